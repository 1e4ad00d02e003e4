// Measurement yardstick, not part of the method: a plain streaming read of a device buffer.
// The HBM fractions of the attention kernels are read against the 8 TB/s data-sheet peak; this
// kernel shows what a kernel that does nothing but 16-byte loads reaches on the same machine.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/mtserve.h"
#include "mts_internal.hpp"

namespace {

typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

constexpr int kUnroll = 8;

// Every workgroup reads one contiguous chunk of the buffer, kUnroll independent 16-byte loads per
// lane in flight at a time (the form that measured fastest of the plain variants tried: grid
// stride or chunked, 2 to 16 loads in flight, 4 to 64 workgroups per CU).
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* __restrict__ src, int64_t n16,
                                                          uint32_t* __restrict__ sink) {
  const int64_t per = (n16 + gridDim.x - 1) / gridDim.x;
  const int64_t lo = (int64_t)blockIdx.x * per;
  const int64_t hi = lo + per < n16 ? lo + per : n16;
  u32x4 acc = {0u, 0u, 0u, 0u};
  int64_t i = lo + threadIdx.x;
  for (; i + (kUnroll - 1) * 256 < hi; i += kUnroll * 256) {
    u32x4 v[kUnroll];
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) v[k] = __builtin_nontemporal_load(src + i + k * 256);
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) acc ^= v[k];
  }
  for (; i < hi; i += 256) acc ^= __builtin_nontemporal_load(src + i);
  // the fold is data-dependent, so the loads cannot be dropped; one word per wavefront is kept
  uint32_t r = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) r ^= __shfl_xor(r, o);
  if ((threadIdx.x & 63) == 0) atomicXor(sink + (blockIdx.x & 1023), r);
}

}  // namespace

extern "C" int32_t mts_diag_stream_read(const void* src, int64_t bytes, void* sink, void* stream) {
  if (!src || !sink) return mts::set_error(MTS_ERR_INVALID_ARG, "src / sink is NULL");
  if (bytes < 0 || (bytes & 15) || (reinterpret_cast<uintptr_t>(src) & 15))
    return mts::set_error(MTS_ERR_INVALID_ARG, "src and bytes must be multiples of 16");
  if (bytes == 0) return MTS_OK;
  int dev = 0, cus = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return mts::set_error(MTS_ERR_HIP, "device query: %s", hipGetErrorString(e));
  const int grid = (cus > 0 ? cus : 256) * 16;
  hipLaunchKernelGGL(stream_read_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const u32x4*>(src), bytes / 16, static_cast<uint32_t*>(sink));
  e = hipGetLastError();
  if (e != hipSuccess) return mts::set_error(MTS_ERR_HIP, "mts_diag_stream_read launch: %s", hipGetErrorString(e));
  return MTS_OK;
}

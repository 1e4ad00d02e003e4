// Plain incremental attention (Sec. 2, Eq. 6-7): one wavefront per (new token, head),
// fp32 logits, running-max softmax and fp32 accumulation, no matrix cores.  PW selects the
// pointwise aggregation instead (silu of the scaled logit, times a normaliser; no softmax).  It serves the
// fp32 element type (the reuse-versus-recompute check shape) and is the slow, simple path
// for bf16 shapes the matrix-core kernel does not take.
#include <math.h>

#include "mts_internal.hpp"

namespace mts {
namespace {

__device__ __forceinline__ float to_float(uint32_t bits) { return __uint_as_float(bits); }
__device__ __forceinline__ float to_float(uint16_t bits) { return __uint_as_float((uint32_t)bits << 16); }

__device__ __forceinline__ void store_elem(uint32_t* p, float v) { *p = __float_as_uint(v); }
__device__ __forceinline__ void store_elem(uint16_t* p, float v) {   // round to nearest even
  uint32_t u = __float_as_uint(v);
  if ((u & 0x7fffffffu) > 0x7f800000u) { *p = (uint16_t)((u >> 16) | 0x40); return; }  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  *p = (uint16_t)(u >> 16);
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

template <typename T, bool PW>
__global__ __launch_bounds__(64) void attn_generic_kernel(PoolGeom g, BatchDev b,
                                                          const T* __restrict__ q,
                                                          T* __restrict__ out, float scale, float inv_norm) {
  constexpr int G = 16 / sizeof(T);
  const int tok = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
  const int H = g.H, D = g.D, S = g.S;

  // user of this token: the largest u with new_indptr[u] <= tok
  int lo = 0, hi = b.batch;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (b.new_indptr[mid] <= tok) lo = mid; else hi = mid;
  }
  const int u = lo;
  const int i = tok - b.new_indptr[u];
  const int P = b.prefix_lens[u];
  const int kv_len = P + i + 1;                       // keys 0 .. P+i are visible
  const int pbeg = b.page_indptr[u];
  const int npg = b.page_indptr[u + 1] - pbeg;

  __shared__ float qs[128];
  __shared__ float ps[64];
  for (int d = lane; d < D; d += 64) qs[d] = to_float(q[((int64_t)tok * H + h) * D + d]);
  __syncthreads();

  float acc0 = 0.f, acc1 = 0.f, m = -INFINITY, l = 0.f;
  for (int base = 0; base < kv_len; base += 64) {
    const int j = base + lane;
    float z = -INFINITY;
    if (j < kv_len && j / S < npg) {
      const int page = b.page_indices[pbeg + j / S];
      if ((unsigned)page < (unsigned)g.num_pages) {
        const int slot = j % S;
        const T* kblk = reinterpret_cast<const T*>(g.layer_base + (int64_t)page * g.page_bytes +
                                                   head_block_offset(0, h, S, D, sizeof(T))) +
                        (int64_t)(slot >> 4) * 16 * D;
        float dot = 0.f;
        for (int d = 0; d < D; ++d) dot = fmaf(qs[d], to_float(kblk[k_sub_index(slot & 15, d, D, G)]), dot);
        z = dot * scale;
      }
    }
    float p;
    if (PW) {
      p = (z == -INFINITY) ? 0.f : z / (1.0f + expf(-z));      // silu; hidden or absent keys weigh 0
    } else {
      const float m_new = fmaxf(m, wave_max(z));        // finite: token `base` is always visible
      p = expf(z - m_new);
      const float alpha = expf(m - m_new);
      l = l * alpha + wave_sum(p);
      acc0 *= alpha;
      acc1 *= alpha;
      m = m_new;
    }
    ps[lane] = p;
    __syncthreads();
    const int cnt = (kv_len - base) < 64 ? (kv_len - base) : 64;
    for (int jj = 0; jj < cnt; ++jj) {
      const int t = base + jj;
      if (t / S >= npg) break;
      const int page = b.page_indices[pbeg + t / S];
      if ((unsigned)page >= (unsigned)g.num_pages) continue;
      const int slot = t % S;
      const T* vblk = reinterpret_cast<const T*>(g.layer_base + (int64_t)page * g.page_bytes +
                                                 head_block_offset(1, h, S, D, sizeof(T))) +
                      (int64_t)(slot >> 4) * 16 * D;
      const float pj = ps[jj];
      if (lane < D) acc0 = fmaf(pj, to_float(vblk[v_sub_index(slot & 15, lane)]), acc0);
      if (lane + 64 < D) acc1 = fmaf(pj, to_float(vblk[v_sub_index(slot & 15, lane + 64)]), acc1);
    }
    __syncthreads();
  }
  T* o = out + ((int64_t)tok * H + h) * D;
  if (lane < D) store_elem(o + lane, PW ? acc0 * inv_norm : acc0 / l);
  if (lane + 64 < D) store_elem(o + lane + 64, PW ? acc1 * inv_norm : acc1 / l);
}

}  // namespace

hipError_t launch_attn_generic(const PoolGeom& g, const void* q, void* out, const BatchDev& b,
                               float sm_scale, float inv_norm, hipStream_t stream) {
  if (b.total_new <= 0) return hipSuccess;
  dim3 grid((unsigned)b.total_new, (unsigned)g.H, 1), block(64, 1, 1);
  const bool pw = inv_norm > 0.f;
  if (g.es == 2) {
    auto kern = pw ? attn_generic_kernel<uint16_t, true> : attn_generic_kernel<uint16_t, false>;
    hipLaunchKernelGGL(kern, grid, block, 0, stream, g, b, (const uint16_t*)q, (uint16_t*)out, sm_scale, inv_norm);
  } else {
    auto kern = pw ? attn_generic_kernel<uint32_t, true> : attn_generic_kernel<uint32_t, false>;
    hipLaunchKernelGGL(kern, grid, block, 0, stream, g, b, (const uint32_t*)q, (uint32_t*)out, sm_scale, inv_norm);
  }
  return hipGetLastError();
}

}  // namespace mts

// Byte-exact KV movement between the contiguous layout and the paged pool:
//   unpack - Cache Scattering (Sec. 3.2 step 3, scatter kernel of Sec. 4.2)
//   append - Cache Update     (Sec. 3.2 step 5, Alg. 1 step 8.2)
//   pack   - gather kernel of the offload path (Sec. 3.2 step 6, Sec. 4.2)
//
// All three are HBM-bound permutations of 16-byte granules (K) and of elements (V, whose pool
// layout is [dim][token]); see kv_move_kernel for how the work is split.
#include <type_traits>

#include "mts_internal.hpp"

namespace mts {
namespace {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));          // one granule, opaque
template <typename T> struct ElemVec;                                // one granule, as elements
template <> struct ElemVec<uint16_t> { typedef uint16_t type __attribute__((ext_vector_type(8))); };
template <> struct ElemVec<uint32_t> { typedef uint32_t type __attribute__((ext_vector_type(4))); };

enum { MODE_UNPACK = 0, MODE_APPEND = 1, MODE_PACK = 2 };

constexpr int kBulkWaves = 4;      // wavefronts (= units) per bulk workgroup

// One wavefront moves one (16-token sub-block, head): the contiguous side moves in whole rows
// (D*es bytes per token and head), the pool side in whole 16-byte granules in pool order, so that
// BOTH sides of every copy are 16-byte-per-lane accesses over full cache lines; the reordering
// in between - the K granule permutation and the V transpose - goes through a wavefront-private
// LDS tile of 16 rows (padded by one granule, which keeps the strided accesses off a single
// bank).  Workgroups [0, bulk_blocks) take the sub-blocks that a run covers completely; those
// behind them take partly covered sub-blocks with the same code under a token mask: rows outside
// the run are neither read nor written, K granules of other tokens are skipped and a V granule
// that the run covers only in part is written element by element, so no slot outside the run
// is ever written.
template <typename T, int MODE, int DCH>
__global__ __launch_bounds__(256) void kv_move_kernel(PoolGeom g, SegDev segs, BatchDev b,
                                                      const T* __restrict__ src_a,
                                                      const T* __restrict__ src_b,
                                                      T* __restrict__ dst_contig, int bulk_blocks,
                                                      int64_t pool_layer_stride, int64_t contig_layer_stride) {
  constexpr int G = 16 / sizeof(T);
  constexpr int D = DCH * G;
  constexpr int PITCH = D + G;       // LDS row pitch in elements (one granule of padding)
  constexpr int NIT = 16 * DCH / 64; // 64-granule rounds per 16-token sub-block
  const int H = g.H, S = g.S;
  constexpr int dch = DCH;
  const int s = blockIdx.y;
  // several layers in one launch: blockIdx.z picks the layer on both sides
  g.layer_base += (int64_t)blockIdx.z * pool_layer_stride;
  src_a += (int64_t)blockIdx.z * contig_layer_stride;
  if (MODE == MODE_APPEND) src_b += (int64_t)blockIdx.z * contig_layer_stride;
  if (MODE == MODE_PACK) dst_contig += (int64_t)blockIdx.z * contig_layer_stride;

  // Resolve the run: user, first pool token, length, and the contiguous K / V planes.  The
  // loads are ordered so that as few of them as possible wait for one another: nothing below
  // returns early between two loads that do not depend on each other.
  int u, pos;
  int64_t n, t0;
  if (MODE == MODE_APPEND) {
    u = s;
    t0 = b.new_indptr[u];
    n = (int64_t)b.new_indptr[u + 1] - t0;
    pos = b.prefix_lens[u];
  } else {
    u = segs.seg_user[s];
    pos = segs.seg_pos[s];
    t0 = segs.seg_tok_indptr[s];
    n = segs.seg_tok_indptr[s + 1] - t0;
  }
  const bool user_ok = (u >= 0 && u < b.batch);
  const int uc = user_ok ? u : 0;
  const int pbeg = b.page_indptr[uc];
  const int npg = b.page_indptr[uc + 1] - pbeg;

  const T* k_plane;
  const T* v_plane;
  T* k_out = nullptr;
  T* v_out = nullptr;
  if (MODE == MODE_APPEND) {
    k_plane = src_a + t0 * H * D;
    v_plane = src_b + t0 * H * D;
  } else {
    const int64_t base = t0 * 2 * H * D;
    k_plane = src_a + base;
    v_plane = k_plane + n * H * D;
    if (MODE == MODE_PACK) {
      k_out = dst_contig + base;
      v_out = k_out + n * H * D;
    }
  }
  const bool run_ok = user_ok && n > 0 && pos >= 0;
  const int64_t npos = run_ok ? n : 1, ppos = run_ok ? pos : 0;
  // 16-token sub-blocks the run covers completely: [full_lo, full_hi) in units of sub-blocks
  const int64_t full_lo = (ppos + 15) >> 4;
  int64_t full_hi = (ppos + npos) >> 4;
  if (full_hi < full_lo || bulk_blocks == 0) full_hi = full_lo;   // a launch of short runs: every sub-block takes the masked form

  // Which sub-block this wavefront moves, and which of its 16 tokens belong to the run.
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t first_sb = ppos >> 4, last_sb = (ppos + npos - 1) >> 4;
  int64_t sb;
  int h;
  bool masked;
  if ((int)blockIdx.x < bulk_blocks) {
    // whole sub-blocks: one wavefront per (sub-block, head)
    const int64_t unit = (int64_t)blockIdx.x * kBulkWaves + wave;
    sb = full_lo + unit / H;
    h = (int)(unit % H);
    masked = false;
    if (!run_ok || sb >= full_hi) return;                       // wavefront-uniform; no block barrier below
  } else {
    // the sub-blocks the whole-sub-block part leaves: all of a run's when the launch has no such
    // part (unit k = k-th sub-block of the run), else the partly covered ones at its two ends
    const int64_t unit = (int64_t)(blockIdx.x - bulk_blocks) * kBulkWaves + wave;
    const int64_t k = unit / H;
    h = (int)(unit % H);
    masked = true;
    if (bulk_blocks == 0) {
      sb = first_sb + k;
    } else {
      const bool head_part = first_sb < full_lo;                            // unit 0: partly covered first
      const bool tail_part = last_sb >= full_hi && !(head_part && last_sb == first_sb);   // unit 1: last
      sb = (k == 0 && head_part) ? first_sb : ((k == 1 && tail_part) ? last_sb : -1);
    }
    if (!run_ok || sb < 0 || sb > last_sb) return;
  }
  const int64_t sbase = sb << 4;
  int t_lo = 0, t_hi = 16;                                      // tokens of the sub-block inside the run
  if (masked) {
    t_lo = (int)(ppos > sbase ? ppos - sbase : 0);
    t_hi = (int)(ppos + npos < sbase + 16 ? ppos + npos - sbase : 16);
  }
  __shared__ __attribute__((aligned(16))) T tile[kBulkWaves][16 * PITCH];
  // masked_c: compile-time copy of `masked`, so that the whole-sub-block form carries no checks
  auto move_sub_block = [&](auto masked_c) __attribute__((always_inline)) {
    constexpr bool MASKED = decltype(masked_c)::value;
    const int64_t lp = sbase / S;
    if (lp >= npg) return;
    const int page = b.page_indices[pbeg + lp];
    if ((unsigned)page >= (unsigned)g.num_pages) return;
    const int sub = (int)(sb & ((S >> 4) - 1));
    char* head = g.layer_base + (int64_t)page * g.page_bytes;
    T* kblk = reinterpret_cast<T*>(head + head_block_offset(0, h, S, D, sizeof(T))) + (int64_t)sub * 16 * D;
    T* vblk = reinterpret_cast<T*>(head + head_block_offset(1, h, S, D, sizeof(T))) + (int64_t)sub * 16 * D;
    const int64_t row0 = sbase - ppos;                          // contiguous-side row of the sub-block's token 0
    T* lt = tile[wave];                                         // [16 tokens][PITCH]: K first, then V
    // LDS operations of one wavefront execute in order; the fence only pins the compiler's order
    auto wave_sync = [] {
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
    };
    auto in_run = [&](int t) { return !MASKED || (t >= t_lo && t < t_hi); };
    typedef typename ElemVec<T>::type EV;
    const u32x4 zero = {0u, 0u, 0u, 0u};
    u32x4 kg[NIT], vg[NIT];
    if (MODE != MODE_PACK) {
      // rows in (whole D*es-byte runs), granules out in pool order
#pragma unroll
      for (int j = 0; j < NIT; ++j) {
        const int gi = j * 64 + lane, t = gi / dch, c = gi % dch;
        const int64_t off = (row0 + t) * H * D + (int64_t)h * D + c * G;
        const bool ok = in_run(t);
        kg[j] = ok ? *reinterpret_cast<const u32x4*>(k_plane + (ok ? off : 0)) : zero;
        vg[j] = ok ? *reinterpret_cast<const u32x4*>(v_plane + (ok ? off : 0)) : zero;
      }
#pragma unroll
      for (int j = 0; j < NIT; ++j) {
        const int gi = j * 64 + lane, t = gi / dch, c = gi % dch;
        *reinterpret_cast<u32x4*>(lt + t * PITCH + c * G) = kg[j];
      }
      wave_sync();
#pragma unroll
      for (int j = 0; j < NIT; ++j) {
        const int p = j * 64 + lane;                            // K granule in pool order
        const int half = p / (dch * 8), c = (p / 8) % dch, slot = p % 8;
        const int t = ((slot >> 2) << 3) + half * 4 + (slot & 3);
        kg[j] = *reinterpret_cast<const u32x4*>(lt + t * PITCH + c * G);
      }
      wave_sync();
#pragma unroll
      for (int j = 0; j < NIT; ++j) {
        const int gi = j * 64 + lane, t = gi / dch, c = gi % dch;
        *reinterpret_cast<u32x4*>(lt + t * PITCH + c * G) = vg[j];
      }
      wave_sync();
#pragma unroll
      for (int j = 0; j < NIT; ++j) {
        const int p = j * 64 + lane;                            // V granule: G tokens of one dim
        const int d = p / (16 / G), part = p % (16 / G);
        EV o;
#pragma unroll
        for (int e = 0; e < G; ++e) o[e] = lt[(part * G + e) * PITCH + d];
        vg[j] = __builtin_bit_cast(u32x4, o);
      }
#pragma unroll
      for (int j = 0; j < NIT; ++j) {
        const int p = j * 64 + lane;
        const int slot = p % 8, half = p / (dch * 8);
        const int t = ((slot >> 2) << 3) + half * 4 + (slot & 3);         // token of K granule p
        if (in_run(t)) *reinterpret_cast<u32x4*>(kblk + (int64_t)p * G) = kg[j];
        // V granule p holds tokens part*G .. part*G+G-1 of one dim: whole if the run covers all
        // of them, else element by element - no slot outside the run is written
        const int part = p % (16 / G);
        int e_lo = t_lo - part * G, e_hi = t_hi - part * G;
        e_lo = e_lo < 0 ? 0 : e_lo;
        e_hi = e_hi > G ? G : e_hi;
        if (!MASKED || (e_lo == 0 && e_hi == G)) {
          *reinterpret_cast<u32x4*>(vblk + (int64_t)p * G) = vg[j];
        } else if (e_lo < e_hi) {
          const EV o = __builtin_bit_cast(EV, vg[j]);
#pragma unroll
          for (int e = 0; e < G; ++e)
            if (e >= e_lo && e < e_hi) vblk[(int64_t)p * G + e] = o[e];
        }
      }
    } else {
      // granules in, in pool order; whole rows out
#pragma unroll
      for (int j = 0; j < NIT; ++j) {
        const int p = j * 64 + lane;
        kg[j] = *reinterpret_cast<const u32x4*>(kblk + (int64_t)p * G);
        vg[j] = *reinterpret_cast<const u32x4*>(vblk + (int64_t)p * G);
      }
#pragma unroll
      for (int j = 0; j < NIT; ++j) {
        const int p = j * 64 + lane;
        const int half = p / (dch * 8), c = (p / 8) % dch, slot = p % 8;
        const int t = ((slot >> 2) << 3) + half * 4 + (slot & 3);
        *reinterpret_cast<u32x4*>(lt + t * PITCH + c * G) = kg[j];
      }
      wave_sync();
#pragma unroll
      for (int j = 0; j < NIT; ++j) {
        const int gi = j * 64 + lane, t = gi / dch, c = gi % dch;
        kg[j] = *reinterpret_cast<const u32x4*>(lt + t * PITCH + c * G);
      }
      wave_sync();
#pragma unroll
      for (int j = 0; j < NIT; ++j) {
        const int p = j * 64 + lane;
        const int d = p / (16 / G), part = p % (16 / G);
        const EV iv = __builtin_bit_cast(EV, vg[j]);
#pragma unroll
        for (int e = 0; e < G; ++e) lt[(part * G + e) * PITCH + d] = iv[e];
      }
      wave_sync();
#pragma unroll
      for (int j = 0; j < NIT; ++j) {
        const int gi = j * 64 + lane, t = gi / dch, c = gi % dch;
        if (in_run(t)) {
          const int64_t off = (row0 + t) * H * D + (int64_t)h * D + c * G;
          *reinterpret_cast<u32x4*>(k_out + off) = kg[j];
          *reinterpret_cast<u32x4*>(v_out + off) = *reinterpret_cast<const u32x4*>(lt + t * PITCH + c * G);
        }
      }
    }
  };
  if (masked) move_sub_block(std::true_type{});
  else move_sub_block(std::false_type{});
}

template <typename T, int MODE, int DCH>
void launch_typed(const PoolGeom& g, const SegDev& segs, const BatchDev& b, dim3 grid, int bulk_blocks,
                  const void* a, const void* bsrc, void* dst, int64_t pool_layer_stride,
                  int64_t contig_layer_stride_bytes, hipStream_t stream) {
  hipLaunchKernelGGL((kv_move_kernel<T, MODE, DCH>), grid, dim3(256, 1, 1), 0, stream, g, segs, b, (const T*)a,
                     (const T*)bsrc, (T*)dst, bulk_blocks, pool_layer_stride,
                     contig_layer_stride_bytes / (int64_t)sizeof(T));
}

template <int MODE>
hipError_t launch_move(const PoolGeom& g, const SegDev& segs, const BatchDev& b, int runs,
                       int64_t max_run_tokens, const void* a, const void* bsrc, void* dst,
                       hipStream_t stream, int layers = 1, int64_t pool_layer_stride = 0,
                       int64_t contig_layer_stride_bytes = 0) {
  if (runs <= 0 || max_run_tokens <= 0 || layers <= 0) return hipSuccess;
  if (layers > 65535) return hipErrorInvalidValue;
  const int G = 16 / g.es;
  // One wavefront per (16-token sub-block, head).  Runs of at least 128 tokens: the sub-blocks a
  // run covers completely (of the longest run) take the unmasked form, the at most two partly
  // covered ones at its ends the masked form.  Shorter runs (a step's few new tokens): every
  // sub-block a run touches, at most ceil(max / 16) + 1, takes the masked form.
  const bool bulk = max_run_tokens >= 128;
  const int64_t bulk_units = bulk ? (max_run_tokens / 16) * (int64_t)g.H : 0;
  const int64_t bulk_blocks = (bulk_units + kBulkWaves - 1) / kBulkWaves;
  const int64_t end_units = (bulk ? 2 : (max_run_tokens + 15) / 16 + 1) * (int64_t)g.H;
  const int64_t blocks = bulk_blocks + (end_units + kBulkWaves - 1) / kBulkWaves;
  if (blocks > 0x7fffffffll) return hipErrorInvalidValue;
  dim3 grid((unsigned)blocks, (unsigned)runs, (unsigned)layers);
  const int dch = g.D / G;
#define MTS_MOVE_CASE(T, DCH_) \
  case DCH_: launch_typed<T, MODE, DCH_>(g, segs, b, grid, (int)bulk_blocks, a, bsrc, dst, pool_layer_stride, \
                                         contig_layer_stride_bytes, stream); break;
  if (g.es == 2) {
    switch (dch) {
      MTS_MOVE_CASE(uint16_t, 4) MTS_MOVE_CASE(uint16_t, 8) MTS_MOVE_CASE(uint16_t, 16)
      default: return hipErrorInvalidValue;
    }
  } else {
    switch (dch) {
      MTS_MOVE_CASE(uint32_t, 8) MTS_MOVE_CASE(uint32_t, 16) MTS_MOVE_CASE(uint32_t, 32)
      default: return hipErrorInvalidValue;
    }
  }
#undef MTS_MOVE_CASE
  return hipGetLastError();
}

}  // namespace

hipError_t launch_unpack(const PoolGeom& g, const void* staging, const SegDev& segs, const BatchDev& b,
                         hipStream_t stream, int layers, int64_t pool_layer_stride, int64_t staging_layer_stride) {
  return launch_move<MODE_UNPACK>(g, segs, b, segs.num_segs, segs.max_seg_tokens, staging, nullptr,
                                  nullptr, stream, layers, pool_layer_stride, staging_layer_stride);
}

hipError_t launch_pack(const PoolGeom& g, void* staging_out, const SegDev& segs, const BatchDev& b,
                       hipStream_t stream, int layers, int64_t pool_layer_stride, int64_t staging_layer_stride) {
  return launch_move<MODE_PACK>(g, segs, b, segs.num_segs, segs.max_seg_tokens, staging_out, nullptr,
                                staging_out, stream, layers, pool_layer_stride, staging_layer_stride);
}

hipError_t launch_append(const PoolGeom& g, const void* k_new, const void* v_new, const BatchDev& b,
                         hipStream_t stream, int layers, int64_t pool_layer_stride, int64_t rows_layer_stride) {
  SegDev none{};
  return launch_move<MODE_APPEND>(g, none, b, b.batch, b.max_new, k_new, v_new, nullptr, stream, layers,
                                  pool_layer_stride, rows_layer_stride);
}

}  // namespace mts

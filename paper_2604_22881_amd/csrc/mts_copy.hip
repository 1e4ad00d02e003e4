// Byte-exact KV movement between the contiguous layout and the paged pool:
//   unpack - Cache Scattering (Sec. 3.2 step 3, scatter kernel of Sec. 4.2)
//   append - Cache Update     (Sec. 3.2 step 5, Alg. 1 step 8.2)
//   pack   - gather kernel of the offload path (Sec. 3.2 step 6, Sec. 4.2)
//
// All three are HBM-bound permutations of 16-byte granules (K) and of elements (V, whose pool
// layout is [dim][token]); see kv_move_kernel for how the work is split.
#include "mts_internal.hpp"

namespace mts {
namespace {

template <typename T>
union Granule {
  uint4 v;
  T     e[16 / sizeof(T)];
};

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));          // one granule, opaque
template <typename T> struct ElemVec;                                // one granule, as elements
template <> struct ElemVec<uint16_t> { typedef uint16_t type __attribute__((ext_vector_type(8))); };
template <> struct ElemVec<uint32_t> { typedef uint32_t type __attribute__((ext_vector_type(4))); };

enum { MODE_UNPACK = 0, MODE_APPEND = 1, MODE_PACK = 2 };

constexpr int kBulkWaves = 4;      // wavefronts (= units) per bulk workgroup

// One launch serves both kinds of work.  Workgroups [0, bulk_blocks) take the 16-token
// sub-blocks that a run covers completely, one wavefront per (sub-block, head): the
// contiguous side moves in whole rows (D*es bytes per token and head), the pool side in whole
// 16-byte granules in pool order, so that BOTH sides of every copy are 16-byte-per-lane
// accesses over full cache lines; the reordering in between - the K granule permutation and
// the V transpose - goes through a wavefront-private LDS tile of 16 rows (padded by one
// granule, which keeps the strided accesses off a single bank).  Workgroups behind them take
// the token groups of partly covered sub-blocks at the two ends of a run, element-wise on the
// pool side: no slot outside the run is ever written.
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
  const int HC = H * dch;
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
  if (full_hi < full_lo || bulk_blocks == 0) full_hi = full_lo;   // short runs: everything goes group by group

  if ((int)blockIdx.x < bulk_blocks) {
    // ---------------- whole sub-blocks: one wavefront per (sub-block, head) ----------------
    __shared__ __attribute__((aligned(16))) T tile[kBulkWaves][16 * PITCH];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t unit = (int64_t)blockIdx.x * kBulkWaves + wave;
    const int64_t sb = full_lo + unit / H;
    const int h = (int)(unit % H);
    if (!run_ok || sb >= full_hi) return;                       // wavefront-uniform; no block barrier below
    const int64_t lp = (sb << 4) / S;
    if (lp >= npg) return;
    const int page = b.page_indices[pbeg + lp];
    if ((unsigned)page >= (unsigned)g.num_pages) return;
    const int sub = (int)(sb & ((S >> 4) - 1));
    char* head = g.layer_base + (int64_t)page * g.page_bytes;
    T* kblk = reinterpret_cast<T*>(head + head_block_offset(0, h, S, D, sizeof(T))) + (int64_t)sub * 16 * D;
    T* vblk = reinterpret_cast<T*>(head + head_block_offset(1, h, S, D, sizeof(T))) + (int64_t)sub * 16 * D;
    const int64_t row0 = (sb << 4) - ppos;                      // contiguous-side row of the sub-block's token 0
    T* lt = tile[wave];                                         // [16 tokens][PITCH]: K first, then V
    // LDS operations of one wavefront execute in order; the fence only pins the compiler's order
    auto wave_sync = [] {
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
    };
    typedef typename ElemVec<T>::type EV;
    u32x4 kg[NIT], vg[NIT];
    if (MODE != MODE_PACK) {
      // rows in (whole D*es-byte runs), granules out in pool order
#pragma unroll
      for (int j = 0; j < NIT; ++j) {
        const int gi = j * 64 + lane, t = gi / dch, c = gi % dch;
        const int64_t off = (row0 + t) * H * D + (int64_t)h * D + c * G;
        kg[j] = *reinterpret_cast<const u32x4*>(k_plane + off);
        vg[j] = *reinterpret_cast<const u32x4*>(v_plane + off);
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
        *reinterpret_cast<u32x4*>(kblk + (int64_t)p * G) = kg[j];
        *reinterpret_cast<u32x4*>(vblk + (int64_t)p * G) = vg[j];
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
        const int64_t off = (row0 + t) * H * D + (int64_t)h * D + c * G;
        *reinterpret_cast<u32x4*>(k_out + off) = kg[j];
        *reinterpret_cast<u32x4*>(v_out + off) = *reinterpret_cast<const u32x4*>(lt + t * PITCH + c * G);
      }
    }
    return;
  }

  // ---------------- token groups of partly covered sub-blocks at the run's ends ----------------
  // One thread moves a G x G micro-tile: G tokens of an aligned group x one granule of G dims.
  const int64_t grp0 = ppos / G;
  const int64_t grp1 = (ppos + npos - 1) / G;
  const int64_t skip_lo = full_lo * (16 / G), skip_hi = full_hi * (16 / G);   // groups the bulk part moved
  const int64_t n_groups = (grp1 - grp0 + 1) - (skip_hi - skip_lo);
  const int64_t idx = (int64_t)(blockIdx.x - bulk_blocks) * blockDim.x + threadIdx.x;
  const bool mine = run_ok && idx < n_groups * HC;
  int64_t grp = grp0 + (mine ? idx / HC : 0);
  if (grp >= skip_lo) grp += skip_hi - skip_lo;
  const int hc = mine ? (int)(idx % HC) : 0;
  const int h = hc / dch, c = hc % dch;
  const int64_t tbase = grp * G;                       // first token of the aligned group
  int lo = (int)((ppos > tbase ? ppos : tbase) - tbase);                          // valid tokens of
  int hi = (int)(((ppos + npos) < (tbase + G) ? (ppos + npos) : (tbase + G)) - tbase);   // the group: [lo, hi)
  if (!mine) lo = hi = 0;
  const int64_t row0 = tbase - ppos;                   // contiguous-side row of group token 0
  const int64_t col = (int64_t)h * D + c * G;

  // contiguous-side loads first (unpack / append): they need nothing from the page table
  Granule<T> krow[G], vrow[G];
  if (MODE != MODE_PACK) {
#pragma unroll
    for (int i = 0; i < G; ++i) {
      if (i >= lo && i < hi) {
        const int64_t off = (row0 + i) * H * D + col;
        krow[i].v = *reinterpret_cast<const uint4*>(k_plane + off);
        vrow[i].v = *reinterpret_cast<const uint4*>(v_plane + off);
      } else {
        krow[i].v = make_uint4(0, 0, 0, 0);
        vrow[i].v = make_uint4(0, 0, 0, 0);
      }
    }
  }

  // One aligned group never straddles a 16-token sub-block, hence never a page.
  const int64_t lp = tbase / S;
  const bool page_ok = mine && lp < npg;
  const int page = page_ok ? b.page_indices[pbeg + lp] : -1;
  if ((unsigned)page >= (unsigned)g.num_pages) return;
  const int slot = (int)(tbase % S);
  const int sub = slot >> 4, t16 = slot & 15;
  char* head = g.layer_base + (int64_t)page * g.page_bytes;
  T* kblk = reinterpret_cast<T*>(head + head_block_offset(0, h, S, D, sizeof(T))) + (int64_t)sub * 16 * D;
  T* vblk = reinterpret_cast<T*>(head + head_block_offset(1, h, S, D, sizeof(T))) + (int64_t)sub * 16 * D;

  if (MODE != MODE_PACK) {
#pragma unroll
    for (int i = 0; i < G; ++i)
      if (i >= lo && i < hi)
        *reinterpret_cast<uint4*>(kblk + k_sub_index(t16 + i, c * G, D, G)) = krow[i].v;
    if (lo == 0 && hi == G) {
#pragma unroll
      for (int dd = 0; dd < G; ++dd) {
        Granule<T> o;
#pragma unroll
        for (int i = 0; i < G; ++i) o.e[i] = vrow[i].e[dd];
        *reinterpret_cast<uint4*>(vblk + v_sub_index(t16, c * G + dd)) = o.v;
      }
    } else {
#pragma unroll
      for (int dd = 0; dd < G; ++dd) {
#pragma unroll
        for (int i = 0; i < G; ++i)
          if (i >= lo && i < hi) vblk[v_sub_index(t16 + i, c * G + dd)] = vrow[i].e[dd];
      }
    }
  } else {
    Granule<T> vcol[G];
#pragma unroll
    for (int dd = 0; dd < G; ++dd)
      vcol[dd].v = *reinterpret_cast<const uint4*>(vblk + v_sub_index(t16, c * G + dd));
#pragma unroll
    for (int i = 0; i < G; ++i)
      krow[i].v = *reinterpret_cast<const uint4*>(kblk + k_sub_index(t16 + i, c * G, D, G));
#pragma unroll
    for (int i = 0; i < G; ++i) {
      if (i >= lo && i < hi) {
        const int64_t off = (row0 + i) * H * D + col;
        *reinterpret_cast<uint4*>(k_out + off) = krow[i].v;
        Granule<T> o;
#pragma unroll
        for (int dd = 0; dd < G; ++dd) o.e[dd] = vcol[dd].e[i];
        *reinterpret_cast<uint4*>(v_out + off) = o.v;
      }
    }
  }
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
  // Runs of at least 128 tokens: whole sub-blocks of the longest run x heads, one per wavefront,
  // then the groups of at most two partly covered sub-blocks per run (2 * 16/G groups, + 2).
  // Shorter runs (a step's few new tokens) are latency-bound, and one thread per group with
  // fewer, smaller workgroups finishes sooner: all their groups take the group path.
  const bool bulk = max_run_tokens >= 128;
  const int64_t bulk_units = bulk ? (max_run_tokens / 16) * (int64_t)g.H : 0;
  const int64_t bulk_blocks = (bulk_units + kBulkWaves - 1) / kBulkWaves;
  const int64_t edge_groups = bulk ? (2 * (16 / G) + 2) : (max_run_tokens / G + 2);
  const int64_t edge_work = edge_groups * (int64_t)g.H * (g.D / G);
  const int64_t blocks = bulk_blocks + (edge_work + 255) / 256;
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

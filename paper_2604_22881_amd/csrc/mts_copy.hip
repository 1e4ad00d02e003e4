// Byte-exact KV movement between the contiguous layout and the paged pool:
//   unpack - Cache Scattering (Sec. 3.2 step 3, scatter kernel of Sec. 4.2)
//   append - Cache Update     (Sec. 3.2 step 5, Alg. 1 step 8.2)
//   pack   - gather kernel of the offload path (Sec. 3.2 step 6, Sec. 4.2)
//
// All three are HBM-bound permutations.  One thread moves a G x G micro-tile (G tokens of
// an aligned token group x one 16-byte granule of G dims, G = 16 / element size): G granule
// copies for K, and a register transpose for V, whose pool layout is [dim][token].  Adjacent
// lanes take adjacent granules of the same token rows, so every contiguous-side access is a
// fully coalesced 16-byte-per-lane access.  Token groups that a run covers only partly are
// written element by element on the pool side: no slot outside the run is ever written.
#include "mts_internal.hpp"

namespace mts {
namespace {

template <typename T>
union Granule {
  uint4 v;
  T     e[16 / sizeof(T)];
};

enum { MODE_UNPACK = 0, MODE_APPEND = 1, MODE_PACK = 2 };

template <typename T, int MODE>
__global__ __launch_bounds__(256) void kv_move_kernel(PoolGeom g, SegDev segs, BatchDev b,
                                                      const T* __restrict__ src_a,
                                                      const T* __restrict__ src_b,
                                                      T* __restrict__ dst_contig) {
  constexpr int G = 16 / sizeof(T);
  const int H = g.H, D = g.D, S = g.S;
  const int dch = D / G;            // granules per head row
  const int HC = H * dch;
  const int s = blockIdx.y;

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
  const int64_t grp0 = ppos / G;
  const int64_t grp1 = (ppos + npos - 1) / G;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const bool mine = run_ok && idx < (grp1 - grp0 + 1) * HC;
  const int64_t grp = grp0 + (mine ? idx / HC : 0);
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

template <int MODE>
hipError_t launch_move(const PoolGeom& g, const SegDev& segs, const BatchDev& b, int runs,
                       int64_t max_run_tokens, const void* a, const void* bsrc, void* dst,
                       hipStream_t stream) {
  if (runs <= 0 || max_run_tokens <= 0) return hipSuccess;
  const int G = 16 / g.es;
  const int64_t work = (max_run_tokens / G + 2) * (int64_t)g.H * (g.D / G);
  dim3 grid((unsigned)((work + 255) / 256), (unsigned)runs, 1), block(256, 1, 1);
  if (g.es == 2) {
    hipLaunchKernelGGL((kv_move_kernel<uint16_t, MODE>), grid, block, 0, stream, g, segs, b,
                       (const uint16_t*)a, (const uint16_t*)bsrc, (uint16_t*)dst);
  } else {
    hipLaunchKernelGGL((kv_move_kernel<uint32_t, MODE>), grid, block, 0, stream, g, segs, b,
                       (const uint32_t*)a, (const uint32_t*)bsrc, (uint32_t*)dst);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_unpack(const PoolGeom& g, const void* staging, const SegDev& segs,
                         const BatchDev& b, hipStream_t stream) {
  return launch_move<MODE_UNPACK>(g, segs, b, segs.num_segs, segs.max_seg_tokens, staging, nullptr,
                                  nullptr, stream);
}

hipError_t launch_pack(const PoolGeom& g, void* staging_out, const SegDev& segs,
                       const BatchDev& b, hipStream_t stream) {
  return launch_move<MODE_PACK>(g, segs, b, segs.num_segs, segs.max_seg_tokens, staging_out, nullptr,
                                staging_out, stream);
}

hipError_t launch_append(const PoolGeom& g, const void* k_new, const void* v_new,
                         const BatchDev& b, hipStream_t stream) {
  SegDev none{};
  return launch_move<MODE_APPEND>(g, none, b, b.batch, b.max_new, k_new, v_new, nullptr, stream);
}

}  // namespace mts

// Cache-miss / long-segment prefill attention on the matrix cores: the same operation as the
// streaming kernel (Sec. 2, Eq. 6-7; with no cached prefix it is the causal attention of the
// recompute baseline, Sec. 5.1), laid out for the case of MANY new tokens per user, where the
// work is a dense contraction and K/V reuse across queries decides the speed.
//
// A workgroup (4 wavefronts) owns one (user, head, block of 4*16*NQB new tokens): wavefront w
// takes queries 16*NQB*w .. 16*NQB*(w+1)-1 of the block.  All four walk the same kv tiles, so each
// 32-token K/V tile is fetched from global memory ONCE per workgroup: every wavefront loads a
// quarter of the tile's 16-byte MFMA fragments, parks them in LDS in fragment order (lane l of
// fragment f at f*1 KiB + l*16 B: reads and writes are conflict-free), and after one barrier
// all four read the whole tile back as ready-made operands.  Two LDS stages, one barrier per
// tile; global loads run PFD tiles ahead through a register ring, and the block's page ids are
// copied to LDS once, so that no load in the loop depends on another load.
//
// Operand flow, pool layout and the fixed-reference softmax are those of the streaming kernel
// (S^T = K Q^T, O^T = V^T P^T with v_mfma_f32_16x16x32_bf16; reference max from the first tile,
// no rescaling; an overflowed denominator makes the whole workgroup redo its block with the
// exact max, found by a K-only pass).  Workgroups of one (user, head) land on one XCD, longest
// block first, so that its K/V stays in that XCD's L2 while the blocks re-read it.  Every block
// writes its output rows itself; nothing is merged.
//
// PW selects the pointwise aggregation out = inv_norm * sum_j silu(c * q.k_j) v_j: no reference
// max, no denominator, no redo; hidden keys carry logit 0 (silu(0) = 0).
#include <math.h>

#include <mutex>
#include <type_traits>

#include "mts_internal.hpp"

namespace mts {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4;   // one 16-byte fragment

constexpr int kTile = 32;        // kv tokens per step
constexpr int kXcds = 8;
constexpr int kMaxIdBytes = 64 * 1024;   // LDS page table of one block

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ float fast_silu(float x) {
  return x * __builtin_amdgcn_rcpf(1.0f + fast_exp2(-1.4426950408889634f * x));
}

__device__ __forceinline__ float quad_row_max(float v) {
  unsigned u = __float_as_uint(v);
  auto a = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  v = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  u = __float_as_uint(v);
  auto b = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}

template <int D, int PFD, int WPS, int kNQB, bool PW>
__global__ __launch_bounds__(256, WPS) void attn_prefill_kernel(PoolGeom g, BatchDev b,
                                                                const uint16_t* __restrict__ q,
                                                                uint16_t* __restrict__ out, float c, float inv_norm,
                                                                int q_blocks_max, int n_pairs, int id_cap) {
  constexpr int kWaveQ = 16 * kNQB;    // queries per wavefront
  constexpr int kBlockQ = 4 * kWaveQ;  // new tokens per workgroup
  constexpr int KS = D / 32;           // k-steps of Q.K
  constexpr int DB = D / 16;           // 16-dim blocks of the output
  constexpr int FR = 2 * KS + DB;      // 16-byte fragments per lane and tile: K (half, step), then V (dim block)
  constexpr int FQ = FR / 4;           // fragments each wavefront fetches: FQ/2 of K, FQ/2 of V
  static_assert(FQ % 2 == 0 && FQ >= 2, "fragment split");

  extern __shared__ int s_ids[];       // physical page of every logical page the block reads
  __shared__ u32x4 stage[2][FR * 64];  // two tiles in fragment order
  __shared__ int redo_flag;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = uniform(tid >> 6);
  const int r = lane & 15, gq = lane >> 4;
  const int H = g.H, S = g.S;

  // blockIdx -> XCD is round-robin: all blocks of one (user, head) share blockIdx % 8
  const int slot = blockIdx.x / kXcds;
  const int pair = (slot / q_blocks_max) * kXcds + (blockIdx.x % kXcds);
  if (pair >= n_pairs) return;
  const int qblk = q_blocks_max - 1 - (slot % q_blocks_max);    // longest causal rows first
  const int u = pair / H, h = pair % H;
  const int tok0 = b.new_indptr[u];
  const int n_u = b.new_indptr[u + 1] - tok0;
  const int Q0 = qblk * kBlockQ;
  if (Q0 >= n_u) return;                                        // workgroup-uniform
  const int P = b.prefix_lens[u];
  const int pbeg = b.page_indptr[u];
  const int npg = b.page_indptr[u + 1] - pbeg;
  const int T_u = P + n_u;                                      // tokens that hold data

  const int blk_end = (n_u < Q0 + kBlockQ) ? n_u : (Q0 + kBlockQ);
  const int tiles_wg = (P + blk_end + kTile - 1) / kTile;      // kv tiles the block's last query sees
  const int q0 = Q0 + kWaveQ * wave;                                // this wavefront's queries
  int nq = n_u - q0;
  nq = nq < 0 ? 0 : (nq > kWaveQ ? kWaveQ : nq);
  const int tiles_w = nq > 0 ? (P + q0 + nq + kTile - 1) / kTile : 0;
  const int first_query_pos = P + q0;

  // page table of the block -> LDS; ids the metadata does not back become page 0 (in bounds;
  // such slots lie past the user's last token and are masked)
  const int n_ids = ((tiles_wg * 2 - 1) >> g.sub_shift) + 1;
  if (n_ids > id_cap) return;          // lengths beyond the bound the call stated: no output, no overrun
  for (int i = tid; i < n_ids; i += 256) {
    int id = i < npg ? b.page_indices[pbeg + i] : 0;
    if ((unsigned)id >= (unsigned)g.num_pages) id = 0;
    s_ids[i] = id;
  }

  const int sub_mask = (1 << g.sub_shift) - 1;
  const int64_t v_off = (int64_t)S * D * 2;
  const char* head_base = g.layer_base + (int64_t)h * 2 * S * D * 2;

  auto tile_bases = [&](int tile, const char*& kb0, const char*& kb1) __attribute__((always_inline)) {
    const int sb0 = tile * 2, sb1 = sb0 + 1;
    const int id0 = s_ids[sb0 >> g.sub_shift], id1 = s_ids[sb1 >> g.sub_shift];
    kb0 = head_base + (int64_t)id0 * g.page_bytes + (int64_t)(sb0 & sub_mask) * 16 * D * 2;
    kb1 = head_base + (int64_t)id1 * g.page_bytes + (int64_t)(sb1 & sub_mask) * 16 * D * 2;
  };
  // K fragment (half hf, k-step s): rows 0-7 from sub-block 0, rows 8-15 from sub-block 1
  auto k_ptr = [&](const char* kb0, const char* kb1, int hf, int s) __attribute__((always_inline)) {
    return reinterpret_cast<const u32x4*>(((r < 8) ? kb0 : kb1) + (r & 7) * 16 +
                                          ((hf * (D / 8) + 4 * s + gq) * 8) * 16);
  };
  // V^T fragment db: dim 16*db + r, tokens 8*gq .. +7 of the tile
  auto v_ptr = [&](const char* kb0, const char* kb1, int db) __attribute__((always_inline)) {
    return reinterpret_cast<const u32x4*>(((gq < 2) ? kb0 : kb1) + v_off + (r * 16 + (gq & 1) * 8) * 2 +
                                          db * 16 * 16 * 2);
  };

  // Register ring: slot p holds this wavefront's quarter of tile j, j % PFD == p, on its way to
  // LDS.  Fragment f = 4*j + wave: the first FQ/2 are K fragments, the rest V fragments.
  u32x4 ring[PFD][FQ];
  const int last_tile = tiles_wg - 1;
  auto load = [&](auto slot_c, int tile) __attribute__((always_inline)) {
    constexpr int p = decltype(slot_c)::value;
    const char *kb0, *kb1;
    tile_bases(tile < last_tile ? tile : last_tile, kb0, kb1);   // past the end: repeat (never used)
#pragma unroll
    for (int j = 0; j < FQ / 2; ++j) {
      const int f = 4 * j + wave;
      ring[p][j] = *k_ptr(kb0, kb1, f / KS, f % KS);
    }
#pragma unroll
    for (int j = FQ / 2; j < FQ; ++j) ring[p][j] = *v_ptr(kb0, kb1, 4 * j + wave - 2 * KS);
  };
  auto park = [&](auto slot_c, int st) __attribute__((always_inline)) {
    constexpr int p = decltype(slot_c)::value;
#pragma unroll
    for (int j = 0; j < FQ; ++j) stage[st][(4 * j + wave) * 64 + lane] = ring[p][j];
  };

  // Q^T fragments: lane (r, gq) holds query q0+16*qb+r, dims 32*s + 8*gq .. +7.
  bf16x8 qf[kNQB][KS];
#pragma unroll
  for (int qb = 0; qb < kNQB; ++qb) {
    const int i = q0 + 16 * qb + r;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      if (i < n_u) {
        qf[qb][s] = *reinterpret_cast<const bf16x8*>(q + ((int64_t)(tok0 + i) * H + h) * D + 32 * s + 8 * gq);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[qb][s][e] = (__bf16)0.0f;
      }
    }
  }
  bf16x8 ones;
#pragma unroll
  for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;

  f32x4 o[DB][kNQB];
  f32x4 lacc[kNQB];                // softmax denominators (all 4 entries of a lane are equal)
  float m[kNQB], mcq[kNQB];        // reference max: raw logit units / scaled for the base-2 exponent
#pragma unroll
  for (int qb = 0; qb < kNQB; ++qb) { m[qb] = -INFINITY; mcq[qb] = 0.f; }

  bf16x8 kf[2][KS];
  bf16x8 vf[DB];
  auto read_k = [&](int st) __attribute__((always_inline)) {
#pragma unroll
    for (int f = 0; f < 2 * KS; ++f) {
      const u32x4 v = stage[st][f * 64 + lane];
      kf[f / KS][f % KS] = *reinterpret_cast<const bf16x8*>(&v);
    }
  };
  auto read_v = [&](int st) __attribute__((always_inline)) {
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      const u32x4 v = stage[st][(2 * KS + db) * 64 + lane];
      vf[db] = *reinterpret_cast<const bf16x8*>(&v);
    }
  };

  // S^T of query block qb against kf.  The lane holds, for query q0+16*qb+r, keys
  // tb + 8*gq + {0..3} (s0) and {4..7} (s1); with `masked`, keys the query must not see
  // (causal order among the new tokens) are set to -inf.
  auto scores = [&](int qb, int tb, bool masked, f32x4& s0, f32x4& s1) __attribute__((always_inline)) {
    s0 = f32x4{0.f, 0.f, 0.f, 0.f};
    s1 = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[0][s], qf[qb][s], s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[1][s], qf[qb][s], s1, 0, 0, 0);
    }
    if (masked) {
      const int qpos = first_query_pos + 16 * qb + r;
      const int kbase = tb + 8 * gq;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (kbase + e > qpos) s0[e] = PW ? 0.f : -INFINITY;
        if (kbase + 4 + e > qpos) s1[e] = PW ? 0.f : -INFINITY;
      }
    }
  };
  auto max8 = [](const f32x4& s0, const f32x4& s1) __attribute__((always_inline)) {
    return fmaxf(fmaxf(fmaxf(s0[0], s0[1]), fmaxf(s0[2], s0[3])),
                 fmaxf(fmaxf(s1[0], s1[1]), fmaxf(s1[2], s1[3])));
  };
  auto accumulate = [&](int qb, int tb, bool masked) __attribute__((always_inline)) {
    f32x4 s0, s1;
    scores(qb, tb, masked, s0, s1);
    bf16x8 pf;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if constexpr (PW) {
        pf[e] = (__bf16)fast_silu(s0[e] * c);
        pf[4 + e] = (__bf16)fast_silu(s1[e] * c);
      } else {
        pf[e] = (__bf16)fast_exp2(fmaf(s0[e], c, -mcq[qb]));
        pf[4 + e] = (__bf16)fast_exp2(fmaf(s1[e], c, -mcq[qb]));
      }
    }
#pragma unroll
    for (int db = 0; db < DB; ++db)
      o[db][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[db], pf, o[db][qb], 0, 0, 0);
    // row sums of the (rounded) weights on the matrix core: every row of ones . P^T
    if constexpr (!PW) lacc[qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pf, lacc[qb], 0, 0, 0);
  };
  // One tile from LDS stage st for all four query blocks, with no branch between them.  Query
  // blocks past the segment's end hold zero queries and are never written; a wavefront whose
  // queries all lie before the tile would compute weights of exactly zero (step() skips those
  // tiles in the causal tail).  MASKED adds what only
  // the causal tail needs: the mask, and zeroing of V slots past the user's last token (they
  // may hold anything).
  auto compute = [&](auto masked_c, int st, int tile) __attribute__((always_inline)) {
    constexpr bool MASKED = decltype(masked_c)::value;
    read_k(st);
    read_v(st);
    const int tb = tile * kTile;
    if constexpr (MASKED) {
      if (tb + kTile > T_u) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (tb + 8 * gq + e >= T_u) vf[db][e] = (__bf16)0.0f;
      }
    }
#pragma unroll
    for (int qb = 0; qb < kNQB; ++qb) accumulate(qb, tb, MASKED);
  };
  // Step `tile` (ring slot k = tile % PFD): compute it from its stage, move tile+1 from the ring
  // to the other stage, refill that ring slot PFD tiles ahead.  The barrier both publishes
  // tile+1 and retires every read of the stage that tile+2 will overwrite.
  auto step = [&](auto masked_c, auto slot_c, int tile) __attribute__((always_inline)) {
    constexpr int pn = (decltype(slot_c)::value + 1) % PFD;
    const int st = tile & 1;
    // tiles past the wavefront's own last query hold no key it may see (the later wavefronts of
    // the block still need them): it only helps to move them
    if (!decltype(masked_c)::value || tile < tiles_w) compute(masked_c, st, tile);
    park(std::integral_constant<int, pn>{}, st ^ 1);
    load(std::integral_constant<int, pn>{}, tile + 1 + PFD);
    __syncthreads();
  };
  // tiles below hide no key from any query of the block (its first wavefront sees the least)
  int fast_all = (P + Q0 + 1) / kTile;
  if (fast_all > tiles_wg) fast_all = tiles_wg;
  constexpr std::false_type body{};
  constexpr std::true_type tail{};

  __syncthreads();                                               // page table visible
  for (int attempt = 0; attempt < 2; ++attempt) {                // workgroup-uniform
#pragma unroll
    for (int qb = 0; qb < kNQB; ++qb) {
      lacc[qb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int db = 0; db < DB; ++db) o[db][qb] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    if (!PW && attempt == 1) {
      // exact max of every query over its whole visible range: K only, straight from global
      float mx[kNQB];
#pragma unroll
      for (int qb = 0; qb < kNQB; ++qb) mx[qb] = -INFINITY;
      for (int tile = 0; tile < tiles_w; ++tile) {             // tiles past tiles_w hold no visible key
        const char *kb0, *kb1;
        tile_bases(tile, kb0, kb1);
#pragma unroll
        for (int f = 0; f < 2 * KS; ++f) {
          const u32x4 v = *k_ptr(kb0, kb1, f / KS, f % KS);
          kf[f / KS][f % KS] = *reinterpret_cast<const bf16x8*>(&v);
        }
        const int tb = tile * kTile;
#pragma unroll
        for (int qb = 0; qb < kNQB; ++qb) {
          f32x4 s0, s1;
          scores(qb, tb, true, s0, s1);
          mx[qb] = fmaxf(mx[qb], max8(s0, s1));
        }
      }
#pragma unroll
      for (int qb = 0; qb < kNQB; ++qb) {
        m[qb] = quad_row_max(mx[qb]);
        mcq[qb] = (m[qb] == -INFINITY ? 0.f : m[qb]) * c;
      }
    }

    // prologue: tile 0 into stage 0, tiles 1..PFD into the ring
    load(std::integral_constant<int, 0>{}, 0);
    park(std::integral_constant<int, 0>{}, 0);
    if constexpr (PFD > 1) load(std::integral_constant<int, 1 % PFD>{}, 1);
    if constexpr (PFD > 2) load(std::integral_constant<int, 2 % PFD>{}, 2);
    if constexpr (PFD > 3) load(std::integral_constant<int, 3 % PFD>{}, 3);
    load(std::integral_constant<int, 0>{}, PFD);
    __syncthreads();

    if (!PW && attempt == 0) {
      // reference max = max of the first tile (tile 0 holds key 0, which every query sees)
      read_k(0);
#pragma unroll
      for (int qb = 0; qb < kNQB; ++qb) {
        f32x4 s0, s1;
        scores(qb, 0, true, s0, s1);
        m[qb] = quad_row_max(max8(s0, s1));
        mcq[qb] = (m[qb] == -INFINITY ? 0.f : m[qb]) * c;
      }
    }

    int tile = 0;
    while (tile + PFD <= fast_all) {                               // steady state: fully visible tiles
      step(body, std::integral_constant<int, 0>{}, tile);
      if constexpr (PFD > 1) step(body, std::integral_constant<int, 1>{}, tile + 1);
      if constexpr (PFD > 2) step(body, std::integral_constant<int, 2>{}, tile + 2);
      if constexpr (PFD > 3) step(body, std::integral_constant<int, 3>{}, tile + 3);
      tile += PFD;
    }
    for (; tile < tiles_wg; tile += PFD) {                         // causal tail, and what is left over
      step(tail, std::integral_constant<int, 0>{}, tile);
      if constexpr (PFD > 1) { if (tile + 1 < tiles_wg) step(tail, std::integral_constant<int, 1>{}, tile + 1); }
      if constexpr (PFD > 2) { if (tile + 2 < tiles_wg) step(tail, std::integral_constant<int, 2>{}, tile + 2); }
      if constexpr (PFD > 3) { if (tile + 3 < tiles_wg) step(tail, std::integral_constant<int, 3>{}, tile + 3); }
    }

    if constexpr (PW) break;                                     // no statistics, nothing to redo
    // A reference far below the true max shows up as an overflowed (or NaN) denominator of a
    // real query; then every wavefront of the block goes round again.
    // (the numerator overflows first when the values are large: the sum of a query's absolute
    // accumulator values is infinite or NaN as soon as one of them is)
    bool bad = false;
#pragma unroll
    for (int qb = 0; qb < kNQB; ++qb) {
      float mag = 0.f;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int k = 0; k < 4; ++k) mag += fabsf(o[db][qb][k]);
      bad |= (16 * qb + r < nq) && (!(lacc[qb][0] < 1e37f) || !(mag < 3.0e38f));
    }
    if (tid == 0) redo_flag = 0;
    __syncthreads();
    if (bad) redo_flag = 1;
    __syncthreads();
    const int redo = redo_flag;
    __syncthreads();                                             // everyone has read the flag and left the stages
    if (!redo) break;
  }

#pragma unroll
  for (int qb = 0; qb < kNQB; ++qb) {
    const int qi = 16 * qb + r;
    if (qi < nq) {
      const float inv = PW ? inv_norm : 1.0f / lacc[qb][0];
      uint16_t* orow = out + ((int64_t)(tok0 + q0 + qi) * H + h) * D + 4 * gq;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        bf16x4 ob;
#pragma unroll
        for (int k = 0; k < 4; ++k) ob[k] = (__bf16)(o[db][qb][k] * inv);
        *reinterpret_cast<bf16x4*>(orow + 16 * db) = ob;
      }
    }
  }
}

template <int D, int PFD, int WPS, int NQB, bool PW>
hipError_t launch_one(const PoolGeom& g, const BatchDev& b, const uint16_t* q, uint16_t* out, float c,
                      float inv_norm, int64_t id_bytes, hipStream_t stream) {
  auto kern = attn_prefill_kernel<D, PFD, WPS, NQB, PW>;
  constexpr int kBlockQ = 64 * NQB;
  int q_blocks_max = (b.max_new + kBlockQ - 1) / kBlockQ;
  if (q_blocks_max < 1) q_blocks_max = 1;
  static std::once_flag attr_once;                               // static + dynamic LDS may pass 64 KiB
  static hipError_t attr_status = hipSuccess;
  std::call_once(attr_once, [&] {
    attr_status = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, kMaxIdBytes);
  });
  if (attr_status != hipSuccess) return attr_status;
  const int n_pairs = b.batch * g.H;
  const int64_t grid = (int64_t)((n_pairs + kXcds - 1) / kXcds) * kXcds * q_blocks_max;
  if (grid <= 0 || grid > 0x7fffffffll) return hipErrorInvalidValue;
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), (size_t)id_bytes, stream, g, b, q, out, c,
                     inv_norm, q_blocks_max, n_pairs, (int)(id_bytes / 4));
  return hipGetLastError();
}

}  // namespace

bool attn_prefill_applicable(const PoolGeom& g, const BatchDev& b) {
  if (g.es != 2 || (g.D != 64 && g.D != 128)) return false;
  const int64_t ids = ((int64_t)b.max_total_len + g.S - 1) / g.S + 4;
  return ids * 4 <= kMaxIdBytes;
}

hipError_t launch_attn_prefill(const PoolGeom& g, const void* q, void* out, const BatchDev& b,
                               float sm_scale, float inv_norm, hipStream_t stream) {
  if (b.total_new <= 0 || b.batch <= 0) return hipSuccess;
  if (!attn_prefill_applicable(g, b)) return hipErrorInvalidValue;
  const bool pw = inv_norm > 0.f;
  // softmax logits are exponentiated in base 2; the pointwise scale stays in natural units
  const float c = pw ? sm_scale : sm_scale * 1.4426950408889634f;
  // table entries one block may touch: its tiles end at most one tile past max_total_len
  const int64_t id_bytes = (((int64_t)b.max_total_len + g.S - 1) / g.S + 4) * 4;
  const uint16_t* qp = reinterpret_cast<const uint16_t*>(q);
  uint16_t* op = reinterpret_cast<uint16_t*>(out);
  // Two wavefronts per SIMD in both shapes (<= 256 registers each): one wavefront alone issues
  // in order and leaves its LDS operand reads and MFMA -> VALU dependencies exposed.  At
  // D = 128 that means 32 queries per wavefront (64-register accumulator) and 128-query blocks.
  switch (g.D) {
    case 64:
      return pw ? launch_one<64, 3, 2, 4, true>(g, b, qp, op, c, inv_norm, id_bytes, stream)
                : launch_one<64, 3, 2, 4, false>(g, b, qp, op, c, 0.f, id_bytes, stream);
    case 128:
      return pw ? launch_one<128, 2, 2, 2, true>(g, b, qp, op, c, inv_norm, id_bytes, stream)
                : launch_one<128, 2, 2, 2, false>(g, b, qp, op, c, 0.f, id_bytes, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace mts

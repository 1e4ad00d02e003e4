// Incremental-prefill attention on the matrix cores (Sec. 2, Eq. 6-7; Alg. 1 step 8.4),
// bf16 inputs, fp32 logits / softmax statistics / accumulators.
//
// Schedule.  The work of one call is a single sequence of 32-token kv tiles, ordered by
// (user, query tile, head, tile).  The launch is persistent: a fixed number of wavefronts
// (one per SIMD) each take an equal, contiguous share of that sequence, so lognormal
// history lengths cost no imbalance and every K/V byte is read from HBM exactly once.  Every
// workgroup derives the schedule by itself from the device-resident lengths (a prefix sum in
// LDS), so the host needs no copy of them.  A wavefront that covers a whole (query tile,
// head) writes its output rows; where a share boundary cuts through one, the wavefronts on
// both sides write unnormalised partials and a small merge kernel finishes those rows, in
// wavefront order (deterministic).
//
// Operand flow.  Scores are computed transposed, S^T = K Q^T with v_mfma_f32_16x16x32_bf16:
// tokens are the M rows, queries the N columns, so a lane's accumulator values belong to ONE
// query and softmax statistics are per-lane scalars.  With the pool's K slot order, the 8
// values a lane holds after the two half-tiles are 8 consecutive tokens, which is exactly the
// B fragment of O^T = V^T P^T; V is stored [dim][token], so its A fragment is one 16-byte
// load.  Nothing is staged through LDS: each 16-byte global load is already an MFMA fragment
// and a wavefront's loads cover whole 512-byte runs of a page.
//
// Pipeline.  Each wavefront keeps a ring of PF tiles in flight in registers.  All loads of the
// steady state are unconditional (positions past a segment's end repeat its last tile), so the
// in-order vector-memory counter can be waited on exactly; page ids travel through scalar
// loads, whose counter is separate.
//
// Softmax.  The reference max of a segment is fixed once, from its first tile, and never
// moved: softmax is shift-invariant, and weights above 1 are as exact in bf16 / fp32 as
// weights below 1, so the inner loop has no running max, no rescaling and no cross-lane step.
// Row sums come from the matrix core (a ones fragment times P^T).  Should the first tile have
// been so unrepresentative that a denominator overflows, the segment is redone with the exact
// max, found by a K-only pass.
//
// Pointwise mode (template flag PW).  The same schedule, operand flow and pipeline serve the
// pointwise aggregation out = inv_norm * sum_j silu(c * q.k_j) v_j: the weights need no
// statistics at all, so there is no reference max, no denominator and no redo; hidden keys
// get logit 0 (silu(0) = 0); cut pairs are finished by adding their pieces.
//
// Unappended mode (template flag FRESH).  The step's own K/V rows are taken from k_new / v_new
// ([token][H][D], the layout the projection writes) instead of the pool, so the call does not
// depend on the layer's append (Sec. 2: the context is the cached prefix followed by the new
// rows) and the append can happen later, for all layers at once.  A (query tile, head) is then
// the tiles of the prefix followed by tiles of new rows, tiled from the first new token; for
// the latter a K fragment is still one 16-byte load per lane (from the token's row), a V^T
// fragment is gathered element by element.
#include <math.h>

#include <type_traits>

#include "mts_internal.hpp"



namespace mts {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

constexpr int kTile = 32;       // kv tokens per step (two 16-token sub-blocks)
constexpr int kWavesPerWg = 4;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
// x * sigmoid(x); -inf never reaches it (hidden keys carry logit 0 in pointwise mode)
__device__ __forceinline__ float fast_silu(float x) {
  return x * __builtin_amdgcn_rcpf(1.0f + fast_exp2(-1.4426950408889634f * x));
}

// max over the 4 lanes that hold the same query (lane, lane^16, lane^32, lane^48)
__device__ __forceinline__ float quad_row_max(float v) {
  unsigned u = __float_as_uint(v);
  auto a = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  v = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  u = __float_as_uint(v);
  auto b = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
// share of wavefront w: [lo, hi) in global tile positions
__device__ __forceinline__ int tiles_per_wave(int total, int num_waves, int min_tiles) {
  const int per = (total + num_waves - 1) / num_waves;
  return per < min_tiles ? min_tiles : per;
}
__device__ __forceinline__ void wave_share(int total, int num_waves, int min_tiles, int w, int* lo, int* hi) {
  const int per = tiles_per_wave(total, num_waves, min_tiles);
  const long long l = (long long)w * per;
  *lo = l < total ? (int)l : total;
  *hi = (l + per) < total ? (int)(l + per) : total;
}

// Histories that are still in the contiguous onload buffer (Sec. 4.1: the buffer doubles as an
// inference area).  User u's prefix is runs first_run[u], first_run[u] + 1, ... of `chunk` tokens
// each (the last one shorter), run s holding [2][n_s][H][D] at element run_tok[s] * 2 * H * D of
// `rows`; first_run[u] < 0: the user's prefix is in the pool.  first_run == nullptr: nobody's is.
struct StagedRuns {
  const uint16_t* rows;
  const int32_t*  first_run;
  const int64_t*  run_tok;
  int32_t         chunk;       // tokens per run, a multiple of 32
};

// What the merge kernel needs to finish one (query tile, head) cut by share boundaries;
// written by the wavefront that holds the pair's first tile.
struct MergeDesc {
  int valid;       // 1: this wavefront starts a cut pair
  int w_last;      // last wavefront that holds a piece of it
  int out_row;     // (token row of the tile's first query) * H + head
  int nq;          // queries in the tile
  int first_slot;  // partial slot of this wavefront's piece (0 leading, 1 trailing)
  int pad[3];
};

// WPS = wavefronts per SIMD the kernel is compiled for (bounds its registers)
// SRC = where keys and values come from: 0 the pool; 1 the step's own rows from k_new / v_new
// (unappended); 2 also the prefixes of the users `staged` names, from the onload buffer
template <int D, int NQB, int PF, int WPS, bool PW, int SRC>
__global__ __launch_bounds__(256, WPS) void attn_stream_kernel(PoolGeom g, BatchDev b,
                                                          const uint16_t* __restrict__ q,
                                                          const uint16_t* __restrict__ k_new,
                                                          const uint16_t* __restrict__ v_new,
                                                          StagedRuns staged,
                                                          uint16_t* __restrict__ out, float c, float inv_norm,
                                                          int q_tiles_max, int n_items, int min_tiles, int pair_cost,
                                                          MergeDesc* __restrict__ ws_desc,
                                                          float* __restrict__ ws_o,
                                                          float* __restrict__ ws_ml) {
  constexpr bool FRESH = SRC >= 1, STAGED = SRC == 2;
  constexpr int QT = 16 * NQB;       // queries per query tile
  constexpr int KS = D / 32;         // k-steps of Q.K
  constexpr int DB = D / 16;         // 16-dim blocks of the output

  // LDS: a wavefront-private tile for the V transpose of row tiles (unappended mode), then
  // per-user metadata and the schedule's prefix sums
  constexpr int VT_PITCH = D + 8;    // elements per token row of the transpose tile
  __shared__ __attribute__((aligned(16))) uint16_t vt_tile[FRESH ? kWavesPerWg * kTile * VT_PITCH : 8];
  extern __shared__ int lds[];
  const int B = b.batch;
  int* s_tok = lds;                  // [B+1] new_indptr
  int* s_pg = s_tok + (B + 1);       // [B+1] page_indptr
  int* s_P = s_pg + (B + 1);         // [B]   prefix_lens
  int* s_cum = s_P + B;              // [n_items+1] exclusive prefix of tiles * H
  int* s_wtot = s_cum + (n_items + 1);   // [4] wavefront totals of the scan

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = uniform(tid >> 6);
  const int r = lane & 15, gq = lane >> 4;
  const int H = g.H, S = g.S;

  for (int k = tid; k <= B; k += 256) {
    s_tok[k] = b.new_indptr[k];
    s_pg[k] = b.page_indptr[k];
    if (k < B) s_P[k] = b.prefix_lens[k];
  }
  __syncthreads();

  // kv tiles visible to the last query of (user, query tile) `item`; 0 if the tile is empty
  auto item_tiles = [&](int item) -> int {
    const int u = item / q_tiles_max, q0 = (item % q_tiles_max) * QT;
    const int n_u = s_tok[u + 1] - s_tok[u];
    if (q0 >= n_u) return 0;
    const int q1 = (n_u < q0 + QT) ? n_u : (q0 + QT);
    // unappended: the cached prefix and the new rows are tiled separately (each from its own
    // first token), so that no tile mixes the two sources
    if (FRESH) return (s_P[u] + kTile - 1) / kTile + (q1 + kTile - 1) / kTile;
    return (s_P[u] + q1 + kTile - 1) / kTile;
  };

  // What a (query tile, head) costs in the schedule: its kv tiles plus an allowance, in tiles,
  // for what it costs besides streaming (Q and page-id loads, the first tiles' latency, the
  // masked tail, writing the result).  Shares are equal in this unit, so a share that holds
  // several short pairs gets fewer tiles than one inside a long pair.
  auto item_cost = [&](int item) -> int {
    const int t = item_tiles(item);
    return t > 0 ? t + pair_cost : 0;
  };
  // ---- schedule: every workgroup computes the same prefix sum --------------------------
  {
    const int per_thread = (n_items + 255) / 256;
    const int first = tid * per_thread;
    int local = 0;
    for (int k = 0; k < per_thread; ++k)
      if (first + k < n_items) local += item_cost(first + k) * H;
    int incl = local;                                  // inclusive scan over the wavefront
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int up = __shfl_up(incl, o);
      if (lane >= o) incl += up;
    }
    if (lane == 63) s_wtot[wave] = incl;
    __syncthreads();
    int base = incl - local;
    for (int w = 0; w < wave; ++w) base += s_wtot[w];
    for (int k = 0; k < per_thread; ++k) {
      if (first + k < n_items) {
        s_cum[first + k] = base;
        base += item_cost(first + k) * H;
      }
    }
    if (tid == 255) s_cum[n_items] = base;
    __syncthreads();
  }
  const int total = s_cum[n_items];
  const int num_waves = gridDim.x * kWavesPerWg;
  const int wid = blockIdx.x * kWavesPerWg + wave;
  const int per_wave = tiles_per_wave(total, num_waves, min_tiles);
  int lo, hi;
  wave_share(total, num_waves, min_tiles, wid, &lo, &hi);
  if (lane == 0) ws_desc[wid].valid = 0;
  if (lo >= hi) return;                                // no barrier below this line

  const int sub_mask = (1 << g.sub_shift) - 1;
  const int64_t v_off = (int64_t)S * D * 2;            // K block -> V block of the same head
  bf16x8 ones;
#pragma unroll
  for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;

  int pos = lo;
  int item = 0;
  {
    int a = 0, e = n_items;                            // largest i with s_cum[i] <= lo
    while (e - a > 1) {
      const int mid = (a + e) >> 1;
      if (s_cum[mid] <= lo) a = mid; else e = mid;
    }
    item = a;
  }
  while (pos < hi) {
    while (s_cum[item + 1] <= pos) ++item;             // skips (user, query tile)s without work
    const int u = item / q_tiles_max;
    const int tok0 = uniform(s_tok[u]);
    const int n_u = uniform(s_tok[u + 1]) - tok0;
    const int P = uniform(s_P[u]);
    const int q0 = (item % q_tiles_max) * QT;
    const int q1 = (n_u < q0 + QT) ? n_u : (q0 + QT);
    const int nq = q1 - q0;
    const int pool_tiles = (P + kTile - 1) / kTile;    // unappended: tiles of the cached prefix
    // kv tiles of the whole (query tile, head)
    const int tiles = FRESH ? pool_tiles + (q1 + kTile - 1) / kTile : (P + q1 + kTile - 1) / kTile;
    // Positions count cost units: a pair's allowance comes first, then its tiles.
    const int item_pos = uniform(s_cum[item]);
    const int ctiles = tiles + pair_cost;
    const int h = (pos - item_pos) / ctiles;
    const int c_beg = (pos - item_pos) % ctiles;
    const int pair_end = item_pos + (h + 1) * ctiles;
    const int seg_end = pair_end < hi ? pair_end : hi;
    const int c_end = c_beg + (seg_end - pos);
    const int t_beg = c_beg > pair_cost ? c_beg - pair_cost : 0;
    const int t_end = c_end > pair_cost ? c_end - pair_cost : 0;
    if (t_end <= t_beg) {                              // only the pair's allowance lies in this share
      pos = seg_end;
      continue;
    }
    const int nqb = (nq + 15) >> 4;
    const int T_u = P + n_u;                           // tokens that hold data
    const int first_query_pos = P + q0;
    const int pbeg = uniform(s_pg[u]);
    const int npg = uniform(s_pg[u + 1]) - pbeg;
    const char* head_base = g.layer_base + (int64_t)h * 2 * S * D * 2;

    // Q^T fragments: lane (r, gq) holds query q0+16*qb+r, dims 32*s + 8*gq .. +7.
    bf16x8 qf[NQB][KS];
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
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

    f32x4 o[DB][NQB];
    f32x4 lacc[NQB];                 // softmax denominators (all 4 entries of a lane are equal)
    float m[NQB];                    // reference max of the accumulators, raw logit units
    float mcq[NQB];                  // the same reference, scaled for the base-2 exponent

    // Page ids come through scalar loads (their counter is separate from the vector-memory
    // one, so they never force a wait on K/V data in flight).  Ring slot p keeps the ids of
    // the NEXT tile it will load, requested one ring revolution earlier.
    // Unappended mode: the ring serves the tiles of the cached prefix, [t_beg, ring_end); the
    // tiles of new rows, [fresh_beg, t_end), follow one at a time.
    int ring_end = t_end;
    if (FRESH && pool_tiles < ring_end) ring_end = pool_tiles > t_beg ? pool_tiles : t_beg;
    const int fresh_beg = FRESH ? ring_end : t_end;
    // Which keys a query may see, as variables because the two kinds of tiles differ: a key at
    // position kp is hidden from query block qb's lane r if kp > mask_q0 + mask_qstep * (16 qb + r);
    // V slots at or past valid_end may hold anything and are cleared.  Tiles of the prefix in
    // unappended mode: every query sees exactly the positions below P.
    int mask_q0 = FRESH ? P - 1 : first_query_pos, mask_qstep = FRESH ? 0 : 1, valid_end = FRESH ? P : T_u;
    const int last_tile = ring_end - 1;
    int idr0[PF], idr1[PF];
    auto page_ids_at = [&](int tl, int& id0, int& id1) __attribute__((always_inline)) {
      int lp0 = (tl * 2) >> g.sub_shift, lp1 = (tl * 2 + 1) >> g.sub_shift;
      if (lp1 >= npg) lp1 = lp0;                                 // no second page at the tail
      if (lp0 >= npg) lp0 = lp1 = 0;                             // metadata out of range: stay in bounds
      id0 = npg > 0 ? b.page_indices[pbeg + lp0] : 0;
      id1 = npg > 0 ? b.page_indices[pbeg + lp1] : 0;
    };
    auto tile_bases_at = [&](int tl, int id0, int id1, const char*& kb0, const char*& kb1) __attribute__((always_inline)) {
      const int sb0 = tl * 2, sb1 = sb0 + 1;
      if ((unsigned)id0 >= (unsigned)g.num_pages) id0 = 0;
      if ((unsigned)id1 >= (unsigned)g.num_pages) id1 = 0;
      kb0 = head_base + (int64_t)id0 * g.page_bytes + (int64_t)(sb0 & sub_mask) * 16 * D * 2;
      kb1 = head_base + (int64_t)id1 * g.page_bytes + (int64_t)(sb1 & sub_mask) * 16 * D * 2;
    };
    // the ring's versions: past its end, repeat its last tile
    auto page_ids = [&](int tile, int& id0, int& id1) __attribute__((always_inline)) {
      page_ids_at(tile < last_tile ? tile : last_tile, id0, id1);
    };
    auto tile_bases = [&](int tile, int id0, int id1, const char*& kb0, const char*& kb1) __attribute__((always_inline)) {
      tile_bases_at(tile < last_tile ? tile : last_tile, id0, id1, kb0, kb1);
    };

    bf16x8 kf[PF][2][KS];
    bf16x8 vf[PF][DB];
    // Loads tile `tile` (clamped to the segment's last tile, so that the loads of the steady
    // state are unconditional and the hardware's in-order load counter can be waited on
    // exactly) into ring slot p, then requests the ids of the tile this slot loads next.
    auto issue = [&](auto buf, int tile) __attribute__((always_inline)) {            // buf is an integral_constant: register ring slot
      constexpr int p = decltype(buf)::value;
      const char *kb0, *kb1;
      tile_bases(tile, idr0[p], idr1[p], kb0, kb1);
      // K fragments: rows 0-7 of a half-tile come from sub-block 0, rows 8-15 from sub-block 1.
      const char* kl = ((r < 8) ? kb0 : kb1) + (r & 7) * 16;
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int s = 0; s < KS; ++s)
          kf[p][hf][s] = *reinterpret_cast<const bf16x8*>(kl + ((hf * (D / 8) + 4 * s + gq) * 8) * 16);
      // V^T fragments: lane (r, gq) holds dim 16*db + r, tokens 8*gq .. +7 of the tile.
      const char* vl = ((gq < 2) ? kb0 : kb1) + v_off + (r * 16 + (gq & 1) * 8) * 2;
#pragma unroll
      for (int db = 0; db < DB; ++db)
        vf[p][db] = *reinterpret_cast<const bf16x8*>(vl + db * 16 * 16 * 2);
      page_ids(tile + PF, idr0[p], idr1[p]);
    };
    // ---- unappended mode: tiles of new rows ----------------------------------------------
    // Tile ft holds the user's new tokens 32 ft .. 32 ft + 31 (positions P + ...), read from
    // k_new / v_new through buffer descriptors that span exactly the user's rows of this head:
    // tokens past the last one read as 0 without a branch.  A K fragment is one 16-byte load per
    // lane (8 dims of the token's row), a V^T fragment one element from each of 8 rows.  All
    // loads of a tile are in flight together; the ring has drained by then, so its registers
    // are free.
    const int row_bytes = H * D * 2;
    auto row_source = [&](const uint16_t* first_row, int rows) __attribute__((always_inline)) {
      return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(first_row), 0, (rows - 1) * row_bytes + D * 2,
                                               0x00020000);
    };
    __amdgpu_buffer_rsrc_t k_rows, v_rows;             // the user's new rows of this head
    int first_run = -1;                                // >= 0: the prefix is read from the onload buffer
    if constexpr (FRESH) {
      const int64_t first = ((int64_t)tok0 * H + h) * D;
      k_rows = row_source(k_new + first, n_u);
      v_rows = row_source(v_new + first, n_u);
      if constexpr (STAGED) first_run = uniform(staged.first_run[u]);
    }
    // the pool's slot order: token of the K row this lane holds in half-tile 0 (half-tile 1: + 4)
    const int k_lane_pos = ((r >> 3) << 4) + (((r & 7) >> 2) << 3) + (r & 3);
    // Loads the 32 rows from `row_first` on of a row source as one tile into ring slot p.
    auto load_rows_k = [&](auto buf, __amdgpu_buffer_rsrc_t ks, int row_first) __attribute__((always_inline)) {
      constexpr int p = decltype(buf)::value;
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        int koff = (row_first + k_lane_pos + 4 * hf) * row_bytes + 8 * gq * 2;
        asm volatile("" : "+v"(koff));                 // computed here, not kept in a register across the ring
#pragma unroll
        for (int s = 0; s < KS; ++s)
          kf[p][hf][s] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(ks, koff + 32 * s * 2, 0, 0));
      }
    };
    // V rows arrive as they lie in memory, 16 bytes (8 dims of one token) per lane and load:
    // load j of lane l holds token (64 j + l) / (D/8), dims 8 * ((64 j + l) % (D/8)) .. + 7.
    // finish_rows() turns them into V^T fragments before the tile is used.
    auto load_rows = [&](auto buf, __amdgpu_buffer_rsrc_t ks, __amdgpu_buffer_rsrc_t vs, int row_first)
        __attribute__((always_inline)) {
      constexpr int p = decltype(buf)::value;
      load_rows_k(buf, ks, row_first);
      int voff = (row_first + lane / (D / 8)) * row_bytes + (lane % (D / 8)) * 16;
      asm volatile("" : "+v"(voff));
#pragma unroll
      for (int j = 0; j < DB; ++j)
        vf[p][j] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(vs, voff + j * (64 / (D / 8)) * row_bytes, 0, 0));
    };
    // The transpose of slot p's V rows through the wavefront's LDS tile: rows in, [dim][8 tokens]
    // fragments out.  Token row t keeps its 16-byte chunks rotated by t / 8, so that the four
    // lane groups of a fragment read (rows 8 apart) fall on different banks.
    auto finish_rows = [&](auto buf) __attribute__((always_inline)) {
      constexpr int p = decltype(buf)::value;
      constexpr int NCH = D / 8;
      uint16_t* lt = vt_tile + wave * (kTile * VT_PITCH);
#pragma unroll
      for (int j = 0; j < DB; ++j) {
        const int t = j * (64 / NCH) + lane / NCH, ch = lane % NCH;
        *reinterpret_cast<u32x4*>(lt + t * VT_PITCH + ((ch + (t >> 3)) % NCH) * 8) = __builtin_bit_cast(u32x4, vf[p][j]);
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const int dim = 16 * db + r;
        const uint16_t* col = lt + (8 * gq) * VT_PITCH + (((dim >> 3) + gq) % NCH) * 8 + (dim & 7);
        uint32_t f[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = col[e * VT_PITCH];
        u32x4 v;
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = f[2 * j] | (f[2 * j + 1] << 16);
        vf[p][db] = __builtin_bit_cast(bf16x8, v);
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
    };
    // Tile `tile` of a prefix that lies in the onload buffer: the run that holds it (tiles never
    // straddle runs: the run length is a multiple of 32) is its own row source, K plane then V
    // plane, so rows past the run's (and with the last run, the prefix's) end read as 0.
    auto staged_sources = [&](int tile, __amdgpu_buffer_rsrc_t& ks, __amdgpu_buffer_rsrc_t& vs, int& row_first)
        __attribute__((always_inline)) {
      const int run = (tile * kTile) / staged.chunk;
      const int64_t a = staged.run_tok[first_run + run], e = staged.run_tok[first_run + run + 1];
      const int rows = (int)(e - a);
      const uint16_t* kp = staged.rows + a * 2 * H * D + (int64_t)h * D;
      ks = row_source(kp, rows);
      vs = row_source(kp + (int64_t)rows * H * D, rows);
      row_first = tile * kTile - run * staged.chunk;
    };

    // S^T of query block qb against the K fragments of ring slot p.  The lane holds, for query
    // q0+16*qb+r, keys tb + 8*gq + {0..3} (s0) and {4..7} (s1); with `masked`, keys the query
    // must not see (causal order among the new tokens) are set to -inf.
    auto scores = [&](auto buf, int qb, int tb, bool masked, f32x4& s0, f32x4& s1) __attribute__((always_inline)) {
      constexpr int p = decltype(buf)::value;
      s0 = f32x4{0.f, 0.f, 0.f, 0.f};
      s1 = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[p][0][s], qf[qb][s], s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[p][1][s], qf[qb][s], s1, 0, 0, 0);
      }
      if (masked) {
        const int qpos = mask_q0 + mask_qstep * (16 * qb + r);
        const int kbase = tb + 8 * gq;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (kbase + e > qpos) s0[e] = PW ? 0.f : -INFINITY;
          if (kbase + 4 + e > qpos) s1[e] = PW ? 0.f : -INFINITY;
        }
      }
    };
    auto max8 = [](const f32x4& s0, const f32x4& s1) {
      return fmaxf(fmaxf(fmaxf(s0[0], s0[1]), fmaxf(s0[2], s0[3])),
                   fmaxf(fmaxf(s1[0], s1[1]), fmaxf(s1[2], s1[3])));
    };

    // One tile against NQ query blocks (NQ a compile-time constant: no branch between the
    // blocks).  The reference max is fixed for the whole segment, so nothing is ever rescaled:
    // softmax is shift-invariant, and weights above 1 are as exact in bf16 / fp32 as weights
    // below 1.  TAIL adds what only the causal tail needs: the mask, and zeroing of V slots past
    // the user's last token (they may hold anything).
    auto tile_step = [&](auto nq_c, auto tail_c, auto buf, int tb) __attribute__((always_inline)) {
      constexpr int NQ = decltype(nq_c)::value;
      constexpr bool TAIL = decltype(tail_c)::value;
      constexpr int p = decltype(buf)::value;      // tb: position of the tile's first token
      bool masked = false;
      if constexpr (TAIL) {
        masked = (tb + kTile - 1 > mask_q0);             // some key hidden from some query
        if (masked && tb + kTile > valid_end) {
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int e = 0; e < 8; ++e)
              if (tb + 8 * gq + e >= valid_end) vf[p][db][e] = (__bf16)0.0f;
        }
      }
#pragma unroll
      for (int qb = 0; qb < NQ; ++qb) {
        f32x4 s0, s1;
        scores(buf, qb, tb, masked, s0, s1);
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
          o[db][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[p][db], pf, o[db][qb], 0, 0, 0);
        // row sums of the (rounded) weights on the matrix core: every row of ones . P^T
        if constexpr (!PW) lacc[qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pf, lacc[qb], 0, 0, 0);
      }
    };

    // Exact running max of every query over the whole segment (K only, no pipelining): used
    // when the first tile's max turned out to be too low a reference.
    auto exact_max = [&](auto nq_c) __attribute__((always_inline)) {
      constexpr int NQ = decltype(nq_c)::value;
      float mx[NQ];
#pragma unroll
      for (int qb = 0; qb < NQ; ++qb) mx[qb] = -INFINITY;
      if constexpr (FRESH) { mask_q0 = P - 1; mask_qstep = 0; }
      for (int tile = t_beg; tile < ring_end; ++tile) {
        const int tb = tile * kTile;
        if (STAGED && first_run >= 0) {
          if constexpr (STAGED) {
            __amdgpu_buffer_rsrc_t ks, vs;
            int row_first;
            staged_sources(tile, ks, vs, row_first);
            load_rows_k(std::integral_constant<int, 0>{}, ks, row_first);
          }
        } else {
          int id0, id1;
          page_ids_at(tile, id0, id1);
          const char *kb0, *kb1;
          tile_bases_at(tile, id0, id1, kb0, kb1);
          const char* kl = ((r < 8) ? kb0 : kb1) + (r & 7) * 16;
#pragma unroll
          for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int s = 0; s < KS; ++s)
              kf[0][hf][s] = *reinterpret_cast<const bf16x8*>(kl + ((hf * (D / 8) + 4 * s + gq) * 8) * 16);
        }
#pragma unroll
        for (int qb = 0; qb < NQ; ++qb) {
          f32x4 s0, s1;
          scores(std::integral_constant<int, 0>{}, qb, tb, tb + kTile - 1 > mask_q0, s0, s1);
          mx[qb] = fmaxf(mx[qb], max8(s0, s1));
        }
      }
      if constexpr (FRESH) {
        mask_q0 = first_query_pos; mask_qstep = 1;
        for (int tile = fresh_beg; tile < t_end; ++tile) {
          const int tb = P + (tile - pool_tiles) * kTile;
          load_rows_k(std::integral_constant<int, 0>{}, k_rows, (tile - pool_tiles) * kTile);
#pragma unroll
          for (int qb = 0; qb < NQ; ++qb) {
            f32x4 s0, s1;
            scores(std::integral_constant<int, 0>{}, qb, tb, tb + kTile - 1 > mask_q0, s0, s1);
            mx[qb] = fmaxf(mx[qb], max8(s0, s1));
          }
        }
      }
#pragma unroll
      for (int qb = 0; qb < NQ; ++qb) {
        m[qb] = quad_row_max(mx[qb]);
        mcq[qb] = (m[qb] == -INFINITY ? 0.f : m[qb]) * c;
      }
    };

    // tiles [0, fast_stop) hide no key from any query of this tile
    int fast_stop = FRESH ? P / kTile : (first_query_pos + 1) / kTile;
    if (fast_stop > ring_end) fast_stop = ring_end;

    // The whole segment for NQ query blocks.  Ring slots are integral_constants so that every
    // register array is indexed by constants only; tile t lives in slot (t - t_beg) % PF.
    auto run_segment = [&](auto nq_c) __attribute__((always_inline)) {
      constexpr int NQ = decltype(nq_c)::value;
      constexpr std::false_type body{};
      constexpr std::true_type tail{};
      // reference max = max of the segment's first tile (in ring slot 0 when this is called)
      auto reference_from_slot0 = [&](int tb) __attribute__((always_inline)) {
#pragma unroll
        for (int qb = 0; qb < NQ; ++qb) {
          f32x4 s0, s1;
          scores(std::integral_constant<int, 0>{}, qb, tb, tb + kTile - 1 > mask_q0, s0, s1);
          m[qb] = quad_row_max(max8(s0, s1));
          mcq[qb] = (m[qb] == -INFINITY ? 0.f : m[qb]) * c;    // nothing visible: any reference
        }
      };
      for (int attempt = 0; attempt < 2; ++attempt) {
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) {
          lacc[qb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int db = 0; db < DB; ++db) o[db][qb] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        if constexpr (!PW) {
          if (attempt == 1) exact_max(nq_c);
        }

        if constexpr (FRESH) { mask_q0 = P - 1; mask_qstep = 0; valid_end = P; }
        if (STAGED && first_run >= 0) {
          // the prefix lies in the onload buffer: its tiles come through the row loader, two ring
          // slots in turn so that one tile's loads are in flight while the other is consumed (the
          // loads are unconditional, clamped to the last tile, as in the ring)
          if constexpr (STAGED) {
            static_assert(PF >= 2, "two ring slots");
            auto load_staged = [&](auto buf, int tile) __attribute__((always_inline)) {
              __amdgpu_buffer_rsrc_t ks, vs;
              int row_first;
              staged_sources(tile < ring_end - 1 ? tile : ring_end - 1, ks, vs, row_first);
              load_rows(buf, ks, vs, row_first);
            };
            if (t_beg < ring_end) {
              load_staged(std::integral_constant<int, 0>{}, t_beg);
              for (int tile = t_beg; tile < ring_end; tile += 2) {
                load_staged(std::integral_constant<int, 1>{}, tile + 1);
                if (!PW && attempt == 0 && tile == t_beg) reference_from_slot0(tile * kTile);
                finish_rows(std::integral_constant<int, 0>{});
                tile_step(nq_c, tail, std::integral_constant<int, 0>{}, tile * kTile);
                load_staged(std::integral_constant<int, 0>{}, tile + 2);
                finish_rows(std::integral_constant<int, 1>{});
                if (tile + 1 < ring_end) tile_step(nq_c, tail, std::integral_constant<int, 1>{}, (tile + 1) * kTile);
              }
            }
          }
        } else if (!FRESH || ring_end > t_beg) {
          page_ids(t_beg, idr0[0], idr1[0]);
          if constexpr (PF > 1) page_ids(t_beg + 1, idr0[1], idr1[1]);
          if constexpr (PF > 2) page_ids(t_beg + 2, idr0[2], idr1[2]);
          if constexpr (PF > 3) page_ids(t_beg + 3, idr0[3], idr1[3]);
          issue(std::integral_constant<int, 0>{}, t_beg);
          if constexpr (PF > 1) issue(std::integral_constant<int, 1>{}, t_beg + 1);
          if constexpr (PF > 2) issue(std::integral_constant<int, 2>{}, t_beg + 2);
          if constexpr (PF > 3) issue(std::integral_constant<int, 3>{}, t_beg + 3);

          if (!PW && attempt == 0) reference_from_slot0(t_beg * kTile);

          int tile = t_beg;
          while (tile + PF <= fast_stop) {                 // steady state: fully visible tiles
            tile_step(nq_c, body, std::integral_constant<int, 0>{}, (tile) * kTile);
            issue(std::integral_constant<int, 0>{}, tile + PF);
            if constexpr (PF > 1) {
              tile_step(nq_c, body, std::integral_constant<int, 1>{}, (tile + 1) * kTile);
              issue(std::integral_constant<int, 1>{}, tile + 1 + PF);
            }
            if constexpr (PF > 2) {
              tile_step(nq_c, body, std::integral_constant<int, 2>{}, (tile + 2) * kTile);
              issue(std::integral_constant<int, 2>{}, tile + 2 + PF);
            }
            if constexpr (PF > 3) {
              tile_step(nq_c, body, std::integral_constant<int, 3>{}, (tile + 3) * kTile);
              issue(std::integral_constant<int, 3>{}, tile + 3 + PF);
            }
            tile += PF;
          }
          for (; tile < ring_end; tile += PF) {            // causal tail, and what is left over
            tile_step(nq_c, tail, std::integral_constant<int, 0>{}, (tile) * kTile);
            issue(std::integral_constant<int, 0>{}, tile + PF);
            if constexpr (PF > 1) {
              if (tile + 1 < ring_end) tile_step(nq_c, tail, std::integral_constant<int, 1>{}, (tile + 1) * kTile);
              issue(std::integral_constant<int, 1>{}, tile + 1 + PF);
            }
            if constexpr (PF > 2) {
              if (tile + 2 < ring_end) tile_step(nq_c, tail, std::integral_constant<int, 2>{}, (tile + 2) * kTile);
              issue(std::integral_constant<int, 2>{}, tile + 2 + PF);
            }
            if constexpr (PF > 3) {
              if (tile + 3 < ring_end) tile_step(nq_c, tail, std::integral_constant<int, 3>{}, (tile + 3) * kTile);
              issue(std::integral_constant<int, 3>{}, tile + 3 + PF);
            }
          }
        }
        if constexpr (FRESH) {
          mask_q0 = first_query_pos; mask_qstep = 1; valid_end = T_u;
          for (int tile = fresh_beg; tile < t_end; ++tile) {      // the tiles of new rows
            const int ft = tile - pool_tiles;
            load_rows(std::integral_constant<int, 0>{}, k_rows, v_rows, ft * kTile);
            if (!PW && attempt == 0 && tile == t_beg) reference_from_slot0(P + ft * kTile);
            finish_rows(std::integral_constant<int, 0>{});
            tile_step(nq_c, tail, std::integral_constant<int, 0>{}, P + ft * kTile);
          }
        }

        // A reference far below the true max shows up as an overflowed (or NaN) denominator.
        if constexpr (PW) break;                         // no statistics, nothing to redo
        bool bad = false;
#pragma unroll
        for (int qb = 0; qb < NQ; ++qb) bad |= !(lacc[qb][0] < 1e37f);
        if (__builtin_amdgcn_ballot_w64(bad) == 0) break;
      }
    };
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) { m[qb] = -INFINITY; mcq[qb] = 0.f; }
    switch (nqb) {
      case 1: run_segment(std::integral_constant<int, 1>{}); break;
      case 2: if constexpr (NQB >= 2) run_segment(std::integral_constant<int, 2>{}); break;
      case 3: if constexpr (NQB >= 3) run_segment(std::integral_constant<int, 3>{}); break;
      default: if constexpr (NQB >= 4) run_segment(std::integral_constant<int, 4>{}); break;
    }

    // ---- finish the segment ----
    float l[NQB];
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) l[qb] = lacc[qb][0];
    const bool complete = (t_beg == 0) && (t_end == tiles);
    const int out_row = (tok0 + q0) * H + h;           // row of query 0, in [token * H + head] units
    if (complete) {
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        const int qi = 16 * qb + r;
        if (qi < nq) {
          const float inv = PW ? inv_norm : 1.0f / l[qb];
          uint16_t* orow = out + ((int64_t)out_row + (int64_t)qi * H) * D + 4 * gq;
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            bf16x4 ob;
#pragma unroll
            for (int k = 0; k < 4; ++k) ob[k] = (__bf16)(o[db][qb][k] * inv);
            *reinterpret_cast<bf16x4*>(orow + 16 * db) = ob;
          }
        }
      }
    } else {
      const int slot = (pos == lo) ? 0 : 1;            // leading or trailing piece of this share
      const int64_t prow = ((int64_t)wid * 2 + slot) * QT;
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        const int qi = 16 * qb + r;
        if (qi < nq) {
          float* po = ws_o + (prow + qi) * D + 4 * gq;
#pragma unroll
          for (int db = 0; db < DB; ++db) *reinterpret_cast<f32x4*>(po + 16 * db) = o[db][qb];
          if (!PW && gq == 0) {
            ws_ml[(prow + qi) * 2] = m[qb];
            ws_ml[(prow + qi) * 2 + 1] = l[qb];
          }
        }
      }
      if (t_beg == 0 && lane == 0) {
        // this share holds the pair's first tile: it owns the merge of all the pieces
        MergeDesc d;
        d.valid = 1;
        d.w_last = (pair_end - 1) / per_wave;
        d.out_row = out_row;
        d.nq = nq;
        d.first_slot = slot;
        d.pad[0] = d.pad[1] = d.pad[2] = 0;
        ws_desc[wid] = d;
      }
    }
    pos = seg_end;
  }
}

// Finishes the (query tile, head)s that a share boundary cut.  Workgroup w serves the pair
// whose first tile lies in share w (if that pair continues into later shares): a numerically
// safe weighted sum of the pieces, in share order.  Share w holds its piece in slot
// `first_slot`; every later share holds its piece as the leading one (slot 0).
template <int D, bool PW>
__global__ __launch_bounds__(256) void attn_merge_kernel(uint16_t* __restrict__ out, float c, float inv_norm, int q_tile,
                                                         int H, const MergeDesc* __restrict__ ws_desc,
                                                         const float* __restrict__ ws_o,
                                                         const float* __restrict__ ws_ml) {
  // One thread per (query, 4 dims); pieces are taken four at a time with all their loads issued
  // together, and folded into a running (max, numerator, denominator) - in share order.
  const int w = blockIdx.x;
  const MergeDesc d = ws_desc[w];
  constexpr int D4 = D / 4;
  const int e = blockIdx.y * 256 + threadIdx.x;
  if (!d.valid || e >= d.nq * D4) return;
  const int qi = e / D4, d4 = e % D4;
  float M = -INFINITY, den = 0.f;
  f32x4 num = {0.f, 0.f, 0.f, 0.f};
  for (int w0 = w; w0 <= d.w_last; w0 += 4) {
    float pm[4], pl[4];
    f32x4 po[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int ww = (w0 + k <= d.w_last) ? (w0 + k) : d.w_last;      // past the end: repeat, weight 0
      const int slot = (ww == w) ? d.first_slot : 0;
      const int64_t prow = ((int64_t)ww * 2 + slot) * q_tile + qi;
      pm[k] = PW ? 0.f : ws_ml[prow * 2];
      pl[k] = PW ? 0.f : ws_ml[prow * 2 + 1];
      po[k] = *reinterpret_cast<const f32x4*>(ws_o + prow * D + 4 * d4);
    }
    float Mn = M;
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (w0 + k <= d.w_last) Mn = fmaxf(Mn, pm[k]);
    const float mref = (Mn == -INFINITY) ? 0.f : Mn;
    const float rescale = fast_exp2((M - mref) * c);                   // 0 while nothing was folded in
    num *= rescale;
    den *= rescale;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (w0 + k <= d.w_last) {
        const float wgt = fast_exp2((pm[k] - mref) * c);               // a piece with no visible key has max -inf
        num += po[k] * wgt;
        den = fmaf(wgt, pl[k], den);
      }
    }
    M = Mn;
  }
  // pointwise: every piece has reference 0, so the weights above are all 1 and num is the plain sum
  const float inv = PW ? inv_norm : 1.0f / den;
  bf16x4 ob;
#pragma unroll
  for (int k = 0; k < 4; ++k) ob[k] = (__bf16)(num[k] * inv);
  *reinterpret_cast<bf16x4*>(out + ((int64_t)d.out_row + (int64_t)qi * H) * D + 4 * d4) = ob;
}

template <int D, int NQB, int PF, int WPS, bool PW, int SRC>
hipError_t launch_one(const PoolGeom& g, const AttnPlan& plan, const uint16_t* q, const uint16_t* k_new,
                      const uint16_t* v_new, const StagedRuns& staged, uint16_t* out, const BatchDev& b, float c,
                      float inv_norm, void* workspace, hipStream_t stream) {
  auto kern = attn_stream_kernel<D, NQB, PF, WPS, PW, SRC>;
  const size_t lds_bytes = sizeof(int) * ((size_t)3 * b.batch + 2 + plan.n_items + 1 + kWavesPerWg);
  static int wgs_per_cu = 0, num_cus = 0;              // per instantiation; same value from any thread
  // static LDS of the kernel: the V transpose tiles of the unappended forms
  constexpr size_t static_lds = SRC >= 1 ? (size_t)kWavesPerWg * kTile * (D + 8) * 2 : 64;
  static size_t lds_limit = 60 * 1024 - static_lds;
  if (wgs_per_cu == 0) {
    int dev = 0, n = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kern, 256, 16 * 1024);
    if (e != hipSuccess) return e;
    num_cus = cus > 0 ? cus : 256;
    wgs_per_cu = n < 1 ? 1 : (n > 2 ? 2 : n);
  }
  if (lds_bytes > lds_limit) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return e;
    lds_limit = lds_bytes;
  }
  int wgs = num_cus * wgs_per_cu;
  if (wgs * kWavesPerWg > plan.max_waves) wgs = plan.max_waves / kWavesPerWg;
  if (wgs < 1) wgs = 1;
  char* ws = static_cast<char*>(workspace);
  MergeDesc* ws_desc = reinterpret_cast<MergeDesc*>(ws);
  float* ws_o = reinterpret_cast<float*>(ws + plan.ws_desc_bytes);
  float* ws_ml = ws_o + (int64_t)plan.max_waves * 2 * plan.q_tile * g.D;
  hipLaunchKernelGGL(kern, dim3(wgs), dim3(256), lds_bytes, stream, g, b, q, k_new, v_new, staged, out, c, inv_norm, plan.q_tiles_max,
                     plan.n_items, plan.min_tiles, plan.pair_cost, ws_desc, ws_o, ws_ml);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((attn_merge_kernel<D, PW>), dim3(wgs * kWavesPerWg, (plan.q_tile * (D / 4) + 255) / 256), dim3(256),
                     0, stream, out, c, inv_norm, plan.q_tile, g.H, ws_desc, ws_o, ws_ml);
  return hipGetLastError();
}

// Launch shapes.  One wavefront per SIMD in every shape (the planner caps the launch at 1024
// wavefronts).  D <= 64: two tiles in flight, compiled to at most 256 registers - the same code
// compiled for 512 registers, or with a ring of 3 or 4 tiles, measured 0-3 % slower.  D = 128:
// a ring of 3 tiles up to 32 queries per tile, else 2.
template <int D, bool PW, int SRC>
hipError_t launch_d(const PoolGeom& g, const AttnPlan& plan, const uint16_t* q, const uint16_t* k_new,
                    const uint16_t* v_new, const StagedRuns& staged, uint16_t* out, const BatchDev& b, float c,
                    float inv_norm, void* ws, hipStream_t stream) {
#ifndef MTS_PF_A
#define MTS_PF_A 2   // D <= 64
#define MTS_PF_B 3   // D = 128, up to 32 queries per tile
#define MTS_PF_C 2   // D = 128, 48 or 64 queries per tile
#define MTS_WPS_A 2  // D <= 64
#endif
  constexpr int PF_SMALL = (D == 128) ? MTS_PF_B : MTS_PF_A;
  constexpr int PF_LARGE = (D == 128) ? MTS_PF_C : MTS_PF_A;
  // the kernels that also read the onload buffer keep two row tiles in flight beside everything
  // else: compiled for one wavefront per SIMD (which is what runs), they need no spills
  constexpr int WPS = (D == 128 || SRC == 2) ? 1 : MTS_WPS_A;
  switch (plan.q_tile / 16) {
    case 1: return launch_one<D, 1, PF_SMALL, WPS, PW, SRC>(g, plan, q, k_new, v_new, staged, out, b, c, inv_norm, ws, stream);
    case 2: return launch_one<D, 2, PF_SMALL, WPS, PW, SRC>(g, plan, q, k_new, v_new, staged, out, b, c, inv_norm, ws, stream);
    case 3: return launch_one<D, 3, PF_LARGE, WPS, PW, SRC>(g, plan, q, k_new, v_new, staged, out, b, c, inv_norm, ws, stream);
    default: return launch_one<D, 4, PF_LARGE, WPS, PW, SRC>(g, plan, q, k_new, v_new, staged, out, b, c, inv_norm, ws, stream);
  }
}

}  // namespace

hipError_t launch_attn_mfma(const PoolGeom& g, const AttnPlan& plan, const void* q, void* out,
                            const BatchDev& b, float sm_scale, float inv_norm, void* workspace,
                            hipStream_t stream, const void* k_new, const void* v_new, const StagedHistories* hist) {
  if (b.total_new <= 0 || b.batch <= 0) return hipSuccess;
  const bool pw = inv_norm > 0.f;
  // pointwise: the scale stays in natural units; softmax: logits are exponentiated in base 2
  const float c = pw ? sm_scale : sm_scale * 1.4426950408889634f;
  const uint16_t* qp = reinterpret_cast<const uint16_t*>(q);
  const uint16_t* kp = reinterpret_cast<const uint16_t*>(k_new);
  const uint16_t* vp = reinterpret_cast<const uint16_t*>(v_new);
  uint16_t* op = reinterpret_cast<uint16_t*>(out);
  const bool fresh = kp != nullptr;
  StagedRuns staged{nullptr, nullptr, nullptr, 32};
  if (fresh && hist != nullptr)
    staged = StagedRuns{reinterpret_cast<const uint16_t*>(hist->rows), hist->first_run, hist->run_tok, hist->chunk};
#define MTS_ATTN_CASE(D_)                                                                                       \
  case D_:                                                                                                      \
    if (pw) return fresh ? launch_d<D_, true, 1>(g, plan, qp, kp, vp, staged, op, b, c, inv_norm, workspace, stream)   \
                         : launch_d<D_, true, 0>(g, plan, qp, kp, vp, staged, op, b, c, inv_norm, workspace, stream);  \
    if (staged.first_run) return launch_d<D_, false, 2>(g, plan, qp, kp, vp, staged, op, b, c, 0.f, workspace, stream); \
    return fresh ? launch_d<D_, false, 1>(g, plan, qp, kp, vp, staged, op, b, c, 0.f, workspace, stream)              \
                 : launch_d<D_, false, 0>(g, plan, qp, kp, vp, staged, op, b, c, 0.f, workspace, stream);
  switch (g.D) {
    MTS_ATTN_CASE(32)
    MTS_ATTN_CASE(64)
    MTS_ATTN_CASE(128)
    default: return hipErrorInvalidValue;
  }
#undef MTS_ATTN_CASE
}

}  // namespace mts

// Incremental-prefill attention on the matrix cores (Sec. 2, Eq. 6-7; Alg. 1 step 8.4),
// bf16 inputs, fp32 logits / softmax statistics / accumulators.
//
// Work split.  A workgroup (4 wavefronts) owns one (user, head, query tile, kv chunk): up to
// 64 of the user's new tokens against `chunk` consecutive kv tokens.  The 4 wavefronts take
// the chunk's 32-token tiles round-robin, each keeping its own running (max, sum, O), and
// combine through LDS at the end.  If the query tile has one chunk the workgroup writes the
// output rows; otherwise it writes unnormalised partials and the merge kernel finishes them
// (split-kv, so that a few long histories still fill 256 CUs, and every K/V byte is read
// from HBM exactly once).
//
// Operand flow.  Scores are computed transposed, S^T = K Q^T with v_mfma_f32_16x16x32_bf16:
// tokens are the M rows, queries the N columns, so a lane's 4 accumulator values belong to
// ONE query; softmax statistics are per-lane scalars and the row max needs two cross-lane
// steps.  With the pool's K slot order, the 8 values a lane holds after the two half-tiles
// are 8 consecutive tokens, which is exactly the B fragment of O^T = V^T P^T; V is stored
// [dim][token], so its A fragment is one 16-byte load.  Nothing is staged through LDS: each
// 16-byte global load is already an MFMA fragment, and a wavefront's loads cover whole
// 512-byte runs of a page.
#include <math.h>

#include "mts_internal.hpp"

namespace mts {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;

constexpr int kWaves = 4;
constexpr int kTile = 32;     // kv tokens per wavefront step (two 16-token sub-blocks)
constexpr int kPad = 4;       // LDS row padding, floats

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

struct TilePtrs {
  const char* sub0;   // K block base of the tile's first 16-token sub-block (this head)
  const char* sub1;   // ... second sub-block
};

template <int D, int NQB>
__global__ __launch_bounds__(256) void attn_mfma_kernel(PoolGeom g, BatchDev b,
                                                        const uint16_t* __restrict__ q,
                                                        uint16_t* __restrict__ out, float c,
                                                        int chunk, int chunks_max, int q_tiles_max,
                                                        float* __restrict__ ws_o,
                                                        float* __restrict__ ws_ml) {
  constexpr int QT = 16 * NQB;       // queries per workgroup
  constexpr int KS = D / 32;         // k-steps of Q.K
  constexpr int DB = D / 16;         // 16-dim blocks of the output
  constexpr int LD = D + kPad;       // LDS row stride, floats

  extern __shared__ float lds[];
  float* buf0 = lds;                         // [QT][LD]
  float* buf1 = lds + QT * LD;               // [QT][LD]
  float* lds_m = lds + 2 * QT * LD;          // [kWaves][QT]
  float* lds_l = lds_m + kWaves * QT;        // [2][QT]
  float* lds_M = lds_l + 2 * QT;             // [QT]

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, gq = lane >> 4;
  const int H = g.H, S = g.S;

  const int cidx = blockIdx.x % chunks_max;
  const int t = blockIdx.x / chunks_max;
  const int u = t / q_tiles_max;
  const int qt = q_tiles_max - 1 - (t % q_tiles_max);   // longest causal rows first
  const int h = blockIdx.y;

  const int tok0 = b.new_indptr[u];
  const int n_u = b.new_indptr[u + 1] - tok0;
  const int q0 = qt * QT;
  if (q0 >= n_u) return;
  const int q1 = (n_u < q0 + QT) ? n_u : (q0 + QT);
  const int nq = q1 - q0;
  const int nqb = (nq + 15) >> 4;
  const int P = b.prefix_lens[u];
  const int kv_end = P + q1;                  // keys [0, kv_end) are visible to the tile's last query
  const int T_u = P + n_u;                    // tokens that hold data
  const int nchunks = (kv_end + chunk - 1) / chunk;
  if (cidx >= nchunks) return;
  const int k0 = cidx * chunk;
  const int k1 = (kv_end < k0 + chunk) ? kv_end : (k0 + chunk);
  const int tile_beg = k0 / kTile;
  const int tile_end = (k1 + kTile - 1) / kTile;
  const int first_query_pos = P + q0;

  const int pbeg = b.page_indptr[u];
  const int npg = b.page_indptr[u + 1] - pbeg;
  const int sub_mask = (1 << g.sub_shift) - 1;
  const int64_t head_off = (int64_t)h * 2 * S * D * 2;      // bytes to this head's K block
  const int64_t v_off = (int64_t)S * D * 2;                 // K block -> V block

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
  float m[NQB], l[NQB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    m[qb] = -INFINITY;
    l[qb] = 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db) o[db][qb] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  for (int tile = tile_beg + wave; tile < tile_end; tile += kWaves) {
    const int tb = tile * kTile;
    // page-table lookup for the two sub-blocks (wave-uniform)
    const int sb0 = tile * 2, sb1 = sb0 + 1;
    int lp0 = sb0 >> g.sub_shift, lp1 = sb1 >> g.sub_shift;
    if (lp0 >= npg) break;
    if (lp1 >= npg) lp1 = lp0;
    int pg0 = b.page_indices[pbeg + lp0];
    int pg1 = b.page_indices[pbeg + lp1];
    if ((unsigned)pg0 >= (unsigned)g.num_pages) pg0 = 0;
    if ((unsigned)pg1 >= (unsigned)g.num_pages) pg1 = 0;
    const char* kb0 = g.layer_base + (int64_t)pg0 * g.page_bytes + head_off + (int64_t)(sb0 & sub_mask) * 16 * D * 2;
    const char* kb1 = g.layer_base + (int64_t)pg1 * g.page_bytes + head_off + (int64_t)(sb1 & sub_mask) * 16 * D * 2;

    // K fragments: rows 0-7 of a half-tile come from sub-block 0, rows 8-15 from sub-block 1.
    const char* kl = ((r < 8) ? kb0 : kb1) + (r & 7) * 16;
    bf16x8 kf[2][KS];
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
      for (int s = 0; s < KS; ++s)
        kf[hf][s] = *reinterpret_cast<const bf16x8*>(kl + ((hf * (D / 8) + 4 * s + gq) * 8) * 16);
    // V^T fragments: lane (r, gq) holds dim 16*db + r, tokens 8*gq .. +7 of the tile.
    const char* vl = ((gq < 2) ? kb0 : kb1) + v_off + (r * 16 + (gq & 1) * 8) * 2;
    bf16x8 vf[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
      vf[db] = *reinterpret_cast<const bf16x8*>(vl + db * 16 * 16 * 2);

    const bool masked = (tb + kTile - 1 > first_query_pos);   // some key is hidden from some query
    if (masked && tb + kTile > T_u) {
      // slots past the user's last token may hold anything: keep them out of P.V
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (tb + 8 * gq + e >= T_u) vf[db][e] = (__bf16)0.0f;
    }

#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      if (qb < nqb) {
        f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < KS; ++s) {
          s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[0][s], qf[qb][s], s0, 0, 0, 0);
          s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[1][s], qf[qb][s], s1, 0, 0, 0);
        }
        // lane holds, for query q0+16*qb+r, keys tb + 8*gq + {0..3} (s0) and {4..7} (s1)
        if (masked) {
          const int qpos = first_query_pos + 16 * qb + r;
          const int kbase = tb + 8 * gq;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            if (kbase + e > qpos) s0[e] = -INFINITY;
            if (kbase + 4 + e > qpos) s1[e] = -INFINITY;
          }
        }
        float tmax = fmaxf(fmaxf(fmaxf(s0[0], s0[1]), fmaxf(s0[2], s0[3])),
                           fmaxf(fmaxf(s1[0], s1[1]), fmaxf(s1[2], s1[3])));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float m_new = fmaxf(m[qb], tmax);
        const float mref = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = fast_exp2((m[qb] - mref) * c);
        const float mc = mref * c;
        float psum = 0.f;
        bf16x8 pf;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float p0 = fast_exp2(fmaf(s0[e], c, -mc));
          const float p1 = fast_exp2(fmaf(s1[e], c, -mc));
          psum += p0 + p1;
          pf[e] = (__bf16)p0;
          pf[4 + e] = (__bf16)p1;
        }
        l[qb] = l[qb] * alpha + psum;
        m[qb] = m_new;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          o[db][qb] *= alpha;
          o[db][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[db], pf, o[db][qb], 0, 0, 0);
        }
      }
    }
  }

  // ---- combine the 4 wavefronts (same queries, disjoint keys) ----
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    l[qb] += __shfl_xor(l[qb], 16);
    l[qb] += __shfl_xor(l[qb], 32);
    if (gq == 0) lds_m[wave * QT + 16 * qb + r] = m[qb];
  }
  __syncthreads();
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int qi = 16 * qb + r;
    float M = lds_m[qi];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) M = fmaxf(M, lds_m[w * QT + qi]);
    const float mref = (M == -INFINITY) ? 0.f : M;
    const float f = fast_exp2((m[qb] - mref) * c);      // 0 for a wavefront that saw no key
    l[qb] *= f;
#pragma unroll
    for (int db = 0; db < DB; ++db) o[db][qb] *= f;
    if (wave == 0 && gq == 0) lds_M[qi] = M;
  }
  if (wave < 2) {
    float* buf = wave ? buf1 : buf0;
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      const int qi = 16 * qb + r;
#pragma unroll
      for (int db = 0; db < DB; ++db)
        *reinterpret_cast<f32x4*>(buf + qi * LD + 16 * db + 4 * gq) = o[db][qb];
      if (gq == 0) lds_l[wave * QT + qi] = l[qb];
    }
  }
  __syncthreads();
  if (wave >= 2) {
    float* buf = (wave == 3) ? buf1 : buf0;
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      const int qi = 16 * qb + r;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        f32x4* p = reinterpret_cast<f32x4*>(buf + qi * LD + 16 * db + 4 * gq);
        *p = *p + o[db][qb];
      }
      if (gq == 0) lds_l[(wave - 2) * QT + qi] += l[qb];
    }
  }
  __syncthreads();

  // ---- write output rows (single chunk) or partials (split kv) ----
  constexpr int D4 = D / 4;
  for (int e = threadIdx.x; e < nq * D4; e += 256) {
    const int qi = e / D4, d4 = e % D4;
    const f32x4 a = *reinterpret_cast<const f32x4*>(buf0 + qi * LD + 4 * d4);
    const f32x4 bb = *reinterpret_cast<const f32x4*>(buf1 + qi * LD + 4 * d4);
    const f32x4 acc = a + bb;
    const float lsum = lds_l[qi] + lds_l[QT + qi];
    const int64_t row = (int64_t)(tok0 + q0 + qi) * H + h;
    if (nchunks == 1) {
      const float inv = 1.0f / lsum;
      bf16x4 ob;
#pragma unroll
      for (int k = 0; k < 4; ++k) ob[k] = (__bf16)(acc[k] * inv);
      *reinterpret_cast<bf16x4*>(out + row * D + 4 * d4) = ob;
    } else {
      const int64_t slot = row * chunks_max + cidx;
      *reinterpret_cast<f32x4*>(ws_o + slot * D + 4 * d4) = acc;
      if (d4 == 0) {
        ws_ml[slot * 2] = lds_M[qi];
        ws_ml[slot * 2 + 1] = lsum;
      }
    }
  }
}

// Finish the query tiles that were split over several kv chunks: a numerically safe
// weighted sum of the chunk partials, in chunk order (deterministic).
template <int D>
__global__ __launch_bounds__(D) void attn_merge_kernel(BatchDev b, int H, uint16_t* __restrict__ out,
                                                       float c, int chunk, int chunks_max, int q_tile,
                                                       const float* __restrict__ ws_o,
                                                       const float* __restrict__ ws_ml) {
  const int tok = blockIdx.x, h = blockIdx.y, d = threadIdx.x;
  int lo = 0, hi = b.batch;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (b.new_indptr[mid] <= tok) lo = mid; else hi = mid;
  }
  const int u = lo;
  const int tok0 = b.new_indptr[u];
  const int n_u = b.new_indptr[u + 1] - tok0;
  const int i = tok - tok0;
  const int q0 = (i / q_tile) * q_tile;
  const int q1 = (n_u < q0 + q_tile) ? n_u : (q0 + q_tile);
  const int kv_end = b.prefix_lens[u] + q1;
  const int nchunks = (kv_end + chunk - 1) / chunk;
  if (nchunks <= 1) return;                       // written by the attention kernel itself
  const int64_t row = (int64_t)tok * H + h;
  const float* ml = ws_ml + row * chunks_max * 2;
  float M = -INFINITY;
  for (int k = 0; k < nchunks; ++k) M = fmaxf(M, ml[2 * k]);
  float num = 0.f, den = 0.f;
  for (int k = 0; k < nchunks; ++k) {
    const float w = fast_exp2((ml[2 * k] - M) * c);   // chunks hidden from this query have max = -inf
    num = fmaf(w, ws_o[(row * chunks_max + k) * D + d], num);
    den = fmaf(w, ml[2 * k + 1], den);
  }
  const float v = num / den;
  uint32_t bits = __float_as_uint(v);
  bits += 0x7fffu + ((bits >> 16) & 1u);
  out[row * D + d] = (uint16_t)(bits >> 16);
}

template <int D, int NQB>
hipError_t launch_one(const PoolGeom& g, const AttnPlan& plan, const uint16_t* q, uint16_t* out,
                      const BatchDev& b, float c, float* ws_o, float* ws_ml, hipStream_t stream) {
  constexpr int QT = 16 * NQB;
  const size_t lds_bytes = sizeof(float) * (2 * QT * (D + kPad) + kWaves * QT + 2 * QT + QT);
  auto kern = attn_mfma_kernel<D, NQB>;
  if (lds_bytes > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return e;
  }
  const int64_t gx = (int64_t)b.batch * plan.q_tiles_max * plan.chunks_max;
  dim3 grid((unsigned)gx, (unsigned)g.H, 1), block(256, 1, 1);
  hipLaunchKernelGGL(kern, grid, block, lds_bytes, stream, g, b, q, out, c, plan.chunk,
                     plan.chunks_max, plan.q_tiles_max, ws_o, ws_ml);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || plan.chunks_max <= 1) return e;
  dim3 mgrid((unsigned)b.total_new, (unsigned)g.H, 1), mblock(D, 1, 1);
  hipLaunchKernelGGL(attn_merge_kernel<D>, mgrid, mblock, 0, stream, b, g.H, out, c, plan.chunk,
                     plan.chunks_max, plan.q_tile, ws_o, ws_ml);
  return hipGetLastError();
}

template <int D>
hipError_t launch_d(const PoolGeom& g, const AttnPlan& plan, const uint16_t* q, uint16_t* out,
                    const BatchDev& b, float c, float* ws_o, float* ws_ml, hipStream_t stream) {
  switch (plan.q_tile / 16) {
    case 1: return launch_one<D, 1>(g, plan, q, out, b, c, ws_o, ws_ml, stream);
    case 2: return launch_one<D, 2>(g, plan, q, out, b, c, ws_o, ws_ml, stream);
    case 3: return launch_one<D, 3>(g, plan, q, out, b, c, ws_o, ws_ml, stream);
    default: return launch_one<D, 4>(g, plan, q, out, b, c, ws_o, ws_ml, stream);
  }
}

}  // namespace

hipError_t launch_attn_mfma(const PoolGeom& g, const AttnPlan& plan, const void* q, void* out,
                            const BatchDev& b, float sm_scale, void* workspace, hipStream_t stream) {
  if (b.total_new <= 0 || b.batch <= 0) return hipSuccess;
  const float c = sm_scale * 1.4426950408889634f;     // logits are exponentiated in base 2
  float* ws_o = reinterpret_cast<float*>(workspace);
  float* ws_ml = ws_o ? ws_o + (int64_t)b.total_new * g.H * plan.chunks_max * g.D : nullptr;
  const uint16_t* qp = reinterpret_cast<const uint16_t*>(q);
  uint16_t* op = reinterpret_cast<uint16_t*>(out);
  switch (g.D) {
    case 32: return launch_d<32>(g, plan, qp, op, b, c, ws_o, ws_ml, stream);
    case 64: return launch_d<64>(g, plan, qp, op, b, c, ws_o, ws_ml, stream);
    case 128: return launch_d<128>(g, plan, qp, op, b, c, ws_o, ws_ml, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace mts

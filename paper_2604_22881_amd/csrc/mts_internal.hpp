// Launchers behind the C ABI.  Each takes validated arguments, enqueues its kernels on
// `stream` and returns the hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mts_layout.hpp"

namespace mts {

// records the calling thread's error text (what mts_last_error returns) and returns `code`
int32_t set_error(int32_t code, const char* fmt, ...);

struct BatchDev {            // device metadata arrays, as in mts_batch_meta
  int32_t        batch;
  const int32_t* page_indptr;
  const int32_t* page_indices;
  const int32_t* prefix_lens;
  const int32_t* new_indptr;
  int32_t        total_new;
  int32_t        max_new;
  int32_t        max_total_len;
  int32_t        total_pages;
};

struct SegDev {              // segment lists of unpack / pack
  int32_t        num_segs;
  const int32_t* seg_user;
  const int32_t* seg_pos;
  const int64_t* seg_tok_indptr;
  int32_t        max_seg_tokens;
};

// `layers` consecutive layers starting at g.layer_base in one launch: layer i of the pool lies
// i * pool_layer_stride bytes further, its runs i * staging_layer_stride bytes further.
hipError_t launch_unpack(const PoolGeom& g, const void* staging, const SegDev& segs, const BatchDev& b,
                         hipStream_t stream, int layers = 1, int64_t pool_layer_stride = 0,
                         int64_t staging_layer_stride = 0);
hipError_t launch_pack(const PoolGeom& g, void* staging_out, const SegDev& segs, const BatchDev& b,
                       hipStream_t stream, int layers = 1, int64_t pool_layer_stride = 0,
                       int64_t staging_layer_stride = 0);
hipError_t launch_append(const PoolGeom& g, const void* k_new, const void* v_new, const BatchDev& b,
                         hipStream_t stream, int layers = 1, int64_t pool_layer_stride = 0,
                         int64_t rows_layer_stride = 0);

// Shape plan of one attention call: computed on the host from the scalar bounds only.
struct AttnPlan {
  bool    use_mfma;      // bf16 matrix-core kernel, else the plain fp32-accumulate kernel
  bool    use_prefill;   // workgroup-per-query-block kernel for long new segments (no workspace)
  bool    too_large;     // more (user, query tile) items than the schedule can hold
  int32_t q_tile;        // queries per query tile (multiple of 16, <= 64)
  int32_t q_tiles_max;   // ceil(max_new / q_tile)
  int32_t n_items;       // batch * q_tiles_max
  int32_t min_tiles;     // least kv tiles a wavefront's share may hold
  int32_t pair_cost;     // schedule allowance per (query tile, head), in tiles
  int32_t max_waves;     // most wavefronts the launch may use (sizes the partial buffers)
  int64_t ws_desc_bytes; // per-wavefront merge descriptors at the start of the workspace
  int64_t ws_bytes;      // whole workspace
};
AttnPlan plan_attention(const PoolGeom& g, const BatchDev& b);
constexpr int kAttnMaxWaves = 1024;   // 256 CUs x 4 SIMDs: one wavefront per SIMD


// inv_norm selects the aggregation: 0 = softmax (Sec. 2, Eq. 6-7); > 0 = pointwise,
// out = inv_norm * sum_j silu(sm_scale * q.k_j) v_j (no softmax statistics).
hipError_t launch_attn_generic(const PoolGeom& g, const void* q, void* out, const BatchDev& b,
                               float sm_scale, float inv_norm, hipStream_t stream);
bool attn_prefill_applicable(const PoolGeom& g, const BatchDev& b);
hipError_t launch_attn_prefill(const PoolGeom& g, const void* q, void* out, const BatchDev& b,
                               float sm_scale, float inv_norm, hipStream_t stream);
// Prefixes still in the contiguous onload buffer (device arrays; see mts_attn_incremental_staged).
struct StagedHistories {
  const void*    rows;        // the layer's runs, [2][n][H][D] each
  const int32_t* first_run;   // [batch]: first run of user u's prefix, -1 = prefix in the pool
  const int64_t* run_tok;     // [runs + 1]: token offset of every run in `rows`
  int32_t        chunk;       // tokens per run (the last run of a user may be shorter)
};

// k_new / v_new non-NULL: this step's K/V rows ([token][H][D]) are read from there and the
// pool's slots for them are not touched, so the layer's append need not have happened; with
// `hist`, the prefixes of the users it names are read from the onload buffer as well.
hipError_t launch_attn_mfma(const PoolGeom& g, const AttnPlan& plan, const void* q, void* out,
                            const BatchDev& b, float sm_scale, float inv_norm, void* workspace,
                            hipStream_t stream, const void* k_new = nullptr, const void* v_new = nullptr,
                            const StagedHistories* hist = nullptr);

}  // namespace mts

// Dispatcher of the streaming matrix-core attention kernel (mts_attn_stream.inc): picks the
// instantiation unit by head_dim and by where keys and values come from.
#include "mts_attn_stream_decl.hpp"

namespace mts {

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
  const bool staged = fresh && hist != nullptr && !pw;
#define MTS_ATTN_CASE(D_)                                                                                        \
  case D_:                                                                                                       \
    if (staged) return launch_attn_stream<D_, 2>(g, plan, qp, kp, vp, hist, op, b, c, inv_norm, workspace, stream); \
    return fresh ? launch_attn_stream<D_, 1>(g, plan, qp, kp, vp, nullptr, op, b, c, inv_norm, workspace, stream)   \
                 : launch_attn_stream<D_, 0>(g, plan, qp, kp, vp, nullptr, op, b, c, inv_norm, workspace, stream);
  switch (g.D) {
    MTS_ATTN_CASE(32)
    MTS_ATTN_CASE(64)
    MTS_ATTN_CASE(128)
    default: return hipErrorInvalidValue;
  }
#undef MTS_ATTN_CASE
}

}  // namespace mts

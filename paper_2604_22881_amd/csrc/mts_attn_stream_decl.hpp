// Entry of one instantiation unit of the streaming attention kernel (defined in
// mts_attn_stream_d<D>_s<SRC>.hip through mts_attn_stream.inc).
#pragma once
#include "mts_internal.hpp"

namespace mts {

template <int D, int SRC>
hipError_t launch_attn_stream(const PoolGeom& g, const AttnPlan& plan, const uint16_t* q, const uint16_t* k_new,
                              const uint16_t* v_new, const StagedHistories* hist, uint16_t* out, const BatchDev& b,
                              float c, float inv_norm, void* ws, hipStream_t stream);

}  // namespace mts

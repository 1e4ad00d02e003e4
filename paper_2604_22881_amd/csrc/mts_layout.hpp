// Paged-pool geometry shared by the host entry points and the kernels.
//
// The pool replaces the paper's [L, N_pages, 2, S_page, H, D] tensor (Sec. 4.1) by an
// arrangement in which every 16-byte granule a wavefront loads is already a matrix-core
// operand fragment:
//   page -> head -> {K block, V block}; each block is S/16 sub-blocks of 16 tokens.
//   K sub-block: [half][D/G][8 slots][G] elements, G = 16 bytes / element size.
//                token t (0..15) has half = (t/4)%2 and slot = (t/8)*4 + t%4, so that the
//                eight slots of one half are the rows one 16x16 MFMA tile takes from this
//                sub-block and the accumulator lanes end up holding 8 consecutive tokens.
//   V sub-block: transposed, [D][16 tokens], so that 8 consecutive tokens of one dim are
//                one 16-byte granule (the contraction index of P.V is the token).
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define MTS_HD __host__ __device__ __forceinline__
#else
#define MTS_HD inline
#endif

namespace mts {

struct PoolGeom {
  char*   layer_base;   // pool + layer * layer_stride_bytes
  int64_t page_bytes;   // 2 * H * S * D * es
  int32_t num_pages;
  int32_t S;            // tokens per page
  int32_t H;
  int32_t D;
  int32_t es;           // element bytes
  int32_t sub_shift;    // log2(S / 16): sub-blocks per page
};

// element index of (token t16 in [0,16), dim d) inside a 16-token K sub-block
MTS_HD int32_t k_sub_index(int32_t t16, int32_t d, int32_t D, int32_t G) {
  const int32_t half = (t16 >> 2) & 1;
  const int32_t slot = ((t16 >> 3) << 2) | (t16 & 3);
  return ((half * (D / G) + d / G) * 8 + slot) * G + d % G;
}

// element index of (token t16, dim d) inside a 16-token V sub-block
MTS_HD int32_t v_sub_index(int32_t t16, int32_t d) { return d * 16 + t16; }

// byte offset inside a page of the K (kv = 0) or V (kv = 1) block of head h
MTS_HD int64_t head_block_offset(int32_t kv, int32_t h, int32_t S, int32_t D, int32_t es) {
  return ((int64_t)h * 2 + kv) * S * D * es;
}

// byte offset inside a page of element (kv, head, slot-in-page, dim)
MTS_HD int64_t elem_offset(int32_t kv, int32_t h, int32_t slot, int32_t d, int32_t S, int32_t D, int32_t es) {
  const int32_t G = 16 / es;
  const int32_t sub = slot >> 4, t16 = slot & 15;
  const int64_t idx = (int64_t)sub * 16 * D + (kv == 0 ? k_sub_index(t16, d, D, G) : v_sub_index(t16, d));
  return head_block_offset(kv, h, S, D, es) + idx * es;
}

}  // namespace mts

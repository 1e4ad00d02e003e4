// Instantiation unit of the streaming attention kernel: head_dim 64, key/value source 0
// (0 the pool, 1 the step's rows read from k_new / v_new, 2 also restored prefixes from the onload buffer).
#define MTS_INST_D 64
#define MTS_INST_SRC 0
#include "mts_attn_stream.inc"

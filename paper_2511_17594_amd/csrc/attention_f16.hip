// Single-pass CSR attention kernels for fp16 Q, K, V (eight elements per 16-byte lane load), fp32 state.
#define AUTOSAGE_ATTN_T f16_t
#define AUTOSAGE_ATTN_SUFFIX f16
#define AUTOSAGE_ATTN_VEC 8
#include "attention_dispatch.inc"

// Single-pass CSR attention kernels for bf16 Q, K, V (eight elements per 16-byte lane load), fp32 state.
#define AUTOSAGE_ATTN_T bf16_t
#define AUTOSAGE_ATTN_SUFFIX bf16
#define AUTOSAGE_ATTN_VEC 8
#include "attention_dispatch.inc"

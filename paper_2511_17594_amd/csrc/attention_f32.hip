// Single-pass CSR attention kernels for fp32 Q, K, V (four elements per 16-byte lane load).
#define AUTOSAGE_ATTN_T float
#define AUTOSAGE_ATTN_SUFFIX f32
#define AUTOSAGE_ATTN_VEC 4
#include "attention_dispatch.inc"

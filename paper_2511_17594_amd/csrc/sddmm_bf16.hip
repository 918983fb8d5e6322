// SDDMM kernels instantiated for bf16 dense operands, fp32 accumulation.
#define AUTOSAGE_SDDMM_T bf16_t
#define AUTOSAGE_SDDMM_SUFFIX bf16
#define AUTOSAGE_SDDMM_VECS(X) X(1) X(2) X(4) X(8)
#include "sddmm_dispatch.inc"

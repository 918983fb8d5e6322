// SDDMM kernels instantiated for fp16 (IEEE binary16) dense operands, fp32 accumulation.
#define AUTOSAGE_SDDMM_T f16_t
#define AUTOSAGE_SDDMM_SUFFIX f16
#define AUTOSAGE_SDDMM_VECS(X) X(1) X(2) X(4) X(8)
#include "sddmm_dispatch.inc"

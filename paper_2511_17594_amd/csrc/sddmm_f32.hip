// SDDMM kernels instantiated for fp32 dense operands.
#define AUTOSAGE_SDDMM_T float
#define AUTOSAGE_SDDMM_SUFFIX f32
#define AUTOSAGE_SDDMM_VECS(X) X(1) X(2) X(4)
#include "sddmm_dispatch.inc"

// SpMM kernels instantiated for fp32 dense operands (4-, 8- and 16-byte lane loads).
#define AUTOSAGE_SPMM_T float
#define AUTOSAGE_SPMM_SUFFIX f32
#define AUTOSAGE_SPMM_VECS(X) X(1) X(2) X(4)
#include "spmm_dispatch.inc"

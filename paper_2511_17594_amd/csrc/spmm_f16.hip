// SpMM kernels instantiated for fp16 (IEEE binary16) dense operands (2-, 4-, 8- and 16-byte lane loads), fp32 accumulation.
#define AUTOSAGE_SPMM_T f16_t
#define AUTOSAGE_SPMM_SUFFIX f16
#define AUTOSAGE_SPMM_VECS(X) X(1) X(2) X(4) X(8)
#include "spmm_dispatch.inc"

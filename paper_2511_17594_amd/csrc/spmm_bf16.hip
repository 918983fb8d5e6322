// SpMM kernels instantiated for bf16 dense operands (2-, 4-, 8- and 16-byte lane loads), fp32 accumulation.
#define AUTOSAGE_SPMM_T bf16_t
#define AUTOSAGE_SPMM_SUFFIX bf16
#define AUTOSAGE_SPMM_VECS(X) X(1) X(2) X(4) X(8)
#include "spmm_dispatch.inc"

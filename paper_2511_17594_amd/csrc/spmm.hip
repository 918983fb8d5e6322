// SpMM launch entry points: light rows, hub rows (partial + ordered combine).
#include "spmm_kernels.inc"

namespace autosage {

hipError_t spmm_rows_f32(const SpmmArgs&, const Resolved&, hipStream_t);
hipError_t spmm_rows_bf16(const SpmmArgs&, const Resolved&, hipStream_t);
hipError_t spmm_rows_f16(const SpmmArgs&, const Resolved&, hipStream_t);
hipError_t spmm_hub_partial_f32(const SpmmArgs&, const Resolved&, const HubMeta&, float*, hipStream_t);
hipError_t spmm_hub_partial_bf16(const SpmmArgs&, const Resolved&, const HubMeta&, float*, hipStream_t);
hipError_t spmm_hub_partial_f16(const SpmmArgs&, const Resolved&, const HubMeta&, float*, hipStream_t);

// Adds the partial rows of a hub row's chunks in ascending chunk order (fixed order -> reproducible).
__global__ void __launch_bounds__(256) spmm_hub_combine_kernel(SpmmDev a)
{
    const int k_hub = blockIdx.x;
    if (k_hub >= a.counts->n_hub) return;
    const int row = row_of(a.rows, a.hub_rows[k_hub]);
    const int c0 = a.chunk_ptr[k_hub];
    const int c1 = a.chunk_ptr[k_hub + 1];
    for (int f = threadIdx.x; f < a.F; f += blockDim.x) {
        float s = 0.f;
        for (int c = c0; c < c1; ++c) s += a.part[(int64_t)c * a.F + f];   // ascending chunk order
        a.C[(int64_t)row * a.ldc + f] = s;
    }
}

hipError_t launch_spmm_rows(const SpmmArgs& a, const Resolved& r, hipStream_t stream)
{
    if (a.dt == DT_BF16) return spmm_rows_bf16(a, r, stream);
    if (a.dt == DT_F16) return spmm_rows_f16(a, r, stream);
    return spmm_rows_f32(a, r, stream);
}

hipError_t launch_spmm_hub(const SpmmArgs& a, const Resolved& r, const HubMeta& meta, float* part, hipStream_t stream)
{
    if (meta.cap_hub == 0 || meta.cap_chunks == 0) return hipSuccess;
    hipError_t e = a.dt == DT_BF16  ? spmm_hub_partial_bf16(a, r, meta, part, stream)
                   : a.dt == DT_F16 ? spmm_hub_partial_f16(a, r, meta, part, stream)
                                    : spmm_hub_partial_f32(a, r, meta, part, stream);
    if (e != hipSuccess) return e;
    SpmmDev d{};
    d.rows = a.rows;
    d.rowptr = a.rowptr;
    d.C = a.C;
    d.ldc = a.ldc;
    d.F = a.F;
    d.counts = meta.counts;
    d.hub_rows = meta.hub_rows;
    d.chunk_ptr = meta.chunk_ptr;
    d.part = part;
    hipLaunchKernelGGL(spmm_hub_combine_kernel, dim3(meta.cap_hub), dim3(256), 0, stream, d);
    return hipGetLastError();
}

}  // namespace autosage

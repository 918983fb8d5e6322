// CSR transpose on the device: A^T as CSR plus the permutation that carries values along.
//
// Needed when the operators sit in a training step (the paper's Introduction motivates them by
// training throughput): the adjoint of C = A B with respect to B is A^T dC.  The transpose is a
// stable sort of the nonzeros by column (rocPRIM/hipCUB radix sort, a library primitive) followed by
// index kernels: inside a row of A^T the entries keep ascending source-row order, so the result is
// unique and reproducible.
#include <hipcub/hipcub.hpp>

#include "device_utils.h"
#include "launch.h"

namespace autosage {
namespace {

__global__ void __launch_bounds__(256) iota_kernel(int32_t* p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = (int32_t)i;
}

// t_rowptr[c] = number of sorted keys < c  (lower bound), c in [0, n_cols]
__global__ void __launch_bounds__(256) transpose_rowptr_kernel(const int32_t* __restrict__ keys, int64_t nnz, int64_t n_cols,
                                                               int32_t* __restrict__ t_rowptr)
{
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c > n_cols) return;
    int64_t lo = 0, hi = nnz;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (keys[mid] < c) lo = mid + 1; else hi = mid;
    }
    t_rowptr[c] = (int32_t)lo;
}

// For entry q of A^T: source position p = perm[q]; its source row is the i with rowptr[i] <= p < rowptr[i+1].
__global__ void __launch_bounds__(256) transpose_fill_kernel(const int32_t* __restrict__ perm, int64_t nnz, int64_t n_rows,
                                                             const int32_t* __restrict__ rowptr, const float* __restrict__ val,
                                                             int32_t* __restrict__ t_colind, float* __restrict__ t_val)
{
    const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= nnz) return;
    const int32_t p = perm[q];
    int64_t lo = 0, hi = n_rows;                 // largest i with rowptr[i] <= p
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (rowptr[mid] <= p) lo = mid; else hi = mid;
    }
    t_colind[q] = (int32_t)lo;
    if (val && t_val) t_val[q] = val[p];
}

// out[q, :] = in[perm[q], :] for rows of `width` floats (values carried to the transposed order)
__global__ void __launch_bounds__(256) gather_rows_kernel(const int32_t* __restrict__ perm, int64_t n, int32_t width,
                                                          const float* __restrict__ in, float* __restrict__ out)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n * width) return;
    const int64_t q = e / width;
    const int32_t w = (int32_t)(e - q * width);
    out[e] = in[(int64_t)perm[q] * width + w];
}

int key_bits(int64_t n_cols)
{
    int b = 1;
    while ((int64_t(1) << b) < n_cols && b < 31) ++b;
    return b;
}

}  // namespace

size_t transpose_sort_temp_bytes(int64_t nnz, int64_t n_cols)
{
    size_t bytes = 0;
    (void)hipcub::DeviceRadixSort::SortPairs(nullptr, bytes, (const int32_t*)nullptr, (int32_t*)nullptr, (const int32_t*)nullptr,
                                       (int32_t*)nullptr, (int)nnz, 0, key_bits(n_cols), (hipStream_t) nullptr);
    return bytes;
}

// keys_out, iota: int32[nnz] scratch; temp: sort scratch of transpose_sort_temp_bytes().
hipError_t launch_csr_transpose(int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
                                const float* val, int32_t* t_rowptr, int32_t* t_colind, float* t_val, int32_t* perm,
                                int32_t* keys_out, int32_t* iota, void* temp, size_t temp_bytes, hipStream_t stream)
{
    const int blocks_c = (int)((n_cols + 1 + 255) / 256);
    if (nnz == 0) {
        hipLaunchKernelGGL(transpose_rowptr_kernel, dim3(blocks_c), dim3(256), 0, stream, colind, (int64_t)0, n_cols, t_rowptr);
        return hipGetLastError();
    }
    const int blocks_n = (int)((nnz + 255) / 256);
    hipLaunchKernelGGL(iota_kernel, dim3(blocks_n), dim3(256), 0, stream, iota, nnz);
    hipError_t e = hipcub::DeviceRadixSort::SortPairs(temp, temp_bytes, colind, keys_out, (const int32_t*)iota, perm, (int)nnz, 0,
                                                      key_bits(n_cols), stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(transpose_rowptr_kernel, dim3(blocks_c), dim3(256), 0, stream, keys_out, nnz, n_cols, t_rowptr);
    hipLaunchKernelGGL(transpose_fill_kernel, dim3(blocks_n), dim3(256), 0, stream, perm, nnz, n_rows, rowptr, val, t_colind, t_val);
    return hipGetLastError();
}

hipError_t launch_gather_rows(const int32_t* perm, int64_t n, int32_t width, const float* in, float* out, hipStream_t stream)
{
    const int64_t total = n * width;
    if (total == 0) return hipSuccess;
    hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, perm, n, width, in, out);
    return hipGetLastError();
}

}  // namespace autosage

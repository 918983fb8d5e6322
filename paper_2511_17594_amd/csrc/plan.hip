// Index metadata kernels (integer only): heavy/light row partition with chunking of the heavy
// rows, degree histogram + rowptr samples for the graph signature, CSR validation.
//
// The paper's kernel-variant table separates rows by a split threshold hubT; the scheduler's
// feature extraction uses row/nnz counts and the degree distribution.  The chunk scheme for
// heavy rows (ceil(deg / hub_chunk) pieces of consecutive nonzeros) belongs to this library.
#include "device_utils.h"
#include <algorithm>
#include "launch.h"

namespace autosage {
namespace {

constexpr int kPartThreads = 256;
constexpr int kRowsPerThread = 4;
constexpr int kRowsPerBlock = kPartThreads * kRowsPerThread;

struct PartDev {
    RowMap rows;
    const int32_t* __restrict__ rowptr;
    int32_t hub_t;
    int32_t hub_chunk;
    int32_t n_blocks;
    HubCounts* counts;
    int32_t* hub_rows;
    int32_t* chunk_ptr;
    int32_t* light_rows;
    int32_t* block_counts;     // [n_blocks][2] = (hubs, chunks) of the block
};

__device__ __forceinline__ int row_degree(const PartDev& a, int idx)
{
    const int row = row_of(a.rows, idx);
    return a.rowptr[row + 1] - a.rowptr[row];
}

// Exclusive scan over the workgroup of (x, y); returns this thread's offsets and the totals.
__device__ __forceinline__ void block_scan2(int x, int y, int& ex, int& ey, int& tx, int& ty, int* lds)
{
    int* sx = lds;
    int* sy = lds + kPartThreads;
    const int t = threadIdx.x;
    sx[t] = x;
    sy[t] = y;
    __syncthreads();
    for (int off = 1; off < kPartThreads; off <<= 1) {
        const int ax = t >= off ? sx[t - off] : 0;
        const int ay = t >= off ? sy[t - off] : 0;
        __syncthreads();
        sx[t] += ax;
        sy[t] += ay;
        __syncthreads();
    }
    ex = sx[t] - x;
    ey = sy[t] - y;
    tx = sx[kPartThreads - 1];
    ty = sy[kPartThreads - 1];
    __syncthreads();
}

__global__ void __launch_bounds__(kPartThreads) hub_count_kernel(PartDev a)
{
    __shared__ int lds[2 * kPartThreads];
    int nh = 0, nc = 0;
    const int first = blockIdx.x * kRowsPerBlock + threadIdx.x * kRowsPerThread;
#pragma unroll
    for (int r = 0; r < kRowsPerThread; ++r) {
        const int idx = first + r;
        if (idx < a.rows.count) {
            const int deg = row_degree(a, idx);
            if (deg >= a.hub_t) {
                ++nh;
                nc += (deg - 1) / a.hub_chunk + 1;
            }
        }
    }
    int ex, ey, tx, ty;
    block_scan2(nh, nc, ex, ey, tx, ty, lds);
    if (threadIdx.x == 0) {
        a.block_counts[2 * blockIdx.x + 0] = tx;
        a.block_counts[2 * blockIdx.x + 1] = ty;
    }
}

__global__ void __launch_bounds__(kPartThreads) hub_fill_kernel(PartDev a)
{
    __shared__ int lds[2 * kPartThreads];
    // hubs / chunks in all earlier blocks
    int bh = 0, bc = 0;
    for (int b = threadIdx.x; b < (int)blockIdx.x; b += kPartThreads) {
        bh += a.block_counts[2 * b + 0];
        bc += a.block_counts[2 * b + 1];
    }
    int ex, ey, base_h, base_c;
    block_scan2(bh, bc, ex, ey, base_h, base_c, lds);

    int deg[kRowsPerThread];
    int nh = 0, nc = 0;
    const int first = blockIdx.x * kRowsPerBlock + threadIdx.x * kRowsPerThread;
#pragma unroll
    for (int r = 0; r < kRowsPerThread; ++r) {
        const int idx = first + r;
        deg[r] = idx < a.rows.count ? row_degree(a, idx) : -1;
        if (deg[r] >= a.hub_t) {
            ++nh;
            nc += (deg[r] - 1) / a.hub_chunk + 1;
        }
    }
    int tx, ty;
    block_scan2(nh, nc, ex, ey, tx, ty, lds);
    int h = base_h + ex;          // hubs before this thread's first row
    int c = base_c + ey;          // chunks before it
#pragma unroll
    for (int r = 0; r < kRowsPerThread; ++r) {
        const int idx = first + r;
        if (deg[r] < 0) continue;
        if (deg[r] >= a.hub_t) {
            a.hub_rows[h] = idx;
            c += (deg[r] - 1) / a.hub_chunk + 1;
            a.chunk_ptr[h + 1] = c;
            ++h;
        } else if (a.light_rows) {
            a.light_rows[idx - h] = idx;      // lights before idx = idx - hubs before idx
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) a.chunk_ptr[0] = 0;
    if ((int)blockIdx.x == a.n_blocks - 1 && threadIdx.x == 0) {
        a.counts->n_hub = base_h + tx;
        a.counts->n_chunks = base_c + ty;
        a.counts->n_light = a.rows.count - (base_h + tx);
        a.counts->pad = 0;
    }
}

__global__ void __launch_bounds__(64) hub_empty_kernel(PartDev a)
{
    if (threadIdx.x == 0) {
        a.counts->n_hub = 0;
        a.counts->n_chunks = 0;
        a.counts->n_light = 0;
        a.counts->pad = 0;
        a.chunk_ptr[0] = 0;
    }
}

// ---- degree features ---------------------------------------------------------------------
// out[0..32] = histogram, out[33] = max degree, out[34] = nnz, out[35 .. 35+1023] = rowptr samples.
__global__ void __launch_bounds__(256) features_kernel(int64_t n_rows, const int32_t* __restrict__ rowptr,
                                                       unsigned long long* out)
{
    __shared__ unsigned int hist[33];
    __shared__ int smax;
    if (threadIdx.x < 33) hist[threadIdx.x] = 0;
    if (threadIdx.x == 0) smax = 0;
    __syncthreads();
    int mx = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_rows; i += (int64_t)gridDim.x * blockDim.x) {
        const int deg = rowptr[i + 1] - rowptr[i];
        const int b = deg > 0 ? 32 - __clz(deg) : 0;
        atomicAdd(&hist[b], 1u);
        mx = max(mx, deg);
    }
    atomicMax(&smax, mx);
    __syncthreads();
    if (threadIdx.x < 33 && hist[threadIdx.x]) atomicAdd(&out[threadIdx.x], (unsigned long long)hist[threadIdx.x]);
    if (threadIdx.x == 0) atomicMax(&out[33], (unsigned long long)smax);
    const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (g < 1024) out[35 + g] = (unsigned long long)(long long)rowptr[(g * n_rows) / 1023];
    if (g == 0) out[34] = (unsigned long long)(long long)rowptr[n_rows];
}

__global__ void __launch_bounds__(256) zero_u64_kernel(unsigned long long* p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0ull;
}

__global__ void __launch_bounds__(256) validate_kernel(int64_t n_rows, int64_t n_cols, int64_t nnz,
                                                       const int32_t* __restrict__ rowptr,
                                                       const int32_t* __restrict__ colind, int32_t* flag)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    bool bad = false;
    if (g == 0) bad = rowptr[0] != 0 || (int64_t)rowptr[n_rows] != nnz;
    for (int64_t i = g; i < n_rows; i += stride) bad |= rowptr[i + 1] < rowptr[i] || rowptr[i] < 0 || (int64_t)rowptr[i + 1] > nnz;
    // colind is only read where rowptr says it exists; a bad rowptr is reported without touching colind out of range
    for (int64_t p = g; p < nnz; p += stride) bad |= colind[p] < 0 || (int64_t)colind[p] >= n_cols;
    if (bad) atomicOr(flag, 1);
}

__global__ void zero_flag_kernel(int32_t* flag) { *flag = 0; }

// dst[i] = (int32) src[i]; flags any value outside [0, limit]
__global__ void __launch_bounds__(256) narrow_kernel(int64_t n, const int64_t* __restrict__ src, int32_t* __restrict__ dst,
                                                     int64_t limit, int32_t* flag)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    bool bad = false;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const int64_t v = src[i];
        bad |= v < 0 || v > limit;
        dst[i] = static_cast<int32_t>(v);
    }
    if (bad) atomicOr(flag, 1);
}

}  // namespace

hipError_t launch_hub_partition(const RowMap& rows, const int32_t* rowptr, int32_t hub_t, int32_t hub_chunk,
                                const HubMeta& meta, hipStream_t stream)
{
    PartDev d{};
    d.rows = rows;
    d.rowptr = rowptr;
    d.hub_t = hub_t;
    d.hub_chunk = hub_chunk;
    d.counts = meta.counts;
    d.hub_rows = meta.hub_rows;
    d.chunk_ptr = meta.chunk_ptr;
    d.light_rows = meta.light_rows;
    d.block_counts = meta.block_counts;
    d.n_blocks = (rows.count + kRowsPerBlock - 1) / kRowsPerBlock;
    if (d.n_blocks == 0) {
        hipLaunchKernelGGL(hub_empty_kernel, dim3(1), dim3(64), 0, stream, d);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(hub_count_kernel, dim3(d.n_blocks), dim3(kPartThreads), 0, stream, d);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(hub_fill_kernel, dim3(d.n_blocks), dim3(kPartThreads), 0, stream, d);
    return hipGetLastError();
}

hipError_t launch_graph_features(int64_t n_rows, const int32_t* rowptr, int64_t* dev_out, hipStream_t stream)
{
    unsigned long long* out = reinterpret_cast<unsigned long long*>(dev_out);
    hipLaunchKernelGGL(zero_u64_kernel, dim3(1), dim3(256), 0, stream, out, 35);
    int blocks = (int)((n_rows + 255) / 256);
    if (blocks < 4) blocks = 4;          // at least 1024 threads for the rowptr samples
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(features_kernel, dim3(blocks), dim3(256), 0, stream, n_rows, rowptr, out);
    return hipGetLastError();
}

hipError_t launch_validate_csr(int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t* rowptr,
                               const int32_t* colind, int32_t* dev_flag, hipStream_t stream)
{
    hipLaunchKernelGGL(zero_flag_kernel, dim3(1), dim3(1), 0, stream, dev_flag);
    int64_t work = n_rows > nnz ? n_rows : nnz;
    int blocks = (int)((work + 255) / 256);
    if (blocks < 1) blocks = 1;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(validate_kernel, dim3(blocks), dim3(256), 0, stream, n_rows, n_cols, nnz, rowptr, colind, dev_flag);
    return hipGetLastError();
}

hipError_t launch_narrow_indices(int64_t n, const int64_t* src, int32_t* dst, int64_t limit, int32_t* dev_flag,
                                 hipStream_t stream)
{
    hipLaunchKernelGGL(zero_flag_kernel, dim3(1), dim3(1), 0, stream, dev_flag);
    if (n > 0) {
        int blocks = (int)std::min<int64_t>((n + 255) / 256, 8192);
        hipLaunchKernelGGL(narrow_kernel, dim3(blocks), dim3(256), 0, stream, n, src, dst, limit, dev_flag);
    }
    return hipGetLastError();
}

}  // namespace autosage

// CSR transpose on the device: A^T as CSR plus the permutation that carries values along.
//
// Needed when the operators sit in a training step (the paper's Introduction motivates them by
// training throughput): the adjoint of C = A B with respect to B is A^T dC.  The transpose is a
// stable sort of the nonzeros by column followed by index kernels: inside a row of A^T the entries
// keep ascending source-row order, so the result is unique and reproducible.
//
// The sort is a least-significant-digit radix sort of (column, position) pairs, 8 bits per pass, over as
// many passes as the column count needs.  A pass is three steps: a histogram of the digit per tile of 4096
// keys, an exclusive scan of the histograms laid out digit-major (so the scanned value of (digit, tile) is
// where that tile's first key with that digit goes), and a scatter in which every key finds its rank among
// the tile's keys of the same digit: a wavefront walks its 1024 keys 64 at a time, the lanes that hold equal
// digits find each other with eight ballots, the first of them advances the wavefront's counter of the digit
// in LDS, and the four wavefronts' counters are then stacked in order.  Keys of a digit keep their order
// inside a tile and tiles keep theirs, so every pass is stable.
#include "device_utils.h"
#include "launch.h"

namespace autosage {
namespace {

constexpr int kSortBits = 8;
constexpr int kSortBuckets = 1 << kSortBits;
constexpr int kSortLanes = 256;                              // one lane per bucket
constexpr int kSortItems = 16;                               // keys per lane
constexpr int kSortTile = kSortLanes * kSortItems;
constexpr int kSortWaves = kSortLanes / kWave;
constexpr int kWaveKeys = kSortTile / kSortWaves;

__global__ void __launch_bounds__(kSortLanes) sort_histogram_kernel(const int32_t* __restrict__ keys, int64_t n, int shift,
                                                                    int n_tiles, int32_t* __restrict__ hist)
{
    __shared__ int32_t cnt[kSortBuckets];
    cnt[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * kSortTile;
#pragma unroll
    for (int k = 0; k < kSortItems; ++k) {
        const int64_t i = base + k * kSortLanes + threadIdx.x;
        if (i < n) atomicAdd(&cnt[(keys[i] >> shift) & (kSortBuckets - 1)], 1);     // integer counts: order does not matter
    }
    __syncthreads();
    hist[(int64_t)threadIdx.x * n_tiles + blockIdx.x] = cnt[threadIdx.x];
}

// Exclusive scan of int32 a[0, n) in place, in three launches: sums of chunks of 4096, a scan of those sums by one
// workgroup, and the scan of every chunk on top of its sum.  A lane owns 16 consecutive elements.
constexpr int kScanLanes = 256;
constexpr int kScanItems = 16;
constexpr int kScanChunk = kScanLanes * kScanItems;

// Exclusive prefix of x over the workgroup's lanes in lane order; *total gets the workgroup's sum.
__device__ __forceinline__ int32_t block_exclusive(int32_t x, int32_t* total)
{
    __shared__ int32_t wave_sum[kScanLanes / kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    int32_t incl = x;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const int32_t y = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += y;
    }
    __syncthreads();                                         // the last use of wave_sum is over
    if (lane == kWave - 1) wave_sum[wave] = incl;
    __syncthreads();
    int32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kScanLanes / kWave; ++w) {
        before += w < wave ? wave_sum[w] : 0;
        all += wave_sum[w];
    }
    *total = all;
    return before + incl - x;
}

__global__ void __launch_bounds__(kScanLanes) scan_sums_kernel(const int32_t* __restrict__ a, int64_t n, int32_t* __restrict__ sums)
{
    const int64_t base = (int64_t)blockIdx.x * kScanChunk + (int64_t)threadIdx.x * kScanItems;
    int32_t s = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) s += base + k < n ? a[base + k] : 0;
    int32_t total;
    (void)block_exclusive(s, &total);
    if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

__global__ void __launch_bounds__(kScanLanes) scan_spine_kernel(int32_t* __restrict__ sums, int n_sums)
{
    int32_t carry = 0;
    for (int base = 0; base < n_sums; base += kScanLanes) {
        const int i = base + threadIdx.x;
        const int32_t x = i < n_sums ? sums[i] : 0;
        int32_t total;
        const int32_t ex = block_exclusive(x, &total);
        if (i < n_sums) sums[i] = carry + ex;
        carry += total;
    }
}

__global__ void __launch_bounds__(kScanLanes) scan_chunks_kernel(int32_t* __restrict__ a, int64_t n, const int32_t* __restrict__ sums)
{
    const int64_t base = (int64_t)blockIdx.x * kScanChunk + (int64_t)threadIdx.x * kScanItems;
    int32_t v[kScanItems];
    int32_t s = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
        v[k] = base + k < n ? a[base + k] : 0;
        s += v[k];
    }
    int32_t total;
    int32_t run = sums[blockIdx.x] + block_exclusive(s, &total);
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
        if (base + k < n) a[base + k] = run;
        run += v[k];
    }
}

// One pass of the sort for one tile.  vals_in == nullptr: the value of key i is i (first pass).
__global__ void __launch_bounds__(kSortLanes) sort_scatter_kernel(const int32_t* __restrict__ keys_in, const int32_t* __restrict__ vals_in,
                                                                  int64_t n, int shift, int n_tiles,
                                                                  const int32_t* __restrict__ offsets,
                                                                  int32_t* __restrict__ keys_out, int32_t* __restrict__ vals_out)
{
    __shared__ int32_t cnt[kSortWaves][kSortBuckets];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
#pragma unroll
    for (int w = 0; w < kSortWaves; ++w) cnt[w][threadIdx.x] = 0;
    const int64_t wbase = (int64_t)blockIdx.x * kSortTile + (int64_t)wave * kWaveKeys;
    int32_t key[kSortItems], val[kSortItems], rank[kSortItems];
#pragma unroll
    for (int k = 0; k < kSortItems; ++k) {
        const int64_t i = wbase + k * kWave + lane;
        const bool valid = i < n;
        key[k] = valid ? keys_in[i] : 0;
        val[k] = valid ? (vals_in ? vals_in[i] : (int32_t)i) : 0;
    }
    __syncthreads();
    // rank of every key among the keys of its digit that precede it in the wavefront's 1024
#pragma unroll
    for (int k = 0; k < kSortItems; ++k) {
        const bool valid = wbase + k * kWave + lane < n;
        const int d = (key[k] >> shift) & (kSortBuckets - 1);
        unsigned long long peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < kSortBits; ++b) {
            const bool bit = (d >> b) & 1;
            const unsigned long long m = __ballot(bit);
            peers &= bit ? m : ~m;
        }
        int32_t start = 0;
        const int leader = valid ? __ffsll((long long)peers) - 1 : lane;
        if (valid && lane == leader) {
            start = cnt[wave][d];
            cnt[wave][d] = start + __popcll(peers);
        }
        start = __shfl(start, leader, kWave);
        rank[k] = start + __popcll(peers & ((1ull << lane) - 1ull));
        __syncthreads();                                     // the counters the next 64 keys read are written
    }
    // where the wavefront's keys of every digit start: the scanned histogram entry of (digit, tile), then the
    // wavefronts in order
    {
        const int d = threadIdx.x;
        int32_t run = offsets[(int64_t)d * n_tiles + blockIdx.x];
#pragma unroll
        for (int w = 0; w < kSortWaves; ++w) {
            const int32_t c = cnt[w][d];
            cnt[w][d] = run;
            run += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kSortItems; ++k) {
        if (wbase + k * kWave + lane < n) {
            const int32_t pos = cnt[wave][(key[k] >> shift) & (kSortBuckets - 1)] + rank[k];
            keys_out[pos] = key[k];
            vals_out[pos] = val[k];
        }
    }
}

struct SortPlan {
    int passes;
    int n_tiles;
    int64_t hist_len;
    int n_sums;
    size_t vals_bytes, hist_bytes, sums_bytes;
};

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

// Source row of every stored position, in two steps so that no position pays a search over all rows:
// bucket_row[b] = row that holds position 64 b (one search per 64 positions; n_rows - 1 past the end) ...
constexpr int kRowBucket = 64;
__global__ void __launch_bounds__(256) bucket_rows_kernel(const int32_t* __restrict__ rowptr, int64_t n_rows, int64_t nnz,
                                                          int64_t n_buckets, int32_t* __restrict__ bucket_row)
{
    const int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (b > n_buckets) return;
    const int64_t p = b * kRowBucket;
    int64_t lo = 0, hi = n_rows;                 // largest i < n_rows with rowptr[i] <= p
    if (p >= nnz) {
        lo = n_rows - 1;
    } else {
        while (hi - lo > 1) {
            const int64_t mid = (lo + hi) >> 1;
            if (rowptr[mid] <= p) lo = mid; else hi = mid;
        }
    }
    bucket_row[b] = (int32_t)lo;
}

// ... and row_of[p] = the row between the rows of the two bucket starts around p (neighbouring lanes read the same
// few entries of rowptr, so the loads are served by the caches).
__global__ void __launch_bounds__(256) position_rows_kernel(const int32_t* __restrict__ rowptr, int64_t nnz,
                                                            const int32_t* __restrict__ bucket_row, int32_t* __restrict__ row_of)
{
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= nnz) return;
    const int64_t b = p / kRowBucket;
    int32_t lo = bucket_row[b], hi = bucket_row[b + 1];
    while (hi > lo) {                            // largest i in [lo, hi] with rowptr[i] <= p
        const int32_t mid = lo + ((hi - lo + 1) >> 1);
        if (rowptr[mid] <= p) lo = mid; else hi = mid - 1;
    }
    row_of[p] = lo;
}

// Entry q of A^T comes from position perm[q] of A: its column is that position's row.
__global__ void __launch_bounds__(256) transpose_fill_kernel(const int32_t* __restrict__ perm, int64_t nnz,
                                                             const int32_t* __restrict__ row_of, const float* __restrict__ val,
                                                             int32_t* __restrict__ t_colind, float* __restrict__ t_val)
{
    const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= nnz) return;
    const int32_t p = perm[q];
    t_colind[q] = row_of[p];
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

SortPlan sort_plan(int64_t nnz, int64_t n_cols)
{
    SortPlan p{};
    p.passes = (key_bits(n_cols) + kSortBits - 1) / kSortBits;
    p.n_tiles = (int)((nnz + kSortTile - 1) / kSortTile);
    p.hist_len = (int64_t)kSortBuckets * p.n_tiles;
    p.n_sums = (int)((p.hist_len + kScanChunk - 1) / kScanChunk);
    auto up = [](size_t b) { return (b + 255) & ~size_t(255); };
    p.vals_bytes = up(sizeof(int32_t) * (size_t)nnz);
    p.hist_bytes = up(sizeof(int32_t) * (size_t)p.hist_len);
    p.sums_bytes = up(sizeof(int32_t) * (size_t)p.n_sums);
    return p;
}

}  // namespace

// Scratch of the sort beyond the two key buffers and the permutation: a second value buffer, the per-tile digit
// histograms and the chunk sums of their scan.
size_t transpose_sort_temp_bytes(int64_t nnz, int64_t n_cols)
{
    const SortPlan p = sort_plan(nnz, n_cols);
    return p.vals_bytes + p.hist_bytes + p.sums_bytes;
}

// keys_a, keys_b: int32[nnz] scratch (the sorted columns end in one of them); temp: transpose_sort_temp_bytes().
hipError_t launch_csr_transpose(int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
                                const float* val, int32_t* t_rowptr, int32_t* t_colind, float* t_val, int32_t* perm,
                                int32_t* keys_a, int32_t* keys_b, void* temp, size_t temp_bytes, hipStream_t stream)
{
    const int blocks_c = (int)((n_cols + 1 + 255) / 256);
    if (nnz == 0) {
        hipLaunchKernelGGL(transpose_rowptr_kernel, dim3(blocks_c), dim3(256), 0, stream, colind, (int64_t)0, n_cols, t_rowptr);
        return hipGetLastError();
    }
    const SortPlan p = sort_plan(nnz, n_cols);
    if (!temp || temp_bytes < p.vals_bytes + p.hist_bytes + p.sums_bytes) return hipErrorInvalidValue;
    char* t = static_cast<char*>(temp);
    int32_t* vals_b = reinterpret_cast<int32_t*>(t);
    int32_t* hist = reinterpret_cast<int32_t*>(t + p.vals_bytes);
    int32_t* sums = reinterpret_cast<int32_t*>(t + p.vals_bytes + p.hist_bytes);
    const int32_t* keys_in = colind;
    const int32_t* vals_in = nullptr;                        // first pass: the value of key i is i
    for (int pass = 0; pass < p.passes; ++pass) {
        const int shift = pass * kSortBits;
        int32_t* keys_out = pass % 2 == 0 ? keys_a : keys_b;
        int32_t* vals_out = (p.passes - 1 - pass) % 2 == 0 ? perm : vals_b;     // the last pass writes the permutation
        hipLaunchKernelGGL(sort_histogram_kernel, dim3(p.n_tiles), dim3(kSortLanes), 0, stream, keys_in, nnz, shift, p.n_tiles, hist);
        hipLaunchKernelGGL(scan_sums_kernel, dim3(p.n_sums), dim3(kScanLanes), 0, stream, hist, p.hist_len, sums);
        hipLaunchKernelGGL(scan_spine_kernel, dim3(1), dim3(kScanLanes), 0, stream, sums, p.n_sums);
        hipLaunchKernelGGL(scan_chunks_kernel, dim3(p.n_sums), dim3(kScanLanes), 0, stream, hist, p.hist_len, sums);
        hipLaunchKernelGGL(sort_scatter_kernel, dim3(p.n_tiles), dim3(kSortLanes), 0, stream, keys_in, vals_in, nnz, shift, p.n_tiles,
                           hist, keys_out, vals_out);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        keys_in = keys_out;
        vals_in = vals_out;
    }
    const int blocks_n = (int)((nnz + 255) / 256);
    hipLaunchKernelGGL(transpose_rowptr_kernel, dim3(blocks_c), dim3(256), 0, stream, keys_in, nnz, n_cols, t_rowptr);
    // source rows: the bucket table takes the place of the histograms, the rows of the positions that of the key
    // buffer the sorted columns are not in
    const int64_t n_buckets = (nnz + kRowBucket - 1) / kRowBucket;
    int32_t* bucket_row = hist;
    int32_t* row_of = keys_in == keys_a ? keys_b : keys_a;
    hipLaunchKernelGGL(bucket_rows_kernel, dim3((unsigned)((n_buckets + 1 + 255) / 256)), dim3(256), 0, stream, rowptr, n_rows, nnz,
                       n_buckets, bucket_row);
    hipLaunchKernelGGL(position_rows_kernel, dim3(blocks_n), dim3(256), 0, stream, rowptr, nnz, bucket_row, row_of);
    hipLaunchKernelGGL(transpose_fill_kernel, dim3(blocks_n), dim3(256), 0, stream, perm, nnz, row_of, val, t_colind, t_val);
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

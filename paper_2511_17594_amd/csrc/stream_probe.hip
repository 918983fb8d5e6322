// Plain streaming kernels that measure what the memory system of the device sustains, so that the
// rates of the sparse kernels can be set against a measured ceiling next to the published 8 TB/s:
//   read     every 16-byte vector of src is loaded once, one partial sum per workgroup is written
//   copy     dst = src (one read and one write per byte)
//   inplace  dst = 0.5 * dst, read and written at the same address (the access pattern of an in-place
//            row-softmax)
// Tiles of consecutive 16-byte vectors per workgroup, four loads in flight per lane, non-temporal loads and
// stores (the fastest of the plain variants tried on this chip: strided grids and cached accesses are 10-25 % slower).  The measurement section of the paper
// reports medians of repeated timed launches; the caller times these launches the same way.
#include "device_utils.h"
#include "launch.h"

namespace autosage {
namespace {

constexpr int kProbeUnroll = 4;
constexpr int64_t kProbeTile = 256 * kProbeUnroll;      // vectors one workgroup takes per step

// Workgroup b takes the tiles b, b + gridDim.x, ... of kProbeTile consecutive vectors: every wavefront
// load covers 1 KiB of consecutive bytes and a workgroup has 16 KiB in flight.
__global__ void __launch_bounds__(256) stream_read_kernel(const stream_f4* __restrict__ src, int64_t n_vec, float* __restrict__ sums)
{
    float acc = 0.f;
    for (int64_t t = (int64_t)blockIdx.x * kProbeTile; t < n_vec; t += (int64_t)gridDim.x * kProbeTile) {
        stream_f4 v[kProbeUnroll];
#pragma unroll
        for (int k = 0; k < kProbeUnroll; ++k) {
            const int64_t i = t + k * 256 + threadIdx.x;
            v[k] = i < n_vec ? __builtin_nontemporal_load(src + i) : stream_f4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int k = 0; k < kProbeUnroll; ++k) acc += (v[k].x + v[k].y) + (v[k].z + v[k].w);
    }
    acc = group_sum<kWave>(acc);
    __shared__ float part[4];
    if ((threadIdx.x & (kWave - 1)) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) sums[blockIdx.x] = (part[0] + part[1]) + (part[2] + part[3]);
}

template <bool IN_PLACE>
__global__ void __launch_bounds__(256) stream_write_kernel(const stream_f4* src, stream_f4* dst, int64_t n_vec)
{
    for (int64_t t = (int64_t)blockIdx.x * kProbeTile; t < n_vec; t += (int64_t)gridDim.x * kProbeTile) {
        stream_f4 v[kProbeUnroll];
#pragma unroll
        for (int k = 0; k < kProbeUnroll; ++k) {
            const int64_t i = t + k * 256 + threadIdx.x;
            if (i < n_vec) v[k] = __builtin_nontemporal_load(src + i);
        }
#pragma unroll
        for (int k = 0; k < kProbeUnroll; ++k) {
            const int64_t i = t + k * 256 + threadIdx.x;
            if (i < n_vec) {
                if (IN_PLACE) v[k] *= 0.5f;
                __builtin_nontemporal_store(v[k], dst + i);
            }
        }
    }
}

// Random-row gather: n_idx reads of whole rows of G 16-byte vectors out of a table, in the access pattern of
// the sparse kernels (64 indices per coalesced load, handed to lane groups of G lanes, 64 / G rows per wavefront
// load, U loads in flight per lane, cached loads).  Every vector read is added into a per-workgroup sum so that
// the loads cannot be dropped.  Indices are clamped into the table.
template <int G>
__global__ void __launch_bounds__(256) gather_probe_kernel(const stream_f4* __restrict__ table, int32_t n_table_rows,
                                                           const int32_t* __restrict__ idx, int64_t n_idx,
                                                           float* __restrict__ sums)
{
    constexpr int S = kWave / G;
    constexpr int U = 4;
    const int lane = threadIdx.x & (kWave - 1);
    const int g = lane / G;
    const int l = lane - g * G;
    const int64_t n_blocks = (n_idx + kWave - 1) / kWave;
    const int64_t wave_id = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t n_waves = (int64_t)gridDim.x * 4;
    float acc = 0.f;
    for (int64_t b = wave_id; b < n_blocks; b += n_waves) {
        const int64_t base = b * kWave;
        const int n = (int)(n_idx - base < kWave ? n_idx - base : kWave);
        int my_c = idx[base + (lane < n ? lane : n - 1)];
        my_c = my_c < 0 ? 0 : (my_c >= n_table_rows ? n_table_rows - 1 : my_c);
        for (int jj = 0; jj < n; jj += S * U) {
            stream_f4 v[U];
            bool ok[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int j = jj + u * S + g;
                ok[u] = j < n;
                const int c = lane_get(my_c, ok[u] ? j : n - 1);
                v[u] = table[(int64_t)c * G + l];
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (ok[u]) acc += (v[u].x + v[u].y) + (v[u].z + v[u].w);
        }
    }
    acc = group_sum<kWave>(acc);
    __shared__ float part[4];
    if (lane == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) sums[blockIdx.x] = (part[0] + part[1]) + (part[2] + part[3]);
}

template <int G>
hipError_t run_gather(int blocks, const void* table, int32_t n_rows, const int32_t* idx, int64_t n_idx, float* sums,
                      hipStream_t stream)
{
    hipLaunchKernelGGL(gather_probe_kernel<G>, dim3(blocks), dim3(256), 0, stream, static_cast<const stream_f4*>(table), n_rows,
                       idx, n_idx, sums);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gather_probe(int blocks, const void* table, int32_t n_table_rows, int32_t row_bytes, const int32_t* idx,
                               int64_t n_idx, float* sums, hipStream_t stream)
{
    switch (row_bytes / 16) {
        case 1: return run_gather<1>(blocks, table, n_table_rows, idx, n_idx, sums, stream);
        case 2: return run_gather<2>(blocks, table, n_table_rows, idx, n_idx, sums, stream);
        case 4: return run_gather<4>(blocks, table, n_table_rows, idx, n_idx, sums, stream);
        case 8: return run_gather<8>(blocks, table, n_table_rows, idx, n_idx, sums, stream);
        case 16: return run_gather<16>(blocks, table, n_table_rows, idx, n_idx, sums, stream);
        case 32: return run_gather<32>(blocks, table, n_table_rows, idx, n_idx, sums, stream);
        case 64: return run_gather<64>(blocks, table, n_table_rows, idx, n_idx, sums, stream);
        default: return hipErrorInvalidValue;
    }
}

int stream_probe_blocks(int cu_count) { return (cu_count > 0 ? cu_count : 256) * 32; }

hipError_t launch_stream_probe(int mode, int blocks, const void* src, void* dst, int64_t n_vec, hipStream_t stream)
{
    const dim3 grid(blocks), block(256);
    if (mode == 0) {
        hipLaunchKernelGGL(stream_read_kernel, grid, block, 0, stream, static_cast<const stream_f4*>(src), n_vec,
                           static_cast<float*>(dst));
    } else if (mode == 1) {
        hipLaunchKernelGGL(stream_write_kernel<false>, grid, block, 0, stream, static_cast<const stream_f4*>(src),
                           static_cast<stream_f4*>(dst), n_vec);
    } else {
        hipLaunchKernelGGL(stream_write_kernel<true>, grid, block, 0, stream, static_cast<const stream_f4*>(dst),
                           static_cast<stream_f4*>(dst), n_vec);
    }
    return hipGetLastError();
}

}  // namespace autosage

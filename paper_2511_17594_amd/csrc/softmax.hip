// CSR row-softmax for gfx950 (paper, Method / Kernel templates: numerically stable row-softmax
// used between the SDDMM and SpMM stages of CSR attention).
//
// Scores are [nnz, H] with the head index minor.  For every row and head:
//   m = max_p s[p,h];  out[p,h] = exp(s[p,h] - m) / sum_q exp(s[q,h] - m).
// A wavefront owns a row: lane = pl * HP + hh, hh = head inside the current pass of HP heads
// (HP = power of two >= min(H, 64)), pl = which of the 64/HP entries of a step.  Rows whose
// scores fit the lanes' registers are read once; longer rows use a running (max, sum) pass
// followed by a normalising pass.  Hub rows are split into chunks: one workgroup per chunk
// produces a (max, sum) pair per head, and a second kernel merges the pairs of a row in
// ascending chunk order and normalises its chunk.
#include "device_utils.h"
#include "launch.h"

namespace autosage {
namespace {

constexpr int kRegs = 8;   // entries per lane kept in registers by the single-read path

struct SoftmaxDev {
    RowMap rows;
    const int32_t* __restrict__ rowptr;
    const float* in;        // may alias out
    float* out;
    int32_t H;
    int32_t hp_shift;       // log2(HP)
    int32_t hub_t;
    int32_t hub_chunk;
    const HubCounts* __restrict__ counts;
    const int32_t* __restrict__ hub_rows;
    const int32_t* __restrict__ chunk_ptr;
    float* part;            // [cap_chunks, H, 2]
};

struct MaxSum {
    float m, l;             // running maximum and sum of exp(s - m)
};

__device__ __forceinline__ MaxSum ms_empty() { return {-INFINITY, 0.f}; }

__device__ __forceinline__ void ms_push(MaxSum& a, float s)
{
    if (s > a.m) {
        a.l = a.l * __expf(a.m - s) + 1.f;      // exp(-inf) = 0 on the first push
        a.m = s;
    } else {
        a.l += __expf(s - a.m);
    }
}

// Merge b into a (a stays the left operand, so a fixed call order gives a fixed result).
__device__ __forceinline__ void ms_merge(MaxSum& a, const MaxSum& b)
{
    const float m = fmaxf(a.m, b.m);
    if (m == -INFINITY) return;                 // both empty
    a.l = a.l * __expf(a.m - m) + b.l * __expf(b.m - m);
    a.m = m;
}

// Merge over the lanes of a wavefront that hold the same head (lane % HP); every such lane gets the result.
__device__ __forceinline__ MaxSum ms_wave_merge(MaxSum a, int HP)
{
    for (int off = HP; off < kWave; off <<= 1) {
        MaxSum b;
        b.m = __shfl_xor(a.m, off, kWave);
        b.l = __shfl_xor(a.l, off, kWave);
        // symmetric form so that both partners compute bit-identical results
        const float m = fmaxf(a.m, b.m);
        if (m != -INFINITY) {
            const float la = a.l * __expf(a.m - m);
            const float lb = b.l * __expf(b.m - m);
            a.l = la + lb;
            a.m = m;
        }
    }
    return a;
}

__global__ void __launch_bounds__(1024) softmax_rows_kernel(SoftmaxDev a)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int idx = wave_uniform(blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6));
    if (idx >= a.rows.count) return;
    const int row = row_of(a.rows, idx);
    const int p0 = wave_uniform(a.rowptr[row]);
    const int p1 = wave_uniform(a.rowptr[row + 1]);
    const int deg = p1 - p0;
    if (deg <= 0) return;
    if (a.hub_t > 0 && deg >= a.hub_t) return;
    const int HP = 1 << a.hp_shift;
    const int PL = kWave >> a.hp_shift;
    const int hh = lane & (HP - 1);
    const int pl = lane >> a.hp_shift;
    for (int hp = 0; hp < a.H; hp += HP) {
        const int h = hp + hh;
        const bool hv = h < a.H;
        if (deg <= PL * kRegs) {
            float s[kRegs];
            MaxSum acc = ms_empty();
#pragma unroll
            for (int r = 0; r < kRegs; ++r) {
                const int p = p0 + r * PL + pl;
                const bool ok = hv && p < p1;
                s[r] = ok ? a.in[(int64_t)p * a.H + h] : -INFINITY;
            }
            float m = s[0];
#pragma unroll
            for (int r = 1; r < kRegs; ++r) m = fmaxf(m, s[r]);
            for (int off = HP; off < kWave; off <<= 1) m = fmaxf(m, __shfl_xor(m, off, kWave));
            float l = 0.f;
#pragma unroll
            for (int r = 0; r < kRegs; ++r) {
                s[r] = (s[r] == -INFINITY) ? 0.f : __expf(s[r] - m);
                l += s[r];
            }
            for (int off = HP; off < kWave; off <<= 1) l += __shfl_xor(l, off, kWave);
            const float inv = 1.f / l;
#pragma unroll
            for (int r = 0; r < kRegs; ++r) {
                const int p = p0 + r * PL + pl;
                if (hv && p < p1) a.out[(int64_t)p * a.H + h] = s[r] * inv;
            }
            (void)acc;
        } else {
            MaxSum acc = ms_empty();
            if (hv) {
                for (int p = p0 + pl; p < p1; p += PL) ms_push(acc, a.in[(int64_t)p * a.H + h]);
            }
            acc = ms_wave_merge(acc, HP);
            const float inv = 1.f / acc.l;
            if (hv) {
                for (int p = p0 + pl; p < p1; p += PL) {
                    const int64_t e = (int64_t)p * a.H + h;
                    a.out[e] = __expf(a.in[e] - acc.m) * inv;
                }
            }
        }
    }
}

__device__ __forceinline__ int softmax_upper_slot(const int32_t* __restrict__ ptr, int n, int x)
{
    int lo = 0, hi = n;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (ptr[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

// One workgroup per chunk: (max, sum) of the chunk's scores for every head.
__global__ void __launch_bounds__(1024) softmax_hub_partial_kernel(SoftmaxDev a)
{
    __shared__ float lds_m[16 * kWave];
    __shared__ float lds_l[16 * kWave];
    const int chunk = blockIdx.x;
    if (chunk >= a.counts->n_chunks) return;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int wpg = blockDim.x >> 6;
    const int k_hub = softmax_upper_slot(a.chunk_ptr, a.counts->n_hub, chunk);
    const int row = row_of(a.rows, a.hub_rows[k_hub]);
    const int t = chunk - a.chunk_ptr[k_hub];
    const int q0 = a.rowptr[row] + t * a.hub_chunk;
    const int q1 = min(q0 + a.hub_chunk, a.rowptr[row + 1]);
    const int HP = 1 << a.hp_shift;
    const int PL = kWave >> a.hp_shift;
    const int hh = lane & (HP - 1);
    const int pl = lane >> a.hp_shift;
    for (int hp = 0; hp < a.H; hp += HP) {
        const int h = hp + hh;
        const bool hv = h < a.H;
        MaxSum acc = ms_empty();
        if (hv) {
            for (int p = q0 + wave * PL + pl; p < q1; p += wpg * PL) ms_push(acc, a.in[(int64_t)p * a.H + h]);
        }
        acc = ms_wave_merge(acc, HP);
        if (pl == 0) {
            lds_m[wave * kWave + hh] = acc.m;
            lds_l[wave * kWave + hh] = acc.l;
        }
        __syncthreads();
        if (wave == 0 && pl == 0 && hv) {
            MaxSum tot = {lds_m[hh], lds_l[hh]};
            for (int w = 1; w < wpg; ++w) {                 // fixed wavefront order
                MaxSum b = {lds_m[w * kWave + hh], lds_l[w * kWave + hh]};
                ms_merge(tot, b);
            }
            a.part[((int64_t)chunk * a.H + h) * 2 + 0] = tot.m;
            a.part[((int64_t)chunk * a.H + h) * 2 + 1] = tot.l;
        }
        __syncthreads();
    }
}

// One workgroup per chunk: merge the (max, sum) pairs of the row's chunks in ascending order, then normalise.
__global__ void __launch_bounds__(1024) softmax_hub_normalise_kernel(SoftmaxDev a)
{
    const int chunk = blockIdx.x;
    if (chunk >= a.counts->n_chunks) return;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int wpg = blockDim.x >> 6;
    const int k_hub = softmax_upper_slot(a.chunk_ptr, a.counts->n_hub, chunk);
    const int row = row_of(a.rows, a.hub_rows[k_hub]);
    const int c0 = a.chunk_ptr[k_hub];
    const int c1 = a.chunk_ptr[k_hub + 1];
    const int t = chunk - c0;
    const int q0 = a.rowptr[row] + t * a.hub_chunk;
    const int q1 = min(q0 + a.hub_chunk, a.rowptr[row + 1]);
    const int HP = 1 << a.hp_shift;
    const int PL = kWave >> a.hp_shift;
    const int hh = lane & (HP - 1);
    const int pl = lane >> a.hp_shift;
    for (int hp = 0; hp < a.H; hp += HP) {
        const int h = hp + hh;
        if (h >= a.H) continue;
        MaxSum tot = ms_empty();
        for (int c = c0; c < c1; ++c) {
            MaxSum b = {a.part[((int64_t)c * a.H + h) * 2 + 0], a.part[((int64_t)c * a.H + h) * 2 + 1]};
            ms_merge(tot, b);
        }
        const float inv = 1.f / tot.l;
        for (int p = q0 + wave * PL + pl; p < q1; p += wpg * PL) {
            const int64_t e = (int64_t)p * a.H + h;
            a.out[e] = __expf(a.in[e] - tot.m) * inv;
        }
    }
}

// ---- backward: dS = P * (dP - sum_q P_q dP_q) per row and head ------------------------------------
struct SoftmaxBwdDev {
    RowMap rows;
    const int32_t* __restrict__ rowptr;
    const float* P;
    const float* dP;        // may alias dS
    float* dS;
    float scale;
    int32_t H;
    int32_t hp_shift;
    int32_t hub_t;
    int32_t hub_chunk;
    const HubCounts* __restrict__ counts;
    const int32_t* __restrict__ hub_rows;
    const int32_t* __restrict__ chunk_ptr;
    float* part;            // [cap_chunks, H] partial dots
};

__global__ void __launch_bounds__(1024) softmax_bwd_rows_kernel(SoftmaxBwdDev a)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int idx = wave_uniform(blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6));
    if (idx >= a.rows.count) return;
    const int row = row_of(a.rows, idx);
    const int p0 = wave_uniform(a.rowptr[row]);
    const int p1 = wave_uniform(a.rowptr[row + 1]);
    const int deg = p1 - p0;
    if (deg <= 0) return;
    if (a.hub_t > 0 && deg >= a.hub_t) return;
    const int HP = 1 << a.hp_shift;
    const int PL = kWave >> a.hp_shift;
    const int hh = lane & (HP - 1);
    const int pl = lane >> a.hp_shift;
    for (int hp = 0; hp < a.H; hp += HP) {
        const int h = hp + hh;
        const bool hv = h < a.H;
        float dot = 0.f;
        if (hv) {
            for (int p = p0 + pl; p < p1; p += PL) {
                const int64_t e = (int64_t)p * a.H + h;
                dot = fmaf(a.P[e], a.dP[e], dot);
            }
        }
        for (int off = HP; off < kWave; off <<= 1) dot += __shfl_xor(dot, off, kWave);
        if (hv) {
            for (int p = p0 + pl; p < p1; p += PL) {
                const int64_t e = (int64_t)p * a.H + h;
                a.dS[e] = a.scale * (a.P[e] * (a.dP[e] - dot));
            }
        }
    }
}

__global__ void __launch_bounds__(1024) softmax_bwd_hub_partial_kernel(SoftmaxBwdDev a)
{
    __shared__ float lds[16 * kWave];
    const int chunk = blockIdx.x;
    if (chunk >= a.counts->n_chunks) return;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int wpg = blockDim.x >> 6;
    const int k_hub = softmax_upper_slot(a.chunk_ptr, a.counts->n_hub, chunk);
    const int row = row_of(a.rows, a.hub_rows[k_hub]);
    const int t = chunk - a.chunk_ptr[k_hub];
    const int q0 = a.rowptr[row] + t * a.hub_chunk;
    const int q1 = min(q0 + a.hub_chunk, a.rowptr[row + 1]);
    const int HP = 1 << a.hp_shift;
    const int PL = kWave >> a.hp_shift;
    const int hh = lane & (HP - 1);
    const int pl = lane >> a.hp_shift;
    for (int hp = 0; hp < a.H; hp += HP) {
        const int h = hp + hh;
        const bool hv = h < a.H;
        float dot = 0.f;
        if (hv) {
            for (int p = q0 + wave * PL + pl; p < q1; p += wpg * PL) {
                const int64_t e = (int64_t)p * a.H + h;
                dot = fmaf(a.P[e], a.dP[e], dot);
            }
        }
        for (int off = HP; off < kWave; off <<= 1) dot += __shfl_xor(dot, off, kWave);
        if (pl == 0) lds[wave * kWave + hh] = dot;
        __syncthreads();
        if (wave == 0 && pl == 0 && hv) {
            float tot = lds[hh];
            for (int w = 1; w < wpg; ++w) tot += lds[w * kWave + hh];       // fixed wavefront order
            a.part[(int64_t)chunk * a.H + h] = tot;
        }
        __syncthreads();
    }
}

__global__ void __launch_bounds__(1024) softmax_bwd_hub_apply_kernel(SoftmaxBwdDev a)
{
    const int chunk = blockIdx.x;
    if (chunk >= a.counts->n_chunks) return;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int wpg = blockDim.x >> 6;
    const int k_hub = softmax_upper_slot(a.chunk_ptr, a.counts->n_hub, chunk);
    const int row = row_of(a.rows, a.hub_rows[k_hub]);
    const int c0 = a.chunk_ptr[k_hub];
    const int c1 = a.chunk_ptr[k_hub + 1];
    const int t = chunk - c0;
    const int q0 = a.rowptr[row] + t * a.hub_chunk;
    const int q1 = min(q0 + a.hub_chunk, a.rowptr[row + 1]);
    const int HP = 1 << a.hp_shift;
    const int PL = kWave >> a.hp_shift;
    const int hh = lane & (HP - 1);
    const int pl = lane >> a.hp_shift;
    for (int hp = 0; hp < a.H; hp += HP) {
        const int h = hp + hh;
        if (h >= a.H) continue;
        float dot = 0.f;
        for (int c = c0; c < c1; ++c) dot += a.part[(int64_t)c * a.H + h];   // ascending chunk order
        for (int p = q0 + wave * PL + pl; p < q1; p += wpg * PL) {
            const int64_t e = (int64_t)p * a.H + h;
            a.dS[e] = a.scale * (a.P[e] * (a.dP[e] - dot));
        }
    }
}

inline int log2_ceil_pow2(int x)
{
    int s = 0;
    while ((1 << s) < x) ++s;
    return s;
}

inline SoftmaxDev make_dev(const SoftmaxArgs& a)
{
    SoftmaxDev d{};
    d.rows = a.rows;
    d.rowptr = a.rowptr;
    d.in = a.in;
    d.out = a.out;
    d.H = a.H;
    d.hp_shift = log2_ceil_pow2(a.H < kWave ? a.H : kWave);
    return d;
}

}  // namespace

hipError_t launch_softmax_rows(const SoftmaxArgs& a, int32_t hub_t, int32_t wpg, hipStream_t stream)
{
    SoftmaxDev d = make_dev(a);
    d.hub_t = hub_t;
    const int n_blocks = (a.rows.count + wpg - 1) / wpg;
    if (n_blocks == 0) return hipSuccess;
    hipLaunchKernelGGL(softmax_rows_kernel, dim3(n_blocks), dim3(wpg * kWave), 0, stream, d);
    return hipGetLastError();
}

hipError_t launch_softmax_hub(const SoftmaxArgs& a, int32_t hub_chunk, const HubMeta& meta, float* part, hipStream_t stream)
{
    if (meta.cap_hub == 0 || meta.cap_chunks == 0) return hipSuccess;
    SoftmaxDev d = make_dev(a);
    d.hub_chunk = hub_chunk;
    d.counts = meta.counts;
    d.hub_rows = meta.hub_rows;
    d.chunk_ptr = meta.chunk_ptr;
    d.part = part;
    hipLaunchKernelGGL(softmax_hub_partial_kernel, dim3(meta.cap_chunks), dim3(256), 0, stream, d);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(softmax_hub_normalise_kernel, dim3(meta.cap_chunks), dim3(256), 0, stream, d);
    return hipGetLastError();
}

hipError_t launch_softmax_bwd(const SoftmaxBwdArgs& a, int32_t hub_t, int32_t hub_chunk, const HubMeta* meta, float* part,
                              hipStream_t stream)
{
    SoftmaxBwdDev d{};
    d.rows = a.rows;
    d.rowptr = a.rowptr;
    d.P = a.P;
    d.dP = a.dP;
    d.dS = a.dS;
    d.scale = a.scale == 0.f ? 1.f : a.scale;
    d.H = a.H;
    d.hp_shift = log2_ceil_pow2(a.H < kWave ? a.H : kWave);
    d.hub_t = hub_t;
    d.hub_chunk = hub_chunk;
    const int n_blocks = (a.rows.count + 3) / 4;
    if (n_blocks == 0) return hipSuccess;
    hipLaunchKernelGGL(softmax_bwd_rows_kernel, dim3(n_blocks), dim3(4 * kWave), 0, stream, d);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || hub_t <= 0 || !meta || meta->cap_chunks == 0 || meta->cap_hub == 0) return e;
    d.counts = meta->counts;
    d.hub_rows = meta->hub_rows;
    d.chunk_ptr = meta->chunk_ptr;
    d.part = part;
    hipLaunchKernelGGL(softmax_bwd_hub_partial_kernel, dim3(meta->cap_chunks), dim3(256), 0, stream, d);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(softmax_bwd_hub_apply_kernel, dim3(meta->cap_chunks), dim3(256), 0, stream, d);
    return hipGetLastError();
}

}  // namespace autosage

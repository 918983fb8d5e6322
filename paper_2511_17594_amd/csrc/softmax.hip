// CSR row-softmax for gfx950 (paper, Method / Kernel templates: numerically stable row-softmax
// used between the SDDMM and SpMM stages of CSR attention).
//
// Scores are [nnz, H] with the head index minor.  For every row and head:
//   m = max_p s[p,h];  out[p,h] = exp(s[p,h] - m) / sum_q exp(s[q,h] - m).
// A wavefront owns a row: lane = pl * HP + hh, hh = head inside the current pass of HP heads
// (HP = power of two >= min(H, 64)), pl = which of the 64/HP entries of a step.  Rows whose
// scores fit the lanes' registers are read once; longer rows use a running (max, sum) pass
// followed by a normalising pass.  Hub rows are split into chunks: one workgroup per chunk
// produces a (max, sum) pair per head, one wavefront per hub row merges the pairs of the row in
// a fixed order, and a third kernel normalises chunk by chunk.
//
// Power-of-two head counts (the usual case) take the lane-group kernels further down: 16-byte loads,
// several short rows per wavefront, long rows taken by the whole wavefront one after the other.
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
    int32_t hs_shift;       // lane-group kernels: log2(H / VEC), vectors per entry
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
    const int k_hub = wave_upper_slot(a.chunk_ptr, a.counts->n_hub, chunk);
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

// One wavefront per hub row: merges the (max, sum) pairs of the row's chunks and leaves the row's total in
// the slot of its first chunk.  Lane pl * HP + hh takes head hh of the chunks c0 + pl, c0 + pl + PL, ... in
// ascending order; the lanes of a head are then merged by a fixed butterfly.
__global__ void __launch_bounds__(256) softmax_hub_merge_kernel(SoftmaxDev a)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int k_hub = wave_uniform(blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6));
    if (k_hub >= a.counts->n_hub) return;
    const int c0 = a.chunk_ptr[k_hub];
    const int c1 = a.chunk_ptr[k_hub + 1];
    if (c1 - c0 <= 1) return;                               // the only chunk already holds the total
    const int HP = 1 << a.hp_shift;
    const int PL = kWave >> a.hp_shift;
    const int hh = lane & (HP - 1);
    const int pl = lane >> a.hp_shift;
    for (int hp = 0; hp < a.H; hp += HP) {
        const int h = hp + hh;
        const bool hv = h < a.H;
        // maximum first, then the sum: the loads of both loops do not wait for the arithmetic
        float m = -INFINITY;
        if (hv) {
            for (int c = c0 + pl; c < c1; c += PL) m = fmaxf(m, a.part[((int64_t)c * a.H + h) * 2]);
        }
        for (int off = HP; off < kWave; off <<= 1) m = fmaxf(m, __shfl_xor(m, off, kWave));
        float l = 0.f;
        if (hv && m > -INFINITY) {
            for (int c = c0 + pl; c < c1; c += PL) {
                const float* pr = a.part + ((int64_t)c * a.H + h) * 2;
                l += pr[1] * __expf(pr[0] - m);
            }
        }
        for (int off = HP; off < kWave; off <<= 1) l += __shfl_xor(l, off, kWave);
        if (hv && pl == 0) {
            a.part[((int64_t)c0 * a.H + h) * 2 + 0] = m;
            a.part[((int64_t)c0 * a.H + h) * 2 + 1] = l;
        }
    }
}

// One workgroup per chunk: normalise with the row's total (left in the slot of the row's first chunk).
__global__ void __launch_bounds__(1024) softmax_hub_normalise_kernel(SoftmaxDev a)
{
    const int chunk = blockIdx.x;
    if (chunk >= a.counts->n_chunks) return;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int wpg = blockDim.x >> 6;
    const int k_hub = wave_upper_slot(a.chunk_ptr, a.counts->n_hub, chunk);
    const int row = row_of(a.rows, a.hub_rows[k_hub]);
    const int c0 = a.chunk_ptr[k_hub];
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
        const MaxSum tot = {a.part[((int64_t)c0 * a.H + h) * 2 + 0], a.part[((int64_t)c0 * a.H + h) * 2 + 1]};   // row total
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
    int32_t hs_shift;       // lane-group kernels: log2(H / VEC), vectors per entry
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
    const int k_hub = wave_upper_slot(a.chunk_ptr, a.counts->n_hub, chunk);
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

// One wavefront per hub row: the row's dot product, left in the slot of its first chunk (lane layout and
// order as in softmax_hub_merge_kernel).
__global__ void __launch_bounds__(256) softmax_bwd_hub_merge_kernel(SoftmaxBwdDev a)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int k_hub = wave_uniform(blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6));
    if (k_hub >= a.counts->n_hub) return;
    const int c0 = a.chunk_ptr[k_hub];
    const int c1 = a.chunk_ptr[k_hub + 1];
    if (c1 - c0 <= 1) return;
    const int HP = 1 << a.hp_shift;
    const int PL = kWave >> a.hp_shift;
    const int hh = lane & (HP - 1);
    const int pl = lane >> a.hp_shift;
    for (int hp = 0; hp < a.H; hp += HP) {
        const int h = hp + hh;
        const bool hv = h < a.H;
        float dot = 0.f;
        if (hv) {
            for (int c = c0 + pl; c < c1; c += PL) dot += a.part[(int64_t)c * a.H + h];
        }
        for (int off = HP; off < kWave; off <<= 1) dot += __shfl_xor(dot, off, kWave);
        if (hv && pl == 0) a.part[(int64_t)c0 * a.H + h] = dot;
    }
}

__global__ void __launch_bounds__(1024) softmax_bwd_hub_apply_kernel(SoftmaxBwdDev a)
{
    const int chunk = blockIdx.x;
    if (chunk >= a.counts->n_chunks) return;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int wpg = blockDim.x >> 6;
    const int k_hub = wave_upper_slot(a.chunk_ptr, a.counts->n_hub, chunk);
    const int row = row_of(a.rows, a.hub_rows[k_hub]);
    const int c0 = a.chunk_ptr[k_hub];
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
        const float dot = a.part[(int64_t)c0 * a.H + h];                     // row total
        for (int p = q0 + wave * PL + pl; p < q1; p += wpg * PL) {
            const int64_t e = (int64_t)p * a.H + h;
            a.dS[e] = a.scale * (a.P[e] * (a.dP[e] - dot));
        }
    }
}

// ---- lane-group kernels for power-of-two head counts ----------------------------------------------
// The scores of a row are deg * H contiguous floats.  They are read as vectors of VEC = min(H, 4)
// floats; hs = H / VEC consecutive vectors make one entry, so vector v of the row holds the heads
// (v % hs) * VEC ... of entry v / hs.  A group of G lanes (G >= hs, both powers of two) owns a row:
// lane j reads the vectors j, j + G, j + 2G, ... of the row, which all hold the same heads, and
// shares those heads with the lanes j +- hs, j +- 2 hs, ... of its group.  Rows of at most G * R / hs
// entries are read once into registers, 64 / G rows per wavefront; each longer row is then taken by
// the whole wavefront (a group of 64 lanes), so that one long row does not leave the other groups idle.
// Scores that are read once and every result are moved with streaming (non-temporal) accesses; the first
// of two reads of a long row or a hub chunk is an ordinary load, so that the second finds it in the cache.
// Scores that are read once, and every result: streaming accesses when a lane moves 16 bytes.  With narrower
// vectors (H < 4) neighbouring rows share cache lines across lane groups and wavefronts, and the hint makes
// those lines be fetched again (measured: 20-45 % slower at H = 1), so they stay ordinary accesses.
template <int VEC> __device__ __forceinline__ void load_once(const float* p, float* v)
{
    if constexpr (VEC == 4) stream_load_f32<4>(p, v);
    else VecIO<float, VEC>::load(p, v);
}

template <int VEC> __device__ __forceinline__ void store_result(float* p, const float* v)
{
    if constexpr (VEC == 4) stream_store_f32<4>(p, v);
    else store_f32<VEC>(p, v);
}

// exp(x - m) with m given pre-multiplied by log2(e): one fused multiply-add and one v_exp_f32 per element.
constexpr float kLog2e = 1.4426950408889634f;
__device__ __forceinline__ float exp_minus(float x, float m_log2e) { return __builtin_amdgcn_exp2f(fmaf(x, kLog2e, -m_log2e)); }
// 1 / x to one unit in the last place (v_rcp_f32) instead of the ten-instruction IEEE division.
__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }

template <int G> __device__ __forceinline__ float heads_max(float x, int hs)
{
    for (int off = hs; off < G; off <<= 1) x = fmaxf(x, __shfl_xor(x, off, kWave));
    return x;
}

template <int G> __device__ __forceinline__ float heads_sum(float x, int hs)
{
    for (int off = hs; off < G; off <<= 1) x += __shfl_xor(x, off, kWave);
    return x;
}

// Row (position of its first score, number of entries) of every lane group of the wavefront; rows
// past the end, empty rows and rows left to the hub kernels come back with deg = 0.
template <int G>
__device__ __forceinline__ void group_row(const RowMap& rows, const int32_t* __restrict__ rowptr, int hub_t, int lane,
                                          int& p0, int& deg)
{
    const int widx = wave_uniform(blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6));
    const int64_t idx = (int64_t)widx * (kWave / G) + lane / G;
    p0 = 0;
    deg = 0;
    if (idx < rows.count) {
        const int row = row_of(rows, (int32_t)idx);
        p0 = rowptr[row];
        deg = rowptr[row + 1] - p0;
        if (hub_t > 0 && deg >= hub_t) deg = 0;
    }
}

template <int G, int VEC, int R>
__global__ void __launch_bounds__(256) softmax_groups_kernel(SoftmaxDev a)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int j = lane & (G - 1);
    int p0, deg;
    group_row<G>(a.rows, a.rowptr, a.hub_t, lane, p0, deg);
    const int hs = 1 << a.hs_shift;
    const int cap = (G * R) >> a.hs_shift;                      // entries a group keeps in registers
    const bool is_long = deg > cap;
    {
        const int nv = is_long ? 0 : deg << a.hs_shift;         // vectors of this group's row
        const int64_t base = ((int64_t)p0 << a.hs_shift) * VEC;
        float s[R][VEC];
#pragma unroll
        for (int k = 0; k < R; ++k) {
            const int v = k * G + j;
            if (v < nv) {
                load_once<VEC>(a.in + base + (int64_t)v * VEC, s[k]);
            } else {
#pragma unroll
                for (int c = 0; c < VEC; ++c) s[k][c] = -INFINITY;
            }
        }
        float inv[VEC];
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            float m = s[0][c];
#pragma unroll
            for (int k = 1; k < R; ++k) m = fmaxf(m, s[k][c]);
            m = heads_max<G>(m, hs);
            const float m2 = m * kLog2e;
            float l = 0.f;
#pragma unroll
            for (int k = 0; k < R; ++k) {
                s[k][c] = exp_minus(s[k][c], m2);                // exp(-inf) = 0 for the padding
                l += s[k][c];
            }
            inv[c] = fast_rcp(heads_sum<G>(l, hs));
        }
#pragma unroll
        for (int k = 0; k < R; ++k) {
            const int v = k * G + j;
            if (v < nv) {
#pragma unroll
                for (int c = 0; c < VEC; ++c) s[k][c] *= inv[c];
                store_result<VEC>(a.out + base + (int64_t)v * VEC, s[k]);
            }
        }
    }
    // long rows, one after the other, all 64 lanes on each
    uint64_t todo = __ballot(is_long && j == 0);
    while (todo) {
        const int leader = __builtin_ctzll(todo);
        todo &= todo - 1;
        const int64_t nv = (int64_t)lane_get_uniform(deg, leader) << a.hs_shift;
        const int64_t base = ((int64_t)lane_get_uniform(p0, leader) << a.hs_shift) * VEC;
        if (nv <= kWave * R) {
            // the row fits the registers of the wavefront: read once
            float s[R][VEC];
#pragma unroll
            for (int k = 0; k < R; ++k) {
                const int64_t v = k * kWave + lane;
                if (v < nv) {
                    load_once<VEC>(a.in + base + v * VEC, s[k]);
                } else {
#pragma unroll
                    for (int c = 0; c < VEC; ++c) s[k][c] = -INFINITY;
                }
            }
            float inv[VEC];
#pragma unroll
            for (int c = 0; c < VEC; ++c) {
                float m = s[0][c];
#pragma unroll
                for (int k = 1; k < R; ++k) m = fmaxf(m, s[k][c]);
                m = heads_max<kWave>(m, hs);
                const float m2 = m * kLog2e;
                float l = 0.f;
#pragma unroll
                for (int k = 0; k < R; ++k) {
                    s[k][c] = exp_minus(s[k][c], m2);
                    l += s[k][c];
                }
                inv[c] = fast_rcp(heads_sum<kWave>(l, hs));
            }
#pragma unroll
            for (int k = 0; k < R; ++k) {
                const int64_t v = k * kWave + lane;
                if (v < nv) {
#pragma unroll
                    for (int c = 0; c < VEC; ++c) s[k][c] *= inv[c];
                    store_result<VEC>(a.out + base + v * VEC, s[k]);
                }
            }
            continue;
        }
        MaxSum acc[VEC];
#pragma unroll
        for (int c = 0; c < VEC; ++c) acc[c] = ms_empty();
        for (int64_t v0 = 0; v0 < nv; v0 += kWave * R) {
            float s[R][VEC];
#pragma unroll
            for (int k = 0; k < R; ++k) {
                const int64_t v = v0 + k * kWave + lane;
                if (v < nv) {
                    VecIO<float, VEC>::load(a.in + base + v * VEC, s[k]);
                } else {
#pragma unroll
                    for (int c = 0; c < VEC; ++c) s[k][c] = -INFINITY;
                }
            }
#pragma unroll
            for (int c = 0; c < VEC; ++c) {
                float m = s[0][c];
#pragma unroll
                for (int k = 1; k < R; ++k) m = fmaxf(m, s[k][c]);
                if (m > acc[c].m) {
                    acc[c].l *= __expf(acc[c].m - m);           // exp(-inf) = 0 while the lane has seen nothing
                    acc[c].m = m;
                }
                if (acc[c].m > -INFINITY) {
                    const float am2 = acc[c].m * kLog2e;
#pragma unroll
                    for (int k = 0; k < R; ++k) acc[c].l += exp_minus(s[k][c], am2);
                }
            }
        }
        float mx[VEC], inv[VEC];
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            const MaxSum t = ms_wave_merge(acc[c], hs);
            mx[c] = t.m * kLog2e;
            inv[c] = fast_rcp(t.l);
        }
        for (int64_t v0 = 0; v0 < nv; v0 += kWave * R) {
            float s[R][VEC];
#pragma unroll
            for (int k = 0; k < R; ++k) {
                const int64_t v = v0 + k * kWave + lane;
                if (v < nv) load_once<VEC>(a.in + base + v * VEC, s[k]);
            }
#pragma unroll
            for (int k = 0; k < R; ++k) {
                const int64_t v = v0 + k * kWave + lane;
                if (v < nv) {
#pragma unroll
                    for (int c = 0; c < VEC; ++c) s[k][c] = exp_minus(s[k][c], mx[c]) * inv[c];
                    store_result<VEC>(a.out + base + v * VEC, s[k]);
                }
            }
        }
    }
}

template <int G, int VEC, int R>
__global__ void __launch_bounds__(256) softmax_bwd_groups_kernel(SoftmaxBwdDev a)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int j = lane & (G - 1);
    int p0, deg;
    group_row<G>(a.rows, a.rowptr, a.hub_t, lane, p0, deg);
    const int hs = 1 << a.hs_shift;
    const int cap = (G * R) >> a.hs_shift;
    const bool is_long = deg > cap;
    {
        const int nv = is_long ? 0 : deg << a.hs_shift;
        const int64_t base = ((int64_t)p0 << a.hs_shift) * VEC;
        float P[R][VEC], dP[R][VEC];
#pragma unroll
        for (int k = 0; k < R; ++k) {
            const int v = k * G + j;
            if (v < nv) {
                load_once<VEC>(a.P + base + (int64_t)v * VEC, P[k]);
                load_once<VEC>(a.dP + base + (int64_t)v * VEC, dP[k]);
            } else {
#pragma unroll
                for (int c = 0; c < VEC; ++c) P[k][c] = dP[k][c] = 0.f;
            }
        }
        float dot[VEC];
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            float t = 0.f;
#pragma unroll
            for (int k = 0; k < R; ++k) t = fmaf(P[k][c], dP[k][c], t);
            dot[c] = heads_sum<G>(t, hs);
        }
#pragma unroll
        for (int k = 0; k < R; ++k) {
            const int v = k * G + j;
            if (v < nv) {
#pragma unroll
                for (int c = 0; c < VEC; ++c) P[k][c] = a.scale * (P[k][c] * (dP[k][c] - dot[c]));
                store_result<VEC>(a.dS + base + (int64_t)v * VEC, P[k]);
            }
        }
    }
    uint64_t todo = __ballot(is_long && j == 0);
    while (todo) {
        const int leader = __builtin_ctzll(todo);
        todo &= todo - 1;
        const int64_t nv = (int64_t)lane_get_uniform(deg, leader) << a.hs_shift;
        const int64_t base = ((int64_t)lane_get_uniform(p0, leader) << a.hs_shift) * VEC;
        if (nv <= kWave * R) {
            // the row fits the registers of the wavefront: read once
            float P[R][VEC], dP[R][VEC];
#pragma unroll
            for (int k = 0; k < R; ++k) {
                const int64_t v = k * kWave + lane;
                if (v < nv) {
                    load_once<VEC>(a.P + base + v * VEC, P[k]);
                    load_once<VEC>(a.dP + base + v * VEC, dP[k]);
                } else {
#pragma unroll
                    for (int c = 0; c < VEC; ++c) P[k][c] = dP[k][c] = 0.f;
                }
            }
            float dot[VEC];
#pragma unroll
            for (int c = 0; c < VEC; ++c) {
                float t = 0.f;
#pragma unroll
                for (int k = 0; k < R; ++k) t = fmaf(P[k][c], dP[k][c], t);
                dot[c] = heads_sum<kWave>(t, hs);
            }
#pragma unroll
            for (int k = 0; k < R; ++k) {
                const int64_t v = k * kWave + lane;
                if (v < nv) {
#pragma unroll
                    for (int c = 0; c < VEC; ++c) P[k][c] = a.scale * (P[k][c] * (dP[k][c] - dot[c]));
                    store_result<VEC>(a.dS + base + v * VEC, P[k]);
                }
            }
            continue;
        }
        float dot[VEC];
#pragma unroll
        for (int c = 0; c < VEC; ++c) dot[c] = 0.f;
        for (int64_t v0 = 0; v0 < nv; v0 += kWave * R) {
            float P[R][VEC], dP[R][VEC];
#pragma unroll
            for (int k = 0; k < R; ++k) {
                const int64_t v = v0 + k * kWave + lane;
                if (v < nv) {
                    VecIO<float, VEC>::load(a.P + base + v * VEC, P[k]);
                    VecIO<float, VEC>::load(a.dP + base + v * VEC, dP[k]);
                } else {
#pragma unroll
                    for (int c = 0; c < VEC; ++c) P[k][c] = dP[k][c] = 0.f;
                }
            }
#pragma unroll
            for (int k = 0; k < R; ++k) {
#pragma unroll
                for (int c = 0; c < VEC; ++c) dot[c] = fmaf(P[k][c], dP[k][c], dot[c]);
            }
        }
#pragma unroll
        for (int c = 0; c < VEC; ++c) dot[c] = heads_sum<kWave>(dot[c], hs);
        for (int64_t v0 = 0; v0 < nv; v0 += kWave * R) {
            float P[R][VEC], dP[R][VEC];
#pragma unroll
            for (int k = 0; k < R; ++k) {
                const int64_t v = v0 + k * kWave + lane;
                if (v < nv) {
                    load_once<VEC>(a.P + base + v * VEC, P[k]);
                    load_once<VEC>(a.dP + base + v * VEC, dP[k]);
                }
            }
#pragma unroll
            for (int k = 0; k < R; ++k) {
                const int64_t v = v0 + k * kWave + lane;
                if (v < nv) {
#pragma unroll
                    for (int c = 0; c < VEC; ++c) P[k][c] = a.scale * (P[k][c] * (dP[k][c] - dot[c]));
                    store_result<VEC>(a.dS + base + v * VEC, P[k]);
                }
            }
        }
    }
}

// ---- hub rows with vector loads (power-of-two head counts) -------------------------------------------
// One workgroup of 256 lanes per chunk.  Lane t reads the vectors t, t + 256, ... of the chunk; 256 is a
// multiple of hs, so a lane keeps the same heads throughout.  Results per chunk and the order in which
// they are merged (lanes by butterfly, wavefronts and chunks ascending) are fixed by the schedule.
constexpr int kHubLanes = 256;
constexpr int kHubR = 4;

struct ChunkSpan {
    int64_t base;       // first float of the chunk in the score array
    int64_t nv;         // vectors in the chunk
    int c0;             // first chunk of the row (its slot holds the row's total after the merge kernel)
};

template <int VEC, typename Dev>
__device__ __forceinline__ ChunkSpan chunk_span(const Dev& a, int chunk)
{
    const int k_hub = wave_upper_slot(a.chunk_ptr, a.counts->n_hub, chunk);
    const int row = row_of(a.rows, a.hub_rows[k_hub]);
    ChunkSpan s;
    s.c0 = a.chunk_ptr[k_hub];
    const int q0 = a.rowptr[row] + (chunk - s.c0) * a.hub_chunk;
    const int q1 = min(q0 + a.hub_chunk, a.rowptr[row + 1]);
    s.base = ((int64_t)q0 << a.hs_shift) * VEC;
    s.nv = (int64_t)(q1 - q0) << a.hs_shift;
    return s;
}

template <int VEC>
__global__ void __launch_bounds__(kHubLanes) softmax_hub_partial_vec_kernel(SoftmaxDev a)
{
    __shared__ float lds_m[(kHubLanes / kWave) * kWave * VEC];
    __shared__ float lds_l[(kHubLanes / kWave) * kWave * VEC];
    const int chunk = blockIdx.x;
    if (chunk >= a.counts->n_chunks) return;
    const ChunkSpan sp = chunk_span<VEC>(a, chunk);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int hs = 1 << a.hs_shift;
    MaxSum acc[VEC];
#pragma unroll
    for (int c = 0; c < VEC; ++c) acc[c] = ms_empty();
    for (int64_t v0 = 0; v0 < sp.nv; v0 += kHubLanes * kHubR) {
        float s[kHubR][VEC];
#pragma unroll
        for (int k = 0; k < kHubR; ++k) {
            const int64_t v = v0 + k * kHubLanes + threadIdx.x;
            if (v < sp.nv) {
                VecIO<float, VEC>::load(a.in + sp.base + v * VEC, s[k]);
            } else {
#pragma unroll
                for (int c = 0; c < VEC; ++c) s[k][c] = -INFINITY;
            }
        }
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            float m = s[0][c];
#pragma unroll
            for (int k = 1; k < kHubR; ++k) m = fmaxf(m, s[k][c]);
            if (m > acc[c].m) {
                acc[c].l *= __expf(acc[c].m - m);
                acc[c].m = m;
            }
            if (acc[c].m > -INFINITY) {
                const float am2 = acc[c].m * kLog2e;
#pragma unroll
                for (int k = 0; k < kHubR; ++k) acc[c].l += exp_minus(s[k][c], am2);
            }
        }
    }
#pragma unroll
    for (int c = 0; c < VEC; ++c) {
        acc[c] = ms_wave_merge(acc[c], hs);
        lds_m[(wave * kWave + lane) * VEC + c] = acc[c].m;
        lds_l[(wave * kWave + lane) * VEC + c] = acc[c].l;
    }
    __syncthreads();
    if (wave == 0 && lane < hs) {
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            MaxSum tot = {lds_m[lane * VEC + c], lds_l[lane * VEC + c]};
            for (int w = 1; w < kHubLanes / kWave; ++w) {          // fixed wavefront order
                const MaxSum b = {lds_m[(w * kWave + lane) * VEC + c], lds_l[(w * kWave + lane) * VEC + c]};
                ms_merge(tot, b);
            }
            const int h = lane * VEC + c;
            a.part[((int64_t)chunk * a.H + h) * 2 + 0] = tot.m;
            a.part[((int64_t)chunk * a.H + h) * 2 + 1] = tot.l;
        }
    }
}

template <int VEC>
__global__ void __launch_bounds__(kHubLanes) softmax_hub_normalise_vec_kernel(SoftmaxDev a)
{
    const int chunk = blockIdx.x;
    if (chunk >= a.counts->n_chunks) return;
    const ChunkSpan sp = chunk_span<VEC>(a, chunk);
    const int h0 = (threadIdx.x & ((1 << a.hs_shift) - 1)) * VEC;
    float mx[VEC], inv[VEC];
#pragma unroll
    for (int c = 0; c < VEC; ++c) {                                // row total, left by the merge kernel
        mx[c] = a.part[((int64_t)sp.c0 * a.H + h0 + c) * 2 + 0] * kLog2e;
        inv[c] = fast_rcp(a.part[((int64_t)sp.c0 * a.H + h0 + c) * 2 + 1]);
    }
    for (int64_t v0 = 0; v0 < sp.nv; v0 += kHubLanes * kHubR) {
        float s[kHubR][VEC];
#pragma unroll
        for (int k = 0; k < kHubR; ++k) {
            const int64_t v = v0 + k * kHubLanes + threadIdx.x;
            if (v < sp.nv) load_once<VEC>(a.in + sp.base + v * VEC, s[k]);
        }
#pragma unroll
        for (int k = 0; k < kHubR; ++k) {
            const int64_t v = v0 + k * kHubLanes + threadIdx.x;
            if (v < sp.nv) {
#pragma unroll
                for (int c = 0; c < VEC; ++c) s[k][c] = exp_minus(s[k][c], mx[c]) * inv[c];
                store_result<VEC>(a.out + sp.base + v * VEC, s[k]);
            }
        }
    }
}

template <int VEC>
__global__ void __launch_bounds__(kHubLanes) softmax_bwd_hub_partial_vec_kernel(SoftmaxBwdDev a)
{
    __shared__ float lds[(kHubLanes / kWave) * kWave * VEC];
    const int chunk = blockIdx.x;
    if (chunk >= a.counts->n_chunks) return;
    const ChunkSpan sp = chunk_span<VEC>(a, chunk);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int hs = 1 << a.hs_shift;
    float dot[VEC];
#pragma unroll
    for (int c = 0; c < VEC; ++c) dot[c] = 0.f;
    for (int64_t v0 = 0; v0 < sp.nv; v0 += kHubLanes * kHubR) {
        float P[kHubR][VEC], dP[kHubR][VEC];
#pragma unroll
        for (int k = 0; k < kHubR; ++k) {
            const int64_t v = v0 + k * kHubLanes + threadIdx.x;
            if (v < sp.nv) {
                VecIO<float, VEC>::load(a.P + sp.base + v * VEC, P[k]);
                VecIO<float, VEC>::load(a.dP + sp.base + v * VEC, dP[k]);
            } else {
#pragma unroll
                for (int c = 0; c < VEC; ++c) P[k][c] = dP[k][c] = 0.f;
            }
        }
#pragma unroll
        for (int k = 0; k < kHubR; ++k) {
#pragma unroll
            for (int c = 0; c < VEC; ++c) dot[c] = fmaf(P[k][c], dP[k][c], dot[c]);
        }
    }
#pragma unroll
    for (int c = 0; c < VEC; ++c) lds[(wave * kWave + lane) * VEC + c] = heads_sum<kWave>(dot[c], hs);
    __syncthreads();
    if (wave == 0 && lane < hs) {
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            float tot = lds[lane * VEC + c];
            for (int w = 1; w < kHubLanes / kWave; ++w) tot += lds[(w * kWave + lane) * VEC + c];   // fixed wavefront order
            a.part[(int64_t)chunk * a.H + lane * VEC + c] = tot;
        }
    }
}

template <int VEC>
__global__ void __launch_bounds__(kHubLanes) softmax_bwd_hub_apply_vec_kernel(SoftmaxBwdDev a)
{
    const int chunk = blockIdx.x;
    if (chunk >= a.counts->n_chunks) return;
    const ChunkSpan sp = chunk_span<VEC>(a, chunk);
    const int h0 = (threadIdx.x & ((1 << a.hs_shift) - 1)) * VEC;
    float dot[VEC];
#pragma unroll
    for (int c = 0; c < VEC; ++c) dot[c] = a.part[(int64_t)sp.c0 * a.H + h0 + c];          // row total, left by the merge kernel
    for (int64_t v0 = 0; v0 < sp.nv; v0 += kHubLanes * kHubR) {
        float P[kHubR][VEC], dP[kHubR][VEC];
#pragma unroll
        for (int k = 0; k < kHubR; ++k) {
            const int64_t v = v0 + k * kHubLanes + threadIdx.x;
            if (v < sp.nv) {
                load_once<VEC>(a.P + sp.base + v * VEC, P[k]);
                load_once<VEC>(a.dP + sp.base + v * VEC, dP[k]);
            }
        }
#pragma unroll
        for (int k = 0; k < kHubR; ++k) {
            const int64_t v = v0 + k * kHubLanes + threadIdx.x;
            if (v < sp.nv) {
#pragma unroll
                for (int c = 0; c < VEC; ++c) P[k][c] = a.scale * (P[k][c] * (dP[k][c] - dot[c]));
                store_result<VEC>(a.dS + sp.base + v * VEC, P[k]);
            }
        }
    }
}

// Vector width of the lane-group kernels for H heads, or 0 when they do not apply (H not a power of
// two, more than 256 heads, or an array that is not aligned for the vector).
inline int group_vec(int H, const void* p0, const void* p1, const void* p2)
{
    if (H <= 0 || (H & (H - 1)) != 0 || H > 256) return 0;
    const int vec = H < 4 ? H : 4;
    const uint64_t bits = reinterpret_cast<uint64_t>(p0) | reinterpret_cast<uint64_t>(p1) | reinterpret_cast<uint64_t>(p2);
    return (bits & (uint64_t)(vec * 4 - 1)) == 0 ? vec : 0;
}

// Lanes per row: the wanted group size, at least the lanes one entry takes.
inline int group_lanes(int want, int hs)
{
    int g = 1;
    while (g < want && g < kWave) g <<= 1;
    return g < hs ? hs : g;
}

template <template <int, int, int> class Launch, typename Dev>
inline void dispatch_groups(int G, int vec, int n_rows, const Dev& d, hipStream_t stream)
{
    const int rpw = kWave / G;
    const int64_t n_waves = ((int64_t)n_rows + rpw - 1) / rpw;
    const dim3 grid((unsigned)((n_waves + 3) / 4)), block(4 * kWave);
#define AUTOSAGE_GROUP_CASE(g)                                                          \
    case g:                                                                             \
        if (vec == 4) Launch<g, 4, 4>::run(grid, block, stream, d);                     \
        else if (vec == 2) Launch<g, 2, 8>::run(grid, block, stream, d);                \
        else Launch<g, 1, 8>::run(grid, block, stream, d);                              \
        break;
    switch (G) {
        AUTOSAGE_GROUP_CASE(1)
        AUTOSAGE_GROUP_CASE(2)
        AUTOSAGE_GROUP_CASE(4)
        AUTOSAGE_GROUP_CASE(8)
        AUTOSAGE_GROUP_CASE(16)
        AUTOSAGE_GROUP_CASE(32)
        default:
        AUTOSAGE_GROUP_CASE(64)
    }
#undef AUTOSAGE_GROUP_CASE
}

template <int G, int VEC, int R> struct LaunchFwd {
    static void run(dim3 grid, dim3 block, hipStream_t st, const SoftmaxDev& d)
    {
        hipLaunchKernelGGL((softmax_groups_kernel<G, VEC, R>), grid, block, 0, st, d);
    }
};
template <int G, int VEC, int R> struct LaunchBwd {
    static void run(dim3 grid, dim3 block, hipStream_t st, const SoftmaxBwdDev& d)
    {
        hipLaunchKernelGGL((softmax_bwd_groups_kernel<G, VEC, R>), grid, block, 0, st, d);
    }
};

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

hipError_t launch_softmax_rows(const SoftmaxArgs& a, int32_t hub_t, int32_t wpg, int32_t group, hipStream_t stream)
{
    SoftmaxDev d = make_dev(a);
    d.hub_t = hub_t;
    if (a.rows.count == 0) return hipSuccess;
    const int vec = group > 0 ? group_vec(a.H, a.in, a.out, nullptr) : 0;
    if (vec > 0) {
        d.hs_shift = log2_ceil_pow2(a.H / vec);
        dispatch_groups<LaunchFwd>(group_lanes(group, a.H / vec), vec, a.rows.count, d, stream);
        return hipGetLastError();
    }
    const int n_blocks = (a.rows.count + wpg - 1) / wpg;
    hipLaunchKernelGGL(softmax_rows_kernel, dim3(n_blocks), dim3(wpg * kWave), 0, stream, d);
    return hipGetLastError();
}

hipError_t launch_softmax_hub(const SoftmaxArgs& a, int32_t hub_chunk, int32_t group, const HubMeta& meta, float* part,
                              hipStream_t stream)
{
    if (meta.cap_hub == 0 || meta.cap_chunks == 0) return hipSuccess;
    SoftmaxDev d = make_dev(a);
    d.hub_chunk = hub_chunk;
    d.counts = meta.counts;
    d.hub_rows = meta.hub_rows;
    d.chunk_ptr = meta.chunk_ptr;
    d.part = part;
    const int vec = group > 0 ? group_vec(a.H, a.in, a.out, nullptr) : 0;
    const dim3 grid(meta.cap_chunks), block(kHubLanes), merge_grid((meta.cap_hub + 3) / 4);
    hipError_t e;
    if (vec > 0) {
        d.hs_shift = log2_ceil_pow2(a.H / vec);
        if (vec == 4) hipLaunchKernelGGL(softmax_hub_partial_vec_kernel<4>, grid, block, 0, stream, d);
        else if (vec == 2) hipLaunchKernelGGL(softmax_hub_partial_vec_kernel<2>, grid, block, 0, stream, d);
        else hipLaunchKernelGGL(softmax_hub_partial_vec_kernel<1>, grid, block, 0, stream, d);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(softmax_hub_merge_kernel, merge_grid, block, 0, stream, d);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        if (vec == 4) hipLaunchKernelGGL(softmax_hub_normalise_vec_kernel<4>, grid, block, 0, stream, d);
        else if (vec == 2) hipLaunchKernelGGL(softmax_hub_normalise_vec_kernel<2>, grid, block, 0, stream, d);
        else hipLaunchKernelGGL(softmax_hub_normalise_vec_kernel<1>, grid, block, 0, stream, d);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(softmax_hub_partial_kernel, grid, block, 0, stream, d);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(softmax_hub_merge_kernel, merge_grid, block, 0, stream, d);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(softmax_hub_normalise_kernel, grid, block, 0, stream, d);
    return hipGetLastError();
}

hipError_t launch_softmax_bwd(const SoftmaxBwdArgs& a, int32_t hub_t, int32_t hub_chunk, int32_t group, const HubMeta* meta,
                              float* part, hipStream_t stream)
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
    const int vec = group > 0 ? group_vec(a.H, a.P, a.dP, a.dS) : 0;
    if (vec > 0) {
        d.hs_shift = log2_ceil_pow2(a.H / vec);
        dispatch_groups<LaunchBwd>(group_lanes(group, a.H / vec), vec, a.rows.count, d, stream);
    } else {
        hipLaunchKernelGGL(softmax_bwd_rows_kernel, dim3(n_blocks), dim3(4 * kWave), 0, stream, d);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || hub_t <= 0 || !meta || meta->cap_chunks == 0 || meta->cap_hub == 0) return e;
    d.counts = meta->counts;
    d.hub_rows = meta->hub_rows;
    d.chunk_ptr = meta->chunk_ptr;
    d.part = part;
    const dim3 grid(meta->cap_chunks), block(kHubLanes), merge_grid((meta->cap_hub + 3) / 4);
    if (vec > 0) {
        if (vec == 4) hipLaunchKernelGGL(softmax_bwd_hub_partial_vec_kernel<4>, grid, block, 0, stream, d);
        else if (vec == 2) hipLaunchKernelGGL(softmax_bwd_hub_partial_vec_kernel<2>, grid, block, 0, stream, d);
        else hipLaunchKernelGGL(softmax_bwd_hub_partial_vec_kernel<1>, grid, block, 0, stream, d);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(softmax_bwd_hub_merge_kernel, merge_grid, block, 0, stream, d);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        if (vec == 4) hipLaunchKernelGGL(softmax_bwd_hub_apply_vec_kernel<4>, grid, block, 0, stream, d);
        else if (vec == 2) hipLaunchKernelGGL(softmax_bwd_hub_apply_vec_kernel<2>, grid, block, 0, stream, d);
        else hipLaunchKernelGGL(softmax_bwd_hub_apply_vec_kernel<1>, grid, block, 0, stream, d);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(softmax_bwd_hub_partial_kernel, grid, block, 0, stream, d);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(softmax_bwd_hub_merge_kernel, merge_grid, block, 0, stream, d);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(softmax_bwd_hub_apply_kernel, grid, block, 0, stream, d);
    return hipGetLastError();
}

}  // namespace autosage

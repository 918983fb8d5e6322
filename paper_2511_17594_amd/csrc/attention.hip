// Single-pass CSR attention launch entry points and the shape rule that says when it applies.
#include "device_utils.h"
#include "launch.h"

namespace autosage {

hipError_t attn_bwd_fused_f32(const AttnBwdArgs&, const AttnShape&, int, const HubMeta*, float*, hipStream_t);
hipError_t attn_bwd_fused_bf16(const AttnBwdArgs&, const AttnShape&, int, const HubMeta*, float*, hipStream_t);
hipError_t attn_bwd_fused_f16(const AttnBwdArgs&, const AttnShape&, int, const HubMeta*, float*, hipStream_t);

hipError_t attn_fused_f32(const AttnArgs&, const AttnShape&, int, const HubMeta*, float*, hipStream_t);
hipError_t attn_fused_bf16(const AttnArgs&, const AttnShape&, int, const HubMeta*, float*, hipStream_t);
hipError_t attn_fused_f16(const AttnArgs&, const AttnShape&, int, const HubMeta*, float*, hipStream_t);

static int pow2_ceil_i(int x)
{
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}

bool attn_fused_shape(int32_t H, int32_t d, int dt, AttnShape* s)
{
    const int vec = 16 / dtype_bytes(dt);
    if (d % vec != 0) return false;
    const int lanes = d / vec;
    if (lanes > 64) return false;
    s->vec = vec;
    s->LH = pow2_ceil_i(lanes);
    const int hp = pow2_ceil_i(H);
    if (hp * s->LH >= 64) {
        s->HW = 64 / s->LH;
        s->KH = (H + s->HW - 1) / s->HW;
        return s->KH <= 2;
    }
    s->HW = hp;
    s->KH = 1;
    return hp * s->LH >= 8;
}

static bool attn_fused_shape_one(int32_t H, int32_t d, int dt, AttnShape* s)
{
    if (!attn_fused_shape(H, d, dt, s)) return false;
    s->heads_tile = H;
    s->tiles = 1;
    return true;
}

bool attn_fused_shape_tiled(int32_t H, int32_t d, int dt, int32_t heads_tile, AttnShape* s)
{
    if (heads_tile <= 0 || heads_tile >= H) return attn_fused_shape_one(H, d, dt, s);
    if (H % heads_tile != 0) return false;
    if (!attn_fused_shape(heads_tile, d, dt, s)) return false;
    s->heads_tile = heads_tile;
    s->tiles = H / heads_tile;
    return true;
}

size_t attn_fused_part_floats(const AttnShape& s)
{
    return (size_t)(s.tiles > 0 ? s.tiles : 1) * s.KH * s.LH * s.HW * (s.vec + 2);
}

hipError_t launch_attn_fused_rows(const AttnArgs& a, const AttnShape& s, hipStream_t stream)
{
    if (a.dt == DT_BF16) return attn_fused_bf16(a, s, 0, nullptr, nullptr, stream);
    if (a.dt == DT_F16) return attn_fused_f16(a, s, 0, nullptr, nullptr, stream);
    return attn_fused_f32(a, s, 0, nullptr, nullptr, stream);
}

hipError_t launch_attn_fused_hub(const AttnArgs& a, const AttnShape& s, const HubMeta& meta, float* part, hipStream_t stream)
{
    if (a.dt == DT_BF16) return attn_fused_bf16(a, s, 1, &meta, part, stream);
    if (a.dt == DT_F16) return attn_fused_f16(a, s, 1, &meta, part, stream);
    return attn_fused_f32(a, s, 1, &meta, part, stream);
}

size_t attn_bwd_part_floats(const AttnShape& s) { return (size_t)s.KH * s.LH * s.HW * (2 * s.vec + 3); }

hipError_t launch_attn_bwd_rows(const AttnBwdArgs& a, const AttnShape& s, hipStream_t stream)
{
    if (a.dt == DT_BF16) return attn_bwd_fused_bf16(a, s, 0, nullptr, nullptr, stream);
    if (a.dt == DT_F16) return attn_bwd_fused_f16(a, s, 0, nullptr, nullptr, stream);
    return attn_bwd_fused_f32(a, s, 0, nullptr, nullptr, stream);
}

hipError_t launch_attn_bwd_hub(const AttnBwdArgs& a, const AttnShape& s, const HubMeta& meta, float* part, hipStream_t stream)
{
    if (a.dt == DT_BF16) return attn_bwd_fused_bf16(a, s, 1, &meta, part, stream);
    if (a.dt == DT_F16) return attn_bwd_fused_f16(a, s, 1, &meta, part, stream);
    return attn_bwd_fused_f32(a, s, 1, &meta, part, stream);
}

namespace {

struct FinishDev {
    RowMap rows;
    const int32_t* __restrict__ rowptr;
    float* S;
    float* D;
    const float* __restrict__ stats;
    int32_t H;
    float scale;
    int32_t hub_t;
    int32_t hub_chunk;
    const HubCounts* __restrict__ counts;
    const int32_t* __restrict__ hub_rows;
    const int32_t* __restrict__ chunk_ptr;
};

// Entries [e0, e1) of the [nnz, H] arrays, all of one row: P = exp(s - m) / l, dS = scale * P * (dP - delta).
__device__ __forceinline__ void finish_span(const FinishDev& a, int row, int64_t e0, int64_t e1, int first, int stride)
{
    const float* __restrict__ rec = a.stats + (int64_t)row * a.H * 3;
    if (stride % a.H == 0) {
        // e0 is a multiple of H, so a lane stays on one head: its record is read once
        const int h = first % a.H;
        const float m = rec[h * 3], inv = rec[h * 3 + 1], delta = rec[h * 3 + 2];
        for (int64_t e = e0 + first; e < e1; e += stride) {
            const float p = __expf(a.S[e] - m) * inv;
            const float dp = a.D[e];
            a.S[e] = p;
            a.D[e] = a.scale * p * (dp - delta);
        }
        return;
    }
    for (int64_t e = e0 + first; e < e1; e += stride) {
        const int h = (int)(e % a.H);
        const float p = __expf(a.S[e] - rec[h * 3]) * rec[h * 3 + 1];
        const float dp = a.D[e];
        a.S[e] = p;
        a.D[e] = a.scale * p * (dp - rec[h * 3 + 2]);
    }
}

__global__ void __launch_bounds__(256) attn_bwd_finish_rows_kernel(FinishDev a)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int idx = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (idx >= a.rows.count) return;
    const int row = row_of(a.rows, idx);
    const int p0 = a.rowptr[row];
    const int p1 = a.rowptr[row + 1];
    if (a.hub_t > 0 && p1 - p0 >= a.hub_t) return;
    finish_span(a, row, (int64_t)p0 * a.H, (int64_t)p1 * a.H, lane, kWave);
}

__global__ void __launch_bounds__(256) attn_bwd_finish_hub_kernel(FinishDev a)
{
    const int chunk = blockIdx.x;
    if (chunk >= a.counts->n_chunks) return;
    const int k_hub = wave_upper_slot(a.chunk_ptr, a.counts->n_hub, chunk);
    const int row = row_of(a.rows, a.hub_rows[k_hub]);
    const int t = chunk - a.chunk_ptr[k_hub];
    const int q0 = a.rowptr[row] + t * a.hub_chunk;
    const int q1 = min(q0 + a.hub_chunk, a.rowptr[row + 1]);
    finish_span(a, row, (int64_t)q0 * a.H, (int64_t)q1 * a.H, threadIdx.x, blockDim.x);
}

}  // namespace

hipError_t launch_attn_bwd_finish(const AttnBwdArgs& a, const AttnShape& s, const HubMeta* meta, hipStream_t stream)
{
    if (a.rows.count == 0) return hipSuccess;
    FinishDev d{};
    d.rows = a.rows;
    d.rowptr = a.rowptr;
    d.S = a.S;
    d.D = a.D;
    d.stats = a.stats;
    d.H = a.H;
    d.scale = a.scale;
    d.hub_t = s.hub_t;
    d.hub_chunk = s.hub_chunk;
    hipLaunchKernelGGL(attn_bwd_finish_rows_kernel, dim3((a.rows.count + 3) / 4), dim3(4 * kWave), 0, stream, d);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || s.hub_t <= 0 || !meta || meta->cap_chunks == 0 || meta->cap_hub == 0) return e;
    d.counts = meta->counts;
    d.hub_rows = meta->hub_rows;
    d.chunk_ptr = meta->chunk_ptr;
    hipLaunchKernelGGL(attn_bwd_finish_hub_kernel, dim3(meta->cap_chunks), dim3(4 * kWave), 0, stream, d);
    return hipGetLastError();
}

}  // namespace autosage

// Single-pass CSR attention launch entry points and the shape rule that says when it applies.
#include "launch.h"

namespace autosage {

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

}  // namespace autosage

// Device-side helpers shared by the gfx950 kernels: typed vector loads, wavefront
// broadcasts and cross-lane reductions.  Wavefront size is 64 throughout.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace autosage {

constexpr int kWave = 64;

struct bf16_t { uint16_t bits; };   // storage only; arithmetic is done in fp32

struct f16_t { uint16_t bits; };    // IEEE binary16 storage; arithmetic is done in fp32

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ float f16_bits_to_f32(uint32_t b)
{
    return static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(b)));     // exact
}

// Loads VEC consecutive elements of T starting at ptr (ptr is VEC*sizeof(T) aligned) as fp32.
template <typename T, int VEC> struct VecIO;

template <> struct VecIO<float, 1> {
    static __device__ __forceinline__ void load(const float* p, float* v) { v[0] = *p; }
};
template <> struct VecIO<float, 2> {
    static __device__ __forceinline__ void load(const float* p, float* v) {
        float2 t = *reinterpret_cast<const float2*>(p); v[0] = t.x; v[1] = t.y;
    }
};
template <> struct VecIO<float, 4> {
    static __device__ __forceinline__ void load(const float* p, float* v) {
        float4 t = *reinterpret_cast<const float4*>(p); v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    }
};
template <> struct VecIO<float, 8> {
    static __device__ __forceinline__ void load(const float* p, float* v) {
        float4 t = *reinterpret_cast<const float4*>(p), u = *reinterpret_cast<const float4*>(p + 4);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w; v[4] = u.x; v[5] = u.y; v[6] = u.z; v[7] = u.w;
    }
};
template <> struct VecIO<bf16_t, 1> {
    static __device__ __forceinline__ void load(const bf16_t* p, float* v) { v[0] = bf16_bits_to_f32(p->bits); }
};
template <> struct VecIO<bf16_t, 2> {
    static __device__ __forceinline__ void load(const bf16_t* p, float* v) {
        uint32_t t = *reinterpret_cast<const uint32_t*>(p);
        v[0] = __uint_as_float(t << 16); v[1] = __uint_as_float(t & 0xFFFF0000u);
    }
};
template <> struct VecIO<bf16_t, 4> {
    static __device__ __forceinline__ void load(const bf16_t* p, float* v) {
        uint2 t = *reinterpret_cast<const uint2*>(p);
        v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xFFFF0000u);
        v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xFFFF0000u);
    }
};
template <> struct VecIO<bf16_t, 8> {
    static __device__ __forceinline__ void load(const bf16_t* p, float* v) {
        uint4 t = *reinterpret_cast<const uint4*>(p);
        v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xFFFF0000u);
        v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xFFFF0000u);
        v[4] = __uint_as_float(t.z << 16); v[5] = __uint_as_float(t.z & 0xFFFF0000u);
        v[6] = __uint_as_float(t.w << 16); v[7] = __uint_as_float(t.w & 0xFFFF0000u);
    }
};

template <> struct VecIO<f16_t, 1> {
    static __device__ __forceinline__ void load(const f16_t* p, float* v) { v[0] = f16_bits_to_f32(p->bits); }
};
template <> struct VecIO<f16_t, 2> {
    static __device__ __forceinline__ void load(const f16_t* p, float* v) {
        uint32_t t = *reinterpret_cast<const uint32_t*>(p);
        v[0] = f16_bits_to_f32(t & 0xFFFFu); v[1] = f16_bits_to_f32(t >> 16);
    }
};
template <> struct VecIO<f16_t, 4> {
    static __device__ __forceinline__ void load(const f16_t* p, float* v) {
        uint2 t = *reinterpret_cast<const uint2*>(p);
        v[0] = f16_bits_to_f32(t.x & 0xFFFFu); v[1] = f16_bits_to_f32(t.x >> 16);
        v[2] = f16_bits_to_f32(t.y & 0xFFFFu); v[3] = f16_bits_to_f32(t.y >> 16);
    }
};
template <> struct VecIO<f16_t, 8> {
    static __device__ __forceinline__ void load(const f16_t* p, float* v) {
        uint4 t = *reinterpret_cast<const uint4*>(p);
        v[0] = f16_bits_to_f32(t.x & 0xFFFFu); v[1] = f16_bits_to_f32(t.x >> 16);
        v[2] = f16_bits_to_f32(t.y & 0xFFFFu); v[3] = f16_bits_to_f32(t.y >> 16);
        v[4] = f16_bits_to_f32(t.z & 0xFFFFu); v[5] = f16_bits_to_f32(t.z >> 16);
        v[6] = f16_bits_to_f32(t.w & 0xFFFFu); v[7] = f16_bits_to_f32(t.w >> 16);
    }
};

// Stores VEC consecutive fp32 values (p is VEC*4-byte aligned; VEC up to 8 is split into 16-byte pieces).
template <int VEC> __device__ __forceinline__ void store_f32(float* p, const float* v)
{
    if constexpr (VEC == 1) {
        *p = v[0];
    } else if constexpr (VEC == 2) {
        *reinterpret_cast<float2*>(p) = make_float2(v[0], v[1]);
    } else if constexpr (VEC == 4) {
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
        static_assert(VEC == 8, "unsupported vector width");
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
    }
}

// Streaming accesses: data that is touched once (index arrays, scores, outputs) is loaded and stored
// with the non-temporal hint, so that it passes through the caches without displacing the gathered
// dense rows that are reused.  Plain streams measure about 10 % faster with the hint on this chip.
typedef float stream_f2 __attribute__((ext_vector_type(2)));
typedef float stream_f4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int stream_load(const int* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ float stream_load(const float* p) { return __builtin_nontemporal_load(p); }

// Loads VEC consecutive floats (p is VEC*4-byte aligned; VEC = 1, 2 or 4).
template <int VEC> __device__ __forceinline__ void stream_load_f32(const float* p, float* v)
{
    if constexpr (VEC == 1) {
        v[0] = __builtin_nontemporal_load(p);
    } else if constexpr (VEC == 2) {
        const stream_f2 t = __builtin_nontemporal_load(reinterpret_cast<const stream_f2*>(p));
        v[0] = t.x; v[1] = t.y;
    } else {
        static_assert(VEC == 4, "unsupported vector width");
        const stream_f4 t = __builtin_nontemporal_load(reinterpret_cast<const stream_f4*>(p));
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    }
}

// Stores VEC consecutive fp32 values (p is min(VEC, 4)*4-byte aligned; VEC = 8 is two 16-byte pieces).
template <int VEC> __device__ __forceinline__ void stream_store_f32(float* p, const float* v)
{
    if constexpr (VEC == 1) {
        __builtin_nontemporal_store(v[0], p);
    } else if constexpr (VEC == 2) {
        const stream_f2 t = {v[0], v[1]};
        __builtin_nontemporal_store(t, reinterpret_cast<stream_f2*>(p));
    } else if constexpr (VEC == 4) {
        const stream_f4 t = {v[0], v[1], v[2], v[3]};
        __builtin_nontemporal_store(t, reinterpret_cast<stream_f4*>(p));
    } else {
        static_assert(VEC == 8, "unsupported vector width");
        const stream_f4 t = {v[0], v[1], v[2], v[3]}, u = {v[4], v[5], v[6], v[7]};
        __builtin_nontemporal_store(t, reinterpret_cast<stream_f4*>(p));
        __builtin_nontemporal_store(u, reinterpret_cast<stream_f4*>(p + 4));
    }
}

// Value of x held by lane `src` (0..63).  `src` may differ between lanes.
__device__ __forceinline__ int lane_get(int x, int src) { return __shfl(x, src, kWave); }
__device__ __forceinline__ float lane_get(float x, int src) { return __shfl(x, src, kWave); }

// Value of x held by lane `src`, where src is the same for the whole wavefront (lands in an SGPR).
__device__ __forceinline__ int lane_get_uniform(int x, int src) { return __builtin_amdgcn_readlane(x, src); }
__device__ __forceinline__ float lane_get_uniform(float x, int src)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), src));
}

__device__ __forceinline__ int wave_uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }

template <int CTRL> __device__ __forceinline__ float dpp_move(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}

// Sum over aligned groups of G consecutive lanes (G a power of two); every lane of the
// group receives the total.  Steps inside a 16-lane row use DPP; wider steps use the
// cross-lane network.
template <int G> __device__ __forceinline__ float group_sum(float x)
{
    if constexpr (G >= 2) x += dpp_move<0xB1>(x);    // quad_perm [1,0,3,2]
    if constexpr (G >= 4) x += dpp_move<0x4E>(x);    // quad_perm [2,3,0,1]
    if constexpr (G >= 8) x += dpp_move<0x141>(x);   // row_half_mirror
    if constexpr (G >= 16) x += dpp_move<0x140>(x);  // row_mirror
    if constexpr (G >= 32) x += __shfl_xor(x, 16, kWave);
    if constexpr (G >= 64) x += __shfl_xor(x, 32, kWave);
    return x;
}

template <int G> __device__ __forceinline__ float group_max(float x)
{
    if constexpr (G >= 2) x = fmaxf(x, dpp_move<0xB1>(x));
    if constexpr (G >= 4) x = fmaxf(x, dpp_move<0x4E>(x));
    if constexpr (G >= 8) x = fmaxf(x, dpp_move<0x141>(x));
    if constexpr (G >= 16) x = fmaxf(x, dpp_move<0x140>(x));
    if constexpr (G >= 32) x = fmaxf(x, __shfl_xor(x, 16, kWave));
    if constexpr (G >= 64) x = fmaxf(x, __shfl_xor(x, 32, kWave));
    return x;
}

// Sum of the values held by lanes {l, l+G, l+2G, ...} (same position in every group of G
// lanes); every such lane receives the total.  Used to merge per-group partial rows.
template <int G> __device__ __forceinline__ float across_groups_sum(float x)
{
    // rotations inside a 16-lane row: after ror:G, ror:2G, ... every lane holds the sum of the
    // lanes of its row that share its position modulo G
    if constexpr (G <= 1) x += dpp_move<0x121>(x);   // row_ror:1
    if constexpr (G <= 2) x += dpp_move<0x122>(x);   // row_ror:2
    if constexpr (G <= 4) x += dpp_move<0x124>(x);   // row_ror:4
    if constexpr (G <= 8) x += dpp_move<0x128>(x);   // row_ror:8
    if constexpr (G <= 16) x += __shfl_xor(x, 16, kWave);
    if constexpr (G <= 32) x += __shfl_xor(x, 32, kWave);
    return x;
}

// Largest k in [0, n) with ptr[k] <= x (ptr ascending, ptr[0] <= x), found by the whole wavefront together: every
// round the 64 lanes probe 64 evenly spaced entries of the remaining range with one load instruction and a ballot
// picks the interval, so a table of n entries takes ceil(log64 n) dependent loads (three for 262 144) where a
// scalar binary search takes log2 n.  All 64 lanes must call it with the same arguments; all get the result.
__device__ __forceinline__ int wave_upper_slot(const int32_t* __restrict__ ptr, int n, int x)
{
    const int lane = threadIdx.x & (kWave - 1);
    int lo = 0, hi = n;                              // answer in [lo, hi), ptr[lo] <= x
    while (hi - lo > 1) {
        const int step = (hi - lo + kWave - 1) / kWave;
        const int idx = lo + lane * step;
        const bool le = idx < hi && ptr[idx] <= x;   // true for a prefix of the lanes (lane 0 included)
        const unsigned long long m = __ballot(le);
        const int j = 63 - __clzll((long long)m);
        lo += j * step;
        hi = min(hi, lo + step);
    }
    return __builtin_amdgcn_readfirstlane(lo);
}

// Maps a launched block id to a logical block id so that each of the 8 XCDs (hardware
// dispatches consecutive workgroup ids round-robin over them) walks one contiguous eighth of
// the logical range.  The grid must be padded to a multiple of 8; ids >= n_logical are idle.
__device__ __forceinline__ int xcd_contiguous_block(int launched_id, int n_launched)
{
    const int per = n_launched >> 3;
    return (launched_id & 7) * per + (launched_id >> 3);
}

// The same for a launch padded beyond the n real work items (hub chunks: the grid covers a host-side upper bound,
// the true count is read on the device): every XCD walks one contiguous eighth of [0, n).  Returns -1 for an idle
// workgroup.  The grid must hold at least 8 * ceil(n / 8) workgroups.
__device__ __forceinline__ int xcd_contiguous_item(int launched_id, int n)
{
    const int per = (n + 7) >> 3;
    const int q = launched_id >> 3;
    if (q >= per) return -1;
    const int item = (launched_id & 7) * per + q;
    return item < n ? item : -1;
}

}  // namespace autosage

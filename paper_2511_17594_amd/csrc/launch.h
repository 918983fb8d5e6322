// Host-side launcher interface between the C ABI layer and the kernel translation units.
// Everything here is plain data + free functions; no device code.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace autosage {

enum Mapping { MAP_PLAIN = 0, MAP_WAVE_ROW = 1, MAP_MULTI_ROW = 2 };
enum DType { DT_F32 = 0, DT_BF16 = 1, DT_F16 = 2 };
inline bool dtype_known(int dt) { return dt == DT_F32 || dt == DT_BF16 || dt == DT_F16; }
inline int dtype_bytes(int dt) { return dt == DT_F32 ? 4 : 2; }

// The rows a launch covers, in blocks of 2^block_shift consecutive rows:
//   row(idx) = first + (idx >> block_shift) * stride + (idx & (2^block_shift - 1)),  idx in [0, count).
// The full matrix is {0, 1, n_rows, 0}; a probe uses strided blocks of rows of the same arrays.
struct RowMap {
    int32_t first;
    int32_t stride;        // distance between the first rows of consecutive blocks
    int32_t count;
    int32_t block_shift;
};

__host__ __device__ inline int32_t row_of(const RowMap& m, int32_t idx)
{
    return m.first + (idx >> m.block_shift) * m.stride + (idx & ((1 << m.block_shift) - 1));
}

// A schedule with every "auto" field resolved against F, dtype and alignment.
struct Resolved {
    int32_t mapping;    // Mapping
    int32_t vec;        // elements per lane load
    int32_t G;          // lanes per group (power of two, <= 64)
    int32_t K;          // vector chunks per lane per pass
    int32_t HW;         // SDDMM: heads side by side in one group (1 for SpMM and single-head SDDMM)
    int32_t f_tile;     // features per pass = G * vec * K (PLAIN: 64)
    int32_t tiles;      // passes over F (grid.y; PLAIN loops inside the kernel)
    int32_t wpg;        // wavefronts per workgroup
    int32_t unroll;     // nonzeros in flight per group
    int32_t hub_t;      // 0 = no hub split
    int32_t hub_chunk;
    int32_t xcd_remap;
};

// Device-resident index metadata of the heavy/light split, laid out in the workspace.
struct HubCounts {      // first 16 bytes of the metadata block
    int32_t n_hub;
    int32_t n_chunks;
    int32_t n_light;
    int32_t pad;
};

struct HubMeta {
    HubCounts* counts;      // dev
    int32_t* hub_rows;      // dev, capacity cap_hub (values are idx of the RowMap, i.e. row = first + v * stride)
    int32_t* chunk_ptr;     // dev, capacity cap_hub + 1
    int32_t* light_rows;    // dev or nullptr
    int32_t* block_counts;  // dev scratch, 4 ints per partition block
    int32_t cap_hub;        // host upper bound of n_hub
    int32_t cap_chunks;     // host upper bound of n_chunks
};

struct SpmmArgs {
    RowMap rows;
    const int32_t* rowptr;
    const int32_t* colind;
    const float* val;      // [nnz] (heads == 1) or [nnz, heads] per-head weights
    const int32_t* val_index;  // nullptr, or [nnz]: nonzero p takes the weights at val_index[p] (wavefront-per-row mapping only)
    const void* B;         // [n_cols, F] (heads == 1) or [n_cols, heads, d] with F = heads * d
    int64_t ldb;
    float* C;
    int64_t ldc;
    int32_t F;
    int32_t dt;
    int32_t heads;         // 1 = plain SpMM; > 1 = per-head weights, head of feature f is f / head_dim
    int32_t head_dim;
};

struct SddmmArgs {
    RowMap rows;
    const int32_t* rowptr;
    const int32_t* colind;
    const void* X;         // [n_rows, heads * d]
    int64_t ldx;
    const void* Y;         // [n_cols, heads * d]
    int64_t ldy;
    float* out;            // [nnz, heads]
    int32_t F;             // per-head feature count d
    int32_t dt;
    int32_t heads;
    float scale;           // out = scale * dot
    int32_t x_f32;         // 1: X holds fp32 whatever dt says (Y keeps dt): the upstream gradient against 16-bit V
    int32_t accumulate;    // 1: out += scale * dot (feature tiles after the first)
};

struct SoftmaxArgs {
    RowMap rows;
    const int32_t* rowptr;
    const float* in;       // [nnz, H]
    float* out;            // [nnz, H]
    int32_t H;
};

struct AttnArgs {
    RowMap rows;
    const int32_t* rowptr;
    const int32_t* colind;
    const void* Q;         // [n_rows, H, d]
    const void* K;         // [n_cols, H, d]
    const void* V;         // [n_cols, H, d]
    float* O;              // [n_rows, H, d]
    int32_t H;
    int32_t d;
    int32_t dt;
    float scale;
};

// Lane shape of the single-pass attention kernels: LH lanes per head, HW heads side by side,
// KH head passes kept in registers.
struct AttnShape {
    int32_t vec;
    int32_t LH;
    int32_t HW;
    int32_t KH;
    int32_t wpg;
    int32_t hub_t;
    int32_t hub_chunk;
    int32_t heads_tile;    // heads one launch row (grid.y) covers; tiles * heads_tile >= H
    int32_t tiles;         // head tiles, walked one after the other by the launch
};

// True (and fills vec/LH/HW/KH, one tile of all H heads) when the single-pass kernels cover this head count and width.
bool attn_fused_shape(int32_t H, int32_t d, int dt, AttnShape* s);
// The same for a launch that walks the heads in tiles of heads_tile (> 0, dividing H) heads: the K and V slices a
// tile gathers from are heads_tile / H of the operands, small enough to stay in the caches when the whole is not.
bool attn_fused_shape_tiled(int32_t H, int32_t d, int dt, int32_t heads_tile, AttnShape* s);
// Floats of partial state per hub chunk.
size_t attn_fused_part_floats(const AttnShape& s);
hipError_t launch_attn_fused_rows(const AttnArgs& a, const AttnShape& s, hipStream_t stream);
hipError_t launch_attn_fused_hub(const AttnArgs& a, const AttnShape& s, const HubMeta& meta, float* part, hipStream_t stream);

// Backward of the attention on the pattern itself, single pass (see attention_kernels.inc): dQ, the scores' gradient
// and the probabilities for the transposed side.
struct AttnBwdArgs {
    RowMap rows;
    const int32_t* rowptr;
    const int32_t* colind;
    const void* Q;         // [n_rows, H, d]
    const void* K;         // [n_cols, H, d]
    const void* V;         // [n_cols, H, d]
    const float* dO;       // [n_rows, H, d]
    float* dQ;             // [n_rows, H, d]
    float* S;              // [nnz, H] out: P
    float* D;              // [nnz, H] out: dS (scale included)
    float* stats;          // [n_rows, H, 3] scratch: m, 1 / l, delta per row and head
    int32_t H;
    int32_t d;
    int32_t dt;
    float scale;
};
// Floats of partial state per hub chunk of the backward pass.
size_t attn_bwd_part_floats(const AttnShape& s);
// Light rows / hub rows of the pass (raw scores and dP in S and D, per-row records in stats) ...
hipError_t launch_attn_bwd_rows(const AttnBwdArgs& a, const AttnShape& s, hipStream_t stream);
hipError_t launch_attn_bwd_hub(const AttnBwdArgs& a, const AttnShape& s, const HubMeta& meta, float* part, hipStream_t stream);
// ... and the streaming kernels that turn S and D into P and dS (meta: nullptr without a hub split).
hipError_t launch_attn_bwd_finish(const AttnBwdArgs& a, const AttnShape& s, const HubMeta* meta, hipStream_t stream);

struct SoftmaxBwdArgs {
    RowMap rows;
    const int32_t* rowptr;
    const float* P;        // [nnz, H] softmax output
    const float* dP;       // [nnz, H] gradient with respect to P (may alias dS)
    float* dS;             // [nnz, H] gradient with respect to the scores
    int32_t H;
    float scale;           // dS is multiplied by it (the chain rule through scaled scores); 0 means 1
};

// dS = P * (dP - rowsum(P * dP)); hub rows (degree >= hub_t) through per-chunk partial dots in `part` ([cap_chunks, H]).
// group: lanes per light row for power-of-two head counts (see launch_softmax_rows).
hipError_t launch_softmax_bwd(const SoftmaxBwdArgs& a, int32_t hub_t, int32_t hub_chunk, int32_t group, const HubMeta* meta,
                              float* part, hipStream_t stream);

// CSR transpose: stable radix sort of the nonzeros by column + index kernels.  keys_a, keys_b: int32[nnz] scratch;
// temp: transpose_sort_temp_bytes(nnz, n_cols) bytes (second value buffer, digit histograms, scan sums).
size_t transpose_sort_temp_bytes(int64_t nnz, int64_t n_cols);
hipError_t launch_csr_transpose(int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
                                const float* val, int32_t* t_rowptr, int32_t* t_colind, float* t_val, int32_t* perm,
                                int32_t* keys_a, int32_t* keys_b, void* temp, size_t temp_bytes, hipStream_t stream);
// out[q, :] = in[perm[q], :] for rows of `width` floats.
hipError_t launch_gather_rows(const int32_t* perm, int64_t n, int32_t width, const float* in, float* out, hipStream_t stream);

// Heavy/light partition of the rows of `rows` (index metadata, integer only).
hipError_t launch_hub_partition(const RowMap& rows, const int32_t* rowptr, int32_t hub_t, int32_t hub_chunk,
                                const HubMeta& meta, hipStream_t stream);

// SpMM: light rows (skips rows of degree >= r.hub_t when r.hub_t > 0) ...
hipError_t launch_spmm_rows(const SpmmArgs& a, const Resolved& r, hipStream_t stream);
// ... and the hub rows: per-chunk partial rows into `part` ([cap_chunks, F] fp32), then an ordered combine.
hipError_t launch_spmm_hub(const SpmmArgs& a, const Resolved& r, const HubMeta& meta, float* part, hipStream_t stream);

hipError_t launch_sddmm_rows(const SddmmArgs& a, const Resolved& r, hipStream_t stream);
hipError_t launch_sddmm_hub(const SddmmArgs& a, const Resolved& r, const HubMeta& meta, hipStream_t stream);

// Row-softmax: light rows, and hub rows through per-chunk (max, sum) partials in `part` ([cap_chunks, H, 2]).
// group > 0: lanes per row (rounded up to a power of two, at least the lanes one entry takes) of the kernels
// that put several rows on a wavefront; they need a power-of-two H <= 256 and arrays aligned to min(H, 4)
// floats, otherwise (and for group <= 0) one wavefront of `wpg` per workgroup takes one row.
hipError_t launch_softmax_rows(const SoftmaxArgs& a, int32_t hub_t, int32_t wpg, int32_t group, hipStream_t stream);
hipError_t launch_softmax_hub(const SoftmaxArgs& a, int32_t hub_chunk, int32_t group, const HubMeta& meta, float* part,
                              hipStream_t stream);

// Degree features: hist[33] (int64), max_deg, nnz and the 1024 rowptr samples, written to `dev_out`
// (int64[33 + 2 + 1024]); the caller copies it back.
hipError_t launch_graph_features(int64_t n_rows, const int32_t* rowptr, int64_t* dev_out, hipStream_t stream);
// CSR consistency check; dev_flag[0] becomes nonzero when a violation is found.
hipError_t launch_narrow_indices(int64_t n, const int64_t* src, int32_t* dst, int64_t limit, int32_t* dev_flag,
                                 hipStream_t stream);
hipError_t launch_validate_csr(int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t* rowptr,
                               const int32_t* colind, int32_t* dev_flag, hipStream_t stream);

// Streaming kernels for the bandwidth probe: mode 0 = read src (one partial sum per workgroup into dst, `blocks`
// floats), 1 = copy src to dst, 2 = scale dst in place; n_vec 16-byte vectors.
int stream_probe_blocks(int cu_count);
hipError_t launch_stream_probe(int mode, int blocks, const void* src, void* dst, int64_t n_vec, hipStream_t stream);
// Random-row gather out of a table of n_table_rows rows of row_bytes (16 * 2^k, at most 1024) bytes: n_idx row
// numbers (clamped into the table), one partial sum per workgroup into sums (`blocks` floats).
hipError_t launch_gather_probe(int blocks, const void* table, int32_t n_table_rows, int32_t row_bytes, const int32_t* idx,
                               int64_t n_idx, float* sums, hipStream_t stream);

}  // namespace autosage

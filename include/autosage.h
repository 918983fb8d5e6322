/*
 * autosage.h -- C ABI of the MI355X (gfx950) CSR SpMM / SDDMM / CSR-attention library.
 *
 * Operations (paper: "Notation", "Preliminaries", "Method: Kernel templates",
 * "Scheduler: estimate -> micro-probe -> guardrail", the decision sketch, Proposition 1):
 *
 *   SpMM            C = A B,  A sparse CSR (rowptr, colind, val), B dense
 *   SDDMM           out[p] = <X_i, Y_j> for every stored (i, j) of A, in CSR order
 *   row-softmax     numerically stable softmax over the stored entries of each row
 *   CSR attention   SDDMM -> row-softmax -> SpMM on one sparsity pattern, multi-head
 *   selector        estimate from the degree histogram -> timed probes on a row sample
 *                   -> guardrail (accept iff t* <= alpha * t_baseline) -> persistent cache
 *
 * Conventions that hold for every entry point unless its comment says otherwise
 *   - "dev" pointers are device (HBM) pointers owned by the caller; "host" pointers are
 *     ordinary host memory.  The library never frees or keeps a caller pointer.
 *   - Indices are int32.  Dense operands are row-major with the feature index minor and a
 *     leading dimension (in elements) >= the feature count.
 *   - Dense INPUT operands have dtype `dt` (fp32, bf16 or IEEE fp16 bit patterns); val, scores and all
 *     outputs are fp32; accumulation is fp32.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls with an
 *     explicit schedule only enqueue work and never synchronise.  Calls with sched == NULL
 *     consult the selector, which synchronises the stream only when it has to probe.
 *   - `workspace` is caller-provided device scratch of at least autosage_workspace_bytes()
 *     bytes, 256-byte aligned; it may be NULL when the schedule needs none (no hub split and
 *     a non-fused attention is never the case: attention always needs it).
 *   - Every function returns an autosage_status_t; nothing throws or aborts across the ABI.
 *     Arguments are checked before anything is launched.
 *   - Outputs must not alias inputs (row-softmax may run in place).
 *   - For a fixed schedule the result is bit-reproducible: no floating-point atomics are used.
 *   - A handle is not thread safe: use one handle per host thread (handles share nothing).
 *   - The selector remembers the degree features of the last 16 (rowptr pointer, n_rows, n_cols, nnz)
 *     combinations so that steady-state calls need no device-to-host copy.  Overwriting a rowptr array
 *     in place with another graph of the same sizes therefore replays the old graph's decision (results
 *     stay correct, the schedule may be a poor one); autosage_forget_graph drops the memory of one rowptr
 *     address, autosage_cache_clear or memoize_signature = 0 drop / disable all of it.
 *   - While `stream` is being captured into a HIP graph a call with sched == NULL succeeds only when it needs
 *     neither the feature pass nor probes (features remembered and decision cached); otherwise it returns
 *     AUTOSAGE_ERR_UNSUPPORTED without touching the stream.  Calls with an explicit schedule can be captured.
 */
#ifndef AUTOSAGE_H
#define AUTOSAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct autosage_ctx* autosage_handle_t;

typedef enum {
    AUTOSAGE_OK = 0,
    AUTOSAGE_ERR_INVALID_ARG = 1,
    AUTOSAGE_ERR_UNSUPPORTED = 2,
    AUTOSAGE_ERR_WORKSPACE_TOO_SMALL = 3,
    AUTOSAGE_ERR_HIP = 4,
    AUTOSAGE_ERR_IO = 5,
    AUTOSAGE_ERR_REPLAY_MISS = 6
} autosage_status_t;

typedef enum { AUTOSAGE_F32 = 0, AUTOSAGE_BF16 = 1, AUTOSAGE_F16 = 2 } autosage_dtype_t;

typedef enum {
    AUTOSAGE_OP_SPMM = 0,
    AUTOSAGE_OP_SDDMM = 1,
    AUTOSAGE_OP_SOFTMAX = 2,
    AUTOSAGE_OP_ATTENTION = 3
} autosage_op_t;

/* Row mappings (the paper's kernel-variant table, re-cut for 64-wide wavefronts). */
typedef enum {
    AUTOSAGE_MAP_PLAIN = 0,      /* fallback: one wavefront per row, one lane per feature, 4-byte loads */
    AUTOSAGE_MAP_WAVE_ROW = 1,   /* one wavefront per row; lane groups split the row's nonzeros */
    AUTOSAGE_MAP_MULTI_ROW = 2,  /* several rows per wavefront: every lane group owns one row */
    AUTOSAGE_MAP_FUSED = 3       /* CSR attention only: one pass with a running softmax, no score array */
} autosage_mapping_t;

/* Most nonzeros, and most rows, of one call: 2^31 - 2^20.  Positions and row numbers are int32 inside the
 * kernels and are stepped by at most one hub chunk past the end of a row. */
#define AUTOSAGE_MAX_NNZ 2146435072LL

/* A schedule = one point of the knob space (feature tile, mapping, vector width, hub split). */
typedef struct {
    int32_t mapping;       /* autosage_mapping_t */
    int32_t f_tile;        /* features one wavefront covers per pass; 0 = smallest tile covering F (max 2048 B per lane group pass) */
    int32_t waves_per_wg;  /* wavefronts per workgroup: 1, 2, 4, 8 or 16; 0 = 4 */
    int32_t vec_bytes;     /* bytes per lane load: 4, 8 or 16; 0 = widest legal for F, ld and pointer alignment */
    int32_t unroll;        /* nonzeros in flight per lane group: 1, 2, 4 or 8; 0 = library default */
    int32_t hub_t;         /* rows with degree >= hub_t are split over workgroups; 0 = no hub split */
    int32_t hub_chunk;     /* nonzeros per hub chunk, 64 .. 2^20; 0 = min(hub_t, 2^20) */
    int32_t xcd_remap;     /* 1 = consecutive row blocks stay on one XCD (contiguous row range per L2) */
    int32_t group_lanes;   /* SDDMM with 16-byte lane loads: lanes that share one gathered dense row per pass, a power of
                              two; each lane then holds (tile width / 16 bytes) / group_lanes vectors of the row (2, 4 or
                              8 of them) and the dot product is finished across group_lanes lanes only.  0, or a value
                              that is not below the lanes one vector per lane would take = one vector per lane.  Any
                              other operator, mapping or shape with a nonzero value -> AUTOSAGE_ERR_UNSUPPORTED */
} autosage_schedule_t;

/* ---- lifetime -------------------------------------------------------------------------- */

/* Creates a handle bound to HIP device `device_id` and reads the AUTOSAGE_* environment
 * toggles once (AUTOSAGE_FTILE, AUTOSAGE_WPB, AUTOSAGE_HUB_T, AUTOSAGE_PROBE_FRAC,
 * AUTOSAGE_PROBE_ITERS, AUTOSAGE_PROBE_CAP_MS, AUTOSAGE_PROBE_TOPK, AUTOSAGE_PROBE_MIN_ROWS, AUTOSAGE_PROBE_REFINE,
 * AUTOSAGE_ALPHA, AUTOSAGE_CACHE (file loaded now and saved by autosage_destroy),
 * AUTOSAGE_REPLAY_ONLY); the paper's Implementation section names them.
 * device_id < 0 creates a host-only handle: selector, cache and estimate functions work,
 * every compute call returns AUTOSAGE_ERR_UNSUPPORTED.
 * Ownership: a device handle holds two small device buffers of its own (8.5 KB for the degree
 * features the selector reads back, 256 bytes for the index-check flag), a pinned host mirror
 * and two events, all made here and released by autosage_destroy; no compute call allocates,
 * and every other byte of device memory a call touches is the caller's. */
autosage_status_t autosage_create(autosage_handle_t* out, int device_id);
autosage_status_t autosage_destroy(autosage_handle_t h);
const char* autosage_status_string(autosage_status_t s);

/* Sets a parameter by name.  Selector: "alpha", "probe_frac", "probe_iters", "probe_cap_ms",
 * "probe_topk", "probe_min_rows", "probe_refine" (most extra probes of the refinement rounds: schedules one knob away
 * from the best probed one; default 8, 0 = none), "replay_only", "confirm_full", "memoize_signature", "baseline_bound"
 * (1, default: the guardrail's baseline is first bounded from below by timing it without its rows of
 * 1024 entries or more, and timed whole only when that bound does not decide; 0: always timed whole).
 * Row-softmax (forward and backward): "softmax_group" = lanes that share one light row (rounded up to
 * a power of two <= 64, at least the lanes one entry of H heads takes); 0 (default) derives it from
 * the mean row length, a negative value keeps one wavefront per row.
 * Attention backward: "attention_backward_fused" (1, default: dQ, P and dS come from one pass over the K and V rows
 * of every nonzero wherever the single-pass forward kernels cover the head count and width; 0: always the chain rule
 * stage by stage).
 * Unknown name -> AUTOSAGE_ERR_INVALID_ARG. */
autosage_status_t autosage_set_param(autosage_handle_t h, const char* name, double value);
autosage_status_t autosage_get_param(autosage_handle_t h, const char* name, double* value);

/* ---- the hot path ---------------------------------------------------------------------- */

/* SpMM (Notation: C = A B).  C[n_rows, F] (fp32, dev) = A[n_rows, n_cols] * B[n_cols, F] (dt, dev).
 * rowptr[n_rows+1], colind[nnz], val[nnz] are dev pointers.  Empty rows give zero rows.
 * sched == NULL: the selector chooses (cache -> probe -> guardrail); else the given schedule runs.
 * Errors: INVALID_ARG (null pointer, F <= 0, ld < F, nnz or n_rows above AUTOSAGE_MAX_NNZ, bad schedule field),
 * UNSUPPORTED (vec_bytes illegal for this F / alignment), WORKSPACE_TOO_SMALL, HIP. */
autosage_status_t autosage_spmm(autosage_handle_t h, int64_t n_rows, int64_t n_cols, int64_t nnz,
                                const int32_t* rowptr, const int32_t* colind, const float* val,
                                const void* B, int64_t ldb, float* C, int64_t ldc, int32_t F,
                                autosage_dtype_t dt, const autosage_schedule_t* sched,
                                void* workspace, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory or size a workspace (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): autosage_spmm with an explicit schedule (sched must not be NULL: the
 * selector may probe and synchronise) whose hub-split scratch -- partition metadata and per-chunk partial rows,
 * the `workspace` of autosage_spmm -- is a fixed array of AUTOSAGE_STATIC_SCRATCH_BYTES inside the library's device
 * image.  Each GPU the library runs on holds that array until the process ends.  Same arguments, results (bit for
 * bit, for the same schedule) and errors as autosage_spmm; additionally AUTOSAGE_ERR_WORKSPACE_TOO_SMALL when
 * autosage_workspace_bytes(AUTOSAGE_OP_SPMM, n_rows, nnz, F, 1, sched) exceeds AUTOSAGE_STATIC_SCRATCH_BYTES
 * (nothing is launched then).  The call allocates and frees nothing, on the device or through any library, and
 * does not synchronise.  All calls on one GPU share the array, which keeps the previous call's contents (every
 * word a call reads it has written first, so nothing needs clearing): calls that overlap on one GPU -- two
 * streams, two handles, two threads -- race on it and must be serialised by the caller. */
#define AUTOSAGE_STATIC_SCRATCH_BYTES (32u << 20)
autosage_status_t autosage_spmm_static(autosage_handle_t h, int64_t n_rows, int64_t n_cols, int64_t nnz,
                                       const int32_t* rowptr, const int32_t* colind, const float* val,
                                       const void* B, int64_t ldb, float* C, int64_t ldc, int32_t F,
                                       autosage_dtype_t dt, const autosage_schedule_t* sched, void* stream);

/* SDDMM (Notation: A~_ij = <X_i, Y_j> on the pattern of A).  out[p] (fp32, dev, CSR order) for
 * every stored p of row i; X is [n_rows, F], Y is [n_cols, F] (dt, dev).  val is not read
 * (pattern only) and may be NULL.  Same schedule / error rules as autosage_spmm. */
autosage_status_t autosage_sddmm(autosage_handle_t h, int64_t n_rows, int64_t n_cols, int64_t nnz,
                                 const int32_t* rowptr, const int32_t* colind, const float* val,
                                 const void* X, int64_t ldx, const void* Y, int64_t ldy, int32_t F,
                                 autosage_dtype_t dt, float* out, const autosage_schedule_t* sched,
                                 void* workspace, size_t workspace_bytes, void* stream);

/* Row-softmax (Kernel templates: numerically stable CSR row-softmax).  in/out are [nnz, H] fp32
 * dev arrays (head index minor); for each row and head: m = max, e = exp(s - m), out = e / sum e.
 * Rows without nonzeros write nothing.  out may equal in.  hub_t > 0 splits rows of degree
 * >= hub_t into chunks of hub_chunk (0 = hub_t) entries: per-chunk (max, sum), one merge per row in a
 * fixed order, then a normalising pass (needs workspace).  A power-of-two H <= 256 with in and out
 * aligned to min(H, 4) floats takes vector loads with several short rows per wavefront; any other H
 * or alignment runs one wavefront per row with scalar loads (same result within rounding). */
autosage_status_t autosage_csr_row_softmax(autosage_handle_t h, int64_t n_rows, int64_t nnz,
                                           const int32_t* rowptr, const float* in, float* out,
                                           int32_t H, int32_t hub_t, int32_t hub_chunk,
                                           void* workspace, size_t workspace_bytes, void* stream);

/* CSR attention (Preliminaries: SDDMM -> row-softmax -> SpMM).  Q, K, V are [N, H, d] (in_dt, dev,
 * d minor), O is [N, H, d] fp32 dev.  S[p,h] = scale * <Q[i,h,:], K[j,h,:]>, P = row-softmax(S)
 * per (row, head), O[i,h,:] = sum_p P[p,h] V[colind[p],h,:].  Rows without nonzeros give O = 0.
 * val is ignored and may be NULL.  Requires d * element size to be a multiple of 16 bytes and 16-byte
 * aligned Q, K, V, O (else AUTOSAGE_ERR_UNSUPPORTED).
 * sched->mapping selects the pipeline: AUTOSAGE_MAP_FUSED = a single pass per row with a running
 * softmax (scores never reach memory; available when the heads fit at most two register passes of a
 * wavefront, else UNSUPPORTED); AUTOSAGE_MAP_WAVE_ROW or AUTOSAGE_MAP_PLAIN = three stages (SDDMM ->
 * row-softmax -> SpMM with the [nnz, H] fp32 scores in the workspace); the guardrail baseline is the
 * three-stage pipeline without hub split (autosage_baseline_schedule).  hub_t / hub_chunk / waves_per_wg /
 * unroll apply to every stage; vec_bytes is chosen from d.  f_tile: for AUTOSAGE_MAP_FUSED, 0 or the features of
 * one head tile (a multiple of d whose head count divides H): the launch then walks the heads tile after tile,
 * so that the slices of K and V a tile gathers from fit cache levels the whole operands do not (any other value
 * -> UNSUPPORTED); the three-stage pipeline ignores it.
 * sched == NULL: the selector chooses pipeline and hub threshold (autosage_decide_attention). */
autosage_status_t autosage_csr_attention(autosage_handle_t h, int64_t N, int64_t nnz,
                                         const int32_t* rowptr, const int32_t* colind, const float* val,
                                         const void* Q, const void* K, const void* V, float* O,
                                         int32_t H, int32_t d, float scale, autosage_dtype_t in_dt,
                                         const autosage_schedule_t* sched,
                                         void* workspace, size_t workspace_bytes, void* stream);

/* Workspace size in bytes (host only, no GPU work).  With sched != NULL: what that schedule needs
 * (0 hub split -> a 256-byte minimum).  With sched == NULL: an upper bound over every schedule the
 * selector may choose (hub thresholds >= 512), which is what calls with sched == NULL require.
 * For SPMM / SDDMM pass the feature count in F and H = 1; for SOFTMAX pass H (F ignored, pass 1);
 * for ATTENTION pass H and F = d (the bound includes the [nnz, H] fp32 score array). */
autosage_status_t autosage_workspace_bytes(autosage_handle_t h, autosage_op_t op, int64_t n_rows,
                                           int64_t nnz, int32_t F, int32_t H,
                                           const autosage_schedule_t* sched, size_t* bytes);

/* ---- plan / index metadata (exposed so that it can be compared bit-exactly) ------------- */

/* Heavy/light split (kernel-variant table: rows whose degree reaches the split threshold hubT).
 *   hub_rows   (dev, capacity n_rows)     ascending { i : deg(i) >= hub_t }
 *   chunk_ptr  (dev, capacity n_rows + 1) chunk_ptr[0] = 0, chunk_ptr[k+1] = chunk_ptr[k] + ceil(deg(hub_rows[k]) / hub_chunk)
 *   light_rows (dev, capacity n_rows, may be NULL) ascending complement, empty rows included
 * Chunk t of hub row r covers nonzeros [rowptr[r] + t*hub_chunk, min(rowptr[r] + (t+1)*hub_chunk, rowptr[r+1])).
 * n_hub, n_light (host) are written after the stream has been synchronised.
 * workspace: autosage_workspace_bytes(AUTOSAGE_OP_SPMM, ...) is always enough. */
autosage_status_t autosage_hub_partition(autosage_handle_t h, int64_t n_rows, const int32_t* rowptr,
                                         int32_t hub_t, int32_t hub_chunk,
                                         int32_t* n_hub, int32_t* hub_rows, int32_t* chunk_ptr,
                                         int32_t* n_light, int32_t* light_rows,
                                         void* workspace, size_t workspace_bytes, void* stream);

/* Degree features of the scheduler (feature extraction: rows, nnz, degree distribution).
 * hist[0] = rows of degree 0; hist[b] = rows with 2^(b-1) <= deg < 2^b (host, 33 entries).
 * signature = 64-bit FNV-1a over the little-endian int64 stream n_rows, n_cols, nnz, max_deg,
 * hist[0..32], rowptr[floor(k * n_rows / 1023)] for k = 0..1023.  Synchronises the stream. */
autosage_status_t autosage_graph_features(autosage_handle_t h, int64_t n_rows, int64_t n_cols,
                                          const int32_t* rowptr, int64_t* hist33, int64_t* max_deg,
                                          int64_t* nnz, uint64_t* signature, void* stream);

/* Checks rowptr[0] == 0, monotone rowptr, rowptr[n_rows] == nnz and 0 <= colind < n_cols on the
 * device; synchronises.  Returns AUTOSAGE_ERR_INVALID_ARG when the CSR arrays are inconsistent. */
autosage_status_t autosage_validate_csr(autosage_handle_t h, int64_t n_rows, int64_t n_cols, int64_t nnz,
                                        const int32_t* rowptr, const int32_t* colind, void* stream);

/* 64-bit CSR index arrays (the default of many frameworks) enter through this call: dst[i] = src[i]
 * for i < n as int32, on the device.  The kernels index with int32 (every workload of the paper's
 * evaluation has nnz < 2^31); a value outside [0, limit] (limit <= INT32_MAX: nnz for a row-pointer
 * array, n_cols - 1 for column indices) returns AUTOSAGE_ERR_UNSUPPORTED and leaves dst unspecified.
 * src and dst are device arrays of n elements that do not overlap.  Synchronises the stream. */
autosage_status_t autosage_narrow_indices(autosage_handle_t h, int64_t n, const int64_t* src, int32_t* dst,
                                          int64_t limit, void* stream);

/* ---- selector -------------------------------------------------------------------------- */

/* Shortlist (Scheduler subsection: the estimate step that ranks candidates before any probe).  Host only.
 * From the degree histogram and the widths/alignments it ranks the legal schedules of `op` by an
 * estimated time (seconds, ascending) and writes up to max_out of them.  align_bytes is the
 * largest power of two (<= 16) dividing every dense base pointer and every ld * element size. */
autosage_status_t autosage_shortlist(autosage_handle_t h, autosage_op_t op, int64_t n_rows, int64_t n_cols,
                                     int64_t nnz, const int64_t* hist33, int64_t max_deg, int32_t F,
                                     autosage_dtype_t dt, int32_t align_bytes,
                                     autosage_schedule_t* out, double* est_seconds, int32_t max_out, int32_t* n_out);

/* The decision rule of the decision sketch and Proposition 1, on given probe times (host only):
 * best = first candidate with the strictly smallest time; accepted iff t_best <= alpha * t_baseline.
 * Returns in *choice the accepted candidate's index or -1 for the baseline. */
autosage_status_t autosage_decide_from_times(int32_t n_cand, const double* t_cand, double t_baseline,
                                             double alpha, int32_t* choice);

/* Full decision for one input: cache lookup by (device signature, graph signature, F, op, dt);
 * on a miss: shortlist, probe the baseline and the top-k on a strided row sample of the real
 * operands (outputs are used as probe targets and are left undefined), guardrail, optional
 * full-input confirmation, store.  In replay-only mode a miss returns the baseline schedule and
 * records the miss.  The operand arguments are those of autosage_spmm (op = SPMM: dense0 = B,
 * dense1 = NULL, out = C) or autosage_sddmm (dense0 = X, dense1 = Y, out = out). */
autosage_status_t autosage_decide(autosage_handle_t h, autosage_op_t op, int64_t n_rows, int64_t n_cols,
                                  int64_t nnz, const int32_t* rowptr, const int32_t* colind, const float* val,
                                  const void* dense0, int64_t ld0, const void* dense1, int64_t ld1,
                                  float* out, int64_t ld_out, int32_t F, autosage_dtype_t dt,
                                  void* workspace, size_t workspace_bytes, void* stream,
                                  autosage_schedule_t* chosen);

/* The same decision for CSR attention (key: device signature, graph signature, d, H, dtype).
 * Candidates: single pass and three stages over a few hub thresholds; baseline: three stages without
 * hub split.  O is used as the probe target and is left undefined. */
autosage_status_t autosage_decide_attention(autosage_handle_t h, int64_t N, int64_t nnz, const int32_t* rowptr,
                                            const int32_t* colind, const void* Q, const void* K, const void* V,
                                            float* O, int32_t H, int32_t d, float scale, autosage_dtype_t dt,
                                            void* workspace, size_t workspace_bytes, void* stream,
                                            autosage_schedule_t* chosen);

/* JSON text of the most recent decision of this handle (key, candidates, probe times, choice,
 * alpha, cache hit / replay miss flags).  Truncated to n-1 characters. */
autosage_status_t autosage_last_decision(autosage_handle_t h, char* json_buf, size_t n);

/* Persistent schedule cache: a text file, one record per key.  Load merges into the handle's
 * cache and skips malformed lines; save writes to a temporary file and renames it. */
autosage_status_t autosage_cache_load(autosage_handle_t h, const char* path);
autosage_status_t autosage_cache_save(autosage_handle_t h, const char* path);
autosage_status_t autosage_cache_clear(autosage_handle_t h);
/* Drops the remembered degree features of every graph whose rowptr array started at this device address (host
 * only; the schedule cache, keyed by graph signature, is untouched).  For callers that recycle device memory:
 * call it when the array at that address is freed or overwritten. */
autosage_status_t autosage_forget_graph(autosage_handle_t h, const int32_t* rowptr);
/* Direct access for tests and tools (host only). found = 0/1.  F = feature width (attention: d),
 * H = heads (1 for SpMM / SDDMM). */
autosage_status_t autosage_cache_lookup(autosage_handle_t h, uint64_t graph_sig, int32_t F, int32_t H,
                                        autosage_op_t op, autosage_dtype_t dt, autosage_schedule_t* sched,
                                        int32_t* found);
autosage_status_t autosage_cache_insert(autosage_handle_t h, uint64_t graph_sig, int32_t F, int32_t H,
                                        autosage_op_t op, autosage_dtype_t dt, const autosage_schedule_t* sched);

/* ---- adjoints for training steps ---------------------------------------------------------
 * The paper motivates the operators by training throughput (Introduction) and leaves end-to-end
 * training to future work; these entry points supply what a backward pass needs beyond the forward
 * operators themselves: d/dB (C = A B) = A^T dC needs A^T; d/dval = SDDMM(dC, B) is autosage_sddmm;
 * the row-softmax has its own Jacobian-transpose product. */

/* dS[p,h] = P[p,h] * (dP[p,h] - sum_q P[q,h] dP[q,h]) over the stored entries q of the row of p.
 * P, dP, dS are [nnz, H] fp32 dev arrays; dS may alias dP.  hub_t / hub_chunk / workspace as in
 * autosage_csr_row_softmax (autosage_workspace_bytes(AUTOSAGE_OP_SOFTMAX, ...) is enough). */
autosage_status_t autosage_csr_row_softmax_backward(autosage_handle_t h, int64_t n_rows, int64_t nnz,
                                                    const int32_t* rowptr, const float* P, const float* dP,
                                                    float* dS, int32_t H, int32_t hub_t, int32_t hub_chunk,
                                                    void* workspace, size_t workspace_bytes, void* stream);

/* A^T as CSR.  t_rowptr[n_cols+1], t_colind[nnz] (dev) describe the n_cols x n_rows matrix A^T; inside a
 * row of A^T the entries are in ascending source-row order (storage order for duplicates), so the result
 * is unique.  perm[nnz] (dev, may be NULL) receives the position in A of every entry of A^T; t_val[nnz]
 * (dev) = val[perm] (both NULL for a pattern-only transpose).  Integer outputs are bit-reproducible.
 * The workspace size comes from autosage_csr_transpose_workspace_bytes (three index buffers of nnz
 * entries, a fourth for the sort, and nnz / 16 counters; needs a device handle).  Enqueues only; no
 * synchronisation. */
autosage_status_t autosage_csr_transpose_workspace_bytes(autosage_handle_t h, int64_t n_rows, int64_t n_cols,
                                                         int64_t nnz, size_t* bytes);
autosage_status_t autosage_csr_transpose(autosage_handle_t h, int64_t n_rows, int64_t n_cols, int64_t nnz,
                                         const int32_t* rowptr, const int32_t* colind, const float* val,
                                         int32_t* t_rowptr, int32_t* t_colind, float* t_val, int32_t* perm,
                                         void* workspace, size_t workspace_bytes, void* stream);

/* out[q, 0..width) = in[perm[q], 0..width) for q < n (fp32, dev): carries per-nonzero values (for
 * instance attention probabilities [nnz, H]) into the order of a transposed pattern.  in != out. */
autosage_status_t autosage_gather_values(autosage_handle_t h, int64_t n, int32_t width, const int32_t* perm,
                                         const float* in, float* out, void* stream);

/* Adjoint of autosage_csr_attention (training step around the attention pipeline of the Preliminaries:
 * the chain rule through SpMM, row-softmax and SDDMM, all heads at once).  Given dO = dL/dO it writes
 *   dV[j,h,:] = sum_p P[p,h] dO[i,h,:],   dP[p,h] = <dO[i,h,:], V[j,h,:]>,   dS = softmax'(P, dP),
 *   dQ[i,h,:] = scale sum_p dS[p,h] K[j,h,:],   dK[j,h,:] = scale sum_p dS[p,h] Q[i,h,:]
 * over the stored p = (i, j); the probabilities P are recomputed from Q and K, not stored by the forward.
 * Where the single-pass forward kernels cover (H, d, in_dt), dQ, P and dS come from one pass that reads the K and
 * the V row of every nonzero once (parameter "attention_backward_fused"); dK and dV are per-head-weight SpMMs on
 * the transposed pattern that read P and dS through perm.
 * Q, K, V: [N, H, d] of in_dt (dev); dO, dQ, dK, dV: [N, H, d] fp32 (dev), none aliasing another.
 * (t_rowptr, t_colind, perm) is the transposed pattern as autosage_csr_transpose returns it for the
 * N x N pattern (computed once per graph by the caller).  hub_t / hub_chunk: rows of the pattern and of
 * its transpose with at least hub_t entries are split into chunks (0 = no split).  Shapes as the forward:
 * d * sizeof(in_dt) a multiple of 16, d a multiple of 4, 16-byte aligned tensors, else UNSUPPORTED.
 * Rows without entries get zero gradients.  Deterministic: no atomics, fixed summation orders.
 * Workspace from autosage_csr_attention_backward_workspace_bytes (2 * nnz * H + 3 * N * H floats + hub scratch). */
autosage_status_t autosage_csr_attention_backward_workspace_bytes(autosage_handle_t h, int64_t N, int64_t nnz,
                                                                  int32_t H, int32_t d, int32_t hub_t,
                                                                  int32_t hub_chunk, size_t* bytes);
autosage_status_t autosage_csr_attention_backward(autosage_handle_t h, int64_t N, int64_t nnz,
                                                  const int32_t* rowptr, const int32_t* colind,
                                                  const int32_t* t_rowptr, const int32_t* t_colind,
                                                  const int32_t* perm,
                                                  const void* Q, const void* K, const void* V, const float* dO,
                                                  float* dQ, float* dK, float* dV,
                                                  int32_t H, int32_t d, float scale, autosage_dtype_t in_dt,
                                                  int32_t hub_t, int32_t hub_chunk,
                                                  void* workspace, size_t workspace_bytes, void* stream);

/* Telemetry (Contributions: deployment toggles and telemetry).  Between profile_begin and
 * profile_read every kernel stage the handle launches is bracketed by a pair of HIP events on its
 * stream.  profile_read waits for the recorded stages, writes JSON {"stage":{"calls":n,"total_ms":t},...}
 * (stage names: hub_partition, spmm_rows, spmm_hub, sddmm_rows, sddmm_hub, softmax_rows, softmax_hub,
 * attn_sddmm_rows, attn_sddmm_hub, attn_spmm_rows, attn_spmm_hub, attn_fused_rows, attn_fused_hub, attn_bwd_rows,
 * attn_bwd_hub, attn_bwd_finish, attn_bwd_spmm_rows, attn_bwd_spmm_hub, ...) and
 * switches profiling off. */
autosage_status_t autosage_profile_begin(autosage_handle_t h);
autosage_status_t autosage_profile_read(autosage_handle_t h, char* json_buf, size_t n);

/* Bandwidth probe (Experimental setup: rates are judged against what the device sustains).  Launches one
 * plain streaming kernel over n_bytes (a multiple of 16, both pointers 16-byte aligned, dev) on `stream`:
 *   AUTOSAGE_STREAM_READ     src is read once; dst receives one fp32 partial sum per workgroup and must hold
 *                            autosage_stream_probe_dst_bytes() bytes (their total is the sum of src as fp32)
 *   AUTOSAGE_STREAM_COPY     dst[0 .. n_bytes) = src[0 .. n_bytes)  (n_bytes read + n_bytes written)
 *   AUTOSAGE_STREAM_INPLACE  dst[i] = 0.5 * dst[i] over n_bytes of fp32 (src unused, may be NULL)
 * n_bytes = 0 is valid (src may then be NULL).  The caller times it (HIP events, median of repeats);
 * nothing is allocated, nothing synchronises. */
typedef enum { AUTOSAGE_STREAM_READ = 0, AUTOSAGE_STREAM_COPY = 1, AUTOSAGE_STREAM_INPLACE = 2 } autosage_stream_mode_t;
autosage_status_t autosage_stream_probe(autosage_handle_t h, autosage_stream_mode_t mode, const void* src, void* dst,
                                        size_t n_bytes, void* stream);
autosage_status_t autosage_stream_probe_dst_bytes(autosage_handle_t h, size_t* bytes);

/* Gather probe (same purpose: the ceiling of the access pattern the sparse kernels are bound by).  Launches one
 * kernel that reads n_idx whole rows of row_bytes bytes (a power of two, 16 .. 1024) out of `table`
 * ([n_table_rows, row_bytes], dev, 16-byte aligned) at the row numbers idx[0 .. n_idx) (int32, dev; values outside
 * the table are clamped into it), in the access pattern of the SpMM / SDDMM / attention kernels: 64 indices per
 * coalesced load, row_bytes / 16 lanes per row, four 16-byte loads in flight per lane.  dst (dev,
 * autosage_stream_probe_dst_bytes() bytes) receives one fp32 partial sum per workgroup; their total is the sum of
 * all fp32 elements of the gathered rows.  A table that fits the L2 caches, the Infinity Cache or neither gives
 * the ceiling of the respective regime.  n_idx = 0 is valid.  The caller times it; nothing is allocated, nothing
 * synchronises. */
autosage_status_t autosage_gather_probe(autosage_handle_t h, const void* table, int64_t n_table_rows, int32_t row_bytes,
                                        const int32_t* idx, int64_t n_idx, float* dst, void* stream);

/* The baseline (fallback) schedule of the guardrail: plain one-wavefront-per-row kernel. */
autosage_status_t autosage_baseline_schedule(autosage_schedule_t* out);

#ifdef __cplusplus
}
#endif
#endif /* AUTOSAGE_H */

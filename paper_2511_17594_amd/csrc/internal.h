// Host-side internals of the library: the handle, schedule resolution, workspace layout,
// stage execution and the selector.  Not part of the public ABI.
#pragma once
#include <hip/hip_runtime_api.h>

#include <map>
#include <string>
#include <tuple>
#include <vector>

#include "../../include/autosage.h"
#include "launch.h"

namespace autosage {

struct CacheKey {
    uint64_t graph_sig;
    int32_t F;      // feature width (attention: head width d)
    int32_t H;      // heads (1 for SpMM / SDDMM)
    int32_t op;
    int32_t dt;
    bool operator<(const CacheKey& o) const
    {
        return std::tie(graph_sig, F, H, op, dt) < std::tie(o.graph_sig, o.F, o.H, o.op, o.dt);
    }
};

// One CSR-attention call (device pointers).
struct AttnCall {
    int64_t N, nnz;
    const int32_t* rowptr;
    const int32_t* colind;
    const void* Q;
    const void* K;
    const void* V;
    float* O;
    int32_t H, d;
    float scale;
    int dt;
};

struct CacheEntry {
    autosage_schedule_t sched;
    double t_baseline_ms;
    double t_chosen_ms;
};

struct SigMemo {
    const void* rowptr;
    int64_t n_rows;
    int64_t n_cols;
    int64_t nnz;
    uint64_t sig;
    int64_t hist[33];
    int64_t max_deg;
};

struct Params {
    double alpha = 0.95;
    double probe_frac = 0.02;
    int probe_iters = 5;
    double probe_cap_ms = 1.0;
    int probe_topk = 4;
    int probe_min_rows = 16384;
    int probe_refine = 8;     // most extra probes of the refinement rounds around the best probed schedule (0 = none)
    int replay_only = 0;
    int confirm_full = 1;
    int memoize_signature = 1;
    int baseline_bound = 1;   // 1: time the baseline's light rows first and the whole baseline only when that bound does not decide
    // forced knobs from the environment (0 = not forced)
    int force_ftile = 0;
    int force_wpb = 0;
    int force_hub_t = -1;     // -1 = not forced, 0 = forced off
    // row-softmax: lanes per light row (0 = from the mean row length, < 0 = one wavefront per row)
    int softmax_group = 0;
    // attention backward: 1 = dQ, P and dS from one pass over K and V where the single-pass kernels cover the shape,
    // 0 = always the chain rule stage by stage
    int attention_backward_fused = 1;
};

}  // namespace autosage

struct autosage_ctx {
    int device = -1;                       // < 0: host-only handle
    std::string device_sig = "host";
    int cu_count = 0;
    autosage::Params params;
    std::map<autosage::CacheKey, autosage::CacheEntry> cache;
    std::string cache_path;                // from AUTOSAGE_CACHE; saved on destroy
    std::string last_decision = "{}";
    std::vector<autosage::SigMemo> memo;
    int64_t* dev_features = nullptr;       // int64[35 + 1024]
    int64_t* host_features = nullptr;      // pinned mirror
    int32_t* dev_flag = nullptr;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    // per-stage telemetry (autosage_profile_begin / autosage_profile_read)
    bool profiling = false;
    struct StageSpan {
        const char* stage;
        hipEvent_t start, stop;
    };
    std::vector<StageSpan> spans;
    size_t spans_used = 0;
    // > 0 while the selector times a lower bound of the baseline: the row kernels of the next launches skip
    // rows of at least this many entries and no hub kernel runs (outputs of skipped rows stay untouched)
    int probe_skip_deg = 0;
    // device address of the library's fixed scratch array on this handle's device (autosage_spmm_static)
    void* static_scratch = nullptr;
};

namespace autosage {

constexpr int kMinHubT = 64;               // smallest split threshold the library accepts
// The kernels hold nonzero positions and row numbers in int32 and step them by at most one chunk or one
// workgroup's stride past the end of a row: both limits together keep every such sum below 2^31.
constexpr int kMaxHubChunk = 1 << 20;                                  // longest chunk of a split row
constexpr int64_t kMaxNnz = (int64_t(1) << 31) - (int64_t(1) << 20);   // most nonzeros, and most rows, of a call
constexpr int kBaselineBoundDeg = 1024;     // rows this long are left out when the selector bounds the baseline from below
constexpr int kSelectorMinHubT = 512;      // smallest threshold the selector proposes for SpMM / SDDMM
constexpr int kSelectorMinChunk = 256;     // shortest hub chunk the selector proposes
constexpr double kRefineGain = 0.97;        // a refinement probe must take at most this share of the best time so far to count
constexpr double kFullInputCapMs = 1.0;     // full-input confirmation: timed runs stop once this is spent; a warm-up of 4x this is the measurement
constexpr double kTileOperandBytes = 96.0 * 1024 * 1024;
constexpr double kHeadTileOperandBytes = 256.0 * 1024 * 1024;   // K + V above this: the single-pass attention is also tried with head tiles   // dense operands above this get narrow-tile candidates

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Chunk length in force for a threshold: an explicit one as given, else the threshold itself (at most
// kMaxHubChunk); 0 when rows are not split.
inline int effective_hub_chunk(int hub_t, int hub_chunk)
{
    if (hub_t <= 0) return 0;
    if (hub_chunk > 0) return hub_chunk;
    return hub_t < kMaxHubChunk ? hub_t : kMaxHubChunk;
}

// Largest power of two <= 16 that divides the pointer value and ld * elem_size.
int common_alignment(const void* p, int64_t ld, int elem_size);

// Resolves the "auto" fields of a schedule for an op of width F (per-head width for SDDMM with heads).
// align_in: alignment of the dense inputs, align_out: of the dense output (SpMM) or 16 when scalar stores are used.
autosage_status_t resolve_schedule(const autosage_schedule_t& s, int op, int32_t F, int dt, int heads,
                                   int align_in, int align_out, Resolved* out);

// Upper bounds of hub rows / chunks for `count` rows holding at most nnz nonzeros.
void hub_caps(int64_t count, int64_t nnz, int hub_t, int hub_chunk, int* cap_hub, int* cap_chunks);

// Workspace needed by one explicit schedule (bytes).  part_floats_per_chunk: F for SpMM, 2*H for softmax, 0 for SDDMM.
size_t hub_workspace_bytes(int64_t count, int64_t nnz, int hub_t, int hub_chunk, int64_t part_floats_per_chunk);

// Carves the hub metadata and the partial buffer out of ws; returns false when ws is too small.
bool carve_hub(void* ws, size_t ws_bytes, int64_t count, int64_t nnz, int hub_t, int hub_chunk,
               int64_t part_floats_per_chunk, HubMeta* meta, float** part, size_t* used);

autosage_status_t exec_spmm(autosage_ctx* h, const SpmmArgs& a, const Resolved& r, int64_t nnz, void* ws, size_t ws_bytes,
                            hipStream_t st);
autosage_status_t exec_sddmm(autosage_ctx* h, const SddmmArgs& a, const Resolved& r, int64_t nnz, void* ws, size_t ws_bytes,
                             hipStream_t st);

// Body of autosage_spmm (argument checks, selector when sched is NULL, schedule resolution, launches).
autosage_status_t spmm_entry(autosage_ctx* h, int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t* rowptr,
                             const int32_t* colind, const float* val, const void* B, int64_t ldb, float* C, int64_t ldc,
                             int32_t F, int dt, const autosage_schedule_t* sched, void* workspace, size_t workspace_bytes,
                             void* stream);
// Device address of the fixed scratch array on `device` (which must be the current device); looked up once per device.
autosage_status_t static_scratch_address(int device, void** ptr);

// Checks the 16-byte alignment / width rules of the attention kernels.
autosage_status_t attention_alignment(const AttnCall& c);
// Runs the attention pipeline the schedule names (FUSED = single pass, else three stages) on `rows`.
autosage_status_t exec_attention(autosage_ctx* h, const AttnCall& c, const autosage_schedule_t& sched, const RowMap& rows,
                                 void* workspace, size_t workspace_bytes, hipStream_t st);

// Brackets one kernel stage with a pair of events on its stream while profiling is on.
class StageTimer {
public:
    StageTimer(autosage_ctx* h, const char* stage, hipStream_t st);
    ~StageTimer();
    StageTimer(const StageTimer&) = delete;
    StageTimer& operator=(const StageTimer&) = delete;

private:
    autosage_ctx* h_;
    hipStream_t st_;
    hipEvent_t stop_ = nullptr;
};

// Host-only selector pieces
int decide_from_times(int n, const double* t, double tb, double alpha);
void shortlist(const autosage_ctx* h, int op, int64_t n_rows, int64_t n_cols, int64_t nnz, const int64_t* hist33,
               int64_t max_deg, int32_t F, int dt, int align_bytes, std::vector<autosage_schedule_t>* out,
               std::vector<double>* est);
uint64_t signature_from_features(int64_t n_rows, int64_t n_cols, const int64_t* feat /* hist33, max, nnz, 1024 samples */);
autosage_schedule_t baseline_schedule();
std::string schedule_json(const autosage_schedule_t& s);

}  // namespace autosage

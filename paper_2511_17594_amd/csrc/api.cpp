// C ABI of the library: argument checking, schedule resolution, workspace layout and the
// sequencing of the kernel stages.  See include/autosage.h for the contract of every entry point.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "internal.h"

using namespace autosage;

#define HIP_TRY(expr)                                   \
    do {                                                \
        hipError_t e__ = (expr);                        \
        if (e__ != hipSuccess) return AUTOSAGE_ERR_HIP; \
    } while (0)

namespace autosage {

int common_alignment(const void* p, int64_t ld, int elem_size)
{
    uint64_t v = reinterpret_cast<uint64_t>(p) | static_cast<uint64_t>(ld * elem_size) | 16u;
    int a = 1;
    while ((v & 1u) == 0 && a < 16) {
        v >>= 1;
        a <<= 1;
    }
    return a;
}

static int pow2_ceil(int x)
{
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}

static bool is_pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

// chunk counts per lane that have kernels: 1, 2, 3, 4, 6, 8
static int round_chunks(int k)
{
    if (k <= 4) return k;
    if (k <= 6) return 6;
    return 8;
}

autosage_schedule_t baseline_schedule()
{
    autosage_schedule_t s{};
    s.mapping = AUTOSAGE_MAP_PLAIN;
    s.f_tile = 64;
    s.waves_per_wg = 4;
    s.vec_bytes = 0;
    s.unroll = 0;
    s.hub_t = 0;
    s.hub_chunk = 0;
    s.xcd_remap = 0;
    return s;
}

autosage_status_t resolve_schedule(const autosage_schedule_t& s, int op, int32_t F, int dt, int heads,
                                   int align_in, int align_out, Resolved* out)
{
    const int esize = dtype_bytes(dt);
    Resolved r{};
    if (F <= 0 || heads < 1) return AUTOSAGE_ERR_INVALID_ARG;
    if (s.mapping < AUTOSAGE_MAP_PLAIN || s.mapping > AUTOSAGE_MAP_MULTI_ROW) return AUTOSAGE_ERR_INVALID_ARG;
    r.mapping = s.mapping;
    r.wpg = s.waves_per_wg == 0 ? 4 : s.waves_per_wg;
    if (!(r.wpg == 1 || r.wpg == 2 || r.wpg == 4 || r.wpg == 8 || r.wpg == 16)) return AUTOSAGE_ERR_INVALID_ARG;
    r.unroll = s.unroll == 0 ? 4 : s.unroll;
    if (!(r.unroll == 1 || r.unroll == 2 || r.unroll == 4 || r.unroll == 8)) return AUTOSAGE_ERR_INVALID_ARG;
    if (s.hub_t < 0 || s.hub_chunk < 0 || (s.hub_t > 0 && s.hub_t < kMinHubT)) return AUTOSAGE_ERR_INVALID_ARG;
    r.hub_t = s.hub_t;
    r.hub_chunk = effective_hub_chunk(s.hub_t, s.hub_chunk);
    if (r.hub_t > 0 && (r.hub_chunk < kMinHubT || r.hub_chunk > kMaxHubChunk)) return AUTOSAGE_ERR_INVALID_ARG;
    r.xcd_remap = s.xcd_remap ? 1 : 0;
    r.HW = 1;
    if (s.group_lanes < 0 || s.group_lanes > 64 || (s.group_lanes > 0 && !is_pow2(s.group_lanes))) return AUTOSAGE_ERR_INVALID_ARG;
    if (s.group_lanes > 0 && op != AUTOSAGE_OP_SDDMM) return AUTOSAGE_ERR_UNSUPPORTED;

    // vector width
    int vb = s.vec_bytes;
    if (vb != 0 && vb != 2 && vb != 4 && vb != 8 && vb != 16) return AUTOSAGE_ERR_INVALID_ARG;
    auto legal = [&](int bytes) {
        if (bytes < esize) return false;
        const int vec = bytes / esize;
        if (F % vec != 0) return false;
        if (align_in % bytes != 0 && bytes > esize) return false;
        const int store_bytes = vec * 4 < 16 ? vec * 4 : 16;       // SpMM stores VEC fp32 values per lane
        if (op == AUTOSAGE_OP_SPMM && store_bytes > 4 && align_out % store_bytes != 0) return false;
        return true;
    };
    if (s.mapping == AUTOSAGE_MAP_PLAIN) {
        if (vb != 0 && vb != esize) return AUTOSAGE_ERR_UNSUPPORTED;
        vb = esize;
    } else if (vb == 0) {
        for (int cand = 16; cand >= esize; cand >>= 1) {
            if (legal(cand)) {
                vb = cand;
                break;
            }
        }
        if (vb == 0) vb = esize;
    } else if (!legal(vb)) {
        return AUTOSAGE_ERR_UNSUPPORTED;
    }
    r.vec = vb / esize;

    const int lanes_needed = (F + r.vec - 1) / r.vec;
    if (s.mapping == AUTOSAGE_MAP_PLAIN) {
        r.G = 64;
        r.K = 1;
        r.f_tile = 64;
        r.tiles = (F + 63) / 64;
        if (r.hub_t > 0) {
            // the plain kernel only serves the light rows; hub chunks run the wavefront-per-row shape
            autosage_schedule_t hub = s;
            hub.mapping = AUTOSAGE_MAP_WAVE_ROW;
            hub.vec_bytes = 0;
            hub.f_tile = 0;
            Resolved hr;
            autosage_status_t rc = resolve_schedule(hub, op, F, dt, heads, align_in, align_out, &hr);
            if (rc != AUTOSAGE_OK) return rc;
            hr.mapping = AUTOSAGE_MAP_PLAIN;
            r = hr;
        }
        *out = r;
        return AUTOSAGE_OK;
    }
    int lanes_tile;
    if (s.f_tile == 0) {
        lanes_tile = lanes_needed <= 64 ? pow2_ceil(lanes_needed) : 64 * round_chunks((lanes_needed + 63) / 64 > 8 ? 4 : (lanes_needed + 63) / 64);
    } else {
        if (s.f_tile < 0 || s.f_tile % r.vec != 0) return AUTOSAGE_ERR_INVALID_ARG;
        lanes_tile = s.f_tile / r.vec;
        if (lanes_tile <= 64) {
            if (!is_pow2(lanes_tile)) return AUTOSAGE_ERR_INVALID_ARG;
        } else {
            if (lanes_tile % 64 != 0) return AUTOSAGE_ERR_INVALID_ARG;
            const int k = lanes_tile / 64;
            if (k > 8 || round_chunks(k) != k) return AUTOSAGE_ERR_INVALID_ARG;
        }
        // a tile wider than needed is trimmed to the smallest shape covering F
        if (lanes_tile > pow2_ceil(lanes_needed) && lanes_needed <= 64) lanes_tile = pow2_ceil(lanes_needed);
    }
    if (lanes_tile <= 64) {
        r.G = lanes_tile;
        r.K = 1;
    } else {
        r.G = 64;
        r.K = lanes_tile / 64;
    }
    r.f_tile = r.G * r.vec * r.K;
    r.tiles = (F + r.f_tile - 1) / r.f_tile;

    if (op == AUTOSAGE_OP_SDDMM) {
        // A dot product sits in one pass of one group, except for an explicit narrower tile with one head:
        // then the tiles run as consecutive launches that add their partial dots into the output.
        if (r.tiles != 1 && !(s.f_tile > 0 && heads == 1)) {
            r.G = 64;
            r.K = round_chunks((lanes_needed + 63) / 64);
            if ((lanes_needed + 63) / 64 > 8) return AUTOSAGE_ERR_UNSUPPORTED;
            r.f_tile = r.G * r.vec * r.K;
            r.tiles = 1;
        }
        if (s.group_lanes > 0 && s.group_lanes < r.G) {
            // narrow groups: the tile's vectors are spread over group_lanes lanes, K of them per lane
            const int g = s.group_lanes, k = r.G / g;
            const bool built = (g == 32 && k == 2) || (g == 16 && (k == 2 || k == 4)) || (g == 8 && (k == 2 || k == 4 || k == 8)) ||
                               (g == 4 && (k == 4 || k == 8));
            if (heads != 1 || vb != 16 || r.K != 1 || s.mapping != AUTOSAGE_MAP_WAVE_ROW || !built) return AUTOSAGE_ERR_UNSUPPORTED;
            r.K = k;
            r.G = g;
        }
        if (heads > 1 && vb == 16 && r.K == 1 && r.G >= 2 && r.G <= 32) {
            int hw = pow2_ceil(heads);
            if (hw > 64 / r.G) hw = 64 / r.G;
            r.HW = hw;
        }
    }
    if (s.mapping == AUTOSAGE_MAP_MULTI_ROW && (r.G * r.HW > 32 || r.K != 1 || r.HW != 1)) return AUTOSAGE_ERR_UNSUPPORTED;
    *out = r;
    return AUTOSAGE_OK;
}

void hub_caps(int64_t count, int64_t nnz, int hub_t, int hub_chunk, int* cap_hub, int* cap_chunks)
{
    if (hub_t <= 0) {
        *cap_hub = 0;
        *cap_chunks = 0;
        return;
    }
    int64_t ch = nnz / hub_t;
    if (ch > count) ch = count;
    int64_t cc = nnz / hub_chunk + ch;
    *cap_hub = static_cast<int>(ch);
    *cap_chunks = static_cast<int>(cc);
}

static size_t hub_meta_bytes(int64_t count, int cap_hub)
{
    const int64_t part_blocks = (count + 1023) / 1024;
    size_t b = 256;                                                    // HubCounts
    b += align_up(sizeof(int32_t) * 2 * (size_t)(part_blocks > 0 ? part_blocks : 1), 256);
    b += align_up(sizeof(int32_t) * (size_t)(cap_hub > 0 ? cap_hub : 1), 256);          // hub_rows
    b += align_up(sizeof(int32_t) * ((size_t)cap_hub + 1), 256);                      // chunk_ptr
    return b;
}

size_t hub_workspace_bytes(int64_t count, int64_t nnz, int hub_t, int hub_chunk, int64_t part_floats_per_chunk)
{
    if (hub_t <= 0) return 0;
    int cap_hub, cap_chunks;
    hub_caps(count, nnz, hub_t, hub_chunk, &cap_hub, &cap_chunks);
    return hub_meta_bytes(count, cap_hub) + align_up(sizeof(float) * (size_t)cap_chunks * (size_t)part_floats_per_chunk, 256);
}

bool carve_hub(void* ws, size_t ws_bytes, int64_t count, int64_t nnz, int hub_t, int hub_chunk,
               int64_t part_floats_per_chunk, HubMeta* meta, float** part, size_t* used)
{
    int cap_hub, cap_chunks;
    hub_caps(count, nnz, hub_t, hub_chunk, &cap_hub, &cap_chunks);
    const size_t need = hub_workspace_bytes(count, nnz, hub_t, hub_chunk, part_floats_per_chunk);
    if (used) *used = need;
    if (ws == nullptr || ws_bytes < need || (reinterpret_cast<uint64_t>(ws) & 255u) != 0) return false;
    char* p = static_cast<char*>(ws);
    const int64_t part_blocks = (count + 1023) / 1024;
    meta->counts = reinterpret_cast<HubCounts*>(p);
    p += 256;
    meta->block_counts = reinterpret_cast<int32_t*>(p);
    p += align_up(sizeof(int32_t) * 2 * (size_t)(part_blocks > 0 ? part_blocks : 1), 256);
    meta->hub_rows = reinterpret_cast<int32_t*>(p);
    p += align_up(sizeof(int32_t) * (size_t)(cap_hub > 0 ? cap_hub : 1), 256);
    meta->chunk_ptr = reinterpret_cast<int32_t*>(p);
    p += align_up(sizeof(int32_t) * ((size_t)cap_hub + 1), 256);
    meta->light_rows = nullptr;
    meta->cap_hub = cap_hub;
    meta->cap_chunks = cap_chunks;
    if (part) *part = reinterpret_cast<float*>(p);
    return true;
}

StageTimer::StageTimer(autosage_ctx* h, const char* stage, hipStream_t st) : h_(h), st_(st)
{
    if (!h_ || !h_->profiling) return;
    if (h_->spans_used == h_->spans.size()) {
        autosage_ctx::StageSpan s{stage, nullptr, nullptr};
        if (hipEventCreate(&s.start) != hipSuccess || hipEventCreate(&s.stop) != hipSuccess) return;
        h_->spans.push_back(s);
    }
    autosage_ctx::StageSpan& s = h_->spans[h_->spans_used++];
    s.stage = stage;
    (void)hipEventRecord(s.start, st_);
    stop_ = s.stop;
}

StageTimer::~StageTimer()
{
    if (stop_) (void)hipEventRecord(stop_, st_);
}

#define STAGE(h, name, st, call)      \
    do {                              \
        StageTimer timer__(h, name, st); \
        HIP_TRY(call);                \
    } while (0)

autosage_status_t exec_spmm(autosage_ctx* h, const SpmmArgs& a, const Resolved& r, int64_t nnz, void* ws, size_t ws_bytes,
                            hipStream_t st)
{
    if (a.rows.count == 0) return AUTOSAGE_OK;
    if (h->probe_skip_deg > 0) {                // lower bound of a schedule: its light rows only
        Resolved light = r;
        light.hub_t = h->probe_skip_deg;
        STAGE(h, "spmm_rows", st, launch_spmm_rows(a, light, st));
        return AUTOSAGE_OK;
    }
    HubMeta meta{};
    float* part = nullptr;
    if (r.hub_t > 0) {
        if (!carve_hub(ws, ws_bytes, a.rows.count, nnz, r.hub_t, r.hub_chunk, a.F, &meta, &part, nullptr))
            return AUTOSAGE_ERR_WORKSPACE_TOO_SMALL;
        STAGE(h, "hub_partition", st, launch_hub_partition(a.rows, a.rowptr, r.hub_t, r.hub_chunk, meta, st));
    }
    STAGE(h, "spmm_rows", st, launch_spmm_rows(a, r, st));
    if (r.hub_t > 0) STAGE(h, "spmm_hub", st, launch_spmm_hub(a, r, meta, part, st));
    return AUTOSAGE_OK;
}

autosage_status_t exec_sddmm(autosage_ctx* h, const SddmmArgs& a, const Resolved& r, int64_t nnz, void* ws, size_t ws_bytes,
                             hipStream_t st)
{
    if (a.rows.count == 0) return AUTOSAGE_OK;
    if (h->probe_skip_deg > 0 && (r.tiles <= 1 || r.mapping == MAP_PLAIN)) {
        Resolved light = r;
        light.hub_t = h->probe_skip_deg;
        STAGE(h, "sddmm_rows", st, launch_sddmm_rows(a, light, st));
        return AUTOSAGE_OK;
    }
    HubMeta meta{};
    if (r.hub_t > 0) {
        if (!carve_hub(ws, ws_bytes, a.rows.count, nnz, r.hub_t, r.hub_chunk, 0, &meta, nullptr, nullptr))
            return AUTOSAGE_ERR_WORKSPACE_TOO_SMALL;
        STAGE(h, "hub_partition", st, launch_hub_partition(a.rows, a.rowptr, r.hub_t, r.hub_chunk, meta, st));
    }
    if (r.tiles > 1 && r.mapping != MAP_PLAIN) {
        // feature tiles one after the other (stream order makes the read-modify-write of `out` safe): the slice
        // of Y that a tile gathers from is n_cols * f_tile elements, small enough to stay in the caches
        const int ex = a.x_f32 ? 4 : dtype_bytes(a.dt), ey = dtype_bytes(a.dt);
        Resolved rt = r;
        rt.tiles = 1;
        for (int t = 0; t < r.tiles; ++t) {
            SddmmArgs at = a;
            const int f0 = t * r.f_tile;
            at.X = static_cast<const char*>(a.X) + (size_t)f0 * ex;
            at.Y = static_cast<const char*>(a.Y) + (size_t)f0 * ey;
            at.F = std::min(r.f_tile, a.F - f0);
            at.accumulate = t > 0 ? 1 : 0;
            STAGE(h, "sddmm_rows", st, launch_sddmm_rows(at, rt, st));
            if (r.hub_t > 0) STAGE(h, "sddmm_hub", st, launch_sddmm_hub(at, rt, meta, st));
        }
        return AUTOSAGE_OK;
    }
    STAGE(h, "sddmm_rows", st, launch_sddmm_rows(a, r, st));
    if (r.hub_t > 0) STAGE(h, "sddmm_hub", st, launch_sddmm_hub(a, r, meta, st));
    return AUTOSAGE_OK;
}

}  // namespace autosage

// ------------------------------------------------------------------------------------------
// lifetime
// ------------------------------------------------------------------------------------------
static double env_double(const char* name, double dflt)
{
    const char* v = std::getenv(name);
    if (!v || !*v) return dflt;
    char* end = nullptr;
    const double x = std::strtod(v, &end);
    return end == v ? dflt : x;
}

extern "C" autosage_status_t autosage_create(autosage_handle_t* out, int device_id)
{
    if (!out) return AUTOSAGE_ERR_INVALID_ARG;
    autosage_ctx* h = new (std::nothrow) autosage_ctx();
    if (!h) return AUTOSAGE_ERR_HIP;
    h->device = device_id;
    Params& p = h->params;
    p.alpha = env_double("AUTOSAGE_ALPHA", p.alpha);
    p.probe_frac = env_double("AUTOSAGE_PROBE_FRAC", p.probe_frac);
    p.probe_iters = std::max(1, (int)env_double("AUTOSAGE_PROBE_ITERS", p.probe_iters));
    p.probe_cap_ms = env_double("AUTOSAGE_PROBE_CAP_MS", p.probe_cap_ms);
    p.probe_topk = (int)env_double("AUTOSAGE_PROBE_TOPK", p.probe_topk);
    p.probe_min_rows = (int)env_double("AUTOSAGE_PROBE_MIN_ROWS", p.probe_min_rows);
    p.probe_refine = std::max(0, (int)env_double("AUTOSAGE_PROBE_REFINE", p.probe_refine));
    p.replay_only = (int)env_double("AUTOSAGE_REPLAY_ONLY", 0);
    p.force_ftile = (int)env_double("AUTOSAGE_FTILE", 0);
    p.force_wpb = (int)env_double("AUTOSAGE_WPB", 0);
    p.force_hub_t = (int)env_double("AUTOSAGE_HUB_T", -1);
    if (device_id >= 0) {
        hipDeviceProp_t prop;
        if (hipSetDevice(device_id) != hipSuccess || hipGetDeviceProperties(&prop, device_id) != hipSuccess) {
            delete h;
            return AUTOSAGE_ERR_HIP;
        }
        int rt = 0;
        (void)hipRuntimeGetVersion(&rt);
        h->cu_count = prop.multiProcessorCount;
        char buf[256];
        std::snprintf(buf, sizeof buf, "%s_%dcu_hip%d_lib2", prop.gcnArchName, prop.multiProcessorCount, rt);
        h->device_sig = buf;
        for (char& c : h->device_sig)
            if (c == ' ' || c == '\t') c = '_';
        if (hipMalloc(&h->dev_features, sizeof(int64_t) * (35 + 1024)) != hipSuccess ||
            hipHostMalloc(&h->host_features, sizeof(int64_t) * (35 + 1024)) != hipSuccess ||
            hipMalloc(&h->dev_flag, 256) != hipSuccess || hipEventCreate(&h->ev0) != hipSuccess ||
            hipEventCreate(&h->ev1) != hipSuccess) {
            autosage_destroy(h);
            return AUTOSAGE_ERR_HIP;
        }
        // the fixed scratch array of autosage_spmm_static: its address on this device (no allocation)
        if (static_scratch_address(device_id, &h->static_scratch) != AUTOSAGE_OK) {
            autosage_destroy(h);
            return AUTOSAGE_ERR_HIP;
        }
    }
    const char* cp = std::getenv("AUTOSAGE_CACHE");
    if (cp && *cp) {
        h->cache_path = cp;
        autosage_cache_load(h, cp);        // a missing or broken file is not an error at start-up
    }
    *out = h;
    return AUTOSAGE_OK;
}

extern "C" autosage_status_t autosage_destroy(autosage_handle_t h)
{
    if (!h) return AUTOSAGE_ERR_INVALID_ARG;
    autosage_status_t st = AUTOSAGE_OK;
    if (!h->cache_path.empty()) st = autosage_cache_save(h, h->cache_path.c_str());
    if (h->dev_features) (void)hipFree(h->dev_features);
    if (h->host_features) (void)hipHostFree(h->host_features);
    if (h->dev_flag) (void)hipFree(h->dev_flag);
    if (h->ev0) (void)hipEventDestroy(h->ev0);
    if (h->ev1) (void)hipEventDestroy(h->ev1);
    for (auto& s : h->spans) {
        if (s.start) (void)hipEventDestroy(s.start);
        if (s.stop) (void)hipEventDestroy(s.stop);
    }
    delete h;
    return st;
}

extern "C" const char* autosage_status_string(autosage_status_t s)
{
    switch (s) {
        case AUTOSAGE_OK: return "ok";
        case AUTOSAGE_ERR_INVALID_ARG: return "invalid argument";
        case AUTOSAGE_ERR_UNSUPPORTED: return "unsupported schedule, dtype or shape";
        case AUTOSAGE_ERR_WORKSPACE_TOO_SMALL: return "workspace too small or misaligned";
        case AUTOSAGE_ERR_HIP: return "HIP runtime error";
        case AUTOSAGE_ERR_IO: return "file I/O error";
        case AUTOSAGE_ERR_REPLAY_MISS: return "replay-only mode: key not in cache";
        default: return "unknown status";
    }
}

namespace {
struct ParamRef {
    const char* name;
    int kind;   // 0 double, 1 int
    void* (*get)(Params&);
};
}  // namespace

static bool param_access(Params& p, const char* name, double* value, bool set)
{
#define P_DOUBLE(nm, field)                 \
    if (std::strcmp(name, nm) == 0) {       \
        if (set) p.field = *value;          \
        else *value = p.field;              \
        return true;                        \
    }
#define P_INT(nm, field)                    \
    if (std::strcmp(name, nm) == 0) {       \
        if (set) p.field = (int)*value;     \
        else *value = (double)p.field;      \
        return true;                        \
    }
    P_DOUBLE("alpha", alpha)
    P_DOUBLE("probe_frac", probe_frac)
    P_INT("probe_iters", probe_iters)
    P_DOUBLE("probe_cap_ms", probe_cap_ms)
    P_INT("probe_topk", probe_topk)
    P_INT("probe_min_rows", probe_min_rows)
    P_INT("probe_refine", probe_refine)
    P_INT("replay_only", replay_only)
    P_INT("confirm_full", confirm_full)
    P_INT("memoize_signature", memoize_signature)
    P_INT("baseline_bound", baseline_bound)
    P_INT("force_ftile", force_ftile)
    P_INT("force_wpb", force_wpb)
    P_INT("force_hub_t", force_hub_t)
    P_INT("softmax_group", softmax_group)
    P_INT("attention_backward_fused", attention_backward_fused)
#undef P_DOUBLE
#undef P_INT
    return false;
}

extern "C" autosage_status_t autosage_set_param(autosage_handle_t h, const char* name, double value)
{
    if (!h || !name || std::isnan(value)) return AUTOSAGE_ERR_INVALID_ARG;
    if (std::strcmp(name, "alpha") == 0 && value <= 0) return AUTOSAGE_ERR_INVALID_ARG;
    if (std::strcmp(name, "probe_frac") == 0 && (value <= 0 || value > 1)) return AUTOSAGE_ERR_INVALID_ARG;
    if (std::strcmp(name, "probe_iters") == 0 && value < 1) return AUTOSAGE_ERR_INVALID_ARG;
    return param_access(h->params, name, &value, true) ? AUTOSAGE_OK : AUTOSAGE_ERR_INVALID_ARG;
}

extern "C" autosage_status_t autosage_get_param(autosage_handle_t h, const char* name, double* value)
{
    if (!h || !name || !value) return AUTOSAGE_ERR_INVALID_ARG;
    return param_access(h->params, name, value, false) ? AUTOSAGE_OK : AUTOSAGE_ERR_INVALID_ARG;
}

extern "C" autosage_status_t autosage_baseline_schedule(autosage_schedule_t* out)
{
    if (!out) return AUTOSAGE_ERR_INVALID_ARG;
    *out = baseline_schedule();
    return AUTOSAGE_OK;
}

// ------------------------------------------------------------------------------------------
// hot path
// ------------------------------------------------------------------------------------------
static bool sizes_ok(int64_t n_rows, int64_t n_cols, int64_t nnz)
{
    return n_rows >= 0 && n_cols >= 0 && nnz >= 0 && nnz <= kMaxNnz && n_rows <= kMaxNnz && n_cols < (int64_t(1) << 31);
}

namespace autosage {

autosage_status_t spmm_entry(autosage_ctx* h, int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t* rowptr,
                             const int32_t* colind, const float* val, const void* B, int64_t ldb, float* C, int64_t ldc,
                             int32_t F, int dt, const autosage_schedule_t* sched, void* workspace, size_t workspace_bytes,
                             void* stream)
{
    if (!h || !sizes_ok(n_rows, n_cols, nnz) || F <= 0 || ldb < F || ldc < F) return AUTOSAGE_ERR_INVALID_ARG;
    if (!dtype_known(dt)) return AUTOSAGE_ERR_INVALID_ARG;
    if (h->device < 0) return AUTOSAGE_ERR_UNSUPPORTED;
    if (n_rows == 0) return AUTOSAGE_OK;
    if (!rowptr || !C || (nnz > 0 && (!colind || !val || !B))) return AUTOSAGE_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    autosage_schedule_t chosen;
    if (!sched) {
        autosage_status_t s = autosage_decide(h, AUTOSAGE_OP_SPMM, n_rows, n_cols, nnz, rowptr, colind, val, B, ldb,
                                              nullptr, 0, C, ldc, F, (autosage_dtype_t)dt, workspace, workspace_bytes, stream,
                                              &chosen);
        if (s != AUTOSAGE_OK) return s;
        sched = &chosen;
    }
    const int esize = dtype_bytes(dt);
    Resolved r;
    autosage_status_t s = resolve_schedule(*sched, AUTOSAGE_OP_SPMM, F, dt, 1, common_alignment(B, ldb, esize),
                                           common_alignment(C, ldc, 4), &r);
    if (s == AUTOSAGE_ERR_UNSUPPORTED && sched == &chosen) {
        // a replayed decision was made for other strides or alignments: the baseline always applies
        chosen = baseline_schedule();
        s = resolve_schedule(chosen, AUTOSAGE_OP_SPMM, F, dt, 1, common_alignment(B, ldb, esize), common_alignment(C, ldc, 4), &r);
    }
    if (s != AUTOSAGE_OK) return s;
    SpmmArgs a{};
    a.rows = RowMap{0, 1, (int32_t)n_rows, 0};
    a.rowptr = rowptr;
    a.colind = colind;
    a.val = val;
    a.B = B;
    a.ldb = ldb;
    a.C = C;
    a.ldc = ldc;
    a.F = F;
    a.dt = dt;
    a.heads = 1;
    a.head_dim = F;
    return exec_spmm(h, a, r, nnz, workspace, workspace_bytes, st);
}

}  // namespace autosage

extern "C" autosage_status_t autosage_spmm(autosage_handle_t h, int64_t n_rows, int64_t n_cols, int64_t nnz,
                                           const int32_t* rowptr, const int32_t* colind, const float* val,
                                           const void* B, int64_t ldb, float* C, int64_t ldc, int32_t F,
                                           autosage_dtype_t dt, const autosage_schedule_t* sched,
                                           void* workspace, size_t workspace_bytes, void* stream)
{
    return spmm_entry(h, n_rows, n_cols, nnz, rowptr, colind, val, B, ldb, C, ldc, F, (int)dt, sched, workspace, workspace_bytes,
                      stream);
}

extern "C" autosage_status_t autosage_sddmm(autosage_handle_t h, int64_t n_rows, int64_t n_cols, int64_t nnz,
                                            const int32_t* rowptr, const int32_t* colind, const float* val,
                                            const void* X, int64_t ldx, const void* Y, int64_t ldy, int32_t F,
                                            autosage_dtype_t dt, float* out, const autosage_schedule_t* sched,
                                            void* workspace, size_t workspace_bytes, void* stream)
{
    (void)val;
    if (!h || !sizes_ok(n_rows, n_cols, nnz) || F <= 0 || ldx < F || ldy < F) return AUTOSAGE_ERR_INVALID_ARG;
    if (!dtype_known(dt)) return AUTOSAGE_ERR_INVALID_ARG;
    if (h->device < 0) return AUTOSAGE_ERR_UNSUPPORTED;
    if (n_rows == 0 || nnz == 0) return AUTOSAGE_OK;
    if (!rowptr || !colind || !X || !Y || !out) return AUTOSAGE_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    autosage_schedule_t chosen;
    if (!sched) {
        autosage_status_t s = autosage_decide(h, AUTOSAGE_OP_SDDMM, n_rows, n_cols, nnz, rowptr, colind, nullptr, X, ldx,
                                              Y, ldy, out, 1, F, dt, workspace, workspace_bytes, stream, &chosen);
        if (s != AUTOSAGE_OK) return s;
        sched = &chosen;
    }
    const int esize = dtype_bytes(dt);
    int al = common_alignment(X, ldx, esize);
    const int al2 = common_alignment(Y, ldy, esize);
    if (al2 < al) al = al2;
    Resolved r;
    autosage_status_t s = resolve_schedule(*sched, AUTOSAGE_OP_SDDMM, F, dt, 1, al, 16, &r);
    if (s == AUTOSAGE_ERR_UNSUPPORTED && sched == &chosen) {
        chosen = baseline_schedule();          // replayed decision made for other strides or alignments
        s = resolve_schedule(chosen, AUTOSAGE_OP_SDDMM, F, dt, 1, al, 16, &r);
    }
    if (s != AUTOSAGE_OK) return s;
    SddmmArgs a{};
    a.rows = RowMap{0, 1, (int32_t)n_rows, 0};
    a.rowptr = rowptr;
    a.colind = colind;
    a.X = X;
    a.ldx = ldx;
    a.Y = Y;
    a.ldy = ldy;
    a.out = out;
    a.F = F;
    a.dt = dt;
    a.heads = 1;
    a.scale = 1.0f;
    return exec_sddmm(h, a, r, nnz, workspace, workspace_bytes, st);
}

// Lanes per light row of the row-softmax kernels: the smallest power of two whose registers hold a row of
// the mean length (16 floats per lane with vector loads, 8 with scalar loads); longer rows of the launch
// are taken by whole wavefronts.
static int softmax_group(const autosage_ctx* h, int64_t count, int64_t nnz, int H)
{
    if (h->params.softmax_group != 0) return h->params.softmax_group;
    const int lane_floats = H >= 2 ? 16 : 8;
    const double want = (double)nnz / (double)(count > 0 ? count : 1) * H;
    int g = 1;
    while (g < 64 && g * lane_floats < want) g <<= 1;
    return g;
}

static autosage_status_t exec_softmax(autosage_ctx* h, const SoftmaxArgs& a, int64_t nnz, int hub_t, int hub_chunk, int wpg,
                                      const HubMeta* shared_meta, float* shared_part, void* ws, size_t ws_bytes,
                                      hipStream_t st)
{
    if (a.rows.count == 0 || nnz == 0) return AUTOSAGE_OK;
    HubMeta meta{};
    float* part = nullptr;
    if (hub_t > 0) {
        if (shared_meta) {
            meta = *shared_meta;
            part = shared_part;
        } else {
            if (!carve_hub(ws, ws_bytes, a.rows.count, nnz, hub_t, hub_chunk, 2 * (int64_t)a.H, &meta, &part, nullptr))
                return AUTOSAGE_ERR_WORKSPACE_TOO_SMALL;
            STAGE(h, "hub_partition", st, launch_hub_partition(a.rows, a.rowptr, hub_t, hub_chunk, meta, st));
        }
    }
    const int group = softmax_group(h, a.rows.count, nnz, a.H);
    STAGE(h, "softmax_rows", st, launch_softmax_rows(a, hub_t, wpg, group, st));
    if (hub_t > 0) STAGE(h, "softmax_hub", st, launch_softmax_hub(a, hub_chunk, group, meta, part, st));
    return AUTOSAGE_OK;
}

extern "C" autosage_status_t autosage_csr_row_softmax(autosage_handle_t h, int64_t n_rows, int64_t nnz,
                                                      const int32_t* rowptr, const float* in, float* out,
                                                      int32_t H, int32_t hub_t, int32_t hub_chunk,
                                                      void* workspace, size_t workspace_bytes, void* stream)
{
    if (!h || !sizes_ok(n_rows, 0, nnz) || H <= 0 || hub_t < 0 || hub_chunk < 0) return AUTOSAGE_ERR_INVALID_ARG;
    if ((int64_t)nnz * H >= (int64_t(1) << 40)) return AUTOSAGE_ERR_INVALID_ARG;
    if (hub_t > 0 && hub_t < kMinHubT) return AUTOSAGE_ERR_INVALID_ARG;
    if (!rowptr || (nnz > 0 && (!in || !out))) return AUTOSAGE_ERR_INVALID_ARG;
    if (h->device < 0) return AUTOSAGE_ERR_UNSUPPORTED;
    const int chunk = effective_hub_chunk(hub_t, hub_chunk);
    if (hub_t > 0 && (chunk < kMinHubT || chunk > kMaxHubChunk)) return AUTOSAGE_ERR_INVALID_ARG;
    SoftmaxArgs a{};
    a.rows = RowMap{0, 1, (int32_t)n_rows, 0};
    a.rowptr = rowptr;
    a.in = in;
    a.out = out;
    a.H = H;
    return exec_softmax(h, a, nnz, hub_t, chunk, 4, nullptr, nullptr, workspace, workspace_bytes,
                        static_cast<hipStream_t>(stream));
}

// Workspace of the attention pipeline: [scores nnz*H fp32][hub metadata + partial buffer].
static size_t attention_part_floats(int32_t H, int32_t d) { return (size_t)H * d > 2 * (size_t)H ? (size_t)H * d : 2 * (size_t)H; }

// Which attention pipeline a schedule asks for: 1 = single pass, 0 = three stages, -1 = cannot run.
static int attention_pipeline(const autosage_schedule_t& sched, int32_t H, int32_t d, int dt, AttnShape* shape)
{
    if (sched.mapping == AUTOSAGE_MAP_FUSED) {
        // f_tile = features per head tile (a multiple of d that divides H * d); 0 = all heads in one tile
        if (sched.f_tile < 0 || sched.f_tile % d != 0) return -1;
        return attn_fused_shape_tiled(H, d, dt, sched.f_tile / d, shape) ? 1 : -1;
    }
    if (sched.mapping == AUTOSAGE_MAP_WAVE_ROW || sched.mapping == AUTOSAGE_MAP_PLAIN) return 0;
    return -1;
}

namespace autosage {

autosage_status_t attention_alignment(const AttnCall& c)
{
    const int esize = dtype_bytes(c.dt);
    const int64_t HD = (int64_t)c.H * c.d;
    // 16-byte lane loads are required: d must be a multiple of 16 / esize elements and the operands aligned
    if ((c.d * esize) % 16 != 0) return AUTOSAGE_ERR_UNSUPPORTED;
    int al = common_alignment(c.Q, HD, esize);
    al = std::min(al, common_alignment(c.K, HD, esize));
    al = std::min(al, common_alignment(c.V, HD, esize));
    if (al < 16 || common_alignment(c.O, HD, 4) < 16) return AUTOSAGE_ERR_UNSUPPORTED;
    return AUTOSAGE_OK;
}

autosage_status_t exec_attention(autosage_ctx* h, const AttnCall& c, const autosage_schedule_t& sched, const RowMap& rows,
                                 void* workspace, size_t workspace_bytes, hipStream_t st)
{
    if (rows.count == 0) return AUTOSAGE_OK;
    const int32_t H = c.H, d = c.d;
    const int64_t HD = (int64_t)H * d;
    const int64_t nnz = c.nnz;
    autosage_schedule_t s = sched;
    AttnShape shape{};
    const int pipeline = attention_pipeline(sched, H, d, c.dt, &shape);
    if (pipeline < 0) return AUTOSAGE_ERR_UNSUPPORTED;
    s.mapping = AUTOSAGE_MAP_WAVE_ROW;
    s.f_tile = 0;
    s.vec_bytes = 16;
    s.group_lanes = 0;
    Resolved rs, rp;
    autosage_status_t rc = resolve_schedule(s, AUTOSAGE_OP_SDDMM, d, c.dt, H, 16, 16, &rs);
    if (rc != AUTOSAGE_OK) return rc;
    rc = resolve_schedule(s, AUTOSAGE_OP_SPMM, (int32_t)HD, c.dt, 1, 16, 16, &rp);
    if (rc != AUTOSAGE_OK) return rc;

    if (pipeline == 1) {
        // single pass with a running softmax: no score array, one hub partition, three kernels at most
        shape.wpg = rs.wpg;
        shape.hub_t = rs.hub_t;
        shape.hub_chunk = rs.hub_chunk;
        AttnArgs fa{};
        fa.rows = rows;
        fa.rowptr = c.rowptr;
        fa.colind = c.colind;
        fa.Q = c.Q;
        fa.K = c.K;
        fa.V = c.V;
        fa.O = c.O;
        fa.H = H;
        fa.d = d;
        fa.dt = c.dt;
        fa.scale = c.scale;
        HubMeta fmeta{};
        float* fpart = nullptr;
        if (shape.hub_t > 0) {
            if (!carve_hub(workspace, workspace_bytes, rows.count, nnz, shape.hub_t, shape.hub_chunk,
                           (int64_t)attn_fused_part_floats(shape), &fmeta, &fpart, nullptr))
                return AUTOSAGE_ERR_WORKSPACE_TOO_SMALL;
            STAGE(h, "hub_partition", st, launch_hub_partition(rows, c.rowptr, shape.hub_t, shape.hub_chunk, fmeta, st));
        }
        STAGE(h, "attn_fused_rows", st, launch_attn_fused_rows(fa, shape, st));
        if (shape.hub_t > 0) STAGE(h, "attn_fused_hub", st, launch_attn_fused_hub(fa, shape, fmeta, fpart, st));
        return AUTOSAGE_OK;
    }

    const size_t score_bytes = align_up(sizeof(float) * (size_t)nnz * H, 256);
    if (!workspace || (reinterpret_cast<uint64_t>(workspace) & 255u) != 0 || workspace_bytes < score_bytes)
        return AUTOSAGE_ERR_WORKSPACE_TOO_SMALL;
    float* S = static_cast<float*>(workspace);
    char* hub_ws = static_cast<char*>(workspace) + score_bytes;
    const size_t hub_ws_bytes = workspace_bytes - score_bytes;

    if (h->probe_skip_deg > 0) {                // lower bound of the three stages: light rows only, no hub kernels
        rs.hub_t = rp.hub_t = h->probe_skip_deg;
    }
    const bool light_only = h->probe_skip_deg > 0;
    HubMeta meta{};
    float* part = nullptr;
    if (rs.hub_t > 0 && !light_only) {
        if (!carve_hub(hub_ws, hub_ws_bytes, rows.count, nnz, rs.hub_t, rs.hub_chunk, (int64_t)attention_part_floats(H, d),
                       &meta, &part, nullptr))
            return AUTOSAGE_ERR_WORKSPACE_TOO_SMALL;
        STAGE(h, "hub_partition", st, launch_hub_partition(rows, c.rowptr, rs.hub_t, rs.hub_chunk, meta, st));
    }
    // stage 1: scores
    SddmmArgs sa{};
    sa.rows = rows;
    sa.rowptr = c.rowptr;
    sa.colind = c.colind;
    sa.X = c.Q;
    sa.ldx = HD;
    sa.Y = c.K;
    sa.ldy = HD;
    sa.out = S;
    sa.F = d;
    sa.dt = c.dt;
    sa.heads = H;
    sa.scale = c.scale;
    if (nnz > 0) {
        STAGE(h, "attn_sddmm_rows", st, launch_sddmm_rows(sa, rs, st));
        if (rs.hub_t > 0 && !light_only) STAGE(h, "attn_sddmm_hub", st, launch_sddmm_hub(sa, rs, meta, st));
    }
    // stage 2: row-softmax in place
    SoftmaxArgs ma{};
    ma.rows = rows;
    ma.rowptr = c.rowptr;
    ma.in = S;
    ma.out = S;
    ma.H = H;
    if (light_only) {
        STAGE(h, "softmax_rows", st, launch_softmax_rows(ma, rs.hub_t, rs.wpg, softmax_group(h, ma.rows.count, nnz, H), st));
    } else {
        rc = exec_softmax(h, ma, nnz, rs.hub_t, rs.hub_chunk, rs.wpg, rs.hub_t > 0 ? &meta : nullptr, part, nullptr, 0, st);
        if (rc != AUTOSAGE_OK) return rc;
    }
    // stage 3: weighted sum of V rows with per-head weights
    SpmmArgs pa{};
    pa.rows = rows;
    pa.rowptr = c.rowptr;
    pa.colind = c.colind;
    pa.val = S;
    pa.B = c.V;
    pa.ldb = HD;
    pa.C = c.O;
    pa.ldc = HD;
    pa.F = (int32_t)HD;
    pa.dt = c.dt;
    pa.heads = H > 1 ? H : 1;
    pa.head_dim = d;
    STAGE(h, "attn_spmm_rows", st, launch_spmm_rows(pa, rp, st));
    if (rp.hub_t > 0 && !light_only) STAGE(h, "attn_spmm_hub", st, launch_spmm_hub(pa, rp, meta, part, st));
    return AUTOSAGE_OK;
}

}  // namespace autosage

extern "C" autosage_status_t autosage_csr_attention(autosage_handle_t h, int64_t N, int64_t nnz,
                                                    const int32_t* rowptr, const int32_t* colind, const float* val,
                                                    const void* Q, const void* K, const void* V, float* O,
                                                    int32_t H, int32_t d, float scale, autosage_dtype_t in_dt,
                                                    const autosage_schedule_t* sched,
                                                    void* workspace, size_t workspace_bytes, void* stream)
{
    (void)val;
    if (!h || !sizes_ok(N, N, nnz) || H <= 0 || d <= 0 || (int64_t)H * d >= (1 << 24)) return AUTOSAGE_ERR_INVALID_ARG;
    if (!dtype_known(in_dt)) return AUTOSAGE_ERR_INVALID_ARG;
    if (h->device < 0) return AUTOSAGE_ERR_UNSUPPORTED;
    if (N == 0) return AUTOSAGE_OK;
    if (!rowptr || !O || (nnz > 0 && (!colind || !Q || !K || !V))) return AUTOSAGE_ERR_INVALID_ARG;
    AttnCall c{N, nnz, rowptr, colind, Q, K, V, O, H, d, scale, (int)in_dt};
    autosage_status_t rc = attention_alignment(c);
    if (rc != AUTOSAGE_OK) return rc;
    autosage_schedule_t chosen;
    if (!sched) {
        rc = autosage_decide_attention(h, N, nnz, rowptr, colind, Q, K, V, O, H, d, scale, in_dt, workspace,
                                       workspace_bytes, stream, &chosen);
        if (rc != AUTOSAGE_OK) return rc;
        sched = &chosen;
    }
    return exec_attention(h, c, *sched, RowMap{0, 1, (int32_t)N, 0}, workspace, workspace_bytes,
                          static_cast<hipStream_t>(stream));
}

extern "C" autosage_status_t autosage_workspace_bytes(autosage_handle_t h, autosage_op_t op, int64_t n_rows,
                                                      int64_t nnz, int32_t F, int32_t H,
                                                      const autosage_schedule_t* sched, size_t* bytes)
{
    if (!h || !bytes || !sizes_ok(n_rows, 0, nnz) || F <= 0 || H <= 0) return AUTOSAGE_ERR_INVALID_ARG;
    int hub_t = kSelectorMinHubT, chunk = kSelectorMinChunk;
    if (sched) {
        hub_t = sched->hub_t;
        chunk = effective_hub_chunk(sched->hub_t, sched->hub_chunk);
        if (hub_t < 0 || (hub_t > 0 && (hub_t < kMinHubT || chunk < kMinHubT || chunk > kMaxHubChunk)))
            return AUTOSAGE_ERR_INVALID_ARG;
    } else if (op == AUTOSAGE_OP_ATTENTION) {
        hub_t = chunk = 256;               // smallest threshold the attention selector proposes
    }
    size_t b = 0;
    switch (op) {
        case AUTOSAGE_OP_SPMM: b = hub_workspace_bytes(n_rows, nnz, hub_t, chunk, F); break;
        case AUTOSAGE_OP_SDDMM: b = hub_workspace_bytes(n_rows, nnz, hub_t, chunk, 0); break;
        case AUTOSAGE_OP_SOFTMAX: b = hub_workspace_bytes(n_rows, nnz, hub_t, chunk, 2 * (int64_t)H); break;
        case AUTOSAGE_OP_ATTENTION: {
            // dtype is not an argument here: take the largest per-chunk state over the element types
            // (and, without a schedule, over the head tilings the selector may choose)
            AttnShape sh{};
            size_t fused_floats = 0;
            for (int dt = DT_F32; dt <= DT_F16; ++dt) {
                for (int ht = 1; ht <= H; ++ht) {
                    if (H % ht != 0) continue;
                    if (sched && sched->f_tile > 0 && sched->f_tile != ht * F) continue;
                    if (sched && sched->f_tile <= 0 && ht != H) continue;
                    if (attn_fused_shape_tiled(H, F, dt, ht, &sh)) fused_floats = std::max(fused_floats, attn_fused_part_floats(sh));
                }
            }
            const size_t three = align_up(sizeof(float) * (size_t)nnz * H, 256) +
                                 hub_workspace_bytes(n_rows, nnz, hub_t, chunk, (int64_t)attention_part_floats(H, F));
            const size_t fused = hub_workspace_bytes(n_rows, nnz, hub_t, chunk, (int64_t)fused_floats);
            if (!sched) b = std::max(three, fused);
            else if (sched->mapping == AUTOSAGE_MAP_FUSED) b = fused;
            else b = three;
            break;
        }
        default: return AUTOSAGE_ERR_INVALID_ARG;
    }
    *bytes = b < 256 ? 256 : b;
    return AUTOSAGE_OK;
}

// ------------------------------------------------------------------------------------------
// attention backward: the chain rule through the three stages, all heads at once; the half on the pattern itself in
// one pass over K and V where the single-pass kernels cover the shape
// ------------------------------------------------------------------------------------------
namespace autosage {

// Workspace: P [nnz, H] | D [nnz, H] (dP, then dS) | per-row records [N, H, 3] of the single pass | hub partition
// + partial buffer (partitioned for A first, for A^T afterwards).  The transposed side reads P and dS through the
// permutation, so no copy in the order of A^T is kept.
// Floats of partial state per hub chunk: the stage-by-stage kernels and, over the element types (the type is not an
// argument of the size query), the single pass over K and V.
static size_t attention_bwd_part_floats(int32_t H, int32_t d)
{
    size_t f = attention_part_floats(H, d);
    AttnShape sh{};
    for (int dt = DT_F32; dt <= DT_F16; ++dt)
        if (attn_fused_shape(H, d, dt, &sh)) f = std::max(f, attn_bwd_part_floats(sh));
    return f;
}

static size_t attention_bwd_hub_bytes(int64_t N, int64_t nnz, int32_t H, int32_t d, int hub_t, int chunk)
{
    return hub_workspace_bytes(N, nnz, hub_t, chunk, (int64_t)attention_bwd_part_floats(H, d));
}

static size_t attention_bwd_stats_bytes(int64_t N, int32_t H) { return align_up(sizeof(float) * 3 * (size_t)(N > 0 ? N : 1) * H, 256); }

static size_t attention_bwd_bytes(int64_t N, int64_t nnz, int32_t H, int32_t d, int hub_t, int chunk)
{
    const size_t cells = align_up(sizeof(float) * (size_t)(nnz > 0 ? nnz : 1) * H, 256);
    return 2 * cells + attention_bwd_stats_bytes(N, H) + attention_bwd_hub_bytes(N, nnz, H, d, hub_t, chunk);
}

struct AttnBwdCall {
    int64_t N, nnz;
    const int32_t *rowptr, *colind, *t_rowptr, *t_colind, *perm;
    const void *Q, *K, *V;
    const float* dO;
    float *dQ, *dK, *dV;
    int32_t H, d;
    float scale;
    int dt;
};

static autosage_status_t exec_attention_backward(autosage_ctx* h, const AttnBwdCall& c, int hub_t, int chunk, void* workspace,
                                                 size_t workspace_bytes, hipStream_t st)
{
    const int32_t H = c.H, d = c.d;
    const int64_t HD = (int64_t)H * d, N = c.N, nnz = c.nnz;
    const RowMap rows{0, 1, (int32_t)N, 0};
    autosage_schedule_t s{};
    s.mapping = AUTOSAGE_MAP_WAVE_ROW;
    s.vec_bytes = 16;
    s.hub_t = hub_t;
    s.hub_chunk = chunk;
    Resolved rs, rp, rp32;
    autosage_status_t rc = resolve_schedule(s, AUTOSAGE_OP_SDDMM, d, c.dt, H, 16, 16, &rs);
    if (rc != AUTOSAGE_OK) return rc;
    rc = resolve_schedule(s, AUTOSAGE_OP_SPMM, (int32_t)HD, c.dt, 1, 16, 16, &rp);
    if (rc != AUTOSAGE_OK) return rc;
    rc = resolve_schedule(s, AUTOSAGE_OP_SPMM, (int32_t)HD, DT_F32, 1, 16, 16, &rp32);
    if (rc != AUTOSAGE_OK) return rc;

    const size_t need = attention_bwd_bytes(N, nnz, H, d, rs.hub_t, rs.hub_chunk);
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uint64_t>(workspace) & 255u) != 0)
        return AUTOSAGE_ERR_WORKSPACE_TOO_SMALL;
    const size_t cells = align_up(sizeof(float) * (size_t)(nnz > 0 ? nnz : 1) * H, 256);
    char* base = static_cast<char*>(workspace);
    float* P = reinterpret_cast<float*>(base);
    float* D = reinterpret_cast<float*>(base + cells);
    float* stats = reinterpret_cast<float*>(base + 2 * cells);
    const size_t head = 2 * cells + attention_bwd_stats_bytes(N, H);
    void* hub_ws = base + head;
    const size_t hub_ws_bytes = workspace_bytes - head;

    HubMeta meta{};
    float* part = nullptr;
    auto partition = [&](const int32_t* rowptr) -> autosage_status_t {
        if (rs.hub_t <= 0) return AUTOSAGE_OK;
        if (!carve_hub(hub_ws, hub_ws_bytes, N, nnz, rs.hub_t, rs.hub_chunk, (int64_t)attention_bwd_part_floats(H, d), &meta, &part,
                       nullptr))
            return AUTOSAGE_ERR_WORKSPACE_TOO_SMALL;
        STAGE(h, "hub_partition", st, launch_hub_partition(rows, rowptr, rs.hub_t, rs.hub_chunk, meta, st));
        return AUTOSAGE_OK;
    };
    auto sddmm = [&](const void* X, bool x_f32, const void* Y, float scale, float* out) -> autosage_status_t {
        SddmmArgs a{};
        a.rows = rows;
        a.rowptr = c.rowptr;
        a.colind = c.colind;
        a.X = X;
        a.ldx = HD;
        a.Y = Y;
        a.ldy = HD;
        a.out = out;
        a.F = d;
        a.dt = c.dt;
        a.heads = H;
        a.scale = scale;
        a.x_f32 = x_f32 ? 1 : 0;
        STAGE(h, "attn_bwd_sddmm_rows", st, launch_sddmm_rows(a, rs, st));
        if (rs.hub_t > 0) STAGE(h, "attn_bwd_sddmm_hub", st, launch_sddmm_hub(a, rs, meta, st));
        return AUTOSAGE_OK;
    };
    auto spmm = [&](const int32_t* rowptr, const int32_t* colind, const float* w, const int32_t* w_at, const void* B, int dt,
                    const Resolved& r, float* out) -> autosage_status_t {
        SpmmArgs a{};
        a.rows = rows;
        a.rowptr = rowptr;
        a.colind = colind;
        a.val = w;
        a.val_index = w_at;
        a.B = B;
        a.ldb = HD;
        a.C = out;
        a.ldc = HD;
        a.F = (int32_t)HD;
        a.dt = dt;
        a.heads = H > 1 ? H : 1;
        a.head_dim = d;
        STAGE(h, "attn_bwd_spmm_rows", st, launch_spmm_rows(a, r, st));
        if (r.hub_t > 0) STAGE(h, "attn_bwd_spmm_hub", st, launch_spmm_hub(a, r, meta, part, st));
        return AUTOSAGE_OK;
    };

    // forward pattern: P = softmax(scale * Q K^T), dP = <dO, V>, dS = scale * softmax'(P, dP), dQ = dS K
    rc = partition(c.rowptr);
    if (rc != AUTOSAGE_OK) return rc;
    AttnShape shape{};
    const bool one_pass = h->params.attention_backward_fused != 0 && attn_fused_shape(H, d, c.dt, &shape);
    if (one_pass) {
        // one walk over K and V per row: dQ, and P and dS left in the two [nnz, H] arrays
        shape.wpg = rs.wpg;
        shape.hub_t = rs.hub_t;
        shape.hub_chunk = rs.hub_chunk;
        shape.heads_tile = H;
        shape.tiles = 1;
        AttnBwdArgs fa{};
        fa.rows = rows;
        fa.rowptr = c.rowptr;
        fa.colind = c.colind;
        fa.Q = c.Q;
        fa.K = c.K;
        fa.V = c.V;
        fa.dO = c.dO;
        fa.dQ = c.dQ;
        fa.S = P;
        fa.D = D;
        fa.stats = stats;
        fa.H = H;
        fa.d = d;
        fa.dt = c.dt;
        fa.scale = c.scale;
        STAGE(h, "attn_bwd_rows", st, launch_attn_bwd_rows(fa, shape, st));
        if (rs.hub_t > 0) STAGE(h, "attn_bwd_hub", st, launch_attn_bwd_hub(fa, shape, meta, part, st));
        if (nnz > 0) STAGE(h, "attn_bwd_finish", st, launch_attn_bwd_finish(fa, shape, rs.hub_t > 0 ? &meta : nullptr, st));
    } else if (nnz > 0) {
        rc = sddmm(c.Q, false, c.K, c.scale, P);
        if (rc != AUTOSAGE_OK) return rc;
        SoftmaxArgs ma{};
        ma.rows = rows;
        ma.rowptr = c.rowptr;
        ma.in = P;
        ma.out = P;
        ma.H = H;
        rc = exec_softmax(h, ma, nnz, rs.hub_t, rs.hub_chunk, rs.wpg, rs.hub_t > 0 ? &meta : nullptr, part, nullptr, 0, st);
        if (rc != AUTOSAGE_OK) return rc;
        rc = sddmm(c.dO, true, c.V, 1.0f, D);
        if (rc != AUTOSAGE_OK) return rc;
        SoftmaxBwdArgs ba{};
        ba.rows = rows;
        ba.rowptr = c.rowptr;
        ba.P = P;
        ba.dP = D;
        ba.dS = D;
        ba.H = H;
        ba.scale = c.scale;
        STAGE(h, "attn_bwd_softmax", st, launch_softmax_bwd(ba, rs.hub_t, rs.hub_chunk, softmax_group(h, ba.rows.count, nnz, ba.H),
                                                                rs.hub_t > 0 ? &meta : nullptr, part, st));
    }
    if (!one_pass) {
        rc = spmm(c.rowptr, c.colind, D, nullptr, c.K, c.dt, rp, c.dQ);
        if (rc != AUTOSAGE_OK) return rc;
    }

    // transposed pattern: dV = P^T dO, dK = dS^T Q
    rc = partition(c.t_rowptr);
    if (rc != AUTOSAGE_OK) return rc;
    // the weights of an entry of the transposed pattern sit at its source position: read through the permutation
    rc = spmm(c.t_rowptr, c.t_colind, P, c.perm, c.dO, DT_F32, rp32, c.dV);
    if (rc != AUTOSAGE_OK) return rc;
    return spmm(c.t_rowptr, c.t_colind, D, c.perm, c.Q, c.dt, rp, c.dK);
}

}  // namespace autosage

extern "C" autosage_status_t autosage_csr_attention_backward_workspace_bytes(autosage_handle_t h, int64_t N, int64_t nnz,
                                                                             int32_t H, int32_t d, int32_t hub_t,
                                                                             int32_t hub_chunk, size_t* bytes)
{
    if (!h || !bytes || !sizes_ok(N, N, nnz) || H <= 0 || d <= 0 || hub_t < 0 || hub_chunk < 0) return AUTOSAGE_ERR_INVALID_ARG;
    const int chunk = effective_hub_chunk(hub_t, hub_chunk);
    if (hub_t > 0 && (hub_t < kMinHubT || chunk < kMinHubT || chunk > kMaxHubChunk)) return AUTOSAGE_ERR_INVALID_ARG;
    *bytes = attention_bwd_bytes(N, nnz, H, d, hub_t, chunk);
    return AUTOSAGE_OK;
}

extern "C" autosage_status_t autosage_csr_attention_backward(
    autosage_handle_t h, int64_t N, int64_t nnz, const int32_t* rowptr, const int32_t* colind, const int32_t* t_rowptr,
    const int32_t* t_colind, const int32_t* perm, const void* Q, const void* K, const void* V, const float* dO, float* dQ,
    float* dK, float* dV, int32_t H, int32_t d, float scale, autosage_dtype_t in_dt, int32_t hub_t, int32_t hub_chunk,
    void* workspace, size_t workspace_bytes, void* stream)
{
    if (!h || !sizes_ok(N, N, nnz) || H <= 0 || d <= 0 || (int64_t)H * d >= (1 << 24) || hub_t < 0 || hub_chunk < 0)
        return AUTOSAGE_ERR_INVALID_ARG;
    if (!dtype_known(in_dt)) return AUTOSAGE_ERR_INVALID_ARG;
    const int chunk = effective_hub_chunk(hub_t, hub_chunk);
    if (hub_t > 0 && (hub_t < kMinHubT || chunk < kMinHubT || chunk > kMaxHubChunk)) return AUTOSAGE_ERR_INVALID_ARG;
    if (h->device < 0) return AUTOSAGE_ERR_UNSUPPORTED;
    if (N == 0) return AUTOSAGE_OK;
    if (!rowptr || !t_rowptr || !dQ || !dK || !dV) return AUTOSAGE_ERR_INVALID_ARG;
    if (nnz > 0 && (!colind || !t_colind || !perm || !Q || !K || !V || !dO)) return AUTOSAGE_ERR_INVALID_ARG;
    // the forward's alignment rule for Q, K, V; the fp32 tensors are read and written in 16-byte pieces
    AttnCall fc{N, nnz, rowptr, colind, Q, K, V, dQ, H, d, scale, (int)in_dt};
    autosage_status_t rc = attention_alignment(fc);
    if (rc != AUTOSAGE_OK) return rc;
    const int64_t HD = (int64_t)H * d;
    if (d % 4 != 0 || common_alignment(dO, HD, 4) < 16 || common_alignment(dK, HD, 4) < 16 || common_alignment(dV, HD, 4) < 16)
        return AUTOSAGE_ERR_UNSUPPORTED;
    AttnBwdCall c{N, nnz, rowptr, colind, t_rowptr, t_colind, perm, Q, K, V, dO, dQ, dK, dV, H, d, scale, (int)in_dt};
    return exec_attention_backward(h, c, hub_t, chunk, workspace, workspace_bytes, static_cast<hipStream_t>(stream));
}

// ------------------------------------------------------------------------------------------
// plan / metadata
// ------------------------------------------------------------------------------------------
extern "C" autosage_status_t autosage_hub_partition(autosage_handle_t h, int64_t n_rows, const int32_t* rowptr,
                                                    int32_t hub_t, int32_t hub_chunk,
                                                    int32_t* n_hub, int32_t* hub_rows, int32_t* chunk_ptr,
                                                    int32_t* n_light, int32_t* light_rows,
                                                    void* workspace, size_t workspace_bytes, void* stream)
{
    if (!h || !sizes_ok(n_rows, 0, 0) || !rowptr || hub_t < 1 || hub_chunk < 1 || !n_hub || !hub_rows || !chunk_ptr || !n_light)
        return AUTOSAGE_ERR_INVALID_ARG;
    if (h->device < 0) return AUTOSAGE_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t part_blocks = (n_rows + 1023) / 1024;
    const size_t need = 256 + align_up(sizeof(int32_t) * 2 * (size_t)(part_blocks > 0 ? part_blocks : 1), 256);
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uint64_t>(workspace) & 255u) != 0)
        return AUTOSAGE_ERR_WORKSPACE_TOO_SMALL;
    HubMeta meta{};
    meta.counts = static_cast<HubCounts*>(workspace);
    meta.block_counts = reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + 256);
    meta.hub_rows = hub_rows;
    meta.chunk_ptr = chunk_ptr;
    meta.light_rows = light_rows;
    meta.cap_hub = (int32_t)n_rows;
    meta.cap_chunks = 0;
    HIP_TRY(launch_hub_partition(RowMap{0, 1, (int32_t)n_rows, 0}, rowptr, hub_t, hub_chunk, meta, st));
    HubCounts c{};
    HIP_TRY(hipMemcpyAsync(&c, meta.counts, sizeof c, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    *n_hub = c.n_hub;
    *n_light = c.n_light;
    return AUTOSAGE_OK;
}

extern "C" autosage_status_t autosage_graph_features(autosage_handle_t h, int64_t n_rows, int64_t n_cols,
                                                     const int32_t* rowptr, int64_t* hist33, int64_t* max_deg,
                                                     int64_t* nnz, uint64_t* signature, void* stream)
{
    if (!h || !sizes_ok(n_rows, n_cols, 0) || !rowptr) return AUTOSAGE_ERR_INVALID_ARG;
    if (h->device < 0) return AUTOSAGE_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    HIP_TRY(launch_graph_features(n_rows, rowptr, h->dev_features, st));
    HIP_TRY(hipMemcpyAsync(h->host_features, h->dev_features, sizeof(int64_t) * (35 + 1024), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    const int64_t* f = h->host_features;
    if (hist33) std::memcpy(hist33, f, sizeof(int64_t) * 33);
    if (max_deg) *max_deg = f[33];
    if (nnz) *nnz = f[34];
    if (signature) *signature = signature_from_features(n_rows, n_cols, f);
    return AUTOSAGE_OK;
}

extern "C" autosage_status_t autosage_validate_csr(autosage_handle_t h, int64_t n_rows, int64_t n_cols, int64_t nnz,
                                                   const int32_t* rowptr, const int32_t* colind, void* stream)
{
    if (!h || !sizes_ok(n_rows, n_cols, nnz) || !rowptr || (nnz > 0 && !colind)) return AUTOSAGE_ERR_INVALID_ARG;
    if (h->device < 0) return AUTOSAGE_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    HIP_TRY(launch_validate_csr(n_rows, n_cols, nnz, rowptr, colind, h->dev_flag, st));
    int32_t flag = 0;
    HIP_TRY(hipMemcpyAsync(&flag, h->dev_flag, sizeof flag, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    return flag ? AUTOSAGE_ERR_INVALID_ARG : AUTOSAGE_OK;
}

extern "C" autosage_status_t autosage_narrow_indices(autosage_handle_t h, int64_t n, const int64_t* src, int32_t* dst,
                                                     int64_t limit, void* stream)
{
    if (!h || n < 0 || limit < 0 || limit > INT32_MAX || (n > 0 && (!src || !dst))) return AUTOSAGE_ERR_INVALID_ARG;
    if (h->device < 0) return AUTOSAGE_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    HIP_TRY(launch_narrow_indices(n, src, dst, limit, h->dev_flag, st));
    int32_t flag = 0;
    HIP_TRY(hipMemcpyAsync(&flag, h->dev_flag, sizeof flag, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    return flag ? AUTOSAGE_ERR_UNSUPPORTED : AUTOSAGE_OK;
}

// ------------------------------------------------------------------------------------------
// bandwidth probe
// ------------------------------------------------------------------------------------------
extern "C" autosage_status_t autosage_stream_probe_dst_bytes(autosage_handle_t h, size_t* bytes)
{
    if (!h || !bytes) return AUTOSAGE_ERR_INVALID_ARG;
    *bytes = sizeof(float) * (size_t)stream_probe_blocks(h->cu_count);
    return AUTOSAGE_OK;
}

extern "C" autosage_status_t autosage_stream_probe(autosage_handle_t h, autosage_stream_mode_t mode, const void* src,
                                                   void* dst, size_t n_bytes, void* stream)
{
    if (!h) return AUTOSAGE_ERR_INVALID_ARG;
    if (mode != AUTOSAGE_STREAM_READ && mode != AUTOSAGE_STREAM_COPY && mode != AUTOSAGE_STREAM_INPLACE)
        return AUTOSAGE_ERR_INVALID_ARG;
    // zero bytes: nothing to read; the read mode still writes its (zero) partial sums
    if ((!dst && (n_bytes > 0 || mode == AUTOSAGE_STREAM_READ)) || (mode != AUTOSAGE_STREAM_INPLACE && !src && n_bytes > 0))
        return AUTOSAGE_ERR_INVALID_ARG;
    if (n_bytes % 16 != 0 || n_bytes > (size_t(1) << 40)) return AUTOSAGE_ERR_INVALID_ARG;
    if (((reinterpret_cast<uint64_t>(src) | reinterpret_cast<uint64_t>(dst)) & 15u) != 0) return AUTOSAGE_ERR_INVALID_ARG;
    if (h->device < 0) return AUTOSAGE_ERR_UNSUPPORTED;
    if (n_bytes == 0 && mode != AUTOSAGE_STREAM_READ) return AUTOSAGE_OK;
    HIP_TRY(launch_stream_probe((int)mode, stream_probe_blocks(h->cu_count), src, dst, (int64_t)(n_bytes / 16),
                                static_cast<hipStream_t>(stream)));
    return AUTOSAGE_OK;
}

extern "C" autosage_status_t autosage_gather_probe(autosage_handle_t h, const void* table, int64_t n_table_rows,
                                                   int32_t row_bytes, const int32_t* idx, int64_t n_idx, float* dst,
                                                   void* stream)
{
    if (!h || n_table_rows < 0 || n_table_rows >= (int64_t(1) << 31) || n_idx < 0 || n_idx > (int64_t(1) << 40))
        return AUTOSAGE_ERR_INVALID_ARG;
    if (row_bytes < 16 || row_bytes > 1024 || (row_bytes & (row_bytes - 1)) != 0) return AUTOSAGE_ERR_INVALID_ARG;
    if (!dst || (n_idx > 0 && (!table || !idx || n_table_rows == 0))) return AUTOSAGE_ERR_INVALID_ARG;
    if ((reinterpret_cast<uint64_t>(table) & 15u) != 0) return AUTOSAGE_ERR_INVALID_ARG;
    if (h->device < 0) return AUTOSAGE_ERR_UNSUPPORTED;
    HIP_TRY(launch_gather_probe(stream_probe_blocks(h->cu_count), table, (int32_t)n_table_rows, row_bytes, idx, n_idx, dst,
                                static_cast<hipStream_t>(stream)));
    return AUTOSAGE_OK;
}

// ------------------------------------------------------------------------------------------
// telemetry
// ------------------------------------------------------------------------------------------
extern "C" autosage_status_t autosage_profile_begin(autosage_handle_t h)
{
    if (!h) return AUTOSAGE_ERR_INVALID_ARG;
    if (h->device < 0) return AUTOSAGE_ERR_UNSUPPORTED;
    h->profiling = true;
    h->spans_used = 0;
    return AUTOSAGE_OK;
}

extern "C" autosage_status_t autosage_profile_read(autosage_handle_t h, char* json_buf, size_t n)
{
    if (!h || !json_buf || n == 0) return AUTOSAGE_ERR_INVALID_ARG;
    if (h->device < 0) return AUTOSAGE_ERR_UNSUPPORTED;
    h->profiling = false;
    std::map<std::string, std::pair<int, double>> agg;
    for (size_t i = 0; i < h->spans_used; ++i) {
        autosage_ctx::StageSpan& s = h->spans[i];
        HIP_TRY(hipEventSynchronize(s.stop));
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, s.start, s.stop));
        auto& e = agg[s.stage];
        e.first += 1;
        e.second += ms;
    }
    h->spans_used = 0;
    std::string js = "{";
    bool first = true;
    for (const auto& kv : agg) {
        char buf[256];
        std::snprintf(buf, sizeof buf, "%s\"%s\":{\"calls\":%d,\"total_ms\":%.6f}", first ? "" : ",", kv.first.c_str(),
                      kv.second.first, kv.second.second);
        js += buf;
        first = false;
    }
    js += "}";
    const size_t m = js.size() < n - 1 ? js.size() : n - 1;
    std::memcpy(json_buf, js.data(), m);
    json_buf[m] = '\0';
    return AUTOSAGE_OK;
}

// ------------------------------------------------------------------------------------------
// adjoint helpers (training steps): row-softmax backward, CSR transpose, value gather
// ------------------------------------------------------------------------------------------
extern "C" autosage_status_t autosage_csr_row_softmax_backward(autosage_handle_t h, int64_t n_rows, int64_t nnz,
                                                               const int32_t* rowptr, const float* P, const float* dP,
                                                               float* dS, int32_t H, int32_t hub_t, int32_t hub_chunk,
                                                               void* workspace, size_t workspace_bytes, void* stream)
{
    if (!h || !sizes_ok(n_rows, 0, nnz) || H <= 0 || hub_t < 0 || hub_chunk < 0) return AUTOSAGE_ERR_INVALID_ARG;
    if (hub_t > 0 && hub_t < kMinHubT) return AUTOSAGE_ERR_INVALID_ARG;
    if (h->device < 0) return AUTOSAGE_ERR_UNSUPPORTED;
    if (n_rows == 0 || nnz == 0) return AUTOSAGE_OK;
    if (!rowptr || !P || !dP || !dS) return AUTOSAGE_ERR_INVALID_ARG;
    const int chunk = effective_hub_chunk(hub_t, hub_chunk);
    if (hub_t > 0 && (chunk < kMinHubT || chunk > kMaxHubChunk)) return AUTOSAGE_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    SoftmaxBwdArgs a{};
    a.rows = RowMap{0, 1, (int32_t)n_rows, 0};
    a.rowptr = rowptr;
    a.P = P;
    a.dP = dP;
    a.dS = dS;
    a.H = H;
    HubMeta meta{};
    float* part = nullptr;
    if (hub_t > 0) {
        if (!carve_hub(workspace, workspace_bytes, n_rows, nnz, hub_t, chunk, H, &meta, &part, nullptr))
            return AUTOSAGE_ERR_WORKSPACE_TOO_SMALL;
        STAGE(h, "hub_partition", st, launch_hub_partition(a.rows, rowptr, hub_t, chunk, meta, st));
    }
    STAGE(h, "softmax_bwd", st, launch_softmax_bwd(a, hub_t, chunk, softmax_group(h, a.rows.count, nnz, a.H),
                                                           hub_t > 0 ? &meta : nullptr, part, st));
    return AUTOSAGE_OK;
}

static size_t transpose_workspace(int64_t nnz, int64_t n_cols, size_t* temp_bytes)
{
    const size_t ints = align_up(sizeof(int32_t) * (size_t)(nnz > 0 ? nnz : 1), 256);
    const size_t temp = align_up(transpose_sort_temp_bytes(nnz > 0 ? nnz : 1, n_cols), 256);
    if (temp_bytes) *temp_bytes = temp;
    return 3 * ints + temp;                 // two key buffers, permutation (when the caller keeps none), sort scratch
}

extern "C" autosage_status_t autosage_csr_transpose_workspace_bytes(autosage_handle_t h, int64_t n_rows, int64_t n_cols,
                                                                    int64_t nnz, size_t* bytes)
{
    if (!h || !bytes || !sizes_ok(n_rows, n_cols, nnz)) return AUTOSAGE_ERR_INVALID_ARG;
    if (h->device < 0) return AUTOSAGE_ERR_UNSUPPORTED;
    *bytes = transpose_workspace(nnz, n_cols, nullptr);
    return AUTOSAGE_OK;
}

extern "C" autosage_status_t autosage_csr_transpose(autosage_handle_t h, int64_t n_rows, int64_t n_cols, int64_t nnz,
                                                    const int32_t* rowptr, const int32_t* colind, const float* val,
                                                    int32_t* t_rowptr, int32_t* t_colind, float* t_val, int32_t* perm,
                                                    void* workspace, size_t workspace_bytes, void* stream)
{
    if (!h || !sizes_ok(n_rows, n_cols, nnz) || !rowptr || !t_rowptr) return AUTOSAGE_ERR_INVALID_ARG;
    if (nnz > 0 && (!colind || !t_colind)) return AUTOSAGE_ERR_INVALID_ARG;
    if (nnz > 0 && (val == nullptr) != (t_val == nullptr)) return AUTOSAGE_ERR_INVALID_ARG;
    if (h->device < 0) return AUTOSAGE_ERR_UNSUPPORTED;
    size_t temp_bytes = 0;
    const size_t need = transpose_workspace(nnz, n_cols, &temp_bytes);
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uint64_t>(workspace) & 255u) != 0)
        return AUTOSAGE_ERR_WORKSPACE_TOO_SMALL;
    const size_t ints = align_up(sizeof(int32_t) * (size_t)(nnz > 0 ? nnz : 1), 256);
    char* p = static_cast<char*>(workspace);
    int32_t* keys_a = reinterpret_cast<int32_t*>(p);
    int32_t* keys_b = reinterpret_cast<int32_t*>(p + ints);
    int32_t* perm_buf = perm ? perm : reinterpret_cast<int32_t*>(p + 2 * ints);
    void* temp = p + 3 * ints;
    hipStream_t st = static_cast<hipStream_t>(stream);
    STAGE(h, "csr_transpose", st,
          launch_csr_transpose(n_rows, n_cols, nnz, rowptr, colind, val, t_rowptr, t_colind, t_val, perm_buf, keys_a, keys_b,
                               temp, temp_bytes, st));
    return AUTOSAGE_OK;
}

extern "C" autosage_status_t autosage_gather_values(autosage_handle_t h, int64_t n, int32_t width, const int32_t* perm,
                                                    const float* in, float* out, void* stream)
{
    if (!h || n < 0 || width <= 0 || n >= (int64_t(1) << 31)) return AUTOSAGE_ERR_INVALID_ARG;
    if (h->device < 0) return AUTOSAGE_ERR_UNSUPPORTED;
    if (n == 0) return AUTOSAGE_OK;
    if (!perm || !in || !out || in == out) return AUTOSAGE_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    STAGE(h, "gather_values", st, launch_gather_rows(perm, n, width, in, out, st));
    return AUTOSAGE_OK;
}

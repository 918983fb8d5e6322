// Input-aware schedule selection (paper, Scheduler subsection, decision sketch, Proposition 1):
// degree-histogram estimate -> timed probes on a strided row sample of the real operands ->
// guardrail against the plain one-wavefront-per-row kernel -> persistent cache keyed by
// (device signature, graph signature, F, op, dtype).  The cost model is this library's own,
// written for MI355X; it only ranks candidates, the probes decide.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <fstream>
#include <limits>
#include <sstream>

#include "internal.h"

using namespace autosage;

namespace autosage {

int decide_from_times(int n, const double* t, double tb, double alpha)
{
    int best = -1;
    double tstar = std::numeric_limits<double>::infinity();
    for (int c = 0; c < n; ++c) {
        if (t[c] < tstar) {      // strict: the first of equal candidates is kept
            best = c;
            tstar = t[c];
        }
    }
    return tstar <= alpha * tb ? best : -1;
}

static uint64_t fnv1a_i64(uint64_t h, int64_t v)
{
    uint64_t u = static_cast<uint64_t>(v);
    for (int b = 0; b < 8; ++b) {
        h ^= (u >> (8 * b)) & 0xFFu;
        h *= 0x100000001B3ULL;
    }
    return h;
}

uint64_t signature_from_features(int64_t n_rows, int64_t n_cols, const int64_t* f)
{
    uint64_t h = 0xCBF29CE484222325ULL;
    h = fnv1a_i64(h, n_rows);
    h = fnv1a_i64(h, n_cols);
    h = fnv1a_i64(h, f[34]);                       // nnz
    h = fnv1a_i64(h, f[33]);                       // max degree
    for (int b = 0; b < 33; ++b) h = fnv1a_i64(h, f[b]);
    for (int k = 0; k < 1024; ++k) h = fnv1a_i64(h, f[35 + k]);
    return h;
}

std::string schedule_json(const autosage_schedule_t& s)
{
    char buf[256];
    std::snprintf(buf, sizeof buf,
                  "{\"mapping\":%d,\"f_tile\":%d,\"waves_per_wg\":%d,\"vec_bytes\":%d,\"unroll\":%d,\"hub_t\":%d,"
                  "\"hub_chunk\":%d,\"xcd_remap\":%d,\"group_lanes\":%d}",
                  s.mapping, s.f_tile, s.waves_per_wg, s.vec_bytes, s.unroll, s.hub_t, s.hub_chunk, s.xcd_remap, s.group_lanes);
    return buf;
}

// ---- estimate ------------------------------------------------------------------------------
namespace {

struct Model {
    double bw_stream = 5.0e12;     // B/s, contiguous reads and writes
    double bw_gather = 3.5e12;     // B/s of useful bytes when whole 128-byte lines are used
    double t_fixed = 2.0e-6;       // s per row visit: rowptr, first index block, store
    double t_step = 0.8e-6;        // s per dependent gather step of a group
    double t_block = 0.6e-6;       // s per 64-nonzero index block
    double t_launch = 6.0e-6;      // s per extra kernel launch
    int waves = 8192;              // resident wavefronts (256 CUs x 4 SIMDs x 8)
};

// Chunk length for the rows at or above hub_t: `factor` thresholds per chunk where the histogram
// promises enough chunks to occupy the chip (about eight workgroups per compute unit), halved down to
// kSelectorMinChunk nonzeros where the hub rows are few.
int pick_hub_chunk(const int64_t* hist, int64_t max_deg, int hub_t, int factor, int cu_count)
{
    if (hub_t <= 0) return 0;
    double hub_nnz = 0.0;
    for (int b = 1; b < 33; ++b) {
        const double lo = std::ldexp(1.0, b - 1);
        if (lo >= hub_t) hub_nnz += std::min<double>(1.5 * lo, (double)max_deg) * (double)hist[b];
    }
    const double want = 8.0 * (cu_count > 0 ? cu_count : 256);
    int chunk = factor * hub_t;
    while (chunk > kSelectorMinChunk && hub_nnz / chunk < want) chunk >>= 1;
    return std::max(chunk, kSelectorMinChunk);
}

double estimate_one(const Model& m, int op, int64_t n_rows, int64_t nnz, const int64_t* hist, int64_t max_deg, int32_t F,
                    int esize, const Resolved& r)
{
    const double row_bytes = static_cast<double>(F) * esize;
    const double tile_bytes = std::min<double>(row_bytes, static_cast<double>(r.f_tile) * esize);
    const double lines = std::ceil(tile_bytes / 128.0) * 128.0;
    const double eff = tile_bytes / lines;
    const double vec_pen = r.mapping == MAP_PLAIN ? 0.6 : (r.vec * esize >= 16 ? 1.0 : (r.vec * esize >= 8 ? 0.9 : 0.75));
    double t_bw = nnz * row_bytes / (m.bw_gather * eff * vec_pen);
    if (op == AUTOSAGE_OP_SPMM) t_bw += (8.0 * nnz * r.tiles + 4.0 * n_rows + 4.0 * n_rows * F) / m.bw_stream;
    else t_bw += (8.0 * nnz + 4.0 * n_rows + row_bytes * n_rows) / m.bw_stream;

    const int G = r.G * r.HW;
    const int S = 64 / G;
    const int U = r.unroll;
    double wave_time = 0.0;          // summed over all wavefront visits
    double longest = 0.0;
    int64_t hub_nnz = 0, hub_rows = 0;
    for (int b = 0; b < 33; ++b) {
        if (hist[b] == 0) continue;
        const double lo = b == 0 ? 0.0 : std::ldexp(1.0, b - 1);
        double deg = b == 0 ? 0.0 : std::min<double>(1.5 * lo, static_cast<double>(max_deg));
        if (r.hub_t > 0 && lo >= r.hub_t) {
            hub_nnz += static_cast<int64_t>(deg * hist[b]);
            hub_rows += hist[b];
            continue;
        }
        double steps, blocks;
        if (r.mapping == MAP_MULTI_ROW) {
            steps = std::ceil(deg / U);
            blocks = 0.0;
        } else if (r.mapping == MAP_PLAIN) {
            steps = deg * 0.5;           // one nonzero at a time, partly overlapped by the hardware
            blocks = 0.0;
        } else {
            steps = std::ceil(deg / (S * U));
            blocks = std::ceil(deg / 64.0);
        }
        const double t_row = m.t_fixed + steps * m.t_step + blocks * m.t_block;
        const double visits = r.mapping == MAP_MULTI_ROW ? static_cast<double>(hist[b]) / S * (1.0 + 0.25 * std::log2((double)S))
                                                         : static_cast<double>(hist[b]);
        wave_time += visits * t_row * r.tiles;
        longest = std::max(longest, t_row);
    }
    double t_lat = wave_time / m.waves;
    double t = std::max(std::max(t_bw, t_lat), longest);
    if (r.hub_t > 0) {
        const double chunks = static_cast<double>(hub_nnz) / r.hub_chunk + hub_rows;
        t += 3 * m.t_launch + (op == AUTOSAGE_OP_SPMM ? 2.0 * chunks * F * 4.0 / m.bw_stream + m.t_launch : 0.0);
        const double chunk_steps = std::ceil(static_cast<double>(r.hub_chunk) / (r.wpg * S * U));
        t = std::max(t, m.t_fixed + chunk_steps * m.t_step);
    }
    return t;
}

}  // namespace

void shortlist(const autosage_ctx* h, int op, int64_t n_rows, int64_t n_cols, int64_t nnz, const int64_t* hist33,
               int64_t max_deg, int32_t F, int dt, int align_bytes, std::vector<autosage_schedule_t>* out,
               std::vector<double>* est)
{
    Model m;
    if (h && h->cu_count > 0) m.waves = h->cu_count * 32;
    const int esize = dtype_bytes(dt);
    const Params dflt;
    const Params& p = h ? h->params : dflt;
    std::vector<std::pair<double, autosage_schedule_t>> all;
    const int hubs[] = {0, 512, 1024, 2048, 4096};
    const int unrolls[] = {4, 8, 2};
    // Narrow feature tiles (SpMM, one wavefront per row): the launch walks the tiles one after the other, so a
    // dense operand too large for the caches is worked through in slices of n_cols * tile bytes that fit them,
    // at the price of reading the indices once per tile.  The histogram knows nothing of locality, so these
    // are ranked by the same estimate and the caller probes the best of each tile width.  SDDMM runs a narrow
    // tile as one launch per tile that adds into the output; that pays only together with narrow lane groups
    // (the cross-lane reduction is paid once per tile), so its 256-byte tile is proposed with them.
    std::vector<int> ftiles{0};
    if (p.force_ftile <= 0 && (int64_t)F * esize >= 512 && (double)n_cols * F * esize >= kTileOperandBytes) {
        ftiles.push_back(256 / esize);
        if (op == AUTOSAGE_OP_SPMM) ftiles.push_back(512 / esize);
    }
    // SDDMM lane groups: one vector per lane (0), or a dense row shared by 8 lanes that hold several vectors each
    // (three cross-lane steps per dot product instead of up to six)
    std::vector<int> lane_opts{0};
    if (op == AUTOSAGE_OP_SDDMM) lane_opts.push_back(8);
    for (int mapping = AUTOSAGE_MAP_WAVE_ROW; mapping <= AUTOSAGE_MAP_MULTI_ROW; ++mapping) {
        for (int vb = 16; vb >= esize; vb >>= 1) {
          for (int ft : ftiles) {
            if (ft > 0 && (mapping != AUTOSAGE_MAP_WAVE_ROW || ft >= F || vb < 8)) continue;
           for (int gl : lane_opts) {
            if (gl > 0 && (mapping != AUTOSAGE_MAP_WAVE_ROW || vb != 16)) continue;
            if (op == AUTOSAGE_OP_SDDMM && ft > 0 && gl == 0) continue;
            for (int u : unrolls) {
                for (int hub : hubs) {
                    if (hub > 0 && max_deg < hub) continue;
                    if (p.force_hub_t >= 0 && hub != hubs[0]) continue;   // forced value handled below
                    for (int xcd = 0; xcd <= 1; ++xcd) {
                        autosage_schedule_t s{};
                        s.mapping = mapping;
                        s.f_tile = p.force_ftile > 0 ? p.force_ftile : ft;
                        s.waves_per_wg = p.force_wpb > 0 ? p.force_wpb : 4;
                        s.vec_bytes = vb;
                        s.unroll = u;
                        s.hub_t = p.force_hub_t >= 0 ? p.force_hub_t : hub;
                        // four thresholds per chunk amortise what a chunk costs before its first gather (the search for
                        // its row, the row's own operand; for SpMM also a reduction and a partial row); fewer where
                        // the hub rows are too few to occupy the chip with chunks that long
                        s.hub_chunk = pick_hub_chunk(hist33, max_deg, s.hub_t, 4, h ? h->cu_count : 0);
                        s.xcd_remap = xcd;
                        s.group_lanes = gl;
                        Resolved r;
                        if (resolve_schedule(s, op, F, dt, 1, align_bytes, align_bytes, &r) != AUTOSAGE_OK) continue;
                        if (r.unroll != u) continue;
                        if (gl > 0 && r.G != gl) continue;        // the tile is no wider than the group: same kernel as gl = 0
                        double t = estimate_one(m, op, n_rows, nnz, hist33, max_deg, F, esize, r);
                        if (xcd) t *= 1.001;      // no locality information in the histogram: keep it next to its twin
                        // schedules that resolve to the same kernel shape under a smaller unroll are duplicates
                        if ((r.K == 2 && u == 8) || (r.K > 2 && r.K <= 4 && u > 2) || (r.K > 4 && u > 2)) continue;
                        all.emplace_back(t, s);
                    }
                }
            }
           }
          }
        }
    }
    std::stable_sort(all.begin(), all.end(), [](const auto& a, const auto& b) { return a.first < b.first; });
    out->clear();
    est->clear();
    for (const auto& e : all) {
        out->push_back(e.second);
        est->push_back(e.first);
    }
}

}  // namespace autosage

// ------------------------------------------------------------------------------------------
// C ABI: host-only pieces
// ------------------------------------------------------------------------------------------
extern "C" autosage_status_t autosage_decide_from_times(int32_t n_cand, const double* t_cand, double t_baseline,
                                                        double alpha, int32_t* choice)
{
    if (n_cand < 0 || (n_cand > 0 && !t_cand) || !choice) return AUTOSAGE_ERR_INVALID_ARG;
    *choice = decide_from_times(n_cand, t_cand, t_baseline, alpha);
    return AUTOSAGE_OK;
}

extern "C" autosage_status_t autosage_shortlist(autosage_handle_t h, autosage_op_t op, int64_t n_rows, int64_t n_cols,
                                                int64_t nnz, const int64_t* hist33, int64_t max_deg, int32_t F,
                                                autosage_dtype_t dt, int32_t align_bytes, autosage_schedule_t* out,
                                                double* est_seconds, int32_t max_out, int32_t* n_out)
{
    if (!h || !hist33 || !n_out || max_out < 0 || (max_out > 0 && !out) || F <= 0 || n_rows < 0 || nnz < 0)
        return AUTOSAGE_ERR_INVALID_ARG;
    if ((op != AUTOSAGE_OP_SPMM && op != AUTOSAGE_OP_SDDMM) || !dtype_known(dt)) return AUTOSAGE_ERR_INVALID_ARG;
    if (align_bytes < 1 || (align_bytes & (align_bytes - 1)) != 0) return AUTOSAGE_ERR_INVALID_ARG;
    std::vector<autosage_schedule_t> c;
    std::vector<double> e;
    shortlist(h, op, n_rows, n_cols, nnz, hist33, max_deg, F, dt, align_bytes > 16 ? 16 : align_bytes, &c, &e);
    const int n = std::min<int>(max_out, (int)c.size());
    for (int i = 0; i < n; ++i) {
        out[i] = c[i];
        if (est_seconds) est_seconds[i] = e[i];
    }
    *n_out = n;
    return AUTOSAGE_OK;
}

// ---- cache ---------------------------------------------------------------------------------
extern "C" autosage_status_t autosage_cache_clear(autosage_handle_t h)
{
    if (!h) return AUTOSAGE_ERR_INVALID_ARG;
    h->cache.clear();
    h->memo.clear();
    return AUTOSAGE_OK;
}

extern "C" autosage_status_t autosage_forget_graph(autosage_handle_t h, const int32_t* rowptr)
{
    if (!h) return AUTOSAGE_ERR_INVALID_ARG;
    for (size_t i = h->memo.size(); i-- > 0;)
        if (h->memo[i].rowptr == rowptr) h->memo.erase(h->memo.begin() + (long)i);
    return AUTOSAGE_OK;
}

extern "C" autosage_status_t autosage_cache_lookup(autosage_handle_t h, uint64_t graph_sig, int32_t F, int32_t H,
                                                   autosage_op_t op, autosage_dtype_t dt, autosage_schedule_t* sched,
                                                   int32_t* found)
{
    if (!h || !found) return AUTOSAGE_ERR_INVALID_ARG;
    auto it = h->cache.find(CacheKey{graph_sig, F, H, (int32_t)op, (int32_t)dt});
    *found = it != h->cache.end();
    if (*found && sched) *sched = it->second.sched;
    return AUTOSAGE_OK;
}

extern "C" autosage_status_t autosage_cache_insert(autosage_handle_t h, uint64_t graph_sig, int32_t F, int32_t H,
                                                   autosage_op_t op, autosage_dtype_t dt, const autosage_schedule_t* sched)
{
    if (!h || !sched || F <= 0 || H <= 0) return AUTOSAGE_ERR_INVALID_ARG;
    h->cache[CacheKey{graph_sig, F, H, (int32_t)op, (int32_t)dt}] = CacheEntry{*sched, 0.0, 0.0};
    return AUTOSAGE_OK;
}

// One record per line:
//   autosage-cache-v3 <device_sig> <graph_sig hex> <F> <H> <op> <dt> <mapping> <f_tile> <wpg> <vec_bytes> <unroll>
//   <hub_t> <hub_chunk> <xcd_remap> <group_lanes> <t_baseline_ms> <t_chosen_ms>
// Records of another device signature are kept out of the in-memory cache (stale-reuse guard).
extern "C" autosage_status_t autosage_cache_load(autosage_handle_t h, const char* path)
{
    if (!h || !path) return AUTOSAGE_ERR_INVALID_ARG;
    std::ifstream in(path);
    if (!in) return AUTOSAGE_ERR_IO;
    std::string line;
    while (std::getline(in, line)) {
        std::istringstream ss(line);
        std::string tag, dev, sig_hex;
        CacheKey k{};
        CacheEntry e{};
        autosage_schedule_t& s = e.sched;
        if (!(ss >> tag >> dev >> sig_hex >> k.F >> k.H >> k.op >> k.dt >> s.mapping >> s.f_tile >> s.waves_per_wg >> s.vec_bytes >>
              s.unroll >> s.hub_t >> s.hub_chunk >> s.xcd_remap >> s.group_lanes >> e.t_baseline_ms >> e.t_chosen_ms))
            continue;
        if (tag != "autosage-cache-v3" || dev != h->device_sig) continue;
        char* end = nullptr;
        k.graph_sig = std::strtoull(sig_hex.c_str(), &end, 16);
        if (end == sig_hex.c_str() || *end != '\0') continue;
        if (s.group_lanes < 0 || s.group_lanes > 64) continue;
        if (s.mapping < 0 || s.mapping > 3 || k.op < 0 || k.op > 3 || !dtype_known(k.dt) || k.F <= 0 || k.H <= 0) continue;
        h->cache[k] = e;
    }
    return AUTOSAGE_OK;
}

extern "C" autosage_status_t autosage_cache_save(autosage_handle_t h, const char* path)
{
    if (!h || !path) return AUTOSAGE_ERR_INVALID_ARG;
    const std::string tmp = std::string(path) + ".tmp";
    {
        std::ofstream out(tmp, std::ios::trunc);
        if (!out) return AUTOSAGE_ERR_IO;
        for (const auto& kv : h->cache) {
            const CacheKey& k = kv.first;
            const autosage_schedule_t& s = kv.second.sched;
            char buf[512];
            std::snprintf(buf, sizeof buf, "autosage-cache-v3 %s %016llx %d %d %d %d %d %d %d %d %d %d %d %d %d %.6f %.6f\n",
                          h->device_sig.c_str(), (unsigned long long)k.graph_sig, k.F, k.H, k.op, k.dt, s.mapping, s.f_tile,
                          s.waves_per_wg, s.vec_bytes, s.unroll, s.hub_t, s.hub_chunk, s.xcd_remap, s.group_lanes,
                          kv.second.t_baseline_ms, kv.second.t_chosen_ms);
            out << buf;
        }
        out.flush();
        if (!out) return AUTOSAGE_ERR_IO;
    }
    if (std::rename(tmp.c_str(), path) != 0) return AUTOSAGE_ERR_IO;
    return AUTOSAGE_OK;
}

extern "C" autosage_status_t autosage_last_decision(autosage_handle_t h, char* json_buf, size_t n)
{
    if (!h || !json_buf || n == 0) return AUTOSAGE_ERR_INVALID_ARG;
    const size_t m = std::min(n - 1, h->last_decision.size());
    std::memcpy(json_buf, h->last_decision.data(), m);
    json_buf[m] = '\0';
    return AUTOSAGE_OK;
}

// ------------------------------------------------------------------------------------------
// the full decision
// ------------------------------------------------------------------------------------------
namespace {

struct OpInput {
    int op;
    int64_t n_rows, n_cols, nnz;
    const int32_t* rowptr;
    const int32_t* colind;
    const float* val;
    const void* d0;
    int64_t ld0;
    const void* d1;
    int64_t ld1;
    float* out;
    int64_t ld_out;
    int32_t F;
    int dt;
    // attention only
    const void* d2;
    int32_t H;
    float scale;
};

autosage_status_t run_once(autosage_ctx* h, const OpInput& in, const RowMap& rows, const autosage_schedule_t& s, void* ws, size_t ws_bytes,
                           hipStream_t st)
{
    const int esize = dtype_bytes(in.dt);
    Resolved r;
    if (in.op == AUTOSAGE_OP_ATTENTION) {
        const AttnCall c{in.n_rows, in.nnz, in.rowptr, in.colind, in.d0, in.d1, in.d2, in.out, in.H, in.F, in.scale, in.dt};
        return exec_attention(h, c, s, rows, ws, ws_bytes, st);
    }
    if (in.op == AUTOSAGE_OP_SPMM) {
        autosage_status_t rc = resolve_schedule(s, in.op, in.F, in.dt, 1, common_alignment(in.d0, in.ld0, esize),
                                                common_alignment(in.out, in.ld_out, 4), &r);
        if (rc != AUTOSAGE_OK) return rc;
        SpmmArgs a{};
        a.rows = rows;
        a.rowptr = in.rowptr;
        a.colind = in.colind;
        a.val = in.val;
        a.B = in.d0;
        a.ldb = in.ld0;
        a.C = in.out;
        a.ldc = in.ld_out;
        a.F = in.F;
        a.dt = in.dt;
        a.heads = 1;
        a.head_dim = in.F;
        return exec_spmm(h, a, r, in.nnz, ws, ws_bytes, st);
    }
    int al = common_alignment(in.d0, in.ld0, esize);
    const int al2 = common_alignment(in.d1, in.ld1, esize);
    if (al2 < al) al = al2;
    autosage_status_t rc = resolve_schedule(s, in.op, in.F, in.dt, 1, al, 16, &r);
    if (rc != AUTOSAGE_OK) return rc;
    SddmmArgs a{};
    a.rows = rows;
    a.rowptr = in.rowptr;
    a.colind = in.colind;
    a.X = in.d0;
    a.ldx = in.ld0;
    a.Y = in.d1;
    a.ldy = in.ld1;
    a.out = in.out;
    a.F = in.F;
    a.dt = in.dt;
    a.heads = 1;
    a.scale = 1.0f;
    return exec_sddmm(h, a, r, in.nnz, ws, ws_bytes, st);
}

// Median of up to `iters` timed runs after one warm-up run; stops early once the timed runs add up
// to cap_ms.  The warm-up is timed as well.  The first launch of a kernel also pays for loading its code
// object (milliseconds), so a long warm-up alone says nothing: it is repeated once, and only when the
// repeat too takes four caps or more (a schedule that is slow on this input) is that time returned as the
// measurement instead of burning more repeats (first_launch = false: the kernels have run before, a long
// warm-up is returned at once).  Returns +inf when the schedule cannot run; `why`
// (optional) then holds the status of the run that failed.
double time_schedule(autosage_ctx* h, const OpInput& in, const RowMap& rows, const autosage_schedule_t& s, void* ws,
                     size_t ws_bytes, hipStream_t st, int iters, double cap_ms, autosage_status_t* why = nullptr,
                     bool first_launch = true)
{
    const double inf = std::numeric_limits<double>::infinity();
    std::vector<double> t;
    double total = 0.0;
    if (why) *why = AUTOSAGE_ERR_HIP;
    for (int i = -2; i < iters; ++i) {
        if (hipEventRecord(h->ev0, st) != hipSuccess) return inf;
        const autosage_status_t rc = run_once(h, in, rows, s, ws, ws_bytes, st);
        if (rc != AUTOSAGE_OK) {
            if (why) *why = rc;
            return inf;
        }
        if (hipEventRecord(h->ev1, st) != hipSuccess) return inf;
        if (hipEventSynchronize(h->ev1) != hipSuccess) return inf;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, h->ev0, h->ev1) != hipSuccess) return inf;
        if (i == -2) {                                // warm-up (may include the code object load)
            if (ms >= 4.0 * cap_ms && !first_launch) return ms;
            if (ms < 4.0 * cap_ms) ++i;               // short: no second warm-up
            continue;
        }
        if (i == -1) {                                // repeat of a long warm-up
            if (ms >= 4.0 * cap_ms) return ms;
            continue;
        }
        t.push_back(ms);
        total += ms;
        if (total >= cap_ms) break;
    }
    if (t.empty()) return inf;
    std::sort(t.begin(), t.end());
    return t[t.size() / 2];
}

std::string num(double x)
{
    if (!std::isfinite(x)) return "null";
    char b[64];
    std::snprintf(b, sizeof b, "%.6f", x);
    return b;
}

}  // namespace

// Candidates of the attention pipeline: the single pass (when the head shape has kernels) and the three
// stages, each over a few hub thresholds; ranked by gathered bytes, score traffic and the longest row.
static void shortlist_attention(const autosage_ctx* h, int64_t nnz, const int64_t* hist, int64_t max_deg, int32_t H,
                                int32_t d, int dt, std::vector<autosage_schedule_t>* out, std::vector<double>* est)
{
    const int esize = dtype_bytes(dt);
    AttnShape shape{};
    const bool can_fuse = attn_fused_shape(H, d, dt, &shape);
    const double row_bytes = 2.0 * H * d * esize;                  // one K row and one V row per nonzero
    const double bw = 6.0e12, t_step = 1.0e-6, t_launch = 6.0e-6;
    std::vector<std::pair<double, autosage_schedule_t>> all;
    const int hubs[] = {0, 256, 512, 1024, 2048};
    for (int fused = 1; fused >= 0; --fused) {
        if (fused && !can_fuse) continue;
        for (int hub : hubs) {
            if (hub > 0 && max_deg < hub) continue;
            if (h->params.force_hub_t >= 0 && hub != hubs[0]) continue;
            autosage_schedule_t s{};
            s.mapping = fused ? AUTOSAGE_MAP_FUSED : AUTOSAGE_MAP_WAVE_ROW;
            s.waves_per_wg = h->params.force_wpb > 0 ? h->params.force_wpb : 4;
            s.hub_t = h->params.force_hub_t >= 0 ? h->params.force_hub_t : hub;
            // a chunk of the single pass carries a state merge
            s.hub_chunk = pick_hub_chunk(hist, max_deg, s.hub_t, fused ? 4 : 1, h->cu_count);
            double t = nnz * row_bytes / bw + (fused ? 0.0 : 16.0 * H * nnz / bw + 2 * t_launch);
            const double longest = s.hub_t > 0 ? std::min<double>((double)max_deg, s.hub_t) : (double)max_deg;
            t = std::max(t, longest / 4.0 * t_step * (fused ? 1.0 : 2.0));
            if (s.hub_t > 0) {
                int64_t hub_nnz = 0;
                for (int b = 1; b < 33; ++b)
                    if (std::ldexp(1.0, b - 1) >= s.hub_t) hub_nnz += (int64_t)(1.5 * std::ldexp(1.0, b - 1) * hist[b]);
                t += (fused ? 3 : 7) * t_launch + 0.05 * hub_nnz * row_bytes / bw;   // chunked rows run a little slower
            }
            all.emplace_back(t, s);
        }
    }
    std::stable_sort(all.begin(), all.end(), [](const auto& a, const auto& b) { return a.first < b.first; });
    for (const auto& e : all) {
        out->push_back(e.second);
        est->push_back(e.first);
    }
}

static autosage_status_t decide_impl(autosage_handle_t h, const OpInput& in, void* workspace, size_t workspace_bytes,
                                     void* stream, autosage_schedule_t* chosen)
{
    const autosage_op_t op = static_cast<autosage_op_t>(in.op);
    const autosage_dtype_t dt = static_cast<autosage_dtype_t>(in.dt);
    const int64_t n_rows = in.n_rows, n_cols = in.n_cols, nnz = in.nnz;
    const int32_t* rowptr = in.rowptr;
    const void* dense0 = in.d0;
    const void* dense1 = in.d1;
    const int64_t ld0 = in.ld0, ld1 = in.ld1, ld_out = in.ld_out;
    float* out = in.out;
    const int32_t F = in.F;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const auto wall0 = std::chrono::steady_clock::now();

    // 1. features and signature (memoised per rowptr pointer when allowed)
    int64_t hist[33];
    int64_t max_deg = 0;
    uint64_t sig = 0;
    bool have = false;
    if (h->params.memoize_signature) {
        for (const SigMemo& m : h->memo) {
            if (m.rowptr == rowptr && m.n_rows == n_rows && m.n_cols == n_cols && m.nnz == nnz) {
                sig = m.sig;
                max_deg = m.max_deg;
                std::memcpy(hist, m.hist, sizeof hist);
                have = true;
                break;
            }
        }
    }
    // Neither the feature pass (a device-to-host copy and a wait) nor probes may run on a stream that is being
    // captured into a graph: such a call is refused before it touches the stream.
    auto capturing = [&]() {
        hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
        return hipStreamIsCapturing(st, &cs) == hipSuccess && cs != hipStreamCaptureStatusNone;
    };
    if (!have) {
        if (capturing()) return AUTOSAGE_ERR_UNSUPPORTED;
        int64_t nnz_dev = 0;
        autosage_status_t rc = autosage_graph_features(h, n_rows, n_cols, rowptr, hist, &max_deg, &nnz_dev, &sig, stream);
        if (rc != AUTOSAGE_OK) return rc;
        if (nnz_dev != nnz) return AUTOSAGE_ERR_INVALID_ARG;
        if (h->params.memoize_signature) {
            SigMemo m{};
            m.rowptr = rowptr;
            m.n_rows = n_rows;
            m.n_cols = n_cols;
            m.nnz = nnz;
            m.sig = sig;
            m.max_deg = max_deg;
            std::memcpy(m.hist, hist, sizeof hist);
            if (h->memo.size() >= 16) h->memo.erase(h->memo.begin());
            h->memo.push_back(m);
        }
    }

    std::ostringstream js;
    char sigbuf[32];
    std::snprintf(sigbuf, sizeof sigbuf, "%016llx", (unsigned long long)sig);
    js << "{\"op\":" << (int)op << ",\"F\":" << F << ",\"H\":" << in.H << ",\"dt\":" << (int)dt << ",\"graph_sig\":\"" << sigbuf
       << "\",\"device_sig\":\"" << h->device_sig << "\",\"alpha\":" << num(h->params.alpha);

    // 2. cache
    const CacheKey key{sig, F, in.H, (int32_t)op, (int32_t)dt};
    auto it = h->cache.find(key);
    if (it != h->cache.end()) {
        *chosen = it->second.sched;
        js << ",\"cache_hit\":true,\"replay_miss\":false,\"choice\":" << schedule_json(*chosen) << "}";
        h->last_decision = js.str();
        return AUTOSAGE_OK;
    }
    const autosage_schedule_t base = baseline_schedule();
    if (h->params.replay_only) {
        *chosen = base;
        js << ",\"cache_hit\":false,\"replay_miss\":true,\"choice\":" << schedule_json(base) << "}";
        h->last_decision = js.str();
        return AUTOSAGE_OK;
    }

    // 3. shortlist
    if (capturing()) return AUTOSAGE_ERR_UNSUPPORTED;
    const int esize = dtype_bytes(dt);
    int al = common_alignment(dense0, ld0, esize);
    if (op == AUTOSAGE_OP_SDDMM) al = std::min(al, common_alignment(dense1, ld1, esize));
    else if (op == AUTOSAGE_OP_SPMM) al = std::min(al, common_alignment(out, ld_out, 4));
    std::vector<autosage_schedule_t> cands;
    std::vector<double> est;
    {
        // the probes get the best-ranked candidates that differ in more than the unroll depth
        std::vector<autosage_schedule_t> all;
        std::vector<double> all_est;
        if (op == AUTOSAGE_OP_ATTENTION) shortlist_attention(h, nnz, hist, max_deg, in.H, F, dt, &all, &all_est);
        else shortlist(h, op, n_rows, n_cols, nnz, hist, max_deg, F, dt, al, &all, &all_est);
        for (size_t i = 0; i < all.size() && (int)cands.size() < h->params.probe_topk; ++i) {
            if (all[i].f_tile != 0 && h->params.force_ftile <= 0) continue;      // narrow tiles: below
            bool fresh = true;
            for (const autosage_schedule_t& c : cands)
                if (c.mapping == all[i].mapping && c.hub_t == all[i].hub_t && c.xcd_remap == all[i].xcd_remap &&
                    c.vec_bytes == all[i].vec_bytes && c.group_lanes == all[i].group_lanes)
                    fresh = false;
            if (fresh) {
                cands.push_back(all[i]);
                est.push_back(all_est[i]);
            }
        }
        // the best-ranked candidate of every narrow tile width, with and without the XCD-aware launch, is
        // probed on top of the k above (their gain is a cache effect that the estimate cannot see)
        if (h->params.force_ftile <= 0) {
            for (size_t i = 0; i < all.size(); ++i) {
                if (all[i].f_tile == 0) continue;
                bool fresh = true;
                for (const autosage_schedule_t& c : cands)
                    if (c.f_tile == all[i].f_tile && c.xcd_remap == all[i].xcd_remap) fresh = false;
                if (fresh) {
                    cands.push_back(all[i]);
                    est.push_back(all_est[i]);
                }
            }
        }
        // attention: both pipelines are probed; when the single pass fills the k above, the best-ranked
        // three-stage candidate is added (which of the two wins depends on how much of K and V the caches keep)
        if (op == AUTOSAGE_OP_ATTENTION) {
            bool have_three = false;
            for (const autosage_schedule_t& c : cands) have_three = have_three || c.mapping == AUTOSAGE_MAP_WAVE_ROW;
            for (size_t i = 0; i < all.size() && !have_three; ++i) {
                if (all[i].mapping != AUTOSAGE_MAP_WAVE_ROW) continue;
                cands.push_back(all[i]);
                est.push_back(all_est[i]);
                have_three = true;
            }
        }
    }
    const int topk = (int)cands.size();

    // 4. probes on a sample of row blocks, run in place (all candidates see the identical sample).
    // Blocks of 256 consecutive rows keep the locality between neighbouring rows that a single-row
    // stride would destroy; the blocks are spread evenly over the matrix.
    const int64_t min_rows = std::max(1, h->params.probe_min_rows);
    int64_t target = std::max<int64_t>(min_rows, (int64_t)std::ceil(h->params.probe_frac * (double)n_rows));
    RowMap sample{0, 1, (int32_t)n_rows, 0};
    int64_t stride = 1;
    if (target < n_rows) {
        const int shift = 8;
        const int64_t block = int64_t(1) << shift;
        const int64_t nb = std::max<int64_t>(1, target / block);
        if (nb * block < n_rows) {
            stride = n_rows / nb;                 // >= block
            sample = RowMap{(int32_t)((stride - block) / 2), (int32_t)stride, (int32_t)(nb * block), shift};
        }
    }

    // The baseline walks every row with one wavefront, so a single row of tens of thousands of entries makes
    // one run of it take many milliseconds.  When such rows exist the baseline is first bounded from below:
    // it is timed on the sample with the rows of kBaselineBoundDeg entries or more left out.  The full
    // baseline cannot be faster than that, so a candidate accepted against the bound (t* <= alpha * bound)
    // is accepted against the baseline itself; only when the bound does not settle the decision is the whole
    // baseline timed.  `light` runs the baseline in that mode; the probe calls pass `why` and may be the first
    // launch of the baseline's kernels, the confirmation calls are not.
    auto time_baseline = [&](const RowMap& rows, bool light, int iters, double cap, autosage_status_t* why,
                             int skip_deg = kBaselineBoundDeg) {
        h->probe_skip_deg = light ? skip_deg : 0;
        const double t = time_schedule(h, in, rows, base, workspace, workspace_bytes, st, iters, cap, why, why != nullptr);
        h->probe_skip_deg = 0;
        return t;
    };
    const bool can_bound = h->params.baseline_bound != 0 && max_deg >= kBaselineBoundDeg;
    // the baseline must be able to run on this input: report its own error (e.g. a short workspace)
    autosage_status_t base_rc = AUTOSAGE_OK;
    double tb = time_baseline(sample, can_bound, h->params.probe_iters, h->params.probe_cap_ms, &base_rc);
    if (!std::isfinite(tb)) return base_rc;
    bool tb_is_bound = can_bound;
    std::vector<double> tc(topk);
    for (int c = 0; c < topk; ++c)
        tc[c] = time_schedule(h, in, sample, cands[c], workspace, workspace_bytes, st, h->params.probe_iters,
                              h->params.probe_cap_ms);

    // 4b. refinement (SpMM, SDDMM): the estimate ranks from the degree histogram alone, so knobs whose gain is a
    // cache or tail effect (XCD-aware launch, narrow tiles, narrow lane groups, the split threshold next door) may
    // be missing from the k above in the combination that wins.  The schedules that differ from the best probed one
    // in a single knob are probed on the same sample, and once more around the new best when one of them wins.
    // A neighbour joins the candidate list the decision rule runs over only when it beats the best so far by
    // kRefineGain: differences of a per cent or two are within the noise of a probe on a row sample, and the knob
    // left alone is the cheaper guess (the XCD-aware launch costs 1-2 % on a graph without locality).
    if (op != AUTOSAGE_OP_ATTENTION && h->params.probe_refine > 0) {
        const bool tile_ok = h->params.force_ftile <= 0 && (int64_t)F * esize >= 512 &&
                             (double)n_cols * F * esize >= kTileOperandBytes;
        const int hub_steps[] = {0, 512, 1024, 2048, 4096};
        auto same = [](const autosage_schedule_t& a, const autosage_schedule_t& b) { return std::memcmp(&a, &b, sizeof a) == 0; };
        int extra = 0;
        for (int round = 0; round < 2 && extra < h->params.probe_refine; ++round) {
            int best = -1;
            for (size_t c = 0; c < cands.size(); ++c)
                if (std::isfinite(tc[c]) && (best < 0 || tc[c] < tc[best])) best = (int)c;
            if (best < 0 || cands[best].mapping != AUTOSAGE_MAP_WAVE_ROW) break;
            const autosage_schedule_t b = cands[best];
            std::vector<autosage_schedule_t> nb;
            autosage_schedule_t s = b;
            s.xcd_remap = !b.xcd_remap;
            nb.push_back(s);
            if (op == AUTOSAGE_OP_SDDMM && b.vec_bytes == 16) {
                s = b;
                s.group_lanes = b.group_lanes ? 0 : 8;
                if (s.group_lanes == 0) s.f_tile = 0;            // the tiled form is only proposed with narrow groups
                Resolved r;
                // a tile no wider than the group runs the same kernel as group_lanes = 0: not a neighbour
                if (resolve_schedule(s, op, F, dt, 1, al, 16, &r) == AUTOSAGE_OK && (s.group_lanes == 0 || r.G == s.group_lanes))
                    nb.push_back(s);
            }
            if (tile_ok && b.vec_bytes >= 8) {
                s = b;
                s.f_tile = b.f_tile ? 0 : 256 / esize;
                if (op == AUTOSAGE_OP_SDDMM && s.f_tile) s.group_lanes = 8;
                nb.push_back(s);
            }
            if (h->params.force_hub_t < 0) {
                int at = 0;
                for (int i = 0; i < 5; ++i)
                    if (hub_steps[i] <= b.hub_t) at = i;
                for (int i : {at - 1, at + 1}) {
                    if (i < 0 || i > 4 || (hub_steps[i] > 0 && max_deg < hub_steps[i])) continue;
                    s = b;
                    s.hub_t = hub_steps[i];
                    s.hub_chunk = pick_hub_chunk(hist, max_deg, s.hub_t, 4, h->cu_count);
                    nb.push_back(s);
                }
            }
            bool improved = false;
            for (const autosage_schedule_t& cand : nb) {
                if (extra >= h->params.probe_refine) break;
                bool seen = false;
                for (const autosage_schedule_t& c : cands) seen = seen || same(c, cand);
                if (seen) continue;
                const double t = time_schedule(h, in, sample, cand, workspace, workspace_bytes, st, h->params.probe_iters,
                                               h->params.probe_cap_ms);
                ++extra;
                if (!std::isfinite(t) || !(t <= kRefineGain * tc[best])) continue;     // no kernel for the shape, or no clear gain
                cands.push_back(cand);
                est.push_back(std::numeric_limits<double>::quiet_NaN());
                tc.push_back(t);
                improved = true;
            }
            if (!improved) break;
        }
    }
    // Attention with K and V larger than the Infinity Cache: the fastest single pass of the sample is also probed with
    // the heads walked in two tiles (each tile gathers from half of K and V).  What that gains is a cache effect of
    // the whole input, so the two forms are run off there (step 6) whatever the sample says.
    if (op == AUTOSAGE_OP_ATTENTION && h->params.force_ftile <= 0 && in.H % 2 == 0 &&
        2.0 * (double)n_cols * in.H * F * esize > kHeadTileOperandBytes) {
        int best = -1;
        for (int c = 0; c < topk; ++c)
            if (cands[c].mapping == AUTOSAGE_MAP_FUSED && cands[c].f_tile == 0 && std::isfinite(tc[c]) && (best < 0 || tc[c] < tc[best]))
                best = c;
        AttnShape shape{};
        if (best >= 0 && attn_fused_shape_tiled(in.H, F, dt, in.H / 2, &shape)) {
            autosage_schedule_t tiled = cands[best];
            tiled.f_tile = (in.H / 2) * F;
            const double t = time_schedule(h, in, sample, tiled, workspace, workspace_bytes, st, h->params.probe_iters,
                                           h->params.probe_cap_ms);
            if (std::isfinite(t)) {
                cands.push_back(tiled);
                est.push_back(est[best]);
                tc.push_back(t);
            }
        }
    }
    const int n_probed = (int)cands.size();
    js << ",\"cache_hit\":false,\"replay_miss\":false,\"probe_rows\":" << sample.count << ",\"probe_stride\":" << stride
       << ",\"candidates\":[";
    for (int c = 0; c < n_probed; ++c)
        js << (c ? "," : "") << "{\"sched\":" << schedule_json(cands[c]) << ",\"est_ms\":" << num(est[c] * 1e3)
           << ",\"t_ms\":" << num(tc[c]) << (c >= topk ? ",\"refinement\":true" : "") << "}";
    js << "]";

    // 5. guardrail
    int choice = decide_from_times(n_probed, tc.data(), tb, h->params.alpha);
    if (choice < 0 && tb_is_bound) {              // the bound rejects everything: ask the baseline itself
        tb = time_baseline(sample, false, h->params.probe_iters, h->params.probe_cap_ms, &base_rc);
        if (!std::isfinite(tb)) return base_rc;
        tb_is_bound = false;
        choice = decide_from_times(n_probed, tc.data(), tb, h->params.alpha);
    }
    double t_choice = choice >= 0 ? tc[choice] : tb;
    js << ",\"t_baseline_ms\":" << num(tb) << ",\"baseline_light_rows_only\":" << (tb_is_bound ? "true" : "false")
       << ",\"choice_index\":" << choice;

    // 6. the guardrail speaks about the sample; confirm once on the whole input
    if (choice >= 0 && h->params.confirm_full) {
        const RowMap full{0, 1, (int32_t)n_rows, 0};
        // its kernels have run on the sample: up to two timed runs after a warm-up, fewer once kFullInputCapMs are
        // spent, and a warm-up of four times that or more is itself the measurement (large inputs: one run)
        double tf_c = time_schedule(h, in, full, cands[choice], workspace, workspace_bytes, st, 2, kFullInputCapMs, nullptr, false);
        // A schedule found by the refinement rounds won on the sample, where a launch is short and latency counts
        // for more than on the whole input.  It is run off against the best of the ranked candidates on the whole
        // input (when that one passes the guardrail too) and the faster of the two is kept.
        std::string runoff;
        if (op == AUTOSAGE_OP_ATTENTION && cands[choice].mapping == AUTOSAGE_MAP_FUSED) {
            // the same single pass with and without head tiles: the tiled form must win by kRefineGain on the whole
            // input to be kept, the untiled one takes over from a tiled choice whenever it is faster there
            for (int c = 0; c < n_probed; ++c) {
                autosage_schedule_t twin = cands[c];
                twin.f_tile = cands[choice].f_tile;
                if (c == choice || cands[c].f_tile == cands[choice].f_tile || std::memcmp(&twin, &cands[choice], sizeof twin) != 0)
                    continue;
                if (!(tc[c] <= h->params.alpha * tb)) break;
                const double tf_t = time_schedule(h, in, full, cands[c], workspace, workspace_bytes, st, 2, kFullInputCapMs, nullptr, false);
                const bool to_tiled = cands[c].f_tile != 0;
                const bool switched = to_tiled ? tf_t <= kRefineGain * tf_c : tf_t < tf_c;
                runoff = ",\"runoff\":{\"index\":" + std::to_string(c) + ",\"t_ms\":" + num(tf_t) + ",\"t_refined_ms\":" +
                         num(tf_c) + ",\"head_tiles\":true,\"switched\":" + (switched ? "true" : "false") + "}";
                if (switched) {
                    choice = c;
                    t_choice = tc[c];
                    tf_c = tf_t;
                }
                break;
            }
        }
        if (choice >= topk && op != AUTOSAGE_OP_ATTENTION) {
            int best0 = -1;
            for (int c = 0; c < topk; ++c)
                if (std::isfinite(tc[c]) && (best0 < 0 || tc[c] < tc[best0])) best0 = c;
            if (best0 >= 0 && tc[best0] <= h->params.alpha * tb) {
                const double tf_0 = time_schedule(h, in, full, cands[best0], workspace, workspace_bytes, st, 2, kFullInputCapMs, nullptr, false);
                const bool switched = tf_0 < tf_c;
                runoff = ",\"runoff\":{\"index\":" + std::to_string(best0) + ",\"t_ms\":" + num(tf_0) + ",\"t_refined_ms\":" +
                         num(tf_c) + ",\"switched\":" + (switched ? "true" : "false") + "}";
                if (switched) {
                    choice = best0;
                    t_choice = tc[best0];
                    tf_c = tf_0;
                }
            }
        }
        // Lower bounds of the baseline on the whole input, cheapest first: its time on the sample (a subset of
        // the rows), then its rows below 8 * kBaselineBoundDeg entries on the whole input (the longest of them
        // still costs one wavefront well under a millisecond).  When a bound already covers the choice's time the
        // baseline itself is not run; otherwise one run of it that takes more than twice the choice settles it.
        bool bound_settles = sample.count < n_rows && tb >= tf_c;
        double tf_b = tb;
        if (!bound_settles && can_bound) {
            tf_b = time_baseline(full, true, 2, 0.5 * tf_c, nullptr, 8 * kBaselineBoundDeg);
            bound_settles = std::isfinite(tf_b) && tf_b >= tf_c;
        }
        if (!bound_settles) tf_b = time_baseline(full, false, 2, 0.5 * tf_c, nullptr);
        const bool demote = !(tf_c <= tf_b);
        js << ",\"confirm\":{\"t_choice_ms\":" << num(tf_c) << ",\"t_baseline_ms\":" << num(tf_b)
           << ",\"baseline_bound_only\":" << (bound_settles ? "true" : "false") << ",\"demoted\":"
           << (demote ? "true" : "false") << runoff << "}";
        if (demote) {
            choice = -1;
            t_choice = tb;
        }
    }
    *chosen = choice >= 0 ? cands[choice] : base;
    h->cache[key] = CacheEntry{*chosen, tb, t_choice};
    const double wall_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - wall0).count();
    js << ",\"choice\":" << schedule_json(*chosen) << ",\"probe_wall_ms\":" << num(wall_ms) << "}";
    h->last_decision = js.str();
    return AUTOSAGE_OK;
}

extern "C" autosage_status_t autosage_decide(autosage_handle_t h, autosage_op_t op, int64_t n_rows, int64_t n_cols,
                                             int64_t nnz, const int32_t* rowptr, const int32_t* colind, const float* val,
                                             const void* dense0, int64_t ld0, const void* dense1, int64_t ld1,
                                             float* out, int64_t ld_out, int32_t F, autosage_dtype_t dt,
                                             void* workspace, size_t workspace_bytes, void* stream,
                                             autosage_schedule_t* chosen)
{
    if (!h || !chosen || !rowptr || F <= 0 || n_rows < 0 || nnz < 0) return AUTOSAGE_ERR_INVALID_ARG;
    if (op != AUTOSAGE_OP_SPMM && op != AUTOSAGE_OP_SDDMM) return AUTOSAGE_ERR_INVALID_ARG;
    if (!dtype_known(dt)) return AUTOSAGE_ERR_INVALID_ARG;
    if (h->device < 0) return AUTOSAGE_ERR_UNSUPPORTED;
    if (nnz > 0 && (!colind || !dense0 || !out || (op == AUTOSAGE_OP_SPMM && !val) || (op == AUTOSAGE_OP_SDDMM && !dense1)))
        return AUTOSAGE_ERR_INVALID_ARG;
    OpInput in{(int)op, n_rows, n_cols, nnz, rowptr, colind, val, dense0, ld0, dense1, ld1, out, ld_out, F, (int)dt,
               nullptr, 1, 1.0f};
    return decide_impl(h, in, workspace, workspace_bytes, stream, chosen);
}

extern "C" autosage_status_t autosage_decide_attention(autosage_handle_t h, int64_t N, int64_t nnz, const int32_t* rowptr,
                                                       const int32_t* colind, const void* Q, const void* K, const void* V,
                                                       float* O, int32_t H, int32_t d, float scale, autosage_dtype_t dt,
                                                       void* workspace, size_t workspace_bytes, void* stream,
                                                       autosage_schedule_t* chosen)
{
    if (!h || !chosen || !rowptr || H <= 0 || d <= 0 || N < 0 || nnz < 0) return AUTOSAGE_ERR_INVALID_ARG;
    if (!dtype_known(dt)) return AUTOSAGE_ERR_INVALID_ARG;
    if (h->device < 0) return AUTOSAGE_ERR_UNSUPPORTED;
    if (!O || (nnz > 0 && (!colind || !Q || !K || !V))) return AUTOSAGE_ERR_INVALID_ARG;
    const AttnCall c{N, nnz, rowptr, colind, Q, K, V, O, H, d, scale, (int)dt};
    autosage_status_t rc = attention_alignment(c);
    if (rc != AUTOSAGE_OK) return rc;
    const int64_t HD = (int64_t)H * d;
    OpInput in{AUTOSAGE_OP_ATTENTION, N, N, nnz, rowptr, colind, nullptr, Q, HD, K, HD, O, HD, d, (int)dt, V, H, scale};
    return decide_impl(h, in, workspace, workspace_bytes, stream, chosen);
}

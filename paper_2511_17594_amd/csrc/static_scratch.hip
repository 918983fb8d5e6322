// autosage_spmm_static: the SpMM entry point for callers that cannot allocate device memory.  The scratch that the
// hub split needs (partition metadata and the per-chunk partial rows) lives in a fixed array inside the
// library's device image instead of a caller-provided workspace.
#include <hip/hip_runtime.h>

#include <mutex>

#include "internal.h"

namespace {

// One copy per GPU the library is loaded on, held until the process ends.  In host code the array's name is
// only a handle for hipGetSymbolAddress; kernels and copies get the device address looked up below.
static __device__ __align__(256) unsigned char scratch[AUTOSAGE_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;     // handles may be created from several threads

}  // namespace

namespace autosage {

autosage_status_t static_scratch_address(int device, void** ptr)
{
    if (!ptr || device < 0 || device >= kMaxDevices) return AUTOSAGE_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return AUTOSAGE_ERR_HIP;
        g_scratch_ptr[device] = p;
    }
    *ptr = g_scratch_ptr[device];
    return AUTOSAGE_OK;
}

}  // namespace autosage

extern "C" autosage_status_t autosage_spmm_static(autosage_handle_t h, int64_t n_rows, int64_t n_cols, int64_t nnz,
                                                  const int32_t* rowptr, const int32_t* colind, const float* val,
                                                  const void* B, int64_t ldb, float* C, int64_t ldc, int32_t F,
                                                  autosage_dtype_t dt, const autosage_schedule_t* sched, void* stream)
{
    using namespace autosage;
    if (!h || !sched) return AUTOSAGE_ERR_INVALID_ARG;          // the selector may probe and synchronise: explicit schedules only
    if (h->device < 0) return AUTOSAGE_ERR_UNSUPPORTED;
    if (!h->static_scratch) return AUTOSAGE_ERR_HIP;
    if (n_rows < 0 || nnz < 0 || n_rows > kMaxNnz || nnz > kMaxNnz || F <= 0) return AUTOSAGE_ERR_INVALID_ARG;
    const int chunk = effective_hub_chunk(sched->hub_t, sched->hub_chunk);
    if (sched->hub_t < 0 || sched->hub_chunk < 0 ||
        (sched->hub_t > 0 && (sched->hub_t < kMinHubT || chunk < kMinHubT || chunk > kMaxHubChunk)))
        return AUTOSAGE_ERR_INVALID_ARG;
    // what this schedule would ask of a caller's workspace must fit the fixed array
    if (hub_workspace_bytes(n_rows, nnz, sched->hub_t, chunk, F) > (size_t)AUTOSAGE_STATIC_SCRATCH_BYTES)
        return AUTOSAGE_ERR_WORKSPACE_TOO_SMALL;
    // stage telemetry creates events on first use: kept off here, this call creates nothing
    const bool profiling = h->profiling;
    h->profiling = false;
    const autosage_status_t rc = spmm_entry(h, n_rows, n_cols, nnz, rowptr, colind, val, B, ldb, C, ldc, F, (int)dt, sched,
                                            h->static_scratch, (size_t)AUTOSAGE_STATIC_SCRATCH_BYTES, stream);
    h->profiling = profiling;
    return rc;
}

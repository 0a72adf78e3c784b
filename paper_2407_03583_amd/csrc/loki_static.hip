// loki_alloc_search_static: the search for callers that cannot allocate device memory (code under HIP
// graph capture around it, tight serving loops, harnesses that forbid hipMalloc).  All the device
// scratch of a search -- constant block, per-task tables, run order, block records, results -- lives in
// one file-scope device array instead of a caller's workspace.  Every GPU the library runs on holds its
// own copy of the array, at its own address, until the process ends.
#include <hip/hip_runtime.h>

#include <mutex>

#include "loki_host.h"

namespace {

static_assert(LOKI_STATIC_SCRATCH_BYTES % 256 == 0, "scratch size");

static __device__ __align__(256) __attribute__((used)) unsigned char scratch[LOKI_STATIC_SCRATCH_BYTES];

// Device address of `scratch` per device, looked up once with that device current.  In host code the
// array's name is only a handle for the symbol lookup; kernels and copies get the pointer kept here.
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_lock;

int scratch_of_current_device(void **ptr) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return loki::note_hip_error(static_cast<int>(e));
    if (dev < 0 || dev >= kMaxDevices) return LOKI_E_ARG;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return loki::note_hip_error(static_cast<int>(e));
        if (!p) return loki::note_hip_error(static_cast<int>(hipErrorInvalidSymbol));
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return LOKI_OK;
}

}  // namespace

extern "C" int loki_alloc_search_static(loki_problem_t *problem, const int64_t *demand_mqps, int32_t n_demand,
                                        int32_t workers, int64_t slo_us, int64_t comm_us, uint32_t flags,
                                        uint64_t index_begin, uint64_t index_end, void *hip_stream,
                                        loki_result_t *out) {
    if (!problem || !demand_mqps || !out) return LOKI_E_NULL;
    if (n_demand < 1) return LOKI_E_ARG;
    if (n_demand > loki::kNoAllocPoints) return LOKI_E_STATIC_LIMIT;
    size_t need = 0;
    int rc = loki::plain_search_bytes(problem, n_demand, &need);
    if (rc) return rc;
    if (need > size_t(LOKI_STATIC_SCRATCH_BYTES)) return LOKI_E_STATIC_LIMIT;
    void *ws = nullptr;
    rc = scratch_of_current_device(&ws);
    if (rc) return rc;
    // Nothing in the buffer has to start at zero: every kernel of a search writes what the next one reads
    // (tables, run order, one record per block, results), so the last call's contents are simply overwritten.
    return loki::search_without_allocation(problem, demand_mqps, n_demand, workers, slo_us, comm_us, flags,
                                           index_begin, index_end, ws, size_t(LOKI_STATIC_SCRATCH_BYTES),
                                           static_cast<hipStream_t>(hip_stream), out);
}

// Stand-ins for the HIP runtime and for the kernel launches, so that the host side of the library
// (validation, layouts, batching, the class walk, staging, result plumbing) can be built for the CPU with
// AddressSanitizer and UndefinedBehaviorSanitizer.  "Device" memory is ordinary memory; a launch does not
// compute anything, it writes every array its kernel would write (over the extents the launch
// configuration implies), so that a layout that is too small for its launch is an ASan report.
#include <hip/hip_runtime_api.h>

#include <cstdlib>
#include <cstring>

#include "../../paper_2407_03583_amd/csrc/loki_launch.h"

extern "C" {

hipError_t hipMemcpyAsync(void *dst, const void *src, size_t bytes, hipMemcpyKind, hipStream_t) {
    std::memmove(dst, src, bytes);
    return hipSuccess;
}
hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
hipError_t hipEventCreate(hipEvent_t *e) {
    *e = reinterpret_cast<hipEvent_t>(std::malloc(8));
    return hipSuccess;
}
hipError_t hipEventCreateWithFlags(hipEvent_t *e, unsigned) { return hipEventCreate(e); }
hipError_t hipEventRecord(hipEvent_t e, hipStream_t) { return e ? hipSuccess : hipErrorInvalidHandle; }
hipError_t hipEventSynchronize(hipEvent_t e) { return e ? hipSuccess : hipErrorInvalidHandle; }
hipError_t hipEventElapsedTime(float *ms, hipEvent_t a, hipEvent_t b) {
    *ms = 0.f;
    return a && b ? hipSuccess : hipErrorInvalidHandle;
}
hipError_t hipEventDestroy(hipEvent_t e) {
    std::free(e);
    return hipSuccess;
}
hipError_t hipHostMalloc(void **p, size_t bytes, unsigned) {
    *p = std::malloc(bytes ? bytes : 1);
    return *p ? hipSuccess : hipErrorOutOfMemory;
}
hipError_t hipHostFree(void *p) {
    std::free(p);
    return hipSuccess;
}

}  // extern "C"

namespace loki {

namespace {
template <typename T>
void touch(T *p, size_t n) {
    if (n) std::memset(static_cast<void *>(p), 0x5a, n * sizeof(T));
}
const DevProblem &problem_of(const SearchArgs &A) { return *A.P; }
}  // namespace

hipError_t launch_task_table(const SearchArgs &A, uint32_t table_total, hipStream_t) {
    if (table_total != problem_of(A).table_total) return hipErrorInvalidValue;
    touch(A.table, size_t(A.M) * table_total);
    if (A.lat2) touch(A.lat2, size_t(A.M) * table_total);
    touch(A.floor, size_t(A.M));
    volatile int64_t sink = 0;
    for (size_t q = 0; q < size_t(A.M) * kMaxTasks; q++) sink = sink + A.Dn[q];
    if (A.class_amount)
        for (size_t q = 0; q < size_t(A.M) * kMaxTasks; q++) sink = sink + A.class_amount[q];
    return hipSuccess;
}

hipError_t launch_root_order(const SearchArgs &A, hipStream_t) {
    const DevProblem &P = problem_of(A);
    if (A.swap) {
        touch(A.perm_all, size_t(A.M) * P.table_total);
        touch(A.run_end_t, size_t(A.M) * P.C[P.tile_task]);
    } else {
        touch(A.perm, size_t(A.M) * P.C[0]);
        touch(A.run_end, size_t(A.M) * P.C[0]);
    }
    return hipSuccess;
}

static hipError_t visit(const SearchArgs &A) {
    if (A.blocks_per_m == 0 || A.M <= 0) return hipErrorInvalidValue;
    if (uint64_t(A.blocks_per_m) * uint64_t(A.M) > (uint64_t(1) << 31)) return hipErrorInvalidValue;
    touch(A.recs, size_t(A.M) * A.blocks_per_m);
    if (A.class_count) {
        volatile uint32_t sink = 0;
        for (size_t q = 0; q < size_t(A.M) * kMaxTasks; q++) sink = sink + A.class_count[q];
    }
    if (A.path_acc) {
        volatile double sink = 0;
        for (uint32_t q = 0; q < problem_of(A).path_total; q++) sink = sink + A.path_acc[q];
    }
    return hipSuccess;
}

hipError_t launch_combine(const SearchArgs &A, int slots, bool, bool, bool, bool, hipStream_t) {
    if (slots != 4 && slots != 8) return hipErrorInvalidValue;
    if (A.tile_len == 0 || A.tile_len > uint32_t(kMidTile) || A.cpb == 0 || A.cpb > uint32_t(kWavesPerBlock))
        return hipErrorInvalidValue;
    if (A.items_per_block * A.blocks_per_m + A.items_extra != A.items && !A.swap) return hipErrorInvalidValue;
    return visit(A);
}
hipError_t launch_path_combine(const SearchArgs &A, int slots, bool, int, hipStream_t) {
    if (slots != 4 && slots != 8) return hipErrorInvalidValue;
    return visit(A);
}
hipError_t launch_per_lane_search(const SearchArgs &A, bool, bool, int, int, hipStream_t) { return visit(A); }
hipError_t launch_open_plans(const SearchArgs &A, int slots, bool, int levels, hipStream_t) {
    if ((slots != 4 && slots != 8) || levels < 2 || !A.lat2) return hipErrorInvalidValue;
    volatile uint32_t sink = 0;   // the second table, as the task table kernel leaves it
    for (size_t q = 0; q < size_t(A.M) * problem_of(A).table_total; q++)
        sink = sink + uint32_t(A.lat2[q].top) + uint32_t(A.lat2[q].bot);
    return visit(A);
}
hipError_t launch_fold_results(void *results, const void *other, int M, bool, hipStream_t) {
    touch(static_cast<unsigned char *>(results), size_t(M) * 32);
    volatile unsigned char sink = 0;
    for (size_t q = 0; q < size_t(M) * 32; q++) sink = sink + static_cast<const unsigned char *>(other)[q];
    return hipSuccess;
}

hipError_t launch_final_reduce(const SearchArgs &A, hipStream_t) {
    // "nothing found" for every point
    struct R { uint64_t index; double accuracy; uint64_t n_feasible; int32_t workers_used, status; };
    R *out = static_cast<R *>(A.results);
    for (int m = 0; m < A.M; m++) out[m] = R{~0ull, 0.0, 0, -1, 1};
    return hipSuccess;
}
hipError_t launch_results_init(const MergeArgs &A, hipStream_t) {
    touch(static_cast<unsigned char *>(A.results), size_t(A.M) * 32);
    return hipSuccess;
}
hipError_t launch_class_merge(const MergeArgs &A, hipStream_t) {
    volatile int sink = 0;
    for (int q = 0; q < A.n; q++) {
        if (A.point[q] < 0) return hipErrorInvalidValue;
        sink = sink + A.point[q];
    }
    touch(static_cast<unsigned char *>(A.class_results), size_t(A.n) * 32);
    return hipSuccess;
}
hipError_t launch_eval(const EvalArgs &A, hipStream_t) {
    volatile uint64_t sink = 0;
    for (int64_t q = 0; q < A.n; q++) sink = sink + A.indices[q];
    touch(static_cast<unsigned char *>(A.out), size_t(A.n) * 16);
    return hipSuccess;
}
hipError_t launch_route(const RouteArgs &A, hipStream_t) {
    volatile uint64_t sink = 0;
    for (int64_t q = 0; q < A.n; q++) sink = sink + A.indices[q] + uint64_t(A.demand[q]);
    touch(A.out, size_t(A.n));
    return hipSuccess;
}

}  // namespace loki

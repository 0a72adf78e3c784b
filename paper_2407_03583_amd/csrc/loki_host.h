// Host-side functions shared by the C-ABI entry points that live in different source files.
#pragma once

#include <hip/hip_runtime_api.h>

#include "../../include/loki_alloc.h"

namespace loki {

// most demand points of a search that allocates nothing (their demands are staged in a block of ordinary
// host memory that every handle owns from its creation)
constexpr int32_t kNoAllocPoints = 64;

// Bytes of device workspace of a search of n_demand demand points that does not run class by class.
int plain_search_bytes(const loki_problem_t *p, int32_t n_demand, size_t *bytes);

// loki_alloc_search in the given workspace without any allocation on the way: no pinned staging, no
// events, never class by class (per-variant factors score whole plans per lane, profiled path accuracies
// walk the variant paths of feasible plans).  Same results as loki_alloc_search.
int search_without_allocation(loki_problem_t *p, const int64_t *demand_mqps, int32_t n_demand, int32_t workers,
                              int64_t slo_us, int64_t comm_us, uint32_t flags, uint64_t index_begin,
                              uint64_t index_end, void *d_workspace, size_t workspace_bytes, hipStream_t stream,
                              loki_result_t *out);

// Remember a HIP error code for loki_last_hip_error(); returns LOKI_E_HIP.
int note_hip_error(int hip_error);

}  // namespace loki

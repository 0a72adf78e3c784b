// Launch wrappers implemented in loki_kernels.hip (one call = one kernel enqueued
// on the given stream; the return value is hipGetLastError() after the launch).
#pragma once

#include <hip/hip_runtime_api.h>

#include "loki_device.h"

namespace loki {

hipError_t launch_task_table(const SearchArgs &A, uint32_t table_total, hipStream_t stream);
hipError_t launch_root_order(const SearchArgs &A, hipStream_t stream);
// leaf_values: profiled path accuracies with one value per leaf (needs A.swap, a leaf in the tiles, two or
// more leaves and at most kMaxPrefix branches above every leaf; see leaf_values_apply in loki_api.cpp)
hipError_t launch_combine(const SearchArgs &A, int slots, bool has_presum, bool divide, bool range,
                          bool leaf_values, hipStream_t stream);
// path_levels: 0, or with profiled path accuracies the number of tasks on the longest root-to-leaf chain
// (selects how many levels of the walk over the variant paths are compiled in)
hipError_t launch_path_combine(const SearchArgs &A, int slots, bool range, int path_levels, hipStream_t stream);
// latency_levels: 0, or for eq. (7) on the variant paths with traffic (DevProblem::lat_per_path must be set) the
// number of tasks on the longest root-to-leaf chain
hipError_t launch_per_lane_search(const SearchArgs &A, bool pv_batch, bool has_vf, int path_levels,
                                  int latency_levels, hipStream_t stream);
// Per-path latency rule on top of the tables (A.lat2 set): the plans the per-task bound rejects but whose variant
// paths with traffic all meet the budget; block records like the other search kernels.
hipError_t launch_open_plans(const SearchArgs &A, int slots, bool range, int latency_levels, hipStream_t stream);
// results[m] takes in other[m] (both loki_result_t arrays on the device)
hipError_t launch_fold_results(void *results, const void *other, int M, bool tie_index_only, hipStream_t stream);
hipError_t launch_final_reduce(const SearchArgs &A, hipStream_t stream);
hipError_t launch_results_init(const MergeArgs &A, hipStream_t stream);
hipError_t launch_class_merge(const MergeArgs &A, hipStream_t stream);
hipError_t launch_eval(const EvalArgs &A, hipStream_t stream);
hipError_t launch_route(const RouteArgs &A, hipStream_t stream);

}  // namespace loki

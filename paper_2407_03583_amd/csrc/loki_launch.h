// Launch wrappers implemented in loki_kernels.hip (one call = one kernel enqueued
// on the given stream; the return value is hipGetLastError() after the launch).
#pragma once

#include <hip/hip_runtime_api.h>

#include "loki_device.h"

namespace loki {

hipError_t launch_task_table(const SearchArgs &A, uint32_t table_total, hipStream_t stream);
hipError_t launch_root_order(const SearchArgs &A, hipStream_t stream);
hipError_t launch_combine(const SearchArgs &A, int slots, bool has_presum, bool divide, bool range,
                          hipStream_t stream);
hipError_t launch_per_lane_search(const SearchArgs &A, hipStream_t stream);
hipError_t launch_final_reduce(const SearchArgs &A, hipStream_t stream);
hipError_t launch_eval(const EvalArgs &A, hipStream_t stream);
hipError_t launch_route(const RouteArgs &A, hipStream_t stream);

}  // namespace loki

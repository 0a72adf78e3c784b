// Plain-data structures shared by the host side of the library and its
// gfx950 kernels.  Everything here is laid out for direct copies into device
// memory and LDS.
#pragma once

#include <stdint.h>

namespace loki {

constexpr int kMaxTasks = 8;
constexpr int kMaxVariants = 8;
constexpr int kMaxBatches = 8;
constexpr int kBlockThreads = 256;          // 4 wavefronts of 64
constexpr int kWavesPerBlock = kBlockThreads / 64;
constexpr int kMidTile = 512;               // most root-task choices staged in LDS per work item
constexpr int kStepMul = 0, kStepLeaf = 1, kStepPre = 2;
constexpr int32_t kNever = 0x7fffffff;      // latency marker: this choice can never be part of a feasible plan
constexpr int kMaxPrefix = 64;              // profiled path accuracies leaf by leaf: most branches of the walk over the
                                            // variant paths above a leaf (product of the variant counts of the tasks
                                            // root..leaf's parent)

// What the fill needs of the variant at one position of a task's route order, side by side (one 16-byte read).
struct RouteStep {
    int32_t k;      // the variant
    int32_t acc;    // its accuracy, ppm
    int32_t vf;     // its multiplicative factor, quarters (4 when absent)
    int32_t pad;
};

// Per-handle constants (Table 1 inputs after validation, plus derived radices).
struct DevProblem {
    int32_t n_tasks;
    int32_t n_paths;
    int32_t parent[kMaxTasks];
    int32_t is_leaf[kMaxTasks];
    int32_t path_len[kMaxTasks];            // number of tasks on the root..i chain
    int32_t K[kMaxTasks];
    int32_t nb[kMaxTasks];
    uint32_t C[kMaxTasks];                  // choices per task
    uint32_t radix[kMaxTasks][kMaxVariants];  // R(i,k)+1, or 1+R(i,k)*|B_i| with per-variant batch sizes
    uint32_t magic32[kMaxTasks][kMaxVariants];  // ceil(2^32 / radix): umulhi(c, magic32) = c / radix for c * radix < 2^32
    int32_t order[kMaxTasks][kMaxVariants];   // route order (accuracy descending, index ascending) -> variant
    int32_t acc[kMaxTasks][kMaxVariants];     // ppm, by variant
    uint32_t table_off[kMaxTasks];          // first record of task i in a per-demand task table
    uint32_t table_total;                   // sum of C_i
    int32_t n_lat0;                         // number of distinct profiled latencies of task 0
    int32_t sum_r0;                         // sum of the replica limits of task 0
    int32_t has_vf;                         // per-variant multiplicative factors are present
    int32_t pv_batch;                       // a batch size per hosted variant instead of one per task
    int32_t tile_task;                      // class-by-class searches with swapped roles: the leaf whose choices fill the tiles
    int32_t lat0_sorted[kMaxVariants * kMaxBatches];  // those latencies, ascending
    // How the path values that do not involve the last task are formed from the first task's accuracy:
    // a list of steps, each "multiply by the accuracy of task prog_task[q]" (kStepMul), "the value is a
    // leaf's path value: add it to the sum of the earlier leaves and start again from the first task's
    // accuracy" (kStepLeaf) or "the value is the product over the last task's ancestors" (kStepPre).
    // Leaves in ascending order, every chain root first: the operation order of eq. (12)'s objective.
    int32_t n_prog;
    int32_t pad2;
    int8_t prog_task[64];
    int8_t prog_op[64];
    int32_t fanout[kMaxTasks];              // quarters, edge parent[i] -> i
    int32_t vf[kMaxTasks][kMaxVariants];    // quarters, by variant (4 everywhere when absent)
    int32_t batch_size[kMaxTasks][kMaxBatches];
    int64_t scale[kMaxTasks];               // 4^depth, or 16^depth with per-variant factors
    uint64_t stride[kMaxTasks];             // prod_{j<i} C_j
    uint64_t magic[kMaxTasks][kMaxVariants];  // ceil(2^36 / radix): (c * magic) >> 36 = c / radix for c * radix <= 2^36
    uint64_t magic_nb[kMaxTasks];           // ceil(2^36 / |B_i|)
    int32_t lat[kMaxTasks][kMaxVariants][kMaxBatches];    // microseconds (at most 2^30)
    int64_t thr_s[kMaxTasks][kMaxVariants][kMaxBatches];  // throughput * 4^depth
    // profiled accuracies of the variant paths (only the kernels that stage the whole block use these)
    int32_t has_path;                       // a table per leaf is present
    uint32_t path_total;                    // entries over all leaves
    uint32_t path_off[kMaxTasks];           // first entry of leaf i's table
    int32_t leaf_path[kMaxTasks][kMaxTasks];  // tasks on the chain root..i, root first (path_len[i] of them)
    // the same ordering data as n_lat0 / sum_r0 / lat0_sorted for the task tile_task
    int32_t n_lat_t;
    int32_t sum_r_t;
    int32_t lat_t_sorted[kMaxVariants * kMaxBatches];
    int32_t lat_per_path;                   // eq. (7) on every variant path with traffic instead of the per-task bound
    int32_t pad3;
    RouteStep route[kMaxTasks][kMaxVariants];  // order / acc / vf again, by route position
};

// What a task contributes to any plan that uses one of its choices
// (depends on the task's own digits and its demand only).
struct TaskRec {
    double a;      // traffic-weighted accuracy of the task
    int32_t w;     // replicas used
    int32_t lat;   // largest latency among the variants in use; kNever if the
                   // choice leaves demand unserved or hosts nothing
};

// With eq. (7) taken on the variant paths with traffic: the latencies of the first and of the last variant in
// use of a choice (route order); kNever like TaskRec::lat.  Two variant paths always carry requests when all
// demand is served (the first variants in use of every task, and the last ones), so their sums bound the
// slowest path with traffic from below as TaskRec::lat's sums bound it from above.
struct TaskLat2 {
    int32_t top, bot;
};

// What the plans sharing one choice of every task but the last have in common,
// staged in LDS per work item and read as a broadcast.  MidVal feeds the
// objective; MidLim holds the limits left for the last task and is the same
// for every record of a run.
struct MidVal {
    double pre;       // product of the accuracies of the last task's ancestors, root first
    double presum;    // sum of the path values of all earlier leaves, in leaf order
};

struct MidLim {
    int32_t w_rem;    // workers left for the last task; -1 if the shared part is already infeasible
    int32_t tl;       // latency left for the last task on its path
    uint32_t cl_lo;   // first choice of the last task inside the index range; when the whole space is
                      // searched: end (exclusive, tile relative) of the run this entry belongs to
    uint32_t cl_cnt;  // number of its choices inside the index range
};

struct BestRec {
    double acc;
    uint64_t idx;
    uint64_t nfeas;
    int32_t w;
    int32_t found;
};

struct SearchArgs {
    const DevProblem *P;
    const int64_t *Dn;      // [M][kMaxTasks]
    TaskRec *table;         // [M][table_total]
    BestRec *recs;          // [M][blocks_per_m]
    uint32_t *perm;         // [M][C_0] first-task choices in run order
    uint32_t *run_end;      // [M][C_0] end (exclusive) of the run each position belongs to
    void *results;          // [M] loki_result_t
    unsigned long long *floor;  // [M] bit pattern of the largest key a block of the point has reported so far
    TaskLat2 *lat2;         // [M][table_total], or null: only written and read under the per-path latency rule
    const double *path_acc; // [path_total] profiled path accuracies as fractions, or null
    // Per-variant factors searched class by class: a "point" of the launch is a demand point together
    // with one value, per task that has children, of the requests the task creates per unit of fan-out
    // (that fixes every task's demand).  class_amount[point][i] is that value for task i (-1: any choice of
    // task i belongs to the point), class_count[point][i] the number of task i's choices that belong.
    const int64_t *class_amount;   // [M][kMaxTasks]; null: points are plain demand points
    const uint32_t *class_count;   // [M][kMaxTasks]
    // With swapped roles (swap != 0; two or more leaves, whole space) the tiles hold the choices of the
    // first leaf (DevProblem::tile_task) in the run order perm_all / run_end_t, and every other task but the
    // last is part of the work item: a task with children through the list of its choices that belong to
    // the point (perm_all lists them first), a leaf through all of its choices.
    uint32_t *perm_all;     // [M][table_total]: per task (at table_off) its choices, usable ones first
    uint32_t *run_end_t;    // [M][C_tile_task]
    uint32_t swap;
    uint32_t swap_tasks;    // number of tasks (the ordering kernel runs for every task but the last)
    int32_t w_free_t;       // like w_free, for the tile task
    int64_t budget[kMaxTasks];  // per task i: floor((slo - comm*path_len[i]) / 2), -1 if negative
    uint64_t begin, end;    // index range
    uint64_t far_count;     // F = prod of C_j over the tasks strictly between the first and the last
    // The part of the space an index range touches.  Tabulated kernel: far_span combinations of the tasks
    // in between, cyclically from far_first (0 and F for the whole space).  Per-lane kernel: far_span
    // combinations of all tasks but the last, cyclically from far_first.
    uint64_t far_first, far_span;
    uint64_t items;         // work items per demand point
    uint64_t items_per_block, items_extra;  // items / blocks_per_m and items % blocks_per_m (tabulated kernels, whole
                                            // launch; with swapped roles a point's own count is divided in the kernel)
    uint32_t cl_first;      // first choice of the last task touched by the range
    uint32_t chunk_groups;  // groups of chunks of the last task
    uint32_t tile_len;      // root-task choices per work item, at most kMidTile
    uint32_t mid_tiles;     // ceil(C_0 / tile_len)
    uint32_t cpb;           // chunks handled side by side in a block (1, 2 or 4)
    int32_t W;
    int32_t w_most_last;    // sum of the replica limits of the last task: no choice of it hosts more
    int32_t w_free;         // first-task replica counts up to this never make the worker budget bind (may be < 0)
    int32_t M;
    uint32_t blocks_per_m;
    uint32_t tie_index_only;
    uint32_t narrow;        // per-lane search: every demand and every x * q * scale of the call is below 2^32
    uint32_t prune;         // profiled path accuracies, tabulated: feasible plans whose upper bound is below the
                            // best objective seen are not walked (one task path, one factor per edge, at most
                            // kMaxPrefix variant combinations above the last task)
};

// Mirrors loki_route_t (include/loki_alloc.h).
struct RouteOut {
    int64_t demand[kMaxTasks];
    int64_t scale[kMaxTasks];
    int64_t unserved[kMaxTasks];
    int32_t replicas[kMaxTasks][kMaxVariants];
    int32_t batch[kMaxTasks][kMaxVariants];
    int64_t capacity[kMaxTasks][kMaxVariants];
    int64_t routed[kMaxTasks][kMaxVariants];
    int64_t leftover[kMaxTasks][kMaxVariants];
    int64_t budget_us[kMaxTasks][kMaxVariants];
    double prob[kMaxTasks][kMaxVariants][kMaxVariants];
};

struct RouteArgs {
    const DevProblem *P;
    const uint64_t *indices;
    const int64_t *demand;
    RouteOut *out;
    int64_t n;
};

// Merge of the per-class results into the results of the demand points they belong to.
struct MergeArgs {
    void *class_results;        // [n] loki_result_t, one per (demand point, class); folded in place
    const int32_t *point;       // [n] demand point of each
    void *results;              // [M] loki_result_t, updated in place
    int32_t n;
    int32_t M;                  // used by the initialising launch only
    uint32_t tie_index_only;
};

struct EvalArgs {
    const DevProblem *P;
    const uint64_t *indices;
    void *out;              // loki_eval_t
    const double *path_acc; // profiled path accuracies as fractions, or null
    int64_t n;
    int64_t Dn[kMaxTasks];
    int64_t budget[kMaxTasks];
    int32_t W;
};

}  // namespace loki

/*
 * loki_alloc -- exhaustive GPU search over resource-allocation plans for an
 * ML inference pipeline, after the allocation model of Loki (HPDC'24,
 * "A System for Serving ML Inference Pipelines with Hardware and Accuracy
 * Scaling"), Section 4.1 (constraints (1)-(7), objectives (11), (12)) and
 * Section 5.1 (Algorithm 1, MostAccurateFirst).
 *
 * The paper hands its constraints to an MILP solver; this library instead
 * enumerates a bounded plan space on one gfx950 GPU: per task i every model
 * variant k gets a replica count x(i,k) in 0..R(i,k) and the task gets one
 * batch size from its list.  Every plan in the requested index range receives
 * a feasibility verdict and, if feasible, its objective; the best plan under
 * a strict total order is returned, so the result does not depend on how the
 * work was split over lanes, waves or blocks.
 *
 * Scoring of one plan (all integer except the objective):
 *   demand   Dn_i = D * prod(fanout_q4 on the edges root..i), in units of
 *            milli-QPS / 4^depth_i                                (eq. (1), one factor per edge)
 *   workers  sum_i sum_k x(i,k) <= S                               (eq. (3))
 *   serving  variants of a task are filled most accurate first (ties: lower
 *            variant index); variant k takes min(remaining, x*q(i,k,b)*4^depth);
 *            the plan is infeasible if demand is left over or a task hosts
 *            nothing                                               (eq. (2), Algorithm 1's fill rule)
 *   latency  for every root-to-leaf path: sum over its tasks of the largest
 *            latency among the variants in use (a hosted variant is in use if
 *            it receives traffic, or if it is the first hosted one)
 *            <= floor((SLO - comm * tasks_on_path) / 2)            (eq. (6), (7), SLO halving,
 *                                                                   communication-latency paragraph)
 *   accuracy a_i = sum_k routed_k*acc_ppm_k / (Dn_i * 10^6) as one fp64
 *            division of two exactly converted integers (a_i = acc of the
 *            first hosted variant when Dn_i = 0); path value = product of a_i
 *            root first; objective = (sum of path values in ascending leaf
 *            order) / number_of_paths                              (Section 2.1 pipeline accuracy,
 *                                                                   eq. (12))
 *   order    higher accuracy, then fewer workers (eq. (11) as tie-break), then
 *            lower index; LOKI_TIE_INDEX_ONLY drops the workers level.
 * fp64 operations are individually rounded (no fused multiply-add), so the
 * objective is reproducible bit for bit.
 *
 * Candidate index (part of the contract):
 *   index    = sum_i choice_i * prod_{j<i} C_j            task 0 least significant
 *   choice_i = sum_k x(i,k) * prod_{k'<k} (R(i,k')+1) + beta_i * prod_k (R(i,k)+1)
 *   C_i      = n_batches_i * prod_k (R(i,k)+1),  beta_i = position in the task's batch list.
 * With per_variant_batch every variant carries its own batch position:
 *   choice_i = sum_k g(i,k) * prod_{k'<k} (1 + R(i,k')*n_batches_i),
 *   g(i,k)   = 0 if the variant is not hosted, else 1 + (x(i,k)-1)*n_batches_i + beta(i,k),
 *   C_i      = prod_k (1 + R(i,k)*n_batches_i).
 *
 * Memory: the caller owns every buffer.  "host" pointers are ordinary host
 * memory, "device" pointers are HIP device memory on the current device.  The
 * library allocates no device memory; all device scratch lives in the
 * caller's workspace.  A handle owns host memory only (including a small
 * pinned staging buffer).  Calls on one handle must not overlap in time.
 *
 * Errors: every function returns LOKI_OK (0) or a negative code; nothing is
 * written to outputs on error.  "No feasible plan" is not an error.
 */
#ifndef LOKI_ALLOC_H
#define LOKI_ALLOC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LOKI_MAX_TASKS 8
#define LOKI_MAX_VARIANTS 8
#define LOKI_MAX_BATCHES 8
#define LOKI_MAX_REPLICAS 255
#define LOKI_MAX_CHOICES (1u << 24) /* per task */
#define LOKI_MAX_DEMAND_POINTS 65535
#define LOKI_MAX_PATH_ENTRIES 32768 /* profiled path accuracies, all leaves together */

enum {
    LOKI_OK = 0,
    LOKI_E_NULL = -1,          /* a required pointer is null */
    LOKI_E_INVALID_GRAPH = -2, /* not a rooted tree in topological order (Section 2.1: trees only) */
    LOKI_E_RANGE = -3,         /* a value outside the documented range, or fixed-point overflow risk */
    LOKI_E_WORKSPACE = -4,     /* workspace too small or misaligned (needs 256-byte alignment) */
    LOKI_E_HIP = -5,           /* a HIP runtime call failed; loki_last_hip_error() has the code */
    LOKI_E_ARG = -6,           /* inconsistent scalar arguments (empty range reversed, bad flags, ...) */
    LOKI_E_STATIC_LIMIT = -7   /* loki_alloc_search_static: the search needs more than LOKI_STATIC_SCRATCH_BYTES
                                  of device scratch, or has more than LOKI_STATIC_MAX_DEMAND_POINTS demand points */
};

/* flags of loki_alloc_search */
#define LOKI_TIE_WORKERS_THEN_INDEX 0u /* default order: accuracy, workers, index */
#define LOKI_TIE_INDEX_ONLY 1u         /* order: accuracy, index */
#define LOKI_SEARCH_PER_LANE 2u        /* evaluate each plan from scratch in its lane (no per-task tables) */

/* result status */
#define LOKI_FOUND 0
#define LOKI_NO_FEASIBLE 1

/* why a plan is infeasible (loki_eval_t.infeasible) */
#define LOKI_BAD_WORKERS 1u /* eq. (3) */
#define LOKI_BAD_DEMAND 2u  /* eq. (2): demand left unserved at some task */
#define LOKI_BAD_EMPTY 4u   /* a task hosts no variant */
#define LOKI_BAD_LATENCY 8u /* eq. (7) on some path */

/* The inputs of Section 4.1 ("Inputs", Table 1): tree T/E, variants V_i, batch
 * sizes B, multiplicative factors (per edge), throughput q, accuracy A.
 * Host memory, read during loki_problem_create only. */
typedef struct {
    int32_t n_tasks;             /* 1..LOKI_MAX_TASKS; task 0 is the root */
    const int32_t *parent;       /* [n] parent[0] = -1, 0 <= parent[i] < i */
    const int32_t *fanout_q4;    /* [n] requests created at task i per request at parent[i], in quarters
                                    (4 = 1.00), 1..4096; [0] ignored */
    const int32_t *n_variants;   /* [n] K_i in 1..LOKI_MAX_VARIANTS */
    const int32_t *n_batches;    /* [n] |B_i| in 1..LOKI_MAX_BATCHES */
    const int32_t *batch_size;   /* concatenated over tasks; positive, strictly increasing within a task */
    const int32_t *max_replicas; /* concatenated over (task, variant): R(i,k) in 0..LOKI_MAX_REPLICAS;
                                    0 removes the variant (eq. (10) of the hardware-scaling step) */
    const int32_t *acc_ppm;      /* concatenated over (task, variant): A(v_ik) in 0..1000000 */
    const int64_t *latency_us;   /* concatenated over (task, variant, batch): 1..2^30 */
    const int64_t *thr_mqps;     /* concatenated over (task, variant, batch): per-replica throughput, 0..2^40 */
    const int32_t *variant_factor_q4; /* NULL, or concatenated over (task, variant): the multiplicative factor
                                    r(i,k) of eq. (1) in quarters, 1..64.  With it the requests task i creates
                                    for a child j are sum_k routed(i,k) * r(i,k) * fanout_q4[j] (Section 5.1:
                                    outgoing = incoming * multFactor * branchRatio), a child's demand depends
                                    on its parent's part of the plan and tasks work in units of milli-QPS /
                                    16^depth.  A task's demand then depends on its ancestors' choices only
                                    through the amounts of requests they create, which take few distinct
                                    values: a search runs the tabulated kernels once per combination of such
                                    amounts, the host settling the choices that cannot serve their demand
                                    (same results).  Demand points with more than 65,535 such combinations
                                    score whole plans per lane (LOKI_SEARCH_PER_LANE). */
    int32_t per_variant_batch;   /* 0: one batch size per task.  1: a batch size per hosted variant, the y(i,k)
                                    of Section 4.1 "Output" and eq. (4); see the index layout above */
    const int32_t *path_acc_ppm; /* NULL, or the profiled end-to-end accuracy A-hat(p) of every variant path
                                    (Section 4.1 "Accuracy"), 0..1000000: concatenated over the leaves in
                                    ascending task index; a leaf's table has one entry per combination of
                                    variants of the tasks root..leaf, entry = sum_j k_j * prod_{j'<j} K_j'
                                    with the root's variant least significant; at most LOKI_MAX_PATH_ENTRIES
                                    entries in total.  The objective of a feasible plan is then the mean over
                                    the root-to-leaf task paths of sum_p c(p) * A-hat(p), where c(p) is the
                                    frontend's split over the root's variants times, per edge, the probability
                                    with which the upstream variant's routing table (Algorithm 1, what
                                    loki_route_table returns in prob) picks the downstream variant; a variant
                                    without traffic hands on to the first hosted downstream variant in route
                                    order.  fp64 order: c(p) multiplied up root first, times A-hat(p)/10^6,
                                    terms added with the root's variants outermost and every level in route
                                    order, task paths added in leaf order, one division by their number.
                                    The objective couples the tasks through c(p), feasibility does not: a
                                    search takes feasibility from the per-task tables and walks the variant
                                    paths for feasible plans only; on a tree with two or more leaves (at most
                                    64 variant combinations above every leaf) it forms each leaf's sum once
                                    for all the plans that share the choices along that leaf's path (whole
                                    plans per lane with LOKI_SEARCH_PER_LANE; same results). */
    int32_t latency_per_path;    /* How eq. (7) is applied (Section 4.1 "Latency", eq. (6), (7), Table 1's I(p)).
                                    0: per root-to-leaf task path, the sum over its tasks of the largest latency
                                    among the task's variants in use must meet the halved SLO.  That sum bounds
                                    the latency of every variant path from above, and is attained by a path
                                    with traffic wherever a task's latency grows with its accuracy (Algorithm 1
                                    pairs the most accurate variants in use of consecutive tasks); it lets
                                    feasibility be tabulated per task.
                                    1: eq. (7) as stated: every variant path that carries requests under
                                    Algorithm 1's routing (the frontend reaches the root's variant, and each
                                    variant's routing table gives the next one a nonzero probability) must meet
                                    it, at each variant's configured batch size; variant paths without traffic
                                    limit nothing.  At zero demand the first hosted variants stand for the plan.
                                    LOKI_BAD_LATENCY is then reported only for plans that host every task and
                                    serve all demand (the routing of the others is not defined).  A plan that
                                    is feasible under 0 is feasible under 1.  A search under this rule takes
                                    the plans that 0 admits from the per-task tables as ever, and picks out, in
                                    a second pass over the plan space, the plans 0 rejects whose two variant
                                    paths that always carry requests (the first and the last variants in use of
                                    every task) meet the budget: only those walk their variant paths.  With
                                    per-variant factors or profiled path accuracies as well, whole plans are
                                    scored per lane (LOKI_SEARCH_PER_LANE is implied), with the same two bounds
                                    deciding most plans. */
} loki_pipeline_t;

typedef struct loki_problem loki_problem_t; /* opaque handle */

typedef struct { /* 32 bytes */
    uint64_t index;       /* best plan; UINT64_MAX if none */
    double accuracy;      /* its objective; 0.0 if none */
    uint64_t n_feasible;  /* feasible plans in the searched range */
    int32_t workers_used; /* sum of x of the best plan; -1 if none */
    int32_t status;       /* LOKI_FOUND or LOKI_NO_FEASIBLE */
} loki_result_t;

typedef struct { /* 16 bytes */
    double accuracy;     /* objective if infeasible == 0, else 0.0 */
    int32_t workers;     /* sum of x */
    uint32_t infeasible; /* OR of LOKI_BAD_* */
} loki_eval_t;

/* Routing for one plan (Algorithm 1 with the replicas of a variant lumped into
 * one entry; Section 5.1) plus what Section 4.2 derives from the plan: the
 * per-task latency budgets and the leftover-capacity (backup) table.
 * Traffic quantities of task i are in units of milli-QPS / scale[i]. */
typedef struct {
    int64_t demand[LOKI_MAX_TASKS];                     /* Dn_i */
    int64_t scale[LOKI_MAX_TASKS];                      /* 4^depth_i */
    int64_t unserved[LOKI_MAX_TASKS];                   /* demand that found no capacity (0 when feasible) */
    int32_t replicas[LOKI_MAX_TASKS][LOKI_MAX_VARIANTS];  /* x(i,k) */
    int32_t batch[LOKI_MAX_TASKS][LOKI_MAX_VARIANTS];     /* configured batch size; 0 if not hosted */
    int64_t capacity[LOKI_MAX_TASKS][LOKI_MAX_VARIANTS];  /* x * q * scale */
    int64_t routed[LOKI_MAX_TASKS][LOKI_MAX_VARIANTS];    /* traffic placed on the variant */
    int64_t leftover[LOKI_MAX_TASKS][LOKI_MAX_VARIANTS];  /* capacity - routed */
    int64_t budget_us[LOKI_MAX_TASKS][LOKI_MAX_VARIANTS]; /* latency at the configured batch; 0 if not hosted */
    /* prob[j][k][k'] = share of the requests variant k of parent[j] creates for task j that go to
     * variant k' of task j; for the root, prob[0][0][k'] is the frontend's split. */
    double prob[LOKI_MAX_TASKS][LOKI_MAX_VARIANTS][LOKI_MAX_VARIANTS];
} loki_route_t;

/* Validate the inputs (tree shape, ranges, and that no fixed-point intermediate
 * can reach 2^53 / overflow int64 for demands up to LOKI limits checked again
 * per call), copy them, precompute radices, route order and paths.
 * Touches no GPU: the pinned staging buffer and the events of a handle are
 * created by its first search or evaluation.
 * Errors: LOKI_E_NULL, LOKI_E_INVALID_GRAPH, LOKI_E_RANGE (also when the number
 * of candidates reaches 2^63). */
int loki_problem_create(const loki_pipeline_t *pipeline, loki_problem_t **out);
void loki_problem_destroy(loki_problem_t *problem);

/* N = prod_i C_i. */
int loki_num_candidates(const loki_problem_t *problem, uint64_t *n);

/* Bytes of device workspace loki_alloc_search / loki_alloc_eval need for up to
 * n_demand demand points (or n_demand indices for loki_alloc_eval). */
int loki_workspace_bytes(const loki_problem_t *problem, int64_t n_demand, size_t *bytes);

/* index -> plan.  x: [sum_i K_i] replica counts in input order; batch: [n] batch
 * sizes (values, not positions), or with per_variant_batch [sum_i K_i] batch sizes
 * (0 where the variant is not hosted).  Host arrays.  LOKI_E_RANGE if index >= N. */
int loki_decode(const loki_problem_t *problem, uint64_t index, int32_t *x, int32_t *batch);

/* The search (accuracy-scaling step, eq. (12), with the hardware-scaling
 * objective eq. (11) as tie-break; the pure hardware-scaling step is the same
 * call on a pipeline whose less accurate variants have max_replicas = 0).
 *   demand_mqps  host, [n_demand] root demand D per demand point, milli-QPS, >= 0
 *   workers      S >= 0;  slo_us  L >= 0;  comm_us >= 0 per task on a path
 *   flags        LOKI_TIE_* | LOKI_SEARCH_PER_LANE
 *   [index_begin, index_end) subset of [0, N); pass 0, N for everything
 *   d_workspace  device, 256-byte aligned, >= loki_workspace_bytes(n_demand)
 *   hip_stream   a hipStream_t (NULL = default stream); all work is enqueued on it
 *   out          host, [n_demand]; valid on return (the call waits for the stream)
 * Errors: LOKI_E_NULL, LOKI_E_ARG, LOKI_E_RANGE (a demand for which an
 * intermediate could overflow), LOKI_E_WORKSPACE, LOKI_E_HIP. */
int loki_alloc_search(loki_problem_t *problem, const int64_t *demand_mqps, int32_t n_demand,
                      int32_t workers, int64_t slo_us, int64_t comm_us, uint32_t flags,
                      uint64_t index_begin, uint64_t index_end,
                      void *d_workspace, size_t workspace_bytes, void *hip_stream,
                      loki_result_t *out);

/* Same, but only enqueues: results are left in device memory at d_results
 * ([n_demand] loki_result_t, device, 8-byte aligned) when the stream reaches
 * that point; nothing is copied back and the call does not wait for the GPU
 * (it may wait for the staging copy of the previous call on this handle, and a
 * search with per-variant factors whose demand points are taken in groups waits
 * for every group's descriptors but the last to be copied). */
int loki_alloc_search_enqueue(loki_problem_t *problem, const int64_t *demand_mqps, int32_t n_demand,
                              int32_t workers, int64_t slo_us, int64_t comm_us, uint32_t flags,
                              uint64_t index_begin, uint64_t index_end,
                              void *d_workspace, size_t workspace_bytes, void *hip_stream,
                              void *d_results);

/* loki_alloc_search for callers that cannot allocate device memory or must not cause an allocation: code
 * running around a HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  There is no
 * workspace argument: the device scratch of the search is a file-scope device array of
 * LOKI_STATIC_SCRATCH_BYTES inside the library (one copy per GPU, held until the process ends), and the
 * call itself allocates nothing -- no device or pinned memory, no events; the handle's host staging is
 * ordinary memory owned since loki_problem_create.  The caller still passes the inputs and the output
 * array.  Results are those of loki_alloc_search bit for bit.
 *   demand_mqps  host, [n_demand], n_demand <= LOKI_STATIC_MAX_DEMAND_POINTS
 *   out          host, [n_demand]; valid on return (the call waits for the stream)
 * All searches of all handles on one GPU share that GPU's array: calls that overlap in time on one GPU
 * (other threads, other streams) race and must be serialised by the caller.  The array keeps the previous
 * call's contents; a search overwrites every part it reads, nothing has to be cleared.
 * A search never runs class by class here (that needs a large workspace and pinned descriptors):
 * per-variant factors score whole plans per lane and profiled path accuracies walk the variant paths of
 * feasible plans, as with LOKI_SEARCH_PER_LANE or on chains.
 * Errors: as loki_alloc_search, and LOKI_E_STATIC_LIMIT when the search of this problem with n_demand
 * demand points needs more scratch than the array holds (4 MiB cover one demand point of about 180,000
 * choices summed over the tasks) or n_demand exceeds LOKI_STATIC_MAX_DEMAND_POINTS; nothing is launched then. */
#define LOKI_STATIC_SCRATCH_BYTES (4u << 20)
#define LOKI_STATIC_MAX_DEMAND_POINTS 64
int loki_alloc_search_static(loki_problem_t *problem, const int64_t *demand_mqps, int32_t n_demand,
                             int32_t workers, int64_t slo_us, int64_t comm_us, uint32_t flags,
                             uint64_t index_begin, uint64_t index_end, void *hip_stream,
                             loki_result_t *out);

/* Evaluate listed plans one by one (each lane scores one plan from scratch).
 *   indices  host, [n_indices], each < N;  out host, [n_indices]. */
int loki_alloc_eval(loki_problem_t *problem, const uint64_t *indices, int64_t n_indices,
                    int64_t demand_mqps, int32_t workers, int64_t slo_us, int64_t comm_us,
                    void *d_workspace, size_t workspace_bytes, void *hip_stream,
                    loki_eval_t *out);

/* Routing, latency budgets and backup table for one plan (host computation,
 * microseconds of work; Algorithm 1).  out: host. */
int loki_route_table(const loki_problem_t *problem, uint64_t index, int64_t demand_mqps,
                     loki_route_t *out);

/* The same for many plans at once, on the GPU: plan indices[j] under root demand
 * demand_mqps[j], one lane per plan -- typically the winners of a demand sweep, so
 * that the routing tables of every demand point come back with one call.
 *   indices, demand_mqps  host, [n];  out  host, [n]
 *   d_workspace  device, 256-byte aligned, >= loki_route_workspace_bytes(n) */
int loki_route_workspace_bytes(const loki_problem_t *problem, int64_t n, size_t *bytes);
int loki_route_table_batch(loki_problem_t *problem, const uint64_t *indices, const int64_t *demand_mqps,
                           int64_t n, void *d_workspace, size_t workspace_bytes, void *hip_stream,
                           loki_route_t *out);

/* The Resource Manager's periodic loop over a demand history (Section 4.2, "Solving the MILP"):
 * the demand to serve is an exponentially weighted moving average of the recent demand,
 *   est_0 = trace_0,  est_t = floor((alpha_ppm * trace_t + (10^6 - alpha_ppm) * est_{t-1}) / 10^6),
 * and every estimate gets its allocation from one batched search.  phase tells which of the two
 * steps of Section 4 produced the plan: LOKI_PHASE_HARDWARE if the best accuracy is not below the
 * one of the most accurate variants (the plan is then the minimum-worker plan, eq. (11); with
 * profiled path accuracies another combination of variants may score above it),
 * LOKI_PHASE_ACCURACY if accuracy had to be given up (eq. (12)), LOKI_PHASE_OVERLOAD if no plan
 * serves the estimate.
 *   trace_mqps  host, [n], >= 0;  alpha_ppm in 1..10^6;  out  host, [n]
 *   d_workspace as for loki_alloc_search with n demand points. */
#define LOKI_PHASE_HARDWARE 0
#define LOKI_PHASE_ACCURACY 1
#define LOKI_PHASE_OVERLOAD 2
typedef struct { /* 48 bytes */
    int64_t estimate_mqps;
    loki_result_t plan;
    int32_t phase;
    int32_t pad;
} loki_plan_step_t;
int loki_plan_trace(loki_problem_t *problem, const int64_t *trace_mqps, int32_t n, int32_t alpha_ppm,
                    int32_t workers, int64_t slo_us, int64_t comm_us, uint32_t flags,
                    void *d_workspace, size_t workspace_bytes, void *hip_stream, loki_plan_step_t *out);

/* GPU time of the most recent loki_alloc_search on this handle, from HIP events
 * on the caller's stream: ms[0] per-task tables (0 for LOKI_SEARCH_PER_LANE),
 * ms[1] the kernel that visits every plan, ms[2] the final merge.  ms: host, [3].
 * LOKI_E_ARG if no blocking search has completed yet. */
int loki_last_search_ms(const loki_problem_t *problem, float *ms);

/* Number of plans whose score the kernels of the most recent search on this handle (blocking or
 * enqueued) formed, for callers that relate kernel time to work done.  The index range times the
 * number of demand points, except where per-variant factors are searched once per combination of
 * created amounts (see variant_factor_q4): plans with a choice that cannot serve its demand at a
 * task that has children are settled on the host per choice (they still count as infeasible in the
 * results), and the figure is the number of plans of the remaining choices; for an index range
 * shorter than the space it is then an upper estimate.  LOKI_E_ARG before the first search. */
int loki_last_search_plans_scored(const loki_problem_t *problem, uint64_t *plans);

/* Width, in bits, of the integer arithmetic with which the most recent search of this handle that scored
 * whole plans per lane (LOKI_SEARCH_PER_LANE, or a search the library took that way) filled the variants
 * (eq. (2), Algorithm 1's fill rule): 32 when every R(i,k) * q * scale of the problem and every task's demand
 * at every demand point of the call are below 2^32 (and the objective is the product form under the default
 * latency rule), else 64.  The results are the same either way; the figure is for tests and measurements.
 * LOKI_E_ARG before the first such search. */
int loki_last_search_fill_bits(const loki_problem_t *problem, int32_t *bits);

const char *loki_strerror(int code);
int loki_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif

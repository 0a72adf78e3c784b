/*
 * CPU checker for the exhaustive allocation search.  TEST INFRASTRUCTURE ONLY:
 * it exists so that tests, the smoke check and the benchmark's CPU-baseline
 * leg have something independent to compare the GPU library with.  Nothing in
 * the product path may include, link or call it, and it shares no code,
 * header or table with the GPU library.
 *
 * What it computes (Loki, HPDC'24, Section 4.1 and Algorithm 1):
 *   a candidate allocation plan gives, per task i, a replica count x(i,k) for
 *   every model variant k and one batch size for the task.  It is scored by
 *   - per-task demand: root demand D times the fan-out of every edge on the
 *     way to the task (eq. (1), per-edge factors); with per-variant factors
 *     r(i,k) the requests a task creates are the sum over its variants of the
 *     traffic placed on the variant times its factor (eq. (1) as printed,
 *     Algorithm 1's outgoing = incoming * multFactor * branchRatio), so a
 *     child's demand depends on the parent's part of the plan,
 *   - the worker budget  sum x(i,k) <= S  (eq. (3)),
 *   - serving all of each task's demand within the hosted capacity
 *     x(i,k) * q(i,k,b) (eq. (2)), traffic placed most-accurate-variant-first
 *     (Algorithm 1's fill rule),
 *   - every root-to-leaf path's processing latency within half of the SLO
 *     after the per-hop communication latency is deducted (eq. (6), (7),
 *     the SLO halving and the communication-latency paragraph of Section 4.2);
 *     per task path the sum of the largest in-use latency of every task, or
 *     with latency_per_path eq. (7) itself: the latency of every variant path
 *     that carries traffic under Algorithm 1's routing,
 *   - pipeline accuracy = mean over root-to-leaf paths of the product of the
 *     tasks' traffic-weighted accuracies (Section 2.1's pipeline accuracy,
 *     eq. (12) objective); or, when profiled end-to-end accuracies of the
 *     variant paths are given (A-hat(p) of Section 4.1 "Accuracy"), the mean
 *     over root-to-leaf task paths of  sum_p c(p) * A-hat(p), where p runs
 *     over the combinations of one variant per task of the path and c(p) is
 *     the share of requests taking it: the frontend's split over the root's
 *     variants times, per edge, the probability with which Algorithm 1's
 *     routing table of the upstream variant picks the downstream variant.
 *   The search is the plain definition: evaluate every index, keep the best
 *   under (accuracy descending, workers ascending, index ascending), which is
 *   eq. (12) followed by eq. (11) as a tie-break.
 *
 * Fixed point: demand and throughput in milli-QPS, fan-out in quarters
 * (a task at depth d works in units of milli-QPS / 4^d so that everything
 * stays integral), latency in microseconds, accuracy in ppm.  The objective
 * is fp64, one correctly rounded operation at a time, no FMA contraction.
 *
 * Pins: tests/test_oracle_*.py (hand-derived worked example, closed forms,
 * exact-rational brute force, invariants, and an LP / MILP solver on the
 * paper's own formulation where the two must agree: product tables, task paths
 * of two tasks, latency not binding; with latency_per_path the feasible set
 * against the formulation's own eq. (7) for the routing Algorithm 1 produces).
 * Unpinned: the paper's MILP optimum with unbounded replica counts, and the
 * optimum over solver-chosen path ratios on longer paths or with a binding
 * latency limit, which can beat hop-by-hop routing.
 */
#ifndef LOKI_ORACLE_H
#define LOKI_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LO_MAX_TASKS 8
#define LO_MAX_VARIANTS 8

/* infeasibility bits */
#define LO_BAD_WORKERS 1 /* eq. (3) violated */
#define LO_BAD_DEMAND 2  /* eq. (2): some task cannot serve all of its demand */
#define LO_BAD_EMPTY 4   /* some task hosts no variant at all */
#define LO_BAD_LATENCY 8 /* eq. (7) violated on some root-to-leaf path */

typedef struct {
    int32_t n_tasks;
    const int32_t *parent;       /* [n] parent[0] = -1 */
    const int32_t *fanout_q4;    /* [n] quarters; [0] ignored */
    const int32_t *n_variants;   /* [n] */
    const int32_t *n_batches;    /* [n] */
    const int32_t *batch_size;   /* concat over tasks */
    const int32_t *max_replicas; /* concat over (task, variant) */
    const int32_t *acc_ppm;      /* concat over (task, variant) */
    const int64_t *latency_us;   /* concat over (task, variant, batch) */
    const int64_t *thr_mqps;     /* concat over (task, variant, batch) */
    const int32_t *variant_factor_q4; /* NULL, or concat over (task, variant): multiplicative factor r(i,k)
                                         of eq. (1) in quarters; requests created for a child =
                                         sum_k routed_k * r(i,k) * fanout(child) (Section 5.1) */
    int32_t per_variant_batch;   /* 0: one batch size per task.  1: y(i,k) of Section 4.1, a batch size per
                                    hosted variant; a variant's digit is 0 (not hosted) or
                                    1 + (replicas - 1) * |B_i| + batch position */
    const int32_t *path_acc_ppm; /* NULL, or A-hat(p) in ppm: concat over the leaves in ascending task index;
                                    a leaf's table has one entry per combination of variants of the tasks
                                    root..leaf, entry = sum_j k_j * prod_{j'<j} K_j' (root least significant) */
    int32_t latency_per_path;    /* 0: a task path's latency is the sum over its tasks of the largest latency
                                    among the variants in use (an upper bound on what eq. (7) limits).
                                    1: eq. (7) as printed: every variant path p with traffic (I(p) = 1 in
                                    Table 1, i.e. every hop of p carries requests under Algorithm 1's routing)
                                    has sum_{(i,k) in p} l(i,k) within the budget.  The latency bit is then
                                    taken only for plans that serve all demand at every task (the routing of
                                    a plan that does not is not the one the plan would run with). */
} lo_pipeline;

typedef struct {
    int32_t infeasible; /* OR of LO_BAD_*; 0 = feasible */
    int32_t workers;    /* sum of x(i,k) */
    double accuracy;    /* objective; 0.0 unless feasible */
    double task_acc[LO_MAX_TASKS];     /* traffic-weighted accuracy per task (feasible only) */
    int64_t task_maxlat[LO_MAX_TASKS]; /* max latency over the variants in use */
    int64_t task_demand[LO_MAX_TASKS]; /* scaled demand Dn_i */
    int64_t task_unserved[LO_MAX_TASKS];
} lo_eval_t;

typedef struct {
    uint64_t index;      /* winner; UINT64_MAX when none */
    double accuracy;     /* 0.0 when none */
    uint64_t n_feasible; /* feasible candidates in the searched range */
    int32_t workers;     /* -1 when none */
    int32_t found;       /* 1 / 0 */
} lo_best_t;

/* Routing for one plan: Algorithm 1 with the replicas of a variant lumped
 * into one entry.  Arrays are indexed [task][variant] / [task][parent variant][variant]. */
typedef struct {
    int64_t demand[LO_MAX_TASKS];                       /* Dn_i (scaled units) */
    int64_t scale[LO_MAX_TASKS];                        /* 4^depth */
    int64_t capacity[LO_MAX_TASKS][LO_MAX_VARIANTS];    /* x*q*scale */
    int64_t routed[LO_MAX_TASKS][LO_MAX_VARIANTS];      /* incoming traffic placed on the variant */
    int64_t leftover[LO_MAX_TASKS][LO_MAX_VARIANTS];    /* capacity - routed (backup table) */
    int64_t unserved[LO_MAX_TASKS];                     /* demand that found no capacity */
    int64_t budget_us[LO_MAX_TASKS][LO_MAX_VARIANTS];   /* latency at the configured batch, 0 if not hosted */
    double prob[LO_MAX_TASKS][LO_MAX_VARIANTS][LO_MAX_VARIANTS]; /* [child task][parent variant][child variant];
                                                                    for the root: [0][0][k] = frontend split */
} lo_route_t;

uint64_t lo_num_candidates(const lo_pipeline *p);
/* batch_digit: [n] batch positions (one per task), or with per_variant_batch [sum K_i] (0 where not hosted). */
void lo_decode(const lo_pipeline *p, uint64_t index, int32_t *x /* sum K_i */, int32_t *batch_digit);
uint64_t lo_encode(const lo_pipeline *p, const int32_t *x, const int32_t *batch_digit);

void lo_eval(const lo_pipeline *p, uint64_t index, int64_t demand_mqps, int32_t workers,
             int64_t slo_us, int64_t comm_us, lo_eval_t *out);

/* tie_index_only: 0 = (accuracy desc, workers asc, index asc); 1 = (accuracy desc, index asc). */
void lo_search(const lo_pipeline *p, int64_t demand_mqps, int32_t workers, int64_t slo_us,
               int64_t comm_us, int tie_index_only, uint64_t index_begin, uint64_t index_end,
               uint64_t index_stride, int n_threads, lo_best_t *out);

/* Same search with each task's per-choice result tabulated once and looked up
 * while walking the indices in order: the same two functions lo_eval calls
 * (task part, then pipeline part), composed through a table.  Only without
 * per-variant factors (with them a task's demand is not fixed); falls back to
 * lo_search otherwise. */
void lo_search_tabulated(const lo_pipeline *p, int64_t demand_mqps, int32_t workers, int64_t slo_us,
                         int64_t comm_us, int tie_index_only, uint64_t index_begin,
                         uint64_t index_end, int n_threads, lo_best_t *out);

void lo_route_table(const lo_pipeline *p, uint64_t index, int64_t demand_mqps, lo_route_t *out);

int lo_max_threads(void);

#ifdef __cplusplus
}
#endif
#endif

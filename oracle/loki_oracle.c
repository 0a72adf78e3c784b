/*
 * CPU checker for the exhaustive allocation search (see loki_oracle.h).
 * TEST INFRASTRUCTURE ONLY; deliberately plain and slow.
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC
 */
#include "loki_oracle.h"

#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- flat-array addressing ------------------------------------------------ */

typedef struct {
    int n;
    int voff[LO_MAX_TASKS];    /* first (task,variant) slot of task i */
    int boff[LO_MAX_TASKS];    /* first batch-size slot of task i */
    int toff[LO_MAX_TASKS];    /* first (task,variant,batch) slot of task i */
    uint64_t choices[LO_MAX_TASKS]; /* C_i = |B_i| * prod_k (R_ik + 1) */
} lo_layout;

static void layout_of(const lo_pipeline *p, lo_layout *L)
{
    int v = 0, b = 0, t = 0;
    L->n = p->n_tasks;
    for (int i = 0; i < p->n_tasks; i++) {
        L->voff[i] = v;
        L->boff[i] = b;
        L->toff[i] = t;
        uint64_t c = p->per_variant_batch ? 1 : (uint64_t)p->n_batches[i];
        for (int k = 0; k < p->n_variants[i]; k++)
            c *= p->per_variant_batch ? (uint64_t)(1 + p->max_replicas[v + k] * p->n_batches[i])
                                      : (uint64_t)(p->max_replicas[v + k] + 1);
        L->choices[i] = c;
        v += p->n_variants[i];
        b += p->n_batches[i];
        t += p->n_variants[i] * p->n_batches[i];
    }
}

uint64_t lo_num_candidates(const lo_pipeline *p)
{
    lo_layout L;
    layout_of(p, &L);
    uint64_t n = 1;
    for (int i = 0; i < L.n; i++)
        n *= L.choices[i];
    return n;
}

/* ---- candidate index <-> plan (the x(i,k), y(i) of Section 4.1 "Output") ---
 * index = sum_i choice_i * prod_{j<i} C_j            (task 0 least significant)
 * choice_i = sum_k x_ik * prod_{k'<k} (R_ik'+1) + beta_i * prod_k (R_ik+1)
 */
static void decode_choice(const lo_pipeline *p, const lo_layout *L, int i, uint64_t choice,
                          int32_t *x /* K_i */, int32_t *beta /* K_i: batch position per variant */)
{
    int K = p->n_variants[i], nb = p->n_batches[i];
    if (p->per_variant_batch) {
        for (int k = 0; k < K; k++) {
            uint64_t radix = (uint64_t)(1 + p->max_replicas[L->voff[i] + k] * nb);
            uint64_t g = choice % radix;
            choice /= radix;
            x[k] = g == 0 ? 0 : (int32_t)((g - 1) / (uint64_t)nb) + 1;
            beta[k] = g == 0 ? 0 : (int32_t)((g - 1) % (uint64_t)nb);
        }
        return;
    }
    for (int k = 0; k < K; k++) {
        uint64_t radix = (uint64_t)(p->max_replicas[L->voff[i] + k] + 1);
        x[k] = (int32_t)(choice % radix);
        choice /= radix;
    }
    for (int k = 0; k < K; k++)
        beta[k] = (int32_t)choice;
}

void lo_decode(const lo_pipeline *p, uint64_t index, int32_t *x, int32_t *batch_digit)
{
    lo_layout L;
    layout_of(p, &L);
    for (int i = 0; i < L.n; i++) {
        int32_t beta[LO_MAX_VARIANTS];
        uint64_t choice = index % L.choices[i];
        index /= L.choices[i];
        decode_choice(p, &L, i, choice, x + L.voff[i], beta);
        if (p->per_variant_batch)
            for (int k = 0; k < p->n_variants[i]; k++)
                batch_digit[L.voff[i] + k] = beta[k];
        else
            batch_digit[i] = beta[0];
    }
}

uint64_t lo_encode(const lo_pipeline *p, const int32_t *x, const int32_t *batch_digit)
{
    lo_layout L;
    layout_of(p, &L);
    uint64_t index = 0, stride = 1;
    for (int i = 0; i < L.n; i++) {
        uint64_t choice = 0, r = 1;
        int nb = p->n_batches[i];
        for (int k = 0; k < p->n_variants[i]; k++) {
            int xk = x[L.voff[i] + k];
            if (p->per_variant_batch) {
                uint64_t g = xk == 0 ? 0 : (uint64_t)(1 + (xk - 1) * nb + batch_digit[L.voff[i] + k]);
                choice += g * r;
                r *= (uint64_t)(1 + p->max_replicas[L.voff[i] + k] * nb);
            } else {
                choice += (uint64_t)xk * r;
                r *= (uint64_t)(p->max_replicas[L.voff[i] + k] + 1);
            }
        }
        if (!p->per_variant_batch)
            choice += (uint64_t)batch_digit[i] * r;
        index += choice * stride;
        stride *= L.choices[i];
    }
    return index;
}

/* ---- demand at each task (eq. (1)) ---------------------------------------------
 * Per-edge model: Dn_i = D * prod of fan-out quarters on the edges root -> i; the task
 * works in units of milli-QPS / 4^depth_i, so Dn_i / scale_i is its demand in milli-QPS.
 * With per-variant factors a level multiplies by two quarter-valued numbers, the units
 * are milli-QPS / 16^depth_i, and Dn_i follows from the parent's routing (see lo_eval). */
static void task_scale(const lo_pipeline *p, int64_t *scale)
{
    int64_t per_level = p->variant_factor_q4 ? 16 : 4;
    scale[0] = 1;
    for (int i = 1; i < p->n_tasks; i++)
        scale[i] = scale[p->parent[i]] * per_level;
}

static void task_demand(const lo_pipeline *p, int64_t demand_mqps, int64_t *Dn, int64_t *scale)
{
    task_scale(p, scale);
    Dn[0] = demand_mqps;
    for (int i = 1; i < p->n_tasks; i++)
        Dn[i] = Dn[p->parent[i]] * (int64_t)p->fanout_q4[i];
}

/* ---- route order: accuracy descending, variant index ascending ------------- */
static void route_order(const lo_pipeline *p, const lo_layout *L, int i, int *order)
{
    int K = p->n_variants[i];
    for (int k = 0; k < K; k++)
        order[k] = k;
    for (int a = 1; a < K; a++) { /* insertion sort, stable */
        int v = order[a], j = a - 1;
        while (j >= 0 && p->acc_ppm[L->voff[i] + order[j]] < p->acc_ppm[L->voff[i] + v]) {
            order[j + 1] = order[j];
            j--;
        }
        order[j + 1] = v;
    }
}

/* ---- the per-task part ------------------------------------------------------ */
typedef struct {
    int32_t workers;   /* sum_k x_ik */
    int32_t any;       /* hosts at least one variant */
    int64_t unserved;  /* demand left after filling every hosted variant */
    int64_t maxlat;    /* max latency over variants in use */
    int64_t weighted;  /* N_i = sum routed_k * acc_ppm_k */
    int32_t first_acc; /* acc_ppm of the first hosted variant in route order */
    int64_t outflow;   /* sum routed_k * r(i,k): requests created per unit of child fan-out */
} lo_task_t;

static void task_eval(const lo_pipeline *p, const lo_layout *L, int i, const int32_t *x,
                      const int32_t *beta /* K_i */, int64_t Dn, int64_t scale, lo_task_t *t,
                      int64_t *routed_out /* K_i or NULL */)
{
    int order[LO_MAX_VARIANTS];
    int K = p->n_variants[i], nb = p->n_batches[i];
    route_order(p, L, i, order);
    t->workers = 0;
    for (int k = 0; k < K; k++)
        t->workers += x[k];
    int64_t rem = Dn;
    t->any = 0;
    t->maxlat = 0;
    t->weighted = 0;
    t->first_acc = 0;
    t->outflow = 0;
    if (routed_out)
        for (int k = 0; k < K; k++)
            routed_out[k] = 0;
    for (int o = 0; o < K; o++) {
        int k = order[o];
        if (x[k] <= 0)
            continue;
        int64_t thr = p->thr_mqps[L->toff[i] + k * nb + beta[k]];
        int64_t lat = p->latency_us[L->toff[i] + k * nb + beta[k]];
        int64_t cap = (int64_t)x[k] * thr * scale;          /* eq. (2) right-hand side */
        int64_t routed = rem < cap ? rem : cap;             /* Algorithm 1 fill rule */
        int used = (routed > 0) || !t->any;
        if (used && lat > t->maxlat)
            t->maxlat = lat;
        if (!t->any)
            t->first_acc = p->acc_ppm[L->voff[i] + k];
        t->weighted += routed * (int64_t)p->acc_ppm[L->voff[i] + k];
        if (p->variant_factor_q4)
            t->outflow += routed * (int64_t)p->variant_factor_q4[L->voff[i] + k];
        rem -= routed;
        t->any = 1;
        if (routed_out)
            routed_out[k] = routed;
    }
    t->unserved = rem;
}

/* ---- the pipeline part: budget, latency, objective -------------------------- */
/* task_latency_bound: take the latency verdict from the per-task bound (sum over a task path of the
 * largest latency in use); 0 leaves the latency out, for the caller that applies eq. (7) path by path. */
static void pipeline_eval(const lo_pipeline *p, const lo_task_t *t, const int64_t *Dn, int32_t workers_cap,
                          int64_t slo_us, int64_t comm_us, int task_latency_bound, lo_eval_t *out)
{
    int n = p->n_tasks;
    int mask = 0;
    int32_t workers = 0;
    for (int i = 0; i < n; i++)
        workers += t[i].workers;
    if (workers > workers_cap)
        mask |= LO_BAD_WORKERS; /* eq. (3) */
    for (int i = 0; i < n; i++) {
        if (!t[i].any)
            mask |= LO_BAD_EMPTY;
        if (t[i].unserved > 0)
            mask |= LO_BAD_DEMAND; /* eq. (2) with all demand served */
    }
    /* leaves in ascending task index; a path is root -> ... -> leaf */
    int is_leaf[LO_MAX_TASKS];
    for (int i = 0; i < n; i++)
        is_leaf[i] = 1;
    for (int i = 1; i < n; i++)
        is_leaf[p->parent[i]] = 0;
    int n_paths = 0;
    for (int leaf = 0; leaf < n; leaf++) {
        if (!is_leaf[leaf])
            continue;
        n_paths++;
        int64_t lat = 0;
        int len = 0;
        for (int i = leaf; i >= 0; i = p->parent[i]) {
            lat += t[i].maxlat;
            len++;
        }
        int64_t room = slo_us - comm_us * (int64_t)len; /* communication latency per server on the path */
        if (task_latency_bound && (room < 0 || lat > room / 2)) /* SLO halved for queueing; eq. (7) */
            mask |= LO_BAD_LATENCY;
    }
    out->infeasible = mask;
    out->workers = workers;
    out->accuracy = 0.0;
    for (int i = 0; i < n; i++) {
        out->task_acc[i] = 0.0;
        out->task_maxlat[i] = t[i].maxlat;
        out->task_demand[i] = Dn[i];
        out->task_unserved[i] = t[i].unserved;
    }
    if (mask)
        return;
    double a[LO_MAX_TASKS];
    for (int i = 0; i < n; i++) {
        if (Dn[i] > 0)
            a[i] = (double)t[i].weighted / (double)(Dn[i] * 1000000);
        else
            a[i] = (double)t[i].first_acc / 1000000.0;
        out->task_acc[i] = a[i];
    }
    double sum = 0.0;
    int first = 1;
    for (int leaf = 0; leaf < n; leaf++) {
        if (!is_leaf[leaf])
            continue;
        int path[LO_MAX_TASKS], len = 0;
        for (int i = leaf; i >= 0; i = p->parent[i])
            path[len++] = i;
        double prod = a[path[len - 1]]; /* root first */
        for (int s = len - 2; s >= 0; s--)
            prod = prod * a[path[s]];
        if (first)
            sum = prod;
        else
            sum = sum + prod;
        first = 0;
    }
    out->accuracy = sum / (double)n_paths;
}

/* ---- objective from profiled path accuracies: sum_p c(p) * A-hat(p) (Section 4.1 "Accuracy") ----
 * Per root-to-leaf task path, p runs over the combinations of one variant per task.  c(p) is the
 * product of: the frontend's split over the root's variants, and per edge the probability that the
 * routing table of the upstream variant (Algorithm 1, lo_route_table) sends a request to the
 * downstream variant.  An upstream variant without traffic (zero demand) has no table; its requests,
 * if there were any, would go to the first hosted downstream variant in route order, the same
 * convention as for a task's accuracy at zero demand.
 * fp64 order: c(p) is multiplied up root first, then times A-hat(p)/10^6; the terms of a task path
 * are added up with the root's variants outermost, every level in route order (accuracy descending);
 * the task paths' sums are added in leaf order and divided by the number of task paths. */
typedef struct {
    const lo_pipeline *p;
    const lo_layout *L;
    const lo_route_t *r;
    const int32_t *x;     /* replicas, concat over (task, variant) */
    const int *path;      /* tasks root..leaf */
    int len;
    const int32_t *table; /* A-hat of this task path */
    double sum;
} lo_walk;

static void path_walk(lo_walk *c, int depth, int prev_variant, double mass, uint64_t entry, uint64_t stride)
{
    const lo_pipeline *p = c->p;
    int i = c->path[depth], K = p->n_variants[i];
    int order[LO_MAX_VARIANTS];
    route_order(p, c->L, i, order);
    int first_hosted = -1;
    for (int o = 0; o < K && first_hosted < 0; o++)
        if (c->x[c->L->voff[i] + order[o]] > 0)
            first_hosted = order[o];
    int has_traffic = depth == 0 ? c->r->demand[0] > 0 : c->r->routed[c->path[depth - 1]][prev_variant] > 0;
    for (int o = 0; o < K; o++) {
        int k = order[o];
        double share;
        if (has_traffic)
            share = depth == 0 ? c->r->prob[0][0][k] : c->r->prob[i][prev_variant][k];
        else
            share = k == first_hosted ? 1.0 : 0.0;
        if (share == 0.0)
            continue; /* no request takes this branch */
        double m = depth == 0 ? share : mass * share;
        uint64_t e = entry + (uint64_t)k * stride;
        if (depth == c->len - 1)
            c->sum = c->sum + m * ((double)c->table[e] / 1000000.0);
        else
            path_walk(c, depth + 1, k, m, e, stride * (uint64_t)K);
    }
}

static double path_objective(const lo_pipeline *p, const lo_layout *L, uint64_t index, int64_t demand_mqps)
{
    lo_route_t r;
    int32_t x[LO_MAX_TASKS * LO_MAX_VARIANTS], beta[LO_MAX_TASKS * LO_MAX_VARIANTS];
    int n = p->n_tasks;
    lo_route_table(p, index, demand_mqps, &r);
    lo_decode(p, index, x, beta);
    int is_leaf[LO_MAX_TASKS];
    for (int i = 0; i < n; i++)
        is_leaf[i] = 1;
    for (int i = 1; i < n; i++)
        is_leaf[p->parent[i]] = 0;
    const int32_t *table = p->path_acc_ppm;
    double total = 0.0;
    int n_paths = 0;
    for (int leaf = 0; leaf < n; leaf++) {
        if (!is_leaf[leaf])
            continue;
        int rev[LO_MAX_TASKS], path[LO_MAX_TASKS], len = 0;
        for (int i = leaf; i >= 0; i = p->parent[i])
            rev[len++] = i;
        uint64_t size = 1;
        for (int s = 0; s < len; s++) {
            path[s] = rev[len - 1 - s];
            size *= (uint64_t)p->n_variants[path[s]];
        }
        lo_walk c = {p, L, &r, x, path, len, table, 0.0};
        path_walk(&c, 0, 0, 0.0, 0, 1);
        if (n_paths == 0)
            total = c.sum;
        else
            total = total + c.sum;
        n_paths++;
        table += size;
    }
    return total / (double)n_paths;
}

/* ---- eq. (7) as printed: the latency of every variant path with traffic ------------------------
 * A variant path p (one variant per task of a root-to-leaf task path) has traffic, I(p) = 1 in
 * Table 1, when every hop of it carries requests under the routing Algorithm 1 produces for the plan:
 * the frontend sends requests to the root's variant, and the routing table of every variant on the
 * path sends some of its requests to the next one.  At zero demand nothing is routed; the path of the
 * first hosted variants then stands for the plan, as for the accuracy. */
typedef struct {
    const lo_pipeline *p;
    const lo_layout *L;
    const lo_route_t *r;
    const int32_t *x;
    const int *path;
    int len;
    int64_t limit;
    int violated;
} lo_latency_walk;

static void latency_walk(lo_latency_walk *c, int depth, int prev_variant, int64_t so_far)
{
    const lo_pipeline *p = c->p;
    int i = c->path[depth], K = p->n_variants[i];
    int order[LO_MAX_VARIANTS];
    route_order(p, c->L, i, order);
    int first_hosted = -1;
    for (int o = 0; o < K && first_hosted < 0; o++)
        if (c->x[c->L->voff[i] + order[o]] > 0)
            first_hosted = order[o];
    int has_traffic = depth == 0 ? c->r->demand[0] > 0 : c->r->routed[c->path[depth - 1]][prev_variant] > 0;
    for (int k = 0; k < K; k++) {
        int taken;
        if (has_traffic)
            taken = (depth == 0 ? c->r->prob[0][0][k] : c->r->prob[i][prev_variant][k]) > 0.0;
        else
            taken = k == first_hosted;
        if (!taken)
            continue;
        int64_t lat = so_far + c->r->budget_us[i][k]; /* l(i,k) at the variant's configured batch size */
        if (depth == c->len - 1) {
            if (lat > c->limit)
                c->violated = 1;
        } else {
            latency_walk(c, depth + 1, k, lat);
        }
    }
}

static int latency_violated_on_some_path(const lo_pipeline *p, const lo_layout *L, uint64_t index,
                                         int64_t demand_mqps, int64_t slo_us, int64_t comm_us)
{
    lo_route_t r;
    int32_t x[LO_MAX_TASKS * LO_MAX_VARIANTS], beta[LO_MAX_TASKS * LO_MAX_VARIANTS];
    int n = p->n_tasks;
    lo_route_table(p, index, demand_mqps, &r);
    lo_decode(p, index, x, beta);
    int is_leaf[LO_MAX_TASKS];
    for (int i = 0; i < n; i++)
        is_leaf[i] = 1;
    for (int i = 1; i < n; i++)
        is_leaf[p->parent[i]] = 0;
    int violated = 0;
    for (int leaf = 0; leaf < n; leaf++) {
        if (!is_leaf[leaf])
            continue;
        int rev[LO_MAX_TASKS], path[LO_MAX_TASKS], len = 0;
        for (int i = leaf; i >= 0; i = p->parent[i])
            rev[len++] = i;
        for (int s = 0; s < len; s++)
            path[s] = rev[len - 1 - s];
        int64_t room = slo_us - comm_us * (int64_t)len; /* communication latency per server on the path */
        if (room < 0) {
            violated = 1;
            continue;
        }
        lo_latency_walk c = {p, L, &r, x, path, len, room / 2 /* SLO halved for queueing */, 0};
        latency_walk(&c, 0, 0, 0);
        violated |= c.violated;
    }
    return violated;
}

void lo_eval(const lo_pipeline *p, uint64_t index, int64_t demand_mqps, int32_t workers, int64_t slo_us,
             int64_t comm_us, lo_eval_t *out)
{
    lo_layout L;
    int64_t Dn[LO_MAX_TASKS], scale[LO_MAX_TASKS];
    lo_task_t t[LO_MAX_TASKS];
    layout_of(p, &L);
    task_demand(p, demand_mqps, Dn, scale);
    uint64_t rest = index;
    for (int i = 0; i < L.n; i++) {
        int32_t x[LO_MAX_VARIANTS], beta[LO_MAX_VARIANTS];
        uint64_t choice = rest % L.choices[i];
        rest /= L.choices[i];
        decode_choice(p, &L, i, choice, x, beta);
        if (p->variant_factor_q4 && i > 0) /* what the parent's variants create for this child */
            Dn[i] = t[p->parent[i]].outflow * (int64_t)p->fanout_q4[i];
        task_eval(p, &L, i, x, beta, Dn[i], scale[i], &t[i], NULL);
    }
    pipeline_eval(p, t, Dn, workers, slo_us, comm_us, !p->latency_per_path, out);
    if (p->latency_per_path && !(out->infeasible & (LO_BAD_DEMAND | LO_BAD_EMPTY)) &&
        latency_violated_on_some_path(p, &L, index, demand_mqps, slo_us, comm_us)) {
        out->infeasible |= LO_BAD_LATENCY; /* eq. (7) on a variant path with traffic */
        out->accuracy = 0.0;
        for (int i = 0; i < L.n; i++)
            out->task_acc[i] = 0.0;
    }
    if (p->path_acc_ppm && !out->infeasible)
        out->accuracy = path_objective(p, &L, index, demand_mqps);
}

/* ---- the search: plain argmax ------------------------------------------------ */
static int better(double acc, int32_t workers, uint64_t index, const lo_best_t *b, int tie_index_only)
{
    if (!b->found)
        return 1;
    if (acc > b->accuracy)
        return 1;
    if (acc < b->accuracy)
        return 0;
    if (!tie_index_only) {
        if (workers < b->workers)
            return 1;
        if (workers > b->workers)
            return 0;
    }
    return index < b->index;
}

static void best_init(lo_best_t *b)
{
    b->index = UINT64_MAX;
    b->accuracy = 0.0;
    b->n_feasible = 0;
    b->workers = -1;
    b->found = 0;
}

static void best_merge(lo_best_t *into, const lo_best_t *from, int tie_index_only)
{
    into->n_feasible += from->n_feasible;
    if (from->found && better(from->accuracy, from->workers, from->index, into, tie_index_only)) {
        into->index = from->index;
        into->accuracy = from->accuracy;
        into->workers = from->workers;
        into->found = 1;
    }
}

int lo_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void lo_search(const lo_pipeline *p, int64_t demand_mqps, int32_t workers, int64_t slo_us, int64_t comm_us,
               int tie_index_only, uint64_t index_begin, uint64_t index_end, uint64_t index_stride,
               int n_threads, lo_best_t *out)
{
    if (n_threads < 1)
        n_threads = 1;
    if (index_stride < 1)
        index_stride = 1;
    uint64_t count = index_end > index_begin ? (index_end - index_begin + index_stride - 1) / index_stride : 0;
    lo_best_t *part = (lo_best_t *)malloc(sizeof(lo_best_t) * (size_t)n_threads);
#pragma omp parallel for num_threads(n_threads) schedule(static, 1)
    for (int th = 0; th < n_threads; th++) {
        lo_best_t b;
        best_init(&b);
        uint64_t lo = count / (uint64_t)n_threads * (uint64_t)th;
        uint64_t hi = th == n_threads - 1 ? count : count / (uint64_t)n_threads * (uint64_t)(th + 1);
        for (uint64_t j = lo; j < hi; j++) {
            uint64_t index = index_begin + j * index_stride;
            lo_eval_t e;
            lo_eval(p, index, demand_mqps, workers, slo_us, comm_us, &e);
            if (e.infeasible)
                continue;
            b.n_feasible++;
            if (better(e.accuracy, e.workers, index, &b, tie_index_only)) {
                b.index = index;
                b.accuracy = e.accuracy;
                b.workers = e.workers;
                b.found = 1;
            }
        }
        part[th] = b;
    }
    best_init(out);
    for (int th = 0; th < n_threads; th++)
        best_merge(out, &part[th], tie_index_only);
    free(part);
}

void lo_search_tabulated(const lo_pipeline *p, int64_t demand_mqps, int32_t workers, int64_t slo_us,
                         int64_t comm_us, int tie_index_only, uint64_t index_begin, uint64_t index_end,
                         int n_threads, lo_best_t *out)
{
    lo_layout L;
    int64_t Dn[LO_MAX_TASKS], scale[LO_MAX_TASKS];
    lo_task_t *table[LO_MAX_TASKS];
    if (p->variant_factor_q4 || p->path_acc_ppm || p->latency_per_path) { /* a task's demand is not fixed / the objective or the latency limit couples tasks: no table */
        lo_search(p, demand_mqps, workers, slo_us, comm_us, tie_index_only, index_begin, index_end, 1, n_threads, out);
        return;
    }
    layout_of(p, &L);
    task_demand(p, demand_mqps, Dn, scale);
    for (int i = 0; i < L.n; i++) {
        table[i] = (lo_task_t *)malloc(sizeof(lo_task_t) * (size_t)L.choices[i]);
        for (uint64_t c = 0; c < L.choices[i]; c++) {
            int32_t x[LO_MAX_VARIANTS], beta[LO_MAX_VARIANTS];
            decode_choice(p, &L, i, c, x, beta);
            task_eval(p, &L, i, x, beta, Dn[i], scale[i], &table[i][c], NULL);
        }
    }
    if (n_threads < 1)
        n_threads = 1;
    uint64_t count = index_end > index_begin ? index_end - index_begin : 0;
    lo_best_t *part = (lo_best_t *)malloc(sizeof(lo_best_t) * (size_t)n_threads);
#pragma omp parallel for num_threads(n_threads) schedule(static, 1)
    for (int th = 0; th < n_threads; th++) {
        lo_best_t b;
        best_init(&b);
        uint64_t lo = index_begin + count / (uint64_t)n_threads * (uint64_t)th;
        uint64_t hi = th == n_threads - 1 ? index_end : index_begin + count / (uint64_t)n_threads * (uint64_t)(th + 1);
        uint64_t choice[LO_MAX_TASKS];
        uint64_t rest = lo;
        for (int i = 0; i < L.n; i++) {
            choice[i] = rest % L.choices[i];
            rest /= L.choices[i];
        }
        for (uint64_t index = lo; index < hi; index++) {
            lo_task_t t[LO_MAX_TASKS];
            lo_eval_t e;
            for (int i = 0; i < L.n; i++)
                t[i] = table[i][choice[i]];
            pipeline_eval(p, t, Dn, workers, slo_us, comm_us, 1, &e);
            if (!e.infeasible) {
                b.n_feasible++;
                if (better(e.accuracy, e.workers, index, &b, tie_index_only)) {
                    b.index = index;
                    b.accuracy = e.accuracy;
                    b.workers = e.workers;
                    b.found = 1;
                }
            }
            for (int i = 0; i < L.n; i++) { /* next index: add one in mixed radix */
                if (++choice[i] < L.choices[i])
                    break;
                choice[i] = 0;
            }
        }
        part[th] = b;
    }
    best_init(out);
    for (int th = 0; th < n_threads; th++)
        best_merge(out, &part[th], tie_index_only);
    free(part);
    for (int i = 0; i < L.n; i++)
        free(table[i]);
}

/* ---- Algorithm 1 for one plan, replicas of a variant lumped together -------- */
void lo_route_table(const lo_pipeline *p, uint64_t index, int64_t demand_mqps, lo_route_t *r)
{
    lo_layout L;
    int32_t x[LO_MAX_TASKS * LO_MAX_VARIANTS], beta[LO_MAX_TASKS][LO_MAX_VARIANTS];
    layout_of(p, &L);
    memset(r, 0, sizeof(*r));
    task_demand(p, demand_mqps, r->demand, r->scale);
    int n = p->n_tasks;
    uint64_t rest = index;
    for (int i = 0; i < n; i++) {
        int nb = p->n_batches[i];
        uint64_t choice = rest % L.choices[i];
        rest /= L.choices[i];
        decode_choice(p, &L, i, choice, x + L.voff[i], beta[i]);
        for (int k = 0; k < p->n_variants[i]; k++) {
            int xk = x[L.voff[i] + k];
            r->capacity[i][k] = (int64_t)xk * p->thr_mqps[L.toff[i] + k * nb + beta[i][k]] * r->scale[i];
            r->leftover[i][k] = r->capacity[i][k];
            r->budget_us[i][k] = xk > 0 ? p->latency_us[L.toff[i] + k * nb + beta[i][k]] : 0;
        }
    }
    /* frontend -> first task */
    {
        int order[LO_MAX_VARIANTS];
        route_order(p, &L, 0, order);
        int64_t outgoing = r->demand[0], total = outgoing;
        for (int o = 0; o < p->n_variants[0]; o++) {
            int k = order[o];
            if (r->leftover[0][k] > 0 && outgoing > 0) {
                int64_t routed = outgoing < r->leftover[0][k] ? outgoing : r->leftover[0][k];
                r->prob[0][0][k] = (double)routed / (double)total;
                outgoing -= routed;
                r->leftover[0][k] -= routed;
                r->routed[0][k] += routed;
            }
        }
        r->unserved[0] = outgoing;
    }
    /* tasks in topological order (indices already are), workers by accuracy */
    for (int i = 0; i < n; i++) {
        int order[LO_MAX_VARIANTS];
        route_order(p, &L, i, order);
        for (int o = 0; o < p->n_variants[i]; o++) {
            int k = order[o];
            for (int j = i + 1; j < n; j++) {
                if (p->parent[j] != i)
                    continue;
                int corder[LO_MAX_VARIANTS];
                route_order(p, &L, j, corder);
                int64_t outgoing = r->routed[i][k] * (int64_t)p->fanout_q4[j];
                if (p->variant_factor_q4) { /* the child's demand is what its parent's variants create */
                    outgoing *= (int64_t)p->variant_factor_q4[L.voff[i] + k];
                    if (o == 0)
                        r->demand[j] = 0;
                    r->demand[j] += outgoing;
                }
                int64_t total = outgoing;
                for (int co = 0; co < p->n_variants[j]; co++) {
                    int ck = corder[co];
                    if (r->leftover[j][ck] > 0 && outgoing > 0) {
                        int64_t routed = outgoing < r->leftover[j][ck] ? outgoing : r->leftover[j][ck];
                        r->prob[j][k][ck] = (double)routed / (double)total;
                        outgoing -= routed;
                        r->leftover[j][ck] -= routed;
                        r->routed[j][ck] += routed;
                    }
                }
                r->unserved[j] += outgoing;
            }
        }
    }
}

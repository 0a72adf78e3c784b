// Host side of the C-ABI declared in include/loki_alloc.h: validation, the
// fixed-point range proof, workspace layout, launch configuration, and the
// per-plan routing table (Algorithm 1 of the Loki paper, Section 5.1).
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstring>
#include <map>
#include <new>
#include <utility>
#include <vector>

#include "../../include/loki_alloc.h"
#include "loki_device.h"
#include "loki_host.h"
#include "loki_launch.h"

using namespace loki;

static_assert(LOKI_MAX_TASKS == kMaxTasks && LOKI_MAX_VARIANTS == kMaxVariants && LOKI_MAX_BATCHES == kMaxBatches,
              "header and kernels disagree on limits");
static_assert(sizeof(loki_route_t) == sizeof(RouteOut), "route record layout");
static_assert(sizeof(loki_result_t) == 32 && sizeof(loki_eval_t) == 16 && sizeof(BestRec) == 32 &&
                  sizeof(TaskRec) == 16 && sizeof(MidVal) == 16 && sizeof(MidLim) == 16,
              "record layouts");

namespace {

// Blocks per launch: far more than the 1024 that are resident at once, so that the hardware's own
// block dispatch evens out compute units and demand points that finish at different times.
constexpr uint32_t kTargetBlocks = 32768;
constexpr uint32_t kMinTile = 128;     // shortest tile of root-task choices per work item
constexpr uint32_t kPruneTile = 256;   // longest tile where most feasible plans are spared the walk (profiled path
                                       // accuracies on one task path): the walks left sit in few work items
// Below this many work items per launch the tile is shortened: a launch should have more blocks than the
// 1280 that are resident at once.  Not sooner: the entries of a tile are walked in runs of equal limits,
// and a longer tile has longer runs.
constexpr uint64_t kFewItems = 2048;
constexpr int64_t kTwo53 = int64_t(1) << 53;
constexpr size_t kAlign = 256;

thread_local int g_last_hip = 0;

size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Layout {
    size_t off_P, off_Dn, off_table, off_lat2, off_perm, off_run, off_perm_all, off_run_t, off_recs, off_floor, off_results,
        off_results_open, total;
};

// `cb` is the size of the constant block: the problem constants followed by the profiled path
// accuracies (if any), see const_block().
// c1: choices of the tile task of a class-by-class search with swapped roles (then off_perm_all holds a list of
// the choices of every task, table_total entries per point, and off_run_t the tile task's runs), else 0.
// per_path: eq. (7) on the variant paths with traffic (a second table of two latencies per choice, and a second
// set of results for the plans only that rule admits).
Layout search_layout(size_t cb, uint32_t table_total, uint32_t c0, int64_t M, uint32_t c1 = 0, bool per_path = false) {
    Layout l;
    l.off_P = 0;
    l.off_Dn = cb;
    l.off_table = align_up(l.off_Dn + size_t(M) * kMaxTasks * sizeof(int64_t));
    l.off_lat2 = align_up(l.off_table + size_t(M) * table_total * sizeof(TaskRec));
    l.off_perm = align_up(l.off_lat2 + (per_path ? size_t(M) * table_total * sizeof(TaskLat2) : 0));
    l.off_run = align_up(l.off_perm + size_t(M) * c0 * sizeof(uint32_t));
    l.off_perm_all = align_up(l.off_run + size_t(M) * c0 * sizeof(uint32_t));
    l.off_run_t = align_up(l.off_perm_all + size_t(M) * (c1 ? table_total : 0u) * sizeof(uint32_t));
    l.off_recs = align_up(l.off_run_t + size_t(M) * c1 * sizeof(uint32_t));
    l.off_floor = align_up(l.off_recs + (size_t(kTargetBlocks) + size_t(M)) * sizeof(BestRec));
    l.off_results = align_up(l.off_floor + size_t(M) * sizeof(unsigned long long));
    l.off_results_open = align_up(l.off_results + size_t(M) * sizeof(loki_result_t));
    l.total = align_up(l.off_results_open + (per_path ? size_t(M) * sizeof(loki_result_t) : 0));
    return l;
}

// Per-variant factors searched class by class: a point of a launch is a demand point with one class (one
// amount of created requests) per task that has children.  A batch of points per set of launches: as many
// as keep the per-point task tables within kClassTableBytes, between 256 and 4096.
#ifndef LOKI_CLASS_POINTS_LIMIT
#define LOKI_CLASS_POINTS_LIMIT 65535  // (a CPU test build of the host side lowers it to reach the paths beyond it)
#endif
constexpr int64_t kMaxClassPoints = LOKI_CLASS_POINTS_LIMIT;
constexpr size_t kClassTableBytes = size_t(256) << 20;
int32_t class_batch(uint32_t table_total) {
    const size_t fit = kClassTableBytes / (size_t(std::max<uint32_t>(table_total, 1u)) * sizeof(TaskRec));
    return int32_t(std::min<size_t>(4096, std::max<size_t>(256, fit)));
}

// Whether some search of the handle can run class by class (see class_search_mode): the workspace is then
// sized for it.
bool class_search_applies(const loki_problem *p);

struct ClassLayout {
    size_t off_P, off_vDn, off_vOut, off_vCount, off_vPoint, off_batch, off_class_results, off_results, total;
    Layout batch;  // offsets inside the batch region (its off_P / off_Dn are not used)
};

ClassLayout class_layout(size_t cb, uint32_t table_total, uint32_t c0, uint32_t c1, int64_t M) {
    ClassLayout l;
    l.off_P = 0;
    l.off_vDn = cb;
    l.off_vOut = align_up(l.off_vDn + size_t(kMaxClassPoints) * kMaxTasks * sizeof(int64_t));
    l.off_vCount = align_up(l.off_vOut + size_t(kMaxClassPoints) * kMaxTasks * sizeof(int64_t));
    l.off_vPoint = align_up(l.off_vCount + size_t(kMaxClassPoints) * kMaxTasks * sizeof(uint32_t));
    l.off_batch = align_up(l.off_vPoint + size_t(kMaxClassPoints) * sizeof(int32_t));
    l.batch = search_layout(0, table_total, c0, class_batch(table_total), c1);
    l.off_class_results = l.off_batch + l.batch.off_results;
    l.off_results = align_up(l.off_batch + l.batch.total);
    l.total = align_up(l.off_results + size_t(M) * sizeof(loki_result_t));
    return l;
}

struct EvalLayout {
    size_t off_P, off_idx, off_out, total;
};

EvalLayout eval_layout(size_t cb, int64_t n) {
    EvalLayout l;
    l.off_P = 0;
    l.off_idx = cb;
    l.off_out = align_up(l.off_idx + size_t(n) * sizeof(uint64_t));
    l.total = align_up(l.off_out + size_t(n) * sizeof(loki_eval_t));
    return l;
}

}  // namespace

struct loki_problem {
    DevProblem dev;
    int32_t n;
    int32_t fanout_q4[kMaxTasks];
    int32_t depth[kMaxTasks];
    int32_t batch_size[kMaxTasks][kMaxBatches];
    int32_t voff[kMaxTasks];
    int32_t max_vf[kMaxTasks];  // largest variant factor of the task (4 without per-variant factors)
    int32_t sum_r[kMaxTasks];   // sum of the replica limits of the task
    bool caps_fit32 = true;     // every R(i,k) * q * scale is below 2^32 (a per-lane search may fill in 32 bits)
    int32_t last_fill_bits = 0; // width of the fill arithmetic of the last search that scored whole plans per lane
    uint64_t n_candidates;
    std::vector<double> path_acc;  // profiled path accuracies as fractions (ppm / 10^6), all leaves
    // class-by-class searches: every choice of every task decoded once (replicas and batch position per
    // variant, at (table_off[i] + c) * kMaxVariants), filled on first use
    // pinned staging of the (demand point, class) descriptors: [Dn 8 int64 | amount int64 | count u32 | point i32] arrays
    unsigned char *class_staging = nullptr;
    bool star = false;  // every other task is a child of the first task
    bool class_small_space = false;  // the class-by-class search under way reaches fewer than 2^33 plans
    // pinned staging: [DevProblem, path accuracies | Dn (cap_points * 8 int64) | results (cap_points)]
    unsigned char *staging = nullptr;
    int64_t cap_points = 0;
    // ordinary host memory with the same head ([DevProblem, path accuracies | Dn of kNoAllocPoints points]) for
    // searches that must not allocate: sized when the handle is created, copied from as it is
    std::vector<unsigned char> plain_block;
    hipEvent_t staged = nullptr, ev[4] = {nullptr, nullptr, nullptr, nullptr};
    bool staged_pending = false;
    // A second set of the pinned buffers and their event: every search call takes the set the call before it
    // did not use (rotate_staging), so that the host never waits for the copies of the call just enqueued, which
    // sit behind that call's predecessors' kernels on the stream, but for those of the call before.
    struct StagingSet {
        unsigned char *class_staging = nullptr, *staging = nullptr;
        int64_t cap_points = 0;
        hipEvent_t staged = nullptr;
        bool staged_pending = false;
    } spare;
    float last_ms[3] = {0.f, 0.f, 0.f};  // per-task tables, main search kernel, final merge
    bool have_ms = false;
    uint64_t last_scored = 0;  // plans the kernels of the last search scored
    bool have_scored = false;
};

namespace {

int hip_fail(hipError_t e) {
    g_last_hip = static_cast<int>(e);
    return LOKI_E_HIP;
}

#define LOKI_HIP(expr)                                \
    do {                                              \
        hipError_t e_ = (expr);                       \
        if (e_ != hipSuccess) return hip_fail(e_);    \
    } while (0)

// Constant block of a handle: DevProblem, directly followed by the path accuracies.
size_t const_block(const loki_problem *p) {
    return align_up(sizeof(DevProblem) + p->path_acc.size() * sizeof(double));
}

void fill_const_block(loki_problem *p, unsigned char *dst = nullptr) {
    if (!dst) dst = p->staging;
    std::memcpy(dst, &p->dev, sizeof(DevProblem));
    if (!p->path_acc.empty())
        std::memcpy(dst + sizeof(DevProblem), p->path_acc.data(), p->path_acc.size() * sizeof(double));
}

const double *device_path_acc(const loki_problem *p, const unsigned char *ws) {
    return p->path_acc.empty() ? nullptr : reinterpret_cast<const double *>(ws + sizeof(DevProblem));
}

size_t staging_bytes(const loki_problem *p, int64_t points) {
    return const_block(p) + align_up(size_t(points) * kMaxTasks * sizeof(int64_t)) +
           align_up(size_t(points) * sizeof(loki_result_t));
}

void rotate_staging(loki_problem *p) {
    std::swap(p->class_staging, p->spare.class_staging);
    std::swap(p->staging, p->spare.staging);
    std::swap(p->cap_points, p->spare.cap_points);
    std::swap(p->staged, p->spare.staged);
    std::swap(p->staged_pending, p->spare.staged_pending);
}

int ensure_staging(loki_problem *p, int64_t points) {
    if (!p->staged)  // first GPU use of this set of buffers: the event for their reuse
        LOKI_HIP(hipEventCreateWithFlags(&p->staged, hipEventDisableTiming));
    if (!p->ev[0])  // first GPU use of this handle: events for timing
        for (auto &e : p->ev) LOKI_HIP(hipEventCreate(&e));
    if (points <= p->cap_points) return LOKI_OK;
    if (p->staged_pending) {
        LOKI_HIP(hipEventSynchronize(p->staged));
        p->staged_pending = false;
    }
    if (p->staging) {
        LOKI_HIP(hipHostFree(p->staging));
        p->staging = nullptr;
        p->cap_points = 0;
    }
    int64_t cap = std::max<int64_t>(points, 1024);
    void *ptr = nullptr;
    LOKI_HIP(hipHostMalloc(&ptr, staging_bytes(p, cap), hipHostMallocDefault));
    p->staging = static_cast<unsigned char *>(ptr);
    p->cap_points = cap;
    return LOKI_OK;
}

// Demand at each task (eq. (1)) with the overflow proof for everything downstream:
// Dn_i * 10^6 must stay below 2^53.  With one factor per edge Dn_i is exact; with per-variant
// factors it is the largest value any plan can reach (every request served by the variant
// with the largest factor) and only Dn_0 is used by the kernels.
int task_demand(const loki_problem *p, int64_t demand_mqps, int64_t *Dn) {
    if (demand_mqps < 0) return LOKI_E_RANGE;
    Dn[0] = demand_mqps;
    for (int i = 0; i < kMaxTasks; i++) {
        if (i >= p->n) {
            Dn[i] = 0;
            continue;
        }
        if (i > 0) {
            const int par = p->dev.parent[i];
            const int64_t factor = int64_t(p->fanout_q4[i]) * (p->dev.has_vf ? p->max_vf[par] : 1);
            if (Dn[par] > kTwo53 / 1000000 / factor) return LOKI_E_RANGE;
            Dn[i] = Dn[par] * factor;
        }
        if (Dn[i] >= kTwo53 / 1000000) return LOKI_E_RANGE;
    }
    return LOKI_OK;
}

void path_budgets(const loki_problem *p, int64_t slo_us, int64_t comm_us, int64_t *budget) {
    for (int i = 0; i < kMaxTasks; i++) {
        budget[i] = -1;
        if (i < p->n) {
            const int64_t room = slo_us - comm_us * p->dev.path_len[i];
            budget[i] = room < 0 ? -1 : room / 2;  // SLO halved for queueing (Section 4.1)
        }
    }
}

int check_scalars(int32_t workers, int64_t slo_us, int64_t comm_us) {
    if (workers < 0 || workers > (1 << 30)) return LOKI_E_RANGE;
    if (slo_us < 0 || slo_us > (int64_t(1) << 40)) return LOKI_E_RANGE;
    if (comm_us < 0 || comm_us > (int64_t(1) << 30)) return LOKI_E_RANGE;
    return LOKI_OK;
}

// The classes of task i at demand D in the task's own units: the amounts of requests its usable choices create
// per unit of a child's fan-out, sum_k routed(k) * r(i,k) (eq. (1) with per-variant factors; eq. (2) and
// Algorithm 1's fill rule, as the kernels' eval_task has them), each with the number of choices that create it,
// in ascending order of the amount.  The choices are not gone through one by one: with the variants taken most
// accurate first, everything is settled once the variants so far reach D (they are full but the last, which
// takes the rest), whatever the replicas of the variants after them, so the digits form a tree that is only
// entered where the capacity so far is below D.
typedef std::vector<std::pair<int64_t, uint32_t>> ClassList;

struct ClassTree {
    const DevProblem *d;
    int i;
    int64_t D;
    bool per_variant;
    uint32_t below[kMaxVariants + 1];  // choices of the variants from route position r on (one batch size per task:
                                       // for one value of it)
    ClassList *classes;
    size_t last;  // the class hit last
};

void class_hit(ClassTree &t, int64_t amount, uint32_t count) {
    ClassList &cl = *t.classes;
    if (!t.per_variant) amount = -1;
    if (t.last < cl.size() && cl[t.last].first == amount) {
        cl[t.last].second += count;
        return;
    }
    auto at = std::lower_bound(cl.begin(), cl.end(), amount,
                               [](const std::pair<int64_t, uint32_t> &c, int64_t v) { return c.first < v; });
    if (at != cl.end() && at->first == amount) at->second += count;
    else at = cl.insert(at, std::make_pair(amount, count));
    t.last = size_t(at - cl.begin());
}

// r: route position; upto < D: capacity of the variants before it; created: what they create when full;
// batch: the task's batch position (one batch size per task).
void class_tree(ClassTree &t, int r, int64_t upto, int64_t created, int batch) {
    const DevProblem &d = *t.d;
    const int i = t.i, k = d.order[i][r], nb = d.nb[i];
    const int64_t factor = d.vf[i][k];
    for (uint32_t g = 0; g < d.radix[i][k]; g++) {
        int64_t x = g;
        int beta = batch;
        if (d.pv_batch) {  // g = 0: not hosted; else 1 + (replicas - 1) * |B_i| + batch position
            x = g == 0 ? 0 : int64_t((g - 1) / uint32_t(nb)) + 1;
            beta = g == 0 ? 0 : int((g - 1) % uint32_t(nb));
        }
        const int64_t mine = x * d.thr_s[i][k][beta];  // below 2^62 by the range proof of the throughputs
        if (mine >= t.D - upto) {
            class_hit(t, created + (t.D - upto) * factor, t.below[r + 1]);
        } else if (r + 1 < d.K[i]) {
            class_tree(t, r + 1, upto + mine, created + mine * factor, batch);
        }
    }
}

void task_classes(const loki_problem *p, int i, int64_t D, bool per_variant, ClassList &classes) {
    const DevProblem &d = p->dev;
    classes.clear();
    classes.reserve(64);
    ClassTree t;
    t.d = &d;
    t.i = i;
    t.D = D;
    t.per_variant = per_variant;
    t.classes = &classes;
    t.last = ~size_t(0);
    t.below[d.K[i]] = 1;
    for (int r = d.K[i] - 1; r >= 0; r--) t.below[r] = t.below[r + 1] * d.radix[i][d.order[i][r]];
    const int batches = d.pv_batch ? 1 : d.nb[i];
    if (D == 0) {
        // nothing to serve: every choice that hosts something is usable and creates nothing
        const uint32_t hosting = (t.below[0] - 1) * uint32_t(batches);
        if (hosting) class_hit(t, 0, hosting);
        return;
    }
    for (int b = 0; b < batches; b++) class_tree(t, 0, 0, 0, b);
}

// The points of a class-by-class search: per demand point every combination of one class per task that
// has children, a class being one amount of requests the task's usable choices create under the demand
// the classes of its ancestors give it.  That fixes every task's demand.  Per point: the demands, the
// amounts (-1 for a leaf), and per task the number of its choices that belong (all of a leaf's).
struct ClassPoints {
    std::vector<int64_t> Dn;        // [n][kMaxTasks]
    std::vector<int64_t> amount;    // [n][kMaxTasks]
    std::vector<uint32_t> count;    // [n][kMaxTasks]
    std::vector<int32_t> point;     // [n]
    size_t size() const { return point.size(); }
};

struct ClassWalk {
    const loki_problem *p;
    ClassPoints *cp;
    int32_t point;
    int64_t Dn[kMaxTasks], amount[kMaxTasks];
    uint32_t count[kMaxTasks];
    // classes of (task, demand), kept while one demand point is walked
    std::map<std::pair<int, int64_t>, std::vector<std::pair<int64_t, uint32_t>>> memo;
};

// Tasks in index order (parents first).  Returns LOKI_E_ARG when the call has too many points.
int walk_classes(ClassWalk &w, int i) {
    const loki_problem *p = w.p;
    if (i == p->n) {
        if (int64_t(w.cp->size()) >= kMaxClassPoints) return LOKI_E_ARG;  // caller falls back
        // (the slots past the last task hold 0 / -1 / 1 from the start of the demand point's walk)
        w.cp->point.push_back(w.point);
        w.cp->Dn.insert(w.cp->Dn.end(), w.Dn, w.Dn + kMaxTasks);
        w.cp->amount.insert(w.cp->amount.end(), w.amount, w.amount + kMaxTasks);
        w.cp->count.insert(w.cp->count.end(), w.count, w.count + kMaxTasks);
        return LOKI_OK;
    }
    // (one factor per edge: the demand is the parent's times the edge's factor, and every usable choice of a
    // task is in its one class, written as amount -1 = "any")
    const bool per_variant = p->dev.has_vf != 0;
    if (i > 0) w.Dn[i] = (per_variant ? w.amount[p->dev.parent[i]] : w.Dn[p->dev.parent[i]]) * int64_t(p->fanout_q4[i]);
    if (p->dev.is_leaf[i]) {
        w.amount[i] = -1;
        w.count[i] = p->dev.C[i];
        return walk_classes(w, i + 1);
    }
    auto key = std::make_pair(i, w.Dn[i]);
    auto it = w.memo.find(key);
    if (it == w.memo.end()) {
        ClassList classes;
        task_classes(p, i, w.Dn[i], per_variant, classes);
        it = w.memo.emplace(key, std::move(classes)).first;
    }
    for (const auto &cls : it->second) {
        w.amount[i] = cls.first;
        w.count[i] = cls.second;
        const int rc = walk_classes(w, i + 1);
        if (rc) return rc;
    }
    return LOKI_OK;
}

// The points of the demand points [first, n_demand), as many whole demand points as stay within
// kMaxClassPoints; *next is the first demand point left out.  LOKI_E_ARG when a single demand point has more.
int build_class_points(loki_problem *p, const int64_t *demand_mqps, int32_t first, int32_t n_demand, ClassPoints &cp,
                       int32_t *next) {
    ClassWalk w;
    w.p = p;
    w.cp = &cp;
    int32_t m = first;
    for (; m < n_demand; m++) {
        int64_t bound[kMaxTasks];
        const int rc = task_demand(p, demand_mqps[m], bound);  // range proof with the largest factors
        if (rc) return rc;
        const size_t before = cp.size();
        w.memo.clear();
        w.point = m;
        for (int j = 0; j < kMaxTasks; j++) {
            w.Dn[j] = 0;
            w.amount[j] = -1;
            w.count[j] = 1u;
        }
        w.Dn[0] = demand_mqps[m];
        const int rc2 = walk_classes(w, 0);
        if (rc2 == LOKI_E_ARG && m > first) {  // this demand point starts the next group
            cp.point.resize(before);
            cp.Dn.resize(before * kMaxTasks);
            cp.amount.resize(before * kMaxTasks);
            cp.count.resize(before * kMaxTasks);
            break;
        }
        if (rc2) return rc2;
    }
    *next = m;
    return LOKI_OK;
}

// Order of the points of a class-by-class search and their split into batches.  The blocks of a launch
// are shared out evenly among its points, so a batch should hold points of similar size: they go by
// descending number of work items (items[]; 1 each where the roles are not swapped), a batch takes as
// many as leave each of its points about one block per kClassItemsPerBlock work items, and inside a batch
// the points of a demand point are kept together (the merge folds stretches of equal demand points).
// With profiled path accuracies a work item's cost is the walks of its feasible plans, which sit in a few
// items: one block per work item then, so that as many blocks as possible share them.
constexpr uint64_t kClassItemsPerBlock = 8;
// With profiled path accuracies and swapped roles: whether the objective is taken leaf by leaf (the tile task
// is a leaf, so every leaf's value depends on the entry, on the lane or on the work item alone; the kernel
// keeps at most kMaxPrefix branches of the walk over the variant paths above a leaf).
bool leaf_values_apply(const loki_problem *p) {
    if (!p->dev.has_path || p->n < 3 || !p->dev.is_leaf[p->dev.tile_task] || p->dev.n_paths < 2) return false;
    for (int i = 0; i < p->n; i++) {
        if (!p->dev.is_leaf[i]) continue;
        uint64_t branches = 1;
        for (int j = p->dev.parent[i]; j >= 0; j = p->dev.parent[j]) branches *= uint64_t(p->dev.K[j]);
        if (branches > uint64_t(kMaxPrefix)) return false;
    }
    return true;
}

uint64_t class_items_per_block(const loki_problem *p) {
    return (p->dev.has_path && !leaf_values_apply(p)) ? 1 : kClassItemsPerBlock;
}

void plan_class_batches(ClassPoints &cp, const std::vector<uint64_t> &items, int32_t batch_limit,
                        uint64_t items_per_block, std::vector<int64_t> &batch_first) {
    const size_t V = cp.size();
    std::vector<uint32_t> order(V);
    for (size_t v = 0; v < V; v++) order[v] = uint32_t(v);
    std::stable_sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) { return items[a] > items[b]; });
    batch_first.clear();
    for (size_t at = 0; at < V;) {
        const uint64_t most = std::max<uint64_t>(1, items[order[at]]);
        const uint64_t blocks = std::max<uint64_t>(1, (most + items_per_block - 1) / items_per_block);
        const size_t take = size_t(std::min<uint64_t>(uint64_t(batch_limit), std::max<uint64_t>(1, kTargetBlocks / blocks)));
        const size_t end = std::min(V, at + take);
        std::stable_sort(order.begin() + at, order.begin() + end,
                         [&](uint32_t a, uint32_t b) { return cp.point[a] < cp.point[b]; });
        batch_first.push_back(int64_t(at));
        at = end;
    }
    batch_first.push_back(int64_t(V));
    ClassPoints out;
    out.Dn.resize(cp.Dn.size());
    out.amount.resize(cp.amount.size());
    out.count.resize(cp.count.size());
    out.point.resize(V);
    for (size_t v = 0; v < V; v++) {
        const size_t src = order[v];
        for (int j = 0; j < kMaxTasks; j++) {
            out.Dn[v * kMaxTasks + j] = cp.Dn[src * kMaxTasks + j];
            out.amount[v * kMaxTasks + j] = cp.amount[src * kMaxTasks + j];
            out.count[v * kMaxTasks + j] = cp.count[src * kMaxTasks + j];
        }
        out.point[v] = cp.point[src];
    }
    cp = std::move(out);
}

// Launch configuration and launches of the tabulated kernels (per-task tables, run order, the kernel
// that visits every plan) for the A.M points A describes.  most: the most first-task choices any point
// visits (all of them, or the largest class); with swapped roles (A.swap, set by the caller: classes, two
// or more leaves, whole space) the most combinations of the work item's tasks any point has.
// before_search / after_search: events recorded around the kernel that visits every plan, or null.
// open_results: with A.lat2 set (per-path latency rule on the tables), where the results of the second kernel go.
int launch_tabulated(loki_problem *p, SearchArgs A, uint64_t most, uint64_t index_begin, uint64_t index_end,
                     hipStream_t stream, hipEvent_t before_search, hipEvent_t after_search, void *open_results = nullptr) {
    const int n = p->n, L = n - 1;
    const uint64_t span = index_end - index_begin;
    const uint32_t n_points = static_cast<uint32_t>(A.M);
    // (with profiled path accuracies a quarter of the blocks: every block ends with one walk over the
    // variant paths for the few plans left in its queues, which longer blocks spread over more work)
    const bool leaf_values = A.swap && leaf_values_apply(p);
    // (a single task path with one factor per edge: an upper bound on the objective spares most feasible plans
    // the walk, see path_combine_kernel; the plans that are walked sit in few places of the plan space, so the
    // work items are made small, and the bound keeps 8 more registers per slot)
    uint64_t above = 1;
    for (int j = 0; j < L; j++) above *= uint64_t(p->dev.K[j]);
    const bool prune = p->dev.has_path && !leaf_values && !A.swap && !p->dev.has_vf && p->dev.n_paths == 1 &&
                       above <= uint64_t(kMaxPrefix);
    A.prune = prune ? 1u : 0u;   // (the table kernel needs it too: it leaves the variants in use in the records)
    const uint32_t target_blocks = (p->dev.has_path && !leaf_values) ? kTargetBlocks / 4 : kTargetBlocks;
    const uint32_t max_bpm = std::max<uint32_t>(1u, (target_blocks + n_points - 1) / n_points);
    const uint32_t CL = p->dev.C[L];
    // (class by class with profiled path accuracies on a small plan space: the cost is the walks of the
    // feasible plans, which sit in few of the work items, and the overhead of smaller items is small in
    // absolute terms; 4 slots per lane and one chunk of the last task per block then, so that more blocks
    // share the walks)
    const bool fine_items =
        p->dev.has_path && !leaf_values && A.class_amount != nullptr && A.swap && p->class_small_space;
    const int slots = (CL >= 512 && !fine_items && !prune) ? 8 : 4;
    const uint32_t chunk = 64u * slots;
    const uint64_t strideL = p->dev.stride[L];
    uint64_t F = 1;
    for (int j = 1; j < L; j++) F *= p->dev.C[j];
    const uint32_t C0 = n >= 2 ? p->dev.C[0] : 1u;
    uint32_t mid_count = static_cast<uint32_t>(std::max<uint64_t>(1u, std::min<uint64_t>(most, C0)));
    if (A.swap) {
        // a point's choices of the tasks with children are few, so the first leaf's choices fill the tiles
        // and all the other tasks but the last make up the work item (see combine_kernel)
        A.swap_tasks = uint32_t(L);
        F = std::max<uint64_t>(1, most);  // the most any point has; a point's own count is taken in the kernel
        mid_count = p->dev.C[p->dev.tile_task];
    }
    A.far_count = F;
    A.tile_len = kMidTile;
    A.mid_tiles = (mid_count + A.tile_len - 1) / A.tile_len;
    A.far_first = 0;
    A.far_span = F;
    if (span == 0) {
        A.cl_first = 0;
        A.chunk_groups = 0;
        A.cpb = 1;
        A.items = 0;
    } else {
        const uint32_t cl_first = static_cast<uint32_t>(index_begin / strideL);
        const uint32_t cl_last = static_cast<uint32_t>((index_end - 1) / strideL);
        const uint32_t n_chunks = (cl_last - cl_first + 1 + chunk - 1) / chunk;
        A.cl_first = cl_first;
        A.cpb = 1;
        while (!fine_items && !prune && A.cpb * 2 <= n_chunks && A.cpb * 2 <= uint32_t(kWavesPerBlock)) A.cpb *= 2;
        A.chunk_groups = (n_chunks + A.cpb - 1) / A.cpb;
        // a range shorter than one step of the last task's choice touches only some of the
        // combinations of the tasks in between, in cyclic order from that of its first index
        if (span < strideL) {
            const uint64_t o_first = index_begin % strideL;  // position among all tasks but the last
            const uint64_t touched = (o_first % C0 + span + C0 - 1) / C0;
            if (touched < F) {
                A.far_first = o_first / C0;
                A.far_span = touched;
            }
        }
        A.items = uint64_t(A.chunk_groups) * A.far_span * A.mid_tiles;
        // a search with few work items gets shorter ones: blocks that meet many feasible plans
        // run long, and only spare items let the others take over the rest
        while (A.tile_len > kMinTile && ((prune && A.tile_len > kPruneTile) || A.items * n_points < kFewItems)) {
            A.tile_len /= 2;
            A.mid_tiles = (mid_count + A.tile_len - 1) / A.tile_len;
            A.items = uint64_t(A.chunk_groups) * A.far_span * A.mid_tiles;
        }
    }
    A.blocks_per_m = static_cast<uint32_t>(std::min<uint64_t>(std::max<uint64_t>(A.items, 1), max_bpm));
    if (A.swap)  // the pairs of a batch are of similar size (plan_class_batches): several work items per block
        A.blocks_per_m = static_cast<uint32_t>(std::min<uint64_t>(
            A.blocks_per_m, std::max<uint64_t>(1, (A.items + class_items_per_block(p) - 1) / class_items_per_block(p))));
    if (A.items > (uint64_t(1) << 62) / A.blocks_per_m) A.blocks_per_m = 1;  // keep items*block in 64 bits
    A.items_per_block = A.items / A.blocks_per_m;
    A.items_extra = A.items % A.blocks_per_m;
    const bool range = !(index_begin == 0 && index_end == p->n_candidates);
    const int np = p->dev.n_paths;
    const bool divide = (np & (np - 1)) != 0;
    LOKI_HIP(launch_task_table(A, p->dev.table_total, stream));
    if (n >= 2) LOKI_HIP(launch_root_order(A, stream));
    if (before_search) LOKI_HIP(hipEventRecord(before_search, stream));
    if (leaf_values) {
        // profiled path accuracies, the objective leaf by leaf: the plans cost what they cost in the product form
        LOKI_HIP(launch_combine(A, slots, true, divide, range, true, stream));
    } else if (p->dev.has_path) {
        // profiled path accuracies (one factor per edge): the same walk over the plan space for feasibility,
        // the objective from the walk over the variant paths for feasible plans only
        int path_levels = 0;
        for (int i = 0; i < n; i++) path_levels = std::max(path_levels, p->dev.path_len[i]);
        LOKI_HIP(launch_path_combine(A, slots, range, path_levels, stream));
    } else {
        LOKI_HIP(launch_combine(A, slots, np > 1, divide, range, false, stream));
    }
    if (A.lat2) {
        // the per-path latency rule: the plans only that rule admits, into results of their own, folded in below
        // (the block records are free again once the first merge has read them; the stream keeps the order)
        LOKI_HIP(launch_final_reduce(A, stream));
        SearchArgs B = A;
        B.results = open_results;
        int latency_levels = 0;
        for (int i = 0; i < n; i++) latency_levels = std::max(latency_levels, p->dev.path_len[i]);
        LOKI_HIP(launch_open_plans(B, slots, range, latency_levels, stream));
        if (after_search) LOKI_HIP(hipEventRecord(after_search, stream));
        LOKI_HIP(launch_final_reduce(B, stream));
        LOKI_HIP(launch_fold_results(A.results, B.results, A.M, A.tie_index_only != 0, stream));
        return LOKI_OK;
    }
    if (after_search) LOKI_HIP(hipEventRecord(after_search, stream));
    LOKI_HIP(launch_final_reduce(A, stream));
    return LOKI_OK;
}

// How a class-by-class search of [index_begin, index_end) would run: 2 with swapped roles (three or more
// tasks, the tile task's choices orderable into runs and its index part within 32 bits),
// 1 with the first task's choices in the tiles (every other task a child of the first one, its choices
// orderable into runs), 0 not at all.
int class_search_mode(const loki_problem *p, uint64_t index_begin, uint64_t index_end) {
    // (without per-variant factors only for the sake of profiled path accuracies taken leaf by leaf: every
    // demand point is then a single point, the roles swapped)
    const bool per_variant = p->dev.has_vf != 0;
    if (!(per_variant || leaf_values_apply(p)) || p->n < 2 || p->dev.table_total > (1u << 16)) return 0;
    const int t = p->dev.tile_task;
    (void)index_begin;
    (void)index_end;
    if (p->n >= 3 &&
        uint64_t(p->dev.sum_r_t + 1) * uint64_t(p->dev.n_lat_t) + 1 <= 4096 &&
        p->dev.stride[t] <= (uint64_t(1) << 32) / p->dev.C[t])
        return 2;
    if (per_variant && p->star && uint64_t(p->dev.sum_r0 + 1) * uint64_t(p->dev.n_lat0) + 1 <= 4096) return 1;
    return 0;
}

bool class_search_applies(const loki_problem *p) {
    return class_search_mode(p, 0, p->n_candidates) != 0 || class_search_mode(p, 0, 0) != 0;
}

int enqueue_search(loki_problem *p, const int64_t *demand_mqps, int32_t n_demand, int32_t workers, int64_t slo_us,
                   int64_t comm_us, uint32_t flags, uint64_t index_begin, uint64_t index_end, void *d_workspace,
                   size_t workspace_bytes, hipStream_t stream, void *d_results, bool timed, void **results_at,
                   bool no_alloc);

int enqueue_class_search(loki_problem *p, const int64_t *demand_mqps, int32_t n_demand, int32_t workers,
                         int64_t slo_us, int64_t comm_us, uint32_t flags, uint64_t index_begin, uint64_t index_end,
                         void *d_workspace, size_t workspace_bytes, hipStream_t stream, void *d_results, bool timed,
                         void **results_at) {
    const size_t cb = const_block(p);
    const int mode = class_search_mode(p, index_begin, index_end);
    if (mode == 0) return LOKI_E_ARG;  // caller takes the general path
    const bool swap = mode == 2;
    const int L = p->n - 1, T = p->dev.tile_task;
    const ClassLayout lay = class_layout(cb, p->dev.table_total, p->dev.C[0], p->dev.C[T], n_demand);
    if (workspace_bytes < lay.total || (reinterpret_cast<uintptr_t>(d_workspace) % kAlign) != 0)
        return LOKI_E_WORKSPACE;
    if (d_results && (reinterpret_cast<uintptr_t>(d_results) % 8) != 0) return LOKI_E_WORKSPACE;
    // every demand point is range-checked before anything is enqueued: the points are taken in groups below,
    // and an error in a later group must not leave the work of the earlier ones behind
    for (int32_t m = 0; m < n_demand; m++) {
        int64_t bound[kMaxTasks];
        const int rc_m = task_demand(p, demand_mqps[m], bound);
        if (rc_m) return rc_m;
    }
    int rc = LOKI_OK;
    const size_t per_point = kMaxTasks * (2 * sizeof(int64_t) + sizeof(uint32_t)) + sizeof(int32_t);
    unsigned char *ws = static_cast<unsigned char *>(d_workspace);

    MergeArgs G;
    std::memset(&G, 0, sizeof(G));
    G.results = d_results ? d_results : static_cast<void *>(ws + lay.off_results);
    if (results_at) *results_at = G.results;
    G.M = n_demand;
    G.tie_index_only = (flags & LOKI_TIE_INDEX_ONLY) ? 1u : 0u;

    SearchArgs A;
    std::memset(&A, 0, sizeof(A));
    unsigned char *bw = ws + lay.off_batch;
    A.P = reinterpret_cast<const DevProblem *>(ws + lay.off_P);
    A.table = reinterpret_cast<TaskRec *>(bw + lay.batch.off_table);
    A.recs = reinterpret_cast<BestRec *>(bw + lay.batch.off_recs);
    A.floor = reinterpret_cast<unsigned long long *>(bw + lay.batch.off_floor);
    A.perm = reinterpret_cast<uint32_t *>(bw + lay.batch.off_perm);
    A.run_end = reinterpret_cast<uint32_t *>(bw + lay.batch.off_run);
    A.perm_all = reinterpret_cast<uint32_t *>(bw + lay.batch.off_perm_all);
    A.run_end_t = reinterpret_cast<uint32_t *>(bw + lay.batch.off_run_t);
    A.swap = swap ? 1u : 0u;
    A.path_acc = device_path_acc(p, ws);
    A.results = ws + lay.off_class_results;
    path_budgets(p, slo_us, comm_us, A.budget);
    A.begin = index_begin;
    A.end = index_end;
    A.W = workers;
    A.w_most_last = p->sum_r[p->n - 1];
    {
        int64_t others = 0;
        for (int i = 1; i < p->n; i++) others += p->sum_r[i];
        A.w_free = static_cast<int32_t>(std::max<int64_t>(int64_t(workers) - others, -1));
        const int64_t others_t = others + p->sum_r[0] - p->sum_r[T];  // all tasks but the tile task
        A.w_free_t = static_cast<int32_t>(std::max<int64_t>(int64_t(workers) - others_t, -1));
    }
    A.tie_index_only = G.tie_index_only;

    // The demand points are taken in groups whose points fit the descriptor arrays (one group unless the call
    // has many demand points or tasks with children); the first group is built before anything is enqueued,
    // so that a call that cannot run class by class at all leaves no work behind.
    p->last_scored = 0;
    p->have_scored = true;
    bool enqueued = false, first_search = true;
    for (int32_t m0 = 0; m0 < n_demand;) {
        ClassPoints cp;
        int32_t m1 = m0;
        rc = build_class_points(p, demand_mqps, m0, n_demand, cp, &m1);
        if (rc == LOKI_E_ARG && enqueued) {
            // This demand point alone has more points than the descriptor arrays hold, and earlier groups are
            // already on the stream: it is searched per lane, here, into its own result slot.  (The per-lane
            // search lays its few buffers over the front of the workspace, which the groups before it no
            // longer need when the stream gets there and the groups after it fill again.)
            const uint64_t scored = p->last_scored;
            rc = enqueue_search(p, demand_mqps + m0, 1, workers, slo_us, comm_us, flags | LOKI_SEARCH_PER_LANE,
                                index_begin, index_end, d_workspace, workspace_bytes, stream,
                                static_cast<unsigned char *>(G.results) + size_t(m0) * sizeof(loki_result_t), false,
                                nullptr, false);
            if (rc) return rc;
            p->last_scored += scored;
            // the constant block of the class-by-class layout is the same block; the descriptors are rewritten per group
            m0 += 1;
            continue;
        }
        if (rc) return rc;  // (LOKI_E_ARG: the first demand point alone has too many points; the caller falls back)
        const int64_t V = int64_t(cp.size());
        // per point: the combinations of the work item's tasks (swapped roles) or the first task's choices
        auto far_of = [&](int64_t v) {
            const uint32_t *cnt = cp.count.data() + size_t(v) * kMaxTasks;
            if (!swap) return uint64_t(cnt[0]);
            uint64_t far = 1;
            for (int j = 0; j < L; j++)
                if (j != T) far *= cnt[j];
            return far;
        };
        {
            const uint64_t span = index_end - index_begin, c0 = p->dev.C[0];
            for (int64_t v = 0; v < V; v++) {
                const uint32_t *cnt = cp.count.data() + size_t(v) * kMaxTasks;
                uint64_t plans = uint64_t(cnt[0]) * ((span + c0 - 1) / c0);  // exact for the whole space
                if (swap) {
                    plans = 1;
                    for (int j = 0; j < p->n; j++) plans *= cnt[j];
                }
                p->last_scored += plans;
            }
        }
        {
            uint64_t group_plans = 0;
            for (int64_t v = 0; v < V; v++) {
                const uint32_t *cnt = cp.count.data() + size_t(v) * kMaxTasks;
                uint64_t plans = 1;
                for (int j = 0; j < p->n; j++) plans = std::min<uint64_t>(plans * cnt[j], uint64_t(1) << 40);
                group_plans += plans;
            }
            p->class_small_space = group_plans < (uint64_t(1) << 33);
        }
        std::vector<int64_t> batch_first;
        {
            // work items per point with swapped roles (else one batch size fits all)
            const uint64_t mid_tiles = (p->dev.C[T] + kMidTile - 1) / kMidTile;
            std::vector<uint64_t> items(size_t(V), 1);
            if (swap)
                for (int64_t v = 0; v < V; v++) items[size_t(v)] = far_of(v) * mid_tiles;
            plan_class_batches(cp, items, class_batch(p->dev.table_total), class_items_per_block(p), batch_first);
        }

        // (the pinned buffers of this call's set; a demand point searched per lane in between has moved on to the other)
        rc = ensure_staging(p, n_demand);
        if (rc) return rc;
        if (!p->class_staging) {
            void *ptr = nullptr;
            LOKI_HIP(hipHostMalloc(&ptr, size_t(kMaxClassPoints) * per_point, hipHostMallocDefault));
            p->class_staging = static_cast<unsigned char *>(ptr);
        }
        if (p->staged_pending) {  // earlier copies (the call before the last, the previous group) may still read them
            LOKI_HIP(hipEventSynchronize(p->staged));
            p->staged_pending = false;
        }
        if (!enqueued) {
            fill_const_block(p);
            LOKI_HIP(hipMemcpyAsync(ws + lay.off_P, p->staging, cb, hipMemcpyHostToDevice, stream));
            if (timed) LOKI_HIP(hipEventRecord(p->ev[0], stream));
            LOKI_HIP(launch_results_init(G, stream));
            enqueued = true;
        }
        if (V > 0) {
            unsigned char *h = p->class_staging;
            const size_t nDn = size_t(V) * kMaxTasks * sizeof(int64_t), nOut = size_t(V) * kMaxTasks * sizeof(int64_t),
                         nCount = size_t(V) * kMaxTasks * sizeof(uint32_t), nPoint = size_t(V) * sizeof(int32_t);
            std::memcpy(h, cp.Dn.data(), nDn);
            std::memcpy(h + nDn, cp.amount.data(), nOut);
            std::memcpy(h + nDn + nOut, cp.count.data(), nCount);
            std::memcpy(h + nDn + nOut + nCount, cp.point.data(), nPoint);
            LOKI_HIP(hipMemcpyAsync(ws + lay.off_vDn, h, nDn, hipMemcpyHostToDevice, stream));
            LOKI_HIP(hipMemcpyAsync(ws + lay.off_vOut, h + nDn, nOut, hipMemcpyHostToDevice, stream));
            LOKI_HIP(hipMemcpyAsync(ws + lay.off_vCount, h + nDn + nOut, nCount, hipMemcpyHostToDevice, stream));
            LOKI_HIP(hipMemcpyAsync(ws + lay.off_vPoint, h + nDn + nOut + nCount, nPoint, hipMemcpyHostToDevice, stream));
        }
        LOKI_HIP(hipEventRecord(p->staged, stream));
        p->staged_pending = true;

        for (size_t b = 0; b + 1 < batch_first.size(); b++) {
            const int64_t v0 = batch_first[b];
            const int32_t nb = int32_t(batch_first[b + 1] - v0);
            A.M = nb;
            A.Dn = reinterpret_cast<const int64_t *>(ws + lay.off_vDn) + size_t(v0) * kMaxTasks;
            A.class_amount = reinterpret_cast<const int64_t *>(ws + lay.off_vOut) + size_t(v0) * kMaxTasks;
            A.class_count = reinterpret_cast<const uint32_t *>(ws + lay.off_vCount) + size_t(v0) * kMaxTasks;
            uint64_t most = 1;
            for (int32_t j = 0; j < nb; j++) most = std::max(most, far_of(v0 + j));
            // (the event after the search kernel is recorded again by every batch: the last one counts)
            rc = launch_tabulated(p, A, most, index_begin, index_end, stream, timed && first_search ? p->ev[1] : nullptr,
                                  timed ? p->ev[2] : nullptr);
            if (rc) return rc;
            first_search = false;
            G.class_results = A.results;
            G.point = reinterpret_cast<const int32_t *>(ws + lay.off_vPoint) + v0;
            G.n = nb;
            LOKI_HIP(launch_class_merge(G, stream));
        }
        m0 = m1;
    }
    if (timed && first_search) {  // nothing to search at all
        LOKI_HIP(hipEventRecord(p->ev[1], stream));
        LOKI_HIP(hipEventRecord(p->ev[2], stream));
    }
    if (timed) LOKI_HIP(hipEventRecord(p->ev[3], stream));
    return LOKI_OK;
}

// results_at (optional): where on the device the results of the demand points are written.
// no_alloc: nothing is allocated on the way (no pinned staging, no events, no class-by-class search, which
// needs both): the head of the workspace is copied from the handle's ordinary host block, so the copy
// is done when hipMemcpyAsync returns; timed must be false and n_demand at most kNoAllocPoints.
int enqueue_search(loki_problem *p, const int64_t *demand_mqps, int32_t n_demand, int32_t workers, int64_t slo_us,
                   int64_t comm_us, uint32_t flags, uint64_t index_begin, uint64_t index_end, void *d_workspace,
                   size_t workspace_bytes, hipStream_t stream, void *d_results, bool timed, void **results_at,
                   bool no_alloc) {
    if (!p || !demand_mqps || !d_workspace) return LOKI_E_NULL;
    if (n_demand < 1 || n_demand > LOKI_MAX_DEMAND_POINTS) return LOKI_E_ARG;
    if (no_alloc && (timed || n_demand > kNoAllocPoints)) return LOKI_E_ARG;
    if (flags & ~(LOKI_TIE_INDEX_ONLY | LOKI_SEARCH_PER_LANE)) return LOKI_E_ARG;
    if (index_begin > index_end || index_end > p->n_candidates) return LOKI_E_ARG;
    int rc = check_scalars(workers, slo_us, comm_us);
    if (rc) return rc;
    if (!no_alloc) rotate_staging(p);
    // eq. (7) on the variant paths with traffic couples the tasks of a path.  With one factor per edge and the
    // product-form objective the tables still do most of the work: the plans the per-task bound admits as ever,
    // then the few it rejects whose sure paths are fast enough, one by one (open_plans_kernel); a single task
    // has one variant per path and the two rules are the same.  Otherwise whole plans per lane.
    const bool per_path_on_tables = p->dev.lat_per_path && !p->dev.has_vf && !p->dev.has_path && !(flags & LOKI_SEARCH_PER_LANE);
    if (p->dev.lat_per_path && !per_path_on_tables) flags |= LOKI_SEARCH_PER_LANE;
    // Per-variant factors: a task's demand depends on its parent's part of the plan.  Where every other
    // task is a child of the first one, that dependence is one number per first-task choice (the requests
    // it creates), and the tabulated kernels run once per distinct value; otherwise whole plans per lane.
    if (!no_alloc && class_search_mode(p, index_begin, index_end) != 0 && !(flags & LOKI_SEARCH_PER_LANE)) {
        rc = enqueue_class_search(p, demand_mqps, n_demand, workers, slo_us, comm_us, flags, index_begin, index_end,
                                  d_workspace, workspace_bytes, stream, d_results, timed, results_at);
        if (rc != LOKI_E_ARG) return rc;  // LOKI_E_ARG: too many classes, take the general path
    }
    // per-variant factors that cannot be searched class by class couple the tasks' feasibility
    if (p->dev.has_vf) flags |= LOKI_SEARCH_PER_LANE;
    p->last_scored = (index_end - index_begin) * uint64_t(n_demand);
    p->have_scored = true;
    const size_t cb = const_block(p);
    const Layout lay = search_layout(cb, p->dev.table_total, p->dev.C[0], n_demand, 0, p->dev.lat_per_path != 0);
    if (workspace_bytes < lay.total || (reinterpret_cast<uintptr_t>(d_workspace) % kAlign) != 0)
        return LOKI_E_WORKSPACE;
    if (d_results && (reinterpret_cast<uintptr_t>(d_results) % 8) != 0) return LOKI_E_WORKSPACE;

    unsigned char *host_head = p->plain_block.data();
    if (!no_alloc) {
        rc = ensure_staging(p, n_demand);
        if (rc) return rc;
        if (p->staged_pending) {  // the previous call's copy may still be reading the staging buffer
            LOKI_HIP(hipEventSynchronize(p->staged));
            p->staged_pending = false;
        }
        host_head = p->staging;
    }
    int64_t *hDn = reinterpret_cast<int64_t *>(host_head + cb);
    for (int32_t m = 0; m < n_demand; m++) {
        rc = task_demand(p, demand_mqps[m], hDn + size_t(m) * kMaxTasks);
        if (rc) return rc;
    }
    fill_const_block(p, host_head);

    unsigned char *ws = static_cast<unsigned char *>(d_workspace);
    const size_t head = cb + size_t(n_demand) * kMaxTasks * sizeof(int64_t);
    static_assert(sizeof(DevProblem) % 8 == 0, "alignment of the demand block");
    LOKI_HIP(hipMemcpyAsync(ws + lay.off_P, host_head, head, hipMemcpyHostToDevice, stream));
    if (!no_alloc) {
        LOKI_HIP(hipEventRecord(p->staged, stream));
        p->staged_pending = true;
    }

    SearchArgs A;
    std::memset(&A, 0, sizeof(A));
    A.P = reinterpret_cast<const DevProblem *>(ws + lay.off_P);
    A.Dn = reinterpret_cast<const int64_t *>(ws + lay.off_Dn);
    A.table = reinterpret_cast<TaskRec *>(ws + lay.off_table);
    A.recs = reinterpret_cast<BestRec *>(ws + lay.off_recs);
    A.floor = reinterpret_cast<unsigned long long *>(ws + lay.off_floor);
    A.perm = reinterpret_cast<uint32_t *>(ws + lay.off_perm);
    A.run_end = reinterpret_cast<uint32_t *>(ws + lay.off_run);
    A.results = d_results ? d_results : static_cast<void *>(ws + lay.off_results);
    if (results_at) *results_at = A.results;
    A.path_acc = device_path_acc(p, ws);
    path_budgets(p, slo_us, comm_us, A.budget);
    if (per_path_on_tables && p->n >= 2) {
        // (a task path whose communication latency alone exceeds the SLO leaves nothing feasible under either rule)
        bool room = true;
        for (int i = 0; i < p->n; i++) room = room && (!p->dev.is_leaf[i] || A.budget[i] >= 0);
        if (room) A.lat2 = reinterpret_cast<TaskLat2 *>(ws + lay.off_lat2);
    }
    A.begin = index_begin;
    A.end = index_end;
    A.W = workers;
    A.w_most_last = p->sum_r[p->n - 1];
    {
        int64_t others = 0;
        for (int i = 1; i < p->n; i++) others += p->sum_r[i];
        A.w_free = static_cast<int32_t>(std::max<int64_t>(int64_t(workers) - others, -1));
    }
    A.M = n_demand;
    A.tie_index_only = (flags & LOKI_TIE_INDEX_ONLY) ? 1u : 0u;
    const uint32_t max_bpm = std::max<uint32_t>(1u, (kTargetBlocks + n_demand - 1) / n_demand);
    const uint64_t span = index_end - index_begin;
    const int n = p->n, L = n - 1;

    if (timed) LOKI_HIP(hipEventRecord(p->ev[0], stream));
    if (flags & LOKI_SEARCH_PER_LANE) {
        // one work item = one choice of all tasks but the last x a strip of 64 choices of the last;
        // only the strips the index range touches are visited (cl_first/chunk_groups carry them)
        uint64_t items = 0;
        A.far_first = 0;
        A.far_span = 1;
        if (span > 0) {
            const uint64_t strideL = p->dev.stride[L];
            const uint32_t strip_first = static_cast<uint32_t>(index_begin / strideL) / 64;
            const uint32_t strip_last = static_cast<uint32_t>((index_end - 1) / strideL) / 64;
            A.cl_first = strip_first;
            A.chunk_groups = strip_last - strip_first + 1;
            // a range shorter than one step of the last task's choice touches only `span` of the
            // combinations of the other tasks, in cyclic order from its first index
            A.far_first = span < strideL ? index_begin % strideL : 0;
            A.far_span = span < strideL ? span : strideL;
            items = A.far_span * A.chunk_groups;
        }
        const uint64_t want = (items + kBlockThreads - 1) / kBlockThreads;
        A.blocks_per_m = static_cast<uint32_t>(std::min<uint64_t>(std::max<uint64_t>(want, 1), max_bpm));
        if (timed) LOKI_HIP(hipEventRecord(p->ev[1], stream));
        int path_levels = 0;
        if (p->dev.has_path)
            for (int i = 0; i < n; i++) path_levels = std::max(path_levels, p->dev.path_len[i]);
        // the 32-bit fill: every capacity below 2^32 (shown when the handle was made) and so every task's demand
        // at every point (with per-variant factors hDn holds what the task's demand cannot exceed)
        bool narrow = p->caps_fit32 && path_levels == 0 && !p->dev.lat_per_path;
        for (int32_t m = 0; narrow && m < n_demand; m++)
            for (int i = 0; i < n; i++) narrow = narrow && hDn[size_t(m) * kMaxTasks + i] < (int64_t(1) << 32);
        A.narrow = narrow ? 1u : 0u;
        p->last_fill_bits = narrow ? 32 : 64;
        int latency_levels = 0;
        if (p->dev.lat_per_path)
            for (int i = 0; i < n; i++) latency_levels = std::max(latency_levels, p->dev.path_len[i]);
        LOKI_HIP(launch_per_lane_search(A, p->dev.pv_batch != 0, p->dev.has_vf != 0, path_levels, latency_levels,
                                        stream));
        if (timed) LOKI_HIP(hipEventRecord(p->ev[2], stream));
        LOKI_HIP(launch_final_reduce(A, stream));
    } else {
        rc = launch_tabulated(p, A, n >= 2 ? p->dev.C[0] : 1u, index_begin, index_end, stream,
                              timed ? p->ev[1] : nullptr, timed ? p->ev[2] : nullptr, ws + lay.off_results_open);
        if (rc) return rc;
    }
    if (timed) LOKI_HIP(hipEventRecord(p->ev[3], stream));
    return LOKI_OK;
}

}  // namespace

extern "C" {

int loki_problem_create(const loki_pipeline_t *in, loki_problem_t **out) {
    if (!in || !out) return LOKI_E_NULL;
    if (!in->parent || !in->fanout_q4 || !in->n_variants || !in->n_batches || !in->batch_size ||
        !in->max_replicas || !in->acc_ppm || !in->latency_us || !in->thr_mqps)
        return LOKI_E_NULL;
    const int n = in->n_tasks;
    if (n < 1 || n > kMaxTasks) return LOKI_E_RANGE;
    if (in->parent[0] != -1) return LOKI_E_INVALID_GRAPH;
    for (int i = 1; i < n; i++)
        if (in->parent[i] < 0 || in->parent[i] >= i) return LOKI_E_INVALID_GRAPH;

    loki_problem *p = new (std::nothrow) loki_problem();
    if (!p) return LOKI_E_RANGE;
    std::memset(&p->dev, 0, sizeof(p->dev));
    DevProblem &d = p->dev;
    p->n = n;
    d.n_tasks = n;
    d.has_vf = in->variant_factor_q4 ? 1 : 0;
    d.pv_batch = in->per_variant_batch ? 1 : 0;
    d.lat_per_path = in->latency_per_path ? 1 : 0;
    if ((in->per_variant_batch != 0 && in->per_variant_batch != 1) ||
        (in->latency_per_path != 0 && in->latency_per_path != 1)) {
        delete p;
        return LOKI_E_RANGE;
    }
    int v = 0, b = 0, t = 0;
    uint64_t N = 1;
    uint32_t table_total = 0;
    int rc = LOKI_OK;
    for (int i = 0; i < n && rc == LOKI_OK; i++) {
        const int K = in->n_variants[i], nb = in->n_batches[i];
        if (K < 1 || K > kMaxVariants || nb < 1 || nb > kMaxBatches) {
            rc = LOKI_E_RANGE;
            break;
        }
        d.parent[i] = in->parent[i];
        d.is_leaf[i] = 1;
        p->depth[i] = i == 0 ? 0 : p->depth[in->parent[i]] + 1;
        d.path_len[i] = p->depth[i] + 1;
        if (i > 0) {
            d.is_leaf[in->parent[i]] = 0;
            if (in->fanout_q4[i] < 1 || in->fanout_q4[i] > 4096) rc = LOKI_E_RANGE;
        }
        p->fanout_q4[i] = i > 0 ? in->fanout_q4[i] : 4;
        d.K[i] = K;
        d.nb[i] = nb;
        p->voff[i] = v;
        const int per_level_bits = in->variant_factor_q4 ? 4 : 2;  // units of milli-QPS / 16^depth or / 4^depth
        const int64_t scale = int64_t(1) << (per_level_bits * p->depth[i]);
        uint64_t choices = d.pv_batch ? 1u : uint64_t(nb);
        d.magic_nb[i] = ((uint64_t(1) << 36) + uint64_t(nb) - 1) / uint64_t(nb);
        d.fanout[i] = i > 0 ? in->fanout_q4[i] : 4;
        d.scale[i] = scale;
        p->max_vf[i] = 4;
        p->sum_r[i] = 0;
        for (int bi = 0; bi < nb; bi++) {
            const int32_t bs = in->batch_size[b + bi];
            if (bs < 1 || (bi > 0 && bs <= in->batch_size[b + bi - 1])) rc = LOKI_E_RANGE;
            p->batch_size[i][bi] = bs;
            d.batch_size[i][bi] = bs;
        }
        for (int k = 0; k < K; k++) {
            const int32_t R = in->max_replicas[v + k], acc = in->acc_ppm[v + k];
            if (R < 0 || R > LOKI_MAX_REPLICAS || acc < 0 || acc > 1000000) {
                rc = LOKI_E_RANGE;
                break;
            }
            p->sum_r[i] += R;
            d.radix[i][k] = d.pv_batch ? 1u + uint32_t(R) * uint32_t(nb) : uint32_t(R) + 1;
            d.magic[i][k] = ((uint64_t(1) << 36) + d.radix[i][k] - 1) / d.radix[i][k];
            d.magic32[i][k] = d.radix[i][k] == 1 ? 0u : uint32_t(((uint64_t(1) << 32) + d.radix[i][k] - 1) / d.radix[i][k]);
            d.acc[i][k] = acc;
            d.vf[i][k] = 4;
            if (in->variant_factor_q4) {
                const int32_t f = in->variant_factor_q4[v + k];
                if (f < 1 || f > 64) {
                    rc = LOKI_E_RANGE;
                    break;
                }
                d.vf[i][k] = f;
                p->max_vf[i] = k == 0 ? f : std::max(p->max_vf[i], f);
            }
            choices *= d.radix[i][k];
            if (choices > LOKI_MAX_CHOICES) {
                rc = LOKI_E_RANGE;
                break;
            }
            for (int bi = 0; bi < nb; bi++) {
                const int64_t lat = in->latency_us[t + k * nb + bi], thr = in->thr_mqps[t + k * nb + bi];
                if (lat < 1 || lat > (int64_t(1) << 30) || thr < 0 || thr > (int64_t(1) << 40)) rc = LOKI_E_RANGE;
                d.lat[i][k][bi] = int32_t(lat);  // range-checked above
                if (thr > (int64_t(1) << 54) / scale) rc = LOKI_E_RANGE;  // keeps 255 replicas * thr * scale below 2^63
                if (rc == LOKI_OK) d.thr_s[i][k][bi] = thr * scale;
                if (rc == LOKI_OK && R > 0 && d.thr_s[i][k][bi] > ((int64_t(1) << 32) - 1) / R) p->caps_fit32 = false;
            }
        }
        if (rc) break;
        // route order: accuracy descending, variant index ascending (Algorithm 1 sorts by single-model accuracy)
        int ord[kMaxVariants];
        for (int k = 0; k < K; k++) ord[k] = k;
        std::stable_sort(ord, ord + K, [&](int x, int y) { return d.acc[i][x] > d.acc[i][y]; });
        for (int k = 0; k < K; k++) d.order[i][k] = ord[k];
        for (int r = 0; r < K; r++) d.route[i][r] = RouteStep{ord[r], d.acc[i][ord[r]], d.vf[i][ord[r]], 0};
        d.C[i] = uint32_t(choices);
        d.stride[i] = N;
        d.table_off[i] = table_total;
        table_total += uint32_t(choices);
        if (N > (uint64_t(1) << 63) / choices) {
            rc = LOKI_E_RANGE;
            break;
        }
        N *= choices;
        v += K;
        b += nb;
        t += K * nb;
    }
    if (rc == LOKI_OK && N >= (uint64_t(1) << 63)) rc = LOKI_E_RANGE;
    if (rc != LOKI_OK) {
        delete p;
        return rc;
    }
    d.table_total = table_total;
    {  // distinct latencies and replica total of the first task (run ordering of its choices)
        std::vector<int32_t> lats;
        for (int k = 0; k < d.K[0]; k++)
            for (int bi = 0; bi < d.nb[0]; bi++) lats.push_back(int32_t(d.lat[0][k][bi]));
        std::sort(lats.begin(), lats.end());
        lats.erase(std::unique(lats.begin(), lats.end()), lats.end());
        d.n_lat0 = int32_t(lats.size());
        for (size_t q = 0; q < lats.size(); q++) d.lat0_sorted[q] = lats[q];
        d.sum_r0 = 0;
        for (int k = 0; k < d.K[0]; k++) d.sum_r0 += in->max_replicas[k];  // task 0's variants come first
    }
    {  // the same for the first leaf (the task whose choices fill the tiles when the roles are swapped)
        int t = 0;
        while (t < n - 1 && !d.is_leaf[t]) t++;
        if (t == n - 1 && n >= 2) t = n - 2;  // a chain: the last task's parent
        d.tile_task = t;
        std::vector<int32_t> lats;
        for (int k = 0; k < d.K[t]; k++)
            for (int bi = 0; bi < d.nb[t]; bi++) lats.push_back(int32_t(d.lat[t][k][bi]));
        std::sort(lats.begin(), lats.end());
        lats.erase(std::unique(lats.begin(), lats.end()), lats.end());
        d.n_lat_t = int32_t(lats.size());
        for (size_t q = 0; q < lats.size(); q++) d.lat_t_sorted[q] = lats[q];
        d.sum_r_t = p->sum_r[t];
    }
    d.n_paths = 0;
    for (int i = 0; i < n; i++) d.n_paths += d.is_leaf[i];
    p->n_candidates = N;
    p->star = n >= 2;
    for (int i = 1; i < n; i++) p->star = p->star && d.parent[i] == 0;
    for (int i = 0; i < n; i++) {  // chain root..i, root first
        int at = d.path_len[i] - 1;
        for (int j = i; j >= 0; j = d.parent[j]) d.leaf_path[i][at--] = j;
    }
    {  // steps that turn the first task's accuracy into the path values without the last task
        const int L = n - 1;
        auto push = [&](int op, int task) {
            d.prog_op[d.n_prog] = int8_t(op);
            d.prog_task[d.n_prog] = int8_t(task);
            d.n_prog++;
        };
        for (int j = 0; j < L; j++) {
            if (!d.is_leaf[j]) continue;
            for (int q = 1; q < d.path_len[j]; q++) push(kStepMul, d.leaf_path[j][q]);
            push(kStepLeaf, -1);
        }
        if (n >= 2) {
            const int parL = d.parent[L];
            for (int q = 1; q < d.path_len[parL]; q++) push(kStepMul, d.leaf_path[parL][q]);
            push(kStepPre, -1);
        }
    }
    if (in->path_acc_ppm) {
        // profiled accuracy of every variant path, per leaf (Section 4.1 "Accuracy"); stored as the
        // fraction ppm / 10^6, one correctly rounded division each
        d.has_path = 1;
        uint64_t total = 0;
        for (int i = 0; i < n; i++) {
            if (!d.is_leaf[i]) continue;
            uint64_t size = 1;
            for (int j = 0; j < d.path_len[i]; j++) size *= uint64_t(d.K[d.leaf_path[i][j]]);
            d.path_off[i] = uint32_t(total);
            total += size;
            if (total > LOKI_MAX_PATH_ENTRIES) {
                delete p;
                return LOKI_E_RANGE;
            }
        }
        d.path_total = uint32_t(total);
        p->path_acc.resize(total);
        for (uint64_t e = 0; e < total; e++) {
            const int32_t a = in->path_acc_ppm[e];
            if (a < 0 || a > 1000000) {
                delete p;
                return LOKI_E_RANGE;
            }
            p->path_acc[e] = double(a) / 1000000.0;
        }
    }

    p->plain_block.assign(const_block(p) + size_t(kNoAllocPoints) * kMaxTasks * sizeof(int64_t), 0);
    *out = p;
    return LOKI_OK;
}

void loki_problem_destroy(loki_problem_t *p) {
    if (!p) return;
    for (int set = 0; set < 2; set++) {
        if (p->staged_pending && p->staged) (void)hipEventSynchronize(p->staged);
        if (p->staging) (void)hipHostFree(p->staging);
        if (p->class_staging) (void)hipHostFree(p->class_staging);
        if (p->staged) (void)hipEventDestroy(p->staged);
        p->staging = p->class_staging = nullptr;
        p->staged = nullptr;
        p->staged_pending = false;
        rotate_staging(p);
    }
    for (auto e : p->ev)
        if (e) (void)hipEventDestroy(e);
    delete p;
}

int loki_num_candidates(const loki_problem_t *p, uint64_t *n) {
    if (!p || !n) return LOKI_E_NULL;
    *n = p->n_candidates;
    return LOKI_OK;
}

int loki_workspace_bytes(const loki_problem_t *p, int64_t n_demand, size_t *bytes) {
    if (!p || !bytes) return LOKI_E_NULL;
    if (n_demand < 1) return LOKI_E_ARG;
    *bytes = std::max(search_layout(const_block(p), p->dev.table_total, p->dev.C[0], n_demand, 0, p->dev.lat_per_path != 0).total,
                      eval_layout(const_block(p), n_demand).total);
    if (class_search_applies(p))
        *bytes = std::max(*bytes, class_layout(const_block(p), p->dev.table_total, p->dev.C[0], p->dev.C[p->dev.tile_task], n_demand).total);
    return LOKI_OK;
}

namespace {

// choice of task i -> replica counts and batch positions per variant
void decode_choice(const loki_problem *p, int i, uint64_t c, int32_t *x, int32_t *beta) {
    const int K = p->dev.K[i], nb = p->dev.nb[i];
    for (int k = 0; k < K; k++) {
        const uint64_t g = c % p->dev.radix[i][k];
        c /= p->dev.radix[i][k];
        if (p->dev.pv_batch) {
            x[k] = g == 0 ? 0 : int32_t((g - 1) / nb) + 1;
            beta[k] = g == 0 ? 0 : int32_t((g - 1) % nb);
        } else {
            x[k] = int32_t(g);
        }
    }
    if (!p->dev.pv_batch)
        for (int k = 0; k < K; k++) beta[k] = int32_t(c);
}

}  // namespace

int loki_decode(const loki_problem_t *p, uint64_t index, int32_t *x, int32_t *batch) {
    if (!p || !x || !batch) return LOKI_E_NULL;
    if (index >= p->n_candidates) return LOKI_E_RANGE;
    for (int i = 0; i < p->n; i++) {
        int32_t beta[kMaxVariants];
        decode_choice(p, i, index % p->dev.C[i], x + p->voff[i], beta);
        index /= p->dev.C[i];
        if (p->dev.pv_batch) {
            for (int k = 0; k < p->dev.K[i]; k++)
                batch[p->voff[i] + k] = x[p->voff[i] + k] > 0 ? p->batch_size[i][beta[k]] : 0;
        } else {
            batch[i] = p->batch_size[i][beta[0]];
        }
    }
    return LOKI_OK;
}

int loki_alloc_search_enqueue(loki_problem_t *p, const int64_t *demand_mqps, int32_t n_demand, int32_t workers,
                              int64_t slo_us, int64_t comm_us, uint32_t flags, uint64_t index_begin,
                              uint64_t index_end, void *d_workspace, size_t workspace_bytes, void *hip_stream,
                              void *d_results) {
    if (!d_results) return LOKI_E_NULL;
    return enqueue_search(p, demand_mqps, n_demand, workers, slo_us, comm_us, flags, index_begin, index_end,
                          d_workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream), d_results, false, nullptr,
                          false);
}

int loki_alloc_search(loki_problem_t *p, const int64_t *demand_mqps, int32_t n_demand, int32_t workers,
                      int64_t slo_us, int64_t comm_us, uint32_t flags, uint64_t index_begin, uint64_t index_end,
                      void *d_workspace, size_t workspace_bytes, void *hip_stream, loki_result_t *out) {
    if (!out) return LOKI_E_NULL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    void *d_res = nullptr;
    int rc = enqueue_search(p, demand_mqps, n_demand, workers, slo_us, comm_us, flags, index_begin, index_end,
                            d_workspace, workspace_bytes, stream, nullptr, true, &d_res, false);
    if (rc) return rc;
    unsigned char *hres = p->staging + const_block(p) +
                          align_up(size_t(p->cap_points) * kMaxTasks * sizeof(int64_t));
    LOKI_HIP(hipMemcpyAsync(hres, d_res, size_t(n_demand) * sizeof(loki_result_t), hipMemcpyDeviceToHost, stream));
    LOKI_HIP(hipStreamSynchronize(stream));
    p->staged_pending = false;
    std::memcpy(out, hres, size_t(n_demand) * sizeof(loki_result_t));
    p->have_ms = true;
    for (int k = 0; k < 3; k++)
        p->have_ms = p->have_ms && hipEventElapsedTime(&p->last_ms[k], p->ev[k], p->ev[k + 1]) == hipSuccess;
    return LOKI_OK;
}

int loki_alloc_eval(loki_problem_t *p, const uint64_t *indices, int64_t n_indices, int64_t demand_mqps,
                    int32_t workers, int64_t slo_us, int64_t comm_us, void *d_workspace, size_t workspace_bytes,
                    void *hip_stream, loki_eval_t *out) {
    if (!p || !indices || !d_workspace || !out) return LOKI_E_NULL;
    if (n_indices < 1 || n_indices > (int64_t(1) << 31) - 1024) return LOKI_E_ARG;
    int rc = check_scalars(workers, slo_us, comm_us);
    if (rc) return rc;
    for (int64_t j = 0; j < n_indices; j++)
        if (indices[j] >= p->n_candidates) return LOKI_E_RANGE;
    const EvalLayout lay = eval_layout(const_block(p), n_indices);
    if (workspace_bytes < lay.total || (reinterpret_cast<uintptr_t>(d_workspace) % kAlign) != 0)
        return LOKI_E_WORKSPACE;
    EvalArgs A;
    std::memset(&A, 0, sizeof(A));
    rc = task_demand(p, demand_mqps, A.Dn);
    if (rc) return rc;
    path_budgets(p, slo_us, comm_us, A.budget);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    unsigned char *ws = static_cast<unsigned char *>(d_workspace);
    rc = ensure_staging(p, 1);
    if (rc) return rc;
    if (p->staged_pending) {
        LOKI_HIP(hipEventSynchronize(p->staged));
        p->staged_pending = false;
    }
    fill_const_block(p);
    LOKI_HIP(hipMemcpyAsync(ws + lay.off_P, p->staging, sizeof(DevProblem) + p->path_acc.size() * sizeof(double),
                            hipMemcpyHostToDevice, stream));
    LOKI_HIP(hipMemcpyAsync(ws + lay.off_idx, indices, size_t(n_indices) * sizeof(uint64_t), hipMemcpyHostToDevice,
                            stream));
    A.P = reinterpret_cast<const DevProblem *>(ws + lay.off_P);
    A.indices = reinterpret_cast<const uint64_t *>(ws + lay.off_idx);
    A.out = ws + lay.off_out;
    A.path_acc = device_path_acc(p, ws);
    A.n = n_indices;
    A.W = workers;
    LOKI_HIP(launch_eval(A, stream));
    LOKI_HIP(hipMemcpyAsync(out, ws + lay.off_out, size_t(n_indices) * sizeof(loki_eval_t), hipMemcpyDeviceToHost,
                            stream));
    LOKI_HIP(hipStreamSynchronize(stream));
    return LOKI_OK;
}

// Algorithm 1 (MostAccurateFirst) for one plan, with all replicas of a variant
// treated as one worker of capacity x*q: tasks in topological order, workers of a
// task by accuracy, each worker's outgoing requests placed on the child's workers
// by accuracy while capacity lasts; the entries are the routing probabilities.
// What is left of each capacity afterwards is the backup table of Section 5.1,
// and the latency at the configured batch is the task's latency budget (Section 4.2).
int loki_route_table(const loki_problem_t *p, uint64_t index, int64_t demand_mqps, loki_route_t *out) {
    if (!p || !out) return LOKI_E_NULL;
    if (index >= p->n_candidates) return LOKI_E_RANGE;
    int64_t Dn[kMaxTasks];
    int rc = task_demand(p, demand_mqps, Dn);
    if (rc) return rc;
    loki_route_t r;
    std::memset(&r, 0, sizeof(r));
    const int n = p->n;
    uint64_t rest = index;
    for (int i = 0; i < n; i++) {
        int32_t beta[kMaxVariants];
        decode_choice(p, i, rest % p->dev.C[i], r.replicas[i], beta);
        rest /= p->dev.C[i];
        r.demand[i] = Dn[i];
        r.scale[i] = int64_t(1) << ((p->dev.has_vf ? 4 : 2) * p->depth[i]);
        for (int k = 0; k < p->dev.K[i]; k++) {
            const bool hosted = r.replicas[i][k] > 0;
            r.batch[i][k] = hosted ? p->batch_size[i][beta[k]] : 0;
            r.capacity[i][k] = int64_t(r.replicas[i][k]) * p->dev.thr_s[i][k][beta[k]];
            r.leftover[i][k] = r.capacity[i][k];
            r.budget_us[i][k] = hosted ? p->dev.lat[i][k][beta[k]] : 0;
        }
    }
    // place `amount` requests from one source on the workers of task j
    auto place = [&](int j, int64_t amount, double *prob_row) -> int64_t {
        const int64_t total = amount;
        for (int o = 0; o < p->dev.K[j] && amount > 0; o++) {
            const int k = p->dev.order[j][o];
            const int64_t take = std::min(amount, r.leftover[j][k]);
            if (take <= 0) continue;
            prob_row[k] = double(take) / double(total);
            r.leftover[j][k] -= take;
            r.routed[j][k] += take;
            amount -= take;
        }
        return amount;
    };
    r.unserved[0] = place(0, Dn[0], r.prob[0][0]);
    for (int i = 0; i < n; i++)
        for (int o = 0; o < p->dev.K[i]; o++) {
            const int k = p->dev.order[i][o];
            for (int j = i + 1; j < n; j++) {
                if (p->dev.parent[j] != i) continue;
                int64_t created = r.routed[i][k] * int64_t(p->fanout_q4[j]);
                if (p->dev.has_vf) {  // the child's demand is what the parent's variants create
                    created *= p->dev.vf[i][k];
                    if (o == 0) r.demand[j] = 0;
                    r.demand[j] += created;
                }
                r.unserved[j] += place(j, created, r.prob[j][k]);
            }
        }
    *out = r;
    return LOKI_OK;
}

int loki_route_workspace_bytes(const loki_problem_t *p, int64_t n, size_t *bytes) {
    if (!p || !bytes) return LOKI_E_NULL;
    if (n < 1) return LOKI_E_ARG;
    *bytes = align_up(sizeof(DevProblem)) + align_up(size_t(n) * 8) + align_up(size_t(n) * 8) +
             align_up(size_t(n) * sizeof(RouteOut));
    return LOKI_OK;
}

int loki_route_table_batch(loki_problem_t *p, const uint64_t *indices, const int64_t *demand_mqps, int64_t n,
                           void *d_workspace, size_t workspace_bytes, void *hip_stream, loki_route_t *out) {
    if (!p || !indices || !demand_mqps || !d_workspace || !out) return LOKI_E_NULL;
    if (n < 1 || n > (int64_t(1) << 24)) return LOKI_E_ARG;
    size_t need = 0;
    (void)loki_route_workspace_bytes(p, n, &need);
    if (workspace_bytes < need || (reinterpret_cast<uintptr_t>(d_workspace) % kAlign) != 0) return LOKI_E_WORKSPACE;
    for (int64_t j = 0; j < n; j++) {
        if (indices[j] >= p->n_candidates) return LOKI_E_RANGE;
        int64_t Dn[kMaxTasks];
        const int rc = task_demand(p, demand_mqps[j], Dn);
        if (rc) return rc;
    }
    int rc = ensure_staging(p, 1);
    if (rc) return rc;
    if (p->staged_pending) {
        LOKI_HIP(hipEventSynchronize(p->staged));
        p->staged_pending = false;
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    unsigned char *ws = static_cast<unsigned char *>(d_workspace);
    const size_t off_idx = align_up(sizeof(DevProblem)), off_dem = off_idx + align_up(size_t(n) * 8),
                 off_out = off_dem + align_up(size_t(n) * 8);
    std::memcpy(p->staging, &p->dev, sizeof(DevProblem));
    LOKI_HIP(hipMemcpyAsync(ws, p->staging, sizeof(DevProblem), hipMemcpyHostToDevice, stream));
    LOKI_HIP(hipMemcpyAsync(ws + off_idx, indices, size_t(n) * 8, hipMemcpyHostToDevice, stream));
    LOKI_HIP(hipMemcpyAsync(ws + off_dem, demand_mqps, size_t(n) * 8, hipMemcpyHostToDevice, stream));
    RouteArgs A;
    A.P = reinterpret_cast<const DevProblem *>(ws);
    A.indices = reinterpret_cast<const uint64_t *>(ws + off_idx);
    A.demand = reinterpret_cast<const int64_t *>(ws + off_dem);
    A.out = reinterpret_cast<RouteOut *>(ws + off_out);
    A.n = n;
    LOKI_HIP(launch_route(A, stream));
    LOKI_HIP(hipMemcpyAsync(out, ws + off_out, size_t(n) * sizeof(RouteOut), hipMemcpyDeviceToHost, stream));
    LOKI_HIP(hipStreamSynchronize(stream));
    return LOKI_OK;
}

int loki_plan_trace(loki_problem_t *p, const int64_t *trace_mqps, int32_t n, int32_t alpha_ppm, int32_t workers,
                    int64_t slo_us, int64_t comm_us, uint32_t flags, void *d_workspace, size_t workspace_bytes,
                    void *hip_stream, loki_plan_step_t *out) {
    if (!p || !trace_mqps || !out) return LOKI_E_NULL;
    if (n < 1 || n > LOKI_MAX_DEMAND_POINTS || alpha_ppm < 1 || alpha_ppm > 1000000) return LOKI_E_ARG;
    std::vector<int64_t> est(static_cast<size_t>(n));
    std::vector<loki_result_t> res(static_cast<size_t>(n));
    for (int32_t t = 0; t < n; t++) {
        if (trace_mqps[t] < 0 || trace_mqps[t] > (int64_t(1) << 40)) return LOKI_E_RANGE;
        est[t] = t == 0 ? trace_mqps[0]
                        : (int64_t(alpha_ppm) * trace_mqps[t] + int64_t(1000000 - alpha_ppm) * est[t - 1]) / 1000000;
    }
    const int rc = loki_alloc_search(p, est.data(), n, workers, slo_us, comm_us, flags, 0, p->n_candidates,
                                     d_workspace, workspace_bytes, hip_stream, res.data());
    if (rc) return rc;
    // accuracy of the most accurate variants: the same operations in the same order as for any plan
    // (with profiled path accuracies: the entry of the most accurate variants on every task path)
    double pp[kMaxTasks], sum = 0.0;
    bool first = true;
    for (int i = 0; i < p->n; i++) {
        const double a = double(p->dev.acc[i][p->dev.order[i][0]]) / 1000000.0;
        pp[i] = i == 0 ? a : pp[p->dev.parent[i]] * a;
        if (p->dev.is_leaf[i]) {
            double leaf_value = pp[i];
            if (p->dev.has_path) {
                uint32_t entry = 0, stride = 1;
                for (int j = 0; j < p->dev.path_len[i]; j++) {
                    const int task = p->dev.leaf_path[i][j];
                    entry += uint32_t(p->dev.order[task][0]) * stride;
                    stride *= uint32_t(p->dev.K[task]);
                }
                leaf_value = p->path_acc[p->dev.path_off[i] + entry];
            }
            sum = first ? leaf_value : sum + leaf_value;
            first = false;
        }
    }
    const double top = sum / double(p->dev.n_paths);
    for (int32_t t = 0; t < n; t++) {
        out[t].estimate_mqps = est[t];
        out[t].plan = res[t];
        out[t].phase = res[t].status != LOKI_FOUND ? LOKI_PHASE_OVERLOAD
                                                   : (res[t].accuracy >= top ? LOKI_PHASE_HARDWARE : LOKI_PHASE_ACCURACY);
        out[t].pad = 0;
    }
    return LOKI_OK;
}

int loki_last_search_ms(const loki_problem_t *p, float *ms) {
    if (!p || !ms) return LOKI_E_NULL;
    if (!p->have_ms) return LOKI_E_ARG;
    for (int k = 0; k < 3; k++) ms[k] = p->last_ms[k];
    return LOKI_OK;
}

int loki_last_search_fill_bits(const loki_problem_t *p, int32_t *bits) {
    if (!p || !bits) return LOKI_E_NULL;
    if (p->last_fill_bits == 0) return LOKI_E_ARG;
    *bits = p->last_fill_bits;
    return LOKI_OK;
}

int loki_last_search_plans_scored(const loki_problem_t *p, uint64_t *plans) {
    if (!p || !plans) return LOKI_E_NULL;
    if (!p->have_scored) return LOKI_E_ARG;
    *plans = p->last_scored;
    return LOKI_OK;
}

const char *loki_strerror(int code) {
    switch (code) {
        case LOKI_OK: return "ok";
        case LOKI_E_NULL: return "null pointer";
        case LOKI_E_INVALID_GRAPH: return "pipeline is not a rooted tree in topological order";
        case LOKI_E_RANGE: return "value out of range or fixed-point overflow risk";
        case LOKI_E_WORKSPACE: return "workspace too small or misaligned";
        case LOKI_E_HIP: return "HIP runtime error";
        case LOKI_E_ARG: return "inconsistent arguments";
        case LOKI_E_STATIC_LIMIT: return "search needs more scratch memory or demand points than the library's static buffer holds";
        default: return "unknown error";
    }
}

int loki_last_hip_error(void) { return g_last_hip; }

}  // extern "C"

namespace loki {

int plain_search_bytes(const loki_problem_t *p, int32_t n_demand, size_t *bytes) {
    if (!p || !bytes) return LOKI_E_NULL;
    if (n_demand < 1) return LOKI_E_ARG;
    *bytes = search_layout(const_block(p), p->dev.table_total, p->dev.C[0], n_demand, 0, p->dev.lat_per_path != 0).total;
    return LOKI_OK;
}

int search_without_allocation(loki_problem_t *p, const int64_t *demand_mqps, int32_t n_demand, int32_t workers,
                              int64_t slo_us, int64_t comm_us, uint32_t flags, uint64_t index_begin,
                              uint64_t index_end, void *d_workspace, size_t workspace_bytes, hipStream_t stream,
                              loki_result_t *out) {
    void *d_res = nullptr;
    const int rc = enqueue_search(p, demand_mqps, n_demand, workers, slo_us, comm_us, flags, index_begin, index_end,
                                  d_workspace, workspace_bytes, stream, nullptr, false, &d_res, true);
    if (rc) return rc;
    // straight into the caller's array (ordinary host memory: the copy is staged by the runtime)
    LOKI_HIP(hipMemcpyAsync(out, d_res, size_t(n_demand) * sizeof(loki_result_t), hipMemcpyDeviceToHost, stream));
    LOKI_HIP(hipStreamSynchronize(stream));
    return LOKI_OK;
}

int note_hip_error(int hip_error) { return hip_fail(static_cast<hipError_t>(hip_error)); }

}  // namespace loki

// gfx950 kernels of the exhaustive allocation search.
//
// Scoring rules: Loki (HPDC'24) Section 4.1 eq. (1)-(3), (6), (7), (12) and the
// fill rule of Algorithm 1 (Section 5.1); the exact fixed-point and fp64
// conventions are stated in include/loki_alloc.h.
//
// Two ways to cover the plan space, with identical results:
//  * per-lane: a lane scores whole plans from their digits (all tasks but the last once per
//    strip of the last task's choices, then the last task and the plan per step);
//  * tabulated (default): a plan's score separates into a part per task that
//    depends on that task's digits only (replicas, largest latency in use,
//    traffic-weighted accuracy) and a cheap combination (worker sum, path
//    latency sums, path products, leaf sum).  task_table_kernel scores every
//    choice of every task once; combine_kernel then visits every plan, with the
//    last task's records held in registers (one per lane and slot), the other
//    tasks' combination staged in LDS and read as a broadcast.  Each plan still
//    gets its own verdict and objective with the same operations in the same
//    order, so the bits match the per-lane path.
//
// All fp64 arithmetic is individually rounded: the file is compiled with
// -ffp-contract=off and additionally pins the pragma below.
#include <hip/hip_runtime.h>

#include <stddef.h>

#include <type_traits>

#include "loki_device.h"
#include "loki_launch.h"

#pragma clang fp contract(off)

namespace loki {

namespace {

constexpr uint32_t kBadWorkers = 1u, kBadDemand = 2u, kBadEmpty = 4u, kBadLatency = 8u;

struct ResultOut {  // mirrors loki_result_t
    uint64_t index;
    double accuracy;
    uint64_t n_feasible;
    int32_t workers_used;
    int32_t status;
};

struct EvalOut {  // mirrors loki_eval_t
    double accuracy;
    int32_t workers;
    uint32_t infeasible;
};

// v[idx] for a uniform idx known to be below `bound` (a compile-time constant after unrolling).
// Blended with integer masks rather than selected: a chain of selects over array elements is
// folded by the optimizer into one dynamically indexed load, which would push the array into
// scratch memory.
__device__ __forceinline__ uint64_t pick_bits(const uint64_t (&v)[kMaxTasks], int idx, int bound) {
    uint64_t r = 0;
#pragma unroll
    for (int q = 0; q < kMaxTasks; q++)
        if (q < bound) r |= v[q] & (idx == q ? ~0ull : 0ull);
    return r;
}
__device__ __forceinline__ double pick_below(const double (&v)[kMaxTasks], int idx, int bound) {
    uint64_t b[kMaxTasks];
#pragma unroll
    for (int q = 0; q < kMaxTasks; q++) b[q] = static_cast<uint64_t>(__double_as_longlong(v[q]));
    return __longlong_as_double(static_cast<long long>(pick_bits(b, idx, bound)));
}
__device__ __forceinline__ int64_t pick_below(const int64_t (&v)[kMaxTasks], int idx, int bound) {
    uint64_t b[kMaxTasks];
#pragma unroll
    for (int q = 0; q < kMaxTasks; q++) b[q] = static_cast<uint64_t>(v[q]);
    return static_cast<int64_t>(pick_bits(b, idx, bound));
}

// The problem constants in device memory, not written while a kernel runs, seen through the constant address
// space: a read whose address is the same in every lane becomes a scalar load.
using ScalarProblem = const __attribute__((address_space(4))) DevProblem *;
__device__ __forceinline__ ScalarProblem scalar_view(const DevProblem *p) {
    return (ScalarProblem)p;  // NOLINT: an address space cast has no named form
}

__device__ __forceinline__ uint32_t uni(uint32_t v) {
    return static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(v)));
}
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ uint64_t uni64(uint64_t v) {
    return (static_cast<uint64_t>(uni(static_cast<uint32_t>(v >> 32))) << 32) | uni(static_cast<uint32_t>(v));
}

// Copy the first `bytes` of the problem constants into LDS (bytes is a multiple of 4).
__device__ __forceinline__ void stage_problem(DevProblem *dst, const DevProblem *src, uint32_t bytes) {
    const uint32_t *s = reinterpret_cast<const uint32_t *>(src);
    uint32_t *d = reinterpret_cast<uint32_t *>(dst);
    for (uint32_t i = threadIdx.x; i < bytes / 4; i += blockDim.x) d[i] = s[i];
}

// ---- the per-task part -----------------------------------------------------------------------
struct TaskOut {
    int32_t w;          // sum of replicas
    int32_t any;        // hosts something
    int64_t rem;        // unserved demand
    int32_t maxlat;     // largest latency among variants in use
    int64_t weighted;   // sum routed * acc_ppm
    int32_t first_acc;  // accuracy of the first hosted variant in route order
    int64_t outflow;    // sum routed * variant factor: what the task creates per unit of child fan-out
    uint32_t used;      // bit k: variant k is in use
    int32_t lat_top;    // latency of the first variant in use in route order (the most accurate one)
    int32_t lat_bot;    // latency of the last variant in use in route order
};

// A choice of a task taken apart: the replicas of every variant and the batch position(s).
struct ChoiceParts {
    uint32_t lo, hi;      // replicas, 8 bits per variant: variants 0..3 and 4..7
    uint32_t betas;       // batch position, 4 bits per variant (per-variant batch sizes only)
    uint32_t beta_task;   // the task's batch position (one batch size per task)
    int32_t w;            // sum of replicas
};

// Decode choice c of task i (variant 0 least significant; the batch digit on top, or a batch
// position inside every variant's digit).
// PV: a batch size per hosted variant.
// U: where the fields that are the same in every lane (counts, radices, reciprocals, route order, accuracies,
// factors) are read from: P itself, or the constants in device memory seen through the constant address space,
// which turns those reads into scalar loads (the per-lane search; the block's copy in LDS then only serves the
// reads whose address depends on the lane: throughput and latency at the lane's batch size).
template <bool PV, typename UniformView>
__device__ __forceinline__ void decode_choice(UniformView U, int i, uint32_t c, ChoiceParts &g) {
    const int K = U->K[i];
    constexpr bool pv = PV;
    const uint32_t nb = static_cast<uint32_t>(U->nb[i]);
    uint32_t dlo = 0, dhi = 0, betas = 0;
    int32_t w = 0;
    auto digit = [&](int k) -> uint32_t {
        const uint32_t radix = U->radix[i][k];
        // exact quotients by multiply-shift: c * radix < 2^32 with one batch size per task (radix <= 256),
        // c * radix <= 2^36 otherwise (both checked at problem creation)
        const uint32_t q = pv ? static_cast<uint32_t>((static_cast<uint64_t>(c) * U->magic[i][k]) >> 36)
                              : (radix == 1 ? c : __umulhi(c, U->magic32[i][k]));
        const uint32_t d = c - q * radix;
        c = q;
        uint32_t x = d;
        if (pv) {  // d = 0: not hosted; else 1 + (x-1)*nb + batch position
            const uint32_t t = d - 1;
            const uint32_t xq = static_cast<uint32_t>((static_cast<uint64_t>(t) * U->magic_nb[i]) >> 36);
            x = d == 0 ? 0u : xq + 1;
            betas |= (d == 0 ? 0u : t - xq * nb) << (4 * k);
        }
        w += static_cast<int32_t>(x);
        return x;
    };
    const int K_lo = K < 4 ? K : 4;
    for (int k = 0; k < K_lo; k++) dlo |= digit(k) << (8 * k);
    for (int k = 4; k < K; k++) dhi |= digit(k) << (8 * (k - 4));
    g.lo = dlo;
    g.hi = dhi;
    g.betas = betas;
    g.beta_task = c;
    g.w = w;
}

// One batch size per task: the parts of choice c + 1 from those of choice c (add one to the mixed-radix number,
// variant 0 least significant, the batch position on top).  A level is only visited while some lane of the
// wavefront still carries.  The sum of replicas is taken anew from the bytes.
template <typename UniformView>
__device__ __forceinline__ void next_choice(UniformView U, int i, ChoiceParts &g) {
    const int K = U->K[i];
    bool carry = true;
    auto level = [&](uint32_t &word, int k, int pos) {
        const uint32_t top = U->radix[i][k] - 1;  // the largest digit
        const uint32_t d = (word >> (8 * pos)) & 0xffu;
        const bool at_top = d == top;
        const uint32_t next = at_top ? word & ~(0xffu << (8 * pos)) : word + (1u << (8 * pos));
        word = carry ? next : word;
        carry = carry && at_top;
    };
    bool done = false;
    const int K_lo = K < 4 ? K : 4;
    for (int k = 0; k < K_lo && !done; k++) {
        level(g.lo, k, k);
        done = __ballot(carry) == 0;
    }
    for (int k = 4; k < K && !done; k++) {
        level(g.hi, k, k - 4);
        done = __ballot(carry) == 0;
    }
    g.beta_task += carry ? 1u : 0u;
    g.w = static_cast<int32_t>(__builtin_amdgcn_sad_u8(g.lo, 0u, __builtin_amdgcn_sad_u8(g.hi, 0u, 0u)));
}

// Fill the hosted variants of a decoded choice most accurate first (eq. (2), Algorithm 1's fill rule).
// PV: a batch size per hosted variant; VF: per-variant multiplicative factors.
// NARROW: the caller has shown that the demand and every x * q * scale the task can meet are below 2^32: the
// fill runs on 32-bit values (the sums of routed * accuracy and routed * factor stay 64-bit).  Same results.
template <bool PV, bool VF, bool NARROW, typename UniformView>
__device__ __forceinline__ void fill_task(const DevProblem *P, UniformView U, int i, const ChoiceParts &g, int64_t Dn,
                                          TaskOut &o) {
    const int K = U->K[i];
    constexpr bool pv = PV;
    const uint32_t dlo = g.lo, dhi = g.hi, betas = g.betas, beta_task = g.beta_task;
    constexpr bool has_vf = VF;
    if constexpr (NARROW) {
        // byte k of the pair: one byte permute (selector bytes 0..3 pick from the second operand, 4..7 from
        // the first, 0x0c yields zero)
        auto replicas_of = [&](int k) -> uint32_t {
            return __builtin_amdgcn_perm(dhi, dlo, 0x0c0c0c00u | static_cast<uint32_t>(k));
        };
        uint32_t rem = static_cast<uint32_t>(Dn);
        uint64_t weighted = 0, outflow = 0;
        int32_t first_acc = 0, maxlat = 0, lat_top = 0, lat_bot = 0;
        bool any = false;
        uint32_t in_use = 0;
        for (int r = 0; r < K; r++) {
            const int k = uni(U->route[i][r].k);  // the same in every lane: the table addresses below stay scalar
            const uint32_t x = replicas_of(k);
            const uint32_t beta = pv ? (betas >> (4 * k)) & 0xf : beta_task;
            const uint32_t cap = x * static_cast<uint32_t>(P->thr_s[i][k][beta]);
            const int32_t lat = P->lat[i][k][beta];
            const uint32_t routed = rem < cap ? rem : cap;
            const bool hosted = x > 0;
            const bool used = routed > 0 || (hosted && !any);
            if (used && lat > maxlat) maxlat = lat;
            if (used) lat_bot = lat;
            in_use |= used ? 1u << k : 0u;
            if (hosted && !any) lat_top = lat;
            weighted += static_cast<uint64_t>(routed) * static_cast<uint32_t>(U->route[i][r].acc);
            if (has_vf) outflow += static_cast<uint64_t>(routed) * static_cast<uint32_t>(U->route[i][r].vf);
            rem -= routed;
            any = any || hosted;
        }
        // the accuracy of the first hosted variant only counts for a task without demand
        if (Dn == 0) {
            bool found = false;
            for (int r = 0; r < K; r++) {
                const bool hosted = replicas_of(uni(U->route[i][r].k)) > 0;
                if (hosted && !found) first_acc = U->route[i][r].acc;
                found = found || hosted;
            }
        }
        o.w = g.w;
        o.any = any ? 1 : 0;
        o.rem = static_cast<int64_t>(rem);
        o.maxlat = maxlat;
        o.weighted = static_cast<int64_t>(weighted);
        o.first_acc = first_acc;
        o.outflow = static_cast<int64_t>(outflow);
        o.used = in_use;
        o.lat_top = lat_top;
        o.lat_bot = lat_bot;
        return;
    }
    const uint64_t digits = (static_cast<uint64_t>(dhi) << 32) | dlo;
    int64_t rem = Dn, weighted = 0, outflow = 0;
    int32_t any = 0, first_acc = 0, maxlat = 0, lat_top = 0, lat_bot = 0;
    uint32_t in_use = 0;
    for (int r = 0; r < K; r++) {
        const int k = U->route[i][r].k;
        const int64_t x = static_cast<int64_t>((digits >> (8 * k)) & 0xff);
        const uint32_t beta = pv ? (betas >> (4 * k)) & 0xf : beta_task;
        const int64_t cap = x * P->thr_s[i][k][beta];
        const int32_t lat = P->lat[i][k][beta];
        const int32_t acc = U->route[i][r].acc;
        const int64_t routed = rem < cap ? rem : cap;
        const bool hosted = x > 0;
        const bool used = hosted && (routed > 0 || !any);
        if (used && lat > maxlat) maxlat = lat;
        if (used) lat_bot = lat;
        in_use |= used ? 1u << k : 0u;
        if (hosted && !any) {
            first_acc = acc;
            lat_top = lat;
        }
        weighted += routed * static_cast<int64_t>(acc);
        if (has_vf) outflow += routed * static_cast<int64_t>(U->route[i][r].vf);
        rem -= routed;
        any |= hosted ? 1 : 0;
    }
    o.w = g.w;
    o.any = any;
    o.rem = rem;
    o.maxlat = maxlat;
    o.weighted = weighted;
    o.first_acc = first_acc;
    o.outflow = outflow;
    o.used = in_use;
    o.lat_top = lat_top;
    o.lat_bot = lat_bot;
}

// Decode and fill.
template <bool PV, bool VF, bool NARROW = false, typename UniformView = const DevProblem *>
__device__ __forceinline__ void eval_task(const DevProblem *P, int i, uint32_t c, int64_t Dn, TaskOut &o,
                                          UniformView U) {
    ChoiceParts g;
    decode_choice<PV>(U, i, c, g);
    fill_task<PV, VF, NARROW>(P, U, i, g, Dn, o);
}

template <bool PV, bool VF, bool NARROW = false>
__device__ __forceinline__ void eval_task(const DevProblem *P, int i, uint32_t c, int64_t Dn, TaskOut &o) {
    eval_task<PV, VF, NARROW, const DevProblem *>(P, i, c, Dn, o, P);
}

// The same with the two switches read from the problem (kernels that are not time critical).
__device__ __forceinline__ void eval_task_any(const DevProblem *P, int i, uint32_t c, int64_t Dn, TaskOut &o) {
    if (P->pv_batch) {
        if (P->has_vf) eval_task<true, true>(P, i, c, Dn, o);
        else eval_task<true, false>(P, i, c, Dn, o);
    } else {
        if (P->has_vf) eval_task<false, true>(P, i, c, Dn, o);
        else eval_task<false, false>(P, i, c, Dn, o);
    }
}

// One correctly rounded fp64 division of two exactly converted integers (< 2^53).
__device__ __forceinline__ double task_accuracy(const TaskOut &o, int64_t Dn) {
    if (Dn > 0) return static_cast<double>(o.weighted) / static_cast<double>(Dn * 1000000);
    return static_cast<double>(o.first_acc) / 1000000.0;
}

// ---- a whole plan in one lane ---------------------------------------------------------------------
// Under the per-path latency rule the per-task bound is not applied here: the caller settles
// kBadLatency (and clears the accuracy) with some_path_too_slow for plans that have none of the demand and
// empty bits.
__device__ __forceinline__ void eval_plan(const DevProblem *P, const uint32_t (&c)[kMaxTasks], const int64_t *Dn,
                                          const int64_t *budget, int32_t W, uint32_t &mask, int32_t &workers,
                                          double &accuracy) {
    const int n = P->n_tasks;
    const bool has_vf = P->has_vf != 0;
    double pp[kMaxTasks];    // product of accuracies root..i, root first
    int64_t pl[kMaxTasks];   // latency sum root..i
    int64_t out[kMaxTasks];  // requests task i creates per unit of child fan-out (per-variant factors)
    mask = 0;
    workers = 0;
#pragma unroll
    for (int i = 0; i < kMaxTasks; i++) {
        pp[i] = 0.0;
        pl[i] = 0;
        out[i] = 0;
    }
#pragma unroll
    for (int i = 0; i < kMaxTasks; i++) {
        if (i < n) {
            const int par = i > 0 ? P->parent[i] : 0;
            // eq. (1): fixed per task with per-edge factors, else what the parent's variants create
            int64_t dn = Dn[i];
            if (has_vf && i > 0) dn = pick_below(out, par, i) * static_cast<int64_t>(P->fanout[i]);
            TaskOut o;
            eval_task_any(P, i, c[i], dn, o);
            out[i] = o.outflow;
            workers += o.w;
            if (!o.any) mask |= kBadEmpty;
            if (o.rem > 0) mask |= kBadDemand;
            const double a = task_accuracy(o, dn);
            if (i == 0) {
                pp[0] = a;
                pl[0] = o.maxlat;
            } else {
                pp[i] = pick_below(pp, par, i) * a;
                pl[i] = pick_below(pl, par, i) + o.maxlat;
            }
        }
    }
    if (workers > W) mask |= kBadWorkers;  // eq. (3)
    double sum = 0.0;
    bool first = true;
#pragma unroll
    for (int i = 0; i < kMaxTasks; i++) {
        if (i < n && P->is_leaf[i]) {
            if (!P->lat_per_path && (budget[i] < 0 || pl[i] > budget[i])) mask |= kBadLatency;  // eq. (7), halved SLO
            sum = first ? pp[i] : sum + pp[i];
            first = false;
        }
    }
    accuracy = mask ? 0.0 : sum / static_cast<double>(P->n_paths);
}

// ---- objective from profiled path accuracies ------------------------------------------------------
// System accuracy = sum over variant paths p of c(p) * A-hat(p) (Section 4.1 "Accuracy"), averaged over
// the root-to-leaf task paths.  c(p): the frontend's split over the root's variants times, per edge,
// the share of the upstream variant's requests that Algorithm 1 (Section 5.1) places on the
// downstream variant.  Algorithm 1 hands the upstream variants' requests, most accurate variant first,
// to the downstream variants, most accurate first: both sides are consecutive intervals of the
// downstream task's request stream, and a share is the overlap of two intervals over the length of
// the upstream one.  The walk below visits one task of the path per level; a level goes through the
// task's hosted variants in route order, which yields their intervals one after the other.
struct PathWalk {
    const DevProblem *P;
    const double *tab;   // A-hat of this task path, as fractions
    int leaf;
    uint32_t c[kMaxTasks];    // the plan: choice per task
    int64_t dn[kMaxTasks];    // demand per task under this plan
    double sum;
};

__device__ __forceinline__ uint32_t pick32(const uint32_t (&v)[kMaxTasks], int idx) {
    uint32_t r = 0;
#pragma unroll
    for (int q = 0; q < kMaxTasks; q++) r |= v[q] & (idx == q ? ~0u : 0u);
    return r;
}

// lo, len: the interval of this task's request stream that holds the requests coming from the variant
// chosen one level up (the whole stream at the root); mass: c(p) so far; entry, stride: position in
// the table.  A variant that sends nothing (len == 0, only at zero demand) hands on to the first
// hosted variant.
// MAXD: number of levels compiled (the longest task path the caller will meet).
template <int J, int MAXD>
__device__ void path_level(PathWalk &X, int64_t lo, int64_t len, double mass, uint32_t entry, uint32_t stride) {
    const DevProblem *P = X.P;
    const int i = P->leaf_path[X.leaf][J];
    const int K = P->K[i];
    const bool pv = P->pv_batch != 0, has_vf = P->has_vf != 0;
    const uint32_t nb = static_cast<uint32_t>(P->nb[i]);
    uint32_t c = pick32(X.c, i);
    uint64_t digits = 0;
    uint32_t betas = 0;
    for (int k = 0; k < K; k++) {
        const uint32_t radix = P->radix[i][k];
        const uint32_t q = c / radix;
        const uint32_t g = c - q * radix;
        c = q;
        uint32_t x = g;
        if (pv) {
            x = g == 0 ? 0u : (g - 1) / nb + 1;
            betas |= (g == 0 ? 0u : (g - 1) % nb) << (4 * k);
        }
        digits |= static_cast<uint64_t>(x) << (8 * k);
    }
    const uint32_t beta_task = c;
    const int64_t dn = pick_below(X.dn, i, kMaxTasks);
    const bool last = J == P->path_len[X.leaf] - 1;
    const int next = last ? 0 : P->leaf_path[X.leaf][J + 1 < MAXD ? J + 1 : J];
    const int64_t fan = last ? 0 : static_cast<int64_t>(P->fanout[next]);
    int64_t at = 0;     // requests of this task placed so far = start of the next variant's interval
    int64_t made = 0;   // requests created so far for a child, per unit of its fan-out
    bool any = false;
    for (int r = 0; r < K; r++) {
        const int k = P->order[i][r];
        const int64_t x = static_cast<int64_t>((digits >> (8 * k)) & 0xff);
        if (x == 0) continue;
        const uint32_t beta = pv ? (betas >> (4 * k)) & 0xf : beta_task;
        const int64_t cap = x * P->thr_s[i][k][beta];
        const int64_t room = dn - at;
        const int64_t routed = room < cap ? room : cap;
        double share;
        if (len > 0) {
            const int64_t hi_a = at + routed, hi_b = lo + len;
            const int64_t ov = (hi_a < hi_b ? hi_a : hi_b) - (at > lo ? at : lo);
            share = ov > 0 ? static_cast<double>(ov) / static_cast<double>(len) : 0.0;
        } else {
            share = any ? 0.0 : 1.0;
        }
        any = true;
        const int64_t out = has_vf ? routed * static_cast<int64_t>(P->vf[i][k]) : routed;
        if (share != 0.0) {
            const double m = J == 0 ? share : mass * share;
            const uint32_t e = entry + static_cast<uint32_t>(k) * stride;
            if (last) {
                X.sum = X.sum + m * X.tab[e];
            } else {
                if constexpr (J + 1 < MAXD)
                    path_level<J + 1, MAXD>(X, made * fan, out * fan, m, e, stride * static_cast<uint32_t>(K));
            }
        }
        at += routed;
        made += out;
    }
}

// Objective of a feasible plan.  Dn: per-task demand with one factor per edge (only Dn[0] is used
// with per-variant factors, where every task's demand follows from its parent's part of the plan).
template <int MAXD>
__device__ __noinline__ double path_objective(const DevProblem *P, const double *path_acc, const uint32_t (&c)[kMaxTasks],
                                              const int64_t *Dn) {
    PathWalk X;
    X.P = P;
    const int n = P->n_tasks;
    const bool has_vf = P->has_vf != 0;
    int64_t out[kMaxTasks];
#pragma unroll
    for (int i = 0; i < kMaxTasks; i++) {
        X.c[i] = c[i];
        X.dn[i] = 0;
        out[i] = 0;
    }
#pragma unroll
    for (int i = 0; i < kMaxTasks; i++) {
        if (i < n) {
            int64_t dn = Dn[i];
            if (has_vf) {
                if (i > 0) dn = pick_below(out, P->parent[i], i) * static_cast<int64_t>(P->fanout[i]);
                TaskOut o;
                eval_task_any(P, i, c[i], dn, o);
                out[i] = o.outflow;
            }
            X.dn[i] = dn;
        }
    }
    double total = 0.0;
    bool first = true;
    for (int leaf = 0; leaf < n; leaf++) {
        if (!P->is_leaf[leaf]) continue;
        X.leaf = leaf;
        X.tab = path_acc + P->path_off[leaf];
        X.sum = 0.0;
        path_level<0, MAXD>(X, 0, X.dn[0], 0.0, 0u, 1u);
        total = first ? X.sum : total + X.sum;
        first = false;
    }
    return total / static_cast<double>(P->n_paths);
}

struct ChoiceDigits {
    uint64_t digits;     // replicas, 8 bits per variant
    uint32_t betas;      // batch position, 4 bits per variant (per-variant batch sizes only)
    uint32_t beta_task;  // the task's batch position otherwise
};

__device__ __forceinline__ ChoiceDigits choice_digits(const DevProblem *P, int i, uint32_t c) {
    const int K = P->K[i];
    const bool pv = P->pv_batch != 0;
    const uint32_t nb = static_cast<uint32_t>(P->nb[i]);
    ChoiceDigits d;
    d.digits = 0;
    d.betas = 0;
    for (int k = 0; k < K; k++) {
        const uint32_t radix = P->radix[i][k];
        const uint32_t q = c / radix;
        const uint32_t g = c - q * radix;
        c = q;
        uint32_t x = g;
        if (pv) {
            x = g == 0 ? 0u : (g - 1) / nb + 1;
            d.betas |= (g == 0 ? 0u : (g - 1) % nb) << (4 * k);
        }
        d.digits |= static_cast<uint64_t>(x) << (8 * k);
    }
    d.beta_task = c;
    return d;
}

// The part of task i's requests that each variant serves under choice c at demand dn (the first hosted one
// serves "all" of no demand).  share is written with constant subscripts only, so that it stays in registers.
__device__ __forceinline__ void choice_shares(const DevProblem *P, int i, uint32_t c, int64_t dn,
                                              float (&share)[kMaxVariants]) {
    const int K = P->K[i];
    const bool pv = P->pv_batch != 0;
    const ChoiceDigits d = choice_digits(P, i, c);
    int64_t rem = dn;
    bool any = false;
#pragma unroll
    for (int k = 0; k < kMaxVariants; k++) share[k] = 0.0f;
    for (int r = 0; r < K; r++) {
        const int k = P->order[i][r];
        const int64_t x = static_cast<int64_t>((d.digits >> (8 * k)) & 0xff);
        const uint32_t beta = pv ? (d.betas >> (4 * k)) & 0xf : d.beta_task;
        const int64_t cap = x * P->thr_s[i][k][beta];
        const int64_t routed = rem < cap ? rem : cap;
        const bool in_use = x > 0 && (routed > 0 || !any);
        const float part = dn > 0 ? static_cast<float>(static_cast<double>(routed) / static_cast<double>(dn)) : 1.0f;
#pragma unroll
        for (int kk = 0; kk < kMaxVariants; kk++) share[kk] = (in_use && kk == k) ? part : share[kk];
        rem -= routed;
        any = any || x > 0;
    }
}

// ---- eq. (7) on the variant paths with traffic ---------------------------------------------------------------
// The latency of a variant path (eq. (6)) counts when the path carries requests (Table 1's I(p)): the
// frontend reaches the root's variant and every variant on the path sends some of its requests to the
// next one under Algorithm 1.  The walk is path_level's, with the latency so far in place of c(p): a
// downstream variant is reached when its interval of the request stream overlaps the interval that holds
// the upstream variant's requests; a variant that sends nothing (only at zero demand) hands on to the
// first hosted variant.  worst: the largest latency met at the leaf.
struct LatencyWalk {
    const DevProblem *P;
    int leaf;
    uint32_t c[kMaxTasks];
    int64_t dn[kMaxTasks];
    int64_t worst;
};

template <int J, int MAXD>
__device__ void latency_level(LatencyWalk &X, int64_t lo, int64_t len, int64_t lat) {
    const DevProblem *P = X.P;
    const int i = P->leaf_path[X.leaf][J];
    const int K = P->K[i];
    const bool pv = P->pv_batch != 0, has_vf = P->has_vf != 0;
    const ChoiceDigits d = choice_digits(P, i, pick32(X.c, i));
    const int64_t dn = pick_below(X.dn, i, kMaxTasks);
    const bool last = J == P->path_len[X.leaf] - 1;
    const int next = last ? 0 : P->leaf_path[X.leaf][J + 1 < MAXD ? J + 1 : J];
    const int64_t fan = last ? 0 : static_cast<int64_t>(P->fanout[next]);
    int64_t at = 0, made = 0;
    bool any = false;
    for (int r = 0; r < K; r++) {
        const int k = P->order[i][r];
        const int64_t x = static_cast<int64_t>((d.digits >> (8 * k)) & 0xff);
        if (x == 0) continue;
        const uint32_t beta = pv ? (d.betas >> (4 * k)) & 0xf : d.beta_task;
        const int64_t cap = x * P->thr_s[i][k][beta];
        const int64_t room = dn - at;
        const int64_t routed = room < cap ? room : cap;
        bool reached;
        if (len > 0) {
            const int64_t hi_a = at + routed, hi_b = lo + len;
            reached = (hi_a < hi_b ? hi_a : hi_b) > (at > lo ? at : lo);
        } else {
            reached = !any;
        }
        any = true;
        const int64_t out = has_vf ? routed * static_cast<int64_t>(P->vf[i][k]) : routed;
        if (reached) {
            const int64_t l = lat + static_cast<int64_t>(P->lat[i][k][beta]);  // l(i,k) at the configured batch size
            if (last) {
                X.worst = l > X.worst ? l : X.worst;
            } else {
                if constexpr (J + 1 < MAXD) latency_level<J + 1, MAXD>(X, made * fan, out * fan, l);
            }
        }
        at += routed;
        made += out;
    }
}

// True when some variant path with traffic of a plan that hosts every task and serves all demand exceeds
// its budget (budget[leaf]: the halved SLO less the communication latency of the leaf's chain, negative when
// nothing is left).  Dn as for path_objective.
template <int MAXD>
__device__ __noinline__ bool some_path_too_slow(const DevProblem *P, const uint32_t (&c)[kMaxTasks], const int64_t *Dn,
                                                const int64_t *budget) {
    LatencyWalk X;
    X.P = P;
    const int n = P->n_tasks;
    const bool has_vf = P->has_vf != 0;
    int64_t out[kMaxTasks];
#pragma unroll
    for (int i = 0; i < kMaxTasks; i++) {
        X.c[i] = c[i];
        X.dn[i] = 0;
        out[i] = 0;
    }
#pragma unroll
    for (int i = 0; i < kMaxTasks; i++) {
        if (i < n) {
            int64_t dn = Dn[i];
            if (has_vf) {
                if (i > 0) dn = pick_below(out, P->parent[i], i) * static_cast<int64_t>(P->fanout[i]);
                TaskOut o;
                eval_task_any(P, i, c[i], dn, o);
                out[i] = o.outflow;
            }
            X.dn[i] = dn;
        }
    }
    bool slow = false;
    for (int leaf = 0; leaf < n; leaf++) {
        if (!P->is_leaf[leaf]) continue;
        if (budget[leaf] < 0) {
            slow = true;
            continue;
        }
        X.leaf = leaf;
        X.worst = 0;
        latency_level<0, MAXD>(X, 0, X.dn[0], 0);
        if (X.worst > budget[leaf]) slow = true;
    }
    return slow;
}

// The part of that objective that belongs to one leaf, the sum over the variant paths of the task path
// root..leaf, depends on the choices of the tasks on that path only, so a search may form it once for all the
// plans that share them.  It is taken in two steps.  path_prefixes expands the walk level by level for every
// task of the path but the leaf: the branches with a nonzero share, in the nested order of path_level (an
// order-preserving expansion of a list keeps that order), each with what the leaf's level needs of it.
// leaf_level_sum then adds up the leaf's own level over those branches, for one choice of the leaf.
struct PathPrefix {
    int64_t lo, len;   // the interval of the leaf's request stream that holds this branch's requests
    double mass;       // c(p) up to here
    uint32_t entry;    // position in the leaf's table so far
    uint32_t pad;
};

// One thread.  c: the plan's choices (only those of the path's tasks above the leaf are read); Dn: the
// demands of the point (only Dn[0] with per-variant factors, where a task's demand is what its parent's part
// of the plan creates, eq. (1)).  tmp, out: kMaxPrefix entries each; the branches end up in out.  Returns their
// number; dn_leaf: the leaf's demand, stride_leaf: the table stride of the leaf's variant.
__device__ __noinline__ int path_prefixes(const DevProblem *P, int leaf, const uint32_t (&c)[kMaxTasks], const int64_t *Dn,
                                          PathPrefix *tmp, PathPrefix *out, int64_t &dn_leaf, uint32_t &stride_leaf) {
    const bool pv = P->pv_batch != 0, has_vf = P->has_vf != 0;
    const int levels = P->path_len[leaf] - 1;   // at least one: the leaf is not the root
    int n = 1;
    int64_t dn = Dn[0];
    uint32_t stride = 1;
    PathPrefix *from = nullptr;
    for (int J = 0; J < levels; J++) {
        const int i = P->leaf_path[leaf][J], next = P->leaf_path[leaf][J + 1];
        const int K = P->K[i];
        const int64_t fan = static_cast<int64_t>(P->fanout[next]);
        const ChoiceDigits d = choice_digits(P, i, pick32(c, i));
        PathPrefix *to = ((levels - 1 - J) & 1) ? tmp : out;
        int m = 0;
        int64_t created = 0;
        for (int q = 0; q < n; q++) {
            PathPrefix up;   // the whole stream at the root
            up.lo = 0;
            up.len = dn;
            up.mass = 0.0;
            up.entry = 0;
            if (J > 0) up = from[q];
            int64_t at = 0, made = 0;
            bool any = false;
            for (int r = 0; r < K; r++) {
                const int k = P->order[i][r];
                const int64_t x = static_cast<int64_t>((d.digits >> (8 * k)) & 0xff);
                if (x == 0) continue;
                const uint32_t beta = pv ? (d.betas >> (4 * k)) & 0xf : d.beta_task;
                const int64_t cap = x * P->thr_s[i][k][beta];
                const int64_t room = dn - at;
                const int64_t routed = room < cap ? room : cap;
                double share;
                if (up.len > 0) {
                    const int64_t hi_a = at + routed, hi_b = up.lo + up.len;
                    const int64_t ov = (hi_a < hi_b ? hi_a : hi_b) - (at > up.lo ? at : up.lo);
                    share = ov > 0 ? static_cast<double>(ov) / static_cast<double>(up.len) : 0.0;
                } else {
                    share = any ? 0.0 : 1.0;
                }
                any = true;
                const int64_t sent = has_vf ? routed * static_cast<int64_t>(P->vf[i][k]) : routed;
                if (share != 0.0 && m < kMaxPrefix) {
                    PathPrefix b;
                    b.lo = made * fan;
                    b.len = sent * fan;
                    b.mass = J == 0 ? share : up.mass * share;
                    b.entry = up.entry + static_cast<uint32_t>(k) * stride;
                    b.pad = 0;
                    to[m++] = b;
                }
                at += routed;
                made += sent;
            }
            created = made;
        }
        dn = has_vf ? created * fan : Dn[next];
        stride *= static_cast<uint32_t>(K);
        from = to;
        n = m;
    }
    dn_leaf = dn;
    stride_leaf = stride;
    return n;
}

// tab: the leaf's table; i, c: the leaf and its choice; dn: its demand; recs[0..n): the branches above it.
__device__ __noinline__ double leaf_level_sum(const DevProblem *P, const double *tab, int i, uint32_t c, int64_t dn,
                                              const PathPrefix *recs, int n, uint32_t stride) {
    const bool pv = P->pv_batch != 0;
    const int K = P->K[i];
    const ChoiceDigits d = choice_digits(P, i, c);
    double sum = 0.0;
    for (int q = 0; q < n; q++) {
        const PathPrefix up = recs[q];
        int64_t at = 0;
        bool any = false;
        for (int r = 0; r < K; r++) {
            const int k = P->order[i][r];
            const int64_t x = static_cast<int64_t>((d.digits >> (8 * k)) & 0xff);
            if (x == 0) continue;
            const uint32_t beta = pv ? (d.betas >> (4 * k)) & 0xf : d.beta_task;
            const int64_t cap = x * P->thr_s[i][k][beta];
            const int64_t room = dn - at;
            const int64_t routed = room < cap ? room : cap;
            double share;
            if (up.len > 0) {
                const int64_t hi_a = at + routed, hi_b = up.lo + up.len;
                const int64_t ov = (hi_a < hi_b ? hi_a : hi_b) - (at > up.lo ? at : up.lo);
                share = ov > 0 ? static_cast<double>(ov) / static_cast<double>(up.len) : 0.0;
            } else {
                share = any ? 0.0 : 1.0;
            }
            any = true;
            if (share != 0.0) {
                const double m = up.mass * share;
                sum = sum + m * tab[up.entry + static_cast<uint32_t>(k) * stride];
            }
            at += routed;
        }
    }
    return sum;
}

// ---- ordering and reductions -----------------------------------------------------------------------
// Strict total order on found plans: accuracy desc, workers asc (unless tie_index_only), index asc.
// A record with acc < 0 means "nothing found" and loses to everything.
__device__ __forceinline__ bool better(double acc, int32_t w, uint64_t idx, double bacc, int32_t bw, uint64_t bidx,
                                       bool tie_index_only) {
    if (acc > bacc) return true;
    if (acc < bacc) return false;
    if (!tie_index_only) {
        if (w < bw) return true;
        if (w > bw) return false;
    }
    return idx < bidx;
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp32(uint32_t v) {
    return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, 0xf, 0xf, false));
}

// Exchange step s of the wavefront butterfly: steps 0-3 stay inside a row of 16
// lanes and use DPP controls (quad_perm [1,0,3,2], quad_perm [2,3,0,1],
// row_half_mirror, row_mirror); steps 4-5 cross rows through ds_bpermute.
template <int STEP>
__device__ __forceinline__ uint32_t wave_xchg(uint32_t v) {
    if constexpr (STEP == 0) return dpp32<0xB1>(v);
    if constexpr (STEP == 1) return dpp32<0x4E>(v);
    if constexpr (STEP == 2) return dpp32<0x141>(v);
    if constexpr (STEP == 3) return dpp32<0x140>(v);
    if constexpr (STEP == 4) return static_cast<uint32_t>(__shfl_xor(static_cast<int>(v), 16, 64));
    return static_cast<uint32_t>(__shfl_xor(static_cast<int>(v), 32, 64));
}

template <int STEP>
__device__ __forceinline__ void wave_best_step(double &acc, int32_t &w, uint64_t &idx, bool tie_index_only) {
    const uint64_t ab = static_cast<uint64_t>(__double_as_longlong(acc));
    const uint64_t oab = (static_cast<uint64_t>(wave_xchg<STEP>(static_cast<uint32_t>(ab >> 32))) << 32) |
                         wave_xchg<STEP>(static_cast<uint32_t>(ab));
    const uint64_t oidx = (static_cast<uint64_t>(wave_xchg<STEP>(static_cast<uint32_t>(idx >> 32))) << 32) |
                          wave_xchg<STEP>(static_cast<uint32_t>(idx));
    const int32_t ow = static_cast<int32_t>(wave_xchg<STEP>(static_cast<uint32_t>(w)));
    const double oacc = __longlong_as_double(static_cast<long long>(oab));
    if (better(oacc, ow, oidx, acc, w, idx, tie_index_only)) {
        acc = oacc;
        w = ow;
        idx = oidx;
    }
}

// After this every lane of the wavefront holds the wavefront's best record.
// Must be called by all 64 lanes.
__device__ __forceinline__ void wave_best(double &acc, int32_t &w, uint64_t &idx, bool tie_index_only) {
    wave_best_step<0>(acc, w, idx, tie_index_only);
    wave_best_step<1>(acc, w, idx, tie_index_only);
    wave_best_step<2>(acc, w, idx, tie_index_only);
    wave_best_step<3>(acc, w, idx, tie_index_only);
    wave_best_step<4>(acc, w, idx, tie_index_only);
    wave_best_step<5>(acc, w, idx, tie_index_only);
}

__device__ __forceinline__ uint64_t wave_sum(uint64_t v) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t lo = static_cast<uint32_t>(__shfl_xor(static_cast<int>(static_cast<uint32_t>(v)), off, 64));
        const uint32_t hi = static_cast<uint32_t>(__shfl_xor(static_cast<int>(static_cast<uint32_t>(v >> 32)), off, 64));
        v += (static_cast<uint64_t>(hi) << 32) | lo;
    }
    return v;
}

// v_max_f64 as it stands, for operands known to be numbers.
__device__ __forceinline__ double max_f64_instruction(double x, double y) {
    double r;
    asm("v_max_f64 %0, %1, %2" : "=v"(r) : "v"(x), "v"(y));
    return r;
}

// Largest value of a wavefront, in every lane.  Must be called by all 64 lanes.
template <int STEP>
__device__ __forceinline__ double wave_max_f64_step(double v) {
    const uint64_t b = static_cast<uint64_t>(__double_as_longlong(v));
    const uint64_t o = (static_cast<uint64_t>(wave_xchg<STEP>(static_cast<uint32_t>(b >> 32))) << 32) |
                       wave_xchg<STEP>(static_cast<uint32_t>(b));
    return __builtin_fmax(v, __longlong_as_double(static_cast<long long>(o)));
}
__device__ __forceinline__ double wave_max_f64(double v) {
    v = wave_max_f64_step<0>(v);
    v = wave_max_f64_step<1>(v);
    v = wave_max_f64_step<2>(v);
    v = wave_max_f64_step<3>(v);
    v = wave_max_f64_step<4>(v);
    return wave_max_f64_step<5>(v);
}

template <int STEP>
__device__ __forceinline__ uint32_t wave_min_u32_step(uint32_t v) {
    const uint32_t o = wave_xchg<STEP>(v);
    return o < v ? o : v;
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
    v = wave_min_u32_step<0>(v);
    v = wave_min_u32_step<1>(v);
    v = wave_min_u32_step<2>(v);
    v = wave_min_u32_step<3>(v);
    v = wave_min_u32_step<4>(v);
    return wave_min_u32_step<5>(v);
}

// Among plans of equal objective: the first in the order (workers unless tie_index_only, then the last
// task's choice, then the rest of the index), in every lane.  "Nothing yet" is (kNever, ~0, ~0) and loses.
template <int STEP>
__device__ __forceinline__ void wave_first_step(int32_t &w, uint32_t &cl, uint64_t &low, bool tie_index_only) {
    const int32_t ow = static_cast<int32_t>(wave_xchg<STEP>(static_cast<uint32_t>(w)));
    const uint32_t ocl = wave_xchg<STEP>(cl);
    const uint64_t olow = (static_cast<uint64_t>(wave_xchg<STEP>(static_cast<uint32_t>(low >> 32))) << 32) |
                          wave_xchg<STEP>(static_cast<uint32_t>(low));
    bool take = (ocl < cl) | ((ocl == cl) & (olow < low));
    if (!tie_index_only) take = (ow < w) | ((ow == w) & take);
    if (take) {
        w = ow;
        cl = ocl;
        low = olow;
    }
}
__device__ __forceinline__ void wave_first(int32_t &w, uint32_t &cl, uint64_t &low, bool tie_index_only) {
    wave_first_step<0>(w, cl, low, tie_index_only);
    wave_first_step<1>(w, cl, low, tie_index_only);
    wave_first_step<2>(w, cl, low, tie_index_only);
    wave_first_step<3>(w, cl, low, tie_index_only);
    wave_first_step<4>(w, cl, low, tie_index_only);
    wave_first_step<5>(w, cl, low, tie_index_only);
}

// Block-level merge of per-wavefront records and store of one BestRec.
// nfeas is the wavefront's total (uniform across its lanes).
__device__ __forceinline__ void block_store_best(double acc, int32_t w, uint64_t idx, uint64_t nfeas, bool tie_index_only,
                                                 BestRec *sBest, BestRec *dst) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    wave_best(acc, w, idx, tie_index_only);
    if (lane == 0) {
        sBest[wave].acc = acc;
        sBest[wave].idx = idx;
        sBest[wave].w = w;
        sBest[wave].nfeas = nfeas;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        BestRec b = sBest[0];
        for (int v = 1; v < static_cast<int>(blockDim.x >> 6); v++) {
            b.nfeas += sBest[v].nfeas;
            if (better(sBest[v].acc, sBest[v].w, sBest[v].idx, b.acc, b.w, b.idx, tie_index_only)) {
                b.acc = sBest[v].acc;
                b.w = sBest[v].w;
                b.idx = sBest[v].idx;
            }
        }
        b.found = b.acc >= 0.0 ? 1 : 0;
        *dst = b;
    }
}

// ---- kernel: score every choice of every task, per demand point ----------------------------------------
__global__ void __launch_bounds__(kBlockThreads) task_table_kernel(SearchArgs A) {
    __shared__ DevProblem sP;
    stage_problem(&sP, A.P, sizeof(DevProblem));
    __syncthreads();
    const uint32_t t = blockIdx.x * kBlockThreads + threadIdx.x;
    const int m = blockIdx.y;
    if (t == 0) A.floor[m] = 0;  // largest key reported by a block of this point so far: none yet
    if (t >= sP.table_total) return;
    int i = sP.n_tasks - 1;
    while (i > 0 && t < sP.table_off[i]) i--;
    const uint32_t c = t - sP.table_off[i];
    const int64_t Dn = A.Dn[static_cast<size_t>(m) * kMaxTasks + i];
    TaskOut o;
    eval_task_any(&sP, i, c, Dn, o);
    TaskRec rec;
    // (A.prune: the objective comes from profiled path accuracies and an upper bound on it wants the variants in
    // use of every choice; the accuracy is not read then and its field carries the bit mask as a number)
    rec.a = A.prune ? static_cast<double>(o.used) : task_accuracy(o, Dn);
    rec.w = o.w;
    bool usable = o.any && o.rem == 0;
    // class by class: only the choices that create the class's amount of requests belong to the point
    if (A.class_amount) {
        const int64_t amount = A.class_amount[static_cast<size_t>(m) * kMaxTasks + i];
        if (amount >= 0) usable = usable && o.outflow == amount;
    }
    rec.lat = usable ? static_cast<int32_t>(o.maxlat) : kNever;
    A.table[static_cast<size_t>(m) * sP.table_total + t] = rec;
    if (A.lat2) {
        TaskLat2 l2;
        l2.top = usable ? o.lat_top : kNever;
        l2.bot = usable ? o.lat_bot : kNever;
        A.lat2[static_cast<size_t>(m) * sP.table_total + t] = l2;
    }
}

// ---- kernel: order the first task's choices into runs of equal (feasible, replicas, latency) ------------
// Everything the combine kernel derives from a first-task choice besides its
// accuracy depends only on that triple, so plans visited in this order share
// their feasibility masks over a whole run.  One block per demand point: a
// counting sort with the histogram in LDS.  The latency of a choice is one of
// the task's profiled latencies, so (replicas, rank of the latency) numbers the
// buckets; unusable choices share the last bucket.  With more buckets than fit,
// the identity order with runs of length one is used instead.
constexpr uint32_t kMaxBuckets = 4096;
constexpr int kSortThreads = 1024;

// w_free: the largest replica count of the first task with which the worker budget (eq. (3)) can
// never bind, whatever the other tasks choose (negative: none).  Choices at or below it leave the
// last task the same feasibility masks, so they share a bucket per latency; the workers of a
// winning plan are taken from its own entry, not from the run.
// lat_sorted: the task's distinct latencies, ascending (in LDS: every choice looks all of them up, and the
// count below has no dependent reads).
__device__ __forceinline__ uint32_t root_bucket(const int32_t *lat_sorted, uint32_t n_lat, const TaskRec &rec,
                                                uint32_t n_buckets, int32_t w_free) {
    if (rec.lat == kNever) return n_buckets - 1;
    uint32_t rank = 0;  // number of latencies below this one, the last one left out
    for (uint32_t q = 0; q + 1 < n_lat; q++) rank += lat_sorted[q] < rec.lat ? 1u : 0u;
    const int32_t wk = w_free < 0 ? rec.w : (rec.w > w_free ? rec.w - w_free : 0);
    // latency first, replicas ascending within a latency: consecutive runs of one latency differ only in
    // the workers they leave, and those that leave more than the last task can ever host look alike to it
    return rank * ((n_buckets - 1) / n_lat) + static_cast<uint32_t>(wk);
}

// Without swapped roles one launch row: the first task's choices into A.perm / A.run_end.  With swapped
// roles blockIdx.y is the task: the tile task's choices go into runs (A.perm_all at the task's offset,
// A.run_end_t), every other task's choices are only split into usable ones first and the rest.
__global__ void __launch_bounds__(kSortThreads) root_order_kernel(SearchArgs A) {
    __shared__ uint32_t sHist[kMaxBuckets];   // counts, then next free position per bucket
    __shared__ uint32_t sEnd[kMaxBuckets];    // end position per bucket
    __shared__ uint32_t sWaveTot[kSortThreads / 64];
    const int m = blockIdx.x;
    const DevProblem *P = A.P;
    const int task = A.swap ? static_cast<int>(blockIdx.y) : 0;
    const bool tile = A.swap && task == P->tile_task;
    const bool runs = !A.swap || tile;
    const uint32_t C0 = P->C[task];
    const TaskRec *tab = A.table + static_cast<size_t>(m) * P->table_total + P->table_off[task];
    uint32_t *perm = A.swap ? A.perm_all + static_cast<size_t>(m) * P->table_total + P->table_off[task]
                            : A.perm + static_cast<size_t>(m) * C0;
    uint32_t *run_end = A.swap ? (tile ? A.run_end_t + static_cast<size_t>(m) * C0 : nullptr)
                               : A.run_end + static_cast<size_t>(m) * C0;
    const uint32_t n_lat = static_cast<uint32_t>(tile ? P->n_lat_t : P->n_lat0);
    __shared__ int32_t sLat[kMaxVariants * kMaxBatches];
    if (threadIdx.x < n_lat) sLat[threadIdx.x] = tile ? P->lat_t_sorted[threadIdx.x] : P->lat0_sorted[threadIdx.x];
    const int32_t *lat_sorted = sLat;  // (visible after the barrier that follows the histogram's reset)
    const int32_t w_free = tile ? A.w_free_t : A.w_free;
    const uint32_t n_buckets = runs ? static_cast<uint32_t>((tile ? P->sum_r_t : P->sum_r0) + 1) * n_lat + 1 : 2u;
    auto bucket_of = [&](const TaskRec &rec) -> uint32_t {
        if (!runs) return rec.lat == kNever ? 1u : 0u;
        return root_bucket(lat_sorted, n_lat, rec, n_buckets, w_free);
    };
    if (n_buckets > kMaxBuckets) {  // (never with swapped roles: the host checks the tile task's buckets)
        for (uint32_t r = threadIdx.x; r < C0; r += kSortThreads) {
            perm[r] = r;
            if (run_end) run_end[r] = r + 1;
        }
        return;
    }
    for (uint32_t b = threadIdx.x; b < kMaxBuckets; b += kSortThreads) sHist[b] = 0;
    __syncthreads();
    for (uint32_t r = threadIdx.x; r < C0; r += kSortThreads) atomicAdd(&sHist[bucket_of(tab[r])], 1u);
    __syncthreads();
    // exclusive prefix sum over the buckets: each thread owns kMaxBuckets / kSortThreads consecutive ones
    constexpr uint32_t kPer = kMaxBuckets / kSortThreads;
    uint32_t cnt[kPer], local = 0;
#pragma unroll
    for (uint32_t q = 0; q < kPer; q++) {
        cnt[q] = sHist[threadIdx.x * kPer + q];
        local += cnt[q];
    }
    uint32_t incl = local;
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t up = static_cast<uint32_t>(__shfl_up(static_cast<int>(incl), off, 64));
        if (static_cast<int>(threadIdx.x & 63) >= off) incl += up;
    }
    if ((threadIdx.x & 63) == 63) sWaveTot[threadIdx.x >> 6] = incl;
    __syncthreads();
    uint32_t pos = incl - local;
    for (uint32_t v = 0; v < (threadIdx.x >> 6); v++) pos += sWaveTot[v];
#pragma unroll
    for (uint32_t q = 0; q < kPer; q++) {
        sHist[threadIdx.x * kPer + q] = pos;
        pos += cnt[q];
        sEnd[threadIdx.x * kPer + q] = pos;
    }
    __syncthreads();
    for (uint32_t r = threadIdx.x; r < C0; r += kSortThreads) {
        const uint32_t b = bucket_of(tab[r]);
        const uint32_t at = atomicAdd(&sHist[b], 1u);  // order inside a bucket is immaterial
        perm[at] = r;
        if (run_end) run_end[at] = sEnd[b];
    }
}

// ---- kernel: visit every plan, combining the per-task records -------------------------------------------
// Work item = (group of chunks of the last task's choices, combination f of the
// tasks strictly between the first and the last, tile of the first task's choices
// in run order).  A wavefront keeps S*64 records of the last task in registers;
// the block builds the MidVal/MidLim of every first-task choice in the tile once, then
// each wavefront walks its part of the tile.  Per run (same latency left, and the same workers
// left or more than the last task can ever use) it takes the feasibility of its S*64 plans
// once (eq. (3), eq. (7)); per record it
// then only forms the S*64 objectives (one fp64 multiply, one add each) and keeps
// their running maximum.  That first pass leaves every lane with the largest key of its feasible
// plans; a second pass over the same work items, taken only by blocks whose largest key can still
// be the demand point's, settles which plan with that key comes first in the order (see the kernel).
//
// SWAP (per-variant factors class by class, three or more tasks): a point owns only a few
// choices of every task that has children, too few to fill a tile.  The tile then holds the choices of
// the first leaf (in their own run order), and every other task but the last is part of the work item:
// a task with children through the list of its choices that belong to the point, a leaf through all of
// its choices.  What an entry needs besides its own record is the same for the whole tile: the
// products and latency sums along the chains of the tile's and the last task's ancestors, and the path
// values of the other leaves.
//
// BY_LEAF (with SWAP, a leaf in the tiles, profiled path accuracies): the objective is the sum, in leaf
// order, of one value per leaf, and a leaf's value depends on the choices along its own task path only.
// Per work item one thread expands the branches above the tile leaf (path_prefixes; also above the last
// task when the choices of its ancestors have changed: they are the slowest digits of the work item) and
// forms the values of the item's other leaves; the tile leaf's value is then formed per entry when the tile
// is built and the last task's per lane and slot (leaf_level_sum).  `a` holds that value, the entries carry
// `pre` = 1, and the loop over the plans is the one of the product form.
template <int S, bool HAS_PRESUM, bool DIVIDE, bool RANGE, bool SWAP, bool BY_LEAF = false>
__global__ void __launch_bounds__(kBlockThreads) __attribute__((amdgpu_waves_per_eu(BY_LEAF ? 4 : 5)))
combine_kernel(SearchArgs A) {
    static_assert(!BY_LEAF || (SWAP && HAS_PRESUM), "path values per leaf need swapped roles and two leaves");
    constexpr uint32_t kHeadBytes = BY_LEAF ? sizeof(DevProblem) : offsetof(DevProblem, lat);
    // BY_LEAF: the branches above the tile leaf and above the last task, their number, the leaf's demand and
    // table stride ([0] tile leaf, [1] last task)
    __shared__ PathPrefix sTmp[BY_LEAF ? kMaxPrefix : 1], sAbove[2][BY_LEAF ? kMaxPrefix : 1];
    __shared__ int sAboveN[2];
    __shared__ int64_t sLeafDn[2];
    __shared__ uint32_t sLeafStride[2];
    __shared__ __attribute__((aligned(16))) unsigned char sPraw[kHeadBytes];
    __shared__ MidVal sVal[kMidTile + 4];  // four spare entries: the record fetch runs ahead of the run's end
    __shared__ MidLim sLim[kMidTile];
    __shared__ uint32_t sChoice[kMidTile];  // first-task choice of each tile entry (second pass only)
    __shared__ double sFac[64];             // the accuracies the path-value steps multiply by (per work item)
    __shared__ BestRec sBest[kWavesPerBlock];
    __shared__ double sTop[kWavesPerBlock][2];  // per wavefront: largest pre / presum of a tile; the largest key
    __shared__ uint32_t sGo;                    // the block takes the second pass
    __shared__ uint32_t sBlk;                   // second pass: fewest workers (order by index: lowest choice of the last
                                                // task) of the best plans the block's wavefronts have found so far
    DevProblem *sP = reinterpret_cast<DevProblem *>(sPraw);  // only the head is valid
    stage_problem(sP, A.P, kHeadBytes);
    __syncthreads();

    // Values that are the same in every lane are passed through readfirstlane so that the
    // compiler keeps them (and the loops they control) on the scalar unit.
    const int lane = threadIdx.x & 63;
    const int wave = uni(threadIdx.x >> 6);
    const int m = blockIdx.y;
    const int n = uni(sP->n_tasks), L = n - 1;
    const uint32_t CL = uni(sP->C[L]);
    const uint32_t C0 = n >= 2 ? uni(sP->C[0]) : 1u;
    // first-task choices to visit, in run order: all of them, or with classes those of this point's class
    // (the ordering kernel puts them first; the rest belong to other points)
    const uint32_t roots = A.class_count ? uni(A.class_count[static_cast<size_t>(m) * kMaxTasks]) : C0;
    // the task whose choices fill the tiles: the first one, or the first leaf
    const int T = SWAP ? uni(sP->tile_task) : 0;
    const uint32_t Cmid = SWAP ? uni(sP->C[T]) : C0;
    // SWAP: the tile task is the first leaf (all of its choices), or on a chain, which has no leaf to
    // spare, the last task's parent (its choices that belong to the point; perm_all lists them first)
    const bool tile_leaf = !SWAP || uni(sP->is_leaf[T]) != 0;
    const uint32_t mid_count =
        SWAP ? (tile_leaf ? Cmid : uni(A.class_count[static_cast<size_t>(m) * kMaxTasks + T])) : roots;
    const uint64_t strideL = uni64(sP->stride[L]);
    const TaskRec *tab = A.table + static_cast<size_t>(m) * uni(sP->table_total);
    const TaskRec *tabL = tab + uni(sP->table_off[L]);
    const TaskRec *tabM = SWAP ? tab + uni(sP->table_off[T]) : tab;
    const uint32_t *perm_m = SWAP ? A.perm_all + static_cast<size_t>(m) * uni(sP->table_total) : nullptr;
    const uint32_t *perm = SWAP ? perm_m + uni(sP->table_off[T]) : A.perm + static_cast<size_t>(m) * C0;
    const uint32_t *run_end = SWAP ? A.run_end_t + static_cast<size_t>(m) * Cmid : A.run_end + static_cast<size_t>(m) * C0;
    // SWAP: how many choices each task of the work item ranges over for this point
    uint32_t cntj[kMaxTasks];
    uint64_t far_swap = 1;
#pragma unroll
    for (int j = 0; j < kMaxTasks; j++) {
        cntj[j] = 1;
        if (SWAP && j < L && j != T) {
            cntj[j] = uni(A.class_count[static_cast<size_t>(m) * kMaxTasks + j]);
            far_swap *= cntj[j];
        }
    }
    // SWAP: the last task's ancestors are the slowest digits of the work item
    uint32_t anc_last = 0;
    if (SWAP)
        for (int i = uni(sP->parent[L]); i >= 0; i = uni(sP->parent[i])) anc_last |= 1u << i;
    const bool tie_index_only = A.tie_index_only != 0;
    const double npd = static_cast<double>(uni(sP->n_paths));
    const int32_t W = A.W;

    const uint32_t cpb = A.cpb;
    const uint32_t chunk_in_group = wave % cpb, midpart = wave / cpb, mid_split = kWavesPerBlock / cpb;

    // SWAP: the number of work items depends on the point (its first-task choices times the rest)
    const uint64_t far_m = SWAP ? far_swap : A.far_span;
    const uint64_t items_m = SWAP ? static_cast<uint64_t>(A.chunk_groups) * far_m * A.mid_tiles : A.items;
    // Quotients of numbers that fit 32 bits are taken in 32 bits (a 64-bit division costs as much as
    // several tile records, and a block with few work items takes a dozen of them to find its place).
    const bool narrow = items_m <= 0xffffffffull && (SWAP || A.far_count <= 0xffffffffull);
    auto divmod = [&](uint64_t x, uint64_t y, uint64_t &quot, uint64_t &rem) {
        if (narrow) {
            const uint32_t x32 = static_cast<uint32_t>(x), y32 = static_cast<uint32_t>(y);
            const uint32_t q32 = x32 / y32;
            quot = q32;
            rem = x32 - q32 * y32;
        } else {
            quot = x / y;
            rem = x - quot * y;
        }
    };
    // the block's share of the work items: items_m / blocks each, the first items_m % blocks blocks one more
    uint64_t per_block = A.items_per_block, extra = A.items_extra;
    if (SWAP) divmod(items_m, A.blocks_per_m, per_block, extra);
    const uint64_t item_lo = per_block * blockIdx.x + (blockIdx.x < extra ? blockIdx.x : extra);
    const uint64_t item_hi = item_lo + per_block + (blockIdx.x < extra ? 1 : 0);

    double a[S];
    int32_t w[S], lat[S];
    // The block walks its work items twice.  The first pass keeps, per lane, nothing but the largest key
    // (path sum, or accuracy when DIVIDE) among its feasible plans -- no compare-and-branch in the loop
    // over the plans, so its cost does not depend on how many plans are feasible or tie -- and counts the
    // feasible plans.  The second pass, taken only by blocks whose largest key can still be the demand
    // point's, settles which of the plans that reach the block's largest key comes first in the order
    // (fewest workers, then lowest index); it skips whatever cannot hold such a plan.
    double bsum = -1.0;
    double gb = -1.0;       // second pass: the block's largest key
    bool lane_in = false;   // second pass: this lane reached it in the first pass
    // second pass: the best plan with that key this wavefront has seen (the same in every lane): workers, and
    // the index split into the last task's choice and the rest (index = rest + strideL * choice, rest < strideL)
    int32_t bw = kNever;
    uint32_t bcl = ~0u;
    uint64_t blow = ~0ull;
    uint64_t nfeas = 0;  // wavefront total
    uint32_t cur_group = ~0u;
    uint32_t cbase = 0;  // first choice of the last task in this wavefront's chunk
    uint32_t cl0 = 0;    // this lane's choice in slot 0
    // BY_LEAF: the choices of the last task's ancestors that `a` was formed for, and of the tile leaf's
    // ancestors that its branches were expanded for
    uint64_t last_for = ~0ull, tile_for = ~0ull;
    uint32_t anc_tile = 0;
    if (BY_LEAF)
        for (int i = uni(sP->parent[T]); i >= 0; i = uni(sP->parent[i])) anc_tile |= 1u << i;

    // Position of the first item in (tile r, digits of the tasks in between, chunk group g);
    // later items advance it like an odometer, so no division sits in the item loop.
    uint32_t r = 0, g = 0;
    uint32_t cj[kMaxTasks];  // choice of every task strictly between the first and the last
    uint64_t f = 0;          // those digits as one number: sum cj[j] * prod_{1<=i<j} C_i
    // With an index range only the combinations the range touches are visited: far_span of them,
    // cyclically from far_first (the whole space: all far_count from 0).
    auto locate = [&](uint64_t item) {
        uint64_t t, rr;
        divmod(item, A.mid_tiles, t, rr);
        r = uni(static_cast<uint32_t>(rr));
        if (SWAP) {
            // one digit per task of the work item: its position in the task's list for this point
            uint64_t rest, gg;
            divmod(t, far_m, gg, rest);
            g = uni(static_cast<uint32_t>(gg));
            f = 0;
#pragma unroll
            for (int j = 0; j < kMaxTasks; j++) cj[j] = 0;
#pragma unroll
            for (int pass = 0; pass < 2; pass++) {
#pragma unroll
                for (int j = 0; j < kMaxTasks; j++) {
                    if (j < L && j != T && ((anc_last >> j) & 1u) == static_cast<uint32_t>(pass)) {
                        uint64_t d;
                        divmod(rest, cntj[j], rest, d);
                        cj[j] = uni(perm_m[uni(sP->table_off[j]) + static_cast<uint32_t>(d)]);
                    }
                }
            }
            return;
        }
        uint64_t gg, ff;
        divmod(t, A.far_span, gg, ff);
        if (RANGE) ff = (A.far_first + ff) % A.far_count;  // (the whole space: far_first = 0, far_span = far_count)
        f = uni64(ff);
        g = uni(static_cast<uint32_t>(gg));
        uint64_t rest = f;
#pragma unroll
        for (int j = 1; j < kMaxTasks; j++) {
            cj[j] = 0;
            if (j < L) {
                uint64_t d;
                divmod(rest, uni(sP->C[j]), rest, d);
                cj[j] = uni(static_cast<uint32_t>(d));
            }
        }
        cj[0] = 0;
    };
    // the next item of the whole space (the tile, then the digits of the tasks in between, then the chunk group)
    auto advance = [&]() {
        if (++r == A.mid_tiles) {
            r = 0;
            ++f;
            bool carry = true;
#pragma unroll
            for (int j = 1; j < kMaxTasks; j++) {
                if (j < L && carry) {
                    if (++cj[j] == uni(sP->C[j])) {
                        cj[j] = 0;
                    } else {
                        carry = false;
                    }
                }
            }
            if (carry) {  // every digit wrapped (or there is none): next chunk group
                f = 0;
                ++g;
            }
        }
    };
    // settle_tag: std::false_type for the first pass, std::true_type for the second
    auto walk = [&](auto settle_tag) {
    constexpr bool SETTLE = decltype(settle_tag)::value;
    cur_group = ~0u;
    last_for = ~0ull;
    tile_for = ~0ull;
    if (item_lo < item_hi) locate(item_lo);
    for (uint64_t item = item_lo; item < item_hi; ++item) {
        if (g != cur_group) {
            cur_group = g;
            cbase = A.cl_first + (g * cpb + chunk_in_group) * (64u * S);
            cl0 = cbase + lane;
#pragma unroll
            for (int s = 0; s < S; s++) {
                const uint32_t cL = cl0 + s * 64;
                if (cL < CL) {
                    const TaskRec rec = tabL[cL];
                    a[s] = rec.a;
                    w[s] = rec.w;
                    lat[s] = rec.lat;
                } else {
                    a[s] = 0.0;
                    w[s] = 0;
                    lat[s] = kNever;
                }
            }
            last_for = ~0ull;
        }
        // What the tasks strictly between the first and the last contribute (the same for the
        // whole tile): replicas, feasibility, latency along each chain without the first task.
        int64_t flp[kMaxTasks];  // latency sum over root..j without the root
        int64_t w_far = 0;
        bool ok_far = true;
        int64_t lat0_cap = kNever - 1;  // largest first-task latency every other leaf's path tolerates
#pragma unroll
        for (int j = 0; j < kMaxTasks; j++) flp[j] = 0;
        int64_t tl_base = A.budget[L];  // latency left for the tile's task and the last task together
        double a_first = 1.0, a_last = 1.0;  // SWAP: products over the ancestors of the tile task and of the last task
        bool new_last = false;               // BY_LEAF: the last task's ancestors have changed, `a` is to be formed anew
        if (SWAP) {
            // every task of the work item, in topological order: replicas, products and latency sums along
            // the chains from the first task (eq. (12) root first, eq. (7)); a leaf closes its path
            double pp[kMaxTasks];
#pragma unroll
            for (int j = 0; j < kMaxTasks; j++) pp[j] = 0.0;
#pragma unroll
            for (int j = 0; j < kMaxTasks; j++) {
                if (j < L && j != T) {
                    const TaskRec rec = tab[sP->table_off[j] + cj[j]];
                    const int32_t rw = uni(rec.w), rlat = uni(rec.lat);
                    const double ra = __longlong_as_double(
                        static_cast<long long>(uni64(static_cast<uint64_t>(__double_as_longlong(rec.a)))));
                    w_far += rw;
                    ok_far = ok_far && rlat != kNever;
                    const int par = j > 0 ? uni(sP->parent[j]) : 0;
                    pp[j] = j == 0 ? ra : pick_below(pp, par, j) * ra;
                    flp[j] = (j == 0 ? 0 : pick_below(flp, par, j)) + rlat;   // here with the first task included
                    if (uni(sP->is_leaf[j])) {
                        ok_far = ok_far && A.budget[j] >= 0 && flp[j] <= A.budget[j];
                        if (!BY_LEAF && threadIdx.x == 0) sFac[j] = pp[j];   // the leaf's path value (published below)
                    }
                }
            }
            const int parT = uni(sP->parent[T]), parL = uni(sP->parent[L]);
            a_first = pick_below(pp, parT, kMaxTasks);    // product over the tile task's ancestors
            if (tile_leaf) {
                a_last = pick_below(pp, parL, kMaxTasks);     // product over the last task's ancestors
                lat0_cap = A.budget[T] < 0 ? -1 : A.budget[T] - pick_below(flp, parT, kMaxTasks);
                if (lat0_cap < 0) ok_far = false;
                tl_base = tl_base < 0 ? -1 : tl_base - pick_below(flp, parL, kMaxTasks);
            } else {
                // the tile task is the last task's parent: its accuracy and latency enter the last task's
                // path per entry, and it closes no path of its own
                tl_base = tl_base < 0 ? -1 : tl_base - pick_below(flp, parT, kMaxTasks);
            }
            if constexpr (BY_LEAF) {
                new_last = false;
                if (ok_far) {
                    uint64_t now_for = 0, now_tile = 0;
#pragma unroll
                    for (int j = 0; j < kMaxTasks; j++) {
                        if ((anc_last >> j) & 1u) now_for += cj[j] * uni64(sP->stride[j]);
                        if ((anc_tile >> j) & 1u) now_tile += cj[j] * uni64(sP->stride[j]);
                    }
                    new_last = now_for != last_for;
                    const bool new_tile = now_tile != tile_for;
                    last_for = now_for;
                    tile_for = now_tile;
                    if (threadIdx.x == 0) {
                        const int64_t *Dn = A.Dn + static_cast<size_t>(m) * kMaxTasks;
                        // the other leaves of the work item (their branches pass through the tile leaf's arrays)
                        bool others = false;
                        for (int j = 0; j < L; j++) {
                            if (j == T || !sP->is_leaf[j]) continue;
                            int64_t dn;
                            uint32_t st;
                            const int nb = path_prefixes(sP, j, cj, Dn, sTmp, sAbove[0], dn, st);
                            sFac[j] = leaf_level_sum(sP, A.path_acc + sP->path_off[j], j, pick32(cj, j), dn, sAbove[0], nb, st);
                            others = true;
                        }
                        if (new_tile || others)
                            sAboveN[0] = path_prefixes(sP, T, cj, Dn, sTmp, sAbove[0], sLeafDn[0], sLeafStride[0]);
                        if (new_last)
                            sAboveN[1] = path_prefixes(sP, L, cj, Dn, sTmp, sAbove[1], sLeafDn[1], sLeafStride[1]);
                    }
                }
            }
        } else {
#pragma unroll
            for (int j = 1; j < kMaxTasks; j++) {
                if (j < L) {
                    // the same record in every lane: through readfirstlane, so that the sums, limits and
                    // selections that follow stay on the scalar unit
                    const TaskRec rec = tab[sP->table_off[j] + cj[j]];
                    const int32_t rw = uni(rec.w), rlat = uni(rec.lat);
                    w_far += rw;
                    ok_far = ok_far && rlat != kNever;
                    flp[j] = pick_below(flp, uni(sP->parent[j]), j) + rlat;
                }
            }
#pragma unroll
            for (int j = 0; j < kMaxTasks; j++) {
                if (j < L && uni(sP->is_leaf[j])) {
                    const int64_t room = A.budget[j] < 0 ? -1 : A.budget[j] - flp[j];
                    if (room < lat0_cap) lat0_cap = room;
                }
            }
            if (lat0_cap < 0) ok_far = false;
            if (n >= 2) {
                const int parL = uni(sP->parent[L]);
                tl_base = tl_base < 0 ? -1 : tl_base - pick_below(flp, parL, kMaxTasks);
            }
        }
        const int64_t w_room = static_cast<int64_t>(W) - w_far;

        const uint32_t tile_base = r * A.tile_len;
        // (a point with few first-task choices may leave the later tiles of the launch empty)
        const uint32_t left = tile_base < mid_count ? mid_count - tile_base : 0u;
        const uint32_t cnt = left < A.tile_len ? left : A.tile_len;
        // index contribution of everything but the tile's task and the last one
        uint64_t base_f = static_cast<uint64_t>(C0) * f;
        if (SWAP) {
            base_f = 0;
#pragma unroll
            for (int j = 0; j < kMaxTasks; j++)
                if (j < L && j != T) base_f += cj[j] * uni64(sP->stride[j]);
        }

        // The accuracies the steps multiply by, one per step, for this combination of the tasks in
        // between.  (The factors of the previous item were last read before its tile was published.)
        if (SWAP) {
            // (the other leaves' path values were written to sFac above)
        } else if (threadIdx.x < static_cast<uint32_t>(sP->n_prog)) {
            const int t = sP->prog_task[threadIdx.x];
            if (t >= 0) sFac[threadIdx.x] = tab[sP->table_off[t] + pick32(cj, t)].a;
        }
        __syncthreads();  // the previous item's tile is no longer being read; the factors are visible
        if constexpr (SETTLE) {
            // Second pass: a work item none of whose plans can come before the best plan some wavefront of the
            // block has found is skipped as a whole.  sBlk changes only while tiles are walked, never between
            // this barrier and the next one, so every thread of the block decides alike.
            const uint32_t seen = sBlk;
            bool skip = !ok_far;
            if (tie_index_only) {
                // the lowest choice of the last task any wavefront of the block holds in this chunk group
                skip = skip || A.cl_first + g * cpb * (64u * S) > seen;
            } else {
                // every task hosts at least one replica in a feasible plan
                const int64_t least = w_far + (n >= 2 ? 2 : 1);
                skip = skip || least > static_cast<int64_t>(seen);
            }
            if (skip) {
                if (BY_LEAF && new_last) last_for = ~0ull;  // the lane values were not formed for these ancestors
                if (RANGE || SWAP) {
                    if (item + 1 < item_hi) locate(item + 1);
                } else {
                    advance();
                }
                continue;
            }
        }
        if constexpr (BY_LEAF) {
            if (new_last) {
                // the last task's value of every lane and slot
                const double *tabL_acc = A.path_acc + uni(sP->path_off[L]);
#pragma unroll
                for (int s = 0; s < S; s++) {
                    a[s] = 0.0;
                    if (lat[s] != kNever)
                        a[s] = leaf_level_sum(sP, tabL_acc, L, cl0 + s * 64, sLeafDn[1], sAbove[1], sAboveN[1],
                                              sLeafStride[1]);
                }
            }
        }
        // Every thread builds its entries of the tile two at a time, side by side: the steps are read once
        // per pair and applied to both.
        constexpr int kSide = 2;
        double top_pre = 0.0, top_presum = 0.0;  // second pass: largest values among this thread's usable entries
        for (uint32_t e_first = threadIdx.x; e_first < cnt; e_first += kSide * kBlockThreads) {
            uint32_t cMs[kSide];
            double a0s[kSide], val[kSide], presum[kSide], pre[kSide];
            int32_t w0s[kSide], lat0s[kSide];
            bool oks[kSide];
#pragma unroll
            for (int k = 0; k < kSide; k++) {
                const uint32_t e = e_first + k * kBlockThreads;
                cMs[k] = 0;
                a0s[k] = 1.0;
                w0s[k] = 0;
                lat0s[k] = 0;
                oks[k] = ok_far;
                if (n >= 2 && e < cnt) {
                    cMs[k] = perm[tile_base + e];
                    const TaskRec rec = tabM[cMs[k]];
                    a0s[k] = rec.a;
                    w0s[k] = rec.w;
                    lat0s[k] = rec.lat;
                    oks[k] = ok_far && rec.lat != kNever && static_cast<int64_t>(rec.lat) <= lat0_cap;
                }
                val[k] = a0s[k];
                presum[k] = 0.0;
                pre[k] = 1.0;
            }
            // path values root first (eq. (12) objective, product stand-in): value = a_0 * a_j1 * a_j2 ...
            if (SWAP) {
                // leaves in ascending order: the tile task (the first leaf, the entry's own), then the
                // other leaves of the work item; the last task's path value is added per plan
                bool none = !tile_leaf;   // no path value in the sum yet
#pragma unroll
                for (int k = 0; k < kSide; k++) {
                    presum[k] = tile_leaf ? a_first * a0s[k] : 0.0;
                    pre[k] = tile_leaf ? a_last : a_first * a0s[k];
                    if constexpr (BY_LEAF) {
                        // the entry's own value, for entries some plan can use
                        presum[k] = 0.0;
                        pre[k] = 1.0;
                        if (oks[k] && w_room >= static_cast<int64_t>(w0s[k]) && e_first + k * kBlockThreads < cnt)
                            presum[k] = leaf_level_sum(sP, A.path_acc + uni(sP->path_off[T]), T, cMs[k], sLeafDn[0],
                                                       sAbove[0], sAboveN[0], sLeafStride[0]);
                    }
                }
                for (int j = 0; j < L; j++) {
                    if (j == T || !uni(sP->is_leaf[j])) continue;
                    const double v = sFac[j];
#pragma unroll
                    for (int k = 0; k < kSide; k++) presum[k] = none ? v : presum[k] + v;
                    none = false;
                }
            }
            bool first = true;
            const int n_prog = SWAP ? 0 : uni(sP->n_prog);
            for (int q = 0; q < n_prog; q++) {
                // one step, written without branches: what a step of another kind would have computed is
                // formed too and dropped (only a multiply step's slot of sFac holds a value)
                const int op = uni(static_cast<int>(sP->prog_op[q]));
                const bool is_mul = op == kStepMul, is_leaf = op == kStepLeaf, is_pre = op == kStepPre;
                const double fac = sFac[q];
#pragma unroll
                for (int k = 0; k < kSide; k++) {
                    const double prod = val[k] * fac;
                    const double sum = first ? val[k] : presum[k] + val[k];
                    presum[k] = is_leaf ? sum : presum[k];
                    pre[k] = is_pre ? val[k] : pre[k];
                    val[k] = is_mul ? prod : a0s[k];
                }
                first = first && !is_leaf;
            }
#pragma unroll
            for (int k = 0; k < kSide; k++) {
                const uint32_t e = e_first + k * kBlockThreads;
                if (e < cnt) {
                    MidVal uv;
                    MidLim ul;
                    uv.pre = pre[k];
                    uv.presum = presum[k];
                    // (SWAP with a leaf in the tiles: the entry's task is not on the last task's path)
                    int64_t tl = tl_base < 0 ? -1 : tl_base - ((SWAP && tile_leaf) ? 0 : static_cast<int64_t>(lat0s[k]));
                    if (tl < 0) tl = -1;
                    if (tl > kNever - 1) tl = kNever - 1;
                    ul.tl = static_cast<int32_t>(tl);
                    const int64_t wr = w_room - static_cast<int64_t>(w0s[k]);
                    ul.w_rem = (oks[k] && wr >= 0) ? static_cast<int32_t>(wr) : -1;
                    // without a range every choice of the last task is admissible and the slot carries the
                    // end of the entry's run instead (tile relative; a run may go on beyond the tile)
                    ul.cl_lo = n >= 2 ? run_end[tile_base + e] - tile_base : e + 1;
                    ul.cl_cnt = CL;
                    if (RANGE) {
                        // index of the plan with the last task's choice 0
                        const uint64_t base = base_f + (SWAP ? uni64(sP->stride[T]) * cMs[k] : static_cast<uint64_t>(cMs[k]));
                        const uint64_t lo = A.begin > base ? (A.begin - base + strideL - 1) / strideL : 0;
                        uint64_t hi = A.end > base ? (A.end - base + strideL - 1) / strideL : 0;
                        if (hi > CL) hi = CL;
                        ul.cl_lo = static_cast<uint32_t>(lo < hi ? lo : hi);
                        ul.cl_cnt = static_cast<uint32_t>(hi > lo ? hi - lo : 0);
                    }
                    sVal[e] = uv;
                    sLim[e] = ul;
                    if (SETTLE && ul.w_rem >= 0) {
                        top_pre = __builtin_fmax(top_pre, uv.pre);
                        top_presum = __builtin_fmax(top_presum, uv.presum);
                    }
                    // the entry's part of the plan's index (SWAP: below 2^32, checked on the host)
                    sChoice[e] = SWAP ? static_cast<uint32_t>(uni64(sP->stride[T])) * cMs[k] : cMs[k];
                }
            }
        }
        if constexpr (SETTLE) {
            // the largest pre / presum of the tile, for the bound below: one slot per wavefront, written by
            // every wavefront for every item (read after the barrier, rewritten after the next item's first one)
            top_pre = wave_max_f64(top_pre);
            top_presum = wave_max_f64(top_presum);
            if (lane == 0) {
                sTop[wave][0] = top_pre;
                sTop[wave][1] = top_presum;
            }
        }
        __syncthreads();

        // this wavefront's contiguous part of the tile
        const uint32_t e_lo = static_cast<uint32_t>(static_cast<uint64_t>(cnt) * midpart / mid_split);
        const uint32_t e_hi = static_cast<uint32_t>(static_cast<uint64_t>(cnt) * (midpart + 1) / mid_split);
        if constexpr (!SETTLE) {
        uint32_t fcount = 0;  // feasible plans of this item seen by this wavefront (< 2^20)
        int32_t amh[S];       // high word of the accuracy, or of a huge negative number where the plan is infeasible
        uint32_t run_feas = 0;
        int32_t prev_w = -2, prev_tl = -2;  // limits the masks were last taken for (none yet in this item)
        uint32_t e = e_lo;
        // the limits and the first record of a run are fetched during the run before it
        MidLim ul_ahead = sLim[e_lo < e_hi ? e_lo : 0];
        MidVal u_ahead = sVal[e_lo < e_hi ? e_lo : 0];
        while (e < e_hi) {
            // ---- start of a run: masks of the S*64 plans, valid for every record of the run
            const MidLim ul = ul_ahead;
            uint32_t run_hi = e + 1;
            if (!RANGE) {
                run_hi = uni(ul.cl_lo);  // end of the run; it may lie beyond this wavefront's part
                if (run_hi > e_hi) run_hi = e_hi;
            }
            MidVal uA = u_ahead;
            {
                const uint32_t e_next = run_hi < e_hi ? run_hi : e;
                ul_ahead = sLim[e_next];
                u_ahead = sVal[e_next];
            }
            const int32_t w_rem = uni(ul.w_rem), tl = uni(ul.tl);  // the same in every lane: scalar operands
            // a run whose limits bind the last task like those of the run before it keeps that run's masks
            // (the ordering kernel lines up the runs of one latency by the workers they leave)
            const int32_t w_eff = w_rem < A.w_most_last ? w_rem : A.w_most_last;
            const bool same_masks = !RANGE && w_eff == prev_w && tl == prev_tl;
            prev_w = w_eff;
            prev_tl = tl;
            if (same_masks) {
                // nothing to do
            } else if (!RANGE && w_rem >= A.w_most_last) {
                run_feas = 0;
                // the workers left cover whatever the last task may host (eq. (3) cannot bind in this run):
                // the latency alone decides (a choice that can never be used carries the latency kNever)
#pragma unroll
                for (int s = 0; s < S; s++) {
                    const bool ok = lat[s] <= tl;
                    run_feas += static_cast<uint32_t>(__builtin_popcountll(__builtin_amdgcn_ballot_w64(ok)));
                    amh[s] = ok ? __double2hiint(a[s]) : static_cast<int32_t>(0xFFE00000u);
                }
            } else {
                run_feas = 0;
#pragma unroll
                for (int s = 0; s < S; s++) {
                    // one ballot per compare: the masks then come straight from the compare results
                    const bool ok_w = w[s] <= w_rem, ok_l = lat[s] <= tl;
                    uint64_t fm = __builtin_amdgcn_ballot_w64(ok_w) & __builtin_amdgcn_ballot_w64(ok_l);
                    bool ok = ok_w & ok_l;
                    if (RANGE) {
                        const bool ok_r = (cl0 + s * 64 - ul.cl_lo) < ul.cl_cnt;
                        fm &= __builtin_amdgcn_ballot_w64(ok_r);
                        ok = ok & ok_r;
                    }
                    run_feas += static_cast<uint32_t>(__builtin_popcountll(fm));
                    amh[s] = ok ? __double2hiint(a[s]) : static_cast<int32_t>(0xFFE00000u);
                }
            }
            fcount += run_feas * (run_hi - e);
            // ---- every record of the run: S*64 objectives into the lane's running maximum; an infeasible
            // plan's stand-in is far below any key
            auto score = [&](const MidVal &u) {
                double kmax = 0.0;
#pragma unroll
                for (int s = 0; s < S; s++) {
                    const double am = __hiloint2double(amh[s], __double2loint(a[s]));
                    const double tprod = u.pre * am;
                    double key = HAS_PRESUM ? u.presum + tprod : tprod;
                    if (DIVIDE) key = key / npd;
                    kmax = s == 0 ? key : __builtin_fmax(kmax, key);
                }
                // (the instruction itself: through the builtin the compiler first re-canonicalises the
                // loop-carried operand, one more instruction per record)
                bsum = max_f64_instruction(bsum, kmax);
            };
            // Three records in flight: a record is fetched two steps before it is used, so that the read's
            // latency is covered by the scoring of the two records before it.  The fetch may reach up to four
            // entries past the run (the tile array is padded for that); what it brings is then not used.  The
            // entry's byte offset lives in a vector register, so that the reads take their distance as an
            // immediate and one add per round moves them on.
            uint32_t eb = e * static_cast<uint32_t>(sizeof(MidVal));
            asm volatile("" : "+v"(eb));
            const char *val_bytes = reinterpret_cast<const char *>(sVal);
            auto fetch = [&](uint32_t ahead) {
                return *reinterpret_cast<const MidVal *>(val_bytes + eb + ahead * sizeof(MidVal));
            };
            MidVal uB = fetch(1), uC = uA;
            while (true) {
                uC = fetch(2);
                score(uA);
                if (e + 1 >= run_hi) break;
                uA = fetch(3);
                score(uB);
                if (e + 2 >= run_hi) break;
                uB = fetch(4);
                score(uC);
                if (e + 3 >= run_hi) break;
                e += 3;
                eb += 3 * static_cast<uint32_t>(sizeof(MidVal));
            }
            // (the records in flight count as used on every way out: their reads stay where they stand
            // instead of sinking to just before their use)
            asm volatile("" : : "v"(uA.pre), "v"(uB.pre), "v"(uC.pre));
            e = run_hi;
        }
        nfeas += fcount;
        } else {
        // ---- second pass.  A slot can reach the block's key in this tile only if it does so with the
        // tile's largest pre and presum: every operation of the key is monotone in each operand (all
        // values are non-negative), so that is an upper bound on the slot's key with any entry.
        double tile_pre = sTop[0][0], tile_presum = sTop[0][1];
#pragma unroll
        for (int v = 1; v < kWavesPerBlock; v++) {
            tile_pre = __builtin_fmax(tile_pre, sTop[v][0]);
            tile_presum = __builtin_fmax(tile_presum, sTop[v][1]);
        }
        uint32_t can = 0;  // bit s: slot s of this lane may reach the key
#pragma unroll
        for (int s = 0; s < S; s++) {
            const double tprod = tile_pre * a[s];
            double key = HAS_PRESUM ? tile_presum + tprod : tprod;
            if (DIVIDE) key = key / npd;
            if (lane_in && lat[s] != kNever && key >= gb) can |= 1u << s;
        }
        uint32_t e = __builtin_amdgcn_ballot_w64(can != 0) != 0 ? e_lo : e_hi;
        while (e < e_hi) {
            // ---- start of a run: the slots that are feasible with the run's limits and may reach the key
            const MidLim ul = sLim[e];
            uint32_t run_hi = e + 1;
            if (!RANGE) {
                run_hi = uni(ul.cl_lo);
                if (run_hi > e_hi) run_hi = e_hi;
            }
            const int32_t w_rem = uni(ul.w_rem), tl = uni(ul.tl);
            uint64_t fm[S];
            int32_t amh[S];
            // of this lane's eligible slots: fewest replicas and the lowest choice having them, and the
            // lowest choice at all
            int32_t minw = kNever;
            uint32_t cmin = ~0u, cfirst = ~0u;
            uint64_t any = 0;
#pragma unroll
            for (int s = S - 1; s >= 0; s--) {
                bool ok = (w[s] <= w_rem) & (lat[s] <= tl) & (((can >> s) & 1u) != 0);
                if (RANGE) ok = ok & ((cl0 + s * 64 - ul.cl_lo) < ul.cl_cnt);
                fm[s] = __builtin_amdgcn_ballot_w64(ok);
                any |= fm[s];
                amh[s] = ok ? __double2hiint(a[s]) : static_cast<int32_t>(0xFFE00000u);
                if (ok) {
                    cfirst = cl0 + s * 64;
                    if (w[s] <= minw) {
                        minw = w[s];
                        cmin = cl0 + s * 64;
                    }
                }
            }
            if (any == 0) {
                e = run_hi;
                continue;
            }
            // what any plan of this wavefront in this run has at least: the fewest replicas of the last task
            // and the lowest choice having them (order by workers), or the lowest choice (order by index)
            const uint32_t mw = wave_min_u32(static_cast<uint32_t>(minw));
            const uint32_t cf = wave_min_u32(tie_index_only ? cfirst : (static_cast<uint32_t>(minw) == mw ? cmin : ~0u));
            // The records of the run, 64 at a time: every lane looks at one entry and tells from the entry's
            // replicas and index part alone whether a plan of this wavefront there could come before the best
            // one found so far; only those records are scored.  (A bound taken with an older best holds for
            // a newer one.)
            for (uint32_t base = e; base < run_hi; base += 64) {
            bool may = false;
            if (base + lane < run_hi) {
                // replicas of all tasks but the last, from the entry itself (the entries of a run share
                // their masks, not necessarily their replica counts), and the entry's part of the index
                const int32_t w_out_l = W - sLim[base + lane].w_rem;
                const uint64_t low_l = base_f + sChoice[base + lane];
                const bool idx_may = (cf < bcl) | ((cf == bcl) & (low_l < blow));
                const int32_t t = w_out_l + static_cast<int32_t>(mw);
                may = tie_index_only ? idx_may : ((t < bw) | ((t == bw) & idx_may));
            }
            uint64_t todo = __builtin_amdgcn_ballot_w64(may);
            while (todo != 0) {
                const uint32_t ee = base + static_cast<uint32_t>(__builtin_ctzll(todo));
                todo &= todo - 1;
                const int32_t w_out = W - uni(sLim[ee].w_rem);
                const uint64_t low = base_f + uni(sChoice[ee]);
                const MidVal u = sVal[ee];
                double kmax = 0.0;
#pragma unroll
                for (int s = 0; s < S; s++) {
                    const double am = __hiloint2double(amh[s], __double2loint(a[s]));
                    const double tprod = u.pre * am;
                    double key = HAS_PRESUM ? u.presum + tprod : tprod;
                    if (DIVIDE) key = key / npd;
                    kmax = s == 0 ? key : __builtin_fmax(kmax, key);
                }
                if (__builtin_amdgcn_ballot_w64(kmax >= gb) == 0) continue;
                // some plan of this record has the block's key: the full order among them
                bool won = false;
#pragma unroll
                for (int s = 0; s < S; s++) {
                    const double tprod = u.pre * a[s];
                    double key = HAS_PRESUM ? u.presum + tprod : tprod;
                    if (DIVIDE) key = key / npd;
                    const uint64_t hit = fm[s] & __builtin_amdgcn_ballot_w64(key >= gb);
                    if (hit == 0) continue;
                    if ((hit >> lane) & 1) {
                        const uint32_t cL = cl0 + s * 64;
                        const int32_t wt = w_out + w[s];
                        const bool idx_wins = (cL < bcl) | ((cL == bcl) & (low < blow));
                        const bool win = tie_index_only ? idx_wins : ((wt < bw) | ((wt == bw) & idx_wins));
                        if (win) {
                            bw = wt;
                            bcl = cL;
                            blow = low;
                            won = true;
                        }
                    }
                }
                // every lane takes over the wavefront's best, which the bounds above are compared with; the
                // block's other wavefronts learn of it through sBlk (work items that cannot do better are skipped)
                if (__builtin_amdgcn_ballot_w64(won) != 0) {
                    wave_first(bw, bcl, blow, tie_index_only);
                    if (lane == 0) atomicMin(&sBlk, tie_index_only ? bcl : static_cast<uint32_t>(bw));
                }
            }
            }
            e = run_hi;
        }
        }
        // next item
        if (RANGE || SWAP) {
            if (item + 1 < item_hi) locate(item + 1);
        } else {
            advance();
        }
    }
    };
    walk(std::false_type{});

    // The block's largest key, and whether it can still be the demand point's: the largest key any block of
    // the demand point has reported so far is kept in A.floor[m] (bit patterns of non-negative doubles order
    // like the doubles).  A block below it cannot hold the best plan and skips the second pass; blocks that
    // tie with it take the pass, the order among their plans is settled by the final merge.
    {
        const double wmax = wave_max_f64(bsum);
        if (lane == 0) sTop[wave][0] = wmax;
        __syncthreads();
        double m4 = sTop[0][0];
#pragma unroll
        for (int v = 1; v < kWavesPerBlock; v++) m4 = __builtin_fmax(m4, sTop[v][0]);
        // (a stand-in times a zero product is -0.0: as a key that is the key 0.0)
        m4 = m4 > -0.5 ? m4 + 0.0 : -1.0;
        if (threadIdx.x == 0) {
            uint32_t go = 0;
            if (m4 >= 0.0) {
                const unsigned long long mine = static_cast<unsigned long long>(__double_as_longlong(m4));
                const unsigned long long seen = atomicMax(A.floor + m, mine);
                go = seen <= mine ? 1u : 0u;
            }
            sGo = go;
            sBlk = ~0u;
        }
        __syncthreads();
        gb = m4;
    }
    if (sGo != 0) {
        lane_in = bsum == gb;
        walk(std::true_type{});
    }
    // the key is the path sum unless DIVIDE; dividing by the (power-of-two) path count is exact and monotone
    double bacc = bw != kNever ? gb : -1.0;
    if (!DIVIDE && bacc >= 0.0) bacc = bacc / npd;
    const uint64_t bidx = bw != kNever ? blow + strideL * bcl : ~0ull;
    __syncthreads();
    block_store_best(bacc, bw, bidx, nfeas, tie_index_only, sBest,
                     A.recs + static_cast<size_t>(m) * A.blocks_per_m + blockIdx.x);
}

// plans waiting for the walk over the variant paths, per wavefront: below 64 waiting + at most 64 new per push
constexpr uint32_t kWalkQueue = 128;

// The objective of plan idx from its profiled path accuracies (a call, so that the loops that queue plans
// keep their registers).
template <int MAXD>
__device__ __noinline__ double walk_plan(const DevProblem *P, const double *path_acc, const int64_t *Dn, uint64_t idx) {
    uint32_t c[kMaxTasks];
    uint64_t rest = idx;
#pragma unroll
    for (int i = 0; i < kMaxTasks; i++) {
        c[i] = 0;
        if (i < P->n_tasks) {
            c[i] = static_cast<uint32_t>(rest % P->C[i]);
            rest /= P->C[i];
        }
    }
    return path_objective<MAXD>(P, path_acc, c, Dn);
}

// ---- kernel: profiled path accuracies on top of the per-task tables -----------------------------------------
// Feasibility is separable even where the objective is not (one factor per edge: a task's demand, and so
// its record, does not depend on the other tasks).  This kernel walks the plan space like combine_kernel
// (same work items, tiles of first-task choices in run order, the last task's records in registers) but
// only takes the feasibility masks, once per run; the plans of a run that are feasible go, by index, into
// a queue of the wavefront, and whenever 64 are waiting every lane walks the variant paths of one
// (path_objective).  The cost is a few instructions per 512 plans plus the walk for feasible plans only.
//
// A.prune (one task path, one factor per edge, at most kMaxPrefix variant combinations above the last task):
// most feasible plans are not walked at all.  The shares c(p) of a plan's variant paths add up, over the
// variants of the tasks above, to the part s(k) of the last task's requests that its variant k serves (every
// hop hands on the whole stream), so   sum_p c(p) A-hat(p)  <=  sum_k s(k) * max A-hat(p', k)   with the
// maximum over the combinations p' of variants in use of the tasks above.  s comes with the lane's choice of the
// last task (registers, formed when a chunk group first meets a feasible run); the variants in use of the other
// tasks' choices come with their table records (task_table_kernel leaves the bit mask where the accuracy would
// be); the maxima are formed per work item (over the tasks in between) and per tile entry (LDS).  A feasible
// plan whose bound (taken in fp32 and widened by 1e-5 for the rounding on both sides) is below the best
// objective seen so far for the demand point (the wavefront's own, and A.floor[m] shared through memory, read
// again after every 64 walks) can neither win nor tie: it is counted and dropped.  Every item is gone through
// twice, the first time only to find, per lane, the feasible plan with the largest bound: walking those first
// gives the threshold a good plan of the same item.  The plans that are walked sit in few places of the plan
// space, so the items are short, and a block's items lie blocks_per_m apart.
template <int S, bool RANGE, int MAXD, bool SWAP>
__global__ void __launch_bounds__(kBlockThreads, MAXD == 4 ? 2 : 1) path_combine_kernel(SearchArgs A) {
    __shared__ DevProblem sPfull;
    __shared__ MidLim sLim[kMidTile];
    __shared__ uint32_t sChoice[kMidTile];
    __shared__ float sCol[SWAP ? 1 : kMidTile][kMaxVariants];
    __shared__ float sTab[SWAP ? 1 : kMaxPrefix * kMaxVariants];   // prune: the last task's table of path accuracies
    // prune: per variant of the first and of the last task, the largest table entry over the combinations of
    // variants in use of the tasks in between (those of the work item)
    __shared__ float sFar[SWAP ? 1 : kMaxVariants][kMaxVariants];
    __shared__ uint64_t sWalkIdx[kWavesPerBlock][kWalkQueue];
    __shared__ int32_t sWalkW[kWavesPerBlock][kWalkQueue];
    __shared__ BestRec sBest[kWavesPerBlock];
    stage_problem(&sPfull, A.P, sizeof(DevProblem));
    __syncthreads();
    const DevProblem *sP = &sPfull;

    const uint32_t lane = threadIdx.x & 63;
    const int wave = uni(static_cast<int>(threadIdx.x >> 6));
    const int m = blockIdx.y;
    const int n = uni(sP->n_tasks), L = n - 1;
    const uint32_t CL = uni(sP->C[L]);
    const uint32_t C0 = n >= 2 ? uni(sP->C[0]) : 1u;
    const uint64_t strideL = uni64(sP->stride[L]);
    const TaskRec *tab = A.table + static_cast<size_t>(m) * uni(sP->table_total);
    const TaskRec *tabL = tab + uni(sP->table_off[L]);
    // SWAP (with per-variant factors, class by class): the tile task and the work item's digits as in
    // combine_kernel; only replicas and latencies matter here, the objective comes from the walk
    const int T = SWAP ? uni(sP->tile_task) : 0;
    const bool tile_leaf = !SWAP || uni(sP->is_leaf[T]) != 0;
    const uint32_t Cmid = SWAP ? uni(sP->C[T]) : C0;
    const uint32_t mid_count =
        SWAP ? (tile_leaf ? Cmid : uni(A.class_count[static_cast<size_t>(m) * kMaxTasks + T])) : C0;
    const TaskRec *tabM = SWAP ? tab + uni(sP->table_off[T]) : tab;
    const uint32_t *perm_m = SWAP ? A.perm_all + static_cast<size_t>(m) * uni(sP->table_total) : nullptr;
    const uint32_t *perm = SWAP ? perm_m + uni(sP->table_off[T]) : A.perm + static_cast<size_t>(m) * C0;
    const uint32_t *run_end = SWAP ? A.run_end_t + static_cast<size_t>(m) * Cmid : A.run_end + static_cast<size_t>(m) * C0;
    uint32_t cntj[kMaxTasks];
    uint64_t far_swap = 1;
#pragma unroll
    for (int j = 0; j < kMaxTasks; j++) {
        cntj[j] = 1;
        if (SWAP && j < L && j != T) {
            cntj[j] = uni(A.class_count[static_cast<size_t>(m) * kMaxTasks + j]);
            far_swap *= cntj[j];
        }
    }
    const bool tie_index_only = A.tie_index_only != 0;
    const int32_t W = A.W;
    const int64_t *Dn = A.Dn + static_cast<size_t>(m) * kMaxTasks;

    const uint32_t cpb = A.cpb;
    const uint32_t chunk_in_group = wave % cpb, midpart = wave / cpb, mid_split = kWavesPerBlock / cpb;

    int32_t w[S], lat[S];
    double bacc = -1.0;
    int32_t bw = kNever;
    uint64_t bidx = ~0ull;
    uint64_t nfeas = 0;      // wavefront total
    uint32_t waiting = 0;    // plans in this wavefront's queue (the same in every lane)
    uint32_t cur_group = ~0u;
    uint32_t cl0 = 0;        // this lane's choice of the last task in slot 0
    const bool prune = !SWAP && A.prune != 0;
    const int KL = uni(sP->K[L]);
    const double *tabPath = A.path_acc + uni(sP->path_off[L]);
    float sh[S][kMaxVariants];    // prune: the part of the last task's requests each of its variants serves
    uint32_t sh_group = ~0u;      // the chunk group sh belongs to
    double thr = 0.0;             // prune: best objective known for the demand point (the same in every lane)
#pragma unroll
    for (int s = 0; s < S; s++)
#pragma unroll
        for (int k = 0; k < kMaxVariants; k++) sh[s][k] = 0.0f;

    // the first `count` lanes take the queue entries [from, from + count) and walk them
    auto walk_queued = [&](uint32_t from, uint32_t count) {
        if (lane < count) {
            const uint64_t idx = sWalkIdx[wave][from + lane];
            const int32_t workers = sWalkW[wave][from + lane];
            const double acc = walk_plan<MAXD>(sP, A.path_acc, Dn, idx);
            if (better(acc, workers, idx, bacc, bw, bidx, tie_index_only)) {
                bacc = acc;
                bw = workers;
                bidx = idx;
            }
        }
    };

    // prune: combinations of variants of the tasks above the last one, and the table in LDS
    uint32_t Qabove = 1;
#pragma unroll
    for (int j = 0; j < kMaxTasks; j++)
        if (j < L) Qabove *= static_cast<uint32_t>(uni(sP->K[j]));
    if constexpr (!SWAP) {
        if (prune) {
            for (uint32_t t = threadIdx.x; t < Qabove * static_cast<uint32_t>(KL); t += kBlockThreads)
                sTab[t] = static_cast<float>(tabPath[t]);
            __syncthreads();
        }
    }

    const uint64_t far_m = SWAP ? far_swap : A.far_span;
    const uint64_t items_m = SWAP ? static_cast<uint64_t>(A.chunk_groups) * far_m * A.mid_tiles : A.items;
    const uint64_t item_lo = items_m * blockIdx.x / A.blocks_per_m;
    const uint64_t item_hi = items_m * (blockIdx.x + 1) / A.blocks_per_m;
    // (prune: the block's items lie blocks_per_m apart, so that the few places of the plan space where plans are
    // walked are shared out among the blocks)
    const bool apart = prune;
    const uint64_t item_step = apart ? A.blocks_per_m : 1;
    for (uint64_t item = apart ? blockIdx.x : item_lo; item < (apart ? items_m : item_hi); item += item_step) {
        // position of the item: tile r, combination f of the tasks in between, chunk group g
        const uint32_t r = uni(static_cast<uint32_t>(item % A.mid_tiles));
        const uint64_t t = item / A.mid_tiles;
        const uint64_t f = SWAP ? 0 : uni64((A.far_first + t % A.far_span) % A.far_count);
        const uint32_t g = uni(static_cast<uint32_t>(t / far_m));
        uint32_t cj[kMaxTasks];
        if (SWAP) {
            uint64_t rest = t % far_m;
#pragma unroll
            for (int j = 0; j < kMaxTasks; j++) {
                cj[j] = 0;
                if (j < L && j != T) {
                    const uint32_t d = static_cast<uint32_t>(rest % cntj[j]);
                    rest /= cntj[j];
                    cj[j] = uni(perm_m[uni(sP->table_off[j]) + d]);
                }
            }
        } else {
            uint64_t rest = f;
#pragma unroll
            for (int j = 1; j < kMaxTasks; j++) {
                cj[j] = 0;
                if (j < L) {
                    cj[j] = uni(static_cast<uint32_t>(rest % sP->C[j]));
                    rest /= sP->C[j];
                }
            }
            cj[0] = 0;
        }
        if (g != cur_group) {
            cur_group = g;
            cl0 = A.cl_first + (g * cpb + chunk_in_group) * (64u * S) + lane;
#pragma unroll
            for (int s = 0; s < S; s++) {
                const uint32_t cL = cl0 + s * 64;
                if (cL < CL) {
                    const TaskRec rec = tabL[cL];
                    w[s] = rec.w;
                    lat[s] = rec.lat;
                } else {
                    w[s] = 0;
                    lat[s] = kNever;
                }
            }
        }
        // prune: the variants in use of the tasks strictly between the first and the last, and what the
        // other blocks of the demand point have found so far
        uint32_t used_far[kMaxTasks];
#pragma unroll
        for (int j = 0; j < kMaxTasks; j++) used_far[j] = 0;
        if (prune) {
#pragma unroll
            for (int j = 1; j < kMaxTasks; j++)
                if (j < L) used_far[j] = uni(static_cast<uint32_t>(tab[sP->table_off[j] + cj[j]].a));
            const double shared = __longlong_as_double(static_cast<long long>(
                __hip_atomic_load(A.floor + m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)));
            if (shared > thr) thr = shared;
            if constexpr (!SWAP) {
                // (read while the tile is staged, between this item's two barriers; every thread is past the
                // previous item's staging here)
                const uint32_t K0v = n >= 2 ? static_cast<uint32_t>(uni(sP->K[0])) : 1u;
                if (threadIdx.x < K0v * static_cast<uint32_t>(KL)) {
                    const uint32_t k_first = threadIdx.x % K0v, k_last = threadIdx.x / K0v;
                    float v = 0.0f;
                    for (uint32_t q = k_first; q < Qabove; q += K0v) {
                        uint32_t rest = q / K0v;
                        bool in_use = true;
#pragma unroll
                        for (int j = 1; j < kMaxTasks; j++) {
                            if (j < L) {
                                const uint32_t Kj = static_cast<uint32_t>(sP->K[j]);
                                const uint32_t k = rest % Kj;
                                rest /= Kj;
                                in_use = in_use && ((used_far[j] >> k) & 1u) != 0;
                            }
                        }
                        const float t = sTab[q + Qabove * k_last];
                        v = (in_use && t > v) ? t : v;
                    }
                    sFar[k_first][k_last] = v;
                }
            }
        }
        // what the tasks strictly between the first and the last contribute (eq. (3), eq. (7))
        int64_t flp[kMaxTasks];
        int64_t w_far = 0;
        bool ok_far = true;
        int64_t lat0_cap = kNever - 1;
#pragma unroll
        for (int j = 0; j < kMaxTasks; j++) flp[j] = 0;
        int64_t tl_base = A.budget[L];
        if (SWAP) {
            // the work item's tasks in topological order: replicas, latency sums along the chains from the
            // first task (here with the first task included); a leaf closes its path (eq. (7))
#pragma unroll
            for (int j = 0; j < kMaxTasks; j++) {
                if (j < L && j != T) {
                    const TaskRec rec = tab[sP->table_off[j] + cj[j]];
                    const int32_t rw = uni(rec.w), rlat = uni(rec.lat);
                    w_far += rw;
                    ok_far = ok_far && rlat != kNever;
                    flp[j] = (j == 0 ? 0 : pick_below(flp, uni(sP->parent[j]), j)) + rlat;
                    if (uni(sP->is_leaf[j])) ok_far = ok_far && A.budget[j] >= 0 && flp[j] <= A.budget[j];
                }
            }
            const int parT = uni(sP->parent[T]);
            if (tile_leaf) {
                lat0_cap = A.budget[T] < 0 ? -1 : A.budget[T] - pick_below(flp, parT, kMaxTasks);
                if (lat0_cap < 0) ok_far = false;
                tl_base = tl_base < 0 ? -1 : tl_base - pick_below(flp, uni(sP->parent[L]), kMaxTasks);
            } else {
                tl_base = tl_base < 0 ? -1 : tl_base - pick_below(flp, parT, kMaxTasks);
            }
        } else {
#pragma unroll
            for (int j = 1; j < kMaxTasks; j++) {
                if (j < L) {
                    const TaskRec rec = tab[sP->table_off[j] + cj[j]];
                    const int32_t rw = uni(rec.w), rlat = uni(rec.lat);
                    w_far += rw;
                    ok_far = ok_far && rlat != kNever;
                    flp[j] = pick_below(flp, uni(sP->parent[j]), j) + rlat;
                }
            }
#pragma unroll
            for (int j = 0; j < kMaxTasks; j++) {
                if (j < L && uni(sP->is_leaf[j])) {
                    const int64_t room = A.budget[j] < 0 ? -1 : A.budget[j] - flp[j];
                    if (room < lat0_cap) lat0_cap = room;
                }
            }
            if (lat0_cap < 0) ok_far = false;
            if (n >= 2) tl_base = tl_base < 0 ? -1 : tl_base - pick_below(flp, uni(sP->parent[L]), kMaxTasks);
        }
        const int64_t w_room = static_cast<int64_t>(W) - w_far;

        const uint32_t tile_base = r * A.tile_len;
        const uint32_t left = tile_base < mid_count ? mid_count - tile_base : 0u;
        const uint32_t cnt = left < A.tile_len ? left : A.tile_len;
        uint64_t base_f = static_cast<uint64_t>(C0) * f;
        if (SWAP) {
            base_f = 0;
#pragma unroll
            for (int j = 0; j < kMaxTasks; j++)
                if (j < L && j != T) base_f += cj[j] * uni64(sP->stride[j]);
        }

        __syncthreads();  // the previous item's tile is no longer being read
        for (uint32_t e = threadIdx.x; e < cnt; e += kBlockThreads) {
            uint32_t cM = 0;
            int32_t w0 = 0, lat0 = 0;
            bool ok = ok_far;
            if (n >= 2) {
                cM = perm[tile_base + e];
                const TaskRec rec = tabM[cM];
                w0 = rec.w;
                lat0 = rec.lat;
                ok = ok_far && rec.lat != kNever && static_cast<int64_t>(rec.lat) <= lat0_cap;
            }
            MidLim ul;
            int64_t tl = tl_base < 0 ? -1 : tl_base - ((SWAP && tile_leaf) ? 0 : static_cast<int64_t>(lat0));
            if (tl < 0) tl = -1;
            if (tl > kNever - 1) tl = kNever - 1;
            ul.tl = static_cast<int32_t>(tl);
            const int64_t wr = w_room - static_cast<int64_t>(w0);
            ul.w_rem = (ok && wr >= 0) ? static_cast<int32_t>(wr) : -1;
            ul.cl_lo = n >= 2 ? run_end[tile_base + e] - tile_base : e + 1;
            ul.cl_cnt = CL;
            if (RANGE) {
                const uint64_t base = base_f + (SWAP ? uni64(sP->stride[T]) * cM : static_cast<uint64_t>(cM));
                const uint64_t lo = A.begin > base ? (A.begin - base + strideL - 1) / strideL : 0;
                uint64_t hi = A.end > base ? (A.end - base + strideL - 1) / strideL : 0;
                if (hi > CL) hi = CL;
                ul.cl_lo = static_cast<uint32_t>(lo < hi ? lo : hi);
                ul.cl_cnt = static_cast<uint32_t>(hi > lo ? hi - lo : 0);
            }
            sLim[e] = ul;
            sChoice[e] = SWAP ? static_cast<uint32_t>(uni64(sP->stride[T])) * cM : cM;
            if constexpr (!SWAP) {
                if (prune) {
                    // per variant of the last task: the largest table entry over the combinations of variants in
                    // use of the tasks above (the first task's from this entry's record)
                    float col[kMaxVariants];
#pragma unroll
                    for (int k = 0; k < kMaxVariants; k++) col[k] = 0.0f;
                    if (ul.w_rem >= 0) {
                        const uint32_t used0 = n >= 2 ? static_cast<uint32_t>(tabM[cM].a) : 1u;
                        for (int k_first = 0; k_first < kMaxVariants; k_first++) {
                            if (((used0 >> k_first) & 1u) == 0) continue;
#pragma unroll
                            for (int k = 0; k < kMaxVariants; k++) {
                                const float v = k < KL ? sFar[k_first][k] : 0.0f;
                                col[k] = v > col[k] ? v : col[k];
                            }
                        }
                    }
#pragma unroll
                    for (int k = 0; k < kMaxVariants; k++) sCol[e][k] = col[k];
                }
            }
        }
        __syncthreads();

        const uint32_t e_lo = static_cast<uint32_t>(static_cast<uint64_t>(cnt) * midpart / mid_split);
        const uint32_t e_hi = static_cast<uint32_t>(static_cast<uint64_t>(cnt) * (midpart + 1) / mid_split);
        // prune: the item is gone through twice.  The first time nothing is walked: every lane keeps the feasible
        // plan with the largest bound it meets, these (at most 64) plans are walked, and the best of them, a
        // good plan of this very item, is the threshold the second time round (plans come in an order in which
        // the objective tends to rise, so a threshold learnt on the way would lag behind).  An item without
        // feasible plans ends after the first time.
        float cand_ub = -1.0f;
        uint32_t cand_at = 0;    // entry * 8 + slot
        bool item_any = true;
        for (int pass = prune ? 0 : 1; pass < 2 && item_any; pass++) {
        if (pass == 0) item_any = false;
        uint32_t e = e_lo;
        while (e < e_hi) {
            // ---- start of a run: which of the S*64 plans are feasible, valid for every record of the run
            const MidLim ul = sLim[e];
            uint32_t run_hi = e + 1;
            if (!RANGE) {
                run_hi = uni(ul.cl_lo);
                if (run_hi > e_hi) run_hi = e_hi;
            }
            const int32_t w_rem = uni(ul.w_rem), tl = uni(ul.tl);
            uint64_t fm[S];
            uint32_t run_feas = 0;
#pragma unroll
            for (int s = 0; s < S; s++) {
                bool ok = (w[s] <= w_rem) & (lat[s] <= tl);
                if (RANGE) ok = ok & ((cl0 + s * 64 - ul.cl_lo) < ul.cl_cnt);
                fm[s] = __builtin_amdgcn_ballot_w64(ok);
                run_feas += static_cast<uint32_t>(__builtin_popcountll(fm[s]));
            }
            if (run_feas != 0) {
                if constexpr (!SWAP) {
                    if (pass == 0) {  // (prune)
                        item_any = true;
                        if (sh_group != cur_group) {
                            sh_group = cur_group;
#pragma unroll
                            for (int s = 0; s < S; s++) {
                                const uint32_t cL = cl0 + s * 64;
                                choice_shares(sP, L, cL < CL ? cL : 0u, Dn[L], sh[s]);
                            }
                        }
                    }
                }
                for (uint32_t ee = e; ee < run_hi; ee++) {
                    const uint64_t low = base_f + sChoice[ee];
                    const int32_t w_out = W - sLim[ee].w_rem;  // replicas of all tasks but the last
                    float thr_f = static_cast<float>(thr) * 0.99999f;
#pragma unroll
                    for (int s = 0; s < S; s++) {
                        if (fm[s] == 0) continue;
                        uint64_t km = fm[s];   // the plans of this slot that go on to the walk
                        if (prune) {
                            float ub = 0.0f;
#pragma unroll
                            for (int k = 0; k < kMaxVariants; k++) ub = __builtin_fmaf(sh[s][k], sCol[ee][k], ub);
                            if (pass == 0) {
                                if (((fm[s] >> lane) & 1) != 0 && ub > cand_ub) {
                                    cand_ub = ub;
                                    cand_at = ee * 8 + s;
                                }
                                continue;
                            }
                            km = __builtin_amdgcn_ballot_w64(((fm[s] >> lane) & 1) != 0 && ub * 1.00001f >= thr_f);
                            if (km == 0) continue;
                        }
                        if ((km >> lane) & 1) {
                            const uint32_t at = waiting + static_cast<uint32_t>(__builtin_popcountll(km & ((1ull << lane) - 1)));
                            sWalkIdx[wave][at] = low + strideL * (cl0 + s * 64);
                            sWalkW[wave][at] = w_out + w[s];
                        }
                        waiting += static_cast<uint32_t>(__builtin_popcountll(km));
                        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                        if (waiting >= 64) {
                            waiting -= 64;
                            walk_queued(waiting, 64);
                            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                            if (prune) {
                                const double seen = wave_max_f64(bacc);
                                if (seen > thr) {
                                    thr = seen;
                                    if (lane == 0) atomicMax(A.floor + m, static_cast<unsigned long long>(__double_as_longlong(seen)));
                                }
                                const double shared = __longlong_as_double(static_cast<long long>(
                                    __hip_atomic_load(A.floor + m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)));
                                if (shared > thr) thr = shared;
                                thr_f = static_cast<float>(thr) * 0.99999f;
                            }
                        }
                    }
                    if (pass == 1) nfeas += run_feas;
                }
            }
            e = run_hi;
        }
        if (pass == 0 && item_any) {
            // walk every lane's candidate, unless what the demand point has reached elsewhere rules it out (and what
            // was waiting), and take the threshold from the result
            {
                const double shared = __longlong_as_double(static_cast<long long>(
                    __hip_atomic_load(A.floor + m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)));
                if (shared > thr) thr = shared;
            }
            const bool have = cand_ub >= 0.0f && cand_ub * 1.00001f >= static_cast<float>(thr) * 0.99999f;
            const uint64_t vote = __builtin_amdgcn_ballot_w64(have);
            if (have) {
                const uint32_t ee = cand_at >> 3, s_at = cand_at & 7u;
                const uint32_t at = waiting + static_cast<uint32_t>(__builtin_popcountll(vote & ((1ull << lane) - 1)));
                int32_t w_s = 0;
#pragma unroll
                for (int s = 0; s < S; s++) w_s = static_cast<uint32_t>(s) == s_at ? w[s] : w_s;
                sWalkIdx[wave][at] = base_f + sChoice[ee] + strideL * (cl0 + s_at * 64);
                sWalkW[wave][at] = W - sLim[ee].w_rem + w_s;
            }
            waiting += static_cast<uint32_t>(__builtin_popcountll(vote));
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            while (waiting > 0) {
                const uint32_t take = waiting < 64 ? waiting : 64;
                waiting -= take;
                walk_queued(waiting, take);
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            }
            const double seen = wave_max_f64(bacc);
            if (seen > thr) {
                thr = seen;
                if (lane == 0) atomicMax(A.floor + m, static_cast<unsigned long long>(__double_as_longlong(seen)));
            }
        }
        }
    }
    // What is left in the four queues (fewer than 64 plans each) is walked by the block as a whole: the
    // wavefronts' leftovers are put one after the other, and every thread below their total takes one.
    __shared__ uint32_t sLeft[kWavesPerBlock];
    if (lane == 0) sLeft[wave] = waiting;
    __syncthreads();
    {
        uint32_t total = 0, mine = threadIdx.x, src_wave = 0;
        bool have = false;
#pragma unroll
        for (int v = 0; v < kWavesPerBlock; v++) {
            const uint32_t c = sLeft[v];
            if (!have && mine < total + c && mine >= total) {
                have = true;
                src_wave = v;
                mine -= total;
            }
            total += c;
        }
        if (have) {
            const uint64_t idx = sWalkIdx[src_wave][mine];
            const int32_t workers = sWalkW[src_wave][mine];
            const double acc = walk_plan<MAXD>(sP, A.path_acc, Dn, idx);
            if (better(acc, workers, idx, bacc, bw, bidx, tie_index_only)) {
                bacc = acc;
                bw = workers;
                bidx = idx;
            }
        }
    }
    __syncthreads();
    block_store_best(bacc, bw, bidx, nfeas, tie_index_only, sBest,
                     A.recs + static_cast<size_t>(m) * A.blocks_per_m + blockIdx.x);
}


// ---- kernel: eq. (7) on the variant paths with traffic, on top of the per-task tables ---------------------
// Under that rule a plan is feasible if the per-task sum of the slowest variants in use meets the budget (those
// plans are found by combine_kernel as ever: the sum bounds every variant path from above), or if it does not
// but every variant path that carries requests does.  This kernel visits the plan space like
// path_combine_kernel (same work items, tiles of first-task choices, the last task's records in registers) and
// picks out the plans of the second kind that are still open: usable choices everywhere, worker budget met, the
// per-task sum too slow on some task path, and the two variant paths that always carry requests (first and
// last variants in use, TaskLat2) within the budget on every task path.  Those few go, by index, into a queue
// of the wavefront, and whenever 64 are waiting every lane walks the variant paths of one
// (some_path_too_slow) and scores it if it passes.  One factor per edge, product-form objective, two tasks or
// more, every budget non-negative (the host sees to all four).
template <int LATD>
__device__ __noinline__ bool score_open_plan(const DevProblem *P, const int64_t *Dn, const int64_t *budget, int32_t W,
                                             uint64_t idx, double *accuracy, int32_t *workers) {
    uint32_t c[kMaxTasks];
    uint64_t rest = idx;
#pragma unroll
    for (int i = 0; i < kMaxTasks; i++) {
        c[i] = 0;
        if (i < P->n_tasks) {
            c[i] = static_cast<uint32_t>(rest % P->C[i]);
            rest /= P->C[i];
        }
    }
    if (some_path_too_slow<LATD>(P, c, Dn, budget)) return false;
    uint32_t mask;
    eval_plan(P, c, Dn, budget, W, mask, *workers, *accuracy);  // (the per-task latency bound is off in P)
    return mask == 0;
}

template <int S, bool RANGE, int LATD>
__global__ void __launch_bounds__(kBlockThreads, 2) open_plans_kernel(SearchArgs A) {
    __shared__ DevProblem sPfull;
    __shared__ MidLim sLim[kMidTile];       // w_rem: -1 unless the entry can be part of an open plan
    __shared__ int32_t sTopRoom[kMidTile], sBotRoom[kMidTile];  // what the two sure paths leave the last task
    __shared__ uint32_t sChoice[kMidTile];
    __shared__ uint32_t sBoundMet[kMidTile];  // the per-task sums of the entry's part meet every budget they close
    __shared__ uint64_t sWalkIdx[kWavesPerBlock][kWalkQueue];
    __shared__ BestRec sBest[kWavesPerBlock];
    stage_problem(&sPfull, A.P, sizeof(DevProblem));
    __syncthreads();
    const DevProblem *sP = &sPfull;

    const uint32_t lane = threadIdx.x & 63;
    const int wave = uni(static_cast<int>(threadIdx.x >> 6));
    const int m = blockIdx.y;
    const int n = uni(sP->n_tasks), L = n - 1;
    const uint32_t CL = uni(sP->C[L]);
    const uint32_t C0 = uni(sP->C[0]);
    const uint64_t strideL = uni64(sP->stride[L]);
    const uint32_t table_total = uni(sP->table_total);
    const TaskRec *tab = A.table + static_cast<size_t>(m) * table_total;
    const TaskLat2 *tab2 = A.lat2 + static_cast<size_t>(m) * table_total;
    const uint32_t offL = uni(sP->table_off[L]);
    const uint32_t *perm = A.perm + static_cast<size_t>(m) * C0;
    const bool tie_index_only = A.tie_index_only != 0;
    const int32_t W = A.W;
    const int64_t *Dn = A.Dn + static_cast<size_t>(m) * kMaxTasks;
    const int parL = uni(sP->parent[L]);

    const uint32_t cpb = A.cpb;
    const uint32_t chunk_in_group = wave % cpb, midpart = wave / cpb, mid_split = kWavesPerBlock / cpb;

    int32_t w[S], lat[S], top[S], bot[S];
    double bacc = -1.0;
    int32_t bw = kNever;
    uint64_t bidx = ~0ull;
    uint64_t nfeas = 0;      // this lane's
    uint32_t waiting = 0;    // plans in this wavefront's queue (the same in every lane)
    uint32_t cur_group = ~0u;
    uint32_t cl0 = 0;
    uint32_t least_w = 0, least_top = 0, least_bot = 0, most_lat = 0;   // over the wavefront's usable choices

    auto walk_queued = [&](uint32_t from, uint32_t count) {
        if (lane < count) {
            const uint64_t idx = sWalkIdx[wave][from + lane];
            double acc;
            int32_t workers;
            if (score_open_plan<LATD>(sP, Dn, A.budget, W, idx, &acc, &workers)) {
                nfeas++;
                if (better(acc, workers, idx, bacc, bw, bidx, tie_index_only)) {
                    bacc = acc;
                    bw = workers;
                    bidx = idx;
                }
            }
        }
    };

    const uint64_t items_m = A.items;
    const uint64_t item_lo = items_m * blockIdx.x / A.blocks_per_m;
    const uint64_t item_hi = items_m * (blockIdx.x + 1) / A.blocks_per_m;
    for (uint64_t item = item_lo; item < item_hi; ++item) {
        const uint32_t r = uni(static_cast<uint32_t>(item % A.mid_tiles));
        const uint64_t t = item / A.mid_tiles;
        const uint64_t f = uni64((A.far_first + t % A.far_span) % A.far_count);
        const uint32_t g = uni(static_cast<uint32_t>(t / A.far_span));
        if (g != cur_group) {
            cur_group = g;
            cl0 = A.cl_first + (g * cpb + chunk_in_group) * (64u * S) + lane;
#pragma unroll
            for (int s = 0; s < S; s++) {
                const uint32_t cL = cl0 + s * 64;
                if (cL < CL) {
                    const TaskRec rec = tab[offL + cL];
                    const TaskLat2 l2 = tab2[offL + cL];
                    w[s] = rec.w;
                    lat[s] = rec.lat;
                    top[s] = l2.top;
                    bot[s] = l2.bot;
                } else {
                    w[s] = 0;
                    lat[s] = top[s] = bot[s] = kNever;
                }
            }
            // what the wavefront's choices of the last task ask for at the least (and, for the per-task sum, at
            // the most): an entry that cannot meet that has no open plan here
            uint32_t lw = ~0u, lt = ~0u, lb = ~0u, hl = ~0u;
#pragma unroll
            for (int s = 0; s < S; s++) {
                if (lat[s] != kNever) {
                    lw = lw < static_cast<uint32_t>(w[s]) ? lw : static_cast<uint32_t>(w[s]);
                    lt = lt < static_cast<uint32_t>(top[s]) ? lt : static_cast<uint32_t>(top[s]);
                    lb = lb < static_cast<uint32_t>(bot[s]) ? lb : static_cast<uint32_t>(bot[s]);
                    hl = hl < ~static_cast<uint32_t>(lat[s]) ? hl : ~static_cast<uint32_t>(lat[s]);
                }
            }
            least_w = uni(wave_min_u32(lw));
            least_top = uni(wave_min_u32(lt));
            least_bot = uni(wave_min_u32(lb));
            most_lat = ~uni(wave_min_u32(hl));   // 0 when no choice is usable (least_* then rule every entry out)
        }
        // the tasks strictly between the first and the last: replicas, and along the chains from the first
        // task (left out here, added per entry) the three latency sums; a leaf among them closes its path
        int64_t fl[kMaxTasks], ft[kMaxTasks], fb[kMaxTasks];
        int64_t w_far = 0;
        bool ok_far = true;
        int64_t lat0_cap = kNever - 1, top0_cap = kNever - 1, bot0_cap = kNever - 1;
#pragma unroll
        for (int j = 0; j < kMaxTasks; j++) fl[j] = ft[j] = fb[j] = 0;
        {
            uint64_t rest = f;
#pragma unroll
            for (int j = 1; j < kMaxTasks; j++) {
                if (j < L) {
                    const uint32_t cj = uni(static_cast<uint32_t>(rest % sP->C[j]));
                    rest /= sP->C[j];
                    const TaskRec rec = tab[sP->table_off[j] + cj];
                    const TaskLat2 l2 = tab2[sP->table_off[j] + cj];
                    const int32_t rw = uni(rec.w), rlat = uni(rec.lat);
                    const int par = uni(sP->parent[j]);
                    w_far += rw;
                    ok_far = ok_far && rlat != kNever;
                    fl[j] = pick_below(fl, par, j) + rlat;
                    ft[j] = pick_below(ft, par, j) + uni(l2.top);
                    fb[j] = pick_below(fb, par, j) + uni(l2.bot);
                    if (uni(sP->is_leaf[j])) {
                        lat0_cap = lat0_cap < A.budget[j] - fl[j] ? lat0_cap : A.budget[j] - fl[j];
                        top0_cap = top0_cap < A.budget[j] - ft[j] ? top0_cap : A.budget[j] - ft[j];
                        bot0_cap = bot0_cap < A.budget[j] - fb[j] ? bot0_cap : A.budget[j] - fb[j];
                    }
                }
            }
        }
        if (top0_cap < 0 || bot0_cap < 0) ok_far = false;  // a sure path is too slow whatever the first task does
        const int64_t w_room = static_cast<int64_t>(W) - w_far;
        const int64_t tl_base = A.budget[L] - pick_below(fl, parL, kMaxTasks);
        const int64_t tt_base = A.budget[L] - pick_below(ft, parL, kMaxTasks);
        const int64_t tb_base = A.budget[L] - pick_below(fb, parL, kMaxTasks);

        const uint32_t tile_base = r * A.tile_len;
        const uint32_t left = tile_base < C0 ? C0 - tile_base : 0u;
        const uint32_t cnt = left < A.tile_len ? left : A.tile_len;
        const uint64_t base_f = static_cast<uint64_t>(C0) * f;

        __syncthreads();  // the previous item's tile is no longer being read
        for (uint32_t e = threadIdx.x; e < cnt; e += kBlockThreads) {
            const uint32_t c0 = perm[tile_base + e];
            const TaskRec rec = tab[c0];
            const TaskLat2 l2 = tab2[c0];
            const bool usable = ok_far && rec.lat != kNever;
            const bool sure_ok = usable && static_cast<int64_t>(l2.top) <= top0_cap && static_cast<int64_t>(l2.bot) <= bot0_cap;
            auto room = [](int64_t v) { return static_cast<int32_t>(v < -1 ? -1 : (v > kNever - 1 ? kNever - 1 : v)); };
            MidLim ul;
            ul.tl = room(tl_base - rec.lat);
            const int64_t wr = w_room - static_cast<int64_t>(rec.w);
            ul.w_rem = (sure_ok && wr >= 0) ? static_cast<int32_t>(wr) : -1;
            ul.cl_lo = 0;
            ul.cl_cnt = CL;
            if (RANGE) {
                const uint64_t base = base_f + static_cast<uint64_t>(c0);
                const uint64_t lo = A.begin > base ? (A.begin - base + strideL - 1) / strideL : 0;
                uint64_t hi = A.end > base ? (A.end - base + strideL - 1) / strideL : 0;
                if (hi > CL) hi = CL;
                ul.cl_lo = static_cast<uint32_t>(lo < hi ? lo : hi);
                ul.cl_cnt = static_cast<uint32_t>(hi > lo ? hi - lo : 0);
            }
            sLim[e] = ul;
            sTopRoom[e] = usable ? room(tt_base - l2.top) : -1;
            sBotRoom[e] = usable ? room(tb_base - l2.bot) : -1;
            sBoundMet[e] = (usable && static_cast<int64_t>(rec.lat) <= lat0_cap) ? 1u : 0u;
            sChoice[e] = c0;
        }
        __syncthreads();

        const uint32_t e_lo = static_cast<uint32_t>(static_cast<uint64_t>(cnt) * midpart / mid_split);
        const uint32_t e_hi = static_cast<uint32_t>(static_cast<uint64_t>(cnt) * (midpart + 1) / mid_split);
        for (uint32_t e = e_lo; e < e_hi; e++) {
            const MidLim ul = sLim[e];
            const int32_t w_rem = uni(ul.w_rem);
            if (w_rem < 0) continue;
            const int32_t tl = uni(ul.tl), tt = uni(sTopRoom[e]), tb = uni(sBotRoom[e]);
            const bool bound_met = uni(sBoundMet[e]) != 0;
            if (tt < 0 || tb < 0 || static_cast<uint32_t>(w_rem) < least_w || static_cast<uint32_t>(tt) < least_top ||
                static_cast<uint32_t>(tb) < least_bot)
                continue;   // no choice of the wavefront fits
            if (bound_met && tl >= 0 && static_cast<uint32_t>(tl) >= most_lat) continue;   // the per-task sum admits all
            const uint64_t low = base_f + sChoice[e];
#pragma unroll
            for (int s = 0; s < S; s++) {
                // usable, within the worker budget, both sure paths fast enough, the per-task sum not
                bool open = (w[s] <= w_rem) & (top[s] <= tt) & (bot[s] <= tb) & !(bound_met & (lat[s] <= tl));
                if (RANGE) open = open & ((cl0 + s * 64 - ul.cl_lo) < ul.cl_cnt);
                const uint64_t vote = __builtin_amdgcn_ballot_w64(open);
                if (vote == 0) continue;
                if (open) {
                    const uint32_t at = waiting + static_cast<uint32_t>(__builtin_popcountll(vote & ((1ull << lane) - 1)));
                    sWalkIdx[wave][at] = low + strideL * (cl0 + s * 64);
                }
                waiting += static_cast<uint32_t>(__builtin_popcountll(vote));
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                if (waiting >= 64) {
                    waiting -= 64;
                    walk_queued(waiting, 64);
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                }
            }
        }
    }
    walk_queued(0, waiting);
    nfeas = wave_sum(nfeas);
    block_store_best(bacc, bw, bidx, nfeas, tie_index_only, sBest,
                     A.recs + static_cast<size_t>(m) * A.blocks_per_m + blockIdx.x);
}

// ---- kernel: every lane scores whole plans (no tables) ---------------------------------------------------
// A work item is one choice of every task but the last plus a strip of kStrip choices of the
// last task.  The lane scores the shared part once (each task in topological order, so that
// with per-variant factors a child's demand can follow from its parent's routing, eq. (1))
// and then walks the strip, scoring the last task and finishing the plan per step.
constexpr uint32_t kStrip = 64;

// MAXD > 0: the objective comes from profiled path accuracies (path_objective with MAXD levels compiled
// in); the feasibility part is the same.  The walk over the variant paths costs far more than the
// feasibility check and only feasible plans need it, so a wavefront does not walk a plan where it finds
// it: the lane puts the plan's index in a queue of its wavefront, and whenever the queue holds 64 plans
// all 64 lanes walk one each (any lane may own any plan: the running best is a maximum under a strict
// total order).  The loops below therefore have the same trip count in every lane of a wavefront.
// The four-level walk is held to the registers of 3 wavefronts per SIMD: its spills cost less than the
// scoring loop gains from the third wavefront.
//
// LAT: eq. (7) on every variant path with traffic (the template switches PV and VF are not used then: the
// problem's own are read).  Two bounds settle most plans in the scoring loop.  From above, the per-task bound
// (every task's slowest variant in use).  From below, two variant paths that always carry requests when all
// demand is served: the first variants in use of every task (the head of every task's request stream goes
// from one to the next) and the last ones (so does the tail).  A plan between the bounds that is feasible
// otherwise goes through the same queue, marked, and the lane that takes it walks its variant paths
// (some_path_too_slow) before anything else.  Without profiled path accuracies the queue also carries the
// accuracy found in the scoring loop.
constexpr int32_t kWalkCheckLatency = 1 << 30;  // queue entry: latency not settled yet (or'ed into the workers)

// NARROW: the host has shown that every capacity and demand of the call is below 2^32 (eval_task's 32-bit fill).
// LATD: 0, or with LAT the number of levels of the walk over the variant paths compiled in (the longest task
// path of the problem, 4 or 8; MAXD when that is not 0).  The kernels with a latency walk are held to the
// registers of 2 wavefronts per SIMD: 3 spill into the scoring loop, and 1 (twice the registers, the upper half
// of them reachable only through copies) leaves the loop's waits uncovered; built that way the eight-level
// kernel with both walks also returned a plan below the best one, which tests/test_gpu_latency_per_path.py
// now checks for on a six-task chain.  The plain kernel with the 32-bit fill and one batch size per task is held
// to the registers of 6 wavefronts per SIMD (80; its scalar loads and LDS reads want the cover): what spills is
// the part that scores the other tasks once per strip, plus one reload per feasible plan; at 8 the feasible-plan
// path of the strip loop reloads more.
template <bool PV, bool VF, int MAXD, int LATD = 0, bool NARROW = false>
__global__ void __launch_bounds__(kBlockThreads, LATD > 0 ? 2 : (MAXD == 4 ? 3 : (MAXD == 0 && NARROW && !PV ? 6 : 1)))
    per_lane_search_kernel(SearchArgs A) {
    constexpr bool LAT = LATD > 0;
    constexpr bool kQueue = MAXD > 0 || LAT;
    constexpr int kLatLevels = LATD > 0 ? LATD : 1;
    constexpr bool kStepChoice = !LAT && !PV;
    static_assert(MAXD == 0 || LATD == 0 || LATD == MAXD, "one depth for both walks");
    __shared__ DevProblem sP;
    __shared__ BestRec sBest[kWavesPerBlock];
    __shared__ uint64_t sWalkIdx[kQueue ? kWavesPerBlock : 1][kQueue ? kWalkQueue : 1];
    __shared__ int32_t sWalkW[kQueue ? kWavesPerBlock : 1][kQueue ? kWalkQueue : 1];
    __shared__ double sWalkAcc[LAT && MAXD == 0 ? kWavesPerBlock : 1][LAT && MAXD == 0 ? kWalkQueue : 1];
    stage_problem(&sP, A.P, sizeof(DevProblem));
    __syncthreads();
    const DevProblem *P = &sP;
    const ScalarProblem PS = scalar_view(A.P);
    const int m = blockIdx.y;
    const int n = P->n_tasks, L = n - 1;
    const bool has_vf = LAT ? P->has_vf != 0 : VF;
    const bool tie_index_only = A.tie_index_only != 0;
    const uint64_t lanes = static_cast<uint64_t>(gridDim.x) * kBlockThreads;
    const uint64_t strideL = P->stride[L];  // number of choice combinations of all other tasks
    const uint32_t CL = P->C[L];
    const uint32_t n_strips = A.chunk_groups;  // strips of the last task's choices touched by the index range
    const uint32_t strip_first = A.cl_first;
    // choice combinations of the other tasks touched by the range: far_span of them, cyclically from far_first
    const uint64_t items = A.far_span * n_strips;
    const double npd = static_cast<double>(P->n_paths);
    // a power of two of task paths: dividing by it is multiplying by its inverse, exactly
    const bool np_pow2 = (P->n_paths & (P->n_paths - 1)) == 0;
    const double np_inv = 1.0 / npd;
    const int parL = n >= 2 ? P->parent[L] : 0;
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int64_t Dn[kMaxTasks];
#pragma unroll
    for (int i = 0; i < kMaxTasks; i++) Dn[i] = A.Dn[static_cast<size_t>(m) * kMaxTasks + i];

    double bacc = -1.0;
    int32_t bw = kNever;
    uint64_t bidx = ~0ull;
    uint64_t nfeas = 0;
    uint32_t waiting = 0;  // plans in this wavefront's queue (the same in every lane)

    // the first `count` lanes take the queue entries [from, from + count) and walk them
    auto walk_queued = [&](uint32_t from, uint32_t count) {
        if constexpr (kQueue) {
            if (lane < count) {
                const uint64_t idx = sWalkIdx[wave][from + lane];
                const int32_t entry = sWalkW[wave][from + lane];
                const int32_t workers = entry & ~kWalkCheckLatency;
                uint32_t c[kMaxTasks];
                uint64_t rest = idx;
#pragma unroll
                for (int i = 0; i < kMaxTasks; i++) {
                    c[i] = 0;
                    if (i < n) {
                        c[i] = static_cast<uint32_t>(rest % P->C[i]);
                        rest /= P->C[i];
                    }
                }
                bool feasible = true;
                if constexpr (LAT) {
                    if (entry & kWalkCheckLatency) {
                        feasible = !some_path_too_slow<kLatLevels>(P, c, Dn, A.budget);
                        if (feasible) nfeas++;
                    }
                }
                if (feasible) {
                    double acc;
                    if constexpr (MAXD > 0) acc = path_objective<MAXD>(P, A.path_acc, c, Dn);
                    else acc = sWalkAcc[wave][from + lane];
                    if (better(acc, workers, idx, bacc, bw, bidx, tie_index_only)) {
                        bacc = acc;
                        bw = workers;
                        bidx = idx;
                    }
                }
            }
        }
    };
    auto task_of = [&](int i, uint32_t ci, int64_t dn, TaskOut &t) {
        if constexpr (LAT) eval_task_any(P, i, ci, dn, t);
        else eval_task<PV, VF, NARROW, ScalarProblem>(P, i, ci, dn, t, PS);
    };
    bool no_room = false;   // some chain's communication latency alone exceeds the SLO: nothing is feasible
    if constexpr (LAT) {
#pragma unroll
        for (int i = 0; i < kMaxTasks; i++)
            if (i < n && P->is_leaf[i] && A.budget[i] < 0) no_room = true;
    }

    const uint64_t first_item = static_cast<uint64_t>(blockIdx.x) * kBlockThreads + threadIdx.x;
    const uint64_t rounds = (items + lanes - 1) / lanes;
    for (uint64_t round = 0; round < rounds; round++) {
        const uint64_t item = first_item + round * lanes;
        bool live = item < items;
        const uint64_t oi = live ? item / n_strips : 0;
        const uint32_t strip = strip_first + static_cast<uint32_t>(item - oi * n_strips);
        uint64_t o = A.far_first + oi;  // index of the plan with the last task's choice 0
        if (o >= strideL) o -= strideL;
        const uint32_t c_lo = strip * kStrip;
        const uint32_t c_hi = c_lo + kStrip < CL ? c_lo + kStrip : CL;
        // strips wholly outside [begin, end) are not scored
        if (live && (o + strideL * c_lo >= A.end || o + strideL * (c_hi - 1) < A.begin)) live = false;
        if constexpr (!kQueue) {
            if (!live) continue;
        }

        // ---- the shared part: tasks 0 .. L-1
        double pp[kMaxTasks];    // product of accuracies root..i, root first
        int64_t pl[kMaxTasks];   // latency sum root..i
        int64_t plt[kMaxTasks], plb[kMaxTasks];  // the same over the first / the last variants in use (LAT)
        int64_t out[kMaxTasks];  // requests task i creates per unit of child fan-out
        uint32_t mask0 = 0;
        int32_t workers0 = 0;
        bool below0 = false;     // LAT: a variant path that surely carries requests is too slow already
#pragma unroll
        for (int i = 0; i < kMaxTasks; i++) {
            pp[i] = 0.0;
            pl[i] = 0;
            plt[i] = 0;
            plb[i] = 0;
            out[i] = 0;
        }
        double presum = 0.0;
        bool first = true;
        if (live) {
            uint64_t rest = o;
#pragma unroll
            for (int i = 0; i < kMaxTasks; i++) {
                if (i < L) {
                    const uint32_t ci = static_cast<uint32_t>(rest % P->C[i]);
                    rest /= P->C[i];
                    const int par = i > 0 ? P->parent[i] : 0;
                    int64_t dn = Dn[i];
                    if (has_vf && i > 0) dn = pick_below(out, par, i) * static_cast<int64_t>(P->fanout[i]);
                    TaskOut t;
                    task_of(i, ci, dn, t);
                    out[i] = t.outflow;
                    workers0 += t.w;
                    if (!t.any) mask0 |= kBadEmpty;
                    if (t.rem > 0) mask0 |= kBadDemand;
                    const double a = task_accuracy(t, dn);
                    if (i == 0) {
                        pp[0] = a;
                        pl[0] = t.maxlat;
                    } else {
                        pp[i] = pick_below(pp, par, i) * a;
                        pl[i] = pick_below(pl, par, i) + t.maxlat;
                    }
                    if constexpr (LAT) {
                        plt[i] = (i == 0 ? 0 : pick_below(plt, par, i)) + t.lat_top;
                        plb[i] = (i == 0 ? 0 : pick_below(plb, par, i)) + t.lat_bot;
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < kMaxTasks; i++) {
                if (i < L && P->is_leaf[i]) {
                    if (A.budget[i] < 0 || pl[i] > A.budget[i]) mask0 |= kBadLatency;
                    if (LAT && (plt[i] > A.budget[i] || plb[i] > A.budget[i])) below0 = true;
                    presum = first ? pp[i] : presum + pp[i];
                    first = false;
                }
            }
        }
        const double pre = pick_below(pp, parL, kMaxTasks);
        const int64_t lat_pre = n >= 2 ? pick_below(pl, parL, kMaxTasks) : 0;
        const int64_t top_pre = LAT && n >= 2 ? pick_below(plt, parL, kMaxTasks) : 0;
        const int64_t bot_pre = LAT && n >= 2 ? pick_below(plb, parL, kMaxTasks) : 0;
        int64_t dnL = Dn[L];
        if (has_vf && n >= 2) dnL = pick_below(out, parL, kMaxTasks) * static_cast<int64_t>(P->fanout[L]);

        // ---- the strip: the last task's choices
        const uint32_t steps = kQueue ? kStrip : c_hi - c_lo;
        // one batch size per task: the last task's choice is decoded at the head of the strip and stepped from
        // there; the plan's index likewise
        [[maybe_unused]] ChoiceParts partsL;
        if constexpr (kStepChoice) decode_choice<false>(PS, L, c_lo, partsL);
        uint64_t idx_next = o + strideL * c_lo;
        for (uint32_t step = 0; step < steps; step++) {
            const uint32_t cL = c_lo + step;
            const uint64_t idx = idx_next;
            idx_next += strideL;
            bool feasible = false;  // by the per-task latency bound and everything else
            bool to_queue = false;
            int32_t workers = 0, entry = 0;
            double acc = 0.0;
            if (live && cL < c_hi && idx >= A.begin && idx < A.end) {
                TaskOut t;
                if constexpr (kStepChoice) fill_task<PV, VF, NARROW>(P, PS, L, partsL, dnL, t);
                else task_of(L, cL, dnL, t);
                uint32_t mask = mask0;
                workers = workers0 + t.w;
                if (!t.any) mask |= kBadEmpty;
                if (t.rem > 0) mask |= kBadDemand;
                if (workers > A.W) mask |= kBadWorkers;                                            // eq. (3)
                if (A.budget[L] < 0 || lat_pre + t.maxlat > A.budget[L]) mask |= kBadLatency;  // eq. (7)
                feasible = mask == 0;
                // feasible but for the per-task bound: the variant paths with traffic decide
                const bool open = LAT && mask == kBadLatency && !no_room && !below0 &&
                                  top_pre + t.lat_top <= A.budget[L] && bot_pre + t.lat_bot <= A.budget[L];
                if constexpr (MAXD == 0) {
                    if (feasible || open) {
                        const double a = task_accuracy(t, dnL);
                        const double path = n >= 2 ? pre * a : a;
                        const double sum = first ? path : presum + path;
                        acc = np_pow2 ? sum * np_inv : sum / npd;
                        if (feasible && better(acc, workers, idx, bacc, bw, bidx, tie_index_only)) {
                            bacc = acc;
                            bw = workers;
                            bidx = idx;
                        }
                    }
                }
                if (feasible) nfeas++;
                to_queue = (MAXD > 0 && feasible) || open;
                entry = open ? workers | kWalkCheckLatency : workers;
            }
            if constexpr (kQueue) {
                // every lane of the wavefront is here: queue the plans to walk, walk 64 when there are that many
                const uint64_t vote = __ballot(to_queue);
                if (vote) {
                    if (to_queue) {
                        const uint32_t at = waiting + __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(vote >> 32),
                                                          __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(vote), 0u));
                        sWalkIdx[wave][at] = idx;
                        sWalkW[wave][at] = entry;
                        if constexpr (LAT && MAXD == 0) sWalkAcc[wave][at] = acc;
                    }
                    waiting += static_cast<uint32_t>(__popcll(vote));
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                    if (waiting >= 64) {
                        waiting -= 64;
                        walk_queued(waiting, 64);
                        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                    }
                }
            }
            if constexpr (kStepChoice) next_choice(PS, L, partsL);
        }
    }
    if constexpr (kQueue) walk_queued(0, waiting);
    nfeas = wave_sum(nfeas);
    block_store_best(bacc, bw, bidx, nfeas, tie_index_only, sBest,
                     A.recs + static_cast<size_t>(m) * A.blocks_per_m + blockIdx.x);
}

// ---- kernel: merge the block records of each demand point -------------------------------------------------
__global__ void __launch_bounds__(kBlockThreads) final_reduce_kernel(SearchArgs A) {
    __shared__ BestRec sBest[kWavesPerBlock];
    __shared__ BestRec sOut;
    const int m = blockIdx.x;
    const bool tie_index_only = A.tie_index_only != 0;
    const BestRec *recs = A.recs + static_cast<size_t>(m) * A.blocks_per_m;
    double bacc = -1.0;
    int32_t bw = kNever;
    uint64_t bidx = ~0ull;
    uint64_t nfeas = 0;
    for (uint32_t b = threadIdx.x; b < A.blocks_per_m; b += kBlockThreads) {
        const BestRec r = recs[b];
        nfeas += r.nfeas;
        if (r.found && better(r.acc, r.w, r.idx, bacc, bw, bidx, tie_index_only)) {
            bacc = r.acc;
            bw = r.w;
            bidx = r.idx;
        }
    }
    nfeas = wave_sum(nfeas);
    block_store_best(bacc, bw, bidx, nfeas, tie_index_only, sBest, &sOut);
    __syncthreads();
    if (threadIdx.x == 0) {
        ResultOut o;
        if (sOut.found) {
            o.index = sOut.idx;
            o.accuracy = sOut.acc;
            o.workers_used = sOut.w;
            o.status = 0;
        } else {
            o.index = ~0ull;
            o.accuracy = 0.0;
            o.workers_used = -1;
            o.status = 1;
        }
        o.n_feasible = sOut.nfeas;
        static_cast<ResultOut *>(A.results)[m] = o;
    }
}

// ---- kernel: score listed plans ------------------------------------------------------------------------------
__global__ void __launch_bounds__(kBlockThreads) eval_kernel(EvalArgs A) {
    __shared__ DevProblem sP;
    stage_problem(&sP, A.P, sizeof(DevProblem));
    __syncthreads();
    const int64_t t = static_cast<int64_t>(blockIdx.x) * kBlockThreads + threadIdx.x;
    if (t >= A.n) return;
    uint64_t rest = A.indices[t];
    uint32_t c[kMaxTasks];
#pragma unroll
    for (int i = 0; i < kMaxTasks; i++) {
        c[i] = 0;
        if (i < sP.n_tasks) {
            c[i] = static_cast<uint32_t>(rest % sP.C[i]);
            rest /= sP.C[i];
        }
    }
    uint32_t mask;
    int32_t workers;
    double acc;
    eval_plan(&sP, c, A.Dn, A.budget, A.W, mask, workers, acc);
    if (sP.lat_per_path && !(mask & (kBadDemand | kBadEmpty)) && some_path_too_slow<kMaxTasks>(&sP, c, A.Dn, A.budget)) {
        mask |= kBadLatency;
        acc = 0.0;
    }
    if (A.path_acc && mask == 0) acc = path_objective<kMaxTasks>(&sP, A.path_acc, c, A.Dn);
    EvalOut o;
    o.accuracy = acc;
    o.workers = workers;
    o.infeasible = mask;
    static_cast<EvalOut *>(A.out)[t] = o;
}

// ---- kernel: routing tables of listed plans, one lane per plan ---------------------------------------------
// Algorithm 1 (MostAccurateFirst) with all replicas of a variant treated as one worker of
// capacity x*q: tasks in topological order, a task's workers by accuracy, each worker's outgoing
// requests placed on the child's workers by accuracy while capacity lasts.  Not a hot path: the
// lane works directly on its output record in global memory.
__device__ int64_t route_place(const DevProblem *P, RouteOut &r, int j, int64_t amount, double *prob_row) {
    const int64_t total = amount;
    for (int o = 0; o < P->K[j] && amount > 0; o++) {
        const int k = P->order[j][o];
        const int64_t room = r.leftover[j][k];
        const int64_t take = amount < room ? amount : room;
        if (take <= 0) continue;
        prob_row[k] = static_cast<double>(take) / static_cast<double>(total);
        r.leftover[j][k] = room - take;
        r.routed[j][k] += take;
        amount -= take;
    }
    return amount;
}

__global__ void __launch_bounds__(kBlockThreads) route_kernel(RouteArgs A) {
    const int64_t t = static_cast<int64_t>(blockIdx.x) * kBlockThreads + threadIdx.x;
    if (t >= A.n) return;
    const DevProblem *P = A.P;
    RouteOut &r = A.out[t];
    uint64_t *words = reinterpret_cast<uint64_t *>(&r);
    for (uint32_t q = 0; q < sizeof(RouteOut) / 8; q++) words[q] = 0;
    const int n = P->n_tasks;
    uint64_t rest = A.indices[t];
    for (int i = 0; i < n; i++) {
        uint64_t c = rest % P->C[i];
        rest /= P->C[i];
        const uint32_t nb = static_cast<uint32_t>(P->nb[i]);
        uint32_t beta[kMaxVariants];
        for (int k = 0; k < P->K[i]; k++) {
            const uint64_t g = c % P->radix[i][k];
            c /= P->radix[i][k];
            if (P->pv_batch) {
                r.replicas[i][k] = g == 0 ? 0 : static_cast<int32_t>((g - 1) / nb) + 1;
                beta[k] = g == 0 ? 0u : static_cast<uint32_t>((g - 1) % nb);
            } else {
                r.replicas[i][k] = static_cast<int32_t>(g);
            }
        }
        r.scale[i] = P->scale[i];
        r.demand[i] = i == 0 ? A.demand[t] : r.demand[P->parent[i]] * P->fanout[i];  // replaced below with r(i,k)
        for (int k = 0; k < P->K[i]; k++) {
            const uint32_t b = P->pv_batch ? beta[k] : static_cast<uint32_t>(c);
            const bool hosted = r.replicas[i][k] > 0;
            r.batch[i][k] = hosted ? P->batch_size[i][b] : 0;
            r.capacity[i][k] = static_cast<int64_t>(r.replicas[i][k]) * P->thr_s[i][k][b];
            r.leftover[i][k] = r.capacity[i][k];
            r.budget_us[i][k] = hosted ? P->lat[i][k][b] : 0;
        }
    }
    r.unserved[0] = route_place(P, r, 0, r.demand[0], r.prob[0][0]);
    for (int i = 0; i < n; i++)
        for (int o = 0; o < P->K[i]; o++) {
            const int k = P->order[i][o];
            for (int j = i + 1; j < n; j++) {
                if (P->parent[j] != i) continue;
                int64_t created = r.routed[i][k] * static_cast<int64_t>(P->fanout[j]);
                if (P->has_vf) {  // the child's demand is what the parent's variants create
                    created *= P->vf[i][k];
                    if (o == 0) r.demand[j] = 0;
                    r.demand[j] += created;
                }
                r.unserved[j] += route_place(P, r, j, created, r.prob[j][k]);
            }
        }
}

// ---- kernels: results of (demand point, class) pairs -> results of the demand points ------------------
__global__ void results_init_kernel(MergeArgs A) {
    const int m = blockIdx.x * blockDim.x + threadIdx.x;
    if (m >= A.M) return;
    ResultOut o;
    o.index = ~0ull;
    o.accuracy = 0.0;
    o.n_feasible = 0;
    o.workers_used = -1;
    o.status = 1;
    static_cast<ResultOut *>(A.results)[m] = o;
}

// The classes of a demand point follow one another.  Two launches: first every stretch is cut into pieces
// of at most kMergePiece classes (a piece starts at a multiple of kMergePiece or where the point changes)
// and the thread of a piece's first class folds the piece into that class's slot; then the thread of a
// stretch's first class folds the piece heads into the point's result (a point's classes may continue in
// the next batch, hence the read of what is there).
constexpr int kMergePiece = 32;

__device__ __forceinline__ void merge_result(ResultOut &o, const ResultOut &c, bool tie_index_only) {
    o.n_feasible += c.n_feasible;
    if (c.status == 0 && (o.status != 0 || better(c.accuracy, c.workers_used, c.index, o.accuracy, o.workers_used,
                                                  o.index, tie_index_only))) {
        o.index = c.index;
        o.accuracy = c.accuracy;
        o.workers_used = c.workers_used;
        o.status = 0;
    }
}

template <bool PIECES>
__global__ void __launch_bounds__(kBlockThreads) class_merge_kernel(MergeArgs A) {
    const int v0 = blockIdx.x * kBlockThreads + threadIdx.x;
    if (v0 >= A.n) return;
    const int point = A.point[v0];
    const bool stretch_start = v0 == 0 || A.point[v0 - 1] != point;
    ResultOut *in = static_cast<ResultOut *>(A.class_results);
    const bool tie_index_only = A.tie_index_only != 0;
    if (PIECES) {
        if (!stretch_start && v0 % kMergePiece != 0) return;
        const int end = (v0 / kMergePiece + 1) * kMergePiece;
        ResultOut o = in[v0];
        for (int v = v0 + 1; v < A.n && v < end && A.point[v] == point; v++) merge_result(o, in[v], tie_index_only);
        in[v0] = o;
    } else {
        if (!stretch_start) return;
        ResultOut *out = static_cast<ResultOut *>(A.results);
        ResultOut o = out[point];
        for (int v = v0; v < A.n && A.point[v] == point; v = (v / kMergePiece + 1) * kMergePiece)
            merge_result(o, in[v], tie_index_only);
        out[point] = o;
    }
}

// results[m] takes in other[m]: feasible counts added, the better plan kept.
__global__ void fold_results_kernel(void *results, const void *other, int M, uint32_t tie_index_only) {
    const int m = blockIdx.x * blockDim.x + threadIdx.x;
    if (m >= M) return;
    ResultOut o = static_cast<ResultOut *>(results)[m];
    merge_result(o, static_cast<const ResultOut *>(other)[m], tie_index_only != 0);
    static_cast<ResultOut *>(results)[m] = o;
}

template <int S>
hipError_t launch_combine_s(const SearchArgs &A, bool has_presum, bool divide, bool range, bool leaf_values,
                            hipStream_t stream) {
    const dim3 grid(A.blocks_per_m, A.M), block(kBlockThreads);
    if (leaf_values) {
        // profiled path accuracies, one value per leaf (the caller has checked: swapped roles, a leaf in the
        // tiles, at most kMaxPrefix branches above every leaf)
        if (!A.swap || !has_presum) return hipErrorInvalidValue;
#define LOKI_LAUNCH_PATHS(D, R) hipLaunchKernelGGL((combine_kernel<S, true, D, R, true, true>), grid, block, 0, stream, A);
        if (divide) {
            if (range) { LOKI_LAUNCH_PATHS(true, true) } else { LOKI_LAUNCH_PATHS(true, false) }
        } else {
            if (range) { LOKI_LAUNCH_PATHS(false, true) } else { LOKI_LAUNCH_PATHS(false, false) }
        }
#undef LOKI_LAUNCH_PATHS
        return hipGetLastError();
    }
    if (A.swap) {
#define LOKI_LAUNCH_SWAP(P, D)                                                                                   \
    if (range) hipLaunchKernelGGL((combine_kernel<S, P, D, true, true>), grid, block, 0, stream, A);             \
    else hipLaunchKernelGGL((combine_kernel<S, P, D, false, true>), grid, block, 0, stream, A);
        if (!has_presum) { LOKI_LAUNCH_SWAP(false, false) }
        else if (divide) { LOKI_LAUNCH_SWAP(true, true) }
        else { LOKI_LAUNCH_SWAP(true, false) }
#undef LOKI_LAUNCH_SWAP
        return hipGetLastError();
    }
#define LOKI_LAUNCH(P, D, R)                                                            \
    hipLaunchKernelGGL((combine_kernel<S, P, D, R, false>), grid, block, 0, stream, A); \
    return hipGetLastError();
    if (has_presum) {
        if (divide) {
            if (range) { LOKI_LAUNCH(true, true, true) } else { LOKI_LAUNCH(true, true, false) }
        } else {
            if (range) { LOKI_LAUNCH(true, false, true) } else { LOKI_LAUNCH(true, false, false) }
        }
    } else {
        if (range) { LOKI_LAUNCH(false, false, true) } else { LOKI_LAUNCH(false, false, false) }
    }
#undef LOKI_LAUNCH
}

}  // namespace

hipError_t launch_task_table(const SearchArgs &A, uint32_t table_total, hipStream_t stream) {
    const dim3 grid((table_total + kBlockThreads - 1) / kBlockThreads, A.M), block(kBlockThreads);
    hipLaunchKernelGGL(task_table_kernel, grid, block, 0, stream, A);
    return hipGetLastError();
}

hipError_t launch_root_order(const SearchArgs &A, hipStream_t stream) {
    hipLaunchKernelGGL(root_order_kernel, dim3(A.M, A.swap ? A.swap_tasks : 1), dim3(kSortThreads), 0, stream, A);
    return hipGetLastError();
}

hipError_t launch_combine(const SearchArgs &A, int slots, bool has_presum, bool divide, bool range,
                          bool leaf_values, hipStream_t stream) {
    if (slots == 8) return launch_combine_s<8>(A, has_presum, divide, range, leaf_values, stream);
    return launch_combine_s<4>(A, has_presum, divide, range, leaf_values, stream);
}

template <int MAXD>
void launch_per_lane_depth(const SearchArgs &A, bool pv_batch, bool has_vf, hipStream_t stream) {
    const dim3 grid(A.blocks_per_m, A.M), block(kBlockThreads);
    if constexpr (MAXD == 0) {
        if (A.narrow) {
            if (pv_batch) {
                if (has_vf) hipLaunchKernelGGL((per_lane_search_kernel<true, true, 0, 0, true>), grid, block, 0, stream, A);
                else hipLaunchKernelGGL((per_lane_search_kernel<true, false, 0, 0, true>), grid, block, 0, stream, A);
            } else {
                if (has_vf) hipLaunchKernelGGL((per_lane_search_kernel<false, true, 0, 0, true>), grid, block, 0, stream, A);
                else hipLaunchKernelGGL((per_lane_search_kernel<false, false, 0, 0, true>), grid, block, 0, stream, A);
            }
            return;
        }
    }
    if (pv_batch) {
        if (has_vf) hipLaunchKernelGGL((per_lane_search_kernel<true, true, MAXD>), grid, block, 0, stream, A);
        else hipLaunchKernelGGL((per_lane_search_kernel<true, false, MAXD>), grid, block, 0, stream, A);
    } else {
        if (has_vf) hipLaunchKernelGGL((per_lane_search_kernel<false, true, MAXD>), grid, block, 0, stream, A);
        else hipLaunchKernelGGL((per_lane_search_kernel<false, false, MAXD>), grid, block, 0, stream, A);
    }
}

hipError_t launch_per_lane_search(const SearchArgs &A, bool pv_batch, bool has_vf, int path_levels, int latency_levels,
                                  hipStream_t stream) {
    if (latency_levels > 0) {
        const dim3 grid(A.blocks_per_m, A.M), block(kBlockThreads);
        const bool deep = latency_levels > 4;
        if (path_levels <= 0) {
            if (deep) hipLaunchKernelGGL((per_lane_search_kernel<false, false, 0, kMaxTasks>), grid, block, 0, stream, A);
            else hipLaunchKernelGGL((per_lane_search_kernel<false, false, 0, 4>), grid, block, 0, stream, A);
        } else if (deep) {
            hipLaunchKernelGGL((per_lane_search_kernel<false, false, kMaxTasks, kMaxTasks>), grid, block, 0, stream, A);
        } else {
            hipLaunchKernelGGL((per_lane_search_kernel<false, false, 4, 4>), grid, block, 0, stream, A);
        }
        return hipGetLastError();
    }
    if (path_levels <= 0) launch_per_lane_depth<0>(A, pv_batch, has_vf, stream);
    else if (path_levels <= 4) launch_per_lane_depth<4>(A, pv_batch, has_vf, stream);
    else launch_per_lane_depth<kMaxTasks>(A, pv_batch, has_vf, stream);
    return hipGetLastError();
}

template <int S, int MAXD>
hipError_t launch_path_combine_s(const SearchArgs &A, bool range, hipStream_t stream) {
    const dim3 grid(A.blocks_per_m, A.M), block(kBlockThreads);
    if (A.swap) {
        if (range) hipLaunchKernelGGL((path_combine_kernel<S, true, MAXD, true>), grid, block, 0, stream, A);
        else hipLaunchKernelGGL((path_combine_kernel<S, false, MAXD, true>), grid, block, 0, stream, A);
    } else {
        if (range) hipLaunchKernelGGL((path_combine_kernel<S, true, MAXD, false>), grid, block, 0, stream, A);
        else hipLaunchKernelGGL((path_combine_kernel<S, false, MAXD, false>), grid, block, 0, stream, A);
    }
    return hipGetLastError();
}

hipError_t launch_path_combine(const SearchArgs &A, int slots, bool range, int path_levels, hipStream_t stream) {
    if (path_levels <= 4)
        return slots == 8 ? launch_path_combine_s<8, 4>(A, range, stream) : launch_path_combine_s<4, 4>(A, range, stream);
    return slots == 8 ? launch_path_combine_s<8, kMaxTasks>(A, range, stream)
                      : launch_path_combine_s<4, kMaxTasks>(A, range, stream);
}

template <int S, int LATD>
hipError_t launch_open_plans_s(const SearchArgs &A, bool range, hipStream_t stream) {
    const dim3 grid(A.blocks_per_m, A.M), block(kBlockThreads);
    if (range) hipLaunchKernelGGL((open_plans_kernel<S, true, LATD>), grid, block, 0, stream, A);
    else hipLaunchKernelGGL((open_plans_kernel<S, false, LATD>), grid, block, 0, stream, A);
    return hipGetLastError();
}

hipError_t launch_open_plans(const SearchArgs &A, int slots, bool range, int latency_levels, hipStream_t stream) {
    if (latency_levels <= 4)
        return slots == 8 ? launch_open_plans_s<8, 4>(A, range, stream) : launch_open_plans_s<4, 4>(A, range, stream);
    return slots == 8 ? launch_open_plans_s<8, kMaxTasks>(A, range, stream)
                      : launch_open_plans_s<4, kMaxTasks>(A, range, stream);
}

hipError_t launch_fold_results(void *results, const void *other, int M, bool tie_index_only, hipStream_t stream) {
    hipLaunchKernelGGL(fold_results_kernel, dim3((M + 255) / 256), dim3(256), 0, stream, results, other, M,
                       tie_index_only ? 1u : 0u);
    return hipGetLastError();
}

hipError_t launch_final_reduce(const SearchArgs &A, hipStream_t stream) {
    const dim3 grid(A.M), block(kBlockThreads);
    hipLaunchKernelGGL(final_reduce_kernel, grid, block, 0, stream, A);
    return hipGetLastError();
}

hipError_t launch_results_init(const MergeArgs &A, hipStream_t stream) {
    hipLaunchKernelGGL(results_init_kernel, dim3((A.M + 255) / 256), dim3(256), 0, stream, A);
    return hipGetLastError();
}

hipError_t launch_class_merge(const MergeArgs &A, hipStream_t stream) {
    const dim3 grid((A.n + kBlockThreads - 1) / kBlockThreads), block(kBlockThreads);
    hipLaunchKernelGGL(class_merge_kernel<true>, grid, block, 0, stream, A);
    hipLaunchKernelGGL(class_merge_kernel<false>, grid, block, 0, stream, A);
    return hipGetLastError();
}

hipError_t launch_route(const RouteArgs &A, hipStream_t stream) {
    const dim3 grid(static_cast<uint32_t>((A.n + kBlockThreads - 1) / kBlockThreads)), block(kBlockThreads);
    hipLaunchKernelGGL(route_kernel, grid, block, 0, stream, A);
    return hipGetLastError();
}

hipError_t launch_eval(const EvalArgs &A, hipStream_t stream) {
    const dim3 grid(static_cast<uint32_t>((A.n + kBlockThreads - 1) / kBlockThreads)), block(kBlockThreads);
    hipLaunchKernelGGL(eval_kernel, grid, block, 0, stream, A);
    return hipGetLastError();
}

}  // namespace loki

// Drives the C-ABI of the CPU build of the library's host side (hip_stubs.cpp in the place of the HIP
// runtime and of the kernels) over one problem read from a text file.  Prints what the host computes itself
// (plan space, decoded plans, routing tables) for the test to compare with the CPU checker; searches and
// evaluations only have to run clean under the sanitizers.
#include <cinttypes>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../include/loki_alloc.h"

static std::vector<int64_t> read_list(FILE *f) {
    long long n = 0;
    if (std::fscanf(f, "%lld", &n) != 1 || n < 0) std::exit(3);
    std::vector<int64_t> v(static_cast<size_t>(n));
    for (auto &x : v) {
        long long t;
        if (std::fscanf(f, "%lld", &t) != 1) std::exit(3);
        x = t;
    }
    return v;
}
static std::vector<int32_t> narrow(const std::vector<int64_t> &v) { return std::vector<int32_t>(v.begin(), v.end()); }

int main(int argc, char **argv) {
    if (argc < 2) return 2;
    FILE *f = std::fopen(argv[1], "r");
    if (!f) return 2;
    const auto head = read_list(f);  // n_tasks, per_variant_batch, has_vf, has_path, workers, slo, comm, latency_per_path
    const auto parent = narrow(read_list(f)), fanout = narrow(read_list(f)), nv = narrow(read_list(f)),
               nb = narrow(read_list(f)), bs = narrow(read_list(f)), rep = narrow(read_list(f)),
               acc = narrow(read_list(f));
    const auto lat = read_list(f), thr = read_list(f);
    const auto vf = narrow(read_list(f)), path = narrow(read_list(f));
    const auto demands = read_list(f);
    const auto indices = read_list(f);   // plans to decode / route / evaluate
    const auto ranges = read_list(f);    // begin,end pairs for range searches
    std::fclose(f);
    loki_pipeline_t P{};
    P.n_tasks = int32_t(head[0]);
    P.parent = parent.data();
    P.fanout_q4 = fanout.data();
    P.n_variants = nv.data();
    P.n_batches = nb.data();
    P.batch_size = bs.data();
    P.max_replicas = rep.data();
    P.acc_ppm = acc.data();
    P.latency_us = lat.data();
    P.thr_mqps = thr.data();
    P.per_variant_batch = int32_t(head[1]);
    P.variant_factor_q4 = head[2] ? vf.data() : nullptr;
    P.path_acc_ppm = head[3] ? path.data() : nullptr;
    P.latency_per_path = head.size() > 7 ? int32_t(head[7]) : 0;
    const int32_t workers = int32_t(head[4]);
    const int64_t slo = head[5], comm = head[6];
    loki_problem_t *h = nullptr;
    int rc = loki_problem_create(&P, &h);
    std::printf("create %d\n", rc);
    if (rc) return 0;
    uint64_t N = 0;
    rc = loki_num_candidates(h, &N);
    std::printf("candidates %d %" PRIu64 "\n", rc, N);
    const int32_t M = int32_t(demands.size());
    size_t bytes = 0;
    rc = loki_workspace_bytes(h, M > 0 ? M : 1, &bytes);
    size_t eval_bytes = 0;
    (void)loki_workspace_bytes(h, int64_t(indices.size() > 0 ? indices.size() : 1), &eval_bytes);
    if (eval_bytes > bytes) bytes = eval_bytes;
    std::printf("workspace %d %zu\n", rc, bytes);
    void *ws = std::aligned_alloc(256, (bytes + 255) / 256 * 256);
    int nvar = 0;
    for (int i = 0; i < P.n_tasks; i++) nvar += nv[size_t(i)];
    std::vector<int32_t> x(static_cast<size_t>(nvar)), b(static_cast<size_t>(nvar));
    for (int64_t idx : indices) {
        rc = loki_decode(h, uint64_t(idx), x.data(), b.data());
        std::printf("decode %d %" PRId64, rc, idx);
        if (!rc) {
            for (int v : x) std::printf(" %d", v);
            std::printf(" |");
            for (int q = 0; q < (P.per_variant_batch ? nvar : P.n_tasks); q++) std::printf(" %d", b[size_t(q)]);
        }
        std::printf("\n");
        loki_route_t r;
        rc = loki_route_table(h, uint64_t(idx), demands.empty() ? 0 : demands[0], &r);
        std::printf("route %d", rc);
        if (!rc)
            for (int i = 0; i < P.n_tasks; i++)
                for (int k = 0; k < nv[size_t(i)]; k++)
                    std::printf(" %" PRId64 ":%" PRId64, r.routed[i][k], r.leftover[i][k]);
        std::printf("\n");
    }
    std::vector<loki_result_t> out(static_cast<size_t>(M > 0 ? M : 1));
    if (M > 0) {
        for (uint32_t flags : {0u, 1u, 2u, 3u}) {
            rc = loki_alloc_search(h, demands.data(), M, workers, slo, comm, flags, 0, N, ws, bytes, nullptr, out.data());
            std::printf("search flags %u rc %d status", flags, rc);
            for (int m = 0; m < M && m < 8; m++) std::printf(" %d", out[size_t(m)].status);
            std::printf("\n");
            uint64_t scored = 0;
            float ms[3];
            const int rc_scored = loki_last_search_plans_scored(h, &scored);
            std::printf("scored %d %" PRIu64 " ms %d\n", rc_scored, scored, loki_last_search_ms(h, ms));
        }
        for (size_t q = 0; q + 1 < ranges.size(); q += 2)
            for (uint32_t flags : {0u, 2u}) {
                rc = loki_alloc_search(h, demands.data(), M, workers, slo, comm, flags, uint64_t(ranges[q]),
                                       uint64_t(ranges[q + 1]), ws, bytes, nullptr, out.data());
                std::printf("range %" PRId64 " %" PRId64 " flags %u rc %d\n", ranges[q], ranges[q + 1], flags, rc);
            }
        // the enqueue form, the planner, and error paths that must not touch the workspace
        rc = loki_alloc_search_enqueue(h, demands.data(), M, workers, slo, comm, 0, 0, N, ws, bytes, nullptr, out.data());
        std::printf("enqueue %d\n", rc);
        std::vector<loki_plan_step_t> steps(static_cast<size_t>(M));
        rc = loki_plan_trace(h, demands.data(), M, 300000, workers, slo, comm, 0, ws, bytes, nullptr, steps.data());
        std::printf("trace %d\n", rc);
        std::printf("too small %d\n", loki_alloc_search(h, demands.data(), M, workers, slo, comm, 0, 0, N, ws, 1024,
                                                         nullptr, out.data()));
        std::printf("misaligned %d\n", loki_alloc_search(h, demands.data(), M, workers, slo, comm, 0, 0, N,
                                                          static_cast<char *>(ws) + 8, bytes - 8, nullptr, out.data()));
        std::printf("reversed %d\n", loki_alloc_search(h, demands.data(), M, workers, slo, comm, 0, N, 0, ws, bytes,
                                                        nullptr, out.data()));
        std::vector<int64_t> bad(demands);
        bad.back() = -1;
        std::printf("negative demand %d\n", loki_alloc_search(h, bad.data(), M, workers, slo, comm, 0, 0, N, ws, bytes,
                                                               nullptr, out.data()));
        bad.back() = INT64_MAX / 2;
        std::printf("huge demand %d\n", loki_alloc_search(h, bad.data(), M, workers, slo, comm, 0, 0, N, ws, bytes,
                                                           nullptr, out.data()));
    }
    if (!indices.empty()) {
        std::vector<uint64_t> ix(indices.begin(), indices.end());
        std::vector<loki_eval_t> ev(ix.size());
        rc = loki_alloc_eval(h, ix.data(), int64_t(ix.size()), demands.empty() ? 0 : demands[0], workers, slo, comm, ws,
                             bytes, nullptr, ev.data());
        std::printf("eval %d\n", rc);
        size_t rb = 0;
        (void)loki_route_workspace_bytes(h, int64_t(ix.size()), &rb);
        void *rws = std::aligned_alloc(256, (rb + 255) / 256 * 256);
        std::vector<loki_route_t> routes(ix.size());
        std::vector<int64_t> dd(ix.size(), demands.empty() ? 0 : demands[0]);
        rc = loki_route_table_batch(h, ix.data(), dd.data(), int64_t(ix.size()), rws, rb, nullptr, routes.data());
        std::printf("route batch %d\n", rc);
        std::free(rws);
    }
    std::free(ws);
    loki_problem_destroy(h);
    std::printf("done\n");
    return 0;
}

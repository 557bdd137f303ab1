// Host planner and online sampler on random graphs, batch sizes, thread counts and both
// schedules, plus two malformed batches; built with sanitizers by tests/test_host_sanitizers.py.
#include <cstdio>
#include <cstdlib>
#include <random>
#include <string>
#include <vector>
#include "ngdb.h"
#include "planner.h"
int main() {
    const int N = 5000, R = 37; const int64_t T = 60000;
    std::mt19937_64 rng(7);
    std::vector<int32_t> h(T), r(T), t(T);
    for (int64_t i = 0; i < T; ++i) { h[i] = rng() % N; r[i] = rng() % R; t[i] = (rng() % 7 == 0) ? rng() % 50 : rng() % N; }
    const char* names = "1p,2p,3p,2i,3i,ip,pi,2u,up,2in,3in,inp,pin,pni";
    for (int threads : {1, 3, 8}) {
        ngdb_sampler_t* s = nullptr;
        int rc = ngdb_sampler_create(N, R, T, h.data(), r.data(), t.data(), names, nullptr, 11, threads, &s);
        if (rc) { printf("create rc %d\n", rc); return 1; }
        for (int it = 0; it < 40; ++it) {
            ngdb_query_batch qb; const int32_t* neg; const uint8_t* tid;
            const int B = 1 + (int)(rng() % 700), K = (int)(rng() % 40);
            rc = ngdb_sampler_next(s, B, K, &qb, &neg, &tid);
            if (rc) { printf("next rc %d %s\n", rc, ngdb_sampler_last_error(s)); return 1; }
            for (int sched = 0; sched < 2; ++sched) {
                ngdb::HostPlan hp; std::string err;
                rc = ngdb::build_plan(qb, N, R, sched, sched ? (int)(rng() % 50) : 0, hp, err);
                if (rc) { printf("plan rc %d %s\n", rc, err.c_str()); return 1; }
            }
        }
        // equal sizes call after call: the library reads the next batch ahead while this one is in
        // use; a batch must stay unchanged over the call that follows it
        uint64_t sum_prev = 0; const int32_t* arg_prev = nullptr; int64_t n_prev = 0;
        for (int it = 0; it < 12; ++it) {
            ngdb_query_batch qb; const int32_t* neg; const uint8_t* tid;
            rc = ngdb_sampler_next(s, 300, 16, &qb, &neg, &tid);
            if (rc) { printf("next rc %d %s\n", rc, ngdb_sampler_last_error(s)); return 1; }
            if (arg_prev) {
                uint64_t again = 0;
                for (int64_t i = 0; i < n_prev; ++i) again = again * 1000003u + (uint32_t)arg_prev[i];
                if (again != sum_prev) { printf("batch %d changed during the next call\n", it - 1); return 1; }
            }
            n_prev = qb.node_off[qb.n_queries]; arg_prev = qb.arg; sum_prev = 0;
            for (int64_t i = 0; i < n_prev; ++i) sum_prev = sum_prev * 1000003u + (uint32_t)arg_prev[i];
        }
        ngdb_sampler_destroy(s);     // with a batch being read ahead
    }
    // malformed batches must be rejected, not crash
    {
        std::vector<int32_t> node_off{0, 3}, arg{1, 2, 0}, in_off{0, 0, 1, 3}, in_idx{0, 1, 7}, pos{1};
        std::vector<uint8_t> op{0, 1, 2};
        ngdb_query_batch qb{1, node_off.data(), op.data(), arg.data(), in_off.data(), in_idx.data(), pos.data()};
        ngdb::HostPlan hp; std::string err;
        int rc = ngdb::build_plan(qb, N, R, 0, 0, hp, err);
        printf("malformed: rc %d (%s)\n", rc, err.c_str());
        in_idx[2] = 1; arg[1] = 99999;
        rc = ngdb::build_plan(qb, N, R, 0, 0, hp, err);
        printf("range: rc %d (%s)\n", rc, err.c_str());
    }
    printf("ok\n");
    return 0;
}

// Replays a script of scheduler, cache-manager and loop events through the library's host code
// (csrc/serving.cpp and csrc/kvm.cpp compiled with -fsanitize=address,undefined) and prints what
// the code decided after every event; tests/test_sanitizers.py writes the script from the
// oracle's random drive and compares the printed decisions with the oracle's.  No GPU: the
// manager runs without layer pools.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "fastserve_kvm.h"

static fs_sched *S = nullptr;
static fs_kvm *K = nullptr;
static fs_serve *L = nullptr;

#define NEED(cond)                                                            \
    do {                                                                      \
        if (!(cond)) {                                                        \
            std::fprintf(stderr, "replay: line %d: %s failed\n", lineno, #cond); \
            return 2;                                                         \
        }                                                                     \
    } while (0)

static void print_job(fs_kvm *k, long long j)
{
    int32_t state = -1, n = 0, ids[64];
    int64_t len = -1;
    if (fs_kvm_job_info(k, j, &state, &len, ids, 64, &n) != FS_OK) {
        std::printf(" %lld:gone", j);
        return;
    }
    std::printf(" %lld:%d:%lld:", j, state, (long long)len);
    for (int i = 0; i < n && i < 64; ++i) std::printf("%s%d", i ? "," : "", ids[i]);
}

int main()
{
    char line[4096];
    int lineno = 0;
    while (std::fgets(line, sizeof line, stdin)) {
        ++lineno;
        std::vector<std::string> t;
        for (char *p = std::strtok(line, " \n"); p; p = std::strtok(nullptr, " \n")) t.emplace_back(p);
        if (t.empty()) continue;
        auto I = [&](size_t i) { return std::atoll(t.at(i).c_str()); };
        auto D = [&](size_t i) { return std::atof(t.at(i).c_str()); };
        const std::string &c = t[0];
        if (c == "sched") {
            NEED(fs_sched_create((int32_t)I(1), D(2), (int32_t)I(3), D(4), (int32_t)I(5), &S) == FS_OK);
        } else if (c == "kvm") {
            fs_kvm_config cfg{};
            cfg.num_blocks = (int32_t)I(1), cfg.num_host_blocks = (int32_t)I(2), cfg.block_size = (int32_t)I(3);
            cfg.table_width = (int32_t)I(4), cfg.reserve_idle_blocks = (int32_t)I(5), cfg.reserve_window = (int32_t)I(6);
            cfg.reserve_quantile = D(7);
            NEED(fs_kvm_create(&cfg, nullptr, 0, S, &K) == FS_OK);
        } else if (c == "add") {
            int32_t q = 0;
            NEED(fs_sched_add_job(S, I(1), D(2), D(3), &q) == FS_OK);
            std::printf("add %d\n", q);
        } else if (c == "ready") {
            NEED(fs_sched_set_ready(S, I(1), (int32_t)I(2)) == FS_OK);
        } else if (c == "batch") {
            int64_t ids[64];
            int32_t n = 0;
            NEED(fs_sched_schedule(S, ids, 64, &n) == FS_OK);
            std::printf("batch");
            for (int i = 0; i < n; ++i) std::printf(" %lld", (long long)ids[i]);
            std::printf("\n");
        } else if (c == "done") {  // done elapsed n_ran ids... n_fin ids...
            std::vector<int64_t> ran, fin;
            size_t p = 2;
            for (long long n = I(p++); n > 0; --n) ran.push_back(I(p++));
            for (long long n = I(p++); n > 0; --n) fin.push_back(I(p++));
            NEED(fs_sched_complete_iteration(S, ran.data(), (int32_t)ran.size(), D(1), fin.data(), (int32_t)fin.size()) == FS_OK);
        } else if (c == "admit") {
            const int rc = fs_kvm_admit(K, I(1), I(2));
            NEED(rc == FS_OK || rc == FS_ERR_OOM);
            std::printf("admit %d\n", rc == FS_OK);
        } else if (c == "grow") {
            int32_t ok = 0;
            NEED(fs_kvm_grow(K, I(1), (int32_t)I(2), &ok) == FS_OK);
            if (ok) NEED(fs_kvm_advance(K, I(1), (int32_t)I(2)) == FS_OK);
            std::printf("grow %d\n", ok);
        } else if (c == "swaps") {  // swaps want n ids...
            std::vector<int64_t> run;
            size_t p = 2;
            for (long long n = I(p++); n > 0; --n) run.push_back(I(p++));
            NEED(fs_kvm_start_swaps(K, run.data(), (int32_t)run.size(), (int32_t)I(1), nullptr) == FS_OK);
        } else if (c == "retire") {
            int32_t n = 0;
            NEED(fs_kvm_retire(K, (int32_t)I(1), 0, &n) == FS_OK);
            std::printf("retire %d\n", n);
        } else if (c == "observe") {
            NEED(fs_kvm_observe_arrivals(K, (int32_t)I(1)) == FS_OK);
        } else if (c == "release") {
            NEED(fs_kvm_release(K, I(1)) == FS_OK);
        } else if (c == "state") {  // state n ids... : free lists, reserve, traffic, the named jobs
            fs_kvm *k = L ? fs_serve_manager(L) : K;
            int64_t out = 0, in = 0;
            int32_t fly = 0;
            NEED(fs_kvm_stats(k, &out, &in, &fly) == FS_OK);
            std::printf("state %d %d %d %lld %lld %d", fs_kvm_free_blocks(k), fs_kvm_free_slots(k), fs_kvm_reserve(k),
                        (long long)out, (long long)in, fly);
            size_t p = 1;
            for (long long n = I(p++); n > 0; --n) print_job(k, I(p++));
            std::printf("\n");
        } else if (c == "loop") {  // loop nq q1 eta alpha B maxprompt blocks slots bs W reserve window quantile
            fs_serve_config cfg{};
            cfg.num_queues = (int32_t)I(1), cfg.q1 = D(2), cfg.eta = (int32_t)I(3), cfg.alpha = D(4);
            cfg.max_batch = (int32_t)I(5), cfg.max_prompt_tokens = I(6);
            cfg.kvm.num_blocks = (int32_t)I(7), cfg.kvm.num_host_blocks = (int32_t)I(8), cfg.kvm.block_size = (int32_t)I(9);
            cfg.kvm.table_width = (int32_t)I(10), cfg.kvm.reserve_idle_blocks = (int32_t)I(11);
            cfg.kvm.reserve_window = (int32_t)I(12), cfg.kvm.reserve_quantile = D(13);
            NEED(fs_serve_create(&cfg, nullptr, 0, &L) == FS_OK);
        } else if (c == "submit") {
            NEED(fs_serve_submit(L, I(1), I(2), (int32_t)I(3), (int32_t)I(4), D(5), D(6)) == FS_OK);
        } else if (c == "plan") {
            fs_serve_iteration it;
            NEED(fs_serve_plan(L, nullptr, &it) == FS_OK);
            std::printf("plan first");
            for (int i = 0; i < it.n_first; ++i) std::printf(" %lld", (long long)it.first_ids[i]);
            std::printf(" decode");
            for (int i = 0; i < it.n_decode; ++i) std::printf(" %lld@%d", (long long)it.decode_ids[i], it.lens_before[i]);
            std::printf(" waiting %d left %d\n", it.n_waiting, it.n_unfinished);
            NEED(fs_serve_complete(L) == FS_OK);
        } else {
            std::fprintf(stderr, "replay: line %d: unknown command %s\n", lineno, c.c_str());
            return 2;
        }
    }
    if (L) {
        fs_serve_stats st;
        if (fs_serve_get_stats(L, &st) == FS_OK)
            std::printf("stats %lld %lld %lld %lld\n", (long long)st.iterations, (long long)st.job_tokens,
                        (long long)st.prompt_tokens, (long long)st.finished_jobs);
        fs_serve_destroy(L);
    }
    if (K) fs_kvm_destroy(K);
    if (S) fs_sched_destroy(S);
    std::printf("replay ok\n");
    return 0;
}

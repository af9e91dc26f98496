// Host-side serving policy of FastServe (arXiv 2305.05920): skip-join MLFQ scheduler
// (Section 4.1, Algorithm 1) and the ENST swap-order estimate (Section 4.2).
// C ABI in include/fastserve_sched.h.  Plain C++; no GPU calls.
#include <algorithm>
#include <deque>
#include <new>
#include <unordered_map>
#include <unordered_set>
#include <vector>

#include "fastserve.h"
#include "fastserve_sched.h"

namespace {

struct JobState {
    double init_time = 0, decode_time = 0;
    int priority = 1;      // queue index, 1 = highest
    double used = 0;       // consumed part of the current quantum
    double starve = 0;     // waited since it last ran, arrived or was promoted
    int64_t iterations = 0;
    bool ready = true;
    double next_iter_time() const { return iterations == 0 ? init_time : decode_time; }
};

}  // namespace

struct fs_sched {
    int n = 1, eta = 1, max_batch = 1;
    double alpha = 0;
    std::vector<double> quantum;              // quantum[k-1] of Q_k
    std::vector<std::deque<int64_t>> queues;  // job ids, front = oldest
    std::unordered_map<int64_t, JobState> jobs;

    int queue_for(double t) const {
        for (int i = 0; i < n; ++i)
            if (quantum[i] >= t) return i + 1;
        return n;
    }
    void erase_from(int p, int64_t id) {
        auto &q = queues[p - 1];
        q.erase(std::find(q.begin(), q.end(), id));
    }
    double t_execute(const JobState &ji) const {
        // prefix[k] = q_1 + ... + q_k
        double total = 0;
        for (const auto &kv : jobs) {
            const JobState &o = kv.second;
            if (o.priority < ji.priority)
                for (int k = o.priority; k < ji.priority; ++k) total += quantum[k - 1];
        }
        return total / max_batch;
    }
};

extern "C" {

int fs_sched_create(int32_t num_queues, double q1, int32_t eta, double alpha, int32_t max_batch, fs_sched **out)
{
    if (!out || num_queues < 1 || num_queues > 62 || !(q1 > 0) || eta < 1 || !(alpha > 0) || max_batch < 1)
        return FS_ERR_INVALID_ARG;
    fs_sched *s = new (std::nothrow) fs_sched();
    if (!s) return FS_ERR_OOM;
    s->n = num_queues;
    s->eta = eta;
    s->alpha = alpha;
    s->max_batch = max_batch;
    s->quantum.resize(num_queues);
    double q = q1;
    for (int i = 0; i < num_queues; ++i, q *= 2) s->quantum[i] = q;
    s->queues.resize(num_queues);
    *out = s;
    return FS_OK;
}

int fs_sched_destroy(fs_sched *s)
{
    if (!s) return FS_ERR_INVALID_ARG;
    delete s;
    return FS_OK;
}

int fs_sched_add_job(fs_sched *s, int64_t job_id, double init_time, double decode_time, int32_t *queue_out)
{
    if (!s || !(init_time >= 0) || !(decode_time >= 0) || s->jobs.count(job_id)) return FS_ERR_INVALID_ARG;
    JobState st;
    st.init_time = init_time;
    st.decode_time = decode_time;
    st.priority = s->queue_for(init_time);
    s->jobs.emplace(job_id, st);
    s->queues[st.priority - 1].push_back(job_id);
    if (queue_out) *queue_out = st.priority;
    return FS_OK;
}

int fs_sched_set_ready(fs_sched *s, int64_t job_id, int32_t ready)
{
    if (!s) return FS_ERR_INVALID_ARG;
    auto it = s->jobs.find(job_id);
    if (it == s->jobs.end()) return FS_ERR_INVALID_ARG;
    it->second.ready = ready != 0;
    return FS_OK;
}

int fs_sched_schedule(const fs_sched *s, int64_t *out_ids, int32_t cap, int32_t *n_out)
{
    if (!s || !out_ids || !n_out || cap < 0) return FS_ERR_INVALID_ARG;
    const int limit = cap < s->max_batch ? cap : s->max_batch;
    int n = 0;
    for (const auto &q : s->queues)
        for (int64_t id : q) {
            if (n >= limit) {
                *n_out = n;
                return FS_OK;
            }
            if (s->jobs.at(id).ready) out_ids[n++] = id;
        }
    *n_out = n;
    return FS_OK;
}

int fs_sched_complete_iteration(fs_sched *s, const int64_t *ran, int32_t n_ran, double elapsed,
                                const int64_t *finished, int32_t n_finished)
{
    if (!s || n_ran < 0 || n_finished < 0 || (n_ran && !ran) || (n_finished && !finished) || !(elapsed >= 0))
        return FS_ERR_INVALID_ARG;
    std::unordered_set<int64_t> ran_set(ran, ran + n_ran), fin(finished, finished + n_finished);
    for (int64_t id : ran_set)
        if (!s->jobs.count(id)) return FS_ERR_INVALID_ARG;
    for (int64_t id : fin)
        if (!ran_set.count(id)) return FS_ERR_INVALID_ARG;
    // visit order fixed before anything moves: Q_1 .. Q_n, oldest first
    std::vector<int64_t> order;
    for (const auto &q : s->queues) order.insert(order.end(), q.begin(), q.end());
    for (int64_t id : order) {
        JobState &job = s->jobs.at(id);
        const int p = job.priority;
        if (ran_set.count(id)) {
            job.iterations += 1;
            job.used += elapsed;
            job.starve = 0;
            if (fin.count(id)) {
                s->erase_from(p, id);
                s->jobs.erase(id);
                continue;
            }
            if (job.used >= s->quantum[p - 1]) {  // quantum used up: demote
                int target = std::max(p + s->eta, s->queue_for(job.next_iter_time()));
                if (target > s->n) target = s->n;
                s->erase_from(p, id);
                s->queues[target - 1].push_back(id);
                job.priority = target;
                job.used = 0;
            }
        } else {
            job.starve += elapsed;
            if (job.starve >= s->alpha) {  // starved: promote
                if (p != 1) {
                    s->erase_from(p, id);
                    s->queues[0].push_back(id);
                    job.priority = 1;
                    job.used = 0;
                }
                job.starve = 0;
            }
        }
    }
    return FS_OK;
}

int fs_sched_job_info(const fs_sched *s, int64_t job_id, int32_t *priority, double *used, double *starve,
                      int64_t *iterations)
{
    if (!s) return FS_ERR_INVALID_ARG;
    auto it = s->jobs.find(job_id);
    if (it == s->jobs.end()) return FS_ERR_INVALID_ARG;
    if (priority) *priority = it->second.priority;
    if (used) *used = it->second.used;
    if (starve) *starve = it->second.starve;
    if (iterations) *iterations = it->second.iterations;
    return FS_OK;
}

int32_t fs_sched_num_jobs(const fs_sched *s) { return s ? (int32_t)s->jobs.size() : -1; }

int fs_sched_enst(const fs_sched *s, int64_t job_id, double *t_promote, double *t_execute, double *enst)
{
    if (!s) return FS_ERR_INVALID_ARG;
    auto it = s->jobs.find(job_id);
    if (it == s->jobs.end()) return FS_ERR_INVALID_ARG;
    const double tp = std::max(0.0, s->alpha - it->second.starve);
    const double te = s->t_execute(it->second);
    if (t_promote) *t_promote = tp;
    if (t_execute) *t_execute = te;
    if (enst) *enst = std::min(tp, te);
    return FS_OK;
}

int fs_sched_swap_order(const fs_sched *s, const int64_t *candidates, int32_t n, int32_t swap_in, int64_t *ordered)
{
    if (!s || n < 0 || (n && (!candidates || !ordered))) return FS_ERR_INVALID_ARG;
    struct Key {
        double enst;
        int priority;
        int64_t id;
    };
    std::vector<Key> keys;
    keys.reserve(n);
    for (int i = 0; i < n; ++i) {
        auto it = s->jobs.find(candidates[i]);
        if (it == s->jobs.end()) return FS_ERR_INVALID_ARG;
        const double tp = std::max(0.0, s->alpha - it->second.starve);
        keys.push_back({std::min(tp, s->t_execute(it->second)), it->second.priority, candidates[i]});
    }
    if (swap_in)
        std::sort(keys.begin(), keys.end(), [](const Key &a, const Key &b) {
            if (a.enst != b.enst) return a.enst < b.enst;
            if (a.priority != b.priority) return a.priority < b.priority;
            return a.id < b.id;
        });
    else
        std::sort(keys.begin(), keys.end(), [](const Key &a, const Key &b) {
            if (a.enst != b.enst) return a.enst > b.enst;
            if (a.priority != b.priority) return a.priority > b.priority;
            return a.id > b.id;
        });
    for (int i = 0; i < n; ++i) ordered[i] = keys[i].id;
    return FS_OK;
}

}  // extern "C"

// Proactive key-value cache manager of FastServe (arXiv 2305.05920, Section 4.2) and the
// iteration loop that drives scheduler, manager and attention kernels (Section 3.2,
// Algorithm 1).  C ABI in include/fastserve_kvm.h.  Host code: the only GPU work issued
// here is block copies (through fs_pool_offload / fs_pool_upload), the small copy kernel that
// brings a batch's tables over (fs_stream_copy), events and stream waits.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstring>
#include <deque>
#include <functional>
#include <new>
#include <unordered_map>
#include <unordered_set>
#include <vector>

#include "fastserve_kvm.h"

namespace {

enum JobWhere : int32_t { kResident = 0, kLeaving = 1, kSwappedOut = 2, kReturning = 3 };

struct JobBlocks {
    int64_t length = 0;             // tokens cached
    std::vector<int32_t> blocks;    // pool block ids (resident, returning)
    std::vector<int32_t> slots;     // host slots (leaving, swapped out)
    JobWhere where = kResident;
    bool released = false;          // left while a copy of its blocks was in flight
};

struct Swap {
    int64_t job = 0;
    bool out = false;               // offload (true) or upload
    std::vector<int32_t> vacated;   // blocks an offload frees / slots an upload frees, at retirement
    hipEvent_t done = nullptr;      // recorded on the side stream after the copies (null without layers)
};

// Staging ring: kStageSlots slots in groups of kStageGroup.  A batch's words are written into a
// slot's pinned memory and brought to its device memory by a copy kernel on the kernels' own
// stream (one launch; an asynchronous copy of a few KiB costs the host several times that), so the
// device words are in order with their readers by themselves.  The pinned words are rewritten
// one whole turn of the ring later; what guards that is one event per group, not per slot.
constexpr int kStageSlots = 64;
constexpr int kStageGroup = 16;
constexpr int kStageGroups = kStageSlots / kStageGroup;

struct StageSlot {
    int32_t *host = nullptr;        // pinned
    int32_t *dev = nullptr;
};

}  // namespace

struct fs_kvm {
    fs_kvm_config cfg{};
    std::vector<fs_pool *> layers;
    fs_sched *sched = nullptr;
    int reserve = 0;
    std::deque<int32_t> demand;                   // arrival history (blocks per iteration)
    std::vector<int32_t> free_blocks, free_slots; // stacks: back = next to hand out
    std::unordered_map<int64_t, JobBlocks> jobs;
    std::deque<Swap> in_flight;                   // issue order
    std::vector<hipEvent_t> spare_events;
    hipStream_t side = nullptr;
    hipEvent_t fence = nullptr;                   // compute stream -> side stream
    StageSlot ring[kStageSlots];
    hipEvent_t group_used[kStageGroups] = {};     // the kernels' stream has passed every batch of the group
    size_t stage_words = 0;
    int64_t staged = 0;
    int64_t blocks_out = 0, blocks_in = 0;

    int needed(int64_t tokens) const { return (int)((tokens + cfg.block_size - 1) / cfg.block_size); }
    int blocks_leaving() const {
        int n = 0;
        for (const Swap &s : in_flight)
            if (s.out) n += (int)s.vacated.size();
        return n;
    }
    // The free lists are kept in falling order, so that the back is the lowest free id: jobs
    // get runs of neighbouring ids where there are any, and neighbours travel as one copy.
    static void put_back(std::vector<int32_t> &list, const std::vector<int32_t> &ids) {
        if (ids.empty()) return;
        list.insert(list.end(), ids.begin(), ids.end());
        std::sort(list.begin(), list.end(), std::greater<int32_t>());
    }
    void give_back(JobBlocks &jb) {
        put_back(free_blocks, jb.blocks);
        put_back(free_slots, jb.slots);
        jb.blocks.clear();
        jb.slots.clear();
    }
};

namespace {

int take_event(fs_kvm *k, hipEvent_t *ev)
{
    if (!k->spare_events.empty()) {
        *ev = k->spare_events.back();
        k->spare_events.pop_back();
        return FS_OK;
    }
    return hipEventCreateWithFlags(ev, hipEventDisableTiming) == hipSuccess ? FS_OK : FS_ERR_HIP;
}

int move_job(fs_kvm *k, int64_t id, bool out)
{
    JobBlocks &jb = k->jobs.at(id);
    const size_t n = out ? jb.blocks.size() : jb.slots.size();
    std::vector<int32_t> fresh(n);
    std::vector<int32_t> &pool_of_fresh = out ? k->free_slots : k->free_blocks;
    for (size_t i = 0; i < n; ++i) {
        fresh[i] = pool_of_fresh.back();
        pool_of_fresh.pop_back();
    }
    Swap sw;
    sw.job = id;
    sw.out = out;
    const std::vector<int32_t> &blocks = out ? jb.blocks : fresh;
    const std::vector<int32_t> &slots = out ? fresh : jb.slots;
    for (fs_pool *layer : k->layers) {
        const int rc = out ? fs_pool_offload(layer, blocks.data(), slots.data(), (int32_t)n, k->side)
                           : fs_pool_upload(layer, slots.data(), blocks.data(), (int32_t)n, k->side);
        if (rc != FS_OK) return rc;
    }
    if (!k->layers.empty()) {
        if (take_event(k, &sw.done) != FS_OK) return FS_ERR_HIP;
        if (hipEventRecord(sw.done, k->side) != hipSuccess) return FS_ERR_HIP;
    }
    const int64_t moved = (int64_t)n * (k->layers.empty() ? 1 : (int64_t)k->layers.size());
    if (out) {
        k->blocks_out += moved;
        sw.vacated = jb.blocks;
        jb.slots = fresh;
        jb.blocks.clear();
        jb.where = kLeaving;
        if (k->sched) (void)fs_sched_set_ready(k->sched, id, 0);
    } else {
        k->blocks_in += moved;
        sw.vacated = jb.slots;
        jb.blocks = fresh;
        jb.slots.clear();
        jb.where = kReturning;
    }
    k->in_flight.push_back(std::move(sw));
    return FS_OK;
}

}  // namespace

extern "C" {

int fs_kvm_create(const fs_kvm_config *cfg, fs_pool *const *layers, int32_t num_layers, fs_sched *sched, fs_kvm **out)
{
    if (!cfg || !out || num_layers < 0 || (num_layers && !layers)) return FS_ERR_INVALID_ARG;
    if (cfg->num_blocks < 1 || cfg->num_host_blocks < 0 || cfg->block_size < 1 || cfg->table_width < 1 ||
        cfg->reserve_idle_blocks < 0 || cfg->reserve_window < 0 || !(cfg->reserve_quantile >= 0.0) ||
        !(cfg->reserve_quantile <= 1.0) || cfg->max_batch < 0 || cfg->max_staged_extra < 0)
        return FS_ERR_INVALID_ARG;
    for (int i = 0; i < num_layers; ++i)
        if (!layers[i] || fs_pool_block_bytes(layers[i]) == 0) return FS_ERR_INVALID_ARG;
    fs_kvm *k = new (std::nothrow) fs_kvm();
    if (!k) return FS_ERR_OOM;
    k->cfg = *cfg;
    k->sched = sched;
    k->reserve = cfg->reserve_idle_blocks;
    k->layers.assign(layers, layers + num_layers);
    for (int b = cfg->num_blocks - 1; b >= 0; --b) k->free_blocks.push_back(b);
    for (int s = cfg->num_host_blocks - 1; s >= 0; --s) k->free_slots.push_back(s);
    if (num_layers) {
        bool ok = hipStreamCreateWithFlags(&k->side, hipStreamNonBlocking) == hipSuccess &&
                  hipEventCreateWithFlags(&k->fence, hipEventDisableTiming) == hipSuccess;
        k->stage_words = (size_t)cfg->max_batch * cfg->table_width + cfg->max_batch + cfg->max_staged_extra;
        const size_t bytes = (std::max<size_t>(k->stage_words, 1) * sizeof(int32_t) + 15) / 16 * 16;
        for (int i = 0; ok && i < kStageSlots; ++i) {
            StageSlot &s = k->ring[i];
            ok = hipHostMalloc((void **)&s.host, bytes, hipHostMallocDefault) == hipSuccess &&
                 hipMalloc((void **)&s.dev, bytes) == hipSuccess;
        }
        for (int g = 0; ok && g < kStageGroups; ++g)
            ok = hipEventCreateWithFlags(&k->group_used[g], hipEventDisableTiming) == hipSuccess;
        if (!ok) {
            (void)hipGetLastError();
            fs_kvm_destroy(k);
            return FS_ERR_OOM;
        }
    }
    *out = k;
    return FS_OK;
}

int fs_kvm_destroy(fs_kvm *k)
{
    if (!k) return FS_ERR_INVALID_ARG;
    if (k->side) (void)hipStreamSynchronize(k->side);
    for (Swap &s : k->in_flight)
        if (s.done) (void)hipEventDestroy(s.done);
    for (hipEvent_t e : k->spare_events) (void)hipEventDestroy(e);
    // (the caller has drained the stream its kernels run on: they read the device words)
    for (StageSlot &s : k->ring) {
        if (s.host) (void)hipHostFree(s.host);
        if (s.dev) (void)hipFree(s.dev);
    }
    for (hipEvent_t e : k->group_used)
        if (e) (void)hipEventDestroy(e);
    if (k->fence) (void)hipEventDestroy(k->fence);
    if (k->side) (void)hipStreamDestroy(k->side);
    delete k;
    return FS_OK;
}

int32_t fs_kvm_blocks_needed(const fs_kvm *k, int64_t tokens) { return (k && tokens >= 0) ? k->needed(tokens) : -1; }
int32_t fs_kvm_free_blocks(const fs_kvm *k) { return k ? (int32_t)k->free_blocks.size() : -1; }
int32_t fs_kvm_free_slots(const fs_kvm *k) { return k ? (int32_t)k->free_slots.size() : -1; }
int32_t fs_kvm_reserve(const fs_kvm *k) { return k ? k->reserve : -1; }

int fs_kvm_observe_arrivals(fs_kvm *k, int32_t blocks_demanded)
{
    if (!k || blocks_demanded < 0) return FS_ERR_INVALID_ARG;
    if (k->cfg.reserve_window <= 0) return FS_OK;
    k->demand.push_back(blocks_demanded);
    if ((int)k->demand.size() > k->cfg.reserve_window) k->demand.pop_front();
    std::vector<int32_t> ordered(k->demand.begin(), k->demand.end());
    std::sort(ordered.begin(), ordered.end());
    const int n = (int)ordered.size();
    int rank = (int)std::ceil(k->cfg.reserve_quantile * n) - 1;  // the ceil(quantile * n)-th smallest
    rank = std::max(0, std::min(n - 1, rank));
    int r = std::max(k->cfg.reserve_idle_blocks, ordered[rank]);
    k->reserve = std::min(r, std::max(k->cfg.reserve_idle_blocks, k->cfg.num_blocks / 2));
    return FS_OK;
}

int fs_kvm_admit(fs_kvm *k, int64_t id, int64_t tokens)
{
    if (!k || tokens < 0 || k->jobs.count(id)) return FS_ERR_INVALID_ARG;
    const int n = k->needed(tokens);
    if (n > (int)k->free_blocks.size() || n > k->cfg.table_width) return FS_ERR_OOM;
    JobBlocks jb;
    for (int i = 0; i < n; ++i) {
        jb.blocks.push_back(k->free_blocks.back());
        k->free_blocks.pop_back();
    }
    k->jobs.emplace(id, std::move(jb));
    return FS_OK;
}

int fs_kvm_grow(fs_kvm *k, int64_t id, int32_t new_tokens, int32_t *ok)
{
    if (!k || !ok || new_tokens < 0) return FS_ERR_INVALID_ARG;
    auto it = k->jobs.find(id);
    if (it == k->jobs.end() || it->second.where != kResident || it->second.released) return FS_ERR_INVALID_ARG;
    JobBlocks &jb = it->second;
    const int need = k->needed(jb.length + new_tokens) - (int)jb.blocks.size();
    if (need > (int)k->free_blocks.size() || (int)jb.blocks.size() + need > k->cfg.table_width) {
        *ok = 0;
        return FS_OK;
    }
    for (int i = 0; i < need; ++i) {
        jb.blocks.push_back(k->free_blocks.back());
        k->free_blocks.pop_back();
    }
    *ok = 1;
    return FS_OK;
}

int fs_kvm_advance(fs_kvm *k, int64_t id, int32_t tokens)
{
    if (!k || tokens < 0) return FS_ERR_INVALID_ARG;
    auto it = k->jobs.find(id);
    if (it == k->jobs.end() || it->second.released) return FS_ERR_INVALID_ARG;
    it->second.length += tokens;
    return FS_OK;
}

int fs_kvm_release(fs_kvm *k, int64_t id)
{
    if (!k) return FS_ERR_INVALID_ARG;
    auto it = k->jobs.find(id);
    if (it == k->jobs.end() || it->second.released) return FS_ERR_INVALID_ARG;
    JobBlocks &jb = it->second;
    if (jb.where == kLeaving || jb.where == kReturning) {
        jb.released = true;  // a copy still reads or writes its blocks and slots: freed when the swap retires
        return FS_OK;
    }
    k->give_back(jb);
    k->jobs.erase(it);
    return FS_OK;
}

int fs_kvm_start_swaps(fs_kvm *k, const int64_t *running, int32_t n_running, int32_t want_free, void *compute_stream)
{
    if (!k || n_running < 0 || (n_running && !running) || want_free < 0) return FS_ERR_INVALID_ARG;
    if (!k->sched) return FS_ERR_INVALID_ARG;
    const std::unordered_set<int64_t> run(running, running + n_running);
    const long long margin = (long long)k->reserve + want_free;
    std::vector<int64_t> cand, ordered;
    // ---- out: largest estimated next scheduled time first ----
    for (const auto &kv : k->jobs)
        if (kv.second.where == kResident && !kv.second.released && !kv.second.blocks.empty() && !run.count(kv.first))
            cand.push_back(kv.first);
    std::sort(cand.begin(), cand.end());
    ordered.resize(cand.size());
    if (!cand.empty() && fs_sched_swap_order(k->sched, cand.data(), (int32_t)cand.size(), 0, ordered.data()) != FS_OK)
        return FS_ERR_INVALID_ARG;
    bool fenced = false;
    auto fence_once = [&]() -> int {
        // the copies must see everything the compute stream has been given so far
        if (fenced || k->layers.empty()) return FS_OK;
        if (hipEventRecord(k->fence, (hipStream_t)compute_stream) != hipSuccess ||
            hipStreamWaitEvent(k->side, k->fence, 0) != hipSuccess)
            return FS_ERR_HIP;
        fenced = true;
        return FS_OK;
    };
    long long free_soon = (long long)k->free_blocks.size() + k->blocks_leaving();
    for (int64_t id : ordered) {
        if (free_soon >= margin) break;
        const JobBlocks &jb = k->jobs.at(id);
        if (jb.blocks.size() > k->free_slots.size()) continue;
        free_soon += (long long)jb.blocks.size();
        int rc = fence_once();
        if (rc == FS_OK) rc = move_job(k, id, true);
        if (rc != FS_OK) return rc;
    }
    // ---- in: smallest estimated next scheduled time first ----
    cand.clear();
    for (const auto &kv : k->jobs)
        if (kv.second.where == kSwappedOut && !kv.second.released) cand.push_back(kv.first);
    std::sort(cand.begin(), cand.end());
    ordered.resize(cand.size());
    if (!cand.empty() && fs_sched_swap_order(k->sched, cand.data(), (int32_t)cand.size(), 1, ordered.data()) != FS_OK)
        return FS_ERR_INVALID_ARG;
    for (int64_t id : ordered) {
        const long long n = (long long)k->jobs.at(id).slots.size();
        if ((long long)k->free_blocks.size() - n < margin) break;
        int rc = fence_once();
        if (rc == FS_OK) rc = move_job(k, id, false);
        if (rc != FS_OK) return rc;
    }
    return FS_OK;
}

int fs_kvm_retire(fs_kvm *k, int32_t max_swaps, int32_t wait, int32_t *retired)
{
    if (!k) return FS_ERR_INVALID_ARG;
    int n = 0;
    while (!k->in_flight.empty() && (max_swaps < 0 || n < max_swaps)) {
        Swap &sw = k->in_flight.front();
        if (sw.done) {
            if (wait) {
                if (hipEventSynchronize(sw.done) != hipSuccess) return FS_ERR_HIP;
            } else {
                const hipError_t e = hipEventQuery(sw.done);
                if (e == hipErrorNotReady) {
                    (void)hipGetLastError();
                    break;
                }
                if (e != hipSuccess) return FS_ERR_HIP;
            }
            k->spare_events.push_back(sw.done);
        }
        fs_kvm::put_back(sw.out ? k->free_blocks : k->free_slots, sw.vacated);
        auto it = k->jobs.find(sw.job);
        if (it != k->jobs.end()) {
            JobBlocks &jb = it->second;
            if (jb.released) {
                k->give_back(jb);
                k->jobs.erase(it);
            } else if (sw.out) {
                jb.where = kSwappedOut;
            } else {
                jb.where = kResident;
                if (k->sched) (void)fs_sched_set_ready(k->sched, sw.job, 1);
            }
        }
        k->in_flight.pop_front();
        ++n;
    }
    if (retired) *retired = n;
    return FS_OK;
}

int fs_kvm_job_info(const fs_kvm *k, int64_t id, int32_t *state, int64_t *length, int32_t *ids, int32_t cap,
                    int32_t *n)
{
    if (!k || cap < 0 || (cap && !ids)) return FS_ERR_INVALID_ARG;
    auto it = k->jobs.find(id);
    if (it == k->jobs.end() || it->second.released) return FS_ERR_INVALID_ARG;
    const JobBlocks &jb = it->second;
    if (state) *state = jb.where;
    if (length) *length = jb.length;
    const std::vector<int32_t> &v = (jb.where == kResident || jb.where == kReturning) ? jb.blocks : jb.slots;
    if (n) *n = (int32_t)v.size();
    for (int i = 0; i < cap && i < (int)v.size(); ++i) ids[i] = v[i];
    return FS_OK;
}

int fs_kvm_stats(const fs_kvm *k, int64_t *blocks_out, int64_t *blocks_in, int32_t *swaps_in_flight)
{
    if (!k) return FS_ERR_INVALID_ARG;
    if (blocks_out) *blocks_out = k->blocks_out;
    if (blocks_in) *blocks_in = k->blocks_in;
    if (swaps_in_flight) *swaps_in_flight = (int32_t)k->in_flight.size();
    return FS_OK;
}

int fs_kvm_table_rows(const fs_kvm *k, const int64_t *ids, int32_t n, int32_t *rows)
{
    if (!k || n < 0 || (n && (!ids || !rows))) return FS_ERR_INVALID_ARG;
    const int W = k->cfg.table_width;
    for (int r = 0; r < n; ++r) {
        auto it = k->jobs.find(ids[r]);
        if (it == k->jobs.end() || it->second.where != kResident || it->second.released) return FS_ERR_INVALID_ARG;
        const std::vector<int32_t> &b = it->second.blocks;
        for (int i = 0; i < W; ++i) rows[(size_t)r * W + i] = i < (int)b.size() ? b[i] : -1;
    }
    return FS_OK;
}

int fs_kvm_stage_batch(fs_kvm *k, const int64_t *ids, int32_t n, const int32_t *extra, int32_t n_extra, void *stream,
                       const int32_t **d_table, const int32_t **d_lens, const int32_t **d_extra)
{
    if (!k || n < 0 || n_extra < 0 || (n && !ids) || (n_extra && !extra) || !d_table || !d_lens || !d_extra)
        return FS_ERR_INVALID_ARG;
    if (k->layers.empty() || n > k->cfg.max_batch || n_extra > k->cfg.max_staged_extra) return FS_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    const int64_t seq = k->staged;
    const int slot_index = (int)(seq % kStageSlots);
    const int group = slot_index / kStageGroup;
    if (slot_index % kStageGroup == 0) {
        // Entering a group.  Everything that reads the group just left -- its copy kernels and the
        // kernels behind them -- has been given to the kernels' stream by now: mark that point.
        if (seq > 0 && hipEventRecord(k->group_used[(group + kStageGroups - 1) % kStageGroups], s) != hipSuccess)
            return FS_ERR_HIP;
        // This group was used one turn ago.  Its pinned words may be rewritten once the stream has
        // passed the mark set when it was left (it has, unless the GPU is most of a ring behind:
        // this bounds the host's lead over the GPU).  Its device words need no guard: the copy
        // kernel that rewrites them runs on the same stream, behind their last reader.
        if (seq >= kStageSlots && hipEventSynchronize(k->group_used[group]) != hipSuccess) return FS_ERR_HIP;
    }
    StageSlot &slot = k->ring[slot_index];
    const int W = k->cfg.table_width;
    int32_t *tab = slot.host, *len = tab + (size_t)k->cfg.max_batch * W, *ext = len + k->cfg.max_batch;
    const int rc = fs_kvm_table_rows(k, ids, n, tab);
    if (rc != FS_OK) return rc;
    for (int r = 0; r < n; ++r) len[r] = (int32_t)k->jobs.at(ids[r]).length;
    if (n_extra) std::memcpy(ext, extra, (size_t)n_extra * sizeof(int32_t));
    const size_t bytes = (((size_t)k->cfg.max_batch * W + k->cfg.max_batch + n_extra) * sizeof(int32_t) + 15) / 16 * 16;
    const int wgs = (int)((bytes / 16 + 255) / 256);
    if (fs_stream_copy(slot.dev, slot.host, bytes, wgs, stream) != FS_OK) return FS_ERR_HIP;
    k->staged += 1;
    *d_table = slot.dev;
    *d_lens = slot.dev + (size_t)k->cfg.max_batch * W;
    *d_extra = slot.dev + (size_t)k->cfg.max_batch * W + k->cfg.max_batch;
    return FS_OK;
}

}  // extern "C"

// ======================================================================================
// Iteration loop
// ======================================================================================
namespace {

struct ServeJob {
    int64_t arrival = 0;
    int32_t prompt = 0, outputs = 0, produced = 0;
    double init_time = 0, decode_time = 0;
    bool admitted = false;
};

}  // namespace

struct fs_serve {
    fs_serve_config cfg{};
    fs_sched *sched = nullptr;
    fs_kvm *kvm = nullptr;
    std::vector<fs_pool *> layers;
    std::unordered_map<int64_t, ServeJob> jobs;
    std::vector<int64_t> future;    // submitted, not yet arrived (submit order)
    std::vector<int64_t> waiting;   // arrived, not yet admitted (arrival order)
    int64_t iteration = 0;
    int64_t max_prompt_tokens = 0;
    // the planned iteration
    bool planned = false;
    std::vector<int64_t> batch, first_ids, decode_ids, runnable, stage_ids;
    std::vector<int32_t> token_offsets, lens_before;
    bool staged = false;            // this iteration's tables and lengths are on the GPU
    const int32_t *d_first_table = nullptr, *d_offsets = nullptr, *d_decode_table = nullptr, *d_lens = nullptr;
    fs_serve_stats stats{};
};

extern "C" {

int fs_serve_create(const fs_serve_config *cfg, fs_pool *const *layers, int32_t num_layers, fs_serve **out)
{
    if (!cfg || !out || num_layers < 0 || (num_layers && !layers) || cfg->max_batch < 1 || cfg->max_prompt_tokens < 0)
        return FS_ERR_INVALID_ARG;
    fs_serve *s = new (std::nothrow) fs_serve();
    if (!s) return FS_ERR_OOM;
    s->cfg = *cfg;
    s->max_prompt_tokens = cfg->max_prompt_tokens;
    s->layers.assign(layers, layers + num_layers);
    int rc = fs_sched_create(cfg->num_queues, cfg->q1, cfg->eta, cfg->alpha, cfg->max_batch, &s->sched);
    if (rc == FS_OK) {
        fs_kvm_config kc = cfg->kvm;
        kc.max_batch = cfg->max_batch;
        kc.max_staged_extra = cfg->max_batch + 1;  // the prompts' token offsets
        rc = fs_kvm_create(&kc, layers, num_layers, s->sched, &s->kvm);
    }
    if (rc != FS_OK) {
        fs_serve_destroy(s);
        return rc;
    }
    *out = s;
    return FS_OK;
}

int fs_serve_destroy(fs_serve *s)
{
    if (!s) return FS_ERR_INVALID_ARG;
    if (s->kvm) (void)fs_kvm_destroy(s->kvm);
    if (s->sched) (void)fs_sched_destroy(s->sched);
    delete s;
    return FS_OK;
}

fs_sched *fs_serve_scheduler(fs_serve *s) { return s ? s->sched : nullptr; }
fs_kvm *fs_serve_manager(fs_serve *s) { return s ? s->kvm : nullptr; }

int fs_serve_submit(fs_serve *s, int64_t id, int64_t arrival_iteration, int32_t prompt_tokens, int32_t output_tokens,
                    double init_time, double decode_time)
{
    if (!s || prompt_tokens < 1 || output_tokens < 1 || arrival_iteration < s->iteration || !(init_time >= 0) ||
        !(decode_time >= 0) || s->jobs.count(id) || s->planned)
        return FS_ERR_INVALID_ARG;
    if (fs_kvm_blocks_needed(s->kvm, (int64_t)prompt_tokens + output_tokens) > s->cfg.kvm.table_width)
        return FS_ERR_INVALID_ARG;  // the job could never hold its whole cache
    ServeJob j;
    j.arrival = arrival_iteration;
    j.prompt = prompt_tokens;
    j.outputs = output_tokens;
    j.init_time = init_time;
    j.decode_time = decode_time;
    s->jobs.emplace(id, j);
    s->future.push_back(id);
    return FS_OK;
}

int fs_serve_plan(fs_serve *s, void *stream, fs_serve_iteration *it)
{
    if (!s || !it || s->planned) return FS_ERR_INVALID_ARG;
    fs_kvm *k = s->kvm;
    // ---- arrivals of this iteration ----
    int demand = 0;
    {
        std::vector<int64_t> later;
        for (int64_t id : s->future) {
            const ServeJob &j = s->jobs.at(id);
            if (j.arrival <= s->iteration) {
                s->waiting.push_back(id);
                demand += fs_kvm_blocks_needed(k, (int64_t)j.prompt + 1);
            } else {
                later.push_back(id);
            }
        }
        s->future.swap(later);
    }
    int rc = fs_kvm_observe_arrivals(k, demand);
    if (rc == FS_OK) rc = fs_kvm_retire(k, -1, 0, nullptr);
    if (rc != FS_OK) return rc;
    // ---- admission, oldest first, beside the reserve ----
    {
        std::vector<int64_t> still;
        for (int64_t id : s->waiting) {
            ServeJob &j = s->jobs.at(id);
            const int need = fs_kvm_blocks_needed(k, (int64_t)j.prompt + 1);
            if (need + fs_kvm_reserve(k) <= fs_kvm_free_blocks(k) && fs_kvm_admit(k, id, (int64_t)j.prompt + 1) == FS_OK) {
                rc = fs_sched_add_job(s->sched, id, j.init_time, j.decode_time, nullptr);
                if (rc != FS_OK) return rc;
                j.admitted = true;
            } else {
                still.push_back(id);
            }
        }
        s->waiting.swap(still);
    }
    // ---- the batch ----
    s->batch.assign((size_t)s->cfg.max_batch, 0);
    int32_t nb = 0;
    rc = fs_sched_schedule(s->sched, s->batch.data(), s->cfg.max_batch, &nb);
    if (rc != FS_OK) return rc;
    s->batch.resize((size_t)nb);
    s->first_ids.clear();
    s->decode_ids.clear();
    s->runnable.clear();
    s->lens_before.clear();
    s->token_offsets.assign(1, 0);
    int sat_out = 0;
    int64_t prompt_tokens = 0;
    for (int64_t id : s->batch) {
        const ServeJob &j = s->jobs.at(id);
        int64_t length = 0;
        (void)fs_kvm_job_info(k, id, nullptr, &length, nullptr, 0, nullptr);
        if (length == 0) {
            // initialization phase; a prompt that does not fit this iteration's buffer waits for the next
            if (s->max_prompt_tokens > 0 && prompt_tokens + j.prompt > s->max_prompt_tokens && !s->first_ids.empty()) {
                ++sat_out;
                continue;
            }
            s->first_ids.push_back(id);
            prompt_tokens += j.prompt;
            s->token_offsets.push_back((int32_t)prompt_tokens);
        } else {
            int32_t ok = 0;
            rc = fs_kvm_grow(k, id, 1, &ok);
            if (rc != FS_OK) return rc;
            if (!ok) {
                ++sat_out;
                continue;
            }
            s->decode_ids.push_back(id);
            s->lens_before.push_back((int32_t)length);
        }
        s->runnable.push_back(id);
    }
    // ---- swaps beside this iteration's kernels: room for those that sat out and for the waiting ----
    long long want = sat_out;
    for (int64_t id : s->waiting) want += fs_kvm_blocks_needed(k, (int64_t)s->jobs.at(id).prompt + 1);
    want = std::min<long long>(want, s->cfg.kvm.num_blocks / 2);
    rc = fs_kvm_start_swaps(k, s->runnable.data(), (int32_t)s->runnable.size(), (int32_t)want, stream);
    if (rc != FS_OK) return rc;
    s->planned = true;
    s->staged = false;
    it->iteration = s->iteration;
    it->n_first = (int32_t)s->first_ids.size();
    it->first_ids = s->first_ids.data();
    it->token_offsets = s->token_offsets.data();
    it->prompt_tokens = prompt_tokens;
    it->n_decode = (int32_t)s->decode_ids.size();
    it->decode_ids = s->decode_ids.data();
    it->lens_before = s->lens_before.data();
    it->n_waiting = (int32_t)s->waiting.size();
    it->n_unfinished = (int32_t)s->jobs.size();
    return FS_OK;
}

int fs_serve_launch(fs_serve *s, int32_t layer, const fs_serve_buffers *buf, void *stream)
{
    if (!s || !buf || !s->planned || s->layers.empty() || layer < -1 || layer >= (int32_t)s->layers.size())
        return FS_ERR_INVALID_ARG;
    fs_kvm *k = s->kvm;
    const int32_t nf = (int32_t)s->first_ids.size(), nd = (int32_t)s->decode_ids.size();
    const int64_t T = s->token_offsets.back();
    if (nf && (T > buf->max_prompt_tokens || !buf->prompt_q || !buf->prompt_k || !buf->prompt_v || !buf->prompt_out))
        return FS_ERR_INVALID_ARG;
    if (nd && (!buf->decode_q || !buf->decode_k || !buf->decode_v || !buf->decode_out)) return FS_ERR_INVALID_ARG;
    if (!s->staged) {
        // Tables, lengths and prompt offsets are the same for every layer: staged once per
        // iteration, as one batch -- the first-iteration jobs' rows, then the decoding jobs'.
        s->stage_ids.assign(s->first_ids.begin(), s->first_ids.end());
        s->stage_ids.insert(s->stage_ids.end(), s->decode_ids.begin(), s->decode_ids.end());
        const int32_t *d_table = nullptr, *d_lens = nullptr, *d_extra = nullptr;
        const int rc = fs_kvm_stage_batch(k, s->stage_ids.data(), nf + nd, s->token_offsets.data(), nf ? nf + 1 : 0,
                                          stream, &d_table, &d_lens, &d_extra);
        if (rc != FS_OK) return rc;
        s->d_first_table = d_table;
        s->d_offsets = d_extra;
        s->d_decode_table = d_table + (size_t)nf * s->cfg.kvm.table_width;
        s->d_lens = d_lens + nf;
        s->staged = true;
    }
    const int32_t l0 = layer < 0 ? 0 : layer, l1 = layer < 0 ? (int32_t)s->layers.size() : layer + 1;
    for (int32_t l = l0; l < l1; ++l) {
        int rc = FS_OK;
        if (nf)
            rc = fs_prefill_step(s->layers[l], s->d_first_table, s->cfg.kvm.table_width, s->d_offsets, nf, T,
                                 buf->prompt_k, buf->prompt_v, buf->prompt_q, buf->prompt_out, stream);
        if (rc == FS_OK && nd)
            rc = fs_decode_step(s->layers[l], s->d_decode_table, s->cfg.kvm.table_width, s->d_lens, nd, buf->decode_k,
                                buf->decode_v, buf->decode_q, 0, buf->decode_out, stream);
        if (rc != FS_OK) return rc;
    }
    return FS_OK;
}

int fs_serve_complete(fs_serve *s)
{
    if (!s || !s->planned) return FS_ERR_INVALID_ARG;
    fs_kvm *k = s->kvm;
    std::vector<int64_t> finished;
    double elapsed = 0;
    for (int64_t id : s->runnable) {
        ServeJob &j = s->jobs.at(id);
        const bool first = j.produced == 0;
        int rc = fs_kvm_advance(k, id, first ? j.prompt : 1);
        if (rc != FS_OK) return rc;
        if (first) s->stats.prompt_tokens += j.prompt;
        j.produced += 1;
        s->stats.job_tokens += 1;
        elapsed = std::max(elapsed, first ? j.init_time : j.decode_time);
        if (j.produced == j.outputs) finished.push_back(id);
    }
    if (s->runnable.empty()) {
        elapsed = s->cfg.q1;
        s->stats.iterations_without_work += 1;
    }
    int rc = fs_sched_complete_iteration(s->sched, s->runnable.data(), (int32_t)s->runnable.size(), elapsed,
                                         finished.data(), (int32_t)finished.size());
    if (rc != FS_OK) return rc;
    for (int64_t id : finished) {
        rc = fs_kvm_release(k, id);
        if (rc != FS_OK) return rc;
        s->jobs.erase(id);
        s->stats.finished_jobs += 1;
    }
    s->iteration += 1;
    s->stats.iterations = s->iteration;
    s->planned = false;
    return FS_OK;
}

int fs_serve_get_stats(const fs_serve *s, fs_serve_stats *stats)
{
    if (!s || !stats) return FS_ERR_INVALID_ARG;
    *stats = s->stats;
    (void)fs_kvm_stats(s->kvm, &stats->blocks_swapped_out, &stats->blocks_swapped_in, nullptr);
    return FS_OK;
}

int fs_serve_run(fs_serve *s, const fs_serve_buffers *buf, void *stream, int64_t max_iterations, fs_serve_stats *stats)
{
    if (!s || !buf || max_iterations < 0) return FS_ERR_INVALID_ARG;
    if (s->max_prompt_tokens == 0 || s->max_prompt_tokens > buf->max_prompt_tokens)
        s->max_prompt_tokens = buf->max_prompt_tokens;
    fs_serve_iteration it;
    using clock = std::chrono::steady_clock;
    auto seconds = [](clock::time_point a, clock::time_point b) { return std::chrono::duration<double>(b - a).count(); };
    for (int64_t i = 0; i < max_iterations && !s->jobs.empty(); ++i) {
        const auto t0 = clock::now();
        int rc = fs_serve_plan(s, stream, &it);
        const auto t1 = clock::now();
        if (rc == FS_OK && (it.n_first || it.n_decode)) rc = fs_serve_launch(s, -1, buf, stream);
        const auto t2 = clock::now();
        if (rc == FS_OK) rc = fs_serve_complete(s);
        const auto t3 = clock::now();
        s->stats.host_seconds_plan += seconds(t0, t1);
        s->stats.host_seconds_launch += seconds(t1, t2);
        s->stats.host_seconds_complete += seconds(t2, t3);
        if (rc != FS_OK) return rc;
    }
    return stats ? fs_serve_get_stats(s, stats) : FS_OK;
}

}  // extern "C"

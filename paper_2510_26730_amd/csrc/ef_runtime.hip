// Expert cache runtime: completion polling of copies and timing events, the estimators of link bandwidth and
// layer time, swap-in of experts through the copy queue, residency queries and the horizon controller
// (paper Sec. 3.2.1, 3.2.2, 3.3, 3.4).  Declarations and argument contracts are in include/expertflow.h.
#include "ef_ctx.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>

namespace efi {

namespace {
thread_local std::string g_err;
void ema(double &est, double sample, double alpha = 0.25) { est = (1.0 - alpha) * est + alpha * sample; }
}  // namespace

const char *thread_error() { return g_err.c_str(); }
void set_thread_error(const std::string &s) { g_err = s; }

int fail(ef_ctx *ctx, int code, const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (ctx) ctx->err = buf;
    g_err = buf;
    return code;
}

// ---- completion polling ---------------------------------------------------------------------

// Has the copy into `slot` completed?  (Caller holds the engine's mutex on device contexts.)
static void poll_copy_locked(ef_ctx *c, int slot) {
    EfSlotDev &s = c->slots[(size_t)slot];
    if (!s.copy_pending || s.copy_queued) return;      // still (partly) in the queue: no ready event yet
    if (c->fake) {
        if (c->fake_now >= s.fake_ready_at) s.copy_pending = false;
        return;
    }
    if (hipEventQuery(s.ready) == hipSuccess) s.copy_pending = false;
    else (void)hipGetLastError();  // hipErrorNotReady is not an error
}

// results the copy worker left: link-rate samples for the C_s estimate, timed bytes, priority-copy latencies
static void collect_engine_results_locked(ef_ctx *c) {
    EfCopyEngine &g = c->eng;
    if (!(c->cfg.flags & EF_FLAG_FIXED_ESTIMATES))
        for (double bw : g.bw_samples) ema(c->bw_Bps, bw);
    g.bw_samples.clear();
    c->st.copy_seconds += g.copy_seconds;
    c->st.bytes_timed += g.bytes_timed;
    c->st.miss_copy_seconds += g.miss_seconds;
    c->st.miss_copy_bytes += g.miss_bytes;
    c->st.miss_copies += g.miss_copies;
    g.copy_seconds = g.miss_seconds = 0.0;
    g.bytes_timed = g.miss_bytes = g.miss_copies = 0;
}

void poll_copy(ef_ctx *c, int slot) {
    if (c->fake) {
        fake_copy_advance(c, c->fake_now);
        poll_copy_locked(c, slot);
        return;
    }
    std::lock_guard<std::mutex> lock(c->eng.mu);
    poll_copy_locked(c, slot);
}

void poll_all_copies(ef_ctx *c) {
    if (c->fake) {
        fake_copy_advance(c, c->fake_now);
        for (int s = 0; s < (int)c->slots.size(); ++s) poll_copy_locked(c, s);
        collect_engine_results_locked(c);
        return;
    }
    std::lock_guard<std::mutex> lock(c->eng.mu);
    for (int s = 0; s < (int)c->slots.size(); ++s) poll_copy_locked(c, s);
    collect_engine_results_locked(c);
}

void poll_pairs(ef_ctx *c, bool wait) {
    if (c->fake) return;
    while (!c->stall_pending.empty()) {
        EfEventPair p = c->stall_pending.front();
        hipError_t q = wait ? hipEventSynchronize(p.b) : hipEventQuery(p.b);
        if (q != hipSuccess) { (void)hipGetLastError(); break; }
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, p.a, p.b) == hipSuccess) c->st.stall_seconds += ms * 1e-3;
        c->stall_pending.pop_front();
    }
    while (!c->layer_pending.empty()) {
        EfEventPair p = c->layer_pending.front();
        hipError_t q = wait ? hipEventSynchronize(p.b) : hipEventQuery(p.b);
        if (q != hipSuccess) { (void)hipGetLastError(); break; }
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, p.a, p.b) == hipSuccess && ms > 0.f) {
            c->st.layer_seconds += ms * 1e-3 * (double)kLayerTimerEvery;   // a sample stands for its neighbours
            if (!(c->cfg.flags & EF_FLAG_FIXED_ESTIMATES)) ema(c->layer_s, ms * 1e-3);
        }
        c->layer_pending.pop_front();
    }
}

void poll_prof(ef_ctx *c, bool wait) {
    while (!c->prof_pending.empty()) {
        ef_ctx::ProfItem it = c->prof_pending.front();
        hipError_t q = wait ? hipEventSynchronize(it.p.b) : hipEventQuery(it.p.b);
        if (q != hipSuccess) { (void)hipGetLastError(); break; }
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, it.p.a, it.p.b) == hipSuccess) {
            c->st.kernel_seconds[it.kind] += ms * 1e-3;
            c->st.kernel_bytes[it.kind] += it.bytes;
            c->st.kernel_flops[it.kind] += it.flops;
            c->st.kernel_launches[it.kind] += 1;
        }
        c->prof_pending.pop_front();
    }
}


KernelTimer::KernelTimer(ef_ctx *ctx, hipStream_t st, int k, double b, double f)
    : c(ctx), s(st), kind(k), bytes(b), flops(f), on(((ctx->profile_mask >> k) & 1u) != 0) {
    if (on && ctx->profile_every > 1) on = (ctx->profile_seen[k]++ % ctx->profile_every) == 0;
    if (!on) return;
    if (c->prof_pending.size() >= c->prof_ring.size()) poll_prof(c, true);
    p = c->prof_ring[c->prof_next];
    c->prof_next = (c->prof_next + 1) % c->prof_ring.size();
    (void)hipEventRecord(p.a, s);
}

KernelTimer::~KernelTimer() {
    if (!on) return;
    (void)hipEventRecord(p.b, s);
    c->prof_pending.push_back({p, kind, bytes, flops});
}

EfEventPair next_pair(std::vector<EfEventPair> &ring, size_t &next, std::deque<EfEventPair> &pending) {
    // never hand out a pair that is still waiting to be read
    if (pending.size() >= ring.size()) {
        EfEventPair p = pending.front();
        (void)hipEventSynchronize(p.b);
        pending.pop_front();
    }
    EfEventPair p = ring[next];
    next = (next + 1) % ring.size();
    return p;
}

uint64_t resident_mask(ef_ctx *c, int layer) {
    uint64_t m = 0;
    for (int e = 0; e < c->cfg.n_experts; ++e)
        if (c->cache->lookup(layer, e) >= 0) m |= (1ull << e);
    return m;
}

// ---- swap-in ---------------------------------------------------------------------------------

namespace {
EfCopyJob *next_job(EfCopyEngine &g);
void issue_chunk(ef_ctx *c, EfCopyJob *job);
// A priority copy does not wait for the worker to wake up: while the link may take more chunks the caller hands
// them over itself (mutex held); the worker carries on from there.
void pump_from_caller(ef_ctx *c) {
    EfCopyEngine &g = c->eng;
    while (!g.failed && (int)g.inflight.size() < g.depth) {
        EfCopyJob *j = next_job(g);
        if (!j) break;
        issue_chunk(c, j);
    }
}
}  // namespace

int swap_in_impl(ef_ctx *c, int layer, int expert, int priority, int due_in, int *slot_out, bool *loaded) {
    int slot = -1, evl = -1, eve = -1;
    if (loaded) *loaded = false;
    ef::SwapResult r = c->cache->swap_in(layer, expert, priority ? 0 : due_in, &slot, &evl, &eve);
    if (r == ef::SwapResult::Busy)
        return fail(c, EF_EBUSY, "no evictable cache slot for layer %d expert %d", layer, expert);
    if (slot_out) *slot_out = slot;
    if (r == ef::SwapResult::Hit) {
        if (!priority) c->st.prefetch_redundant += 1;
        return EF_OK;
    }
    EfSlotDev &s = c->slots[(size_t)slot];
    if (evl >= 0) {
        c->st.evictions += 1;
        if (s.prefetched_unused) c->st.prefetch_wasted += 1;   // fetched ahead, evicted before any layer used it
    }
    const size_t bytes = c->expert_bytes;
    EfCopyJob job;
    job.slot = slot; job.layer = layer; job.expert = expert;
    job.miss = priority != 0;
    job.total = bytes;
    job.war = s.last_read;        // the slot may still be read by an enqueued FFN
    EfCopyEngine &g = c->eng;
    if (c->fake) {
        fake_copy_advance(c, c->fake_now);
        for (auto it = g.pending.begin(); it != g.pending.end();)      // a copy still queued for the slot is void
            it = it->slot == slot ? g.pending.erase(it) : it + 1;
        job.fake_request = c->fake_now;
        g.pending.push_back(job);
        s.copy_queued = true;
        c->st.copy_seconds += (double)bytes / c->bw_Bps;
        c->st.bytes_timed += (int64_t)bytes;
        if (priority) { c->st.miss_copies += 1; c->st.miss_copy_bytes += (int64_t)bytes; }
        fake_copy_advance(c, c->fake_now);
    } else {
        job.t_request = std::chrono::steady_clock::now();
        {
            std::lock_guard<std::mutex> lock(g.mu);
            if (g.failed) return fail(c, EF_EHIP, "copy engine: %s", g.error.c_str());
            for (auto it = g.pending.begin(); it != g.pending.end();)
                it = it->slot == slot ? g.pending.erase(it) : it + 1;
            g.pending.push_back(job);
            s.copy_queued = true;
            if (job.miss) pump_from_caller(c);
        }
        g.cv_work.notify_one();
    }
    s.copy_pending = true;
    s.copy_bytes = bytes;
    s.last_read = nullptr;
    s.prefetched_unused = priority == 0;
    c->st.bytes_copied += (int64_t)bytes;
    if (!priority) c->st.prefetch_issued += 1;
    if (loaded) *loaded = true;
    return EF_OK;
}

// ---- copy engine: device -------------------------------------------------------------------------

namespace {

// the copy the link takes next: the oldest priority copy, else the oldest prefetch
EfCopyJob *next_job(EfCopyEngine &g) {
    for (auto &j : g.pending)
        if (j.miss) return &j;
    return g.pending.empty() ? nullptr : &g.pending.front();
}

void engine_fail(EfCopyEngine &g, const char *what, hipError_t e) {
    if (!g.failed) {
        g.failed = true;
        g.error = std::string(what) + ": " + hipGetErrorString(e);
    }
    g.cv_done.notify_all();
}

// hand one chunk of `job` to the copy stream (mutex held)
void issue_chunk(ef_ctx *c, EfCopyJob *job) {
    EfCopyEngine &g = c->eng;
    EfSlotDev &s = c->slots[(size_t)job->slot];
    hipStream_t cs = c->copy_stream;
    hipError_t e = hipSuccess;
    if (!job->started) {
        if (job->war) e = hipStreamWaitEvent(cs, job->war, 0);
        job->started = true;
    }
    const size_t n = std::min(g.chunk_bytes, job->total - job->done);
    if (e == hipSuccess)
        e = hipMemcpyAsync(c->pool + (size_t)job->slot * c->expert_bytes + job->done,
                           c->layers[(size_t)job->layer].experts + (size_t)job->expert * c->expert_bytes + job->done, n,
                           hipMemcpyHostToDevice, cs);
    job->done += n;
    const bool last = job->done == job->total;
    if (e == hipSuccess && last) e = hipEventRecord(s.ready, cs);
    hipEvent_t ev = g.chunk_ev[g.chunk_next];
    g.chunk_next = (g.chunk_next + 1) % g.chunk_ev.size();
    if (e == hipSuccess) e = hipEventRecord(ev, cs);
    if (e != hipSuccess) {
        engine_fail(g, "expert copy", e);
        return;
    }
    // its transfer starts when the chunk before it ends, if that one was still on the link when this one was issued
    EfCopyEngine::InFlight f{ev, n, !g.inflight.empty(), last && job->miss, job->total, job->t_request};
    g.inflight.push_back(f);
    if (last) {
        s.copy_queued = false;
        for (auto it = g.pending.begin(); it != g.pending.end(); ++it)
            if (&*it == job) { g.pending.erase(it); break; }
        g.cv_done.notify_all();
    }
}

// the front chunk has completed (mutex held)
void retire_chunk(EfCopyEngine &g) {
    EfCopyEngine::InFlight f = g.inflight.front();
    g.inflight.pop_front();
    if (f.back_to_back && g.prev_done) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, g.prev_done, f.ev) == hipSuccess && ms > 0.f) {
            g.copy_seconds += ms * 1e-3;
            g.bytes_timed += (long long)f.bytes;
            g.bw_samples.push_back((double)f.bytes / (ms * 1e-3));
        } else {
            (void)hipGetLastError();
        }
    }
    g.prev_done = f.ev;
    if (f.last_of_miss) {
        g.miss_seconds += std::chrono::duration<double>(std::chrono::steady_clock::now() - f.t_request).count();
        g.miss_bytes += (long long)f.miss_bytes;
        g.miss_copies += 1;
    }
}

void copy_worker(ef_ctx *c) {
    EfCopyEngine &g = c->eng;
    (void)hipSetDevice(g.device);
    std::unique_lock<std::mutex> lk(g.mu);
    while (!g.stop) {
        while (!g.inflight.empty()) {
            hipError_t q = hipEventQuery(g.inflight.front().ev);
            if (q == hipSuccess) { retire_chunk(g); continue; }
            (void)hipGetLastError();
            break;
        }
        if (g.failed) { g.cv_work.wait(lk); continue; }
        EfCopyJob *job = (int)g.inflight.size() < g.depth ? next_job(g) : nullptr;
        if (job) { issue_chunk(c, job); continue; }
        if (!g.inflight.empty()) {            // the link is busy and the queue may not run further ahead: wait for a chunk
            hipEvent_t ev = g.inflight.front().ev;
            lk.unlock();
            hipError_t e = hipEventSynchronize(ev);
            lk.lock();
            if (e != hipSuccess) engine_fail(g, "hipEventSynchronize", e);
            continue;
        }
        g.cv_done.notify_all();               // idle: whoever drains the queue may go on
        g.cv_work.wait(lk);
    }
}

}  // namespace

int copy_engine_start(ef_ctx *c) {
    EfCopyEngine &g = c->eng;
    EF_HIP(c, hipGetDevice(&g.device));
    g.chunk_ev.resize(16);                    // more than any copy_depth plus the chunk that completed last
    for (auto &ev : g.chunk_ev) EF_HIP(c, hipEventCreateWithFlags(&ev, hipEventBlockingSync));
    g.worker = std::thread(copy_worker, c);
    return EF_OK;
}

void copy_engine_stop(ef_ctx *c) {
    EfCopyEngine &g = c->eng;
    if (g.worker.joinable()) {
        {
            std::lock_guard<std::mutex> lock(g.mu);
            g.stop = true;
        }
        g.cv_work.notify_all();
        g.worker.join();
    }
    for (auto ev : g.chunk_ev)
        if (ev) (void)hipEventDestroy(ev);
    g.chunk_ev.clear();
}

int copy_engine_flush(ef_ctx *c, const int *slots, int n) {
    EfCopyEngine &g = c->eng;
    std::unique_lock<std::mutex> lk(g.mu);
    bool any = false;
    for (auto &j : g.pending)
        for (int i = 0; i < n; ++i)
            if (j.slot == slots[i] && !j.miss) {     // a prefetch the layer caught in the queue: a priority copy from now on
                j.miss = true;
                j.t_request = std::chrono::steady_clock::now();
                any = true;
            }
    if (any) {
        pump_from_caller(c);
        g.cv_work.notify_one();
    }
    g.cv_done.wait(lk, [&] {
        if (g.failed) return true;
        for (int i = 0; i < n; ++i)
            if (c->slots[(size_t)slots[i]].copy_queued) return false;
        return true;
    });
    if (g.failed) return fail(c, EF_EHIP, "copy engine: %s", g.error.c_str());
    return EF_OK;
}

int copy_engine_drain(ef_ctx *c) {
    EfCopyEngine &g = c->eng;
    {
        std::unique_lock<std::mutex> lk(g.mu);
        g.cv_done.wait(lk, [&] { return g.failed || (g.pending.empty() && g.inflight.empty()); });
        if (g.failed) return fail(c, EF_EHIP, "copy engine: %s", g.error.c_str());
    }
    EF_HIP(c, hipStreamSynchronize(c->copy_stream));
    return EF_OK;
}

// ---- copy engine: fake clock ---------------------------------------------------------------------
// The same policy as the worker above, as a discrete-event simulation: at most `depth` chunks are committed to
// the link, which transfers them one after the other at the bandwidth estimate; whenever there is room, the
// next chunk of the oldest priority copy, else of the oldest prefetch, is committed.

namespace {

void fake_fill(ef_ctx *c) {
    EfCopyEngine &g = c->eng;
    while ((int)g.fake_committed.size() < g.depth) {
        EfCopyJob *job = next_job(g);
        if (!job) break;
        const size_t n = std::min(g.chunk_bytes, job->total - job->done);
        const double start = std::max(g.fake_link_free, g.fake_t);
        const double finish = start + (double)n / c->bw_Bps;
        g.fake_link_free = finish;
        job->done += n;
        const bool last = job->done == job->total;
        g.fake_committed.push_back({finish, job->slot, last});
        if (last) {
            EfSlotDev &s = c->slots[(size_t)job->slot];
            s.fake_ready_at = finish;
            s.copy_queued = false;
            if (job->miss) c->st.miss_copy_seconds += finish - job->fake_request;
            for (auto it = g.pending.begin(); it != g.pending.end(); ++it)
                if (&*it == job) { g.pending.erase(it); break; }
        }
    }
}

}  // namespace

void fake_copy_advance(ef_ctx *c, double now) {
    EfCopyEngine &g = c->eng;
    for (;;) {
        fake_fill(c);
        if (g.fake_committed.empty() || g.fake_committed.front().finish > now) break;
        g.fake_t = std::max(g.fake_t, g.fake_committed.front().finish);
        g.fake_committed.pop_front();
    }
    g.fake_t = std::max(g.fake_t, now);
    fake_fill(c);
}

double fake_copy_wait(ef_ctx *c, const int *slots, int n) {
    EfCopyEngine &g = c->eng;
    fake_copy_advance(c, c->fake_now);
    for (auto &j : g.pending)
        for (int i = 0; i < n; ++i)
            if (j.slot == slots[i] && !j.miss) {
                j.miss = true;
                j.fake_request = c->fake_now;
                c->st.miss_copies += 1;
                c->st.miss_copy_bytes += (int64_t)j.total;
            }
    auto queued = [&] {
        for (int i = 0; i < n; ++i)
            if (c->slots[(size_t)slots[i]].copy_queued) return true;
        return false;
    };
    fake_fill(c);
    while (queued() && !g.fake_committed.empty()) {   // run the link until every chunk of them is committed
        g.fake_t = std::max(g.fake_t, g.fake_committed.front().finish);
        g.fake_committed.pop_front();
        fake_fill(c);
    }
    double need = c->fake_now;
    for (int i = 0; i < n; ++i)
        if (c->slots[(size_t)slots[i]].copy_pending) need = std::max(need, c->slots[(size_t)slots[i]].fake_ready_at);
    return need;
}

int check_ctx_layer(ef_ctx *c, int layer) {
    if (!c) return fail(nullptr, EF_EINVAL, "null context");
    if (layer < 0 || layer >= c->cfg.n_layers) return fail(c, EF_EINVAL, "layer %d out of range", layer);
    if (!c->layers[(size_t)layer].set) return fail(c, EF_EINVAL, "layer %d is not registered", layer);
    return EF_OK;
}


}  // namespace efi

using namespace efi;

extern "C" int ef_cache_swap_in(ef_ctx *c, int layer, int expert, int priority, int due_in, int *slot_out) {
    int rc = check_ctx_layer(c, layer);
    if (rc) return rc;
    if (expert < 0 || expert >= c->cfg.n_experts) return fail(c, EF_EINVAL, "expert %d out of range", expert);
    if (priority != 0 && priority != 1) return fail(c, EF_EINVAL, "priority must be 0 or 1");
    if (due_in < 0) return fail(c, EF_EINVAL, "due_in must be >= 0");
    poll_all_copies(c);
    return swap_in_impl(c, layer, expert, priority, due_in, slot_out, nullptr);
}

extern "C" int ef_cache_query(ef_ctx *c, int layer, uint8_t *resident_host) {
    if (!c) return fail(nullptr, EF_EINVAL, "null context");
    if (layer < 0 || layer >= c->cfg.n_layers) return fail(c, EF_EINVAL, "layer %d out of range", layer);
    if (!resident_host) return fail(c, EF_EINVAL, "ef_cache_query: null pointer");
    for (int e = 0; e < c->cfg.n_experts; ++e) resident_host[e] = c->cache->lookup(layer, e) >= 0 ? 1 : 0;
    return EF_OK;
}

extern "C" int ef_choose_horizon(ef_ctx *c, int layer, const int32_t *hist_host, int H, int T, int *H_next,
                                 int32_t *prefetch_list, int *n_prefetch) {
    if (!c) return fail(nullptr, EF_EINVAL, "null context");
    if (layer < 0 || layer >= c->cfg.n_layers) return fail(c, EF_EINVAL, "layer %d out of range", layer);
    if (H < 0 || H > EF_MAX_HORIZON) return fail(c, EF_EINVAL, "ef_choose_horizon: H out of range");
    if (!H_next || !n_prefetch || (H > 0 && (!hist_host || !prefetch_list)))
        return fail(c, EF_EINVAL, "ef_choose_horizon: null pointer");
    (void)T;
    poll_all_copies(c);
    poll_pairs(c, false);
    const int E = c->cfg.n_experts;
    const double tau = (double)c->cfg.cum_threshold;
    *n_prefetch = 0;
    H = std::min(H, c->cfg.n_layers - 1 - layer);
    if (H < 0) H = 0;

    // descending-demand order and the cumulative-share cut of each look-ahead layer
    std::vector<std::vector<int>> chosen((size_t)H);
    int n_miss_first = 0;
    for (int j = 0; j < H; ++j) {
        const int32_t *hj = hist_host + (size_t)j * E;
        long long total = 0;
        for (int e = 0; e < E; ++e) {
            if (hj[e] < 0) return fail(c, EF_EINVAL, "ef_choose_horizon: negative histogram entry");
            total += hj[e];
        }
        std::vector<int> order((size_t)E);
        for (int e = 0; e < E; ++e) order[(size_t)e] = e;
        std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return hj[x] > hj[y]; });
        {   // remembered for the overlap statistics: every expert with predicted demand
            uint64_t named = 0;
            for (int e = 0; e < E; ++e)
                if (hj[e] > 0) named |= 1ull << e;
            const size_t at = (size_t)(layer + 1 + j) * EF_MAX_HORIZON + j;
            c->pred_mask[at] = named;
            c->pred_valid[at] = 1;
        }
        long long cum = 0;
        for (int r = 0; r < E && total > 0; ++r) {
            int e = order[(size_t)r];
            if (hj[e] == 0) break;
            cum += hj[e];
            chosen[(size_t)j].push_back(e);
            if ((double)cum / (double)total >= tau) break;
        }
        if (j == 0) {
            for (int e : chosen[0])
                if (c->cache->lookup(layer + 1, e) < 0) ++n_miss_first;
        }
    }
    double raw = (double)n_miss_first * (double)c->expert_bytes / (c->bw_Bps * c->layer_s);
    int S = (int)std::ceil(raw);
    S += c->fb_adjust;
    S = std::max(1, std::min(c->cfg.h_max, S));
    c->horizon = S;
    c->cache->set_S(S);
    *H_next = S;
    int n = 0;
    for (int j = 0; j < std::min(H, S); ++j)
        for (int e : chosen[(size_t)j])
            if (c->cache->lookup(layer + 1 + j, e) < 0) prefetch_list[n++] = ((j + 1) << 16) | e;
    *n_prefetch = n;
    return EF_OK;
}

extern "C" int ef_fake_advance_time(ef_ctx *c, double seconds) {
    if (!c) return fail(nullptr, EF_EINVAL, "null context");
    if (!c->fake) return fail(c, EF_ENOSYS, "ef_fake_advance_time: not a fake-copy context");
    if (!(seconds >= 0.0)) return fail(c, EF_EINVAL, "seconds must be >= 0");
    c->fake_now += seconds;
    c->st.layer_seconds += seconds;
    poll_all_copies(c);
    return EF_OK;
}

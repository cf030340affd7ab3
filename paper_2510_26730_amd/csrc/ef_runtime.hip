// Expert cache runtime: completion polling of copies and timing events, the estimators of link bandwidth and
// layer time, swap-in of experts over the copy streams, residency queries and the horizon controller
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

void poll_copy(ef_ctx *c, int slot) {
    EfSlotDev &s = c->slots[(size_t)slot];
    if (!s.copy_pending) return;
    if (c->fake) {
        if (c->fake_now >= s.fake_ready_at) s.copy_pending = false;
        return;
    }
    if (hipEventQuery(s.ready) == hipSuccess) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, s.copy_start, s.ready) == hipSuccess && ms > 0.f) {
            double sec = ms * 1e-3;
            c->st.copy_seconds += sec;
            c->st.bytes_timed += (int64_t)s.copy_bytes;
            if (!(c->cfg.flags & EF_FLAG_FIXED_ESTIMATES)) ema(c->bw_Bps, (double)s.copy_bytes / sec);
        }
        s.copy_pending = false;
    } else {
        (void)hipGetLastError();  // hipErrorNotReady is not an error
    }
}

void poll_all_copies(ef_ctx *c) {
    for (int s = 0; s < (int)c->slots.size(); ++s) poll_copy(c, s);
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
    if (evl >= 0) c->st.evictions += 1;
    EfSlotDev &s = c->slots[(size_t)slot];
    const size_t bytes = c->expert_bytes;
    const int q = priority ? 1 : 0;
    if (c->fake) {
        double start = std::max(c->fake_now, c->fake_engine_free[q]);
        s.fake_ready_at = start + (double)bytes / c->bw_Bps;
        c->fake_engine_free[q] = s.fake_ready_at;
        c->st.copy_seconds += (double)bytes / c->bw_Bps;
        c->st.bytes_timed += (int64_t)bytes;
    } else {
        hipStream_t cs = c->copy_stream[q];
        hipError_t e = hipSuccess;
        // the slot may still be read by an enqueued FFN, or written by an earlier copy on the other stream
        if (s.last_read) e = hipStreamWaitEvent(cs, s.last_read, 0);
        if (e == hipSuccess && s.copy_pending) e = hipStreamWaitEvent(cs, s.ready, 0);
        if (e == hipSuccess) e = hipEventRecord(s.copy_start, cs);
        if (e == hipSuccess)
            e = hipMemcpyAsync(c->pool + (size_t)slot * bytes,
                               c->layers[(size_t)layer].experts + (size_t)expert * bytes, bytes,
                               hipMemcpyHostToDevice, cs);
        if (e == hipSuccess) e = hipEventRecord(s.ready, cs);
        if (e != hipSuccess) {
            c->cache->drop(slot);
            return fail(c, EF_EHIP, "swap-in of layer %d expert %d failed: %s", layer, expert,
                        hipGetErrorString(e));
        }
    }
    s.copy_pending = true;
    s.copy_bytes = bytes;
    s.last_read = nullptr;
    c->st.bytes_copied += (int64_t)bytes;
    if (!priority) c->st.prefetch_issued += 1;
    if (loaded) *loaded = true;
    return EF_OK;
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

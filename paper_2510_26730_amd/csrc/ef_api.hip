// C-ABI layer: context, expert cache runtime (slots, copy streams, events, estimators, horizon
// controller) and the launch plans of the hot-path kernels.  Declarations and argument contracts
// are in include/expertflow.h.
#include "../../include/expertflow.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <deque>
#include <new>
#include <string>
#include <thread>
#include <vector>

#include "ef_cache.h"
#include "ef_kernels.h"

namespace {

struct LayerReg {
    const uint16_t *gate_w = nullptr;
    const float *gate_b = nullptr;
    const char *experts = nullptr;
    const void *shared_blob = nullptr;
    bool set = false;
};

struct SlotDev {
    hipEvent_t copy_start = nullptr, ready = nullptr;
    hipEvent_t last_read = nullptr;   // borrowed from the read-event ring (may be null)
    bool copy_pending = false;        // a copy was enqueued and not yet seen complete
    double fake_ready_at = 0.0;       // fake-copy contexts: completion time of the copy
    size_t copy_bytes = 0;
};

struct EventPair {
    hipEvent_t a, b;
};

}  // namespace

struct ef_ctx {
    ef_config cfg{};
    size_t expert_bytes = 0;
    bool fake = false;
    std::vector<LayerReg> layers;
    ef::ExpertCache *cache = nullptr;
    char *pool = nullptr;
    std::vector<SlotDev> slots;
    hipStream_t copy_stream[2] = {nullptr, nullptr};  // [0] prefetch, [1] miss
    // scratch
    int32_t *blockcounts = nullptr, *blockbase = nullptr;
    void *xp = nullptr, *act = nullptr;
    float *gate_part = nullptr;      // partial logits of K-split gate launches (small batches)
    bool q4 = false;                 // routed experts are 4-bit blobs
    char *q4_stage = nullptr;        // 16-bit copies of the 4-bit experts that go through the tiled kernels in a phase
    int q4_stage_slots = 0;          // how many such copies fit (as many groups as can reach the tiled size at once)
    size_t q4_stage_bytes = 0;       // bytes of one copy (the larger of routed and shared FFN)
    bool prepacked = false;          // ef_layer_step already enqueued the token packing of the coming ef_moe_ffn
    size_t gate_part_floats = 0;
    float *y = nullptr;
    long long y_floats = 0;          // capacity of y: several K-slice planes when the batch is small
    int max_tiles = 0;
    // buffers of ef_layer_step (library-owned routing state and the host-mapped hand-over area)
    int32_t *st_ids = nullptr, *st_counts = nullptr, *st_offsets = nullptr, *st_perm = nullptr,
            *st_inv = nullptr, *st_pred_ids = nullptr, *st_pred_hist = nullptr;
    float *st_w = nullptr;
    int32_t *meta_host = nullptr, *meta_dev = nullptr;
    int meta_seq = 0;
    // side stream on which a phase's tiled launches run beside its streamed launches, and the fork / join events
    hipStream_t side_stream = nullptr;
    std::vector<hipEvent_t> fork_ring;
    size_t fork_next = 0;
    // event rings
    std::vector<hipEvent_t> read_ring;
    size_t read_next = 0;
    std::vector<EventPair> stall_ring, layer_ring;
    size_t stall_next = 0, layer_next = 0;
    std::deque<EventPair> stall_pending, layer_pending;
    struct ProfItem { EventPair p; int kind; double bytes; double flops; };
    std::vector<EventPair> prof_ring;
    size_t prof_next = 0;
    std::deque<ProfItem> prof_pending;
    unsigned profile_mask = 0;       // bit per kernel kind that is bracketed with events
    int profile_every = 1;           // bracket every n-th launch of a selected kernel kind
    long long profile_seen[EF_K_COUNT] = {};
    bool layer_open = false;
    long long layer_calls = 0;       // layers started (every kLayerTimerEvery-th is timed)
    EventPair layer_cur{nullptr, nullptr};
    // estimators and feedback
    double bw_Bps = 50e9, layer_s = 200e-6;
    int horizon = 1, fb_adjust = 0;
    int stall_counter = 0, overfetch_counter = 0;
    ef_stats st{};
    // fake clock
    double fake_now = 0.0, fake_engine_free[2] = {0.0, 0.0};
    std::string err;
};

namespace {

thread_local std::string g_err;

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

#define EF_HIP(ctx, call)                                                                       \
    do {                                                                                        \
        hipError_t _e = (call);                                                                 \
        if (_e != hipSuccess)                                                                   \
            return fail(ctx, EF_EHIP, "%s failed: %s (%s:%d)", #call, hipGetErrorString(_e),    \
                        __FILE__, __LINE__);                                                    \
    } while (0)

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Debug knob: an integer environment variable overrides a launch heuristic (read on every call,
// so a tuning script can sweep it inside one process).
int tune(const char *name, int dflt) {
    const char *v = getenv(name);
    return (v && *v) ? atoi(v) : dflt;
}

// Routed groups take the tiled kernels from this many token tiles on (the kernels accept 8).  A group of 8 or 9
// tiles is one 256-token panel (plus an almost empty one): its weight panels are read by a single workgroup
// each, cold from HBM with three stages in flight, and such workgroups outlast those of a group with several
// token panels in the same launch; the streaming kernels serve them better (Qwen-shaped T = 640: 8 % of the layer).
int tiled_min_routed() { return std::max(ef::kTiledMinTiles, tune("EF_TUNE_TILED_MIN_TILES", 10)); }

void ema(double &est, double sample, double alpha = 0.25) { est = (1.0 - alpha) * est + alpha * sample; }

// Every kLayerTimerEvery-th layer is bracketed with events for the T_l estimate: an event record between two
// kernels costs the stream a bubble of 2-3 us, and the estimate is a moving average anyway.
constexpr long long kLayerTimerEvery = 4;

// ---- completion polling ---------------------------------------------------------------------

void poll_copy(ef_ctx *c, int slot) {
    SlotDev &s = c->slots[(size_t)slot];
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
        EventPair p = c->stall_pending.front();
        hipError_t q = wait ? hipEventSynchronize(p.b) : hipEventQuery(p.b);
        if (q != hipSuccess) { (void)hipGetLastError(); break; }
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, p.a, p.b) == hipSuccess) c->st.stall_seconds += ms * 1e-3;
        c->stall_pending.pop_front();
    }
    while (!c->layer_pending.empty()) {
        EventPair p = c->layer_pending.front();
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

// Brackets one kernel launch with events on the launch stream when profiling is on.
struct KernelTimer {
    ef_ctx *c;
    hipStream_t s;
    int kind;
    double bytes, flops;
    EventPair p{nullptr, nullptr};
    bool on;
    KernelTimer(ef_ctx *ctx, hipStream_t st, int k, double b, double f = 0.0)
        : c(ctx), s(st), kind(k), bytes(b), flops(f), on(((ctx->profile_mask >> k) & 1u) != 0) {
        if (on && ctx->profile_every > 1) on = (ctx->profile_seen[k]++ % ctx->profile_every) == 0;
        if (!on) return;
        if (c->prof_pending.size() >= c->prof_ring.size()) poll_prof(c, true);
        p = c->prof_ring[c->prof_next];
        c->prof_next = (c->prof_next + 1) % c->prof_ring.size();
        (void)hipEventRecord(p.a, s);
    }
    ~KernelTimer() {
        if (!on) return;
        (void)hipEventRecord(p.b, s);
        c->prof_pending.push_back({p, kind, bytes, flops});
    }
};

EventPair next_pair(std::vector<EventPair> &ring, size_t &next, std::deque<EventPair> &pending) {
    // never hand out a pair that is still waiting to be read
    if (pending.size() >= ring.size()) {
        EventPair p = pending.front();
        (void)hipEventSynchronize(p.b);
        pending.pop_front();
    }
    EventPair p = ring[next];
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
    SlotDev &s = c->slots[(size_t)slot];
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

}  // namespace

// =================================================================================================
// utilities
// =================================================================================================

extern "C" const char *ef_strerror(int code) {
    switch (code) {
        case EF_OK: return "ok";
        case EF_EINVAL: return "invalid argument";
        case EF_ENOMEM: return "out of memory";
        case EF_EHIP: return "HIP runtime error";
        case EF_EBUSY: return "no evictable cache slot";
        case EF_ENOTRESIDENT: return "expert not resident";
        case EF_ENOSYS: return "not available in this context";
        default: return "unknown error";
    }
}

extern "C" size_t ef_expert_bytes(int d, int F) {
    if (d <= 0 || F <= 0 || d % 64 != 0 || F % 32 != 0) return 0;
    return (size_t)3 * (size_t)d * (size_t)F * 2;
}

extern "C" int ef_pack_expert(const uint16_t *W1, const uint16_t *W3, const uint16_t *W2, int d, int F,
                              void *blob) {
    if (!W1 || !W3 || !W2 || !blob) return fail(nullptr, EF_EINVAL, "ef_pack_expert: null pointer");
    if (ef_expert_bytes(d, F) == 0) return fail(nullptr, EF_EINVAL, "ef_pack_expert: d %% 64 or F %% 32 != 0");
    uint16_t *out = static_cast<uint16_t *>(blob);
    const int nkb = d / 16, nrb = F / 32, ncb = d / 32, nkb2 = F / 16;
    auto section_a = [&](int rb0, int rb1) {
        for (int rb = rb0; rb < rb1; ++rb)
            for (int which = 0; which < 2; ++which) {
                const uint16_t *W = which ? W3 : W1;
                uint16_t *dst = out + ((size_t)rb * 2 + which) * nkb * 512;
                for (int kb = 0; kb < nkb; ++kb)
                    for (int lane = 0; lane < 64; ++lane) {
                        int g = lane >> 5, i = lane & 31;
                        memcpy(dst + ((size_t)kb * 64 + lane) * 8,
                               W + (size_t)(rb * 32 + i) * d + kb * 16 + 8 * g, 16);
                    }
            }
    };
    auto section_b = [&](int cb0, int cb1) {
        uint16_t *base = out + (size_t)2 * d * F;
        for (int cb = cb0; cb < cb1; ++cb)
            for (int kb = 0; kb < nkb2; ++kb)
                for (int lane = 0; lane < 64; ++lane) {
                    int g = lane >> 5, i = lane & 31;
                    const uint16_t *src = W2 + (size_t)(cb * 32 + i) * F + kb * 16 + 4 * g;
                    uint16_t *dst = base + (((size_t)cb * nkb2 + kb) * 64 + lane) * 8;
                    memcpy(dst, src, 8);          // t = 0..3 -> columns 4g + t
                    memcpy(dst + 4, src + 8, 8);  // t = 4..7 -> columns 8 + 4g + (t-4)
                }
    };
    unsigned hw = std::thread::hardware_concurrency();
    int nth = (int)std::min<unsigned>(hw ? hw : 1, 16);
    if ((size_t)d * F < (1u << 20)) nth = 1;
    std::vector<std::thread> th;
    for (int t = 0; t < nth; ++t)
        th.emplace_back([&, t] {
            section_a((int)((long long)nrb * t / nth), (int)((long long)nrb * (t + 1) / nth));
            section_b((int)((long long)ncb * t / nth), (int)((long long)ncb * (t + 1) / nth));
        });
    for (auto &t : th) t.join();
    return EF_OK;
}

extern "C" size_t ef_expert_bytes_q4(int d, int F) {
    if (d <= 0 || F <= 0 || d % 128 != 0 || F % 128 != 0) return 0;
    return (size_t)3 * d * F / 2 + (size_t)3 * d * F / 64;
}

extern "C" int ef_pack_expert_q4(const uint8_t *q1, const uint16_t *s1, const uint8_t *q3, const uint16_t *s3,
                                 const uint8_t *q2, const uint16_t *s2, int d, int F, void *blob) {
    if (!q1 || !s1 || !q3 || !s3 || !q2 || !s2 || !blob) return fail(nullptr, EF_EINVAL, "ef_pack_expert_q4: null pointer");
    if (ef_expert_bytes_q4(d, F) == 0) return fail(nullptr, EF_EINVAL, "ef_pack_expert_q4: d %% 128 or F %% 128 != 0");
    unsigned char *out = static_cast<unsigned char *>(blob);
    // dword of one lane for one k-step: code t of the lane's eight values at bits 4*(t/2) + 16*(t%2)
    auto pack8 = [](const uint8_t *v8) {
        uint32_t x = 0;
        for (int t = 0; t < 8; ++t) x |= (uint32_t)(v8[t] & 15u) << (4 * (t / 2) + 16 * (t % 2));
        return x;
    };
    const int nqa = d / 64, nqb = F / 64;
    uint32_t *A = reinterpret_cast<uint32_t *>(out);
    for (int rb = 0; rb < F / 32; ++rb)
        for (int kq = 0; kq < nqa; ++kq)
            for (int which = 0; which < 2; ++which) {
                const uint8_t *Q = which ? q3 : q1;
                uint32_t *dst = A + (((size_t)rb * nqa + kq) * 2 + which) * 256;   // 64 lanes x 4 dwords
                for (int lane = 0; lane < 64; ++lane) {
                    const int g = lane >> 5, i = lane & 31;
                    for (int j = 0; j < 4; ++j)   // natural order: columns kb*16 + 8g + t
                        dst[lane * 4 + j] = pack8(Q + (size_t)(rb * 32 + i) * d + (kq * 4 + j) * 16 + 8 * g);
                }
            }
    uint32_t *B = reinterpret_cast<uint32_t *>(out + (size_t)d * F);
    for (int cb = 0; cb < d / 32; ++cb)
        for (int kq = 0; kq < nqb; ++kq) {
            uint32_t *dst = B + ((size_t)cb * nqb + kq) * 256;
            for (int lane = 0; lane < 64; ++lane) {
                const int g = lane >> 5, i = lane & 31;
                for (int j = 0; j < 4; ++j) {   // paired order: columns kb*16 + 8*(t/4) + 4g + t%4
                    const uint8_t *row = q2 + (size_t)(cb * 32 + i) * F + (kq * 4 + j) * 16;
                    uint8_t v8[8];
                    for (int t = 0; t < 8; ++t) v8[t] = row[8 * (t / 4) + 4 * g + t % 4];
                    dst[lane * 4 + j] = pack8(v8);
                }
            }
        }
    uint16_t *SA = reinterpret_cast<uint16_t *>(out + (size_t)3 * d * F / 2);
    for (int rb = 0; rb < F / 32; ++rb)
        for (int kg = 0; kg < d / 128; ++kg)
            for (int which = 0; which < 2; ++which)
                for (int i = 0; i < 32; ++i)
                    SA[(((size_t)rb * (d / 128) + kg) * 2 + which) * 32 + i] =
                        (which ? s3 : s1)[(size_t)(rb * 32 + i) * (d / 128) + kg];
    uint16_t *SB = reinterpret_cast<uint16_t *>(out + (size_t)3 * d * F / 2 + (size_t)d * F / 32);
    for (int cb = 0; cb < d / 32; ++cb)
        for (int kg = 0; kg < F / 128; ++kg)
            for (int i = 0; i < 32; ++i)
                SB[((size_t)cb * (F / 128) + kg) * 32 + i] = s2[(size_t)(cb * 32 + i) * (F / 128) + kg];
    return EF_OK;
}

// =================================================================================================
// context
// =================================================================================================

extern "C" int ef_destroy(ef_ctx *c) {
    if (!c) return EF_OK;
    if (!c->fake) {
        (void)hipDeviceSynchronize();
        for (auto &s : c->slots) {
            if (s.copy_start) (void)hipEventDestroy(s.copy_start);
            if (s.ready) (void)hipEventDestroy(s.ready);
        }
        for (auto e : c->read_ring) (void)hipEventDestroy(e);
        for (auto e : c->fork_ring) (void)hipEventDestroy(e);
        if (c->side_stream) (void)hipStreamDestroy(c->side_stream);
        for (auto &p : c->stall_ring) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
        for (auto &p : c->layer_ring) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
        for (auto &p : c->prof_ring) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
        for (int q = 0; q < 2; ++q)
            if (c->copy_stream[q]) (void)hipStreamDestroy(c->copy_stream[q]);
        if (c->pool) (void)hipFree(c->pool);
        if (c->blockcounts) (void)hipFree(c->blockcounts);
        if (c->blockbase) (void)hipFree(c->blockbase);
        if (c->xp) (void)hipFree(c->xp);
        if (c->gate_part) (void)hipFree(c->gate_part);
        if (c->act) (void)hipFree(c->act);
        if (c->y) (void)hipFree(c->y);
        if (c->q4_stage) (void)hipFree(c->q4_stage);
        for (void *p : {(void *)c->st_ids, (void *)c->st_counts, (void *)c->st_offsets, (void *)c->st_perm,
                        (void *)c->st_inv, (void *)c->st_pred_ids, (void *)c->st_pred_hist, (void *)c->st_w})
            if (p) (void)hipFree(p);
        if (c->meta_host) (void)hipHostFree(c->meta_host);
    }
    delete c->cache;
    delete c;
    return EF_OK;
}

extern "C" int ef_create(const ef_config *cfg, ef_ctx **out) {
    if (!cfg || !out) return fail(nullptr, EF_EINVAL, "ef_create: null argument");
    *out = nullptr;
    const ef_config &g = *cfg;
    if (g.n_layers <= 0 || g.n_experts <= 0 || g.n_experts > EF_MAX_EXPERTS || g.top_k <= 0 ||
        g.top_k > EF_MAX_TOPK || g.top_k > g.n_experts)
        return fail(nullptr, EF_EINVAL, "ef_create: need 1 <= top_k <= min(n_experts, %d), n_experts <= %d",
                    EF_MAX_TOPK, EF_MAX_EXPERTS);
    if (ef_expert_bytes(g.d_model, g.d_ff) == 0)
        return fail(nullptr, EF_EINVAL, "ef_create: d_model must be a multiple of 64 and d_ff of 32");
    if (g.weight_bits != 0 && g.weight_bits != 16 && g.weight_bits != 4)
        return fail(nullptr, EF_EINVAL, "ef_create: weight_bits must be 0, 16 or 4");
    if (g.weight_bits == 4 && (ef_expert_bytes_q4(g.d_model, g.d_ff) == 0 ||
                               (g.d_ff_shared != 0 && ef_expert_bytes_q4(g.d_model, g.d_ff_shared) == 0)))
        return fail(nullptr, EF_EINVAL, "ef_create: 4-bit experts need d_model, d_ff and d_ff_shared multiples of 128");
    if (g.d_ff_shared < 0 || g.d_ff_shared % 32 != 0)
        return fail(nullptr, EF_EINVAL, "ef_create: d_ff_shared must be a non-negative multiple of 32");
    if (g.slots_total <= 0 || g.slots_per_layer_max < 0 || g.max_tokens <= 0)
        return fail(nullptr, EF_EINVAL, "ef_create: slots_total and max_tokens must be positive");
    if (g.h_max < 1 || g.h_max > EF_MAX_HORIZON)
        return fail(nullptr, EF_EINVAL, "ef_create: h_max must be in 1..%d", EF_MAX_HORIZON);
    if (!(g.cum_threshold > 0.f && g.cum_threshold <= 1.f))
        return fail(nullptr, EF_EINVAL, "ef_create: cum_threshold must be in (0, 1]");
    if ((long long)g.max_tokens * g.top_k > (1ll << 30))
        return fail(nullptr, EF_EINVAL, "ef_create: max_tokens * top_k too large");

    ef_ctx *c = new (std::nothrow) ef_ctx();
    if (!c) return fail(nullptr, EF_ENOMEM, "ef_create: host allocation failed");
    c->cfg = g;
    c->q4 = g.weight_bits == 4;
    c->expert_bytes = c->q4 ? ef_expert_bytes_q4(g.d_model, g.d_ff) : ef_expert_bytes(g.d_model, g.d_ff);
    c->fake = (g.flags & EF_FLAG_FAKE_COPY) != 0;
    c->layers.resize((size_t)g.n_layers);
    c->cache = new ef::ExpertCache(g.slots_total, g.slots_per_layer_max, g.n_layers, g.n_experts);
    c->slots.resize((size_t)g.slots_total);
    if (g.init_bandwidth_gbps > 0.f) c->bw_Bps = (double)g.init_bandwidth_gbps * 1e9;
    if (g.init_layer_us > 0.f) c->layer_s = (double)g.init_layer_us * 1e-6;
    c->horizon = 1;
    c->cache->set_S(1);
    if (c->fake) {
        *out = c;
        return EF_OK;
    }

    const int E = g.n_experts, k = g.top_k, d = g.d_model;
    const long long Tm = g.max_tokens;
    const int ntile_tok = (int)((Tm + ef::kTile - 1) / ef::kTile);
    const int routed_tiles = (int)((Tm * k + ef::kTile - 1) / ef::kTile) + E;
    const int shared_tiles = g.d_ff_shared > 0 ? ntile_tok : 0;
    c->max_tiles = routed_tiles + shared_tiles;
    const size_t xp_bytes = (size_t)c->max_tiles * ef::kTile * d * 2;
    const size_t act_bytes = (size_t)routed_tiles * ef::kTile * g.d_ff * 2 +
                             (size_t)shared_tiles * ef::kTile * g.d_ff_shared * 2;
    // expert outputs: one plane of (T*k [+T]) x d floats, times up to 8 K-slice planes while that stays
    // under 256 MiB (small batches split K of the second FFN half across workgroups)
    const long long y_plane_max = (Tm * k + (g.d_ff_shared > 0 ? Tm : 0)) * d;
    long long planes = std::max(1ll, std::min(8ll, (64ll << 20) / y_plane_max));
    c->y_floats = y_plane_max * planes;
    const size_t y_bytes = (size_t)c->y_floats * 4;

    auto bail = [&](hipError_t e, const char *what) {
        int rc = fail(nullptr, e == hipErrorOutOfMemory ? EF_ENOMEM : EF_EHIP, "ef_create: %s: %s", what,
                      hipGetErrorString(e));
        std::string keep = g_err;
        ef_destroy(c);
        g_err = keep;
        return rc;
    };
    hipError_t e;
    if ((e = hipMalloc(&c->pool, (size_t)g.slots_total * c->expert_bytes)) != hipSuccess) return bail(e, "slot pool");
    if ((e = hipMalloc(&c->blockcounts, (size_t)ntile_tok * E * 4)) != hipSuccess) return bail(e, "blockcounts");
    if ((e = hipMalloc(&c->blockbase, (size_t)ntile_tok * E * 4)) != hipSuccess) return bail(e, "blockbase");
    if ((e = hipMalloc(&c->xp, xp_bytes)) != hipSuccess) return bail(e, "packed-token scratch");
    // partial logits of K-split gate launches: 8 MiB (64 workgroups x 32 rows x 128 columns x 8 splits), or four
    // splits of every token tile of the largest batch
    c->gate_part_floats = std::max((size_t)2 << 20, (size_t)ntile_tok * 4 * ef::kTile * 128);
    if ((e = hipMalloc(&c->gate_part, c->gate_part_floats * 4)) != hipSuccess) return bail(e, "gate partials");
    if ((e = hipMalloc(&c->act, act_bytes)) != hipSuccess) return bail(e, "activation scratch");
    if ((e = hipMalloc(&c->y, y_bytes)) != hipSuccess) return bail(e, "expert-output scratch");
    if (c->q4) {
        // 4-bit groups with enough tokens for the tiled kernels are expanded to 16 bits first.  A group needs more
        // than (kTiledMinTiles - 1) tiles of tokens, so at most `can` routed experts of one call qualify, plus the
        // shared FFN (every token).
        const long long need = (ef::kTiledMinTiles - 1) * ef::kTile + 1;
        if (ef::ffn_tiled_ok(d, g.d_ff, ef::kTiledMinTiles)) c->q4_stage_slots = (int)std::min<long long>(E, Tm * k / need);
        if (g.d_ff_shared > 0 && ef::ffn_tiled_ok(d, g.d_ff_shared, ef::kTiledMinTiles) && Tm >= need)
            c->q4_stage_slots += 1;
        c->q4_stage_bytes = ef_expert_bytes(d, std::max(g.d_ff, g.d_ff_shared));
        if (c->q4_stage_slots > 0 &&
            (e = hipMalloc(&c->q4_stage, (size_t)c->q4_stage_slots * c->q4_stage_bytes)) != hipSuccess)
            return bail(e, "16-bit staging of 4-bit experts");
    }

    {
        const size_t n = (size_t)Tm * k;
        if ((e = hipMalloc(&c->st_ids, n * 4)) != hipSuccess) return bail(e, "step buffers");
        if ((e = hipMalloc(&c->st_w, n * 4)) != hipSuccess) return bail(e, "step buffers");
        if ((e = hipMalloc(&c->st_perm, n * 4)) != hipSuccess) return bail(e, "step buffers");
        if ((e = hipMalloc(&c->st_inv, n * 4)) != hipSuccess) return bail(e, "step buffers");
        if ((e = hipMalloc(&c->st_pred_ids, n * 4 * EF_MAX_HORIZON)) != hipSuccess) return bail(e, "step buffers");
        if ((e = hipMalloc(&c->st_counts, (size_t)E * 4)) != hipSuccess) return bail(e, "step buffers");
        if ((e = hipMalloc(&c->st_offsets, (size_t)(E + 1) * 4)) != hipSuccess) return bail(e, "step buffers");
        if ((e = hipMalloc(&c->st_pred_hist, (size_t)EF_MAX_HORIZON * E * 4)) != hipSuccess)
            return bail(e, "step buffers");
        if ((e = hipMemset(c->st_pred_hist, 0, (size_t)EF_MAX_HORIZON * E * 4)) != hipSuccess)
            return bail(e, "step buffers");
        if ((e = hipHostMalloc(reinterpret_cast<void **>(&c->meta_host), (size_t)ef::kMetaInts * 4,
                               hipHostMallocMapped)) != hipSuccess)
            return bail(e, "host-mapped hand-over buffer");
        memset(c->meta_host, 0, (size_t)ef::kMetaInts * 4);
        if ((e = hipHostGetDevicePointer(reinterpret_cast<void **>(&c->meta_dev), c->meta_host, 0)) != hipSuccess)
            return bail(e, "host-mapped hand-over buffer");
    }
    for (int q = 0; q < 2; ++q)
        if ((e = hipStreamCreateWithFlags(&c->copy_stream[q], hipStreamNonBlocking)) != hipSuccess)
            return bail(e, "copy stream");
    for (auto &s : c->slots) {
        if ((e = hipEventCreate(&s.copy_start)) != hipSuccess) return bail(e, "event");
        if ((e = hipEventCreate(&s.ready)) != hipSuccess) return bail(e, "event");
    }
    c->read_ring.resize(128);
    for (auto &ev : c->read_ring)
        if ((e = hipEventCreateWithFlags(&ev, hipEventDisableTiming)) != hipSuccess) return bail(e, "event");
    if ((e = hipStreamCreateWithFlags(&c->side_stream, hipStreamNonBlocking)) != hipSuccess) return bail(e, "side stream");
    c->fork_ring.resize(64);
    for (auto &ev : c->fork_ring)
        if ((e = hipEventCreateWithFlags(&ev, hipEventDisableTiming)) != hipSuccess) return bail(e, "event");
    c->stall_ring.resize(128);
    c->layer_ring.resize(128);
    if (g.flags & EF_FLAG_PROFILE) c->profile_mask = 0x3FFu;
    else if (g.flags & EF_FLAG_PROFILE_FFN_UP) c->profile_mask = 1u << EF_K_FFN_UP;
    if (c->profile_mask) c->prof_ring.resize(1024);
    for (auto *ring : {&c->stall_ring, &c->layer_ring, &c->prof_ring})
        for (auto &p : *ring) {
            if ((e = hipEventCreate(&p.a)) != hipSuccess) return bail(e, "event");
            if ((e = hipEventCreate(&p.b)) != hipSuccess) return bail(e, "event");
        }
    *out = c;
    return EF_OK;
}

extern "C" const char *ef_last_error(ef_ctx *c) { return c ? c->err.c_str() : g_err.c_str(); }

extern "C" int ef_register_layer(ef_ctx *c, int layer, const void *gate_w, const float *gate_b,
                                 const void *experts, const void *shared_blob) {
    if (!c) return fail(nullptr, EF_EINVAL, "null context");
    if (layer < 0 || layer >= c->cfg.n_layers) return fail(c, EF_EINVAL, "layer %d out of range", layer);
    if (!experts) return fail(c, EF_EINVAL, "ef_register_layer: experts is null");
    if (!c->fake) {
        if (!gate_w) return fail(c, EF_EINVAL, "ef_register_layer: gate_w is null");
        if (!aligned16(gate_w) || !aligned16(experts) || !aligned16(shared_blob))
            return fail(c, EF_EINVAL, "ef_register_layer: pointers must be 16-byte aligned");
        if (c->cfg.d_ff_shared > 0 && !shared_blob)
            return fail(c, EF_EINVAL, "ef_register_layer: shared_blob required when d_ff_shared > 0");
    }
    LayerReg &L = c->layers[(size_t)layer];
    L.gate_w = static_cast<const uint16_t *>(gate_w);
    L.gate_b = gate_b;
    L.experts = static_cast<const char *>(experts);
    L.shared_blob = shared_blob;
    L.set = true;
    return EF_OK;
}

// =================================================================================================
// hot path
// =================================================================================================

namespace {

const ef::GroupExport kNoExport{nullptr, nullptr, 0, 0, 0};

// One pass over `hidden`: optionally the current layer's own gate (routing outputs and grouping)
// and the gates of the next He layers (prediction outputs).  Wide launches are split over the gates.
int run_gates(ef_ctx *c, int layer, const void *hidden, int T, float beta, bool do_route, int He, int H_stride,
              const float *delta, const int32_t *tok2req, int32_t *topk_ids, float *topk_w, int32_t *counts,
              int32_t *offsets, int32_t *perm, int32_t *inv_perm, int32_t *pred_ids, int32_t *pred_hist,
              const ef::GroupExport &ex, hipStream_t s) {
    const int E = c->cfg.n_experts, k = c->cfg.top_k, d = c->cfg.d_model;
    const int ntiles = (T + ef::kTile - 1) / ef::kTile;
    // the library's own histogram buffer is left zeroed by the hand-over step of the previous layer
    if (He > 0 && !ex.host_meta) EF_HIP(c, ef::launch_fill_i32(pred_hist, He * E, 0, s));
    const int per_launch = ef::kMaxGates;
    const int total_gates = (do_route ? 1 : 0) + He;
    bool grouped = false;
    for (int g0 = 0; g0 < total_gates; g0 += per_launch) {
        ef::GateArgs a{};
        a.h = static_cast<const uint16_t *>(hidden);
        a.T = T; a.d = d; a.E = E; a.k = k;
        a.G = std::min(per_launch, total_gates - g0);
        a.beta = beta;
        a.tok2req = tok2req;
        a.delta = nullptr;
        a.delta_req_stride = H_stride * E;
        a.delta_gate_begin = 0;
        bool first_pred = true;
        for (int gi = 0; gi < a.G; ++gi) {
            const int gg = g0 + gi;                       // index over [route?] + predictions
            const bool is_route = do_route && gg == 0;
            const int j = gg - (do_route ? 1 : 0);        // prediction index (0-based) when !is_route
            const int ly = is_route ? layer : layer + 1 + j;
            const LayerReg &L = c->layers[(size_t)ly];
            a.Wg[gi] = L.gate_w;
            a.bias[gi] = L.gate_b;
            a.resident[gi] = resident_mask(c, ly);
            if (is_route) {
                a.ids[gi] = topk_ids;
                a.hist[gi] = nullptr;
                a.w = topk_w;
                a.blockcounts = c->blockcounts;
                a.renorm = c->cfg.renorm_topk;
                a.routed_scale = c->cfg.routed_scale;
            } else {
                a.ids[gi] = pred_ids + (size_t)j * T * k;
                a.hist[gi] = pred_hist + (size_t)j * E;
                if (first_pred) {
                    a.delta_gate_begin = gi;
                    a.delta = delta ? delta + (size_t)j * E : nullptr;
                    first_pred = false;
                }
            }
        }
        a.gpw = ef::gate_pick_gpw(T, a.G, E);
        a.ksplit = ef::gate_pick_ksplit(T, d, a.G, E, a.gpw, c->gate_part_floats);
        {
            const int forced = tune("EF_TUNE_GATE_KSPLIT", 0);
            if (forced >= 1 && forced <= 16 &&
                (size_t)ntiles * ((a.G + a.gpw - 1) / a.gpw) * forced * ef::kTile * 128 <= c->gate_part_floats)
                a.ksplit = forced;
        }
        a.part = c->gate_part;
        a.tsplit = 1;
        {   // the two-kernel form also pays off without a K split when the per-token part dominates
            const int ts = ef::gate_pick_tsplit(T, a.G, E, a.gpw);
            const size_t need = (size_t)ntiles * ((a.G + a.gpw - 1) / a.gpw) * a.ksplit * ef::kTile * 128;
            if (ts > 1 && need <= c->gate_part_floats && tune("EF_TUNE_GATE_TSPLIT", 1) != 0) a.tsplit = ts;
        }
        a.two_step = (a.ksplit > 1 || a.tsplit > 1) ? 1 : 0;
        const bool has_route = do_route && g0 == 0;
        // decode-sized batches with a K-split gate and few experts: its second step and the grouping run as
        // one workgroup (with more than 16 experts a token takes a whole wave round of the epilogue, and the
        // many workgroups of the separate second step are faster: 27 against 36 us at 64 experts)
        const bool fused = has_route && total_gates <= per_launch && ntiles <= ef::kFusedMaxTiles && a.ksplit > 1 &&
                           E <= 16 &&
                           ef::gate_fused_lds_bytes(T, a.G, E, a.gpw) <= ef::kFusedMaxLds &&
                           tune("EF_TUNE_FUSED_FINISH", 1) != 0;
        if (fused) a.tsplit = 1;
        {
            KernelTimer kt(c, s, has_route ? EF_K_ROUTE : EF_K_PREDICT,
                           (double)T * d * 2 + (double)a.G * E * d * 2 + (double)a.G * T * k * 4 +
                               (has_route ? (double)T * k * 4 + (double)ntiles * E * 4 : 0.0) +
                               (double)(a.G - (has_route ? 1 : 0)) * E * 4 +
                               (fused ? (double)(2 * E + 1) * 4 + (double)T * k * 12 : 0.0));
            if (fused) EF_HIP(c, ef::launch_gate_fused(a, counts, offsets, perm, inv_perm, ex, s));
            else EF_HIP(c, ef::launch_gate(a, s));
        }
        if (fused) grouped = true;
    }
    if (do_route && !grouped) {
        KernelTimer kt(c, s, EF_K_GROUP, (double)ntiles * E * 8 + (double)(2 * E + 1) * 4 + (double)T * k * 12);
        EF_HIP(c, ef::launch_group(c->blockcounts, topk_ids, T, k, E, c->blockbase, counts, offsets, perm,
                                   inv_perm, ex, s));
    }
    return EF_OK;
}

int check_predict_args(ef_ctx *c, int layer, int T, int H, int *He_out, const char *who) {
    if (c->fake) return fail(c, EF_ENOSYS, "%s: fake-copy context has no device", who);
    if (H < 0 || H > EF_MAX_HORIZON) return fail(c, EF_EINVAL, "%s: H must be in 0..%d", who, EF_MAX_HORIZON);
    if (T < 0 || T > c->cfg.max_tokens) return fail(c, EF_EINVAL, "%s: T=%d outside 0..max_tokens", who, T);
    int He = std::max(0, std::min(H, c->cfg.n_layers - 1 - layer));
    for (int j = 1; j <= He; ++j)
        if (!c->layers[(size_t)(layer + j)].set)
            return fail(c, EF_EINVAL, "%s: layer %d is not registered", who, layer + j);
    *He_out = He;
    return EF_OK;
}

int open_layer_timer(ef_ctx *c, hipStream_t s) {
    poll_pairs(c, false);
    if ((c->layer_calls++ % kLayerTimerEvery) != 0) return EF_OK;
    c->layer_cur = next_pair(c->layer_ring, c->layer_next, c->layer_pending);
    EF_HIP(c, hipEventRecord(c->layer_cur.a, s));
    c->layer_open = true;
    return EF_OK;
}

}  // namespace

extern "C" int ef_predict(ef_ctx *c, int layer, const void *hidden, int T, int H, const float *delta,
                          const int32_t *tok2req, float beta, int32_t *topk_ids, int32_t *hist, int *H_eff,
                          void *stream) {
    int rc = check_ctx_layer(c, layer);
    if (rc) return rc;
    int He = 0;
    if ((rc = check_predict_args(c, layer, T, H, &He, "ef_predict"))) return rc;
    if (H_eff) *H_eff = He;
    if (He == 0) return EF_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!hist) return fail(c, EF_EINVAL, "ef_predict: null pointer");
    if (T == 0) {
        EF_HIP(c, ef::launch_fill_i32(hist, He * c->cfg.n_experts, 0, s));
        return EF_OK;
    }
    if (!hidden || !topk_ids) return fail(c, EF_EINVAL, "ef_predict: null pointer");
    if (!aligned16(hidden)) return fail(c, EF_EINVAL, "ef_predict: hidden must be 16-byte aligned");
    return run_gates(c, layer, hidden, T, beta, false, He, H, delta, tok2req, nullptr, nullptr, nullptr, nullptr,
                     nullptr, nullptr, topk_ids, hist, kNoExport, s);
}

extern "C" int ef_token_dist(ef_ctx *c, const void *hidden, int T, float *tok_dist, double *dist, void *stream) {
    if (!c) return EF_EINVAL;
    if (c->fake) return fail(c, EF_ENOSYS, "ef_token_dist: fake-copy context has no device");
    if (T < 1 || T > c->cfg.max_tokens) return fail(c, EF_EINVAL, "ef_token_dist: T=%d outside 1..max_tokens", T);
    if (!hidden || !dist) return fail(c, EF_EINVAL, "ef_token_dist: null pointer");
    if (!aligned16(hidden)) return fail(c, EF_EINVAL, "ef_token_dist: hidden must be 16-byte aligned");
    const int d = c->cfg.d_model;
    const int ntiles = (T + ef::kTile - 1) / ef::kTile;
    if (ntiles > c->max_tiles || (long long)ef::dist_scratch_floats(T) > c->y_floats)
        return fail(c, EF_EINVAL, "ef_token_dist: T=%d needs more scratch than this context has", T);
    hipStream_t s = static_cast<hipStream_t>(stream);
    ef::PackTable pt{};
    pt.n_groups = 1;
    pt.tile_start[0] = 0;
    pt.tile_start[1] = ntiles;
    pt.row_offset[0] = -1;   // identity: packed row = token
    pt.count[0] = T;
    // flops of the strict upper triangle; bytes: tokens read once, packed copy written and read once
    const double flops = (double)T * (T - 1) * d;
    const double bytes = 6.0 * T * d + 8.0 * T;
    KernelTimer kt(c, s, EF_K_DIST, bytes, flops);
    EF_HIP(c, ef::launch_pack_x(pt, ntiles, static_cast<const uint16_t *>(hidden), d, 1, nullptr, c->xp, false, s));
    EF_HIP(c, ef::launch_token_dist(static_cast<const uint16_t *>(hidden), T, d, c->xp, c->y, tok_dist, dist, s));
    return EF_OK;
}

extern "C" int ef_route(ef_ctx *c, int layer, const void *hidden, int T, float beta, int32_t *topk_ids,
                        float *topk_w, int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv_perm,
                        void *stream) {
    int rc = check_ctx_layer(c, layer);
    if (rc) return rc;
    if (c->fake) return fail(c, EF_ENOSYS, "ef_route: fake-copy context has no device");
    if (T < 0 || T > c->cfg.max_tokens) return fail(c, EF_EINVAL, "ef_route: T=%d outside 0..max_tokens", T);
    if (!counts || !offsets) return fail(c, EF_EINVAL, "ef_route: null pointer");
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int E = c->cfg.n_experts;
    if (T == 0) {
        EF_HIP(c, ef::launch_fill_i32(counts, E, 0, s));
        EF_HIP(c, ef::launch_fill_i32(offsets, E + 1, 0, s));
        return EF_OK;
    }
    if (!hidden || !topk_ids || !topk_w || !perm || !inv_perm) return fail(c, EF_EINVAL, "ef_route: null pointer");
    if (!aligned16(hidden)) return fail(c, EF_EINVAL, "ef_route: hidden must be 16-byte aligned");
    if ((rc = open_layer_timer(c, s))) return rc;
    return run_gates(c, layer, hidden, T, beta, true, 0, 0, nullptr, nullptr, topk_ids, topk_w, counts, offsets,
                     perm, inv_perm, nullptr, nullptr, kNoExport, s);
}

extern "C" int ef_route_predict(ef_ctx *c, int layer, const void *hidden, int T, float beta, int H,
                                const float *delta, const int32_t *tok2req, int32_t *topk_ids, float *topk_w,
                                int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv_perm,
                                int32_t *pred_ids, int32_t *pred_hist, int *H_eff, void *stream) {
    int rc = check_ctx_layer(c, layer);
    if (rc) return rc;
    int He = 0;
    if ((rc = check_predict_args(c, layer, T, H, &He, "ef_route_predict"))) return rc;
    if (H_eff) *H_eff = He;
    if (!counts || !offsets || (He > 0 && !pred_hist)) return fail(c, EF_EINVAL, "ef_route_predict: null pointer");
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int E = c->cfg.n_experts;
    if (T == 0) {
        EF_HIP(c, ef::launch_fill_i32(counts, E, 0, s));
        EF_HIP(c, ef::launch_fill_i32(offsets, E + 1, 0, s));
        if (He > 0) EF_HIP(c, ef::launch_fill_i32(pred_hist, He * E, 0, s));
        return EF_OK;
    }
    if (!hidden || !topk_ids || !topk_w || !perm || !inv_perm || (He > 0 && !pred_ids))
        return fail(c, EF_EINVAL, "ef_route_predict: null pointer");
    if (!aligned16(hidden)) return fail(c, EF_EINVAL, "ef_route_predict: hidden must be 16-byte aligned");
    if ((rc = open_layer_timer(c, s))) return rc;
    return run_gates(c, layer, hidden, T, beta, true, He, H, delta, tok2req, topk_ids, topk_w, counts, offsets,
                     perm, inv_perm, pred_ids, pred_hist, kNoExport, s);
}

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

namespace {

struct PhaseGroup {
    int expert;  // -1: dense shared FFN
    int slot;
};

// Build the launch tables of one phase and enqueue both FFN halves.
int launch_phase(ef_ctx *c, int layer, const std::vector<PhaseGroup> &groups, const int32_t *counts_host,
                 const std::vector<int> &offs_host, const std::vector<int> &tile_start,
                 const std::vector<long long> &act_off, int shared_tile_start, long long shared_act_off, int T,
                 int ksg_stream, int ksg_tiled, ef::PlaneTable &planes, long long y_plane, bool use_tiled, hipStream_t s) {
    if (groups.empty()) return EF_OK;
    const int d = c->cfg.d_model, k = c->cfg.top_k;
    // groups with many tokens go to the tiled (matrix-core bound) kernels, the others to the
    // weight-streaming kernels; at most two launches per FFN half
    ef::GroupTable gu{}, big{};
    ef::DequantTable dq{};
    int n = 0, nb = 0, max_tiles = 1;
    const bool allow_tiled = use_tiled;
    // Workgroups start in index order; groups with the most work go first so that the launch's last round holds
    // the short ones (the groups are independent: the order changes no result)
    std::vector<PhaseGroup> ordered(groups);
    if (tune("EF_TUNE_SORT_GROUPS", 1) != 0) {
        auto work = [&](const PhaseGroup &pg) {
            const long long cnt = pg.expert < 0 ? T : counts_host[pg.expert];
            const long long F = pg.expert < 0 ? c->cfg.d_ff_shared : c->cfg.d_ff;
            return ((cnt + ef::kTile - 1) / ef::kTile) * F;
        };
        std::stable_sort(ordered.begin(), ordered.end(),
                         [&](const PhaseGroup &a, const PhaseGroup &b) { return work(a) > work(b); });
    }
    for (const PhaseGroup &pg : ordered) {
        int cnt, ts, F, ro;
        long long ao;
        const void *blob;
        if (pg.expert < 0) {
            cnt = T; ts = shared_tile_start; F = c->cfg.d_ff_shared; ro = T * k; ao = shared_act_off;
            blob = c->layers[(size_t)layer].shared_blob;
        } else {
            cnt = counts_host[pg.expert]; ts = tile_start[(size_t)pg.expert]; F = c->cfg.d_ff;
            ro = offs_host[(size_t)pg.expert]; ao = act_off[(size_t)pg.expert];
            blob = c->pool + (size_t)pg.slot * c->expert_bytes;
        }
        const int nt = (cnt + ef::kTile - 1) / ef::kTile;
        const bool tiled = allow_tiled && ef::ffn_tiled_ok(d, F, nt) && (pg.expert < 0 || nt >= tiled_min_routed()) &&
                           (!c->q4 || nb < c->q4_stage_slots);
        ef::GroupTable &g = tiled ? big : gu;
        int &i = tiled ? nb : n;
        if (tiled && c->q4) {   // the tiled kernels read a 16-bit copy written just before them on the same stream
            void *copy = c->q4_stage + (size_t)nb * c->q4_stage_bytes;
            dq.F[nb] = F; dq.src[nb] = blob; dq.dst[nb] = copy;
            blob = copy;
        }
        (pg.expert < 0 ? planes.shared : planes.routed[pg.expert]) = (uint8_t)(tiled ? ksg_tiled : ksg_stream);
        g.tile_start[i] = ts; g.n_tiles[i] = nt; g.row_offset[i] = ro;
        g.count[i] = cnt; g.F[i] = F; g.act_off[i] = ao; g.blob[i] = blob;
        if (!tiled) max_tiles = std::max(max_tiles, nt);
        ++i;
    }
    gu.n_groups = n;
    big.n_groups = nb;
    // weights: 2 bytes each, or half a byte plus one bf16 scale per 128
    const double wb = c->q4 ? 0.5 + 2.0 / 128.0 : 2.0;
    auto alg_bytes = [&](const ef::GroupTable &g, int cnt_groups, double &b_up, double &b_dn) {
        for (int i = 0; i < cnt_groups; ++i) {
            b_up += 2.0 * wb * d * g.F[i] + 2.0 * g.count[i] * d + 2.0 * g.count[i] * g.F[i];
            b_dn += wb * d * g.F[i] + 2.0 * g.count[i] * g.F[i] + 4.0 * g.count[i] * d;
        }
    };
    hipEvent_t join = nullptr;   // set when this phase's tiled launches went to the side stream
    if (nb > 0) {
        ef::GroupTable bdn = big;
        int wg_up = 0, wg_dn = 0;
        // Workgroups go to the XCDs round-robin by index and hold one of an XCD's 32 compute units for their whole
        // K loop.  A group's panel blocks (block b -> XCD rot + b) are dealt from the start XCD that leaves the
        // fullest XCD of the first half's launch least full, so groups of a few panels do not pile up on XCD 0.
        int load[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        const int rot_on = tune("EF_TUNE_TILED_ROT", 1);
        for (int i = 0; i < nb; ++i) {
            big.wg_start[i] = wg_up;
            bdn.wg_start[i] = wg_dn;
            const int pu = big.F[i] / 128, pbu = ef::tiled_panel_block(pu), nblk = (pu + pbu - 1) / pbu;
            const int mp = (big.n_tiles[i] + 7) / 8;
            int best = 0, best_max = 1 << 30;
            for (int rot = 0; rot < (rot_on ? 8 : 1); ++rot) {
                int trial[8], mx = 0;
                for (int x = 0; x < 8; ++x) trial[x] = load[x];
                for (int b = 0; b < nblk; ++b) trial[(rot + b) & 7] += std::min(pbu, pu - b * pbu) * mp;
                for (int x = 0; x < 8; ++x) mx = std::max(mx, trial[x]);
                if (mx < best_max) { best_max = mx; best = rot; }
            }
            for (int b = 0; b < nblk; ++b) load[(best + b) & 7] += std::min(pbu, pu - b * pbu) * mp;
            big.xcd_rot[i] = best;
            bdn.xcd_rot[i] = 0;   // the second half's panels cover every XCD (or K slices interleave them)
            wg_up += ef::ffn_gate_up_tiled_wgs(big.F[i], big.n_tiles[i]);
            wg_dn += ef::ffn_down_tiled_wgs(d, big.n_tiles[i]) * ksg_tiled;
        }
        big.wg_start[nb] = wg_up;
        bdn.wg_start[nb] = wg_dn;
        double b_up = 0.0, b_dn = 0.0, f_up = 0.0, f_dn = 0.0;
        alg_bytes(big, nb, b_up, b_dn);
        for (int i = 0; i < nb; ++i) {
            f_up += 4.0 * big.count[i] * d * big.F[i];   // two d x F products, 2 flops per multiply-add
            f_dn += 2.0 * big.count[i] * d * big.F[i];
        }
        // A phase with both kinds of groups runs its tiled launches on the side stream, beside the streamed ones:
        // the two touch different groups (tiles of the packed tokens, activations, rows of Y), small tiled launches
        // leave half of the compute units idle, and the streamed kernels are bound by HBM, not by compute units.
        // Fork: the side stream waits for everything enqueued so far (the token packing, the previous layer's
        // un-permute).  Join: the caller's stream waits for the side stream before anything after this phase.
        hipStream_t ts = s;
        if (n > 0 && c->side_stream && tune("EF_TUNE_OVERLAP", 1) != 0) {
            hipEvent_t fork = c->fork_ring[c->fork_next];
            c->fork_next = (c->fork_next + 1) % c->fork_ring.size();
            EF_HIP(c, hipEventRecord(fork, s));
            EF_HIP(c, hipStreamWaitEvent(c->side_stream, fork, 0));
            ts = c->side_stream;
        }
        {
            KernelTimer kt(c, ts, EF_K_FFN_UP_TILED, b_up, f_up);   // 4-bit: the expansion is timed with the first half
            if (c->q4) {
                dq.n = nb;
                EF_HIP(c, ef::launch_dequant_q4(dq, d, ts));
            }
            EF_HIP(c, ef::launch_ffn_gate_up_tiled(big, wg_up, c->xp, c->act, d, c->q4, ts));
        }
        {
            KernelTimer kt(c, ts, EF_K_FFN_DOWN_TILED, b_dn, f_dn);
            EF_HIP(c, ef::launch_ffn_down_tiled(bdn, wg_dn, ksg_tiled, c->act, c->y, y_plane, d, c->q4, ts));
        }
        if (ts != s) {
            join = c->fork_ring[c->fork_next];
            c->fork_next = (c->fork_next + 1) % c->fork_ring.size();
            EF_HIP(c, hipEventRecord(join, ts));
        }
    }
    if (n == 0) return EF_OK;
    ef::GroupTable dn = gu;
    // token tiles per pass over a group's weights: groups of three or more tiles (too few for the tiled
    // kernels) take passes of four, which halves the re-reads of their weights (bf16 kernels only)
    const int tpp = (max_tiles >= 3 && !c->q4 && tune("EF_TUNE_TPP4", 1) != 0) ? 4 : max_tiles >= 2 ? 2 : 1;
    // K slices inside a workgroup of the first half: split while the launch has too few waves to
    // keep enough weight bytes in flight, as long as a slice keeps >= 16 fragments
    long long units = 0;
    for (int i = 0; i < n; ++i) units += (long long)(gu.F[i] / 32) * ((gu.n_tiles[i] + tpp - 1) / tpp);
    int ks = 1;
    const int want_waves = tune("EF_TUNE_UP_WAVES", 768), nkb = d / 16;
    while (ks < 4 && units * ks < want_waves && nkb / (ks * 2) >= 16) ks *= 2;
    ks = tune("EF_TUNE_UP_KS", ks);
    // passes of four tiles: the kernels whose four waves share the token / activation fragments through LDS
    // (per-wave copies of them would be twice the weights' bytes from L2)
    bool shared = tpp == 4 && !c->q4 && tune("EF_TUNE_SHARED", 1) != 0;
    for (int i = 0; i < n && shared; ++i) shared = gu.F[i] % 128 == 0;
    int wg_gu = 0, wg_dn = 0;
    for (int i = 0; i < n; ++i) {
        gu.wg_start[i] = wg_gu;
        dn.wg_start[i] = wg_dn;
        if (shared) {
            wg_gu += ef::ffn_gate_up_shared_wgs(gu.F[i], gu.n_tiles[i], tpp);
            wg_dn += ef::ffn_down_shared_wgs(d, gu.n_tiles[i], tpp, ksg_stream);
            continue;
        }
        wg_gu += c->q4 ? ef::ffn_gate_up_q4_wgs(gu.F[i], gu.n_tiles[i], tpp)
                       : ef::ffn_gate_up_wgs(gu.F[i], gu.n_tiles[i], tpp, ks);
        wg_dn += c->q4 ? ef::ffn_down_q4_wgs(d, gu.n_tiles[i], tpp, ksg_stream)
                       : ef::ffn_down_wgs(d, gu.n_tiles[i], tpp, ksg_stream);
    }
    gu.wg_start[n] = wg_gu;
    dn.wg_start[n] = wg_dn;
    double b_up = 0.0, b_dn = 0.0;
    alg_bytes(gu, n, b_up, b_dn);
    // workgroups per CU of the LDS-shared kernels: two (with a shorter register ring) measured 0-1.5 % faster
    // than one on the mixed DeepSeek- and Qwen-shaped batches
    const int occ = tune("EF_TUNE_SHARED_OCC", 2);
    {
        KernelTimer kt(c, s, EF_K_FFN_UP, b_up);
        if (shared) EF_HIP(c, ef::launch_ffn_gate_up_shared(gu, wg_gu, tpp, occ, c->xp, c->act, d, s));
        else if (c->q4) EF_HIP(c, ef::launch_ffn_gate_up_q4(gu, wg_gu, tpp, c->xp, c->act, d, s));
        else EF_HIP(c, ef::launch_ffn_gate_up(gu, wg_gu, tpp, ks, c->xp, c->act, d, s));
    }
    {
        KernelTimer kt(c, s, EF_K_FFN_DOWN, b_dn);
        if (shared) EF_HIP(c, ef::launch_ffn_down_shared(dn, wg_dn, tpp, occ, ksg_stream, c->act, c->y, y_plane, d, s));
        else if (c->q4) EF_HIP(c, ef::launch_ffn_down_q4(dn, wg_dn, tpp, ksg_stream, c->act, c->y, y_plane, d, s));
        else EF_HIP(c, ef::launch_ffn_down(dn, wg_dn, tpp, ksg_stream, c->act, c->y, y_plane, d, s));
    }
    if (join) EF_HIP(c, hipStreamWaitEvent(s, join, 0));
    return EF_OK;
}

}  // namespace

extern "C" int ef_moe_ffn(ef_ctx *c, int layer, const void *hidden, int T, const int32_t *topk_ids,
                          const float *topk_w, const int32_t *counts_host, const int32_t *offsets,
                          const int32_t *perm, const int32_t *inv_perm, float *out, void *stream) {
    // set by ef_layer_step for the call it makes right afterwards; never survives this call
    const bool prepacked = c && c->prepacked;
    if (c) c->prepacked = false;
    int rc = check_ctx_layer(c, layer);
    if (rc) return rc;
    if (T < 0 || T > c->cfg.max_tokens) return fail(c, EF_EINVAL, "ef_moe_ffn: T=%d outside 0..max_tokens", T);
    if (!counts_host) return fail(c, EF_EINVAL, "ef_moe_ffn: counts_host is null");
    const int E = c->cfg.n_experts, k = c->cfg.top_k, d = c->cfg.d_model;
    long long tot = 0;
    for (int e = 0; e < E; ++e) {
        if (counts_host[e] < 0 || counts_host[e] > T)
            return fail(c, EF_EINVAL, "ef_moe_ffn: counts_host[%d]=%d outside 0..T", e, counts_host[e]);
        tot += counts_host[e];
    }
    if (tot != (long long)T * k) return fail(c, EF_EINVAL, "ef_moe_ffn: counts_host sums to %lld, not T*k", tot);
    if (!c->fake && T > 0) {
        if (!hidden || !topk_ids || !topk_w || !offsets || !perm || !inv_perm || !out)
            return fail(c, EF_EINVAL, "ef_moe_ffn: null pointer");
        if (!aligned16(hidden) || !aligned16(out)) return fail(c, EF_EINVAL, "ef_moe_ffn: hidden/out must be 16-byte aligned");
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool strict = (c->cfg.flags & EF_FLAG_STRICT_RESIDENT) != 0;
    poll_all_copies(c);

    // host copies of the group geometry
    std::vector<int> offs_host((size_t)E + 1, 0), tile_start((size_t)E, 0);
    std::vector<long long> act_off((size_t)E, 0);
    int tiles = 0;
    for (int e = 0; e < E; ++e) {
        offs_host[(size_t)e + 1] = offs_host[(size_t)e] + counts_host[e];
        tile_start[(size_t)e] = tiles;
        act_off[(size_t)e] = (long long)tiles * ef::kTile * c->cfg.d_ff / 8;   // 16-byte units
        tiles += (counts_host[e] + ef::kTile - 1) / ef::kTile;
    }
    const bool has_shared = c->cfg.d_ff_shared > 0 && T > 0;
    const int shared_tile_start = tiles;
    const long long shared_act_off = (long long)tiles * ef::kTile * c->cfg.d_ff / 8;
    if (has_shared) tiles += (T + ef::kTile - 1) / ef::kTile;
    if (!c->fake && tiles > c->max_tiles) return fail(c, EF_EINVAL, "ef_moe_ffn: scratch too small (internal)");

    // K slices of the second FFN half across workgroups (one Y plane each, summed by the un-permute):
    // split while the layer's launch would have too few workgroups, a slice keeps >= 32 fragments per
    // wave and the planes fit the scratch.  One value per call: every phase shares the planes.
    const long long y_plane = ((long long)T * k + (has_shared ? T : 0)) * d;
    // Groups of at least 8 token tiles go to the matrix-core tiled kernels.  The two thresholds (total
    // workgroups of the tiled launches) exist for tuning only: on the mixed batches measured (640 tokens
    // with a 2048 x 5632 shared expert, 1056 tokens over 64 experts) the tiled kernels were equal to or
    // 8 % faster than streaming the same groups in several passes, even at 150-200 workgroups.
    bool use_tiled = false;
    long long tiled_dn_wgs = 0;
    int tiled_stages_min = 1 << 30;   // fewest K stages (32 columns each) among the tiled groups
    int tiled_stages_max = 0;         // ... and most
    if (T > 0 && (!c->q4 || c->q4_stage_slots > 0) && tune("EF_TUNE_TILED", 1) != 0) {
        long long wg_up = 0, wg_dn = 0;
        auto add = [&](int F, int cnt, bool routed) {
            const int nt = (cnt + ef::kTile - 1) / ef::kTile;
            if (!ef::ffn_tiled_ok(d, F, nt) || (routed && nt < tiled_min_routed())) return;
            wg_up += ef::ffn_gate_up_tiled_wgs(F, nt);
            wg_dn += ef::ffn_down_tiled_wgs(d, nt);
            tiled_stages_min = std::min(tiled_stages_min, F / 32);
            tiled_stages_max = std::max(tiled_stages_max, F / 32);
        };
        for (int e = 0; e < E; ++e) add(c->cfg.d_ff, counts_host[e], true);
        if (has_shared) add(c->cfg.d_ff_shared, T, false);
        use_tiled = wg_up >= tune("EF_TUNE_TILED_MIN_UP", 1) && wg_dn >= tune("EF_TUNE_TILED_MIN_DOWN", 1);
        tiled_dn_wgs = wg_dn;
    }
    // K slices of the second half (one Y plane each, summed by the un-permute): the streamed launch and the tiled
    // launch of the layer choose separately, each for its own workgroup count
    int ksg = 1, ksg_tiled = 1;
    if (T > 0) {
        long long base_wgs = 0;
        int tmax = 1;
        for (int e = 0; e < E; ++e) tmax = std::max(tmax, (counts_host[e] + ef::kTile - 1) / ef::kTile);
        if (has_shared) tmax = std::max(tmax, (T + ef::kTile - 1) / ef::kTile);
        const int tpp = (tmax >= 3 && !c->q4) ? 4 : tmax >= 2 ? 2 : 1;
        // workgroups of the streamed launch with one slice (groups that take the tiled kernels do not count)
        for (int e = 0; e < E; ++e)
            if (counts_host[e] > 0) {
                const int nt = (counts_host[e] + ef::kTile - 1) / ef::kTile;
                if (use_tiled && ef::ffn_tiled_ok(d, c->cfg.d_ff, nt) && nt >= tiled_min_routed()) continue;
                base_wgs += c->q4 ? ef::ffn_down_q4_wgs(d, nt, tpp, 1)
                            : tpp == 4 ? ef::ffn_down_shared_wgs(d, nt, tpp, 1) : ef::ffn_down_wgs(d, nt, tpp, 1);
            }
        if (has_shared && !(use_tiled && ef::ffn_tiled_ok(d, c->cfg.d_ff_shared, (T + ef::kTile - 1) / ef::kTile)))
            base_wgs += c->q4 ? ef::ffn_down_q4_wgs(d, (T + ef::kTile - 1) / ef::kTile, tpp, 1)
                        : tpp == 4 ? ef::ffn_down_shared_wgs(d, (T + ef::kTile - 1) / ef::kTile, tpp, 1)
                                   : ef::ffn_down_wgs(d, (T + ef::kTile - 1) / ef::kTile, tpp, 1);
        // the LDS-shared kernels (passes of four tiles) run two workgroups per compute unit
        const int want = tune("EF_TUNE_DOWN_WGS", (tpp == 4 && !c->q4) ? 512 : 256);
        const int nkb_min = std::min(c->cfg.d_ff, has_shared ? c->cfg.d_ff_shared : c->cfg.d_ff) / 16;
        // a slice keeps >= 32 fragments per wave (bf16: four waves split it again), >= 6 quads (4-bit), or >= 8
        // stages of four fragments (LDS-shared kernels: a wave walks the whole slice)
        const int units = c->q4 ? nkb_min / 4 / 6 : tpp == 4 ? nkb_min / 4 / 8 : nkb_min / 4 / 32;
        while (ksg < 8 && base_wgs * ksg < want && units / (ksg * 2) >= 1 && y_plane * (ksg * 2) <= c->y_floats)
            ksg *= 2;
        if (use_tiled) {
            // the tiled second half: slices until its 256 x 256 tiles fill the chip, each slice keeping at least
            // 16 stages
            while (ksg_tiled < 8 && tiled_dn_wgs * ksg_tiled < 256 && (tune("EF_TUNE_KSG_BY_MAX", 1) ? tiled_stages_max : tiled_stages_min) / (ksg_tiled * 2) >= 16 &&
                   y_plane * (ksg_tiled * 2) <= c->y_floats)
                ksg_tiled *= 2;
            if (tune("EF_TUNE_SPLIT_KSG", 1) == 0) ksg = ksg_tiled;   // one slice count for both launches
        }
        int forced = tune("EF_TUNE_DOWN_KSG", 0);
        if (forced >= 1 && forced <= 8 && y_plane * forced <= c->y_floats) ksg = ksg_tiled = forced;
    }
    ef::PlaneTable planes{};

    // classify the needed experts
    std::vector<PhaseGroup> ready, loading;
    std::vector<int> missing;
    bool any_not_ready = false;
    for (int e = 0; e < E; ++e) {
        if (counts_host[e] == 0) continue;
        int slot = c->cache->lookup(layer, e);
        if (slot < 0) {
            if (strict) {
                for (const auto &g : ready) c->cache->pin(g.slot, false);
                for (const auto &g : loading) c->cache->pin(g.slot, false);
                return fail(c, EF_ENOTRESIDENT, "ef_moe_ffn: layer %d expert %d is not resident", layer, e);
            }
            missing.push_back(e);
            any_not_ready = true;
            c->st.misses += 1;
            continue;
        }
        c->st.hits += 1;
        c->cache->touch(slot);
        c->cache->pin(slot, true);
        if (c->slots[(size_t)slot].copy_pending) { loading.push_back({e, slot}); any_not_ready = true; }
        else ready.push_back({e, slot});
    }
    // feedback counters (paper Sec. 3.2.2): a layer that had to wait counts as a stall, a layer
    // whose experts were all loaded in time counts as an overfetch
    if (T > 0) {
        if (any_not_ready) {
            if (++c->stall_counter >= std::max(1, c->cfg.stall_thresh)) { c->stall_counter = 0; c->fb_adjust += 1; }
        } else {
            if (++c->overfetch_counter >= std::max(1, c->cfg.overfetch_thresh)) { c->overfetch_counter = 0; c->fb_adjust -= 1; }
        }
        c->fb_adjust = std::max(-(c->cfg.h_max - 1), std::min(c->cfg.h_max - 1, c->fb_adjust));
    }

    auto unpin_all = [&](const std::vector<PhaseGroup> &v) {
        for (const auto &g : v)
            if (g.expert >= 0) c->cache->pin(g.slot, false);
    };
    // start what misses can start right now (slots not needed by this layer)
    std::vector<int> deferred;
    for (int e : missing) {
        int slot = -1;
        int r = swap_in_impl(c, layer, e, 1, 0, &slot, nullptr);
        if (r == EF_EBUSY) { deferred.push_back(e); continue; }
        if (r != EF_OK) { unpin_all(ready); unpin_all(loading); return r; }
        c->cache->touch(slot);
        c->cache->pin(slot, true);
        loading.push_back({e, slot});
    }

    // A slot may be overwritten once the kernels that read it have finished: an event recorded behind them
    // is what a later swap-in waits for.  One event behind the layer's last kernel serves every slot of the
    // layer; only when misses are still waiting for a slot (phase C) must each phase's slots be released as
    // soon as that phase's kernels are enqueued.
    const bool eager_marks = !deferred.empty();
    std::vector<int> read_slots;
    struct PinGuard {   // an error return between the phases must not leave the collected slots pinned
        ef_ctx *c;
        std::vector<int> *v;
        ~PinGuard() { for (int slot : *v) c->cache->pin(slot, false); }
    } pin_guard{c, &read_slots};
    auto mark_read = [&](const std::vector<PhaseGroup> &v) -> int {
        if (c->fake) { unpin_all(v); return EF_OK; }
        if (!eager_marks) {
            for (const auto &g : v)
                if (g.expert >= 0) read_slots.push_back(g.slot);
            return EF_OK;   // still pinned: released behind the layer's last kernel
        }
        hipEvent_t ev = c->read_ring[c->read_next];
        c->read_next = (c->read_next + 1) % c->read_ring.size();
        EF_HIP(c, hipEventRecord(ev, s));
        for (const auto &g : v)
            if (g.expert >= 0) c->slots[(size_t)g.slot].last_read = ev;
        unpin_all(v);
        return EF_OK;
    };
    auto release_read_slots = [&]() -> int {
        if (read_slots.empty()) return EF_OK;
        hipEvent_t ev = c->read_ring[c->read_next];
        c->read_next = (c->read_next + 1) % c->read_ring.size();
        hipError_t he = hipEventRecord(ev, s);
        for (int slot : read_slots) {
            c->slots[(size_t)slot].last_read = ev;
            c->cache->pin(slot, false);
        }
        read_slots.clear();
        if (he != hipSuccess) return fail(c, EF_EHIP, "hipEventRecord failed: %s", hipGetErrorString(he));
        return EF_OK;
    };
    auto wait_loaded = [&](const std::vector<PhaseGroup> &v) -> int {
        if (v.empty()) return EF_OK;
        if (c->fake) {
            double need = c->fake_now;
            for (const auto &g : v) need = std::max(need, c->slots[(size_t)g.slot].fake_ready_at);
            c->st.stall_seconds += need - c->fake_now;
            c->fake_now = need;
            for (const auto &g : v) poll_copy(c, g.slot);
            return EF_OK;
        }
        EventPair p = next_pair(c->stall_ring, c->stall_next, c->stall_pending);
        EF_HIP(c, hipEventRecord(p.a, s));
        for (const auto &g : v) EF_HIP(c, hipStreamWaitEvent(s, c->slots[(size_t)g.slot].ready, 0));
        EF_HIP(c, hipEventRecord(p.b, s));
        c->stall_pending.push_back(p);
        return EF_OK;
    };
    auto run_phase = [&](std::vector<PhaseGroup> &v, bool with_shared) -> int {
        std::vector<PhaseGroup> g = v;
        if (with_shared && has_shared) g.push_back({-1, -1});
        if (!c->fake) {
            int r = launch_phase(c, layer, g, counts_host, offs_host, tile_start, act_off, shared_tile_start,
                                 shared_act_off, T, ksg, ksg_tiled, planes, y_plane, use_tiled, s);
            if (r) return r;
        }
        return mark_read(v);
    };

    if (T > 0) {
        if (!c->fake && !prepacked) {
            // token permutation into per-expert tiles (all groups of this layer in one launch)
            ef::PackTable pt{};
            int n = 0;
            for (int e = 0; e < E; ++e) {
                if (counts_host[e] == 0) continue;
                pt.tile_start[n] = tile_start[(size_t)e];
                pt.row_offset[n] = offs_host[(size_t)e];
                pt.count[n] = counts_host[e];
                ++n;
            }
            if (has_shared) {
                pt.tile_start[n] = shared_tile_start;
                pt.row_offset[n] = -1;
                pt.count[n] = T;
                ++n;
            }
            pt.tile_start[n] = tiles;
            pt.n_groups = n;
            int r = EF_OK;
            long long rows = (long long)T * k + (has_shared ? T : 0);
            KernelTimer kt(c, s, EF_K_PACK, 4.0 * rows * d + 4.0 * T * k);
            hipError_t he = ef::launch_pack_x(pt, tiles, static_cast<const uint16_t *>(hidden), d, k, perm, c->xp, c->q4, s);
            if (he != hipSuccess) r = fail(c, EF_EHIP, "pack_x launch failed: %s", hipGetErrorString(he));
            if (r) { unpin_all(ready); unpin_all(loading); return r; }
        }
        // phase A: experts that are ready (+ the dense shared FFN): tokens whose experts are resident go first
        rc = run_phase(ready, true);
        if (rc) { unpin_all(loading); return rc; }
        // phase B: experts whose copy is in flight (earlier prefetches and the misses started above)
        if (!loading.empty()) {
            rc = wait_loaded(loading);
            if (!rc) rc = run_phase(loading, false);
            if (rc) { unpin_all(loading); return rc; }
        }
        // phase C: misses that had no slot until an earlier phase released one
        size_t next = 0;
        while (next < deferred.size()) {
            std::vector<PhaseGroup> wave;
            while (next < deferred.size()) {
                int slot = -1;
                int r = swap_in_impl(c, layer, deferred[next], 1, 0, &slot, nullptr);
                if (r == EF_EBUSY) break;
                if (r != EF_OK) { unpin_all(wave); return r; }
                c->cache->touch(slot);
                c->cache->pin(slot, true);
                wave.push_back({deferred[next], slot});
                ++next;
            }
            if (wave.empty()) return fail(c, EF_EBUSY, "ef_moe_ffn: no cache slot can be freed for layer %d", layer);
            rc = wait_loaded(wave);
            if (!rc) rc = run_phase(wave, false);
            if (rc) { unpin_all(wave); return rc; }
        }
        if (!c->fake) {
            KernelTimer kt(c, s, EF_K_COMBINE, 4.0 * ((double)T * k + (has_shared ? T : 0)) * d + 4.0 * T * d +
                                                   8.0 * T * k);
            // the layer's last kernel carries the read marker of the slots collected above
            hipEvent_t done = nullptr;
            if (!read_slots.empty()) {
                done = c->read_ring[c->read_next];
                c->read_next = (c->read_next + 1) % c->read_ring.size();
            }
            EF_HIP(c, ef::launch_combine(c->y, planes, y_plane, topk_w, topk_ids, inv_perm, T, k, d,
                                         has_shared ? (long long)T * k : -1ll, out, done, s));
            if (done) {
                for (int slot : read_slots) {
                    c->slots[(size_t)slot].last_read = done;
                    c->cache->pin(slot, false);
                }
                read_slots.clear();
            }
        }
    }
    if ((rc = release_read_slots())) return rc;
    if (!c->fake && c->layer_open) {
        EF_HIP(c, hipEventRecord(c->layer_cur.b, s));
        c->layer_pending.push_back(c->layer_cur);
        c->layer_open = false;
    }
    c->st.layers_run += 1;
    c->st.tokens_run += T;
    c->cache->advance();
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

extern "C" int ef_layer_step(ef_ctx *c, int layer, const void *hidden, int T, float beta, int H,
                             const float *delta, const int32_t *tok2req, float *out, int *H_next,
                             int32_t *counts_host_out, void *stream) {
    int rc = check_ctx_layer(c, layer);
    if (rc) return rc;
    if (H < 0) H = c->horizon;
    int He = 0;
    if ((rc = check_predict_args(c, layer, T, H, &He, "ef_layer_step"))) return rc;
    if (T <= 0) return fail(c, EF_EINVAL, "ef_layer_step: T must be positive");
    if ((long long)T * c->cfg.top_k >= (1ll << ef::kMetaValueBits))
        return fail(c, EF_EINVAL, "ef_layer_step: T * top_k must be below 2^24");
    if (!hidden || !out) return fail(c, EF_EINVAL, "ef_layer_step: null pointer");
    if (!aligned16(hidden) || !aligned16(out)) return fail(c, EF_EINVAL, "ef_layer_step: hidden/out must be 16-byte aligned");
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int E = c->cfg.n_experts;
    if ((rc = open_layer_timer(c, s))) return rc;
    // 1. one pass over the hidden states: routing of this layer + demand of the next He layers; the
    //    grouping kernel hands counts and histograms to the host through mapped memory
    const int seq = ++c->meta_seq;
    ef::GroupExport ex{c->meta_dev, c->st_pred_hist, He * E, EF_MAX_HORIZON * E, seq};
    rc = run_gates(c, layer, hidden, T, beta, true, He, H, delta, tok2req, c->st_ids, c->st_w, c->st_counts,
                   c->st_offsets, c->st_perm, c->st_inv, c->st_pred_ids, c->st_pred_hist, ex, s);
    if (rc) return rc;
    // the token packing only needs what the grouping kernel left on the device: enqueue it now, so it
    // runs while the host waits for and digests the counts
    bool did_pack = false;
    if (tune("EF_TUNE_EARLY_PACK", 1) != 0) {
        const int k = c->cfg.top_k, d = c->cfg.d_model;
        const bool has_shared = c->cfg.d_ff_shared > 0;
        const long long assignments = (long long)T * k;
        const int bound = (int)((assignments + ef::kTile - 1) / ef::kTile) + (int)std::min<long long>(E, assignments) +
                          (has_shared ? (T + ef::kTile - 1) / ef::kTile : 0);
        const long long rows = assignments + (has_shared ? T : 0);
        KernelTimer kt(c, s, EF_K_PACK, 4.0 * rows * d + 4.0 * T * k);
        EF_HIP(c, ef::launch_pack_x_dev(c->st_counts, c->st_offsets, E, has_shared, T, std::min(bound, c->max_tiles),
                                        static_cast<const uint16_t *>(hidden), d, k, c->st_perm, c->xp, c->q4, s));
        did_pack = true;
    }
    // 2. wait until every expected word carries this call's tag (bounded: fall back to a stream
    //    synchronisation, then give up)
    const volatile int32_t *mh = c->meta_host;
    const uint32_t tag = (uint32_t)(seq & 0xFF);
    const int n_hist = He * E;
    auto arrived = [&]() {
        for (int x = 0; x < E; ++x)
            if (((uint32_t)mh[x] >> ef::kMetaValueBits) != tag) return false;
        for (int x = 0; x < n_hist; ++x)
            if (((uint32_t)mh[ef::kMetaHist + x] >> ef::kMetaValueBits) != tag) return false;
        return true;
    };
    bool seen = false;
    for (long long spin = 0; spin < (1ll << 34); ++spin) {
        if (arrived()) { seen = true; break; }
        __builtin_ia32_pause();
        if ((spin & 0xFFFFF) == 0xFFFFF && hipStreamQuery(s) == hipSuccess) break;   // stream drained
    }
    if (!seen) {
        EF_HIP(c, hipStreamSynchronize(s));
        if (!arrived()) return fail(c, EF_EHIP, "ef_layer_step: routing results never reached the host");
    }
    const int32_t value_mask = (1 << ef::kMetaValueBits) - 1;
    int32_t counts_host[EF_MAX_EXPERTS];
    for (int e = 0; e < E; ++e) counts_host[e] = mh[e] & value_mask;
    int32_t hist_host[EF_MAX_HORIZON * EF_MAX_EXPERTS];
    for (int x = 0; x < n_hist; ++x) hist_host[x] = mh[ef::kMetaHist + x] & value_mask;
    if (counts_host_out) memcpy(counts_host_out, counts_host, (size_t)E * 4);
    // 3. grouped FFN first (resident groups, misses swapped in meanwhile, weighted un-permute): the GPU has
    //    nothing to do until these launches are enqueued, so everything else the host decides comes after
    c->prepacked = did_pack;
    rc = ef_moe_ffn(c, layer, hidden, T, c->st_ids, c->st_w, counts_host, c->st_offsets, c->st_perm, c->st_inv, out,
                    stream);
    if (rc) return rc;
    // 4. horizon for the next layer and prefetches: the copies overlap the FFN that is now running
    int Hn = c->horizon;
    if (He > 0) {
        int32_t lst[EF_MAX_HORIZON * EF_MAX_EXPERTS];
        int n = 0;
        rc = ef_choose_horizon(c, layer, hist_host, He, T, &Hn, lst, &n);
        if (rc) return rc;
        for (int i = 0; i < n; ++i) {
            const int j = lst[i] >> 16, e = lst[i] & 0xFFFF;
            rc = swap_in_impl(c, layer + j, e, 0, j, nullptr, nullptr);
            if (rc != EF_OK && rc != EF_EBUSY) return rc;   // a full, pinned cache only skips the prefetch
        }
    }
    if (H_next) *H_next = Hn;
    return EF_OK;
}

extern "C" int ef_get_stats(ef_ctx *c, ef_stats *out) {
    if (!c || !out) return fail(c, EF_EINVAL, "ef_get_stats: null pointer");
    if (!c->fake) {
        for (int q = 0; q < 2; ++q) (void)hipStreamSynchronize(c->copy_stream[q]);
        poll_pairs(c, true);
        poll_prof(c, true);
    }
    poll_all_copies(c);
    c->st.bandwidth_Bps = c->bw_Bps;
    c->st.layer_seconds_est = c->layer_s;
    c->st.horizon = c->horizon;
    c->st.stall_counter = c->stall_counter;
    c->st.overfetch_counter = c->overfetch_counter;
    int64_t n = c->st.hits + c->st.misses;
    c->st.miss_rate = n > 0 ? 1.0 - (double)c->st.hits / (double)n : 0.0;
    *out = c->st;
    return EF_OK;
}

extern "C" int ef_set_profile(ef_ctx *c, unsigned kinds_mask) {
    if (!c) return fail(nullptr, EF_EINVAL, "null context");
    if (c->fake) return fail(c, EF_ENOSYS, "ef_set_profile: fake-copy context has no device");
    poll_prof(c, true);
    if (kinds_mask && c->prof_ring.empty()) {
        c->prof_ring.resize(1024);
        for (auto &p : c->prof_ring) {
            EF_HIP(c, hipEventCreate(&p.a));
            EF_HIP(c, hipEventCreate(&p.b));
        }
    }
    c->profile_mask = kinds_mask & 0x3FFu;
    return EF_OK;
}

extern "C" int ef_set_profile_sampling(ef_ctx *c, int every) {
    if (!c) return fail(nullptr, EF_EINVAL, "null context");
    if (every < 1) return fail(c, EF_EINVAL, "ef_set_profile_sampling: every must be >= 1");
    c->profile_every = every;
    for (auto &n : c->profile_seen) n = 0;
    return EF_OK;
}

extern "C" int ef_reset_stats(ef_ctx *c) {
    if (!c) return fail(nullptr, EF_EINVAL, "null context");
    if (!c->fake) { poll_pairs(c, true); poll_prof(c, true); }
    c->st = ef_stats{};
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

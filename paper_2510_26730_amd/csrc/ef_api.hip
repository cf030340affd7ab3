// C-ABI layer: utilities, context life cycle, the thin entry points of prediction and routing, the composite
// layer step, statistics, profiling switches and launch tuning.  Declarations and argument contracts are in
// include/expertflow.h; the cache runtime is ef_runtime.hip, the launch planner ef_plan.hip.
#include "ef_ctx.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <thread>

using namespace efi;

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

namespace {
// bf16 bit pattern -> fp16 bit pattern of the same number (round to nearest even below the fp16 normal range,
// where the grid is 2^-24); false for infinities, NaNs and magnitudes of 2^16 and more
bool bf16_to_f16_bits(uint16_t b, uint16_t *out) {
    const uint32_t sign = (uint32_t)(b >> 15) << 15, exp = (b >> 7) & 0xFFu, man = b & 0x7Fu;
    if (exp == 0xFFu) return false;
    if (exp == 0) { *out = (uint16_t)sign; return true; }          // below 2^-126
    const int e = (int)exp - 127;
    if (e > 15) return false;
    if (e >= -14) { *out = (uint16_t)(sign | ((uint32_t)(e + 15) << 10) | (man << 3)); return true; }
    const uint32_t m = 128u + man;                                   // value = m * 2^(e - 7) = m * 2^(e + 17) * 2^-24
    if (e >= -17) { *out = (uint16_t)(sign | (m << (e + 17))); return true; }
    const int r = -(e + 17);
    if (r > 9) { *out = (uint16_t)sign; return true; }
    uint32_t q = m >> r;
    const uint32_t rem = m & ((1u << r) - 1u), half = 1u << (r - 1);
    if (rem > half || (rem == half && (q & 1u))) ++q;
    *out = (uint16_t)(sign | q);
    return true;
}
}  // namespace

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
    std::atomic<bool> w2_ok{true};
    auto section_b = [&](int cb0, int cb1) {   // W2 leaves as fp16 (the second FFN half runs in fp16)
        uint16_t *base = out + (size_t)2 * d * F;
        bool ok = true;
        for (int cb = cb0; cb < cb1; ++cb)
            for (int kb = 0; kb < nkb2; ++kb)
                for (int lane = 0; lane < 64; ++lane) {
                    int g = lane >> 5, i = lane & 31;
                    const uint16_t *src = W2 + (size_t)(cb * 32 + i) * F + kb * 16 + 4 * g;
                    uint16_t *dst = base + (((size_t)cb * nkb2 + kb) * 64 + lane) * 8;
                    for (int t = 0; t < 4; ++t) {
                        ok &= bf16_to_f16_bits(src[t], dst + t);          // t = 0..3 -> columns 4g + t
                        ok &= bf16_to_f16_bits(src[8 + t], dst + 4 + t);  // t = 4..7 -> columns 8 + 4g + (t-4)
                    }
                }
        if (!ok) w2_ok = false;
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
    if (!w2_ok) return fail(nullptr, EF_EINVAL, "ef_pack_expert: W2 holds a value that is not finite in fp16 (|w| >= 65536, inf or NaN)");
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
        copy_engine_stop(c);      // the worker thread first: it uses the copy stream and the slot events
        (void)hipDeviceSynchronize();
        for (auto &s : c->slots)
            if (s.ready) (void)hipEventDestroy(s.ready);
        for (auto e : c->read_ring) (void)hipEventDestroy(e);
        for (auto e : c->fork_ring) (void)hipEventDestroy(e);
        if (c->side_stream) (void)hipStreamDestroy(c->side_stream);
        for (auto &p : c->stall_ring) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
        for (auto &p : c->layer_ring) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
        for (auto &p : c->prof_ring) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
        if (c->copy_stream) (void)hipStreamDestroy(c->copy_stream);
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
    tuning_defaults(&c->tune);
    c->q4 = g.weight_bits == 4;
    c->expert_bytes = c->q4 ? ef_expert_bytes_q4(g.d_model, g.d_ff) : ef_expert_bytes(g.d_model, g.d_ff);
    c->fake = (g.flags & EF_FLAG_FAKE_COPY) != 0;
    c->layers.resize((size_t)g.n_layers);
    c->cache = new ef::ExpertCache(g.slots_total, g.slots_per_layer_max, g.n_layers, g.n_experts, g.top_k);
    c->slots.resize((size_t)g.slots_total);
    c->pred_mask.assign((size_t)g.n_layers * EF_MAX_HORIZON, 0);
    c->pred_valid.assign((size_t)g.n_layers * EF_MAX_HORIZON, 0);
    c->eng.chunk_bytes = (size_t)c->tune.copy_chunk_mib << 20;
    c->eng.depth = c->tune.copy_depth;
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
    // under 256 MiB (small batches split K of the second FFN half across workgroups), or up to 4 while it stays
    // under 2 GiB (large batches cut the last group of a tiled second half into K slices)
    const long long y_plane_max = (Tm * k + (g.d_ff_shared > 0 ? Tm : 0)) * d;
    long long planes = std::max({1ll, std::min(8ll, (64ll << 20) / y_plane_max), std::min(4ll, (512ll << 20) / y_plane_max)});
    c->y_floats = y_plane_max * planes;
    const size_t y_bytes = (size_t)c->y_floats * 4;

    auto bail = [&](hipError_t e, const char *what) {
        int rc = fail(nullptr, e == hipErrorOutOfMemory ? EF_ENOMEM : EF_EHIP, "ef_create: %s: %s", what,
                      hipGetErrorString(e));
        std::string keep = thread_error();
        ef_destroy(c);
        set_thread_error(keep);
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
        memset(c->meta_host, 0xFF, (size_t)ef::kMetaInts * 4);   // every word carries the tag no call uses
        if ((e = hipHostGetDevicePointer(reinterpret_cast<void **>(&c->meta_dev), c->meta_host, 0)) != hipSuccess)
            return bail(e, "host-mapped hand-over buffer");
    }
    if ((e = hipStreamCreateWithFlags(&c->copy_stream, hipStreamNonBlocking)) != hipSuccess)
        return bail(e, "copy stream");
    {   // resolve the address of ef_route_static's scratch on this device now, so that the call itself never has to
        EfRouteScratch rs{};
        if (static_route_scratch(c, &rs) != EF_OK) {
            std::string keep = thread_error();
            ef_destroy(c);
            set_thread_error(keep);
            return EF_EHIP;
        }
    }
    for (auto &s : c->slots)
        if ((e = hipEventCreateWithFlags(&s.ready, hipEventDisableTiming)) != hipSuccess) return bail(e, "event");
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
    if (copy_engine_start(c) != EF_OK) {
        std::string keep = thread_error();
        ef_destroy(c);
        set_thread_error(keep);
        return EF_EHIP;
    }
    *out = c;
    return EF_OK;
}

extern "C" const char *ef_last_error(ef_ctx *c) { return c ? c->err.c_str() : thread_error(); }

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
    EfLayerReg &L = c->layers[(size_t)layer];
    L.gate_w = static_cast<const uint16_t *>(gate_w);
    L.gate_b = gate_b;
    L.experts = static_cast<const char *>(experts);
    L.shared_blob = shared_blob;
    L.set = true;
    return EF_OK;
}

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
                     nullptr, nullptr, topk_ids, hist, kNoExport, ctx_route_scratch(c), s);
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
    if (ef::dist_needs_packed(T, c->tune.dist_form))
        EF_HIP(c, ef::launch_pack_x(pt, ntiles, static_cast<const uint16_t *>(hidden), d, 1, nullptr, c->xp, false, s));
    EF_HIP(c, ef::launch_token_dist(static_cast<const uint16_t *>(hidden), T, d, c->xp, c->y, tok_dist, dist,
                                    c->tune.dist_form, s));
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
                     perm, inv_perm, nullptr, nullptr, kNoExport, ctx_route_scratch(c), s);
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
                     perm, inv_perm, pred_ids, pred_hist, kNoExport, ctx_route_scratch(c), s);
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
    // The tag of a call is its sequence number modulo 255: the value 255 is never a call's tag.  The buffer
    // starts out filled with it, and the host writes it back over every word once it has read it, so a word
    // that shows a call's tag was written by that call (not by the one 255 calls earlier whose words of a
    // look-ahead position no call in between rewrote).
    const int seq = (int)(++c->meta_seq % 255);
    ef::GroupExport ex{c->meta_dev, c->st_pred_hist, He * E, EF_MAX_HORIZON * E, seq};
    rc = run_gates(c, layer, hidden, T, beta, true, He, H, delta, tok2req, c->st_ids, c->st_w, c->st_counts,
                   c->st_offsets, c->st_perm, c->st_inv, c->st_pred_ids, c->st_pred_hist, ex, ctx_route_scratch(c), s);
    if (rc) return rc;
    // the token packing only needs what the grouping kernel left on the device: enqueue it now, so it
    // runs while the host waits for and digests the counts
    bool did_pack = false;
    if (c->tune.early_pack != 0) {
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
    const uint32_t tag = (uint32_t)seq;
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
    // consumed: back to the tag no call uses (the kernels of this call have written each of these words once,
    // and nothing writes them again before the next call's kernels)
    {
        volatile int32_t *mw = c->meta_host;
        for (int x = 0; x < E; ++x) mw[x] = -1;
        for (int x = 0; x < n_hist; ++x) mw[ef::kMetaHist + x] = -1;
    }
    c->last_T = T;
    c->last_He = He;
    memcpy(c->last_hist, hist_host, (size_t)n_hist * 4);
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
        int rc = copy_engine_drain(c);
        if (rc) return rc;
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


// =================================================================================================
// inspection and tuning
// =================================================================================================

extern "C" int ef_layer_step_fetch(ef_ctx *c, int32_t *topk_ids, float *topk_w, int32_t *offsets, int32_t *perm,
                                   int32_t *inv_perm, int32_t *pred_ids, int32_t *pred_hist, int *T_out,
                                   int *H_eff_out, void *stream) {
    if (!c) return fail(nullptr, EF_EINVAL, "null context");
    if (c->fake) return fail(c, EF_ENOSYS, "ef_layer_step_fetch: fake-copy context has no device");
    if (c->last_T <= 0) return fail(c, EF_EINVAL, "ef_layer_step_fetch: no ef_layer_step has run yet");
    EF_HIP(c, hipStreamSynchronize(static_cast<hipStream_t>(stream)));
    const size_t n = (size_t)c->last_T * c->cfg.top_k;
    const int E = c->cfg.n_experts;
    if (topk_ids) EF_HIP(c, hipMemcpy(topk_ids, c->st_ids, n * 4, hipMemcpyDeviceToHost));
    if (topk_w) EF_HIP(c, hipMemcpy(topk_w, c->st_w, n * 4, hipMemcpyDeviceToHost));
    if (offsets) EF_HIP(c, hipMemcpy(offsets, c->st_offsets, (size_t)(E + 1) * 4, hipMemcpyDeviceToHost));
    if (perm) EF_HIP(c, hipMemcpy(perm, c->st_perm, n * 4, hipMemcpyDeviceToHost));
    if (inv_perm) EF_HIP(c, hipMemcpy(inv_perm, c->st_inv, n * 4, hipMemcpyDeviceToHost));
    if (pred_ids && c->last_He > 0)
        EF_HIP(c, hipMemcpy(pred_ids, c->st_pred_ids, n * 4 * (size_t)c->last_He, hipMemcpyDeviceToHost));
    if (pred_hist && c->last_He > 0) memcpy(pred_hist, c->last_hist, (size_t)c->last_He * E * 4);
    if (T_out) *T_out = c->last_T;
    if (H_eff_out) *H_eff_out = c->last_He;
    return EF_OK;
}

void efi::tuning_defaults(ef_tuning *t) {
    t->tiled = 1;
    // Routed groups take the tiled kernels from this many token tiles on (the kernels accept 8).  A group of 8 or
    // 9 tiles is one 256-token panel (plus an almost empty one): its weight panels are read by a single workgroup
    // each, cold from HBM with three stages in flight, and such workgroups outlast those of a group with several
    // token panels in the same launch; the streaming kernels serve them better.
    t->tiled_min_tiles = 10;
    t->tiled_min_up_wgs = 1;
    t->tiled_min_down_wgs = 1;
    t->tiled_xcd_rotation = 1;
    t->overlap_tiled = 1;
    t->sort_groups = 1;
    t->passes_of_four = 1;
    t->lds_shared = 1;
    t->lds_shared_occupancy = 0;
    t->up_want_waves = 640;
    t->up_k_slices = 0;
    t->down_want_wgs = 0;
    t->down_k_slices = 0;
    t->down_slices_by_longest_k = 1;
    t->down_split_slice_counts = 1;
    t->gate_k_split = 0;
    t->gate_token_split = 1;
    t->gate_fused_finish = 1;
    t->down_tail_split = 1;
    t->tiled_tail_slices = 1;
    t->dist_form = 0;
    t->gate_stream = 1;
    t->early_pack = 1;
    t->copy_chunk_mib = 32;
    t->copy_depth = 2;
}

extern "C" int ef_get_tuning(ef_ctx *c, ef_tuning *out) {
    if (!c || !out) return fail(c, EF_EINVAL, "ef_get_tuning: null pointer");
    *out = c->tune;
    return EF_OK;
}

extern "C" int ef_set_tuning(ef_ctx *c, const ef_tuning *t) {
    if (!c || !t) return fail(c, EF_EINVAL, "ef_set_tuning: null pointer");
    auto flag = [](int v) { return v == 0 || v == 1; };
    const char *bad = nullptr;
    if (!flag(t->tiled)) bad = "tiled";
    else if (t->tiled_min_tiles < ef::kTiledMinTiles || t->tiled_min_tiles > 4096) bad = "tiled_min_tiles";
    else if (t->tiled_min_up_wgs < 1) bad = "tiled_min_up_wgs";
    else if (t->tiled_min_down_wgs < 1) bad = "tiled_min_down_wgs";
    else if (!flag(t->tiled_xcd_rotation)) bad = "tiled_xcd_rotation";
    else if (!flag(t->overlap_tiled)) bad = "overlap_tiled";
    else if (!flag(t->sort_groups)) bad = "sort_groups";
    else if (!flag(t->passes_of_four)) bad = "passes_of_four";
    else if (!flag(t->lds_shared)) bad = "lds_shared";
    else if (t->lds_shared_occupancy < 0 || t->lds_shared_occupancy > 2) bad = "lds_shared_occupancy";
    else if (t->up_want_waves < 1) bad = "up_want_waves";
    else if (t->up_k_slices != 0 && t->up_k_slices != 1 && t->up_k_slices != 2 && t->up_k_slices != 4) bad = "up_k_slices";
    else if (t->down_want_wgs < 0) bad = "down_want_wgs";
    else if (t->down_k_slices < 0 || t->down_k_slices > 8) bad = "down_k_slices";
    else if (!flag(t->down_slices_by_longest_k)) bad = "down_slices_by_longest_k";
    else if (!flag(t->down_split_slice_counts)) bad = "down_split_slice_counts";
    else if (t->gate_k_split < 0 || t->gate_k_split > 16) bad = "gate_k_split";
    else if (!flag(t->gate_token_split)) bad = "gate_token_split";
    else if (!flag(t->gate_fused_finish)) bad = "gate_fused_finish";
    else if (!flag(t->down_tail_split)) bad = "down_tail_split";
    else if (t->tiled_tail_slices != 0 && t->tiled_tail_slices != 1 && t->tiled_tail_slices != 2 &&
             t->tiled_tail_slices != 4 && t->tiled_tail_slices != 8) bad = "tiled_tail_slices";
    else if (t->dist_form < 0 || t->dist_form > 2) bad = "dist_form";
    else if (!flag(t->gate_stream)) bad = "gate_stream";
    else if (!flag(t->early_pack)) bad = "early_pack";
    else if (t->copy_chunk_mib < 1 || t->copy_chunk_mib > 1024) bad = "copy_chunk_mib";
    else if (t->copy_depth < 1 || t->copy_depth > 8) bad = "copy_depth";
    if (bad) return fail(c, EF_EINVAL, "ef_set_tuning: %s out of range", bad);
    c->tune = *t;
    {
        std::lock_guard<std::mutex> lock(c->eng.mu);     // the copy worker reads these
        c->eng.chunk_bytes = (size_t)t->copy_chunk_mib << 20;
        c->eng.depth = t->copy_depth;
    }
    return EF_OK;
}

// ef_route_static: the routing entry point for callers that cannot allocate device memory (code under HIP
// graph capture, tight serving loops, harnesses that forbid hipMalloc).  Same kernels and same results as
// ef_route; the only difference is where the kernels' scratch lives: in a file-scope device array of this
// translation unit instead of buffers the context allocated.
#include "ef_ctx.h"

#include <mutex>

namespace {

// Layout of the static scratch (bytes): per-tile expert counts, their prefixes, partial logits of K-split gates.
constexpr size_t kCountsBytes = (size_t)(EF_ROUTE_STATIC_MAX_TOKENS / ef::kTile) * EF_MAX_EXPERTS * 4;   // 64 KiB
constexpr size_t kPartOffset = 2 * kCountsBytes;
constexpr size_t kScratchBytes = EF_ROUTE_STATIC_SCRATCH_BYTES;
static_assert(kPartOffset < kScratchBytes && kPartOffset % 256 == 0, "scratch layout");

// Every GPU the library runs on holds its own copy of this array, at its own address, until the process ends.
// In host code the name is only a handle for hipGetSymbolAddress: kernels get the resolved address.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
void *g_scratch_ptr[kMaxDevices] = {};

}  // namespace

// Address of the static scratch on the current device, resolved once per device (at ef_create, with that
// device current; on first use otherwise).
int efi::static_route_scratch(ef_ctx *c, EfRouteScratch *out) {
    int dev = -1;
    EF_HIP(c, hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(c, EF_EINVAL, "static scratch: device index %d not supported", dev);
    void *ptr = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        if (!g_scratch_ptr[dev]) {
            void *p = nullptr;
            EF_HIP(c, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
            if (!p) return fail(c, EF_EHIP, "static scratch: hipGetSymbolAddress returned a null address");
            g_scratch_ptr[dev] = p;
        }
        ptr = g_scratch_ptr[dev];
    }
    unsigned char *base = static_cast<unsigned char *>(ptr);
    out->blockcounts = reinterpret_cast<int32_t *>(base);
    out->blockbase = reinterpret_cast<int32_t *>(base + kCountsBytes);
    out->gate_part = reinterpret_cast<float *>(base + kPartOffset);
    out->gate_part_floats = (kScratchBytes - kPartOffset) / sizeof(float);
    return EF_OK;
}

extern "C" int ef_route_static(ef_ctx *c, int layer, const void *hidden, int T, float beta, int32_t *topk_ids,
                               float *topk_w, int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv_perm,
                               void *stream) {
    using namespace efi;
    int rc = check_ctx_layer(c, layer);
    if (rc) return rc;
    if (c->fake) return fail(c, EF_ENOSYS, "ef_route_static: fake-copy context has no device");
    if (T < 0) return fail(c, EF_EINVAL, "ef_route_static: T=%d is negative", T);
    if (T > EF_ROUTE_STATIC_MAX_TOKENS)
        return fail(c, EF_EINVAL, "ef_route_static: T=%d exceeds the static scratch (at most %d tokens per call)", T,
                    EF_ROUTE_STATIC_MAX_TOKENS);
    if (!counts || !offsets) return fail(c, EF_EINVAL, "ef_route_static: null pointer");
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int E = c->cfg.n_experts;
    if (T == 0) {
        EF_HIP(c, ef::launch_fill_i32(counts, E, 0, s));
        EF_HIP(c, ef::launch_fill_i32(offsets, E + 1, 0, s));
        return EF_OK;
    }
    if (!hidden || !topk_ids || !topk_w || !perm || !inv_perm) return fail(c, EF_EINVAL, "ef_route_static: null pointer");
    if (!aligned16(hidden)) return fail(c, EF_EINVAL, "ef_route_static: hidden must be 16-byte aligned");
    EfRouteScratch rs{};
    if ((rc = static_route_scratch(c, &rs))) return rc;
    if ((rc = open_layer_timer(c, s))) return rc;
    // Nothing in the scratch has to start at zero: the gate kernels store (or zero, then add to) every per-tile
    // count they are asked for, the partial logits are written before the second gate step reads them, and the
    // prefixes before the scatter does.  What the previous call left there is simply overwritten.
    return run_gates(c, layer, hidden, T, beta, true, 0, 0, nullptr, nullptr, topk_ids, topk_w, counts, offsets, perm,
                     inv_perm, nullptr, nullptr, kNoExport, rs, s);
}

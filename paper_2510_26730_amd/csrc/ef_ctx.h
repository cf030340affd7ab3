// The context behind the C ABI and the helpers its three translation units share:
//   ef_api.hip      the ABI's utilities, context life cycle, statistics, tuning, the composite layer step
//   ef_runtime.hip  expert cache runtime: slots, copy queue and streams, completion polling, estimators,
//                   horizon controller
//   ef_plan.hip     launch planner: gate / grouping launches, the phases of the grouped FFN
// Declarations and argument contracts of the ABI itself are in include/expertflow.h.
#pragma once
#include "../../include/expertflow.h"

#include <hip/hip_runtime.h>

#include <chrono>
#include <condition_variable>
#include <cstdint>
#include <deque>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

#include "ef_cache.h"
#include "ef_kernels.h"

struct EfLayerReg {
    const uint16_t *gate_w = nullptr;
    const float *gate_b = nullptr;
    const char *experts = nullptr;
    const void *shared_blob = nullptr;
    bool set = false;
};

struct EfSlotDev {
    hipEvent_t ready = nullptr;       // recorded behind the last chunk of the slot's copy
    hipEvent_t last_read = nullptr;   // borrowed from the read-event ring (may be null)
    bool copy_pending = false;        // a copy was requested and not yet seen complete
    bool copy_queued = false;         // ... and not all of its chunks have been handed to the link yet (guarded by
                                      // the copy engine's mutex)
    bool prefetched_unused = false;   // filled by a prefetch that no layer has used yet
    double fake_ready_at = 0.0;       // fake-copy contexts: completion time of the copy
    size_t copy_bytes = 0;
};

// One expert copy in the queue of the copy engine: the bytes not yet handed to the link.
struct EfCopyJob {
    int slot = -1, layer = -1, expert = -1;
    bool miss = false;                // priority copy: taken before any prefetch
    bool started = false;
    size_t done = 0, total = 0;
    hipEvent_t war = nullptr;         // the last kernels that read the slot's previous content
    std::chrono::steady_clock::time_point t_request;
    double fake_request = 0.0;
};

// The copy queue of a context (paper Sec. 3.4): one link, chunked copies, misses first.  On a device a worker
// thread hands chunks to the copy stream; fake-copy contexts run the same policy on the fake clock.
struct EfCopyEngine {
    std::mutex mu;
    std::condition_variable cv_work, cv_done;
    std::deque<EfCopyJob> pending;    // arrival order
    size_t chunk_bytes = (size_t)32 << 20;
    int depth = 2;
    // device
    struct InFlight { hipEvent_t ev; size_t bytes; bool back_to_back; bool last_of_miss; size_t miss_bytes;
                      std::chrono::steady_clock::time_point t_request; };
    std::vector<hipEvent_t> chunk_ev;
    size_t chunk_next = 0;
    std::deque<InFlight> inflight;
    hipEvent_t prev_done = nullptr;   // the chunk that completed last (start of the next chunk's transfer)
    std::thread worker;
    bool stop = false, failed = false;
    int device = 0;
    std::string error;
    // results the worker leaves for the context's thread (applied in poll_all_copies)
    std::vector<double> bw_samples;
    double copy_seconds = 0.0, miss_seconds = 0.0;
    long long bytes_timed = 0, miss_bytes = 0, miss_copies = 0;
    // fake clock
    struct FakeChunk { double finish; int slot; bool last; };
    std::deque<FakeChunk> fake_committed;
    double fake_t = 0.0, fake_link_free = 0.0;
};

struct EfEventPair {
    hipEvent_t a, b;
};

// Device scratch of the routing launches: per-tile expert counts and their prefixes ([token tiles][E] each) and
// the partial logits of K-split gate launches.
struct EfRouteScratch {
    int32_t *blockcounts, *blockbase;
    float *gate_part;
    size_t gate_part_floats;
};

struct ef_ctx {
    ef_config cfg{};
    ef_tuning tune{};
    size_t expert_bytes = 0;
    bool fake = false;
    std::vector<EfLayerReg> layers;
    ef::ExpertCache *cache = nullptr;
    char *pool = nullptr;
    std::vector<EfSlotDev> slots;
    hipStream_t copy_stream = nullptr;
    EfCopyEngine eng;
    // look-ahead bookkeeping for the overlap statistics: pred_mask[(layer, j-1)] = experts the look-ahead made j
    // layers before `layer` named, pred_valid its "was made" flags
    std::vector<uint64_t> pred_mask;
    std::vector<uint8_t> pred_valid;
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
    long long meta_seq = 0;
    // what the last ef_layer_step saw (ef_layer_step_fetch)
    int last_T = 0, last_He = 0;
    int32_t last_hist[EF_MAX_HORIZON * EF_MAX_EXPERTS] = {};
    // side stream on which a phase's tiled launches run beside its streamed launches, and the fork / join events
    hipStream_t side_stream = nullptr;
    std::vector<hipEvent_t> fork_ring;
    size_t fork_next = 0;
    // event rings
    std::vector<hipEvent_t> read_ring;
    size_t read_next = 0;
    std::vector<EfEventPair> stall_ring, layer_ring;
    size_t stall_next = 0, layer_next = 0;
    std::deque<EfEventPair> stall_pending, layer_pending;
    struct ProfItem { EfEventPair p; int kind; double bytes; double flops; };
    std::vector<EfEventPair> prof_ring;
    size_t prof_next = 0;
    std::deque<ProfItem> prof_pending;
    unsigned profile_mask = 0;       // bit per kernel kind that is bracketed with events
    int profile_every = 1;           // bracket every n-th launch of a selected kernel kind
    long long profile_seen[EF_K_COUNT] = {};
    bool layer_open = false;
    long long layer_calls = 0;       // layers started (every kLayerTimerEvery-th is timed)
    EfEventPair layer_cur{nullptr, nullptr};
    // estimators and feedback
    double bw_Bps = 50e9, layer_s = 200e-6;
    int horizon = 1, fb_adjust = 0;
    int stall_counter = 0, overfetch_counter = 0;
    ef_stats st{};
    // fake clock
    double fake_now = 0.0;
    std::string err;
};

namespace efi {

// Every kLayerTimerEvery-th layer is bracketed with events for the T_l estimate: an event record between two
// kernels costs the stream a bubble of 2-3 us, and the estimate is a moving average anyway.
constexpr long long kLayerTimerEvery = 4;

int fail(ef_ctx *ctx, int code, const char *fmt, ...) __attribute__((format(printf, 3, 4)));
const char *thread_error();
void set_thread_error(const std::string &s);

#define EF_HIP(ctx, call)                                                                            \
    do {                                                                                             \
        hipError_t _e = (call);                                                                      \
        if (_e != hipSuccess)                                                                        \
            return efi::fail(ctx, EF_EHIP, "%s failed: %s (%s:%d)", #call, hipGetErrorString(_e),   \
                             __FILE__, __LINE__);                                                    \
    } while (0)

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

void tuning_defaults(ef_tuning *t);

// ---- cache runtime (ef_runtime.hip) ---------------------------------------------------------------
void poll_copy(ef_ctx *c, int slot);
void poll_all_copies(ef_ctx *c);
void poll_pairs(ef_ctx *c, bool wait);
void poll_prof(ef_ctx *c, bool wait);
EfEventPair next_pair(std::vector<EfEventPair> &ring, size_t &next, std::deque<EfEventPair> &pending);
uint64_t resident_mask(ef_ctx *c, int layer);
int check_ctx_layer(ef_ctx *c, int layer);
// Make (layer, expert) resident; *loaded (may be null) tells whether a copy was started.
int swap_in_impl(ef_ctx *c, int layer, int expert, int priority, int due_in, int *slot_out, bool *loaded);
// copy engine
int copy_engine_start(ef_ctx *c);        // device contexts: events and the worker thread
void copy_engine_stop(ef_ctx *c);
// The layer being run needs these slots: their copies become priority copies, and the call returns once every
// chunk of them has been handed to the copy stream (their ready events can then be waited for by a stream).
int copy_engine_flush(ef_ctx *c, const int *slots, int n);
int copy_engine_drain(ef_ctx *c);        // until the queue is empty (statistics, destruction)
// fake-copy contexts: run the queue up to the fake clock / until the copies into these slots are complete
void fake_copy_advance(ef_ctx *c, double now);
double fake_copy_wait(ef_ctx *c, const int *slots, int n);

// Brackets one kernel launch with events on the launch stream when profiling is on.
struct KernelTimer {
    ef_ctx *c;
    hipStream_t s;
    int kind;
    double bytes, flops;
    EfEventPair p{nullptr, nullptr};
    bool on;
    KernelTimer(ef_ctx *ctx, hipStream_t st, int k, double b, double f = 0.0);
    ~KernelTimer();
};

// ---- launch planner (ef_plan.hip) -----------------------------------------------------------------
extern const ef::GroupExport kNoExport;
// One pass over `hidden`: optionally the current layer's own gate (routing outputs and grouping)
// and the gates of the next He layers (prediction outputs).  Wide launches are split over the gates.
int run_gates(ef_ctx *c, int layer, const void *hidden, int T, float beta, bool do_route, int He, int H_stride,
              const float *delta, const int32_t *tok2req, int32_t *topk_ids, float *topk_w, int32_t *counts,
              int32_t *offsets, int32_t *perm, int32_t *inv_perm, int32_t *pred_ids, int32_t *pred_hist,
              const ef::GroupExport &ex, const EfRouteScratch &rs, hipStream_t s);
// the static device scratch of ef_route_static on the current device (ef_static.hip)
int static_route_scratch(ef_ctx *c, EfRouteScratch *out);
inline EfRouteScratch ctx_route_scratch(const ef_ctx *c) {
    return EfRouteScratch{c->blockcounts, c->blockbase, c->gate_part, c->gate_part_floats};
}
int check_predict_args(ef_ctx *c, int layer, int T, int H, int *He_out, const char *who);
int open_layer_timer(ef_ctx *c, hipStream_t s);

}  // namespace efi

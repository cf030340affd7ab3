// Two-level LRU expert cache policy (host only, no HIP).
//
// Follows the paper's expert memory management (Sec. 3.3.1): a `high` tier for experts used
// within the recent window of layers or predicted to be needed soon, a `low` tier for the rest;
// victims come from `low` first.  Tiers are re-derived whenever the clock or the look-ahead S
// changes.  Readings where the paper is silent: the window is S layers; a prediction keeps an
// entry high until the tick it is due; inside `high`, entries no prediction waits for go first
// (least recently used first), and if every candidate is awaited the one due furthest ahead goes.
#pragma once
#include <cstdint>
#include <vector>

namespace ef {

struct CacheEntry {
    int layer = -1, expert = -1;   // layer < 0: slot is free
    int64_t stamp = 0;             // recency: larger = more recent
    int64_t last_use = INT64_MIN / 2;
    int64_t due = INT64_MIN / 2;
    bool high = false;
    bool pinned = false;
};

enum class SwapResult { Hit, Load, Busy };

class ExpertCache {
public:
    ExpertCache(int slots_total, int per_layer_cap, int n_layers, int n_experts)
        : cap_(per_layer_cap), n_layers_(n_layers), n_experts_(n_experts),
          slots_((size_t)slots_total), map_((size_t)n_layers * n_experts, -1),
          per_layer_((size_t)n_layers, 0) {}

    int slots_total() const { return (int)slots_.size(); }
    const CacheEntry &entry(int slot) const { return slots_[(size_t)slot]; }
    int lookup(int layer, int expert) const { return map_[(size_t)layer * n_experts_ + expert]; }
    int64_t clock() const { return clock_; }
    int S() const { return S_; }

    void retier() {
        for (auto &e : slots_)
            if (e.layer >= 0) e.high = is_high(e);
    }
    void advance() { ++clock_; retier(); }
    void set_S(int S) { S_ = S; retier(); }

    void touch(int slot) {
        CacheEntry &e = slots_[(size_t)slot];
        e.stamp = ++stamp_;
        e.last_use = clock_;
        e.high = true;
    }
    void pin(int slot, bool on) { slots_[(size_t)slot].pinned = on; }

    // Make (layer, expert) resident.  due_in = layers until needed (0 = needed now).
    // On Load, *slot is the slot to fill and (*ev_layer, *ev_expert) the evicted entry or -1.
    SwapResult swap_in(int layer, int expert, int due_in, int *slot, int *ev_layer, int *ev_expert) {
        *ev_layer = *ev_expert = -1;
        int64_t due = clock_ + due_in;
        int s = lookup(layer, expert);
        if (s >= 0) {
            CacheEntry &e = slots_[(size_t)s];
            e.stamp = ++stamp_;
            if (due > e.due) e.due = due;
            e.high = true;
            *slot = s;
            return SwapResult::Hit;
        }
        s = victim(layer);
        if (s < 0) return SwapResult::Busy;
        CacheEntry &e = slots_[(size_t)s];
        if (e.layer >= 0) {
            *ev_layer = e.layer;
            *ev_expert = e.expert;
            map_[(size_t)e.layer * n_experts_ + e.expert] = -1;
            per_layer_[(size_t)e.layer] -= 1;
        }
        e = CacheEntry();
        e.layer = layer;
        e.expert = expert;
        e.stamp = ++stamp_;
        e.last_use = due_in == 0 ? clock_ : INT64_MIN / 2;
        e.due = due;
        e.high = true;
        map_[(size_t)layer * n_experts_ + expert] = s;
        per_layer_[(size_t)layer] += 1;
        *slot = s;
        return SwapResult::Load;
    }

    // Drop an entry (failed copy): the slot becomes free again.
    void drop(int slot) {
        CacheEntry &e = slots_[(size_t)slot];
        if (e.layer >= 0) {
            map_[(size_t)e.layer * n_experts_ + e.expert] = -1;
            per_layer_[(size_t)e.layer] -= 1;
        }
        e = CacheEntry();
    }

private:
    bool is_high(const CacheEntry &e) const { return (clock_ - e.last_use <= S_) || (e.due >= clock_); }

    int victim(int layer) const {
        bool layer_full = cap_ > 0 && per_layer_[(size_t)layer] >= cap_;
        if (!layer_full)
            for (size_t s = 0; s < slots_.size(); ++s)
                if (slots_[s].layer < 0) return (int)s;
        int best_low = -1, best_idle = -1, best_due = -1;
        for (size_t s = 0; s < slots_.size(); ++s) {
            const CacheEntry &e = slots_[s];
            if (e.layer < 0 || e.pinned) continue;
            if (layer_full && e.layer != layer) continue;
            if (!e.high) {
                if (best_low < 0 || e.stamp < slots_[(size_t)best_low].stamp) best_low = (int)s;
            } else if (e.due < clock_) {
                if (best_idle < 0 || e.stamp < slots_[(size_t)best_idle].stamp) best_idle = (int)s;
            } else {
                if (best_due < 0) best_due = (int)s;
                else {
                    const CacheEntry &b = slots_[(size_t)best_due];
                    if (e.due > b.due || (e.due == b.due && e.stamp > b.stamp)) best_due = (int)s;
                }
            }
        }
        if (best_low >= 0) return best_low;
        if (best_idle >= 0) return best_idle;
        return best_due;
    }

    int cap_, n_layers_, n_experts_;
    std::vector<CacheEntry> slots_;
    std::vector<int> map_;
    std::vector<int> per_layer_;
    int64_t clock_ = 0, stamp_ = 0;
    int S_ = 1;
};

}  // namespace ef

// Two-level LRU expert cache policy (host only, no HIP).
//
// Follows the paper's expert memory management (Sec. 3.3.1): a `high` tier for experts used
// within the recent window of layers or predicted to be needed soon, a `low` tier for the rest;
// victims come from `low` first.  Tiers are re-derived whenever the clock or the look-ahead S
// changes.  Readings where the paper is silent: the window is S layers; a prediction keeps an
// entry high until the tick it is due; inside `high`, entries no prediction waits for go first
// (least recently used first), and if every candidate is awaited the one due furthest ahead goes.
//
// One pool shared by all layers (no per-layer cap): a decode loop runs the layers in a cycle, so the least
// recently used entry of the pool belongs to the layer that runs next, and plain recency order evicts exactly
// what is needed soonest (the premature eviction of the first layers' experts that Sec. 3.3.1 names as the
// motivation of the two tiers).  Once the pool is full, a layer that already holds its share of it
// (slots_total / n_layers, at least top_k) replaces entries of its own, like under a per-layer cap: with a pool
// just large enough for top_k experts per layer, a layer that grew at the others' expense would leave them
// below top_k and the misses would cascade from layer to layer.  A layer below its share takes its victim,
// among the candidates of a tier, (1) from the layer that holds the most entries, as long as that is more
// than top_k (a layer needs top_k resident experts before the residency bias can keep its tokens on them),
// (2) then from the layer whose next turn in the cycle is furthest away, (3) then least recently used.
// With a per-layer cap in force all candidates belong to one layer and (3) alone decides, as before.
#pragma once
#include <algorithm>
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
    ExpertCache(int slots_total, int per_layer_cap, int n_layers, int n_experts, int top_k = 1)
        : cap_(per_layer_cap), n_layers_(n_layers), n_experts_(n_experts), top_k_(top_k),
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
    // one layer executed (`layer_run`: which one, -1 = unknown; the next turn is then layer_run + 1, cyclically)
    void advance(int layer_run = -1) {
        ++clock_;
        if (layer_run >= 0) next_layer_ = (layer_run + 1) % n_layers_;
        retier();
    }
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
        if (!layer_full) {
            for (size_t s = 0; s < slots_.size(); ++s)
                if (slots_[s].layer < 0) return (int)s;
            // the pool is full: a layer at its share of it replaces its own entries
            const int share = std::max(top_k_, (int)slots_.size() / n_layers_);
            if (per_layer_[(size_t)layer] >= share) layer_full = true;
        }
        int best_low = -1, best_idle = -1, best_due = -1;
        // true if entry a goes before entry b
        auto before = [&](const CacheEntry &a, const CacheEntry &b) {
            if (!layer_full) {
                const int ca = crowd(a.layer), cb = crowd(b.layer);
                if (ca != cb) return ca > cb;
                const int da = turn_distance(a.layer), db = turn_distance(b.layer);
                if (da != db) return da > db;
            }
            return a.stamp < b.stamp;
        };
        for (size_t s = 0; s < slots_.size(); ++s) {
            const CacheEntry &e = slots_[s];
            if (e.layer < 0 || e.pinned) continue;
            if (layer_full && e.layer != layer) continue;
            if (!e.high) {
                if (best_low < 0 || before(e, slots_[(size_t)best_low])) best_low = (int)s;
            } else if (e.due < clock_) {
                if (best_idle < 0 || before(e, slots_[(size_t)best_idle])) best_idle = (int)s;
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

    // entries the layer holds if that is more than top_k, else 0: layers at or below top_k are robbed last
    int crowd(int layer) const { return per_layer_[(size_t)layer] > top_k_ ? per_layer_[(size_t)layer] : 0; }
    // layers until `layer` runs again, counted from the layer that runs next
    int turn_distance(int layer) const { return (layer - next_layer_ + n_layers_) % n_layers_; }

    int cap_, n_layers_, n_experts_, top_k_;
    int next_layer_ = 0;
    std::vector<CacheEntry> slots_;
    std::vector<int> map_;
    std::vector<int> per_layer_;
    int64_t clock_ = 0, stamp_ = 0;
    int S_ = 1;
};

}  // namespace ef

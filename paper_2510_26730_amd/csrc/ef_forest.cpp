// Deviation predictor (paper Sec. 3.2.2-3.2.5): random-forest regressor over activation logs, the
// prediction cache keyed by (token sequence, layer, step size) and the asynchronous producer that
// fills it.  Host code only: the paper runs this model on the CPU so that it never competes with
// the GPU kernels; here it lives in worker threads of the same library.
//
// Labels are 0/1 vectors, so the squared-error criterion of a split is a ratio of integers:
// minimising the summed squared error of the two sides is maximising
//     sum_m sL[m]^2 / nL + sum_m sR[m]^2 / nR        (sL, sR: per-expert label sums of the sides),
// and the best split is decided by exact integer cross-multiplication (128-bit), never by rounding.
#include <algorithm>
#include <atomic>
#include <condition_variable>
#include <cstdint>
#include <cstring>
#include <deque>
#include <list>
#include <mutex>
#include <new>
#include <thread>
#include <unordered_map>
#include <vector>

#include "../../include/expertflow.h"

#pragma STDC FP_CONTRACT OFF

namespace {

typedef __int128 i128;
constexpr int kMaxSamples = 1 << 20;   // keeps every cross product below 2^127

struct Tree {
    std::vector<int32_t> feature, left, right, count;
    std::vector<double> threshold, value;   // value [nodes, M]
};

struct Split {
    i128 num = 0;       // sum_m sL^2 * nR + sum_m sR^2 * nL
    int64_t den = 0;    // nL * nR
    double thr = 0.0;
    int feature = -1;
};

// a/b > c/d for positive denominators
inline bool frac_greater(i128 a, int64_t b, i128 c, int64_t d) { return a * (i128)d > c * (i128)b; }

struct Grower {
    const float *X;
    int F, M, max_depth, min_leaf;
    // labels in compressed rows: the set bits of sample i are lab[lab_off[i] .. lab_off[i+1])
    const std::vector<int32_t> *lab_off, *lab;
    Tree *tree;
    std::vector<std::pair<float, int32_t>> keyed;   // scratch: (feature value, sample)
    std::vector<int64_t> sl, tot;

    int grow(std::vector<int32_t> &ids, int depth) {
        const int me = (int)tree->feature.size();
        const int64_t n = (int64_t)ids.size();
        tree->feature.push_back(-1);
        tree->left.push_back(-1);
        tree->right.push_back(-1);
        tree->threshold.push_back(0.0);
        tree->count.push_back((int32_t)n);
        std::vector<int64_t> s(M, 0);
        for (int32_t id : ids)
            for (int32_t q = (*lab_off)[id]; q < (*lab_off)[id + 1]; ++q) s[(*lab)[q]] += 1;
        for (int m = 0; m < M; ++m) tree->value.push_back((double)s[m] / (double)n);
        if (depth >= max_depth || n < 2 * (int64_t)min_leaf) return me;

        int64_t q_node = 0;
        for (int m = 0; m < M; ++m) q_node += s[m] * s[m];
        Split best;
        keyed.resize((size_t)n);
        for (int f = 0; f < F; ++f) {
            float lo = X[(size_t)ids[0] * F + f], hi = lo;
            for (int64_t i = 0; i < n; ++i) {
                const float v = X[(size_t)ids[i] * F + f];
                keyed[i] = {v, ids[i]};
                lo = std::min(lo, v);
                hi = std::max(hi, v);
            }
            if (!(lo < hi)) continue;
            std::sort(keyed.begin(), keyed.end());
            std::fill(sl.begin(), sl.end(), 0);
            int64_t ql = 0, qr = q_node;
            for (int64_t i = 1; i < n; ++i) {
                // sample i-1 moves to the left side
                const int32_t id = keyed[i - 1].second;
                for (int32_t q = (*lab_off)[id]; q < (*lab_off)[id + 1]; ++q) {
                    const int m = (*lab)[q];
                    ql += 2 * sl[m] + 1;
                    qr -= 2 * (s[m] - sl[m]) - 1;
                    sl[m] += 1;
                }
                if (keyed[i - 1].first == keyed[i].first) continue;
                const int64_t nl = i, nr = n - i;
                if (nl < min_leaf || nr < min_leaf) continue;
                const i128 num = (i128)ql * nr + (i128)qr * nl;
                const int64_t den = nl * nr;
                if (best.feature < 0 || frac_greater(num, den, best.num, best.den)) {
                    best.num = num;
                    best.den = den;
                    best.feature = f;
                    best.thr = 0.5 * ((double)keyed[i - 1].first + (double)keyed[i].first);
                }
            }
        }
        // split only if it strictly improves on the node itself: best.num / best.den > q_node / n
        if (best.feature < 0 || !frac_greater(best.num, best.den, (i128)q_node, n)) return me;

        std::vector<int32_t> lids, rids;
        for (int32_t id : ids) {
            if ((double)X[(size_t)id * F + best.feature] <= best.thr) lids.push_back(id);
            else rids.push_back(id);
        }
        std::vector<int32_t>().swap(ids);   // the parent's list is no longer needed
        tree->feature[me] = best.feature;
        tree->threshold[me] = best.thr;
        const int l = grow(lids, depth + 1);
        tree->left[me] = l;
        const int r = grow(rids, depth + 1);
        tree->right[me] = r;
        return me;
    }
};

int resolve_threads(int requested, int work_items) {
    int n = requested > 0 ? requested : (int)std::thread::hardware_concurrency();
    if (n < 1) n = 1;
    return std::max(1, std::min(n, work_items));
}

template <typename Fn> void parallel_for(int n_items, int n_threads, Fn fn) {
    if (n_threads <= 1 || n_items <= 1) {
        for (int i = 0; i < n_items; ++i) fn(i);
        return;
    }
    std::atomic<int> next(0);
    std::vector<std::thread> pool;
    for (int t = 0; t < n_threads; ++t)
        pool.emplace_back([&] {
            for (int i = next.fetch_add(1); i < n_items; i = next.fetch_add(1)) fn(i);
        });
    for (auto &th : pool) th.join();
}

void features_into(const float *emb, int d_emb, const int32_t *tok, int n_tok, int S, int layer,
                   const uint8_t *prev_act, int LM, float *x) {
    std::vector<double> acc(d_emb, 0.0);
    for (int i = 0; i < n_tok; ++i) {
        const float *row = emb + (size_t)tok[i] * d_emb;
        for (int j = 0; j < d_emb; ++j) acc[j] = acc[j] + (double)row[j];
    }
    for (int j = 0; j < d_emb; ++j) x[j] = (float)(acc[j] / (double)n_tok);
    x[d_emb] = (float)S;
    x[d_emb + 1] = (float)layer;
    for (int i = 0; i < LM; ++i) x[d_emb + 2 + i] = prev_act ? (float)(prev_act[i] != 0) : 0.f;
}

void centre_row(const double *y, int M, float gain, float *out) {
    double mean = 0.0;
    for (int e = 0; e < M; ++e) mean = mean + y[e];
    mean = mean / (double)M;
    for (int e = 0; e < M; ++e) out[e] = (float)((double)gain * (y[e] - mean));
}

}  // namespace

struct ef_forest {
    ef_forest_config cfg;
    std::vector<Tree> trees;
    bool fitted = false;
};

static void forest_predict_row(const ef_forest *f, const float *x, double *out) {
    const int M = f->cfg.n_outputs;
    for (int m = 0; m < M; ++m) out[m] = 0.0;
    for (const Tree &t : f->trees) {
        int nd = 0;
        while (t.feature[nd] >= 0) nd = (double)x[t.feature[nd]] <= t.threshold[nd] ? t.left[nd] : t.right[nd];
        const double *v = &t.value[(size_t)nd * M];
        for (int m = 0; m < M; ++m) out[m] = out[m] + v[m];
    }
    const double nt = (double)f->trees.size();
    for (int m = 0; m < M; ++m) out[m] = out[m] / nt;
}

extern "C" {

int ef_forest_create(const ef_forest_config *cfg, ef_forest **out) {
    if (!cfg || !out) return EF_EINVAL;
    if (cfg->n_features < 1 || cfg->n_outputs < 1 || cfg->n_outputs > EF_MAX_EXPERTS || cfg->n_trees < 1 ||
        cfg->max_depth < 1 || cfg->max_depth > 30 || cfg->min_samples_leaf < 1 || cfg->n_threads < 0)
        return EF_EINVAL;
    ef_forest *f = new (std::nothrow) ef_forest;
    if (!f) return EF_ENOMEM;
    f->cfg = *cfg;
    *out = f;
    return EF_OK;
}

int ef_forest_destroy(ef_forest *f) {
    delete f;
    return EF_OK;
}

int ef_delta_features(const float *emb_table, int V, int d_emb, const int32_t *token_ids, int n_tok, int S,
                      int layer, const uint8_t *prev_act, int L, int M, float *x) {
    if (!emb_table || !token_ids || !prev_act || !x || V < 1 || d_emb < 1 || n_tok < 1 || L < 1 || M < 1 ||
        layer < 0 || layer >= L)
        return EF_EINVAL;
    for (int i = 0; i < n_tok; ++i)
        if (token_ids[i] < 0 || token_ids[i] >= V) return EF_EINVAL;
    features_into(emb_table, d_emb, token_ids, n_tok, S, layer, prev_act, L * M, x);
    return EF_OK;
}

int ef_forest_fit(ef_forest *f, const float *X, const uint8_t *Y, int N, const int32_t *bootstrap) {
    if (!f || !X || !Y || N < 1 || N > kMaxSamples) return EF_EINVAL;
    const int F = f->cfg.n_features, M = f->cfg.n_outputs, nt = f->cfg.n_trees;
    if (bootstrap)
        for (size_t i = 0; i < (size_t)nt * N; ++i)
            if (bootstrap[i] < 0 || bootstrap[i] >= N) return EF_EINVAL;
    for (size_t i = 0; i < (size_t)N * F; ++i)
        if (!(X[i] - X[i] == 0.f)) return EF_EINVAL;   // NaN or infinity: feature values must order
    try {
        std::vector<int32_t> lab_off(N + 1, 0), lab;
        for (int i = 0; i < N; ++i) {
            for (int m = 0; m < M; ++m)
                if (Y[(size_t)i * M + m]) lab.push_back(m);
            lab_off[i + 1] = (int32_t)lab.size();
        }
        std::vector<Tree> trees(nt);
        std::atomic<bool> failed(false);
        parallel_for(nt, resolve_threads(f->cfg.n_threads, nt), [&](int t) {
            try {
                Grower g;
                g.X = X;
                g.F = F;
                g.M = M;
                g.max_depth = f->cfg.max_depth;
                g.min_leaf = f->cfg.min_samples_leaf;
                g.lab_off = &lab_off;
                g.lab = &lab;
                g.tree = &trees[t];
                g.sl.assign(M, 0);
                std::vector<int32_t> ids(N);
                for (int i = 0; i < N; ++i) ids[i] = bootstrap ? bootstrap[(size_t)t * N + i] : i;
                g.grow(ids, 0);
            } catch (...) {
                failed = true;
            }
        });
        if (failed) return EF_ENOMEM;
        f->trees.swap(trees);
        f->fitted = true;
    } catch (const std::bad_alloc &) {
        return EF_ENOMEM;
    }
    return EF_OK;
}

int ef_forest_predict(const ef_forest *f, const float *X, int n, double *Y_hat) {
    if (!f || !X || !Y_hat || n < 0 || !f->fitted) return EF_EINVAL;
    const int F = f->cfg.n_features, M = f->cfg.n_outputs;
    const int chunk = 256, n_chunks = (n + chunk - 1) / chunk;
    parallel_for(n_chunks, resolve_threads(f->cfg.n_threads, n_chunks), [&](int c) {
        const int hi = std::min(n, (c + 1) * chunk);
        for (int i = c * chunk; i < hi; ++i) forest_predict_row(f, X + (size_t)i * F, Y_hat + (size_t)i * M);
    });
    return EF_OK;
}

int ef_forest_tree_size(const ef_forest *f, int t) {
    if (!f || !f->fitted || t < 0 || t >= (int)f->trees.size()) return EF_EINVAL;
    return (int)f->trees[t].feature.size();
}

int ef_forest_tree_export(const ef_forest *f, int t, int32_t *feature, double *threshold, int32_t *left,
                          int32_t *right, int32_t *count, double *value) {
    if (!f || !f->fitted || t < 0 || t >= (int)f->trees.size()) return EF_EINVAL;
    const Tree &tr = f->trees[t];
    const size_t n = tr.feature.size();
    if (feature) std::memcpy(feature, tr.feature.data(), n * sizeof(int32_t));
    if (threshold) std::memcpy(threshold, tr.threshold.data(), n * sizeof(double));
    if (left) std::memcpy(left, tr.left.data(), n * sizeof(int32_t));
    if (right) std::memcpy(right, tr.right.data(), n * sizeof(int32_t));
    if (count) std::memcpy(count, tr.count.data(), n * sizeof(int32_t));
    if (value) std::memcpy(value, tr.value.data(), tr.value.size() * sizeof(double));
    return EF_OK;
}

int ef_forest_bit_accuracy(const double *Y_hat, const uint8_t *Y, int n, int M, double *accuracy) {
    if (!Y_hat || !Y || !accuracy || n < 1 || M < 1) return EF_EINVAL;
    long long good = 0;
    for (size_t i = 0; i < (size_t)n * M; ++i) good += ((Y_hat[i] >= 0.5) == (Y[i] != 0));
    *accuracy = (double)good / ((double)n * (double)M);
    return EF_OK;
}

int ef_delta_from_activation(const double *Y_hat, int n_rows, int M, float gain, float *delta) {
    if (!Y_hat || !delta || n_rows < 0 || M < 1) return EF_EINVAL;
    for (int r = 0; r < n_rows; ++r) centre_row(Y_hat + (size_t)r * M, M, gain, delta + (size_t)r * M);
    return EF_OK;
}

}  // extern "C"

// ------------------------------------------------------------------------------------------------
// prediction cache
// ------------------------------------------------------------------------------------------------
namespace {

struct Key {
    std::vector<int32_t> tokens;
    int layer, S;
    bool operator==(const Key &o) const { return layer == o.layer && S == o.S && tokens == o.tokens; }
};

struct KeyHash {
    size_t operator()(const Key &k) const {
        uint64_t h = 1469598103934665603ull;   // FNV-1a over the words of the key
        auto mix = [&](uint32_t w) {
            for (int b = 0; b < 4; ++b) {
                h ^= (w >> (8 * b)) & 0xFF;
                h *= 1099511628211ull;
            }
        };
        mix((uint32_t)k.layer);
        mix((uint32_t)k.S);
        for (int32_t t : k.tokens) mix((uint32_t)t);
        return (size_t)h;
    }
};

struct Entry {
    Key key;
    std::vector<double> y;
};

}  // namespace

struct ef_delta_cache {
    int capacity, M;
    std::mutex mu;
    std::list<Entry> lru;   // front = most recently used
    std::unordered_map<Key, std::list<Entry>::iterator, KeyHash> index;
    long long hits = 0, misses = 0;

    bool contains(const Key &k) {
        std::lock_guard<std::mutex> g(mu);
        return index.count(k) != 0;
    }
    void put(Key &&k, const double *y) {
        std::lock_guard<std::mutex> g(mu);
        auto it = index.find(k);
        if (it != index.end()) {
            it->second->y.assign(y, y + M);
            lru.splice(lru.begin(), lru, it->second);
            return;
        }
        lru.push_front(Entry{std::move(k), std::vector<double>(y, y + M)});
        index[lru.front().key] = lru.begin();
        while ((int)lru.size() > capacity) {
            index.erase(lru.back().key);
            lru.pop_back();
        }
    }
    bool get(const Key &k, double *y) {
        std::lock_guard<std::mutex> g(mu);
        auto it = index.find(k);
        if (it == index.end()) {
            ++misses;
            return false;
        }
        ++hits;
        lru.splice(lru.begin(), lru, it->second);
        std::memcpy(y, it->second->y.data(), (size_t)M * sizeof(double));
        return true;
    }
};

// ------------------------------------------------------------------------------------------------
// asynchronous producer
// ------------------------------------------------------------------------------------------------
namespace {

struct Job {
    Key key;
    std::vector<uint8_t> prev_act;
};

}  // namespace

struct ef_delta_producer {
    const ef_forest *forest;
    ef_delta_cache *cache;
    const float *emb;
    int V, d_emb, L, M;
    std::mutex mu;
    std::condition_variable wake, idle;
    std::deque<Job> queue;
    int active = 0;
    bool stop = false;
    std::vector<std::thread> workers;

    void run() {
        std::vector<float> x((size_t)d_emb + 2 + (size_t)L * M);
        std::vector<double> y(M);
        for (;;) {
            Job job;
            {
                std::unique_lock<std::mutex> lk(mu);
                wake.wait(lk, [&] { return stop || !queue.empty(); });
                if (queue.empty()) return;   // stop requested and nothing left to do
                job = std::move(queue.front());
                queue.pop_front();
                ++active;
            }
            // only what is known when this layer is predicted S layers ahead: the rows of layers < layer - S
            const int known = std::max(0, std::min(L, job.key.layer - job.key.S));
            std::fill(job.prev_act.begin() + (size_t)known * M, job.prev_act.end(), (uint8_t)0);
            features_into(emb, d_emb, job.key.tokens.data(), (int)job.key.tokens.size(), job.key.S, job.key.layer,
                          job.prev_act.data(), L * M, x.data());
            forest_predict_row(forest, x.data(), y.data());
            cache->put(std::move(job.key), y.data());
            {
                std::lock_guard<std::mutex> lk(mu);
                --active;
                if (queue.empty() && active == 0) idle.notify_all();
            }
        }
    }
};

extern "C" {

int ef_delta_cache_create(int capacity, int M, ef_delta_cache **out) {
    if (!out || capacity < 1 || M < 1 || M > EF_MAX_EXPERTS) return EF_EINVAL;
    ef_delta_cache *c = new (std::nothrow) ef_delta_cache;
    if (!c) return EF_ENOMEM;
    c->capacity = capacity;
    c->M = M;
    *out = c;
    return EF_OK;
}

int ef_delta_cache_destroy(ef_delta_cache *c) {
    delete c;
    return EF_OK;
}

int ef_delta_cache_put(ef_delta_cache *c, const int32_t *token_ids, int n_tok, int layer, int S, const double *y_hat) {
    if (!c || !token_ids || !y_hat || n_tok < 1) return EF_EINVAL;
    try {
        c->put(Key{std::vector<int32_t>(token_ids, token_ids + n_tok), layer, S}, y_hat);
    } catch (const std::bad_alloc &) {
        return EF_ENOMEM;
    }
    return EF_OK;
}

int ef_delta_cache_get(ef_delta_cache *c, const int32_t *token_ids, int n_tok, int layer, int S, double *y_hat) {
    if (!c || !token_ids || !y_hat || n_tok < 1) return EF_EINVAL;
    try {
        return c->get(Key{std::vector<int32_t>(token_ids, token_ids + n_tok), layer, S}, y_hat) ? 1 : 0;
    } catch (const std::bad_alloc &) {
        return EF_ENOMEM;
    }
}

int ef_delta_cache_counts(ef_delta_cache *c, long long *hits, long long *misses, long long *entries) {
    if (!c) return EF_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    if (hits) *hits = c->hits;
    if (misses) *misses = c->misses;
    if (entries) *entries = (long long)c->lru.size();
    return EF_OK;
}

int ef_delta_producer_create(const ef_forest *f, ef_delta_cache *cache, const float *emb_table, int V, int d_emb,
                             int L, int M, int n_threads, ef_delta_producer **out) {
    if (!f || !cache || !emb_table || !out || !f->fitted || V < 1 || d_emb < 1 || L < 1 || M < 1 || n_threads < 0)
        return EF_EINVAL;
    if (f->cfg.n_features != d_emb + 2 + L * M || f->cfg.n_outputs != M || cache->M != M) return EF_EINVAL;
    ef_delta_producer *p = new (std::nothrow) ef_delta_producer;
    if (!p) return EF_ENOMEM;
    p->forest = f;
    p->cache = cache;
    p->emb = emb_table;
    p->V = V;
    p->d_emb = d_emb;
    p->L = L;
    p->M = M;
    const int nt = resolve_threads(n_threads, 1 << 16);
    try {
        for (int i = 0; i < nt; ++i) p->workers.emplace_back([p] { p->run(); });
    } catch (...) {
        ef_delta_producer_destroy(p);
        return EF_ENOMEM;
    }
    *out = p;
    return EF_OK;
}

int ef_delta_producer_destroy(ef_delta_producer *p) {
    if (!p) return EF_OK;
    {
        std::lock_guard<std::mutex> lk(p->mu);
        p->stop = true;
    }
    p->wake.notify_all();
    for (auto &w : p->workers) w.join();   // workers finish what is queued, then leave
    delete p;
    return EF_OK;
}

int ef_delta_submit(ef_delta_producer *p, const int32_t *token_ids, int n_tok, int S, int layer_first, int n_layers,
                    const uint8_t *prev_act) {
    if (!p || !token_ids || !prev_act || n_tok < 1 || layer_first < 0 || n_layers < 0) return EF_EINVAL;
    for (int i = 0; i < n_tok; ++i)
        if (token_ids[i] < 0 || token_ids[i] >= p->V) return EF_EINVAL;
    try {
        int queued = 0;
        for (int l = layer_first; l < layer_first + n_layers && l < p->L; ++l) {
            Key k{std::vector<int32_t>(token_ids, token_ids + n_tok), l, S};
            if (p->cache->contains(k)) continue;
            Job job{std::move(k), std::vector<uint8_t>(prev_act, prev_act + (size_t)p->L * p->M)};
            {
                std::lock_guard<std::mutex> lk(p->mu);
                p->queue.push_back(std::move(job));
            }
            ++queued;
        }
        if (queued == 1) p->wake.notify_one();
        else if (queued > 1) p->wake.notify_all();
    } catch (const std::bad_alloc &) {
        return EF_ENOMEM;
    }
    return EF_OK;
}

int ef_delta_drain(ef_delta_producer *p) {
    if (!p) return EF_EINVAL;
    std::unique_lock<std::mutex> lk(p->mu);
    p->idle.wait(lk, [&] { return p->queue.empty() && p->active == 0; });
    return EF_OK;
}

int ef_delta_assemble(ef_delta_cache *c, const int32_t *token_ids, const int32_t *tok_off, int R, int layer, int S,
                      int H, int L, float gain, float *delta, int *n_hits) {
    if (!c || !token_ids || !tok_off || !delta || R < 1 || H < 1 || L < 1 || layer < 0) return EF_EINVAL;
    for (int r = 0; r < R; ++r)
        if (tok_off[r + 1] <= tok_off[r] || tok_off[r] < 0) return EF_EINVAL;
    const int M = c->M;
    int hits = 0;
    std::vector<double> y(M);
    try {
        for (int r = 0; r < R; ++r) {
            Key k{std::vector<int32_t>(token_ids + tok_off[r], token_ids + tok_off[r + 1]), 0, S};
            for (int j = 0; j < H; ++j) {
                float *row = delta + ((size_t)r * H + j) * M;
                k.layer = layer + 1 + j;
                if (k.layer < L && c->get(k, y.data())) {
                    centre_row(y.data(), M, gain, row);
                    ++hits;
                } else {
                    for (int e = 0; e < M; ++e) row[e] = 0.f;
                }
            }
        }
    } catch (const std::bad_alloc &) {
        return EF_ENOMEM;
    }
    if (n_hits) *n_hits = hits;
    return EF_OK;
}

}  // extern "C"

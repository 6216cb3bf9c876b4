// Slab-based dynamic expert cache with a transfer stream and a compute stream (paper Sec. 3.4.2: fixed-size slabs,
// lookahead-driven insertion, safety-guarded eviction; Sec. 3.4.3: two streams, a miss stalls only on its expert).
// Host-side logic in C++; the device work it issues is asynchronous copies and event waits, no kernels.
//
// Policy. A resident expert (layer, expert) is Required (listed by the latest prediction or demanded, its layer not
// yet executed in this pass), Speculative (was Required, dropped by a newer prediction, its layer not yet executed)
// or Expired (its layer has executed). Only Expired experts are evicted, lowest predictor priority first, ties to
// the lowest (layer, expert). Free slabs are taken lowest index first.
//
// Ordering on the device. Every slab has a "ready" event recorded on the transfer stream behind the copy that fills
// it; the compute stream waits on the ready events of the experts a layer needs, and on nothing else. Every layer has
// a "done" event recorded on the compute stream when the layer has been enqueued; before a slab is overwritten the
// transfer stream waits on the done event of the layer its previous tenant belonged to, so a copy can never land in
// a slab that an earlier kernel is still reading.
#include <math.h>

#include <algorithm>
#include <map>
#include <new>
#include <utility>
#include <vector>

#include "common.h"

namespace {

enum : int { kRequired = 0, kSpeculative = 1, kExpired = 2 };
typedef std::pair<int, int> Key;      // (layer, expert)

struct Entry {
    int slab;
    int cls;
    float prio;
};

}  // namespace

struct moe_expert_cache {
    int n_layers, E, n_slabs;
    size_t slab_bytes;
    char* pool;
    std::map<Key, Entry> where;            // ordered: ties in victim selection go to the lowest (layer, expert)
    std::vector<int> free_slabs;           // kept sorted descending: back() is the lowest index
    std::vector<hipEvent_t> ready;         // per slab
    std::vector<hipEvent_t> done;          // per layer
    std::vector<int> last_layer;           // per slab: layer of the tenant whose readers may still be running, or -1
    std::vector<char> done_recorded;       // per layer: a done event has been recorded at least once
    long long stats[6];                    // hits, misses, prefetches, evictions, refused, bytes copied
};

namespace {

// A slab for `key`: a free one, else the slab of the Expired expert of lowest priority. -1 when there is none.
int take_slab(moe_expert_cache* c, const Key& key, int* victim_layer, int* victim_expert) {
    *victim_layer = *victim_expert = -1;
    int slab;
    if (!c->free_slabs.empty()) {
        slab = c->free_slabs.back();
        c->free_slabs.pop_back();
    } else {
        auto best = c->where.end();
        for (auto it = c->where.begin(); it != c->where.end(); ++it)
            if (it->second.cls == kExpired && (best == c->where.end() || it->second.prio < best->second.prio)) best = it;
        if (best == c->where.end()) return -1;
        slab = best->second.slab;
        *victim_layer = best->first.first;
        *victim_expert = best->first.second;
        c->where.erase(best);
        ++c->stats[3];
    }
    (void)key;
    return slab;
}

// Starts the copy of one expert into `slab` on the transfer stream.
hipError_t start_copy(moe_expert_cache* c, int slab, const void* host_src, int layer, hipStream_t trans) {
    hipError_t e;
    const int prev = c->last_layer[slab];
    if (prev >= 0 && c->done_recorded[prev]) {
        // the previous tenant's layer may still be executing: the copy must not overtake its readers
        if ((e = hipStreamWaitEvent(trans, c->done[prev], 0)) != hipSuccess) return e;
    }
    if ((e = hipMemcpyAsync(c->pool + (size_t)slab * c->slab_bytes, host_src, c->slab_bytes, hipMemcpyHostToDevice,
                            trans)) != hipSuccess)
        return e;
    if ((e = hipEventRecord(c->ready[slab], trans)) != hipSuccess) return e;
    c->last_layer[slab] = layer;
    c->stats[5] += (long long)c->slab_bytes;
    return hipSuccess;
}

bool bad_key(const moe_expert_cache* c, int layer, int expert) {
    return layer < 0 || layer >= c->n_layers || expert < 0 || expert >= c->E;
}

}  // namespace

extern "C" {

moe_status moe_cache_create(int32_t n_layers, int32_t E, size_t slab_bytes, int32_t n_slabs, void* device_pool,
                            moe_expert_cache** out) {
    if (!out) return MOE_ERR_NULL;
    *out = nullptr;
    if (n_layers < 1 || E < 1 || n_slabs < 1 || slab_bytes == 0 || slab_bytes % 16 != 0) return MOE_ERR_SHAPE;
    if (!device_pool) return MOE_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(device_pool) & 255u) return MOE_ERR_ALIGN;
    moe_expert_cache* c = new (std::nothrow) moe_expert_cache();
    if (!c) return MOE_ERR_HIP;
    c->n_layers = n_layers;
    c->E = E;
    c->n_slabs = n_slabs;
    c->slab_bytes = slab_bytes;
    c->pool = static_cast<char*>(device_pool);
    for (int s = n_slabs - 1; s >= 0; --s) c->free_slabs.push_back(s);
    c->last_layer.assign(n_slabs, -1);
    c->done_recorded.assign(n_layers, 0);
    for (int i = 0; i < 6; ++i) c->stats[i] = 0;
    bool ok = true;
    for (int s = 0; s < n_slabs && ok; ++s) {
        hipEvent_t ev;
        ok = hipEventCreateWithFlags(&ev, hipEventDisableTiming) == hipSuccess;
        if (ok) c->ready.push_back(ev);
    }
    for (int l = 0; l < n_layers && ok; ++l) {
        hipEvent_t ev;
        ok = hipEventCreateWithFlags(&ev, hipEventDisableTiming) == hipSuccess;
        if (ok) c->done.push_back(ev);
    }
    if (!ok) {
        for (hipEvent_t ev : c->ready) (void)hipEventDestroy(ev);
        for (hipEvent_t ev : c->done) (void)hipEventDestroy(ev);
        delete c;
        return MOE_ERR_HIP;
    }
    *out = c;
    return MOE_OK;
}

void moe_cache_destroy(moe_expert_cache* c) {
    if (!c) return;
    for (hipEvent_t ev : c->ready) (void)hipEventDestroy(ev);
    for (hipEvent_t ev : c->done) (void)hipEventDestroy(ev);
    delete c;
}

moe_status moe_cache_predict(moe_expert_cache* c, const int32_t* layers, const int32_t* experts, const float* priorities,
                             int32_t n, const void* const* host_src, void* trans_stream, int32_t* started_out,
                             int32_t* n_started) {
    if (!c || !n_started) return MOE_ERR_NULL;
    *n_started = 0;
    if (n < 0) return MOE_ERR_SHAPE;
    if (n > 0 && (!layers || !experts || !priorities || !host_src)) return MOE_ERR_NULL;
    std::map<Key, int> listed;
    for (int i = 0; i < n; ++i) {
        if (bad_key(c, layers[i], experts[i]) || !host_src[i] || isnan(priorities[i])) return MOE_ERR_SHAPE;
        if (!listed.emplace(Key(layers[i], experts[i]), i).second) return MOE_ERR_SHAPE;      // listed twice
    }
    for (auto& kv : c->where)
        if (kv.second.cls == kRequired && !listed.count(kv.first)) kv.second.cls = kSpeculative;
    for (auto& kv : listed) {            // residents first: what is listed cannot be evicted below
        auto it = c->where.find(kv.first);
        if (it != c->where.end()) {
            it->second.cls = kRequired;
            it->second.prio = priorities[kv.second];
        }
    }
    std::vector<int> order(n);
    for (int i = 0; i < n; ++i) order[i] = i;
    std::sort(order.begin(), order.end(), [&](int a, int b) {
        if (priorities[a] != priorities[b]) return priorities[a] > priorities[b];
        return Key(layers[a], experts[a]) < Key(layers[b], experts[b]);
    });
    hipStream_t trans = (hipStream_t)trans_stream;
    for (int i : order) {
        const Key key(layers[i], experts[i]);
        if (c->where.count(key)) continue;
        int vl, ve;
        const int slab = take_slab(c, key, &vl, &ve);
        if (slab < 0) {
            ++c->stats[4];
            continue;
        }
        if (start_copy(c, slab, host_src[i], key.first, trans) != hipSuccess) return MOE_ERR_HIP;
        c->where[key] = Entry{slab, kRequired, priorities[i]};
        ++c->stats[2];
        if (started_out) {
            started_out[2 * *n_started] = key.first;
            started_out[2 * *n_started + 1] = key.second;
        }
        ++*n_started;
    }
    return MOE_OK;
}

moe_status moe_cache_acquire(moe_expert_cache* c, int32_t layer, const int32_t* needed, int32_t n,
                             const void* const* host_src, void* trans_stream, void* comp_stream, const void** table_out,
                             int32_t* missed_out, int32_t* n_missed) {
    if (!c || !table_out || !n_missed) return MOE_ERR_NULL;
    *n_missed = 0;
    if (n < 0 || layer < 0 || layer >= c->n_layers) return MOE_ERR_SHAPE;
    if (n > 0 && (!needed || !host_src)) return MOE_ERR_NULL;
    std::map<int, int> want;             // expert -> index of its first mention, ascending experts
    for (int i = 0; i < n; ++i) {
        if (bad_key(c, layer, needed[i]) || !host_src[i]) return MOE_ERR_SHAPE;
        want.emplace(needed[i], i);
    }
    for (auto& kv : want) {              // hits first: they cannot be evicted by this call's misses
        auto it = c->where.find(Key(layer, kv.first));
        if (it != c->where.end()) {
            it->second.cls = kRequired;
            ++c->stats[0];
        }
    }
    hipStream_t trans = (hipStream_t)trans_stream, comp = (hipStream_t)comp_stream;
    for (auto& kv : want) {
        const Key key(layer, kv.first);
        if (c->where.count(key)) continue;
        ++c->stats[1];
        int vl, ve;
        const int slab = take_slab(c, key, &vl, &ve);
        if (slab < 0) return MOE_ERR_CACHE_FULL;     // the cache is too small for what is protected plus this layer
        if (start_copy(c, slab, host_src[kv.second], layer, trans) != hipSuccess) return MOE_ERR_HIP;
        c->where[key] = Entry{slab, kRequired, 0.f};      // no prediction scored it
        if (missed_out) missed_out[*n_missed] = kv.first;
        ++*n_missed;
    }
    // the slab table of this layer; the compute stream waits for exactly the experts it is about to read
    for (int e = 0; e < c->E; ++e) table_out[e] = nullptr;
    for (auto& kv : want) {
        const Entry& en = c->where[Key(layer, kv.first)];
        table_out[kv.first] = c->pool + (size_t)en.slab * c->slab_bytes;
        if (hipStreamWaitEvent(comp, c->ready[en.slab], 0) != hipSuccess) return MOE_ERR_HIP;
    }
    return MOE_OK;
}

moe_status moe_cache_layer_done(moe_expert_cache* c, int32_t layer, void* comp_stream) {
    if (!c) return MOE_ERR_NULL;
    if (layer < 0 || layer >= c->n_layers) return MOE_ERR_SHAPE;
    if (hipEventRecord(c->done[layer], (hipStream_t)comp_stream) != hipSuccess) return MOE_ERR_HIP;
    c->done_recorded[layer] = 1;
    for (auto& kv : c->where)
        if (kv.first.first == layer) kv.second.cls = kExpired;
    return MOE_OK;
}

moe_status moe_cache_query(const moe_expert_cache* c, int32_t layer, int32_t expert, int32_t* slab, int32_t* cls,
                           float* priority) {
    if (!c || !slab || !cls || !priority) return MOE_ERR_NULL;
    if (bad_key(c, layer, expert)) return MOE_ERR_SHAPE;
    auto it = c->where.find(Key(layer, expert));
    if (it == c->where.end()) {
        *slab = -1;
        *cls = -1;
        *priority = 0.f;
    } else {
        *slab = it->second.slab;
        *cls = it->second.cls;
        *priority = it->second.prio;
    }
    return MOE_OK;
}

moe_status moe_cache_stats(const moe_expert_cache* c, int64_t* out6) {
    if (!c || !out6) return MOE_ERR_NULL;
    for (int i = 0; i < 6; ++i) out6[i] = c->stats[i];
    return MOE_OK;
}

}  // extern "C"

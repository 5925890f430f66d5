// Chunked Hash Tree: the scheduler-side structure that decides which waiting
// requests join the running batch (Section 4.2; appendix "Algorithms": Insert,
// FindBest, AddToBatch, Finish, Remove, BuildBatch).  Host code only.
//
// Requests are cumulative chunk-hash vectors.  Kept incrementally, as the paper
// describes: reference counts of (level, hash) nodes over the active requests
// (a node is in the working set while its count is positive), a reverse index
// node -> waiting requests that carry it, the missing count of every waiting
// request, a min-heap of (missing count, request id) with lazy deletion, the
// shared prefix tip, and the cached result of FindBest.
//
// Where the paper's text and its listings disagree, the text wins: the first
// request of a batch enters the working set like any other; the tip after an
// addition is the deepest level at which the newcomer agrees with the old tip
// (tested against the working set as it was before the newcomer's own nodes
// went in); Finish always drops the request from the auxiliary structures.
#include <algorithm>
#include <cstdint>
#include <functional>
#include <queue>
#include <unordered_map>
#include <utility>
#include <vector>

#include "../../include/fea.h"
#include "fea_internal.h"

namespace {

struct Node {
    int32_t level;
    uint64_t hash;
    bool operator==(const Node& o) const { return level == o.level && hash == o.hash; }
};
struct NodeHash {
    size_t operator()(const Node& n) const {
        uint64_t x = n.hash + 0x9E3779B97F4A7C15ull * (uint64_t)(uint32_t)n.level;
        x ^= x >> 32;
        return (size_t)x;
    }
};

struct Request {
    std::vector<uint64_t> H;
    int32_t miss = 0;
    bool active = false;
};

using HeapEntry = std::pair<int32_t, int64_t>;   // (missing count, request id): ties go to the smaller id

}  // namespace

struct fea_cht {
    int32_t K = FEA_BLOCK_TOKENS;
    std::unordered_map<int64_t, Request> req;
    std::unordered_map<Node, int32_t, NodeHash> ref;                    // active requests through a node
    std::unordered_map<Node, std::vector<int64_t>, NodeHash> waiting;   // waiting requests through a node
    std::priority_queue<HeapEntry, std::vector<HeapEntry>, std::greater<HeapEntry>> heap;
    std::vector<int64_t> active;
    int64_t n_waiting = 0;
    int32_t tip_level = 0;
    uint64_t tip_hash = 0;
    int32_t hash_kind = FEA_HASH_CHAINED;
    uint64_t hash_seed = 0;
    bool cache_valid = false;
    bool cache_found = false;
    int64_t c_id = 0;
    int32_t c_before = 0, c_after = 0, c_peers = 0, c_miss = 0;

    int32_t refs(const Node& n) const {
        auto it = ref.find(n);
        return it == ref.end() ? 0 : it->second;
    }
    void unindex(int64_t id, const Request& r) {   // take a request out of the reverse index
        for (size_t l = 0; l < r.H.size(); ++l) {
            auto it = waiting.find(Node{(int32_t)l + 1, r.H[l]});
            if (it == waiting.end()) continue;
            auto& v = it->second;
            auto pos = std::find(v.begin(), v.end(), id);
            if (pos != v.end()) { *pos = v.back(); v.pop_back(); }
            if (v.empty()) waiting.erase(it);
        }
    }
    void bump(const Node& n, int32_t delta) {      // a node entered (-1) or left (+1) the working set
        auto it = waiting.find(n);
        if (it == waiting.end()) return;
        for (int64_t w : it->second) {
            Request& r = req[w];
            r.miss += delta;
            heap.emplace(r.miss, w);
        }
    }
};

using fea::fail;

extern "C" {

int32_t fea_cht_create(int32_t chunk_tokens, fea_cht** out) {
    if (!out) return fail(FEA_EINVAL, "fea_cht_create: out is NULL");
    if (chunk_tokens <= 0) return fail(FEA_EINVAL, "fea_cht_create: chunk_tokens=%d must be positive", chunk_tokens);
    if (chunk_tokens != FEA_BLOCK_TOKENS)
        return fail(FEA_EINVAL, "fea_cht_create: chunk_tokens=%d, the hash vectors of this library use %d", chunk_tokens, FEA_BLOCK_TOKENS);
    fea_cht* t = new (std::nothrow) fea_cht();
    if (!t) return fail(FEA_ENOMEM, "fea_cht_create: out of host memory");
    t->K = chunk_tokens;
    *out = t;
    return FEA_OK;
}

void fea_cht_destroy(fea_cht* t) { delete t; }

int32_t fea_cht_set_hash(fea_cht* t, int32_t kind, uint64_t seed) {
    return fea::guarded("fea_cht_set_hash", [&]() -> int32_t {
        if (!t) return fail(FEA_EINVAL, "fea_cht_set_hash: tree is NULL");
        if (kind != FEA_HASH_CHAINED && kind != FEA_HASH_XXH64) return fail(FEA_EINVAL, "fea_cht_set_hash: unknown kind %d", kind);
        if (!t->req.empty()) return fail(FEA_EINVAL, "fea_cht_set_hash: requests are present; set the hash on an empty tree");
        t->hash_kind = kind;
        t->hash_seed = seed;
        return FEA_OK;
    });
}

int32_t fea_cht_insert_hashes(fea_cht* t, int64_t id, const uint64_t* hashes, int32_t n) {
    return fea::guarded("fea_cht_insert_hashes", [&]() -> int32_t {
        if (!t || (n > 0 && !hashes) || n < 0) return fail(FEA_EINVAL, "fea_cht_insert: bad argument");
        if (t->req.count(id)) return fail(FEA_EINVAL, "fea_cht_insert: request %lld is already present", (long long)id);
        Request r;
        r.H.assign(hashes, hashes + n);
        for (int32_t l = 0; l < n; ++l) {
            const Node nd{l + 1, r.H[l]};
            if (t->refs(nd) == 0) ++r.miss;
            t->waiting[nd].push_back(id);
        }
        t->heap.emplace(r.miss, id);
        t->req.emplace(id, std::move(r));
        ++t->n_waiting;
        t->cache_valid = false;
        return FEA_OK;
    });
}

int32_t fea_cht_insert(fea_cht* t, int64_t id, const int32_t* tokens, int64_t n_tokens) {
    return fea::guarded("fea_cht_insert", [&]() -> int32_t {
        if (!t || n_tokens < 0 || (n_tokens > 0 && !tokens)) return fail(FEA_EINVAL, "fea_cht_insert: bad argument");
        if (n_tokens > (int64_t)0x7FFFFFFF * t->K) return fail(FEA_EINVAL, "fea_cht_insert: sequence too long");
        std::vector<uint64_t> H((size_t)((n_tokens + t->K - 1) / t->K));
        const int32_t rc = t->hash_kind == FEA_HASH_XXH64 ? fea_chunk_hashes_xxh64(tokens, n_tokens, t->hash_seed, H.data())
                                                          : fea_chunk_hashes(tokens, n_tokens, H.data());
        if (rc != FEA_OK) return rc;
        return fea_cht_insert_hashes(t, id, H.data(), (int32_t)H.size());
    });
}

int32_t fea_cht_find_best(fea_cht* t, int64_t* id, int32_t* tip_before, int32_t* tip_after, int32_t* peers, int32_t* missing) {
    return fea::guarded("fea_cht_find_best", [&]() -> int32_t {
        if (!t || !id) return fail(FEA_EINVAL, "fea_cht_find_best: NULL argument");
        if (!t->cache_valid) {
            t->cache_found = false;
            while (t->n_waiting > 0 && !t->heap.empty()) {
                const HeapEntry e = t->heap.top();
                auto it = t->req.find(e.second);
                if (it == t->req.end() || it->second.active || it->second.miss != e.first) {   // stale
                    t->heap.pop();
                    continue;
                }
                const Request& r = it->second;   // the entry stays in the heap for later calls
                int32_t after = 0;
                for (int32_t l = std::min<int32_t>(t->tip_level, (int32_t)r.H.size()); l >= 1; --l)
                    if (t->refs(Node{l, r.H[l - 1]}) > 0) { after = l; break; }
                int32_t p = (int32_t)std::min<int64_t>(t->n_waiting, 0x7FFFFFFF);
                if (after > 0) {
                    auto w = t->waiting.find(Node{after, r.H[after - 1]});
                    p = w == t->waiting.end() ? 0 : (int32_t)w->second.size();
                }
                t->cache_found = true;
                t->c_id = e.second;
                t->c_before = t->tip_level;
                t->c_after = after;
                t->c_peers = p;
                t->c_miss = r.miss;
                break;
            }
            t->cache_valid = true;
        }
        if (!t->cache_found) return 1;   // nothing is waiting
        *id = t->c_id;
        if (tip_before) *tip_before = t->c_before;
        if (tip_after) *tip_after = t->c_after;
        if (peers) *peers = t->c_peers;
        if (missing) *missing = t->c_miss;
        return FEA_OK;
    });
}

int32_t fea_cht_add_to_batch(fea_cht* t, int64_t id) {
    return fea::guarded("fea_cht_add_to_batch", [&]() -> int32_t {
        if (!t) return fail(FEA_EINVAL, "fea_cht_add_to_batch: NULL tree");
        auto it = t->req.find(id);
        if (it == t->req.end() || it->second.active) return fail(FEA_EINVAL, "fea_cht_add_to_batch: request %lld is not waiting", (long long)id);
        Request& r = it->second;
        t->unindex(id, r);
        r.active = true;
        --t->n_waiting;
        const int32_t C = (int32_t)r.H.size();
        // the new tip: first active request -> its full depth; otherwise the deepest level,
        // no deeper than the old tip, whose node the batch already holds
        int32_t new_tip = 0;
        if (t->active.empty()) {
            new_tip = C;
        } else {
            for (int32_t l = std::min(t->tip_level, C); l >= 1; --l)
                if (t->refs(Node{l, r.H[l - 1]}) > 0) { new_tip = l; break; }
        }
        for (int32_t l = C; l >= 1; --l) {
            const Node nd{l, r.H[l - 1]};
            int32_t& c = t->ref[nd];
            if (c == 0) t->bump(nd, -1);
            ++c;
        }
        t->active.push_back(id);
        t->tip_level = new_tip;
        t->tip_hash = new_tip > 0 ? r.H[new_tip - 1] : 0;
        t->cache_valid = false;
        return FEA_OK;
    });
}

int32_t fea_cht_finish(fea_cht* t, int64_t id) {
    return fea::guarded("fea_cht_finish", [&]() -> int32_t {
        if (!t) return fail(FEA_EINVAL, "fea_cht_finish: NULL tree");
        auto it = t->req.find(id);
        if (it == t->req.end() || !it->second.active) return fail(FEA_EINVAL, "fea_cht_finish: request %lld is not active", (long long)id);
        const std::vector<uint64_t> H = std::move(it->second.H);
        t->req.erase(it);
        t->active.erase(std::find(t->active.begin(), t->active.end(), id));
        for (int32_t l = 1; l <= (int32_t)H.size(); ++l) {
            const Node nd{l, H[l - 1]};
            auto c = t->ref.find(nd);
            if (--c->second == 0) {
                t->ref.erase(c);
                t->bump(nd, +1);
            }
        }
        if (t->active.empty()) {
            t->tip_level = 0;
            t->tip_hash = 0;
        } else {
            const std::vector<uint64_t>& H0 = t->req[t->active[0]].H;
            if (t->active.size() == 1) {
                t->tip_level = (int32_t)H0.size();
            } else {
                size_t depth = H0.size();
                for (int64_t q : t->active) depth = std::min(depth, t->req[q].H.size());
                while ((size_t)t->tip_level < depth &&
                       t->refs(Node{t->tip_level + 1, H0[t->tip_level]}) == (int32_t)t->active.size())
                    ++t->tip_level;
            }
            t->tip_hash = t->tip_level > 0 ? H0[t->tip_level - 1] : 0;
        }
        t->cache_valid = false;
        return FEA_OK;
    });
}

int32_t fea_cht_remove(fea_cht* t, int64_t id) {
    return fea::guarded("fea_cht_remove", [&]() -> int32_t {
        if (!t) return fail(FEA_EINVAL, "fea_cht_remove: NULL tree");
        auto it = t->req.find(id);
        if (it == t->req.end() || it->second.active) return fail(FEA_EINVAL, "fea_cht_remove: request %lld is not waiting", (long long)id);
        t->unindex(id, it->second);
        t->req.erase(it);
        --t->n_waiting;
        t->cache_valid = false;
        return FEA_OK;
    });
}

int32_t fea_cht_missing(const fea_cht* t, int64_t id, int32_t* missing) {
    if (!t || !missing) return fail(FEA_EINVAL, "fea_cht_missing: NULL argument");
    auto it = t->req.find(id);
    if (it == t->req.end() || it->second.active) return fail(FEA_EINVAL, "fea_cht_missing: request %lld is not waiting", (long long)id);
    *missing = it->second.miss;
    return FEA_OK;
}

int32_t fea_cht_stats(const fea_cht* t, int64_t* n_waiting, int64_t* n_active, int32_t* tip_level, uint64_t* tip_hash,
                      int64_t* working_set, int64_t* heap_entries) {
    if (!t) return fail(FEA_EINVAL, "fea_cht_stats: NULL tree");
    if (n_waiting) *n_waiting = t->n_waiting;
    if (n_active) *n_active = (int64_t)t->active.size();
    if (tip_level) *tip_level = t->tip_level;
    if (tip_hash) *tip_hash = t->tip_hash;
    if (working_set) *working_set = (int64_t)t->ref.size();
    if (heap_entries) *heap_entries = (int64_t)t->heap.size();
    return FEA_OK;
}

int32_t fea_cht_build_batch(fea_cht* t, const fea_stop_policy* p, int32_t max_batch, int64_t* ids, int32_t* n_out) {
    return fea::guarded("fea_cht_build_batch", [&]() -> int32_t {
        if (!t || !p || !ids || !n_out || max_batch < 0) return fail(FEA_EINVAL, "fea_cht_build_batch: bad argument");
        int32_t n = 0;
        while (n < max_batch) {
            int64_t id;
            int32_t before, after, peers;
            if (fea_cht_find_best(t, &id, &before, &after, &peers, nullptr) != FEA_OK) break;
            const int32_t loss = before - after;
            bool add;
            if (loss <= 0) add = true;
            else if (n < p->small_batch) add = loss <= p->loss_small;
            else if (loss <= p->loss_limit) add = true;
            else add = peers >= p->peers_relax && loss <= p->loss_relaxed;
            if (!add) break;
            const int32_t rc = fea_cht_add_to_batch(t, id);
            if (rc != FEA_OK) return rc;
            ids[n++] = id;
        }
        *n_out = n;
        return FEA_OK;
    });
}

}  // extern "C"

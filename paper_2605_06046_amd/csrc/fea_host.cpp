// Host side of libfea: error slot, KV block pool, chunked prefix hashes and the
// block-table builder.  No HIP in this file.
#include "../../include/fea.h"
#include "fea_internal.h"

#include <cstdio>
#include <cstring>
#include <deque>
#include <new>
#include <unordered_map>
#include <vector>

namespace fea {

static thread_local char g_err[512] = "";

int32_t fail(int32_t code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

// ---- the hash fixed in fea.h (splitmix64 finaliser as the mixing step) ----
static constexpr uint64_t kGamma = 0x9E3779B97F4A7C15ull;
static constexpr uint64_t kH0 = 0x243F6A8885A308D3ull;
static constexpr int kK = FEA_BLOCK_TOKENS;

static inline uint64_t mix(uint64_t x) {
    x ^= x >> 30;
    x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27;
    x *= 0x94D049BB133111EBull;
    x ^= x >> 31;
    return x;
}

static inline uint64_t leaf(const int32_t* t, int n) {
    uint64_t a = mix(kGamma ^ (uint64_t)n);
    for (int j = 0; j < n; ++j) a = mix(a ^ (uint64_t)(uint32_t)t[j]);
    return a;
}

// Four full chunks at a time: the per-chunk chains are independent (that is the
// point of the chunk-parallel formulation), so interleaving them hides the
// multiply latency of the serial mix chain.
static inline void leaf4(const int32_t* t, uint64_t out[4]) {
    uint64_t a0 = mix(kGamma ^ (uint64_t)kK), a1 = a0, a2 = a0, a3 = a0;
    for (int j = 0; j < kK; ++j) {
        a0 = mix(a0 ^ (uint64_t)(uint32_t)t[j]);
        a1 = mix(a1 ^ (uint64_t)(uint32_t)t[kK + j]);
        a2 = mix(a2 ^ (uint64_t)(uint32_t)t[2 * kK + j]);
        a3 = mix(a3 ^ (uint64_t)(uint32_t)t[3 * kK + j]);
    }
    out[0] = a0; out[1] = a1; out[2] = a2; out[3] = a3;
}

static inline uint64_t chain(uint64_t h_prev, uint64_t lf) { return mix(mix(h_prev + kGamma) ^ lf); }

static void chunk_hashes(const int32_t* tok, int64_t T, uint64_t* H) {
    const int64_t C = (T + kK - 1) / kK, full = T / kK;
    uint64_t h = kH0;
    int64_t c = 0;
    for (; c + 4 <= full; c += 4) {
        uint64_t lf[4];
        leaf4(tok + c * kK, lf);
        for (int u = 0; u < 4; ++u) { h = chain(h, lf[u]); H[c + u] = h; }
    }
    for (; c < C; ++c) {
        const int n = (int)((c + 1) * kK <= T ? kK : T - c * kK);
        h = chain(h, leaf(tok + c * kK, n));
        H[c] = h;
    }
}

// ---- the sequential formulation: one running XXH64 state, digested at every
// chunk boundary (appendix "Prefix Hash Computation", Algorithm 1).  Tokens enter
// as 4-byte little-endian words.  A full chunk is 64 bytes = two 32-byte stripes,
// so the stripe buffer is empty at every boundary but the last.
static constexpr uint64_t kP1 = 0x9E3779B185EBCA87ull, kP2 = 0xC2B2AE3D27D4EB4Full, kP3 = 0x165667B19E3779F9ull,
                          kP4 = 0x85EBCA77C2B2AE63ull, kP5 = 0x27D4EB2F165667C5ull;
static inline uint64_t rotl64(uint64_t x, int r) { return (x << r) | (x >> (64 - r)); }
static inline uint64_t xround(uint64_t acc, uint64_t lane) { return rotl64(acc + lane * kP2, 31) * kP1; }
static inline uint64_t xmerge(uint64_t h, uint64_t v) { return (h ^ xround(0, v)) * kP1 + kP4; }
static inline uint64_t word64(const int32_t* t) { return (uint64_t)(uint32_t)t[0] | ((uint64_t)(uint32_t)t[1] << 32); }

struct Xxh64Stream {
    uint64_t v[4], seed;
    int64_t stripes = 0;                       // 32-byte stripes consumed
    explicit Xxh64Stream(uint64_t sd) : seed(sd) {
        v[0] = sd + kP1 + kP2; v[1] = sd + kP2; v[2] = sd; v[3] = sd - kP1;
    }
    void stripe(const int32_t* t) {            // 8 tokens
        for (int i = 0; i < 4; ++i) v[i] = xround(v[i], word64(t + 2 * i));
        ++stripes;
    }
    // Digest after the consumed stripes plus `n` (< 8) further tokens at `t`.
    uint64_t digest(const int32_t* t, int n) const {
        uint64_t h;
        if (stripes > 0) {
            h = rotl64(v[0], 1) + rotl64(v[1], 7) + rotl64(v[2], 12) + rotl64(v[3], 18);
            for (int i = 0; i < 4; ++i) h = xmerge(h, v[i]);
        } else {
            h = seed + kP5;
        }
        h += (uint64_t)(stripes * 32 + 4 * n);
        int j = 0;
        for (; j + 2 <= n; j += 2) h = rotl64(h ^ xround(0, word64(t + j)), 27) * kP1 + kP4;
        if (j < n) h = rotl64(h ^ ((uint64_t)(uint32_t)t[j] * kP1), 23) * kP2 + kP3;
        h ^= h >> 33; h *= kP2; h ^= h >> 29; h *= kP3; h ^= h >> 32;
        return h;
    }
};

static void chunk_hashes_xxh64(const int32_t* tok, int64_t T, uint64_t seed, uint64_t* H) {
    Xxh64Stream s(seed);
    const int64_t full = T / kK;
    for (int64_t c = 0; c < full; ++c) {
        s.stripe(tok + c * kK);
        s.stripe(tok + c * kK + 8);
        H[c] = s.digest(nullptr, 0);
    }
    int rest = (int)(T - full * kK);
    if (rest > 0) {
        const int32_t* t = tok + full * kK;
        if (rest >= 8) { s.stripe(t); t += 8; rest -= 8; }
        H[full] = s.digest(t, rest);
    }
}

static void chunk_hashes_of_kind(int32_t kind, uint64_t seed, const int32_t* tok, int64_t T, uint64_t* H) {
    if (kind == FEA_HASH_XXH64) chunk_hashes_xxh64(tok, T, seed, H);
    else chunk_hashes(tok, T, H);
}

struct BlockMeta {
    int32_t refcount = 0;
    int32_t parent = -1;      // block of the previous column (-1 at level 0)
    int32_t level = -1;       // column index; -1: block holds no registered prefix
    uint64_t hash = 0;
    int32_t tokens[kK];
};

struct Key {
    uint64_t hash;
    int32_t level;
    bool operator==(const Key& o) const { return hash == o.hash && level == o.level; }
};
struct KeyHash {
    size_t operator()(const Key& k) const { return (size_t)(k.hash ^ mix((uint64_t)(uint32_t)k.level)); }
};

}  // namespace fea

struct fea_kv_pool {
    uint32_t num_blocks = 0;
    std::deque<int32_t> free_list;
    std::vector<fea::BlockMeta> meta;
    // (level, cumulative hash) -> blocks storing a prefix with that key.  More
    // than one entry only after a 64-bit collision between different prefixes.
    std::unordered_map<fea::Key, std::vector<int32_t>, fea::KeyHash> index;
    uint32_t collisions = 0;
    int32_t hash_kind = FEA_HASH_CHAINED;
    uint64_t hash_seed = 0;

    void unindex(int32_t b) {
        fea::BlockMeta& m = meta[b];
        if (m.level < 0) return;
        auto it = index.find(fea::Key{m.hash, m.level});
        if (it != index.end()) {
            auto& v = it->second;
            for (size_t k = 0; k < v.size(); ++k)
                if (v[k] == b) { v[k] = v.back(); v.pop_back(); break; }
            if (v.empty()) index.erase(it);
        }
        m.level = -1;
    }
};

using namespace fea;

extern "C" {

const char* fea_last_error(void) { return g_err; }

int32_t fea_kv_alloc(uint32_t num_blocks, uint32_t block_size, uint64_t perm_seed, fea_kv_pool** out) {
    if (!out) return fail(FEA_EINVAL, "fea_kv_alloc: out is NULL");
    if (num_blocks == 0 || num_blocks > 0x7FFFFFFFu) return fail(FEA_EINVAL, "fea_kv_alloc: num_blocks=%u out of range", num_blocks);
    if (block_size != FEA_BLOCK_TOKENS) return fail(FEA_EINVAL, "fea_kv_alloc: block_size=%u, only %d is supported", block_size, FEA_BLOCK_TOKENS);
    fea_kv_pool* p = new (std::nothrow) fea_kv_pool;
    if (!p) return fail(FEA_ENOMEM, "fea_kv_alloc: out of host memory");
    try {
        p->num_blocks = num_blocks;
        p->meta.resize(num_blocks);
        std::vector<int32_t> order(num_blocks);
        for (uint32_t i = 0; i < num_blocks; ++i) order[i] = (int32_t)i;
        if (perm_seed != 0) {
            uint64_t s = perm_seed;
            for (uint32_t k = num_blocks - 1; k >= 1; --k) {
                s += kGamma;
                const uint32_t j = (uint32_t)(mix(s) % (uint64_t)(k + 1));
                std::swap(order[k], order[j]);
            }
        }
        p->free_list.assign(order.begin(), order.end());
        p->index.reserve(num_blocks);
    } catch (...) {
        delete p;
        return fail(FEA_ENOMEM, "fea_kv_alloc: out of host memory");
    }
    *out = p;
    return FEA_OK;
}

int32_t fea_kv_free(fea_kv_pool* pool) {
    delete pool;
    return FEA_OK;
}

int32_t fea_kv_stats(const fea_kv_pool* pool, uint32_t* num_blocks, uint32_t* free_blocks,
                     uint32_t* hash_collisions, int32_t* refcounts) {
    if (!pool) return fail(FEA_EINVAL, "fea_kv_stats: pool is NULL");
    if (num_blocks) *num_blocks = pool->num_blocks;
    if (free_blocks) *free_blocks = (uint32_t)pool->free_list.size();
    if (hash_collisions) *hash_collisions = pool->collisions;
    if (refcounts)
        for (uint32_t b = 0; b < pool->num_blocks; ++b) refcounts[b] = pool->meta[b].refcount;
    return FEA_OK;
}

int32_t fea_chunk_hashes(const int32_t* tokens, int64_t T, uint64_t* hashes) {
    return fea::guarded("fea_chunk_hashes", [&]() -> int32_t {
        if (T < 0) return fail(FEA_EINVAL, "fea_chunk_hashes: T=%lld is negative", (long long)T);
        if (T == 0) return FEA_OK;
        if (!tokens || !hashes) return fail(FEA_EINVAL, "fea_chunk_hashes: NULL pointer");
        chunk_hashes(tokens, T, hashes);
        return FEA_OK;
    });
}

int32_t fea_chunk_hashes_xxh64(const int32_t* tokens, int64_t T, uint64_t seed, uint64_t* hashes) {
    return fea::guarded("fea_chunk_hashes_xxh64", [&]() -> int32_t {
        if (T < 0) return fail(FEA_EINVAL, "fea_chunk_hashes_xxh64: T=%lld is negative", (long long)T);
        if (T == 0) return FEA_OK;
        if (!tokens || !hashes) return fail(FEA_EINVAL, "fea_chunk_hashes_xxh64: NULL pointer");
        chunk_hashes_xxh64(tokens, T, seed, hashes);
        return FEA_OK;
    });
}

int32_t fea_kv_set_hash(fea_kv_pool* pool, int32_t kind, uint64_t seed) {
    return fea::guarded("fea_kv_set_hash", [&]() -> int32_t {
        if (!pool) return fail(FEA_EINVAL, "fea_kv_set_hash: pool is NULL");
        if (kind != FEA_HASH_CHAINED && kind != FEA_HASH_XXH64) return fail(FEA_EINVAL, "fea_kv_set_hash: unknown kind %d", kind);
        if (!pool->index.empty())
            return fail(FEA_EINVAL, "fea_kv_set_hash: the pool holds registered prefixes; set the hash before the first table is built");
        pool->hash_kind = kind;
        pool->hash_seed = seed;
        return FEA_OK;
    });
}

int32_t fea_build_block_tables(fea_kv_pool* pool, const int32_t* tokens, const int64_t* tok_offsets, int32_t B,
                               int32_t max_blocks_per_seq, int32_t* block_tables, int32_t* seq_lens,
                               uint64_t* hashes, int64_t* hash_offsets) {
    if (!pool) return fail(FEA_EINVAL, "fea_build_block_tables: pool is NULL");
    if (B < 0 || max_blocks_per_seq < 0) return fail(FEA_EINVAL, "fea_build_block_tables: negative B or max_blocks_per_seq");
    if (B == 0) { if (hash_offsets) hash_offsets[0] = 0; return FEA_OK; }
    if (!tok_offsets || !block_tables || !seq_lens) return fail(FEA_EINVAL, "fea_build_block_tables: NULL pointer");
    if ((hashes == nullptr) != (hash_offsets == nullptr)) return fail(FEA_EINVAL, "fea_build_block_tables: hashes and hash_offsets must both be given or both be NULL");
    int64_t total_chunks = 0;
    for (int32_t i = 0; i < B; ++i) {
        const int64_t T = tok_offsets[i + 1] - tok_offsets[i];
        if (T < 0 || tok_offsets[0] < 0) return fail(FEA_EINVAL, "fea_build_block_tables: tok_offsets not monotone at request %d", i);
        if (T > 0x7FFFFFFF) return fail(FEA_EINVAL, "fea_build_block_tables: request %d too long", i);
        const int64_t C = (T + kK - 1) / kK;
        if (C > max_blocks_per_seq) return fail(FEA_ERANGE, "fea_build_block_tables: request %d needs %lld blocks, table has %d columns", i, (long long)C, max_blocks_per_seq);
        total_chunks += C;
    }
    if (total_chunks > 0 && !tokens) return fail(FEA_EINVAL, "fea_build_block_tables: tokens is NULL");

    // Work on scratch outputs so that a failure leaves the caller's arrays untouched.
    std::vector<int32_t> tab;
    std::vector<uint64_t> hs;
    std::vector<int32_t> took;        // blocks popped from the free list, in order
    std::vector<int32_t> shared;      // blocks that gained a reference by aliasing
    std::vector<int32_t> registered;  // blocks entered into the index by this call
    const uint32_t collisions_before = pool->collisions;
    bool oom = false;
    int32_t oom_req = -1;
    try {
        tab.assign((size_t)B * max_blocks_per_seq, -1);
        hs.resize((size_t)total_chunks);
        int64_t hpos = 0;
        for (int32_t i = 0; i < B && !oom; ++i) {
            const int32_t* tok = tokens + tok_offsets[i];
            const int64_t T = tok_offsets[i + 1] - tok_offsets[i];
            const int64_t C = (T + kK - 1) / kK;
            uint64_t* H = hs.data() + hpos;
            chunk_hashes_of_kind(pool->hash_kind, pool->hash_seed, tok, T, H);   // a1
            int32_t parent = -1;
            for (int64_t c = 0; c < C; ++c) {                           // a2
                const bool full = (c + 1) * kK <= T;
                int32_t b = -1;
                if (full) {
                    auto it = pool->index.find(Key{H[c], (int32_t)c});
                    if (it != pool->index.end()) {
                        for (int32_t cand : it->second) {
                            const BlockMeta& m = pool->meta[cand];
                            if (m.parent == parent && std::memcmp(m.tokens, tok + c * kK, sizeof m.tokens) == 0) { b = cand; break; }
                        }
                        if (b < 0) pool->collisions++;
                    }
                }
                if (b >= 0) {
                    pool->meta[b].refcount++;
                    shared.push_back(b);
                } else {
                    if (pool->free_list.empty()) { oom = true; oom_req = i; break; }
                    b = pool->free_list.front();
                    pool->free_list.pop_front();
                    took.push_back(b);
                    BlockMeta& m = pool->meta[b];
                    m.refcount = 1;
                    m.level = -1;
                    if (full) {
                        m.parent = parent;
                        m.level = (int32_t)c;
                        m.hash = H[c];
                        std::memcpy(m.tokens, tok + c * kK, sizeof m.tokens);
                        pool->index[Key{H[c], (int32_t)c}].push_back(b);
                        registered.push_back(b);
                    }
                }
                tab[(size_t)i * max_blocks_per_seq + c] = b;
                parent = b;
            }
            hpos += C;
        }
    } catch (...) {
        oom = true;
    }
    if (oom) {
        for (size_t k = registered.size(); k-- > 0;) pool->unindex(registered[k]);
        for (int32_t b : shared) pool->meta[b].refcount--;
        for (size_t k = took.size(); k-- > 0;) {
            pool->meta[took[k]].refcount = 0;
            pool->free_list.push_front(took[k]);
        }
        pool->collisions = collisions_before;
        if (oom_req >= 0) return fail(FEA_ENOMEM, "fea_build_block_tables: KV pool exhausted at request %d (%u blocks in pool)", oom_req, pool->num_blocks);
        return fail(FEA_ENOMEM, "fea_build_block_tables: out of host memory");
    }
    std::memcpy(block_tables, tab.data(), tab.size() * sizeof(int32_t));
    int64_t hpos = 0;
    for (int32_t i = 0; i < B; ++i) {
        const int64_t T = tok_offsets[i + 1] - tok_offsets[i];
        seq_lens[i] = (int32_t)T;
        if (hash_offsets) hash_offsets[i] = hpos;
        hpos += (T + kK - 1) / kK;
    }
    if (hash_offsets) {
        hash_offsets[B] = hpos;
        if (total_chunks) std::memcpy(hashes, hs.data(), hs.size() * sizeof(uint64_t));
    }
    return FEA_OK;
}

int32_t fea_release(fea_kv_pool* pool, const int32_t* row, int32_t nb) {
    return fea::guarded("fea_release", [&]() -> int32_t {
        if (!pool) return fail(FEA_EINVAL, "fea_release: pool is NULL");
        if (nb < 0 || (nb > 0 && !row)) return fail(FEA_EINVAL, "fea_release: bad row");
        // validate first (a block may legally appear several times in one row)
        std::unordered_map<int32_t, int32_t> uses;
        for (int32_t c = 0; c < nb; ++c) {
            const int32_t b = row[c];
            if (b < 0 || (uint32_t)b >= pool->num_blocks) return fail(FEA_EINVAL, "fea_release: block id %d out of range in column %d", b, c);
            if (++uses[b] > pool->meta[b].refcount) return fail(FEA_EINVAL, "fea_release: block %d holds fewer references than the row drops", b);
        }
        for (int32_t c = 0; c < nb; ++c) {
            const int32_t b = row[c];
            if (--pool->meta[b].refcount == 0) {
                pool->unindex(b);
                pool->free_list.push_back(b);
            }
        }
        return FEA_OK;
    });
}

int32_t fea_kv_extend(fea_kv_pool* pool, int32_t* bt, int32_t stride, int32_t* seq_lens, int32_t B, int32_t* n_new_blocks) {
    return fea::guarded("fea_kv_extend", [&]() -> int32_t {
        if (!pool) return fail(FEA_EINVAL, "fea_kv_extend: pool is NULL");
        if (B < 0 || stride < 0 || (B > 0 && (!bt || !seq_lens))) return fail(FEA_EINVAL, "fea_kv_extend: bad arguments");
        // validate everything and count the blocks needed before touching anything
        size_t need = 0;
        for (int32_t i = 0; i < B; ++i) {
            const int32_t L = seq_lens[i];
            if (L < 0 || L == INT32_MAX) return fail(FEA_EINVAL, "fea_kv_extend: seq_lens[%d]=%d out of range", i, L);
            if (L % kK == 0) {
                if (L / kK >= stride) return fail(FEA_ERANGE, "fea_kv_extend: request %d needs column %d, the table has %d", i, L / kK, stride);
                ++need;
            }
        }
        if (need > pool->free_list.size())
            return fail(FEA_ENOMEM, "fea_kv_extend: %zu blocks needed, %zu free", need, pool->free_list.size());
        for (int32_t i = 0; i < B; ++i) {
            const int32_t L = seq_lens[i];
            if (L % kK == 0) {   // the new token opens a block: a private one, it holds no registered prefix
                const int32_t b = pool->free_list.front();
                pool->free_list.pop_front();
                fea::BlockMeta& m = pool->meta[b];
                m.refcount = 1;
                m.parent = -1;
                m.level = -1;
                bt[(size_t)i * stride + L / kK] = b;
            }
            seq_lens[i] = L + 1;
        }
        if (n_new_blocks) *n_new_blocks = (int32_t)need;
        return FEA_OK;
    });
}

int32_t fea_validate_block_tables(const int32_t* bt, int32_t stride, const int32_t* seq_lens, int32_t B, uint32_t num_blocks) {
    if (B < 0 || stride < 0 || (B > 0 && (!bt || !seq_lens))) return fail(FEA_EINVAL, "fea_validate_block_tables: bad arguments");
    for (int32_t i = 0; i < B; ++i) {
        const int32_t L = seq_lens[i];
        if (L < 0) return fail(FEA_EINVAL, "fea_validate_block_tables: seq_lens[%d]=%d is negative", i, L);
        const int64_t nb = ((int64_t)L + kK - 1) / kK;
        if (nb > stride) return fail(FEA_EINVAL, "fea_validate_block_tables: request %d needs %lld columns, stride is %d", i, (long long)nb, stride);
        for (int64_t c = 0; c < nb; ++c) {
            const int32_t b = bt[(size_t)i * stride + c];
            if (b < 0 || (uint32_t)b >= num_blocks) return fail(FEA_EINVAL, "fea_validate_block_tables: entry [%d,%lld]=%d outside [0,%u)", i, (long long)c, b, num_blocks);
        }
    }
    return FEA_OK;
}

}  // extern "C"

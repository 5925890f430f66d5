// Alias detection and work-list construction on the device (one workgroup).
//
// Reads only the block tables and lengths.  Requests whose table rows start with
// the same run of block ids form a group (the device-side sibling of the shared
// prefix tip of Section 4.2: the deepest level all members agree on); the run is
// swept once for the whole group, the remaining columns of each request are swept
// on their own.  A group is only a way to save KV reads: membership requires
// nothing but equal block ids over the run and full blocks for every member, so
// the result is the same attention whatever the tables look like.
//
// The sweeps are then laid end to end as one stream of 32-token tiles (shared
// runs first) and the stream is cut into equal shares, one per sweep wave, so
// that every wave moves the same number of KV bytes; a cut inside a segment just
// adds one partial result to it.  With an explicit split size the segments are
// cut every `split` blocks instead and the pieces dealt out in equal numbers.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <climits>

#include "fea_plan.h"

namespace fea {

__device__ __forceinline__ int cdiv(int a, int b) { return (a + b - 1) / b; }

// Integer division by a run-time divisor without the ~40-instruction expansion:
// exact for 0 <= x < 2^24 and 1 <= d (row and request counts are far below that).
struct FastDiv {
    int d;
    float rcp;
    __device__ explicit FastDiv(int dd) : d(dd), rcp(1.0f / (float)dd) {}
    __device__ __forceinline__ int div(int x) const {
        int q = (int)((float)x * rcp);
        const int r = x - q * d;
        if (r >= d) ++q;
        if (r < 0) --q;
        return q;
    }
    __device__ __forceinline__ int cdiv(int x) const { return div(x + d - 1); }
};

// The same through double precision: exact for 0 <= x < 2^31 (tile positions).
struct WideDiv {
    int d;
    double rcp;
    __device__ explicit WideDiv(int dd) : d(dd), rcp(1.0 / (double)dd) {}
    __device__ __forceinline__ int div(int x) const {
        int q = (int)((double)x * rcp);
        const long long r = (long long)x - (long long)q * d;
        if (r >= d) ++q;
        if (r < 0) --q;
        return q;
    }
};

// floor(x / d) for 0 <= x < 2^52 and d >= 1 through double precision: the 64-bit
// integer division expands to hundreds of dependent instructions, which is felt in
// the serial stretches of a single-workgroup kernel.
__device__ __forceinline__ long long ddiv(long long x, int d) {
    long long q = (long long)((double)x / (double)d);
    const long long r = x - q * d;
    if (r >= d) ++q;
    if (r < 0) --q;
    return q;
}

// Exclusive prefix sum of one int per thread over the 1024-thread block.
__device__ int block_scan_excl(int v, int* s_tmp, int& total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int x = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int y = __shfl_up(x, o);
        if (lane >= o) x += y;
    }
    if (lane == 63) s_tmp[wave] = x;
    __syncthreads();
    if (wave == 0) {
        constexpr int kWaves = kPlanThreads / 64;
        const int w = lane < kWaves ? s_tmp[lane] : 0;
        int xs = w;
#pragma unroll
        for (int o = 1; o < kWaves; o <<= 1) {
            const int y = __shfl_up(xs, o);
            if (lane >= o) xs += y;
        }
        if (lane < kWaves) s_tmp[32 + lane] = xs - w;
        if (lane == kWaves - 1) s_tmp[31] = xs;
    }
    __syncthreads();
    const int base = s_tmp[32 + wave];
    total = s_tmp[31];
    __syncthreads();
    return base + x - v;
}

// Four neighbouring table columns, loadable from any 4-byte boundary.
struct __attribute__((packed, aligned(4))) Cols4 { int32_t c[4]; };

__device__ __forceinline__ uint32_t slot_of(int key) { return ((uint32_t)key * 2654435761u) >> 20; }  // 12 bits

__device__ __forceinline__ void write_item(Item* it, int who, int g, int nrows, int mlist_off, int c0, int c1,
                                           int pbase, int tok_end) {
    int4* p = reinterpret_cast<int4*>(it);
    p[0] = make_int4(who, g, nrows, mlist_off);
    p[1] = make_int4(c0, c1, pbase, tok_end);
}

// Leaders and common runs for large tables, on many workgroups (the planner's one
// workgroup would pull every follower's and leader's row through a single CU: 71 of its
// 105 us for 800 requests of 10K tokens).  Every workgroup finds the leaders for itself
// (smallest request index per first block; a few thousand LDS operations), then its waves
// take followers in turn: 64 lanes x 4 columns per step, the first differing column and the
// follower's block there picked from the lowest lane that saw a difference.
__global__ __launch_bounds__(kRunThreads) void run_kernel(PlanArgs a) {
    __shared__ int keys[kHashSlots], vals[kHashSlots];
    __shared__ int s_len[kGroupReqMax];
    __shared__ short s_lead[kGroupReqMax];
    const int tid = threadIdx.x, lane = tid & 63;
    const int nG = a.grouping ? min(a.B, kGroupReqMax) : 0;
    const int maxL = a.stride * kBlock;
    constexpr int kPer = kGroupReqMax / kRunThreads;
    for (int s = tid; s < kHashSlots; s += kRunThreads) { keys[s] = -1; vals[s] = INT_MAX; }
    __syncthreads();
    int my_key[kPer];
#pragma unroll
    for (int k = 0; k < kPer; ++k) {
        const int i = tid + k * kRunThreads;
        my_key[k] = -1;
        if (i < nG) {
            const int L = max(0, min(a.seq_lens[i], maxL));
            s_len[i] = L;
            if (L >= kBlock) {
                const int key = a.bt[(size_t)i * a.stride];
                my_key[k] = key;
                if (key >= 0) {
                    uint32_t s = slot_of(key);
                    for (;;) {
                        const int old = atomicCAS(&keys[s], -1, key);
                        if (old == -1 || old == key) { atomicMin(&vals[s], i); break; }
                        s = (s + 1) & (kHashSlots - 1);
                    }
                }
            }
        }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kPer; ++k) {
        const int i = tid + k * kRunThreads;
        if (i < nG) {
            int lead = -1;
            const int key = my_key[k];
            if (key >= 0) {
                uint32_t s = slot_of(key);
                while (keys[s] != key) s = (s + 1) & (kHashSlots - 1);
                lead = vals[s];
            }
            s_lead[i] = (short)lead;
        }
    }
    __syncthreads();
    unsigned long long* pre = reinterpret_cast<unsigned long long*>(a.ws + a.lay.pre);
    int* pre_lead = reinterpret_cast<int*>(pre + kGroupReqMax);
    const int waves = gridDim.x * (kRunThreads / 64);
    for (int i = blockIdx.x * (kRunThreads / 64) + (tid >> 6); i < nG; i += waves) {
        const int lead = s_lead[i];
        const int cp = lead >= 0 ? min(s_len[i], s_len[lead]) / kBlock : 0;
        unsigned long long res = ((unsigned long long)(uint32_t)cp << 32) | 0xFFFFFFFFull;
        if (lead >= 0 && lead != i) {
            const int32_t* ri = a.bt + (size_t)i * a.stride;
            const int32_t* rl = a.bt + (size_t)lead * a.stride;
            constexpr int kWin = 4;   // column windows (64 lanes x 4 columns) requested together
            bool done = false;
            for (int c0 = 0; c0 < cp && !done; c0 += 256 * kWin) {
                int4 x[kWin], y[kWin];
#pragma unroll
                for (int u = 0; u < kWin; ++u) {
                    const int c = c0 + u * 256 + lane * 4;
                    x[u] = y[u] = make_int4(0, 0, 0, 0);
                    if (c < cp) {
                        if (c + 4 <= a.stride) {
                            const Cols4 xv = *reinterpret_cast<const Cols4*>(ri + c), yv = *reinterpret_cast<const Cols4*>(rl + c);
                            x[u] = make_int4(xv.c[0], xv.c[1], xv.c[2], xv.c[3]);
                            y[u] = make_int4(yv.c[0], yv.c[1], yv.c[2], yv.c[3]);
                        } else {
                            const bool two = c + 1 < a.stride, three = c + 2 < a.stride;
                            x[u] = make_int4(ri[c], two ? ri[c + 1] : 0, three ? ri[c + 2] : 0, 0);
                            y[u] = make_int4(rl[c], two ? rl[c + 1] : 0, three ? rl[c + 2] : 0, 0);
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < kWin; ++u) {
                    const int c = c0 + u * 256 + lane * 4;
                    int first = INT_MAX, mine = 0;
                    if (x[u].w != y[u].w) { first = c + 3; mine = x[u].w; }
                    if (x[u].z != y[u].z) { first = c + 2; mine = x[u].z; }
                    if (x[u].y != y[u].y) { first = c + 1; mine = x[u].y; }
                    if (x[u].x != y[u].x) { first = c; mine = x[u].x; }
                    const unsigned long long seen = __ballot(!done && first < cp);
                    if (seen) {   // lanes hold rising columns: the lowest lane has the first difference
                        const int src = __ffsll((long long)seen) - 1;
                        const int f0 = __shfl(first, src), m0 = __shfl(mine, src);
                        res = ((unsigned long long)(uint32_t)f0 << 32) | (uint32_t)m0;
                        done = true;
                    }
                }
            }
        }
        if (lane == 0) { pre[i] = res; pre_lead[i] = lead; }
    }
}

constexpr int kGroupMax = kGroupReqMax / 2;   // a group has at least two members

__global__ __launch_bounds__(kPlanThreads) void plan_kernel(PlanArgs a) {
    static_assert(kHashSlots == 4096, "slot_of() yields 12 bits");
    __shared__ union {
        struct { int keys[kHashSlots]; int vals[kHashSlots]; } h;                     // leader finding only
        struct { int run[kGroupReqMax]; int cnt[kGroupReqMax]; int moff[kGroupReqMax];
                 int gseg[kGroupMax]; } c;                                            // afterwards
    } u;
    __shared__ struct { int keys[kHashSlots]; int vals[kHashSlots]; } h2;             // subgroup leaders (nested runs)
    __shared__ unsigned short s_r1[kGroupReqMax];
    __shared__ unsigned long long s_lcpv[kGroupReqMax];   // round one: (common run << 32) | the follower's block where it ends
    __shared__ short s_lead[kGroupReqMax];      // request ids fit 16 bits (kGroupReqMax <= 32767)
    __shared__ int s_len[kGroupReqMax];
    __shared__ union {
        struct { int lcp[kGroupReqMax]; short lead2[kGroupReqMax]; } x;   // until the group runs are known
        struct { int npc[kGroupMax]; int ibase[kGroupMax]; int rbase[kGroupMax]; } g;   // then the cut of each group
    } v;
    __shared__ union {
        unsigned short flw[kGroupReqMax];       // followers (grouped, not leader), for the run detection
        unsigned short glist[kGroupMax];        // then the list of viable leaders
    } w;
    __shared__ int s_tmp[64];
    __shared__ int s_ngroups, s_ngrouped, s_shared_blocks, s_nflw, s_nest, s_adopt;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int* hdr = reinterpret_cast<int*>(a.ws);
    ReqDesc* req = reinterpret_cast<ReqDesc*>(a.ws + a.lay.req);
    GroupDesc* grp = reinterpret_cast<GroupDesc*>(a.ws + a.lay.grp);
    int* members = reinterpret_cast<int*>(a.ws + a.lay.members);
    SegDesc* segs = reinterpret_cast<SegDesc*>(a.ws + a.lay.segs);
    int* wave_first = reinterpret_cast<int*>(a.ws + a.lay.wave_first);
    Item* items = reinterpret_cast<Item*>(a.ws + a.lay.items);

    const int B = a.B, Hkv = a.Hkv;
    const int nG = a.grouping ? min(B, kGroupReqMax) : 0;
    const int maxL = a.stride * kBlock;
    auto clampL = [&](int L) { return max(0, min(L, maxL)); };

    int my_key[kGroupReqMax / kPlanThreads];
    for (int s = tid; s < kHashSlots; s += kPlanThreads) { h2.keys[s] = -1; h2.vals[s] = INT_MAX; }
    if (tid == 0) { s_ngroups = 0; s_ngrouped = 0; s_shared_blocks = 0; s_nflw = 0; }
    if (a.pre) {
        // ---- leaders and common runs were found by run_kernel
        const unsigned long long* pre = reinterpret_cast<const unsigned long long*>(a.ws + a.lay.pre);
        const int* pre_lead = reinterpret_cast<const int*>(pre + kGroupReqMax);
        for (int i = tid; i < nG; i += kPlanThreads) {
            s_len[i] = clampL(a.seq_lens[i]);
            s_lead[i] = (short)pre_lead[i];
            s_lcpv[i] = pre[i];
        }
        __syncthreads();
    } else {
        // ---- leaders: smallest request index among those with the same first block
        for (int s = tid; s < kHashSlots; s += kPlanThreads) { u.h.keys[s] = -1; u.h.vals[s] = INT_MAX; }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < kGroupReqMax / kPlanThreads; ++k) {
            const int i = tid + k * kPlanThreads;
            my_key[k] = -1;
            if (i < nG) {
                const int L = clampL(a.seq_lens[i]);
                s_len[i] = L;
                if (L >= kBlock) {
                    const int key = a.bt[(size_t)i * a.stride];
                    my_key[k] = key;
                    if (key >= 0) {
                        uint32_t s = slot_of(key);
                        for (;;) {
                            const int old = atomicCAS(&u.h.keys[s], -1, key);
                            if (old == -1 || old == key) { atomicMin(&u.h.vals[s], i); break; }
                            s = (s + 1) & (kHashSlots - 1);
                        }
                    }
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < kGroupReqMax / kPlanThreads; ++k) {
            const int i = tid + k * kPlanThreads;
            if (i < nG) {
                int lead = -1, lcp = 0;
                const int key = my_key[k];
                if (key >= 0) {
                    uint32_t s = slot_of(key);
                    while (u.h.keys[s] != key) s = (s + 1) & (kHashSlots - 1);
                    lead = u.h.vals[s];
                    lcp = min(s_len[i], s_len[lead]) / kBlock;
                    if (lead != i) w.flw[atomicAdd(&s_nflw, 1)] = (unsigned short)i;
                }
                s_lead[i] = (short)lead;
                s_lcpv[i] = ((unsigned long long)(uint32_t)lcp << 32) | 0xFFFFFFFFull;
            }
        }
        __syncthreads();   // the hash table is dead from here on; its memory becomes run/cnt/moff/...
    }
    auto reset_groups = [&](int moff0) {
        for (int i = tid; i < nG; i += kPlanThreads) { u.c.run[i] = INT_MAX; u.c.cnt[i] = 0; u.c.moff[i] = moff0; }
    };
    reset_groups(0);

    // ---- longest common run of block ids with the leader's row.  All (follower,
    // column group) pairs are spread flat over the threads, six at a time so that
    // their loads are in flight together; a mismatch lowers the follower's run with
    // an LDS atomic.  Columns below from(i) are known to agree and are not read.
    auto lcp_pass = [&](int nflw, const short* lead_of, auto&& from, auto&& hit) {
        constexpr int cpe = 4;                             // columns per element
        const int epr = cdiv(a.stride, cpe);               // elements per row (the last one may be short)
        const FastDiv by_epr(max(epr, 1));
        const int total = nflw * epr;
        constexpr int kBatch = 6;
        for (int e0 = tid; e0 < total; e0 += kBatch * kPlanThreads) {
            int4 xs[kBatch], ys[kBatch];
            int who[kBatch], col[kBatch], cap[kBatch];
#pragma unroll
            for (int q = 0; q < kBatch; ++q) {
                const int e = e0 + q * kPlanThreads;
                who[q] = -1;
                if (e < total) {
                    const int f = by_epr.div(e);
                    const int i = w.flw[f];
                    const int lead = lead_of[i];
                    const int c = (e - f * epr) * cpe;
                    const int cp = min(s_len[i], s_len[lead]) / kBlock;   // the starting value of lcp[i]
                    if (c < cp && c + cpe > from(i)) {
                        who[q] = i; col[q] = c; cap[q] = cp;
                        const int32_t* ri = a.bt + (size_t)i * a.stride + c;
                        const int32_t* rl = a.bt + (size_t)lead * a.stride + c;
                        if (c + cpe <= a.stride) {          // rows need not start on 16-byte boundaries
                            const Cols4 x = *reinterpret_cast<const Cols4*>(ri), y = *reinterpret_cast<const Cols4*>(rl);
                            xs[q] = make_int4(x.c[0], x.c[1], x.c[2], x.c[3]);
                            ys[q] = make_int4(y.c[0], y.c[1], y.c[2], y.c[3]);
                        } else {                            // the row's last, short element
                            const bool two = c + 1 < a.stride, three = c + 2 < a.stride;
                            xs[q] = make_int4(ri[0], two ? ri[1] : 0, three ? ri[2] : 0, 0);
                            ys[q] = make_int4(rl[0], two ? rl[1] : 0, three ? rl[2] : 0, 0);
                        }
                    }
                }
            }
#pragma unroll
            for (int q = 0; q < kBatch; ++q) {
                if (who[q] >= 0) {
                    int first = INT_MAX, mine = 0;
                    if (xs[q].w != ys[q].w) { first = col[q] + 3; mine = xs[q].w; }
                    if (xs[q].z != ys[q].z) { first = col[q] + 2; mine = xs[q].z; }
                    if (xs[q].y != ys[q].y) { first = col[q] + 1; mine = xs[q].y; }
                    if (xs[q].x != ys[q].x) { first = col[q]; mine = xs[q].x; }
                    if (first < cap[q]) hit(who[q], first, mine);
                }
            }
        }
    };
    auto note_run_end = [&](int who, int first, int mine) {   // the run and the follower's block that ends it
        atomicMin(&s_lcpv[who], ((unsigned long long)(uint32_t)first << 32) | (uint32_t)mine);
    };
    if (!a.pre) {
        lcp_pass(s_nflw, s_lead, [](int) { return 0; }, note_run_end);
        __syncthreads();
    }

    // A 32-token tile costs a wave more the more query rows ride on it: weights in
    // sixteenths of a 16-row tile's sweep.
    const int w32 = a.tune.weights & 255, w64 = (a.tune.weights >> 8) & 255;
    auto tile_weight = [&](int rows) { return rows <= 16 ? 16 : (rows <= 32 ? w32 : w64); };
    const FastDiv by_mpt(a.mpt);
    // Row tiles of one piece of a shared run read the same KV bytes.  On the matrix-core path the sweep
    // runs them as a team of 2 or 4 waves of one workgroup that fetches every tile once; for that the
    // row tiles of a piece sit on neighbouring shares, in slots of 1, 2 or a multiple of 4 (the slots
    // past the last row tile hold waves that only help fetching), and every group starts on a multiple of 4.
    const bool teams = a.teams != 0 && a.split_user == 0;   // (with a fixed split a share holds several items: no teams)
    auto tiles_padded = [&](int tiles_r) { return (!teams || tiles_r <= 2) ? tiles_r : ((tiles_r + 3) & ~3); };
    auto items_padded = [&](int n) { return teams ? ((n + 3) & ~3) : n; };
    // cost of one 32-token tile of a shared run per wave that sweeps it, for a group of cnt members: a team
    // fetches the tile once for all its row tiles and overlaps the two products, which makes the tile far
    // cheaper for a wave than a tile it streams and sweeps alone
    // (a team of 2 fetches half of every tile per wave, a team of 4 a quarter: the tile costs the former more)
    const int w_team = (a.tune.weights >> 16) & 255, w_team2 = (a.tune.weights >> 24) & 127;
    auto group_weight = [&](int cnt) {
        const int tiles_r = by_mpt.cdiv(cnt);
        return (teams && tiles_r >= 2) ? (tiles_r == 2 ? w_team2 : w_team) : tile_weight(min(a.mpt, cnt) * a.G);
    };
    // ... and what a piece costs the two waves of a small team besides its tiles: they fill the table of block ids
    // and the ring before the first tile, and drain it after the last, with half the lanes a team of 4 has for it
    // (measured: 32 requests on one 4096-token prefix 26.2 -> 24.6 us; with the same charge on teams of 4, whose
    // pieces it shortens as well, the 64-request batch lost 0.5 us to the merge of the extra pieces)
    auto group_fixed = [&](int cnt) { return (teams && by_mpt.cdiv(cnt) == 2) ? a.tune.team_fixed : 0; };

    // ---- nested prefixes.  Members of a group may go on sharing blocks past the group's
    // run (a common system prompt, then a few conversations: the radix patterns of
    // Section 3).  A second round finds, inside every group, the members that carry the
    // same block in the first column after the run, and their common run from there.
    // Such a subgroup becomes a group of its own (run measured from column 0, so it sweeps
    // the outer run again) when that saves more sweep cost than it adds, by the tile weights;
    // the members left behind keep the outer run under the smallest index among them.
    //
    // A follower agrees with its leader over lcp >= run columns.  If lcp > run it is in the
    // leader's subgroup and its run there is lcp itself; if lcp == run, the block that
    // tells its subgroup sits in column lcp - the very entry the run detection stopped at,
    // which it hands over together with the column (no further memory round trip).
    // Stage by stage: (1) runs, sizes (and, the first time, ranks) of the groups as they
    // are; (2) keys into a hash table of their own; (3) subgroup leaders.  With nothing
    // nested that is all (two barriers more than without this stage) and the results of
    // (1) stand.  Otherwise the subgroups' runs are measured and the ones that pay split
    // off; those are looked at again (a further level of sharing), kMaxLevels times at most.
    // Members left behind, and subgroups that stay, are final.
    constexpr int kPer = kGroupReqMax / kPlanThreads;
    constexpr int kMaxLevels = 4;
    int my_rank[kPer];
    {
        int lead1[kPer];
        bool act[kPer];          // still part of a group that may split further
        bool regroup = false;    // groups changed after the first stage (1): stats and ranks are redone
#pragma unroll
        for (int k = 0; k < kPer; ++k) {
            const int i = tid + k * kPlanThreads;
            lead1[k] = i < nG ? (int)s_lead[i] : -1;
            act[k] = lead1[k] >= 0;
            my_rank[k] = 0;
        }
        for (int level = 0; level < kMaxLevels; ++level) {
            int r1[kPer], lcp1[kPer];
            bool in[kPer];
            if (tid == 0) { s_nflw = 0; s_nest = 0; s_adopt = 0; }
#pragma unroll
            for (int k = 0; k < kPer; ++k) {
                const int i = tid + k * kPlanThreads;
                lcp1[k] = 0;
                my_key[k] = -1;
                if (act[k]) {
                    const unsigned long long lv = s_lcpv[i];
                    lcp1[k] = (int)(lv >> 32);
                    v.x.lcp[i] = lcp1[k];
                    if (lead1[k] != i && lcp1[k] < s_len[i] / kBlock) {
                        // the block in the column where the follower left its leader: the run detection saw
                        // it, unless the leader's row simply ended there
                        my_key[k] = (uint32_t)lv != 0xFFFFFFFFu ? (int)(uint32_t)lv : a.bt[(size_t)i * a.stride + lcp1[k]];
                    }
                    atomicMin(&u.c.run[lead1[k]], lcp1[k]);
                    const int rank = atomicAdd(&u.c.cnt[lead1[k]], 1);
                    if (level == 0) my_rank[k] = rank;
                }
            }
            __syncthreads();
#pragma unroll
            for (int k = 0; k < kPer; ++k) {
                in[k] = act[k] && u.c.cnt[lead1[k]] >= 2 && u.c.run[lead1[k]] >= a.tune.min_run;
                r1[k] = in[k] ? u.c.run[lead1[k]] : 0;
                if (!in[k] || lcp1[k] > r1[k]) my_key[k] = -1;      // only the members that leave the leader at the run
                const int key = my_key[k];
                if (key >= 0) {
                    uint32_t s = slot_of(key);
                    for (;;) {
                        const int old = atomicCAS(&h2.keys[s], -1, key);
                        if (old == -1 || old == key) { atomicMin(&h2.vals[s], tid + k * kPlanThreads); break; }
                        s = (s + 1) & (kHashSlots - 1);
                    }
                }
            }
            __syncthreads();
            int lead2[kPer];
#pragma unroll
            for (int k = 0; k < kPer; ++k) {
                const int i = tid + k * kPlanThreads;
                lead2[k] = -1;
                const int key = my_key[k];
                if (key >= 0) {
                    uint32_t s = slot_of(key);
                    while (h2.keys[s] != key) s = (s + 1) & (kHashSlots - 1);
                    const int cand = h2.vals[s];
                    lead2[k] = s_lead[cand] == lead1[k] ? cand : i;     // only within the same outer group
                    s_lcpv[i] = ((unsigned long long)(uint32_t)(min(s_len[i], s_len[lead2[k]]) / kBlock) << 32) | 0xFFFFFFFFull;
                    if (lead2[k] != i) w.flw[atomicAdd(&s_nflw, 1)] = (unsigned short)i;
                } else if (in[k] && (lead1[k] == i || lcp1[k] > r1[k])) {
                    lead2[k] = lead1[k];                                // the leader's own subgroup: runs are known
                    if (lead1[k] != i) atomicAdd(&s_nest, 1);
                }
                if (i < nG) { v.x.lead2[i] = (short)lead2[k]; s_r1[i] = (unsigned short)min(r1[k], 65535); }
            }
            __syncthreads();
            const int nflw2 = s_nflw;
            if (nflw2 + s_nest == 0) break;            // uniform: nothing (more) is nested
            regroup = true;
            if (nflw2 > 0) {
                lcp_pass(nflw2, v.x.lead2, [&](int i) { return (int)s_r1[i]; }, note_run_end);
                __syncthreads();
            }
            reset_groups(INT_MAX);
            __syncthreads();
            int lcp2[kPer];
#pragma unroll
            for (int k = 0; k < kPer; ++k) {           // runs and sizes of the subgroups
                const int i = tid + k * kPlanThreads;
                lcp2[k] = 0;
                if (lead2[k] >= 0) {
                    lcp2[k] = (int)(s_lcpv[i] >> 32);
                    atomicMin(&u.c.run[lead2[k]], lcp2[k]);
                    atomicAdd(&u.c.cnt[lead2[k]], 1);
                }
            }
            __syncthreads();
            bool adopt[kPer];
#pragma unroll
            for (int k = 0; k < kPer; ++k) {
                adopt[k] = false;
                if (lead2[k] >= 0) {
                    const int c2 = u.c.cnt[lead2[k]], run2 = u.c.run[lead2[k]];
                    // private sweeps saved plus the outer group's relief against the subgroup's own sweep
                    const long long gain = 16ll * c2 * (run2 - r1[k]) + (long long)r1[k] * group_weight(2 * a.mpt) * by_mpt.div(c2);
                    const long long cost = (long long)run2 * group_weight(c2) * by_mpt.cdiv(c2);
                    adopt[k] = c2 >= 2 && gain > cost;
                    if (adopt[k] && lead2[k] == tid + k * kPlanThreads) atomicAdd(&s_adopt, 1);
                }
                if (in[k] && !adopt[k]) atomicMin(&u.c.moff[lead1[k]], tid + k * kPlanThreads);   // who leads the rest
            }
            __syncthreads();
            int lead_f[kPer];
#pragma unroll
            for (int k = 0; k < kPer; ++k) lead_f[k] = adopt[k] ? lead2[k] : (in[k] ? u.c.moff[lead1[k]] : lead1[k]);
            const bool again = s_adopt > 0 && level + 1 < kMaxLevels;
            __syncthreads();                           // every leader is read before any changes
#pragma unroll
            for (int k = 0; k < kPer; ++k) {
                const int i = tid + k * kPlanThreads;
                if (in[k]) {
                    s_lead[i] = (short)lead_f[k];
                    v.x.lcp[i] = adopt[k] ? lcp2[k] : r1[k];
                }
                lead1[k] = lead_f[k];
                act[k] = adopt[k];
            }
            if (!again) break;                         // uniform
            // the groups that split off are looked at again, with clean tables
            for (int s = tid; s < kHashSlots; s += kPlanThreads) { h2.keys[s] = -1; h2.vals[s] = INT_MAX; }
            reset_groups(0);   // every thread changed only its own requests' entries above
            __syncthreads();
        }
        if (regroup) {
            __syncthreads();
            reset_groups(0);
            __syncthreads();
            // runs, sizes and ranks of the groups as they are now
#pragma unroll
            for (int k = 0; k < kPer; ++k) {
                const int i = tid + k * kPlanThreads;
                my_rank[k] = 0;
                if (i < nG) {
                    const int lead = s_lead[i];
                    if (lead >= 0) {
                        atomicMin(&u.c.run[lead], v.x.lcp[i]);
                        my_rank[k] = atomicAdd(&u.c.cnt[lead], 1);
                    }
                }
            }
            __syncthreads();
        }
    }
    // lcp[] and flw[] are dead from here on; run/cnt hold every group's run (the shortest
    // common run over its members) and size, my_rank the arrival at the group's counter
    // A run swept by teams is cut to an even number of columns (tiles are two columns; a piece with a column left
    // over is not taken by a team, and the waves that sweep it on their own hold up the team they share a
    // workgroup with).  The members read the column left over with their own ones, out of L2 after the first.
    if (teams) {
        for (int i = tid; i < nG; i += kPlanThreads)
            if (s_lead[i] == i && u.c.cnt[i] > a.mpt) u.c.run[i] &= ~1;
        __syncthreads();
    }
    auto viable = [&](int i) { return s_lead[i] == i && u.c.cnt[i] >= 2 && u.c.run[i] >= a.tune.min_run; };

    // ---- member-list offsets (exclusive scan over leaders) and the list of groups
    {
        const int per = (nG + kPlanThreads - 1) / kPlanThreads;   // 0, 1 or 2
        const int i0 = tid * per, i1 = min(nG, i0 + per);
        int local = 0;
        for (int i = i0; i < i1; ++i)
            if (viable(i)) local += u.c.cnt[i];
        int total;
        int base = block_scan_excl(local, s_tmp, total);
        for (int i = i0; i < i1; ++i)
            if (viable(i)) {
                u.c.moff[i] = base;
                base += u.c.cnt[i];
                w.glist[atomicAdd(&s_ngroups, 1)] = (unsigned short)i;
                atomicAdd(&s_shared_blocks, u.c.run[i]);
            }
        if (tid == 0) s_ngrouped = total;
    }
    __syncthreads();
    const int n_groups = s_ngroups;

    // ---- cost model (tile weights as above).  Shared runs are cut into
    // equal pieces per segment, one piece per wave (a "share"); the private columns of
    // all requests form one stream of tiles that is cut into equal shares for the
    // remaining waves.  Both kinds of share are sized to the same cost.
    auto run_of = [&](int i) {   // shared columns of request i (0 if ungrouped)
        if (i >= nG) return 0;
        const int lead = s_lead[i];
        return (lead >= 0 && viable(lead)) ? u.c.run[lead] : 0;
    };
    auto len_of = [&](int i) { return i < nG ? s_len[i] : clampL(a.seq_lens[i]); };
    auto priv_tiles = [&](int i) { return ((((len_of(i) + kBlock - 1) / kBlock) - run_of(i)) + 1) >> 1; };   // per KV head

    // private stream: request i owns Hkv * priv_tiles(i) consecutive tiles, KV head by KV
    // head.  Its segments (request, KV head) are the entries the threads share out, so
    // that a batch of few requests still spreads over many lanes.
    const int NE = B * Hkv;
    const int per = (NE + kPlanThreads - 1) / kPlanThreads;
    const int e0 = tid * per, e1 = min(NE, e0 + per);
    const FastDiv by_hkv(Hkv);
    int lt = 0;
    for (int e = e0; e < e1; ++e) lt += priv_tiles(by_hkv.div(e));
    int T_pr;
    const int tbase = block_scan_excl(lt, s_tmp, T_pr);
    // shared side: wave 0 sizes the shares, lanes over the groups (float reciprocals are
    // exact here: every dividend is a tile or share count far below 2^24)
    __shared__ int s_plan[8];
    auto idiv = [](int x, int d) {
        int qq = (int)((float)x * (1.0f / (float)d));
        const int r = x - qq * d;
        if (r >= d) ++qq;
        if (r < 0) --qq;
        return qq;
    };
    if (wave == 0) {
        // Sums and scans over the groups, one group per lane.  Cross-lane moves cost an LDS
        // round trip each and this stretch is serial, so only as many butterfly steps are
        // taken as the lanes that hold a group need (none for a single group).
        int span = 1;
        while (span < min(n_groups, 64)) span <<= 1;
        auto wsum = [&](long long x) {   // lanes >= n_groups pass 0 (and are handed the total too)
            for (int o = 1; o < span; o <<= 1) x += __shfl_xor(x, o);
            const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)x);
            const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((unsigned long long)x >> 32));
            return (long long)(((unsigned long long)hi << 32) | lo);
        };
        auto scan_excl = [&](int v, int& total) {   // the same for an exclusive prefix sum
            int x = v;
            for (int o = 1; o < span; o <<= 1) {
                const int y = __shfl_up(x, o);
                if (lane >= o) x += y;
            }
            total = span > 1 ? __shfl(x, span - 1) : __builtin_amdgcn_readfirstlane(x);
            return x - v;
        };
        const int fixed_tiles = a.split_user > 0 ? a.split_user >> 1 : 0;   // split_user is even
        // group gi's leader, members and run: the lane keeps those of group `lane` in registers
        // (every pass below starts there, and there are rarely more than 64 groups)
        int my_ld = 0, my_cnt = 0, my_run = 0;
        if (lane < n_groups) { my_ld = w.glist[lane]; my_cnt = u.c.cnt[my_ld]; my_run = u.c.run[my_ld]; }
        auto group = [&](int gi, int& ld, int& cnt, int& run) {
            if (gi == lane) { ld = my_ld; cnt = my_cnt; run = my_run; }
            else { ld = w.glist[gi]; cnt = u.c.cnt[ld]; run = u.c.run[ld]; }
        };
        long long u_loc = 0, t_loc = 0;
        for (int gi = lane; gi < n_groups; gi += 64) {
            int ld, cnt, run;
            group(gi, ld, cnt, run);
            const long long t = (long long)Hkv * by_mpt.cdiv(cnt) * ((run + 1) >> 1);
            u_loc += t * group_weight(cnt);
            t_loc += t;
        }
        const long long U = wsum(u_loc) + 16ll * T_pr, total_tiles = wsum(t_loc) + T_pr;
        const int n_act = (int)max(1ll, min((long long)a.tune.n_waves, ddiv(total_tiles, max(a.tune.min_piece, 1))));
        // Pieces of a group's run of T_seg tiles when a share may cost Q.
        auto pieces = [&](int cnt, int T_seg, int Q) {
            const int want = fixed_tiles > 0 ? fixed_tiles : max(1, idiv(max(Q - group_fixed(cnt), 0), group_weight(cnt)));
            return idiv(T_seg + want - 1, want);
        };
        // shares of the private stream at cost Q per share, and their tiles
        auto own_shares = [&](int Q, int& q) {
            const int n_pr = max(1, (int)ddiv(16ll * T_pr + Q - 1, Q));
            q = max(1, idiv(T_pr + n_pr - 1, n_pr));
            return idiv(T_pr + q - 1, q);
        };
        int Q = (int)min(1ll << 25, max(16ll, ddiv(U + n_act - 1, n_act)));   // the even split
        int q = 1, n_sh = 0;
        bool searched = false;
        if (fixed_tiles == 0 && n_groups > 0 && n_groups <= 32) {
            // Shares are whole tiles and pieces whole fractions of a run, so the even split rarely fits the waves,
            // and which cost near it does is a matter of rounding.  Every lane tries one cost for the shared
            // pieces, from 3/4 of the even split to 7/4 of it; the waves the pieces leave over share the private
            // stream; the lane whose longest share (shared piece or private share) costs least wins.
            const int Qc = Q - (Q >> 2) + (int)(((long long)Q * lane) >> 6);
            int slots = 0, longest = 0;
            for (int gi = 0; gi < n_groups; ++gi) {
                const int ld = w.glist[gi], cnt = u.c.cnt[ld], T_seg = (u.c.run[ld] + 1) >> 1;
                const int n_pc = pieces(cnt, T_seg, Qc);
                slots += items_padded(Hkv * tiles_padded(by_mpt.cdiv(cnt)) * n_pc);
                longest = max(longest, ((T_seg + n_pc - 1) / n_pc) * group_weight(cnt) + group_fixed(cnt));
            }
            int qq = 0;
            if (T_pr > 0) {
                const int n_own = min(n_act - slots, (T_pr + a.tune.min_piece - 1) / max(a.tune.min_piece, 1));
                qq = n_own >= 1 ? (T_pr + n_own - 1) / n_own : -1;
                if (qq > (1 << 26)) qq = -1;
            }
            const bool fits = slots <= n_act && qq >= 0;
            int cost = fits ? max(longest, 16 * qq) : 0x7FFFFFFF;
            int who = lane;
            for (int o = 1; o < 64; o <<= 1) {     // least cost; among equals the largest Qc (fewest pieces)
                const int c2 = __shfl_xor(cost, o), w2 = __shfl_xor(who, o);
                if (c2 < cost || (c2 == cost && w2 > who)) { cost = c2; who = w2; }
            }
            if (cost != 0x7FFFFFFF) {
                Q = __shfl(Qc, who);
                q = max(1, __shfl(qq, who));
                searched = true;
            }
        }
        // Otherwise (very many groups, or nothing fitted): start from the even split and grow the cost until
        // shared pieces plus private shares fit the waves (a wave with two shares would be the tail).
        for (int round = 0; round < 4; ++round) {
            int loc = 0;
            for (int gi = lane; gi < n_groups; gi += 64) {
                int ld, cnt, run;
                group(gi, ld, cnt, run);
                const int n_pc = pieces(cnt, (run + 1) >> 1, Q);
                v.g.npc[gi] = n_pc;
                loc += items_padded(Hkv * tiles_padded(by_mpt.cdiv(cnt)) * n_pc);
            }
            n_sh = (int)wsum(loc);
            if (fixed_tiles > 0 || searched) break;
            const int shares = n_sh + own_shares(Q, q);
            if (shares <= n_act) break;
            Q = (int)min(1ll << 25, ddiv((long long)Q * shares + n_act - 1, n_act) + 1);
        }
        // bases of the groups in list order: shares/items, segments, partial rows
        int ib = 0, sb = 0, rb = 0;
        for (int g0 = 0; g0 < n_groups; g0 += 64) {
            const int gi = g0 + lane;
            int ni = 0, nsg = 0, nr = 0;
            if (gi < n_groups) {
                int ld, cnt, run;
                group(gi, ld, cnt, run);
                nsg = Hkv * by_mpt.cdiv(cnt);
                ni = items_padded(Hkv * tiles_padded(by_mpt.cdiv(cnt)) * v.g.npc[gi]);
                nr = Hkv * v.g.npc[gi] * cnt * a.G;
            }
            int ti, ts, tr;
            const int xi = scan_excl(ni, ti), xs = scan_excl(nsg, ts), xr = scan_excl(nr, tr);
            if (gi < n_groups) {
                v.g.ibase[gi] = ib + xi;
                u.c.gseg[gi] = sb + xs;
                v.g.rbase[gi] = rb + xr;
            }
            ib += ti; sb += ts; rb += tr;
        }
        if (lane == 0) {
            s_plan[0] = fixed_tiles;
            s_plan[1] = q;
            s_plan[2] = n_sh;
            s_plan[3] = rb;
        }
    }
    __syncthreads();
    const int fixed_tiles = s_plan[0], q = s_plan[1], n_sh = s_plan[2], rows_sh = s_plan[3];

    // Cutting one segment of T_seg tiles into pieces, walking along the stream: `rem`
    // tiles of share `k` are used up at the segment's start.  Calls f(jb, je,
    // starts_share, k) for every piece, in order, and moves (k, rem) to the segment's end.
    auto for_pieces = [&](int T_seg, int& k, int& rem, auto&& f) {
        int jb = 0;
        while (jb < T_seg) {
            int take;
            bool starts = false;
            if (fixed_tiles > 0) {
                take = min(T_seg - jb, fixed_tiles);
            } else {
                take = min(T_seg - jb, q - rem);
                starts = rem == 0;
            }
            f(jb, jb + take, starts, k);
            jb += take;
            if (fixed_tiles == 0) {
                rem += take;
                if (rem == q) { rem = 0; ++k; }
            }
        }
    };
    const WideDiv by_q(max(q, 1));
    const int k_start = by_q.div(tbase), rem_start = tbase - k_start * q;

    // ---- item counts of the thread's segments, scanned in stream order
    int li = 0;
    {
        int k = k_start, rem = rem_start;
        for (int e = e0; e < e1; ++e)
            for_pieces(priv_tiles(by_hkv.div(e)), k, rem, [&](int, int, bool, int) { ++li; });
    }
    int priv_items;
    const int ibase = n_sh + block_scan_excl(li, s_tmp, priv_items);
    const int total_items = n_sh + priv_items, total_rows = rows_sh + priv_items * a.G;
    const bool overflow = total_items > a.lay.max_items || total_rows > a.lay.max_rows;

    // shares: a shared piece each, then the cuts of the private stream; with a fixed
    // split all items are dealt out in equal numbers instead
    const int n_shares = overflow ? 0 : (fixed_tiles > 0 ? min(a.tune.n_waves, total_items) : n_sh + (T_pr + q - 1) / q);
    // first item of every share: a shared piece is its own share, the private shares'
    // entries are written by whoever emits their first item (below); with a fixed split
    // the items are dealt out evenly; then the end marks
    for (int x = tid; x <= n_shares; x += kPlanThreads) {
        if (x == n_shares) wave_first[x] = overflow ? 0 : total_items;
        else if (fixed_tiles > 0) wave_first[x] = (int)ddiv((long long)x * total_items, n_shares);
        else if (x < n_sh) wave_first[x] = x;
    }
    if (tid == 0) wave_first[a.lay.max_items] = overflow ? 0 : total_items;

    // ---- descriptors and items of the requests' own columns
    {
        int k = k_start, rem = rem_start, idx = ibase;
        for (int e = e0; e < e1; ++e) {
            const int i = by_hkv.div(e), g = e - i * Hkv;
            const int L = len_of(i), nb = (L + kBlock - 1) / kBlock, c0 = run_of(i);
            if (g == 0) {
                ReqDesc rd;
                rd.ns_sh = rd.sh_base0 = rd.sh_gstride = rd.sh_pstride = 0;   // a group fills these in below
                rd.nb = nb;
                rd.L = L;
                rd.group = c0 > 0 ? (int)s_lead[i] : -1;
                rd.priv_c0 = c0;
                req[i] = rd;
            }
            const int seg_first = idx;
            if (!overflow) {
                for_pieces(((nb - c0) + 1) >> 1, k, rem, [&](int jb, int je, bool starts, int kk) {
                    const int cs = c0 + 2 * jb, ce = min(nb, c0 + 2 * je);
                    // (the piece that ends at the request's last column is marked: it grows with the request, see refresh_kernel)
                    write_item(&items[idx], i, g, a.G, ce == nb ? kOpenEnded : -1, cs, ce, rows_sh + (idx - n_sh) * a.G, min(L, ce * kBlock));
                    if (starts) wave_first[n_sh + kk] = idx;
                    ++idx;
                });
            }
            SegDesc sd;
            sd.pbase = rows_sh + (seg_first - n_sh) * a.G;
            sd.npieces = idx - seg_first;
            segs[e] = sd;
        }
    }
    // member lists of the groups (the rank lives with the thread that drew it)
    for (int k = 0, i = tid; i < nG; i += kPlanThreads, ++k) {
        const int lead = s_lead[i];
        if (lead >= 0 && viable(lead)) members[u.c.moff[lead] + my_rank[k]] = i;
    }
    __syncthreads();   // request descriptors and member lists are written: groups may amend them
    // ---- descriptors and items of the groups: one team of waves per group, its lanes
    // over the group's items (the fewer groups, the bigger the teams).
    // Order: KV head, piece, row tile - the row tiles of one piece read the same KV bytes
    // and sit on neighbouring shares, which the sweep maps to one XCD.
    if (!overflow) {
        int team = kPlanThreads / 64;   // waves per team: the largest power of two with teams >= groups (at least 1)
        while (team > 1 && (kPlanThreads / 64) / team < n_groups) team >>= 1;
        const int lstep = team * 64, l0 = tid & (lstep - 1), n_teams = kPlanThreads / lstep;
        for (int gi = tid / lstep; gi < n_groups; gi += n_teams) {
            const int ld = w.glist[gi];
            const int cnt = u.c.cnt[ld], run = u.c.run[ld];
            const int tiles_r = by_mpt.cdiv(cnt), T_seg = (run + 1) >> 1;
            const int n_pc = v.g.npc[gi];
            // tiles per piece: the fixed split's, or the run's tiles dealt out evenly (the first `extra` pieces hold one
            // more).  A short last piece would not be worth a team, and the pair of waves sweeping it on their own
            // would sit in a workgroup with a team: its barriers wait for every wave of the workgroup that is still
            // running, so that team would start only when those two had finished.
            const int ps = fixed_tiles > 0 ? fixed_tiles : T_seg / n_pc;
            const int extra = fixed_tiles > 0 ? 0 : T_seg - ps * n_pc;
            if (l0 == 0) {
                GroupDesc gd;
                gd.leader = ld;
                gd.members = cnt;
                gd.run = run;
                gd.member_off = u.c.moff[ld];
                gd.tiles = tiles_r;
                gd.seg_base = u.c.gseg[gi];
                gd.pad[0] = gd.pad[1] = 0;
                grp[ld] = gd;
            }
            const int tiles_p = tiles_padded(tiles_r);
            const int team = (teams && tiles_r >= 2) ? (tiles_r == 2 ? 2 : 4) : 0;
            const FastDiv by_tp(tiles_p), by_pc(n_pc);
            const int n = Hkv * n_pc * tiles_p, n_slots = items_padded(n);
            const int full_rows = a.mpt * a.G, last_rows = (cnt - (tiles_r - 1) * a.mpt) * a.G;
            // partial rows of segment (g, tau): pieces p = 0 .. n_pc-1, rows(tau) each; segments in (g, tau) order
            const int rows_per_head = cnt * a.G;
            for (int k = l0; k < n_slots; k += lstep) {
                Item* dst = &items[v.g.ibase[gi] + k];
                if (k >= n) {                          // filler up to the next multiple of 4: nothing to sweep
                    write_item(dst, 0, 0, 0, -1, 0, 0, 0, 0);
                    continue;
                }
                const int rest = by_tp.div(k), tau = k - rest * tiles_p;
                const int g = by_pc.div(rest), pc = rest - g * n_pc;
                const int cs = 2 * (pc * ps + min(pc, extra)), ce = min(run, cs + 2 * (ps + (pc < extra ? 1 : 0)));
                const int g_team = g | (team << 16) | ((team ? (tau & (team - 1)) : 0) << 20);   // KV head, team size, rank in the team
                if (tau >= tiles_r) {                  // no rows of its own: a team member that only fetches
                    write_item(dst, ld, g_team, 0, -1, cs, ce, 0, ce * kBlock);
                    continue;
                }
                const int rows = tau == tiles_r - 1 ? last_rows : full_rows;
                const int seg_pbase = v.g.rbase[gi] + n_pc * (g * rows_per_head + tau * full_rows);
                write_item(dst, ld, g_team, rows, u.c.moff[ld] + tau * a.mpt, cs, ce, seg_pbase + pc * rows, ce * kBlock);
                if (pc == 0) {
                    SegDesc sd;
                    sd.pbase = seg_pbase;
                    sd.npieces = n_pc;
                    segs[(size_t)B * Hkv + u.c.gseg[gi] + g * tiles_r + tau] = sd;
                }
            }
            // where each member finds the partials of the shared run (rank r = position in the member list)
            const FastDiv by_m(a.mpt);
            for (int r = l0; r < cnt; r += lstep) {
                const int i = members[u.c.moff[ld] + r];
                const int tau = by_m.div(r);
                int4 shared;
                shared.x = n_pc;
                shared.y = v.g.rbase[gi] + n_pc * tau * full_rows + (r - tau * a.mpt) * a.G;
                shared.z = n_pc * rows_per_head;
                shared.w = tau == tiles_r - 1 ? last_rows : full_rows;
                *reinterpret_cast<int4*>(&req[i]) = shared;
            }
        }
    }
    if (tid == 0) {
        hdr[H_ITEMS] = overflow ? 0 : total_items;
        hdr[H_QUEUE] = 0;
        hdr[H_GROUPS] = n_groups;
        hdr[H_GROUPED] = s_ngrouped;
        hdr[H_SPLIT] = fixed_tiles > 0 ? 2 * fixed_tiles : 2 * q;
        hdr[H_ROWS] = total_rows;
        hdr[H_SHARED_BLOCKS] = s_shared_blocks;
        hdr[H_VARIANT] = a.variant;
        hdr[H_OVERFLOW] = overflow ? 1 : 0;
        hdr[H_WAVES] = n_shares;
    }
}

// A plan made for shorter histories: the requests have grown since (decode steps append tokens, tables got
// new columns at their ends), nothing else changed.  The split of the work stays; the last piece of every
// request's own columns is stretched to the request's length now.  (Lengths that shrank would leave the plan
// wrong - attention over rows that no longer count - but never out of bounds: a piece keeps at least one tile.)
__global__ __launch_bounds__(256) void refresh_kernel(PlanArgs a) {
    const int* hdr = reinterpret_cast<const int*>(a.ws);
    Item* items = reinterpret_cast<Item*>(a.ws + a.lay.items);
    const int n_items = min(hdr[H_ITEMS], a.lay.max_items);
    const int maxL = a.stride * kBlock;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n_items; i += gridDim.x * blockDim.x) {
        const int4 w0 = reinterpret_cast<const int4*>(&items[i])[0];
        if (w0.w != kOpenEnded) continue;
        const int who = w0.x;
        if (who < 0 || who >= a.B) continue;
        int4 w1 = reinterpret_cast<const int4*>(&items[i])[1];
        const int L = max(0, min(a.seq_lens[who], maxL));
        w1.y = max((L + kBlock - 1) / kBlock, w1.x + 1);      // c1
        w1.w = max(L, w1.x * kBlock + 1);                     // tok_end
        reinterpret_cast<int4*>(&items[i])[1] = w1;
    }
    // a request that had no columns of its own then (empty, or every block shared) has no piece to stretch
    const ReqDesc* req = reinterpret_cast<const ReqDesc*>(a.ws + a.lay.req);
    const SegDesc* segs = reinterpret_cast<const SegDesc*>(a.ws + a.lay.segs);
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < a.B; i += gridDim.x * blockDim.x)
        if (segs[(size_t)i * a.Hkv].npieces == 0 && min(a.seq_lens[i], maxL) > req[i].L)
            atomicOr(reinterpret_cast<int*>(a.ws) + H_OVERFLOW, 2);
}

void launch_refresh(const PlanArgs& a, const Launch& L) {
    hipExtLaunchKernelGGL(refresh_kernel, dim3(32), dim3(256), 0, static_cast<hipStream_t>(L.stream),
                          static_cast<hipEvent_t>(L.ev_start), static_cast<hipEvent_t>(L.ev_stop), 0, a);
}

void launch_plan(const PlanArgs& a, const Launch& L) {
    hipStream_t st = static_cast<hipStream_t>(L.stream);
    hipEvent_t e0 = static_cast<hipEvent_t>(L.ev_start), e1 = static_cast<hipEvent_t>(L.ev_stop);
    if (a.pre) {   // each dispatch gets a whole pair of events; the step runs from the first start to the last stop
        hipExtLaunchKernelGGL(run_kernel, dim3(a.pre_grid), dim3(kRunThreads), 0, st, e0,
                              static_cast<hipEvent_t>(L.ev_mid[0]), 0, a);
        hipExtLaunchKernelGGL(plan_kernel, dim3(1), dim3(kPlanThreads), 0, st, static_cast<hipEvent_t>(L.ev_mid[1]), e1, 0, a);
    } else {
        hipExtLaunchKernelGGL(plan_kernel, dim3(1), dim3(kPlanThreads), 0, st, e0, e1, 0, a);
    }
}

}  // namespace fea

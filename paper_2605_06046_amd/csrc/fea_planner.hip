// Alias detection and work-list construction on the device (one workgroup).
//
// Reads only the block tables and lengths.  Requests whose table rows start with
// the same run of block ids form a group (the device-side sibling of the shared
// prefix tip of Section 4.2: the deepest level all members agree on); the run is
// swept once for the whole group, the remaining columns of each request are swept
// on their own.  A group is only a way to save KV reads: membership requires
// nothing but equal block ids over the run and full blocks for every member, so
// the result is the same attention whatever the tables look like.
#include <hip/hip_runtime.h>

#include <climits>

#include "fea_plan.h"

namespace fea {

__device__ __forceinline__ int cdiv(int a, int b) { return (a + b - 1) / b; }

// Integer division by a run-time divisor without the ~40-instruction expansion:
// exact for 0 <= x < 2^24 and 1 <= d (block and request counts are far below that).
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
        const int w = lane < 16 ? s_tmp[lane] : 0;
        int xs = w;
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) {
            const int y = __shfl_up(xs, o);
            if (lane >= o) xs += y;
        }
        if (lane < 16) s_tmp[32 + lane] = xs - w;
        if (lane == 15) s_tmp[31] = xs;
    }
    __syncthreads();
    const int base = s_tmp[32 + wave];
    total = s_tmp[31];
    __syncthreads();
    return base + x - v;
}

__device__ long long block_sum_ll(long long v, long long* s_tmp) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
    if (lane == 0) s_tmp[wave] = v;
    __syncthreads();
    long long t = 0;
#pragma unroll
    for (int w = 0; w < kPlanThreads / 64; ++w) t += s_tmp[w];
    __syncthreads();
    return t;
}

__device__ __forceinline__ uint32_t slot_of(int key) { return ((uint32_t)key * 2654435761u) >> 20; }  // 12 bits

__device__ __forceinline__ void write_item(Item* it, int kind, int who, int g, int nrows, int mlist_off, int c0, int c1,
                                           int pbase, int tok_end) {
    int4* p = reinterpret_cast<int4*>(it);
    p[0] = make_int4(who, g, nrows, mlist_off);
    p[1] = make_int4(c0, c1, pbase, tok_end);
    p[2] = make_int4(kind, 0, 0, 0);
}

__global__ __launch_bounds__(kPlanThreads) void plan_kernel(PlanArgs a) {
    static_assert(kHashSlots == 4096, "slot_of() yields 12 bits");
    __shared__ union {
        struct { int keys[kHashSlots]; int vals[kHashSlots]; } h;
        struct { int run[kGroupReqMax]; int cnt[kGroupReqMax]; int moff[kGroupReqMax]; } c;
    } u;
    __shared__ short s_lead[kGroupReqMax];      // request ids fit 16 bits (kGroupReqMax <= 32767)
    __shared__ int s_lcp[kGroupReqMax];
    __shared__ int s_len[kGroupReqMax];
    __shared__ unsigned short s_flw[kGroupReqMax];   // followers: grouped requests that are not their group's leader
    __shared__ int s_tmp[64];
    __shared__ long long s_tmpll[kPlanThreads / 64];
    __shared__ int s_glist[kGroupReqMax / 2];   // viable leaders (a group has >= 2 members)
    __shared__ int s_ngroups, s_ngrouped, s_shared_blocks, s_nflw;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int* hdr = reinterpret_cast<int*>(a.ws);
    ReqDesc* req = reinterpret_cast<ReqDesc*>(a.ws + a.lay.req);
    GroupDesc* grp = reinterpret_cast<GroupDesc*>(a.ws + a.lay.grp);
    int* members = reinterpret_cast<int*>(a.ws + a.lay.members);
    Item* items = reinterpret_cast<Item*>(a.ws + a.lay.items);

    const int B = a.B;
    const int nG = a.grouping ? min(B, kGroupReqMax) : 0;
    const int maxL = a.stride * kBlock;
    auto clampL = [&](int L) { return max(0, min(L, maxL)); };

    // ---- leaders: smallest request index among those with the same first block
    for (int s = tid; s < kHashSlots; s += kPlanThreads) { u.h.keys[s] = -1; u.h.vals[s] = INT_MAX; }
    if (tid == 0) { s_ngroups = 0; s_ngrouped = 0; s_shared_blocks = 0; s_nflw = 0; }
    __syncthreads();
    int my_key[kGroupReqMax / kPlanThreads];
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
                if (lead != i) s_flw[atomicAdd(&s_nflw, 1)] = (unsigned short)i;
            }
            s_lead[i] = (short)lead;
            s_lcp[i] = lcp;
        }
    }
    __syncthreads();   // the hash table is dead from here on; its memory becomes run/cnt/moff
    for (int i = tid; i < nG; i += kPlanThreads) { u.c.run[i] = INT_MAX; u.c.cnt[i] = 0; u.c.moff[i] = 0; }

    // ---- longest common run of block ids with the leader's row.  All (follower,
    // column group) pairs are spread flat over the threads, four at a time so that
    // their loads are in flight together; a mismatch lowers the follower's run with
    // an LDS atomic.
    {
        const int nflw = s_nflw;
        const bool vec = (a.stride % 4 == 0) && ((reinterpret_cast<uintptr_t>(a.bt) & 15) == 0);
        const int cpe = vec ? 4 : 1;                       // columns per element
        const int epr = cdiv(a.stride, cpe);               // elements per row
        const FastDiv by_epr(max(epr, 1));
        const int total = nflw * epr;
        for (int e0 = tid; e0 < total; e0 += 4 * kPlanThreads) {
            int4 xs[4], ys[4];
            int who[4], col[4], cap[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int e = e0 + q * kPlanThreads;
                who[q] = -1;
                if (e < total) {
                    const int f = by_epr.div(e);
                    const int i = s_flw[f];
                    const int lead = s_lead[i];
                    const int c = (e - f * epr) * cpe;
                    const int cp = min(s_len[i], s_len[lead]) / kBlock;   // the starting value of s_lcp[i]
                    if (c < cp) {
                        who[q] = i; col[q] = c; cap[q] = cp;
                        const int32_t* ri = a.bt + (size_t)i * a.stride + c;
                        const int32_t* rl = a.bt + (size_t)lead * a.stride + c;
                        if (vec) {
                            xs[q] = *reinterpret_cast<const int4*>(ri);
                            ys[q] = *reinterpret_cast<const int4*>(rl);
                        } else {
                            xs[q] = make_int4(*ri, 0, 0, 0);
                            ys[q] = make_int4(*rl, 0, 0, 0);
                        }
                    }
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (who[q] >= 0) {
                    int first = INT_MAX;
                    if (xs[q].w != ys[q].w) first = col[q] + 3;
                    if (xs[q].z != ys[q].z) first = col[q] + 2;
                    if (xs[q].y != ys[q].y) first = col[q] + 1;
                    if (xs[q].x != ys[q].x) first = col[q];
                    if (first < cap[q]) atomicMin(&s_lcp[who[q]], first);
                }
            }
        }
    }
    __syncthreads();

    // ---- group run = shortest common run over the members; rank = arrival at the counter
    int my_rank[kGroupReqMax / kPlanThreads];
#pragma unroll
    for (int k = 0; k < kGroupReqMax / kPlanThreads; ++k) {
        const int i = tid + k * kPlanThreads;
        my_rank[k] = 0;
        if (i < nG) {
            const int lead = s_lead[i];
            if (lead >= 0) {
                atomicMin(&u.c.run[lead], s_lcp[i]);
                my_rank[k] = atomicAdd(&u.c.cnt[lead], 1);
            }
        }
    }
    __syncthreads();
    auto viable = [&](int i) { return s_lead[i] == i && u.c.cnt[i] >= 2 && u.c.run[i] >= a.tune.min_run; };
    const FastDiv by_mpt(a.mpt);

    // ---- member-list offsets (exclusive scan over leaders)
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
                const int gi = atomicAdd(&s_ngroups, 1);
                s_glist[gi] = i;
                atomicAdd(&s_shared_blocks, u.c.run[i]);
            }
        if (tid == 0) s_ngrouped = total;
    }
    __syncthreads();

    // ---- totals that fix the split size; member lists (grouped part, then identity)
    long long w_local = 0, rb_local = 0;
    for (int k = 0, i = tid; i < B; i += kPlanThreads, ++k) {
        const int nb = ((i < nG ? s_len[i] : clampL(a.seq_lens[i])) + kBlock - 1) / kBlock;
        int run_i = 0;
        if (i < nG) {
            const int lead = s_lead[i];
            if (lead >= 0 && viable(lead)) {
                run_i = u.c.run[lead];
                members[u.c.moff[lead] + my_rank[k]] = i;
            }
            if (viable(i)) w_local += (long long)u.c.run[i] * a.Hkv * by_mpt.cdiv(u.c.cnt[i]);
        }
        members[B + i] = i;
        w_local += (long long)(nb - run_i) * a.Hkv;
        rb_local += (long long)nb * a.Hq;
    }
    const long long W = block_sum_ll(w_local, s_tmpll);
    const long long RB = block_sum_ll(rb_local, s_tmpll);
    int split = a.split_user;
    if (split <= 0) {
        long long s = a.tune.min_split;
        s = max(s, (W + a.tune.target_items - 1) / a.tune.target_items);
        s = max(s, (RB + a.tune.row_budget - 1) / a.tune.row_budget);
        split = (int)min(s, (long long)INT_MAX / 64);
    }
    split = (split + 1) & ~1;   // sweeps advance two blocks at a time
    const FastDiv by_split(split);

    // ---- per-segment item and partial-row counts, scanned: groups first, then requests
    const int N = nG + B;
    const int per = (N + kPlanThreads - 1) / kPlanThreads;
    const int e0 = tid * per, e1 = min(N, e0 + per);
    auto seg_counts = [&](int e, int& n_items, int& n_rows, int& nsplits, int& c0, int& L) {
        n_items = n_rows = nsplits = c0 = L = 0;
        if (e < nG) {
            if (viable(e)) {
                nsplits = by_split.cdiv(u.c.run[e]);
                n_items = a.Hkv * by_mpt.cdiv(u.c.cnt[e]) * nsplits;
                n_rows = nsplits * u.c.cnt[e] * a.Hq;
            }
        } else {
            const int i = e - nG;
            L = i < nG ? s_len[i] : clampL(a.seq_lens[i]);
            if (i < nG) {
                const int lead = s_lead[i];
                if (lead >= 0 && viable(lead)) c0 = u.c.run[lead];
            }
            nsplits = by_split.cdiv((L + kBlock - 1) / kBlock - c0);
            n_items = a.Hkv * nsplits;
            n_rows = nsplits * a.Hq;
        }
    };
    int li = 0, lr = 0;
    for (int e = e0; e < e1; ++e) {
        int ni, nr, ns, c0, L;
        seg_counts(e, ni, nr, ns, c0, L);
        li += ni;
        lr += nr;
    }
    int total_items, total_rows;
    int ibase = block_scan_excl(li, s_tmp, total_items);
    int rbase = block_scan_excl(lr, s_tmp, total_rows);
    const bool overflow = total_items > a.lay.max_items || total_rows > a.lay.max_rows;

    for (int e = e0; e < e1; ++e) {
        int ni, nr, ns, c0, L;
        seg_counts(e, ni, nr, ns, c0, L);
        if (e < nG) {
            const bool ok = viable(e);
            GroupDesc gd;
            gd.leader = e;
            gd.members = ok ? u.c.cnt[e] : 0;
            gd.run = ok ? u.c.run[e] : 0;
            gd.nsplits = ns;
            gd.pbase = rbase;
            gd.member_off = u.c.moff[e];
            gd.tiles = ok ? by_mpt.cdiv(u.c.cnt[e]) : 0;
            gd.item_base = ibase;
            grp[e] = gd;
        } else {
            const int i = e - nG;
            const int nb = (L + kBlock - 1) / kBlock;
            ReqDesc rd;
            rd.group = -1;
            rd.rank = 0;
            if (i < nG) {
                const int lead = s_lead[i];
                if (lead >= 0 && viable(lead)) rd.group = lead;
            }
            rd.priv_c0 = c0;
            rd.priv_nsplits = ns;
            rd.priv_pbase = rbase;
            rd.nb = nb;
            rd.L = L;
            rd.priv_item_base = ibase;
            req[i] = rd;
            if (!overflow) {
                // private items of one request: KV head fastest, so that a request's
                // heads (which read the same blocks' other head slices) run together
                Item* dst = items + ibase;
                for (int s = 0; s < ns; ++s) {
                    const int cs = c0 + s * split, ce = min(nb, cs + split);
                    for (int g = 0; g < a.Hkv; ++g)
                        write_item(dst++, 0, i, g, a.G, B + i, cs, ce, rbase + s * a.Hq + g * a.G, min(L, ce * kBlock));
                }
            }
        }
        ibase += ni;
        rbase += nr;
    }
    __syncthreads();
    // ranks live with the thread that drew them
#pragma unroll
    for (int k = 0; k < kGroupReqMax / kPlanThreads; ++k) {
        const int i = tid + k * kPlanThreads;
        if (i < nG) {
            const int lead = s_lead[i];
            if (lead >= 0 && viable(lead)) req[i].rank = my_rank[k];
        }
    }
    // shared items: one wave per group, row tile fastest so that the tiles of one
    // (split, KV head), which read the same KV bytes, are handed out back to back
    if (!overflow) {
        for (int gi = wave; gi < s_ngroups; gi += kPlanThreads / 64) {
            const int e = s_glist[gi];
            const int members_g = u.c.cnt[e], run_g = u.c.run[e];
            const int tiles = by_mpt.cdiv(members_g), nsplits = by_split.cdiv(run_g);
            const GroupDesc gd = grp[e];   // for pbase / item_base (written above, visible after the barrier)
            const FastDiv by_tiles(tiles), by_hkv(a.Hkv);
            const int n = a.Hkv * tiles * nsplits;
            for (int k = lane; k < n; k += 64) {
                const int rest = by_tiles.div(k), tau = k - rest * tiles;
                const int s = by_hkv.div(rest), g = rest - s * a.Hkv;
                const int cs = s * split, ce = min(run_g, cs + split);
                const int first = tau * a.mpt;
                const int pb = gd.pbase + (s * a.Hkv + g) * members_g * a.G + first * a.G;
                write_item(&items[gd.item_base + k], 1, e, g, min(a.mpt, members_g - first) * a.G, gd.member_off + first,
                           cs, ce, pb, ce * kBlock);
            }
        }
    }
    if (tid == 0) {
        hdr[H_ITEMS] = overflow ? 0 : total_items;
        hdr[H_QUEUE] = 0;
        hdr[H_GROUPS] = s_ngroups;
        hdr[H_GROUPED] = s_ngrouped;
        hdr[H_SPLIT] = split;
        hdr[H_ROWS] = total_rows;
        hdr[H_SHARED_BLOCKS] = s_shared_blocks;
        hdr[H_VARIANT] = a.variant;
        hdr[H_OVERFLOW] = overflow ? 1 : 0;
    }
}

void launch_plan(const PlanArgs& a, void* stream) {
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(kPlanThreads), 0, static_cast<hipStream_t>(stream), a);
}

}  // namespace fea

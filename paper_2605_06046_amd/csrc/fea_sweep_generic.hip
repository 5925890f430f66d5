// Generic KV sweep (plain vector ALU) and the merge of partial results.
//
// The generic sweep serves float32 caches and every shape the MFMA sweep does not
// take.  One workgroup per work item; scores of a 256-token piece are staged in
// LDS, the softmax runs online across pieces (running maximum and sum), and the
// value accumulation is reduced across the workgroup at the end.  Everything is
// float32; scores are kept in the base-2 domain (score * scale * log2 e) so that
// the exponential is a bare v_exp_f32.
//
// Computes, for the item's token range R and each query head h of its KV head:
//   m = max_{t in R} s_t,  l = sum_t 2^(s_t - m),  acc = sum_t 2^(s_t - m) v_t
// with s_t = (q_h . k_t) * scale * log2(e)  -- the pieces of
// softmax(q K^T / sqrt(d)) V (Section 2.1) that the merge kernel combines.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <type_traits>

#include "../../include/fea.h"
#include "fea_plan.h"

namespace fea {

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int kPerLoad = 4;   // elements in one 16-byte load
    using Raw = float4;                  // the 16 bytes as loaded
    __device__ static Raw load_raw(const float* p) { return *reinterpret_cast<const float4*>(p); }
    __device__ static void unpack(const Raw& v, float (&f)[4]) { f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w; }
    __device__ static void load(const float* p, float (&f)[4]) { unpack(load_raw(p), f); }
    __device__ static void store(float* p, float v) { *p = v; }
    __device__ static void store8(float* p, const float (&v)[8]) {   // p is 32-byte aligned
        reinterpret_cast<float4*>(p)[0] = make_float4(v[0], v[1], v[2], v[3]);
        reinterpret_cast<float4*>(p)[1] = make_float4(v[4], v[5], v[6], v[7]);
    }
};
struct bf16_t { uint16_t bits; };
template <> struct Elem<bf16_t> {
    static constexpr int kPerLoad = 8;
    using Raw = uint4;
    __device__ static Raw load_raw(const bf16_t* p) { return *reinterpret_cast<const uint4*>(p); }
    __device__ static void unpack(const Raw& v, float (&f)[8]) {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            f[2 * k] = __uint_as_float(w[k] << 16);
            f[2 * k + 1] = __uint_as_float(w[k] & 0xFFFF0000u);
        }
    }
    __device__ static void load(const bf16_t* p, float (&f)[8]) { unpack(load_raw(p), f); }
    __device__ static void store(bf16_t* p, float v) {   // round to nearest even
        uint32_t u = __float_as_uint(v);
        if ((u & 0x7FFFFFFFu) > 0x7F800000u) { p->bits = 0x7FC0; return; }
        u += 0x7FFFu + ((u >> 16) & 1u);
        p->bits = (uint16_t)(u >> 16);
    }
    __device__ static void store8(bf16_t* p, const float (&v)[8]) {   // p is 16-byte aligned: one store
        bf16_t h[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) store(&h[k], v[k]);
        uint4 w;
        w.x = h[0].bits | ((uint32_t)h[1].bits << 16);
        w.y = h[2].bits | ((uint32_t)h[3].bits << 16);
        w.z = h[4].bits | ((uint32_t)h[5].bits << 16);
        w.w = h[6].bits | ((uint32_t)h[7].bits << 16);
        *reinterpret_cast<uint4*>(p) = w;
    }
};

constexpr int kGenThreads = 256;
constexpr int kGenWaves = kGenThreads / 64;
constexpr int kPiece = 256;   // tokens whose scores are staged at once

// Query rows handled per pass over an item's tokens: the item's rows are its members' query heads stacked
// (member-major), so a pass over a shared run serves several members at once (Section 3: the run is read
// once for all who attend to it - here once per pass, and the passes after the first hit L2).  Two
// instantiations: 4 rows per pass (few registers, four workgroups per compute unit: what a batch that
// fills the chip wants, being bound by memory latency) and WIDE = 16 rows (8 for 16-bit caches, fewer for
// head_dim 256) for batches too small to fill it, where the number of passes is all that counts.
template <typename T, int D> constexpr int gen_rows_wide() {
    return (sizeof(T) == 4 ? 16 : 8) > 2048 / D ? 2048 / D : (sizeof(T) == 4 ? 16 : 8);
}

template <typename T, int D, int HB>
__global__ __launch_bounds__(kGenThreads) void sweep_generic_kernel(SweepArgs a) {
    constexpr int EPL = Elem<T>::kPerLoad;
    constexpr int LPT = D / EPL;          // lanes that share one token row
    constexpr int TPW = 64 / LPT;         // token rows per wave-wide load
    static_assert(LPT >= 1 && LPT <= 64 && (LPT & (LPT - 1)) == 0, "head_dim not supported");

    __shared__ float s_sc[HB][kPiece];
    __shared__ float s_alpha[HB], s_m[HB], s_l[HB];
    __shared__ float s_red[kGenWaves][HB][D];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane % LPT, r = lane / LPT;
    const int* hdr = reinterpret_cast<const int*>(a.ws);
    const Item* items = reinterpret_cast<const Item*>(a.ws + a.lay.items);
    float2* ml = reinterpret_cast<float2*>(a.ws + a.lay.ml);
    float* pacc = reinterpret_cast<float*>(a.ws + a.lay.acc);
    const T* Q = static_cast<const T*>(a.q);
    const T* K = static_cast<const T*>(a.k_cache);
    const T* V = static_cast<const T*>(a.v_cache);
    const int n_items = hdr[H_ITEMS];

    for (int it = blockIdx.x; it < n_items; it += gridDim.x) {
        const Item item = items[it];
        const int32_t* row = a.bt + (size_t)item.who * a.stride;
        const int t_begin = item.c0 * kBlock, t_end = item.tok_end;
        // query rows of the item: one request's query group, or those of the members of a group's row tile
        const int* mlist = reinterpret_cast<const int*>(a.ws + a.lay.members) + item.mlist_off;
        // one pass over the item's tokens for rows row0 .. row0 + RB - 1 (RB: a compile-time bound, so that the
        // rows' registers are arrays the compiler can keep in registers)
        auto pass = [&](auto rb_tag, int row0) {
            constexpr int RB = decltype(rb_tag)::value;
            const int prow0 = item.pbase + row0;
            const int nh = min(RB, item.nrows - row0);
            float qf[RB][EPL];
#pragma unroll
            for (int j = 0; j < RB; ++j) {
                if (j < nh) {
                    const int ra = row0 + j, mem = ra / a.G, hh = ra - mem * a.G;
                    const int qreq = item.mlist_off < 0 ? item.who : mlist[mem];
                    Elem<T>::load(Q + ((size_t)qreq * a.Hq + item.g * a.G + hh) * D + c * EPL, qf[j]);
                } else {
#pragma unroll
                    for (int e = 0; e < EPL; ++e) qf[j][e] = 0.f;
                }
            }
            float acc[RB][EPL];
#pragma unroll
            for (int j = 0; j < RB; ++j)
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[j][e] = 0.f;
            constexpr int RPW = (RB + kGenWaves - 1) / kGenWaves;   // rows whose softmax state one wave keeps
            float m_run[RPW], l_run[RPW];   // of rows wave, wave + kGenWaves, ...
#pragma unroll
            for (int k = 0; k < RPW; ++k) { m_run[k] = -INFINITY; l_run[k] = 0.f; }

            for (int p0 = t_begin; p0 < t_end; p0 += kPiece) {
                const int np = min(kPiece, t_end - p0);
                // scores
                for (int tt = wave * TPW + r; tt < np; tt += kGenWaves * TPW) {
                    const int t = p0 + tt;
                    const int blk = max(row[t / kBlock], 0);   // a -1 inside a request's length (the caller's error) must not become a read before the cache
                    float kf[EPL];
                    Elem<T>::load(K + (((size_t)blk * a.Hkv + item.g) * kBlock + (t % kBlock)) * D + c * EPL, kf);
                    float dot[RB];
#pragma unroll
                    for (int j = 0; j < RB; ++j) {
                        float s = 0.f;
#pragma unroll
                        for (int e = 0; e < EPL; ++e) s = fmaf(qf[j][e], kf[e], s);
                        dot[j] = s;
                    }
#pragma unroll
                    for (int o = LPT / 2; o >= 1; o >>= 1)
#pragma unroll
                        for (int j = 0; j < RB; ++j) dot[j] += __shfl_xor(dot[j], o);
                    if (c == 0) {
#pragma unroll
                        for (int j = 0; j < RB; ++j) s_sc[j][tt] = dot[j] * a.scale_log2;
                    }
                }
                __syncthreads();
                // softmax bookkeeping: wave w owns rows w, w + kGenWaves, ...
#pragma unroll
                for (int k = 0; k < RPW; ++k) {
                    const int j = wave + k * kGenWaves;
                    if (j < nh) {
                        float mx = -INFINITY;
                        for (int tt = lane; tt < np; tt += 64) mx = fmaxf(mx, s_sc[j][tt]);
#pragma unroll
                        for (int o = 32; o >= 1; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
                        const float m_new = fmaxf(m_run[k], mx);
                        float sum = 0.f;
                        for (int tt = lane; tt < np; tt += 64) {
                            const float p = exp2f(s_sc[j][tt] - m_new);
                            s_sc[j][tt] = p;
                            sum += p;
                        }
#pragma unroll
                        for (int o = 32; o >= 1; o >>= 1) sum += __shfl_xor(sum, o);
                        const float alpha = exp2f(m_run[k] - m_new);   // 0 on the first piece
                        l_run[k] = l_run[k] * alpha + sum;
                        m_run[k] = m_new;
                        if (lane == 0) { s_alpha[j] = alpha; s_m[j] = m_new; s_l[j] = l_run[k]; }
                    }
                }
                __syncthreads();
                // values
#pragma unroll
                for (int j = 0; j < RB; ++j) {
                    const float al = j < nh ? s_alpha[j] : 0.f;
#pragma unroll
                    for (int e = 0; e < EPL; ++e) acc[j][e] *= al;
                }
                for (int tt = wave * TPW + r; tt < np; tt += kGenWaves * TPW) {
                    const int t = p0 + tt;
                    const int blk = max(row[t / kBlock], 0);   // a -1 inside a request's length (the caller's error) must not become a read before the cache
                    float vf[EPL];
                    Elem<T>::load(V + (((size_t)blk * a.Hkv + item.g) * kBlock + (t % kBlock)) * D + c * EPL, vf);
#pragma unroll
                    for (int j = 0; j < RB; ++j) {
                        if (j < nh) {
                            const float p = s_sc[j][tt];
#pragma unroll
                            for (int e = 0; e < EPL; ++e) acc[j][e] = fmaf(p, vf[e], acc[j][e]);
                        }
                    }
                }
                __syncthreads();
            }
            // reduce the value sums over the token rows of a wave, then over waves
#pragma unroll
            for (int o = LPT; o < 64; o <<= 1)
#pragma unroll
                for (int j = 0; j < RB; ++j)
#pragma unroll
                    for (int e = 0; e < EPL; ++e) acc[j][e] += __shfl_xor(acc[j][e], o);
            if (r == 0) {
#pragma unroll
                for (int j = 0; j < RB; ++j)
#pragma unroll
                    for (int e = 0; e < EPL; ++e) s_red[wave][j][c * EPL + e] = acc[j][e];
            }
            __syncthreads();
            for (int x = tid; x < nh * D; x += kGenThreads) {
                const int j = x / D, e = x % D;
                float s = 0.f;
#pragma unroll
                for (int w = 0; w < kGenWaves; ++w) s += s_red[w][j][e];
                pacc[(size_t)(prow0 + j) * D + e] = s;
            }
            if (tid < nh) ml[prow0 + tid] = make_float2(s_m[tid], s_l[tid]);
            __syncthreads();
        };
        if (HB > 4 && item.nrows <= 4) {
            pass(std::integral_constant<int, 4>{}, 0);      // a request's own columns with a query group of up to 4 heads
        } else {
            for (int row0 = 0; row0 < item.nrows; row0 += HB) pass(std::integral_constant<int, HB>{}, row0);
        }
    }
}

// out[i,h,:] = sum_s 2^(m_s - M) acc_s / sum_s 2^(m_s - M) l_s over the partials
// of row (i,h): the pieces of its group's shared run, then the pieces of the
// request's own columns.  One wave per row; the wave is cut into SLOTS groups of
// D/8 lanes, each group takes every SLOTS-th partial (8 floats per lane, so that a
// group reads a whole 4*D-byte partial row in one go and several rows are in
// flight), and the groups are folded together at the end.
template <typename T, int D>
__global__ __launch_bounds__(256) void merge_kernel(SweepArgs a) {
    constexpr int LPR = D / 8;           // lanes per partial row
    constexpr int SLOTS = 64 / LPR;
    const int lane = threadIdx.x & 63;
    const int rowid = blockIdx.x * 4 + (threadIdx.x >> 6);
    int* hdr = reinterpret_cast<int*>(a.ws);
    if (rowid >= a.B * a.Hq) return;
    const int i = rowid / a.Hq, h = rowid - i * a.Hq;
    const int g = h / a.G, hh = h - g * a.G;
    // (the first four words of the request's descriptor, taken as values: a reference to the whole struct would put it on the stack)
    const int4 rd4 = *reinterpret_cast<const int4*>(a.ws + a.lay.req + (size_t)i * sizeof(ReqDesc));
    const int rd_ns_sh = rd4.x, rd_sh_base0 = rd4.y, rd_sh_gstride = rd4.z, rd_sh_pstride = rd4.w;
    const SegDesc pd = reinterpret_cast<const SegDesc*>(a.ws + a.lay.segs)[(size_t)i * a.Hkv + g];
    const float2* ml = reinterpret_cast<const float2*>(a.ws + a.lay.ml);
    const float* pacc = reinterpret_cast<const float*>(a.ws + a.lay.acc);
    T* out = static_cast<T*>(a.out) + (size_t)rowid * D;
    const int c = lane % LPR, slot = lane / LPR;

    if (hdr[H_OVERFLOW]) {   // the plan did not fit its buffers: make it loud
        for (int e = lane; e < D; e += 64) Elem<T>::store(out + e, __uint_as_float(0x7FC00000u));
        return;
    }
    const int ns_sh = rd_ns_sh, ns = ns_sh + pd.npieces;
    const int sh_base = rd_sh_base0 + g * rd_sh_gstride + hh, pr_base = pd.pbase + hh;
    auto prow = [&](int s) { return s < ns_sh ? sh_base + s * rd_sh_pstride : pr_base + (s - ns_sh) * a.G; };

    // Each lane group walks its partials kInFlight at a time: their (m, l) pairs and
    // accumulator rows are requested together, so a row with up to kInFlight * SLOTS
    // partials costs one memory round trip.  A group keeps its own reference exponent
    // (raised batch by batch); the groups are brought to the common one when folded.
    constexpr int kInFlight = 4;
    float num[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) num[k] = 0.f;
    float den = 0.f, M = -INFINITY;
    for (int s0 = 0; s0 < ns; s0 += kInFlight * SLOTS) {
        float4 x[kInFlight][2];
        float2 v[kInFlight];
        float mb = -INFINITY;
#pragma unroll
        for (int q = 0; q < kInFlight; ++q) {
            const int s = s0 + q * SLOTS + slot;
            v[q] = make_float2(-INFINITY, 0.f);
            x[q][0] = x[q][1] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (s < ns) {
                const int pr = prow(s);
                v[q] = ml[pr];
                const float4* src = reinterpret_cast<const float4*>(pacc + (size_t)pr * D + c * 8);
                x[q][0] = src[0];
                x[q][1] = src[1];
            }
        }
#pragma unroll
        for (int q = 0; q < kInFlight; ++q) mb = fmaxf(mb, v[q].x);
        const float Mn = fmaxf(M, mb);
        if (Mn > M) {                                   // raise the group's reference (a no-op on empty sums)
            const float f = M == -INFINITY ? 0.f : exp2f(M - Mn);
            den *= f;
#pragma unroll
            for (int k = 0; k < 8; ++k) num[k] *= f;
            M = Mn;
        }
#pragma unroll
        for (int q = 0; q < kInFlight; ++q) {
            const float w = v[q].x == -INFINITY ? 0.f : exp2f(v[q].x - M);
            den = fmaf(w, v[q].y, den);
            num[0] = fmaf(w, x[q][0].x, num[0]); num[1] = fmaf(w, x[q][0].y, num[1]);
            num[2] = fmaf(w, x[q][0].z, num[2]); num[3] = fmaf(w, x[q][0].w, num[3]);
            num[4] = fmaf(w, x[q][1].x, num[4]); num[5] = fmaf(w, x[q][1].y, num[5]);
            num[6] = fmaf(w, x[q][1].z, num[6]); num[7] = fmaf(w, x[q][1].w, num[7]);
        }
    }
    // fold the lane groups (fixed order: deterministic) at the common reference
    {
        float Mg = M;
#pragma unroll
        for (int o = LPR; o < 64; o <<= 1) Mg = fmaxf(Mg, __shfl_xor(Mg, o));
        const float f = M == -INFINITY ? 0.f : exp2f(M - Mg);
        den *= f;
#pragma unroll
        for (int k = 0; k < 8; ++k) num[k] *= f;
    }
#pragma unroll
    for (int o = LPR; o < 64; o <<= 1) {
        den += __shfl_xor(den, o);
#pragma unroll
        for (int k = 0; k < 8; ++k) num[k] += __shfl_xor(num[k], o);
    }
    if (slot == 0) {
        const float inv = den > 0.f ? 1.f / den : 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k) num[k] *= inv;
        Elem<T>::store8(out + c * 8, num);
    }
}

// The same merge for batches of very many rows with few partials each (hundreds of requests
// that share nothing: one or two pieces per row): a wave takes 64 / (D/8) rows, one per lane
// group, each group walking its own row's partials four at a time.  A quarter (D = 128) of the
// waves of merge_kernel, which there spends its time starting waves that fetch one partial.
template <typename T, int D>
__global__ __launch_bounds__(256) void merge_rows_kernel(SweepArgs a) {
    constexpr int LPR = D / 8;           // lanes per row
    constexpr int SLOTS = 64 / LPR;      // rows per wave
    const int lane = threadIdx.x & 63, c = lane % LPR;
    const int rowid = (blockIdx.x * 4 + (threadIdx.x >> 6)) * SLOTS + lane / LPR;
    const int* hdr = reinterpret_cast<const int*>(a.ws);
    if (rowid >= a.B * a.Hq) return;     // nothing below crosses lane groups
    const int i = rowid / a.Hq, h = rowid - i * a.Hq;
    const int g = h / a.G, hh = h - g * a.G;
    // (the first four words of the request's descriptor, taken as values: a reference to the whole struct would put it on the stack)
    const int4 rd4 = *reinterpret_cast<const int4*>(a.ws + a.lay.req + (size_t)i * sizeof(ReqDesc));
    const int rd_ns_sh = rd4.x, rd_sh_base0 = rd4.y, rd_sh_gstride = rd4.z, rd_sh_pstride = rd4.w;
    const SegDesc pd = reinterpret_cast<const SegDesc*>(a.ws + a.lay.segs)[(size_t)i * a.Hkv + g];
    const float2* ml = reinterpret_cast<const float2*>(a.ws + a.lay.ml);
    const float* pacc = reinterpret_cast<const float*>(a.ws + a.lay.acc);
    T* out = static_cast<T*>(a.out) + (size_t)rowid * D;
    if (hdr[H_OVERFLOW]) {   // the plan did not fit its buffers: make it loud
        for (int e = c; e < D; e += LPR) Elem<T>::store(out + e, __uint_as_float(0x7FC00000u));
        return;
    }
    const int ns_sh = rd_ns_sh, ns = ns_sh + pd.npieces;
    const int sh_base = rd_sh_base0 + g * rd_sh_gstride + hh, pr_base = pd.pbase + hh;
    auto prow = [&](int s) { return s < ns_sh ? sh_base + s * rd_sh_pstride : pr_base + (s - ns_sh) * a.G; };
    constexpr int kInFlight = 4;
    float num[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) num[k] = 0.f;
    float den = 0.f, M = -INFINITY;
    for (int s0 = 0; s0 < ns; s0 += kInFlight) {
        float4 x[kInFlight][2];
        float2 v[kInFlight];
        float mb = -INFINITY;
#pragma unroll
        for (int q = 0; q < kInFlight; ++q) {
            const int s = s0 + q;
            v[q] = make_float2(-INFINITY, 0.f);
            x[q][0] = x[q][1] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (s < ns) {
                const int pr = prow(s);
                v[q] = ml[pr];
                const float4* src = reinterpret_cast<const float4*>(pacc + (size_t)pr * D + c * 8);
                x[q][0] = src[0];
                x[q][1] = src[1];
            }
        }
#pragma unroll
        for (int q = 0; q < kInFlight; ++q) mb = fmaxf(mb, v[q].x);
        const float Mn = fmaxf(M, mb);
        if (Mn > M) {
            const float f = M == -INFINITY ? 0.f : exp2f(M - Mn);
            den *= f;
#pragma unroll
            for (int k = 0; k < 8; ++k) num[k] *= f;
            M = Mn;
        }
#pragma unroll
        for (int q = 0; q < kInFlight; ++q) {
            const float w = v[q].x == -INFINITY ? 0.f : exp2f(v[q].x - M);
            den = fmaf(w, v[q].y, den);
            num[0] = fmaf(w, x[q][0].x, num[0]); num[1] = fmaf(w, x[q][0].y, num[1]);
            num[2] = fmaf(w, x[q][0].z, num[2]); num[3] = fmaf(w, x[q][0].w, num[3]);
            num[4] = fmaf(w, x[q][1].x, num[4]); num[5] = fmaf(w, x[q][1].y, num[5]);
            num[6] = fmaf(w, x[q][1].z, num[6]); num[7] = fmaf(w, x[q][1].w, num[7]);
        }
    }
    const float inv = den > 0.f ? 1.f / den : 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) num[k] *= inv;
    Elem<T>::store8(out + c * 8, num);
}

// The whole call in one launch, for batches too small to be worth a plan, a sweep and a merge of their
// own (a few requests with short histories, where three dependent launches and the planner's one
// workgroup cost several times what the attention does).  One workgroup per (request, KV head) walks the
// request's whole history: every lane group keeps the online-softmax state (m, l, acc) of the token rows it
// visits - several rows in flight per lane, requested together and folded into the state with one
// change of the reference exponent - and the states are folded over the wave's lane groups, then over
// the waves through LDS, normalised and written as out[i, h, :] = softmax(q K^T * scale) V (Section 2.1).
// No plan is read or made: a block that several requests alias is read once per request, out of L2
// after the first.
constexpr int kSmallThreads = 512;
constexpr int kSmallWaves = kSmallThreads / 64;
// Query heads per pass over the history and token rows a lane has in flight: 4 and 8, or - for query groups of
// more than 4 heads over float32 caches, where the number of passes counts - 8 and 4 (the registers hold one or
// the other; with 16-bit caches a lane carries 8 elements per head, and 8 heads do not fit).
constexpr int kSmallCols = 512;    // table entries of the request kept in LDS (longer rows read the rest from memory)

template <typename T, int D, int RB>
__global__ __launch_bounds__(kSmallThreads) void decode_small_kernel(SweepArgs a) {
    constexpr int EPL = Elem<T>::kPerLoad;
    constexpr int LPT = D / EPL;          // lanes that share one token row
    constexpr int TPW = 64 / LPT;         // token rows per wave-wide load
    constexpr int U = RB == 4 ? 8 : 4;
    static_assert(RB == 4 || RB == 8, "4 or 8 query heads per pass");
    using Raw = typename Elem<T>::Raw;
    __shared__ float s_acc[kSmallWaves][RB][D];
    __shared__ float2 s_ml[kSmallWaves][RB];
    __shared__ int s_row[kSmallCols];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane % LPT, r = lane / LPT;
    const int i = blockIdx.x / a.Hkv, g = blockIdx.x - i * a.Hkv;
    if (blockIdx.x == 0 && tid < H_WORDS)   // what a later look at the workspace finds: no plan, this kernel
        reinterpret_cast<int*>(a.ws)[tid] = tid == H_VARIANT ? 2 : tid == H_WAVES ? (int)gridDim.x * kSmallWaves : 0;
    const int L = min(max(a.seq_lens[i], 0), a.stride * kBlock);
    const int32_t* row = a.bt + (size_t)i * a.stride;
    const T* Q = static_cast<const T*>(a.q) + ((size_t)i * a.Hq + g * a.G) * D;
    const T* K = static_cast<const T*>(a.k_cache);
    const T* V = static_cast<const T*>(a.v_cache);
    T* out = static_cast<T*>(a.out) + ((size_t)i * a.Hq + g * a.G) * D;
    // (a -1 inside a request's length - the caller's error - must not become a read before the cache)
    for (int x = tid; x < min((L + kBlock - 1) / kBlock, kSmallCols); x += kSmallThreads) s_row[x] = max(row[x], 0);
    __syncthreads();

    // A query group of more than RB heads takes several passes over the history.  They run side by side where they
    // can: the 8 waves form 2, 4 or 8 sets, each set with a pass of its own over all tokens (the work per wave is
    // the same as with one pass after the other on all waves, but the fixed part of a pass - the dependent loads at
    // its start, the folds at its end - is paid once for the passes of a round).
    const int passes = (a.G + RB - 1) / RB;
    int nsets = 1;
    while (nsets < kSmallWaves && nsets < passes) nsets <<= 1;
    const int wps = kSmallWaves / nsets;                 // waves per set
    const int set = wave / wps, wis = wave - set * wps;   // (uniform in a wave)
    const int STEP = wps * TPW;                           // token rows a set takes per wave-wide load of its waves
    for (int ps = 0; ps * nsets < passes; ++ps) {
        const int row0 = (ps * nsets + set) * RB;
        const int nh = max(0, min(RB, a.G - row0));      // 0: no pass left for this set (it still meets the barriers)
        float qf[RB][EPL], acc[RB][EPL], m[RB], l[RB];
#pragma unroll
        for (int j = 0; j < RB; ++j) {
            if (j < nh) {
                Elem<T>::load(Q + (size_t)(row0 + j) * D + c * EPL, qf[j]);
            } else {
#pragma unroll
                for (int e = 0; e < EPL; ++e) qf[j][e] = 0.f;
            }
            m[j] = -INFINITY;
            l[j] = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[j][e] = 0.f;
        }
        // One round: U token rows per lane.  FULL: every lane of the wave has all U (straight-line code, the loads
        // in flight together); otherwise only the first nu rows exist for any lane and the rest is skipped.
        auto round = [&](auto full_tag, int t0, int nu) {
            constexpr bool FULL = decltype(full_tag)::value;
            Raw kraw[U], vraw[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (FULL || u < nu) {
                    const int t = min(t0 + u * STEP, L - 1);   // (a lane past the end loads the last token and gives it weight 0)
                    const int col = t / kBlock;
                    const int blk = col < kSmallCols ? s_row[col] : max(row[col], 0);
                    const size_t at = (((size_t)blk * a.Hkv + g) * kBlock + (t % kBlock)) * D + c * EPL;
                    kraw[u] = Elem<T>::load_raw(K + at);
                    vraw[u] = Elem<T>::load_raw(V + at);
                }
            }
            float sc[U][RB];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (FULL || u < nu) {
                    float kf[EPL];
                    Elem<T>::unpack(kraw[u], kf);
#pragma unroll
                    for (int j = 0; j < RB; ++j) {
                        float s = 0.f;
#pragma unroll
                        for (int e = 0; e < EPL; ++e) s = fmaf(qf[j][e], kf[e], s);
                        sc[u][j] = s;
                    }
#pragma unroll
                    for (int o = LPT / 2; o >= 1; o >>= 1)
#pragma unroll
                        for (int j = 0; j < RB; ++j) sc[u][j] += __shfl_xor(sc[u][j], o);
                    const bool live = t0 + u * STEP < L;
#pragma unroll
                    for (int j = 0; j < RB; ++j) sc[u][j] = live ? sc[u][j] * a.scale_log2 : -INFINITY;
                } else {
#pragma unroll
                    for (int j = 0; j < RB; ++j) sc[u][j] = -INFINITY;
                }
            }
            // one new reference exponent for the round (row 0 is live in every lane still in the loop, so it is finite)
#pragma unroll
            for (int j = 0; j < RB; ++j) {
                float mn = m[j];
#pragma unroll
                for (int u = 0; u < U; ++u) mn = fmaxf(mn, sc[u][j]);
                const float al = exp2f(m[j] - mn);   // 0 the first time
                m[j] = mn;
                l[j] *= al;
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[j][e] *= al;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (FULL || u < nu) {
                    float vf[EPL];
                    Elem<T>::unpack(vraw[u], vf);
#pragma unroll
                    for (int j = 0; j < RB; ++j) {
                        const float p = exp2f(sc[u][j] - m[j]);
                        l[j] += p;
#pragma unroll
                        for (int e = 0; e < EPL; ++e) acc[j][e] = fmaf(p, vf[e], acc[j][e]);
                    }
                }
            }
        };
        for (int t0 = wis * TPW + r; t0 < (nh > 0 ? L : 0); t0 += U * STEP) {
            // rows of this round that any lane of the wave has (the same in every lane: the first active lane is
            // the one with the lowest token)
            const int left = (L - __builtin_amdgcn_readfirstlane(t0 - r) + STEP - 1) / STEP;
            const int last = __builtin_amdgcn_readfirstlane(t0 - r) + (TPW - 1) + (U - 1) * STEP;   // highest token of a full round
            if (last < L) round(std::true_type{}, t0, U);
            else round(std::false_type{}, t0, min(U, left));
        }
        // fold the states of the wave's lane groups (a group that saw no token has m = -inf and weight 0)
#pragma unroll
        for (int o = LPT; o < 64; o <<= 1) {
#pragma unroll
            for (int j = 0; j < RB; ++j) {
                const float mo = __shfl_xor(m[j], o), lo = __shfl_xor(l[j], o);
                const float mn = fmaxf(m[j], mo);
                const float fa = m[j] == -INFINITY ? 0.f : exp2f(m[j] - mn);
                const float fb = mo == -INFINITY ? 0.f : exp2f(mo - mn);
                l[j] = l[j] * fa + lo * fb;
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[j][e] = acc[j][e] * fa + __shfl_xor(acc[j][e], o) * fb;
                m[j] = mn;
            }
        }
        if (r == 0) {
#pragma unroll
            for (int j = 0; j < RB; ++j) {
#pragma unroll
                for (int e = 0; e < EPL; ++e) s_acc[wave][j][c * EPL + e] = acc[j][e];
                if (c == 0) s_ml[wave][j] = make_float2(m[j], l[j]);
            }
        }
        __syncthreads();
        // fold the waves of every set (fixed order), normalise, write 8 elements per thread
        for (int x = tid; x < nsets * RB * (D / 8); x += kSmallThreads) {
            const int sf = x / (RB * (D / 8)), y = x - sf * (RB * (D / 8));
            const int j = y / (D / 8), c8 = y % (D / 8);
            const int head = (ps * nsets + sf) * RB + j;
            if (head >= a.G) continue;
            const int w0 = sf * wps, w1 = w0 + wps;
            float M = -INFINITY;
            for (int w = w0; w < w1; ++w) M = fmaxf(M, s_ml[w][j].x);
            float den = 0.f, num[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) num[k] = 0.f;
            for (int w = w0; w < w1; ++w) {
                const float2 v = s_ml[w][j];
                const float f = v.x == -INFINITY ? 0.f : exp2f(v.x - M);
                den = fmaf(f, v.y, den);
#pragma unroll
                for (int k = 0; k < 8; ++k) num[k] = fmaf(f, s_acc[w][j][c8 * 8 + k], num[k]);
            }
            const float inv = den > 0.f ? 1.f / den : 0.f;   // an empty history gives a zero row
#pragma unroll
            for (int k = 0; k < 8; ++k) num[k] *= inv;
            Elem<T>::store8(out + (size_t)head * D + c8 * 8, num);
        }
        __syncthreads();
    }
}

template <typename T, int D>
static void launch_generic_d(const SweepArgs& a, int grid, bool wide, const Launch& L) {
    hipStream_t st = static_cast<hipStream_t>(L.stream);
    hipEvent_t e0 = static_cast<hipEvent_t>(L.ev_start), e1 = static_cast<hipEvent_t>(L.ev_stop);
    if (wide) hipExtLaunchKernelGGL((sweep_generic_kernel<T, D, gen_rows_wide<T, D>()>), dim3(grid), dim3(kGenThreads), 0, st, e0, e1, 0, a);
    else hipExtLaunchKernelGGL((sweep_generic_kernel<T, D, 4>), dim3(grid), dim3(kGenThreads), 0, st, e0, e1, 0, a);
}

template <typename T>
static void launch_generic_t(const SweepArgs& a, int head_dim, int grid, const Launch& L) {
    // a batch whose items cannot fill the grid: fewer, wider passes (an item per (request, KV head) and per
    // 8 columns is a generous estimate of what the planner makes)
    const bool wide = (int64_t)a.B * a.Hkv * (1 + a.stride / 8) <= grid;
    switch (head_dim) {
        case 32: launch_generic_d<T, 32>(a, grid, wide, L); break;
        case 64: launch_generic_d<T, 64>(a, grid, wide, L); break;
        case 128: launch_generic_d<T, 128>(a, grid, wide, L); break;
        case 256: launch_generic_d<T, 256>(a, grid, wide, L); break;
        default: break;
    }
}

void launch_sweep_generic(const SweepArgs& a, int dtype, int head_dim, int grid, const Launch& L) {
    if (dtype == FEA_DTYPE_F32) launch_generic_t<float>(a, head_dim, grid, L);
    else launch_generic_t<bf16_t>(a, head_dim, grid, L);
}

template <typename T>
static void launch_merge_t(const SweepArgs& a, int head_dim, bool by_rows, const Launch& L) {
    hipStream_t st = static_cast<hipStream_t>(L.stream);
    hipEvent_t e0 = static_cast<hipEvent_t>(L.ev_start), e1 = static_cast<hipEvent_t>(L.ev_stop);
    const int rows = a.B * a.Hq;
    if (by_rows) {
        const int per_wg = 4 * (64 / (head_dim / 8));
        const int grid = (rows + per_wg - 1) / per_wg;
        switch (head_dim) {
            case 32: hipExtLaunchKernelGGL((merge_rows_kernel<T, 32>), dim3(grid), dim3(256), 0, st, e0, e1, 0, a); break;
            case 64: hipExtLaunchKernelGGL((merge_rows_kernel<T, 64>), dim3(grid), dim3(256), 0, st, e0, e1, 0, a); break;
            case 128: hipExtLaunchKernelGGL((merge_rows_kernel<T, 128>), dim3(grid), dim3(256), 0, st, e0, e1, 0, a); break;
            case 256: hipExtLaunchKernelGGL((merge_rows_kernel<T, 256>), dim3(grid), dim3(256), 0, st, e0, e1, 0, a); break;
            default: break;
        }
        return;
    }
    const int grid = (rows + 3) / 4;
    switch (head_dim) {
        case 32: hipExtLaunchKernelGGL((merge_kernel<T, 32>), dim3(grid), dim3(256), 0, st, e0, e1, 0, a); break;
        case 64: hipExtLaunchKernelGGL((merge_kernel<T, 64>), dim3(grid), dim3(256), 0, st, e0, e1, 0, a); break;
        case 128: hipExtLaunchKernelGGL((merge_kernel<T, 128>), dim3(grid), dim3(256), 0, st, e0, e1, 0, a); break;
        case 256: hipExtLaunchKernelGGL((merge_kernel<T, 256>), dim3(grid), dim3(256), 0, st, e0, e1, 0, a); break;
        default: break;
    }
}

void launch_merge(const SweepArgs& a, int dtype, int head_dim, bool by_rows, const Launch& L) {
    if (dtype == FEA_DTYPE_F32) launch_merge_t<float>(a, head_dim, by_rows, L);
    else launch_merge_t<bf16_t>(a, head_dim, by_rows, L);
}

template <typename T, int RB>
static void launch_small_t(const SweepArgs& a, int head_dim, const Launch& L) {
    hipStream_t st = static_cast<hipStream_t>(L.stream);
    hipEvent_t e0 = static_cast<hipEvent_t>(L.ev_start), e1 = static_cast<hipEvent_t>(L.ev_stop);
    const int grid = a.B * a.Hkv;
    switch (head_dim) {
        case 32: hipExtLaunchKernelGGL((decode_small_kernel<T, 32, RB>), dim3(grid), dim3(kSmallThreads), 0, st, e0, e1, 0, a); break;
        case 64: hipExtLaunchKernelGGL((decode_small_kernel<T, 64, RB>), dim3(grid), dim3(kSmallThreads), 0, st, e0, e1, 0, a); break;
        case 128: hipExtLaunchKernelGGL((decode_small_kernel<T, 128, RB>), dim3(grid), dim3(kSmallThreads), 0, st, e0, e1, 0, a); break;
        case 256: hipExtLaunchKernelGGL((decode_small_kernel<T, 256, RB>), dim3(grid), dim3(kSmallThreads), 0, st, e0, e1, 0, a); break;
        default: break;
    }
}

void launch_decode_small(const SweepArgs& a, int dtype, int head_dim, const Launch& L) {
    if (dtype == FEA_DTYPE_F32) { if (a.G > 4) launch_small_t<float, 8>(a, head_dim, L); else launch_small_t<float, 4>(a, head_dim, L); }
    else launch_small_t<bf16_t, 4>(a, head_dim, L);
}

}  // namespace fea

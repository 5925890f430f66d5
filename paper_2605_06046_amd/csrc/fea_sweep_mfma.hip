// KV sweep on the matrix cores: bf16 caches, head_dim 128, query group size a
// power of two up to 16.
//
// One workgroup (4 waves) takes one work item: a set of up to 64 query rows
// (one request's query group, or a row tile of a prefix group: members x group
// heads stacked) x one KV head x a range of table columns.  The 4 waves split
// the range; each runs an online softmax over its part and the four results are
// merged in LDS, so one partial row per query row leaves the workgroup.
//
// Per 32-token tile (two 16-token blocks) a wave computes, transposed,
//     S^T = K Q^T           (tokens x rows;  v_mfma_f32_16x16x32_bf16, k = head_dim)
//     O^T += V^T P^T        (dims x rows;    same instruction,        k = tokens)
// The transposed forms are chosen so that (a) one lane owns one query row: the
// row maximum, the running sum and the rescale of O stay in-lane (only the 4
// lane groups are combined with two cross-lane maxima), and (b) the
// exponentiated scores in the S^T accumulator layout are already the B operand
// of the second product, no data movement in between.
//
// Memory side: every 16-token block of one KV head is 4 KB contiguous.  K is read
// with four wave-wide 16-byte-per-lane loads per block (perfectly linear), staged
// through a wave-private LDS slab to turn "lane = 16-byte chunk of a token row"
// into the A-operand layout "lane = token".  V needs "lane = head dim, 8 tokens
// per lane"; its loads are also whole 256-byte token rows per 16 lanes, and the
// 8x8 transposition of 16-bit values happens in registers with byte permutes, so
// V never touches LDS.  The loads of tile t+1 are issued before tile t is
// consumed.
//
// What is computed is the same (m, l, acc) triple per query row as in the generic
// sweep: the pieces of softmax(q K^T / sqrt(d)) V (Section 2.1), scores in the
// base-2 domain.  Products are bf16 x bf16 accumulated in float32; the softmax
// weights are rounded to bf16 for the second product, the sums stay float32.
#include <hip/hip_runtime.h>

#include "fea_plan.h"

namespace fea {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kD = 128;                 // head dim
constexpr int kTileTok = 32;            // tokens per tile (two blocks)
constexpr int kKRow = 272;              // bytes per staged K row: 256 + 16 pad (conflict-free b128 reads)
constexpr int kKSlab = kTileTok * kKRow;   // 8704 bytes per wave
constexpr int kWaves = 4;
constexpr size_t kBlkBytes = (size_t)kBlock * kD * 2;   // one (block, KV head): 4096 bytes

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ u32x4 ld16(const void* p) { return *reinterpret_cast<const u32x4*>(p); }
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

struct TileRegs {
    u32x4 k[8];   // k[4*b + i]: block b, tokens 4i + lane/16, 16-byte chunk lane%16
    u32x4 v[8];   // v[j]: token (lane/16)*4 + j%4 of block j/4, 16-byte chunk lane%16
};

// Loads one tile (blocks b0, b1 of KV head g) into registers: K half, V half.
__device__ __forceinline__ void load_tile_k(TileRegs& r, const char* K, int Hkv, int g, int b0, int b1, int lane) {
    const size_t o0 = ((size_t)b0 * Hkv + g) * kBlkBytes;
    const size_t o1 = ((size_t)b1 * Hkv + g) * kBlkBytes;
    const int klane = lane * 16;                                  // linear 4 KB per block
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        r.k[i] = ld16(K + o0 + klane + i * 1024);
        r.k[4 + i] = ld16(K + o1 + klane + i * 1024);
    }
}
__device__ __forceinline__ void load_tile_v(TileRegs& r, const char* V, int Hkv, int g, int b0, int b1, int lane) {
    const size_t o0 = ((size_t)b0 * Hkv + g) * kBlkBytes;
    const size_t o1 = ((size_t)b1 * Hkv + g) * kBlkBytes;
    const int vlane = (lane >> 4) * 1024 + (lane & 15) * 16;      // token row 4*(lane/16) + j
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        r.v[j] = ld16(V + o0 + vlane + j * 256);
        r.v[4 + j] = ld16(V + o1 + vlane + j * 256);
    }
}

template <int NT>
__device__ __forceinline__ void sweep_item(const SweepArgs& a, const Item& item, int nrows, const int* mlist,
                                           int log2G, char* s_k, float2 (*s_ml)[kTileRows], int wave, int lane) {
    const int n = lane & 15;      // query row inside a 16-row tile / token inside a 16-token block (A operand)
    const int kg = lane >> 4;     // lane group: k-slots of the MFMA operands, 4 tokens of the accumulators
    const char* K = static_cast<const char*>(a.k_cache);
    const char* V = static_cast<const char*>(a.v_cache);
    const uint16_t* Q = static_cast<const uint16_t*>(a.q);
    char* kst = s_k + wave * kKSlab;

    const int ncols = item.c1 - item.c0;
    const int ntiles = (ncols + 1) >> 1;
    const int tpw = (ntiles + kWaves - 1) / kWaves;
    const int t_begin = wave * tpw, t_end = min(ntiles, t_begin + tpw);

    f32x4 oacc[NT][8];
    float m_run[NT], l_run[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        m_run[nt] = -INFINITY;
        l_run[nt] = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) oacc[nt][i] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    if (t_begin < t_end) {
        // B operand of the first product: Q^T, lane (n, kg) holds q[row n][32 ks + 8 kg .. +8]
        bf16x8 qB[NT][4];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int row = nt * 16 + n;
            const bool ok = row < nrows;
            const int mem = row >> log2G, hh = row & ((1 << log2G) - 1);
            const int req = ok ? (mlist ? mlist[mem] : item.who) : 0;
            const uint16_t* qp = Q + ((size_t)req * a.Hq + item.g * a.G + hh) * kD + kg * 8;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                u32x4 v = {0u, 0u, 0u, 0u};
                if (ok) v = ld16(qp + ks * 32);
                qB[nt][ks] = as_bf16x8(v);
            }
        }

        const int32_t* trow = a.bt + (size_t)item.who * a.stride;
        const int col0 = item.c0 + 2 * t_begin;
        const int last_col = item.c1 - 1;
        auto load_cols = [&](int cbase) { return trow[min(cbase + lane, last_col)]; };
        int cols = load_cols(col0);
        int cols_next = load_cols(col0 + 64);
        // block ids of the wave's rel-th tile; must be called with rel = 0, 1, 2, ... in order
        auto tile_blocks = [&](int rel, int& b0, int& b1) {
            const int w = rel & 31;
            if (w == 0 && rel > 0) {
                cols = cols_next;
                cols_next = load_cols(col0 + 64 * ((rel >> 5) + 1));
            }
            b0 = __builtin_amdgcn_readlane(cols, 2 * w);
            b1 = __builtin_amdgcn_readlane(cols, 2 * w + 1);
        };

        // Consumes tile t from `cur`.  With `refill`, the loads of tile (nb0, nb1) go
        // back into the same registers as soon as their contents are used up (K after
        // staging, V after the transposes) - the single-buffer schedule of the 64-row case.
        auto process = [&](TileRegs& cur, int t, bool refill, int nb0, int nb1) {
            const int tile_pos = (item.c0 + 2 * t) * kBlock;          // position of the tile's first token
            const bool ragged = tile_pos + kTileTok > item.tok_end;   // wave-uniform

            // ---- K: registers -> LDS (row = token, 16-byte chunks) -> A-operand layout
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                const int tok = (x >> 2) * 16 + (x & 3) * 4 + kg;
                *reinterpret_cast<u32x4*>(kst + tok * kKRow + n * 16) = cur.k[x];
            }
            if (refill) load_tile_k(cur, K, a.Hkv, item.g, nb0, nb1, lane);
            // ---- S^T = K Q^T
            f32x4 sacc[NT][2];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) sacc[nt][0] = sacc[nt][1] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const bf16x8 kA = as_bf16x8(ld16(kst + (mt * 16 + n) * kKRow + (ks * 4 + kg) * 16));
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        sacc[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kA, qB[nt][ks], sacc[nt][mt], 0, 0, 0);
                }
            }
            // ---- V: zero rows past the end (they may hold anything), then 8x8 transposes of 16-bit values
            if (ragged) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int pos = tile_pos + (j >> 2) * 16 + kg * 4 + (j & 3);
                    if (pos >= item.tok_end) cur.v[j] = u32x4{0u, 0u, 0u, 0u};
                }
            }
            bf16x8 vA[8];   // vA[i]: head dim 8*(lane%16) + i, k-slots = the lane group's 8 tokens
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;
                u32x4 o;
#pragma unroll
                for (int w = 0; w < 4; ++w) o[w] = __builtin_amdgcn_perm(cur.v[2 * w + 1][i >> 1], cur.v[2 * w][i >> 1], sel);
                vA[i] = as_bf16x8(o);
            }
            if (refill) load_tile_v(cur, V, a.Hkv, item.g, nb0, nb1, lane);
            // ---- online softmax, one query row per lane (per row tile)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                float s[8];
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) s[mt * 4 + jj] = sacc[nt][mt][jj] * a.scale_log2;
                if (ragged) {
#pragma unroll
                    for (int x = 0; x < 8; ++x) {
                        const int pos = tile_pos + (x >> 2) * 16 + kg * 4 + (x & 3);
                        if (pos >= item.tok_end) s[x] = -INFINITY;
                    }
                }
                float tmax = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
                tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
                tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
                const float m_new = fmaxf(m_run[nt], tmax);
                const float alpha = fast_exp2(m_run[nt] - m_new);
                float psum = 0.f;
                bf16x8 pB;
#pragma unroll
                for (int x = 0; x < 8; ++x) {
                    const float p = fast_exp2(s[x] - m_new);
                    psum += p;
                    pB[x] = (__bf16)p;
                }
                l_run[nt] = l_run[nt] * alpha + psum;
                m_run[nt] = m_new;
                if (__any(alpha != 1.f)) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) oacc[nt][i] *= alpha;
                }
                // ---- O^T += V^T P^T
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    oacc[nt][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vA[i], pB, oacc[nt][i], 0, 0, 0);
            }
        };

        TileRegs ra;
        int b0, b1;
        tile_blocks(0, b0, b1);
        load_tile_k(ra, K, a.Hkv, item.g, b0, b1, lane);
        load_tile_v(ra, V, a.Hkv, item.g, b0, b1, lane);
        if constexpr (NT < 4) {
            // two register sets in ping-pong: the loads of the next tile are in
            // flight while the current one is consumed
            TileRegs rb;
            for (int t = t_begin; t < t_end; t += 2) {
                const bool more = t + 1 < t_end;
                if (more) {
                    tile_blocks(t + 1 - t_begin, b0, b1);
                    load_tile_k(rb, K, a.Hkv, item.g, b0, b1, lane);
                    load_tile_v(rb, V, a.Hkv, item.g, b0, b1, lane);
                }
                process(ra, t, false, 0, 0);
                if (more) {
                    if (t + 2 < t_end) {
                        tile_blocks(t + 2 - t_begin, b0, b1);
                        load_tile_k(ra, K, a.Hkv, item.g, b0, b1, lane);
                        load_tile_v(ra, V, a.Hkv, item.g, b0, b1, lane);
                    }
                    process(rb, t + 1, false, 0, 0);
                }
            }
        } else {
            for (int t = t_begin; t < t_end; ++t) {
                const bool more = t + 1 < t_end;
                if (more) tile_blocks(t + 1 - t_begin, b0, b1);
                process(ra, t, more, b0, b1);
            }
        }
    }

    // ---- merge the four waves: common maximum, rescale, chain-add through LDS
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        float l = l_run[nt];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        l_run[nt] = l;
        if (kg == 0) s_ml[wave][nt * 16 + n] = make_float2(m_run[nt], l);
    }
    __syncthreads();
    float M[NT], Lsum[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        float2 w[kWaves];
        float mx = -INFINITY;
#pragma unroll
        for (int k = 0; k < kWaves; ++k) {
            w[k] = s_ml[k][nt * 16 + n];
            mx = fmaxf(mx, w[k].x);
        }
        float ls = 0.f;
#pragma unroll
        for (int k = 0; k < kWaves; ++k) ls += fast_exp2(w[k].x - mx) * w[k].y;
        M[nt] = mx;
        Lsum[nt] = ls;
        const float f = fast_exp2(m_run[nt] - mx);   // 0 for a wave that had no tile
#pragma unroll
        for (int i = 0; i < 8; ++i) oacc[nt][i] *= f;
    }
    float* slab = reinterpret_cast<float*>(s_k);   // K staging is dead: every wave is past its loop
    float2* ml = reinterpret_cast<float2*>(a.ws + a.lay.ml);
    float* pacc = reinterpret_cast<float*>(a.ws + a.lay.acc);
#pragma unroll
    for (int step = kWaves - 1; step >= 0; --step) {
        if (wave == step) {
            if (step != kWaves - 1) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int i = 0; i < 8; ++i)
#pragma unroll
                        for (int jj = 0; jj < 4; ++jj) oacc[nt][i][jj] += slab[((nt * 8 + i) * 4 + jj) * 64 + lane];
            }
            if (step != 0) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int i = 0; i < 8; ++i)
#pragma unroll
                        for (int jj = 0; jj < 4; ++jj) slab[((nt * 8 + i) * 4 + jj) * 64 + lane] = oacc[nt][i][jj];
            } else {
                // lane (n, kg) holds, for row 16 nt + n, dims 8 (4 kg + jj) + i: runs of 8 consecutive floats
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const int row = nt * 16 + n;
                    if (row < nrows) {
                        float* dst = pacc + (size_t)(item.pbase + row) * kD + kg * 32;
#pragma unroll
                        for (int jj = 0; jj < 4; ++jj) {
                            *reinterpret_cast<float4*>(dst + jj * 8) =
                                make_float4(oacc[nt][0][jj], oacc[nt][1][jj], oacc[nt][2][jj], oacc[nt][3][jj]);
                            *reinterpret_cast<float4*>(dst + jj * 8 + 4) =
                                make_float4(oacc[nt][4][jj], oacc[nt][5][jj], oacc[nt][6][jj], oacc[nt][7][jj]);
                        }
                        if (kg == 0) ml[item.pbase + row] = make_float2(M[nt], Lsum[nt]);
                    }
                }
            }
        }
        __syncthreads();
    }
}

__global__ __launch_bounds__(kWaves * 64, 1) void sweep_mfma_kernel(SweepArgs a, int log2G) {
    __shared__ __attribute__((aligned(16))) char s_k[kWaves * kKSlab];
    __shared__ float2 s_ml[kWaves][kTileRows];
    __shared__ int s_item;
    static_assert(kWaves * kKSlab >= 4 * 8 * 4 * 64 * 4, "merge slab must fit in the K staging area");

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int* hdr = reinterpret_cast<int*>(a.ws);
    const Item* items = reinterpret_cast<const Item*>(a.ws + a.lay.items);
    const int n_items = hdr[H_ITEMS];

    for (;;) {
        if (tid == 0) s_item = atomicAdd(&hdr[H_QUEUE], 1);
        __syncthreads();
        const int it = __builtin_amdgcn_readfirstlane(s_item);
        if (it >= n_items) break;   // every wave sees the same value: the whole workgroup leaves together
        const Item item = items[it];
        int nrows = a.G;
        const int* mlist = nullptr;
        if (item.kind == 1) {
            const GroupDesc gd = reinterpret_cast<const GroupDesc*>(a.ws + a.lay.grp)[item.who];
            const int first = item.tile * a.mpt;
            nrows = min(a.mpt, gd.members - first) * a.G;
            mlist = reinterpret_cast<const int*>(a.ws + a.lay.members) + gd.member_off + first;
        }
        if (nrows <= 16) sweep_item<1>(a, item, nrows, mlist, log2G, s_k, s_ml, wave, lane);
        else if (nrows <= 32) sweep_item<2>(a, item, nrows, mlist, log2G, s_k, s_ml, wave, lane);
        else sweep_item<4>(a, item, nrows, mlist, log2G, s_k, s_ml, wave, lane);
    }
}

void launch_sweep_mfma(const SweepArgs& a, int grid, void* stream) {
    int log2G = 0;
    while ((1 << log2G) < a.G) ++log2G;
    hipLaunchKernelGGL(sweep_mfma_kernel, dim3(grid), dim3(kWaves * 64), 0, static_cast<hipStream_t>(stream), a, log2G);
}

}  // namespace fea

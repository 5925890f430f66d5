// KV sweep on the matrix cores: bf16 caches, head_dim 128, 64 or 256, query groups of
// up to 64 heads per KV head (32 at head_dim 256; any ratio: 7 as in 28/4, 5 as in 40/8, ...).  What
// follows describes head_dim 128.  Head_dim 64 is the same kernel with 2 KB blocks (two
// loads each, 128-byte token rows of eight chunks, swizzled by the row modulo 8), two
// k-steps in the first product and four output products per 16 rows, lanes n and n+8
// sharing a V chunk and taking its lower and upper four dims.  Head_dim 256: 8 KB
// blocks (eight loads, 512-byte rows whose halves are swizzled like 256-byte rows),
// eight k-steps, sixteen output products per 16 rows (lane n takes V chunks n and
// n+16), work items of at most 32 rows (O for 32 rows fills half the accumulation
// registers), and two waves per workgroup, whose two 32 KB stages each fill the LDS.
//
// One wave per SIMD (workgroups of four waves, one workgroup per compute unit); the planner has
// cut the stream of 32-token tiles into equal shares, and wave w sweeps the consecutive work
// items of share w.
// An item is a set of up to 64 query rows (one request's query group,
// or a row tile of a prefix group: members x group heads stacked) x one KV head x
// a range of table columns; the wave sweeps the range with an online softmax and
// writes one partial (m, l, acc[128]) per query row.
//
// Per 32-token tile (two 16-token blocks) the wave computes, transposed,
//     S^T = K Q^T           (tokens x rows;  v_mfma_f32_16x16x32_bf16, k = head_dim)
//     O^T += V^T P^T        (dims x rows;    same instruction,        k = tokens)
// The transposed forms are chosen so that (a) one lane owns one query row: the
// row maximum, the running sum and the rescale of O stay in-lane (only the 4
// lane groups are combined, with two cross-lane maxima), and (b) the
// exponentiated scores in the S^T accumulator layout are already the B operand
// of the second product, no data movement in between.
//
// Memory side.  Every 16-token block of one KV head is 4 KB contiguous.  A tile
// (K and V of two blocks, 16 KB) is fetched with sixteen wave-wide 16-byte-per-
// lane loads that write straight into LDS (global_load_lds_dwordx4), so data in
// flight costs no registers: two 16 KB stages per wave, and the fetch of tile
// t+2 is issued as soon as tile t has been read out of its stage, which keeps
// two tiles in flight while a tile is being computed - across item boundaries too:
// the block ids of the next item's first columns are fetched while the current
// item runs, so its last tiles overlap with the first fetches of the next.  Each
// load covers four
// whole 256-byte token rows; inside a row the sixteen 16-byte chunks are placed
// XOR-swizzled by the row number, which makes the "lane = token" reads of the K
// operand bank-conflict free without padding (the DMA path cannot pad).  V needs
// "lane = head dim, 8 tokens per lane": it is read back as whole token rows and
// transposed 8x8 in registers with byte permutes.
//
// The LDS writes of those loads are invisible to the compiler, so the waits are
// explicit: vmcnt before a stage is read, lgkmcnt before it is overwritten.
//
// What is computed is the same (m, l, acc) triple per query row as in the generic
// sweep: the pieces of softmax(q K^T / sqrt(d)) V (Section 2.1), scores in the
// base-2 domain.  Products are bf16 x bf16 accumulated in float32; the softmax
// weights are rounded to bf16 for the second product, the sums stay float32.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cstdlib>

#include "fea_plan.h"

namespace fea {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kD = 128;                 // head dim of the team sequence (the sweep itself is instantiated per head dim)
constexpr int kTileTok = 32;            // tokens per tile (two blocks)
constexpr int kBlkBytes = kBlock * kD * 2;      // one (block, KV head) at that head dim: 4096 bytes
constexpr int kStageBytes = 4 * kBlkBytes;      // a tile stage at that head dim: K b0 | K b1 | V b0 | V b1
constexpr int kStages = 2;
constexpr int kDescWindow = 8;           // item descriptors fetched into LDS at a time
constexpr float kSlack = 24.f;           // log2 of the largest softmax weight tolerated before the reference is raised

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ u32x4 ld16(const void* p) { return *reinterpret_cast<const u32x4*>(p); }
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Wave-uniform values that must sit in scalar registers (folded away by the compiler
// where it already knows them to be uniform).
// (The builtin returns a signed int: the halves go through uint32_t so that the low
// word is zero-extended, not sign-extended, when the pointer is put back together.)
__device__ __forceinline__ uint32_t sgpr(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
__device__ __forceinline__ const char* sgpr(const void* p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint64_t lo = sgpr((uint32_t)v), hi = sgpr((uint32_t)(v >> 32));
    return reinterpret_cast<const char*>(lo | (hi << 32));
}

// Four wave-wide loads of 64 x 16 bytes from global memory straight into LDS: load
// i reads base + off_i (per lane) and lane l's bytes land at lds_i + 16 l.  The LDS
// addresses are wave-uniform and go through M0.  The scalar operands may have been
// produced by a vector instruction (v_readfirstlane) just before; the hardware
// wants five wait states between such a write and a memory instruction that reads
// the register, and the compiler cannot see into this block, hence the s_nop (and
// one wait state between each write of M0 and the load that uses it).
__device__ __forceinline__ void dma16x4(const char* base, uint32_t off0, uint32_t off1, uint32_t off2, uint32_t off3,
                                        uint32_t lds0, uint32_t lds1, uint32_t lds2, uint32_t lds3) {
    asm volatile(
        "s_nop 4\n\t"
        "s_mov_b32 m0, %5\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %4\n\t"
        "s_mov_b32 m0, %6\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %4\n\t"
        "s_mov_b32 m0, %7\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %4\n\t"
        "s_mov_b32 m0, %8\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %3, %4"
        :: "v"(off0), "v"(off1), "v"(off2), "v"(off3), "s"(base), "s"(lds0), "s"(lds1), "s"(lds2), "s"(lds3)
        : "memory", "m0");
}
// Two such loads (a 2 KB block of head_dim 64).
__device__ __forceinline__ void dma16x2(const char* base, uint32_t off0, uint32_t off1, uint32_t lds0, uint32_t lds1) {
    asm volatile(
        "s_nop 4\n\t"
        "s_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %2\n\t"
        "s_mov_b32 m0, %4\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
        :: "v"(off0), "v"(off1), "s"(base), "s"(lds0), "s"(lds1)
        : "memory", "m0");
}
// One load of 4 bytes per lane (block ids of 64 table columns), same conventions.
__device__ __forceinline__ void dma4(const void* base, uint32_t lane_off, uint32_t lds_addr) {
    asm volatile("s_nop 4\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                 :: "v"(lane_off), "s"(base), "s"(lds_addr) : "memory", "m0");
}
// acc *= f for an accumulator tuple that lives in the accumulation registers.  Done
// by hand so that the register allocator keeps the big O accumulators there (a
// plain C++ multiply would pull all of them into the vector register file and
// make every tile pay for copies).  Only the rare "raise the reference" path runs
// this; the leading s_nop covers the matrix-core write -> read distance even if a
// product into the same tuple were the immediately preceding instruction.
__device__ __forceinline__ void scale_acc(f32x4& acc, float f) {
    float a0 = acc[0], a1 = acc[1], a2 = acc[2], a3 = acc[3];
    float t0, t1;
    asm volatile(
        "s_nop 15\n\ts_nop 3\n\t"
        "v_accvgpr_read_b32 %4, %0\n\tv_accvgpr_read_b32 %5, %1\n\t"
        "v_mul_f32 %4, %4, %6\n\tv_mul_f32 %5, %5, %6\n\t"
        "v_accvgpr_write_b32 %0, %4\n\tv_accvgpr_write_b32 %1, %5\n\t"
        "v_accvgpr_read_b32 %4, %2\n\tv_accvgpr_read_b32 %5, %3\n\t"
        "v_mul_f32 %4, %4, %6\n\tv_mul_f32 %5, %5, %6\n\t"
        "v_accvgpr_write_b32 %2, %4\n\tv_accvgpr_write_b32 %3, %5"
        : "+a"(a0), "+a"(a1), "+a"(a2), "+a"(a3), "=&v"(t0), "=&v"(t1)
        : "v"(f));
    acc[0] = a0; acc[1] = a1; acc[2] = a2; acc[3] = a3;
}
// Stores issued by hand so that the wave can count them (see Stream): wave-uniform
// base address in scalar registers, 32-bit byte offset per lane.  The hardware reads
// the data registers of a wide store a little after issue and does not interlock
// against a vector instruction overwriting them meanwhile; the compiler pads its own
// stores for that but cannot see these, hence the trailing s_nop.
__device__ __forceinline__ void store_f32x4(const char* base, uint32_t off, f32x4 v) {
    asm volatile("s_nop 4\n\tglobal_store_dwordx4 %0, %1, %2\n\ts_nop 1" :: "v"(off), "v"(v), "s"(base) : "memory");
}
__device__ __forceinline__ void store_f32x2(const char* base, uint32_t off, float x, float y) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    const f32x2 v = {x, y};
    asm volatile("s_nop 4\n\tglobal_store_dwordx2 %0, %1, %2\n\ts_nop 1" :: "v"(off), "v"(v), "s"(base) : "memory");
}
template <int N> __device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory"); }
__device__ __forceinline__ void wait_lgkmcnt0() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

struct Lanes {
    int n;                 // lane % 16: query row of a 16-row tile / token of a block / 16-byte chunk
    int kg;                // lane / 16: k-slot group of the MFMA operands
    uint32_t dma_off[8];   // global byte offset inside a block for load i (rows 4i + kg, swizzled chunk)
    uint32_t k_off[8];     // LDS byte offset inside a K block of the A operand for k-step ks
    uint32_t v_off[4];     // LDS byte offset inside a V block of token row 4 kg + j
};

// Fetch blocks b0, b1 of KV head g into the stage at LDS address `stage` (16 loads).
template <int D>
__device__ __forceinline__ void fetch_tile(const SweepArgs& a, int g, int b0, int b1, uint32_t stage, const Lanes& L) {
    constexpr int BLK = kBlock * D * 2;
    const size_t o0 = ((size_t)b0 * a.Hkv + g) * BLK;
    const size_t o1 = ((size_t)b1 * a.Hkv + g) * BLK;
    const char* k0 = sgpr(static_cast<const char*>(a.k_cache) + o0);
    const char* k1 = sgpr(static_cast<const char*>(a.k_cache) + o1);
    const char* v0 = sgpr(static_cast<const char*>(a.v_cache) + o0);
    const char* v1 = sgpr(static_cast<const char*>(a.v_cache) + o1);
    stage = sgpr(stage);
    const char* bases[4] = {k0, k1, v0, v1};
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const uint32_t l = stage + x * BLK;
        if constexpr (D == 64) dma16x2(bases[x], L.dma_off[0], L.dma_off[1], l, l + 1024);
        else dma16x4(bases[x], L.dma_off[0], L.dma_off[1], L.dma_off[2], L.dma_off[3], l, l + 1024, l + 2048, l + 3072);
        if constexpr (D == 256) dma16x4(bases[x], L.dma_off[4], L.dma_off[5], L.dma_off[6], L.dma_off[7], l + 4096, l + 5120, l + 6144, l + 7168);
    }
}

// Tile stream of one wave.  `phase` is the stage the current item's tile 0 uses,
// `iss` counts the tiles issued so far, numbered from the current item's tile 0
// (so it can already be 1 or 2 when the item starts: its predecessor fetched them).
//
// Everything the wave loads while it streams goes global -> LDS by hand-issued loads
// the compiler does not see, and the hardware retires a wave's vector-memory
// operations in issue order.  So the wave numbers them itself: `seq` counts the
// loads issued, every consumer remembers the count right after "its" loads (a
// mark), and waiting for a mark means letting at most seq - mark younger
// operations stay outstanding; the stores of the partial rows are issued by hand
// and counted as well.  An operation the compiler issues on its own and that is
// not counted only makes a wait stricter.
struct Stream {
    int phase;
    int iss;
    // Block ids travel through three 64-column windows in LDS: even and odd windows of
    // the current item, and the first window of the next item (which becomes the even
    // window when the items switch).
    int cb0, cb1, cbn;
    bool cols_ready;   // the current item's first window was requested while its predecessor ran
    bool q_ready;      // so were its query rows (into the LDS query buffer)
    uint32_t seq;      // hand-issued loads so far
    uint32_t done;     // loads [0, done) are known to have landed
    uint32_t tmark0, tmark1;          // mark of the tile in stage 0 / 1
    uint32_t cmark0, cmark1, cmark2;  // marks of the three column windows
    uint32_t qmark;                   // mark of the query buffer
};

__device__ __forceinline__ uint32_t pick3(int i, uint32_t a, uint32_t b, uint32_t c) { return i == 0 ? a : (i == 1 ? b : c); }

// Wait until the load with this mark (and with it every older one) has landed.
__device__ __forceinline__ void wait_for(Stream& sm, uint32_t mark) {
    if ((int32_t)(mark - sm.done) <= 0) return;
    uint32_t n = sm.seq - mark;   // younger loads: they may stay in flight
    if (n > 50) n = 50;
    switch (n) {                  // the wait takes its count as an immediate
#define FEA_W(N) case N: wait_vmcnt<N>(); break;
        FEA_W(0) FEA_W(1) FEA_W(2) FEA_W(3) FEA_W(4) FEA_W(5) FEA_W(6) FEA_W(7) FEA_W(8) FEA_W(9)
        FEA_W(10) FEA_W(11) FEA_W(12) FEA_W(13) FEA_W(14) FEA_W(15) FEA_W(16) FEA_W(17) FEA_W(18) FEA_W(19)
        FEA_W(20) FEA_W(21) FEA_W(22) FEA_W(23) FEA_W(24) FEA_W(25) FEA_W(26) FEA_W(27) FEA_W(28) FEA_W(29)
        FEA_W(30) FEA_W(31) FEA_W(32) FEA_W(33) FEA_W(34) FEA_W(35) FEA_W(36) FEA_W(37) FEA_W(38) FEA_W(39)
        FEA_W(40) FEA_W(41) FEA_W(42) FEA_W(43) FEA_W(44) FEA_W(45) FEA_W(46) FEA_W(47) FEA_W(48) FEA_W(49)
        default: wait_vmcnt<50>(); break;
#undef FEA_W
    }
    sm.done = sm.seq - n;
}
__device__ __forceinline__ void wait_all(Stream& sm) {
    wait_vmcnt<0>();
    sm.done = sm.seq;
}

template <int NT, int D>
__device__ __forceinline__ void sweep_item(const SweepArgs& a, const Item& item, const Item& next, bool has_next,
                                           int g_rcp, char* s_stage, const int* s_cols, const char* s_q, uint32_t lds_base,
                                           uint32_t cols_base, uint32_t q_base, const Lanes& L, int lane, Stream& sm) {
    constexpr int BLK = kBlock * D * 2;      // bytes of one (block, KV head)
    constexpr int STG = 4 * BLK;             // K b0 | K b1 | V b0 | V b1
    constexpr int KS = D / 32;               // k-steps of S^T = K Q^T
    constexpr int NI = D / 16;               // products of O^T += V^T P^T per 16 query rows
    const int n = L.n, kg = L.kg;
    const uint16_t* Q = static_cast<const uint16_t*>(a.q);
    const int* mlist = reinterpret_cast<const int*>(a.ws + a.lay.members) + item.mlist_off;
    const int ntiles = (item.c1 - item.c0 + 1) >> 1;
    const int next_pre = has_next ? min(2, (next.c1 - next.c0 + 1) >> 1) : 0;   // tiles of the next item we may fetch

    // Block ids of the item's columns travel through LDS as well, 64 columns per
    // window: the compiler then sees no pending vector-memory load inside the tile
    // loop (it would drain the whole prefetch queue for it).
    const int32_t* trow = a.bt + (size_t)item.who * a.stride;
    const int32_t* nrow = a.bt + (size_t)next.who * a.stride;
    auto fetch_cols = [&](const int32_t* row, int c0, int c1, int win, int buf) {   // clamped: never reads a dead entry
        dma4(sgpr(row), (uint32_t)min(c0 + 64 * win + lane, c1 - 1) * 4u, sgpr(cols_base + buf * 256));
        sm.seq += 1;
        sm.cmark0 = buf == 0 ? sm.seq : sm.cmark0;   // (value selects: the struct must stay in registers)
        sm.cmark1 = buf == 1 ? sm.seq : sm.cmark1;
        sm.cmark2 = buf == 2 ? sm.seq : sm.cmark2;
    };
    auto buf_of = [&](int win) { return (win & 1) ? sm.cb1 : sm.cb0; };
    // Issue stream tile `idx` (own tile idx, or tile idx - ntiles of the next item) if it
    // is the next one due and exists; own tiles must be asked for in increasing order.
    auto issue = [&](int idx) {
        if (idx != sm.iss) return;
        int buf, at;
        int g = item.g;
        if (idx < ntiles) {
            const int w = idx & 31, win = idx >> 5;
            if (w == 0 && idx > 0) fetch_cols(trow, item.c0, item.c1, win + 1, buf_of(win + 1));   // `win` came 32 tiles ago
            buf = buf_of(win);
            at = 2 * w;
        } else {
            const int j = idx - ntiles;
            if (j >= next_pre) return;
            buf = sm.cbn;
            at = 2 * j;
            g = next.g;
        }
        wait_for(sm, pick3(buf, sm.cmark0, sm.cmark1, sm.cmark2));   // the window's block ids must have landed
        const int* sc = s_cols + buf * 64 + at;
        // (a table entry of -1 inside a request's length is the caller's error; it must not become a
        // read before the cache)
        const int b0 = max(__builtin_amdgcn_readfirstlane(sc[0]), 0);
        const int b1 = max(__builtin_amdgcn_readfirstlane(sc[1]), 0);
        const int stg = (sm.phase + idx) & 1;
        fetch_tile<D>(a, g, b0, b1, lds_base + stg * STG, L);
        sm.seq += D / 8;
        sm.tmark0 = stg == 0 ? sm.seq : sm.tmark0;
        sm.tmark1 = stg == 1 ? sm.seq : sm.tmark1;
        sm.iss = idx + 1;
    };
    if (!sm.cols_ready) fetch_cols(trow, item.c0, item.c1, 0, sm.cb0);
    fetch_cols(trow, item.c0, item.c1, 1, sm.cb1);
    if (has_next) fetch_cols(nrow, next.c0, next.c1, 0, sm.cbn);
    // Own tiles only at this point (no-ops when the predecessor has asked for them):
    // the next item's column window has only just been requested.
    issue(0);
    if (ntiles > 1) issue(1);

    // B operand of the first product: Q^T, lane (n, kg) holds q[row n][32 ks + 8 kg .. +8].
    // The rows of a single request's query group are contiguous in q; the predecessor
    // has then already brought them into the LDS query buffer (laid out like a K
    // block: 16 rows, chunks swizzled by the row), and nothing has to be waited for
    // that is younger than that.  Otherwise (first item of a share, rows gathered
    // through a member list, more than 16 rows) they are loaded here and everything
    // in flight is drained once.
    bf16x8 qB[NT][KS];
    bool q_from_lds = false;
    if constexpr (NT == 1) q_from_lds = sm.q_ready;
    if (q_from_lds) {
        wait_for(sm, sm.qmark);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qB[0][ks] = as_bf16x8(ld16(s_q + L.k_off[ks]));
    } else {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int row = nt * 16 + n;
            const bool ok = row < item.nrows;
            const int mem = (row * g_rcp) >> 16, hh = row - mem * a.G;   // row / G and row % G (rows < 64, G <= 64)
            const int req = ok ? (item.mlist_off < 0 ? item.who : mlist[mem]) : 0;
            const uint16_t* qp = Q + ((size_t)req * a.Hq + item.g * a.G + hh) * D + kg * 8;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                u32x4 v = {0u, 0u, 0u, 0u};
                if (ok) v = ld16(qp + ks * 32);
                qB[nt][ks] = as_bf16x8(v);
            }
        }
        // Everything in flight is consumed here, before the tile loop, so that the
        // compiler has no load of its own pending inside it.
        wait_all(sm);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qB[nt][ks]));
    }
    // Bring in the next item's query rows if they are one contiguous run of at most 16.
    const bool q_next = has_next && next.nrows <= 16 && next.mlist_off < 0;
    if (q_next) {
        wait_lgkmcnt0();   // the buffer has been read out
        const char* qn = reinterpret_cast<const char*>(Q + ((size_t)next.who * a.Hq + next.g * a.G) * D);
        const uint32_t qb = sgpr(q_base);
        if constexpr (D == 128) {
            uint32_t off[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int row = 4 * j + kg;                          // row of the buffer this lane fills in load j
                off[j] = (uint32_t)min(row, next.nrows - 1) * 256u + (uint32_t)((n ^ row) & 15) * 16u;   // rows past the end repeat the last one
            }
            dma16x4(sgpr(qn), off[0], off[1], off[2], off[3], qb, qb + 1024, qb + 2048, qb + 3072);
            sm.seq += 4;
        } else if constexpr (D == 64) {
            uint32_t off[2];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int row = 8 * j + (lane >> 3), pos = lane & 7;   // 128-byte rows: eight per load
                off[j] = (uint32_t)min(row, next.nrows - 1) * 128u + (uint32_t)((pos ^ row) & 7) * 16u;
            }
            dma16x2(sgpr(qn), off[0], off[1], qb, qb + 1024);
            sm.seq += 2;
        } else {
            uint32_t off[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int row = 2 * j + (lane >> 5), pos = lane & 31;  // 512-byte rows: two per load
                off[j] = (uint32_t)min(row, next.nrows - 1) * 512u + (uint32_t)((pos & 16) | ((pos ^ row) & 15)) * 16u;
            }
            dma16x4(sgpr(qn), off[0], off[1], off[2], off[3], qb, qb + 1024, qb + 2048, qb + 3072);
            dma16x4(sgpr(qn), off[4], off[5], off[6], off[7], qb + 4096, qb + 5120, qb + 6144, qb + 7168);
            sm.seq += 8;
        }
        sm.qmark = sm.seq;
    }

    // The softmax denominator is accumulated by the matrix core as well: a V^T row
    // of ones turns the second product into sum_t p_t, taken over the same bf16-
    // rounded weights as the numerator (so numerator and denominator stay consistent).
    u32x4 ones_bits = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
    const bf16x8 ones = as_bf16x8(ones_bits);
    f32x4 oacc[NT][NI];
    f32x4 lacc[NT];
    float m_run[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        m_run[nt] = -INFINITY;
        lacc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < NI; ++i) oacc[nt][i] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // One tile in two halves.  front(t): wait for the tile, read it out of its stage
    // (handing the stage back for the refill), S^T = K Q^T, V transposed, and the
    // scaled scores with their per-lane maximum.  back(): weights, denominators and
    // O^T += V^T P^T.  Between the two the reference exponents may have to be raised;
    // that happens in a second copy of the loop, entered at most once per item.
    f32x4 sacc[NT][2]; // S^T of the tile: this lane's 8 tokens (two blocks of 4) per row tile
    float tmax[NT];    // scaled maximum of those, positions past the end left out
    int tile_pos = 0;  // position of the tile's first token
    bool ragged = false;   // the tile reaches past the item's last token (wave-uniform)
    bf16x8 vA[NI];     // vA[i]: head dim 8*(lane%16) + i (head_dim 64: lanes n >= 8 carry dim 8*(n-8) + i + 4), k-slots = the lane group's 8 tokens
    auto scores = [&](int nt, float (&r)[8]) {   // this lane's 8 scores of row tile nt; -inf past the end
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) r[mt * 4 + jj] = sacc[nt][mt][jj];
        if (__builtin_expect(ragged, 0)) {
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                const int pos = tile_pos + (x >> 2) * 16 + kg * 4 + (x & 3);
                if (pos >= item.tok_end) r[x] = -INFINITY;
            }
        }
    };
    auto front = [&](int t) {
        const int stg = (sm.phase + t) & 1;
        const char* st = s_stage + stg * STG;
        wait_for(sm, stg == 0 ? sm.tmark0 : sm.tmark1);   // tile t has landed
        // Read the tile out of its stage and hand the stage back.  With 16 or 32 query
        // rows everything is read up front so that the refill starts at once; with 64
        // rows registers are short, so V is read after the first product (that
        // instantiation computes long enough per tile for the later refill not to matter).
        constexpr bool kLate = NT == 4 || D == 256;   // registers are short: K of the second block and V are read after the first product
        constexpr int VH = D == 256 ? 2 : 1;          // a V row has 32 chunks at head_dim 256: lane n takes chunks n and n + 16
        bf16x8 kA[kLate ? 1 : 2][KS];
        u32x4 vr[8 * VH];
#pragma unroll
        for (int mt = 0; mt < (kLate ? 1 : 2); ++mt)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) kA[mt][ks] = as_bf16x8(ld16(st + mt * BLK + L.k_off[ks]));
        if constexpr (!kLate) {
#pragma unroll
            for (int j = 0; j < 8; ++j) vr[j] = ld16(st + (2 + (j >> 2)) * BLK + L.v_off[j & 3]);
            wait_lgkmcnt0();   // the stage is read out: refill it with stream tile t+2
            issue(t + 1);      // (only due if the look-ahead into the next item stopped short)
            issue(t + 2);
        }

        tile_pos = (item.c0 + 2 * t) * kBlock;
        ragged = tile_pos + kTileTok > item.tok_end;

        // ---- S^T = K Q^T
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) sacc[nt][0] = sacc[nt][1] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            if constexpr (kLate) {
                if (mt == 1) {
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) kA[0][ks] = as_bf16x8(ld16(st + BLK + L.k_off[ks]));
                }
            }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    sacc[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kA[kLate ? 0 : mt][ks], qB[nt][ks], sacc[nt][mt], 0, 0, 0);
        }
        if constexpr (kLate) {
#pragma unroll
            for (int h = 0; h < VH; ++h)
#pragma unroll
                for (int j = 0; j < 8; ++j) vr[8 * h + j] = ld16(st + (2 + (j >> 2)) * BLK + L.v_off[j & 3] + h * 256);
            wait_lgkmcnt0();
            issue(t + 1);
            issue(t + 2);
        }

        // ---- V: zero rows past the end (they may hold anything), then 8x8 transposes of 16-bit values
        if (__builtin_expect(ragged, 0)) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int pos = tile_pos + (j >> 2) * 16 + kg * 4 + (j & 3);
                if (pos >= item.tok_end) {
#pragma unroll
                    for (int h = 0; h < VH; ++h) vr[8 * h + j] = u32x4{0u, 0u, 0u, 0u};
                }
            }
        }
        if constexpr (D >= 128) {
#pragma unroll
            for (int h = 0; h < VH; ++h)
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;
                    u32x4 o;
#pragma unroll
                    for (int w = 0; w < 4; ++w) o[w] = __builtin_amdgcn_perm(vr[8 * h + 2 * w + 1][i >> 1], vr[8 * h + 2 * w][i >> 1], sel);
                    vA[8 * h + i] = as_bf16x8(o);     // (head_dim 256: products 8.. carry dims 128 + 8 n + i)
                }
        } else {
            // a token row has 8 chunks: lanes n and n + 8 read the same one; lane n < 8 hands elements 0..3 of it
            // to products 0..3 (dims 8 n + i), lane n >= 8 elements 4..7 (dims 8 (n - 8) + 4 + i)
            const int hi = n >> 3;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;
                u32x4 o;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const uint32_t lo1 = vr[2 * w + 1][i >> 1], lo0 = vr[2 * w][i >> 1];
                    const uint32_t hi1 = vr[2 * w + 1][2 + (i >> 1)], hi0 = vr[2 * w][2 + (i >> 1)];
                    o[w] = __builtin_amdgcn_perm(hi ? hi1 : lo1, hi ? hi0 : lo0, sel);
                }
                vA[i] = as_bf16x8(o);
            }
        }

        // ---- row maxima, one query row per lane (per row tile); the scores themselves stay
        // in the accumulation registers until back() turns them into weights
        bool raise = false;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            float r[8];
            scores(nt, r);
            tmax[nt] = a.scale_log2 *
                fmaxf(fmaxf(fmaxf(r[0], r[1]), fmaxf(r[2], r[3])), fmaxf(fmaxf(r[4], r[5]), fmaxf(r[6], r[7])));
            raise = raise || tmax[nt] > m_run[nt] + kSlack;
        }
        return __any(raise);
    };
    // Online softmax.  The running "maximum" is a reference exponent m_ref per row:
    // weights are 2^(s - m_ref).  It is raised to the true row maximum (and l, O
    // rescaled) only when some score exceeds it by more than kSlack, which float32
    // sums absorb without loss; on the first tile it is -inf, so that always happens
    // there.  Softmax is shift-invariant, so the result is the same, and the common
    // case costs no cross-lane traffic and no rescale of O.
    auto raise_refs = [&]() {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            if (__any(tmax[nt] > m_run[nt] + kSlack)) {
                float rmax = fmaxf(tmax[nt], __shfl_xor(tmax[nt], 16));
                rmax = fmaxf(rmax, __shfl_xor(rmax, 32));
                const float m_new = fmaxf(m_run[nt], rmax);
                const float alpha = fast_exp2(m_run[nt] - m_new);
                scale_acc(lacc[nt], alpha);
#pragma unroll
                for (int i = 0; i < NI; ++i) scale_acc(oacc[nt][i], alpha);
                m_run[nt] = m_new;
            }
        }
    };
    auto back = [&]() {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const float neg_m = -m_run[nt];
            float r[8];
            scores(nt, r);
            bf16x8 pB;
#pragma unroll
            for (int x = 0; x < 8; ++x) pB[x] = (__bf16)fast_exp2(fmaf(r[x], a.scale_log2, neg_m));
            lacc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pB, lacc[nt], 0, 0, 0);
#pragma unroll
            for (int i = 0; i < NI; ++i)
                oacc[nt][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vA[i], pB, oacc[nt][i], 0, 0, 0);
        }
    };
    // First tile: the reference is its row maximum, nothing to rescale yet.
    front(0);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        float rmax = fmaxf(tmax[nt], __shfl_xor(tmax[nt], 16));
        m_run[nt] = fmaxf(rmax, __shfl_xor(rmax, 32));
    }
    back();
    // Fast loop: no reference is ever raised in here, the accumulators are only touched
    // by the matrix core.  It is left for good (to the loop below) the first time a
    // score outgrows its reference.
    int t = 1;
    bool need = false;
    for (; t < ntiles; ++t) {
        need = front(t);
        if (__builtin_expect(need, 0)) break;
        back();
    }
    if (need) {
        for (;;) {   // tile t has been through front()
            raise_refs();
            back();
            if (++t >= ntiles) break;
            front(t);
        }
    }

    // ---- partial rows: lane (n, kg) holds, for row 16 nt + n, dims 8 (4 kg + jj) + i: runs of 8 floats
    const char* ml = sgpr(a.ws + a.lay.ml + (size_t)item.pbase * sizeof(float2));          // the item's first partial row
    const char* pacc = sgpr(a.ws + a.lay.acc + (size_t)item.pbase * (D * sizeof(float)));
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const float l = lacc[nt][0];   // every element of the column holds the row's sum
        const int row = nt * 16 + n;
        if (nt * 16 < item.nrows) {    // wave-uniform: lane 0 has a row here, so all nine stores are issued
            if (row < item.nrows) {
                if constexpr (D >= 128) {
#pragma unroll
                    for (int h = 0; h < D / 128; ++h) {
                        const uint32_t dst = (uint32_t)row * (D * 4u) + (uint32_t)kg * 128u + (uint32_t)h * 512u;
#pragma unroll
                        for (int jj = 0; jj < 4; ++jj) {
                            store_f32x4(pacc, dst + jj * 32, f32x4{oacc[nt][8 * h + 0][jj], oacc[nt][8 * h + 1][jj], oacc[nt][8 * h + 2][jj], oacc[nt][8 * h + 3][jj]});
                            store_f32x4(pacc, dst + jj * 32 + 16, f32x4{oacc[nt][8 * h + 4][jj], oacc[nt][8 * h + 5][jj], oacc[nt][8 * h + 6][jj], oacc[nt][8 * h + 7][jj]});
                        }
                    }
                } else {
                    // product i, output row m = 4 kg + jj: dim 8 m + i for m < 8, 8 (m - 8) + 4 + i for m >= 8
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) {
                        const int m = 4 * kg + jj, db = m < 8 ? 8 * m : 8 * (m - 8) + 4;
                        store_f32x4(pacc, (uint32_t)row * (D * 4u) + (uint32_t)db * 4u,
                                    f32x4{oacc[nt][0][jj], oacc[nt][1][jj], oacc[nt][2][jj], oacc[nt][3][jj]});
                    }
                }
                if (kg == 0) store_f32x2(ml, (uint32_t)row * 8u, m_run[nt], l);
            }
            sm.seq += D / 16 + 1;
        }
    }
    sm.phase = (sm.phase + ntiles) & 1;
    sm.iss -= ntiles;
    const int old0 = sm.cb0;
    sm.cb0 = sm.cbn;   // the next item's first window is already there
    sm.cbn = sm.cb1;
    sm.cb1 = old0;
    sm.cols_ready = has_next;
    sm.q_ready = q_next;
}

// A piece of a shared run swept by a team of 2 or 4 waves of this workgroup, one row tile of up to 64
// query rows per wave, every tile of the piece fetched once for the whole team: the hand-scheduled
// sequences of fea_sweep_core.inc (see gen_sweep_core.py for what they do and why they are written
// out by hand).  Same partial rows as sweep_item.  A sequence uses most of the wave's registers under
// fixed names; the caller ends the wave right after it, so that nothing of the rest of the kernel
// has to live across it.  `team_base`: LDS address of the team's ring (2 x team tiles of K, then of V).
#include "fea_sweep_core.inc"
constexpr int kTeamCols = 1024;   // columns of a piece a team can sweep: their block ids fill the wave's query buffer (4 KB)
__device__ __forceinline__ void sweep_team_core(const SweepArgs& a, const Item& item, int team, int rank, int g_rcp,
                                                uint32_t team_base, uint32_t tab_base, int lane) {
    // The per-lane inputs are worked out again from a copy of the lane number the compiler cannot
    // see through: they must sit in the few registers the sequence leaves alone, and tying them to
    // the values the rest of the kernel keeps for its whole life would push those into scratch.
    asm volatile("" : "+v"(lane));
    const int n = lane & 15, kg = lane >> 4;
    const uint32_t k_off0 = (uint32_t)(n * 256 + ((kg ^ n) & 15) * 16);             // token row n, chunk kg (k-step 0)
    const uint32_t v_off0 = (uint32_t)(4 * kg * 256 + ((n ^ (4 * kg)) & 15) * 16);  // token row 4 kg, chunk n
    const uint32_t d_off0 = (uint32_t)(kg * 256 + ((n ^ kg) & 15) * 16);            // load 0 of a block: row kg
    const int ntiles = (item.c1 - item.c0) >> 1;
    const int* mlist = reinterpret_cast<const int*>(a.ws + a.lay.members) + item.mlist_off;
    const int32_t* trow = a.bt + (size_t)item.who * a.stride;
    // block ids of all the piece's columns (at most kTeamCols), 64 per load, into this wave's query buffer
    // (not needed here: the sequence keeps the query rows in registers)
    for (int w = 0; w * 64 < item.c1 - item.c0; ++w)
        dma4(sgpr(trow), (uint32_t)min(item.c0 + 64 * w + lane, item.c1 - 1) * 4u, sgpr(tab_base + 256u * (uint32_t)w));
    // byte offset of this lane's part of query row 16 nt + n (rows past the end: the first row again)
    uint32_t qoff[4];
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
        int row = nt * 16 + n;
        row = row < item.nrows ? row : 0;
        const int mem = (row * g_rcp) >> 16, hh = row - mem * a.G;
        const int req = item.mlist_off < 0 ? item.who : mlist[mem];
        qoff[nt] = (uint32_t)(((req * a.Hq + item.g * a.G + hh) * kD + kg * 8) * 2);
    }
    wait_vmcnt<0>();
    // this wave's part of every tile: ranks of the lower half fetch K, of the upper half V; in a team of 4 one block each
    const bool loads_v = rank >= team / 2;
    const uint64_t own = reinterpret_cast<uint64_t>(loads_v ? a.v_cache : a.k_cache);
    const uint32_t odd = team == 4 ? (uint32_t)(rank & 1) : 0u;
    const uint32_t own_ring = sgpr((loads_v ? (uint32_t)(2 * team) * (2u * kBlkBytes) : 0u) + odd * kBlkBytes);
    const uint32_t tabsel = sgpr(odd * 4u);
    const uint64_t qbase = reinterpret_cast<uint64_t>(sgpr(a.q));
    const uint64_t accbase = reinterpret_cast<uint64_t>(sgpr(a.ws + a.lay.acc + (size_t)item.pbase * (kD * sizeof(float))));
    const uint64_t mlbase = reinterpret_cast<uint64_t>(sgpr(a.ws + a.lay.ml + (size_t)item.pbase * sizeof(float2)));
    const uint32_t own_lo = sgpr((uint32_t)own), own_hi = sgpr((uint32_t)(own >> 32));
    const uint32_t lane4 = (uint32_t)lane * 4u, dst0 = (uint32_t)n * (kD * 4u) + (uint32_t)kg * 128u;
#define FEA_TEAM_CORE_OPERANDS                                                                                                  \
    : [koff0] "v"(k_off0), [voff0] "v"(v_off0), [doff0] "v"(d_off0), [q0] "v"(qoff[0]), [q1] "v"(qoff[1]), [q2] "v"(qoff[2]),   \
      [q3] "v"(qoff[3]), [lane4] "v"(lane4), [dst0] "v"(dst0), [nrow] "v"(n), [qbase] "s"(qbase), [accbase] "s"(accbase),       \
      [mlbase] "s"(mlbase), [own_lo] "s"(own_lo), [own_hi] "s"(own_hi), [hkv] "s"(sgpr((uint32_t)a.Hkv)),                        \
      [g] "s"(sgpr((uint32_t)item.g)), [ntiles] "s"(sgpr((uint32_t)ntiles)), [nrows] "s"(sgpr((uint32_t)item.nrows)),             \
      [scale] "s"(__builtin_bit_cast(float, sgpr(__builtin_bit_cast(uint32_t, a.scale_log2)))), [team] "s"(sgpr(team_base)),     \
      [tab] "s"(sgpr(tab_base)), [own_ring] "s"(own_ring), [tabsel] "s"(tabsel)                                                   \
    : FEA_TEAM_CORE_CLOBBERS
    if (team == 4) asm volatile(FEA_TEAM4_CORE_ASM : FEA_TEAM_CORE_OPERANDS);
    else asm volatile(FEA_TEAM2_CORE_ASM : FEA_TEAM_CORE_OPERANDS);
#undef FEA_TEAM_CORE_OPERANDS
}

constexpr int kWavesPerGroup = 4;   // one wave per SIMD of a compute unit: a workgroup fills the unit

// Waves per workgroup: four (one per SIMD) - at head_dim 256 two, whose tile stages (2 x 32 KB each) fill the LDS.
template <int D> constexpr int waves_per_group() { return D == 256 ? 2 : kWavesPerGroup; }

template <int D>
__global__ __launch_bounds__(64 * waves_per_group<D>()) void sweep_mfma_kernel(SweepArgs a, int g_rcp, int xcd_aware) {
    constexpr int WPG = waves_per_group<D>();
    constexpr int STG = 4 * kBlock * D * 2;          // bytes of a tile stage: K b0 | K b1 | V b0 | V b1
    // Every wave sweeps a share of its own and owns a quarter of the workgroup's LDS; the waves of a
    // workgroup never wait for one another on this path.  (They sit in one workgroup so that the row
    // tiles of a shared run's piece, which read the same KV bytes, can share what is fetched.)
    __shared__ __attribute__((aligned(1024))) char s_stage_all[WPG * kStages * STG];
    __shared__ __attribute__((aligned(256))) int s_cols_all[WPG * 3 * 64];
    __shared__ __attribute__((aligned(256))) int s_desc_all[WPG * kDescWindow * 8];     // the next few item descriptors
    __shared__ __attribute__((aligned(1024))) char s_q_all[WPG * kBlock * (D < 128 ? 128 : D) * 2];   // query rows of the next item (at least 4 KB per wave: a team keeps its block ids there)
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = threadIdx.x & 63;
    char* s_stage = s_stage_all + wv * (kStages * STG);
    int* s_cols = s_cols_all + wv * (3 * 64);
    int* s_desc = s_desc_all + wv * (kDescWindow * 8);
    char* s_q = s_q_all + wv * (kBlock * (D < 128 ? 128 : D) * 2);
    int* hdr = reinterpret_cast<int*>(a.ws);
    const Item* items = reinterpret_cast<const Item*>(a.ws + a.lay.items);
    const int n_items = hdr[H_ITEMS];
    const uint32_t lds_base = __builtin_amdgcn_readfirstlane(
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)s_stage);
    const uint32_t cols_base = __builtin_amdgcn_readfirstlane(
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) int*)s_cols);
    const uint32_t desc_base = __builtin_amdgcn_readfirstlane(
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) int*)s_desc);
    const uint32_t q_base = __builtin_amdgcn_readfirstlane(
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)s_q);

    Lanes L;
    L.n = lane & 15;
    L.kg = lane >> 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if constexpr (D == 128) {
            const int row = 4 * i + L.kg;                          // token row of the block this lane fetches in load i
            L.dma_off[i] = row * 256 + ((L.n ^ row) & 15) * 16;    // LDS chunk position n receives global chunk n ^ row
            L.k_off[i] = L.n * 256 + (((4 * i + L.kg) ^ L.n) & 15) * 16;   // token row n, chunk 4 ks + kg
            const int vrow = 4 * L.kg + i;                         // token row of V k-slot i (and i + 4 in the second block)
            L.v_off[i] = vrow * 256 + ((L.n ^ vrow) & 15) * 16;    // chunk n of that row
        } else if constexpr (D == 64) {
            // head_dim 64: 128-byte token rows of 8 chunks, eight rows per load; position p of row r holds chunk p ^ (r % 8)
            const int row = 8 * (i & 1) + (lane >> 3), pos = lane & 7;
            L.dma_off[i] = row * 128 + ((pos ^ row) & 7) * 16;     // (loads 0 and 1 only)
            L.k_off[i] = L.n * 128 + (((4 * (i & 1) + L.kg) ^ L.n) & 7) * 16;   // token row n, chunk 4 ks + kg (k-steps 0 and 1)
            const int vrow = 4 * L.kg + i;
            L.v_off[i] = vrow * 128 + ((L.n ^ vrow) & 7) * 16;     // chunk n % 8 of that row
        } else {
            // head_dim 256: 512-byte token rows of 32 chunks, two rows per load; each half of a row is swizzled like a
            // 256-byte row (position p of row r holds chunk (p & 16) | ((p ^ r) & 15)); V chunk n + 16 sits 256 bytes on
            const int vrow = 4 * L.kg + i;
            L.v_off[i] = vrow * 512 + ((L.n ^ vrow) & 15) * 16;
        }
    }
    if constexpr (D == 256) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = 2 * i + (lane >> 5), pos = lane & 31;
            L.dma_off[i] = row * 512 + ((pos & 16) | ((pos ^ row) & 15)) * 16;
            const int c = 4 * i + L.kg;                                          // chunk of k-step i
            L.k_off[i] = L.n * 512 + ((c & 16) | ((c ^ L.n) & 15)) * 16;
        }
    }

    // Item descriptors come through LDS too, kDescWindow at a time (one load of 4
    // bytes per lane); a descriptor is made wave-uniform (scalar registers) when it
    // is taken out of the window.
    auto fetch_desc = [&](int first, Stream& sm) {
        dma4(sgpr(items), (uint32_t)min(first * 8 + lane, n_items * 8 - 1) * 4u, desc_base);
        sm.seq += 1;
    };
    int team = 0, rank = 0;   // of the descriptor read last: team size (0: a wave on its own) and rank of a shared run's piece
    auto read_desc = [&](int k) {
        const int4* p = reinterpret_cast<const int4*>(s_desc + k * 8);
        const int4 w0 = p[0], w1 = p[1];
        auto u = [](int v) { return __builtin_amdgcn_readfirstlane(v); };
        Item x;
        const int gt = u(w0.y);
        team = (gt >> 16) & 15;
        rank = (gt >> 20) & 15;
        x.who = u(w0.x); x.g = gt & 0xFFFF; x.nrows = u(w0.z); x.mlist_off = u(w0.w);
        x.c0 = u(w1.x); x.c1 = u(w1.y); x.pbase = u(w1.z); x.tok_end = u(w1.w);
        return x;
    };

    // Which shares this wave sweeps: share, share + grid, ...  Workgroups are dealt
    // round-robin to the 8 XCDs (workgroup id mod 8), each with its own L2, while
    // consecutive shares of a shared run are its row tiles over the same KV bytes.
    // Put every 8 consecutive shares on one XCD so that those bytes are fetched into
    // one L2 once.  (Pure performance: any permutation is correct.)
    int group = blockIdx.x;
    if (xcd_aware && (gridDim.x & 15) == 0) {
        const int x = blockIdx.x & 7, k = blockIdx.x >> 3;
        group = 2 * ((k >> 1) * 8 + x) + (k & 1);
    }
    int share = WPG * group + wv;
    const int n_waves = WPG * (int)gridDim.x;
    const int n_shares = hdr[H_WAVES];
    const int* wave_first = reinterpret_cast<const int*>(a.ws + a.lay.wave_first);
    for (; share < n_shares; share += n_waves) {
        int it = __builtin_amdgcn_readfirstlane(wave_first[share]);
        const int it_end = min(n_items, __builtin_amdgcn_readfirstlane(wave_first[share + 1]));
        if (it >= it_end) continue;
        wait_vmcnt<0>();   // nothing of an earlier share is still on its way into LDS
        wait_lgkmcnt0();
        Stream sm;
        sm.phase = 0;
        sm.iss = 0;
        sm.cb0 = 0; sm.cb1 = 1; sm.cbn = 2;
        sm.cols_ready = false;
        sm.q_ready = false;
        sm.seq = sm.done = 0;
        sm.tmark0 = sm.tmark1 = sm.cmark0 = sm.cmark1 = sm.cmark2 = sm.qmark = 0;
        int win_first = it;
        fetch_desc(win_first, sm);
        wait_all(sm);
        Item item = read_desc(0);
        // A piece of a shared run as this wave's only work, its row tiles on the neighbouring waves of this
        // workgroup: the team sweeps it together if it qualifies (every member sees the same columns, so
        // they all decide alike).  Members without rows of their own only take part in that.
        if constexpr (D == 128) {   // (the team sequence is written for head_dim 128)
            if (a.fast_shared && team >= 2 && it + 1 == it_end && share + n_waves >= n_shares &&
                ((item.c1 - item.c0) & 1) == 0 && item.c1 - item.c0 >= 8 && item.c1 - item.c0 <= kTeamCols &&
                item.tok_end == item.c1 * kBlock && (wv & (team - 1)) == rank) {
                wait_lgkmcnt0();
                const uint32_t ring = sgpr((uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)s_stage_all) +
                                      (team == 2 ? (uint32_t)(wv >> 1) * (2u * kStages * kStageBytes) : 0u);
                sweep_team_core(a, item, team, rank, g_rcp, ring, q_base, lane);
                __builtin_amdgcn_endpgm();   // (not `return`: control must not rejoin the loop, or the loop's values live across the sequence)
            }
        }
        if (item.nrows == 0 && it + 1 == it_end) continue;   // a slot that only exists for a team (or a filler)
        for (;;) {
            const bool has_next = it + 1 < it_end;
            if (has_next && it + 1 - win_first == kDescWindow) {   // window used up: fetch the next one (drains the stream once)
                wait_lgkmcnt0();
                win_first = it + 1;
                fetch_desc(win_first, sm);
                wait_all(sm);
            }
            const Item next = has_next ? read_desc(it + 1 - win_first) : item;
            if (item.nrows <= 16) sweep_item<1, D>(a, item, next, has_next, g_rcp, s_stage, s_cols, s_q, lds_base, cols_base, q_base, L, lane, sm);
            else if (D == 256 || item.nrows <= 32) sweep_item<2, D>(a, item, next, has_next, g_rcp, s_stage, s_cols, s_q, lds_base, cols_base, q_base, L, lane, sm);   // (head_dim 256: the planner makes no item of more than 32 rows)
            else sweep_item<(D == 256 ? 2 : 4), D>(a, item, next, has_next, g_rcp, s_stage, s_cols, s_q, lds_base, cols_base, q_base, L, lane, sm);
            if (!has_next) break;
            ++it;
            item = next;
        }
    }
}

void launch_sweep_mfma(const SweepArgs& a, int head_dim, int grid, const Launch& L) {
    const int g_rcp = (65536 + a.G - 1) / a.G;   // (row * g_rcp) >> 16 == row / G for the 64 rows of an item
    static const int xcd_aware = [] { const char* v = std::getenv("FEA_XCD_AWARE"); return v && *v ? std::atoi(v) : 1; }();
    hipStream_t st = static_cast<hipStream_t>(L.stream);
    hipEvent_t e0 = static_cast<hipEvent_t>(L.ev_start), e1 = static_cast<hipEvent_t>(L.ev_stop);
    if (head_dim == 64) hipExtLaunchKernelGGL(sweep_mfma_kernel<64>, dim3(grid / 4), dim3(256), 0, st, e0, e1, 0, a, g_rcp, xcd_aware);
    else if (head_dim == 256) hipExtLaunchKernelGGL(sweep_mfma_kernel<256>, dim3(grid / 2), dim3(128), 0, st, e0, e1, 0, a, g_rcp, xcd_aware);
    else hipExtLaunchKernelGGL(sweep_mfma_kernel<128>, dim3(grid / 4), dim3(256), 0, st, e0, e1, 0, a, g_rcp, xcd_aware);
}

}  // namespace fea

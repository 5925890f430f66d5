// Device-resident plan of one decode-attention call: which requests alias a
// leading run of KV blocks, how the KV sweep is cut into work items, and where
// each item's partial result goes.  Shared by the planner, the sweep kernels and
// the merge kernel.
#pragma once
#include <cstddef>
#include <cstdint>

namespace fea {

constexpr int kBlock = 16;            // tokens per KV block
constexpr int kPlanThreads = 1024;    // the planner is one workgroup
constexpr int kGroupReqMax = 2048;    // requests with index >= this are never grouped
constexpr int kHashSlots = 4096;      // LDS hash slots for leader finding (2x kGroupReqMax)
constexpr int kTileRows = 64;         // query rows one MFMA work item carries at most
constexpr int kOpenEnded = -2;        // Item::mlist_off of a request's last piece of its own columns

// header words (int32) at the start of the workspace
enum Hdr {
    H_ITEMS = 0,       // number of work items
    H_QUEUE = 1,       // unused (kept zero)
    H_GROUPS = 2,      // prefix groups found
    H_GROUPED = 3,     // requests that belong to a group
    H_SPLIT = 4,       // KV blocks per wave (balanced mode) or per item (fixed split)
    H_ROWS = 5,        // partial rows in use
    H_SHARED_BLOCKS = 6,
    H_VARIANT = 7,     // 0 generic, 1 MFMA, 2 one fused launch (no plan)
    H_OVERFLOW = 8,    // planner ran out of item/partial capacity (never by construction)
    H_WAVES = 9,       // sweep waves that received work
    H_WORDS = 64
};

struct ReqDesc {       // one per request: where the merge finds the partials of its shared run
    int32_t ns_sh;     // pieces of the group's shared run (0 if ungrouped)
    int32_t sh_base0;  // partial row of (KV head 0, piece 0, this request's first query head)
    int32_t sh_gstride;   // partial rows between KV heads
    int32_t sh_pstride;   // partial rows between pieces (= rows of the request's row tile)
    int32_t nb;        // ceil(L / 16)
    int32_t L;
    int32_t group;     // leader request id of its group, or -1
    int32_t priv_c0;   // first private column (= shared run length, 0 if ungrouped)
};

struct GroupDesc {     // indexed by leader request id; valid only where members >= 2
    int32_t leader;
    int32_t members;
    int32_t run;       // aliased leading blocks (full blocks of every member)
    int32_t member_off;   // into the member list
    int32_t tiles;     // row tiles (members are cut into tiles of members_per_tile)
    int32_t seg_base;  // its segments are segs[B*Hkv + seg_base + g*tiles + tile]
    int32_t pad[2];
};

// A segment is one row set x one KV head x a whole column range (a request's
// private columns, or a group row tile's shared run).  It is swept in `npieces`
// consecutive pieces; piece p's partial for the segment's row r is partial row
// pbase + p * rows + r.
struct SegDesc {
    int32_t pbase;
    int32_t npieces;
};

struct Item {          // one KV sweep: a row set x one KV head x a column range (32 bytes)
    int32_t who;       // request whose table row is read (the group's leader for a shared run)
    int32_t g;         // KV head (bits 0-15); pieces of shared runs swept by a team of waves: team size (bits 16-19), rank (bits 20-23)
    int32_t nrows;     // query rows: (requests in the row set) x (group heads)
    int32_t mlist_off; // the row set's request ids start at members[mlist_off]; negative: just `who` (kOpenEnded: and
                       // the piece ends where the request's history ends)
    int32_t c0, c1;    // table columns [c0, c1) of `who`'s row
    int32_t pbase;     // partial row of the item's first query row
    int32_t tok_end;   // tokens at positions >= tok_end are not attended to
};
static_assert(sizeof(Item) == 32, "Item is read as two 16-byte words");

// Byte offsets of the workspace sections (all multiples of 256).
struct WsLayout {
    size_t req, grp, members, segs, wave_first, items, ml, acc, pre, total;
    int32_t max_items, max_rows;
};

// Planner tuning (host constants, overridable through the environment for sweeps).
struct PlanTuning {
    int32_t n_waves;        // sweep waves the work is cut for (the sweep kernel's grid)
    int32_t min_piece;      // a wave gets at least this many 32-token tiles (fewer waves get work instead)
    int32_t min_run;        // shortest aliased run worth sweeping jointly
    int32_t team_fixed;     // what a piece costs a wave of a team of 2 before its first tile and after its last, in the units of the tile weights
    int32_t weights;        // cost of a 32-token tile to the wave that sweeps it, in sixteenths of a 16-row tile a wave streams
                            // alone: with <= 32 query rows | with <= 64 << 8 | as one of a team of 4 waves << 16 | of 2 << 24
};

struct PlanArgs {
    const int32_t* bt;
    const int32_t* seq_lens;
    char* ws;
    WsLayout lay;
    PlanTuning tune;
    int32_t stride, B, Hq, Hkv, G;
    int32_t mpt;         // members (requests) per row tile
    int32_t grouping;    // 0: every request on its own
    int32_t split_user;  // 0: choose
    int32_t variant;
    int32_t teams;       // the sweep runs the row tiles of a shared run's piece as a team of waves (MFMA sweep, head_dim 128)
    int32_t pre;         // leaders and common runs come from run_kernel (workspace section `pre`)
    int32_t pre_grid;    // its grid
};

// What run_kernel leaves for the planner, per groupable request: the run it shares with its
// leader and its own block in the column where that run ends (as one 64-bit word, run in the
// upper half, 0xFFFFFFFF where no such block was seen), then the leaders as int32.
constexpr int kRunThreads = 256;

// Everything the sweep and merge kernels need besides the plan in the workspace.
struct SweepArgs {
    const void* q;
    const void* k_cache;
    const void* v_cache;
    const int32_t* bt;
    const int32_t* seq_lens;
    void* out;
    char* ws;
    WsLayout lay;
    float scale_log2;    // softmax scale times log2(e): scores live in the base-2 domain
    int32_t stride, B, Hq, Hkv, G, mpt;
    int32_t fast_shared;   // q is small enough for 32-bit byte offsets: the hand-scheduled shared-run sequence may be used
};

// launchers (defined next to their kernels); stream is a hipStream_t
// Where a kernel goes: the caller's stream and, when its duration is wanted, a pair of
// events (hipEvent_t, or null) that take the start and the end time of that one dispatch.
struct Launch {
    void* stream;
    void* ev_start;
    void* ev_stop;
    void* ev_mid[2] = {nullptr, nullptr};   // where a step is two dispatches: end of the first, start of the second
};

void launch_plan(const PlanArgs& a, const Launch& L);
void launch_refresh(const PlanArgs& a, const Launch& L);
void launch_sweep_generic(const SweepArgs& a, int dtype, int head_dim, int grid, const Launch& L);
void launch_sweep_mfma(const SweepArgs& a, int head_dim, int grid, const Launch& L);
void launch_merge(const SweepArgs& a, int dtype, int head_dim, bool by_rows, const Launch& L);
void launch_decode_small(const SweepArgs& a, int dtype, int head_dim, const Launch& L);

}  // namespace fea

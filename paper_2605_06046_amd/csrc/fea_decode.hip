// fea_decode_attention: argument checks, workspace carving and the three launches
// (plan, KV sweep, merge), or the one launch that small batches take.  No device memory is allocated here and nothing
// synchronises except fea_decode_plan_info.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdlib>
#include <atomic>
#include <cstring>
#include <mutex>
#include <vector>

#include "../../include/fea.h"
#include "fea_internal.h"
#include "fea_plan.h"

namespace fea {

static size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

static int env_int(const char* name, int dflt) {
    const char* v = std::getenv(name);
    if (!v || !*v) return dflt;
    return std::atoi(v);
}

// Development knobs for tuning sweeps.  The environment is read once, the first time
// a call needs them, and never again: a variable that changes later (or a stale one a
// second thread sets) cannot switch kernels or move the workspace layout between the
// sizing call and the attention call.  What tests need to steer is in fea_attn_params.
struct Knobs {
    int force_generic, sweep_grid, spare_waves, min_piece, min_run, w32, w64, no_fast_shared, w_team, w_team2, team_fixed;
};
static const Knobs& knobs() {
    static const Knobs k = {env_int("FEA_FORCE_GENERIC", 0), env_int("FEA_SWEEP_GRID", 0), env_int("FEA_SPARE_WAVES", 16),
                            env_int("FEA_MIN_PIECE", 4),     env_int("FEA_MIN_RUN", 2),    env_int("FEA_W32", 20),
                            env_int("FEA_W64", 24), env_int("FEA_NO_FAST_SHARED", 0), env_int("FEA_WTEAM", 12),
                            env_int("FEA_WTEAM2", 12), env_int("FEA_TEAM_FIXED", 40)};
    return k;
}

struct Resolved {
    int variant;      // 0 generic, 1 MFMA
    int fused;        // the batch is small enough for the one-launch kernel (no plan, sweep and merge)
    int G, mpt, grouping, split_user, grid;
    int pre, pre_grid;   // leaders and common runs on many workgroups first (large tables)
    int merge_by_rows;   // very many output rows: the merge takes several rows per wave
    PlanTuning tune;
    WsLayout lay;
};

// Optional per-kernel timing: each launch can carry a pair of library-owned events that
// take the start and end time of that dispatch itself (no marker packets in between).
constexpr int kEvPerCall = 8;               // (start, stop) for plan, sweep, merge, and the inner pair of a two-dispatch plan
static std::atomic<bool> g_prof_on{false};  // read without the lock on every call; everything below is under g_prof_mu
static std::mutex g_prof_mu;
static std::vector<hipEvent_t> g_ev_pool;   // kEvPerCall events per recorded call
static int g_prof_calls = 0;                // calls recorded since profiling was switched on
static int g_prof_which = -1;               // -1: all three launches; 0, 1, 2: only that one
static std::vector<unsigned char> g_prof_mask;   // per recorded call: bit k set if launch k was timed

static int cu_count() {
    static int n = 0;
    if (n == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) n = prop.multiProcessorCount;
        if (n <= 0) n = 256;
    }
    return n;
}

// Whether the one-launch kernel is expected to beat plan + sweep + merge.  Both sides are estimates in
// microseconds fitted to measurements (1 to 128 requests, 128 to 4096 tokens, bf16 and float32, head dims 64 to
// 256, query groups of 4 to 65).  The one launch pays, per round of workgroups on the chip and per pass of four
// query heads, a fixed part (the chain of dependent loads, the folds, the barrier) plus vector-unit work per
// token in proportion to the head dim.  The three launches cost their start-up and the planner's one workgroup,
// then the KV bytes of the requests' own columns on the matrix-core path; the vector-unit sweep costs far more
// to start with, and from some hundred thousand (query row, token) pairs on in proportion to them.  The one
// launch is taken where it wins by a tenth (more where its workgroups need several rounds on the chip).
static bool fused_pays(const fea_attn_params* p, int64_t B, int64_t stride, int variant) {
    const bool f32 = p->dtype == FEA_DTYPE_F32;
    const int64_t rounds = (B * p->num_kv_heads + cu_count() - 1) / cu_count();
    const int per_pass = f32 && p->num_q_heads / p->num_kv_heads > 4 ? 8 : 4;   // query heads the kernel takes per pass
    const int64_t passes = (p->num_q_heads / p->num_kv_heads + per_pass - 1) / per_pass;
    const double tokens = (double)stride * kBlock, dd = p->head_dim / 64.0;
    // (passes of one query group run side by side on 2, 4 or 8 sets of the workgroup's waves: their fixed part is
    // paid once per round of passes, their work per token adds up as if they ran one after the other)
    int64_t sets = 1;
    while (sets < 8 && sets < passes) sets <<= 1;
    const int64_t seq = (passes + sets - 1) / sets;
    const double fused_us = 2.4 + (double)rounds * ((double)seq * 6.0 + (double)(seq * sets) * (f32 ? 0.0165 : 0.0096) *
                                                                         (per_pass == 8 ? 1.7 : 1.0) * dd * tokens);
    double planned_us;
    if (variant == 1) {
        planned_us = (B < 2 ? 22.0 : B < 16 ? 27.0 : B <= 64 ? 31.0 : 35.0) + (p->head_dim == 256 ? 4.0 : 0.0) +
                     (0.03 + 0.003 * (double)B) * (double)stride * (p->num_kv_heads * p->head_dim / 1024.0);
    } else {
        const double G = (double)(p->num_q_heads / p->num_kv_heads);   // (the vector sweep passes over its tokens once per 4 or 16 stacked rows)
        const double base = B < 4 ? 20.0 + 1.5 * G : std::min(30.0 + 4.0 * G, 120.0);
        planned_us = (B < 16 ? base : std::max(94.0, base)) * (p->head_dim >= 128 ? 1.4 : 1.0) +
                     (f32 ? 0.027e-3 : 0.0175e-3) * std::pow(dd, 1.6) * (double)(B * p->num_q_heads) * tokens;
    }
    return (1.1 + 0.05 * (double)(rounds - 1)) * fused_us < planned_us;   // (several rounds of workgroups take longer than their sum)
}

static int32_t check_params(const fea_attn_params* p, const char* who) {
    if (!p) return fail(FEA_EINVAL, "%s: params is NULL", who);
    if (p->num_q_heads <= 0 || p->num_kv_heads <= 0 || p->num_q_heads % p->num_kv_heads != 0)
        return fail(FEA_EINVAL, "%s: num_q_heads=%d must be a positive multiple of num_kv_heads=%d", who, p->num_q_heads, p->num_kv_heads);
    if (p->block_size != FEA_BLOCK_TOKENS) return fail(FEA_EINVAL, "%s: block_size=%d, only %d is supported", who, p->block_size, FEA_BLOCK_TOKENS);
    if (p->dtype != FEA_DTYPE_F32 && p->dtype != FEA_DTYPE_BF16) return fail(FEA_EINVAL, "%s: unknown dtype %d", who, p->dtype);
    const int d = p->head_dim;
    const bool d_ok = p->dtype == FEA_DTYPE_F32 ? (d == 32 || d == 64 || d == 128 || d == 256) : (d == 64 || d == 128 || d == 256);
    if (!d_ok) return fail(FEA_EINVAL, "%s: head_dim=%d not supported for this dtype", who, d);
    if (!(p->scale >= 0.f) || !std::isfinite(p->scale)) return fail(FEA_EINVAL, "%s: scale must be finite and >= 0", who);
    if (p->split_blocks < 0 || p->max_group < 0) return fail(FEA_EINVAL, "%s: split_blocks and max_group must be >= 0", who);
    if (p->flags & ~(FEA_FLAG_REUSE_PLAN | FEA_FLAG_PLAN_ONLY | FEA_FLAG_REFRESH_PLAN))
        return fail(FEA_EINVAL, "%s: unknown flag bits 0x%x", who, p->flags);
    const int plan_flags = p->flags & (FEA_FLAG_REUSE_PLAN | FEA_FLAG_PLAN_ONLY | FEA_FLAG_REFRESH_PLAN);
    if (plan_flags & (plan_flags - 1))
        return fail(FEA_EINVAL, "%s: FEA_FLAG_REUSE_PLAN, FEA_FLAG_PLAN_ONLY and FEA_FLAG_REFRESH_PLAN exclude one another", who);
    return FEA_OK;
}

static int32_t resolve(const fea_attn_params* p, int32_t B, int32_t stride, Resolved& r, const char* who) {
    if (B < 0 || stride < 0) return fail(FEA_EINVAL, "%s: negative B or table_stride", who);
    if ((int64_t)B * p->num_q_heads > 0x3FFFFFFF || (int64_t)stride * kBlock > 0x3FFFFFFF)
        return fail(FEA_EINVAL, "%s: problem too large (B*Hq or sequence length overflows)", who);
    // the planner counts 32-token tiles of the whole batch in 32-bit integers
    if ((int64_t)B * p->num_kv_heads * ((stride + 1) / 2) > 0x3FFFFFFF)
        return fail(FEA_EINVAL, "%s: problem too large (B * num_kv_heads * table_stride / 2 exceeds 2^30 tiles)", who);
    const Knobs& kn = knobs();
    r.G = p->num_q_heads / p->num_kv_heads;
    // (a work item's query rows - a request's query group, or stacked ones - fill at most 64 matrix-core rows, 32 at head_dim 256)
    const bool mfma_ok = p->dtype == FEA_DTYPE_BF16 && (p->head_dim == 128 || p->head_dim == 64 || p->head_dim == 256) &&
                         r.G <= (p->head_dim == 256 ? 32 : 64);
    r.variant = (mfma_ok && !kn.force_generic) ? 1 : 0;
    // One launch instead of three where that is estimated to be faster; an explicit bound on the row length stands alone.
    r.fused = p->fused_max < 0 ? 0 : p->fused_max > 0 ? (stride <= p->fused_max) : fused_pays(p, B, stride, r.variant);
    // requests per row tile of a shared run: 64 query rows per work item, 32 on the matrix-core path at head_dim 256
    // (a wave's accumulation registers hold O for 32 rows of 256 dims)
    const int tile_rows = (r.variant == 1 && p->head_dim == 256) ? 32 : kTileRows;
    r.mpt = r.G >= tile_rows ? 1 : tile_rows / r.G;
    r.grouping = p->max_group == 1 ? 0 : 1;
    r.split_user = p->split_blocks > 0 ? ((p->split_blocks + 1) & ~1) : 0;
    // the sweep grid the plan is cut for: one single-wave workgroup per SIMD on the
    // matrix-core path, a few workgroups per CU on the generic path
    r.grid = kn.sweep_grid > 0 ? std::max(4, kn.sweep_grid & ~3) : (r.variant == 1 ? (p->head_dim == 256 ? 2 : 4) : 8) * cu_count();   // waves; four to a workgroup on the matrix-core path (two at head_dim 256)
    // The plan is cut for a few waves fewer than the grid has.  With every one of the
    // 4 x CUs single-wave workgroups busy from start to end, a handful of them (the first
    // ones dispatched) were measured to run about 1.5x longer than the rest, whatever
    // their work; with some workgroups exiting at once this does not happen.
    r.tune.n_waves = std::max(1, r.grid - std::min(r.grid / 2, std::max(0, kn.spare_waves)));
    r.tune.min_piece = std::max(1, kn.min_piece);
    r.tune.min_run = std::max(1, kn.min_run);
    r.tune.team_fixed = std::min(4096, std::max(0, kn.team_fixed));
    r.tune.weights = std::min(255, std::max(16, kn.w32)) | (std::min(255, std::max(16, kn.w64)) << 8) |
                     (std::min(255, std::max(1, kn.w_team)) << 16) | (std::min(127, std::max(1, kn.w_team2)) << 24);
    // Large tables: the rows are compared on many workgroups before the planner's one workgroup
    // takes over (a second launch, so only where the rows are long or many enough to pay for it).
    const int64_t groupable = std::min(B, kGroupReqMax);
    // (measured: 256 requests x 320 columns 30 -> 24 us, 800 x 657 105 -> 35 us; 32 x 2082 no gain, hence
    // the request count; a batch that shares nothing pays about 3 us for it)
    const int run_min = p->run_kernel_min == 0 ? 49152 : p->run_kernel_min;
    r.pre = r.grouping && (run_min < 0 || (groupable >= 128 && groupable * stride >= run_min)) ? 1 : 0;
    r.pre_grid = (int)std::max<int64_t>(1, std::min<int64_t>(2 * cu_count(), (groupable + 3) / 4));
    const int64_t rows = (int64_t)B * p->num_q_heads;
    // Very many rows mean many requests and hence few pieces per row: there a wave of the merge takes
    // several rows (a long shared run cut into many pieces comes with few rows, and keeps a wave per row).
    r.merge_by_rows = (p->merge_rows_min < 0 || rows >= (p->merge_rows_min == 0 ? 8192 : p->merge_rows_min)) ? 1 : 0;
    const int64_t segs = 2ll * B * p->num_kv_heads;          // private segments + at most as many shared ones
    const int64_t rows_per_item = std::max(kTileRows, r.mpt * r.G);
    int64_t max_items, max_rows;
    if (r.split_user > 0) {
        const int64_t per = ((stride + 1) / 2 + r.split_user / 2 - 1) / (r.split_user / 2) + 1;   // pieces per segment
        max_items = segs * per + 64;
        max_rows = 2 * rows * per + 64;
    } else {
        max_items = segs + 5ll * r.grid + 2ll * B + 64;      // pieces of shared runs (with team slots) + cuts of the private stream
        max_rows = 2 * rows + (int64_t)r.grid * (rows_per_item + 2 * r.G) + 64;
    }
    if (max_items > 0x3FFFFFFF || max_rows > 0x3FFFFFFF) return fail(FEA_EINVAL, "%s: split_blocks too small for this problem size", who);
    WsLayout& l = r.lay;
    size_t off = up256(H_WORDS * sizeof(int32_t));
    l.req = off;      off += up256((size_t)B * sizeof(ReqDesc));
    l.grp = off;      off += up256((size_t)B * sizeof(GroupDesc));
    l.members = off;  off += up256((size_t)B * sizeof(int32_t));       // member lists of the groups
    l.segs = off;     off += up256((size_t)segs * sizeof(SegDesc));
    l.wave_first = off; off += up256((size_t)(max_items + 2) * sizeof(int32_t));
    l.items = off;    off += up256((size_t)max_items * sizeof(Item));
    l.ml = off;       off += up256((size_t)max_rows * 2 * sizeof(float));
    l.acc = off;      off += up256((size_t)max_rows * p->head_dim * sizeof(float));
    l.pre = off;      off += up256((size_t)kGroupReqMax * (sizeof(uint64_t) + sizeof(int32_t)));
    l.total = off;
    l.max_items = (int32_t)max_items;
    l.max_rows = (int32_t)max_rows;
    return FEA_OK;
}

}  // namespace fea

using namespace fea;

extern "C" {

int32_t fea_decode_workspace_bytes(const fea_attn_params* p, int32_t B, int32_t table_stride, size_t* out_bytes) {
    if (!out_bytes) return fail(FEA_EINVAL, "fea_decode_workspace_bytes: out_bytes is NULL");
    return decode_workspace_bytes(p, B, table_stride, out_bytes, "fea_decode_workspace_bytes");
}

}  // extern "C"

namespace fea {

int32_t decode_workspace_bytes(const fea_attn_params* p, int32_t B, int32_t table_stride, size_t* out_bytes, const char* who) {
    int32_t rc = check_params(p, who);
    if (rc != FEA_OK) return rc;
    Resolved r;
    rc = resolve(p, B, table_stride, r, who);
    if (rc != FEA_OK) return rc;
    *out_bytes = r.lay.total;
    return FEA_OK;
}

int32_t decode_impl(const fea_attn_params* p, const void* q, const void* k_cache, const void* v_cache,
                    const int32_t* block_tables, int32_t table_stride, const int32_t* seq_lens, int32_t B,
                    void* out, void* workspace, size_t workspace_bytes, void* hip_stream) {
    int32_t rc = check_params(p, "fea_decode_attention");
    if (rc != FEA_OK) return rc;
    Resolved r;
    rc = resolve(p, B, table_stride, r, "fea_decode_attention");
    if (rc != FEA_OK) return rc;
    if (B == 0) return FEA_OK;
    const bool plan_only = (p->flags & FEA_FLAG_PLAN_ONLY) != 0;
    if (!block_tables || !seq_lens || !workspace || (!plan_only && (!q || !k_cache || !v_cache || !out)))
        return fail(FEA_EINVAL, "fea_decode_attention: NULL device pointer");
    if (((uintptr_t)workspace & 255) != 0) return fail(FEA_EINVAL, "fea_decode_attention: workspace must be 256-byte aligned");
    if (((uintptr_t)q & 15) || ((uintptr_t)k_cache & 15) || ((uintptr_t)v_cache & 15) || ((uintptr_t)out & 15))
        return fail(FEA_EINVAL, "fea_decode_attention: q, caches and out must be 16-byte aligned");
    if (workspace_bytes < r.lay.total)
        return fail(FEA_ERANGE, "fea_decode_attention: workspace has %zu bytes, %zu needed", workspace_bytes, r.lay.total);

    const float scale = p->scale > 0.f ? p->scale : 1.0f / std::sqrt((float)p->head_dim);
    Launch where[3] = {{hip_stream, nullptr, nullptr}, {hip_stream, nullptr, nullptr}, {hip_stream, nullptr, nullptr}};
    std::unique_lock<std::mutex> prof_lock(g_prof_mu, std::defer_lock);
    if (g_prof_on.load(std::memory_order_relaxed)) prof_lock.lock();   // (calls of several threads take their slots one after the other)
    if (prof_lock.owns_lock() && g_prof_on.load() && !g_ev_pool.empty()) {
        const size_t slot = (size_t)(g_prof_calls % (int)(g_ev_pool.size() / kEvPerCall));
        hipEvent_t* ev = &g_ev_pool[kEvPerCall * slot];
        unsigned char mask = 0;
        for (int k = 0; k < 3; ++k) {
            if (g_prof_which >= 0 && g_prof_which != k) continue;
            if (k == 0 && ((p->flags & FEA_FLAG_REUSE_PLAN) || (r.fused && !plan_only))) continue;
            if (k > 0 && plan_only) continue;
            if (k == 2 && r.fused) continue;
            where[k].ev_start = ev[2 * k];
            where[k].ev_stop = ev[2 * k + 1];
            if (k == 0) { where[0].ev_mid[0] = ev[6]; where[0].ev_mid[1] = ev[7]; }
            mask |= (unsigned char)(1u << k);
        }
        g_prof_mask[slot] = mask;
        ++g_prof_calls;
    }
    if (prof_lock.owns_lock()) prof_lock.unlock();
    if (!(p->flags & FEA_FLAG_REUSE_PLAN) && (plan_only || !r.fused)) {   // a new plan, or the one in the workspace stretched to the lengths of now
        PlanArgs pa;
        std::memset(&pa, 0, sizeof pa);
        pa.bt = block_tables;
        pa.seq_lens = seq_lens;
        pa.ws = static_cast<char*>(workspace);
        pa.lay = r.lay;
        pa.tune = r.tune;
        pa.stride = table_stride;
        pa.B = B;
        pa.Hq = p->num_q_heads;
        pa.Hkv = p->num_kv_heads;
        pa.G = r.G;
        pa.mpt = r.mpt;
        pa.grouping = r.grouping;
        pa.split_user = r.split_user;
        pa.variant = r.variant;
        pa.teams = (r.variant == 1 && p->head_dim == 128 && !knobs().no_fast_shared) ? 1 : 0;
        pa.pre = r.pre;
        pa.pre_grid = r.pre_grid;
        if (p->flags & FEA_FLAG_REFRESH_PLAN) launch_refresh(pa, where[0]);
        else launch_plan(pa, where[0]);
    }
    if (plan_only) {
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail(FEA_EHIP, "fea_decode_attention: launch failed: %s", hipGetErrorString(e));
        return FEA_OK;
    }
    SweepArgs sa;
    std::memset(&sa, 0, sizeof sa);
    sa.q = q;
    sa.k_cache = k_cache;
    sa.v_cache = v_cache;
    sa.bt = block_tables;
    sa.seq_lens = seq_lens;
    sa.out = out;
    sa.ws = static_cast<char*>(workspace);
    sa.lay = r.lay;
    sa.scale_log2 = scale * 1.4426950408889634f;
    sa.stride = table_stride;
    sa.B = B;
    sa.Hq = p->num_q_heads;
    sa.Hkv = p->num_kv_heads;
    sa.G = r.G;
    sa.mpt = r.mpt;
    sa.fast_shared = (p->head_dim == 128 && (int64_t)B * p->num_q_heads < (1 << 23) && !knobs().no_fast_shared) ? 1 : 0;
    if (r.fused) {
        launch_decode_small(sa, p->dtype, p->head_dim, where[1]);
    } else {
        if (r.variant == 1) launch_sweep_mfma(sa, p->head_dim, r.grid, where[1]);
        else launch_sweep_generic(sa, p->dtype, p->head_dim, r.grid, where[1]);
        launch_merge(sa, p->dtype, p->head_dim, r.merge_by_rows != 0, where[2]);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(FEA_EHIP, "fea_decode_attention: launch failed: %s", hipGetErrorString(e));
    return FEA_OK;
}

}  // namespace fea

extern "C" {

int32_t fea_decode_attention(const fea_attn_params* p, const void* q, const void* k_cache, const void* v_cache,
                             const int32_t* block_tables, int32_t table_stride, const int32_t* seq_lens, int32_t B,
                             void* out, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return decode_impl(p, q, k_cache, v_cache, block_tables, table_stride, seq_lens, B, out, workspace, workspace_bytes,
                       hip_stream);
}

// A tool that intercepts the launches (rocprofv3 loads its library through this variable)
// times every dispatch itself; the library's own per-dispatch events are not attached then.
static bool profiler_attached() {
    const char* v = std::getenv("ROCP_TOOL_LIBRARIES");
    return v && *v;
}

int32_t fea_profile_enable(int32_t max_calls, int32_t which) {
    if (max_calls < 0 || max_calls > 65536) return fail(FEA_EINVAL, "fea_profile_enable: max_calls=%d out of range", max_calls);
    if (which < -1 || which > 2) return fail(FEA_EINVAL, "fea_profile_enable: which=%d, expected -1, 0, 1 or 2", which);
    if (max_calls > 0 && profiler_attached())
        return fail(FEA_EINVAL, "fea_profile_enable: a profiling tool is attached to this process (ROCP_TOOL_LIBRARIES); "
                                "it times the dispatches itself, the library's events stay off");
    return guarded("fea_profile_enable", [&]() -> int32_t {
    std::lock_guard<std::mutex> lock(g_prof_mu);
    g_prof_which = which;
    while ((int)g_ev_pool.size() < kEvPerCall * max_calls) {
        hipEvent_t ev;
        const hipError_t e = hipEventCreate(&ev);
        if (e != hipSuccess) return fail(FEA_EHIP, "fea_profile_enable: %s", hipGetErrorString(e));
        g_ev_pool.push_back(ev);
    }
    g_prof_mask.assign(g_ev_pool.size() / kEvPerCall, 0);
    g_prof_on = max_calls > 0;
    g_prof_calls = 0;
    return FEA_OK;
    });
}

int32_t fea_profile_read(int32_t call, float* ms) {
    if (!ms) return fail(FEA_EINVAL, "fea_profile_read: ms is NULL");
    std::lock_guard<std::mutex> lock(g_prof_mu);
    const int slots = (int)(g_ev_pool.size() / kEvPerCall);
    if (call < 0 || call >= g_prof_calls || g_prof_calls - call > slots)
        return fail(FEA_EINVAL, "fea_profile_read: call %d was not recorded (or its events were reused)", call);
    const size_t slot = (size_t)(call % slots);
    hipEvent_t* ev = &g_ev_pool[kEvPerCall * slot];
    hipError_t e = hipSuccess;
    for (int k = 0; k < 3; ++k) {
        ms[k] = 0.f;
        if (!(g_prof_mask[slot] & (1u << k)) || e != hipSuccess) continue;
        e = hipEventSynchronize(ev[2 * k + 1]);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms[k], ev[2 * k], ev[2 * k + 1]);
    }
    if (e != hipSuccess) return fail(FEA_EHIP, "fea_profile_read: %s", hipGetErrorString(e));
    return FEA_OK;
}

int32_t fea_decode_plan_info(const void* workspace, void* hip_stream, int32_t* info) {
    if (!workspace || !info) return fail(FEA_EINVAL, "fea_decode_plan_info: NULL pointer");
    int32_t hdr[H_WORDS];
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    hipError_t e = hipMemcpyAsync(hdr, workspace, sizeof hdr, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) return fail(FEA_EHIP, "fea_decode_plan_info: %s", hipGetErrorString(e));
    info[0] = hdr[H_ITEMS];
    info[1] = hdr[H_GROUPS];
    info[2] = hdr[H_GROUPED];
    info[3] = hdr[H_SPLIT];
    info[4] = hdr[H_ROWS];
    info[5] = hdr[H_SHARED_BLOCKS];
    info[6] = hdr[H_VARIANT];
    info[7] = hdr[H_OVERFLOW];
    info[8] = hdr[H_WAVES];
    return FEA_OK;
}

}  // extern "C"

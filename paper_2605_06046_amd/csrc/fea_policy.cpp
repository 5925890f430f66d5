// Learned stop policies of batch formation (Section 4.3 "Batching and
// Reinforcement Learning": contextual bandit with UCB selection, tabular
// Q-learning with epsilon-greedy exploration; appendix "Batch Formation").
// Host code only.
//
// Both policies share one dense table indexed by the discretised state
// (b bin, loss bin, peers bin) and the action.  A decision appends its table
// index to the open episode; the reward of the executed batch closes the
// episode and is folded into the table.  All arithmetic is in double, in the
// order the update rules state it, so results do not depend on table layout.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <new>
#include <memory>
#include <vector>

#include "../../include/fea.h"
#include "fea_internal.h"

using fea::fail;

struct fea_policy {
    fea_policy_params prm;
    int32_t loss_bins;
    std::vector<double> acc;        // UCB: summed reward; Q-learning: Q
    std::vector<int64_t> cnt;       // times credited / updated
    std::vector<int32_t> episode;   // entry index (state * 2 + action) per open decision
    int64_t decisions = 0, episodes = 0;
    double eps = 0.0;

    int32_t state_index(int32_t sb, int32_t sl, int32_t sw) const { return (sb * loss_bins + sl) * prm.w_bins + sw; }
};

namespace {

int32_t exp_bin(int32_t x, int32_t bins) {
    if (x <= 0) return 0;
    const int32_t k = 31 - __builtin_clz((uint32_t)x);      // floor(log2 x)
    return std::min(1 + k, bins - 1);
}

int32_t loss_bin(const fea_policy* p, int32_t loss) {
    int32_t n = 0;
    for (int32_t i = 0; i < p->prm.n_loss_thresholds; ++i) n += loss > p->prm.loss_thresholds[i];
    return n;
}

bool unit(double x) { return x >= 0.0 && x <= 1.0; }

}  // namespace

extern "C" {

int32_t fea_policy_create(const fea_policy_params* q, fea_policy** out) {
    return fea::guarded("fea_policy_create", [&]() -> int32_t {
        if (!q || !out) return fail(FEA_EINVAL, "fea_policy_create: NULL argument");
        if (q->kind != FEA_POLICY_UCB && q->kind != FEA_POLICY_QLEARN)
            return fail(FEA_EINVAL, "fea_policy_create: unknown kind %d", q->kind);
        if (q->b_bins < 1 || q->b_bins > 64 || q->w_bins < 1 || q->w_bins > 64 || q->n_loss_thresholds < 0 ||
            q->n_loss_thresholds > FEA_POLICY_MAX_THRESHOLDS)
            return fail(FEA_EINVAL, "fea_policy_create: bins %d x %d or %d thresholds out of range", q->b_bins, q->w_bins,
                        q->n_loss_thresholds);
        for (int32_t i = 1; i < q->n_loss_thresholds; ++i)
            if (q->loss_thresholds[i] <= q->loss_thresholds[i - 1])
                return fail(FEA_EINVAL, "fea_policy_create: loss thresholds must ascend");
        if (q->kind == FEA_POLICY_UCB && !(q->c >= 0.0)) return fail(FEA_EINVAL, "fea_policy_create: c must be >= 0");
        if (q->kind == FEA_POLICY_QLEARN &&
            !(q->alpha > 0.0 && q->alpha <= 1.0 && unit(q->gamma) && unit(q->eps) && unit(q->eps_min) && unit(q->eps_decay)))
            return fail(FEA_EINVAL, "fea_policy_create: alpha in (0,1], gamma, eps, eps_min, eps_decay in [0,1] required");
        std::unique_ptr<fea_policy> p(new fea_policy());   // (a failing allocation below must not leak it)
        p->prm = *q;
        p->loss_bins = q->n_loss_thresholds + 1;
        const size_t n = (size_t)q->b_bins * p->loss_bins * q->w_bins * 2;
        p->acc.assign(n, 0.0);
        p->cnt.assign(n, 0);
        p->eps = q->kind == FEA_POLICY_QLEARN ? q->eps : 0.0;
        *out = p.release();
        return FEA_OK;
    });
}

void fea_policy_destroy(fea_policy* p) { delete p; }

int32_t fea_policy_state(const fea_policy* p, int32_t b, int32_t loss, int32_t peers, int32_t* sb, int32_t* sl,
                         int32_t* sw) {
    if (!p) return fail(FEA_EINVAL, "fea_policy_state: NULL policy");
    if (sb) *sb = exp_bin(b, p->prm.b_bins);
    if (sl) *sl = loss_bin(p, loss);
    if (sw) *sw = exp_bin(peers, p->prm.w_bins);
    return FEA_OK;
}

int32_t fea_policy_decide(fea_policy* p, int32_t b, int32_t loss, int32_t peers, double u_explore, double u_action,
                          int32_t* action) {
    return fea::guarded("fea_policy_decide", [&]() -> int32_t {
        if (!p || !action) return fail(FEA_EINVAL, "fea_policy_decide: NULL argument");
        const int32_t s = p->state_index(exp_bin(b, p->prm.b_bins), loss_bin(p, loss), exp_bin(peers, p->prm.w_bins));
        const int32_t ia = 2 * s + FEA_ADD, is = 2 * s + FEA_STOP;
        int32_t a;
        if (p->prm.kind == FEA_POLICY_UCB) {
            if (p->cnt[ia] == 0) a = FEA_ADD;
            else if (p->cnt[is] == 0) a = FEA_STOP;
            else {
                const double lnS = std::log((double)p->decisions);
                const double ua = p->acc[ia] / (double)p->cnt[ia] + p->prm.c * std::sqrt(lnS / (double)p->cnt[ia]);
                const double us = p->acc[is] / (double)p->cnt[is] + p->prm.c * std::sqrt(lnS / (double)p->cnt[is]);
                a = ua >= us ? FEA_ADD : FEA_STOP;
            }
        } else {
            if (u_explore < p->eps) a = u_action < 0.5 ? FEA_ADD : FEA_STOP;
            else a = p->acc[ia] >= p->acc[is] ? FEA_ADD : FEA_STOP;
        }
        p->episode.push_back(2 * s + a);
        *action = a;
        return FEA_OK;
    });
}

int32_t fea_policy_reward(fea_policy* p, double r) {
    return fea::guarded("fea_policy_reward", [&]() -> int32_t {
        if (!p) return fail(FEA_EINVAL, "fea_policy_reward: NULL policy");
        if (!std::isfinite(r)) return fail(FEA_EINVAL, "fea_policy_reward: reward is not finite");
        const size_t T = p->episode.size();
        if (p->prm.kind == FEA_POLICY_UCB) {
            for (size_t i = 0; i < T; ++i) {
                p->acc[p->episode[i]] += r;
                p->cnt[p->episode[i]] += 1;
            }
        } else {
            for (size_t i = 0; i < T; ++i) {
                const bool last = i + 1 == T;
                double future = 0.0;
                if (!last) {
                    const int32_t ns = p->episode[i + 1] & ~1;
                    future = std::max(p->acc[ns + FEA_ADD], p->acc[ns + FEA_STOP]);
                }
                const double ri = (p->prm.reward_every_step || last) ? r : 0.0;
                double& q = p->acc[p->episode[i]];
                q = q + p->prm.alpha * (ri + p->prm.gamma * future - q);
                p->cnt[p->episode[i]] += 1;
            }
            p->eps = std::max(p->prm.eps_min, p->eps * p->prm.eps_decay);
        }
        p->decisions += (int64_t)T;
        p->episodes += 1;
        p->episode.clear();
        return FEA_OK;
    });
}

int32_t fea_policy_entry(const fea_policy* p, int32_t sb, int32_t sl, int32_t sw, int32_t action, double* value,
                         int64_t* count) {
    if (!p) return fail(FEA_EINVAL, "fea_policy_entry: NULL policy");
    if (sb < 0 || sb >= p->prm.b_bins || sl < 0 || sl >= p->loss_bins || sw < 0 || sw >= p->prm.w_bins ||
        (action != FEA_ADD && action != FEA_STOP))
        return fail(FEA_ERANGE, "fea_policy_entry: (%d, %d, %d, %d) outside the table", sb, sl, sw, action);
    const int32_t i = 2 * p->state_index(sb, sl, sw) + action;
    if (value) *value = p->prm.kind == FEA_POLICY_UCB ? (p->cnt[i] ? p->acc[i] / (double)p->cnt[i] : 0.0) : p->acc[i];
    if (count) *count = p->cnt[i];
    return FEA_OK;
}

int32_t fea_policy_info(const fea_policy* p, int64_t* decisions, int64_t* episodes, double* eps, int32_t* open) {
    if (!p) return fail(FEA_EINVAL, "fea_policy_info: NULL policy");
    if (decisions) *decisions = p->decisions;
    if (episodes) *episodes = p->episodes;
    if (eps) *eps = p->eps;
    if (open) *open = (int32_t)p->episode.size();
    return FEA_OK;
}

int32_t fea_cht_build_batch_learned(fea_cht* t, fea_policy* p, int32_t max_batch, const double* draws, int64_t* ids,
                                    int32_t* n_out) {
    return fea::guarded("fea_cht_build_batch_learned", [&]() -> int32_t {
        if (!t || !p || !ids || !n_out || max_batch < 0)
            return fail(FEA_EINVAL, "fea_cht_build_batch_learned: bad argument");
        if (!draws && p->prm.kind != FEA_POLICY_UCB)
            return fail(FEA_EINVAL, "fea_cht_build_batch_learned: this policy needs draws");
        int32_t n = 0;
        while (n < max_batch) {
            int64_t id;
            int32_t before, after, peers, action;
            if (fea_cht_find_best(t, &id, &before, &after, &peers, nullptr) != FEA_OK) break;
            const int32_t k = n;      // decisions so far in this call: every earlier one was an ADD
            int32_t rc = fea_policy_decide(p, n, before - after, peers, draws ? draws[2 * k] : 0.0,
                                           draws ? draws[2 * k + 1] : 0.0, &action);
            if (rc != FEA_OK) return rc;
            if (action == FEA_STOP) break;
            rc = fea_cht_add_to_batch(t, id);
            if (rc != FEA_OK) return rc;
            ids[n++] = id;
        }
        *n_out = n;
        return FEA_OK;
    });
}

}  // extern "C"

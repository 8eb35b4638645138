// Host scheduler: turns predicted response lengths into micro-batches.
//
// Paper Sec. 4.1 (Method): sort the group by predicted length and split it into
// batches; Binning paragraph: lengths are scheduled by the upper edge of a fixed-size
// bin; FCR paragraph: the cap on new tokens is the largest predicted length in the
// batch and overrunning rows are recomputed after the group; VBS paragraph: the batch
// size keeps the tokens per batch constant (inverse proportionality, see the header).
// Integers only; no GPU.
#include "ss_internal.h"

#include <algorithm>
#include <cstring>
#include <memory>
#include <numeric>
#include <vector>

namespace {

struct PlanStorage {
    ss_plan pub;                 // must stay first: the public pointer is this object
    std::vector<int32_t> offsets, idx, cap;
};

int check_policy(const ss_policy* p, int32_t bin)
{
    if (!p) return ss::fail(SS_EINVAL, "policy is NULL");
    if (bin < 0) return ss::fail(SS_EINVAL, "bin must be >= 0");
    if (p->base_batch < 1) return ss::fail(SS_EINVAL, "base_batch must be >= 1");
    if (p->max_batch < p->base_batch) return ss::fail(SS_EINVAL, "max_batch must be >= base_batch");
    if (p->base_len < 1) return ss::fail(SS_EINVAL, "base_len must be >= 1");
    if ((p->flags & SS_BIN) && !(p->flags & SS_SORT)) return ss::fail(SS_EINVAL, "SS_BIN needs SS_SORT");
    if ((p->flags & SS_BIN) && bin == 0) return ss::fail(SS_EINVAL, "SS_BIN needs bin > 0");
    if ((p->flags & SS_VBS) && !(p->flags & SS_SORT)) return ss::fail(SS_EINVAL, "SS_VBS needs SS_SORT");
    if (p->vbs_rule != SS_VBS_CLAMP_FLOOR && p->vbs_rule != SS_VBS_PAPER_POW2)
        return ss::fail(SS_EINVAL, "unknown vbs_rule");
    if (p->flags & ~(SS_SORT | SS_BIN | SS_FCR | SS_VBS | SS_COMPACT)) return ss::fail(SS_EINVAL, "unknown flag");
    return SS_OK;
}

// Length a query is scheduled by (Sec. 4.1 Binning: round up to the covering bin; the top bin is the
// one that holds the global limit).
inline int64_t sched_len(int32_t pred, int32_t bin, const ss_policy& p)
{
    if (!(p.flags & SS_BIN)) return pred;
    const int64_t w = bin;
    const int64_t ub = ((static_cast<int64_t>(pred) + w - 1) / w) * w;
    const int64_t top = ((static_cast<int64_t>(p.base_len) + w - 1) / w) * w;
    return std::min(ub, top);
}

// Batch size for a scheduled length L (Sec. 4.1 VBS; Sec. 4.2 for the power-of-two variant).
inline int32_t batch_size(int64_t L, const ss_policy& p)
{
    if (!(p.flags & SS_VBS)) return p.base_batch;
    if (p.vbs_rule == SS_VBS_PAPER_POW2) {
        if (L >= 300) return 16;
        // nearest power of two to 12800/L: compare in exact integer arithmetic,
        // x - lo <= hi - x  <=>  2*12800 <= (lo + hi) * L
        int64_t lo = 1;
        while (lo * 2 * L <= 12800) lo *= 2;
        const int64_t hi = lo * 2;
        return static_cast<int32_t>((2 * 12800 <= (lo + hi) * L) ? lo : hi);
    }
    const int64_t b = (static_cast<int64_t>(p.base_batch) * p.base_len) / L;
    return static_cast<int32_t>(std::max<int64_t>(p.base_batch, std::min<int64_t>(p.max_batch, b)));
}

ss_plan* finish(std::unique_ptr<PlanStorage> s)
{
    s->pub.n = static_cast<int32_t>(s->idx.size());
    s->pub.n_mb = static_cast<int32_t>(s->cap.size());
    s->pub.mb_offsets = s->offsets.data();
    s->pub.query_idx = s->idx.data();
    s->pub.mb_cap = s->cap.data();
    return &s.release()->pub;   // the caller owns it from here: ss_plan_free
}

void emit(PlanStorage* s, const int32_t* rows, int32_t count, int32_t cap)
{
    s->idx.insert(s->idx.end(), rows, rows + count);
    s->offsets.push_back(static_cast<int32_t>(s->idx.size()));
    s->cap.push_back(cap);
}

int schedule_impl(const int32_t* pred_lens, int32_t n, int32_t bin, const ss_policy* policy, ss_plan** out)
{
    if (!out) return ss::fail(SS_EINVAL, "out is NULL");
    if (n <= 0) return ss::fail(SS_EINVAL, "n must be > 0");
    if (int rc = check_policy(policy, bin)) return rc;
    const ss_policy& p = *policy;
    const bool sorted = (p.flags & SS_SORT) != 0;
    if (sorted && !pred_lens) return ss::fail(SS_EINVAL, "pred_lens is NULL but SS_SORT is set");
    if (sorted)
        for (int32_t i = 0; i < n; ++i)
            if (pred_lens[i] < 1) return ss::fail(SS_EINVAL, "pred_lens[%d] = %d < 1", i, pred_lens[i]);

    std::unique_ptr<PlanStorage> plan(new PlanStorage());
    PlanStorage* s = plan.get();
    s->offsets.push_back(0);
    std::vector<int32_t> order(n);
    std::iota(order.begin(), order.end(), 0);

    if (!sorted) {  // vanilla: arrival order, fixed batch, global cap
        for (int32_t b = 0; b < n; b += p.base_batch) emit(s, &order[b], std::min(p.base_batch, n - b), p.base_len);
        *out = finish(std::move(plan));
        return SS_OK;
    }

    std::vector<int64_t> L(n);
    for (int32_t i = 0; i < n; ++i) L[i] = sched_len(pred_lens[i], bin, p);
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return L[a] < L[b]; });
    const bool fcr = (p.flags & SS_FCR) != 0;
    auto cap_of = [&](int64_t longest) {
        return fcr ? static_cast<int32_t>(std::min<int64_t>(longest, p.base_len)) : p.base_len;
    };

    int32_t at = 0;
    while (at < n) {
        if (p.flags & SS_BIN) {
            // one bin = a run of equal scheduled lengths; chunk it alone
            int32_t end = at;
            while (end < n && L[order[end]] == L[order[at]]) ++end;
            const int64_t ub = L[order[at]];
            const int32_t bs = batch_size(ub, p);
            for (int32_t c = at; c < end; c += bs) emit(s, &order[c], std::min(bs, end - c), cap_of(ub));
            at = end;
        } else {
            int32_t end;
            if (p.flags & SS_VBS) {
                // longest chunk whose size fits the batch size allowed for its largest prediction
                end = at + 1;
                while (end < n && (end - at + 1) <= batch_size(L[order[end]], p)) ++end;
            } else {
                end = std::min(n, at + p.base_batch);
            }
            emit(s, &order[at], end - at, cap_of(L[order[end - 1]]));
            at = end;
        }
    }
    *out = finish(std::move(plan));
    return SS_OK;
}

int schedule_failures_impl(const int32_t* pred_lens, int32_t n, const int32_t* failed_idx, int32_t n_failed,
                           int32_t bin, const ss_policy* policy, ss_plan** out)
{
    if (!out) return ss::fail(SS_EINVAL, "out is NULL");
    if (n <= 0 || n_failed < 0 || n_failed > n) return ss::fail(SS_EINVAL, "bad n / n_failed");
    if (int rc = check_policy(policy, bin)) return rc;
    if (n_failed > 0 && !failed_idx) return ss::fail(SS_EINVAL, "failed_idx is NULL");
    const ss_policy& p = *policy;
    std::vector<int32_t> order(failed_idx, failed_idx + n_failed);
    for (int32_t i : order)
        if (i < 0 || i >= n) return ss::fail(SS_EINVAL, "failed index %d out of range", i);
    if (pred_lens && (p.flags & SS_SORT)) {
        for (int32_t i : order)
            if (pred_lens[i] < 1) return ss::fail(SS_EINVAL, "pred_lens[%d] < 1", i);
        std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
            const int64_t la = sched_len(pred_lens[a], bin, p), lb = sched_len(pred_lens[b], bin, p);
            return la != lb ? la < lb : a < b;
        });
    }
    std::unique_ptr<PlanStorage> plan(new PlanStorage());
    PlanStorage* s = plan.get();
    s->offsets.push_back(0);
    for (int32_t b = 0; b < n_failed; b += p.base_batch)
        emit(s, &order[b], std::min(p.base_batch, n_failed - b), p.base_len);
    *out = finish(std::move(plan));
    return SS_OK;
}

}  // namespace

// The entry points hand no C++ exception to the caller: a plan that does not fit the host's memory is SS_ENOMEM.
extern "C" int ss_schedule(const int32_t* pred_lens, int32_t n, int32_t bin, const ss_policy* policy, ss_plan** out)
{
    return ss::no_throw([&] { return schedule_impl(pred_lens, n, bin, policy, out); });
}

extern "C" int ss_schedule_failures(const int32_t* pred_lens, int32_t n, const int32_t* failed_idx, int32_t n_failed,
                                    int32_t bin, const ss_policy* policy, ss_plan** out)
{
    return ss::no_throw([&] { return schedule_failures_impl(pred_lens, n, failed_idx, n_failed, bin, policy, out); });
}

extern "C" void ss_plan_free(ss_plan* plan)
{
    if (plan) delete reinterpret_cast<PlanStorage*>(plan);
}

// Scheduler-side planning of libes (declared in include/es_sched.h): the analytical
// performance model of paper section 3.4, Eq. 1a-1d, and the plan search under it.
// Host arithmetic only; nothing here touches a device.
//
// Search.  For fixed GPU counts the estimate is maxP / f_overload, so the best
// allocation is the one with the shortest global step.  A step time t admits at most
// cap_i(t) = max{a : a / C[i] <= t} ESTs per GPU of type i, and the GPUs can hold the job
// iff every used type admits one EST and sum N[i] * cap_i(t) >= maxP; that is monotone in
// t, and the optimum is of the form a / C[i], so a bisection over a per type finds it.
// Over-provisioning is then minimised exactly: the sums sum N[i] * A[i] reachable with
// 1 <= A[i] <= cap_i are built type by type as bit sets (only sums below maxP + max N[i]
// matter: a larger reachable sum can always give one place back).
#include "es.h"
#include "es_sched.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

namespace {

struct Problem {
    uint32_t K = 0;
    const double* C = nullptr;
    uint32_t max_p = 0;
};

bool valid_types(uint32_t n_types, const double* capability)
{
    if (n_types == 0 || n_types > ES_SCHED_MAX_TYPES || !capability) return false;
    for (uint32_t i = 0; i < n_types; ++i)
        if (!(capability[i] > 0.0) || !std::isfinite(capability[i])) return false;
    return true;
}

// Eq. 1a-1d in the order the header states them.  N and A are valid on entry.
void evaluate(const Problem& pr, const uint32_t* N, const uint32_t* A, bool per_gpu, es_sched_plan* out)
{
    std::memset(out, 0, sizeof(*out));
    uint64_t n_est = 0, n_gpus = 0;
    for (uint32_t i = 0; i < pr.K; ++i) {
        out->n_used[i] = N[i];
        out->est_per_gpu[i] = N[i] ? A[i] : 0;
        n_est += (uint64_t)N[i] * out->est_per_gpu[i];                    // 1a
        n_gpus += N[i];
    }
    double f = 0.0;
    for (uint32_t i = 0; i < pr.K; ++i)
        if (N[i]) f = std::max(f, (double)A[i] / pr.C[i]);               // 1b
    double waste = 0.0;
    for (uint32_t i = 0; i < pr.K; ++i) {
        if (!N[i]) continue;
        const double idle = pr.C[i] - (double)A[i] / f;
        waste = waste + (per_gpu ? (double)N[i] * idle : idle);
    }
    waste = waste + (double)(n_est - pr.max_p) / f;                      // 1c
    double cap = 0.0;
    for (uint32_t i = 0; i < pr.K; ++i) cap = cap + (double)N[i] * pr.C[i];
    out->n_gpus = (uint32_t)n_gpus;
    out->n_est = (uint32_t)n_est;
    out->f_overload = f;
    out->waste = waste;
    out->throughput = cap - waste;                                       // 1d
}

// max{a in 0..max_p : a / c <= t}, decided by the same division the model uses
uint32_t cap_at(double t, double c, uint32_t max_p)
{
    double g = std::floor(t * c);
    uint32_t a = g <= 0.0 ? 0u : g >= (double)max_p ? max_p : (uint32_t)g;
    while (a < max_p && (double)(a + 1) / c <= t) ++a;
    while (a > 0 && (double)a / c > t) --a;
    return a;
}

bool feasible(const Problem& pr, const uint32_t* N, double t)
{
    uint64_t places = 0;
    for (uint32_t i = 0; i < pr.K; ++i) {
        if (!N[i]) continue;
        const uint32_t c = cap_at(t, pr.C[i], pr.max_p);
        if (c == 0) return false;
        places += (uint64_t)N[i] * c;
    }
    return places >= pr.max_p;
}

struct BitSet {
    std::vector<uint64_t> w;
    explicit BitSet(size_t bits) : w((bits + 63) / 64, 0) {}
    bool test(size_t i) const { return (w[i >> 6] >> (i & 63)) & 1; }
    void set(size_t i) { w[i >> 6] |= 1ull << (i & 63); }
    // this |= other << s, truncated to this set's size
    void or_shifted(const BitSet& o, size_t s)
    {
        const size_t ws = s >> 6, bs = s & 63;
        for (size_t k = w.size(); k-- > ws;) {
            uint64_t v = o.w[k - ws] << bs;
            if (bs && k > ws) v |= o.w[k - ws - 1] >> (64 - bs);
            w[k] |= v;
        }
    }
};

// Best allocation for fixed N (valid: some N[i] > 0, sum N <= max_p).
void best_mapping(const Problem& pr, const uint32_t* N, es_sched_plan* out)
{
    // shortest feasible step time: per type the smallest a with a / C[i] feasible
    double best_t = 0.0;
    bool have = false;
    for (uint32_t i = 0; i < pr.K; ++i) {
        if (!N[i]) continue;
        uint32_t lo = 1, hi = pr.max_p;                 // a = max_p is feasible only if every other type
        if (!feasible(pr, N, (double)hi / pr.C[i])) continue;   // admits an EST by then
        while (lo < hi) {
            const uint32_t mid = lo + (hi - lo) / 2;
            if (feasible(pr, N, (double)mid / pr.C[i])) hi = mid; else lo = mid + 1;
        }
        const double t = (double)lo / pr.C[i];
        if (!have || t < best_t) { best_t = t; have = true; }
    }
    // `have` always ends true: the slowest used type at a = max_p admits everything

    uint32_t used[ES_SCHED_MAX_TYPES], cap[ES_SCHED_MAX_TYPES], nu = 0, max_n = 0;
    for (uint32_t i = 0; i < pr.K; ++i)
        if (N[i]) {
            used[nu] = i;
            cap[nu] = cap_at(best_t, pr.C[i], pr.max_p);
            max_n = std::max(max_n, N[i]);
            ++nu;
        }
    // reachable sums of the types j.. (suffix sets), truncated below max_p + max_n
    const size_t bits = (size_t)pr.max_p + max_n;
    std::vector<BitSet> reach(nu + 1, BitSet(bits));
    reach[nu].set(0);
    for (uint32_t j = nu; j-- > 0;) {
        const uint32_t n = N[used[j]];
        for (uint32_t a = 1; a <= cap[j] && (size_t)n * a < bits; ++a) reach[j].or_shifted(reach[j + 1], (size_t)n * a);
    }
    size_t target = pr.max_p;
    while (target < bits && !reach[0].test(target)) ++target;
    // target < bits always: some reachable sum >= max_p exists (feasibility), and giving one
    // place back at a time from it passes through [max_p, max_p + max_n)
    uint32_t A[ES_SCHED_MAX_TYPES] = {0};
    if (target >= bits) {                               // unreachable; keep a valid plan regardless
        for (uint32_t j = 0; j < nu; ++j) A[used[j]] = cap[j];
        evaluate(pr, N, A, true, out);
        return;
    }
    size_t rest = target;
    for (uint32_t j = 0; j < nu; ++j) {
        const uint32_t n = N[used[j]];
        for (uint32_t a = 1; a <= cap[j]; ++a) {
            const size_t take = (size_t)n * a;
            if (take <= rest && reach[j + 1].test(rest - take)) {
                A[used[j]] = a;
                rest -= take;
                break;
            }
        }
    }
    evaluate(pr, N, A, true, out);
}

bool ranks_before(const es_sched_plan& a, const es_sched_plan& b, uint32_t K)
{
    if (a.f_overload != b.f_overload) return a.f_overload < b.f_overload;
    if (a.n_gpus != b.n_gpus) return a.n_gpus < b.n_gpus;
    if (a.n_est != b.n_est) return a.n_est < b.n_est;
    for (uint32_t i = 0; i < K; ++i)
        if (a.n_used[i] != b.n_used[i]) return a.n_used[i] < b.n_used[i];
    for (uint32_t i = 0; i < K; ++i)
        if (a.est_per_gpu[i] != b.est_per_gpu[i]) return a.est_per_gpu[i] < b.est_per_gpu[i];
    return false;
}

}  // namespace

extern "C" {

int es_sched_evaluate(uint32_t n_types, const double* capability, const uint32_t* n_used,
                      const uint32_t* est_per_gpu, uint32_t max_p, int waste_reading,
                      es_sched_plan* out)
{
    if (!valid_types(n_types, capability) || !n_used || !est_per_gpu || !out) return ES_EINVAL;
    if (max_p == 0 || max_p > 65535) return ES_EINVAL;
    if (waste_reading != ES_SCHED_WASTE_PER_GPU && waste_reading != ES_SCHED_WASTE_AS_PRINTED) return ES_EINVAL;
    uint64_t n_est = 0, n_gpus = 0;
    for (uint32_t i = 0; i < n_types; ++i) {
        if (n_used[i] > 65535) return ES_EINVAL;
        if (n_used[i] && (est_per_gpu[i] == 0 || est_per_gpu[i] > 65535)) return ES_EINVAL;
        n_gpus += n_used[i];
        n_est += (uint64_t)n_used[i] * (n_used[i] ? est_per_gpu[i] : 0);
    }
    if (n_gpus == 0 || n_est < max_p || n_est > 0xffffffffull) return ES_EINVAL;
    Problem pr;
    pr.K = n_types; pr.C = capability; pr.max_p = max_p;
    evaluate(pr, n_used, est_per_gpu, waste_reading == ES_SCHED_WASTE_PER_GPU, out);
    return ES_OK;
}

int es_sched_best_mapping(uint32_t n_types, const double* capability, const uint32_t* n_used,
                          uint32_t max_p, es_sched_plan* out)
try {
    if (!valid_types(n_types, capability) || !n_used || !out) return ES_EINVAL;
    if (max_p == 0 || max_p > ES_SCHED_MAX_P) return ES_EINVAL;
    uint64_t n_gpus = 0;
    for (uint32_t i = 0; i < n_types; ++i) {
        if (n_used[i] > max_p) return ES_EINVAL;
        n_gpus += n_used[i];
    }
    if (n_gpus == 0 || n_gpus > max_p) return ES_EINVAL;
    Problem pr;
    pr.K = n_types; pr.C = capability; pr.max_p = max_p;
    best_mapping(pr, n_used, out);
    return ES_OK;
} catch (const std::bad_alloc&) {
    return ES_ENOMEM;
}

int es_sched_enumerate(uint32_t n_types, const double* capability, const uint32_t* available,
                       uint32_t max_p, uint32_t top_k, es_sched_plan* out, uint32_t* n_out)
try {
    if (!valid_types(n_types, capability) || !available || !out || !n_out || top_k == 0) return ES_EINVAL;
    if (max_p == 0 || max_p > ES_SCHED_MAX_P) return ES_EINVAL;
    uint64_t combos = 1;
    for (uint32_t i = 0; i < n_types; ++i) {
        if (available[i] > 65535) return ES_EINVAL;
        combos *= (uint64_t)available[i] + 1;
        if (combos > (1ull << 20)) return ES_EINVAL;
    }
    // one best-mapping search per count vector costs on the order of max_p steps: bound the product
    if (combos * (uint64_t)max_p > (1ull << 27)) return ES_EINVAL;
    Problem pr;
    pr.K = n_types; pr.C = capability; pr.max_p = max_p;
    std::vector<es_sched_plan> best;                  // ranked, at most top_k entries
    best.reserve(std::min<uint64_t>(top_k, combos));
    uint32_t N[ES_SCHED_MAX_TYPES] = {0};
    for (uint64_t c = 1; c < combos; ++c) {
        // next vector of GPU counts, last type fastest
        for (uint32_t i = n_types; i-- > 0;) {
            if (N[i] < available[i]) { ++N[i]; break; }
            N[i] = 0;
        }
        uint64_t n_gpus = 0;
        for (uint32_t i = 0; i < n_types; ++i) n_gpus += N[i];
        if (n_gpus > max_p) continue;
        es_sched_plan p;
        best_mapping(pr, N, &p);
        if (best.size() == top_k && !ranks_before(p, best.back(), n_types)) continue;
        auto pos = std::upper_bound(best.begin(), best.end(), p,
                                    [&](const es_sched_plan& a, const es_sched_plan& b) { return ranks_before(a, b, n_types); });
        best.insert(pos, p);
        if (best.size() > top_k) best.pop_back();
    }
    for (size_t k = 0; k < best.size(); ++k) out[k] = best[k];
    *n_out = (uint32_t)best.size();
    return ES_OK;
} catch (const std::bad_alloc&) {
    return ES_ENOMEM;
}

int es_sched_grouping(uint32_t n_types, const es_sched_plan* plan, uint32_t max_p,
                      uint32_t* worker_of_est, uint32_t* slot_of_est, uint32_t* n_workers)
try {
    if (n_types == 0 || n_types > ES_SCHED_MAX_TYPES || !plan || !worker_of_est || !slot_of_est || !n_workers)
        return ES_EINVAL;
    if (max_p == 0 || max_p > 65535) return ES_EINVAL;
    std::vector<uint32_t> quota;
    uint64_t places = 0;
    for (uint32_t i = 0; i < n_types; ++i) {
        const uint32_t n = plan->n_used[i], a = plan->est_per_gpu[i];
        if (n > 65535 || (n && (a == 0 || a > 65535))) return ES_EINVAL;
        if (quota.size() + n > max_p) return ES_EINVAL;              // more GPUs than ESTs
        quota.insert(quota.end(), n, a);
        places += (uint64_t)n * a;
    }
    if (quota.empty() || places < max_p) return ES_EINVAL;
    uint64_t slack = places - max_p;
    while (slack > 0)                                                 // ends: sum(quota) > max_p >= #GPUs
        for (size_t g = quota.size(); g-- > 0 && slack > 0;)
            if (quota[g] > 1) { --quota[g]; --slack; }
    uint32_t e = 0;
    for (size_t g = 0; g < quota.size(); ++g)
        for (uint32_t s = 0; s < quota[g]; ++s, ++e) {
            worker_of_est[e] = (uint32_t)g;
            slot_of_est[e] = s;
        }
    *n_workers = (uint32_t)quota.size();
    return ES_OK;
} catch (const std::bad_alloc&) {
    return ES_ENOMEM;
}

}  // extern "C"

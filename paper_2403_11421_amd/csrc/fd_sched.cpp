// Host-side scheduling arithmetic of FastDecode Section 4.2 (Eq. 5, Eq. 6, Figure 7,
// Algorithm 1).  Integer only; see fastdecode_sched.h for the conventions.
#include <algorithm>
#include <cmath>
#include <new>
#include <vector>

#include "fastdecode_rpart.h"
#include "fastdecode_sched.h"

struct fd_load_ctl {
    int64_t S, W_lim;
    std::vector<int64_t> M, E, W;
};

namespace {

// load contributed at step s by m sequences started at step t0 (0 outside their S steps)
inline int64_t contribution(int64_t m, int64_t t0, int64_t S, int64_t s)
{
    const int64_t age = s - t0;
    return (age >= 0 && age < S) ? m * (age + 1) : 0;
}

} // namespace

extern "C" {

int64_t fd_sls_microbatch_size(int64_t B, int64_t F, int64_t S)
{
    if (B <= 0 || F <= 0 || S <= 0) return FD_EINVAL;
    return std::max<int64_t>(1, B * F / S);
}

int64_t fd_sls_peak_load(int64_t M, int64_t F, int64_t S)
{
    if (M <= 0 || F <= 0 || S <= 0) return FD_EINVAL;
    int64_t w = 0;
    for (int64_t k = 1; k <= S / F; ++k) w += M * k * F;
    return w;
}

int fd_sls_step_loads(int64_t M, int64_t F, int64_t S, int64_t n_steps, int64_t *loads)
{
    if (M <= 0 || F <= 0 || S <= 0 || n_steps < 0 || (n_steps > 0 && !loads)) return FD_EINVAL;
    for (int64_t s = 0; s < n_steps; ++s) {
        // micro-batches alive at step s started at multiples of F in (s - S, s]
        int64_t w = 0;
        for (int64_t t0 = s - s % F; t0 >= 0 && t0 > s - S; t0 -= F) w += contribution(M, t0, S, s);
        loads[s] = w;
    }
    return FD_OK;
}

int fd_batch_step_loads(int64_t B, int64_t S, int64_t n_steps, int64_t *loads)
{
    if (B <= 0 || S <= 0 || n_steps < 0 || (n_steps > 0 && !loads)) return FD_EINVAL;
    for (int64_t s = 0; s < n_steps; ++s) loads[s] = B * (s % S + 1);
    return FD_OK;
}

fd_load_ctl *fd_lc_create(int64_t S, int64_t W_lim)
{
    if (S <= 0 || W_lim <= 0) return nullptr;
    fd_load_ctl *lc = new (std::nothrow) fd_load_ctl;
    if (lc) { lc->S = S; lc->W_lim = W_lim; }
    return lc;
}

void fd_lc_destroy(fd_load_ctl *lc) { delete lc; }

int fd_lc_add_microbatch(fd_load_ctl *lc, int64_t t, int64_t m)
{
    if (!lc || m <= 0) return FD_EINVAL;
    // the new micro-batch's length at the last step of every one that already runs
    int64_t own = m * lc->S;
    for (size_t i = 0; i < lc->M.size(); ++i) {
        if (lc->E[i] > t) lc->W[i] += (lc->E[i] - t) * m;
        // a micro-batch started at this same step is as long as the new one at its last step
        // (the paper's listing assumes one start per step and has no such term)
        if (lc->E[i] == t + lc->S) own += lc->M[i] * lc->S;
    }
    lc->M.push_back(m);
    lc->E.push_back(t + lc->S);
    lc->W.push_back(own);
    return FD_OK;
}

int64_t fd_lc_earliest_step(const fd_load_ctl *lc, int64_t t, int64_t m)
{
    if (!lc || m <= 0 || t < 0) return FD_EINVAL;
    if (m > lc->W_lim / lc->S) return FD_EINVAL;             // m*S alone exceeds the limit: never admissible
    // A micro-batch of m sequences started at step r < E[i] is E[i] - r tokens long at the last
    // step E[i] - 1 of micro-batch i, so it adds m * (E[i] - r) to W[i].  Keeping
    // W[i] + m * (E[i] - r) <= W_lim means E[i] - r <= x with x = floor((W_lim - W[i]) / m),
    // i.e. r >= E[i] - x; with no room at all (x <= 0) the start has to wait until i has ended.
    int64_t r = t;
    for (size_t i = 0; i < lc->M.size(); ++i) {
        if (lc->E[i] <= t) continue;                          // already finished: not current
        const int64_t margin = lc->W_lim - lc->W[i];
        int64_t x = margin / m;                               // floor division (margin may be negative)
        if (margin % m != 0 && margin < 0) --x;
        r = std::max(r, lc->E[i] - std::max<int64_t>(x, 0));
    }
    return r;
}

int64_t fd_lc_controlled_starts(int64_t B, int64_t S, int64_t M, int64_t F, int64_t W_lim,
                                int64_t n_steps, int64_t *starts, int64_t max_starts)
{
    if (B <= 0 || S <= 0 || M <= 0 || F <= 0 || W_lim <= 0 || n_steps < 0 || max_starts < 0 ||
        (max_starts > 0 && !starts) || B % M != 0 || M > W_lim / S)
        return FD_EINVAL;
    fd_load_ctl lc;
    lc.S = S;
    lc.W_lim = W_lim;
    std::vector<int64_t> free_at((size_t)(B / M), 0);         // step from which a group of M slots is free
    int64_t waiting = 0, n = 0;
    for (int64_t t = 0; t < n_steps; ++t) {
        if (t % F == 0) ++waiting;                            // a micro-batch arrives
        fd_lc_retire(&lc, t);
        const size_t g = (size_t)(std::min_element(free_at.begin(), free_at.end()) - free_at.begin());
        if (waiting > 0 && free_at[g] <= t && fd_lc_earliest_step(&lc, t, M) <= t) {
            fd_lc_add_microbatch(&lc, t, M);
            free_at[g] = t + S;
            if (n < max_starts) starts[n] = t;
            ++n;
            --waiting;
        }
    }
    return n;
}

int64_t fd_lc_retire(fd_load_ctl *lc, int64_t t)
{
    if (!lc) return FD_EINVAL;
    size_t keep = 0;
    for (size_t i = 0; i < lc->M.size(); ++i) {
        if (lc->E[i] > t) {
            lc->M[keep] = lc->M[i];
            lc->E[keep] = lc->E[i];
            lc->W[keep] = lc->W[i];
            ++keep;
        }
    }
    const int64_t dropped = (int64_t)(lc->M.size() - keep);
    lc->M.resize(keep);
    lc->E.resize(keep);
    lc->W.resize(keep);
    return dropped;
}

int64_t fd_lc_count(const fd_load_ctl *lc) { return lc ? (int64_t)lc->M.size() : FD_EINVAL; }

int64_t fd_lc_snapshot(const fd_load_ctl *lc, int64_t n, int64_t *M, int64_t *E, int64_t *W)
{
    if (!lc || n < 0 || (n > 0 && (!M || !E || !W))) return FD_EINVAL;
    const int64_t c = std::min<int64_t>(n, (int64_t)lc->M.size());
    for (int64_t i = 0; i < c; ++i) { M[i] = lc->M[i]; E[i] = lc->E[i]; W[i] = lc->W[i]; }
    return c;
}

// ---------------------------------------------------------------------------
// Slot free list (Section 4.1: dropped sequences hand their slot to later ones)
// ---------------------------------------------------------------------------
struct fd_slots {
    std::vector<int32_t> free_ids;      // stack of free slots; back() is handed out next
    std::vector<char> taken;
};

fd_slots *fd_slots_create(int32_t B)
{
    if (B <= 0) return nullptr;
    fd_slots *s = new (std::nothrow) fd_slots;
    if (!s) return nullptr;
    s->taken.assign((size_t)B, 0);
    s->free_ids.resize((size_t)B);
    for (int32_t i = 0; i < B; ++i) s->free_ids[(size_t)i] = B - 1 - i;    // slot 0 first
    return s;
}

void fd_slots_destroy(fd_slots *s) { delete s; }

int32_t fd_slots_acquire(fd_slots *s)
{
    if (!s) return FD_EINVAL;
    if (s->free_ids.empty()) return FD_SLOT_FREE;
    const int32_t id = s->free_ids.back();
    s->free_ids.pop_back();
    s->taken[(size_t)id] = 1;
    return id;
}

int fd_slots_release(fd_slots *s, int32_t id)
{
    if (!s || id < 0 || (size_t)id >= s->taken.size() || !s->taken[(size_t)id]) return FD_EINVAL;
    s->taken[(size_t)id] = 0;
    s->free_ids.push_back(id);
    return FD_OK;
}

int32_t fd_slots_in_use(const fd_slots *s)
{
    return s ? (int32_t)(s->taken.size() - s->free_ids.size()) : FD_EINVAL;
}

// ---------------------------------------------------------------------------
// Section 4.3: batch size and number of R-workers from two measured quantities
// ---------------------------------------------------------------------------
double fd_model_sequence_latency(int64_t N, int64_t S, double T_B)
{
    if (N <= 0 || S <= 0 || !(T_B > 0)) return std::nan("");
    return 2.0 * (double)N * (double)S * T_B;
}

int64_t fd_model_max_batch(int64_t N, int64_t S, double L, const int64_t *Bs, const double *T,
                           int64_t n)
{
    if (N <= 0 || S <= 0 || !(L > 0) || n < 0 || (n > 0 && (!Bs || !T))) return FD_EINVAL;
    int64_t best = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (Bs[i] <= 0 || !(T[i] > 0)) return FD_EINVAL;
        if (fd_model_sequence_latency(N, S, T[i]) <= L) best = std::max(best, Bs[i]);
    }
    return best;
}

double fd_model_sworker_throughput(int64_t B, double T_B)
{
    if (B <= 0 || !(T_B > 0)) return std::nan("");
    return (double)B / T_B;
}

int64_t fd_model_min_rworkers_memory(int64_t B, int64_t S, int64_t C)
{
    if (B <= 0 || S <= 0 || C <= 0) return FD_EINVAL;
    if (B > INT64_MAX / S) return FD_EINVAL;
    const int64_t twoC = 2 * C;                      // B*S/2 <= C*P  <=>  P >= B*S / (2C)
    return (B * S + twoC - 1) / twoC;
}

double fd_model_num_rworkers(int64_t B, int64_t S, double R, double T_B)
{
    if (B <= 0 || S <= 0 || !(R > 0) || !(T_B > 0)) return std::nan("");
    return (double)B * (double)S * R / (2.0 * T_B);
}

} // extern "C"

// What this library was built from: the build step passes a hash of the sources, headers and
// compiler flags, and the binding refuses (or rebuilds) a library whose hash is not the tree's.
#ifndef FD_BUILD_ID
#define FD_BUILD_ID "unknown"
#endif
extern "C" const char *fd_build_id(void) { return FD_BUILD_ID; }

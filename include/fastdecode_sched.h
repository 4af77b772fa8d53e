/*
 * fastdecode_sched.h -- host-side scheduling arithmetic of FastDecode (arXiv 2403.11421),
 * Section 4.2: the sequence-level load-stabilising schedule (Eq. 5, Eq. 6, Figure 7) and
 * the load-control bookkeeping of Algorithm 1.  Pure integer host code in the same shared
 * library as the GPU kernels; it decides which sequences exist at which length, i.e. the
 * ragged seq_lens the R-Part kernels see.  Nothing here touches a device.
 *
 * Step convention (fixed by Figure 7's worked example): a sequence started at step t has
 * length s - t + 1 at step s and lives for S steps, s = t .. t+S-1; a step's load is the sum
 * of the lengths of the sequences alive at that step.
 *
 * All functions return negative FD_E* codes (fastdecode_rpart.h) on bad arguments.
 */
#ifndef FASTDECODE_SCHED_H
#define FASTDECODE_SCHED_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Eq. 5: micro-batch size M = B*F/S of the schedule that starts a micro-batch every F
 * steps and keeps about B sequences in flight.  Requires B, F, S > 0; rounds down, at least 1. */
int64_t fd_sls_microbatch_size(int64_t B, int64_t F, int64_t S);

/* Eq. 6: peak total length W'max = sum_{k=1..S/F} M*k*F of that schedule (= B(S+F)/2 when F
 * divides S and S divides B*F).  Computed from the sum, not from the closed form. */
int64_t fd_sls_peak_load(int64_t M, int64_t F, int64_t S);

/* Per-step total load, loads[0..n_steps), of micro-batches of M sequences started every F
 * steps from step 0 (Figure 7, lower half).  `loads` is a host array owned by the caller. */
int fd_sls_step_loads(int64_t M, int64_t F, int64_t S, int64_t n_steps, int64_t *loads);

/* Per-step total load when all B sequences start together and the next batch starts when
 * they finish (Figure 7, upper half). */
int fd_batch_step_loads(int64_t B, int64_t S, int64_t n_steps, int64_t *loads);

/*
 * Algorithm 1 (load control).  The object keeps, for every current micro-batch i, its size
 * M[i], its ending step E[i] = start + S (exclusive) and W[i], the total load at its last
 * step E[i]-1, where the load peaks.
 *   fd_lc_add_microbatch(t, m): records a micro-batch of m sequences started at step t:
 *       appends (m, t+S, m*S) and adds (E[i]-t)*m to W[i] of every micro-batch that
 *       existed before the call (the new one's length at their last step).
 *   fd_lc_earliest_step(t, m): GetEarliestStep: the smallest step r >= t at which a
 *       micro-batch of m sequences can start without pushing any W[i] over W_lim.  A start at
 *       r < E[i] adds m * (E[i] - r) to W[i], so with x = floor((W_lim - W[i]) / m) the bound
 *       is r >= E[i] - max(x, 0), taken over the current micro-batches.  (The paper's listing
 *       prints E[i] - x + 1, the bound for an E[i] that is the last step itself; with
 *       E[i] = start + S as AddMicroBatch sets it, that is one step later than the load
 *       definition of Figure 7 requires.)  FD_EINVAL if t < 0 or if m * S alone exceeds
 *       W_lim, in which case no step is ever admissible.
 *   fd_lc_retire(t): forgets micro-batches with E[i] <= t ("current" means still running).
 * The handle is host memory owned by the library until fd_lc_destroy.
 */
typedef struct fd_load_ctl fd_load_ctl;
fd_load_ctl *fd_lc_create(int64_t S, int64_t W_lim);
void fd_lc_destroy(fd_load_ctl *lc);
int fd_lc_add_microbatch(fd_load_ctl *lc, int64_t t, int64_t m);
int64_t fd_lc_earliest_step(const fd_load_ctl *lc, int64_t t, int64_t m);
int64_t fd_lc_retire(fd_load_ctl *lc, int64_t t);
int64_t fd_lc_count(const fd_load_ctl *lc);
/* Copies up to `n` entries of (M[i], E[i], W[i]) into the caller's arrays; returns the count. */
int64_t fd_lc_snapshot(const fd_load_ctl *lc, int64_t n, int64_t *M, int64_t *E, int64_t *W);

/*
 * The admission loop of Algorithm 1's driver, start to finish, for micro-batches of M
 * sequences that arrive every F steps (Eq. 5's schedule) on an R-worker with room for B
 * sequences (B / M groups of slots, B a multiple of M; a group is busy for S steps):
 * arrivals wait in order; at every step 0 .. n_steps-1 the one at the head starts if a group
 * of slots is free and fd_lc_earliest_step allows that step, at most one start per step.
 * Writes the start steps, in order, to starts[0 .. min(count, max_starts)) (host array owned
 * by the caller) and returns the count.  With W_lim >= Eq. 6's peak every micro-batch starts
 * on arrival (the fixed-interval schedule of Figure 7); with a tighter limit starts are held
 * back and the load never exceeds it.
 */
int64_t fd_lc_controlled_starts(int64_t B, int64_t S, int64_t M, int64_t F, int64_t W_lim,
                                int64_t n_steps, int64_t *starts, int64_t max_starts);

/*
 * Slot bookkeeping for an R-worker with room for B sequences (Section 4.1: the cache of a
 * sequence is dropped when its generation ends; its slot and block are handed to the next
 * sequence).  A host-side free list; the device side of a slot is fd_kv_release / fd_kv_reset.
 *   fd_slots_acquire  a free slot id (the most recently released one first; 0, 1, 2, ... while
 *                     none has been released), or
 *                     FD_SLOT_FREE (-1) when all B are taken.
 *   fd_slots_release  returns slot `id`; FD_EINVAL if it is out of range or already free.
 */
typedef struct fd_slots fd_slots;
fd_slots *fd_slots_create(int32_t B);
void fd_slots_destroy(fd_slots *s);
int32_t fd_slots_acquire(fd_slots *s);
int fd_slots_release(fd_slots *s, int32_t id);
int32_t fd_slots_in_use(const fd_slots *s);

/*
 * Section 4.3 (workload-balanced hardware selection).  T_B is the measured latency of the
 * S-Part of one transformer block at batch size B, R the measured R-Part latency of one
 * R-worker per cached token and block, both in the same time unit; N blocks, sequences of
 * up to S tokens.  The double-valued functions return NaN on bad arguments.
 *   fd_model_sequence_latency   Eq. 7, left side: 2 * N * S * T(B), the time to generate one
 *                               sequence when S-Part and R-Part take equally long.
 *   fd_model_max_batch          Eq. 7: the largest batch size of a measured table
 *                               (Bs[i], T[i]), i < n, whose sequence latency is <= L;
 *                               0 if none qualifies.
 *   fd_model_sworker_throughput Eq. 8: E(B) = B / T(B).
 *   fd_model_min_rworkers_memory  Eq. 9: the least P with B*S/2 <= C*P, C = tokens of K and V
 *                               one R-worker can hold.
 *   fd_model_num_rworkers       Eq. 11: P = B*S*R / (2*T(B)) = S*R*E(B)/2, not rounded.
 */
double fd_model_sequence_latency(int64_t N, int64_t S, double T_B);
int64_t fd_model_max_batch(int64_t N, int64_t S, double L, const int64_t *Bs, const double *T,
                           int64_t n);
double fd_model_sworker_throughput(int64_t B, double T_B);
int64_t fd_model_min_rworkers_memory(int64_t B, int64_t S, int64_t C);
double fd_model_num_rworkers(int64_t B, int64_t S, double R, double T_B);

/*
 * Identifies the build: a hash of the sources, headers and compiler flags this library was made
 * from ("unknown" when the build step passed none).  The Python binding compares it with the hash
 * of the tree it sits in, so that a library left over from other sources is never tested or timed
 * unnoticed.  Not part of the method.
 */
const char *fd_build_id(void);

#ifdef __cplusplus
}
#endif
#endif /* FASTDECODE_SCHED_H */

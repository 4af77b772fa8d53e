// R-Part of FastDecode (arXiv 2403.11421) for gfx950: KV append, ragged planner,
// split-K streaming attention and log-sum-exp merge, behind the C ABI declared
// in fastdecode_rpart.h.
//
// The path is a batched matrix-vector product and bound by memory traffic (Section 3.1):
// one flop per KV byte, so everything here is organised around streaming each K and V row
// from HBM exactly once with 128-bit coalesced loads; no matrix cores.
//
// Lane mapping of the streaming kernel (d = 128): a row of K or V is 256 B =
// 16 lanes x 16 B, so one wave64 load instruction covers 4 consecutive tokens
// (1 KB contiguous).  Each lane keeps the 8 query elements of its column slice
// in registers; the q.k dot product is finished by a 4-step DPP butterfly inside
// the 16-lane row; each 16-lane row runs its own online softmax over "its"
// tokens, so the value accumulation needs no cross-lane traffic in the loop.
// d = 64 uses 8 lanes per row and 8 tokens per wave load.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fastdecode_rpart.h"

// ---------------------------------------------------------------------------
// Built-in scratch for the entry point that allocates nothing.  The array lives in every
// device's copy of the code object; host code must not use its name as an address (that is a
// host-side stand-in): the device address is asked for once per device and kept.
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[FD_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int kVersion = 100;          // 0.1.0
constexpr int kWaves = 4;              // waves per workgroup of the streaming kernel
constexpr int kThreads = kWaves * 64;
constexpr int kPlanThreads = 1024;
constexpr int kPhases = 4;             // starting points of the workgroups' walks through their rounds
constexpr int kHdrInts = 64;           // 256-byte header
constexpr float kNegBig = -1.0e30f;    // "no token seen yet" running max (finite: no inf-inf)

// header words
enum { HDR_NITEMS = 0, HDR_CHUNK = 2, HDR_TOKENS = 3, HDR_GRID = 4, HDR_MAGIC = 5, HDR_B = 6,
       HDR_H = 7, HDR_MAXITEMS = 8, HDR_WAVE_UNITS = 9, HDR_KIND = 10, HDR_BUMP = 11,
       HDR_STATUS_OUT = 16 };
// cache format a plan was made for: head dimension and bits per element (16 = fp16)
constexpr int plan_kind(int d, int bits) { return d | (bits << 16); }
constexpr int32_t kPlanMagic = 0x46445251;

struct WsLayout {
    size_t off_item0;     // int32[B]  first item of sequence b
    size_t off_nchunk;    // int32[B]  chunks of sequence b
    size_t off_newlen;    // int32[B]  length of sequence b after the step's append (fused append + plan)
    size_t off_newseen;   // int32[B]  tokens seen by sequence b after that append (windowed caches)
    size_t off_items;     // int4[max_items]  {b, t0, t1, n_chunks_of_b}, chunks of a sequence adjacent
    size_t off_order;     // int32[max_items] item indices, longest chunk first (the schedule)
    size_t off_cnt;       // int32[max_items][H]  finished chunks of a split (sequence, head), at its first item
    size_t off_acc;       // float[max_items][H][d]  unnormalised weighted value sums (512 B records)
    size_t off_ml;        // float[max_items][H][2]  {running max, sum of exponentials}
    int64_t max_items;
    size_t min_bytes;     // bytes needed for max_items == B
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

inline size_t ws_per_item(int H, int d) { return 16 + 4 + (size_t)H * 4 + (size_t)H * (size_t)(d + 2) * 4; }

inline WsLayout ws_layout(int B, int H, int d, size_t ws_bytes)
{
    WsLayout w;
    size_t o = kHdrInts * sizeof(int32_t);
    w.off_item0 = o;
    o = align_up(o + (size_t)B * 4, 256);
    w.off_nchunk = o;
    o = align_up(o + (size_t)B * 4, 256);
    w.off_newlen = o;
    o = align_up(o + (size_t)B * 4, 256);
    w.off_newseen = o;
    o = align_up(o + (size_t)B * 4, 256);
    w.off_items = o;
    const size_t per_item = ws_per_item(H, d);
    const size_t slop = 5 * 256;                         // alignment of the five arrays
    w.min_bytes = o + slop + (size_t)(B > 0 ? B : 1) * per_item;
    w.max_items = 0;
    w.off_order = w.off_cnt = w.off_acc = w.off_ml = 0;
    if (ws_bytes < w.min_bytes) return w;
    w.max_items = (int64_t)((ws_bytes - o - slop) / per_item);
    if (w.max_items > (int64_t)0x3FFFFFFF) w.max_items = 0x3FFFFFFF;
    const size_t n = (size_t)w.max_items;
    w.off_order = align_up(w.off_items + n * 16, 256);
    w.off_cnt = align_up(w.off_order + n * 4, 256);
    w.off_acc = align_up(w.off_cnt + n * (size_t)H * 4, 256);
    w.off_ml = align_up(w.off_acc + n * (size_t)H * (size_t)d * 4, 256);
    return w;
}

// The plan as the kernels see it: pointers into the workspace.
struct PlanView {
    int32_t *hdr, *item0, *nchunk, *newlen, *newseen;
    int4 *items;
    int32_t *order, *cnt;
    float *acc, *ml;
    int max_items;
};

inline PlanView plan_view(void *workspace, const WsLayout &w)
{
    char *ws = (char *)workspace;
    PlanView v;
    v.hdr = (int32_t *)ws;
    v.item0 = (int32_t *)(ws + w.off_item0);
    v.nchunk = (int32_t *)(ws + w.off_nchunk);
    v.newlen = (int32_t *)(ws + w.off_newlen);
    v.newseen = (int32_t *)(ws + w.off_newseen);
    v.items = (int4 *)(ws + w.off_items);
    v.order = (int32_t *)(ws + w.off_order);
    v.cnt = (int32_t *)(ws + w.off_cnt);
    v.acc = (float *)(ws + w.off_acc);
    v.ml = (float *)(ws + w.off_ml);
    v.max_items = (int)w.max_items;
    return v;
}

// ---------------------------------------------------------------------------
// Append (Section 4.1).
// ---------------------------------------------------------------------------
// Where the new token of a sequence goes: the row, or -1 when the append is skipped (free slot,
// full plain cache, inconsistent window state; *err is the FD_ST_* bit to report, 0 for a free
// slot).  *new_len / *new_seen: the length and the tokens seen after the append (unchanged when
// it is skipped).  L = seq_lens[b], cap = seq_cap[b], p = seq_seen[b] (windowed caches only).
__device__ inline int append_rule(int L, int cap, bool windowed, int p, int n_sink, int *new_len,
                                  int *new_seen, int *err)
{
    *new_len = L;
    *new_seen = p;
    *err = 0;
    if (L == FD_SLOT_FREE) return -1;
    if (!windowed) {
        if (L < 0 || L >= cap) {
            *err = FD_ST_CAPACITY;
            return -1;
        }
        *new_len = L + 1;
        return L;
    }
    // windowed cache: a bounded buffer of n_sink fixed rows and a ring of cap - n_sink rows
    if (n_sink < 0 || n_sink >= cap || p < 0 || L != (p < cap ? p : cap)) {
        *err = FD_ST_WINDOW;
        return -1;
    }
    *new_len = p + 1 < cap ? p + 1 : cap;
    *new_seen = p + 1;
    return p < cap ? p : n_sink + (p - n_sink) % (cap - n_sink);
}

// What the append kernels are told about the cache's bookkeeping arrays.
struct SeqState {
    const int64_t *seq_off;
    const int32_t *seq_cap;
    int32_t *seq_lens, *seq_seen, *status;
    int n_sink;
};

// Row that the new token of sequence b goes to, -1 if the append is skipped.  Uniform over the
// workgroup; thread 0 reports errors.
__device__ inline int append_row(const SeqState &st, int b, int *new_len)
{
    int new_seen, err;
    const int row = append_rule(st.seq_lens[b], st.seq_cap[b], st.seq_seen != nullptr,
                                st.seq_seen ? st.seq_seen[b] : 0, st.n_sink, new_len, &new_seen, &err);
    if (err && threadIdx.x == 0) atomicOr(st.status, err);
    return row;
}

// One workgroup per sequence: 2*H rows of d fp16 are copied as raw 128-bit words.  With `bump`
// one thread then stores the new length; without it the lengths are left alone and take effect
// later (the fused append + plan launch: its planner works from the old lengths).
__device__ inline void kv_append_body(uint4 *__restrict__ k_base, uint4 *__restrict__ v_base,
                                      const SeqState &st, const uint4 *__restrict__ k_new,
                                      const uint4 *__restrict__ v_new, int H, int d, int b, bool bump)
{
    const int cap = st.seq_cap[b];
    int new_len = 0;
    const int L = append_row(st, b, &new_len);
    if (L < 0) return;
    const int vpr = d / 8;                               // 16-byte words per row
    const int n = H * vpr;
    const int64_t blk = st.seq_off[b] / 8;               // block offset in 16-byte words
    const int64_t src0 = (int64_t)b * n;
    for (int x = threadIdx.x; x < 2 * n; x += blockDim.x) {
        const int which = x >= n;
        const int y = which ? x - n : x;
        const int h = y / vpr, c = y - h * vpr;
        const int64_t dst = blk + ((int64_t)h * cap + L) * vpr + c;
        // written through, not left dirty in this XCD's L2: the streaming kernel that follows
        // reads the row from another XCD as a rule, and fetching a line out of a remote L2 was
        // measured at about half a microsecond per unit, exposed at the end of the unit
        typedef unsigned int u32x4v __attribute__((ext_vector_type(4)));
        const uint4 val = which ? v_new[src0 + y] : k_new[src0 + y];
        u32x4v *out4 = reinterpret_cast<u32x4v *>((which ? v_base : k_base) + dst);
        __builtin_nontemporal_store(u32x4v{val.x, val.y, val.z, val.w}, out4);
    }
    if (bump) {
        __syncthreads();
        if (threadIdx.x == 0) {
            st.seq_lens[b] = new_len;
            if (st.seq_seen) st.seq_seen[b] += 1;
        }
    }
}

__global__ __launch_bounds__(256) void kv_append_kernel(
    uint4 *__restrict__ k_base, uint4 *__restrict__ v_base, SeqState st,
    const uint4 *__restrict__ k_new, const uint4 *__restrict__ v_new, int H, int d)
{
    kv_append_body(k_base, v_base, st, k_new, v_new, H, d, blockIdx.x, true);
}

// value = 0 starts an empty sequence in the slot, FD_SLOT_FREE marks the slot free
__global__ void kv_reset_kernel(int32_t *__restrict__ seq_lens, int32_t *__restrict__ seq_seen,
                                const int32_t *__restrict__ ids, int n, int B, int value)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= n) return;
    const int b = ids ? ids[j] : j;
    if (b >= 0 && b < B) {
        seq_lens[b] = value;
        if (seq_seen) seq_seen[b] = 0;
    }
}

// Bulk store of n consecutive token rows of one sequence (prompt ingestion): raw 128-bit copies
// of rows given as fp16 [H][n][d] into tokens t0 .. t0+n-1.  One thread per 16-byte word.
__global__ __launch_bounds__(256) void kv_store_rows_kernel(
    uint4 *__restrict__ k_base, uint4 *__restrict__ v_base, const int64_t *__restrict__ seq_off,
    const int32_t *__restrict__ seq_cap, int32_t *__restrict__ seq_lens,
    int32_t *__restrict__ seq_seen, int32_t *__restrict__ status, const uint4 *__restrict__ k_rows,
    const uint4 *__restrict__ v_rows, int H, int d, int b, int t0, int n, int set_len)
{
    const int cap = seq_cap[b];
    if (t0 + n > cap) {                                      // uniform over the grid: nothing is written
        if (blockIdx.x == 0 && threadIdx.x == 0) atomicOr(status, FD_ST_CAPACITY);
        return;
    }
    const int vpr = d / 8;
    const int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;    // word index in [H][n][vpr]
    if (x < (int64_t)H * n * vpr) {
        const int64_t r = x / vpr;
        const int c = (int)(x - r * vpr);
        const int h = (int)(r / n), j = (int)(r - (int64_t)h * n);
        const int64_t dst = seq_off[b] / 8 + ((int64_t)h * cap + t0 + j) * vpr + c;
        if (k_rows) k_base[dst] = k_rows[x];
        if (v_rows) v_base[dst] = v_rows[x];
    }
    if (set_len && blockIdx.x == 0 && threadIdx.x == 0) {
        seq_lens[b] = t0 + n;
        if (seq_seen) seq_seen[b] = t0 + n;
    }
}

// sticky status word: take it (read and clear in one atomic step) or clear the bits just read
__global__ void status_take_kernel(int32_t *__restrict__ status, int32_t *__restrict__ dst)
{
    *dst = atomicExch(status, 0);
}
__global__ void status_clear_bits_kernel(int32_t *__restrict__ status, int32_t bits)
{
    atomicAnd(status, ~bits);
}

// ---------------------------------------------------------------------------
// Planner: one workgroup.  Reads the ragged lengths on the device, picks the
// chunk length, writes the work-item table and a static schedule.
//
// Splitting is kept to what load balance needs: every chunk state that has to
// be written out and merged later costs far more than its bytes (result stores
// interleaved with the read stream lower the achieved HBM bandwidth by several
// per cent), so a sequence is cut only when it is longer than 1/16 of a
// workgroup's share of the step (`split` = 16; 4 for the quantised caches, whose
// units carry a half to a quarter of the bytes per token against the same fixed cost:
// measured there, a quarter against a sixteenth is +12 % on a geometric length mix with 4-bit
// codes, +29 % on one sequence of 131072 tokens, and nowhere slower; for fp16 the two are
// within 1 % of each other with 1/16 ahead on the ragged mixes).  Sequence b with L_b tokens
// is cut into n_b = ceil(L_b / T) chunks of equal length rounded up to the granule.
//
// The schedule is static (a shared ticket counter was measured 4-5 % slower: the
// atomic sits in the in-order return queue in front of the unit's first loads):
// items are ordered longest first by a counting sort on their length, and the
// streaming kernel deals (item, head) units to workgroups in snake order, which
// is the longest-processing-time rule for units that are small against a
// workgroup's share.
//
// The planner can run in the same launch as the step's append (workgroup 0 plans, the others
// append): it then works from the lengths the sequences will have AFTER that append, which it
// derives from the old lengths by the append's own rule, stores them for the streaming kernel
// to put into seq_lens, and no kernel of that launch writes seq_lens, so nothing races.
// ---------------------------------------------------------------------------
constexpr int kShortSeq = 384;      // a sequence under this many tokens is latency-bound ("short")
constexpr int kBuckets = 256;
constexpr int kLenCache = 4;       // lengths a planner thread keeps in registers

struct PlanArgs {
    const int32_t *seq_lens, *seq_cap, *seq_seen;
    int32_t *status;
    int n_sink;
    int after_append;     // plan for the lengths after one append (fused launch); else for seq_lens as it stands
    int B, H, chunk_req, granule, grid_long, grid_short, short_below, hashed, wave_units, split, kind;
    PlanView v;
};

__device__ inline int block_sum(int v, int *sm)
{
    // sum over the workgroup; result returned to all threads
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    int t = 0;
    for (int w = 0; w < kPlanThreads / 64; ++w) t += sm[w];
    return t;
}

// two sums over the workgroup with one pair of barriers; results to all threads
__device__ inline void block_sum2(int &x, int &y, int *sm)
{
    for (int off = 32; off > 0; off >>= 1) {
        x += __shfl_xor(x, off);
        y += __shfl_xor(y, off);
    }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) {
        sm[threadIdx.x >> 6] = x;
        sm[kPlanThreads / 64 + (threadIdx.x >> 6)] = y;
    }
    __syncthreads();
    x = 0;
    y = 0;
    for (int w = 0; w < kPlanThreads / 64; ++w) {
        x += sm[w];
        y += sm[kPlanThreads / 64 + w];
    }
}

// two sums, a minimum and a maximum over the workgroup with one pair of barriers
__device__ inline void block_sum2_minmax(int &x, int &y, int &lo, int &hi, int *sm)
{
    constexpr int NW = kPlanThreads / 64;
    for (int off = 32; off > 0; off >>= 1) {
        x += __shfl_xor(x, off);
        y += __shfl_xor(y, off);
        lo = min(lo, __shfl_xor(lo, off));
        hi = max(hi, __shfl_xor(hi, off));
    }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) {
        const int w = threadIdx.x >> 6;
        sm[w] = x;
        sm[NW + w] = y;
        sm[2 * NW + w] = lo;
        sm[3 * NW + w] = hi;
    }
    __syncthreads();
    x = 0;
    y = 0;
    for (int w = 0; w < NW; ++w) {
        x += sm[w];
        y += sm[NW + w];
        lo = min(lo, sm[2 * NW + w]);
        hi = max(hi, sm[3 * NW + w]);
    }
}

// exclusive prefix sum over the workgroup's threads (two barriers)
__device__ inline int block_exclusive_scan(int v, int *sm)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = v;
    for (int off = 1; off < 64; off <<= 1) {
        const int u = __shfl_up(inc, off);
        if (lane >= off) inc += u;
    }
    __syncthreads();
    if (lane == 63) sm[wave] = inc;
    __syncthreads();
    int base = 0;
    for (int w = 0; w < wave; ++w) base += sm[w];
    return base + inc - v;
}

__device__ inline int clamp_len(int L, int cap, int *bad)
{
    if (L == FD_SLOT_FREE) return 0;                     // a free slot counts as empty
    if (L < 0) { *bad = 1; return 0; }
    if (L > cap) { *bad = 1; return cap > 0 ? cap : 0; }
    return L;
}

// tokens of sequence b that the plan covers
__device__ inline int plan_len(const PlanArgs &a, int b, int *bad)
{
    int L = a.seq_lens[b];
    const int cap = a.seq_cap[b];
    if (a.after_append) {
        int new_seen, err;
        append_rule(L, cap, a.seq_seen != nullptr, a.seq_seen ? a.seq_seen[b] : 0, a.n_sink, &L,
                    &new_seen, &err);
    }
    return clamp_len(L, cap, bad);
}

__device__ inline int length_bucket(int len, int T)
{
    int k = (int)(((long long)(T - len) * kBuckets) / T);   // longest chunks in bucket 0
    return k < 0 ? 0 : (k >= kBuckets ? kBuckets - 1 : k);
}

// chunk k of a sequence of L tokens cut into n chunks: tokens [t0, t1)
__device__ inline void chunk_span(int L, int n, int granule, int k, int *t0, int *t1)
{
    int len = (L + n - 1) / n;
    len = (len + granule - 1) / granule * granule;      // <= the chunk length T, so (n-1)*len < L
    *t0 = k * len;
    *t1 = min(L, *t0 + len);
}

constexpr int kBigChunks = 16;      // a sequence cut into more chunks than this ...
constexpr int kBigMax = 128;        // ... goes on a list of at most this many entries

// the whole workgroup (kPlanThreads threads) must call this
__device__ inline void plan_body(const PlanArgs &a)
{
    __shared__ int sm[kPlanThreads];
    __shared__ int hist[kBuckets];
    __shared__ int4 big[kBigMax];
    __shared__ int nbig, big_nmax;
    const int B = a.B, H = a.H, granule = a.granule, max_items = a.v.max_items;
    int32_t *__restrict__ item0 = a.v.item0;
    int32_t *__restrict__ nchunk = a.v.nchunk;
    int4 *__restrict__ items = a.v.items;
    int32_t *__restrict__ order = a.v.order;
    int32_t *__restrict__ cnt = a.v.cnt;
    const int tid = threadIdx.x;
    const int per = (B + kPlanThreads - 1) / kPlanThreads;   // sequences per thread (contiguous)
    const int b0 = tid * per;
    const int b1 = min(B, b0 + per);

    // Each thread reads its sequences' lengths once and keeps them in registers (up to kLenCache
    // per thread, 4096 sequences in all; beyond that they are read again per pass), and sums that
    // do not depend on each other share a reduction.  (Of the 8.5 us of a fused append + plan
    // launch about 5 are the launch and the append; the passes up to the item counts cost next
    // to nothing, writing the items 1 us, the bucket scan 1 us, the scatter 1.4 us.)
    int bad = 0;
    int Lc[kLenCache];
    const bool cached = per <= kLenCache;
#pragma unroll
    for (int i = 0; i < kLenCache; ++i) Lc[i] = cached && b0 + i < b1 ? plan_len(a, b0 + i, &bad) : 0;
    // f(b, L) for this thread's sequences
    auto each = [&](auto &&f) {
        if (cached) {
#pragma unroll
            for (int i = 0; i < kLenCache; ++i)
                if (b0 + i < b1) f(b0 + i, Lc[i]);
        } else {
            for (int b = b0; b < b1; ++b) f(b, plan_len(a, b, &bad));
        }
    };

    // One workgroup per CU streams long sequences best (a second one costs 1-2 %); a sequence of
    // a few blocks is dominated by its fixed cost, and more workgroups per CU hide that.  Measured
    // on the fp16 kernel, one against two per CU: 256 tokens each +3.5 %, lengths uniform in
    // 1..1024 (the load-stabilising schedule's mix) +2.2 %, 512 each -1.1 %, uniform in 1..2048
    // -0.6 %, exponential with mean 1024 -1.2 %.  What separates them is the share of the
    // cached tokens that sits in sequences shorter than short_below tokens (100 %, 14 %, 0, 3.5 %,
    // 5.5 %): above a tenth the larger grid is used.  The host launches the larger number and
    // workgroups at or beyond `grid` leave at once.
    int total = 0, few = 0, lmin = 0x7FFFFFFF, lmax = 0;
    each([&](int, int L) {
        total += L;
        few += L < a.short_below ? L : 0;
        lmin = min(lmin, L);
        lmax = max(lmax, L);
    });
    block_sum2_minmax(total, few, lmin, lmax, sm);
    if (bad) atomicOr(a.status, FD_ST_BADLEN);
    const bool many_short = (long long)few * 10 > (long long)total;
    const int grid = many_short ? a.grid_short : a.grid_long;
    // wave_units: 0 = the workgroup's waves always share a unit, 1 = each wave takes units of its
    // own when the batch holds many short sequences, 2 = always
    const int wave_now = a.wave_units == 2 || (a.wave_units == 1 && many_short);

    int T;
    if (a.chunk_req > 0) {
        T = a.chunk_req;
    } else {
        // token-heads per worker: a workgroup, or a wave when each wave takes units of its own
        // (a wave's share is a quarter of a workgroup's: it is cut into quarters at most, or half
        // of a batch of a few hundred tokens per sequence would end up split)
        const long long share = (long long)total * H / ((long long)grid * (wave_now ? kWaves : 1));
        long long t = share / (wave_now && a.split > 4 ? 4 : a.split);
        T = (int)(t < 128 ? 128 : (t > (1 << 28) ? (1 << 28) : t));
    }
    T = (T + granule - 1) / granule * granule;

    // The order in which the sequences are visited when the schedule is filled.  With `hashed` it
    // is scrambled (a bijection of [0, B)): equal-length sequences then run side by side in no
    // regular pattern.  A regular one can put the streams that run in lockstep a constant distance
    // apart, and for some distances (2^a + 2^(a+8) bytes was seen) they then fight over the same
    // DRAM banks all the way: -10 % on the int8 kernel.
    int hbits = 1;
    while ((1 << hbits) < B) ++hbits;
    const unsigned hmask = (1u << hbits) - 1u;
    const int hhalf = (hbits + 1) / 2;
    auto visit = [&](int j) {
        if (!a.hashed) return j;
        unsigned x = (unsigned)j;
        do {                                                // cycle-walk back into [0, B)
            x = (x * 0x9E3779B1u) & hmask;
            x ^= x >> hhalf;
            x = (x * 0x85EBCA6Bu) & hmask;
            x ^= x >> hhalf;
        } while (x >= (unsigned)B);
        return (int)x;
    };

    // Equal lengths (a batch decoded in lockstep, a single sequence): every sequence is cut alike,
    // sequence b's items are b n .. b n + n - 1, and chunk-major order (chunk 0 of every sequence,
    // then chunk 1, ...) is already longest first, since only a sequence's last chunk can be
    // shorter than the others.  No counting, no sort, no further barrier: 8.5 -> 5 us for the
    // fused append + plan launch (about the time of the append alone), a fifth of a batch-1 step.
    int count = 0;
    bool uniform = lmin == lmax && lmin > 0;
    if (uniform) {
        int n = (lmin + T - 1) / T;
        while ((long long)B * n > max_items && T < (1 << 30)) {
            T *= 2;
            n = (lmin + T - 1) / T;
        }
        uniform = n <= kBigChunks && (long long)B * n <= max_items;
        if (uniform) {
            count = B * n;
            each([&](int b, int L) {
                const int pos = b * n;
                item0[b] = pos;
                nchunk[b] = n;
                if (a.after_append) {
                    int new_len, new_seen, err;
                    append_rule(a.seq_lens[b], a.seq_cap[b], a.seq_seen != nullptr,
                                a.seq_seen ? a.seq_seen[b] : 0, a.n_sink, &new_len, &new_seen, &err);
                    a.v.newlen[b] = new_len;
                    a.v.newseen[b] = new_seen;
                }
                for (int k = 0; k < n; ++k) {
                    int t0, t1;
                    chunk_span(L, n, granule, k, &t0, &t1);
                    items[pos + k] = make_int4(b, t0, t1, n);
                }
                if (n > 1)
                    for (int h = 0; h < H; ++h) cnt[(int64_t)pos * H + h] = 0;
            });
            for (int j = b0; j < b1; ++j) {
                const int b = visit(j);
                for (int k = 0; k < n; ++k) order[(int64_t)k * B + j] = b * n + k;
            }
        }
    }
    if (!uniform) {
        // items in all (the chunk length is doubled until they fit the workspace) and sequences cut
        // into many chunks; c = this thread's items
        int c, n_big;
        for (;;) {
            c = 0;
            n_big = 0;
            each([&](int, int L) {
                const int n = (L + T - 1) / T;
                c += n;
                n_big += n > kBigChunks;
            });
            count = c;
            block_sum2(count, n_big, sm);
            if (count <= max_items || T >= (1 << 30)) break;   // T >= longest sequence gives count <= B
            T *= 2;
        }
        // A sequence cut into many chunks (one that has the device almost to itself) is written out
        // by the whole workgroup, a chunk per thread, instead of by the one thread that owns it:
        // 128 chunks walked by one thread took 46 us.  The list is used only when it holds them all.
        const bool use_list = n_big <= kBigMax;
        if (tid < kBuckets) hist[tid] = 0;
        if (tid == 0) { nbig = 0; big_nmax = 0; }
        const int first = block_exclusive_scan(c, sm);      // its barriers also publish hist = 0
        int pos = first;
        each([&](int b, int L) {
            const int n = (L + T - 1) / T;
            item0[b] = pos;
            nchunk[b] = n;
            if (a.after_append) {
                // what the append of this launch makes of the sequence's bookkeeping; the streaming
                // kernel stores it into seq_lens / seq_seen
                int new_len, new_seen, err;
                append_rule(a.seq_lens[b], a.seq_cap[b], a.seq_seen != nullptr,
                            a.seq_seen ? a.seq_seen[b] : 0, a.n_sink, &new_len, &new_seen, &err);
                a.v.newlen[b] = new_len;
                a.v.newseen[b] = new_seen;
            }
            if (use_list && n > kBigChunks) {
                big[atomicAdd(&nbig, 1)] = make_int4(b, L, n, pos);
                atomicMax(&big_nmax, n);
            } else {
                for (int k = 0; k < n; ++k) {
                    int t0, t1;
                    chunk_span(L, n, granule, k, &t0, &t1);
                    if (pos + k < max_items) {
                        items[pos + k] = make_int4(b, t0, t1, n);
                        atomicAdd(&hist[length_bucket(t1 - t0, T)], 1);
                    }
                }
                // a split sequence's heads count their finished chunks here (see finish_split)
                if (n > 1 && pos < max_items)
                    for (int h = 0; h < H; ++h) cnt[(int64_t)pos * H + h] = 0;
            }
            pos += n;
        });
        __syncthreads();
        const int n_listed = nbig;
        for (int s = 0; s < n_listed; ++s) {
            const int4 e = big[s];                          // (b, L, n, first item)
            for (int k = tid; k < e.z; k += kPlanThreads) {
                int t0, t1;
                chunk_span(e.y, e.z, granule, k, &t0, &t1);
                if (e.w + k < max_items) {
                    items[e.w + k] = make_int4(e.x, t0, t1, e.z);
                    atomicAdd(&hist[length_bucket(t1 - t0, T)], 1);
                }
            }
            if (e.w < max_items)
                for (int h = tid; h < H; h += kPlanThreads) cnt[(int64_t)e.w * H + h] = 0;
        }
        __syncthreads();
        // bucket starts = exclusive scan of the 256 counters, then scatter
        {
            const int n = tid < kBuckets ? hist[tid] : 0;
            const int start = block_exclusive_scan(n, sm);
            if (tid < kBuckets) hist[tid] = start;
        }
        __syncthreads();
        // Scatter.  Inside a bucket the order is the arrival order of the atomics, the sequences
        // being visited in the order of `visit`.
        for (int j = b0; j < b1; ++j) {
            const int b = visit(j);
            const int n = nchunk[b];
            const int base = item0[b];
            if (n > 0 && !(use_list && n > kBigChunks)) {
                const int L = plan_len(a, b, &bad);
                for (int k = 0; k < n; ++k) {
                    int t0, t1;
                    chunk_span(L, n, granule, k, &t0, &t1);
                    if (base + k < max_items)
                        order[atomicAdd(&hist[length_bucket(t1 - t0, T)], 1)] = base + k;
                }
            }
        }
        // listed sequences chunk-major (chunk 0 of each, chunk 1 of each, ...), the order in which
        // their owner threads, side by side in one wave, would have issued the atomics: units that
        // run at the same time then belong to different sequences where there are several
        if (n_listed > 0) {
            const long long k_end = (long long)big_nmax * n_listed;
            for (long long i = tid; i < k_end; i += kPlanThreads) {
                const int k = (int)(i / n_listed);
                const int4 e = big[(int)(i - (long long)k * n_listed)];
                if (k < e.z) {
                    int t0, t1;
                    chunk_span(e.y, e.z, granule, k, &t0, &t1);
                    if (e.w + k < max_items)
                        order[atomicAdd(&hist[length_bucket(t1 - t0, T)], 1)] = e.w + k;
                }
            }
        }
    }
    if (tid == 0) {
        int32_t *hdr = a.v.hdr;
        hdr[HDR_NITEMS] = count <= max_items ? count : 0;
        hdr[HDR_CHUNK] = T;
        hdr[HDR_TOKENS] = total;
        hdr[HDR_GRID] = grid;
        hdr[HDR_MAGIC] = kPlanMagic;
        hdr[HDR_B] = B;
        hdr[HDR_H] = H;
        hdr[HDR_MAXITEMS] = max_items;
        hdr[HDR_WAVE_UNITS] = wave_now;
        hdr[HDR_KIND] = a.kind;
        hdr[HDR_BUMP] = a.after_append;
    }
}

__global__ __launch_bounds__(kPlanThreads) void plan_kernel(PlanArgs a) { plan_body(a); }

// One launch for the front of a step: workgroup 0 plans the decode for the lengths after the
// append, workgroups 1 .. B append (sequence blockIdx.x - 1) without touching seq_lens.
__global__ __launch_bounds__(kPlanThreads) void kv_append_plan_kernel(
    uint4 *__restrict__ k_base, uint4 *__restrict__ v_base, SeqState st,
    const uint4 *__restrict__ k_new, const uint4 *__restrict__ v_new, int d, PlanArgs a)
{
    if (blockIdx.x == 0) plan_body(a);
    else kv_append_body(k_base, v_base, st, k_new, v_new, a.H, d, (int)blockIdx.x - 1, false);
}

// The streaming and the merge kernels index the caller's slabs with what the plan tables say:
// they refuse a workspace that does not hold a plan made for this batch shape, cache format and
// workspace size (never planned, or planned for another kind of descriptor), report it and write
// nothing.  `launched` is the number of workgroups this launch has, 0 where that does not
// matter: a plan that deals units to more workgroups than exist would leave outputs unwritten.
// Token ranges are clamped to the current descriptor's capacities when a unit is fetched, so a
// plan made for other lengths gives wrong results but never an access outside a block.
__device__ inline bool plan_matches(const int32_t *hdr, int B, int H, int kind, int max_items,
                                    int launched, int32_t *status)
{
    const bool ok = hdr[HDR_MAGIC] == kPlanMagic && hdr[HDR_B] == B && hdr[HDR_H] == H &&
                    hdr[HDR_KIND] == kind && hdr[HDR_MAXITEMS] == max_items &&
                    hdr[HDR_NITEMS] >= 0 && hdr[HDR_NITEMS] <= max_items &&
                    (launched == 0 || (hdr[HDR_GRID] > 0 && hdr[HDR_GRID] <= launched));
    if (!ok && blockIdx.x == 0 && threadIdx.x == 0) atomicOr(status, FD_ST_PLAN);
    return ok;
}

// ---------------------------------------------------------------------------
// Split-K streaming attention (Eq. 2 + Eq. 3 over one chunk of one (b,h)).
// ---------------------------------------------------------------------------
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float fvec4 __attribute__((ext_vector_type(4)));
typedef _Float16 hvec4 __attribute__((ext_vector_type(4)));

template <int CTRL>
__device__ inline float dpp_xadd(float x)
{
    const int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true);
    return x + __int_as_float(y);
}

// sum over the LPR consecutive lanes that hold one row; every lane gets the sum
template <int LPR>
__device__ inline float row_sum(float x)
{
    x = dpp_xadd<0xB1>(x);                  // quad_perm [1,0,3,2]
    x = dpp_xadd<0x4E>(x);                  // quad_perm [2,3,0,1]
    if (LPR >= 8) x = dpp_xadd<0x141>(x);   // row_half_mirror: other quad of the 8
    if (LPR == 16) x = dpp_xadd<0x140>(x);  // row_mirror: other half of the 16
    return x;
}

// keeps the instruction scheduler from sinking a tile's prefetch loads down to their uses
__device__ inline void sched_fence() { __builtin_amdgcn_sched_barrier(0); }

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ inline half8 ld_stream(const char *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const half8 *>(p));
}

// Where a unit of work (one chunk of one head's stream) lives; uniform over the wave.
struct Unit {
    int64_t row0;            // element offset (fp16) or row index (codes) of the chunk's first row
    int ntok;                // tokens in the chunk; 0 = no unit
    int b, h, item, nch;     // sequence, head, item index, chunks of the sequence
};

// What a streaming kernel does before its first unit, by workgroup (blockIdx.x < active
// workgroups, sequences dealt round-robin): a sequence without tokens gets a zero output, and
// after a fused append + plan launch the new lengths are put into seq_lens (absolute values:
// doing it twice changes nothing).
template <int D>
__device__ inline void unit_prologue(const int32_t *__restrict__ hdr, const int32_t *__restrict__ nchunk,
                                     const int32_t *__restrict__ newlen, const int32_t *__restrict__ newseen,
                                     int32_t *__restrict__ seq_lens, int32_t *__restrict__ seq_seen,
                                     _Float16 *__restrict__ out, int B, int H)
{
    const int Wg = hdr[HDR_GRID];
    const int bump = hdr[HDR_BUMP];
    for (int b = blockIdx.x; b < B; b += Wg) {
        if (bump && threadIdx.x == 0) {
            seq_lens[b] = newlen[b];
            if (seq_seen) seq_seen[b] = newseen[b];
        }
        if (nchunk[b] == 0) {
            uint4 *o = reinterpret_cast<uint4 *>(out + (int64_t)b * H * D);
            for (int x = threadIdx.x; x < H * (D / 8); x += blockDim.x) o[x] = make_uint4(0, 0, 0, 0);
        }
    }
}

// ---------------------------------------------------------------------------
// Chunk states of split sequences travel between workgroups that may sit on different XCDs,
// whose L2 caches are not coherent with each other.  A device-scope fence would write back and
// invalidate a whole L2 (measured: one pair of fences per split unit cost a geometric length mix
// 15 % and a batch of half-split sequences a factor of three).  Instead every access to a chunk
// state or to a chunk counter is itself a device-scope access (relaxed atomics of agent scope:
// stores go through to memory, loads come from there), and order is kept by waiting for the
// wave's stores to complete before its counter increments are issued.
// ---------------------------------------------------------------------------
__device__ inline void st_agent(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline float ld_agent(const float *p)
{
    return __hip_atomic_load(const_cast<float *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
typedef float fvec2 __attribute__((ext_vector_type(2)));
// 128 bits of a chunk state as two 64-bit device-scope loads
__device__ inline fvec4 ld_agent4(const fvec4 *p)
{
    union { unsigned long long u; fvec2 f; } lo, hi;
    unsigned long long *q = reinterpret_cast<unsigned long long *>(const_cast<fvec4 *>(p));
    lo.u = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    hi.u = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return fvec4{lo.f[0], lo.f[1], hi.f[0], hi.f[1]};
}

// ---------------------------------------------------------------------------
// Log-sum-exp merge of the chunk states of one (sequence, head) by one wave.
// States are in the base-2 exponent domain used by the streaming kernels.
//
// A sequence that has the device to itself is cut into over a hundred chunks per head, so the
// wave works on many chunk states at once: maxima and sums of exponentials one chunk per lane,
// the weighted value sums four records per load (16 lanes x 128-bit per record) with sixteen
// records in flight, and a cross-lane sum over the four groups at the end.  The order of the
// arithmetic is fixed, so the result does not depend on which wave runs it or when.
// rec0 = first record (chunk 0) of this (b,h); chunk c is record rec0 + c*H.  o = out + bh*D.
// ---------------------------------------------------------------------------
template <int D>
__device__ inline void merge_states(int lane, int n, int64_t rec0, int H, const float *part_acc,
                                    const float *part_ml, _Float16 *o)
{
    constexpr int NV = D / 64;                        // 128-bit pieces of a record per lane
    const int t = lane & 15, g = lane >> 4;           // piece within the record, record within the load
    float M = kNegBig;
    for (int c0 = 0; c0 < n; c0 += 64) {
        const int c = c0 + lane;
        if (c < n) M = fmaxf(M, ld_agent(&part_ml[(rec0 + (int64_t)c * H) * 2]));
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
    float L = 0.f;
    fvec4 acc[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) acc[v] = fvec4{0.f, 0.f, 0.f, 0.f};
    const int64_t step = (int64_t)H * (D / 4);         // record stride of one chunk, in 128-bit pieces
    for (int c0 = 0; c0 < n; c0 += 64) {
        const int c = c0 + lane;
        float w = 0.f;
        if (c < n) {
            const int64_t rec = rec0 + (int64_t)c * H;
            w = fast_exp2(ld_agent(&part_ml[rec * 2]) - M);
            L += w * ld_agent(&part_ml[rec * 2 + 1]);
        }
        const int nb = min(64, n - c0);
        const fvec4 *pa = (const fvec4 *)(part_acc + (rec0 + (int64_t)c0 * H) * D) + t;
        for (int j0 = 0; j0 < nb; j0 += 16) {
            fvec4 x[4][NV];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int j = min(j0 + u * 4 + g, nb - 1);   // past the end: a valid record, weight 0
#pragma unroll
                for (int v = 0; v < NV; ++v) x[u][v] = ld_agent4(pa + j * step + v * 16);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int j = j0 + u * 4 + g;
                float wj = __shfl(w, j & 63);
                wj = j < nb ? wj : 0.f;
#pragma unroll
                for (int v = 0; v < NV; ++v) acc[v] += wj * x[u][v];
            }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) L += __shfl_xor(L, off);
#pragma unroll
    for (int v = 0; v < NV; ++v)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float a = acc[v][i];
            a += __shfl_xor(a, 16);
            a += __shfl_xor(a, 32);
            acc[v][i] = a;
        }
    if (g == 0) {                                     // lanes of group 0 write elements v*64 + t*4 ..
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            hvec4 r;
#pragma unroll
            for (int i = 0; i < 4; ++i) r[i] = (_Float16)(acc[v][i] / L);
            *(hvec4 *)(o + t * 4 + v * 64) = r;
        }
    }
}

// A sequence cut into few chunks (the usual case: a ragged batch splits only its longest
// sequences, in two to four) leaves the wave-wide merge above almost idle and bound by the
// latency of its dependent loads.  This form merges up to four (sequence, head) pairs at once,
// one per 16-lane group, chunk after chunk in chunk order, with all loads of a pair issued
// together.  Which form merges a pair depends only on its number of chunks (kSmallMerge), so
// the result still does not depend on who merges it.  `active`, n, rec0, o: per 16-lane group.
constexpr int kSmallMerge = 4;

template <int D>
__device__ inline void merge_states_small(int lane, bool active, int n, int64_t rec0, int H,
                                          const float *part_acc, const float *part_ml, _Float16 *o)
{
    constexpr int NV = D / 64;
    const int t = lane & 15;
    float mc[kSmallMerge], lc[kSmallMerge];
    fvec4 x[kSmallMerge][NV];
    const int64_t step = (int64_t)H * (D / 4);
    const fvec4 *pa = (const fvec4 *)(part_acc + rec0 * D) + t;
#pragma unroll
    for (int c = 0; c < kSmallMerge; ++c) {
        const bool on = active && c < n;
        mc[c] = on ? ld_agent(&part_ml[(rec0 + (int64_t)c * H) * 2]) : kNegBig;
        lc[c] = on ? ld_agent(&part_ml[(rec0 + (int64_t)c * H) * 2 + 1]) : 0.f;
#pragma unroll
        for (int v = 0; v < NV; ++v)
            x[c][v] = on ? ld_agent4(pa + c * step + v * 16) : fvec4{0.f, 0.f, 0.f, 0.f};
    }
    float M = kNegBig;
#pragma unroll
    for (int c = 0; c < kSmallMerge; ++c) M = fmaxf(M, mc[c]);
    float L = 0.f;
    fvec4 acc[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) acc[v] = fvec4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < kSmallMerge; ++c) {
        const float w = (active && c < n) ? fast_exp2(mc[c] - M) : 0.f;
        L += w * lc[c];
#pragma unroll
        for (int v = 0; v < NV; ++v) acc[v] += w * x[c][v];
    }
    if (active) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            hvec4 r;
#pragma unroll
            for (int i = 0; i < 4; ++i) r[i] = (_Float16)(acc[v][i] / L);
            *(hvec4 *)(o + t * 4 + v * 64) = r;
        }
    }
}

// ---------------------------------------------------------------------------
// The merge is folded into the streaming kernel, so a step needs no merge launch.  A wave that
// writes chunk states of split sequences notes them on a short list in LDS ({b, h, chunks, first
// item}).  When it has no more units (or the list is full) it publishes them in one go: it waits
// for its state stores to complete, then adds one to the counter of every listed (sequence,
// head), all with a single batched atomic, so the round trip is paid once per wave and not once
// per unit.  Whoever brings a counter to the sequence's chunk count has published, or seen
// published, every chunk of that head: that wave merges them in chunk order and puts the counter
// back to zero for the next launch on this plan.  Integer atomics only; the result does not
// depend on who merges.
// ---------------------------------------------------------------------------
constexpr int kSplitList = 64;      // entries per publishing wave

template <int D>
__device__ __attribute__((noinline)) void publish_split(int lane, const int4 *list, int n, int H, int32_t *cnt,
                                     const float *part_acc, const float *part_ml,
                                     _Float16 *__restrict__ out)
{
    if (n == 0) return;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_s_waitcnt(0);                    // every chunk state store of this wave has completed
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    int4 e = make_int4(0, 0, 0, 0);
    int last = 0;
    if (lane < n) {
        e = list[lane];
        const int ticket = __hip_atomic_fetch_add(&cnt[(int64_t)e.w * H + e.y], 1, __ATOMIC_RELAXED,
                                                  __HIP_MEMORY_SCOPE_AGENT);
        last = ticket == e.z - 1;
    }
    // pairs cut into few chunks: four at a time, one per 16-lane group
    unsigned long long small = __ballot(last && e.z <= kSmallMerge);
    unsigned long long large = __ballot(last && e.z > kSmallMerge);
    const int grp = lane >> 4;
    while (small) {
        int src = -1;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (small) {
                const int bit = __ffsll((long long)small) - 1;
                small &= small - 1;
                if (grp == k) src = bit;
            }
        }
        const int from = src < 0 ? 0 : src;
        const int b = __shfl(e.x, from), h = __shfl(e.y, from), nch = __shfl(e.z, from);
        const int64_t rec0 = (int64_t)__shfl(e.w, from) * H + h;
        merge_states_small<D>(lane, src >= 0, nch, rec0, H, part_acc, part_ml, out + ((int64_t)b * H + h) * D);
        if (src >= 0 && (lane & 15) == 0)
            __hip_atomic_store(&cnt[rec0], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    while (large) {
        const int src = __ffsll((long long)large) - 1;
        large &= large - 1;
        const int b = __shfl(e.x, src), h = __shfl(e.y, src), nch = __shfl(e.z, src);
        const int64_t rec0 = (int64_t)__shfl(e.w, src) * H + h;
        merge_states<D>(lane, nch, rec0, H, part_acc, part_ml, out + ((int64_t)b * H + h) * D);
        if (lane == 0) __hip_atomic_store(&cnt[rec0], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// One tile = this wave's share of a block of a unit.  WPU = waves that stream a unit together:
// kWaves (a block is kWaves * NL consecutive wave loads, 1 KB each, of the K stream and of the
// V stream; wave w takes loads w, w + kWaves, ...: the workgroup reads the block as one
// contiguous run with its waves interleaved at 1 KB, and every wave gets the same number of
// loads whatever the chunk length) or 1 (the wave streams a unit of its own: NL consecutive
// wave loads per block).
template <int D, int NL, int WPU>
struct Tile {
    static constexpr int LPR = D / 8;                    // lanes per row
    static constexpr int RPW = 64 / LPR;                 // rows (tokens) per wave load
    static constexpr int STRIDE = WPU * 1024;            // bytes between a wave's consecutive loads
    static constexpr int TSTEP = WPU * RPW;              // tokens between a wave's consecutive loads
    static constexpr int BLK_TOK = NL * TSTEP;           // tokens per block
    static constexpr int BLK_BYTES = NL * STRIDE;        // bytes of K (or V) per block
    half8 k[NL], v[NL];

    __device__ inline void load(const char *kp, const char *vp)
    {
#pragma unroll
        for (int j = 0; j < NL; ++j) k[j] = ld_stream(kp + j * STRIDE);
#pragma unroll
        for (int j = 0; j < NL; ++j) v[j] = ld_stream(vp + j * STRIDE);
    }

    // Ragged last block of `rem` tokens.  Only the wave's first nj loads hold a valid row (nj is
    // the same for every lane of the wave): the others are neither issued nor computed, so a
    // rest of a few tokens costs a few tokens' work.  Within a load, a lane whose token
    // (tok0 + j*TSTEP) is at or beyond `rem` re-reads token rem-1 (in bounds) and is masked.
    __device__ static inline int tail_loads(int wave_tok0, int rem)
    {
        const int n = (rem - wave_tok0 + TSTEP - 1) / TSTEP;
        return n < 0 ? 0 : (n > NL ? NL : n);
    }
    __device__ inline void load_tail(const char *kp, const char *vp, int tok0, int rem, int nj)
    {
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            if (j < nj) {
                const int t = j * TSTEP + tok0;
                const int back = t < rem ? 0 : (t - (rem - 1)) * (D * 2);
                k[j] = ld_stream(kp + j * STRIDE - back);
                v[j] = ld_stream(vp + j * STRIDE - back);
            }
        }
    }

    // MASKED: the ragged last block (tok0, rem, nj as for load_tail); otherwise all NL loads count
    template <bool MASKED>
    __device__ inline void update(const float (&q)[8], float &m, float &l, float (&acc)[8],
                                  int tok0, int rem, int nj) const
    {
        float s[NL];
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            float a = kNegBig;
            if (!MASKED || j < nj) {
                a = 0.f;
#pragma unroll
                for (int i = 0; i < 8; ++i) a = __builtin_fmaf((float)k[j][i], q[i], a);
                a = row_sum<LPR>(a);
                if (MASKED && j * TSTEP + tok0 >= rem) a = kNegBig;
            }
            s[j] = a;
        }
        float tm = s[0];
#pragma unroll
        for (int j = 1; j < NL; ++j) tm = fmaxf(tm, s[j]);
        const float mn = fmaxf(m, tm);
        const float corr = fast_exp2(m - mn);
        l *= corr;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] *= corr;
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            if (!MASKED || j < nj) {
                float p = fast_exp2(s[j] - mn);
                if (MASKED && j * TSTEP + tok0 >= rem) p = 0.f;
                l += p;
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[i] = __builtin_fmaf(p, (float)v[j][i], acc[i]);
            }
        }
        m = mn;
    }
};

// Everything the fp16 streaming kernel is given.
struct PartialArgs {
    const char *k_base, *v_base;
    const int64_t *seq_off;
    const int32_t *seq_cap;
    int32_t *seq_lens, *seq_seen, *status;
    const _Float16 *q;
    _Float16 *out;
    int B, H;
    float qscale;
    PlanView v;
};

template <int D, int NL, int WPU>
__device__ __forceinline__ void rpart_body(const PartialArgs &a)
{
    using T = Tile<D, NL, WPU>;
    constexpr int LPR = T::LPR;
    // two sets, used by alternate units: one barrier per unit is then enough (a wave cannot
    // overwrite a set before every wave has passed the barrier of the unit in between)
    __shared__ float sm_acc2[2][kWaves][D];
    __shared__ float sm_m2[2][kWaves], sm_l2[2][kWaves];
    __shared__ int4 sm_split[kWaves][kSplitList];        // chunk states written but not yet published
    int set = 0;

    const char *__restrict__ k_base = a.k_base;
    const char *__restrict__ v_base = a.v_base;
    const int64_t *__restrict__ seq_off = a.seq_off;
    const int32_t *__restrict__ seq_cap = a.seq_cap;
    const _Float16 *__restrict__ q = a.q;
    _Float16 *__restrict__ out = a.out;
    const int32_t *__restrict__ hdr = a.v.hdr;
    const int4 *__restrict__ items = a.v.items;
    const int32_t *__restrict__ order = a.v.order;
    float *part_acc = a.v.acc;
    float *part_ml = a.v.ml;
    const int H = a.H;

    const int lane = threadIdx.x & 63;
    // the wave's number is the same in all its lanes: kept in a scalar register, so that everything
    // derived from it (the unit, its addresses, the loop counts) is scalar as well
    const int wave_id = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int wave = WPU == 1 ? 0 : wave_id;                     // position among the unit's waves
    const int tid = wave * 64 + lane;                            // thread index among them
    const int row = lane / LPR;
    const int col = lane % LPR;
    const int n_units = hdr[HDR_NITEMS] * H;
    // workers (workgroups, or single waves) that the planner's grid amounts to, and this one
    const int W = hdr[HDR_GRID] * (kWaves / WPU);
    const int g = WPU == 1 ? (int)(blockIdx.x * kWaves) + wave_id : (int)blockIdx.x;
    if (g >= W) return;
    int4 *split_list = sm_split[wave_id];
    int n_split = 0;

    // Static snake schedule over units in longest-first order: in round k this worker
    // owns unit k*W + g (even k) or k*W + W-1-g (odd k), which balances the token totals.
    // The workers walk their rounds from kPhases different starting points, so that at
    // any moment long and short units are in flight together: short units are dominated by
    // latency, and letting every worker reach them at once would leave HBM idle (+3 % on
    // exponentially distributed lengths).  More phases spread the reads over more of the
    // cache at once, which costs about 1 % on uniform lengths; four keeps both.
    const int n_rounds = (int)(((long long)n_units + W - 1) / W);
    const int k_start = (int)((long long)(g % kPhases) * n_rounds / kPhases);
    auto fetch = [&](int j) {
        Unit u;
        u.ntok = 0;
        if (j < n_rounds) {
            int k = k_start + j;
            if (k >= n_rounds) k -= n_rounds;
            const long long p = (long long)k * W + ((k & 1) ? W - 1 - g : g);
            if (p < n_units) {
                const int sidx = (int)(p / H);
                const int item = order[sidx];
                const int4 it = items[item];
                const int cap = seq_cap[it.x];
                // inside this cache's block, and not empty, whatever lengths the plan was made from
                const int t1 = min(it.z, cap), t0 = min(it.y, max(t1 - 1, 0));
                u.h = (int)(p - (long long)sidx * H);
                u.b = it.x;
                u.item = item;
                u.nch = it.w;
                u.ntok = t1 - t0;
                u.row0 = seq_off[it.x] + ((int64_t)u.h * cap + t0) * D;
            }
        }
        return u;
    };

    // only the last round can be incomplete, so at most one fetched unit is empty
    int j = 0;
    Unit cur = fetch(0);
    if (cur.ntok == 0 && n_rounds > 1) cur = fetch(++j);
    // The units are walked in stretches: a stretch ends when the wave has no more units or its list
    // of unpublished chunk states is full; the states are then published (the call sits outside
    // the unit loop, so that it does not constrain the registers of the streaming code).
    for (;;) {
    while (cur.ntok > 0 && n_split < kSplitList) {
        // the next unit's descriptor (three dependent scalar loads) is fetched while this
        // unit streams
        Unit nxt = fetch(++j);
        if (nxt.ntok == 0 && j < n_rounds) nxt = fetch(++j);

        const int b = cur.b, h = cur.h;
        const char *kp = k_base + cur.row0 * 2 + tid * 16;     // wave w starts at its 1 KB slot
        const char *vp = v_base + cur.row0 * 2 + tid * 16;

        float qf[8];
        {
            const half8 qh = *reinterpret_cast<const half8 *>(q + ((int64_t)b * H + h) * D + col * 8);
#pragma unroll
            for (int i = 0; i < 8; ++i) qf[i] = (float)qh[i] * a.qscale;
        }

        float m = kNegBig, l = 0.f, acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = 0.f;

        const int ntok = cur.ntok;
        const int n_blk = ntok / T::BLK_TOK;              // full blocks
        const int rem = ntok - n_blk * T::BLK_TOK;        // tokens of the ragged last block

        // ping-pong register buffers: the next block's loads are in flight while the current
        // one is consumed.  The loop body is branch-free so that the wait counters leave
        // the prefetch outstanding.
        const char *kt = kp;
        const char *vt = vp;
        T A, Bf;
        if (n_blk > 0) {
            A.load(kt, vt);
            int i = 0;
            while (i + 2 < n_blk) {
                Bf.load(kt + T::BLK_BYTES, vt + T::BLK_BYTES);
                sched_fence();
                A.template update<false>(qf, m, l, acc, 0, 0, 0);
                sched_fence();
                A.load(kt + 2 * T::BLK_BYTES, vt + 2 * T::BLK_BYTES);
                sched_fence();
                Bf.template update<false>(qf, m, l, acc, 0, 0, 0);
                sched_fence();
                kt += 2 * T::BLK_BYTES;
                vt += 2 * T::BLK_BYTES;
                i += 2;
            }
            if (i + 1 < n_blk) {
                Bf.load(kt + T::BLK_BYTES, vt + T::BLK_BYTES);
                sched_fence();
                A.template update<false>(qf, m, l, acc, 0, 0, 0);
                sched_fence();
                Bf.template update<false>(qf, m, l, acc, 0, 0, 0);
            } else {
                A.template update<false>(qf, m, l, acc, 0, 0, 0);
            }
        }
        if (rem > 0) {
            const int nj = T::tail_loads(wave * T::RPW, rem);
            if (nj > 0) {                                 // this wave has at least one valid row
                const int tok0 = wave * T::RPW + row;
                const int64_t o = (int64_t)n_blk * T::BLK_BYTES;
                A.load_tail(kp + o, vp + o, tok0, rem, nj);
                A.template update<true>(qf, m, l, acc, tok0, rem, nj);
            }
        }

        // combine the rows of this wave (each 16- or 8-lane row saw different tokens)
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1) {
            const float mo = __shfl_xor(m, off);
            const float lo = __shfl_xor(l, off);
            const float M = fmaxf(m, mo);
            const float wa = fast_exp2(m - M), wc = fast_exp2(mo - M);
            l = l * wa + lo * wc;
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = acc[i] * wa + __shfl_xor(acc[i], off) * wc;
            m = M;
        }
        // Stores are non-temporal: they are never re-read by this unit, and plain stores were
        // measured to cost the read stream about three times as much bandwidth.
        if constexpr (WPU == 1) {
            // the wave owns the unit: every lane holds the state of all rows for its 8 columns;
            // the lanes of row 0 write them
            if (cur.nch == 1) {
                if (lane < LPR) {
                    half8 o8;
#pragma unroll
                    for (int i = 0; i < 8; ++i) o8[i] = (_Float16)(acc[i] / l);
                    __builtin_nontemporal_store(o8, reinterpret_cast<half8 *>(out + ((int64_t)b * H + h) * D + lane * 8));
                }
            } else {
                const int64_t rec = (int64_t)cur.item * H + h;
                if (lane < LPR) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) st_agent(&part_acc[rec * D + lane * 8 + i], acc[i]);
                    if (lane == 0) {
                        st_agent(&part_ml[rec * 2], m);
                        st_agent(&part_ml[rec * 2 + 1], l);
                    }
                }
                if (lane == 0) split_list[n_split] = make_int4(b, h, cur.nch, a.v.item0[b]);
                ++n_split;
            }
        } else {
            float (&sm_acc)[kWaves][D] = sm_acc2[set];
            float (&sm_m)[kWaves] = sm_m2[set];
            float (&sm_l)[kWaves] = sm_l2[set];
            set ^= 1;
            if (lane < LPR) {
#pragma unroll
                for (int i = 0; i < 8; ++i) sm_acc[wave][lane * 8 + i] = acc[i];
            }
            if (lane == 0) { sm_m[wave] = m; sm_l[wave] = l; }
            __syncthreads();

            // combine the waves; write the final output, or this chunk's state
            if (cur.nch == 1) {
                if (tid < D) {
                    float M = sm_m[0];
#pragma unroll
                    for (int w = 1; w < kWaves; ++w) M = fmaxf(M, sm_m[w]);
                    float L = 0.f, o = 0.f;
#pragma unroll
                    for (int w = 0; w < kWaves; ++w) {
                        const float wa = fast_exp2(sm_m[w] - M);
                        L += wa * sm_l[w];
                        o += wa * sm_acc[w][tid];
                    }
                    __builtin_nontemporal_store((_Float16)(o / L), &out[((int64_t)b * H + h) * D + tid]);
                }
            } else if (wave == 0) {
                // one wave writes the whole state (element lane, and lane + 64) and will publish it
                float M = sm_m[0];
#pragma unroll
                for (int w = 1; w < kWaves; ++w) M = fmaxf(M, sm_m[w]);
                float L = 0.f, wgt[kWaves];
#pragma unroll
                for (int w = 0; w < kWaves; ++w) {
                    wgt[w] = fast_exp2(sm_m[w] - M);
                    L += wgt[w] * sm_l[w];
                }
                const int64_t rec = (int64_t)cur.item * H + h;
#pragma unroll
                for (int e = lane; e < D; e += 64) {
                    float o = 0.f;
#pragma unroll
                    for (int w = 0; w < kWaves; ++w) o += wgt[w] * sm_acc[w][e];
                    st_agent(&part_acc[rec * D + e], o);
                }
                if (lane == 0) {
                    st_agent(&part_ml[rec * 2], M);
                    st_agent(&part_ml[rec * 2 + 1], L);
                }
                if (lane == 0) split_list[n_split] = make_int4(b, h, cur.nch, a.v.item0[b]);
            }
            // counted by every wave of the workgroup (they all leave the stretch together)
            if (cur.nch != 1) ++n_split;
        }
        cur = nxt;                     // no second barrier: the next unit uses the other LDS set
    }
    // the chunk states written in this stretch are published, and merged where this wave is the
    // last to publish a chunk of a (sequence, head)
    if (WPU == 1 || wave == 0)
        publish_split<D>(lane, split_list, n_split, H, a.v.cnt, part_acc, part_ml, out);
    n_split = 0;
    if (cur.ntok == 0) break;
    }
}

// Whether each wave of the fp16 streaming kernel takes units of its own when the batch holds
// many short sequences (the planner's wave_units argument).  Measured against workgroup units
// with two workgroups per CU: 256 tokens per sequence -1.1 %, lengths uniform in 1..1024 -1.0 %
// (streaming kernel time), so it stays off: the fp16 unit streams four times the bytes of a 4-bit
// one against the same fixed cost, and two resident workgroups already hide that cost.
constexpr int kWaveUnitsFp16 = 0;

// One kernel, two bodies: the planner decides per launch whether a workgroup's four waves share
// a unit or take one each (short sequences: a unit's fixed cost, the epilogue with its barrier
// and cross-wave combine, is then spread over four times as many blocks per wave).
template <int D, int NL>
__global__ __launch_bounds__(kThreads) void rpart_partial_kernel(PartialArgs a)
{
    const int32_t *hdr = a.v.hdr;
    if (!plan_matches(hdr, a.B, a.H, plan_kind(D, 16), a.v.max_items, (int)gridDim.x, a.status)) return;
    if ((int)blockIdx.x >= hdr[HDR_GRID]) return;
    unit_prologue<D>(hdr, a.v.nchunk, a.v.newlen, a.v.newseen, a.seq_lens, a.seq_seen, a.out, a.B, a.H);
    if constexpr (kWaveUnitsFp16 != 0) {
        if (hdr[HDR_WAVE_UNITS]) {
            rpart_body<D, NL, 1>(a);
            return;
        }
    }
    rpart_body<D, NL, kWaves>(a);
}

// ---------------------------------------------------------------------------
// Stand-alone merge, one wave per (b,h): recomputes `out` of every split sequence from the chunk
// states in the workspace, in the same order as the streaming kernel's own merge (same bits),
// and writes zeros for empty sequences.  The decode entry points do not launch it.
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void rpart_merge_kernel(PlanView v, _Float16 *__restrict__ out, int B,
                                                          int H, int kind, int32_t *__restrict__ status)
{
    if (!plan_matches(v.hdr, B, H, kind, v.max_items, 0, status)) return;
    const int lane = threadIdx.x & 63;
    const int64_t bh = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (bh >= (int64_t)B * H) return;
    const int b = (int)(bh / H);
    const int h = (int)(bh - (int64_t)b * H);
    const int n = v.nchunk[b];
    if (n == 1) return;                               // written by the streaming kernel
    _Float16 *o = out + bh * D;
    if (n == 0) {
        if (lane < 16) {
#pragma unroll
            for (int p = 0; p < D / 64; ++p) *(hvec4 *)(o + lane * 4 + p * 64) = hvec4{0, 0, 0, 0};
        }
        return;
    }
    const int64_t rec0 = (int64_t)v.item0[b] * H + h;
    if (n <= kSmallMerge) merge_states_small<D>(lane, lane < 16, n, rec0, H, v.acc, v.ml, o);
    else merge_states<D>(lane, n, rec0, H, v.acc, v.ml, o);
}

// ---------------------------------------------------------------------------
// Pure-read probe: what a kernel that only streams memory reaches on this device,
// with the same 128-bit non-temporal loads.  Each workgroup walks a private
// contiguous region, 8 loads per lane in flight.
// ---------------------------------------------------------------------------
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void hbm_read_probe_kernel(const uint4v *__restrict__ p,
                                                             size_t iters_per_wg,
                                                             int32_t *__restrict__ sink)
{
    constexpr int U = 8;
    const uint4v *q = p + (size_t)blockIdx.x * iters_per_wg * (256 * U) + threadIdx.x;
    unsigned acc = 0;
    for (size_t i = 0; i < iters_per_wg; ++i, q += 256 * U) {
        uint4v v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(q + u * 256);
#pragma unroll
        for (int u = 0; u < U; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x9E3779B9u) sink[0] = (int32_t)acc;     // keeps the loads alive
}

// Measurement aid: fill a buffer with a seeded bit pattern whose 16-bit halves are finite fp16
// values of magnitude 0.25 .. 1 (read as float32 the words are finite too), without any help
// from the framework that owns the memory.
__global__ __launch_bounds__(256) void fill_pattern_kernel(uint32_t *__restrict__ p, size_t n_words,
                                                           uint32_t seed)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_words; i += stride) {
        uint32_t x = (uint32_t)i * 0x9E3779B1u + (uint32_t)(i >> 32) + seed;
        x ^= x >> 15;
        x *= 0x85EBCA6Bu;
        x ^= x >> 13;
        // per half: sign, exponent field 13 or 14, ten mantissa bits
        const uint32_t lo = (x & 0x83FFu) | ((13u + ((x >> 10) & 1u)) << 10);
        const uint32_t hi = ((x >> 16) & 0x83FFu) | ((13u + ((x >> 26) & 1u)) << 10);
        p[i] = lo | (hi << 16);
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
constexpr int kTileLoads = 8;                          // wave loads of K (and of V) per tile

inline bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }

int check_desc(const fd_kv_desc *d)
{
    if (!d) return FD_EINVAL;
    if (d->B < 0 || d->H <= 0 || (d->d != 64 && d->d != 128)) return FD_EINVAL;
    if (d->chunk_tokens < 0) return FD_EINVAL;
    if (d->B == 0) return FD_OK;
    if (!d->k_base || !d->v_base || !d->seq_off || !d->seq_cap || !d->seq_lens || !d->status)
        return FD_EINVAL;
    if (!aligned(d->k_base, 16) || !aligned(d->v_base, 16) || !aligned(d->seq_off, 8) ||
        !aligned(d->seq_cap, 4) || !aligned(d->seq_lens, 4) || !aligned(d->status, 4))
        return FD_EINVAL;
    if (d->seq_seen && (!aligned(d->seq_seen, 4) || d->n_sink < 0)) return FD_EINVAL;
    return FD_OK;
}

int check_ws(const fd_kv_desc *d, const void *ws, size_t ws_bytes, WsLayout *w)
{
    if (!ws || !aligned(ws, 256)) return FD_EINVAL;
    *w = ws_layout(d->B, d->H, d->d, ws_bytes);
    if (w->max_items < d->B) return FD_EWORKSPACE;
    return FD_OK;
}

// chunk boundaries are multiples of this many tokens (one wave load of rows)
int chunk_granule(int d) { return d == 128 ? 32 : 64; }

// Compute units of the current device, asked for at every call: the library keeps no state
// between calls, and a process may use several devices.  The streaming kernels are launched
// with two (or three) workgroups per CU; the planner decides how many take part.
int persistent_grid()
{
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        return 0;
    return cus;
}

int launched(void) { return hipGetLastError() == hipSuccess ? FD_OK : FD_EHIP; }

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];          // device address of `scratch` on device i, or null

// Address of the current device's scratch array; null on failure.  The first call on a device
// looks the symbol up with that device current; later calls return the kept address.  Two
// threads racing through the first call both obtain the same address.
void *scratch_address()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void *p = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
    if (p) return p;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
        (void)hipGetLastError();
        return nullptr;
    }
    __atomic_store_n(&g_scratch_ptr[dev], p, __ATOMIC_RELEASE);
    return p;
}

SeqState seq_state(const fd_kv_desc *d)
{
    SeqState st;
    st.seq_off = d->seq_off;
    st.seq_cap = d->seq_cap;
    st.seq_lens = d->seq_lens;
    st.seq_seen = d->seq_seen;
    st.status = d->status;
    st.n_sink = d->n_sink;
    return st;
}


PlanArgs plan_args(const fd_kv_desc *d, void *workspace, const WsLayout &w, int grid, int after_append)
{
    PlanArgs a;
    a.seq_lens = d->seq_lens;
    a.seq_cap = d->seq_cap;
    a.seq_seen = d->seq_seen;
    a.status = d->status;
    a.n_sink = d->n_sink;
    a.after_append = after_append;
    a.B = d->B;
    a.H = d->H;
    a.chunk_req = d->chunk_tokens;
    a.granule = chunk_granule(d->d);
    a.grid_long = grid;
    a.grid_short = 2 * grid;
    a.short_below = kShortSeq;
    a.hashed = 0;
    a.wave_units = kWaveUnitsFp16;
    a.split = 16;
    a.kind = plan_kind(d->d, 16);
    a.v = plan_view(workspace, w);
    return a;
}

// the streaming launch; every argument has been checked
int launch_partial(const fd_kv_desc *desc, const void *q, void *out, void *workspace,
                   const WsLayout &w, int grid, void *stream)
{
    PartialArgs a;
    a.k_base = (const char *)desc->k_base;
    a.v_base = (const char *)desc->v_base;
    a.seq_off = desc->seq_off;
    a.seq_cap = desc->seq_cap;
    a.seq_lens = desc->seq_lens;
    a.seq_seen = desc->seq_seen;
    a.status = desc->status;
    a.q = (const _Float16 *)q;
    a.out = (_Float16 *)out;
    a.B = desc->B;
    a.H = desc->H;
    // scores are kept in the base-2 exponent domain: exp(x) = 2^(x * log2 e)
    a.qscale = (float)(1.4426950408889634 / (desc->d == 128 ? 11.313708498984761 : 8.0));
    a.v = plan_view(workspace, w);
    if (desc->d == 128)
        hipLaunchKernelGGL((rpart_partial_kernel<128, kTileLoads>), dim3(2 * grid), dim3(kThreads), 0,
                           (hipStream_t)stream, a);
    else
        hipLaunchKernelGGL((rpart_partial_kernel<64, kTileLoads>), dim3(2 * grid), dim3(kThreads), 0,
                           (hipStream_t)stream, a);
    return launched();
}

// host checks shared by the entry points that take q, out and a workspace
int check_decode_args(const fd_kv_desc *desc, const void *q, const void *out, const void *workspace,
                      size_t workspace_bytes, WsLayout *w)
{
    int rc = check_desc(desc);
    if (rc != FD_OK) return rc;
    if (desc->B == 0) return FD_OK;
    if (!q || !out || !aligned(q, 16) || !aligned(out, 16)) return FD_EINVAL;
    return check_ws(desc, workspace, workspace_bytes, w);
}

} // namespace

extern "C" {

int fd_version(void) { return kVersion; }

size_t fd_desc_size(int which)
{
    return which == 0 ? sizeof(fd_kv_desc) : which == 1 ? sizeof(fd_kvq_desc) : 0;
}

const char *fd_strerror(int code)
{
    switch (code) {
    case FD_OK: return "ok";
    case FD_EINVAL: return "invalid argument (null or misaligned pointer, bad shape)";
    case FD_EWORKSPACE: return "workspace too small";
    case FD_EHIP: return "HIP runtime call or kernel launch failed";
    case FD_ETOOBIG: return "batch too large for the built-in scratch of the no-allocation entry point";
    default: return "unknown error code";
    }
}

size_t fd_workspace_bytes(int32_t B, int32_t H, int32_t d, int64_t max_total_tokens)
{
    if (B < 0 || H <= 0 || (d != 64 && d != 128) || max_total_tokens < 0) return 0;
    WsLayout w = ws_layout(B, H, d, 0);
    const size_t per_item = ws_per_item(H, d);
    const size_t extra = (size_t)((max_total_tokens + 255) / 256);
    return align_up(w.min_bytes + extra * per_item, 256);
}

int fd_kv_append(const fd_kv_desc *desc, const void *k_new, const void *v_new, void *stream)
{
    int rc = check_desc(desc);
    if (rc != FD_OK) return rc;
    if (desc->B == 0) return FD_OK;
    if (!k_new || !v_new || !aligned(k_new, 16) || !aligned(v_new, 16)) return FD_EINVAL;
    hipLaunchKernelGGL(kv_append_kernel, dim3(desc->B), dim3(256), 0, (hipStream_t)stream,
                       (uint4 *)desc->k_base, (uint4 *)desc->v_base, seq_state(desc),
                       (const uint4 *)k_new, (const uint4 *)v_new, desc->H, desc->d);
    return launched();
}

int fd_kv_append_plan(const fd_kv_desc *desc, const void *k_new, const void *v_new,
                      void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_desc(desc);
    if (rc != FD_OK) return rc;
    if (desc->B == 0) return FD_OK;
    if (!k_new || !v_new || !aligned(k_new, 16) || !aligned(v_new, 16)) return FD_EINVAL;
    WsLayout w;
    rc = check_ws(desc, workspace, workspace_bytes, &w);
    if (rc != FD_OK) return rc;
    const int grid = persistent_grid();
    if (grid <= 0) return FD_EHIP;
    hipLaunchKernelGGL(kv_append_plan_kernel, dim3(desc->B + 1), dim3(kPlanThreads), 0,
                       (hipStream_t)stream, (uint4 *)desc->k_base, (uint4 *)desc->v_base,
                       seq_state(desc), (const uint4 *)k_new, (const uint4 *)v_new, desc->d,
                       plan_args(desc, workspace, w, grid, 1));
    return launched();
}

static int reset_slots(const fd_kv_desc *desc, const int32_t *seq_ids, int32_t n, int value,
                       void *stream)
{
    int rc = check_desc(desc);
    if (rc != FD_OK) return rc;
    if (desc->B == 0) return FD_OK;
    if (seq_ids && n < 0) return FD_EINVAL;
    const int count = seq_ids ? n : desc->B;
    if (count == 0) return FD_OK;
    hipLaunchKernelGGL(kv_reset_kernel, dim3((count + 255) / 256), dim3(256), 0,
                       (hipStream_t)stream, desc->seq_lens, desc->seq_seen, seq_ids, count,
                       desc->B, value);
    return launched();
}

int fd_kv_reset(const fd_kv_desc *desc, const int32_t *seq_ids, int32_t n, void *stream)
{
    return reset_slots(desc, seq_ids, n, 0, stream);
}

int fd_kv_release(const fd_kv_desc *desc, const int32_t *seq_ids, int32_t n, void *stream)
{
    return reset_slots(desc, seq_ids, n, FD_SLOT_FREE, stream);
}

int fd_rpart_plan(const fd_kv_desc *desc, void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_desc(desc);
    if (rc != FD_OK) return rc;
    if (desc->B == 0) return FD_OK;
    WsLayout w;
    rc = check_ws(desc, workspace, workspace_bytes, &w);
    if (rc != FD_OK) return rc;
    const int grid = persistent_grid();
    if (grid <= 0) return FD_EHIP;
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(kPlanThreads), 0, (hipStream_t)stream,
                       plan_args(desc, workspace, w, grid, 0));
    return launched();
}

int fd_rpart_partial(const fd_kv_desc *desc, const void *q, void *out,
                     void *workspace, size_t workspace_bytes, void *stream)
{
    WsLayout w;
    int rc = check_decode_args(desc, q, out, workspace, workspace_bytes, &w);
    if (rc != FD_OK || desc->B == 0) return rc;
    const int grid = persistent_grid();
    if (grid <= 0) return FD_EHIP;
    return launch_partial(desc, q, out, workspace, w, grid, stream);
}

int fd_rpart_merge(const fd_kv_desc *desc, void *out,
                   void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_desc(desc);
    if (rc != FD_OK) return rc;
    if (desc->B == 0) return FD_OK;
    if (!out || !aligned(out, 16)) return FD_EINVAL;
    WsLayout w;
    rc = check_ws(desc, workspace, workspace_bytes, &w);
    if (rc != FD_OK) return rc;
    const int64_t bh = (int64_t)desc->B * desc->H;
    const dim3 grid((unsigned)((bh + 3) / 4));
    const PlanView v = plan_view(workspace, w);
    if (desc->d == 128)
        hipLaunchKernelGGL(rpart_merge_kernel<128>, grid, dim3(256), 0, (hipStream_t)stream, v,
                           (_Float16 *)out, desc->B, desc->H, plan_kind(128, 16), desc->status);
    else
        hipLaunchKernelGGL(rpart_merge_kernel<64>, grid, dim3(256), 0, (hipStream_t)stream, v,
                           (_Float16 *)out, desc->B, desc->H, plan_kind(64, 16), desc->status);
    return launched();
}

int fd_rpart_decode(const fd_kv_desc *desc, const void *q, void *out,
                    void *workspace, size_t workspace_bytes, void *stream)
{
    // validate everything before the first launch so that a failing call enqueues nothing
    WsLayout w;
    int rc = check_decode_args(desc, q, out, workspace, workspace_bytes, &w);
    if (rc != FD_OK || desc->B == 0) return rc;
    const int grid = persistent_grid();
    if (grid <= 0) return FD_EHIP;
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(kPlanThreads), 0, (hipStream_t)stream,
                       plan_args(desc, workspace, w, grid, 0));
    rc = launched();
    if (rc != FD_OK) return rc;
    return launch_partial(desc, q, out, workspace, w, grid, stream);
}

int fd_rpart_decode_noalloc(const fd_kv_desc *desc, const void *q, void *out, void *stream)
{
    int rc = check_desc(desc);
    if (rc != FD_OK) return rc;
    if (desc->B == 0) return FD_OK;
    if (!q || !out || !aligned(q, 16) || !aligned(out, 16)) return FD_EINVAL;
    // the plan tables and one chunk state per sequence must fit the fixed array
    const WsLayout w = ws_layout(desc->B, desc->H, desc->d, FD_NOALLOC_SCRATCH_BYTES);
    if (w.max_items < desc->B) return FD_ETOOBIG;
    void *ws = scratch_address();
    if (!ws) return FD_EHIP;
    // nothing in the array has to start at zero: the planner rewrites the header, every table
    // entry and every counter the other kernels read, and chunk states are written before they
    // are merged
    return fd_rpart_decode(desc, q, out, ws, FD_NOALLOC_SCRATCH_BYTES, stream);
}

// append + plan in one launch, then the streaming kernel: two launches per step
static int step_fused(const fd_kv_desc *desc, const void *q, const void *k_new, const void *v_new,
                      void *out, void *workspace, size_t workspace_bytes, void *stream)
{
    WsLayout w;
    int rc = check_decode_args(desc, q, out, workspace, workspace_bytes, &w);
    if (rc != FD_OK || desc->B == 0) return rc;
    if (!k_new || !v_new || !aligned(k_new, 16) || !aligned(v_new, 16)) return FD_EINVAL;
    const int grid = persistent_grid();
    if (grid <= 0) return FD_EHIP;
    hipLaunchKernelGGL(kv_append_plan_kernel, dim3(desc->B + 1), dim3(kPlanThreads), 0,
                       (hipStream_t)stream, (uint4 *)desc->k_base, (uint4 *)desc->v_base,
                       seq_state(desc), (const uint4 *)k_new, (const uint4 *)v_new, desc->d,
                       plan_args(desc, workspace, w, grid, 1));
    rc = launched();
    if (rc != FD_OK) return rc;
    return launch_partial(desc, q, out, workspace, w, grid, stream);
}

int fd_rpart_step(const fd_kv_desc *desc, const void *q, const void *k_new, const void *v_new,
                  void *out, void *workspace, size_t workspace_bytes, void *stream)
{
    return step_fused(desc, q, k_new, v_new, out, workspace, workspace_bytes, stream);
}

int fd_rpart_layer_step(const fd_kv_desc *layer, const void *q, const void *k_new,
                        const void *v_new, void *out, void *workspace, size_t workspace_bytes,
                        int replan, void *stream)
{
    if (replan) return step_fused(layer, q, k_new, v_new, out, workspace, workspace_bytes, stream);
    WsLayout w;
    int rc = check_decode_args(layer, q, out, workspace, workspace_bytes, &w);
    if (rc != FD_OK || layer->B == 0) return rc;
    if (!k_new || !v_new || !aligned(k_new, 16) || !aligned(v_new, 16)) return FD_EINVAL;
    const int grid = persistent_grid();
    if (grid <= 0) return FD_EHIP;
    rc = fd_kv_append(layer, k_new, v_new, stream);
    if (rc != FD_OK) return rc;
    return launch_partial(layer, q, out, workspace, w, grid, stream);
}

int fd_hbm_read_probe(const void *buf, size_t bytes, int32_t *sink, size_t *bytes_read, void *stream)
{
    if (!buf || !sink || !bytes_read || !aligned(buf, 16)) return FD_EINVAL;
    const int grid = 2 * persistent_grid();
    if (grid <= 0) return FD_EHIP;
    const size_t per_iter = 256 * 8 * 16;                       // bytes per workgroup iteration
    const size_t iters = bytes / per_iter / (size_t)grid;
    *bytes_read = iters * per_iter * (size_t)grid;
    if (iters == 0) return FD_EINVAL;
    hipLaunchKernelGGL(hbm_read_probe_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream,
                       (const uint4v *)buf, iters, sink);
    return launched();
}

int fd_fill_pattern(void *buf, size_t bytes, uint32_t seed, void *stream)
{
    if (!buf || !aligned(buf, 4) || bytes % 4 != 0) return FD_EINVAL;
    if (bytes == 0) return FD_OK;
    const int cus = persistent_grid();
    if (cus <= 0) return FD_EHIP;
    hipLaunchKernelGGL(fill_pattern_kernel, dim3(cus * 8), dim3(256), 0, (hipStream_t)stream,
                       (uint32_t *)buf, bytes / 4, seed);
    return launched();
}

int fd_read_status(const fd_kv_desc *desc, int32_t *host_status, int clear, void *stream)
{
    if (!desc || !desc->status || !host_status) return FD_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    if (hipMemcpyAsync(host_status, desc->status, sizeof(int32_t), hipMemcpyDeviceToHost, s) !=
        hipSuccess)
        return FD_EHIP;
    if (hipStreamSynchronize(s) != hipSuccess) return FD_EHIP;
    if (clear && *host_status != 0) {
        // only the bits just reported are cleared: one raised since the copy stays for the next read
        hipLaunchKernelGGL(status_clear_bits_kernel, dim3(1), dim3(1), 0, s, desc->status, *host_status);
        if (launched() != FD_OK) return FD_EHIP;
        if (hipStreamSynchronize(s) != hipSuccess) return FD_EHIP;
    }
    return FD_OK;
}

int fd_last_device_status(const fd_kv_desc *desc, void *workspace, int32_t *host_out, void *stream)
{
    if (!desc || !desc->status || !host_out || !workspace || !aligned(workspace, 256)) return FD_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    int32_t *slot = (int32_t *)workspace + HDR_STATUS_OUT;   // a header word no kernel reads
    hipLaunchKernelGGL(status_take_kernel, dim3(1), dim3(1), 0, s, desc->status, slot);
    if (launched() != FD_OK) return FD_EHIP;
    if (hipMemcpyAsync(host_out, slot, sizeof(int32_t), hipMemcpyDeviceToHost, s) != hipSuccess)
        return FD_EHIP;
    if (hipStreamSynchronize(s) != hipSuccess) return FD_EHIP;
    return FD_OK;
}

int fd_kv_store_rows(const fd_kv_desc *desc, int32_t b, int32_t t0, int32_t n, const void *k_rows,
                     const void *v_rows, int set_len, void *stream)
{
    int rc = check_desc(desc);
    if (rc != FD_OK) return rc;
    if (b < 0 || b >= desc->B || t0 < 0 || n < 0 || (int64_t)t0 + n > INT32_MAX) return FD_EINVAL;
    if ((k_rows && !aligned(k_rows, 16)) || (v_rows && !aligned(v_rows, 16))) return FD_EINVAL;
    if (n == 0 && !set_len) return FD_OK;
    const int64_t words = (int64_t)desc->H * n * (desc->d / 8);
    const unsigned grid = (unsigned)(words > 0 ? (words + 255) / 256 : 1);
    hipLaunchKernelGGL(kv_store_rows_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream,
                       (uint4 *)desc->k_base, (uint4 *)desc->v_base, desc->seq_off, desc->seq_cap,
                       desc->seq_lens, desc->seq_seen, desc->status, (const uint4 *)k_rows,
                       (const uint4 *)v_rows, desc->H, desc->d, b, t0, n, set_len);
    return launched();
}

int fd_plan_info(const void *workspace, int32_t info[4], void *stream)
{
    if (!workspace || !info) return FD_EINVAL;
    int32_t hdr[8];
    hipStream_t s = (hipStream_t)stream;
    if (hipMemcpyAsync(hdr, workspace, sizeof(hdr), hipMemcpyDeviceToHost, s) != hipSuccess)
        return FD_EHIP;
    if (hipStreamSynchronize(s) != hipSuccess) return FD_EHIP;
    info[0] = hdr[HDR_NITEMS];
    info[1] = hdr[HDR_CHUNK];
    info[2] = hdr[HDR_TOKENS];
    info[3] = hdr[HDR_GRID];
    return FD_OK;
}

} // extern "C"

// quantised KV-cache path (Section 5.2); reuses the planner, merge kernel and helpers above
#include "fd_rpartq.h"

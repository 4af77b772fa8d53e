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
       HDR_H = 7, HDR_MAXITEMS = 8, HDR_WAVE_UNITS = 9, HDR_KIND = 10, HDR_STATUS_OUT = 16 };
// cache format a plan was made for: head dimension and bits per element (16 = fp16)
constexpr int plan_kind(int d, int bits) { return d | (bits << 16); }
constexpr int32_t kPlanMagic = 0x46445250;

struct WsLayout {
    size_t off_item0;     // int32[B]  first item of sequence b
    size_t off_nchunk;    // int32[B]  chunks of sequence b
    size_t off_items;     // int4[max_items]  {b, t0, t1, n_chunks_of_b}, chunks of a sequence adjacent
    size_t off_order;     // int32[max_items] item indices, longest chunk first (the schedule)
    size_t off_acc;       // float[max_items][H][d]  unnormalised weighted value sums (512 B records)
    size_t off_ml;        // float[max_items][H][2]  {running max, sum of exponentials}
    int64_t max_items;
    size_t min_bytes;     // bytes needed for max_items == B
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

inline size_t ws_per_item(int H, int d) { return 16 + 4 + (size_t)H * (size_t)(d + 2) * 4; }

inline WsLayout ws_layout(int B, int H, int d, size_t ws_bytes)
{
    WsLayout w;
    size_t o = kHdrInts * sizeof(int32_t);
    w.off_item0 = o;
    o = align_up(o + (size_t)B * 4, 256);
    w.off_nchunk = o;
    o = align_up(o + (size_t)B * 4, 256);
    w.off_items = o;
    const size_t per_item = ws_per_item(H, d);
    const size_t slop = 4 * 256;                         // alignment of the four arrays
    w.min_bytes = o + slop + (size_t)(B > 0 ? B : 1) * per_item;
    w.max_items = 0;
    w.off_order = w.off_acc = w.off_ml = 0;
    if (ws_bytes < w.min_bytes) return w;
    w.max_items = (int64_t)((ws_bytes - o - slop) / per_item);
    if (w.max_items > (int64_t)0x3FFFFFFF) w.max_items = 0x3FFFFFFF;
    const size_t n = (size_t)w.max_items;
    w.off_order = align_up(w.off_items + n * 16, 256);
    w.off_acc = align_up(w.off_order + n * 4, 256);
    w.off_ml = align_up(w.off_acc + n * (size_t)H * (size_t)d * 4, 256);
    return w;
}

// ---------------------------------------------------------------------------
// Append (Section 4.1).  One workgroup per sequence: 2*H rows of d fp16 are
// copied as raw 128-bit words, then one thread bumps the length.
// ---------------------------------------------------------------------------
// Row that the new token of sequence b goes to, and the sequence's length afterwards; -1 if
// the append is skipped (free slot, full plain cache, inconsistent window state).  Uniform
// over the workgroup; thread 0 reports errors.
__device__ inline int append_row(const int32_t *seq_lens, const int32_t *seq_cap,
                                 const int32_t *seq_seen, int n_sink, int32_t *status, int b,
                                 int *new_len)
{
    const int L = seq_lens[b];
    const int cap = seq_cap[b];
    if (L == FD_SLOT_FREE) return -1;
    if (!seq_seen) {
        if (L < 0 || L >= cap) {
            if (threadIdx.x == 0) atomicOr(status, FD_ST_CAPACITY);
            return -1;
        }
        *new_len = L + 1;
        return L;
    }
    // windowed cache: a bounded buffer of n_sink fixed rows and a ring of cap - n_sink rows
    const int p = seq_seen[b];
    if (n_sink < 0 || n_sink >= cap || p < 0 || L != (p < cap ? p : cap)) {
        if (threadIdx.x == 0) atomicOr(status, FD_ST_WINDOW);
        return -1;
    }
    *new_len = p + 1 < cap ? p + 1 : cap;
    return p < cap ? p : n_sink + (p - n_sink) % (cap - n_sink);
}

__global__ __launch_bounds__(256) void kv_append_kernel(
    uint4 *__restrict__ k_base, uint4 *__restrict__ v_base,
    const int64_t *__restrict__ seq_off, const int32_t *__restrict__ seq_cap,
    int32_t *__restrict__ seq_lens, int32_t *__restrict__ status,
    const uint4 *__restrict__ k_new, const uint4 *__restrict__ v_new, int H, int d,
    int32_t *__restrict__ seq_seen, int n_sink)
{
    const int b = blockIdx.x;
    const int cap = seq_cap[b];
    int new_len = 0;
    const int L = append_row(seq_lens, seq_cap, seq_seen, n_sink, status, b, &new_len);
    if (L < 0) return;
    const int vpr = d / 8;                               // 16-byte words per row
    const int n = H * vpr;
    const int64_t blk = seq_off[b] / 8;                  // block offset in 16-byte words
    const int64_t src0 = (int64_t)b * n;
    for (int x = threadIdx.x; x < 2 * n; x += blockDim.x) {
        const int which = x >= n;
        const int y = which ? x - n : x;
        const int h = y / vpr, c = y - h * vpr;
        const int64_t dst = blk + ((int64_t)h * cap + L) * vpr + c;
        if (which) v_base[dst] = v_new[src0 + y];
        else       k_base[dst] = k_new[src0 + y];
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        seq_lens[b] = new_len;
        if (seq_seen) seq_seen[b] += 1;
    }
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
// ---------------------------------------------------------------------------
constexpr int kShortSeq = 384;      // a sequence under this many tokens is latency-bound ("short")
constexpr int kBuckets = 256;

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

__global__ __launch_bounds__(kPlanThreads) void plan_kernel(
    const int32_t *__restrict__ seq_lens, const int32_t *__restrict__ seq_cap,
    int32_t *__restrict__ status, int B, int H, int chunk_req, int granule, int grid_long, int grid_short,
    int short_below, int hashed, int wave_units, int split, int kind, int max_items,
    int32_t *__restrict__ hdr, int32_t *__restrict__ item0, int32_t *__restrict__ nchunk,
    int4 *__restrict__ items, int32_t *__restrict__ order)
{
    __shared__ int sm[kPlanThreads];
    __shared__ int hist[kBuckets];
    __shared__ int4 big[kBigMax];
    __shared__ int nbig, big_nmax;
    const int tid = threadIdx.x;
    const int per = (B + kPlanThreads - 1) / kPlanThreads;   // sequences per thread (contiguous)
    const int b0 = tid * per;
    const int b1 = min(B, b0 + per);

    int bad = 0, mine = 0;
    for (int b = b0; b < b1; ++b) mine += clamp_len(seq_lens[b], seq_cap[b], &bad);
    const int total = block_sum(mine, sm);
    if (bad) atomicOr(status, FD_ST_BADLEN);

    // One workgroup per CU streams long sequences best (a second one costs 1-2 %); a sequence of
    // a few blocks is dominated by its fixed cost, and more workgroups per CU hide that.  Measured
    // on the fp16 kernel, one against two per CU: 256 tokens each +3.5 %, lengths uniform in
    // 1..1024 (the load-stabilising schedule's mix) +2.2 %, 512 each -1.1 %, uniform in 1..2048
    // -0.6 %, exponential with mean 1024 -1.2 %.  What separates them is the share of the
    // cached tokens that sits in sequences shorter than short_below tokens (100 %, 14 %, 0, 3.5 %,
    // 5.5 %): above a tenth the larger grid is used.  The host launches the larger number and
    // workgroups at or beyond `grid` leave at once.
    int few = 0;
    for (int b = b0; b < b1; ++b) {
        const int L = clamp_len(seq_lens[b], seq_cap[b], &bad);
        few += L < short_below ? L : 0;
    }
    few = block_sum(few, sm);
    const bool many_short = (long long)few * 10 > (long long)total;
    const int grid = many_short ? grid_short : grid_long;
    // wave_units: 0 = the workgroup's waves always share a unit, 1 = each wave takes units of its
    // own when the batch holds many short sequences, 2 = always
    const int wave_now = wave_units == 2 || (wave_units == 1 && many_short);

    int T;
    if (chunk_req > 0) {
        T = chunk_req;
    } else {
        // token-heads per worker: a workgroup, or a wave when each wave takes units of its own
        const long long share = (long long)total * H / ((long long)grid * (wave_now ? kWaves : 1));
        long long t = share / split;
        T = (int)(t < 128 ? 128 : (t > (1 << 28) ? (1 << 28) : t));
    }
    T = (T + granule - 1) / granule * granule;

    int count;
    for (;;) {
        int c = 0;
        for (int b = b0; b < b1; ++b) {
            const int L = clamp_len(seq_lens[b], seq_cap[b], &bad);
            c += (L + T - 1) / T;
        }
        count = block_sum(c, sm);
        if (count <= max_items || T >= (1 << 30)) break;   // T >= longest sequence gives count <= B
        T *= 2;
    }

    // exclusive scan of per-thread item counts
    int c = 0, c_big = 0;
    for (int b = b0; b < b1; ++b) {
        const int L = clamp_len(seq_lens[b], seq_cap[b], &bad);
        const int n = (L + T - 1) / T;
        c += n;
        c_big += n > kBigChunks;
    }
    // A sequence cut into many chunks (one that has the device almost to itself) is written out
    // by the whole workgroup, a chunk per thread, instead of by the one thread that owns it:
    // 128 chunks walked by one thread took 46 us.  The list is used only when it holds them all.
    const bool use_list = block_sum(c_big, sm) <= kBigMax;
    if (tid < kBuckets) hist[tid] = 0;
    if (tid == 0) { nbig = 0; big_nmax = 0; }
    const int first = block_exclusive_scan(c, sm);      // its barriers also publish hist = 0
    int pos = first;
    for (int b = b0; b < b1; ++b) {
        const int L = clamp_len(seq_lens[b], seq_cap[b], &bad);
        const int n = (L + T - 1) / T;
        item0[b] = pos;
        nchunk[b] = n;
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
        }
        pos += n;
    }
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
    }
    __syncthreads();
    // bucket starts = exclusive scan of the 256 counters, then scatter
    {
        const int n = tid < kBuckets ? hist[tid] : 0;
        const int start = block_exclusive_scan(n, sm);
        if (tid < kBuckets) hist[tid] = start;
    }
    __syncthreads();
    // Scatter.  Inside a bucket the order is the arrival order of the atomics.  With `hashed` the
    // sequences are visited in a scrambled order (a bijection of [0, B)): equal-length sequences
    // then run side by side in no regular pattern.  A regular one can put the streams that run
    // in lockstep a constant distance apart, and for some distances (2^a + 2^(a+8) bytes was
    // seen) they then fight over the same DRAM banks all the way: -10 % on the int8 kernel.
    int bits = 1;
    while ((1 << bits) < B) ++bits;
    const unsigned mask = (1u << bits) - 1u;
    const int half = (bits + 1) / 2;
    for (int j = b0; j < b1; ++j) {
        int b = j;
        if (hashed) {
            unsigned x = (unsigned)j;
            do {                                            // cycle-walk back into [0, B)
                x = (x * 0x9E3779B1u) & mask;
                x ^= x >> half;
                x = (x * 0x85EBCA6Bu) & mask;
                x ^= x >> half;
            } while (x >= (unsigned)B);
            b = (int)x;
        }
        const int n = nchunk[b];
        const int base = item0[b];
        if (n > 0 && !(use_list && n > kBigChunks)) {
            const int L = clamp_len(seq_lens[b], seq_cap[b], &bad);
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
    if (tid == 0) {
        hdr[HDR_NITEMS] = count <= max_items ? count : 0;
        hdr[HDR_CHUNK] = T;
        hdr[HDR_TOKENS] = total;
        hdr[HDR_GRID] = grid;
        hdr[HDR_MAGIC] = kPlanMagic;
        hdr[HDR_B] = B;
        hdr[HDR_H] = H;
        hdr[HDR_MAXITEMS] = max_items;
        hdr[HDR_WAVE_UNITS] = wave_now;
        hdr[HDR_KIND] = kind;
    }
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

// One tile = this wave's share of a workgroup block.  A block is kWaves * NL
// consecutive wave loads (1 KB each) of the K stream and of the V stream; wave w
// takes loads w, w + kWaves, ...: the workgroup reads the block as one contiguous
// run with its waves interleaved at 1 KB, and every wave gets the same number of
// loads whatever the chunk length.
template <int D, int NL>
struct Tile {
    static constexpr int LPR = D / 8;                    // lanes per row
    static constexpr int RPW = 64 / LPR;                 // rows (tokens) per wave load
    static constexpr int STRIDE = kWaves * 1024;         // bytes between a wave's consecutive loads
    static constexpr int TSTEP = kWaves * RPW;           // tokens between a wave's consecutive loads
    static constexpr int BLK_TOK = NL * TSTEP;           // tokens per workgroup block
    static constexpr int BLK_BYTES = NL * STRIDE;        // bytes of K (or V) per workgroup block
    half8 k[NL], v[NL];

    __device__ inline void load(const char *kp, const char *vp)
    {
#pragma unroll
        for (int j = 0; j < NL; ++j) k[j] = ld_stream(kp + j * STRIDE);
#pragma unroll
        for (int j = 0; j < NL; ++j) v[j] = ld_stream(vp + j * STRIDE);
    }

    // ragged last block of `rem` tokens: a lane whose token (tok0 + j*TSTEP) is at or beyond
    // `rem` re-reads token rem-1 (in bounds) and is masked in update<true>
    __device__ inline void load_tail(const char *kp, const char *vp, int tok0, int rem)
    {
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            const int t = j * TSTEP + tok0;
            const int back = t < rem ? 0 : (t - (rem - 1)) * (D * 2);
            k[j] = ld_stream(kp + j * STRIDE - back);
            v[j] = ld_stream(vp + j * STRIDE - back);
        }
    }

    template <bool MASKED>
    __device__ inline void update(const float (&q)[8], float &m, float &l, float (&acc)[8],
                                  int tok0, int rem) const
    {
        float s[NL];
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            float a = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) a = __builtin_fmaf((float)k[j][i], q[i], a);
            a = row_sum<LPR>(a);
            if (MASKED && j * TSTEP + tok0 >= rem) a = kNegBig;
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
            float p = fast_exp2(s[j] - mn);
            if (MASKED && j * TSTEP + tok0 >= rem) p = 0.f;
            l += p;
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = __builtin_fmaf(p, (float)v[j][i], acc[i]);
        }
        m = mn;
    }
};

// Where a unit of work (one chunk of one head's stream) lives; uniform over the workgroup.
struct Unit {
    int64_t row0;            // element offset of the chunk's first row in the K / V slab
    int ntok;                // tokens in the chunk; 0 = no unit
    int b, h, item, nch;     // sequence, head, item index, chunks of the sequence
};

template <int D, int NL>
__global__ __launch_bounds__(kThreads) void rpart_partial_kernel(
    const char *__restrict__ k_base, const char *__restrict__ v_base,
    const int64_t *__restrict__ seq_off, const int32_t *__restrict__ seq_cap,
    const _Float16 *__restrict__ q, _Float16 *__restrict__ out, int H,
    const int32_t *__restrict__ hdr, const int4 *__restrict__ items,
    const int32_t *__restrict__ order, float *__restrict__ part_acc, float *__restrict__ part_ml,
    float qscale, int B, int max_items, int32_t *__restrict__ status)
{
    using T = Tile<D, NL>;
    constexpr int LPR = T::LPR;
    // two sets, used by alternate units: one barrier per unit is then enough (a wave cannot
    // overwrite a set before every wave has passed the barrier of the unit in between)
    __shared__ float sm_acc2[2][kWaves][D];
    __shared__ float sm_m2[2][kWaves], sm_l2[2][kWaves];
    int set = 0;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int row = lane / LPR;
    const int col = lane % LPR;
    if (!plan_matches(hdr, B, H, plan_kind(D, 16), max_items, (int)gridDim.x, status)) return;
    const int n_units = hdr[HDR_NITEMS] * H;
    const int W = hdr[HDR_GRID], g = blockIdx.x;          // active workgroups, chosen by the planner
    if (g >= W) return;

    // Static snake schedule over units in longest-first order: in round k this workgroup
    // owns unit k*W + g (even k) or k*W + W-1-g (odd k), which balances the token totals.
    // The workgroups walk their rounds from kPhases different starting points, so that at
    // any moment long and short units are in flight together: short units are dominated by
    // latency, and letting every workgroup reach them at once would leave HBM idle (+3 % on
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
    while (cur.ntok > 0) {
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
            for (int i = 0; i < 8; ++i) qf[i] = (float)qh[i] * qscale;
        }

        float m = kNegBig, l = 0.f, acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = 0.f;

        const int ntok = cur.ntok;
        const int n_blk = ntok / T::BLK_TOK;              // full workgroup blocks
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
                A.template update<false>(qf, m, l, acc, 0, 0);
                sched_fence();
                A.load(kt + 2 * T::BLK_BYTES, vt + 2 * T::BLK_BYTES);
                sched_fence();
                Bf.template update<false>(qf, m, l, acc, 0, 0);
                sched_fence();
                kt += 2 * T::BLK_BYTES;
                vt += 2 * T::BLK_BYTES;
                i += 2;
            }
            if (i + 1 < n_blk) {
                Bf.load(kt + T::BLK_BYTES, vt + T::BLK_BYTES);
                sched_fence();
                A.template update<false>(qf, m, l, acc, 0, 0);
                sched_fence();
                Bf.template update<false>(qf, m, l, acc, 0, 0);
            } else {
                A.template update<false>(qf, m, l, acc, 0, 0);
            }
        }
        if (rem > 0) {
            const int tok0 = wave * T::RPW + row;
            if (wave * T::RPW < rem) {                    // this wave has at least one valid row
                const int64_t o = (int64_t)n_blk * T::BLK_BYTES;
                A.load_tail(kp + o, vp + o, tok0, rem);
                A.template update<true>(qf, m, l, acc, tok0, rem);
            }
        }

        // combine the rows of this wave (each 16- or 8-lane row saw different tokens)
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1) {
            const float mo = __shfl_xor(m, off);
            const float lo = __shfl_xor(l, off);
            const float M = fmaxf(m, mo);
            const float a = fast_exp2(m - M), c = fast_exp2(mo - M);
            l = l * a + lo * c;
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = acc[i] * a + __shfl_xor(acc[i], off) * c;
            m = M;
        }
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

        // combine the waves; write the final output or this chunk's partial state.  Stores
        // are non-temporal: they are never re-read by this kernel, and plain stores were
        // measured to cost the read stream about three times as much bandwidth.
        if (tid < D) {
            float M = sm_m[0];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) M = fmaxf(M, sm_m[w]);
            float L = 0.f, o = 0.f;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                const float a = fast_exp2(sm_m[w] - M);
                L += a * sm_l[w];
                o += a * sm_acc[w][tid];
            }
            if (cur.nch == 1) {
                __builtin_nontemporal_store((_Float16)(o / L), &out[((int64_t)b * H + h) * D + tid]);
            } else {
                const int64_t rec = (int64_t)cur.item * H + h;
                __builtin_nontemporal_store(o, &part_acc[rec * D + tid]);
                if (tid == 0) {
                    __builtin_nontemporal_store(M, &part_ml[rec * 2]);
                    __builtin_nontemporal_store(L, &part_ml[rec * 2 + 1]);
                }
            }
        }
        cur = nxt;                     // no second barrier: the next unit uses the other LDS set
    }
}

// ---------------------------------------------------------------------------
// Log-sum-exp merge of a sequence's chunk states; one wave per (b,h).
// States are in the base-2 exponent domain used by the streaming kernel.
//
// A sequence that has the device to itself is cut into over a hundred chunks per head, so the
// wave works on many chunk states at once: maxima and sums of exponentials one chunk per lane,
// the weighted value sums four records per load (16 lanes x 128-bit per record) with sixteen
// records in flight, and a cross-lane sum over the four groups at the end.
// ---------------------------------------------------------------------------
typedef float fvec4 __attribute__((ext_vector_type(4)));
typedef _Float16 hvec4 __attribute__((ext_vector_type(4)));

template <int D>
__global__ __launch_bounds__(256) void rpart_merge_kernel(
    const int32_t *__restrict__ item0, const int32_t *__restrict__ nchunk,
    const float *__restrict__ part_acc, const float *__restrict__ part_ml,
    _Float16 *__restrict__ out, int B, int H, const int32_t *__restrict__ hdr, int kind,
    int max_items, int32_t *__restrict__ status)
{
    constexpr int NV = D / 64;                        // 128-bit pieces of a record per lane
    if (!plan_matches(hdr, B, H, kind, max_items, 0, status)) return;
    const int lane = threadIdx.x & 63;
    const int t = lane & 15, g = lane >> 4;           // piece within the record, record within the load
    const int64_t bh = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (bh >= (int64_t)B * H) return;
    const int b = (int)(bh / H);
    const int h = (int)(bh - (int64_t)b * H);
    const int n = nchunk[b];
    if (n == 1) return;                               // written by the streaming kernel
    _Float16 *o = out + bh * D + t * 4;               // lanes of group 0 write elements v*64 + t*4 ..
    if (n == 0) {
        if (g == 0) {
#pragma unroll
            for (int v = 0; v < NV; ++v) *(hvec4 *)(o + v * 64) = hvec4{0, 0, 0, 0};
        }
        return;
    }
    const int64_t rec0 = (int64_t)item0[b] * H + h;   // chunk c of this (b,h) is record rec0 + c*H
    float M = kNegBig;
    for (int c0 = 0; c0 < n; c0 += 64) {
        const int c = c0 + lane;
        if (c < n) M = fmaxf(M, part_ml[(rec0 + (int64_t)c * H) * 2]);
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
            w = fast_exp2(part_ml[rec * 2] - M);
            L += w * part_ml[rec * 2 + 1];
        }
        const int nb = min(64, n - c0);
        const fvec4 *pa = (const fvec4 *)(part_acc + (rec0 + (int64_t)c0 * H) * D) + t;
        for (int j0 = 0; j0 < nb; j0 += 16) {
            fvec4 x[4][NV];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int j = min(j0 + u * 4 + g, nb - 1);   // past the end: a valid record, weight 0
#pragma unroll
                for (int v = 0; v < NV; ++v) x[u][v] = pa[j * step + v * 16];
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
    if (g == 0) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            hvec4 r;
#pragma unroll
            for (int i = 0; i < 4; ++i) r[i] = (_Float16)(acc[v][i] / L);
            *(hvec4 *)(o + v * 64) = r;
        }
    }
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

// tokens per workgroup block of the streaming kernel = chunk granule of the planner
int block_tokens(int d) { return kWaves * kTileLoads * (d == 128 ? 4 : 8); }
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
                       (uint4 *)desc->k_base, (uint4 *)desc->v_base, desc->seq_off, desc->seq_cap,
                       desc->seq_lens, desc->status, (const uint4 *)k_new, (const uint4 *)v_new,
                       desc->H, desc->d, desc->seq_seen, desc->n_sink);
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
    char *ws = (char *)workspace;
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(kPlanThreads), 0, (hipStream_t)stream,
                       desc->seq_lens, desc->seq_cap, desc->status, desc->B, desc->H,
                       desc->chunk_tokens, chunk_granule(desc->d), grid, 2 * grid, kShortSeq, 0, 0,
                       16 /* split */, plan_kind(desc->d, 16),
                       (int)w.max_items, (int32_t *)ws,
                       (int32_t *)(ws + w.off_item0), (int32_t *)(ws + w.off_nchunk),
                       (int4 *)(ws + w.off_items), (int32_t *)(ws + w.off_order));
    return launched();
}

int fd_rpart_partial(const fd_kv_desc *desc, const void *q, void *out,
                     void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_desc(desc);
    if (rc != FD_OK) return rc;
    if (desc->B == 0) return FD_OK;
    if (!q || !out || !aligned(q, 16) || !aligned(out, 16)) return FD_EINVAL;
    WsLayout w;
    rc = check_ws(desc, workspace, workspace_bytes, &w);
    if (rc != FD_OK) return rc;
    const int grid = persistent_grid();
    if (grid <= 0) return FD_EHIP;
    char *ws = (char *)workspace;
    // scores are kept in the base-2 exponent domain: exp(x) = 2^(x * log2 e)
    const float qscale = (float)(1.4426950408889634 / (desc->d == 128 ? 11.313708498984761 : 8.0));
    if (desc->d == 128)
        hipLaunchKernelGGL((rpart_partial_kernel<128, kTileLoads>), dim3(2 * grid), dim3(kThreads), 0,
                           (hipStream_t)stream, (const char *)desc->k_base,
                           (const char *)desc->v_base, desc->seq_off, desc->seq_cap,
                           (const _Float16 *)q, (_Float16 *)out, desc->H, (const int32_t *)ws,
                           (const int4 *)(ws + w.off_items), (const int32_t *)(ws + w.off_order),
                           (float *)(ws + w.off_acc), (float *)(ws + w.off_ml), qscale, desc->B,
                           (int)w.max_items, desc->status);
    else
        hipLaunchKernelGGL((rpart_partial_kernel<64, kTileLoads>), dim3(2 * grid), dim3(kThreads), 0,
                           (hipStream_t)stream, (const char *)desc->k_base,
                           (const char *)desc->v_base, desc->seq_off, desc->seq_cap,
                           (const _Float16 *)q, (_Float16 *)out, desc->H, (const int32_t *)ws,
                           (const int4 *)(ws + w.off_items), (const int32_t *)(ws + w.off_order),
                           (float *)(ws + w.off_acc), (float *)(ws + w.off_ml), qscale, desc->B,
                           (int)w.max_items, desc->status);
    return launched();
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
    char *ws = (char *)workspace;
    const int64_t bh = (int64_t)desc->B * desc->H;
    const dim3 grid((unsigned)((bh + 3) / 4));
    if (desc->d == 128)
        hipLaunchKernelGGL(rpart_merge_kernel<128>, grid, dim3(256), 0, (hipStream_t)stream,
                           (const int32_t *)(ws + w.off_item0), (const int32_t *)(ws + w.off_nchunk),
                           (const float *)(ws + w.off_acc), (const float *)(ws + w.off_ml),
                           (_Float16 *)out, desc->B, desc->H, (const int32_t *)ws,
                           plan_kind(128, 16), (int)w.max_items, desc->status);
    else
        hipLaunchKernelGGL(rpart_merge_kernel<64>, grid, dim3(256), 0, (hipStream_t)stream,
                           (const int32_t *)(ws + w.off_item0), (const int32_t *)(ws + w.off_nchunk),
                           (const float *)(ws + w.off_acc), (const float *)(ws + w.off_ml),
                           (_Float16 *)out, desc->B, desc->H, (const int32_t *)ws,
                           plan_kind(64, 16), (int)w.max_items, desc->status);
    return launched();
}

int fd_rpart_decode(const fd_kv_desc *desc, const void *q, void *out,
                    void *workspace, size_t workspace_bytes, void *stream)
{
    // validate everything before the first launch so that a failing call enqueues nothing
    int rc = check_desc(desc);
    if (rc != FD_OK) return rc;
    if (desc->B == 0) return FD_OK;
    if (!q || !out || !aligned(q, 16) || !aligned(out, 16)) return FD_EINVAL;
    WsLayout w;
    rc = check_ws(desc, workspace, workspace_bytes, &w);
    if (rc != FD_OK) return rc;
    rc = fd_rpart_plan(desc, workspace, workspace_bytes, stream);
    if (rc != FD_OK) return rc;
    rc = fd_rpart_partial(desc, q, out, workspace, workspace_bytes, stream);
    if (rc != FD_OK) return rc;
    return fd_rpart_merge(desc, out, workspace, workspace_bytes, stream);
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
    // nothing in the array has to start at zero: the planner rewrites the header and every
    // table entry the other kernels read, and chunk states are written before they are merged
    return fd_rpart_decode(desc, q, out, ws, FD_NOALLOC_SCRATCH_BYTES, stream);
}

int fd_rpart_step(const fd_kv_desc *desc, const void *q, const void *k_new, const void *v_new,
                  void *out, void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_desc(desc);
    if (rc != FD_OK) return rc;
    if (desc->B == 0) return FD_OK;
    if (!q || !out || !k_new || !v_new || !aligned(q, 16) || !aligned(out, 16) ||
        !aligned(k_new, 16) || !aligned(v_new, 16))
        return FD_EINVAL;
    WsLayout w;
    rc = check_ws(desc, workspace, workspace_bytes, &w);
    if (rc != FD_OK) return rc;
    rc = fd_kv_append(desc, k_new, v_new, stream);
    if (rc != FD_OK) return rc;
    return fd_rpart_decode(desc, q, out, workspace, workspace_bytes, stream);
}

int fd_rpart_layer_step(const fd_kv_desc *layer, const void *q, const void *k_new,
                        const void *v_new, void *out, void *workspace, size_t workspace_bytes,
                        int replan, void *stream)
{
    int rc = check_desc(layer);
    if (rc != FD_OK) return rc;
    if (layer->B == 0) return FD_OK;
    if (!q || !out || !k_new || !v_new || !aligned(q, 16) || !aligned(out, 16) ||
        !aligned(k_new, 16) || !aligned(v_new, 16))
        return FD_EINVAL;
    WsLayout w;
    rc = check_ws(layer, workspace, workspace_bytes, &w);
    if (rc != FD_OK) return rc;
    rc = fd_kv_append(layer, k_new, v_new, stream);
    if (rc != FD_OK) return rc;
    if (replan) {
        rc = fd_rpart_plan(layer, workspace, workspace_bytes, stream);
        if (rc != FD_OK) return rc;
    }
    rc = fd_rpart_partial(layer, q, out, workspace, workspace_bytes, stream);
    if (rc != FD_OK) return rc;
    return fd_rpart_merge(layer, out, workspace, workspace_bytes, stream);
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

/*
 * fastdecode_rpart.h -- C ABI of the MI355X (gfx950) R-Part library.
 *
 * The R-Part is the per-sequence, parameter-free part of a decoder block in
 * FastDecode (arXiv 2403.11421, Section 3.1): Eq. 2 (scores of the new token's
 * query against every cached key, normalised by softmax) and Eq. 3 (weighted
 * sum of the cached values).  Section 4.1 states the worker's contract that
 * this ABI mirrors: receive Q_i, K_i, V_i for a batch of sequences, append
 * K_i, V_i to each sequence's KV-cache, attend Q_i over the local cache,
 * return O_i, and drop a sequence's cache when its generation ends.
 *
 * Conventions
 *   - Every pointer marked "device" is HBM memory of the current HIP device,
 *     owned by the caller; the library allocates nothing and frees nothing.
 *   - Every call only enqueues work on `stream` (a hipStream_t passed as
 *     void*; NULL = the default stream) and returns without synchronising,
 *     unless stated otherwise.
 *   - fp16 means IEEE 754 binary16; arithmetic is fp32 (Section 5.1: 16-bit
 *     storage widened in registers).  `out` is rounded to nearest-even fp16.
 *   - Return value: FD_OK or a negative FD_E* code.  Errors that the host can
 *     see (null / misaligned pointers, bad shapes, workspace too small) are
 *     returned before anything is enqueued.  Errors only the device can see
 *     are OR-ed into the sticky word `*desc->status` (FD_ST_* bits).
 *   - Calls that share a descriptor, a workspace or output buffers must be
 *     ordered by the caller (same stream, or events).
 */
#ifndef FASTDECODE_RPART_H
#define FASTDECODE_RPART_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FD_OK          0
#define FD_EINVAL     (-1)  /* null/misaligned pointer, B<0, H<=0, d not in {64,128}, bad chunk_tokens */
#define FD_EWORKSPACE (-2)  /* workspace smaller than fd_workspace_bytes(B,H,d,0)               */
#define FD_EHIP       (-3)  /* a HIP runtime call or kernel launch failed                        */
#define FD_ETOOBIG    (-4)  /* fd_rpart_decode_noalloc: the batch needs more than the built-in scratch */

#define FD_ST_CAPACITY 1    /* append skipped for a sequence whose cache is full                 */
#define FD_ST_BADLEN   2    /* a seq_lens entry was outside [0, seq_cap]; it was clamped         */
#define FD_ST_WINDOW   4    /* windowed cache: n_sink leaves no window row, or seq_seen and
                               seq_lens of a sequence disagree; its append was skipped           */

#define FD_ST_PLAN     8    /* partial/merge found no plan for this batch shape, cache format,
                               launch and workspace size in the workspace (plan missing, or
                               made for another kind of descriptor); they wrote nothing       */

#define FD_SLOT_FREE  (-1)  /* value of seq_lens[b] for a slot that holds no sequence            */

/*
 * KV-cache of one layer for B sequences (the paper prescribes no layout; this
 * one makes every (sequence, head) stream a contiguous run of d*2-byte rows).
 *
 * Element i of the K row of sequence b, head h, token t is the fp16 at
 *     k_base[ seq_off[b] + ((int64)h * seq_cap[b] + t) * d + i ]
 * and likewise for V with v_base.  seq_off[b] must be a multiple of 8 elements
 * (rows are read with 128-bit loads); blocks must not overlap.
 */
typedef struct fd_kv_desc {
    void          *k_base;        /* device, fp16 slab holding every sequence's K block         */
    void          *v_base;        /* device, fp16 slab holding every sequence's V block         */
    const int64_t *seq_off;       /* device int64[B]: element offset of sequence b's block      */
    const int32_t *seq_cap;       /* device int32[B]: capacity of sequence b in tokens          */
    int32_t       *seq_lens;      /* device int32[B]: cached tokens; written by append / reset  */
    int32_t       *status;        /* device int32[1]: sticky FD_ST_* bits; caller zeroes it     */
    int32_t        B;             /* sequences                                                   */
    int32_t        H;             /* attention heads (multi-head: one K/V head per query head)  */
    int32_t        d;             /* head dimension, 64 or 128                                   */
    int32_t        chunk_tokens;  /* split-K chunk length in tokens; 0 = chosen on the device   */
    int32_t       *seq_seen;      /* device int32[B] or NULL: see "windowed cache" below        */
    int32_t        n_sink;        /* windowed cache: leading tokens that are never replaced     */
} fd_kv_desc;

/*
 * Free slots.  seq_lens[b] == FD_SLOT_FREE marks a slot without a sequence
 * (Section 4.1: the cache of a sequence is dropped when its generation ends, and
 * the slot's block is reused by a later sequence without reallocation): append
 * leaves it alone, decode treats it as empty (out[b] = 0).  fd_kv_release frees
 * slots, fd_kv_reset starts a new sequence (length 0) in them.
 *
 * Windowed cache (window attention with sink tokens: the variation of attention
 * that the paper's Related Work names as reducing the tokens a new token interacts
 * with).  With seq_seen != NULL, sequence b attends to its first n_sink tokens and to
 * its last seq_cap[b] - n_sink tokens only, and its block is a bounded buffer:
 * seq_seen[b] counts the tokens appended so far; token p is stored in row p while
 * p < seq_cap[b], afterwards in row n_sink + (p - n_sink) mod (seq_cap[b] - n_sink),
 * replacing the oldest token that is not a sink; seq_lens[b] = min(seq_seen[b],
 * seq_cap[b]).  Attention does not depend on the order of the rows, so the decode
 * entry points need nothing else.  Requires n_sink < seq_cap[b].
 */

/* Library version (major*10000 + minor*100 + patch). */
int fd_version(void);

/* sizeof(fd_kv_desc) (which = 0) or sizeof(fd_kvq_desc) (which = 1, declared below) as this
 * library was built: lets a foreign-language binding check its mirror of the struct. */
size_t fd_desc_size(int which);

/* Static text for an FD_* return code. */
const char *fd_strerror(int code);

/*
 * Bytes of workspace that fd_rpart_decode needs so that it can split contexts
 * into chunks of about 256 tokens when at most `max_total_tokens` tokens are
 * cached over all B sequences.  Any size >= fd_workspace_bytes(B,H,d,0) works:
 * with less room the planner uses longer chunks.  Returns 0 on bad arguments.
 */
size_t fd_workspace_bytes(int32_t B, int32_t H, int32_t d, int64_t max_total_tokens);

/*
 * Append (Section 4.1): for every b, copy the d*H fp16 of k_new[b] and v_new[b]
 * bit-for-bit into row seq_lens[b] of the sequence's K and V blocks, then
 * seq_lens[b] += 1.  A sequence with seq_lens[b] >= seq_cap[b] is left
 * untouched and FD_ST_CAPACITY is set in *desc->status.  Free slots are skipped.
 * With a windowed cache the row is the one described above, seq_seen[b] += 1 and
 * the length saturates at seq_cap[b]; there is no capacity error.
 *   k_new, v_new: device fp16 [B][H][d], 16-byte aligned.
 */
int fd_kv_append(const fd_kv_desc *desc, const void *k_new, const void *v_new, void *stream);

/*
 * Decode attention (Eq. 2 + Eq. 3) for one new token per sequence:
 *   out[b,h,:] = sum_t softmax_t( q[b,h,:] . K[b,h,t,:] / sqrt(d) ) * V[b,h,t,:]
 * over t in [0, seq_lens[b]) as seq_lens stands when the kernels run (so it
 * includes a token appended earlier on the same stream).  seq_lens[b] == 0
 * gives out[b,:,:] = 0.
 *   q:   device fp16 [B][H][d], 16-byte aligned.
 *   out: device fp16 [B][H][d], 16-byte aligned.
 *   workspace: device, 256-byte aligned, workspace_bytes long; contents are
 *     scratch (plan tables and split-K partial states) and need no initialisation.
 * Two launches: fd_rpart_plan, then fd_rpart_partial.
 */
int fd_rpart_decode(const fd_kv_desc *desc, const void *q, void *out,
                    void *workspace, size_t workspace_bytes, void *stream);

/*
 * The stages of fd_rpart_decode, exposed so that a harness can time them
 * separately.  They must be enqueued in this order on one stream with the same
 * descriptor and workspace.  partial and merge check that the workspace holds a plan
 * made for the same B, H, head dimension, cache format and workspace size and for no more
 * workgroups than they are launched with; otherwise they set FD_ST_PLAN and write nothing.
 * Token ranges from the plan are clamped to this descriptor's seq_cap, so a plan made from
 * other lengths gives wrong results but no access outside a sequence's block.
 *   plan:    reads seq_lens on the device, cuts every sequence into chunks and
 *            writes the work-item table into the workspace.
 *   partial: the whole attention.  Streams each chunk's K and V rows once; per (b,h,chunk)
 *            produces the running max, the sum of exponentials and the unnormalised weighted
 *            value sum.  A sequence of one chunk is normalised and written to `out` at once.
 *            For a split sequence the chunk states go to the workspace, and the wave that
 *            finishes the last chunk of a (sequence, head) merges them (log-sum-exp merge,
 *            normalisation, rounding to fp16) in chunk order: the result does not depend on
 *            which wave that is, and no merge launch is needed.  Empty sequences get zeros.
 *   merge:   optional.  Recomputes `out` of every split sequence from the chunk states left in
 *            the workspace (the same arithmetic in the same order: the same bits) and writes
 *            zeros for empty sequences.  The decode and step entry points do not launch it.
 */
int fd_rpart_plan(const fd_kv_desc *desc, void *workspace, size_t workspace_bytes, void *stream);
int fd_rpart_partial(const fd_kv_desc *desc, const void *q, void *out,
                     void *workspace, size_t workspace_bytes, void *stream);
int fd_rpart_merge(const fd_kv_desc *desc, void *out,
                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * fd_kv_append and fd_rpart_plan in ONE launch (the front half of a step): workgroup 0 plans
 * the decode for the lengths the sequences have after the append, which it derives from the old
 * lengths by the append's own rule, while the other workgroups append.  seq_lens (and seq_seen)
 * are NOT updated by this launch: the new values are kept in the workspace and stored by the
 * next fd_rpart_partial on this workspace, so fd_rpart_partial must follow on the same stream
 * before anything else reads seq_lens.  Errors are reported as by fd_kv_append.
 */
int fd_kv_append_plan(const fd_kv_desc *desc, const void *k_new, const void *v_new,
                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * fd_rpart_decode for callers that cannot allocate device memory or hand over a workspace:
 * code running under HIP graph capture, tight serving loops, harnesses that forbid
 * allocation.  Same inputs, outputs, semantics and kernels as fd_rpart_decode, but the plan
 * tables and split-K chunk states live in an array of FD_NOALLOC_SCRATCH_BYTES that is part
 * of the library's device code (every GPU the library runs on holds its own copy until the
 * process ends).  The call allocates and frees nothing.
 *   - Returns FD_ETOOBIG, before anything is enqueued, when the array cannot hold the tables
 *     and one chunk state per sequence, i.e. when fd_workspace_bytes(B, H, d, 0) exceeds
 *     FD_NOALLOC_SCRATCH_BYTES (B * H * (d + 2) * 4 bytes, roughly: B * H <= 129 000 at
 *     d = 128).  With less room than fd_workspace_bytes(B, H, d, tokens) the planner uses
 *     longer chunks, as for any small workspace.
 *   - All calls on one GPU share that GPU's array: calls that may overlap on one GPU (two
 *     streams, two threads) race and must be ordered by the caller.  The array keeps the
 *     previous call's contents; nothing in it needs clearing between calls.
 *   - The first call on a device looks the array's address up (a host-side query, no stream
 *     work); make it once before starting a graph capture.
 */
#define FD_NOALLOC_SCRATCH_BYTES (64u << 20)
int fd_rpart_decode_noalloc(const fd_kv_desc *desc, const void *q, void *out, void *stream);

/* One R-worker step of Section 4.1: append, then attend.  Two launches: fd_kv_append_plan, then
 * fd_rpart_partial.  Same results as fd_kv_append followed by fd_rpart_decode. */
int fd_rpart_step(const fd_kv_desc *desc, const void *q, const void *k_new, const void *v_new,
                  void *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Drop cached sequences (Section 4.1: a worker may drop a sequence's cache when
 * its generation ends): seq_lens[seq_ids[j]] = 0 (and seq_seen, if present) for
 * j < n, i.e. the slot now holds a new, empty sequence.  seq_ids is a device
 * int32[n]; NULL means all B sequences (n is then ignored).  Ids outside [0,B)
 * are ignored.  The cache rows themselves are not cleared.
 * fd_kv_release does the same but marks the slots FD_SLOT_FREE.
 */
int fd_kv_reset(const fd_kv_desc *desc, const int32_t *seq_ids, int32_t n, void *stream);
int fd_kv_release(const fd_kv_desc *desc, const int32_t *seq_ids, int32_t n, void *stream);

/*
 * Bulk store (prompt ingestion; Section 4.1: the worker's cache holds every token of the
 * sequence, the prompt's included): rows t0 .. t0+n-1 of sequence b receive the n token rows
 * given as device fp16 [H][n][d] (16-byte aligned), K from k_rows, V from v_rows; either may
 * be NULL and that side is then left alone.  fp16 caches copy the rows bit for bit; quantised
 * caches quantise every row exactly as fd_kvq_append does.  Rows are raw row indices (in a
 * windowed cache, positions in the bounded buffer).  With set_len non-zero seq_lens[b] (and
 * seq_seen[b], if present) becomes t0 + n, otherwise lengths are untouched and rows beyond
 * seq_lens[b] stay invisible to decode.  If t0 + n exceeds seq_cap[b] nothing is written and
 * FD_ST_CAPACITY is raised.  FD_EINVAL for b outside [0, B) or negative t0, n.
 */
int fd_kv_store_rows(const fd_kv_desc *desc, int32_t b, int32_t t0, int32_t n, const void *k_rows,
                     const void *v_rows, int set_len, void *stream);

/*
 * Device status (errors only the device can see are OR-ed into the sticky word *desc->status).
 * Both calls SYNCHRONISE `stream`.
 *   fd_last_device_status  takes the word: *host_out receives the FD_ST_* bits raised since the
 *       previous take and the device word is cleared in the same atomic step, so a bit raised by
 *       a kernel that runs meanwhile is never lost.  `workspace` (device, 256-byte aligned, any
 *       workspace of this library or 256 bytes of its own) lends one header word as the staging
 *       slot; plan tables in it are untouched.  Section 4.1's worker reports per step whether
 *       its appends took place; this is that report.
 *   fd_read_status  copies the word without a workspace; with `clear` non-zero the bits it
 *       reported (only those) are cleared afterwards.
 * For a quantised cache pass an fd_kv_desc whose `status` field is the quantised descriptor's.
 */
int fd_last_device_status(const fd_kv_desc *desc, void *workspace, int32_t *host_out, void *stream);
int fd_read_status(const fd_kv_desc *desc, int32_t *host_status, int clear, void *stream);

/*
 * Copy what the last fd_rpart_plan on this workspace decided to the host:
 * info[0] = work items (sequence chunks), info[1] = chunk length in tokens,
 * info[2] = total cached tokens, info[3] = workgroups that take part in the streaming
 * kernel (a multiple of the compute units; larger when more than a tenth of the cached
 * tokens sits in sequences shorter than 384 tokens).
 * SYNCHRONISES `stream`.
 */
int fd_plan_info(const void *workspace, int32_t info[4], void *stream);

/* ------------------------------------------------------------------------- */
/* Quantised KV-cache (Section 5.2: K_i and V_i are added to the cache after      */
/* quantisation; fewer bytes to stream make the memory-bound R-Part faster).      */
/* ------------------------------------------------------------------------- */

/*
 * Quantised KV-cache of one layer, 8 or 4 bits per element.  The paper leaves the
 * quantiser to the user; the ones implemented keep one set of parameters per token
 * and head and are evaluated in IEEE binary32 so that the stored bytes are
 * reproducible:
 *   bits = 8 (or 0): symmetric.  scale = max_i |x_i| / 127, code_i = rint(x_i / scale)
 *       (ties to even), the byte stored is code_i + 128; value = (byte - 128) * scale;
 *       an all-zero row gets scale 0 and bytes 128.  One float per row in k_scale.
 *   bits = 4: asymmetric.  zero = min_i x_i, scale = (max_i x_i - zero) / 15,
 *       code_i = rint((x_i - zero) / scale) in 0..15, element 2j in the low nibble of
 *       byte j, element 2j+1 in the high one; value = code * scale + zero; a constant
 *       row gets scale 0 and codes 0.  Two floats (scale, zero) per row in k_scale.
 * The query needs no transformation for these schemes.  d is 128 or 64.
 *
 * With rb = d * bits / 8 bytes of codes per row, the K row of sequence b, head h, token t is
 * row r = h * rows_b + t of the sequence's block, where rows_b = seq_cap[b] (8 bit) or
 * seq_cap[b] rounded up to even (4 bit).  Byte i of that row is
 *     8 bit:  k_codes[ seq_off[b] + r * rb + i ]
 *     4 bit:  k_codes[ seq_off[b] + (r / 2) * 2 rb + (i / 8) * 16 + (r % 2) * 8 + i % 8 ]
 * (4-bit rows lie in pairs whose 8-byte pieces alternate, so that one 16-byte load brings the
 * same 16 elements of two consecutive tokens), and its parameters start at float index
 *     (seq_off[b] / rb + r) * (bits == 4 ? 2 : 1)   of k_scale;
 * likewise for V.  A block holds H * rows_b rows; seq_off[b] must be a multiple of 128 bytes;
 * blocks must not overlap.  k_scale and v_scale must be 8-byte aligned.
 */
typedef struct fd_kvq_desc {
    void          *k_codes;       /* device, byte slab of K codes                               */
    void          *v_codes;       /* device, byte slab of V codes                               */
    float         *k_scale;       /* device, float32 slab of K row parameters (see above)       */
    float         *v_scale;       /* device, float32 slab of V row parameters                   */
    const int64_t *seq_off;       /* device int64[B]: byte offset of sequence b's code block    */
    const int32_t *seq_cap;       /* device int32[B]: capacity of sequence b in tokens          */
    int32_t       *seq_lens;      /* device int32[B]: cached tokens; written by append / reset  */
    int32_t       *status;        /* device int32[1]: sticky FD_ST_* bits; caller zeroes it     */
    int32_t        B, H, d;       /* sequences, heads, head dimension (128 or 64)               */
    int32_t        chunk_tokens;  /* split-K chunk length in tokens; 0 = chosen on the device   */
    int32_t       *seq_seen;      /* device int32[B] or NULL: windowed cache, as in fd_kv_desc  */
    int32_t        n_sink;        /* windowed cache: leading tokens that are never replaced     */
    int32_t        bits;          /* 8 (or 0) or 4                                              */
} fd_kvq_desc;

/*
 * Same contracts as the fp16 entry points of the same names without the "q":
 * fd_kvq_append quantises k_new[b], v_new[b] (device fp16 [B][H][d]) into row
 * seq_lens[b] and bumps the length (FD_ST_CAPACITY when full); fd_rpartq_decode is
 * Eq. 2 + Eq. 3 over the dequantised rows with fp32 arithmetic and an fp16 result; workspace
 * size comes from fd_workspace_bytes(B, H, d, n).
 */
int fd_kvq_append(const fd_kvq_desc *desc, const void *k_new, const void *v_new, void *stream);
int fd_kvq_append_plan(const fd_kvq_desc *desc, const void *k_new, const void *v_new,
                       void *workspace, size_t workspace_bytes, void *stream);
int fd_kvq_store_rows(const fd_kvq_desc *desc, int32_t b, int32_t t0, int32_t n, const void *k_rows,
                      const void *v_rows, int set_len, void *stream);
int fd_kvq_reset(const fd_kvq_desc *desc, const int32_t *seq_ids, int32_t n, void *stream);
int fd_kvq_release(const fd_kvq_desc *desc, const int32_t *seq_ids, int32_t n, void *stream);
int fd_rpartq_plan(const fd_kvq_desc *desc, void *workspace, size_t workspace_bytes, void *stream);
int fd_rpartq_partial(const fd_kvq_desc *desc, const void *q, void *out,
                      void *workspace, size_t workspace_bytes, void *stream);
int fd_rpartq_merge(const fd_kvq_desc *desc, void *out,
                    void *workspace, size_t workspace_bytes, void *stream);
int fd_rpartq_decode(const fd_kvq_desc *desc, const void *q, void *out,
                     void *workspace, size_t workspace_bytes, void *stream);
int fd_rpartq_step(const fd_kvq_desc *desc, const void *q, const void *k_new, const void *v_new,
                   void *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * One transformer block's share of a token step (Section 4.1: for every block the R-worker
 * receives Q_i, K_i, V_i of a mini-batch, appends, attends and returns O_i; Section 5.3: the
 * caches of different blocks are independent).  All blocks of one mini-batch hold the same
 * sequences at the same lengths, so the ragged plan is the same for each of them:
 *   replan != 0  append, plan from this layer's lengths, attend      (first block of a step)
 *   replan == 0  append, attend with the plan already in `workspace` (the other blocks)
 * `layer` describes this block's cache; every block of the mini-batch must use the same B, H,
 * d, chunk_tokens, seq_cap values and seq_off values, its own seq_lens array holding the
 * same lengths as the block that planned, and the same workspace.  If the lengths differ the
 * result is wrong but every access stays inside the block's slabs.  Two mini-batches with their
 * own workspaces may run on two streams at once (the token-level pipeline of Section 4.1).
 * The int8 variant has the same contract.
 */
int fd_rpart_layer_step(const fd_kv_desc *layer, const void *q, const void *k_new,
                        const void *v_new, void *out, void *workspace, size_t workspace_bytes,
                        int replan, void *stream);
int fd_rpartq_layer_step(const fd_kvq_desc *layer, const void *q, const void *k_new,
                         const void *v_new, void *out, void *workspace, size_t workspace_bytes,
                         int replan, void *stream);

/*
 * Measurement aid, not part of the R-Part: enqueue a kernel that only reads
 * `buf` (device, 16-byte aligned) with the same 128-bit streaming loads as the
 * attention kernel, so a harness can time the device's pure-read ceiling next to
 * it.  *bytes_read (host) receives the number of bytes the kernel reads, a
 * multiple of 32 KiB per workgroup not above `bytes`.  `sink` is a device int32
 * the kernel may write.  FD_EINVAL if `bytes` is too small for one pass.
 */
int fd_hbm_read_probe(const void *buf, size_t bytes, int32_t *sink, size_t *bytes_read, void *stream);

/*
 * Measurement aid, not part of the R-Part: fill `buf` (device, 4-byte aligned, `bytes` a
 * multiple of 4) with a seeded bit pattern whose 16-bit halves are finite fp16 values of
 * magnitude 0.25 .. 1 (and whose 32-bit words are finite floats), so that a harness can give a
 * cache contents without running any kernel of its own: counter-collection runs of the
 * profiler have crashed inside the tensor framework's kernel dispatches, and HBM traffic does
 * not depend on the values.
 */
int fd_fill_pattern(void *buf, size_t bytes, uint32_t seed, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FASTDECODE_RPART_H */

// Quantised KV-cache path of the R-Part (FastDecode Section 5.2: K_i and V_i are added to the
// cache after quantisation, which divides the bytes the memory-bound attention has to stream;
// with 4-bit integers the memory access size is a quarter of fp16's).
// Included at the end of fd_rpart.hip: it reuses that file's planner, merge kernel, schedule
// and helpers; only the cache format, the append and the streaming kernel differ.
//
// Formats (the paper leaves the quantiser to the user), one set of parameters per token and
// head, everything evaluated in IEEE binary32 so that the stored bytes are reproducible:
//   8 bit: symmetric.  scale = max|x| / 127, code = rint(x / scale), byte = code + 128;
//          value = (byte - 128) * scale.  A row of d values: d bytes + a 4 B scale.
//   4 bit: asymmetric. zero = min x, scale = (max x - min x) / 15,
//          code = rint((x - zero) / scale) in 0..15, element 2j in the low nibble of byte j;
//          value = code * scale + zero.  A row: 64 B + an 8 B (scale, zero) pair.
// The query needs no transformation for these schemes and stays fp16.

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

template <int CTRL>
__device__ inline float dpp_xmax(float x)
{
    const int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true);
    return fmaxf(x, __int_as_float(y));
}

template <int CTRL>
__device__ inline float dpp_xmin(float x)
{
    const int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true);
    return fminf(x, __int_as_float(y));
}

// geometry of a quantised row of D elements (D = 128 or 64)
template <int BITS, int D_>
struct QFmt {
    static_assert(BITS == 8 || BITS == 4, "8- or 4-bit codes");
    static_assert(D_ == 128 || D_ == 64, "head dimension 128 or 64");
    static constexpr int D = D_;
    static constexpr int RB = D * BITS / 8;              // bytes of codes per row
    static constexpr int MW = BITS == 8 ? 1 : 2;         // floats of parameters per row
    static constexpr int LPR = D / 16;                   // lanes per row when streaming: 16 elements per lane
    static constexpr int LB = RB / LPR;                  // bytes of a row one lane loads: 16 (8 bit) or 8 (4 bit)
    static constexpr int NW = LB / 4;                    // 32-bit words per lane load
    static constexpr int QL = D / 8;                     // lanes per row when quantising: 8 values per lane
};
template <int BITS> struct CodeVec;
template <> struct CodeVec<8> { typedef u32x4 type; };
template <> struct CodeVec<4> { typedef u32x2 type; };

// ---------------------------------------------------------------------------
// Where a row's codes live.  A sequence's block holds, for each head, head_rows(capacity) rows.
// 8 bit: the rows follow one another.  4 bit: the rows lie in pairs (rows 2p and 2p+1 of a
// head) whose 8-byte pieces alternate: piece c of row 2p at byte 16 c of the pair, piece c of
// row 2p+1 at 16 c + 8.  The streaming kernel then reads both rows' 16 elements with one 16-byte
// load per lane.  A head's rows are padded to an even count so that every head starts a pair;
// the row parameters keep one entry per row, with the same padding.
// ---------------------------------------------------------------------------
template <int BITS> __host__ __device__ inline int head_rows(int cap) { return BITS == 4 ? (cap + 1) & ~1 : cap; }

// byte offset, inside the block, of byte o of row `row` (row counted over the block's heads)
template <int BITS, int D>
__device__ inline int64_t code_byte(int64_t row, int o)
{
    constexpr int RB = QFmt<BITS, D>::RB;
    if (BITS == 8) return row * RB + o;
    return (row >> 1) * (2 * RB) + (o >> 3) * 16 + (int)(row & 1) * 8 + (o & 7);
}

// ---------------------------------------------------------------------------
// Row quantiser.  A row (D fp16) is handled by D / 8 consecutive lanes with 8 values each:
// `sub` is the lane's position among them, f its values, block the first code byte of the
// sequence's block, row the row's index in it, meta the row's parameters.  Every step is a
// correctly rounded binary32 operation, so the stored bytes are those of the definition
// evaluated in IEEE binary32.
// ---------------------------------------------------------------------------
template <int BITS, int D>
__device__ inline void quantize_row_store(const float (&f)[8], int sub, uint8_t *block, int64_t row,
                                          float *meta)
{
    using F = QFmt<BITS, D>;
    uint8_t *dst = block + code_byte<BITS, D>(row, sub * (F::RB / F::QL));   // this lane's 8 codes
    if (BITS == 8) {
        float amax = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(f[i]));
        amax = dpp_xmax<0xB1>(amax);           // max over the 16 (or 8) lanes of the row
        amax = dpp_xmax<0x4E>(amax);
        amax = dpp_xmax<0x141>(amax);
        if (F::QL == 16) amax = dpp_xmax<0x140>(amax);
        const float scale = __fdiv_rn(amax, 127.0f);
        unsigned lo = 0, hi = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float c = scale > 0.f ? rintf(__fdiv_rn(f[i], scale)) : 0.f;
            const unsigned u = (unsigned)((int)c + 128) & 0xFFu;
            if (i < 4) lo |= u << (8 * i);
            else       hi |= u << (8 * (i - 4));
        }
        // non-temporal stores: written through instead of left dirty in this XCD's L2, from which
        // the streaming kernel that follows would have to fetch them across XCDs
        __builtin_nontemporal_store(u32x2{lo, hi}, reinterpret_cast<u32x2 *>(dst));
        if (sub == 0) __builtin_nontemporal_store(scale, meta);
    } else {
        float mn = f[0], mx = f[0];
#pragma unroll
        for (int i = 1; i < 8; ++i) {
            mn = fminf(mn, f[i]);
            mx = fmaxf(mx, f[i]);
        }
        mn = dpp_xmin<0xB1>(mn);  mx = dpp_xmax<0xB1>(mx);
        mn = dpp_xmin<0x4E>(mn);  mx = dpp_xmax<0x4E>(mx);
        mn = dpp_xmin<0x141>(mn); mx = dpp_xmax<0x141>(mx);
        if (F::QL == 16) { mn = dpp_xmin<0x140>(mn); mx = dpp_xmax<0x140>(mx); }
        const float scale = __fdiv_rn(__fsub_rn(mx, mn), 15.0f);
        unsigned w = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float c = scale > 0.f ? rintf(__fdiv_rn(__fsub_rn(f[i], mn), scale)) : 0.f;
            c = fminf(fmaxf(c, 0.f), 15.f);
            w |= (unsigned)(int)c << (4 * i);
        }
        __builtin_nontemporal_store(w, reinterpret_cast<unsigned *>(dst));
        if (sub == 0) __builtin_nontemporal_store(f32x2{scale, mn}, reinterpret_cast<f32x2 *>(meta));
    }
}

__device__ inline void load_row_f32(const _Float16 *src, float (&f)[8])
{
    const half8 x = *reinterpret_cast<const half8 *>(src);
#pragma unroll
    for (int i = 0; i < 8; ++i) f[i] = (float)x[i];
}

// ---------------------------------------------------------------------------
// Quantising append.  One workgroup per sequence, one row per 16 lanes per pass.  `bump` as in
// the fp16 append: without it the lengths take effect later (fused append + plan launch).
// ---------------------------------------------------------------------------
struct QSlabs {
    uint8_t *k_codes, *v_codes;
    float *k_meta, *v_meta;
};

template <int BITS, int D>
__device__ inline void kvq_append_body(const QSlabs &c, const SeqState &st,
                                       const _Float16 *__restrict__ k_new,
                                       const _Float16 *__restrict__ v_new, int H, int b, bool bump)
{
    using F = QFmt<BITS, D>;
    const int cap = st.seq_cap[b];
    int new_len = 0;
    const int L = append_row(st, b, &new_len);
    if (L < 0) return;
    const int sub = threadIdx.x % F::QL;       // position inside the lane group of a row
    const int group = threadIdx.x / F::QL;
    const int groups = blockDim.x / F::QL;
    const int64_t off = st.seq_off[b];
    for (int r = group; r < 2 * H; r += groups) {
        const int which = r >= H;
        const int h = which ? r - H : r;
        float f[8];
        load_row_f32((which ? v_new : k_new) + ((int64_t)b * H + h) * D + sub * 8, f);
        const int64_t row = (int64_t)h * head_rows<BITS>(cap) + L;
        quantize_row_store<BITS, D>(f, sub, (which ? c.v_codes : c.k_codes) + off, row,
                                    (which ? c.v_meta : c.k_meta) + (off / F::RB + row) * F::MW);
    }
    if (bump) {
        __syncthreads();
        if (threadIdx.x == 0) {
            st.seq_lens[b] = new_len;
            if (st.seq_seen) st.seq_seen[b] += 1;
        }
    }
}

template <int BITS, int D>
__global__ __launch_bounds__(256) void kvq_append_kernel(QSlabs c, SeqState st,
                                                         const _Float16 *__restrict__ k_new,
                                                         const _Float16 *__restrict__ v_new, int H)
{
    kvq_append_body<BITS, D>(c, st, k_new, v_new, H, blockIdx.x, true);
}

// front of a step in one launch: workgroup 0 plans for the lengths after the append, the
// others append without touching seq_lens (see kv_append_plan_kernel)
template <int BITS, int D>
__global__ __launch_bounds__(kPlanThreads) void kvq_append_plan_kernel(
    QSlabs c, SeqState st, const _Float16 *__restrict__ k_new, const _Float16 *__restrict__ v_new,
    PlanArgs a)
{
    if (blockIdx.x == 0) plan_body(a);
    else kvq_append_body<BITS, D>(c, st, k_new, v_new, a.H, (int)blockIdx.x - 1, false);
}

// Bulk store of n consecutive token rows of one sequence (prompt ingestion): the same quantiser
// as the append, rows given as fp16 [H][n][D].  grid.x covers the H * n rows, 256 / (D / 8) per
// workgroup.
template <int BITS, int D>
__global__ __launch_bounds__(256) void kvq_store_rows_kernel(
    uint8_t *__restrict__ k_codes, uint8_t *__restrict__ v_codes,
    float *__restrict__ k_meta, float *__restrict__ v_meta,
    const int64_t *__restrict__ seq_off, const int32_t *__restrict__ seq_cap,
    int32_t *__restrict__ seq_lens, int32_t *__restrict__ seq_seen, int32_t *__restrict__ status,
    const _Float16 *__restrict__ k_rows, const _Float16 *__restrict__ v_rows, int H, int b, int t0,
    int n, int set_len)
{
    using F = QFmt<BITS, D>;
    const int cap = seq_cap[b];
    if (t0 + n > cap) {                                      // uniform over the grid: nothing is written
        if (blockIdx.x == 0 && threadIdx.x == 0) atomicOr(status, FD_ST_CAPACITY);
        return;
    }
    const int sub = threadIdx.x % F::QL;
    const int64_t r = (int64_t)blockIdx.x * (256 / F::QL) + threadIdx.x / F::QL;   // row index in [H][n]
    const int64_t off = seq_off[b];
    if (r < (int64_t)H * n) {
        const int h = (int)(r / n), j = (int)(r - (int64_t)h * n);
        const int64_t row = (int64_t)h * head_rows<BITS>(cap) + t0 + j;
        float f[8];
        if (k_rows) {
            load_row_f32(k_rows + r * D + sub * 8, f);
            quantize_row_store<BITS, D>(f, sub, k_codes + off, row, k_meta + (off / F::RB + row) * F::MW);
        }
        if (v_rows) {
            load_row_f32(v_rows + r * D + sub * 8, f);
            quantize_row_store<BITS, D>(f, sub, v_codes + off, row, v_meta + (off / F::RB + row) * F::MW);
        }
    }
    if (set_len && blockIdx.x == 0 && threadIdx.x == 0) {
        seq_lens[b] = t0 + n;
        if (seq_seen) seq_seen[b] = t0 + n;
    }
}

// ---------------------------------------------------------------------------
// Streaming kernel over codes.  A lane always holds 16 elements of a row (16 B of 8-bit or 8 B of
// 4-bit codes), so a row is 8 lanes at d = 128 and 4 lanes at d = 64, and a wave load covers
// RPW = 8 or 16 tokens (1 KB of 8-bit codes; 4-bit rows are read two at a time, see TileQ, so
// that a memory load is 1 KB there too and fills two of the tile's slots); a workgroup block is
// 4 waves x NL slots = 4 NL RPW tokens.  The NL RPW tokens of a wave's tile map onto its first
// NL RPW lanes for the row parameters: each lane loads those of "its" token (the other lanes
// repeat them) and the values are handed to the lanes that need them with a cross-lane read.
//
// Dequantisation is folded into the arithmetic.  With value = u * scale + zero (8 bit: u is
// the stored byte and zero = -128 * scale):
//   q . k   = scale_k * sum_i q_i u_i + zero_k * sum_i q_i
//   sum p v = sum_t (p_t scale_v,t) u_t  +  sum_t p_t zero_v,t   (the same for every element)
// A code sitting in the low bits of a 16-bit half is the fp16 subnormal u * 2^-24, exactly, and
// both v_dot2_f32_f16 and the mixed-precision FMA take fp16 subnormals at full precision (checked
// on the device): the K side costs one mask per two codes and one dot instruction per two
// elements with the query left in fp16, the V side one mixed FMA per element; the 2^24 goes into
// the per-token factors.
// ---------------------------------------------------------------------------
__device__ inline float byte_f32(unsigned w, int i) { return (float)((w >> (8 * i)) & 0xFFu); }

__device__ inline f16x2 as_f16x2(unsigned w)
{
    union { unsigned u; f16x2 h; } x;
    x.u = w;
    return x.h;
}

// bytes 1 and 3 of w as two zero-extended halves, (w >> 8) & 0x00FF00FF, in one instruction
__device__ inline unsigned odd_bytes(unsigned w) { return __builtin_amdgcn_perm(w, w, 0x0C030C01u); }

// Streams are read through buffer descriptors: the base lives in scalar registers (it must be
// the same in every lane), a lane adds a 32-bit byte offset, and advancing the stream is scalar
// arithmetic.  Against 64-bit per-lane pointers this takes the address arithmetic off the vector
// unit and frees ten vector registers: the 4-bit kernel, which is bound by instruction issue,
// gains 1-4 % and no longer spills; the 8-bit kernel is unchanged.  No bounds are set in the
// descriptor (the base moves with the stream, offsets stay below a block): offsets are computed
// exactly as for plain loads.  Word 3 = 0x00020000: untyped 32-bit data, no swizzle.
typedef __amdgpu_buffer_rsrc_t Rsrc;
__device__ inline Rsrc stream_rsrc(const void *ubase)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(ubase), 0, 0x7FFFFFFF, 0x00020000);
}
constexpr int kAuxNt = 2;                                 // non-temporal
template <typename V> __device__ inline V ld_buf(Rsrc r, unsigned voff, int soff);
template <> __device__ inline u32x4 ld_buf<u32x4>(Rsrc r, unsigned voff, int soff)
{
    return __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, kAuxNt);
}
template <> __device__ inline u32x2 ld_buf<u32x2>(Rsrc r, unsigned voff, int soff)
{
    return __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, kAuxNt);
}
// The row parameters are read with the non-temporal hint like the codes.  A wave asks for the
// 32 B (8 bit) or 64 B (4 bit) of its eight tokens per load and the neighbouring waves for the
// rest of the same memory line, so part of the lines is fetched twice (counters: 1.013 x and
// 1.031 x the algorithmic bytes).  Reading them cached removes that and looked 2-11 % faster
// in a loop that repeats one layer's step, but only because the parameters (3-11 % of the
// bytes) then survive in the memory-side cache from one step to the next; with other work
// between the steps (cache lines dirtied by other kernels) the cached variant lost 7-26 %.
// A cache that is streamed once per token of a many-layer model must not count on that.
__device__ inline unsigned ld_meta32(Rsrc r, unsigned voff)
{
    return __builtin_amdgcn_raw_buffer_load_b32(r, voff, 0, kAuxNt);
}
__device__ inline u32x2 ld_meta64(Rsrc r, unsigned voff)
{
    return __builtin_amdgcn_raw_buffer_load_b64(r, voff, 0, kAuxNt);
}

// Tile size and residency, measured on MI355X over the two-block rolling prefetch below (8-bit
// codes): two wave loads per tile and two workgroups per CU (187 VGPRs, two waves per SIMD)
// stream 6.9 TB/s at 2048 tokens per sequence and 6.1 TB/s at 256; eight loads per tile with one
// workgroup per CU (the fp16 kernel's shape) reach 6.2 and 3.3: this kernel has 2.5 x the
// arithmetic per byte, and a second wave per SIMD is what hides it.
// The 4-bit kernel's tile has twice the slots of half the size (two memory loads of row pairs
// per stream), so as many bytes are in flight.
template <int BITS> constexpr int q_tile_loads() { return BITS == 8 ? 2 : 4; }   // slots (wave loads of RPW rows) per tile
// Workgroups per compute unit.  8 bit: two when the sequences are long; the kernel (147 VGPRs)
// fits a third one, which pays on short sequences (+5 % at 256 tokens per sequence, -5 % at
// 2048), so the planner switches it on by the same rule as the fp16 kernel's second one.
// 4 bit: always three (the 168-register budget, no spills).  Its units stream in a quarter of the fp16 kernel's time against the same fixed cost
// per unit, and a third resident workgroup covers more of it: against two, 2049 tokens per
// sequence +4 %, geometric mix +5.5 %, uniform 1..4096 +1.5 %, 256 each +2.4 %; uniform
// 1..1024 -1.5 %, 16 sequences of 32768 -1.3 %, one of 131072 -3 %.
template <int BITS> constexpr int q_wg_long() { return BITS == 8 ? 2 : 3; }
template <int BITS> constexpr int q_wg_short() { return 3; }
constexpr int kQSplit = 4;          // a sequence is cut when longer than 1/4 of a worker's share
// Units per wave instead of per workgroup when the batch holds many short sequences (the
// planner's wave_units argument).  Measured against workgroup units with the best residency:
// 4 bit +30 % at 256 tokens per sequence, +22 % on lengths uniform in 1..1024, but -9 % at 2048
// tokens; 8 bit +3 %, -4 %, -10 %: only the 4-bit kernel, whose unit epilogue is dear against its
// short streaming time, uses it.
template <int BITS> constexpr int q_wave_units() { return BITS == 4 ? 1 : 0; }

// WPU = waves that share a unit: kWaves (the workgroup streams one (sequence, head) together,
// wave w the w-th quarter of every block) or 1 (every wave streams a unit of its own).
template <int BITS, int D_, int NL_, int WPU>
struct TileQ {
    using F = QFmt<BITS, D_>;
    static constexpr int D = F::D;
    static constexpr int NL = NL_;
    static constexpr int RB = F::RB;
    static constexpr int MW = F::MW;
    static constexpr int LB = F::LB;
    static constexpr int NW = F::NW;
    static constexpr int LPR = F::LPR;                   // lanes per row: 8 (D = 128) or 4 (D = 64)
    static constexpr int RPW = 64 / LPR;                 // rows (tokens) per wave load: 8 or 16
    static constexpr int EPL = D / LPR;                  // elements per lane: 16
    // A wave's NL loads of a block are consecutive: it owns NL * RPW consecutive tokens, so the
    // row parameters it needs are one contiguous 64 B (8 bit) or 256 B (4 bit) run and no other
    // wave asks for a part of the same run.  (With the waves interleaved load by load, a wave's
    // parameters came in 32 B / 64 B pieces of memory lines that its neighbours fetched again.)
    //
    // 4-bit rows lie in memory in pairs (see pair_byte): a lane's 16-byte load brings its 8 bytes
    // of an even row and of the odd row after it.  The arithmetic still sees NL "loads" of RPW
    // rows (slot j = half j % 2 of memory load j / 2), so only the loads and the slot -> token
    // map know about pairs.  Against 8-byte loads of plain rows this halves the requests that
    // the vector memory pipeline tracks per byte: its queue was full 43 % of the time and HBM
    // was not (no credit stalls), +4 % at 2048 tokens per sequence, +6 % on the geometric mix.
    static constexpr bool PAIRED = BITS == 4;
    static_assert(!PAIRED || NL % 2 == 0, "4-bit tiles are made of row pairs");
    static constexpr int STRIDE = 64 * LB * (PAIRED ? 2 : 1);   // bytes between a wave's consecutive memory loads
    static constexpr int BLK_TOK = NL * WPU * RPW;       // tokens per workgroup block
    static constexpr int BLK_BYTES = NL * WPU * 64 * LB; // bytes of K (or V) codes per block
    static_assert(NL * RPW <= 64, "one lane per token of the tile for the row parameters");
    typedef typename CodeVec<BITS>::type CV;
    CV k[NL], v[NL];
    float ks, kz, vs, vz;                                // parameters of this lane's own token

    // token (inside a block) whose parameters lane `lane` of wave `wave` loads
    __device__ static inline int own_token(int lane, int wave)
    {
        return first_token(wave) + lane % (NL * RPW);
    }
    // first token (inside a block) of the wave's run, and the byte offset of a lane's part of
    // memory load 0
    __device__ static inline int first_token(int wave) { return wave * NL * RPW; }
    __device__ static inline unsigned lane_offset(int lane, int wave)
    {
        return PAIRED ? (unsigned)((wave * (NL / 2) * 64 + lane) * 16) : (unsigned)((wave * NL * 64 + lane) * LB);
    }
    // token (inside the wave's run) that slot j holds for the lanes of row `row`
    __device__ static inline int slot_token(int j, int row)
    {
        return PAIRED ? 2 * ((j / 2) * RPW + row) + (j & 1) : j * RPW + row;
    }
    // memory loads of the K (or V) codes of one tile into the slots
    __device__ inline void load_codes(CV (&dst)[NL], Rsrc r, unsigned co)
    {
#pragma unroll
        for (int j = 0; j < NL; ++j) load_slot(dst, j, r, co);
    }
    // the load that fills slot j, issued when the arithmetic is done with the slot: for a pair
    // that is after its odd half (the even half's registers are written by the same load)
    __device__ inline void load_slot(CV (&dst)[NL], int j, Rsrc r, unsigned co)
    {
        if constexpr (PAIRED) {
            if (j & 1) {
                const u32x4 t = ld_buf<u32x4>(r, co, (j / 2) * STRIDE);
                dst[j - 1] = CV{t[0], t[1]};
                dst[j] = CV{t[2], t[3]};
            }
        } else {
            dst[j] = ld_buf<CV>(r, co, j * STRIDE);
        }
    }

    // mo4 = byte offset of this lane's token in the parameter stream
    __device__ inline void load_kmeta(const float *base, unsigned mo4)
    {
        const Rsrc r = stream_rsrc(base);
        if (BITS == 8) {
            ks = __uint_as_float(ld_meta32(r, mo4));
        } else {
            const u32x2 t = ld_meta64(r, mo4);
            ks = __uint_as_float(t[0]);
            kz = __uint_as_float(t[1]);
        }
    }
    __device__ inline void load_vmeta(const float *base, unsigned mo4)
    {
        const Rsrc r = stream_rsrc(base);
        if (BITS == 8) {
            vs = __uint_as_float(ld_meta32(r, mo4));
        } else {
            const u32x2 t = ld_meta64(r, mo4);
            vs = __uint_as_float(t[0]);
            vz = __uint_as_float(t[1]);
        }
    }

    // issue order = consumption order (loads return in order): K parameters, K codes,
    // V parameters, V codes
    __device__ inline void load(const char *kb, const char *vb, const float *kmb, const float *vmb,
                                unsigned co, unsigned mo)
    {
        load_kmeta(kmb, mo * 4u);
        load_codes(k, stream_rsrc(kb), co);
        load_vmeta(vmb, mo * 4u);
        load_codes(v, stream_rsrc(vb), co);
    }

    // ragged last block of `rem` >= 1 tokens: lanes whose token is at or beyond `rem` re-read
    // the row (the pair) of token rem-1 (in bounds) and are masked in update<true, ...>.  `row` is
    // the lane's row, wtok the first token of the wave's run, own the token whose parameters the
    // lane loads.  The odd row of the last pair may lie beyond `rem`: it is inside the block
    // (a head's rows are padded to an even count) and masked like the others.
    __device__ inline void load_tail(const char *kb, const char *vb, const float *kmb,
                                     const float *vmb, unsigned co, unsigned mo, int row, int wtok,
                                     int own, int rem)
    {
        const int sback = own > rem - 1 ? own - (rem - 1) : 0;
        const unsigned mt = mo - (unsigned)(sback * MW);           // token min(own, rem-1) >= 0
        load_kmeta(kmb, mt * 4u);
        load_vmeta(vmb, mt * 4u);
        const Rsrc rk = stream_rsrc(kb), rv = stream_rsrc(vb);
        if constexpr (PAIRED) {
#pragma unroll
            for (int jp = 0; jp < NL / 2; ++jp) {
                const int over = (wtok + slot_token(2 * jp, row)) / 2 - (rem - 1) / 2;   // pairs beyond the last one
                const int back = over > 0 ? over * 2 * RB : 0;
                const unsigned ct = co + (unsigned)(jp * STRIDE) - (unsigned)back;
                const u32x4 a = ld_buf<u32x4>(rk, ct, 0), b = ld_buf<u32x4>(rv, ct, 0);
                k[2 * jp] = CV{a[0], a[1]};
                k[2 * jp + 1] = CV{a[2], a[3]};
                v[2 * jp] = CV{b[0], b[1]};
                v[2 * jp + 1] = CV{b[2], b[3]};
            }
        } else {
#pragma unroll
            for (int j = 0; j < NL; ++j) {
                const int over = wtok + slot_token(j, row) - (rem - 1);
                const int back = over > 0 ? over * RB : 0;
                const unsigned ct = co + (unsigned)(j * STRIDE) - (unsigned)back;   // row min(., rem-1) >= 0
                k[j] = ld_buf<CV>(rk, ct, 0);
                v[j] = ld_buf<CV>(rv, ct, 0);
            }
        }
    }

    // 2^-24 * sum_e q[e] * u_e over this lane's 16 elements.  A code in the low bits of a
    // 16-bit half is the fp16 subnormal u * 2^-24, exactly, and v_dot2_f32_f16 takes subnormal
    // inputs at full precision: two codes cost one mask (and shift) and one dot instruction,
    // with the query left in fp16.  qh holds the query pairs in the order the masks produce.
    __device__ static inline float dot_codes(const CV &c, const f16x2 (&qh)[EPL / 2])
    {
        if (BITS == 8) {
            float a = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                a = __builtin_amdgcn_fdot2(as_f16x2(c[w] & 0x00FF00FFu), qh[2 * w], a, false);
                a = __builtin_amdgcn_fdot2(as_f16x2(odd_bytes(c[w])), qh[2 * w + 1], a, false);
            }
            return a;
        } else {
            // a nibble in bits 4..7 of a half is still inside the mantissa field: it reads as
            // 16 u * 2^-24, so the odd nibbles need no shift; their query elements carry the 1/16
            float a = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const unsigned lo = c[w], hi = c[w] >> 8;
                a = __builtin_amdgcn_fdot2(as_f16x2(lo & 0x000F000Fu), qh[4 * w], a, false);
                a = __builtin_amdgcn_fdot2(as_f16x2(lo & 0x00F000F0u), qh[4 * w + 1], a, false);
                a = __builtin_amdgcn_fdot2(as_f16x2(hi & 0x000F000Fu), qh[4 * w + 2], a, false);
                a = __builtin_amdgcn_fdot2(as_f16x2(hi & 0x00F000F0u), qh[4 * w + 3], a, false);
            }
            return a;
        }
    }

    // the query pairs for dot_codes from this lane's 16 query elements
    __device__ static inline void pack_query(const _Float16 (&q)[EPL], f16x2 (&qh)[EPL / 2])
    {
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            if (BITS == 8) {
                qh[2 * w] = f16x2{q[4 * w], q[4 * w + 2]};           // bytes 0 and 2 of word w
                qh[2 * w + 1] = f16x2{q[4 * w + 1], q[4 * w + 3]};   // bytes 1 and 3
            } else {
                // nibble n of a word holds the word's element n; odd nibbles are read as 16 u, so
                // their query elements are divided by 16 here (exact but for elements below
                // 2^-10, whose lost bits are far below the result's precision)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    qh[4 * w + i] = f16x2{q[8 * w + i], q[8 * w + i + 4]};
                    if (i & 1) qh[4 * w + i] *= f16x2{(_Float16)0.0625f, (_Float16)0.0625f};
                }
            }
        }
    }

    // acc[e] += pv24 * 2^-24 * u_e: the same subnormal halves feed a mixed-precision FMA
    // (fp16 operand widened exactly, fp32 weight and accumulator); pv24 carries the 2^24.
    __device__ static inline void axpy_codes(const CV &c, float pv24, float (&acc)[EPL])
    {
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            if (BITS == 8) {
                const f16x2 a = as_f16x2(c[w] & 0x00FF00FFu), b = as_f16x2(odd_bytes(c[w]));
                acc[4 * w] = __builtin_fmaf(pv24, (float)a[0], acc[4 * w]);
                acc[4 * w + 1] = __builtin_fmaf(pv24, (float)b[0], acc[4 * w + 1]);
                acc[4 * w + 2] = __builtin_fmaf(pv24, (float)a[1], acc[4 * w + 2]);
                acc[4 * w + 3] = __builtin_fmaf(pv24, (float)b[1], acc[4 * w + 3]);
            } else {
                // the odd nibbles are read as 16 u: their accumulators run 16 times too high
                // and are put right once per unit (fix_odd)
                const unsigned lo = c[w], hi = c[w] >> 8;
                const f16x2 n04 = as_f16x2(lo & 0x000F000Fu), n15 = as_f16x2(lo & 0x00F000F0u);
                const f16x2 n26 = as_f16x2(hi & 0x000F000Fu), n37 = as_f16x2(hi & 0x00F000F0u);
                acc[8 * w] = __builtin_fmaf(pv24, (float)n04[0], acc[8 * w]);
                acc[8 * w + 1] = __builtin_fmaf(pv24, (float)n15[0], acc[8 * w + 1]);
                acc[8 * w + 2] = __builtin_fmaf(pv24, (float)n26[0], acc[8 * w + 2]);
                acc[8 * w + 3] = __builtin_fmaf(pv24, (float)n37[0], acc[8 * w + 3]);
                acc[8 * w + 4] = __builtin_fmaf(pv24, (float)n04[1], acc[8 * w + 4]);
                acc[8 * w + 5] = __builtin_fmaf(pv24, (float)n15[1], acc[8 * w + 5]);
                acc[8 * w + 6] = __builtin_fmaf(pv24, (float)n26[1], acc[8 * w + 6]);
                acc[8 * w + 7] = __builtin_fmaf(pv24, (float)n37[1], acc[8 * w + 7]);
            }
        }
    }

    // end of a unit: the accumulators of the 4-bit kernel's odd elements (see axpy_codes)
    __device__ static inline void fix_odd(float (&acc)[EPL])
    {
        if (BITS == 4) {
#pragma unroll
            for (int i = 1; i < EPL; i += 2) acc[i] *= 0.0625f;
        }
    }

    // Consume this tile.  With REFILL every register is reloaded with the same slot of the block
    // two ahead (kp2, vp2, kmp2, vmp2) as soon as its last use is issued, so that close to two
    // blocks of loads per wave stay in flight during the arithmetic as well.
    template <bool MASKED, bool REFILL>
    __device__ inline void update(const f16x2 (&qh)[EPL / 2], float kmul, float qs, float &m,
                                  float &l, float &aux, float (&acc)[EPL], int row, int wtok,
                                  int rem, unsigned co = 0, unsigned mo = 0,
                                  const char *kp2 = nullptr, const char *vp2 = nullptr,
                                  const float *kmp2 = nullptr, const float *vmp2 = nullptr)
    {
        // score = kmul * scale * a + qs * zero.  Every lane scales the parameters of its own
        // token once, then hands them to the rows that use them (a lane uses NL tokens): after
        // that the registers are free to refill.  8 bit: zero = -128 scale, so the score is
        // (kmul * scale) * (a + c0).
        const float ksm = ks * kmul;
        const float kzq = BITS == 8 ? 0.f : kz * qs;
        const float c0 = -128.0f * qs / kmul;                    // the same for the whole unit
        float s[NL], z[NL];
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            s[j] = __shfl(ksm, slot_token(j, row));
            z[j] = BITS == 8 ? 0.f : __shfl(kzq, slot_token(j, row));
        }
        if (REFILL) {
            sched_fence();
            load_kmeta(kmp2, mo * 4u);
            sched_fence();
        }
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            float a = dot_codes(k[j], qh);
            if (REFILL) {
                sched_fence();
                load_slot(k, j, stream_rsrc(kp2), co);
                sched_fence();
            }
            a = row_sum<LPR>(a);
            a = BITS == 8 ? (a + c0) * s[j] : __builtin_fmaf(a, s[j], z[j]);
            if (MASKED && wtok + slot_token(j, row) >= rem) a = kNegBig;
            s[j] = a;
        }
        float tm = s[0];
#pragma unroll
        for (int j = 1; j < NL; ++j) tm = fmaxf(tm, s[j]);
        const float mn = fmaxf(m, tm);
        // after the first few tiles a new maximum is rare: the rescaling is skipped when no row
        // of the wave has one (a wave-uniform branch without memory operations)
        if (__any(mn > m)) {
            const float corr = fast_exp2(m - mn);
            l *= corr;
            aux *= corr;
#pragma unroll
            for (int i = 0; i < EPL; ++i) acc[i] *= corr;
        }
        // weights times V scales (with the 2^24 of the subnormal codes, applied by the token's
        // own lane); the weighted zero points go to aux; then the V parameter registers are free
        // as well
        const float vsm = vs * 16777216.0f;
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            float p = fast_exp2(s[j] - mn);
            if (MASKED && wtok + slot_token(j, row) >= rem) p = 0.f;
            l += p;
            const float pv24 = p * __shfl(vsm, slot_token(j, row));
            aux = BITS == 8 ? __builtin_fmaf(pv24, -128.0f / 16777216.0f, aux)
                            : __builtin_fmaf(p, __shfl(vz, slot_token(j, row)), aux);
            s[j] = pv24;
        }
        if (REFILL) {
            sched_fence();
            load_vmeta(vmp2, mo * 4u);
            sched_fence();
        }
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            axpy_codes(v[j], s[j], acc);
            if (REFILL) {
                sched_fence();
                load_slot(v, j, stream_rsrc(vp2), co);
                sched_fence();
            }
        }
        m = mn;
    }
};

// a value that is the same in every lane of the wave, moved to scalar registers
__device__ inline int64_t uniform64(int64_t x)
{
    const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(x & 0xFFFFFFFFll));
    const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)((unsigned long long)x >> 32));
    return (int64_t)(((unsigned long long)hi << 32) | lo);
}

// Everything the streaming kernel over codes is given.
struct PartialQArgs {
    const char *k_codes, *v_codes;
    const float *k_meta, *v_meta;
    const int64_t *seq_off;
    const int32_t *seq_cap;
    int32_t *seq_lens, *seq_seen, *status;
    const _Float16 *q;
    _Float16 *out;
    int B, H;
    float qscale;
    PlanView v;
};

template <int BITS, int D_, int WPU>
__device__ __forceinline__ void rpartq_body(const PartialQArgs &a)
{
    const char *__restrict__ k_codes = a.k_codes;
    const char *__restrict__ v_codes = a.v_codes;
    const float *__restrict__ k_meta = a.k_meta;
    const float *__restrict__ v_meta = a.v_meta;
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
    const float qscale = a.qscale;
    using T = TileQ<BITS, D_, q_tile_loads<BITS>(), WPU>;
    constexpr int D = T::D, LPR = T::LPR, EPL = T::EPL, RB = T::RB, MW = T::MW;
    // two sets, used by alternate units, so that one barrier per unit is enough
    __shared__ float sm_acc2[2][kWaves][D];
    __shared__ float sm_m2[2][kWaves], sm_l2[2][kWaves], sm_aux2[2][kWaves];
    __shared__ int4 sm_split[kWaves][kSplitList];        // chunk states written but not yet published
    int set = 0;

    const int lane = threadIdx.x & 63;
    const int wave_id = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // scalar
    const int wave = WPU == 1 ? 0 : wave_id;                     // position among the unit's waves
    const int tid = wave * 64 + lane;                            // thread index among them
    const int row = lane / LPR;
    const int col = lane % LPR;
    const int own = T::own_token(lane, wave);              // token whose parameters this lane loads
    const int n_units = hdr[HDR_NITEMS] * H;
    // workers (workgroups, or single waves) that the planner's grid amounts to, and this one
    const int W = hdr[HDR_GRID] * (kWaves / WPU);
    const int g = WPU == 1 ? (int)(blockIdx.x * kWaves) + wave_id : (int)blockIdx.x;
    if (g >= W) return;
    int4 *split_list = sm_split[wave_id];
    int n_split = 0;

    // same static schedule as the fp16 kernel
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
                // (4 bit: a chunk starts with a pair, as the planner's chunks do)
                const int t1 = min(it.z, cap), t0 = min(it.y, max(t1 - 1, 0)) & (BITS == 4 ? ~1 : ~0);
                u.h = (int)(p - (long long)sidx * H);
                u.b = it.x;
                u.item = item;
                u.nch = it.w;
                u.ntok = t1 - t0;
                u.row0 = seq_off[it.x] / RB + (int64_t)u.h * head_rows<BITS>(cap) + t0;   // row index
            }
        }
        return u;
    };

    // compute units = workgroups launched / the most that may share one; how many share one now
    const int n_cus = (int)gridDim.x / q_wg_short<BITS>();
    const int wg_per_cu = hdr[HDR_GRID] / n_cus;
    const int wg_slot = (int)blockIdx.x / n_cus;           // dispatch order on this workgroup's CU
    int j = 0;
    Unit cur = fetch(0);
    if (cur.ntok == 0 && n_rounds > 1) cur = fetch(++j);
    // The units are walked in stretches: a stretch ends when the wave has no more units or its list
    // of unpublished chunk states is full; the states are then published (the call sits outside
    // the unit loop, so that it does not constrain the registers of the streaming code).
    for (;;) {
    while (cur.ntok > 0 && n_split < kSplitList) {
        Unit nxt = fetch(++j);
        if (nxt.ntok == 0 && j < n_rounds) nxt = fetch(++j);

        // Workgroups that share a compute unit are not served alike: the one dispatched first wins
        // the issue arbitration (with equal shares it finished 15-25 % ahead of the third).  With
        // three per CU their waves' priorities are rotated from unit to unit, which evens that
        // out in part: +2 to +5 % on the workloads that run three per CU; with two per CU the
        // rotation cost 0.5 % and is left out, and so it is when every wave has units of its own
        // (-0.5 %).
        if (WPU != 1 && wg_per_cu >= 3) {
            const int pr = (wg_slot + j) % 3;
            if (pr == 0) __builtin_amdgcn_s_setprio(0);
            else if (pr == 1) __builtin_amdgcn_s_setprio(1);
            else __builtin_amdgcn_s_setprio(2);
        }
        const int b = cur.b, h = cur.h;
        // wave-uniform bases (scalar registers) and per-lane 32-bit offsets: the loads take the
        // base from scalar registers, and advancing a stream is scalar arithmetic
        const int64_t row0 = uniform64(cur.row0);
        const char *kp = k_codes + row0 * RB;
        const char *vp = v_codes + row0 * RB;
        const float *kmp = k_meta + row0 * MW;
        const float *vmp = v_meta + row0 * MW;
        const unsigned co = T::lane_offset(lane, wave);         // wave w starts at its own run
        const unsigned mo = (unsigned)(own * MW);

        // the query stays fp16 for the dot instruction; its scale (log2 e / sqrt d) and the 2^24
        // of the subnormal codes are applied to the dot product
        f16x2 qh[EPL / 2];
        float qs = 0.f;
        {
            const _Float16 *qp = q + ((int64_t)b * H + h) * D + col * EPL;
            _Float16 qe[EPL];
#pragma unroll
            for (int c8 = 0; c8 < EPL / 8; ++c8) {
                const half8 v8 = *reinterpret_cast<const half8 *>(qp + 8 * c8);
#pragma unroll
                for (int i = 0; i < 8; ++i) qe[8 * c8 + i] = v8[i];
            }
#pragma unroll
            for (int i = 0; i < EPL; ++i) qs += (float)qe[i];
            qs = row_sum<LPR>(qs) * qscale;                      // scaled sum of the whole query
            T::pack_query(qe, qh);
        }
        const float kmul = qscale * 16777216.0f;

        float m = kNegBig, l = 0.f, aux = 0.f, acc[EPL];
#pragma unroll
        for (int i = 0; i < EPL; ++i) acc[i] = 0.f;

        const int ntok = __builtin_amdgcn_readfirstlane(cur.ntok);
        const int n_blk = ntok / T::BLK_TOK;
        const int rem = ntok - n_blk * T::BLK_TOK;

        const char *kt = kp;
        const char *vt = vp;
        const float *kmt = kmp;
        const float *vmt = vmp;
        constexpr int MSTEP = T::BLK_TOK * MW;                  // floats of parameters per block
        T A, Bf;
        if (n_blk > 0) {
            int left = n_blk;                              // A holds block n_blk-left, Bf the one after
            if (n_blk >= 4) {
                // both loads are issued unconditionally on the way into the loop: its wait
                // counts can then leave a whole block outstanding behind the one in use
                A.load(kt, vt, kmt, vmt, co, mo);
                Bf.load(kt + T::BLK_BYTES, vt + T::BLK_BYTES, kmt + MSTEP, vmt + MSTEP, co, mo);
                sched_fence();
                do {
                    A.template update<false, true>(qh, kmul, qs, m, l, aux, acc, row, 0, 0, co, mo,
                                                   kt + 2 * T::BLK_BYTES, vt + 2 * T::BLK_BYTES,
                                                   kmt + 2 * MSTEP, vmt + 2 * MSTEP);
                    Bf.template update<false, true>(qh, kmul, qs, m, l, aux, acc, row, 0, 0, co, mo,
                                                    kt + 3 * T::BLK_BYTES, vt + 3 * T::BLK_BYTES,
                                                    kmt + 3 * MSTEP, vmt + 3 * MSTEP);
                    kt += 2 * T::BLK_BYTES;
                    vt += 2 * T::BLK_BYTES;
                    kmt += 2 * MSTEP;
                    vmt += 2 * MSTEP;
                    left -= 2;
                } while (left > 3);
                // the counters are the same in every lane; say so, so that the stream bases
                // below stay in scalar registers
                left = __builtin_amdgcn_readfirstlane(left);
                const int64_t done = n_blk - left;
                kt = kp + done * T::BLK_BYTES;
                vt = vp + done * T::BLK_BYTES;
                kmt = kmp + done * MSTEP;
                vmt = vmp + done * MSTEP;
            } else {
                A.load(kt, vt, kmt, vmt, co, mo);
                if (n_blk > 1) Bf.load(kt + T::BLK_BYTES, vt + T::BLK_BYTES, kmt + MSTEP, vmt + MSTEP, co, mo);
                sched_fence();
            }
            if (left == 3) {
                A.template update<false, true>(qh, kmul, qs, m, l, aux, acc, row, 0, 0, co, mo,
                                               kt + 2 * T::BLK_BYTES, vt + 2 * T::BLK_BYTES,
                                               kmt + 2 * MSTEP, vmt + 2 * MSTEP);
                Bf.template update<false, false>(qh, kmul, qs, m, l, aux, acc, row, 0, 0);
                A.template update<false, false>(qh, kmul, qs, m, l, aux, acc, row, 0, 0);
            } else if (left == 2) {
                A.template update<false, false>(qh, kmul, qs, m, l, aux, acc, row, 0, 0);
                Bf.template update<false, false>(qh, kmul, qs, m, l, aux, acc, row, 0, 0);
            } else {
                A.template update<false, false>(qh, kmul, qs, m, l, aux, acc, row, 0, 0);
            }
        }
        // The ragged rest of the unit goes through tiles of one memory load per wave (8 tokens, 16
        // for 4-bit pairs): a rest of a few tokens then costs a few tokens' arithmetic, not a whole
        // block's (uniform 2048-token batches leave exactly one token, the one just appended).
        {
            using T1 = TileQ<BITS, D_, BITS == 4 ? 2 : 1, WPU>;
            const int wtok1 = T1::first_token(wave);
            for (int t0 = 0; t0 < rem; t0 += T1::BLK_TOK) {
                const int r1 = min(rem - t0, T1::BLK_TOK);
                if (wtok1 < r1) {                          // this wave has at least one valid row
                    // The lane-dependent offsets of this path are worked out here, from a copy of
                    // the lane number that the compiler must take as new: hoisted out of the unit
                    // loop they would sit in registers all through the streaming loop, which has
                    // none to spare (nine were spilled to scratch memory; with scratch memory in
                    // use the kernel ran 4-6 % slower on batches of equal-length sequences).
                    int lane1 = lane;
                    asm volatile("" : "+v"(lane1));
                    const int row1 = lane1 / LPR;
                    const int own1 = T1::own_token(lane1, wave);
                    const int64_t o = (int64_t)n_blk * T::BLK_BYTES + (int64_t)t0 * RB;
                    const int64_t so = (int64_t)n_blk * MSTEP + (int64_t)t0 * MW;
                    T1 C;
                    C.load_tail(kp + o, vp + o, kmp + so, vmp + so, T1::lane_offset(lane1, wave),
                                (unsigned)(own1 * MW), row1, wtok1, own1, r1);
                    C.template update<true, false>(qh, kmul, qs, m, l, aux, acc, row1, wtok1, r1);
                }
            }
        }

        T::fix_odd(acc);
        // combine the rows of this wave
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1) {
            const float mo = __shfl_xor(m, off);
            const float lo = __shfl_xor(l, off);
            const float xo = __shfl_xor(aux, off);
            const float M = fmaxf(m, mo);
            const float a = fast_exp2(m - M), c = fast_exp2(mo - M);
            l = l * a + lo * c;
            aux = aux * a + xo * c;
#pragma unroll
            for (int i = 0; i < EPL; ++i) acc[i] = acc[i] * a + __shfl_xor(acc[i], off) * c;
            m = M;
        }
        if constexpr (WPU == 1) {
            // the wave owns the unit: every lane now holds the state of all rows for its 16
            // elements; the 8 lanes of row 0 write them
            if (lane < LPR) {
                if (cur.nch == 1) {
                    _Float16 o16[EPL];
#pragma unroll
                    for (int i = 0; i < EPL; ++i) o16[i] = (_Float16)((acc[i] + aux) / l);
                    _Float16 *op = out + ((int64_t)b * H + h) * D + lane * EPL;
#pragma unroll
                    for (int c8 = 0; c8 < EPL / 8; ++c8) {
                        half8 v8;
#pragma unroll
                        for (int i = 0; i < 8; ++i) v8[i] = o16[8 * c8 + i];
                        __builtin_nontemporal_store(v8, reinterpret_cast<half8 *>(op + 8 * c8));
                    }
                } else {
                    const int64_t rec = (int64_t)cur.item * H + h;
#pragma unroll
                    for (int i = 0; i < EPL; ++i) st_agent(&part_acc[rec * D + lane * EPL + i], acc[i] + aux);
                    if (lane == 0) {
                        st_agent(&part_ml[rec * 2], m);
                        st_agent(&part_ml[rec * 2 + 1], l);
                    }
                }
            }
            if (cur.nch != 1) {
                if (lane == 0) split_list[n_split] = make_int4(b, h, cur.nch, a.v.item0[b]);
                ++n_split;
            }
        } else {
            float (&sm_acc)[kWaves][D] = sm_acc2[set];
            float (&sm_m)[kWaves] = sm_m2[set];
            float (&sm_l)[kWaves] = sm_l2[set];
            float (&sm_aux)[kWaves] = sm_aux2[set];
            set ^= 1;
            if (lane < LPR) {
#pragma unroll
                for (int i = 0; i < EPL; ++i) sm_acc[wave][lane * EPL + i] = acc[i];
            }
            if (lane == 0) { sm_m[wave] = m; sm_l[wave] = l; sm_aux[wave] = aux; }
            __syncthreads();

            if (cur.nch == 1) {
                if (tid < D) {
                    float M = sm_m[0];
#pragma unroll
                    for (int w = 1; w < kWaves; ++w) M = fmaxf(M, sm_m[w]);
                    float L = 0.f, X = 0.f, o = 0.f;
#pragma unroll
                    for (int w = 0; w < kWaves; ++w) {
                        const float wa = fast_exp2(sm_m[w] - M);
                        L += wa * sm_l[w];
                        X += wa * sm_aux[w];
                        o += wa * sm_acc[w][tid];
                    }
                    o += X;                                      // the weighted zero points
                    __builtin_nontemporal_store((_Float16)(o / L), &out[((int64_t)b * H + h) * D + tid]);
                }
            } else if (wave == 0) {
                // one wave writes the whole chunk state, publishes it and counts the chunk
                float M = sm_m[0];
#pragma unroll
                for (int w = 1; w < kWaves; ++w) M = fmaxf(M, sm_m[w]);
                float L = 0.f, X = 0.f, wgt[kWaves];
#pragma unroll
                for (int w = 0; w < kWaves; ++w) {
                    wgt[w] = fast_exp2(sm_m[w] - M);
                    L += wgt[w] * sm_l[w];
                    X += wgt[w] * sm_aux[w];
                }
                const int64_t rec = (int64_t)cur.item * H + h;
#pragma unroll
                for (int e = lane; e < D; e += 64) {
                    float o = X;
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

// One kernel, two bodies: the planner decides per launch whether a workgroup's four waves share
// a unit or take one each (short sequences: a unit's fixed cost, the epilogue with its barrier
// and cross-wave combine, is then spread over four times as many blocks per wave).
template <int BITS, int D>
__global__ __launch_bounds__(kThreads)
__attribute__((amdgpu_waves_per_eu(q_wg_short<BITS>(), q_wg_short<BITS>())))
void rpartq_partial_kernel(PartialQArgs a)
{
    const int32_t *hdr = a.v.hdr;
    if (!plan_matches(hdr, a.B, a.H, plan_kind(D, BITS), a.v.max_items, (int)gridDim.x, a.status)) return;
    if ((int)blockIdx.x >= hdr[HDR_GRID]) return;
    unit_prologue<D>(hdr, a.v.nchunk, a.v.newlen, a.v.newseen, a.seq_lens, a.seq_seen, a.out, a.B, a.H);
    if constexpr (q_wave_units<BITS>() != 0) {
        if (hdr[HDR_WAVE_UNITS]) {
            rpartq_body<BITS, D, 1>(a);
            return;
        }
    }
    rpartq_body<BITS, D, kWaves>(a);
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
int check_qdesc(const fd_kvq_desc *d)
{
    if (!d) return FD_EINVAL;
    if (d->B < 0 || d->H <= 0 || (d->d != 128 && d->d != 64)) return FD_EINVAL;
    if (d->chunk_tokens < 0) return FD_EINVAL;
    if (d->bits != 0 && d->bits != 8 && d->bits != 4) return FD_EINVAL;
    if (d->B == 0) return FD_OK;
    if (!d->k_codes || !d->v_codes || !d->k_scale || !d->v_scale || !d->seq_off || !d->seq_cap ||
        !d->seq_lens || !d->status)
        return FD_EINVAL;
    if (!aligned(d->k_codes, 16) || !aligned(d->v_codes, 16) || !aligned(d->k_scale, 8) ||
        !aligned(d->v_scale, 8) || !aligned(d->seq_off, 8) || !aligned(d->seq_cap, 4) ||
        !aligned(d->seq_lens, 4) || !aligned(d->status, 4))
        return FD_EINVAL;
    if (d->seq_seen && (!aligned(d->seq_seen, 4) || d->n_sink < 0)) return FD_EINVAL;
    return FD_OK;
}

int check_qws(const fd_kvq_desc *d, const void *ws, size_t ws_bytes, WsLayout *w)
{
    if (!ws || !aligned(ws, 256)) return FD_EINVAL;
    *w = ws_layout(d->B, d->H, d->d, ws_bytes);
    if (w->max_items < d->B) return FD_EWORKSPACE;
    return FD_OK;
}

// instantiate a launch for the descriptor's bit width and head dimension
#define FD_Q_DISPATCH(desc, LAUNCH)                                    \
    do {                                                               \
        if ((desc)->bits == 4) {                                       \
            if ((desc)->d == 64) { LAUNCH(4, 64); } else { LAUNCH(4, 128); } \
        } else {                                                       \
            if ((desc)->d == 64) { LAUNCH(8, 64); } else { LAUNCH(8, 128); } \
        }                                                              \
    } while (0)

QSlabs q_slabs(const fd_kvq_desc *d)
{
    QSlabs c;
    c.k_codes = (uint8_t *)d->k_codes;
    c.v_codes = (uint8_t *)d->v_codes;
    c.k_meta = d->k_scale;
    c.v_meta = d->v_scale;
    return c;
}

SeqState q_seq_state(const fd_kvq_desc *d)
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

PlanArgs q_plan_args(const fd_kvq_desc *d, void *workspace, const WsLayout &w, int grid, int after_append)
{
    const bool four = d->bits == 4;
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
    a.granule = 64;
    a.grid_long = (four ? q_wg_long<4>() : q_wg_long<8>()) * grid;
    a.grid_short = (four ? q_wg_short<4>() : q_wg_short<8>()) * grid;
    a.short_below = kShortSeq;
    a.hashed = 1;
    a.wave_units = four ? q_wave_units<4>() : q_wave_units<8>();
    a.split = kQSplit;
    a.kind = plan_kind(d->d, four ? 4 : 8);
    a.v = plan_view(workspace, w);
    return a;
}

int launch_qpartial(const fd_kvq_desc *desc, const void *q, void *out, void *workspace,
                    const WsLayout &w, int grid, void *stream)
{
    PartialQArgs a;
    a.k_codes = (const char *)desc->k_codes;
    a.v_codes = (const char *)desc->v_codes;
    a.k_meta = desc->k_scale;
    a.v_meta = desc->v_scale;
    a.seq_off = desc->seq_off;
    a.seq_cap = desc->seq_cap;
    a.seq_lens = desc->seq_lens;
    a.seq_seen = desc->seq_seen;
    a.status = desc->status;
    a.q = (const _Float16 *)q;
    a.out = (_Float16 *)out;
    a.B = desc->B;
    a.H = desc->H;
    a.qscale = (float)(1.4426950408889634 / (desc->d == 128 ? 11.313708498984761 : 8.0));
    a.v = plan_view(workspace, w);
#define FD_LAUNCH(BITS, D)                                                                              \
    hipLaunchKernelGGL((rpartq_partial_kernel<BITS, D>), dim3(q_wg_short<BITS>() * grid), dim3(kThreads), 0, \
                       (hipStream_t)stream, a)
    FD_Q_DISPATCH(desc, FD_LAUNCH);
#undef FD_LAUNCH
    return launched();
}

int check_qdecode_args(const fd_kvq_desc *desc, const void *q, const void *out, const void *workspace,
                       size_t workspace_bytes, WsLayout *w)
{
    int rc = check_qdesc(desc);
    if (rc != FD_OK) return rc;
    if (desc->B == 0) return FD_OK;
    if (!q || !out || !aligned(q, 16) || !aligned(out, 16)) return FD_EINVAL;
    return check_qws(desc, workspace, workspace_bytes, w);
}

int launch_qfront(const fd_kvq_desc *desc, const void *k_new, const void *v_new, void *workspace,
                  const WsLayout &w, int grid, void *stream)
{
    const PlanArgs pa = q_plan_args(desc, workspace, w, grid, 1);
#define FD_LAUNCH(BITS, D)                                                                              \
    hipLaunchKernelGGL((kvq_append_plan_kernel<BITS, D>), dim3(desc->B + 1), dim3(kPlanThreads), 0,     \
                       (hipStream_t)stream, q_slabs(desc), q_seq_state(desc), (const _Float16 *)k_new,  \
                       (const _Float16 *)v_new, pa)
    FD_Q_DISPATCH(desc, FD_LAUNCH);
#undef FD_LAUNCH
    return launched();
}

} // namespace

extern "C" {

int fd_kvq_append(const fd_kvq_desc *desc, const void *k_new, const void *v_new, void *stream)
{
    int rc = check_qdesc(desc);
    if (rc != FD_OK) return rc;
    if (desc->B == 0) return FD_OK;
    if (!k_new || !v_new || !aligned(k_new, 16) || !aligned(v_new, 16)) return FD_EINVAL;
#define FD_LAUNCH(BITS, D)                                                                              \
    hipLaunchKernelGGL((kvq_append_kernel<BITS, D>), dim3(desc->B), dim3(256), 0, (hipStream_t)stream,  \
                       q_slabs(desc), q_seq_state(desc), (const _Float16 *)k_new,                       \
                       (const _Float16 *)v_new, desc->H)
    FD_Q_DISPATCH(desc, FD_LAUNCH);
#undef FD_LAUNCH
    return launched();
}

int fd_kvq_append_plan(const fd_kvq_desc *desc, const void *k_new, const void *v_new,
                       void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_qdesc(desc);
    if (rc != FD_OK) return rc;
    if (desc->B == 0) return FD_OK;
    if (!k_new || !v_new || !aligned(k_new, 16) || !aligned(v_new, 16)) return FD_EINVAL;
    WsLayout w;
    rc = check_qws(desc, workspace, workspace_bytes, &w);
    if (rc != FD_OK) return rc;
    const int grid = persistent_grid();
    if (grid <= 0) return FD_EHIP;
    return launch_qfront(desc, k_new, v_new, workspace, w, grid, stream);
}

int fd_kvq_store_rows(const fd_kvq_desc *desc, int32_t b, int32_t t0, int32_t n, const void *k_rows,
                      const void *v_rows, int set_len, void *stream)
{
    int rc = check_qdesc(desc);
    if (rc != FD_OK) return rc;
    if (b < 0 || b >= desc->B || t0 < 0 || n < 0 || (int64_t)t0 + n > INT32_MAX) return FD_EINVAL;
    if ((k_rows && !aligned(k_rows, 16)) || (v_rows && !aligned(v_rows, 16))) return FD_EINVAL;
    if (n == 0 && !set_len) return FD_OK;
    const int64_t rows = (int64_t)desc->H * n;
    const int per_wg = 256 / (desc->d / 8);                   // rows a workgroup handles
    const unsigned grid = (unsigned)(rows > 0 ? (rows + per_wg - 1) / per_wg : 1);
#define FD_LAUNCH(BITS, D)                                                                              \
    hipLaunchKernelGGL((kvq_store_rows_kernel<BITS, D>), dim3(grid), dim3(256), 0, (hipStream_t)stream, \
                       (uint8_t *)desc->k_codes, (uint8_t *)desc->v_codes, desc->k_scale, desc->v_scale, \
                       desc->seq_off, desc->seq_cap, desc->seq_lens, desc->seq_seen, desc->status,      \
                       (const _Float16 *)k_rows, (const _Float16 *)v_rows, desc->H, b, t0, n, set_len)
    FD_Q_DISPATCH(desc, FD_LAUNCH);
#undef FD_LAUNCH
    return launched();
}

static int reset_qslots(const fd_kvq_desc *desc, const int32_t *seq_ids, int32_t n, int value,
                        void *stream)
{
    int rc = check_qdesc(desc);
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

int fd_kvq_reset(const fd_kvq_desc *desc, const int32_t *seq_ids, int32_t n, void *stream)
{
    return reset_qslots(desc, seq_ids, n, 0, stream);
}

int fd_kvq_release(const fd_kvq_desc *desc, const int32_t *seq_ids, int32_t n, void *stream)
{
    return reset_qslots(desc, seq_ids, n, FD_SLOT_FREE, stream);
}

int fd_rpartq_plan(const fd_kvq_desc *desc, void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_qdesc(desc);
    if (rc != FD_OK) return rc;
    if (desc->B == 0) return FD_OK;
    WsLayout w;
    rc = check_qws(desc, workspace, workspace_bytes, &w);
    if (rc != FD_OK) return rc;
    const int grid = persistent_grid();
    if (grid <= 0) return FD_EHIP;
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(kPlanThreads), 0, (hipStream_t)stream,
                       q_plan_args(desc, workspace, w, grid, 0));
    return launched();
}

int fd_rpartq_partial(const fd_kvq_desc *desc, const void *q, void *out,
                      void *workspace, size_t workspace_bytes, void *stream)
{
    WsLayout w;
    int rc = check_qdecode_args(desc, q, out, workspace, workspace_bytes, &w);
    if (rc != FD_OK || desc->B == 0) return rc;
    const int grid = persistent_grid();
    if (grid <= 0) return FD_EHIP;
    return launch_qpartial(desc, q, out, workspace, w, grid, stream);
}

int fd_rpartq_merge(const fd_kvq_desc *desc, void *out,
                    void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_qdesc(desc);
    if (rc != FD_OK) return rc;
    if (desc->B == 0) return FD_OK;
    if (!out || !aligned(out, 16)) return FD_EINVAL;
    WsLayout w;
    rc = check_qws(desc, workspace, workspace_bytes, &w);
    if (rc != FD_OK) return rc;
    const int64_t bh = (int64_t)desc->B * desc->H;
    const dim3 grid((unsigned)((bh + 3) / 4));
    const int kind = plan_kind(desc->d, desc->bits == 4 ? 4 : 8);
    if (desc->d == 128)
        hipLaunchKernelGGL(rpart_merge_kernel<128>, grid, dim3(256), 0, (hipStream_t)stream,
                           plan_view(workspace, w), (_Float16 *)out, desc->B, desc->H, kind, desc->status);
    else
        hipLaunchKernelGGL(rpart_merge_kernel<64>, grid, dim3(256), 0, (hipStream_t)stream,
                           plan_view(workspace, w), (_Float16 *)out, desc->B, desc->H, kind, desc->status);
    return launched();
}

int fd_rpartq_decode(const fd_kvq_desc *desc, const void *q, void *out,
                     void *workspace, size_t workspace_bytes, void *stream)
{
    WsLayout w;
    int rc = check_qdecode_args(desc, q, out, workspace, workspace_bytes, &w);
    if (rc != FD_OK || desc->B == 0) return rc;
    const int grid = persistent_grid();
    if (grid <= 0) return FD_EHIP;
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(kPlanThreads), 0, (hipStream_t)stream,
                       q_plan_args(desc, workspace, w, grid, 0));
    rc = launched();
    if (rc != FD_OK) return rc;
    return launch_qpartial(desc, q, out, workspace, w, grid, stream);
}

static int qstep_fused(const fd_kvq_desc *desc, const void *q, const void *k_new, const void *v_new,
                       void *out, void *workspace, size_t workspace_bytes, void *stream)
{
    WsLayout w;
    int rc = check_qdecode_args(desc, q, out, workspace, workspace_bytes, &w);
    if (rc != FD_OK || desc->B == 0) return rc;
    if (!k_new || !v_new || !aligned(k_new, 16) || !aligned(v_new, 16)) return FD_EINVAL;
    const int grid = persistent_grid();
    if (grid <= 0) return FD_EHIP;
    rc = launch_qfront(desc, k_new, v_new, workspace, w, grid, stream);
    if (rc != FD_OK) return rc;
    return launch_qpartial(desc, q, out, workspace, w, grid, stream);
}

int fd_rpartq_step(const fd_kvq_desc *desc, const void *q, const void *k_new, const void *v_new,
                   void *out, void *workspace, size_t workspace_bytes, void *stream)
{
    return qstep_fused(desc, q, k_new, v_new, out, workspace, workspace_bytes, stream);
}

int fd_rpartq_layer_step(const fd_kvq_desc *layer, const void *q, const void *k_new,
                         const void *v_new, void *out, void *workspace, size_t workspace_bytes,
                         int replan, void *stream)
{
    if (replan) return qstep_fused(layer, q, k_new, v_new, out, workspace, workspace_bytes, stream);
    WsLayout w;
    int rc = check_qdecode_args(layer, q, out, workspace, workspace_bytes, &w);
    if (rc != FD_OK || layer->B == 0) return rc;
    if (!k_new || !v_new || !aligned(k_new, 16) || !aligned(v_new, 16)) return FD_EINVAL;
    const int grid = persistent_grid();
    if (grid <= 0) return FD_EHIP;
    rc = fd_kvq_append(layer, k_new, v_new, stream);
    if (rc != FD_OK) return rc;
    return launch_qpartial(layer, q, out, workspace, w, grid, stream);
}

} // extern "C"

// Host-only exercise of the library for an AddressSanitizer + UBSan build: the scheduling
// arithmetic (fastdecode_sched.h) under random use, and the argument checks of the GPU entry
// points, which return before any HIP call.  No GPU is touched.  Exit status 0 = every check
// held and the sanitizers found nothing.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "fastdecode_rpart.h"
#include "fastdecode_sched.h"

static int failures = 0;
#define CHECK(x) do { if (!(x)) { std::fprintf(stderr, "CHECK failed: %s (line %d)\n", #x, __LINE__); ++failures; } } while (0)

static uint64_t rng_state = 0x243F6A8885A308D3ull;
static uint64_t rnd()
{
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return rng_state;
}
static int64_t rnd_in(int64_t lo, int64_t hi) { return lo + (int64_t)(rnd() % (uint64_t)(hi - lo + 1)); }

static void sched_random_walk()
{
    for (int trial = 0; trial < 300; ++trial) {
        const int64_t S = rnd_in(1, 40), W_lim = rnd_in(S, S * 50);
        fd_load_ctl *lc = fd_lc_create(S, W_lim);
        CHECK(lc != nullptr);
        int64_t t = 0;
        for (int k = 0; k < 60; ++k) {
            const int64_t m = rnd_in(1, 6);
            fd_lc_retire(lc, t);
            const int64_t r = fd_lc_earliest_step(lc, t, m);
            if (m * S > W_lim) { CHECK(r == FD_EINVAL); continue; }
            CHECK(r >= t);
            t = r;
            CHECK(fd_lc_add_microbatch(lc, t, m) == FD_OK);
            const int64_t n = fd_lc_count(lc);
            std::vector<int64_t> M((size_t)n), E((size_t)n), W((size_t)n);
            CHECK(fd_lc_snapshot(lc, n, M.data(), E.data(), W.data()) == n);
            for (int64_t i = 0; i < n; ++i) CHECK(W[(size_t)i] <= W_lim || E[(size_t)i] <= t);
            CHECK(fd_lc_snapshot(lc, 0, nullptr, nullptr, nullptr) == 0);
            t += rnd_in(0, 3);
        }
        fd_lc_destroy(lc);
    }
    CHECK(fd_lc_create(0, 5) == nullptr);
    CHECK(fd_lc_earliest_step(nullptr, 0, 1) == FD_EINVAL);
    CHECK(fd_lc_retire(nullptr, 0) == FD_EINVAL);
    fd_lc_destroy(nullptr);

    for (int trial = 0; trial < 200; ++trial) {
        const int64_t S = rnd_in(1, 30), M = rnd_in(1, 4), B = M * rnd_in(1, 8), F = rnd_in(1, 6);
        const int64_t W_lim = rnd_in(M * S, M * S * 8), n = rnd_in(0, 6 * S);
        std::vector<int64_t> starts((size_t)(n > 0 ? n : 1));
        const int64_t full = fd_lc_controlled_starts(B, S, M, F, W_lim, n, starts.data(), n);
        CHECK(full >= 0 && full <= n);
        const int64_t cut = fd_lc_controlled_starts(B, S, M, F, W_lim, n, starts.data(), full / 2);
        CHECK(cut == full);                                   // the count does not depend on the room given
        std::vector<int64_t> loads((size_t)(n > 0 ? n : 1));
        CHECK(fd_sls_step_loads(M, F, S, n, loads.data()) == FD_OK);
        CHECK(fd_batch_step_loads(B, S, n, loads.data()) == FD_OK);
        CHECK(fd_sls_peak_load(M, F, S) >= 0 && fd_sls_microbatch_size(B, F, S) >= 1);
    }
    CHECK(fd_lc_controlled_starts(8, 4, 3, 1, 100, 10, nullptr, 0) == FD_EINVAL);      // B % M != 0
    CHECK(fd_sls_step_loads(1, 1, 1, 3, nullptr) == FD_EINVAL);

    for (int trial = 0; trial < 100; ++trial) {
        const int32_t B = (int32_t)rnd_in(1, 40);
        fd_slots *s = fd_slots_create(B);
        std::vector<char> held((size_t)B, 0);
        int in_use = 0;
        for (int k = 0; k < 400; ++k) {
            if (rnd() & 1) {
                const int32_t id = fd_slots_acquire(s);
                if (in_use == B) CHECK(id == FD_SLOT_FREE);
                else { CHECK(id >= 0 && id < B && !held[(size_t)id]); held[(size_t)id] = 1; ++in_use; }
            } else {
                const int32_t id = (int32_t)rnd_in(-2, B + 1);
                const int rc = fd_slots_release(s, id);
                if (id >= 0 && id < B && held[(size_t)id]) { CHECK(rc == FD_OK); held[(size_t)id] = 0; --in_use; }
                else CHECK(rc == FD_EINVAL);
            }
            CHECK(fd_slots_in_use(s) == in_use);
        }
        fd_slots_destroy(s);
    }
    CHECK(fd_slots_create(0) == nullptr);

    const int64_t Bs[3] = {1, 64, 256};
    const double T[3] = {0.5, 0.6, 1.0};
    CHECK(fd_model_max_batch(32, 1024, 70000.0, Bs, T, 3) == 256);
    CHECK(fd_model_max_batch(32, 1024, 70000.0, nullptr, nullptr, 0) == 0);
    CHECK(fd_model_min_rworkers_memory(INT64_MAX / 2, 4, 16) == FD_EINVAL);             // overflow guarded
    CHECK(fd_model_num_rworkers(1024, 1024, 1.0, 1000000.0) == 0.524288);
}

static void entry_point_argument_checks()
{
    // aligned, fake device pointers: the host checks never dereference them
    auto P = [](uintptr_t x) { return (void *)x; };
    fd_kv_desc d = {};
    d.k_base = P(0x1000); d.v_base = P(0x2000);
    d.seq_off = (const int64_t *)P(0x3000); d.seq_cap = (const int32_t *)P(0x4000);
    d.seq_lens = (int32_t *)P(0x5000); d.status = (int32_t *)P(0x6000);
    d.B = 2; d.H = 4; d.d = 128;
    int32_t st = 0;
    CHECK(fd_kv_append(nullptr, P(0x7000), P(0x8000), nullptr) == FD_EINVAL);
    CHECK(fd_kv_append(&d, nullptr, P(0x8000), nullptr) == FD_EINVAL);
    CHECK(fd_kv_append(&d, P(0x7008), P(0x8000), nullptr) == FD_EINVAL);
    CHECK(fd_rpart_decode(&d, P(0x7000), P(0x8000), P(0x9000), 16, nullptr) == FD_EWORKSPACE);
    CHECK(fd_rpart_decode(&d, P(0x7000), P(0x8000), P(0x9010), 1u << 30, nullptr) == FD_EINVAL);
    CHECK(fd_rpart_step(&d, P(0x7000), nullptr, P(0x8000), P(0x8000), P(0x9000), 1u << 30, nullptr) == FD_EINVAL);
    CHECK(fd_rpart_layer_step(&d, P(0x7000), P(0x7000), P(0x8000), nullptr, P(0x9000), 1u << 30, 1, nullptr) == FD_EINVAL);
    CHECK(fd_rpart_plan(&d, nullptr, 1u << 30, nullptr) == FD_EINVAL);
    CHECK(fd_rpart_partial(&d, P(0x7000), P(0x8000), P(0x9000), 0, nullptr) == FD_EWORKSPACE);
    CHECK(fd_rpart_merge(&d, P(0x8001), P(0x9000), 1u << 30, nullptr) == FD_EINVAL);
    CHECK(fd_kv_reset(&d, (const int32_t *)P(0x7000), -1, nullptr) == FD_EINVAL);
    CHECK(fd_kv_release(nullptr, nullptr, 0, nullptr) == FD_EINVAL);
    CHECK(fd_kv_store_rows(&d, 2, 0, 1, P(0x7000), nullptr, 0, nullptr) == FD_EINVAL);
    CHECK(fd_kv_store_rows(&d, 0, 3, 0, nullptr, nullptr, 0, nullptr) == FD_OK);
    CHECK(fd_read_status(&d, nullptr, 0, nullptr) == FD_EINVAL);
    CHECK(fd_last_device_status(&d, P(0x9010), &st, nullptr) == FD_EINVAL);
    CHECK(fd_plan_info(nullptr, nullptr, nullptr) == FD_EINVAL);
    fd_kv_desc big = d;
    big.B = 4096; big.H = 64;
    CHECK(fd_rpart_decode_noalloc(&big, P(0x7000), P(0x8000), nullptr) == FD_ETOOBIG);
    CHECK(fd_rpart_decode_noalloc(&d, P(0x7000), nullptr, nullptr) == FD_EINVAL);
    d.d = 96;
    CHECK(fd_kv_append(&d, P(0x7000), P(0x8000), nullptr) == FD_EINVAL);
    d.d = 64; d.chunk_tokens = -1;
    CHECK(fd_rpart_decode(&d, P(0x7000), P(0x8000), P(0x9000), 1u << 30, nullptr) == FD_EINVAL);
    d.chunk_tokens = 0; d.B = 0;
    CHECK(fd_rpart_step(&d, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr) == FD_OK);   // empty batch

    fd_kvq_desc q = {};
    q.k_codes = P(0x1000); q.v_codes = P(0x2000); q.k_scale = (float *)P(0x3000); q.v_scale = (float *)P(0x4000);
    q.seq_off = (const int64_t *)P(0x5000); q.seq_cap = (const int32_t *)P(0x6000);
    q.seq_lens = (int32_t *)P(0x7000); q.status = (int32_t *)P(0x8000);
    q.B = 3; q.H = 2; q.d = 128; q.bits = 4;
    CHECK(fd_kvq_append(&q, nullptr, nullptr, nullptr) == FD_EINVAL);
    CHECK(fd_rpartq_decode(&q, P(0x9000), P(0xA000), P(0xB000), 64, nullptr) == FD_EWORKSPACE);
    CHECK(fd_rpartq_step(&q, P(0x9000), P(0x9000), P(0x9000), P(0xA000), P(0xB001), 1u << 30, nullptr) == FD_EINVAL);
    CHECK(fd_kvq_store_rows(&q, 3, 0, 1, P(0x9000), nullptr, 0, nullptr) == FD_EINVAL);
    q.bits = 5;
    CHECK(fd_kvq_reset(&q, nullptr, 0, nullptr) == FD_EINVAL);
    q.bits = 8; q.d = 96;
    CHECK(fd_rpartq_plan(&q, P(0xB000), 1u << 30, nullptr) == FD_EINVAL);

    CHECK(fd_workspace_bytes(256, 32, 128, 0) > 0 && fd_workspace_bytes(256, 32, 96, 0) == 0);
    CHECK(fd_workspace_bytes(1, 1, 64, INT64_MAX / 2) > 0);
    for (int c = -6; c <= 1; ++c) CHECK(fd_strerror(c) != nullptr);
    CHECK(fd_desc_size(0) == sizeof(fd_kv_desc) && fd_desc_size(1) == sizeof(fd_kvq_desc) && fd_desc_size(7) == 0);
    size_t nread = 1;
    CHECK(fd_hbm_read_probe(nullptr, 1u << 30, &st, &nread, nullptr) == FD_EINVAL);
}

int main()
{
    sched_random_walk();
    entry_point_argument_checks();
    if (failures) { std::fprintf(stderr, "%d check(s) failed\n", failures); return 1; }
    std::puts("sanitize_host: ok");
    return 0;
}

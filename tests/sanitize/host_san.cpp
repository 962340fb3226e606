// Sanitizer driver for the host-only part of the C ABI (test infrastructure; needs no GPU).
//
// Linked with csrc/nfd_attn.hip compiled with -fsanitize=address,undefined on the host side and run by
// tests/test_sanitizers.py.  It sweeps the argument validation, the tile schedule and the speculative
// bookkeeping over valid, degenerate and invalid arguments; result structs live in heap blocks of their
// exact size so that a write past them is reported, and 32-/64-bit overflows in the size arithmetic abort.
#include <climits>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../include/nfd_attn.h"

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); std::exit(1); } } while (0)

static void plans() {
    const int dims[] = {INT_MIN, -1, 0, 1, 7, 16, 65, 336, 576, 1 << 20, INT_MAX};
    const int heads[] = {1, 12, 16, 64};
    long n_ok = 0;
    for (int dt = 0; dt <= 1; ++dt)  // enumerators only: any other value is not a valid nfd_dtype_t in C++
        for (int T : dims)
            for (int D : {0, 32, 64, 256, 257})
                for (int H : heads)
                    for (int kv : {-3, 0, 1, 2, 5, 33, 64, 100000, INT_MAX})
                        for (int qf : {-1, 0, 1, 2, 4, 33, INT_MAX})
                            for (int spare : {0, 1}) {
                                const int F = kv > 0 && kv < INT_MAX ? kv + spare : kv;
                                const int rc = nfd_attn_check_args((nfd_dtype_t)dt, 1, H, F, T, D, kv, qf);
                                nfd_attn_plan_t* pl = (nfd_attn_plan_t*)std::malloc(sizeof(nfd_attn_plan_t));
                                const int rp = nfd_attn_plan((nfd_dtype_t)dt, 1, H, F, T, D, kv, qf, 256, 0, pl);
                                CHECK((rc == NFD_OK) == (rp == NFD_OK) || rp == NFD_ERR_UNSUPPORTED);
                                if (rp == NFD_OK) {
                                    ++n_ok;
                                    CHECK(pl->n_workgroups >= 1 && pl->n_q_tiles >= 1 && pl->n_splits >= 1);
                                    CHECK(pl->key_tiles_visited <= pl->key_tiles_dense);
                                    // every workgroup id decodes to an item inside the launch
                                    if (pl->kernel == 1 && pl->n_workgroups <= 2048) {
                                        for (int grp = 0; grp < 2; ++grp) {
                                            std::vector<char> seen((size_t)H * pl->n_q_tiles * pl->n_splits, 0);
                                            const unsigned ids = (unsigned)pl->n_workgroups + 64;
                                            for (unsigned b = 0; b < ids; ++b) {
                                                int bh, qt, sp;
                                                if (nfd_attn_work_item(H, pl->n_q_tiles, pl->n_splits, grp, b, &bh, &qt, &sp) != NFD_OK) continue;
                                                CHECK(bh >= 0 && bh < H && qt >= 0 && qt < pl->n_q_tiles && sp >= 0 && sp < pl->n_splits);
                                                char& s = seen[((size_t)bh * pl->n_q_tiles + qt) * pl->n_splits + sp];
                                                CHECK(!s);
                                                s = 1;
                                            }
                                        }
                                    }
                                }
                                std::free(pl);
                            }
    CHECK(n_ok > 100);
    int r0, nr;
    CHECK(nfd_attn_q_tile_rows(INT_MAX, 3, 2, &r0, &nr) == NFD_ERR_UNSUPPORTED);
    for (int rows : {1, 31, 32, 33, 336, 1344, 5376, 36864, 1 << 30})
        for (int nq : {1, 2, 3, 6, 21, 144, 1 << 20}) {
            long covered = 0;
            for (int qt = 0; qt < nq && qt < 200; ++qt) {
                int r0 = -1, n = -1;
                const int rc = nfd_attn_q_tile_rows(rows, nq, qt, &r0, &n);
                CHECK(rc == NFD_OK && r0 >= 0 && n >= 0 && (long)r0 + n <= rows);
                CHECK(r0 == covered || n == 0);
                covered += n;
            }
            if (nq <= 200) CHECK(covered == rows);
        }
    CHECK(nfd_attn_q_tile_rows(10, 1, 1, &r0, &nr) == NFD_ERR_SHAPE && nfd_attn_q_tile_rows(10, 1, 0, nullptr, &nr) == NFD_ERR_NULL);
    CHECK(nfd_attn_plan(NFD_BF16, 1, 1, 1, 1, 64, 1, 1, 256, 0, nullptr) == NFD_ERR_NULL);
    int a, b;
    CHECK(nfd_attn_work_item(1, 1, 1, 0, 0, &a, &b, nullptr) == NFD_ERR_NULL);
    CHECK(nfd_attn_work_item(0, 1, 1, 0, 0, &a, &b, &a) == NFD_ERR_SHAPE);
    CHECK(nfd_attn_visible_pairs(3, 4, 2) == 63 && nfd_attn_visible_pairs(0, 1, 1) == -1);
    CHECK(nfd_attn_visible_pairs(46340, 46340, 46340) > 0);  // 64-bit arithmetic
    size_t bytes = 0;
    CHECK(nfd_fp8_cache_bytes(1, 16, 33, 336, 64, &bytes) == NFD_OK && bytes == (size_t)16 * 11136 * 64);
    CHECK(nfd_fp8_cache_bytes(1, 16, 33, 336, 64, nullptr) == NFD_ERR_NULL);
    CHECK(nfd_fp8_cache_bytes(INT_MAX, INT_MAX, INT_MAX, INT_MAX, 64, &bytes) != NFD_OK);
}

static void rope_args() {
    for (int T : {-1, 0, 1, 6, 336})
        for (int gh : {-1, 0, 1, 2, 24, INT_MAX})
            for (int gw : {0, 1, 3, 14, INT_MAX})
                for (int nt : {-2, 0, 1, 16, INT_MAX})
                    for (int pos : {-1, 0, 3, INT_MAX})
                        for (int n : {-1, 0, 1, INT_MAX})
                            (void)nfd_rope_check_args(NFD_BF16, 1, 16, 4, T, 64, pos, n, gh, gw, nt, 24, 24);
    CHECK(nfd_rope_check_args(NFD_BF16, 1, 16, 33, 336, 64, 32, 1, 24, 14, 16, 24, 24) == NFD_OK);
    CHECK(nfd_rope_check_args(NFD_BF16, 1, 16, 33, 336, 64, 33, 1, 24, 14, 16, 24, 24) == NFD_ERR_CAPACITY);
    CHECK(nfd_rope_check_args(NFD_BF16, 1, 16, 33, 336, 64, 0, 1, 24, 14, 16, 24, 22) == NFD_ERR_SHAPE);
}

static void spec_loop() {
    uint64_t s = 0x9e3779b97f4a7c15ull;
    auto next = [&]() { s ^= s << 13; s ^= s >> 7; s ^= s << 17; return s; };
    for (int rep = 0; rep < 300; ++rep) {
        const int n_spec = 1 + (int)(next() % 5), window = 1 + (int)(next() % 9), spare = (int)(next() % 3);
        const int capacity = window + n_spec + spare, n_prompt = 1 + (int)(next() % (unsigned)capacity);
        const int total = n_prompt + (int)(next() % 40), adim = 1 + (int)(next() % 3);
        nfd_spec_t* st = (nfd_spec_t*)std::malloc(sizeof(nfd_spec_t));
        nfd_spec_step_t* step = (nfd_spec_step_t*)std::malloc(sizeof(nfd_spec_step_t));
        int32_t* actions = (int32_t*)std::malloc(sizeof(int32_t) * (size_t)total * adim);  // exactly `total` rows
        for (int i = 0; i < total * adim; ++i) actions[i] = (int32_t)(next() % 2);
        CHECK(nfd_spec_init(st, capacity, window, n_spec, n_prompt, total) == NFD_OK);
        int guard = 0, rc;
        while ((rc = nfd_spec_next(st, step)) == 1) {
            CHECK(step->kv_frames <= capacity && step->frame_pos + step->n_frames == step->kv_frames);
            CHECK(step->n_frames >= 1 && step->n_frames <= n_spec && step->frame_pos <= window && step->n_drop >= 0);
            int kept = 0;
            CHECK(nfd_spec_accept(st, step, actions, adim, &kept) == NFD_OK);
            CHECK(kept >= 1 && kept <= step->n_frames);
            CHECK(++guard <= total);
        }
        CHECK(rc == 0 && st->done == total);
        std::free(st); std::free(step); std::free(actions);
    }
    nfd_spec_t st;
    CHECK(nfd_spec_init(nullptr, 4, 2, 2, 1, 5) == NFD_ERR_NULL);
    CHECK(nfd_spec_init(&st, 3, 2, 2, 1, 5) == NFD_ERR_CAPACITY);
    CHECK(nfd_spec_init(&st, INT_MAX, INT_MAX, INT_MAX, 1, 5) == NFD_ERR_CAPACITY);
    CHECK(nfd_spec_init(&st, 4, 2, 2, 0, 5) == NFD_ERR_SHAPE);
    CHECK(nfd_spec_next(&st, nullptr) == NFD_ERR_NULL);
}

static void null_handles() {  // every device entry point refuses a null handle before it touches anything
    char x[16] = {0};
    float f[1] = {1.f};
    CHECK(nfd_block_causal_attn_fwd(nullptr, x, x, x, x, 1, 1, 1, 1, 64, 1, 1, 0.f, nullptr) == NFD_ERR_NULL);
    CHECK(nfd_block_causal_attn_fwd_lse(nullptr, x, x, x, x, f, 1, 1, 1, 1, 64, 1, 1, 0.f, nullptr) == NFD_ERR_NULL);
    CHECK(nfd_kvcache_append(nullptr, x, x, x, x, 1, 1, 1, 1, 64, 0, 1, nullptr) == NFD_ERR_NULL);
    CHECK(nfd_kvcache_shift(nullptr, x, x, 1, 1, 1, 1, 64, 1, 0, nullptr) == NFD_ERR_NULL);
    CHECK(nfd_attn_destroy(nullptr) == NFD_OK);
    CHECK(nfd_last_error(nullptr) != nullptr);
    CHECK(nfd_attn_create(nullptr, NFD_BF16, 0, 0) == NFD_ERR_NULL);
}

int main() {
    plans();
    rope_args();
    spec_loop();
    null_handles();
    std::printf("host sanitizer run: ok\n");
    return 0;
}

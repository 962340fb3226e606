/* Sanitizer driver for the CPU oracle (test infrastructure).
 *
 * Built with -fsanitize=address,undefined together with oracle/nfd_oracle.c and run by
 * tests/test_sanitizers.py.  Every buffer is a heap block of exactly the documented size, so any
 * read or write of the oracle outside its arguments is reported.  The checks on the values are
 * only what needs no second implementation: finite outputs, rows of a constant V reproduce the
 * constant, gradients of a constant-V attention vanish in q and k, the cache append lands where
 * it should. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int nfd_oracle_block_causal_attn(const double *q, const double *k, const double *v, double *out, int B, int H, int F,
                                 int T, int D, int kv_frames, int q_frames, double scale, const int64_t *rows,
                                 int64_t n_rows);
int nfd_oracle_block_causal_attn_bwd(const double *q, const double *k, const double *v, const double *dout, double *dq,
                                     double *dk, double *dv, double *lse, int B, int H, int F, int T, int D,
                                     int kv_frames, int q_frames, double scale);
int nfd_oracle_kvcache_append(double *cache, const double *fresh, int B, int H, int F, int T, int D, int frame_pos,
                              int n_frames);
int nfd_oracle_rope_kvcache_append(const double *q, double *q_out, double *k_cache, double *v_cache, const double *k_new,
                                   const double *v_new, int B, int H, int F, int T, int D, int frame_pos, int n_frames,
                                   int t_offset, int grid_h, int grid_w, int n_t, int n_h, int n_w, double theta);
int64_t nfd_oracle_visible_pairs(int T, int kv_frames, int q_frames);

static uint64_t rng_state = 0x2506013801ull;
static double rnd(void) /* uniform in (-1, 1): enough for a memory check */
{
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(int64_t)(rng_state >> 11) / 4503599627370496.0 - 1.0;
}
static double *block(size_t n, int random, double fill)
{
    double *p = (double *)malloc((n ? n : 1) * sizeof(double));
    if (!p) { fprintf(stderr, "out of memory\n"); exit(2); }
    for (size_t i = 0; i < n; ++i) p[i] = random ? rnd() : fill;
    return p;
}
#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); exit(1); } } while (0)

static void attention_case(int B, int H, int F, int T, int D, int kvf, int qf)
{
    const size_t nq = (size_t)B * H * qf * T * D, nk = (size_t)B * H * F * T * D, nl = (size_t)B * H * qf * T;
    double *q = block(nq, 1, 0), *k = block(nk, 1, 0), *v = block(nk, 0, 0.75), *out = block(nq, 0, NAN);
    CHECK(nfd_oracle_block_causal_attn(q, k, v, out, B, H, F, T, D, kvf, qf, 0.3, NULL, 0) == 0);
    for (size_t i = 0; i < nq; ++i) CHECK(fabs(out[i] - 0.75) < 1e-12); /* weights sum to one */
    /* a subset of rows, in an order of its own, into a block of exactly that many rows */
    const int64_t Sq = (int64_t)qf * T;
    int64_t rows[3] = {Sq - 1, 0, Sq / 2};
    double *sub = block((size_t)B * H * 3 * D, 0, NAN);
    CHECK(nfd_oracle_block_causal_attn(q, k, v, sub, B, H, F, T, D, kvf, qf, 0.3, rows, 3) == 0);
    for (size_t i = 0; i < (size_t)B * H * 3 * D; ++i) CHECK(isfinite(sub[i]));
    rows[1] = Sq; /* out of range: refused, nothing touched */
    CHECK(nfd_oracle_block_causal_attn(q, k, v, sub, B, H, F, T, D, kvf, qf, 0.3, rows, 3) == -1);
    /* gradients: with V constant the output does not depend on q or k */
    double *g = block(nq, 1, 0), *dq = block(nq, 0, NAN), *dk = block(nk, 0, NAN), *dv = block(nk, 0, NAN);
    double *lse = block(nl, 0, NAN);
    CHECK(nfd_oracle_block_causal_attn_bwd(q, k, v, g, dq, dk, dv, lse, B, H, F, T, D, kvf, qf, 0.3) == 0);
    for (size_t i = 0; i < nq; ++i) CHECK(fabs(dq[i]) < 1e-12);
    for (size_t i = 0; i < nk; ++i) CHECK(fabs(dk[i]) < 1e-12 && isfinite(dv[i]));
    for (size_t i = 0; i < nl; ++i) CHECK(isfinite(lse[i]));
    CHECK(nfd_oracle_block_causal_attn_bwd(q, k, v, g, dq, dk, dv, NULL, B, H, F, T, D, kvf, qf, 0.3) == 0);
    free(q); free(k); free(v); free(out); free(sub); free(g); free(dq); free(dk); free(dv); free(lse);
}

static void cache_case(int B, int H, int F, int T, int D, int pos, int n, int gh, int gw, int nt, int nh, int nw)
{
    const size_t nc = (size_t)B * H * F * T * D, nn = (size_t)B * H * n * T * D;
    double *cache = block(nc, 0, -1.0), *fresh = block(nn, 1, 0);
    CHECK(nfd_oracle_kvcache_append(cache, fresh, B, H, F, T, D, pos, n) == 0);
    size_t changed = 0;
    for (size_t i = 0; i < nc; ++i) changed += cache[i] != -1.0;
    CHECK(changed <= nn);
    CHECK(nfd_oracle_kvcache_append(cache, fresh, B, H, F, T, D, F - n + 1, n) == -1);
    double *q = block(nn, 1, 0), *qo = block(nn, 0, NAN), *kc = block(nc, 0, -1.0), *vc = block(nc, 0, -1.0);
    double *kn = block(nn, 1, 0), *vn = block(nn, 1, 0);
    CHECK(nfd_oracle_rope_kvcache_append(q, qo, kc, vc, kn, vn, B, H, F, T, D, pos, n, 5, gh, gw, nt, nh, nw, 10000.0) == 0);
    for (size_t i = 0; i < nn; ++i) CHECK(isfinite(qo[i]));
    CHECK(nfd_oracle_rope_kvcache_append(q, q, kc, vc, kn, vn, B, H, F, T, D, pos, n, 5, gh, gw, nt, nh, nw, 10000.0) == 0); /* in place */
    CHECK(nfd_oracle_rope_kvcache_append(q, qo, kc, vc, kn, vn, B, H, F, T, D, pos, n, 5, gh, gw + 1, nt, nh, nw, 10000.0) == -1);
    free(cache); free(fresh); free(q); free(qo); free(kc); free(vc); free(kn); free(vn);
}

int main(void)
{
    attention_case(1, 1, 1, 1, 1, 1, 1);
    attention_case(1, 2, 4, 16, 64, 4, 4);
    attention_case(2, 3, 5, 7, 24, 4, 2);   /* spare capacity, cached form, odd sizes */
    attention_case(1, 2, 6, 5, 8, 6, 1);
    attention_case(1, 1, 3, 33, 64, 3, 3);
    cache_case(1, 2, 4, 6, 8, 1, 2, 2, 3, 2, 2, 4);
    cache_case(2, 1, 3, 12, 16, 2, 1, 3, 4, 0, 8, 8);
    cache_case(1, 1, 2, 4, 6, 0, 0, 2, 2, 2, 2, 2);    /* nothing to append */
    CHECK(nfd_oracle_visible_pairs(3, 4, 2) == 3 * 3 * (2 * 2 + 3));
    printf("oracle sanitizer run: ok\n");
    return 0;
}

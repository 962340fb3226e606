/*
 * CPU oracle for the block-wise causal attention of Next-Frame Diffusion.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * attention computes; it shares no code, header, table or helper with the HIP
 * library and is never on the product path.  Only the test-suite, the smoke
 * check and the benchmark's cpu_baseline leg may build or call it.
 *
 * Everything is fp64.  Inputs are the exact values the device kernel receives
 * (bf16 / fp32 widen to fp64 without rounding).
 *
 * The mask follows the paper's "Block-wise Causal Attention" paragraph
 * (Sec. 3.1): a token attends to every token of its own frame and to every
 * token of all preceding frames, never to a later frame.  The queries are the
 * last q_frames of the kv_frames frames present, as in the speculative
 * sampling listing of Appendix A (a chunk of new frames is appended at the end
 * and only those frames are produced) and in the KV-cache paragraph of
 * Appendix B (past frames' K/V are reused, only the new frames are queried).
 * Softmax is the ordinary one with natural exponent; the paper does not write
 * it out.
 *
 * Pins (tests/test_oracle_pins.py): reduction to textbook causal attention at
 * T=1 and to full attention at one frame (both against independent numpy and
 * a library SDPA), brute force over an explicit mask matrix, uniform-score
 * closed form (mean of visible V), future-perturbation invariance, cached /
 * speculative forms equal to the tail rows of the full form, visible-pair
 * count closed form, permutation and convexity invariants, one-hot limit and
 * large-magnitude stability; for the rotary embedding: complex-multiplication
 * form of textbook 1-D RoPE, identity at the origin, norm preservation,
 * dependence of rotated dot products on position differences only, section
 * independence, quarter-turn closed form.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* Frame-block visibility (Sec. 3.1, "Block-wise Causal Attention").
 * Query row i lives in query-frame i/T, which is absolute frame P + i/T where
 * P = kv_frames - q_frames past frames precede the first query frame.
 * Key j lives in absolute frame j/T.  Visible iff key frame <= query frame. */
static int visible(int64_t i, int64_t j, int64_t T, int64_t P)
{
    return (j / T) <= (P + i / T);
}

/*
 * out[b,h,r,:] = sum_j w_j v[b,h,j,:] / sum_j w_j,   w_j = M_ij exp(s_ij - m_i)
 * s_ij = scale * <q[b,h,i,:], k[b,h,j,:]>,  m_i = max over visible j of s_ij,
 * where i = rows[r] (or r when rows == NULL).
 *
 * q   : [B, H, q_frames*T, D]        k, v : [B, H, F*T, D]  (first kv_frames*T rows used)
 * out : [B, H, n_out, D], n_out = n_rows if rows != NULL else q_frames*T
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int nfd_oracle_block_causal_attn(const double *q, const double *k, const double *v,
                                 double *out, int B, int H, int F, int T, int D,
                                 int kv_frames, int q_frames, double scale,
                                 const int64_t *rows, int64_t n_rows)
{
    if (!q || !k || !v || !out) return -1;
    if (B < 1 || H < 1 || T < 1 || D < 1 || q_frames < 1) return -1;
    if (q_frames > kv_frames || kv_frames > F) return -1;

    const int64_t Sq = (int64_t)q_frames * T;
    const int64_t Sk = (int64_t)kv_frames * T;
    const int64_t Scap = (int64_t)F * T;
    const int64_t P = (int64_t)kv_frames - q_frames;
    const int64_t n_out = rows ? n_rows : Sq;
    if (rows) {
        for (int64_t r = 0; r < n_rows; ++r)
            if (rows[r] < 0 || rows[r] >= Sq) return -1;
    }
    int failed = 0;

#pragma omp parallel
    {
        double *w = (double *)malloc((size_t)Sk * sizeof(double));
        unsigned char *M = (unsigned char *)malloc((size_t)Sk);
        if (!w || !M) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for collapse(2) schedule(dynamic, 8)
            for (int64_t bh = 0; bh < (int64_t)B * H; ++bh) {
                for (int64_t r = 0; r < n_out; ++r) {
                    const int64_t i = rows ? rows[r] : r;
                    const double *qi = q + (bh * Sq + i) * D;
                    const double *kb = k + bh * Scap * D;
                    const double *vb = v + bh * Scap * D;
                    double *o = out + (bh * n_out + r) * D;

                    /* explicit boolean mask row, then masked scores */
                    double m = -INFINITY;
                    for (int64_t j = 0; j < Sk; ++j) {
                        M[j] = (unsigned char)visible(i, j, T, P);
                        if (!M[j]) { w[j] = 0.0; continue; }
                        double s = 0.0;
                        for (int d = 0; d < D; ++d) s += qi[d] * kb[j * D + d];
                        s *= scale;
                        w[j] = s;
                        if (s > m) m = s;
                    }
                    double denom = 0.0;
                    for (int d = 0; d < D; ++d) o[d] = 0.0;
                    for (int64_t j = 0; j < Sk; ++j) {
                        if (!M[j]) continue;
                        const double e = exp(w[j] - m);
                        denom += e;
                        for (int d = 0; d < D; ++d) o[d] += e * vb[j * D + d];
                    }
                    for (int d = 0; d < D; ++d) o[d] /= denom;
                }
            }
        }
        free(w);
        free(M);
    }
    return failed ? -1 : 0;
}

/*
 * Gradients of the attention above with respect to q, k and v, for an upstream
 * gradient dout of the output (the paper trains through this attention:
 * Sec. 3.2 "Training"; the mask is the one of Sec. 3.1).  Written out from the
 * definition, element by element:
 *
 *   p_ij   = M_ij exp(s_ij) / sum_l M_il exp(s_il)          (softmax over visible keys)
 *   dv_j   = sum_i p_ij dout_i
 *   dp_ij  = <dout_i, v_j>
 *   ds_ij  = p_ij (dp_ij - sum_l p_il dp_il)                 (Jacobian of the softmax)
 *   dq_i   = scale sum_j ds_ij k_j          dk_j = scale sum_i ds_ij q_i
 *
 * dq : [B, H, q_frames*T, D]; dk, dv : [B, H, F*T, D] (rows at and past kv_frames*T are set to 0);
 * lse (optional, may be NULL) : [B, H, q_frames*T] = log sum_l M_il exp(s_il).
 */
int nfd_oracle_block_causal_attn_bwd(const double *q, const double *k, const double *v,
                                     const double *dout, double *dq, double *dk, double *dv,
                                     double *lse, int B, int H, int F, int T, int D, int kv_frames,
                                     int q_frames, double scale)
{
    if (!q || !k || !v || !dout || !dq || !dk || !dv) return -1;
    if (B < 1 || H < 1 || T < 1 || D < 1 || q_frames < 1) return -1;
    if (q_frames > kv_frames || kv_frames > F) return -1;
    const int64_t Sq = (int64_t)q_frames * T, Sk = (int64_t)kv_frames * T, Scap = (int64_t)F * T;
    const int64_t P = (int64_t)kv_frames - q_frames;
    const int64_t BH = (int64_t)B * H;
    double *L = (double *)malloc((size_t)(BH * Sq) * sizeof(double));   /* log of the row's softmax denominator */
    double *G = (double *)malloc((size_t)(BH * Sq) * sizeof(double));   /* sum_l p_il dp_il */
    if (!L || !G) { free(L); free(G); return -1; }
    int failed = 0;

    /* rows: p_i., dp_i., the row's Jacobian term, dq_i */
#pragma omp parallel
    {
        double *p = (double *)malloc((size_t)Sk * sizeof(double));
        double *dp = (double *)malloc((size_t)Sk * sizeof(double));
        if (!p || !dp) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for collapse(2) schedule(dynamic, 8)
            for (int64_t bh = 0; bh < BH; ++bh)
                for (int64_t i = 0; i < Sq; ++i) {
                    const double *qi = q + (bh * Sq + i) * D, *gi = dout + (bh * Sq + i) * D;
                    const double *kb = k + bh * Scap * D, *vb = v + bh * Scap * D;
                    double m = -INFINITY;
                    for (int64_t j = 0; j < Sk; ++j) {
                        if (!visible(i, j, T, P)) { p[j] = 0.0; continue; }
                        double s = 0.0;
                        for (int d = 0; d < D; ++d) s += qi[d] * kb[j * D + d];
                        p[j] = s * scale;
                        if (p[j] > m) m = p[j];
                    }
                    double denom = 0.0;
                    for (int64_t j = 0; j < Sk; ++j)
                        if (visible(i, j, T, P)) { p[j] = exp(p[j] - m); denom += p[j]; }
                    double g = 0.0;
                    for (int64_t j = 0; j < Sk; ++j) {
                        dp[j] = 0.0;
                        if (!visible(i, j, T, P)) continue;
                        p[j] /= denom;
                        for (int d = 0; d < D; ++d) dp[j] += gi[d] * vb[j * D + d];
                        g += p[j] * dp[j];
                    }
                    L[bh * Sq + i] = m + log(denom);
                    G[bh * Sq + i] = g;
                    double *dqi = dq + (bh * Sq + i) * D;
                    for (int d = 0; d < D; ++d) dqi[d] = 0.0;
                    for (int64_t j = 0; j < Sk; ++j) {
                        if (!visible(i, j, T, P)) continue;
                        const double ds = p[j] * (dp[j] - g);
                        for (int d = 0; d < D; ++d) dqi[d] += scale * ds * kb[j * D + d];
                    }
                }
        }
        free(p);
        free(dp);
    }

    /* keys: dv_j and dk_j gather over the rows that see key j */
    if (!failed) {
#pragma omp parallel for collapse(2) schedule(dynamic, 8)
        for (int64_t bh = 0; bh < BH; ++bh)
            for (int64_t j = 0; j < Scap; ++j) {
                double *dkj = dk + (bh * Scap + j) * D, *dvj = dv + (bh * Scap + j) * D;
                for (int d = 0; d < D; ++d) { dkj[d] = 0.0; dvj[d] = 0.0; }
                if (j >= Sk) continue;
                const double *kj = k + (bh * Scap + j) * D, *vj = v + (bh * Scap + j) * D;
                for (int64_t i = 0; i < Sq; ++i) {
                    if (!visible(i, j, T, P)) continue;
                    const double *qi = q + (bh * Sq + i) * D, *gi = dout + (bh * Sq + i) * D;
                    double s = 0.0, dpij = 0.0;
                    for (int d = 0; d < D; ++d) { s += qi[d] * kj[d]; dpij += gi[d] * vj[d]; }
                    const double pij = exp(s * scale - L[bh * Sq + i]);
                    const double ds = pij * (dpij - G[bh * Sq + i]);
                    for (int d = 0; d < D; ++d) { dvj[d] += pij * gi[d]; dkj[d] += scale * ds * qi[d]; }
                }
            }
    }
    if (lse && !failed) memcpy(lse, L, (size_t)(BH * Sq) * sizeof(double));
    free(L);
    free(G);
    return failed ? -1 : 0;
}

/*
 * KV cache write (Appendix B, "KV Caching": K/V of frames are computed once
 * and reused).  Copies n_frames new frames into the cache at frame frame_pos.
 * cache : [B, H, F*T, D]   fresh : [B, H, n_frames*T, D]
 */
int nfd_oracle_kvcache_append(double *cache, const double *fresh, int B, int H,
                              int F, int T, int D, int frame_pos, int n_frames)
{
    if (!cache || !fresh) return -1;
    if (B < 1 || H < 1 || T < 1 || D < 1 || n_frames < 0 || frame_pos < 0) return -1;
    if (frame_pos + n_frames > F) return -1;
    const int64_t rowsz = (int64_t)T * D;
    for (int64_t bh = 0; bh < (int64_t)B * H; ++bh)
        for (int64_t f = 0; f < n_frames; ++f)
            memcpy(cache + (bh * F + frame_pos + f) * rowsz,
                   fresh + (bh * n_frames + f) * rowsz, (size_t)rowsz * sizeof(double));
    return 0;
}

/*
 * 3D rotary position embedding of the queries and keys of n_frames new frames,
 * with the rotated keys and the (unchanged) values written into the cache
 * (Sec. 3.1, paragraph "3D Positional Embedding": the head dimension of query
 * and key tokens is separated into [n_T, n_H, n_W]; rotary frequency
 * embeddings are computed for each axis separately and concatenated along the
 * last dimension; Appendix B "KV Caching" for the cache write).
 *
 * Readings where the paper is silent:
 *  - a token's position is (t, y, x): t = t_offset + frame_pos + its frame
 *    among the new ones, and (y, x) = (token / grid_w, token % grid_w) on the
 *    grid_h x grid_w latent grid, T = grid_h * grid_w, row-major;
 *  - inside the section of an axis of width n the feature pairs are the
 *    ADJACENT ones (2i, 2i+1), i = 0 .. n/2-1, pair i turning by the angle
 *    position * theta^(-2i/n);
 *  - the rotation is the counter-clockwise one:
 *    (a, b) -> (a cos - b sin, a sin + b cos).
 * The sections lie in the order T, H, W along the head dimension; a section of
 * width 0 is allowed; every width is even; n_t + n_h + n_w = D.
 *
 * q, q_out : [B, H, n_frames*T, D]       k_new, v_new : [B, H, n_frames*T, D]
 * k_cache, v_cache : [B, H, F*T, D]
 */
int nfd_oracle_rope_kvcache_append(const double *q, double *q_out, double *k_cache, double *v_cache,
                                   const double *k_new, const double *v_new, int B, int H, int F,
                                   int T, int D, int frame_pos, int n_frames, int t_offset,
                                   int grid_h, int grid_w, int n_t, int n_h, int n_w, double theta)
{
    if (!q || !q_out || !k_cache || !v_cache || !k_new || !v_new) return -1;
    if (B < 1 || H < 1 || T < 1 || D < 1 || n_frames < 0 || frame_pos < 0) return -1;
    if (frame_pos + n_frames > F) return -1;
    if (grid_h < 1 || grid_w < 1 || (int64_t)grid_h * grid_w != T) return -1;
    if (n_t < 0 || n_h < 0 || n_w < 0 || (n_t | n_h | n_w) & 1 || n_t + n_h + n_w != D) return -1;
    if (!(theta > 0.0)) return -1;
    const int width[3] = {n_t, n_h, n_w};
    for (int64_t bh = 0; bh < (int64_t)B * H; ++bh)
        for (int f = 0; f < n_frames; ++f)
            for (int tok = 0; tok < T; ++tok) {
                const double pos[3] = {(double)(t_offset + frame_pos + f), (double)(tok / grid_w),
                                       (double)(tok % grid_w)};
                const int64_t src = ((bh * n_frames + f) * T + tok) * D;
                const int64_t dst = ((bh * F + frame_pos + f) * T + tok) * D;
                int d0 = 0;
                for (int ax = 0; ax < 3; ++ax) {
                    const int n = width[ax];
                    for (int i = 0; i < n / 2; ++i) {
                        const double ang = pos[ax] * pow(theta, -2.0 * (double)i / (double)n);
                        const double cs = cos(ang), sn = sin(ang);
                        const int e = d0 + 2 * i;
                        const double qa = q[src + e], qb = q[src + e + 1];
                        const double ka = k_new[src + e], kb = k_new[src + e + 1];
                        q_out[src + e] = qa * cs - qb * sn;
                        q_out[src + e + 1] = qa * sn + qb * cs;
                        k_cache[dst + e] = ka * cs - kb * sn;
                        k_cache[dst + e + 1] = ka * sn + kb * cs;
                    }
                    d0 += n;
                }
                for (int e = 0; e < D; ++e) v_cache[dst + e] = v_new[src + e];
            }
    return 0;
}

/* Number of visible (query, key) pairs per (b, h), by direct enumeration of
 * the mask (used to state FLOP counts; closed form is checked in the tests). */
int64_t nfd_oracle_visible_pairs(int T, int kv_frames, int q_frames)
{
    const int64_t Sq = (int64_t)q_frames * T, Sk = (int64_t)kv_frames * T;
    const int64_t P = (int64_t)kv_frames - q_frames;
    int64_t n = 0;
    for (int64_t i = 0; i < Sq; ++i)
        for (int64_t j = 0; j < Sk; ++j) n += visible(i, j, T, P);
    return n;
}

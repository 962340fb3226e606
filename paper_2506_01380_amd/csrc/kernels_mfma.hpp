// bf16 matrix-core forward kernel for head width 64 (gfx950 / CDNA4).
//
// Flash-style online softmax.  A workgroup of NW wavefronts owns NW*64 consecutive
// query rows of one (batch, head); each wavefront owns 64 of them as two 32-wide
// column blocks of the TRANSPOSED score matrix:
//
//   S^T[key, query] = K_tile[key, :] . Q^T[:, query]       v_mfma_f32_32x32x16_bf16, A = K (LDS), B = Q^T (registers)
//   O^T[d,   query] += V_tile^T[d, key] . P^T[key, query]  A = V^T (LDS, transposing read), B = P^T (registers)
//
// In the 32x32 accumulator layout a lane holds ONE query column (lane % 32) and 16 of the
// 32 key rows, so row max / row sum are register-local plus a single exchange with
// lane ^ 32, and the accumulator registers of S^T are already in the B-operand layout
// the second product needs: P never goes through LDS.
//
// Mask (Sec. 3.1): row i sees keys j < kmax(i) = (P + i/T + 1) * T.  Key tiles entirely
// below every row's bound run with no mask arithmetic; tiles at or beyond the largest
// bound of the workgroup are never visited; only the tiles in between compare the key
// index with the lane's bound.
#pragma once
#include "nfd_common.hpp"

namespace nfd {
namespace mfma {

constexpr int kD = 64;     // head width
constexpr int kBN = 64;    // keys per tile
constexpr int kKStr = 72;  // LDS row stride of the K tile in bf16 elements (144 B)
constexpr int kVStr = 72;  // LDS row stride of the V tile
constexpr float kRescaleThreshold = 8.0f;  // log2 units the running max may lag behind

__device__ __forceinline__ bf16x8 lds_read_b128(const __bf16* p) { return *(const bf16x8*)p; }

// Transposing LDS read: the 16 lanes of a group present a 4-row x 16-column block
// (lane s -> row s/4, columns 4*(s%4)..+3); lane i receives column i of the 4 rows.
__device__ __forceinline__ s16x4 lds_read_tr(const __bf16* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p));
}

template <int NW>
struct Smem {
    __bf16 k[2][kBN * kKStr];
    __bf16 v[2][kBN * kVStr];
};

// Work decomposition of one launch.  Workgroup ids are dealt round-robin to the 8 XCDs;
// heads are pinned to an XCD (bh % 8) so that all query tiles and key splits of a head
// share one L2, and inside an XCD the heaviest query tiles (latest frames) come first.
struct WorkItem {
    int bh, q_tile, split;
    bool valid;
};
__device__ __forceinline__ WorkItem decode_work(const FwdParams& p) {
    WorkItem w;
    const int per_head = p.n_q_tiles * p.n_splits;
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int heads_here = p.BH / 8 + (xcd < (p.BH & 7) ? 1 : 0);
    w.valid = heads_here > 0 && j < heads_here * per_head;
    const int item = heads_here > 0 ? j / heads_here : 0;
    const int head_local = heads_here > 0 ? j % heads_here : 0;
    w.bh = head_local * 8 + xcd;
    w.q_tile = p.n_q_tiles - 1 - item / p.n_splits;
    w.split = item % p.n_splits;
    return w;
}

template <int NW>
__global__ void __launch_bounds__(NW * 64, 2)
attn_fwd_bf16_d64(FwdParams p) {
    constexpr int BM = NW * 64;
    constexpr int NTHREADS = NW * 64;
    constexpr int CHUNKS = kBN * kD / 8;  // 16-byte chunks per K or V tile (512)
    constexpr int LD_ITERS = (CHUNKS + NTHREADS - 1) / NTHREADS;
    __shared__ Smem<NW> sm;

    const WorkItem wi = decode_work(p);
    if (!wi.valid) return;  // whole workgroup leaves together

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int n = lane & 31, h = lane >> 5;
    const int r0 = wi.q_tile * BM;                       // first query row of the workgroup
    const int r_last = min(r0 + BM, p.Sq) - 1;           // last valid row
    const int kmax_wg = kmax_of_row(r_last, p.T, p.P);   // keys visited by this workgroup
    const int n_tiles = (kmax_wg + kBN - 1) / kBN;
    const int tiles_per_split = (n_tiles + p.n_splits - 1) / p.n_splits;
    const int t_begin = wi.split * tiles_per_split;
    const int t_end = min(t_begin + tiles_per_split, n_tiles);

    const __bf16* qg = (const __bf16*)p.q + (int64_t)wi.bh * p.Sq * kD;
    const __bf16* kg = (const __bf16*)p.k + (int64_t)wi.bh * p.Scap * kD;
    const __bf16* vg = (const __bf16*)p.v + (int64_t)wi.bh * p.Scap * kD;

    // ---- this wavefront's queries -------------------------------------------------------
    const int rw0 = r0 + wv * 64;
    int row[2], kmax_lane[2];
    bf16x8 qf[2][4];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        row[qt] = rw0 + 32 * qt + n;
        const int rc = min(row[qt], p.Sq - 1);  // ragged tail: compute a duplicate, never store it
        kmax_lane[qt] = kmax_of_row(rc, p.T, p.P);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) qf[qt][ks] = *(const bf16x8*)(qg + (int64_t)rc * kD + 16 * ks + 8 * h);
    }
    const int rw_first = min(rw0, p.Sq - 1), rw_last = min(rw0 + 63, p.Sq - 1);
    const int kmin_wave = kmax_of_row(rw_first, p.T, p.P);  // tiles ending at or below need no mask
    const int kmax_wave = kmax_of_row(rw_last, p.T, p.P);   // tiles starting at or above are skipped
    const bool wave_active = rw0 < p.Sq;

    f32x16 o_acc[2][2];  // [dt][qt]: O^T rows 32*dt.., query block qt
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) o_acc[a][b][r] = 0.f;
    float m_used[2] = {kNegBig, kNegBig};  // reference max, raw score units (stale by design)
    float l_sum[2] = {0.f, 0.f};           // this lane's share of the row sum
    const float c = p.scale_log2e;

    // ---- global -> register -> LDS staging of one K and one V tile ---------------------------
    u32x4 kreg[LD_ITERS], vreg[LD_ITERS];
    auto load_tile = [&](int tile) {
        const int j0 = tile * kBN;
#pragma unroll
        for (int it = 0; it < LD_ITERS; ++it) {
            const int ch = tid + it * NTHREADS;
            if (CHUNKS % NTHREADS == 0 || ch < CHUNKS) {
                const int kr = min(j0 + (ch >> 3), p.Sk - 1);  // clamp: rows past the end are masked anyway
                const int64_t off = (int64_t)kr * kD + (ch & 7) * 8;
                kreg[it] = *(const u32x4*)(kg + off);
                vreg[it] = *(const u32x4*)(vg + off);
            }
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int it = 0; it < LD_ITERS; ++it) {
            const int ch = tid + it * NTHREADS;
            if (CHUNKS % NTHREADS == 0 || ch < CHUNKS) {
                *(u32x4*)(&sm.k[buf][(ch >> 3) * kKStr + (ch & 7) * 8]) = kreg[it];
                *(u32x4*)(&sm.v[buf][(ch >> 3) * kVStr + (ch & 7) * 8]) = vreg[it];
            }
        }
    };

    if (t_begin < t_end) {
        load_tile(t_begin);
        store_tile(0);
    }
    __syncthreads();

    // lane-constant LDS offsets
    const int k_off = n * kKStr + 8 * h;                                   // + 32*kb rows, + 16*ks cols
    const int s16 = lane & 15, dblk = (lane >> 4) & 1;
    const int v_off = (4 * h + (s16 >> 2)) * kVStr + 16 * dblk + 4 * (s16 & 3);  // + (32kb+16g [+8]) rows, + 32*dt cols

    for (int t = t_begin; t < t_end; ++t) {
        const int buf = (t - t_begin) & 1;
        const int j0 = t * kBN;
        const bool has_next = t + 1 < t_end;
        if (has_next) load_tile(t + 1);

        if (wave_active && j0 < kmax_wave) {
            const __bf16* ks_ = sm.k[buf];
            const __bf16* vs_ = sm.v[buf];
            // ---- S^T = K . Q^T ----------------------------------------------------------------
            f32x16 s_acc[2][2];  // [kb][qt]
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int qt = 0; qt < 2; ++qt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) s_acc[kb][qt][r] = 0.f;
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const bf16x8 a = lds_read_b128(ks_ + k_off + 32 * kb * kKStr + 16 * ks);
#pragma unroll
                    for (int qt = 0; qt < 2; ++qt)
                        s_acc[kb][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[qt][ks], s_acc[kb][qt], 0, 0, 0);
                }
            }
            // ---- mask (only tiles that cross some row's bound) ---------------------------------
            if (j0 + kBN > kmin_wave) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int qt = 0; qt < 2; ++qt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int key = j0 + 32 * kb + 8 * (r >> 2) + 4 * h + (r & 3);
                            if (key >= kmax_lane[qt]) s_acc[kb][qt][r] = -INFINITY;
                        }
            }
            // ---- online softmax, lane-local per query column ----------------------------------
            float mx[2];
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) {
                float a = fmaxf(s_acc[0][qt][0], s_acc[1][qt][0]);
#pragma unroll
                for (int r = 1; r < 16; ++r) a = fmaxf(fmaxf(a, s_acc[0][qt][r]), s_acc[1][qt][r]);
                a = fmaxf(a, __shfl_xor(a, 32));
                mx[qt] = fmaxf(a, m_used[qt]);
            }
            // Rescale only when some row's max outgrew the reference by more than the threshold;
            // until then p may exceed 1 (by at most 2^threshold), which fp32 sums and bf16 P hold.
            const bool grow = ((mx[0] - m_used[0]) * c > kRescaleThreshold) | ((mx[1] - m_used[1]) * c > kRescaleThreshold);
            if (__builtin_amdgcn_ballot_w64(grow) != 0) {
#pragma unroll
                for (int qt = 0; qt < 2; ++qt) {
                    const float alpha = __builtin_amdgcn_exp2f((m_used[qt] - mx[qt]) * c);
                    m_used[qt] = mx[qt];
                    l_sum[qt] *= alpha;
#pragma unroll
                    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) o_acc[dt][qt][r] *= alpha;
                }
            }
            // ---- P = exp2(c*s - c*m), bf16; row sums from the rounded values ------------------------
            bf16x8 pf[2][2][2];  // [kb][g][qt]
            const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) {
                const float mc = m_used[qt] * c;
                float l = l_sum[qt];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int g = 0; g < 2; ++g) {
#pragma unroll
                        for (int jj = 0; jj < 4; ++jj) {
                            const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[kb][qt][8 * g + 2 * jj], c, -mc));
                            const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[kb][qt][8 * g + 2 * jj + 1], c, -mc));
                            const f32x2 pp = {p0, p1};
                            const bf16x2 pb = __builtin_convertvector(pp, bf16x2);
                            l = __builtin_amdgcn_fdot2_f32_bf16(pb, ones, l, false);
                            pf[kb][g][qt][2 * jj] = pb[0];
                            pf[kb][g][qt][2 * jj + 1] = pb[1];
                        }
                    }
                l_sum[qt] = l;
            }
            // ---- O^T += V^T . P^T -----------------------------------------------------------------
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int g = 0; g < 2; ++g)
#pragma unroll
                    for (int dt = 0; dt < 2; ++dt) {
                        const __bf16* vp = vs_ + v_off + (32 * kb + 16 * g) * kVStr + 32 * dt;
                        const s16x4 lo = lds_read_tr(vp);
                        const s16x4 hi = lds_read_tr(vp + 8 * kVStr);
                        typedef __attribute__((ext_vector_type(8))) short s16x8;
                        const s16x8 av = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                        const bf16x8 a = __builtin_bit_cast(bf16x8, av);
#pragma unroll
                        for (int qt = 0; qt < 2; ++qt)
                            o_acc[dt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[kb][g][qt], o_acc[dt][qt], 0, 0, 0);
                    }
        }

        if (has_next) store_tile(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue -----------------------------------------------------------------------------
    if (!wave_active) return;
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        const float l_row = l_sum[qt] + __shfl_xor(l_sum[qt], 32);
        if (row[qt] >= p.Sq) continue;
        if (p.n_splits == 1) {
            const float inv = 1.0f / l_row;
            __bf16* og = (__bf16*)p.out + ((int64_t)wi.bh * p.Sq + row[qt]) * kD;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int rb = 0; rb < 4; ++rb) {
                    const f32x4 x = {o_acc[dt][qt][4 * rb] * inv, o_acc[dt][qt][4 * rb + 1] * inv,
                                     o_acc[dt][qt][4 * rb + 2] * inv, o_acc[dt][qt][4 * rb + 3] * inv};
                    const bf16x4 y = __builtin_convertvector(x, bf16x4);
                    *(bf16x4*)(og + 32 * dt + 8 * rb + 4 * h) = y;
                }
        } else {
            const int64_t prow = ((int64_t)wi.bh * p.n_splits + wi.split) * p.Sq + row[qt];
            float* po = p.part_o + prow * kD;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int rb = 0; rb < 4; ++rb) {
                    const f32x4 x = {o_acc[dt][qt][4 * rb], o_acc[dt][qt][4 * rb + 1], o_acc[dt][qt][4 * rb + 2],
                                     o_acc[dt][qt][4 * rb + 3]};
                    *(f32x4*)(po + 32 * dt + 8 * rb + 4 * h) = x;
                }
            if (h == 0) {
                const f32x2 ml = {m_used[qt] * c, l_row};
                *(f32x2*)(p.part_ml + prow * 2) = ml;
            }
        }
    }
}

// Merge the key-split partials of one query row: out = sum_s w_s O_s / sum_s w_s l_s with
// w_s = 2^(m_s - max_s m_s).  One thread per (row, 4 output columns).
__global__ void __launch_bounds__(256)
attn_combine_d64(FwdParams p) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t total = (int64_t)p.BH * p.Sq * (kD / 4);
    if (idx >= total) return;
    const int dq = (int)(idx % (kD / 4));
    const int64_t r = idx / (kD / 4);
    const int bh = (int)(r / p.Sq), i = (int)(r % p.Sq);
    float mmax = kNegBig;
    for (int s = 0; s < p.n_splits; ++s) {
        const int64_t prow = ((int64_t)bh * p.n_splits + s) * p.Sq + i;
        mmax = fmaxf(mmax, p.part_ml[prow * 2]);
    }
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float l = 0.f;
    for (int s = 0; s < p.n_splits; ++s) {
        const int64_t prow = ((int64_t)bh * p.n_splits + s) * p.Sq + i;
        const float w = __builtin_amdgcn_exp2f(p.part_ml[prow * 2] - mmax);
        l += w * p.part_ml[prow * 2 + 1];
        const f32x4 o = *(const f32x4*)(p.part_o + prow * kD + 4 * dq);
        acc += w * o;
    }
    const float inv = 1.0f / l;
    const f32x4 x = acc * inv;
    const bf16x4 y = __builtin_convertvector(x, bf16x4);
    *(bf16x4*)((__bf16*)p.out + r * kD + 4 * dq) = y;
}

}  // namespace mfma
}  // namespace nfd

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

// Wait for every outstanding vector-memory load of this wavefront.  Used once after the Q
// fragments are fetched: otherwise the compiler, unable to prove they have landed on every
// path into the main loop, guards each matrix instruction that reads them with an in-order
// vmcnt wait, and those waits would drain the K/V prefetch issued just before.
__device__ __forceinline__ void wait_vmem_all() { __builtin_amdgcn_s_waitcnt(0x0F70); }

template <int NW>
struct __attribute__((aligned(16))) Smem {
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

// Final write of one wavefront's 64 query rows: normalised bf16 output when the keys were not
// split, otherwise the unnormalised fp32 accumulator plus (reference max in log2 units, row sum).
// Lane (n, h) holds, for query column n of block qt, output features 32*dt + 8*rb + 4*h + 0..3.
__device__ __forceinline__ void store_rows(const FwdParams& p, const WorkItem& wi, const int (&row)[2], int h,
                                           const f32x16 (&o_acc)[2][2], const float (&l_sum)[2],
                                           const float (&m_used)[2], float c) {
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
    wait_vmem_all();
    __syncthreads();

    // lane-constant LDS offsets
    const int k_off = n * kKStr + 8 * h;                                   // + 32*kb rows, + 16*ks cols
    const int s16 = lane & 15, dblk = (lane >> 4) & 1;
    const int v_off = (4 * h + (s16 >> 2)) * kVStr + 16 * dblk + 4 * (s16 & 3);  // + (32kb+16g [+8]) rows, + 32*dt cols

#ifdef NFD_STAGE_TIMING
    unsigned long long tsum[5] = {0, 0, 0, 0, 0}, tc0, tc1;
#define NFD_TICK(i) { __builtin_amdgcn_s_waitcnt(0); tc1 = __builtin_readcyclecounter(); tsum[i] += tc1 - tc0; tc0 = tc1; }
    tc0 = __builtin_readcyclecounter();
#else
#define NFD_TICK(i)
#endif
    for (int t = t_begin; t < t_end; ++t) {
        const int buf = (t - t_begin) & 1;
        const int j0 = t * kBN;
        const bool has_next = t + 1 < t_end;
        if (has_next) load_tile(t + 1);
        NFD_TICK(0)

        if (wave_active && j0 < kmax_wave) {
            const __bf16* ks_ = sm.k[buf];
            const __bf16* vs_ = sm.v[buf];
            // ---- S^T = K . Q^T: all eight K fragments are requested before the first product so the
            // LDS latency is paid once per tile, not once per fragment ------------------------------
            f32x16 s_acc[2][2];  // [kb][qt]
            bf16x8 kf[2][4];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) kf[kb][ks] = lds_read_b128(ks_ + k_off + 32 * kb * kKStr + 16 * ks);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int qt = 0; qt < 2; ++qt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) s_acc[kb][qt][r] = 0.f;
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
                    for (int qt = 0; qt < 2; ++qt)
                        s_acc[kb][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kb][ks], qf[qt][ks], s_acc[kb][qt], 0, 0, 0);
                }
            }
            // V^T fragments for the second product are requested now and land during the softmax.
            bf16x8 vf[2][2][2];  // [kb][g][dt]
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
                        vf[kb][g][dt] = __builtin_bit_cast(bf16x8, av);
                    }
            __builtin_amdgcn_sched_barrier(0);
            NFD_TICK(1)
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
            // ---- P = exp2(c*s - c*m), bf16; row sums in fp32 (plain adds: the packed dot
    // instruction shares the matrix pipe and would stall the other wavefront's MFMAs) ------------------------
            bf16x8 pf[2][2][2];  // [kb][g][qt]
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) {
                const float mc = m_used[qt] * c;
                float l = l_sum[qt], l2 = 0.f;
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
                            l += p0;
                            l2 += p1;
                            pf[kb][g][qt][2 * jj] = pb[0];
                            pf[kb][g][qt][2 * jj + 1] = pb[1];
                        }
                    }
                l_sum[qt] = l + l2;
            }
            NFD_TICK(2)
            // ---- O^T += V^T . P^T -----------------------------------------------------------------
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int g = 0; g < 2; ++g)
#pragma unroll
                    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                        for (int qt = 0; qt < 2; ++qt)
                            o_acc[dt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[kb][g][dt], pf[kb][g][qt], o_acc[dt][qt], 0, 0, 0);
        }

        NFD_TICK(3)
        if (has_next) store_tile(buf ^ 1);
        __syncthreads();
        NFD_TICK(4)
    }
#ifdef NFD_STAGE_TIMING
    if (p.timing && lane == 0) {
        unsigned long long* o = p.timing + ((size_t)blockIdx.x * NW + wv) * 8;
        for (int i = 0; i < 5; ++i) o[i] = tsum[i];
        o[5] = (unsigned long long)(t_end - t_begin);
    }
#endif

    // ---- epilogue -----------------------------------------------------------------------------
    if (!wave_active) return;
    store_rows(p, wi, row, h, o_acc, l_sum, m_used, c);
}

// ---------------------------------------------------------------------------------------------
// Ping-pong variant: 8 wavefronts = two groups of 4.  Wavefront w of group A and wavefront w of
// group B own the SAME 64 query rows and share a SIMD; group A takes the even key tiles of the
// workgroup's range, group B the odd ones, each with its own accumulators, and the two are
// merged through LDS at the end.  Time is cut into barrier-delimited intervals; in every
// interval one group runs its matrix-core stage (P.V of its previous tile, then K.Q^T of its
// next tile) while the other runs its softmax stage on the vector ALU, so the MFMA pipe and
// the VALU of a SIMD are busy at the same time instead of taking turns.
//
// Softmax is optimistic: P is formed against the reference max of earlier tiles without first
// looking at this tile's max; only if a lane's tile sum reaches kOptimisticLimit (which also
// catches inf, i.e. the very first tile) the tile is redone with its exact max and the
// accumulators are rescaled.  Row sums come from the bf16-rounded P, so numerator and
// denominator see the same values.
// ---------------------------------------------------------------------------------------------
constexpr int kPPWaves = 8;
constexpr int kPPBM = 256;
constexpr int kKSlots = 2, kVSlots = 4;
constexpr float kOptimisticLimit = 32768.0f;  // 2^15 per lane and tile (32 values)

struct __attribute__((aligned(16))) SmemPP {
    union {
        struct {
            __bf16 k[kKSlots][kBN * kKStr];
            __bf16 v[kVSlots][kBN * kVStr];
        } t;
        float merge[4 * 64 * 36];  // one query block of group B: [wave][9 vec4][lane][4]
    };
};

// The loop body of both groups is straight-line code: every stage runs in every interval.  The
// pipeline's fill and drain intervals and the tiles a wavefront cannot see are handled by data,
// not by branches: P starts as zero, V slots start as zero, and a tile that must not contribute
// is given a key offset beyond every row's bound so that the mask zeroes its P.  This keeps the
// lifetimes of S, P and the operand fragments short and evident to the register allocator.
// DBG is 0 in the product; development builds instantiate variants that leave out one piece of work
// (results are then wrong) to see what each piece costs in situ.
template <int DBG>
__global__ void __launch_bounds__(kPPWaves * 64, 2)
attn_fwd_bf16_d64_pp(FwdParams p) {
    __shared__ SmemPP sm;
    const WorkItem wi = decode_work(p);
    if (!wi.valid) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave >> 2, wq = wave & 3;
    const int n = lane & 31, h = lane >> 5;
    const int r0 = wi.q_tile * kPPBM;
    const int r_last = min(r0 + kPPBM, p.Sq) - 1;
    const int kmax_wg = kmax_of_row(r_last, p.T, p.P);
    const int n_tiles = (kmax_wg + kBN - 1) / kBN;
    const int tiles_per_split = (n_tiles + p.n_splits - 1) / p.n_splits;
    const int t_begin = wi.split * tiles_per_split;
    const int n_local = max(0, min(t_begin + tiles_per_split, n_tiles) - t_begin);

    const __bf16* qg = (const __bf16*)p.q + (int64_t)wi.bh * p.Sq * kD;
    const __bf16* kg = (const __bf16*)p.k + (int64_t)wi.bh * p.Scap * kD;
    const __bf16* vg = (const __bf16*)p.v + (int64_t)wi.bh * p.Scap * kD;

    const int rw0 = r0 + wq * 64;
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
    const int kmin_wave = kmax_of_row(min(rw0, p.Sq - 1), p.T, p.P);
    const bool wave_active = rw0 < p.Sq;

    f32x16 o_acc[2][2], s_acc[2][2];
    bf16x8 pf[2][2][2];  // [kb][g][qt]
    bf16x8 vf[2][2][2];  // [kb][g][dt]
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
#pragma unroll
            for (int r = 0; r < 16; ++r) { o_acc[a][b][r] = 0.f; s_acc[a][b][r] = 0.f; }
#pragma unroll
            for (int e = 0; e < 2; ++e)
#pragma unroll
                for (int x = 0; x < 8; ++x) { pf[a][b][e][x] = (__bf16)0.0f; vf[a][b][e][x] = (__bf16)0.0f; }
        }
    float m_used[2] = {kNegBig, kNegBig};
    float l_sum[2] = {0.f, 0.f};
    const float c = p.scale_log2e;

    // V slots start as zeros: the fill intervals multiply them by P = 0 and must not meet NaN bits.
    {
        u32x4* vz = (u32x4*)&sm.t.v[0][0];
        const u32x4 z = {0u, 0u, 0u, 0u};
        for (int i = tid; i < kVSlots * kBN * kVStr / 8; i += kPPWaves * 64) vz[i] = z;
    }

    u32x4 kreg, vreg;
    auto load_tile = [&](int i) {  // rows past the end are clamped: they are masked anyway
        const int kr = min((t_begin + i) * kBN + (tid >> 3), p.Sk - 1);
        const int64_t off = (int64_t)kr * kD + (tid & 7) * 8;
        if (DBG & 1) return;
        kreg = *(const u32x4*)(kg + off);
        vreg = *(const u32x4*)(vg + off);
    };
    auto store_tile = [&](int i) {
        if (DBG & 2) return;
        *(u32x4*)(&sm.t.k[i & (kKSlots - 1)][(tid >> 3) * kKStr + (tid & 7) * 8]) = kreg;
        *(u32x4*)(&sm.t.v[i & (kVSlots - 1)][(tid >> 3) * kVStr + (tid & 7) * 8]) = vreg;
    };
    const int k_off = n * kKStr + 8 * h;
    const int s16 = lane & 15, dblk = (lane >> 4) & 1;
    const int v_off = (4 * h + (s16 >> 2)) * kVStr + 16 * dblk + 4 * (s16 & 3);

    // Requested at the end of the softmax stage, so the LDS latency hides behind the barrier.
    auto read_v_frags = [&](int i) {
        if (DBG & 4) return;
        const __bf16* vs_ = sm.t.v[i & (kVSlots - 1)];
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
                    vf[kb][g][dt] = __builtin_bit_cast(bf16x8, av);
                }
    };
    auto pv_half = [&](int kb) {
        if (DBG & 32) return;
#pragma unroll
        for (int g = 0; g < 2; ++g)
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int qt = 0; qt < 2; ++qt)
                    o_acc[dt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[kb][g][dt], pf[kb][g][qt], o_acc[dt][qt], 0, 0, 0);
    };
    // Matrix-core stage: O^T += V^T . P^T of the group's previous tile, then S^T = K . Q^T of its
    // next tile i_qk.  The K fragments are requested while the first product is still issuing.
    auto stage_mfma = [&](int i_qk) {
        bf16x8 kf[2][4];
        // The matrix stage outranks the other group's softmax in instruction arbitration: its MFMAs then
        // issue the moment the pipe frees up and the softmax's VALU work fills the cycles in between.
        __builtin_amdgcn_s_setprio(3);
        pv_half(0);
        __builtin_amdgcn_sched_barrier(0);
        const __bf16* ks_ = sm.t.k[i_qk & (kKSlots - 1)];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                if (DBG & 8) kf[kb][ks] = vf[kb][ks >> 1][ks & 1];
                else kf[kb][ks] = lds_read_b128(ks_ + k_off + 32 * kb * kKStr + 16 * ks);
            }
        __builtin_amdgcn_sched_barrier(0);
        pv_half(1);
        __builtin_amdgcn_sched_barrier(0);
        if (!(DBG & 32))
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int qt = 0; qt < 2; ++qt)
#pragma unroll
                for (int r = 0; r < 16; ++r) s_acc[kb][qt][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int qt = 0; qt < 2; ++qt)
                    s_acc[kb][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kb][ks], qf[qt][ks], s_acc[kb][qt], 0, 0, 0);
        }
        __builtin_amdgcn_s_setprio(0);
    };
    auto form_p = [&]() {  // P = exp2(c*s - c*m_used) in bf16, row sums in fp32 (plain adds: the packed dot
    // instruction shares the matrix pipe and would stall the other wavefront's MFMAs)
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
            const float mc = m_used[qt] * c;
            float l = l_sum[qt], l2 = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int g = 0; g < 2; ++g)
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) {
                        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[kb][qt][8 * g + 2 * jj], c, -mc));
                        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[kb][qt][8 * g + 2 * jj + 1], c, -mc));
                        const f32x2 pp = {p0, p1};
                        const bf16x2 pb = __builtin_convertvector(pp, bf16x2);
                        l += p0;
                        l2 += p1;
                        pf[kb][g][qt][2 * jj] = pb[0];
                        pf[kb][g][qt][2 * jj + 1] = pb[1];
                    }
            l_sum[qt] = l + l2;
        }
    };
#ifdef NFD_STAGE_TIMING
    unsigned long long tsum[8] = {0, 0, 0, 0, 0, 0, 0, 0}, tc0, tc1;
#define NFD_TOCK2(i) { __builtin_amdgcn_s_waitcnt(0xc07f); tc1 = __builtin_readcyclecounter(); tsum[i] += tc1 - tc0; tc0 = tc1; }
#else
#define NFD_TOCK2(i)
#endif
    // Softmax stage of local tile i (S in s_acc -> P in pf); a tile index outside the split's range
    // is given an offset beyond every bound, which masks it completely.
    auto stage_softmax = [&](int i) {
        const int j0 = (i >= 0 && i < n_local) ? (t_begin + i) * kBN : 0x3fffff00;
        if (__builtin_amdgcn_readfirstlane(j0 + kBN > kmin_wave)) {  // tile crosses some row's bound
            asm volatile("" ::: "memory");  // keep this rare block a branch; do not if-convert it into every tile
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
        const float l_old0 = l_sum[0], l_old1 = l_sum[1];
        if (DBG & 16) return;
        form_p();
        const bool bad = !(l_sum[0] - l_old0 < kOptimisticLimit) | !(l_sum[1] - l_old1 < kOptimisticLimit);
        if (__builtin_amdgcn_ballot_w64(bad) != 0) {  // exact path: this tile's max, rescale, redo
#ifdef NFD_STAGE_TIMING
            tsum[4] += 1;
#endif
            l_sum[0] = l_old0;
            l_sum[1] = l_old1;
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) {
                float a = fmaxf(s_acc[0][qt][0], s_acc[1][qt][0]);
#pragma unroll
                for (int r = 1; r < 16; ++r) a = fmaxf(fmaxf(a, s_acc[0][qt][r]), s_acc[1][qt][r]);
                a = fmaxf(a, __shfl_xor(a, 32));
                const float m_new = fmaxf(a, m_used[qt]);
                const float alpha = __builtin_amdgcn_exp2f((m_used[qt] - m_new) * c);
                m_used[qt] = m_new;
                l_sum[qt] *= alpha;
#pragma unroll
                for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o_acc[dt][qt][r] *= alpha;
            }
            form_p();
        }
    };

    load_tile(0);
    store_tile(0);
    wait_vmem_all();
    __syncthreads();

    // Interval nn: group (nn & 1) runs P.V of tile nn-2 and K.Q^T of tile nn; the other group runs
    // the softmax of tile nn-1 and fetches that tile's V fragments.  Everybody stages tile nn+1 and
    // meets at a barrier.  Tile i belongs to group (i & 1).  K(i) is read in interval i and its slot
    // (2 slots) rewritten in interval i+1; V(i) is read at the end of interval i+1 and its slot
    // (4 slots) rewritten in interval i+3.
    const int n_iter = n_local > 0 ? (n_local + 3) / 2 : 0;
#ifdef NFD_STAGE_TIMING
#define NFD_TOCK(i) { __builtin_amdgcn_s_waitcnt(0xc07f); tc1 = __builtin_readcyclecounter(); tsum[i] += tc1 - tc0; tc0 = tc1; }
    tc0 = __builtin_readcyclecounter();
#else
#define NFD_TOCK(i)
#endif
    if (grp == 0) {
        for (int it = 0; it < n_iter; ++it) {
            const int nn = 2 * it;
            load_tile(nn + 1);
            stage_mfma(nn);
            NFD_TOCK(0)
            store_tile(nn + 1);
            __syncthreads();
            NFD_TOCK(1)
            load_tile(nn + 2);
            stage_softmax(nn);
            read_v_frags(nn);
            NFD_TOCK(2)
            store_tile(nn + 2);
            __syncthreads();
            NFD_TOCK(3)
        }
    } else {
        for (int it = 0; it < n_iter; ++it) {
            const int nn = 2 * it;
            load_tile(nn + 1);
            stage_softmax(nn - 1);
            read_v_frags(nn - 1);
            NFD_TOCK(2)
            store_tile(nn + 1);
            __syncthreads();
            NFD_TOCK(3)
            load_tile(nn + 2);
            stage_mfma(nn + 1);
            NFD_TOCK(0)
            store_tile(nn + 2);
            __syncthreads();
            NFD_TOCK(1)
        }
    }
#ifdef NFD_STAGE_TIMING
    if (p.timing && lane == 0) {
        unsigned long long* o = p.timing + ((size_t)blockIdx.x * kPPWaves + wave) * 8;
        for (int i = 0; i < 5; ++i) o[i] = tsum[i];
        o[5] = (unsigned long long)(2 * n_iter);
        o[6] = tsum[5];
        o[7] = tsum[6];
    }
#endif
    __syncthreads();

    // ---- merge group B into group A (one 32-query block at a time through LDS), then store --------
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        const float l_row = l_sum[qt] + __shfl_xor(l_sum[qt], 32);
        float* mb = sm.merge + wq * (64 * 36);
        if (grp == 1) {
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int rb = 0; rb < 4; ++rb) {
                    const f32x4 x = {o_acc[dt][qt][4 * rb], o_acc[dt][qt][4 * rb + 1], o_acc[dt][qt][4 * rb + 2],
                                     o_acc[dt][qt][4 * rb + 3]};
                    *(f32x4*)(mb + ((dt * 4 + rb) * 64 + lane) * 4) = x;
                }
            const f32x4 ml = {m_used[qt], l_row, 0.f, 0.f};
            *(f32x4*)(mb + (8 * 64 + lane) * 4) = ml;
        }
        __syncthreads();
        if (grp == 0 && wave_active) {
            const f32x4 ml = *(const f32x4*)(mb + (8 * 64 + lane) * 4);
            const float m_all = fmaxf(m_used[qt], ml[0]);
            const float wa = __builtin_amdgcn_exp2f((m_used[qt] - m_all) * c);
            const float wb = __builtin_amdgcn_exp2f((ml[0] - m_all) * c);
            const float l_all = l_row * wa + ml[1] * wb;
            const bool store_row = row[qt] < p.Sq;
            float scale_out = 1.0f;
            if (p.n_splits == 1) scale_out = 1.0f / l_all;
            const float fa = wa * scale_out, fb = wb * scale_out;
            __bf16* og = (__bf16*)p.out + ((int64_t)wi.bh * p.Sq + row[qt]) * kD;
            const int64_t prow = ((int64_t)wi.bh * p.n_splits + wi.split) * p.Sq + row[qt];
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int rb = 0; rb < 4; ++rb) {
                    const f32x4 ob = *(const f32x4*)(mb + ((dt * 4 + rb) * 64 + lane) * 4);
                    const f32x4 x = {o_acc[dt][qt][4 * rb] * fa + ob[0] * fb, o_acc[dt][qt][4 * rb + 1] * fa + ob[1] * fb,
                                     o_acc[dt][qt][4 * rb + 2] * fa + ob[2] * fb, o_acc[dt][qt][4 * rb + 3] * fa + ob[3] * fb};
                    if (store_row) {
                        if (p.n_splits == 1) {
                            const bf16x4 y = __builtin_convertvector(x, bf16x4);
                            *(bf16x4*)(og + 32 * dt + 8 * rb + 4 * h) = y;
                        } else {
                            *(f32x4*)(p.part_o + prow * kD + 32 * dt + 8 * rb + 4 * h) = x;
                        }
                    }
                }
            if (p.n_splits > 1 && store_row && h == 0) {
                const f32x2 o2 = {m_all * c, l_all};
                *(f32x2*)(p.part_ml + prow * 2) = o2;
            }
        }
        __syncthreads();
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

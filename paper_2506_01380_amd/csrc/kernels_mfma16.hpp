// The 256-row throughput shape of the forward kernel over a bf16 cache (64 query rows per wavefront), on the 16x16x32
// shape of the bf16 matrix instruction.
//
// Same decomposition, tile ring, swizzle, mask handling and optimistic softmax as the shapes in kernels_mfma.hpp (read
// its header first); what differs is the register layout, a software-pipelined tile loop, and row sums formed on
// the matrix pipe.  v_mfma_f32_16x16x32_bf16: A[i][k] sits in lane i + 16 (k / 8), element k % 8;
// B[k][j] in lane j + 16 (k / 8), element k % 8; D[i][j] in lane j + 16 (i / 4), element i % 4.  With lane = (j, g),
// j = lane % 16, g = lane / 16:
//
//   S^T[key, query] = K . Q^T   A = K rows 16 rb + j, features 32 ks + 8 g ..   (one 16-byte LDS read)
//                               B = Q^T: query 16 cq + j, the same features     (registers, whole kernel)
//                               D: query 16 cq + j, operand rows 4 g + e, e = 0..3
//   O^T[d, query] += V^T . P^T  A = V^T: feature 16 fb + j, keys at positions (g, 0..7) of a 32-key step
//                               B = P^T: query 16 cq + j, the same positions
//                               D: query 16 cq + j, features 16 fb + 4 g + e
// Operand row i of a 16-key block is key 4 sg(i / 4) + i % 4 of it, sg = (0, 2, 3, 1), so lane group g holds keys
// 4 sg(g) .. + 3.  The order is chosen for the LDS banks under the tile swizzle: a 16-byte read is served in groups
// of sixteen lanes ({0-3, 12-15, 20-23, 24-27}, {4-7, 8-11, 16-19, 28-31}, the same + 32) that here mix two feature
// chunks, an 8-byte read in halves of the wavefront (lane groups 0, 1 and 2, 3); with this order every such group
// touches sixteen different 16-byte bank groups for the K fragments as well as for the V^T fragments (the plain
// order collides in pairs on both: 8.0 M conflict cycles on 24 M LDS cycles at 16 frames of 336 tokens).
// Position (g, m) of the 32-key step kb is key 32 kb + 4 sg(g) + m for m < 4 and 32 kb + 16 + 4 sg(g) + (m - 4)
// otherwise: exactly the eight scores lane (j, g) holds of the step's two 16-key blocks, so P goes from the
// accumulators of the first product into the B operand of the second unchanged, and the transposing LDS read (16
// lanes present 4 rows x 16 columns, lane i receives column i) delivers V^T in the same order, two reads a fragment.
// A lane owns one query column in each of four 16-query blocks (cq = 0..3: two per 32-row block), shared with the
// three lanes j + 16, j + 32, j + 48: row max / row sum are register-local plus two exchanges at the very end.
#pragma once
#include "kernels_mfma.hpp"

namespace nfd {
namespace mfma {

// Four-register slice fb of a sixteen-register accumulator.  The accumulators of one query column are kept as one
// sixteen-register value: the rare rescale is then a partial update of a value too large to be worth copying, and the
// allocator leaves it where it is (as four independent values it was moved at every join of the rare and common paths).
template <int FB>
__device__ __forceinline__ f32x4 acc_slice(const f32x16& v) {
    return __builtin_shufflevector(v, v, 4 * FB, 4 * FB + 1, 4 * FB + 2, 4 * FB + 3);
}
template <int FB>
__device__ __forceinline__ void acc_set(f32x16& v, const f32x4& x) {
#pragma unroll
    for (int e = 0; e < 4; ++e) v[4 * FB + e] = x[e];
}
// v.slice(FB) += A . B
template <int FB>
__device__ __forceinline__ void acc_mfma(f32x16& v, const bf16x8& a, const bf16x8& b) {
    acc_set<FB>(v, __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc_slice<FB>(v), 0, 0, 0));
}

template <bool EXACTQ>
__device__ __forceinline__ void attn_fwd_item16(const FwdParams& p, const WorkItem& wi, SmemRingPipe& sm) {
    constexpr int PRIO = kMfmaPriority;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 15, g = lane >> 4;
    auto sg = [](int x) { return (0x78 >> (2 * x)) & 3; };  // 0, 2, 3, 1: see the header
    int blk0, n_blk;
    q_tile_blocks(wi.q_tile, p.blocks_lo, p.n_hi, &blk0, &n_blk);
    const int r0 = 32 * blk0;
    const int r_last = min(r0 + 32 * n_blk, p.Sq) - 1;
    const int kmax_wg = kmax_of_row(r_last, p.T, p.P);
    const int n_tiles = (kmax_wg + kBN - 1) / kBN;
    const int tiles_per_split = (n_tiles + p.n_splits - 1) / p.n_splits;
    const int t_begin = wi.split * tiles_per_split;
    const int t_end = min(t_begin + tiles_per_split, n_tiles);

    const __bf16* qg = (const __bf16*)p.q + (int64_t)wi.bh * p.Sq * kD;
    const __bf16* kg = (const __bf16*)p.k + (int64_t)wi.bh * p.Scap * kD;
    const __bf16* vg = (const __bf16*)p.v + (int64_t)wi.bh * p.Scap * kD;
    const bool fused = p.k_new != nullptr;
    const __bf16* kn = fused ? (const __bf16*)p.k_new + ((int64_t)wi.bh * p.Sq - p.Snew0) * kD : kg;
    const __bf16* vn = fused ? (const __bf16*)p.v_new + ((int64_t)wi.bh * p.Sq - p.Snew0) * kD : vg;
    constexpr int kMaxCopy = 4;
    u32x4 cp_k[kMaxCopy], cp_v[kMaxCopy];
    int64_t cp_dst[kMaxCopy];
    if (fused) {
        const int64_t n_vec = (int64_t)p.BH * p.Sq * (kD / 8), n_thr = (int64_t)gridDim.x * blockDim.x;
        const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
#pragma unroll
        for (int i = 0; i < kMaxCopy; ++i) {
            const int64_t x = gid + i * n_thr;
            cp_dst[i] = -1;
            if (x < n_vec) {
                const int64_t per_head = (int64_t)p.Sq * (kD / 8);
                const int64_t bh = x / per_head, rem = x - bh * per_head;
                cp_dst[i] = (bh * p.Scap + p.Snew0) * (kD / 8) + rem;
                cp_k[i] = ((const u32x4*)p.k_new)[x];
                cp_v[i] = ((const u32x4*)p.v_new)[x];
            }
        }
    }

    // ---- this wavefront's queries: 32-row blocks `wave` and `wave + 4` (or one block, as the later one) -------
    const float c = p.scale_log2e;
    int b0_blk[2];                 // [qt]: first row of the block, or a row no tensor has (dead block)
    int kmin_blk[2], kmax_blk[2];  // [qt]
    bf16x8 qf[4][2];               // [cq][ks]
    // row of this lane's query column cq and its key bound: recomputed where needed (masked tiles, the final write)
    // rather than kept in registers through the loops
    auto row_of = [&](int cq) { return b0_blk[cq >> 1] + 16 * (cq & 1) + j; };
    auto kmax_lane_of = [&](int cq) { return kmax_of_row(min(row_of(cq), p.Sq - 1), p.T, p.P); };
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        const bool pair = wave + kWaves < n_blk;
        const bool dead = qt == 0 && !pair;
        const int b0 = r0 + 32 * (qt == 1 && pair ? wave + kWaves : wave);
        b0_blk[qt] = dead ? 0x40000000 : b0;
        kmin_blk[qt] = dead ? 0 : kmax_of_row(min(b0, p.Sq - 1), p.T, p.P);
        kmax_blk[qt] = dead ? 0 : kmax_of_row(min(b0 + 31, p.Sq - 1), p.T, p.P);
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            const int cq = 2 * qt + cb;
            const int rc = min(row_of(cq), p.Sq - 1);
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const bf16x8 raw = *(const bf16x8*)(qg + (int64_t)rc * kD + 32 * ks + 8 * g);
                if constexpr (EXACTQ) {
                    qf[cq][ks] = raw;
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) qf[cq][ks][e] = (__bf16)((float)raw[e] * c);
                }
            }
        }
    }
    const int kmax_wave = kmax_blk[1];
    const bool wave_active = wave < n_blk;

    f32x16 o_acc[4];  // [cq], element 4 fb + e: feature 16 fb + 4 g + e
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[a][r] = 0.f;
    // Row sums.  MSUM (the plain forward): the second product also multiplies P^T by a block of ones, so the sum of a
    // column of a unit's P - of the bf16 values the output is formed from - comes out of the matrix pipe (in all four
    // elements of the result, in every lane group) and costs the vector unit one add per column instead of sixteen
    // (the tile loop is bound by vector issue: 16 of its 48 instructions per step were these adds).  The result is
    // added to l_sum at once rather than accumulated in place: four persistent registers per column do not fit.  The reference then sits kRefBias above the maximum seen, so that
    // "some P >= 2" (one bit of the packed values, OR-ed together) is a rare event that still leaves 2^119 of range.
    // EXACTQ (the training pair, whose log-sum-exp the backward normalises with) keeps fp32 sums of the unrounded
    // values on the vector unit and the test on them.
    constexpr bool MSUM = !EXACTQ;
    constexpr float kRefBias = MSUM ? 8.f : 0.f;
    float m_used[4], l_sum[4];  // [cq]; m_used in accumulator units (raw scores with EXACTQ)
    bf16x8 ones;
#pragma unroll
    for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;
    asm volatile("" : "+v"(ones));  // keep it in registers: rebuilt from constants it costs two moves per step
#pragma unroll
    for (int cq = 0; cq < 4; ++cq) { m_used[cq] = kNegBig; l_sum[cq] = 0.f; }
    // some value of the two packed operands is >= 2 (or not a number): bit 14 of a bf16 is the top exponent bit
    auto any_big = [](const bf16x8& a, const bf16x8& b) {
        const u32x4 x = __builtin_bit_cast(u32x4, a), y = __builtin_bit_cast(u32x4, b);
        return ((x[0] | x[1] | x[2] | x[3] | y[0] | y[1] | y[2] | y[3]) & 0x40004000u) != 0;
    };

    // ---- tile loads (as in the 32x32 item) -----------------------------------------------------------------
    const int ld_row = 8 * wave + (lane >> 3);
    const int ld_chunk = (lane & 7) ^ chunk_swizzle(ld_row);
    const unsigned ld_voff[2] = {(unsigned)(ld_row * kD + ld_chunk * 8) * 2u, (unsigned)((ld_row + 32) * kD + ld_chunk * 8) * 2u};
    const int ld_plain_end = min(p.Sk, p.Snew0);
    const unsigned lds_k0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)(&sm.k[0][0]) + wave * 1024;
    const unsigned lds_v0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)(&sm.v[0][0]) + wave * 1024;
    auto load_tile = [&](int t, int slot) {
        if ((t + 1) * kBN <= ld_plain_end) {
            const __bf16* kt = kg + (int64_t)t * kTileElems;
            const __bf16* vt = vg + (int64_t)t * kTileElems;
#pragma unroll
            for (int pass = 0; pass < 2; ++pass) {
                const unsigned kdst = lds_k0 + (unsigned)(slot * kTileElems * 2 + pass * 4096);
                const unsigned vdst = lds_v0 + (unsigned)(slot * kTileElems * 2 + pass * 4096);
                asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(ld_voff[pass]), "s"(kt), "s"(kdst) : "memory", "m0");
                asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(ld_voff[pass]), "s"(vt), "s"(vdst) : "memory", "m0");
            }
            return;
        }
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            const int kr = min(t * kBN + 32 * pass + ld_row, p.Sk - 1);
            const int64_t off = (int64_t)kr * kD + ld_chunk * 8;
            const bool from_new = kr >= p.Snew0;
            const unsigned kdst = lds_k0 + (unsigned)(slot * kTileElems * 2 + pass * 4096);
            const unsigned vdst = lds_v0 + (unsigned)(slot * kTileElems * 2 + pass * 4096);
            asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"((from_new ? kn : kg) + off), "s"(kdst) : "memory", "m0");
            asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"((from_new ? vn : vg) + off), "s"(vdst) : "memory", "m0");
        }
    };

    // ---- per-lane fragment offsets (elements) under the swizzle -----------------------------------------------
    // K: operand row j of a 16-key block is key row k_row (the swizzle of a row depends on it alone), chunk 4 ks + g.
    const int k_row = 4 * sg(j >> 2) + (j & 3);
    const int fk = chunk_swizzle(k_row);
    int k_off[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) k_off[ks] = k_row * kD + 8 * ((4 * ks + g) ^ fk);
    // V^T: lane s = j of group g presents row 4 sg(g) + s / 4 (+ 32 kb + 16 half), columns 16 fb + 4 (s % 4) ..
    const int v_row = 4 * sg(g) + (j >> 2);
    const int fv = chunk_swizzle(v_row);  // rows + 16, + 32: the same swizzle
    int v_off[4];                         // [fb]
#pragma unroll
    for (int fb = 0; fb < 4; ++fb) v_off[fb] = v_row * kD + 8 * ((2 * fb + ((j & 3) >> 1)) ^ fv) + 4 * (j & 1);

    if (t_begin < t_end) load_tile(t_begin, 0);
    if (t_begin + 1 < t_end) load_tile(t_begin + 1, 1);
    if (t_begin + 2 < t_end) load_tile(t_begin + 2, 2);
    wait_vmem_all();
    if (fused) {
#pragma unroll
        for (int i = 0; i < kMaxCopy; ++i)
            if (cp_dst[i] >= 0) {
                ((u32x4*)p.k)[cp_dst[i]] = cp_k[i];
                ((u32x4*)p.v)[cp_dst[i]] = cp_v[i];
            }
    }

    auto to_exponent = [&](float s, float ref_exponent) {
        if constexpr (EXACTQ) return __builtin_fmaf(s, c, -ref_exponent);
        else return s - ref_exponent;
    };
    auto read_v_frag = [&](const __bf16* tile, int kb, int fb) {  // V^T fragment of the 32-key step kb, features 16 fb ..
        const __bf16* vp = tile + 32 * kb * kD + v_off[fb];
        const s16x4 lo = lds_read_tr(vp);
        const s16x4 hi = lds_read_tr(vp + 16 * kD);
        typedef __attribute__((ext_vector_type(8))) short s16x8;
        return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    auto pack_p = [&](const f32x4& a, const f32x4& b) {  // positions 0..3 from the first 16-key block, 4..7 from the second
        bf16x8 r;
#pragma unroll
        for (int e = 0; e < 4; e += 2) {
            const f32x2 x = {a[e], a[e + 1]}, y = {b[e], b[e + 1]};
            const bf16x2 xb = __builtin_convertvector(x, bf16x2), yb = __builtin_convertvector(y, bf16x2);
            r[e] = xb[0]; r[e + 1] = xb[1]; r[4 + e] = yb[0]; r[5 + e] = yb[1];
        }
        return r;
    };

    // ---- one whole tile at a time (tiles at the frame bounds, tiles only the later block sees), one 32-row block
    // of the wavefront per call: these tiles are few, and half the scores at a time keep the register peak of this
    // path below that of the pipelined loop (a value that finds no register here is reloaded at every use, there too)
    auto tile_body = [&](int t, int slot, auto qt_tag) {
        constexpr int C0 = 2 * decltype(qt_tag)::value, C1 = C0 + 2;  // this block's query columns
        const int j0 = t * kBN;
        const __bf16* ks_ = sm.k[slot];
        const __bf16* vs_ = sm.v[slot];
        bf16x8 kf[4][2];  // [rb][ks]
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) kf[rb][ks] = lds_read_b128(ks_ + 16 * rb * kD + k_off[ks]);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(PRIO);
        f32x4 s_acc[4][4];  // [rb][cq]
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
#pragma unroll
            for (int cq = C0; cq < C1; ++cq) {
#pragma unroll
                for (int e = 0; e < 4; ++e) s_acc[rb][cq][e] = 0.f;
#pragma unroll
                for (int ks = 0; ks < 2; ++ks)
                    s_acc[rb][cq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[rb][ks], qf[cq][ks], s_acc[rb][cq], 0, 0, 0);
            }
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(0);
        if (j0 + kBN > kmin_blk[C0 / 2]) {
#pragma unroll
            for (int cq = C0; cq < C1; ++cq) {
                const int left = kmax_lane_of(cq) - (j0 + 4 * sg(g));  // visible keys from this lane's first of the tile
#pragma unroll
                for (int rb = 0; rb < 4; ++rb)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (16 * rb + e >= left) s_acc[rb][cq][e] = -INFINITY;
            }
        }
        bf16x8 pf[2][4];  // [kb][cq]
        float l_tile[4];
        auto form_p = [&]() {
#pragma unroll
            for (int cq = C0; cq < C1; ++cq) {
                const float mc = EXACTQ ? m_used[cq] * c : m_used[cq];
                float l = 0.f, l2 = 0.f;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    f32x4 pa, pb;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        pa[e] = __builtin_amdgcn_exp2f(to_exponent(s_acc[2 * kb][cq][e], mc));
                        pb[e] = __builtin_amdgcn_exp2f(to_exponent(s_acc[2 * kb + 1][cq][e], mc));
                        l += pa[e];
                        l2 += pb[e];
                    }
                    pf[kb][cq] = pack_p(pa, pb);
                }
                l_tile[cq] = l + l2;
            }
        };
        bool bad = true;
        if (t != t_begin) {
            form_p();
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = C0; b < C1; ++b) asm volatile("" : "+v"(pf[a][b]));
            bad = false;
#pragma unroll
            for (int cq = C0; cq < C1; ++cq) {
                if constexpr (MSUM) bad |= any_big(pf[0][cq], pf[1][cq]);
                else bad |= !(l_tile[cq] < kOptimisticLimit);
            }
        }
        bf16x8 vf[2][4];  // [kb][fb]
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int fb = 0; fb < 4; ++fb) vf[kb][fb] = read_v_frag(vs_, kb, fb);
        if (__builtin_amdgcn_ballot_w64(bad) != 0) {
#pragma unroll
            for (int cq = C0; cq < C1; ++cq) {
                float a = s_acc[0][cq][0];
#pragma unroll
                for (int rb = 0; rb < 4; ++rb)
#pragma unroll
                    for (int e = 0; e < 4; ++e) a = fmaxf(a, s_acc[rb][cq][e]);
                a = fmaxf(a, __shfl_xor(a, 16));
                a = fmaxf(a, __shfl_xor(a, 32));
                const float m_new = fmaxf(a + kRefBias, m_used[cq]);
                const float alpha = __builtin_amdgcn_exp2f(EXACTQ ? (m_used[cq] - m_new) * c : m_used[cq] - m_new);
                m_used[cq] = m_new;
                l_sum[cq] *= alpha;
#pragma unroll
                for (int r = 0; r < 16; ++r) o_acc[cq][r] *= alpha;
            }
            form_p();
        }
        if constexpr (!MSUM)
#pragma unroll
            for (int cq = C0; cq < C1; ++cq) l_sum[cq] += l_tile[cq];
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(PRIO);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int cq = C0; cq < C1; ++cq) {
                acc_mfma<0>(o_acc[cq], vf[kb][0], pf[kb][cq]);
                acc_mfma<1>(o_acc[cq], vf[kb][1], pf[kb][cq]);
                acc_mfma<2>(o_acc[cq], vf[kb][2], pf[kb][cq]);
                acc_mfma<3>(o_acc[cq], vf[kb][3], pf[kb][cq]);
                if constexpr (MSUM) {
                    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
                    l_sum[cq] += __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pf[kb][cq], zero, 0, 0, 0)[0];
                }
            }
        __builtin_amdgcn_sched_barrier(0);
    };

    // ---- software-pipelined tile loop ------------------------------------------------------------------------------
    // A key tile is four units (kb, qt): 32 keys x one 32-row query block.  Unit u = 2 kb + qt needs
    //   QK(u): 8 MFMA  S[qt] = K[kb] . Q[qt]^T - reference      (the reference enters as the MFMA's C operand)
    //   SM(u): 16 exp2, 8 packed conversions per lane (and 16 adds without MSUM)   P[qt] = exp2(S[qt])
    //   PV(u): 8 MFMA  O[qt] += V[kb]^T . P[qt]^T               (+ 2 for the row sums with MSUM)
    // and step u of the loop issues QK(u+1), SM(u) and PV(u-1) together: the two MFMA groups belong to the other
    // query block, so nothing in a step depends on anything else in it and the MFMAs interleave with the vector
    // instructions of the softmax inside one wavefront.  Consecutive units alternate between the blocks.
    // Only tiles that both blocks see entirely (no mask) run here; the few tiles at the frame bounds and the
    // tiles only the later block sees run through tile_body afterwards.
    //
    // Ring contract (both loops): Bar(t), one barrier per tile t.  A wavefront arrives when its own loads of tile
    // t+1 have landed and it no longer reads tile t-1; after Bar(t) tile t+1 is visible to all and every wavefront
    // requests tile t+3 into the slot of tile t-1.  The pipelined loop passes Bar(t) after its first step of tile t
    // (which still reads V of tile t-1), tile_body's loop at the top of tile t.
    const int t_mid = wave_active ? max(t_begin, min(t_end, (kmax_blk[0] + kBN - 1) / kBN)) : t_begin;
    int t_pipe = wave_active ? max(t_begin, min(t_mid, kmin_blk[0] / kBN)) : t_begin;
    if (t_pipe - t_begin < 2) t_pipe = t_begin;
    auto bar = [&](int t, auto load_slot) {  // load_slot: the ring slot of tile t + 3 (an int or a compile-time constant)
        if (t + 2 < t_end) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        if (t + 3 < t_end) load_tile(t + 3, (int)load_slot);
        // Key-split launches: the wave priority falls with the quarter of the chain the workgroup is in, so that of
        // two workgroups sharing a CU the one that lags is served first and both finish together (the arbiter
        // otherwise prefers the older one throughout: 52 against 70 us at four speculative frames).  Training
        // launches keep one level: there a CU's workgroups differ in length and start time anyway, and changing
        // levels costs 1-2 %.
        if (p.n_splits > 1) {
            const int done4 = (t - t_begin) * 4, len = t_end - t_begin;
            if (done4 < len) __builtin_amdgcn_s_setprio(3);
            else if (done4 < 2 * len) __builtin_amdgcn_s_setprio(2);
            else if (done4 < 3 * len) __builtin_amdgcn_s_setprio(1);
            else __builtin_amdgcn_s_setprio(0);
        }
    };
    __builtin_amdgcn_s_barrier();

    if (t_pipe > t_begin) {
        f32x4 S[2][2][2];      // [qt][rb'][cb]: the unit in flight of each 32-row block
        f32x4 minit[4];        // [cq]: minus the reference, the C operand of the first product
        bf16x8 P[2][2];        // [qt][cb]
        bf16x8 kf[2][2][2];    // [kb][rb'][ks]
        bf16x8 vf[2][4];       // [kb][fb]
#pragma unroll
        for (int cq = 0; cq < 4; ++cq)
#pragma unroll
            for (int e = 0; e < 4; ++e) minit[cq][e] = 0.f;
#pragma unroll
        for (int qt = 0; qt < 2; ++qt)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                for (int e = 0; e < 8; ++e) P[qt][cb][e] = (__bf16)0.f;
#pragma unroll
        for (int fb = 0; fb < 4; ++fb)
#pragma unroll
            for (int e = 0; e < 8; ++e) vf[1][fb][e] = (__bf16)0.f;  // the first step's PV adds 0 . 0
        auto read_k = [&](int slot, int kb) {
            const __bf16* ks_ = sm.k[slot] + 32 * kb * kD;
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) kf[kb][rb][ks] = lds_read_b128(ks_ + 16 * rb * kD + k_off[ks]);
        };
        auto read_v = [&](int slot, int kb) {
            const __bf16* vs_ = sm.v[slot];
#pragma unroll
            for (int fb = 0; fb < 4; ++fb) vf[kb][fb] = read_v_frag(vs_, kb, fb);
        };
        auto qk = [&](int kb, int qt) {
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int cb = 0; cb < 2; ++cb)
                    S[qt][rb][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kb][rb][0], qf[2 * qt + cb][0], minit[2 * qt + cb], 0, 0, 0);
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int cb = 0; cb < 2; ++cb)
                    S[qt][rb][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kb][rb][1], qf[2 * qt + cb][1], S[qt][rb][cb], 0, 0, 0);
        };
        auto pv = [&](int kb, int qt) {
            if constexpr (MSUM) {  // the unit's column sums first: their adds then find room later in the same step
                const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int cb = 0; cb < 2; ++cb)
                    l_sum[2 * qt + cb] += __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, P[qt][cb], zero, 0, 0, 0)[0];
            }
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                acc_mfma<0>(o_acc[2 * qt + cb], vf[kb][0], P[qt][cb]);
                acc_mfma<1>(o_acc[2 * qt + cb], vf[kb][1], P[qt][cb]);
                acc_mfma<2>(o_acc[2 * qt + cb], vf[kb][2], P[qt][cb]);
                acc_mfma<3>(o_acc[2 * qt + cb], vf[kb][3], P[qt][cb]);
            }
        };
        // softmax of one unit: P[qt][cb] from S[qt][.][cb] minus `sub[cb]` (accumulator units); lu: the lane's sums
        auto sm_unit = [&](int qt, const float (&sub)[2], float (&lu)[2], bool subtract) {
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                float l = 0.f, l2 = 0.f;
#pragma unroll
                for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                    for (int e = 0; e < 4; e += 2) {
                        float x0 = S[qt][rb][cb][e], x1 = S[qt][rb][cb][e + 1];
                        if (subtract) { x0 -= sub[cb]; x1 -= sub[cb]; }
                        if constexpr (EXACTQ) { x0 *= c; x1 *= c; }
                        const float p0 = __builtin_amdgcn_exp2f(x0), p1 = __builtin_amdgcn_exp2f(x1);
                        const f32x2 pp = {p0, p1};
                        const bf16x2 pb = __builtin_convertvector(pp, bf16x2);
                        l += p0;
                        l2 += p1;
                        P[qt][cb][4 * rb + e] = pb[0];
                        P[qt][cb][4 * rb + e + 1] = pb[1];
                    }
                lu[cb] = l + l2;
            }
        };
        const float no_sub[2] = {0.f, 0.f};
        // After SM(u): if the unit's test fails (or the unit is a block's first), take the unit's exact max, move the
        // reference, rescale the block's accumulators and form P again.  S[qt] is still intact.
        auto settle = [&](int qt, float (&lu)[2], bool fresh) {
            const bool bad = fresh || (MSUM ? any_big(P[qt][0], P[qt][1]) : !(lu[0] < kOptimisticLimit) || !(lu[1] < kOptimisticLimit));
            if (__builtin_amdgcn_ballot_w64(bad) != 0) {
                float up[2];
#pragma unroll
                for (int cb = 0; cb < 2; ++cb) {
                    const int cq = 2 * qt + cb;
                    float a = S[qt][0][cb][0];
#pragma unroll
                    for (int e = 0; e < 4; ++e) a = fmaxf(a, fmaxf(S[qt][0][cb][e], S[qt][1][cb][e]));
                    a = fmaxf(a, __shfl_xor(a, 16));
                    a = fmaxf(a, __shfl_xor(a, 32));  // relative to the current reference
                    up[cb] = fresh ? a + kRefBias : fmaxf(a + kRefBias, 0.f);
                    const float alpha = fresh ? 0.f : __builtin_amdgcn_exp2f(EXACTQ ? -up[cb] * c : -up[cb]);
                    const float ref = (fresh ? 0.f : -minit[cq][0]) + up[cb];  // the reference lives in minit alone here
                    l_sum[cq] *= alpha;
    #pragma unroll
                    for (int r = 0; r < 16; ++r) o_acc[cq][r] *= alpha;
#pragma unroll
                    for (int e = 0; e < 4; ++e) minit[cq][e] = -ref;
                }
                sm_unit(qt, up, lu, true);
            }
            if constexpr (!MSUM) {
                l_sum[2 * qt] += lu[0];
                l_sum[2 * qt + 1] += lu[1];
            }
        };
        // PV of unit (kp, qp), then QK of unit (kq, qq): order, interleave ratio and wave priorities were swept on the
        // chip; everything lies within 1-2 %
        auto qk_pv = [&](int kq, int qq, int kp, int qp) {
            pv(kp, qp);
            qk(kq, qq);
        };
        // one MFMA : two vector instructions, for every MFMA of the step (ratios 1 to 4 measured: 2 is best by 1 %)
        auto interleave = [&]() {
#pragma unroll
            for (int i = 0; i < (MSUM ? 18 : 16); ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x402, 2, 0);
            }
        };

        // The four steps of one key tile in ring slot `slot`.  The main loop below runs four tiles per round with the
        // slots as compile-time constants: every LDS address is then a per-lane offset fixed before the loop plus an
        // immediate, and the round spends no vector instruction on addresses.  Up to three tiles remain for the
        // second loop, which computes its slots.
        auto tile_steps = [&](int t, auto slot, auto slot_next, auto slot_load, bool first) __attribute__((always_inline)) {
            float lu[2];
            // step (0,0): QK(0,1), PV(1,1) of the previous tile, SM(0,0)
            __builtin_amdgcn_sched_barrier(0);
            qk_pv(0, 1, 1, 1);
            sm_unit(0, no_sub, lu, false);
            interleave();
            __builtin_amdgcn_sched_barrier(0);
            settle(0, lu, first);
            bar(t, slot_load);
            // step (0,1): PV(0,0), QK(1,0), SM(0,1)
            __builtin_amdgcn_sched_barrier(0);
            read_k((int)slot, 1);
            read_v((int)slot, 0);
            qk_pv(1, 0, 0, 0);
            sm_unit(1, no_sub, lu, false);
            interleave();
            __builtin_amdgcn_sched_barrier(0);
            settle(1, lu, first);
            // step (1,0): QK(1,1), PV(0,1), SM(1,0)
            __builtin_amdgcn_sched_barrier(0);
            qk_pv(1, 1, 0, 1);
            sm_unit(0, no_sub, lu, false);
            interleave();
            __builtin_amdgcn_sched_barrier(0);
            settle(0, lu, false);
            // step (1,1): PV(1,0), QK(0,0) of the next tile (a discarded product after the last tile), SM(1,1)
            __builtin_amdgcn_sched_barrier(0);
            read_k((int)slot_next, 0);
            read_v((int)slot, 1);
            qk_pv(0, 0, 1, 0);
            sm_unit(1, no_sub, lu, false);
            interleave();
            __builtin_amdgcn_sched_barrier(0);
            settle(1, lu, false);
        };
        read_k(0, 0);
        qk(0, 0);  // fill: QK of the first unit alone
        typedef std::integral_constant<int, 0> I0;
        typedef std::integral_constant<int, 1> I1;
        typedef std::integral_constant<int, 2> I2;
        typedef std::integral_constant<int, 3> I3;
        int t = t_begin;
        for (; t + 4 <= t_pipe; t += 4) {
            tile_steps(t, I0{}, I1{}, I3{}, t == t_begin);
            tile_steps(t + 1, I1{}, I2{}, I0{}, false);
            tile_steps(t + 2, I2{}, I3{}, I1{}, false);
            tile_steps(t + 3, I3{}, I0{}, I2{}, false);
        }
        for (; t < t_pipe; ++t) {
            const int slot = (t - t_begin) & 3;
            tile_steps(t, slot, (slot + 1) & 3, (slot + 3) & 3, t == t_begin);
        }
        __builtin_amdgcn_sched_barrier(0);
        pv(1, 1);  // drain: PV of the last unit
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int cq = 0; cq < 4; ++cq) m_used[cq] = -minit[cq][0];
    }
    // tiles at the frame bounds (mask) and tiles only the later block sees: one tile at a time
    auto run_rest = [&](int t_from, int t_to, auto qa_tag) {
        constexpr int QA = decltype(qa_tag)::value;
        for (int t = t_from; t < t_to; ++t) {
            __builtin_amdgcn_sched_barrier(0);
            bar(t, (t + 3 - t_begin) & 3);
            if (QA == 0) tile_body(t, (t - t_begin) & 3, std::integral_constant<int, 0>{});
            if (QA == 0 || (wave_active && t * kBN < kmax_wave)) tile_body(t, (t - t_begin) & 3, std::integral_constant<int, 1>{});
        }
    };
    run_rest(t_pipe, t_mid, std::integral_constant<int, 0>{});
    run_rest(t_mid, t_end, std::integral_constant<int, 1>{});

    // ---- final write: lane (j, g) holds, for query column cq, features 16 fb + 4 g + 0..3 -----------------------
    if (!wave_active) return;
#pragma unroll
    for (int cq = 0; cq < 4; ++cq) {
        float l_row;
        if constexpr (MSUM) {
            l_row = l_sum[cq];  // every lane group holds the whole column's sum
        } else {
            l_row = l_sum[cq] + __shfl_xor(l_sum[cq], 16);
            l_row += __shfl_xor(l_row, 32);
        }
        const int row = row_of(cq);
        if (row >= p.Sq) continue;
        const float m_exp = EXACTQ ? m_used[cq] * c : m_used[cq];
        if (p.n_splits == 1) {
            const float inv = 1.0f / l_row;
            __bf16* og = (__bf16*)p.out + ((int64_t)wi.bh * p.Sq + row) * kD;
#pragma unroll
            for (int fb = 0; fb < 4; ++fb) {
                const f32x4 x = {o_acc[cq][4 * fb] * inv, o_acc[cq][4 * fb + 1] * inv, o_acc[cq][4 * fb + 2] * inv, o_acc[cq][4 * fb + 3] * inv};
                *(bf16x4*)(og + 16 * fb + 4 * g) = __builtin_convertvector(x, bf16x4);
            }
            if (p.lse && g == 0) p.lse[(int64_t)wi.bh * p.Sq + row] = (m_exp + __builtin_log2f(l_row)) * kLn2;
        } else {
            const int64_t prow = ((int64_t)wi.bh * p.n_splits + wi.split) * p.Sq + row;
            __bf16* po = p.part_o + prow * kD;
#pragma unroll
            for (int fb = 0; fb < 4; ++fb) {
                const f32x4 x = {o_acc[cq][4 * fb], o_acc[cq][4 * fb + 1], o_acc[cq][4 * fb + 2], o_acc[cq][4 * fb + 3]};
                *(bf16x4*)(po + 16 * fb + 4 * g) = __builtin_convertvector(x, bf16x4);
            }
            if (g == 0) {
                const f32x2 ml = {m_exp, l_row};
                *(f32x2*)(p.part_ml + prow * 2) = ml;
            }
        }
    }
}

template <bool EXACTQ>
__global__ void __launch_bounds__(kWaves * 64, 2)
attn_fwd_bf16_d64_m16(FwdParams p) {
    __shared__ SmemRingPipe sm;
    const WorkItem wi = decode_work(p);
    if (!wi.valid) return;
    attn_fwd_item16<EXACTQ>(p, wi, sm);
}

}  // namespace mfma
}  // namespace nfd

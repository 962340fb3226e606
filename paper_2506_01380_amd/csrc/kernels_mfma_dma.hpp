// Ping-pong bf16 forward kernel with direct global->LDS tile loads (gfx950 / CDNA4).
//
// Same mathematics and the same two-group interval structure as attn_fwd_bf16_d64_pp, but K and V
// tiles never pass through registers: every wavefront issues 16-byte global loads that land straight
// in LDS (one wave instruction = 1 KB = eight 128-byte tile rows), two intervals ahead of their use.
// A wave's 1 KB is contiguous in LDS, so rows cannot be padded; bank conflicts are avoided with an XOR
// swizzle instead: the 16-byte chunk c of tile row r is stored at chunk position c ^ f(r), with
// f(r) = perm((r >> 1) & 7).  The swizzle costs nothing on the way in (each lane simply fetches the
// chunk that belongs at its position) and one precomputed per-lane offset on the way out.
#pragma once
#include "kernels_mfma.hpp"

namespace nfd {
namespace mfma {

constexpr int kDmaSlots = 4;             // K and V ring depth (tiles)
constexpr int kTileElems = kBN * kD;     // 4096 bf16 = 8 KB, rows of 128 B, no padding

// Chunk-position swizzle of a tile row: a bijection of (r >> 1) & 7 whose bit 2 toggles every two rows.
// Measured conflict-free for both the 16-byte fragment reads (32 consecutive rows, one chunk) and the
// transposing 8-byte reads (4 rows x 64 bytes per 32 lanes) on this LDS.
__device__ __forceinline__ int chunk_swizzle(int r) {
    const int k = (r >> 1) & 7;
    return ((k & 1) << 2) | (k >> 1);
}

struct __attribute__((aligned(16))) SmemDma {
    union {
        struct {
            __bf16 k[kDmaSlots][kTileElems];
            __bf16 v[kDmaSlots][kTileElems];
        } t;
        float merge[4 * 64 * 36];
    };
};

// DBG is 0 in the product; development builds leave out pieces of work (wrong results) to cost them.
template <int DBG>
__global__ void __launch_bounds__(kPPWaves * 64, 2)
attn_fwd_bf16_d64_dma(FwdParams p) {
    __shared__ SmemDma sm;
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
        for (int i = tid; i < kDmaSlots * kTileElems / 8; i += kPPWaves * 64) vz[i] = z;
    }
    __syncthreads();  // the zero fill must not race with the first tile loads below

    // ---- tile loads: this lane fills position (lane & 7) of tile row 8*wave + lane/8 ---------------
    const int ld_row = 8 * wave + (lane >> 3);
    const int ld_chunk = (lane & 7) ^ chunk_swizzle(ld_row);
    const unsigned lds_k0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)(&sm.t.k[0][0]) + wave * 1024;
    const unsigned lds_v0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)(&sm.t.v[0][0]) + wave * 1024;
    auto load_tile = [&](int i) {  // rows past the end are clamped: they are masked anyway
        if (DBG & 4) return;
        const int kr = min((t_begin + i) * kBN + ld_row, p.Sk - 1);
        const int64_t off = (int64_t)kr * kD + ld_chunk * 8;
        const unsigned kdst = lds_k0 + (unsigned)((i & (kDmaSlots - 1)) * kTileElems * 2);
        const unsigned vdst = lds_v0 + (unsigned)((i & (kDmaSlots - 1)) * kTileElems * 2);
        // Issued through inline assembly on purpose: the compiler would otherwise guard every later LDS
        // read and every barrier with vmcnt(0), which cancels the two-interval prefetch distance.  The
        // waits that order these loads are the explicit ones below.
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(kg + off), "s"(kdst) : "memory", "m0");
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(vg + off), "s"(vdst) : "memory", "m0");
    };
    // all but the newest tile's two loads have landed
    auto wait_older_tiles = [&]() { asm volatile("s_waitcnt vmcnt(2)" ::: "memory"); };

    // ---- per-lane fragment offsets (elements) under the swizzle ---------------------------------------
    const int fk = chunk_swizzle(n);  // K rows 32*kb + n: (r >> 1) & 7 does not depend on kb
    int k_off[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) k_off[ks] = n * kD + 8 * ((2 * ks + h) ^ fk);
    const int s16 = lane & 15, dblk = (lane >> 4) & 1;
    const int v_row = 4 * h + (s16 >> 2);
    const int v_chunk = 2 * dblk + ((s16 & 3) >> 1);  // + 4*dt
    const int fv = chunk_swizzle(v_row);              // rows 32kb + 16g + v_row: same swizzle; +8 rows: fv ^ 2
    int v_off[2][2];                                  // [dt][second half of the key step]
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int sec = 0; sec < 2; ++sec)
            v_off[dt][sec] = (v_row + 8 * sec) * kD + 8 * ((4 * dt + v_chunk) ^ (fv ^ (2 * sec))) + 4 * (s16 & 1);

    auto read_v_frags = [&](int i) {
        if (DBG & 8) return;
        const __bf16* vs_ = sm.t.v[i & (kDmaSlots - 1)];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int g = 0; g < 2; ++g)
#pragma unroll
                for (int dt = 0; dt < 2; ++dt) {
                    const __bf16* vp = vs_ + (32 * kb + 16 * g) * kD;
                    const s16x4 lo = lds_read_tr(vp + v_off[dt][0]);
                    const s16x4 hi = lds_read_tr(vp + v_off[dt][1]);
                    typedef __attribute__((ext_vector_type(8))) short s16x8;
                    const s16x8 av = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    vf[kb][g][dt] = __builtin_bit_cast(bf16x8, av);
                }
    };
    auto pv_half = [&](int kb) {
        if (DBG & (2 | 64)) return;
#pragma unroll
        for (int g = 0; g < 2; ++g)
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int qt = 0; qt < 2; ++qt)
                    o_acc[dt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[kb][g][dt], pf[kb][g][qt], o_acc[dt][qt], 0, 0, 0);
    };
    auto stage_mfma = [&](int i_qk) {
        bf16x8 kf[2][4];
        pv_half(0);
        __builtin_amdgcn_sched_barrier(0);
        const __bf16* ks_ = sm.t.k[i_qk & (kDmaSlots - 1)];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                if (DBG & 16) kf[kb][ks] = qf[kb][ks];
                else kf[kb][ks] = lds_read_b128(ks_ + 32 * kb * kD + k_off[ks]);
            }
        __builtin_amdgcn_sched_barrier(0);
        pv_half(1);
        __builtin_amdgcn_sched_barrier(0);
        if (!(DBG & 2))
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
    };
    auto form_p = [&]() {  // P = exp2(c*s - c*m_used) in bf16; row sums by plain fp32 adds
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
    auto stage_softmax = [&](int i) {
        if (DBG & 32) { form_p(); return; }
        const int j0 = (i >= 0 && i < n_local) ? (t_begin + i) * kBN : 0x3fffff00;
        if (__builtin_amdgcn_readfirstlane(j0 + kBN > kmin_wave)) {  // tile crosses some row's bound
            asm volatile("" ::: "memory");
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
        if (DBG & 1) return;
        form_p();
        // Pin the packed P before the test: otherwise the compiler, seeing P rebuilt on the rare path,
        // postpones all conversions until after the branch and keeps the 64 exponentials alive across it.
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int e = 0; e < 2; ++e) asm volatile("" : "+v"(pf[a][b][e]));
        const bool bad = !(l_sum[0] - l_old0 < kOptimisticLimit) | !(l_sum[1] - l_old1 < kOptimisticLimit);
        if (__builtin_amdgcn_ballot_w64(bad) != 0) {  // exact path: this tile's max, rescale, redo
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

    // Tiles 0 and 1 before the loop; interval nn issues tile nn+2 and, before its barrier, waits for
    // everything older than that (tile nn+1 is read in interval nn+1).  K(i) is read in interval i,
    // V(i) at the end of interval i+1; tile nn+2 may land any time during intervals nn..nn+1, so a ring
    // of 4 slots keeps it clear of tiles nn-1, nn and nn+1.
    load_tile(0);
    load_tile(1);
    wait_vmem_all();  // Q fragments and tiles 0, 1 have landed on every path (and the compiler knows it)
    __syncthreads();

    // Interval boundary.  Matrix instructions touch no memory, so without the scheduling fences the
    // compiler is free to move them across the barrier into the next interval - which puts both groups'
    // MFMAs at the start of every interval and their softmax behind them: the stages then take turns
    // again instead of overlapping.
    auto interval_end = [&]() {
        __builtin_amdgcn_sched_barrier(0);
        wait_older_tiles();
        // A bare barrier, not __syncthreads(): the fence of the latter would also wait for the V^T
        // fragment reads issued just before it, whose latency is meant to pass behind the barrier.
        // Nothing else needs the fence: LDS is written only by the tile loads, which the explicit
        // vmcnt wait above orders, and the slots being read are not rewritten for two more intervals.
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };
    const int n_iter = n_local > 0 ? (n_local + 3) / 2 : 0;
#ifdef NFD_STAGE_TIMING
    const unsigned long long tc0 = __builtin_readcyclecounter();
#endif
    if (grp == 0) {
        for (int it = 0; it < n_iter; ++it) {
            const int nn = 2 * it;
            load_tile(nn + 2);
            stage_mfma(nn);
            interval_end();
            load_tile(nn + 3);
            stage_softmax(nn);
            read_v_frags(nn);
            interval_end();
        }
    } else {
        for (int it = 0; it < n_iter; ++it) {
            const int nn = 2 * it;
            load_tile(nn + 2);
            stage_softmax(nn - 1);
            read_v_frags(nn - 1);
            interval_end();
            load_tile(nn + 3);
            stage_mfma(nn + 1);
            interval_end();
        }
    }
#ifdef NFD_STAGE_TIMING
    if (p.timing && lane == 0) {
        unsigned long long* o = p.timing + ((size_t)blockIdx.x * kPPWaves + wave) * 8;
        o[0] = __builtin_readcyclecounter() - tc0;
        o[5] = (unsigned long long)(2 * n_iter);
    }
#endif
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // no tile load may still be writing LDS when it is reused below
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

}  // namespace mfma
}  // namespace nfd

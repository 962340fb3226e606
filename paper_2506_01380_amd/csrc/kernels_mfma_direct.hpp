// bf16 forward kernel with direct global->LDS tile loads, one barrier per key tile (gfx950 / CDNA4).
//
// Work decomposition as in attn_fwd_bf16_d64 (4 wavefronts x 64 query rows, two workgroups per CU,
// S^T = K.Q^T and O^T += V^T.P^T on 32x32x16 bf16 MFMA, P stays in registers), but
//  * K and V tiles never pass through registers: each wavefront issues 16-byte global loads that
//    land straight in LDS, two tiles ahead of their use, into a ring of three tile slots; rows are
//    128 bytes, unpadded, and the 16-byte chunks of a row are XOR-swizzled against bank conflicts;
//  * softmax is optimistic: P is formed against the reference max of earlier tiles and the tile's
//    own max is only computed when a lane's tile sum says the reference was too small.
#pragma once
#include "kernels_mfma_dma.hpp"

namespace nfd {
namespace mfma {

constexpr int kRingSlots = 3;

struct __attribute__((aligned(16))) SmemRing {
    __bf16 k[kRingSlots][kTileElems];
    __bf16 v[kRingSlots][kTileElems];
};

template <int VEARLY>
__global__ void __launch_bounds__(256, 2)
attn_fwd_bf16_d64_direct(FwdParams p) {
    constexpr int BM = 256;
    __shared__ SmemRing sm;
    const WorkItem wi = decode_work(p);
    if (!wi.valid) return;  // whole workgroup leaves together

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, h = lane >> 5;
    const int r0 = wi.q_tile * BM;
    const int r_last = min(r0 + BM, p.Sq) - 1;
    const int kmax_wg = kmax_of_row(r_last, p.T, p.P);
    const int n_tiles = (kmax_wg + kBN - 1) / kBN;
    const int tiles_per_split = (n_tiles + p.n_splits - 1) / p.n_splits;
    const int t_begin = wi.split * tiles_per_split;
    const int t_end = min(t_begin + tiles_per_split, n_tiles);

    const __bf16* qg = (const __bf16*)p.q + (int64_t)wi.bh * p.Sq * kD;
    const __bf16* kg = (const __bf16*)p.k + (int64_t)wi.bh * p.Scap * kD;
    const __bf16* vg = (const __bf16*)p.v + (int64_t)wi.bh * p.Scap * kD;

    // ---- this wavefront's queries -------------------------------------------------------
    const int rw0 = r0 + wave * 64;
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

    // ---- tile loads: one wave instruction fills 8 consecutive tile rows (1 KB); a wavefront owns
    // rows 8*wave + 32*pass + lane/8, and each lane fetches the chunk that belongs at its position ----
    const int ld_row = 8 * wave + (lane >> 3);
    const int ld_chunk = (lane & 7) ^ chunk_swizzle(ld_row);  // rows +32: same swizzle
    const unsigned lds_k0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)(&sm.k[0][0]) + wave * 1024;
    const unsigned lds_v0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)(&sm.v[0][0]) + wave * 1024;
    auto load_tile = [&](int t, int slot) {  // rows past the end are clamped: they are masked anyway
        // Issued through inline assembly on purpose: for the builtin the compiler guards every later
        // LDS read and every barrier with vmcnt(0), which would cancel the prefetch distance.  The
        // waits that order these loads are the explicit ones at the top of the tile loop.
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            const int kr = min(t * kBN + 32 * pass + ld_row, p.Sk - 1);
            const int64_t off = (int64_t)kr * kD + ld_chunk * 8;
            const unsigned kdst = lds_k0 + (unsigned)(slot * kTileElems * 2 + pass * 4096);
            const unsigned vdst = lds_v0 + (unsigned)(slot * kTileElems * 2 + pass * 4096);
            asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(kg + off), "s"(kdst) : "memory", "m0");
            asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(vg + off), "s"(vdst) : "memory", "m0");
        }
    };

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

    if (t_begin < t_end) load_tile(t_begin, 0);
    if (t_begin + 1 < t_end) load_tile(t_begin + 1, 1);
    // The Q fragments are complete from here on and the compiler knows it: no later guard on them
    // can drain the tile prefetch.  (This also lands tiles 0 and 1, once per workgroup.)
    wait_vmem_all();

    int slot = 0;
    for (int t = t_begin; t < t_end; ++t) {
        // Tile t has landed for this wavefront once at most tile t+1's four loads are in flight; after
        // the barrier it has landed for all, and every wavefront is done with tile t-1, whose slot
        // the load of tile t+2 reuses.
        __builtin_amdgcn_sched_barrier(0);
        if (t + 1 < t_end) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        const int slot2 = slot == 0 ? 2 : slot - 1;  // (slot + 2) % 3
        if (t + 2 < t_end) load_tile(t + 2, slot2);
        const int j0 = t * kBN;

        if (wave_active && j0 < kmax_wave) {
            const __bf16* ks_ = sm.k[slot];
            const __bf16* vs_ = sm.v[slot];
            // ---- S^T = K . Q^T: all eight K fragments are requested before the first product ------
            f32x16 s_acc[2][2];  // [kb][qt]
            bf16x8 kf[2][4];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) kf[kb][ks] = lds_read_b128(ks_ + 32 * kb * kD + k_off[ks]);
            __builtin_amdgcn_sched_barrier(0);
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
            bf16x8 vf[2][2][2];  // [kb][g][dt]
            auto read_v_frags = [&]() {
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
            if (VEARLY) {  // V^T fragments land during the softmax
                read_v_frags();
                __builtin_amdgcn_sched_barrier(0);
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
            // ---- optimistic softmax, lane-local per query column -------------------------------
            bf16x8 pf[2][2][2];  // [kb][g][qt]
            float l_tile[2];
            auto form_p = [&]() {  // P = exp2(c*s - c*m_used) in bf16; row sums by plain fp32 adds (the
                                   // packed dot instruction shares the matrix pipe and would stall MFMAs)
#pragma unroll
                for (int qt = 0; qt < 2; ++qt) {
                    const float mc = m_used[qt] * c;
                    float l = 0.f, l2 = 0.f;
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
                    l_tile[qt] = l + l2;
                }
            };
            form_p();
            // Pin the packed P before the test: otherwise the compiler, seeing P rebuilt on the rare
            // path, postpones the conversions until after the branch and keeps 64 exponentials alive.
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int e = 0; e < 2; ++e) asm volatile("" : "+v"(pf[a][b][e]));
            if (!VEARLY) read_v_frags();
            const bool bad = !(l_tile[0] < kOptimisticLimit) | !(l_tile[1] < kOptimisticLimit);
            if (__builtin_amdgcn_ballot_w64(bad) != 0) {  // exact path: this tile's max, rescale, redo
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
            l_sum[0] += l_tile[0];
            l_sum[1] += l_tile[1];
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
        slot = slot == 2 ? 0 : slot + 1;
    }

    if (!wave_active) return;
    store_rows(p, wi, row, h, o_acc, l_sum, m_used, c);
}

}  // namespace mfma
}  // namespace nfd

// bf16 matrix-core backward kernels for head width 64 (gfx950 / CDNA4).
//
// Gradients of the block-wise causal attention (mask: Sec. 3.1; the paper trains through this
// attention, Sec. 3.2).  With p_ij = exp(s_ij - lse_i) the softmax weights of the visible keys,
//   dv_j = sum_i p_ij do_i            dp_ij = <do_i, v_j>         delta_i = <do_i, o_i> = sum_j p_ij dp_ij
//   ds_ij = p_ij (dp_ij - delta_i)    dq_i = scale sum_j ds_ij k_j    dk_j = scale sum_i ds_ij q_i
// Two launches, no atomics, bit-reproducible:
//   attn_bwd_dq_bf16_d64   query-major, same decomposition and tile ring as the forward kernel; it also forms
//                          delta_i = <do_i, o_i> of its rows (dout is in its registers anyway) and stores -delta_i
//                          and lse_i log2(e), the two per-row values in the form the dk/dv kernel consumes them
//   attn_bwd_dkdv_bf16_d64 key-major: a wavefront owns 32 (or 64) keys and walks over the query tiles that see them
// Both matrix kernels recompute the weights from the stored log-sum-exp, so no online softmax is
// needed, and both keep the operand whose rows they own in registers for the whole kernel.  Tiles
// of the other operand go global -> LDS directly into the same XOR-swizzled ring as in the forward
// kernel.  As there, every second product takes the accumulator registers of the first as its B
// operand unchanged (the contraction index is permuted identically on the A side by the transposing
// LDS read), so neither P nor dS ever touches LDS.
//
// Register budget: both kernels run two wavefronts per SIMD - the dq kernel by forming the scores of
// 32 keys at a time, the dk/dv kernel by owning 32 keys per wavefront.  S and dP are formed in both
// kernels (seven products for the five of the mathematics): the price of having no atomics on dq.
#pragma once
#include "kernels_mfma.hpp"

namespace nfd {
namespace mfma {

struct BwdParams {
    const void* q;       // [BH, Sq, D]
    const void* k;       // [BH, Scap, D]
    const void* v;       // [BH, Scap, D]
    const void* dout;    // [BH, Sq, D]
    const void* out;     // [BH, Sq, D] the forward's result
    const float* lse;    // [BH, Sq] natural log of the softmax denominator (from the forward call)
    float* neg_delta;    // [BH, Sq] -<dout_i, out_i> (workspace): written by the dq kernel, read by the dk/dv kernel
    float* lse2;         // [BH, Sq] lse * log2(e) (workspace): likewise
    void* dq;            // [BH, Sq, D]
    void* dk;            // [BH, Scap, D], rows < Sk written
    void* dv;            // [BH, Scap, D], rows < Sk written
    int BH, Sq, Sk, Scap, T, P;
    int n_q_tiles;       // 256-row query tiles per head (dq kernel)
    int n_k_blocks;      // key blocks per head (dk/dv kernel)
    float scale;
    float scale_log2e;
};

// Workgroup id -> (head, item): ids are dealt round-robin to the 8 XCDs; when the head count is a
// multiple of 8 heads are pinned to an XCD (bh % 8), otherwise ids run plainly over the heads; either
// way item 0 of every head comes first, then item 1, ...
struct BwdItem {
    int bh, item;
    bool valid;
};
__device__ __forceinline__ BwdItem decode_bwd(int BH, int n_items) {
    BwdItem w;
    const bool pinned = (BH & 7) == 0;
    const int xcd = pinned ? (int)(blockIdx.x & 7) : 0;
    const int j = pinned ? (int)(blockIdx.x >> 3) : (int)blockIdx.x;
    const int hh = pinned ? BH >> 3 : BH;
    w.valid = j < hh * n_items;
    w.bh = pinned ? (j % hh) * 8 + xcd : j % hh;
    w.item = j / hh;
    return w;
}

// One wavefront's share of a 64-row tile pair (a_rows from tensor a, b_rows from tensor b) into the
// ring: rows 8*wave + 32*pass + lane/8, each lane fetching the chunk that belongs at its swizzled
// position.  Rows past row_limit - 1 are clamped (their results are masked or never stored).
__device__ __forceinline__ void dma_tile_pair(const __bf16* a, const __bf16* b, int row0, int row_limit,
                                              unsigned lds_a, unsigned lds_b, int ld_row, int ld_chunk) {
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int r = min(row0 + 32 * pass + ld_row, row_limit - 1);
        const int64_t off = (int64_t)r * kD + ld_chunk * 8;
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(a + off), "s"(lds_a + pass * 4096) : "memory", "m0");
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(b + off), "s"(lds_b + pass * 4096) : "memory", "m0");
    }
}

// Per-lane LDS offsets (elements) of the two fragment kinds under the swizzle: plain 16-byte row
// fragments (row = lane % 32 of a 32-row block, feature step ks) and transposing reads (A operand
// of a product whose contraction index runs over the tile's rows).
struct FragOffsets {
    int row_frag[4];     // [ks]
    int tr_frag[2][2];   // [dt][second half of the 16-row step]
};
__device__ __forceinline__ FragOffsets frag_offsets(int lane) {
    FragOffsets f;
    const int n = lane & 31, h = lane >> 5;
    const int fk = chunk_swizzle(n);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) f.row_frag[ks] = n * kD + 8 * ((2 * ks + h) ^ fk);
    const int s16 = lane & 15, dblk = (lane >> 4) & 1;
    const int v_row = 4 * h + (s16 >> 2);
    const int v_chunk = 2 * dblk + ((s16 & 3) >> 1);
    const int fv = chunk_swizzle(v_row);
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int sec = 0; sec < 2; ++sec)
            f.tr_frag[dt][sec] = (v_row + 8 * sec) * kD + 8 * ((4 * dt + v_chunk) ^ (fv ^ (2 * sec))) + 4 * (s16 & 1);
    return f;
}
__device__ __forceinline__ bf16x8 read_tr_frag(const __bf16* tile, const FragOffsets& f, int blk32, int g, int dt) {
    const __bf16* vp = tile + (32 * blk32 + 16 * g) * kD;
    const s16x4 lo = lds_read_tr(vp + f.tr_frag[dt][0]);
    const s16x4 hi = lds_read_tr(vp + f.tr_frag[dt][1]);
    typedef __attribute__((ext_vector_type(8))) short s16x8;
    const s16x8 av = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, av);
}
// Pack eight consecutive accumulator values of one 32x32 block into the B-operand fragment of the
// following product.
__device__ __forceinline__ bf16x8 pack8(const f32x16& a, int g) {
    bf16x8 r;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
        const f32x2 pp = {a[8 * g + 2 * jj], a[8 * g + 2 * jj + 1]};
        const bf16x2 pb = __builtin_convertvector(pp, bf16x2);
        r[2 * jj] = pb[0];
        r[2 * jj + 1] = pb[1];
    }
    return r;
}

// ---------------------------------------------------------------------------------------------
// dq: a workgroup owns 256 query rows (4 wavefronts x 64), walks over the visible key tiles.
//   S^T = K.Q^T, dP^T = V.dO^T (A = K / V rows from LDS, B = Q^T / dO^T in registers)
//   dS^T = P^T o (dP^T - delta),  dQ^T += K^T.dS^T (A = K^T by transposing read, B = dS^T accumulators)
__global__ void __launch_bounds__(256, 2)
attn_bwd_dq_bf16_d64(BwdParams p) {
    __shared__ SmemRing sm;
    const BwdItem wi = decode_bwd(p.BH, p.n_q_tiles);
    if (!wi.valid) return;
    const int q_tile = p.n_q_tiles - 1 - wi.item;  // heaviest (latest frames) first

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, h = lane >> 5;
    const int r0 = q_tile * kBM;
    const int r_last = min(r0 + kBM, p.Sq) - 1;
    const int n_tiles = (kmax_of_row(r_last, p.T, p.P) + kBN - 1) / kBN;

    const __bf16* qg = (const __bf16*)p.q + (int64_t)wi.bh * p.Sq * kD;
    const __bf16* gg = (const __bf16*)p.dout + (int64_t)wi.bh * p.Sq * kD;
    const __bf16* og_ = (const __bf16*)p.out + (int64_t)wi.bh * p.Sq * kD;
    const __bf16* kg = (const __bf16*)p.k + (int64_t)wi.bh * p.Scap * kD;
    const __bf16* vg = (const __bf16*)p.v + (int64_t)wi.bh * p.Scap * kD;

    const int rw0 = r0 + wave * 64;
    int row[2], kmax_lane[2];
    float lse2[2], dl[2];
    bf16x8 qf[2][4], gf[2][4];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        row[qt] = rw0 + 32 * qt + n;
        const int rc = min(row[qt], p.Sq - 1);  // ragged tail: compute a duplicate, never store it
        kmax_lane[qt] = kmax_of_row(rc, p.T, p.P);
        lse2[qt] = p.lse[(int64_t)wi.bh * p.Sq + rc] * kLog2e;
        float part = 0.f;  // this lane's half of <dout_i, out_i>: the features it holds of dout
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            qf[qt][ks] = *(const bf16x8*)(qg + (int64_t)rc * kD + 16 * ks + 8 * h);
            gf[qt][ks] = *(const bf16x8*)(gg + (int64_t)rc * kD + 16 * ks + 8 * h);
            const bf16x8 of = *(const bf16x8*)(og_ + (int64_t)rc * kD + 16 * ks + 8 * h);
#pragma unroll
            for (int e = 0; e < 8; ++e) part = __builtin_fmaf((float)gf[qt][ks][e], (float)of[e], part);
        }
        dl[qt] = part + __shfl_xor(part, 32);
        if (h == 0 && row[qt] < p.Sq) {  // for the dk/dv kernel
            p.neg_delta[(int64_t)wi.bh * p.Sq + row[qt]] = -dl[qt];
            p.lse2[(int64_t)wi.bh * p.Sq + row[qt]] = lse2[qt];
        }
    }
    const int kmin_wave = kmax_of_row(min(rw0, p.Sq - 1), p.T, p.P);
    const int kmax_wave = kmax_of_row(min(rw0 + 63, p.Sq - 1), p.T, p.P);
    const bool wave_active = rw0 < p.Sq;

    f32x16 dq_acc[2][2];  // [dt][qt]
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) dq_acc[a][b][r] = 0.f;
    const float c = p.scale_log2e;

    const int ld_row = 8 * wave + (lane >> 3);
    const int ld_chunk = (lane & 7) ^ chunk_swizzle(ld_row);
    const unsigned lds_k0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)(&sm.k[0][0]) + wave * 1024;
    const unsigned lds_v0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)(&sm.v[0][0]) + wave * 1024;
    auto load_tile = [&](int t, int slot) {
        dma_tile_pair(kg, vg, t * kBN, p.Sk, lds_k0 + slot * kTileElems * 2, lds_v0 + slot * kTileElems * 2, ld_row, ld_chunk);
    };
    const FragOffsets fo = frag_offsets(lane);

    if (0 < n_tiles) load_tile(0, 0);
    if (1 < n_tiles) load_tile(1, 1);
    wait_vmem_all();  // q, dout, lse, delta fragments and the first tiles have landed (and the compiler knows it)

    int slot = 0;
    for (int t = 0; t < n_tiles; ++t) {
        // same ring protocol as the forward kernel: tile t complete for all after the barrier, and the
        // slot of tile t-1 free for tile t+2
        __builtin_amdgcn_sched_barrier(0);
        if (t + 1 < n_tiles) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        const int slot2 = slot == 0 ? 2 : slot - 1;
        if (t + 2 < n_tiles) load_tile(t + 2, slot2);
        const int j0 = t * kBN;
        if (wave_active && j0 < kmax_wave) {
            const __bf16* ks_ = sm.k[slot];
            const __bf16* vs_ = sm.v[slot];
            const bool need_mask = j0 + kBN > kmin_wave;  // tile crosses some row's bound
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {  // 32 keys at a time: keeps the live accumulators at half
                f32x16 s_acc[2], dp_acc[2];   // [qt]
                bf16x8 kf[4], vf[4];
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    kf[ks] = lds_read_b128(ks_ + 32 * kb * kD + fo.row_frag[ks]);
                    vf[ks] = lds_read_b128(vs_ + 32 * kb * kD + fo.row_frag[ks]);
                }
#pragma unroll
                for (int qt = 0; qt < 2; ++qt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) { s_acc[qt][r] = 0.f; dp_acc[qt][r] = 0.f; }
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                    for (int qt = 0; qt < 2; ++qt) {
                        s_acc[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[qt][ks], s_acc[qt], 0, 0, 0);
                        dp_acc[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[ks], gf[qt][ks], dp_acc[qt], 0, 0, 0);
                    }
                if (need_mask) {
#pragma unroll
                    for (int qt = 0; qt < 2; ++qt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int key = j0 + 32 * kb + 8 * (r >> 2) + 4 * h + (r & 3);
                            if (key >= kmax_lane[qt]) s_acc[qt][r] = -INFINITY;
                        }
                }
                // dS^T = P^T o (dP^T - delta), written over the score accumulators
#pragma unroll
                for (int qt = 0; qt < 2; ++qt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float pr = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[qt][r], c, -lse2[qt]));
                        s_acc[qt][r] = pr * (dp_acc[qt][r] - dl[qt]);
                    }
#pragma unroll
                for (int g = 0; g < 2; ++g) {
                    const bf16x8 ds0 = pack8(s_acc[0], g), ds1 = pack8(s_acc[1], g);
#pragma unroll
                    for (int dt = 0; dt < 2; ++dt) {
                        const bf16x8 kt = read_tr_frag(ks_, fo, kb, g, dt);
                        dq_acc[dt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt, ds0, dq_acc[dt][0], 0, 0, 0);
                        dq_acc[dt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt, ds1, dq_acc[dt][1], 0, 0, 0);
                    }
                }
            }
        }
        slot = slot == 2 ? 0 : slot + 1;
    }

    if (!wave_active) return;
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        if (row[qt] >= p.Sq) continue;
        __bf16* og = (__bf16*)p.dq + ((int64_t)wi.bh * p.Sq + row[qt]) * kD;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) {
                const f32x4 x = {dq_acc[dt][qt][4 * rb] * p.scale, dq_acc[dt][qt][4 * rb + 1] * p.scale,
                                 dq_acc[dt][qt][4 * rb + 2] * p.scale, dq_acc[dt][qt][4 * rb + 3] * p.scale};
                *(bf16x4*)(og + 32 * dt + 8 * rb + 4 * h) = __builtin_convertvector(x, bf16x4);
            }
    }
}

// ---------------------------------------------------------------------------------------------
// dk, dv: a workgroup owns 128 keys (4 wavefronts x 32, two wavefronts per SIMD) and walks over the 64-row query
// tiles that can see them (all rows from the first frame that sees the block's first key).
//   S = Q.K^T, dP = dO.V^T (A = Q / dO rows from LDS, B = K^T / V^T in registers)
//   dV^T += dO^T.P, dK^T += Q^T.dS (A by transposing reads of the dO / Q tile, B = P / dS accumulators)
// In the accumulator layout a lane holds ONE key column and 16 of a block's 32 query rows, so the
// per-row values come from LDS (four 16-byte reads each per 32-row block), in the form the dq kernel left them:
// lse log2(e), subtracted inside the exponent's fma, and -delta, which is what the dP accumulators start from
// (the matrix instruction adds the product to it), so dP - delta costs no instruction.
// Key j is visible to row i iff i >= rmin(j) = (floor(j/T) - P) T: one bound per lane, no division
// in the loop.
//
// A query tile is two units of 32 rows; unit u runs scores(u): 8 MFMA for S and dP; weights(u): 16 x (fma, exp2,
// mul) + 16 packed conversions; grads(u): 8 MFMA for dV and dK.  (Measured and not kept: interleaving the matrix
// instructions of one unit with the vector instructions of the other inside the wavefront, no gain - the second
// wavefront of the SIMD already fills those slots; 64 keys per wavefront with one wavefront per SIMD, slower.)
// ring depth: tiles t+1, t+2 in flight or landed while tile t is worked on, t+3 requested (three slots: 1 % slower;
// three slots and three wavefronts per SIMD, which the registers allow with ten spills: 3 % slower)
constexpr int kBwdKvSlots = 4;
struct __attribute__((aligned(16))) SmemBwdKv {
    __bf16 q[kBwdKvSlots][kTileElems];
    __bf16 g[kBwdKvSlots][kTileElems];
    float ld[kBwdKvSlots][4][64];  // per slot: [0] lse * log2e, [1] -delta, [2], [3] the other two wavefronts' copies
};

__global__ void __launch_bounds__(256, 2)
attn_bwd_dkdv_bf16_d64(BwdParams p) {
    __shared__ SmemBwdKv sm;
    const BwdItem wi = decode_bwd(p.BH, p.n_k_blocks);
    if (!wi.valid) return;
    const int k_block = wi.item;  // block 0 is seen by every row: heaviest first

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, h = lane >> 5;
    const int k0 = k_block * 128;
    const int kw0 = k0 + wave * 32;

    const __bf16* qg = (const __bf16*)p.q + (int64_t)wi.bh * p.Sq * kD;
    const __bf16* gg = (const __bf16*)p.dout + (int64_t)wi.bh * p.Sq * kD;
    const __bf16* kg = (const __bf16*)p.k + (int64_t)wi.bh * p.Scap * kD;
    const __bf16* vg = (const __bf16*)p.v + (int64_t)wi.bh * p.Scap * kD;
    const float* lse_g = p.lse2 + (int64_t)wi.bh * p.Sq;
    const float* dl_g = p.neg_delta + (int64_t)wi.bh * p.Sq;

    // ---- this wavefront's keys: B operands K^T, V^T and the visibility bound of the lane's key ----
    const int key = kw0 + n;
    const int kc = min(key, p.Sk - 1);           // ragged tail: a duplicate column, never stored
    const int rmin_lane = (kc / p.T - p.P) * p.T;  // <= 0: visible to every row
    bf16x8 kf[4], vf[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        kf[ks] = *(const bf16x8*)(kg + (int64_t)kc * kD + 16 * ks + 8 * h);
        vf[ks] = *(const bf16x8*)(vg + (int64_t)kc * kD + 16 * ks + 8 * h);
    }
    const bool wave_active = kw0 < p.Sk;
    const int kw_first = min(kw0, p.Sk - 1), kw_last = min(kw0 + 31, p.Sk - 1);
    const int rmin_wave = (kw_first / p.T - p.P) * p.T;  // tiles ending at or below it are skipped by this wavefront
    const int rmax_wave = (kw_last / p.T - p.P) * p.T;   // tiles starting at or above it need no mask
    const int rmin_wg = max(0, (k0 / p.T - p.P) * p.T);
    const int t_begin = rmin_wg / 64;
    const int t_end = (p.Sq + 63) / 64;

    f32x16 dk_acc[2], dv_acc[2];  // [dt]
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) { dk_acc[a][r] = 0.f; dv_acc[a][r] = 0.f; }
    const float c = p.scale_log2e;

    const int ld_row = 8 * wave + (lane >> 3);
    const int ld_chunk = (lane & 7) ^ chunk_swizzle(ld_row);
    const unsigned lds_q0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)(&sm.q[0][0]) + wave * 1024;
    const unsigned lds_g0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)(&sm.g[0][0]) + wave * 1024;
    const unsigned lds_ld0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)(&sm.ld[0][0][0]) + wave * 256;
    const float* row_vec = (wave & 1) ? dl_g : lse_g;  // wavefronts 0, 2 fetch lse log2(e), 1, 3 -delta
    auto load_tile = [&](int t, int slot) {  // five loads per wavefront and tile
        dma_tile_pair(qg, gg, t * 64, p.Sq, lds_q0 + slot * kTileElems * 2, lds_g0 + slot * kTileElems * 2, ld_row, ld_chunk);
        const int r = min(t * 64 + lane, p.Sq - 1);
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dword %0, off" ::"v"(row_vec + r), "s"(lds_ld0 + slot * 1024) : "memory", "m0");
    };
    const FragOffsets fo = frag_offsets(lane);

#pragma unroll
    for (int i = 0; i < kBwdKvSlots - 1; ++i)
        if (t_begin + i < t_end) load_tile(t_begin + i, i);
    wait_vmem_all();

    int slot = 0, slot_load = kBwdKvSlots - 1;
    for (int t = t_begin; t < t_end; ++t) {
        // tile t has landed for this wavefront once only the loads of later tiles (five each) are in flight; after the
        // barrier it has landed for all, and every wavefront is done with tile t-1, whose slot tile t+3 takes
        __builtin_amdgcn_sched_barrier(0);
        if (kBwdKvSlots > 3 && t + 2 < t_end) asm volatile("s_waitcnt vmcnt(10)" ::: "memory");
        else if (t + 1 < t_end) asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        if (t + kBwdKvSlots - 1 < t_end) load_tile(t + kBwdKvSlots - 1, slot_load);
        const int i0 = t * 64;
        if (wave_active && i0 + 64 > rmin_wave) {
            const __bf16* qs_ = sm.q[slot];
            const __bf16* gs_ = sm.g[slot];
            const bool need_mask = i0 < rmax_wave;
            const bool ragged = i0 + 64 > p.Sq;
            f32x16 s_acc[2], dp_acc[2];  // [qb]: the two 32-row units of the tile (one after the other)
            f32x4 lse4[2][4];            // [qb][g4]
            bf16x8 pk[2][2], dsk[2][2];  // [qb][g]: P and dS as operands of the second products
            // rows of this lane in unit qb: i0 + 32 qb + 8 g4 + 4 h + e, g4 = 0..3, e = 0..3: accumulator element 4 g4 + e
            auto scores = [&](int qb) {
                bf16x8 qa[4], ga[4];
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    qa[ks] = lds_read_b128(qs_ + 32 * qb * kD + fo.row_frag[ks]);
                    ga[ks] = lds_read_b128(gs_ + 32 * qb * kD + fo.row_frag[ks]);
                }
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    lse4[qb][g4] = *(const f32x4*)(&sm.ld[slot][0][32 * qb + 8 * g4 + 4 * h]);
                    const f32x4 nd = *(const f32x4*)(&sm.ld[slot][1][32 * qb + 8 * g4 + 4 * h]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) dp_acc[qb][4 * g4 + e] = nd[e];  // dP starts at -delta
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) s_acc[qb][r] = 0.f;
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    s_acc[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa[ks], kf[ks], s_acc[qb], 0, 0, 0);
                    dp_acc[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ga[ks], vf[ks], dp_acc[qb], 0, 0, 0);
                }
            };
            auto weights = [&](int qb) {
                if (need_mask || ragged) {  // wave-uniform: rows the lane's key may not see, and the clamped
                                            // duplicate rows of a ragged last tile
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int i = i0 + 32 * qb + 8 * (r >> 2) + 4 * h + (r & 3);
                        if (i < rmin_lane || i >= p.Sq) s_acc[qb][r] = -INFINITY;
                    }
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float pr = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[qb][r], c, -lse4[qb][r >> 2][r & 3]));
                    s_acc[qb][r] = pr;                   // P
                    dp_acc[qb][r] = pr * dp_acc[qb][r];  // dS = P (dP - delta)
                }
#pragma unroll
                for (int g = 0; g < 2; ++g) { pk[qb][g] = pack8(s_acc[qb], g); dsk[qb][g] = pack8(dp_acc[qb], g); }
            };
            auto grads = [&](int qb) {
#pragma unroll
                for (int g = 0; g < 2; ++g)
#pragma unroll
                    for (int dt = 0; dt < 2; ++dt) {
                        const bf16x8 gt = read_tr_frag(gs_, fo, qb, g, dt);  // dO^T
                        const bf16x8 qt = read_tr_frag(qs_, fo, qb, g, dt);  // Q^T
                        dv_acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gt, pk[qb][g], dv_acc[dt], 0, 0, 0);
                        dk_acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qt, dsk[qb][g], dk_acc[dt], 0, 0, 0);
                    }
            };
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                scores(qb);
                weights(qb);
                grads(qb);
            }
        }
        slot = slot == kBwdKvSlots - 1 ? 0 : slot + 1;
        slot_load = slot_load == kBwdKvSlots - 1 ? 0 : slot_load + 1;
    }

    if (!wave_active || key >= p.Sk) return;
    __bf16* dkg = (__bf16*)p.dk + ((int64_t)wi.bh * p.Scap + key) * kD;
    __bf16* dvg = (__bf16*)p.dv + ((int64_t)wi.bh * p.Scap + key) * kD;
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) {
            const f32x4 xk = {dk_acc[dt][4 * rb] * p.scale, dk_acc[dt][4 * rb + 1] * p.scale,
                              dk_acc[dt][4 * rb + 2] * p.scale, dk_acc[dt][4 * rb + 3] * p.scale};
            const f32x4 xv = {dv_acc[dt][4 * rb], dv_acc[dt][4 * rb + 1], dv_acc[dt][4 * rb + 2], dv_acc[dt][4 * rb + 3]};
            *(bf16x4*)(dkg + 32 * dt + 8 * rb + 4 * h) = __builtin_convertvector(xk, bf16x4);
            *(bf16x4*)(dvg + 32 * dt + 8 * rb + 4 * h) = __builtin_convertvector(xv, bf16x4);
        }
}

}  // namespace mfma
}  // namespace nfd

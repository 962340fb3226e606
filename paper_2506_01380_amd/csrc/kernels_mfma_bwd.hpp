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
//   attn_bwd_dkdv_bf16_d64 key-major: a wavefront owns 48 keys and walks over the query tiles that see them
// Both matrix kernels recompute the weights from the stored log-sum-exp, so no online softmax is
// needed, and both keep the operand whose rows they own in registers for the whole kernel.  Tiles
// of the other operand go global -> LDS directly into the same XOR-swizzled ring as in the forward
// kernel.  As there, every second product takes the accumulator registers of the first as its B
// operand unchanged (the contraction index is permuted identically on the A side by the transposing
// LDS read), so neither P nor dS ever touches LDS.
//
// Register budget: both kernels run two wavefronts per SIMD - the dq kernel by forming the scores of
// 32 keys and 16 queries at a time, the dk/dv kernel by owning 48 keys per wavefront.  S and dP are formed in both
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

// ---------------------------------------------------------------------------------------------
// dq: a workgroup owns 256 query rows (4 wavefronts x 64), walks over the visible key tiles.
//   S^T = K.Q^T, dP^T = V.dO^T (A = K / V rows from LDS, B = Q^T / dO^T in registers)
//   dS^T = P^T o (dP^T - delta),  dQ^T += K^T.dS^T (A = K^T by transposing read, B = dS^T accumulators)
// 16x16x32 shape of the matrix instruction, in the register layout of the forward kernel (kernels_mfma16.hpp): lane =
// (j, g), j = lane % 16, g = lane / 16; a wavefront's 64 rows are four column blocks cq of 16 queries, a lane owns
// query 16 cq + j of each; 32 keys at a time as two 16-key blocks, operand row i of a block being tile row
// 4 sg(i / 4) + i % 4, sg = (0, 2, 3, 1).  The accumulators of S^T and dP^T give lane (j, g) keys 4 sg(g) .. + 3 of both
// blocks: the eight values of dS^T it needs as B operand of the third product, whose A operand K^T comes from the
// transposing read in the same key order.  The per-row values are per-lane scalars here: lse log2(e) goes into the
// exponent's fma, and dP^T starts from -delta (a four-register C operand per column block, kept for the whole kernel),
// so dP - delta costs no instruction.  The four column blocks are worked one after the other on the same K, V and K^T
// fragments: a quarter of the scores live at a time.
__global__ void __launch_bounds__(256, 2)
attn_bwd_dq_bf16_d64(BwdParams p) {
    __shared__ SmemRing sm;
    const BwdItem wi = decode_bwd(p.BH, p.n_q_tiles);
    if (!wi.valid) return;
    const int q_tile = p.n_q_tiles - 1 - wi.item;  // heaviest (latest frames) first

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 15, g = lane >> 4;
    auto sg = [](int x) { return (0x78 >> (2 * x)) & 3; };  // 0, 2, 3, 1
    const int r0 = q_tile * kBM;
    const int r_last = min(r0 + kBM, p.Sq) - 1;
    const int n_tiles = (kmax_of_row(r_last, p.T, p.P) + kBN - 1) / kBN;

    const __bf16* qg = (const __bf16*)p.q + (int64_t)wi.bh * p.Sq * kD;
    const __bf16* gg = (const __bf16*)p.dout + (int64_t)wi.bh * p.Sq * kD;
    const __bf16* og_ = (const __bf16*)p.out + (int64_t)wi.bh * p.Sq * kD;
    const __bf16* kg = (const __bf16*)p.k + (int64_t)wi.bh * p.Scap * kD;
    const __bf16* vg = (const __bf16*)p.v + (int64_t)wi.bh * p.Scap * kD;

    const int rw0 = r0 + wave * 64;
    float lse2[4];
    f32x4 ndl[4];            // [cq] -delta of the lane's query in all four elements: the C operand dP^T starts from
    bf16x8 qf[4][2], gf[4][2];  // [cq][ks]
#pragma unroll
    for (int cq = 0; cq < 4; ++cq) {
        const int row = rw0 + 16 * cq + j;
        const int rc = min(row, p.Sq - 1);  // ragged tail: compute a duplicate, never store it
        lse2[cq] = p.lse[(int64_t)wi.bh * p.Sq + rc] * kLog2e;
        float part = 0.f;  // this lane's quarter of <dout_i, out_i>: the features it holds of dout
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            qf[cq][ks] = *(const bf16x8*)(qg + (int64_t)rc * kD + 32 * ks + 8 * g);
            gf[cq][ks] = *(const bf16x8*)(gg + (int64_t)rc * kD + 32 * ks + 8 * g);
            const bf16x8 of = *(const bf16x8*)(og_ + (int64_t)rc * kD + 32 * ks + 8 * g);
#pragma unroll
            for (int e = 0; e < 8; ++e) part = __builtin_fmaf((float)gf[cq][ks][e], (float)of[e], part);
        }
        part += __shfl_xor(part, 16);
        const float dl = part + __shfl_xor(part, 32);
#pragma unroll
        for (int e = 0; e < 4; ++e) ndl[cq][e] = -dl;
        if (g == 0 && row < p.Sq) {  // for the dk/dv kernel
            p.neg_delta[(int64_t)wi.bh * p.Sq + row] = -dl;
            p.lse2[(int64_t)wi.bh * p.Sq + row] = lse2[cq];
        }
    }
    const int kmin_wave = kmax_of_row(min(rw0, p.Sq - 1), p.T, p.P);
    const int kmax_wave = kmax_of_row(min(rw0 + 63, p.Sq - 1), p.T, p.P);
    const bool wave_active = rw0 < p.Sq;

    f32x4 dq_acc[4][4];  // [cq][fb]: query 16 cq + j, features 16 fb + 4 g + e
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int e = 0; e < 4; ++e) dq_acc[a][b][e] = 0.f;
    const float c = p.scale_log2e;

    const int ld_row = 8 * wave + (lane >> 3);
    const int ld_chunk = (lane & 7) ^ chunk_swizzle(ld_row);
    const unsigned lds_k0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)(&sm.k[0][0]) + wave * 1024;
    const unsigned lds_v0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)(&sm.v[0][0]) + wave * 1024;
    auto load_tile = [&](int t, int slot) {
        dma_tile_pair(kg, vg, t * kBN, p.Sk, lds_k0 + slot * kTileElems * 2, lds_v0 + slot * kTileElems * 2, ld_row, ld_chunk);
    };
    // per-lane fragment offsets (elements) under the swizzle; blocks at + 16, + 32, + 48 rows have the same swizzle
    const int a_row = 4 * sg(j >> 2) + (j & 3);
    const int fa = chunk_swizzle(a_row);
    int a_off[2];  // [ks]: rows of K / V as A operands
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) a_off[ks] = a_row * kD + 8 * ((4 * ks + g) ^ fa);
    const int t_row = 4 * sg(g) + (j >> 2);
    const int ft = chunk_swizzle(t_row);
    int t_off[4];  // [fb]: transposed fragments of K
#pragma unroll
    for (int fb = 0; fb < 4; ++fb) t_off[fb] = t_row * kD + 8 * ((2 * fb + ((j & 3) >> 1)) ^ ft) + 4 * (j & 1);
    const int key_lane = 4 * sg(g);  // first of the lane's four keys of a 16-key block

    if (0 < n_tiles) load_tile(0, 0);
    if (1 < n_tiles) load_tile(1, 1);
    wait_vmem_all();  // q, dout, out, lse fragments and the first tiles have landed (and the compiler knows it)

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
            for (int kb = 0; kb < 2; ++kb) {  // 32 keys at a time
                bf16x8 kf[2][2], vf[2][2];   // [key block][ks]
                bf16x8 kt[4];                // [fb] K^T of the 32 keys
#pragma unroll
                for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) {
                        kf[b2][ks] = lds_read_b128(ks_ + (32 * kb + 16 * b2) * kD + a_off[ks]);
                        vf[b2][ks] = lds_read_b128(vs_ + (32 * kb + 16 * b2) * kD + a_off[ks]);
                    }
#pragma unroll
                for (int fb = 0; fb < 4; ++fb) {
                    const __bf16* tp = ks_ + 32 * kb * kD + t_off[fb];
                    const s16x4 lo = lds_read_tr(tp);
                    const s16x4 hi = lds_read_tr(tp + 16 * kD);
                    typedef __attribute__((ext_vector_type(8))) short s16x8;
                    kt[fb] = __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                }
#pragma unroll
                for (int cq = 0; cq < 4; ++cq) {  // one column block of queries at a time: a quarter of the scores live
                    f32x4 s_acc[2], dp_acc[2];    // [key block]
#pragma unroll
                    for (int b2 = 0; b2 < 2; ++b2) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) s_acc[b2][e] = 0.f;
                        dp_acc[b2] = ndl[cq];
                    }
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                        for (int b2 = 0; b2 < 2; ++b2) {
                            s_acc[b2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[b2][ks], qf[cq][ks], s_acc[b2], 0, 0, 0);
                            dp_acc[b2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[b2][ks], gf[cq][ks], dp_acc[b2], 0, 0, 0);
                        }
                    if (need_mask) {
                        const int left = kmax_of_row(min(rw0 + 16 * cq + j, p.Sq - 1), p.T, p.P) - (j0 + 32 * kb + key_lane);
#pragma unroll
                        for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (16 * b2 + e >= left) s_acc[b2][e] = -INFINITY;
                    }
                    // dS^T = P^T o (dP^T - delta), written over the dP accumulators
#pragma unroll
                    for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float pr = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[b2][e], c, -lse2[cq]));
                            dp_acc[b2][e] = pr * dp_acc[b2][e];
                        }
                    bf16x8 ds;  // positions 0..3 from the first key block, 4..7 from the second
#pragma unroll
                    for (int e = 0; e < 4; e += 2) {
                        const f32x2 x = {dp_acc[0][e], dp_acc[0][e + 1]}, y = {dp_acc[1][e], dp_acc[1][e + 1]};
                        const bf16x2 xb = __builtin_convertvector(x, bf16x2), yb = __builtin_convertvector(y, bf16x2);
                        ds[e] = xb[0]; ds[e + 1] = xb[1]; ds[4 + e] = yb[0]; ds[5 + e] = yb[1];
                    }
#pragma unroll
                    for (int fb = 0; fb < 4; ++fb)
                        dq_acc[cq][fb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kt[fb], ds, dq_acc[cq][fb], 0, 0, 0);
                }
            }
        }
        slot = slot == 2 ? 0 : slot + 1;
    }

    if (!wave_active) return;
#pragma unroll
    for (int cq = 0; cq < 4; ++cq) {
        const int row = rw0 + 16 * cq + j;
        if (row >= p.Sq) continue;
        __bf16* og = (__bf16*)p.dq + ((int64_t)wi.bh * p.Sq + row) * kD;
#pragma unroll
        for (int fb = 0; fb < 4; ++fb) {
            const f32x4 x = dq_acc[cq][fb] * p.scale;
            *(bf16x4*)(og + 16 * fb + 4 * g) = __builtin_convertvector(x, bf16x4);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// dk, dv: a workgroup owns 192 keys (4 wavefronts x 48, two wavefronts per SIMD) and walks over the 64-row query
// tiles that can see them (all rows from the first frame that sees the block's first key).
//   S = Q.K^T, dP = dO.V^T (A = Q / dO rows from LDS, B = K^T / V^T in registers)
//   dV^T += dO^T.P, dK^T += Q^T.dS (A by transposing reads of the dO / Q tile, B = P / dS accumulators)
// In the accumulator layout a lane holds ONE key column per column block and four of a block's sixteen query rows, so
// the per-row values come from LDS (one 16-byte read each per row block), in the form the dq kernel left them:
// lse log2(e), subtracted inside the exponent's fma, and -delta, which is what the dP accumulators start from
// (the matrix instruction adds the product to it), so dP - delta costs no instruction.
// Key j is visible to row i iff i >= rmin(j) = (floor(j/T) - P) T: one bound per lane and column block, no division
// in the loop.
//
// The 16x16x32 shape of the matrix instruction, in the register layout of the forward kernel (kernels_mfma16.hpp).
// Lane = (j, g), j = lane % 16, g = lane / 16.  A wavefront's 48 keys are three column blocks ck of 16; a 32-row unit of
// a query tile is two row blocks rb of 16.  Operand row i of a row block is tile row 4 sg(i / 4) + i % 4, sg = (0, 2, 3, 1)
// (the order that keeps both kinds of fragment reads free of bank conflicts under the tile swizzle), so
//   S[rb][ck], dP[rb][ck]   A = Q / dO rows (16-byte LDS reads), B = K^T / V^T (registers)
//                           D: key 16 ck + j, rows 4 sg(g) + e of the block, e = 0..3
//   dV^T[fb][ck], dK^T[fb][ck]  A = dO^T / Q^T (transposing reads: features 16 fb + j, rows at positions (g, 0..7) =
//                           rows 4 sg(g) .. + 3 of the unit's first block, then of its second), B = P / dS: exactly the
//                           eight values lane (j, g) holds of the unit's two blocks, packed
//                           D: key 16 ck + j, features 16 fb + 4 g + e
// A query tile is two units of 32 rows; per unit 24 MFMA for S and dP, 24 x (fma, exp2, mul) + 24 packed conversions,
// 24 MFMA for dV and dK, 20 KB of LDS fragment reads.  (The same kernel on the 32x32x16 instruction with 32 keys per
// wavefront - 16 of a block's 32 rows per lane, 24 KB of reads per unit of 32 MFMA - measured 0.835 against 0.804 ms for
// the whole backward at 16 frames of 336 tokens with 32 keys per wavefront on this instruction.  Also measured there and not kept: interleaving the matrix instructions of one unit with the vector
// instructions of the other inside the wavefront, no gain - the second wavefront of the SIMD already fills those
// slots; 64 keys per wavefront with one wavefront per SIMD, slower.)
// ring depth: tiles t+1, t+2 in flight or landed while tile t is worked on, t+3 requested (three slots: 1 % slower;
// three slots and three wavefronts per SIMD, which the registers allow with ten spills: 3 % slower)
constexpr int kBwdKvSlots = 4;
// 16-key column blocks per wavefront.  Every fragment of Q, dO and their transposes that comes out of LDS feeds one
// matrix instruction per column block, so the LDS bytes per FLOP fall with the block count; the accumulators of dK^T
// and dV^T and the K^T, V^T operands grow with it.  Three blocks (48 keys per wavefront, 192 per workgroup) are what
// two wavefronts per SIMD leave room for: 252 VGPRs, no spills (two blocks: 178; four: 118 spilled dwords).  Measured
// on one box, whole backward at 16 frames of 336 tokens: 0.776 ms with two blocks, 0.742 with three.
constexpr int kBwdColBlocks = 3;
constexpr int kBwdKeysPerWorkgroup = 4 * 16 * kBwdColBlocks;
struct __attribute__((aligned(16))) SmemBwdKv {
    __bf16 q[kBwdKvSlots][kTileElems];
    __bf16 g[kBwdKvSlots][kTileElems];
    float ld[kBwdKvSlots][4][64];  // per slot: [0] lse * log2e, [1] -delta, [2], [3] the other two wavefronts' copies
};

__global__ void __launch_bounds__(256, 2)
attn_bwd_dkdv_bf16_d64(BwdParams p) {
    constexpr int NCK = kBwdColBlocks, kWaveKeys = 16 * NCK;
    __shared__ SmemBwdKv sm;
    const BwdItem wi = decode_bwd(p.BH, p.n_k_blocks);
    if (!wi.valid) return;
    const int k_block = wi.item;  // block 0 is seen by every row: heaviest first

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 15, g = lane >> 4;
    auto sg = [](int x) { return (0x78 >> (2 * x)) & 3; };  // 0, 2, 3, 1
    const int k0 = k_block * 4 * kWaveKeys;
    const int kw0 = k0 + wave * kWaveKeys;

    const __bf16* qg = (const __bf16*)p.q + (int64_t)wi.bh * p.Sq * kD;
    const __bf16* gg = (const __bf16*)p.dout + (int64_t)wi.bh * p.Sq * kD;
    const __bf16* kg = (const __bf16*)p.k + (int64_t)wi.bh * p.Scap * kD;
    const __bf16* vg = (const __bf16*)p.v + (int64_t)wi.bh * p.Scap * kD;
    const float* lse_g = p.lse2 + (int64_t)wi.bh * p.Sq;
    const float* dl_g = p.neg_delta + (int64_t)wi.bh * p.Sq;

    // ---- this wavefront's keys: B operands K^T, V^T and the visibility bound of the lane's two keys ----
    int key[NCK], rmin_lane[NCK];
    bf16x8 kf[NCK][2], vf[NCK][2];  // [ck][ks]
#pragma unroll
    for (int ck = 0; ck < NCK; ++ck) {
        key[ck] = kw0 + 16 * ck + j;
        const int kc = min(key[ck], p.Sk - 1);  // ragged tail: a duplicate column, never stored
        rmin_lane[ck] = (kc / p.T - p.P) * p.T;  // <= 0: visible to every row
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            kf[ck][ks] = *(const bf16x8*)(kg + (int64_t)kc * kD + 32 * ks + 8 * g);
            vf[ck][ks] = *(const bf16x8*)(vg + (int64_t)kc * kD + 32 * ks + 8 * g);
        }
    }
    const bool wave_active = kw0 < p.Sk;
    const int kw_first = min(kw0, p.Sk - 1), kw_last = min(kw0 + kWaveKeys - 1, p.Sk - 1);
    const int rmin_wave = (kw_first / p.T - p.P) * p.T;  // tiles ending at or below it are skipped by this wavefront
    const int rmax_wave = (kw_last / p.T - p.P) * p.T;   // tiles starting at or above it need no mask
    const int rmin_wg = max(0, (k0 / p.T - p.P) * p.T);
    const int t_begin = rmin_wg / 64;
    const int t_end = (p.Sq + 63) / 64;

    f32x4 dk_acc[4][NCK], dv_acc[4][NCK];  // [fb][ck]
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < NCK; ++b)
#pragma unroll
            for (int e = 0; e < 4; ++e) { dk_acc[a][b][e] = 0.f; dv_acc[a][b][e] = 0.f; }
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
    // per-lane fragment offsets (elements) under the swizzle; blocks at + 16, + 32, + 48 rows have the same swizzle
    const int a_row = 4 * sg(j >> 2) + (j & 3);
    const int fa = chunk_swizzle(a_row);
    int a_off[2];  // [ks]: rows of Q / dO as A operands
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) a_off[ks] = a_row * kD + 8 * ((4 * ks + g) ^ fa);
    const int t_row = 4 * sg(g) + (j >> 2);
    const int ft = chunk_swizzle(t_row);
    int t_off[4];  // [fb]: transposed fragments of Q / dO
#pragma unroll
    for (int fb = 0; fb < 4; ++fb) t_off[fb] = t_row * kD + 8 * ((2 * fb + ((j & 3) >> 1)) ^ ft) + 4 * (j & 1);
    const int vec_row = 4 * sg(g);  // first of the lane's four rows of a 16-row block
    auto read_t = [&](const __bf16* tile, int qb, int fb) {
        const __bf16* tp = tile + 32 * qb * kD + t_off[fb];
        const s16x4 lo = lds_read_tr(tp);
        const s16x4 hi = lds_read_tr(tp + 16 * kD);
        typedef __attribute__((ext_vector_type(8))) short s16x8;
        return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    auto pack2 = [&](const f32x4& a, const f32x4& b) {  // positions 0..3 from the first row block, 4..7 from the second
        bf16x8 r;
#pragma unroll
        for (int e = 0; e < 4; e += 2) {
            const f32x2 x = {a[e], a[e + 1]}, y = {b[e], b[e + 1]};
            const bf16x2 xb = __builtin_convertvector(x, bf16x2), yb = __builtin_convertvector(y, bf16x2);
            r[e] = xb[0]; r[e + 1] = xb[1]; r[4 + e] = yb[0]; r[5 + e] = yb[1];
        }
        return r;
    };

#pragma unroll
    for (int i = 0; i < kBwdKvSlots - 1; ++i)
        if (t_begin + i < t_end) load_tile(t_begin + i, i);
    wait_vmem_all();

    int slot = 0, slot_load = kBwdKvSlots - 1;
    for (int t = t_begin; t < t_end; ++t) {
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
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                f32x4 s_acc[2][NCK], dp_acc[2][NCK];  // [rb][ck]
                f32x4 lse4[2];                    // [rb]
                bf16x8 qa[2][2], ga[2][2];        // [rb][ks]
#pragma unroll
                for (int rb = 0; rb < 2; ++rb) {
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) {
                        qa[rb][ks] = lds_read_b128(qs_ + (32 * qb + 16 * rb) * kD + a_off[ks]);
                        ga[rb][ks] = lds_read_b128(gs_ + (32 * qb + 16 * rb) * kD + a_off[ks]);
                    }
                    lse4[rb] = *(const f32x4*)(&sm.ld[slot][0][32 * qb + 16 * rb + vec_row]);
                    const f32x4 nd = *(const f32x4*)(&sm.ld[slot][1][32 * qb + 16 * rb + vec_row]);
#pragma unroll
                    for (int ck = 0; ck < NCK; ++ck) {
                        dp_acc[rb][ck] = nd;  // dP starts at -delta
#pragma unroll
                        for (int e = 0; e < 4; ++e) s_acc[rb][ck][e] = 0.f;
                    }
                }
#pragma unroll
                for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                        for (int ck = 0; ck < NCK; ++ck) {
                            s_acc[rb][ck] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa[rb][ks], kf[ck][ks], s_acc[rb][ck], 0, 0, 0);
                            dp_acc[rb][ck] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ga[rb][ks], vf[ck][ks], dp_acc[rb][ck], 0, 0, 0);
                        }
                if (need_mask || ragged) {  // wave-uniform: rows a lane's key may not see, and the clamped duplicate
                                            // rows of a ragged last tile
#pragma unroll
                    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int i = i0 + 32 * qb + 16 * rb + vec_row + e;
#pragma unroll
                            for (int ck = 0; ck < NCK; ++ck)
                                if (i < rmin_lane[ck] || i >= p.Sq) s_acc[rb][ck][e] = -INFINITY;
                        }
                }
#pragma unroll
                for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                    for (int ck = 0; ck < NCK; ++ck)
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float pr = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[rb][ck][e], c, -lse4[rb][e]));
                            s_acc[rb][ck][e] = pr;                         // P
                            dp_acc[rb][ck][e] = pr * dp_acc[rb][ck][e];    // dS = P (dP - delta)
                        }
                bf16x8 pk[NCK], dsk[NCK];  // [ck]
#pragma unroll
                for (int ck = 0; ck < NCK; ++ck) {
                    pk[ck] = pack2(s_acc[0][ck], s_acc[1][ck]);
                    dsk[ck] = pack2(dp_acc[0][ck], dp_acc[1][ck]);
                }
#pragma unroll
                for (int fb = 0; fb < 4; ++fb) {
                    const bf16x8 gt = read_t(gs_, qb, fb);  // dO^T
                    const bf16x8 qt = read_t(qs_, qb, fb);  // Q^T
#pragma unroll
                    for (int ck = 0; ck < NCK; ++ck) {
                        dv_acc[fb][ck] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(gt, pk[ck], dv_acc[fb][ck], 0, 0, 0);
                        dk_acc[fb][ck] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qt, dsk[ck], dk_acc[fb][ck], 0, 0, 0);
                    }
                }
            }
        }
        slot = slot == kBwdKvSlots - 1 ? 0 : slot + 1;
        slot_load = slot_load == kBwdKvSlots - 1 ? 0 : slot_load + 1;
    }

    if (!wave_active) return;
#pragma unroll
    for (int ck = 0; ck < NCK; ++ck) {
        if (key[ck] >= p.Sk) continue;
        __bf16* dkg = (__bf16*)p.dk + ((int64_t)wi.bh * p.Scap + key[ck]) * kD;
        __bf16* dvg = (__bf16*)p.dv + ((int64_t)wi.bh * p.Scap + key[ck]) * kD;
#pragma unroll
        for (int fb = 0; fb < 4; ++fb) {
            const f32x4 xk = dk_acc[fb][ck] * p.scale;
            *(bf16x4*)(dkg + 16 * fb + 4 * g) = __builtin_convertvector(xk, bf16x4);
            *(bf16x4*)(dvg + 16 * fb + 4 * g) = __builtin_convertvector(dv_acc[fb][ck], bf16x4);
        }
    }
}

}  // namespace mfma
}  // namespace nfd

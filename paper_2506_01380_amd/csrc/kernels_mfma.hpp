// bf16 matrix-core forward kernels for head width 64 (gfx950 / CDNA4): what all shapes share, and the shapes built
// on the 32x32x16 matrix instruction - the 128-row latency shape, and both shapes over the 8-bit cache.  The 256-row
// throughput shape over a bf16 cache is in kernels_mfma16.hpp (same structure, 16x16x32 instruction).
//
// Flash-style online softmax.  A workgroup of 4 wavefronts owns up to 256 consecutive query rows of
// one (batch, head) - the 32-row blocks of a head are dealt evenly to its query tiles -; each wavefront
// owns 64 of them as two 32-wide column blocks (blocks w and w + 4 of the workgroup's eight; a single
// block where the tile has fewer) of the TRANSPOSED score matrix:
//
//   S^T[key, query] = K_tile[key, :] . Q^T[:, query]       v_mfma_f32_32x32x16_bf16, A = K (LDS), B = Q^T (registers)
//   O^T[d,   query] += V_tile^T[d, key] . P^T[key, query]  A = V^T (LDS, transposing read), B = P^T (registers)
//
// In the 32x32 accumulator layout a lane holds ONE query column (lane % 32) and 16 of the
// 32 key rows, so row max / row sum are register-local plus a single exchange with
// lane ^ 32, and the accumulator registers of S^T are already in the B-operand layout
// the second product needs: P never goes through LDS.
//
// K and V tiles (64 keys) never pass through registers either: every wavefront issues 16-byte
// global loads that land straight in LDS (one wave instruction = 1 KB = eight 128-byte tile
// rows), two tiles ahead of their use, into a ring of three tile slots (three ahead, four slots in the
// pipelined 256-row shape), with one bare barrier per tile.  A wave's 1 KB is contiguous in LDS, so rows
// cannot be padded; bank conflicts are avoided with an XOR swizzle instead: the 16-byte chunk c of tile row r is stored at chunk
// position c ^ f(r).  The swizzle costs nothing on the way in (each lane simply fetches the
// chunk that belongs at its position) and one precomputed per-lane offset on the way out.
//
// Softmax is optimistic: P is formed against the reference max of earlier tiles without
// looking at this tile's max; only if a lane's tile sum reaches kOptimisticLimit (which also
// catches inf, i.e. the first tile of a row) the tile is redone with its exact max and the
// accumulators are rescaled.  The softmax scale lives in the query fragments (rounded to bf16), so the
// score accumulators hold base-2 exponents.  The forward of the training pair (EXACTQ) keeps the
// queries as given and scales the fp32 scores instead.
//
// Mask (Sec. 3.1): row i sees keys j < kmax(i) = (P + i/T + 1) * T.  Key tiles entirely
// below every row's bound run with no mask arithmetic; tiles at or beyond the largest
// bound of the workgroup (of the wavefront) are never visited (computed); only the tiles in
// between compare the key index with the lane's bound.
#pragma once
#include <type_traits>

#include "nfd_common.hpp"

namespace nfd {
namespace mfma {

constexpr int kD = 64;                        // head width
constexpr int kBN = 64;                       // keys per tile
constexpr int kBM = 256;                      // query rows per workgroup (throughput shape; 128 in the latency shape)
constexpr int kWaves = 4;                     // wavefronts per workgroup, 64 query rows each
constexpr int kTileElems = kBN * kD;          // 4096 bf16 = 8 KB, rows of 128 B, no padding
constexpr int kRingSlots = 3;                 // K and V ring depth (tiles)
constexpr float kOptimisticLimit = 32768.0f;  // 2^15 per lane and tile (32 values)
constexpr int kMfmaPriority = 2;              // wave priority while it feeds the matrix pipe

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

// Chunk-position swizzle of a tile row: a bijection of (r >> 1) & 7 whose bit 2 toggles every two rows.
// Measured conflict-free for both the 16-byte fragment reads (32 consecutive rows, one chunk) and the
// transposing 8-byte reads (4 rows x 64 bytes per 32 lanes) on this LDS.
__device__ __forceinline__ int chunk_swizzle(int r) {
    const int k = (r >> 1) & 7;
    return ((k & 1) << 2) | (k >> 1);
}

struct __attribute__((aligned(16))) SmemRing {
    __bf16 k[kRingSlots][kTileElems];
    __bf16 v[kRingSlots][kTileElems];
};
// The pipelined 256-row shape (kernels_mfma16.hpp) keeps the V tile of the previous key tile alive while it works on
// the K tile of the next one, so its ring is one slot deeper for the same prefetch distance (64 KB, two workgroups
// per CU).
constexpr int kPipeSlots = 4;
struct __attribute__((aligned(16))) SmemRingPipe {
    __bf16 k[kPipeSlots][kTileElems];
    __bf16 v[kPipeSlots][kTileElems];
};

// 8-bit cache (E4M3 codes): a K tile is 64 keys x 64 features, a V tile 64 features x 64 keys (V is stored
// feature-major), both 64 rows of 64 bytes.  One wave instruction of 16-byte loads fills 16 tile rows, so a tile
// is one load per wavefront and tensor.  The 16-byte chunk c of row r sits at chunk position c ^ ((r >> 2) & 3):
// measured conflict-free for the 16-byte fragment reads (lane n of a half-wavefront reads one chunk of row n;
// such loads are served in groups of lanes {0-3, 12-15, 20-23, 24-27}, {4-7, 8-11, 16-19, 28-31}, same + 32).
struct __attribute__((aligned(16))) SmemRing8 {
    unsigned char k[kRingSlots][kTileElems];
    unsigned char v[kRingSlots][kTileElems];
};
__device__ __forceinline__ int chunk_swizzle8(int r) { return (r >> 2) & 3; }

// 64-row workgroup shape over the 8-bit cache: the four wavefronts widen each tile ONCE, together, from the
// ring of code tiles into a double-buffered pair of bf16 tiles in the bf16 kernel's layout (V with the 8 keys of
// one matrix operand contiguous), one tile ahead of its use; the products then read bf16 fragments.  16
// conversions per wavefront and tile instead of 64.
struct __attribute__((aligned(16))) SmemRing8Wide {
    unsigned char k[kRingSlots][kTileElems];
    unsigned char v[kRingSlots][kTileElems];
    __bf16 kb[2][kTileElems];
    __bf16 vb[2][kTileElems];
};

// Eight E4M3 codes (two dwords, lowest byte first) widened to bf16; every E4M3 value is a bf16 value.
__device__ __forceinline__ bf16x8 widen_e4m3x8(uint32_t w0, uint32_t w1) {
    const bf16x2 a = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w0, 1.0f, false);
    const bf16x2 b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w0, 1.0f, true);
    const bf16x2 c = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w1, 1.0f, false);
    const bf16x2 d = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w1, 1.0f, true);
    const bf16x4 ab = __builtin_shufflevector(a, b, 0, 1, 2, 3);
    const bf16x4 cd = __builtin_shufflevector(c, d, 0, 1, 2, 3);
    return __builtin_shufflevector(ab, cd, 0, 1, 2, 3, 4, 5, 6, 7);
}

// Work decomposition of one launch.  Workgroup ids are dealt round-robin to the 8 XCDs.
// When the head count is a multiple of 8, heads are pinned to an XCD (bh % 8) so that all query
// tiles and key splits of a head share one L2; otherwise pinning would leave XCDs unevenly loaded
// (or idle), and the items are dealt out plainly, consecutive ids going to consecutive heads.
// Order of the items of an XCD (or of the launch):
//  * by default the heaviest query tiles (latest frames) come first, heads fastest, so the tail
//    of the launch is made of the lightest tiles; with more than kHeadGroup heads in the stream they go in
//    groups of that many, one group after the other: the workgroups resident together then belong to few
//    heads and share their K/V tiles in L2 (256 heads x 21 tiles: 917 -> 1017 TFLOP/s), while a group
//    is still large enough to end on light tiles;
//  * group_q_tiles (key-split launches whose K/V exceed the last-level cache): the query tiles of
//    one (head, split) are consecutive instead, so they are resident together and their common
//    K/V range is fetched from HBM once and found in L2 by the others.
constexpr int kHeadGroup = 8;

// The 32-row blocks of a head are dealt to its query tiles as evenly as they go: tile i owns blocks_lo blocks, the
// first n_hi tiles one more, so no tile is mostly padding.  (blocks_lo = n_blocks / n_q_tiles, n_hi = n_blocks mod
// n_q_tiles, n_blocks = ceil(rows / 32).)
__host__ __device__ __forceinline__ void q_tile_blocks(int q_tile, int blocks_lo, int n_hi, int* first_block, int* n_blocks) {
    *first_block = q_tile * blocks_lo + (q_tile < n_hi ? q_tile : n_hi);
    *n_blocks = blocks_lo + (q_tile < n_hi ? 1 : 0);
}

struct WorkItem {
    int bh, q_tile, split;
    bool valid;
};
__host__ __device__ __forceinline__ WorkItem work_item_of(unsigned block, int BH, int n_q_tiles, int n_splits,
                                                          int group_q_tiles) {
    WorkItem w;
    const int per_head = n_q_tiles * n_splits;
    const bool pinned = (BH & 7) == 0;
    const int xcd = pinned ? (int)(block & 7) : 0;
    const int j = pinned ? (int)(block >> 3) : (int)block;
    const int hh = pinned ? BH >> 3 : BH;  // heads this id stream runs over
    w.valid = j < hh * per_head;
    int head_local;
    if (!group_q_tiles) {
        // heads in groups of kHeadGroup: all items of a group before the next group's
        const int per_group = kHeadGroup * per_head;
        const int g0 = j / per_group * kHeadGroup, jj = j % per_group;
        const int gh = max(1, min(kHeadGroup, hh - g0));  // heads of this group (the last one may be smaller; an id past the launch: 1)
        const int item = jj / gh;
        head_local = g0 + jj % gh;
        w.q_tile = n_q_tiles - 1 - item / n_splits;
        w.split = item % n_splits;
    } else {
        const int rest = j / n_q_tiles;
        w.q_tile = n_q_tiles - 1 - j % n_q_tiles;
        head_local = rest % hh;
        w.split = rest / hh;
    }
    w.bh = pinned ? head_local * 8 + xcd : head_local;
    return w;
}
__device__ __forceinline__ WorkItem decode_work(const FwdParams& p) {
    WorkItem w = work_item_of(blockIdx.x, p.BH, p.n_q_tiles, p.n_splits, p.group_q_tiles);
    // the divisions run on the vector unit: bring the (uniform) results back to scalar registers, so that everything
    // derived from them - tensor base pointers above all - is scalar too
    w.bh = __builtin_amdgcn_readfirstlane(w.bh);
    w.q_tile = __builtin_amdgcn_readfirstlane(w.q_tile);
    w.split = __builtin_amdgcn_readfirstlane(w.split);
    return w;
}

// Final write of one wavefront's 64 query rows: normalised bf16 output when the keys were not
// split, otherwise the unnormalised accumulator (bf16) plus (reference max in log2 units, row sum; fp32).
// Lane (n, h) holds, for query column n of block qt, output features 32*dt + 8*rb + 4*h + 0..3.
template <int QT>
__device__ __forceinline__ void store_rows(const FwdParams& p, const WorkItem& wi, const int (&row)[QT], int h,
                                           const f32x16 (&o_acc)[2][QT], const float (&l_sum)[QT],
                                           const float (&m_used)[QT]) {
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
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
            if (p.lse && h == 0) p.lse[(int64_t)wi.bh * p.Sq + row[qt]] = (m_used[qt] + __builtin_log2f(l_row)) * kLn2;
        } else {
            const int64_t prow = ((int64_t)wi.bh * p.n_splits + wi.split) * p.Sq + row[qt];
            __bf16* po = p.part_o + prow * kD;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int rb = 0; rb < 4; ++rb) {
                    const f32x4 x = {o_acc[dt][qt][4 * rb], o_acc[dt][qt][4 * rb + 1], o_acc[dt][qt][4 * rb + 2],
                                     o_acc[dt][qt][4 * rb + 3]};
                    *(bf16x4*)(po + 32 * dt + 8 * rb + 4 * h) = __builtin_convertvector(x, bf16x4);
                }
            if (h == 0) {
                const f32x2 ml = {m_used[qt], l_row};
                *(f32x2*)(p.part_ml + prow * 2) = ml;
            }
        }
    }
}

// QT = 2: 64 query rows per wavefront, 256 per workgroup, two wavefronts per SIMD: the throughput shape.
// QT = 1: 32 rows per wavefront, 128 per workgroup, three wavefronts per SIMD: half the softmax and half the
// matrix work per tile and wavefront, i.e. a shorter chain per key tile, for calls with few query rows whose
// time is the length of that chain (cached forms); it reads twice the LDS bytes per FLOP.
//
// KV8: K and V come from the 8-bit cache and are widened to bf16 (exact) before they reach the matrix operands;
// the per-head scales are folded into the softmax scale (K) and the final write (V), so the arithmetic between
// the operands is the same as for a bf16 cache.  QT = 1: every wavefront widens its own fragments on their way
// out of LDS (SmemRing8); the feature order inside the first product's contraction is then permuted (a 16-byte
// read serves two steps), the same way for K and Q.  QT = 2: the workgroup widens each tile once (SmemRing8Wide).
//
// EXACTQ: the forward of the training pair, which also writes the log-sum-exp the backward normalises with.  The
// queries enter the first product as given, the scores are exact sums of products of the inputs, and the softmax
// scale is applied to the fp32 scores (one multiply per score); the reference max is then kept in raw score units.
// Without it the scale is folded into the query fragments (one more bf16 rounding of an input, no multiply).
template <int QT, bool KV8>
struct SmemOf {
    static_assert(QT == 1 || KV8, "the 256-row shape over a bf16 cache is attn_fwd_item16");
    static constexpr bool WIDE = KV8 && QT == 2;   // tiles widened once per workgroup (see SmemRing8Wide)
    typedef typename std::conditional<WIDE, SmemRing8Wide, typename std::conditional<KV8, SmemRing8, SmemRing>::type>::type type;
};

// One work item (head, query tile, key split) from the first load to the final write.  Every wavefront of the
// workgroup passes the same barriers and returns; the LDS ring may be reused after a workgroup barrier.
template <int QT, bool KV8, bool EXACTQ>
__device__ __forceinline__ void attn_fwd_item(const FwdParams& p, const WorkItem& wi, typename SmemOf<QT, KV8>::type& sm) {
    constexpr int PRIO = kMfmaPriority;
    constexpr bool WIDE = SmemOf<QT, KV8>::WIDE;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, h = lane >> 5;
    int blk0, n_blk;  // this tile's 32-row blocks (at most eight)
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
    // fused append: the new frames' rows, addressed by cache row index (row Snew0 of the cache is row 0 of k_new)
    const bool fused = !KV8 && p.k_new != nullptr;
    const __bf16* kn = fused ? (const __bf16*)p.k_new + ((int64_t)wi.bh * p.Sq - p.Snew0) * kD : kg;
    const __bf16* vn = fused ? (const __bf16*)p.v_new + ((int64_t)wi.bh * p.Sq - p.Snew0) * kD : vg;
    // This workgroup's share of the copy of k_new, v_new into the cache: 16-byte vectors gid, gid + threads, ...
    // The loads go out first and land behind the same wait as the query fragments; the stores follow it.
    constexpr int kMaxCopy = 4;
    u32x4 cp_k[kMaxCopy], cp_v[kMaxCopy];
    int64_t cp_dst[kMaxCopy];
    if constexpr (!KV8) {
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
    }

    // ---- this wavefront's queries -------------------------------------------------------
    // QT = 2: the wavefront owns the 32-row blocks `wave` and `wave + 4` of the workgroup's (up to) eight, not two
    // adjacent ones.  Where a frame boundary falls inside the workgroup, the later frame's extra key tiles are
    // then shared by all four wavefronts (each running one block) instead of keeping the last wavefronts busy
    // with two blocks while the first ones idle.  In a tile of fewer than eight blocks the wavefronts without a
    // block `wave + 4` own block `wave` alone, as their LATER block: the earlier one is dead (no rows, key bound 0),
    // so every tile runs in the second, one-block loop and nothing is computed for rows that do not exist.
    // The softmax scale (times log2 e, times the K scale of an 8-bit cache) is folded into the query fragments once,
    // rounded to bf16: the score accumulators then hold base-2 exponents directly and the softmax needs no multiply.
    float c = p.scale_log2e;
    if constexpr (KV8) c *= p.k_scale[wi.bh];  // scores of the codes -> scores of the values
    int row[QT], kmax_lane[QT];
    int kmin_blk[QT], kmax_blk[QT];  // key bound of a block's first / last row: mask needed above, nothing beyond
    bf16x8 qf[QT][4];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const bool pair = QT == 2 && wave + kWaves < n_blk;   // this wavefront has two blocks
        const bool dead = QT == 2 && qt == 0 && !pair;         // single block: it is block index 1
        const int b0 = r0 + 32 * (QT == 2 && qt == 1 && pair ? wave + kWaves : wave);
        row[qt] = dead ? 0x40000000 : b0 + n;                  // dead rows are never stored
        const int rc = min(row[qt], p.Sq - 1);  // rows past the end: compute a duplicate, never store it
        kmax_lane[qt] = kmax_of_row(rc, p.T, p.P);
        kmin_blk[qt] = dead ? 0 : kmax_of_row(min(b0, p.Sq - 1), p.T, p.P);
        kmax_blk[qt] = dead ? 0 : kmax_of_row(min(b0 + 31, p.Sq - 1), p.T, p.P);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            // contraction step ks, lane half h: features 16*ks + 8*h ..+7; with the 8-bit cache the features of
            // the 16-byte chunk 2*(ks/2) + h, first or second half (ks % 2) - the order the K reads deliver
            const int d0 = KV8 && !WIDE ? 16 * (2 * (ks >> 1) + h) + 8 * (ks & 1) : 16 * ks + 8 * h;
            const bf16x8 raw = *(const bf16x8*)(qg + (int64_t)rc * kD + d0);
            if constexpr (EXACTQ) {
                qf[qt][ks] = raw;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) qf[qt][ks][e] = (__bf16)((float)raw[e] * c);
            }
        }
    }
    const int kmax_wave = kmax_blk[QT - 1];  // tiles starting at or above are skipped (blocks ascend)
    const bool wave_active = wave < n_blk;

    f32x16 o_acc[2][QT];  // [dt][qt]: O^T rows 32*dt.., query block qt
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < QT; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) o_acc[a][b][r] = 0.f;
    float m_used[QT];  // reference max (stale by design), in the units of the score accumulators: base-2 exponents,
                       // or raw scores (exponent = c * score) with EXACTQ
    float l_sum[QT];   // this lane's share of the row sum
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) { m_used[qt] = kNegBig; l_sum[qt] = 0.f; }

    // ---- tile loads: one wave instruction fills 8 consecutive tile rows (1 KB); a wavefront owns
    // rows 8*wave + 32*pass + lane/8, and each lane fetches the chunk that belongs at its position ----
    const int ld_row = 8 * wave + (lane >> 3);
    const int ld_chunk = (lane & 7) ^ chunk_swizzle(ld_row);  // rows +32: same swizzle
    const unsigned ld_voff[2] = {(unsigned)(ld_row * kD + ld_chunk * 8) * 2u, (unsigned)((ld_row + 32) * kD + ld_chunk * 8) * 2u};  // bytes
    const int ld_plain_end = min(p.Sk, p.Snew0);  // tiles that end at or below: whole, and in the cache
    const unsigned lds_k0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)(&sm.k[0][0]) + wave * 1024;
    const unsigned lds_v0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)(&sm.v[0][0]) + wave * 1024;
    // 8-bit cache: one instruction fills 16 tile rows of 64 bytes; the tensors are padded to whole tiles, so no
    // row is clamped (codes past the end are masked: K by the score mask, V explicitly in the last tile)
    const int ld_row8 = 16 * wave + (lane >> 2);
    const int64_t ld_chunk8 = 16 * ((lane & 3) ^ chunk_swizzle8(ld_row8));
    const unsigned char* k_src8 = (const unsigned char*)p.k + ((int64_t)wi.bh * p.Spad + ld_row8) * kD + ld_chunk8;
    const unsigned char* v_src8 = (const unsigned char*)p.v + ((int64_t)wi.bh * kD + ld_row8) * p.Spad + ld_chunk8;
    auto load_tile = [&](int t, int slot) {  // rows past the end are clamped: they are masked anyway
        if constexpr (KV8) {
            const unsigned kdst = lds_k0 + (unsigned)(slot * kTileElems);
            const unsigned vdst = lds_v0 + (unsigned)(slot * kTileElems);
            asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(k_src8 + (int64_t)t * kBN * kD), "s"(kdst) : "memory", "m0");
            asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(v_src8 + (int64_t)t * kBN), "s"(vdst) : "memory", "m0");
            return;
        }
        // Issued through inline assembly on purpose: for the builtin the compiler guards every later
        // LDS read and every barrier with vmcnt(0), which would cancel the prefetch distance.  The
        // waits that order these loads are the explicit ones at the top of the tile loop.
        if ((t + 1) * kBN <= ld_plain_end) {
            // A whole tile of the cache: scalar base + one precomputed 32-bit lane offset, no vector arithmetic at all
            // (the tile loop is bound by vector issue).
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
        // The last tile of the cache (rows past the end are clamped: they are masked anyway) and, with a fused append,
        // the tiles that hold new rows (read from k_new / v_new): one address per lane.
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            const int kr = min(t * kBN + 32 * pass + ld_row, p.Sk - 1);
            const int64_t off = (int64_t)kr * kD + ld_chunk * 8;
            const bool from_new = kr >= p.Snew0;  // never true without a fused append (Snew0 = INT_MAX then)
            const unsigned kdst = lds_k0 + (unsigned)(slot * kTileElems * 2 + pass * 4096);
            const unsigned vdst = lds_v0 + (unsigned)(slot * kTileElems * 2 + pass * 4096);
            asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"((from_new ? kn : kg) + off), "s"(kdst) : "memory", "m0");
            asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"((from_new ? vn : vg) + off), "s"(vdst) : "memory", "m0");
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
    // 8-bit cache, byte offsets.  K: lane (n, h) reads chunk 2*kp + h of key row 32*kb + n (the swizzle of a row
    // does not depend on kb): 16 features = two contraction steps.  V: lane (n, h) reads, of feature row
    // 32*dt + n, the keys 4h..4h+3 and 8+4h..8+4h+3 of the 16-key chunk 2*kb + g: the rows of P it multiplies.
    // The cache stores them as 8 consecutive bytes at byte 8 * (h ^ s) of the chunk, s = bit 4 of the feature
    // (the 32 lanes of one h would otherwise read half of the banks twice).
    const int f8 = chunk_swizzle8(n);
    int k_off8[2], v_off8[4];
#pragma unroll
    for (int kp = 0; kp < 2; ++kp) k_off8[kp] = n * kD + 16 * ((2 * kp + h) ^ f8);
#pragma unroll
    for (int ch = 0; ch < 4; ++ch) v_off8[ch] = n * kBN + 16 * (ch ^ f8) + 8 * (h ^ ((n >> 4) & 1));
    // Widened tiles (WIDE): V^T rows of 64 bf16 whose 16-byte chunk 2*ch + h holds the 8 keys lane half h needs of
    // the 16-key chunk ch; read like K, with K's offsets (k_off[ch]).  A lane widens the 16 codes of chunk cv_c of tile row cv_row of both
    // tensors.  Eight consecutive lanes take the eight even (or odd) rows of the wavefront's 16: the 16-byte
    // stores of such a group then fall on eight different chunk positions of the 128-byte rows (stores are
    // served eight lanes at a time), and the 16-byte loads stay conflict-free (measured: 0 conflict cycles
    // for both; 16 consecutive rows per 16 lanes cost a two-way conflict on either side).
    const int cv_row = 16 * wave + 2 * (lane & 7) + ((lane >> 3) & 1), cv_c = lane >> 4;
    const int cv_src = cv_row * 64 + 16 * (cv_c ^ chunk_swizzle8(cv_row));
    const int cv_f = chunk_swizzle(cv_row), cv_s = (cv_row >> 4) & 1;
    // destinations (elements): the two halves of a chunk go to chunk positions that differ in their lowest bit
    const int cv_k0 = cv_row * kD + 8 * ((2 * cv_c) ^ cv_f);
    const int cv_v0 = cv_row * kD + 8 * ((2 * cv_c + cv_s) ^ cv_f);
    auto widen_tile = [&](int t, int fslot, int buf) {
        if constexpr (WIDE) {
            const u32x4 rk = *(const u32x4*)(sm.k[fslot] + cv_src);
            u32x4 rv = *(const u32x4*)(sm.v[fslot] + cv_src);
            const int j0 = t * kBN;
            if (j0 + kBN > p.Sk) {  // last tile of the cache: V codes at or past the end count as zero
#pragma unroll
                for (int x = 0; x < 2; ++x) {  // bytes 8x..8x+7: keys 4hh..4hh+3 and 8+4hh.. of the chunk, hh = x ^ s
                    const int left = p.Sk - (j0 + 16 * cv_c + 4 * (x ^ cv_s));
                    rv[2 * x] = left >= 4 ? rv[2 * x] : left <= 0 ? 0u : rv[2 * x] & ((1u << (8 * left)) - 1u);
                    rv[2 * x + 1] = left >= 12 ? rv[2 * x + 1] : left <= 8 ? 0u : rv[2 * x + 1] & ((1u << (8 * (left - 8))) - 1u);
                }
            }
            *(bf16x8*)(sm.kb[buf] + cv_k0) = widen_e4m3x8(rk[0], rk[1]);
            *(bf16x8*)(sm.kb[buf] + (cv_k0 ^ 8)) = widen_e4m3x8(rk[2], rk[3]);
            *(bf16x8*)(sm.vb[buf] + cv_v0) = widen_e4m3x8(rv[0], rv[1]);
            *(bf16x8*)(sm.vb[buf] + (cv_v0 ^ 8)) = widen_e4m3x8(rv[2], rv[3]);
        }
    };

    if (t_begin < t_end) load_tile(t_begin, 0);
    if (t_begin + 1 < t_end) load_tile(t_begin + 1, 1);
    if constexpr (WIDE)
        if (t_begin + 2 < t_end) load_tile(t_begin + 2, 2);
    // The Q fragments are complete from here on and the compiler knows it: no later guard on them
    // can drain the tile prefetch.  (This also lands tiles 0 and 1, once per workgroup.)
    wait_vmem_all();
    if constexpr (!KV8) {
        if (fused) {
#pragma unroll
            for (int i = 0; i < kMaxCopy; ++i)
                if (cp_dst[i] >= 0) {
                    ((u32x4*)p.k)[cp_dst[i]] = cp_k[i];
                    ((u32x4*)p.v)[cp_dst[i]] = cp_v[i];
                }
        }
    }

    // base-2 exponent of one score against a reference already in exponent units
    auto to_exponent = [&](float s, float ref_exponent) {
        if constexpr (EXACTQ) return __builtin_fmaf(s, c, -ref_exponent);
        else return s - ref_exponent;
    };
    // QA = first block of the wavefront that still has visible keys in this tile (1: its earlier block is done)
    auto tile_body = [&](int t, int slot, auto qa_tag) {
        constexpr int QA = decltype(qa_tag)::value;
        const int j0 = t * kBN;
        {
            const auto* ks_ = [&]() { if constexpr (WIDE) return sm.kb[slot]; else return sm.k[slot]; }();
            const auto* vs_ = [&]() { if constexpr (WIDE) return sm.vb[slot]; else return sm.v[slot]; }();
            // ---- S^T = K . Q^T: all eight K fragments are requested before the first product ------
            f32x16 s_acc[2][QT];  // [kb][qt]
            bf16x8 kf[2][4];
            if constexpr (KV8 && !WIDE) {
                u32x4 raw[2][2];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int kp = 0; kp < 2; ++kp) raw[kb][kp] = *(const u32x4*)(ks_ + 32 * kb * kD + k_off8[kp]);
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int kp = 0; kp < 2; ++kp) {
                        kf[kb][2 * kp] = widen_e4m3x8(raw[kb][kp][0], raw[kb][kp][1]);
                        kf[kb][2 * kp + 1] = widen_e4m3x8(raw[kb][kp][2], raw[kb][kp][3]);
                    }
            } else {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks) kf[kb][ks] = lds_read_b128(ks_ + 32 * kb * kD + k_off[ks]);
            }
            __builtin_amdgcn_sched_barrier(0);
            // Raised priority from here to the end of the K.Q^T run, and again from the P.V run to
            // this point of the next tile: when the two wavefronts of a SIMD are in different
            // stages, the one feeding the matrix pipe (one issue slot per 32-cycle instruction) is
            // never kept waiting by the other one's stream of vector instructions.
            // Key-split launches (all workgroups resident at once, equal chains): a workgroup in the first half of its
            // chain runs one level higher.  Of the workgroups that share a CU the instruction arbiter otherwise serves the
            // oldest first, which then finishes far ahead and leaves the youngest to run alone at the end.
            const bool early = p.n_splits > 1 && (t - t_begin) * 2 < t_end - t_begin;
            if (early) __builtin_amdgcn_s_setprio(PRIO + 1);
            else __builtin_amdgcn_s_setprio(PRIO);
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int qt = QA; qt < QT; ++qt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) s_acc[kb][qt][r] = 0.f;
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                    for (int qt = QA; qt < QT; ++qt)
                        s_acc[kb][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kb][ks], qf[qt][ks], s_acc[kb][qt], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (early) __builtin_amdgcn_s_setprio(1);
            else __builtin_amdgcn_s_setprio(0);
            bf16x8 vf[2][2][2];  // [kb][g][dt]
            auto read_v_frags = [&]() {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int g = 0; g < 2; ++g)
#pragma unroll
                        for (int dt = 0; dt < 2; ++dt) {
                            if constexpr (WIDE) {
                                vf[kb][g][dt] = lds_read_b128(vs_ + 32 * dt * kD + k_off[2 * kb + g]);
                                continue;
                            } else if constexpr (KV8) {
                                const u32x2 w01 = *(const u32x2*)(vs_ + 32 * dt * kBN + v_off8[2 * kb + g]);
                                uint32_t w0 = w01[0], w1 = w01[1];
                                if (j0 + kBN > p.Sk) {  // last tile of the cache: codes past the end count as zero
                                    const int left = p.Sk - (j0 + 32 * kb + 16 * g + 4 * h);  // keys left from w0's first
                                    w0 = left >= 4 ? w0 : left <= 0 ? 0u : w0 & ((1u << (8 * left)) - 1u);
                                    w1 = left >= 12 ? w1 : left <= 8 ? 0u : w1 & ((1u << (8 * (left - 8))) - 1u);
                                }
                                vf[kb][g][dt] = widen_e4m3x8(w0, w1);
                                continue;
                            }
                            const __bf16* vp = (const __bf16*)vs_ + (32 * kb + 16 * g) * kD;
                            const s16x4 lo = lds_read_tr(vp + v_off[dt][0]);
                            const s16x4 hi = lds_read_tr(vp + v_off[dt][1]);
                            typedef __attribute__((ext_vector_type(8))) short s16x8;
                            const s16x8 av = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                            vf[kb][g][dt] = __builtin_bit_cast(bf16x8, av);
                        }
            };
            // ---- mask (only tiles that cross some row's bound) ---------------------------------
            if (j0 + kBN > kmin_blk[QA]) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int qt = QA; qt < QT; ++qt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int key = j0 + 32 * kb + 8 * (r >> 2) + 4 * h + (r & 3);
                            if (key >= kmax_lane[qt]) s_acc[kb][qt][r] = -INFINITY;
                        }
            }
            // ---- optimistic softmax, lane-local per query column -------------------------------
            bf16x8 pf[2][2][QT];  // [kb][g][qt]
            float l_tile[QT];
            auto form_p = [&]() {  // P = exp2(s - m_used) in bf16; row sums by plain fp32 adds (the
                                   // packed dot instruction shares the matrix pipe and would stall MFMAs)
#pragma unroll
                for (int qt = QA; qt < QT; ++qt) {
                    const float mc = EXACTQ ? m_used[qt] * c : m_used[qt];
                    float l = 0.f, l2 = 0.f;
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                        for (int g = 0; g < 2; ++g)
#pragma unroll
                            for (int jj = 0; jj < 4; ++jj) {
                                const float p0 = __builtin_amdgcn_exp2f(to_exponent(s_acc[kb][qt][8 * g + 2 * jj], mc));
                                const float p1 = __builtin_amdgcn_exp2f(to_exponent(s_acc[kb][qt][8 * g + 2 * jj + 1], mc));
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
            bool bad = true;  // a workgroup's first tile has no reference yet: straight to the exact pass
            if (t != t_begin) {
                form_p();
                // Pin the packed P before the test: otherwise the compiler, seeing P rebuilt on the rare
                // path, postpones the conversions until after the branch and keeps 64 exponentials alive.
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int b = 0; b < 2; ++b)
#pragma unroll
                        for (int e = QA; e < QT; ++e) asm volatile("" : "+v"(pf[a][b][e]));
                bad = false;
#pragma unroll
                for (int qt = QA; qt < QT; ++qt) bad |= !(l_tile[qt] < kOptimisticLimit);
            }
            // V^T fragments are requested once P is formed (earlier they would not fit the register
            // file next to the scores kept for the rare exact pass); the latency passes behind the
            // overflow test and the other wavefront of the SIMD.
            read_v_frags();
            if (__builtin_amdgcn_ballot_w64(bad) != 0) {  // exact path: this tile's max, rescale, redo
#pragma unroll
                for (int qt = QA; qt < QT; ++qt) {
                    float a = fmaxf(s_acc[0][qt][0], s_acc[1][qt][0]);
#pragma unroll
                    for (int r = 1; r < 16; ++r) a = fmaxf(fmaxf(a, s_acc[0][qt][r]), s_acc[1][qt][r]);
                    a = fmaxf(a, __shfl_xor(a, 32));
                    const float m_new = fmaxf(a, m_used[qt]);
                    const float alpha = __builtin_amdgcn_exp2f(EXACTQ ? (m_used[qt] - m_new) * c : m_used[qt] - m_new);
                    m_used[qt] = m_new;
                    l_sum[qt] *= alpha;
#pragma unroll
                    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) o_acc[dt][qt][r] *= alpha;
                }
                form_p();
            }
#pragma unroll
            for (int qt = QA; qt < QT; ++qt) l_sum[qt] += l_tile[qt];
            // ---- O^T += V^T . P^T -----------------------------------------------------------------
            __builtin_amdgcn_sched_barrier(0);
            if (early) __builtin_amdgcn_s_setprio(PRIO + 1);
            else __builtin_amdgcn_s_setprio(PRIO);
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int g = 0; g < 2; ++g)
#pragma unroll
                    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                        for (int qt = QA; qt < QT; ++qt)
                            o_acc[dt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[kb][g][dt], pf[kb][g][qt], o_acc[dt][qt], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // The tile loop runs twice in sequence for QT = 2: tiles in which both blocks of the wavefront have visible
    // keys, then the tiles only its later block still sees (two loops rather than a branch inside one: each keeps
    // its own, smaller, set of live registers).  Every wavefront passes the same number of barriers.
    int slot = 0;         // ring slot of tile t (of tile t+1 with widened tiles)
    int buf = 0;          // widened tiles: buffer of tile t
    auto run_tiles = [&](int t_from, int t_to, auto qa_tag) {
        constexpr int QA = decltype(qa_tag)::value;
        for (int t = t_from; t < t_to; ++t) {
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (WIDE) {
                // Code tiles t+1 and t+2 are in the ring (t+3 on its way into the slot tile t left), tile t sits
                // widened in buffer `buf`.  Per tile: one barrier; then every wavefront requests tile t+3, widens
                // its share of tile t+1 into the other buffer and runs the products of tile t.  The barrier at the
                // top of the next round makes the widened tile visible and frees the buffer and the code slot read.
                if (t + 2 < t_end) asm volatile("s_waitcnt vmcnt(2) lgkmcnt(0)" ::: "memory");  // tile t+1 landed, own LDS traffic done
                else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
                if (t + 3 < t_end) load_tile(t + 3, slot == 0 ? 2 : slot - 1);  // (slot + 2) % 3: the slot of tile t
                if (t + 1 < t_end) widen_tile(t + 1, slot, buf ^ 1);
                if (QA == 0 || (wave_active && t * kBN < kmax_wave)) tile_body(t, buf, qa_tag);
                buf ^= 1;
            } else {
                // Tile t has landed for this wavefront once at most tile t+1's loads are in flight (four; two with
                // the 8-bit cache); after the barrier it has landed for all, and every wavefront is done with tile
                // t-1, whose slot the load of tile t+2 reuses.
                if (t + 1 < t_end) {
                    if constexpr (KV8) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
                    else asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
                } else {
                    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                }
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
                if (t + 2 < t_end) load_tile(t + 2, slot == 0 ? 2 : slot - 1);  // (slot + 2) % 3
                if (QA == 0 || (wave_active && t * kBN < kmax_wave)) tile_body(t, slot, qa_tag);
            }
            slot = slot == 2 ? 0 : slot + 1;
        }
    };
    if constexpr (WIDE) {
        __builtin_amdgcn_s_barrier();  // tile t_begin landed for all (the wait above covered this wavefront's loads)
        if (t_begin < t_end) widen_tile(t_begin, 0, 0);
        slot = 1;
    }
    if constexpr (QT == 2) {
        // tiles below the earlier block's bound (none for a wavefront past the end of a ragged last query tile)
        const int t_mid = wave_active ? max(t_begin, min(t_end, (kmax_blk[0] + kBN - 1) / kBN)) : t_begin;
        run_tiles(t_begin, t_mid, std::integral_constant<int, 0>{});
        run_tiles(t_mid, t_end, std::integral_constant<int, 1>{});
    } else {
        const int t_mid = wave_active ? max(t_begin, min(t_end, (kmax_wave + kBN - 1) / kBN)) : t_begin;
        run_tiles(t_begin, t_mid, std::integral_constant<int, 0>{});
        for (int t = t_mid; t < t_end; ++t) {  // tiles this wavefront sees nothing of: keep the ring turning
            if (t + 1 < t_end) {
                if constexpr (KV8) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
                else asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
            } else {
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            }
            __builtin_amdgcn_s_barrier();
            if (t + 2 < t_end) load_tile(t + 2, slot == 0 ? 2 : slot - 1);
            slot = slot == 2 ? 0 : slot + 1;
        }
    }

    if (!wave_active) return;
    if constexpr (KV8) {  // values of V = codes * scale: linear, so applied once to the accumulator
        const float vs = p.v_scale[wi.bh];
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int qt = 0; qt < QT; ++qt)
#pragma unroll
                for (int r = 0; r < 16; ++r) o_acc[dt][qt][r] *= vs;
    }
    if constexpr (EXACTQ)
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) m_used[qt] *= c;
    store_rows<QT>(p, wi, row, h, o_acc, l_sum, m_used);
}

template <int QT, bool KV8 = false, bool EXACTQ = false>
__global__ void __launch_bounds__(kWaves * 64, QT == 2 ? 2 : 3)
attn_fwd_bf16_d64(FwdParams p) {
    __shared__ typename SmemOf<QT, KV8>::type sm;
    const WorkItem wi = decode_work(p);
    if (!wi.valid) return;  // whole workgroup leaves together
    attn_fwd_item<QT, KV8, EXACTQ>(p, wi, sm);
}

// Merge the key-split partials of one query row: out = sum_s w_s O_s / sum_s w_s l_s with
// w_s = 2^(m_s - max_s m_s).  One thread per (row, 4 output columns).  The partials of up to eight
// splits are requested together, so a merge costs one memory round trip per eight splits rather
// than one per split; chunks are folded with the usual running-max rescale.
__global__ void __launch_bounds__(256)
attn_combine_d64(FwdParams p) {
    constexpr int U = 8;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t total = (int64_t)p.BH * p.Sq * (kD / 4);
    if (idx >= total) return;
    const int dq = (int)(idx % (kD / 4));
    const int64_t r = idx / (kD / 4);
    const int bh = (int)(r / p.Sq), i = (int)(r % p.Sq);
    const int64_t prow0 = (int64_t)bh * p.n_splits * p.Sq + i;  // split s: + s * Sq
    float m_run = kNegBig, l = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < p.n_splits; s0 += U) {
        f32x2 ml[U];
        bf16x4 o[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t prow = prow0 + (int64_t)min(s0 + u, p.n_splits - 1) * p.Sq;  // clamped: dropped below
            ml[u] = *(const f32x2*)(p.part_ml + prow * 2);
            o[u] = *(const bf16x4*)(p.part_o + prow * kD + 4 * dq);
        }
        float m_new = m_run;
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (s0 + u < p.n_splits) m_new = fmaxf(m_new, ml[u][0]);
        const float a = __builtin_amdgcn_exp2f(m_run - m_new);
        l *= a;
        acc *= a;
        m_run = m_new;
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (s0 + u < p.n_splits) {
                const float w = __builtin_amdgcn_exp2f(ml[u][0] - m_new);
                l += w * ml[u][1];
                acc += w * __builtin_convertvector(o[u], f32x4);
            }
    }
    const float inv = 1.0f / l;
    const f32x4 x = acc * inv;
    const bf16x4 y = __builtin_convertvector(x, bf16x4);
    *(bf16x4*)((__bf16*)p.out + r * kD + 4 * dq) = y;
    if (p.lse && dq == 0) p.lse[r] = (m_run + __builtin_log2f(l)) * kLn2;
}

}  // namespace mfma
}  // namespace nfd

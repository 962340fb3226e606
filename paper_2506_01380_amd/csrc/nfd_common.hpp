// Shared device-side vocabulary of the gfx950 attention kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nfd {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr float kLog2e = 1.4426950408889634f;
// Running maxima start at a large finite negative so that (m_old - m_new) is never inf - inf.
constexpr float kLn2 = 0.69314718055994531f;
constexpr float kNegBig = -1.0e30f;

// Launch geometry and tensor description shared by every forward kernel.
// Mask (Sec. 3.1, block-wise causal attention): query row i sees keys
// j < kmax(i) = (P + i / T + 1) * T, i.e. all frames up to and including its own.
struct FwdParams {
    const void* q;      // [BH, Sq, D]
    const void* k;      // [BH, Scap, D]
    const void* v;      // [BH, Scap, D]
    void* out;          // [BH, Sq, D]
    __bf16* part_o;     // [BH, n_splits, Sq, D] un-normalised partial outputs (split launches), rounded to bf16:
                        // one more rounding of the kind the output gets anyway, for half the combine's traffic
    float* part_ml;     // [BH, n_splits, Sq, 2]  (running max in log2 units, running sum)
    float* lse;         // [BH, Sq] optional: natural log of the row's softmax denominator (for the backward)
    int BH;             // B * H
    int Sq;             // q_frames * T
    int Sk;             // kv_frames * T
    int Scap;           // F * T (head stride of k, v in rows)
    int T;              // tokens per frame
    int P;              // kv_frames - q_frames
    int D;
    int n_q_tiles;      // query tiles per head
    int blocks_lo;      // 32-row blocks per query tile; the first n_hi tiles own one more
    int n_hi;
    int n_splits;       // key splits per query tile
    int group_q_tiles;  // split launches: 1 = query tiles of one (head, split) get adjacent workgroup ids
    float scale_log2e;  // softmax scale * log2(e)
    // 8-bit cache only (k: [BH, Spad, D] E4M3 codes, v: [BH, D, Spad] codes, value = code * scale[bh]):
    const float* k_scale;  // [BH]
    const float* v_scale;  // [BH]
    int Spad;              // F * T rounded up to a multiple of 64: row count of k, row length of v
    // fused cache append (bf16 matrix-core kernels only; null otherwise): the K/V of the query frames themselves,
    // [BH, Sq, D].  Key rows >= Snew0 = P * T are read from here instead of the cache, and every workgroup copies its
    // share of these rows into k, v on the side, so the cache ends up as after an append.
    const void* k_new;
    const void* v_new;
    int Snew0;
};

__device__ __forceinline__ int kmax_of_row(int row, int T, int P) { return (P + row / T + 1) * T; }

}  // namespace nfd

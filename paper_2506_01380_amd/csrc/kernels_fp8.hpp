// Writing new frames into the 8-bit KV cache (the cache of Appendix B held as E4M3 codes; post-training
// quantisation is the acceleration Sec. 6 leaves for later).  One scale per (batch, head) and tensor:
// code = E4M3(x / scale), round to nearest even, saturating at +-448; x / scale is x * (1 / scale) in fp32,
// both correctly rounded.  K codes are stored key-major [BH, Spad, 64]; V codes feature-major
// [BH, 64, Spad], the orientation the second product of the attention kernel consumes, keys permuted inside
// groups of 16 (v8t_position).
#pragma once
#include "nfd_common.hpp"

namespace nfd {

constexpr float kE4m3Max = 448.0f;

// Where key j of a feature row sits inside that row of the V cache.  Keys are permuted inside every aligned
// group of 16 so that one lane of the attention kernel finds the 8 keys its matrix operand needs (keys
// 4h..4h+3 and 8+4h..8+4h+3 of the group, h = lane / 32) in 8 consecutive bytes, at byte 8 * (h ^ s) of the
// group; s = bit 4 of the feature index, so that the 32 lanes of one h read all LDS banks, not half of them.
__host__ __device__ __forceinline__ int64_t v8t_position(int64_t j, int s) {
    const int q = (int)(j & 15);
    return (j & ~(int64_t)15) | (8 * (((q >> 2) & 1) ^ s) + 4 * (q >> 3) + (q & 3));
}

// Two fp32 values -> two codes in the low (hi = false) or high half of `old`.
template <bool HI>
__device__ __forceinline__ uint32_t e4m3_pack2(float a, float b, uint32_t old) {
    a = __builtin_amdgcn_fmed3f(a, -kE4m3Max, kE4m3Max);
    b = __builtin_amdgcn_fmed3f(b, -kE4m3Max, kE4m3Max);
    return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(a, b, (int)old, HI);
}

// One launch for both tensors.  blockIdx.y = head (strided); the first k_blocks workgroups along x take K,
// the others V.
// K: one thread quantises 8 consecutive features of one new key row.
// V: a workgroup takes 64 new key rows; wavefront w the features 16w .. 16w+15.  A lane reads its row's 16
// features (32 contiguous bytes) and stores 16 single codes; across the lanes of a wavefront each store
// instruction covers 64 consecutive bytes of one feature row of the cache.
__global__ void __launch_bounds__(256)
kvcache_append_fp8(const __bf16* __restrict__ kn, const __bf16* __restrict__ vn, unsigned char* __restrict__ k8,
                   unsigned char* __restrict__ v8t, const float* __restrict__ k_scale, const float* __restrict__ v_scale,
                   int n_rows, int64_t Spad, int j0, int BH, unsigned k_blocks) {
    if (blockIdx.x < k_blocks) {
        const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
        if (idx >= (int64_t)n_rows * 8) return;
        const int r = (int)(idx >> 3), c8 = (int)(idx & 7);
        for (int bh = blockIdx.y; bh < BH; bh += gridDim.y) {
            const float inv = __frcp_rn(k_scale[bh]);
            const bf16x8 x = *(const bf16x8*)(kn + ((int64_t)bh * n_rows + r) * 64 + 8 * c8);
            uint32_t w0 = e4m3_pack2<false>((float)x[0] * inv, (float)x[1] * inv, 0u);
            w0 = e4m3_pack2<true>((float)x[2] * inv, (float)x[3] * inv, w0);
            uint32_t w1 = e4m3_pack2<false>((float)x[4] * inv, (float)x[5] * inv, 0u);
            w1 = e4m3_pack2<true>((float)x[6] * inv, (float)x[7] * inv, w1);
            const u32x2 w = {w0, w1};
            *(u32x2*)(k8 + ((int64_t)bh * Spad + j0 + r) * 64 + 8 * c8) = w;
        }
        return;
    }
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int r = (int)(blockIdx.x - k_blocks) * 64 + lane;
    if (r >= n_rows) return;
    for (int bh = blockIdx.y; bh < BH; bh += gridDim.y) {
        const float inv = __frcp_rn(v_scale[bh]);
        const __bf16* src = vn + ((int64_t)bh * n_rows + r) * 64 + 16 * w;
        const bf16x8 x0 = *(const bf16x8*)src, x1 = *(const bf16x8*)(src + 8);
        unsigned char* dst = v8t + ((int64_t)bh * 64 + 16 * w) * Spad + v8t_position(j0 + r, w & 1);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            dst[(int64_t)e * Spad] = (unsigned char)(e4m3_pack2<false>((float)x0[e] * inv, 0.f, 0u) & 0xffu);
            dst[(int64_t)(e + 8) * Spad] = (unsigned char)(e4m3_pack2<false>((float)x1[e] * inv, 0.f, 0u) & 0xffu);
        }
    }
}

// Move n_keys keys of every feature row between two row-major byte tensors, either of which may be in the
// V cache's permuted key order (perm_*; feature of a row = (row_base + row) % 64) or in plain order (staging).
// blockIdx.y = row (strided), x over keys.
__global__ void __launch_bounds__(256)
v8t_move_keys(unsigned char* __restrict__ dst, const unsigned char* __restrict__ src, int64_t rows, int64_t dst_stride,
              int64_t src_stride, int64_t dst_key0, int64_t src_key0, int64_t n_keys, int perm_dst, int perm_src,
              int64_t row_base) {
    for (int64_t row = blockIdx.y; row < rows; row += gridDim.y) {
        const int s = (int)(((row_base + row) >> 4) & 1);
        for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_keys; i += (int64_t)gridDim.x * blockDim.x) {
            const int64_t sp = perm_src ? v8t_position(src_key0 + i, s) : src_key0 + i;
            const int64_t dp = perm_dst ? v8t_position(dst_key0 + i, s) : dst_key0 + i;
            dst[row * dst_stride + dp] = src[row * src_stride + sp];
        }
    }
}

}  // namespace nfd

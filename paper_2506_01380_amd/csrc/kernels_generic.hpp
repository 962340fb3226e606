// General forward kernel: any T, any D <= 256, fp32 or bf16 storage, fp32 arithmetic.
// One wavefront owns one query row and walks the visible keys 64 at a time with an
// online softmax.  It is the fp32 path of the library and the fallback for head
// widths the matrix-core kernel is not built for; it is not tuned.
#pragma once
#include "kernels_fp8.hpp"
#include "nfd_common.hpp"

namespace nfd {

template <typename T> __device__ __forceinline__ float to_f32(T x);
template <> __device__ __forceinline__ float to_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ float to_f32<__bf16>(__bf16 x) { return (float)x; }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ __bf16 from_f32<__bf16>(float x) { return (__bf16)x; }  // RNE

__device__ __forceinline__ float wave_max(float x) {
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}
__device__ __forceinline__ float wave_sum(float x) {
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

constexpr int kGenericWaves = 4;
constexpr int kGenericMaxD = 256;

template <typename T>
__global__ void __launch_bounds__(kGenericWaves * 64)
attn_fwd_generic(FwdParams p) {
    __shared__ float q_s[kGenericWaves][kGenericMaxD];
    __shared__ float p_s[kGenericWaves][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t row_id = (int64_t)blockIdx.x * kGenericWaves + w;  // over BH * Sq
    if (row_id >= (int64_t)p.BH * p.Sq) return;                      // whole wave exits together
    const int bh = (int)(row_id / p.Sq), i = (int)(row_id % p.Sq);
    const int D = p.D;
    const T* q = (const T*)p.q + ((int64_t)bh * p.Sq + i) * D;
    const T* k = (const T*)p.k + (int64_t)bh * p.Scap * D;
    const T* v = (const T*)p.v + (int64_t)bh * p.Scap * D;
    T* out = (T*)p.out + ((int64_t)bh * p.Sq + i) * D;

    for (int d = lane; d < D; d += 64) q_s[w][d] = to_f32<T>(q[d]);
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): q_s visible within the wave

    const int kmax = kmax_of_row(i, p.T, p.P);  // <= Sk by construction
    float m = kNegBig, l = 0.f;
    float acc[kGenericMaxD / 64] = {0.f, 0.f, 0.f, 0.f};

    for (int j0 = 0; j0 < kmax; j0 += 64) {
        const int j = j0 + lane;
        float s = -INFINITY;
        if (j < kmax) {
            const T* kr = k + (int64_t)j * D;
            float a = 0.f;
            for (int d = 0; d < D; ++d) a = fmaf(q_s[w][d], to_f32<T>(kr[d]), a);
            s = a * p.scale_log2e;  // log2 units
        }
        const float m_new = fmaxf(m, wave_max(s));
        const float alpha = exp2f(m - m_new);
        const float pj = exp2f(s - m_new);  // 0 for masked lanes
        l = l * alpha + wave_sum(pj);
        m = m_new;
        p_s[w][lane] = pj;
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_s_waitcnt(0xc07f);
        const int nj = min(64, kmax - j0);
#pragma unroll
        for (int c = 0; c < kGenericMaxD / 64; ++c) {
            const int d = lane + 64 * c;
            if (d < D) {
                float a = acc[c] * alpha;
                for (int jj = 0; jj < nj; ++jj) a = fmaf(p_s[w][jj], to_f32<T>(v[(int64_t)(j0 + jj) * D + d]), a);
                acc[c] = a;
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
    const float inv = 1.0f / l;
#pragma unroll
    for (int c = 0; c < kGenericMaxD / 64; ++c) {
        const int d = lane + 64 * c;
        if (d < D) out[d] = from_f32<T>(acc[c] * inv);
    }
    if (p.lse && lane == 0) p.lse[row_id] = (m + log2f(l)) * kLn2;
}

// General backward: the same one-wavefront-per-row scheme, fp32 arithmetic, any T, D <= 256.  Two kernels,
// neither with atomics.  With p_ij = exp(scale <q_i, k_j> - lse_i) over the visible keys of row i and
// delta_i = <dout_i, out_i>:  ds_ij = p_ij (<dout_i, v_j> - delta_i),  dq_i = scale sum_j ds_ij k_j,
// dk_j = scale sum_i ds_ij q_i,  dv_j = sum_i p_ij dout_i.
struct BwdGenericParams {
    const void *q, *k, *v, *out, *dout;
    const float* lse;
    float* delta;  // [BH, Sq], written by the dq kernel, read by the dk/dv kernel
    void *dq, *dk, *dv;
    int BH, Sq, Sk, Scap, T, P, D;
    float scale, scale_log2e;
};

// One wavefront per query row: delta_i, then dq_i over the visible keys, 64 at a time.
template <typename T>
__global__ void __launch_bounds__(kGenericWaves * 64)
attn_bwd_dq_generic(BwdGenericParams p) {
    __shared__ float q_s[kGenericWaves][kGenericMaxD];
    __shared__ float g_s[kGenericWaves][kGenericMaxD];
    __shared__ float ds_s[kGenericWaves][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t row_id = (int64_t)blockIdx.x * kGenericWaves + w;  // over BH * Sq
    if (row_id >= (int64_t)p.BH * p.Sq) return;
    const int bh = (int)(row_id / p.Sq), i = (int)(row_id % p.Sq);
    const int D = p.D;
    const T* q = (const T*)p.q + row_id * D;
    const T* o = (const T*)p.out + row_id * D;
    const T* g = (const T*)p.dout + row_id * D;
    const T* k = (const T*)p.k + (int64_t)bh * p.Scap * D;
    const T* v = (const T*)p.v + (int64_t)bh * p.Scap * D;

    float dsum = 0.f;
    for (int d = lane; d < D; d += 64) {
        const float gd = to_f32<T>(g[d]);
        q_s[w][d] = to_f32<T>(q[d]);
        g_s[w][d] = gd;
        dsum = fmaf(gd, to_f32<T>(o[d]), dsum);
    }
    const float delta = wave_sum(dsum);
    if (lane == 0) p.delta[row_id] = delta;
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_s_waitcnt(0xc07f);

    const float lse2 = p.lse[row_id] * kLog2e;
    const int kmax = kmax_of_row(i, p.T, p.P);
    float acc[kGenericMaxD / 64] = {0.f, 0.f, 0.f, 0.f};
    for (int j0 = 0; j0 < kmax; j0 += 64) {
        const int j = j0 + lane;
        float ds = 0.f;
        if (j < kmax) {
            const T* kr = k + (int64_t)j * D;
            const T* vr = v + (int64_t)j * D;
            float a = 0.f, b = 0.f;
            for (int d = 0; d < D; ++d) {
                a = fmaf(q_s[w][d], to_f32<T>(kr[d]), a);
                b = fmaf(g_s[w][d], to_f32<T>(vr[d]), b);
            }
            ds = exp2f(a * p.scale_log2e - lse2) * (b - delta);
        }
        ds_s[w][lane] = ds;
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_s_waitcnt(0xc07f);
        const int nj = min(64, kmax - j0);
#pragma unroll
        for (int c = 0; c < kGenericMaxD / 64; ++c) {
            const int d = lane + 64 * c;
            if (d < D) {
                float a = acc[c];
                for (int jj = 0; jj < nj; ++jj) a = fmaf(ds_s[w][jj], to_f32<T>(k[(int64_t)(j0 + jj) * D + d]), a);
                acc[c] = a;
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
    T* dq = (T*)p.dq + row_id * D;
#pragma unroll
    for (int c = 0; c < kGenericMaxD / 64; ++c) {
        const int d = lane + 64 * c;
        if (d < D) dq[d] = from_f32<T>(acc[c] * p.scale);
    }
}

// One wavefront per key row j < Sk: dk_j and dv_j over the query rows that see it, 64 at a time.  Those are
// the rows from (floor(j/T) - P) * T on (none below 0): every later frame sees the key as well.
template <typename T>
__global__ void __launch_bounds__(kGenericWaves * 64)
attn_bwd_dkdv_generic(BwdGenericParams p) {
    __shared__ float k_s[kGenericWaves][kGenericMaxD];
    __shared__ float v_s[kGenericWaves][kGenericMaxD];
    __shared__ float p_s[kGenericWaves][64];
    __shared__ float ds_s[kGenericWaves][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t key_id = (int64_t)blockIdx.x * kGenericWaves + w;  // over BH * Sk
    if (key_id >= (int64_t)p.BH * p.Sk) return;
    const int bh = (int)(key_id / p.Sk), j = (int)(key_id % p.Sk);
    const int D = p.D;
    const T* kr = (const T*)p.k + ((int64_t)bh * p.Scap + j) * D;
    const T* vr = (const T*)p.v + ((int64_t)bh * p.Scap + j) * D;
    const T* q = (const T*)p.q + (int64_t)bh * p.Sq * D;
    const T* g = (const T*)p.dout + (int64_t)bh * p.Sq * D;
    const float* lse = p.lse + (int64_t)bh * p.Sq;
    const float* delta = p.delta + (int64_t)bh * p.Sq;

    for (int d = lane; d < D; d += 64) {
        k_s[w][d] = to_f32<T>(kr[d]);
        v_s[w][d] = to_f32<T>(vr[d]);
    }
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_s_waitcnt(0xc07f);

    const int rmin = max(0, (j / p.T - p.P) * p.T);
    float acc_k[kGenericMaxD / 64] = {0.f, 0.f, 0.f, 0.f};
    float acc_v[kGenericMaxD / 64] = {0.f, 0.f, 0.f, 0.f};
    for (int i0 = rmin; i0 < p.Sq; i0 += 64) {
        const int i = i0 + lane;
        float pij = 0.f, ds = 0.f;
        if (i < p.Sq) {
            const T* qr = q + (int64_t)i * D;
            const T* gr = g + (int64_t)i * D;
            float a = 0.f, b = 0.f;
            for (int d = 0; d < D; ++d) {
                a = fmaf(to_f32<T>(qr[d]), k_s[w][d], a);
                b = fmaf(to_f32<T>(gr[d]), v_s[w][d], b);
            }
            pij = exp2f(a * p.scale_log2e - lse[i] * kLog2e);
            ds = pij * (b - delta[i]);
        }
        p_s[w][lane] = pij;
        ds_s[w][lane] = ds;
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_s_waitcnt(0xc07f);
        const int ni = min(64, p.Sq - i0);
#pragma unroll
        for (int c = 0; c < kGenericMaxD / 64; ++c) {
            const int d = lane + 64 * c;
            if (d < D) {
                float ak = acc_k[c], av = acc_v[c];
                for (int ii = 0; ii < ni; ++ii) {
                    ak = fmaf(ds_s[w][ii], to_f32<T>(q[(int64_t)(i0 + ii) * D + d]), ak);
                    av = fmaf(p_s[w][ii], to_f32<T>(g[(int64_t)(i0 + ii) * D + d]), av);
                }
                acc_k[c] = ak;
                acc_v[c] = av;
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
    T* dk = (T*)p.dk + ((int64_t)bh * p.Scap + j) * D;
    T* dv = (T*)p.dv + ((int64_t)bh * p.Scap + j) * D;
#pragma unroll
    for (int c = 0; c < kGenericMaxD / 64; ++c) {
        const int d = lane + 64 * c;
        if (d < D) {
            dk[d] = from_f32<T>(acc_k[c] * p.scale);
            dv[d] = from_f32<T>(acc_v[c]);
        }
    }
}

// Copy a run of whole frames of every head between two head-strided tensors: the cache write of new
// frames (Appendix B, KV caching) and the moves of the sliding context window.  K and V together.
// All counts in units of the element type E (a 16-byte vector when every size and address allows it,
// otherwise one tensor element): head_dst / head_src = head strides, off_dst / off_src = offsets
// inside a head, len = units per head.  blockIdx.y walks over the heads, blockIdx.x over the units of a
// head, so no thread divides.
// PAIR = false: one tensor only (kd, ks); vd and vs are not touched.
template <typename E, bool PAIR = true>
__global__ void __launch_bounds__(256)
kvcache_copy(E* __restrict__ kd, E* __restrict__ vd, const E* __restrict__ ks, const E* __restrict__ vs,
             int64_t head_dst, int64_t head_src, int64_t off_dst, int64_t off_src, int64_t len, int64_t heads) {
    for (int64_t bh = blockIdx.y; bh < heads; bh += gridDim.y) {
        const int64_t dbase = bh * head_dst + off_dst, sbase = bh * head_src + off_src;
        for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < len; r += (int64_t)gridDim.x * blockDim.x) {
            kd[dbase + r] = ks[sbase + r];
            if constexpr (PAIR) vd[dbase + r] = vs[sbase + r];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// 3D rotary position embedding of the queries and keys of the new frames, fused with the cache
// write (Sec. 3.1 "3D Positional Embedding": the head dimension is separated into [n_T, n_H, n_W],
// one rotary embedding per axis, concatenated; Appendix B for the cache).  The rotation of feature
// pair (2i, 2i+1) of an axis section of width n at position p is by the angle p * theta^(-2i/n),
// counter-clockwise.  Pure streaming work: q in -> q out, k -> cache, v -> cache.
//
// One thread owns VEC consecutive features of one (frame, token) and walks over a range of heads:
// the cosines and sines depend on the position only, so they are computed once (in fp64: angles
// reach hundreds of radians) and reused for every head.  Consecutive threads cover consecutive
// 16-byte chunks of consecutive tokens, i.e. contiguous memory inside each head.
constexpr int kRopeMaxPairs = 128;  // D <= 256
struct RopeTable {
    double inv_freq[kRopeMaxPairs];     // theta^(-2i/n) of every feature pair, in head-dimension order
    unsigned char axis[kRopeMaxPairs];  // 0 = frame index, 1 = grid row, 2 = grid column
};
struct RopeParams {
    int BH, F, T, D;
    int frame_pos, n_frames;
    int t_pos0;            // temporal position of the first new frame
    int grid_w;
    int heads_per_thread;  // blockIdx.y selects a range of heads
};

//
// KV8 (bf16, VEC = 8 only): the caches are the 8-bit ones (kernels_fp8.hpp): the rotated key, rounded to bf16
// exactly as for a bf16 cache, and the value are quantised with the head's scales; K codes go to 8 consecutive
// bytes of the key's row, V codes to 8 feature rows at the key's (permuted) position.
struct RopeFp8 {
    const float* k_scale;  // [BH]
    const float* v_scale;  // [BH]
    int64_t Spad;          // keys per cache row set (F * T rounded up to 64)
};

template <typename E, int VEC, bool KV8 = false>
__global__ void __launch_bounds__(256)
rope_kvcache_append(const E* q, E* q_out, E* __restrict__ kc, E* __restrict__ vc,
                    const E* __restrict__ kn, const E* __restrict__ vn, RopeParams rp, RopeTable tab, RopeFp8 f8 = RopeFp8{}) {
    typedef __attribute__((ext_vector_type(VEC))) E vec_t;
    const int chunks = rp.D / VEC;
    const int64_t items = (int64_t)rp.n_frames * rp.T * chunks;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= items) return;
    const int chunk = (int)(idx % chunks);
    const int64_t row = idx / chunks;  // (new frame, token)
    const int f = (int)(row / rp.T), tok = (int)(row % rp.T);
    const int pos[3] = {rp.t_pos0 + f, tok / rp.grid_w, tok % rp.grid_w};
    float cs[VEC / 2], sn[VEC / 2];
#pragma unroll
    for (int j = 0; j < VEC / 2; ++j) {
        const int p = chunk * (VEC / 2) + j;
        const double ang = (double)pos[tab.axis[p]] * tab.inv_freq[p];
        double s, c;
        sincos(ang, &s, &c);
        cs[j] = (float)c;
        sn[j] = (float)s;
    }
    const int bh0 = blockIdx.y * rp.heads_per_thread;
    const int bh1 = min(bh0 + rp.heads_per_thread, rp.BH);
    for (int bh = bh0; bh < bh1; ++bh) {
        const int64_t src = ((int64_t)bh * rp.n_frames * rp.T + row) * rp.D + chunk * VEC;
        const int64_t dst = (((int64_t)bh * rp.F + rp.frame_pos) * rp.T + row) * rp.D + chunk * VEC;
        const vec_t qv = *(const vec_t*)(q + src);
        const vec_t kv = *(const vec_t*)(kn + src);
        const vec_t vv = *(const vec_t*)(vn + src);
        vec_t qo, ko;
#pragma unroll
        for (int j = 0; j < VEC / 2; ++j) {
            const float qa = (float)qv[2 * j], qb = (float)qv[2 * j + 1];
            const float ka = (float)kv[2 * j], kb = (float)kv[2 * j + 1];
            qo[2 * j] = (E)(qa * cs[j] - qb * sn[j]);
            qo[2 * j + 1] = (E)(qa * sn[j] + qb * cs[j]);
            ko[2 * j] = (E)(ka * cs[j] - kb * sn[j]);
            ko[2 * j + 1] = (E)(ka * sn[j] + kb * cs[j]);
        }
        *(vec_t*)(q_out + src) = qo;
        if constexpr (KV8) {
            static_assert(!KV8 || VEC == 8, "the 8-bit cache takes eight features per thread");
            const float ik = __frcp_rn(f8.k_scale[bh]), iv = __frcp_rn(f8.v_scale[bh]);
            const int64_t j = (int64_t)rp.frame_pos * rp.T + row;  // key index in the cache
            uint32_t w0 = e4m3_pack2<false>((float)ko[0] * ik, (float)ko[1] * ik, 0u);
            w0 = e4m3_pack2<true>((float)ko[2] * ik, (float)ko[3] * ik, w0);
            uint32_t w1 = e4m3_pack2<false>((float)ko[4] * ik, (float)ko[5] * ik, 0u);
            w1 = e4m3_pack2<true>((float)ko[6] * ik, (float)ko[7] * ik, w1);
            const u32x2 w = {w0, w1};
            *(u32x2*)((unsigned char*)kc + ((int64_t)bh * f8.Spad + j) * 64 + chunk * 8) = w;
            unsigned char* vd = (unsigned char*)vc + ((int64_t)bh * 64 + chunk * 8) * f8.Spad + v8t_position(j, (chunk >> 1) & 1);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                vd[(int64_t)e * f8.Spad] = (unsigned char)(e4m3_pack2<false>((float)vv[e] * iv, 0.f, 0u) & 0xffu);
        } else {
            *(vec_t*)(kc + dst) = ko;
            *(vec_t*)(vc + dst) = vv;
        }
    }
}

}  // namespace nfd

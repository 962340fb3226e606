// Measurement aid, not part of the attention path: what one SIMD of this chip sustains for the
// forward kernel's instruction mix with no memory traffic at all.  One wavefront per SIMD runs, per
// iteration, the 32 bf16 32x32x16 MFMAs of a 64 x 64 x 64 tile pair and/or the softmax arithmetic
// of its 64 x 64 scores per wavefront (per lane: 64 fma, 64 exp2, 32 packed bf16 conversions, 64
// adds), either one after the other or interleaved 1 MFMA : 7 vector instructions.  The figures
// bound what any schedule of the real kernel can reach; they are quoted in the design notes.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstring>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

// MODE 0: MFMA only; 1: vector only; 2: both, one after the other; 3: both, interleaved 1 : 7
// At most 256 registers per lane, so that two workgroups fit a CU: launched with twice as many workgroups as
// CUs, every SIMD holds two wavefronts, as in the attention kernel.
template <int MODE>
__global__ void __launch_bounds__(256, 2)
issue_mix(float* out, const u32x4* in, int iters, float c, unsigned long long* cycles) {
    bf16x8 a[8], b[8];
    for (int j = 0; j < 8; ++j) {
        a[j] = __builtin_bit_cast(bf16x8, in[threadIdx.x + 64 * j]);
        b[j] = __builtin_bit_cast(bf16x8, in[threadIdx.x + 64 * j + 1024]);
    }
    f32x16 acc[4], s[4];
    for (int j = 0; j < 4; ++j)
        for (int r = 0; r < 16; ++r) {
            acc[j][r] = 0.f;
            s[j][r] = (float)(in[threadIdx.x + 64 * j + 512 * (r >> 2)][r & 3] & 1023) * 0.004f;
        }
    float l0 = 0.f, l1 = 0.f, mc = 0.5f;
    bf16x8 pf[8];
    for (int j = 0; j < 8; ++j) pf[j] = a[j];
    const unsigned long long t0 = __builtin_readcyclecounter();
    for (int it = 0; it < iters; ++it) {
        if (MODE != 1) {
#pragma unroll
            for (int j = 0; j < 8; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[(j + q) & 7], acc[q], 0, 0, 0);
        }
        if (MODE == 2) __builtin_amdgcn_sched_barrier(0);
        if (MODE != 0) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int g = 0; g < 2; ++g)
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) {
                        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[j][8 * g + 2 * jj], c, -mc));
                        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[j][8 * g + 2 * jj + 1], c, -mc));
                        const f32x2 pp = {p0, p1};
                        const bf16x2 pb = __builtin_convertvector(pp, bf16x2);
                        l0 += p0;
                        l1 += p1;
                        pf[2 * j + g][2 * jj] = pb[0];
                        pf[2 * j + g][2 * jj + 1] = pb[1];
                    }
#pragma unroll
            for (int j = 0; j < 8; ++j) asm volatile("" : "+v"(pf[j]));
            mc += l0 * 1e-30f;  // loop-carried, so nothing is hoisted
        }
        if (MODE == 3) {
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
                __builtin_amdgcn_sched_group_barrier(0x002, 7, 0);  // seven vector instructions
            }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) asm volatile("" : "+a"(acc[q]));  // the products stay in the loop (accumulation registers)
        __builtin_amdgcn_sched_barrier(0);
    }
    const unsigned long long t1 = __builtin_readcyclecounter();
    float res = l0 + l1 + mc;
    for (int j = 0; j < 4; ++j)
        for (int r = 0; r < 16; ++r) res += acc[j][r];
    for (int j = 0; j < 8; ++j) res += (float)pf[j][0];
    out[blockIdx.x * 256 + threadIdx.x] = res;
    if (threadIdx.x == 0) cycles[blockIdx.x] = t1 - t0;
}

// Operand values: gaussian = 0: bf16 in [1, 2) with random mantissas (few bits toggle); 1: N(0, 1)
// rounded to bf16, like the attention inputs (sign, exponent and mantissa all toggle: more power).
static void fill_operands(unsigned* h, int n_words, int gaussian) {
    uint64_t st = 0x2506013800ull;
    auto next = [&]() { st = st * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(st >> 32); };
    auto bf16_of = [](float x) { uint32_t u; memcpy(&u, &x, 4); return (uint32_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16); };
    for (int i = 0; i < n_words; ++i) {
        if (!gaussian) { h[i] = 0x3f803f80u ^ (next() & 0x007f007fu); continue; }
        const float u1 = ((next() >> 8) + 1) * (1.0f / 16777217.0f), u2 = (next() >> 8) * (1.0f / 16777216.0f);
        const float r = sqrtf(-2.0f * logf(u1));
        h[i] = bf16_of(r * cosf(6.2831853f * u2)) | (bf16_of(r * sinf(6.2831853f * u2)) << 16);
    }
}

template <int MODE>
static int run_mode(int workgroups, int iters, int gaussian, float* ms, double* cycles_per_iter) {
    float* out = nullptr;
    u32x4* in = nullptr;
    unsigned long long* cyc = nullptr;
    if (hipMalloc(&out, (size_t)workgroups * 256 * 4) != hipSuccess) return -6;
    if (hipMalloc(&in, 65536 * 16) != hipSuccess) return -6;
    if (hipMalloc(&cyc, (size_t)workgroups * 8) != hipSuccess) return -6;
    unsigned* h = new unsigned[65536 * 4];
    fill_operands(h, 65536 * 4, gaussian);
    int rc = 0;
    hipEvent_t e0, e1;
    if (hipMemcpy(in, h, 65536 * 16, hipMemcpyHostToDevice) != hipSuccess || hipEventCreate(&e0) != hipSuccess ||
        hipEventCreate(&e1) != hipSuccess) rc = -5;
    if (rc == 0) {
        hipLaunchKernelGGL(issue_mix<MODE>, dim3(workgroups), dim3(256), 0, 0, out, in, 50, 0.18f, cyc);  // warm-up
        hipEventRecord(e0, 0);
        hipLaunchKernelGGL(issue_mix<MODE>, dim3(workgroups), dim3(256), 0, 0, out, in, iters, 0.18f, cyc);
        hipEventRecord(e1, 0);
        unsigned long long c0 = 0;
        if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(ms, e0, e1) != hipSuccess ||
            hipMemcpy(&c0, cyc, 8, hipMemcpyDeviceToHost) != hipSuccess) rc = -5;
        *cycles_per_iter = (double)c0 / iters;
        hipEventDestroy(e0);
        hipEventDestroy(e1);
    }
    delete[] h;
    hipFree(out);
    hipFree(in);
    hipFree(cyc);
    return rc;
}

// mode 0..3 as above, gaussian as in fill_operands; one wavefront per SIMD when workgroups == number of CUs, two when
// workgroups == twice that.
// Returns 0, -5 on a HIP error, -6 on allocation failure, -2 on a bad mode.
extern "C" int nfd_probe_issue_mix(int mode, int workgroups, int iters, int gaussian, float* ms, double* cycles_per_iter) {
    if (!ms || !cycles_per_iter || workgroups < 1 || iters < 1) return -2;
    switch (mode) {
        case 0: return run_mode<0>(workgroups, iters, gaussian, ms, cycles_per_iter);
        case 1: return run_mode<1>(workgroups, iters, gaussian, ms, cycles_per_iter);
        case 2: return run_mode<2>(workgroups, iters, gaussian, ms, cycles_per_iter);
        case 3: return run_mode<3>(workgroups, iters, gaussian, ms, cycles_per_iter);
        default: return -2;
    }
}

// Micro-benchmark: do matrix (MFMA) and vector (VALU) instructions of one SIMD overlap on gfx950?
//
// Every block has 8 wavefronts, two per SIMD.  Wavefronts 0-3 (one per SIMD) run a chain of MFMA
// instructions, wavefronts 4-7 (the other one on each SIMD) a chain of independent fp32 FMAs or of
// transcendentals; each kind of work is sized to take the same time alone.  If the two pipelines overlap, running
// both takes as long as one of them; if they exclude each other, the times add.  A second variant puts both
// instruction streams, independent of each other, into the same wavefront.
//
// Build and run (one MI355X):
//   hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops \
//       paper_2506_02023_amd/microbench/mfma_valu_overlap.hip -o paper_2506_02023_amd/microbench/mfma_valu_overlap
//   paper_2506_02023_amd/microbench/mfma_valu_overlap
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

enum { MATRIX_F32 = 1, MATRIX_F16 = 2, VEC_FMA = 4, VEC_TRANS = 8, SAME_WAVE = 16 };

// 16 MFMAs of 64 cycles (fp32, 32x32x2) or 32 of 32 cycles (fp16, 32x32x16): 1024 cycles of the matrix pipeline
__device__ inline void matrix_f32(f32x16 &acc0, f32x16 &acc1, float av, float bv)
{
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc1, 0, 0, 0);
    }
}
__device__ inline void matrix_f16(f32x16 &acc0, f32x16 &acc1, f16x8 ah, f16x8 bh)
{
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bh, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bh, acc1, 0, 0, 0);
    }
}
// 256 independent-enough FMAs (8 chains): 1024 cycles of the vector pipeline
__device__ inline void vector_fma(float (&x)[8], float a, float b)
{
#pragma unroll
    for (int u = 0; u < 32; ++u)
#pragma unroll
        for (int k = 0; k < 8; ++k) x[k] = fmaf(x[k], a, b);
}
// 128 transcendentals (v_exp_f32, 4 chains)
__device__ inline void vector_trans(float (&x)[8])
{
#pragma unroll
    for (int u = 0; u < 32; ++u)
#pragma unroll
        for (int k = 0; k < 4; ++k) x[k] = __builtin_amdgcn_exp2f(x[k]);
}

__global__ void __launch_bounds__(512) k_overlap(float *out, int iters, int mode, float a, float b)
{
    const bool first = (threadIdx.x >> 8) == 0;   // wavefronts 0-3: one per SIMD
    const bool same = (mode & SAME_WAVE) != 0;
    f32x16 acc0, acc1;
    for (int r = 0; r < 16; ++r) { acc0[r] = 0.f; acc1[r] = 0.f; }
    float x[8];
    for (int k = 0; k < 8; ++k) x[k] = a + 0.001f * k;
    const float av = a + threadIdx.x, bv = b;
    f16x8 ah, bh;
    for (int k = 0; k < 8; ++k) { ah[k] = (_Float16)(a + k); bh[k] = (_Float16)b; }
    const bool do_matrix = same ? first : first;
    const bool do_vector = same ? first : !first;
    for (int it = 0; it < iters; ++it) {
        if (do_matrix && (mode & MATRIX_F32)) matrix_f32(acc0, acc1, av, bv);
        if (do_matrix && (mode & MATRIX_F16)) matrix_f16(acc0, acc1, ah, bh);
        if (do_vector && (mode & VEC_FMA)) vector_fma(x, a, b);
        if (do_vector && (mode & VEC_TRANS)) vector_trans(x);
    }
    float res = 0.f;
    for (int r = 0; r < 16; ++r) res += acc0[r] + acc1[r];
    for (int k = 0; k < 8; ++k) res += x[k];
    out[blockIdx.x * 512 + threadIdx.x] = res;
}

static float run(int mode, int blocks, int iters)
{
    static float *out = nullptr;
    if (!out && hipMalloc(&out, (size_t)4096 * 512 * 4) != hipSuccess) exit(1);
    hipEvent_t e0, e1;
    (void)hipEventCreate(&e0);
    (void)hipEventCreate(&e1);
    k_overlap<<<blocks, 512>>>(out, 10, mode, 0.999f, 0.001f);
    (void)hipDeviceSynchronize();
    (void)hipEventRecord(e0);
    k_overlap<<<blocks, 512>>>(out, iters, mode, 0.999f, 0.001f);
    (void)hipEventRecord(e1);
    (void)hipDeviceSynchronize();
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return ms;
}

int main()
{
    const int blocks = 256, iters = 4000;   // one block per compute unit: every SIMD holds one wavefront of each kind
    struct { const char *name; int mode; } cases[] = {
        {"fp32 MFMA alone (v_mfma_f32_32x32x2_f32)", MATRIX_F32},
        {"fp32 FMA alone (v_fma_f32)", VEC_FMA},
        {"fp32 MFMA + FMA, other wavefront of the SIMD", MATRIX_F32 | VEC_FMA},
        {"fp32 MFMA + FMA, same wavefront", MATRIX_F32 | VEC_FMA | SAME_WAVE},
        {"transcendental alone (v_exp_f32)", VEC_TRANS},
        {"fp32 MFMA + transcendental, other wavefront", MATRIX_F32 | VEC_TRANS},
        {"fp16 MFMA alone (v_mfma_f32_32x32x16_f16)", MATRIX_F16},
        {"fp16 MFMA + FMA, other wavefront of the SIMD", MATRIX_F16 | VEC_FMA},
        {"fp16 MFMA + FMA, same wavefront", MATRIX_F16 | VEC_FMA | SAME_WAVE},
        {"fp16 MFMA + transcendental, other wavefront", MATRIX_F16 | VEC_TRANS},
    };
    printf("%-52s %10s\n", "case (256 blocks of 8 wavefronts, 4000 iterations)", "ms");
    for (auto &c : cases) printf("%-52s %10.3f\n", c.name, run(c.mode, blocks, iters));
    // sustained matrix rates with every SIMD fully occupied by matrix wavefronts (2 per SIMD)
    const double flop32 = 2.0 * 32 * 32 * 2 * 16, flop16 = 2.0 * 32 * 32 * 16 * 32;
    const float t32 = run(MATRIX_F32 | SAME_WAVE, 512, iters), t16 = run(MATRIX_F16 | SAME_WAVE, 512, iters);
    printf("sustained fp32 MFMA: %.1f TFLOP/s   fp16 MFMA: %.1f TFLOP/s\n",
           flop32 * iters * 512 * 4 / (t32 * 1e-3) / 1e12, flop16 * iters * 512 * 4 / (t16 * 1e-3) / 1e12);
    return 0;
}

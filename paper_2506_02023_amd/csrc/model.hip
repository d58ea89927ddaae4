// Radial message-passing potential on gfx950: forward, hand-written reverse pass, forces.
//
// Model (benchmark configuration 0):  h0 = Emb[z];  per layer  g = h Wm,
//   a_i = sum_{e: recv=i} (SiLU(b_e W1) W2) * g_send(e),  h += SiLU(a Wo);
//   eps_i = SiLU(h Wr1) . wr2,  E = sum eps,  F = -dE/dr.
// Partitioned execution follows the paper's scheme (Graph-Parallel Message
// Passing; Distributing Atom Graphs): every partition computes the edges whose
// receiver it owns, ghost rows of g are refreshed from their owners before each
// layer's edge step and ghost-row gradients are added back to the owners in the
// reverse pass.
//
// Kernel design
//  * All dense contractions (filter MLP per edge, F x F maps per node) run on
//    v_mfma_f32_32x32x2_f32 with items (edges or nodes) as the 32 MFMA columns
//    and features as rows.  In that orientation the accumulator layout of one
//    product is directly the B operand of the next one if the contraction index
//    is visited in the order the accumulator registers hold it; the weight (A)
//    operands are pre-packed in that order, so chained products need no
//    transposition or lane exchange.
//  * The per-receiver reduction is LDS-staged: a 32-edge tile of filter outputs
//    is written to LDS edge-major, then each lane owns one feature, reads the
//    tile row by row, multiplies with the gathered sender row (one coalesced
//    256-byte load per edge) and keeps a running sum that is flushed when the
//    receiver changes.  No atomics; the summation order is the canonical edge order.
//  * Reverse pass without scatter: the edge set is symmetric (i<-j,S) <-> (j<-i,-S)
//    with bitwise equal length, hence equal filter value w.  So
//      gbar_i = sum_{e in row i} w_e * abar_send(e)
//      dE/dd summed over an edge and its mirror = dw/dd . (abar_i*g_j + abar_j*g_i)
//    are both receiver-side gathers.  In a partition, abar of ghost rows is zero
//    and ghost rows carry the sub-row of neighbours owned by the partition, which
//    yields exactly the ghost-row gradients the owner must receive.
#include "mlip_internal.h"

#include <algorithm>
#include <cmath>

namespace mlip {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

constexpr int kBufferFlags = 0x00020000;  // raw 32-bit buffer descriptor word 3 on gfx9-family targets
constexpr float kPi = 3.14159265358979323846f;

__device__ inline void wave_lds_fence()
{
    // LDS operations of one wavefront execute in program order; this only stops the
    // compiler from moving them across the point where lanes exchange roles.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ inline float sigmoidf_fast(float x) { return __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }

// The edge kernels evaluate SiLU on pre-scaled pre-activations t' = c t with c = -log2(e):
// sigmoid(t) = 1 / (1 + 2^t'), so the scaling multiply disappears (c is folded into the packed W1,
// 1/c into the packed W2 that consumes s' = c SiLU(t)).
constexpr float kSiluScale = -1.4426950408889634f;
constexpr float kSiluScaleInv = -0.6931471805599453f;
__device__ inline float sigmoid_scaled(float tp) { return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(tp)); }

struct BasisParams {
    float rc, inv_rc;
    float pc0;   // p (p + 1) (p + 2) / 2, the factor of the envelope's derivative
    int p;
};

// b[n] = sin((n+1) pi x) / d * u(x) and, if DERIV, db[n] = d b[n] / d d   (n = 0..7)
template <bool DERIV>
__device__ inline void radial_basis(float d, const BasisParams &bp, float (&b)[8], float (&db)[8])
{
    float x = fminf(d * bp.inv_rc, 1.0f);
    // sin(pi x), cos(pi x) on [0,1]: with z = pi (x - 1/2) in [-pi/2, pi/2], sin(pi x) = cos z and
    // cos(pi x) = -sin z; Taylor polynomials to z^12 / z^13 (truncation below 1e-8)
    const float z = kPi * (x - 0.5f), z2 = z * z;
    float s1 = 1.0f + z2 * (-0.5f + z2 * (4.16666667e-2f + z2 * (-1.38888889e-3f + z2 * (2.48015873e-5f +
               z2 * (-2.75573192e-7f + z2 * 2.08767570e-9f)))));
    float c1v = -z * (1.0f + z2 * (-1.66666667e-1f + z2 * (8.33333333e-3f + z2 * (-1.98412698e-4f +
                z2 * (2.75573192e-6f + z2 * (-2.50521084e-8f + z2 * 1.60590438e-10f))))));
    // envelope in factored form, free of cancellation near the cutoff where it goes to zero with its first two
    // derivatives:  u(x) = (1 - x)^3 sum_{k < p} C(k + 2, 2) x^k  (the same polynomial as 1 - (p+1)(p+2)/2 x^p
    // + p(p+2) x^(p+1) - p(p+1)/2 x^(p+2)),  u'(x) = -p(p+1)(p+2)/2 x^(p-1) (1 - x)^2
    const float w1 = 1.0f - x;
    float xpm1 = 1.0f;
    float q = (float)(bp.p * (bp.p + 1) / 2);
    for (int k = bp.p - 2; k >= 0; --k) {
        q = fmaf(q, x, (float)((k + 1) * (k + 2) / 2));
        xpm1 *= x;
    }
    const float w2 = w1 * w1;
    const float u = w2 * w1 * q;
    const float inv_d = __builtin_amdgcn_rcpf(d);
    float du_term = 0.f;  // u'/rc - u/d
    if (DERIV) {
        const float du = -bp.pc0 * xpm1 * w2;
        du_term = du * bp.inv_rc - u * inv_d;
    }
    const float u_rc = u * bp.inv_rc;
    float sn = s1, cn = c1v;
#pragma unroll
    for (int n = 0; n < 8; ++n) {
        b[n] = sn * u * inv_d;
        if (DERIV) db[n] = fmaf((float)(n + 1) * kPi, cn * u_rc, sn * du_term) * inv_d;   // (n+1) pi: a literal operand
        const float s2 = sn * c1v + cn * s1;
        cn = cn * c1v - sn * s1;
        sn = s2;
    }
}

// ---------------------------------------------------------------- packed weights
//
// pack_ff: F x F matrix M[o][k] as MFMA A operands, index
//   ((((bo * NB + bi) * 4 + a) * 64 + lane) * 4 + c)  ->  M[32 bo + lane % 32][32 bi + 8 a + 4 (lane / 32) + c]
// with M[o][k] = W[k][o] (TRANS, y = x W) or W[o][k] (y = x W^T).
// pack_w1: K = 8 rows, index ((bo * 4 + s) * 64 + lane) -> W1[2 s + lane / 32][32 bo + lane % 32].

__global__ void k_pack_ff(const float *__restrict__ W, int F, int trans, float scale, float *__restrict__ out)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= F * F) return;
    const int NB = F / 32;
    const int c = idx & 3, lane = (idx >> 2) & 63, a = (idx >> 8) & 3, bb = idx >> 10;
    const int bi = bb % NB, bo = bb / NB;
    const int o = 32 * bo + (lane & 31);
    const int k = 32 * bi + 8 * a + 4 * (lane >> 5) + c;
    out[idx] = scale * (trans ? W[k * F + o] : W[o * F + k]);
}

__global__ void k_pack_w1(const float *__restrict__ W1, int F, float scale, float *__restrict__ out)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    const int NB = F / 32;
    if (idx >= NB * 4 * 64) return;
    const int lane = idx & 63, s = (idx >> 6) & 3, bo = idx >> 8;
    out[idx] = scale * W1[(2 * s + (lane >> 5)) * F + 32 * bo + (lane & 31)];
}

// bf16 form of an F x F operand for v_mfma_f32_32x32x16_bf16 (the bf16 precision mode: the W2 products of the
// filter MLP run on the bf16 matrix pipeline with fp32 accumulation, at 1/16 of the fp32 MFMA time).
// Index (((bo * NB + bi) * 2 + q) * 64 + lane) * 8 + t  ->  M[32 bo + lane % 32][32 bi + 8 (r / 4) + 4 (lane / 32) + r % 4],
// r = 8 q + t: element t of lane-half h of MFMA (bi, q) pairs with accumulator register r of a chained product
// (or with the same feature of an item-major LDS row).
__global__ void k_pack_ff_bf16(const float *__restrict__ W, int F, int trans, float scale, __bf16 *__restrict__ out)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= F * F) return;
    const int NB = F / 32;
    const int t = idx & 7, lane = (idx >> 3) & 63, q = (idx >> 9) & 1, bb = idx >> 10;
    const int bi = bb % NB, bo = bb / NB;
    const int r = 8 * q + t;
    const int o = 32 * bo + (lane & 31);
    const int k = 32 * bi + 8 * (r / 4) + 4 * (lane >> 5) + (r & 3);
    out[idx] = (__bf16)(scale * (trans ? W[k * F + o] : W[o * F + k]));
}

// Split-fp16 form of the same operand: every fp32 value v is kept as hi + lo, hi = fp16(v), lo = fp16(v - hi)
// (22 significant bits together); a product of two such values is taken as hi hi + hi lo + lo hi with fp32
// accumulation.  What is dropped (lo lo, and the rounding of the two lo parts) is about 3 * 2^-22 of the term,
// the size of the rounding an fp32 accumulation of 64 terms makes anyway, at 3/16 of the fp32 MFMA's matrix time.
// hi parts first (F * F halves), then lo parts: together the bytes of the fp32 pack.
__global__ void k_pack_ff_f16x2(const float *__restrict__ W, int F, int trans, float scale, _Float16 *__restrict__ out)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= F * F) return;
    const int NB = F / 32;
    const int t = idx & 7, lane = (idx >> 3) & 63, q = (idx >> 9) & 1, bb = idx >> 10;
    const int bi = bb % NB, bo = bb / NB;
    const int r = 8 * q + t;
    const int o = 32 * bo + (lane & 31);
    const int k = 32 * bi + 8 * (r / 4) + 4 * (lane >> 5) + (r & 3);
    const float v = scale * (trans ? W[k * F + o] : W[o * F + k]);
    const _Float16 h = (_Float16)v;
    out[idx] = h;
    out[F * F + idx] = (_Float16)(v - (float)h);
}

__device__ inline void split_f16(const float (&v)[8], f16x8 &hi, f16x8 &lo)
{
#pragma unroll
    for (int i = 0; i < 8; i += 2) {
        const f32x2 p = {v[i], v[i + 1]};
        const f16x2 h = __builtin_convertvector(p, f16x2);
        const f16x2 l = __builtin_convertvector(p - __builtin_convertvector(h, f32x2), f16x2);
        hi[i] = h[0];
        hi[i + 1] = h[1];
        lo[i] = l[0];
        lo[i + 1] = l[1];
    }
}

__device__ inline bf16x8 to_bf16x8(const float (&v)[8])
{
    bf16x8 o;
#pragma unroll
    for (int i = 0; i < 8; i += 2) {
        const f32x2 p = {v[i], v[i + 1]};
        const bf16x2 h = __builtin_convertvector(p, bf16x2);   // round to nearest even, two per instruction
        o[i] = h[0];
        o[i + 1] = h[1];
    }
    return o;
}

template <int F> struct Dims {
    static constexpr int NB = F / 32;
    static constexpr int FS = F + 4;      // LDS row stride of an item-major tile
    static constexpr int TILE = 32 * FS;  // floats per 32-item tile
    static constexpr int PACK1 = NB * 4 * 64;
    static constexpr int PACKF = F * F;
};

// out[bo] = sum_k M[.][k] in[k][.], `in` held in accumulator layout (chained product)
template <int F>
__device__ inline void gemm_regs(const float *__restrict__ Ap, const f32x16 (&in)[Dims<F>::NB],
                                 f32x16 (&out)[Dims<F>::NB], int lane)
{
    constexpr int NB = Dims<F>::NB;
#pragma unroll
    for (int bo = 0; bo < NB; ++bo)
#pragma unroll
        for (int r = 0; r < 16; ++r) out[bo][r] = 0.f;
#pragma unroll
    for (int bi = 0; bi < NB; ++bi)
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int bo = 0; bo < NB; ++bo) {
                const f32x4 av = *reinterpret_cast<const f32x4 *>(Ap + ((((bo * NB + bi) * 4 + a) * 64 + lane) * 4));
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    out[bo] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[c], in[bi][4 * a + c], out[bo], 0, 0, 0);
            }
}

// same product with the B operand read from an item-major LDS tile [32][FS]; A and B operand
// loads of step k+1 are issued before the MFMAs of step k
template <int F, bool ACCUMULATE = false>
__device__ inline void gemm_lds(const float *__restrict__ Ap, const float *tile, f32x16 (&out)[Dims<F>::NB], int lane)
{
    constexpr int NB = Dims<F>::NB;
    constexpr int FS = Dims<F>::FS;
    constexpr int STEPS = NB * 4;
    const int c32 = lane & 31, h = lane >> 5;
    if (!ACCUMULATE)
#pragma unroll
        for (int bo = 0; bo < NB; ++bo)
#pragma unroll
            for (int r = 0; r < 16; ++r) out[bo][r] = 0.f;
    const float *bp = tile + c32 * FS + 4 * h;
    const float *ap = Ap + lane * 4;
    f32x4 bv = *reinterpret_cast<const f32x4 *>(bp);
    f32x4 av[NB];
#pragma unroll
    for (int bo = 0; bo < NB; ++bo) av[bo] = *reinterpret_cast<const f32x4 *>(ap + ((bo * NB) * 4) * 256);
#pragma unroll
    for (int st = 0; st < STEPS; ++st) {
        f32x4 bn = bv, an[NB];
#pragma unroll
        for (int bo = 0; bo < NB; ++bo) an[bo] = av[bo];
        if (st + 1 < STEPS) {
            const int bi = (st + 1) / 4, a = (st + 1) % 4;
            bn = *reinterpret_cast<const f32x4 *>(bp + 32 * bi + 8 * a);
#pragma unroll
            for (int bo = 0; bo < NB; ++bo)
                an[bo] = *reinterpret_cast<const f32x4 *>(ap + (((bo * NB + bi) * 4 + a)) * 256);
        }
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int bo = 0; bo < NB; ++bo)
                out[bo] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[bo][c], bv[c], out[bo], 0, 0, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, NB + 1, 0);  // the next step's LDS reads first
        __builtin_amdgcn_sched_group_barrier(0x008, 4 * NB, 0);  // then this step's MFMAs
        bv = bn;
#pragma unroll
        for (int bo = 0; bo < NB; ++bo) av[bo] = an[bo];
    }
}

// A operands of an F x F matrix held in registers (one f32x4 per (bo, bi, a))
template <int F> struct RegPack {
    f32x4 v[Dims<F>::NB][Dims<F>::NB][4];
};

template <int F> __device__ inline void load_pack(RegPack<F> &P, const float *__restrict__ Ap, int lane)
{
    constexpr int NB = Dims<F>::NB;
#pragma unroll
    for (int bo = 0; bo < NB; ++bo)
#pragma unroll
        for (int bi = 0; bi < NB; ++bi)
#pragma unroll
            for (int a = 0; a < 4; ++a)
                P.v[bo][bi][a] = *reinterpret_cast<const f32x4 *>(Ap + ((((bo * NB + bi) * 4 + a) * 64 + lane) * 4));
}

// chained product with register-resident weights; consecutive MFMAs alternate accumulators
template <int F>
__device__ inline void gemm_rr(const RegPack<F> &P, const f32x16 (&in)[Dims<F>::NB], f32x16 (&out)[Dims<F>::NB])
{
    constexpr int NB = Dims<F>::NB;
#pragma unroll
    for (int bo = 0; bo < NB; ++bo)
#pragma unroll
        for (int r = 0; r < 16; ++r) out[bo][r] = 0.f;
#pragma unroll
    for (int bi = 0; bi < NB; ++bi)
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int bo = 0; bo < NB; ++bo)
                    out[bo] = __builtin_amdgcn_mfma_f32_32x32x2f32(P.v[bo][bi][a][c], in[bi][4 * a + c], out[bo], 0, 0, 0);
}

// chained product with the weights in LDS (packed A operands), B operand in registers; the A
// operands of step k+1 are fetched while the MFMAs of step k run
template <int F>
__device__ inline void gemm_rl(const float *__restrict__ Ap, const f32x16 (&in)[Dims<F>::NB],
                               f32x16 (&out)[Dims<F>::NB], int lane)
{
    constexpr int NB = Dims<F>::NB;
    constexpr int STEPS = NB * 4;
#pragma unroll
    for (int bo = 0; bo < NB; ++bo)
#pragma unroll
        for (int r = 0; r < 16; ++r) out[bo][r] = 0.f;
    const float *ap = Ap + lane * 4;
    f32x4 av[NB];
#pragma unroll
    for (int bo = 0; bo < NB; ++bo) av[bo] = *reinterpret_cast<const f32x4 *>(ap + ((bo * NB) * 4) * 256);
#pragma unroll
    for (int st = 0; st < STEPS; ++st) {
        const int bi = st / 4, a = st % 4;
        f32x4 an[NB];
#pragma unroll
        for (int bo = 0; bo < NB; ++bo) an[bo] = av[bo];
        if (st + 1 < STEPS) {
            const int bi2 = (st + 1) / 4, a2 = (st + 1) % 4;
#pragma unroll
            for (int bo = 0; bo < NB; ++bo)
                an[bo] = *reinterpret_cast<const f32x4 *>(ap + (((bo * NB + bi2) * 4 + a2)) * 256);
        }
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int bo = 0; bo < NB; ++bo)
                out[bo] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[bo][c], in[bi][4 * a + c], out[bo], 0, 0, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, NB, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 4 * NB, 0);
#pragma unroll
        for (int bo = 0; bo < NB; ++bo) av[bo] = an[bo];
    }
}

// gemm_rl in bf16: weights as a bf16 pack in LDS, the chained B operand rounded to bf16, fp32 accumulation
template <int F>
__device__ inline void gemm_rl_bf16(const __bf16 *__restrict__ Ap, const f32x16 (&in)[Dims<F>::NB],
                                    f32x16 (&out)[Dims<F>::NB], int lane)
{
    constexpr int NB = Dims<F>::NB;
    const bf16x8 *A = reinterpret_cast<const bf16x8 *>(Ap) + lane;
#pragma unroll
    for (int bo = 0; bo < NB; ++bo)
#pragma unroll
        for (int r = 0; r < 16; ++r) out[bo][r] = 0.f;
#pragma unroll
    for (int bi = 0; bi < NB; ++bi)
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            float v[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) v[t] = in[bi][8 * q + t];
            const bf16x8 b = to_bf16x8(v);
#pragma unroll
            for (int bo = 0; bo < NB; ++bo)
                out[bo] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[((bo * NB + bi) * 2 + q) * 64], b, out[bo], 0, 0, 0);
        }
}

// the same with the B operand taken from an item-major LDS row of this lane's item (fp32, rounded here)
template <int F>
__device__ inline void gemm_row_bf16(const __bf16 *__restrict__ Ap, const float *row, f32x16 (&out)[Dims<F>::NB], int lane)
{
    constexpr int NB = Dims<F>::NB;
    const int h = lane >> 5;
    const bf16x8 *A = reinterpret_cast<const bf16x8 *>(Ap) + lane;
#pragma unroll
    for (int bo = 0; bo < NB; ++bo)
#pragma unroll
        for (int r = 0; r < 16; ++r) out[bo][r] = 0.f;
#pragma unroll
    for (int bi = 0; bi < NB; ++bi)
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const f32x4 lo4 = *reinterpret_cast<const f32x4 *>(row + 32 * bi + 16 * q + 4 * h);
            const f32x4 hi4 = *reinterpret_cast<const f32x4 *>(row + 32 * bi + 16 * q + 8 + 4 * h);
            const float v[8] = {lo4[0], lo4[1], lo4[2], lo4[3], hi4[0], hi4[1], hi4[2], hi4[3]};
            const bf16x8 b = to_bf16x8(v);
#pragma unroll
            for (int bo = 0; bo < NB; ++bo)
                out[bo] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[((bo * NB + bi) * 2 + q) * 64], b, out[bo], 0, 0, 0);
        }
}

// gemm_rl and gemm_row in split fp16 (three MFMAs of depth 16 per 16 k-values)
template <int F>
__device__ inline void gemm_rl_f16x3(const _Float16 *__restrict__ Ap, const f32x16 (&in)[Dims<F>::NB],
                                     f32x16 (&out)[Dims<F>::NB], int lane)
{
    constexpr int NB = Dims<F>::NB;
    const f16x8 *Ah = reinterpret_cast<const f16x8 *>(Ap) + lane;
    const f16x8 *Al = reinterpret_cast<const f16x8 *>(Ap + F * F) + lane;
#pragma unroll
    for (int bo = 0; bo < NB; ++bo)
#pragma unroll
        for (int r = 0; r < 16; ++r) out[bo][r] = 0.f;
#pragma unroll
    for (int bi = 0; bi < NB; ++bi)
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            float v[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) v[t] = in[bi][8 * q + t];
            f16x8 bh, bl;
            split_f16(v, bh, bl);
#pragma unroll
            for (int bo = 0; bo < NB; ++bo) {
                const f16x8 ah = Ah[((bo * NB + bi) * 2 + q) * 64], al = Al[((bo * NB + bi) * 2 + q) * 64];
                out[bo] = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, bh, out[bo], 0, 0, 0);   // small terms first
                out[bo] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bl, out[bo], 0, 0, 0);
                out[bo] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bh, out[bo], 0, 0, 0);
            }
        }
}

template <int F>
__device__ inline void gemm_row_f16x3(const _Float16 *__restrict__ Ap, const float *row, f32x16 (&out)[Dims<F>::NB], int lane)
{
    constexpr int NB = Dims<F>::NB;
    const int h = lane >> 5;
    const f16x8 *Ah = reinterpret_cast<const f16x8 *>(Ap) + lane;
    const f16x8 *Al = reinterpret_cast<const f16x8 *>(Ap + F * F) + lane;
#pragma unroll
    for (int bo = 0; bo < NB; ++bo)
#pragma unroll
        for (int r = 0; r < 16; ++r) out[bo][r] = 0.f;
#pragma unroll
    for (int bi = 0; bi < NB; ++bi)
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const f32x4 lo4 = *reinterpret_cast<const f32x4 *>(row + 32 * bi + 16 * q + 4 * h);
            const f32x4 hi4 = *reinterpret_cast<const f32x4 *>(row + 32 * bi + 16 * q + 8 + 4 * h);
            const float v[8] = {lo4[0], lo4[1], lo4[2], lo4[3], hi4[0], hi4[1], hi4[2], hi4[3]};
            f16x8 bh, bl;
            split_f16(v, bh, bl);
#pragma unroll
            for (int bo = 0; bo < NB; ++bo) {
                const f16x8 ah = Ah[((bo * NB + bi) * 2 + q) * 64], al = Al[((bo * NB + bi) * 2 + q) * 64];
                out[bo] = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, bh, out[bo], 0, 0, 0);
                out[bo] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bl, out[bo], 0, 0, 0);
                out[bo] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bh, out[bo], 0, 0, 0);
            }
        }
}

template <int F> struct RegPack1 {
    float v[Dims<F>::NB][4];
};

template <int F> __device__ inline void load_pack1(RegPack1<F> &P, const float *__restrict__ A1, int lane)
{
#pragma unroll
    for (int bo = 0; bo < Dims<F>::NB; ++bo)
#pragma unroll
        for (int s = 0; s < 4; ++s) P.v[bo][s] = A1[(bo * 4 + s) * 64 + lane];
}

template <int F>
__device__ inline void gemm_k8r(const RegPack1<F> &P, const float (&v)[8], f32x16 (&out)[Dims<F>::NB], int lane)
{
    constexpr int NB = Dims<F>::NB;
    const int h = lane >> 5;
#pragma unroll
    for (int bo = 0; bo < NB; ++bo)
#pragma unroll
        for (int r = 0; r < 16; ++r) out[bo][r] = 0.f;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const float bv = h ? v[2 * s + 1] : v[2 * s];
#pragma unroll
        for (int bo = 0; bo < NB; ++bo)
            out[bo] = __builtin_amdgcn_mfma_f32_32x32x2f32(P.v[bo][s], bv, out[bo], 0, 0, 0);
    }
}

// one 32-feature block of gemm_k8r
template <int F>
__device__ inline void gemm_k8r_block(const RegPack1<F> &P, const float (&v)[8], int bo, f32x16 &out, int lane)
{
    const int h = lane >> 5;
#pragma unroll
    for (int r = 0; r < 16; ++r) out[r] = 0.f;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const float bv = h ? v[2 * s + 1] : v[2 * s];
        out = __builtin_amdgcn_mfma_f32_32x32x2f32(P.v[bo][s], bv, out, 0, 0, 0);
    }
}

// out[f][item] = sum_n W1[n][f] v[n][item], v = 8 per-lane values of the lane's item
template <int F>
__device__ inline void gemm_k8(const float *__restrict__ A1, const float (&v)[8], f32x16 (&out)[Dims<F>::NB], int lane)
{
    constexpr int NB = Dims<F>::NB;
    const int h = lane >> 5;
#pragma unroll
    for (int bo = 0; bo < NB; ++bo)
#pragma unroll
        for (int r = 0; r < 16; ++r) out[bo][r] = 0.f;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const float bv = h ? v[2 * s + 1] : v[2 * s];
#pragma unroll
        for (int bo = 0; bo < NB; ++bo)
            out[bo] = __builtin_amdgcn_mfma_f32_32x32x2f32(A1[(bo * 4 + s) * 64 + lane], bv, out[bo], 0, 0, 0);
    }
}

// accumulator layout -> item-major LDS tile
template <int F>
__device__ inline void regs_to_tile(const f32x16 (&v)[Dims<F>::NB], float *tile, int lane)
{
    constexpr int NB = Dims<F>::NB;
    constexpr int FS = Dims<F>::FS;
    const int c32 = lane & 31, h = lane >> 5;
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            f32x4 x = {v[b][4 * a], v[b][4 * a + 1], v[b][4 * a + 2], v[b][4 * a + 3]};
            *reinterpret_cast<f32x4 *>(tile + c32 * FS + 32 * b + 8 * a + 4 * h) = x;
        }
}

__device__ inline int64_t lower_bound_i64(const int64_t *__restrict__ a, int64_t n, int64_t v)
{
    int64_t lo = 0, hi = n;  // first index in [0, n] with a[idx] >= v (a has n + 1 entries, searched over [0, n))
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (a[mid] < v) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// ---------------------------------------------------------------- edge kernels

struct EdgeArgs {
    int64_t n_rows;            // receiver rows processed
    int64_t n_chunks;
    int64_t n_stored;          // reverse: edges [0, n_stored) have their w_e in wstore
    int64_t n_nodes;           // rows of g / abar (n_local)
    const int64_t *row_ptr;
    const int32_t *senders;
    const int32_t *recv;       // receiver row of every edge
    const float *d;
    const float *g;            // [n_local][F]
    const float *abar;         // reverse: [n_local][F] (ghost rows zero)
    float *out;                // forward: a [n_rows][F]; reverse: gbar [n_rows][F]
    float *dsum;               // reverse: per-edge dE/dd of the edge and its mirror, summed over layers
    float *wstore;             // forward: filter values w_e [n_stored][F] kept for the reverse pass (or null)
    const int32_t *mirror;     // reverse: position of every edge's reverse edge
    const int32_t *chunk_row;  // first row of every work item
};

// What all partitions of one launch share: the layer's packed weights and the basis.
struct EdgeCommon {
    const float *A1, *A1s, *A2t, *A2n;   // A1s = c W1, A2t = W2 / c (see kSiluScale), A1 and A2n unscaled
    BasisParams bp;
    int need_gbar, first;
};

// One launch covers up to kBatch partitions, taken in order: work item w belongs to partition p
// with chunk_start[p] <= w < chunk_start[p + 1].  The partitions keep their own arrays (local rows,
// ghost rows); batching only removes the idle tail between per-partition launches.
constexpr int kBatch = 8;
enum { kPrecF32 = 0, kPrecBf16 = 1, kPrecF16x3 = 2 };
struct EdgeBatch {
    EdgeCommon c;
    int n;
    int64_t chunk_start[kBatch + 1];
    EdgeArgs s[kBatch];
};

// Persistent launch: the grid holds exactly the blocks that are resident at once, a multiple of 8.
// Blocks go to the 8 XCDs round-robin, so blocks b with the same b % 8 share an L2.  Each XCD takes one
// contiguous eighth of the work items and its blocks walk through it side by side (block slot s, wave w
// takes items 4 s + w, 4 (s + n_slots) + w, ...): at any moment an XCD works on a short contiguous run
// of rows, whose neighbourhoods overlap, so the sender rows it gathers stay in its L2.
struct ItemRange {
    int64_t first, end, stride;
};
__device__ inline ItemRange edge_items(int64_t total, int wave, int nw = 4)   // nw: wavefronts per block
{
    const int64_t n_slots = gridDim.x >> 3;
    const int64_t per = (((total + 7) >> 3) + 3) & ~(int64_t)3;
    const int64_t xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    ItemRange r;
    r.first = xcd * per + slot * nw + wave;
    r.end = min(total, (xcd + 1) * per);
    r.stride = n_slots * nw;
    return r;
}

__device__ inline int batch_find(const int64_t *start, int n, int64_t w)
{
    int p = 0;
#pragma unroll
    for (int q = 1; q < kBatch; ++q)
        if (q < n && w >= start[q]) p = q;
    return p;
}

// Read-only graph arrays are read through the constant address space when the index is
// wave-uniform: the load then goes through the scalar cache into SGPRs and costs no vector issue slot.
// (Valid because no kernel of this file writes the graph arrays.)
typedef const __attribute__((address_space(4))) int32_t *const_i32_ptr;
__device__ inline int32_t uniform_load(const int32_t *p, int64_t i)
{
    return reinterpret_cast<const_i32_ptr>(reinterpret_cast<uintptr_t>(p))[i];
}

// wavefront work item: the rows whose first edge lies in [chunk * kChunkEdges, (chunk + 1) * kChunkEdges)
__device__ inline bool chunk_rows(const EdgeArgs &A, int64_t chunk, int64_t &r0, int64_t &r1)
{
    r0 = uniform_load(A.chunk_row, chunk);
    r1 = uniform_load(A.chunk_row, chunk + 1);
    if (chunk == A.n_chunks - 1) r1 = A.n_rows;   // the forward step stops at the owned rows
    return r0 < r1;
}

// 32-bit buffer accesses: per-lane byte offset in a VGPR, wave-uniform byte offset in an SGPR, no
// vector address arithmetic; accesses outside the descriptor's range read 0 / are dropped.
__device__ inline float buffer_load_f32(__amdgpu_buffer_rsrc_t r, unsigned voff, int soff, int)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0));
}
__device__ inline void buffer_store_f32(float v, __amdgpu_buffer_rsrc_t r, unsigned voff, int soff, int)
{
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), r, voff, soff, 0);
}
// The same with the non-temporal hint (cache policy bit 1) for the kept filter values: written once, read once
// much later, they should not displace the gathered rows in the L2 (measured on the 1M-atom benchmark: 0.7 ms
// of 40 per step in fp32 mode, 1.5 ms of 34 in the split-fp16 mode).
__device__ inline float buffer_load_f32_stream(__amdgpu_buffer_rsrc_t r, unsigned voff, int soff)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 2));
}
__device__ inline void buffer_store_f32_stream(float v, __amdgpu_buffer_rsrc_t r, unsigned voff, int soff)
{
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), r, voff, soff, 2);
}

// Per-tile row bookkeeping shared by both edge kernels.  Every lane holds the receiver of its edge
// (rk, the sentinel r1 for lanes past the end of the chunk); the receiver of the following edge
// comes from the neighbouring lane or, for lane 31, from the next tile.  Bit k of the returned mask
// says "edge k is the last edge of its row"; it is wave-uniform, so the flush is a scalar branch.
__device__ inline uint32_t row_ends(int32_t rk, int32_t rn_first, bool valid, int lane, int32_t &rnext)
{
    const int32_t up = __shfl(rk, (lane & 31) + 1, 64);
    rnext = ((lane & 31) == 31) ? rn_first : up;
    return (uint32_t)__ballot(valid && rnext != rk);
}

// PREC selects how the F x F product with W2 runs: kPrecF32 fp32 MFMA, kPrecBf16 bf16 operands, kPrecF16x3 split fp16
template <int F, int PREC>
__global__ void __launch_bounds__(256, 3) k_edge_fwd(EdgeBatch B)
{
    using D = Dims<F>;
    extern __shared__ float lds[];
    float *A2t = lds;
    float *tiles = A2t + D::PACKF;
    for (int i = threadIdx.x; i < (PREC == kPrecBf16 ? D::PACKF / 2 : D::PACKF); i += 256) A2t[i] = B.c.A2t[i];
    __syncthreads();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int c32 = lane & 31;
    const unsigned f = lane & (F - 1);
    float *tile = tiles + wave * D::TILE;
    const EdgeCommon &C = B.c;
    RegPack1<F> W1;
    load_pack1<F>(W1, C.A1s, lane);
    const ItemRange items = edge_items(B.chunk_start[B.n], wave);
    int64_t item = items.first;
    for (int part = 0; part < B.n; ++part) {
    const int64_t part_end = min(items.end, B.chunk_start[part + 1]);
    if (item >= part_end) continue;
    const EdgeArgs A = B.s[part];
    const __amdgpu_buffer_rsrc_t g_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(A.g), 0, (int)(A.n_nodes * F * 4), kBufferFlags);
    const __amdgpu_buffer_rsrc_t o_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        A.out, 0, (int)(A.n_rows * F * 4), kBufferFlags);
    auto store_row = [&](int32_t row, float v) {
        if (F == 64 || lane < F) buffer_store_f32(v, o_rsrc, f * 4, row * (F * 4), 0);
    };
    for (; item < part_end; item += items.stride) {
    const int64_t chunk = item - B.chunk_start[part];
    int64_t r0, r1;
    if (!chunk_rows(A, chunk, r0, r1)) continue;
    // wave-uniform values loaded through vector instructions: keep them scalar (edge indices fit 32 bits)
    const int32_t e_lo = __builtin_amdgcn_readfirstlane((int32_t)A.row_ptr[r0]);
    const int32_t e_hi = __builtin_amdgcn_readfirstlane((int32_t)A.row_ptr[r1]);
    const int32_t r_end = (int32_t)r1;
    const bool keep_w = A.wstore != nullptr;
    if (e_lo >= e_hi) {   // only empty rows
        for (int32_t r = (int32_t)r0; r < r_end; ++r) store_row(r, 0.f);
        continue;
    }
    float acc = 0.f;
    // edge records of the first tile (lane k mod 32 holds edge tb + k, clamped to the item's last edge;
    // lanes past the end get d = rc, i.e. a zero filter, and the end sentinel r1 as receiver)
    int32_t en = min(e_lo + c32, e_hi - 1);
    float dv = A.d[en];
    int32_t rk = A.recv[en];
    int32_t sv = A.senders[en];
    {   // rows of the chunk before its first edge are empty
        const int32_t first = __builtin_amdgcn_readfirstlane(rk);
        for (int32_t r = (int32_t)r0; r < first; ++r) store_row(r, 0.f);
    }
    for (int32_t tb = e_lo; tb < e_hi; tb += 32) {
        const bool valid = tb + c32 < e_hi;
        const int kmax = min(32, e_hi - tb);
        float b[8], db[8];
        radial_basis<false>(valid ? dv : C.bp.rc, C.bp, b, db);
        // sender rows of this tile: issued now, consumed after the MFMA chain.  An edge past the end gathers the
        // row of the item's last edge; its filter is zero.
        float gv[32];
        const int32_t so = sv * (F * 4);
#pragma unroll
        for (int k = 0; k < 32; ++k) gv[k] = buffer_load_f32(g_rsrc, f * 4, __builtin_amdgcn_readlane(so, k), 0);
        const int32_t rcur = valid ? rk : r_end;
        // next tile's edge records
        en = min(tb + 32 + c32, e_hi - 1);
        dv = A.d[en];
        rk = A.recv[en];
        sv = A.senders[en];
        __builtin_amdgcn_sched_barrier(0);
        f32x16 t[D::NB], w[D::NB];
        gemm_k8r<F>(W1, b, t, lane);
#pragma unroll
        for (int bb = 0; bb < D::NB; ++bb)
#pragma unroll
            for (int r = 0; r < 16; ++r) t[bb][r] = t[bb][r] * sigmoid_scaled(t[bb][r]);
        if (PREC == kPrecBf16)
            gemm_rl_bf16<F>(reinterpret_cast<const __bf16 *>(A2t), t, w, lane);
        else if (PREC == kPrecF16x3)
            gemm_rl_f16x3<F>(reinterpret_cast<const _Float16 *>(A2t), t, w, lane);
        else
            gemm_rl<F>(A2t, t, w, lane);
        regs_to_tile<F>(w, tile, lane);
        wave_lds_fence();
        __builtin_amdgcn_sched_barrier(0);  // keep the use of the prefetched receiver after the MFMA chain
        int32_t rnext;
        const int32_t nf = __builtin_amdgcn_readfirstlane(rk);
        const uint32_t ends = row_ends(rcur, (tb + 32 < e_hi) ? nf : r_end, valid, lane, rnext);
        float wv[32];
#pragma unroll
        for (int k = 0; k < 32; ++k) wv[k] = tile[k * D::FS + f];
        if (keep_w) {   // keep w_e for the reverse pass; rows past the end of the chunk fall outside the
                        // descriptor's range and are dropped by the hardware bounds check
            const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(
                A.wstore + (int64_t)tb * F, 0, kmax * (F * 4), kBufferFlags);
#pragma unroll
            for (int k = 0; k < 32; ++k)
                if (F == 64 || lane < F) buffer_store_f32_stream(wv[k], w_rsrc, f * 4, k * (F * 4));
        }
#pragma unroll
        for (int k = 0; k < 32; ++k) {
            acc = fmaf(wv[k], gv[k], acc);   // lanes past the end hold a zero filter
            if (ends & (1u << k)) {
                const int32_t row = __builtin_amdgcn_readlane(rcur, k);
                const int32_t nrow = __builtin_amdgcn_readlane(rnext, k);
                store_row(row, acc);
                acc = 0.f;
                for (int32_t r = row + 1; r < nrow; ++r) store_row(r, 0.f);   // empty rows in between
            }
        }
        wave_lds_fence();
        // retire the prefetched edge records here (they arrived long ago); a load left pending across
        // the loop edge would make the compiler wait for all loads, gathers included, at the top
        asm volatile("" : "+v"(dv), "+v"(rk), "+v"(sv));
    }
    }   // work items
    }   // partitions
}

// Reverse edge step.
//
// Phase 1 (lane = feature), 16 edges at a time, every edge of the rows:
//   gbar_i += w_e * abar_send(e)               (w_e read back from the forward pass's store)
//   and, for the "upper" edge of each edge / reverse-edge pair (the one with the smaller index),
//   wsym_e = abar_i * g_j + abar_j * g_i is queued in LDS together with the edge's length and the
//   two edge indices of the pair.
// Only owned rows are processed here.  A ghost row (abar_i = 0) holds lower edges only, so its pairs are
// queued from the owned rows' side, and its gbar comes from k_ghost_gbar.
// Phase 2 (lane = edge), whenever 32 pairs are queued: dE/dd of the pair,
//   sum_k (W2 wsym)_k * ds_k/dd,   ds_k/dd = SiLU'(t_k) * sum_n W1[n][k] db_n/dd,
//   on the MFMA units, written to both edges of the pair.  Both edges of a pair have the same length
//   and the same wsym, so the dense work runs once per pair instead of once per directed edge.
// Edges per step of the reverse kernel's phase 1 and wavefronts per block.  Three wavefronts per SIMD instead of two
// were tried twice and measured slower on the 1M-atom benchmark (14.1 - 14.8 ms per step as built): steps of 8 with a
// 32-slot queue in three 4-wave blocks per compute unit (154 registers): 16.2 ms, the per-step bookkeeping doubles and
// phase 2 runs on partly filled tiles; steps of 12 in one 12-wave block (168 registers, 4 of them spilled): 16.0 ms.
constexpr int kStep = 16;
constexpr int kBwdWaves = 4;
constexpr int kQueue = 31 + kStep + 1;   // queued pairs per wavefront: at most 31 pending + one step's new ones
// phase 2 runs once a further step could overflow the queue (and at the latest with 32 pairs queued)
constexpr int kQueueTrigger = (kQueue - kStep < 32) ? kQueue - kStep : 32;

template <int F>
__device__ inline void gemm_queue(const float *__restrict__ Ap, const float *row, f32x16 (&out)[Dims<F>::NB], int lane)
{
    // as gemm_lds, the B operand row of this lane's edge given directly (queue slot)
    constexpr int NB = Dims<F>::NB;
    constexpr int STEPS = NB * 4;
    const int h = lane >> 5;
#pragma unroll
    for (int bo = 0; bo < NB; ++bo)
#pragma unroll
        for (int r = 0; r < 16; ++r) out[bo][r] = 0.f;
    const float *bp = row + 4 * h;
    const float *ap = Ap + lane * 4;
    f32x4 bv = *reinterpret_cast<const f32x4 *>(bp);
    f32x4 av[NB];
#pragma unroll
    for (int bo = 0; bo < NB; ++bo) av[bo] = *reinterpret_cast<const f32x4 *>(ap + ((bo * NB) * 4) * 256);
#pragma unroll
    for (int st = 0; st < STEPS; ++st) {
        f32x4 bn = bv, an[NB];
#pragma unroll
        for (int bo = 0; bo < NB; ++bo) an[bo] = av[bo];
        if (st + 1 < STEPS) {
            const int bi = (st + 1) / 4, a = (st + 1) % 4;
            bn = *reinterpret_cast<const f32x4 *>(bp + 32 * bi + 8 * a);
#pragma unroll
            for (int bo = 0; bo < NB; ++bo)
                an[bo] = *reinterpret_cast<const f32x4 *>(ap + (((bo * NB + bi) * 4 + a)) * 256);
        }
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int bo = 0; bo < NB; ++bo)
                out[bo] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[bo][c], bv[c], out[bo], 0, 0, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, NB + 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 4 * NB, 0);
        bv = bn;
#pragma unroll
        for (int bo = 0; bo < NB; ++bo) av[bo] = an[bo];
    }
}

template <int F, int PREC>
__global__ void __launch_bounds__(kBwdWaves * 64, kBwdWaves == 4 ? 2 : 1) k_edge_bwd(EdgeBatch B)
{
    using D = Dims<F>;
    constexpr int FS = D::FS;
    constexpr int kRowBytes = F * 4;
    extern __shared__ float lds[];
    float *A2n = lds;
    float *A1l = A2n + D::PACKF;
    float *queues = A1l + D::PACK1;
    for (int i = threadIdx.x; i < (PREC == kPrecBf16 ? D::PACKF / 2 : D::PACKF); i += kBwdWaves * 64) A2n[i] = B.c.A2n[i];
    for (int i = threadIdx.x; i < D::PACK1; i += kBwdWaves * 64) A1l[i] = B.c.A1[i];
    __syncthreads();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int c32 = lane & 31;
    const int l16 = lane % kStep;   // lane's edge within a step
    const unsigned f = lane & (F - 1);
    // Queue of pairs, one per wavefront: slot s is LDS row s, floats [0, F) = wsym, then the upper
    // edge's index, the reverse edge's index and the edge length in the row's padding.  It carries
    // over from one work item to the next and is drained at the end of a partition.
    float *Q = queues + wave * (kQueue * FS);
    char *Qf = reinterpret_cast<char *>(Q + f);
    const EdgeCommon &C = B.c;
    const bool need_gbar = C.need_gbar != 0;
    int q_head = 0, q_count = 0;   // first queued slot, queued pairs
    int q_tail = 0;                // (q_head + q_count) % kQueue, the slot the next pair goes to

    const ItemRange items = edge_items(B.chunk_start[B.n], wave, kBwdWaves);
    int64_t item = items.first;
    for (int part = 0; part < B.n; ++part) {
    const int64_t part_end = min(items.end, B.chunk_start[part + 1]);
    if (item >= part_end) continue;
    const EdgeArgs A = B.s[part];
    const __amdgpu_buffer_rsrc_t g_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(A.g), 0, (int)(A.n_nodes * kRowBytes), kBufferFlags);
    const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(A.abar), 0, (int)(A.n_nodes * kRowBytes), kBufferFlags);
    const __amdgpu_buffer_rsrc_t o_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        A.out, 0, need_gbar ? (int)(A.n_rows * kRowBytes) : 0, kBufferFlags);   // gbar rows; nothing is stored without it
    auto store_row = [&](int32_t row, float v) {
        if (F == 64 || lane < F) buffer_store_f32(v, o_rsrc, f * 4, row * kRowBytes, 0);
    };
    // state of the current work item (edge indices fit 32 bits)
    int32_t r1 = 0, e_hi = 0;
    float acc = 0.f;

    // Phase 1 runs in steps of kStep edges through a software pipeline whose loads are all issued ahead of
    // their use: the edge records (sender, receiver, reverse edge, length) two steps ahead, the rows they
    // point to one step ahead.  Vector memory loads complete in order, so a stage may only contain loads
    // and address arithmetic; anything that consumes a loaded value belongs to a later stage.
    struct Ids {    // lane k (mod kStep) holds edge tb + k, clamped to the last edge of the work item
        int32_t sj, rk, mk;
        float dk;
    };
    struct Step {
        float av[kStep], gv[kStep], wv[kStep];   // abar / g rows of the senders, kept filter values
        float ai0, gi0, ai1, gi1;       // abar / g rows of the first and of the last edge's receiver
        int kmax;                       // valid edges in the step
        int32_t tb;
    };
    auto load_ids = [&](Ids &I, int32_t tb) {
        const int32_t e = min((int32_t)tb + l16, e_hi - 1);
        I.sj = A.senders[e];
        I.rk = A.recv[e];
        I.mk = A.mirror[e];
        I.dk = A.d[e];
    };
    auto load_step = [&](Step &S, const Ids &I, int32_t tb) {
        S.tb = tb;
        S.kmax = __builtin_amdgcn_readfirstlane(max(0, min(kStep, e_hi - tb)));   // (the clamp is a vector instruction)
        // A step past the end of the work item (kmax = 0) still issues its loads, from the clamped records:
        // every path through the pipeline then has the same number of loads in flight, which is what lets
        // the waits before the uses be partial ones.
        const int32_t sjo = I.sj * kRowBytes;
        const int32_t row0 = __builtin_amdgcn_readfirstlane(I.rk);
        const int32_t rowl = __builtin_amdgcn_readlane(I.rk, max(S.kmax - 1, 0));
        S.ai0 = buffer_load_f32(a_rsrc, f * 4, row0 * kRowBytes, 0);
        S.gi0 = buffer_load_f32(g_rsrc, f * 4, row0 * kRowBytes, 0);
        S.ai1 = buffer_load_f32(a_rsrc, f * 4, rowl * kRowBytes, 0);
        S.gi1 = buffer_load_f32(g_rsrc, f * 4, rowl * kRowBytes, 0);
        // w_e sits at the edge's own index (a range of zero bytes reads 0: without gbar no w is needed)
        const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(
            A.wstore + (need_gbar ? (int64_t)tb * F : 0), 0, need_gbar ? S.kmax * kRowBytes : 0, kBufferFlags);
#pragma unroll
        for (int k = 0; k < kStep; ++k) {
            const int32_t so = __builtin_amdgcn_readlane(sjo, k);
            S.av[k] = buffer_load_f32(a_rsrc, f * 4, so, 0);
            S.gv[k] = buffer_load_f32(g_rsrc, f * 4, so, 0);
            S.wv[k] = buffer_load_f32_stream(w_rsrc, f * 4, k * kRowBytes);   // 0 outside the descriptor's range
        }
    };
    // rn_first: receiver of the first edge of the following step (r1 after the last step)
    auto compute_step = [&](const Step &S, const Ids &I, int32_t rn_first) {
        if (S.kmax <= 0) return;
        const bool valid_l = l16 < S.kmax;
        const int32_t rk = valid_l ? I.rk : r1;
        const int32_t e_l = S.tb + l16;
        // wave-uniform masks: bit k = edge k ends its row / edge k is the upper edge of its pair
        const int32_t up = __shfl(rk, l16 + 1, 64);
        const int32_t rnext = (l16 == kStep - 1) ? rn_first : up;
        const uint32_t ends = (uint32_t)__ballot(valid_l && rnext != rk) & ((1u << kStep) - 1u);
        const bool upper_l = valid_l && I.mk > e_l;
        const uint32_t uppers = (uint32_t)__ballot(upper_l) & ((1u << kStep) - 1u);
        {   // records of the pairs queued by this step, all at once: slots follow q_tail in edge order
            int slot = q_tail + (int)__builtin_amdgcn_mbcnt_lo(uppers, 0u);   // upper edges before this lane's (lanes < kStep)
            slot -= (slot >= kQueue) ? kQueue : 0;
            if (upper_l && lane < kStep) {
                float *rec = Q + slot * FS + F;
                reinterpret_cast<int32_t *>(rec)[0] = e_l;
                reinterpret_cast<int32_t *>(rec)[1] = I.mk;
                rec[2] = I.dk;
            }
        }
        const int32_t row_last = __builtin_amdgcn_readlane(rk, S.kmax - 1);
        float ai = S.ai0, gi = S.gi0;
        int q_off = q_tail * (FS * 4);   // byte offset of the slot the next pair goes to
#pragma unroll
        for (int k = 0; k < kStep; ++k) {
            acc = fmaf(S.wv[k], S.av[k], acc);   // edges past the end contribute w = 0
            // wsym goes to the next free slot whether or not the edge is an upper one; only an upper edge
            // advances the slot, anything else is overwritten by the next edge
            *reinterpret_cast<float *>(Qf + q_off) = fmaf(ai, S.gv[k], S.av[k] * gi);
            q_off += (uppers & (1u << k)) ? FS * 4 : 0;
            q_off = (q_off == kQueue * FS * 4) ? 0 : q_off;
            if (ends & (1u << k)) {
                const int32_t rrow = __builtin_amdgcn_readlane(rk, k);
                const int32_t nrow = __builtin_amdgcn_readlane(rnext, k);
                store_row(rrow, acc);
                for (int32_t r = rrow + 1; r < nrow; ++r) store_row(r, 0.f);   // empty rows in between
                acc = 0.f;
                if (k + 1 < S.kmax) {   // the next row starts inside this step
                    ai = S.ai1;
                    gi = S.gi1;
                    if (nrow != row_last) {   // a third row inside one step (short rows): fetch it now
                        ai = buffer_load_f32(a_rsrc, f * 4, nrow * kRowBytes, 0);
                        gi = buffer_load_f32(g_rsrc, f * 4, nrow * kRowBytes, 0);
                        // complete the two loads here: left pending, they would make every later use of
                        // ai / gi, on the common path too, wait for all loads in flight
                        asm volatile("" : "+v"(ai), "+v"(gi));
                    }
                }
            }
        }
        const int n_new = __builtin_popcount(uppers);
        q_count += n_new;
        q_tail += n_new;
        q_tail -= (q_tail >= kQueue) ? kQueue : 0;
    };
    auto phase2 = [&]() {
        // ---------------- up to 32 queued pairs
        wave_lds_fence();
        const int nval = min(q_count, 32);
        int slot = q_head + c32;
        slot -= (slot >= kQueue) ? kQueue : 0;
        const bool valid = c32 < nval;
        const float *rec = Q + slot * FS + F;
        const int32_t e_q = reinterpret_cast<const int32_t *>(rec)[0];
        const int32_t m_q = reinterpret_cast<const int32_t *>(rec)[1];
        const float d_q = rec[2];
        const int32_t e2 = valid ? e_q : 0, m2 = valid ? m_q : 0;
        const float d2 = valid ? d_q : C.bp.rc;   // rc: zero derivative
        float b[8], db[8];
        radial_basis<true>(d2, C.bp, b, db);
#pragma unroll
        for (int n = 0; n < 8; ++n) b[n] *= kSiluScale;   // pre-activations come out as t' = c t
        f32x16 t[D::NB];   // ds_k/dd = SiLU'(t_k) c_k, one block of 32 features at a time (fewer live registers)
#pragma unroll
        for (int bb = 0; bb < D::NB; ++bb) {
            f32x16 cg;
            RegPack1<F> W1;   // this block's W1 operands, from LDS
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) W1.v[bb][s4] = A1l[(bb * 4 + s4) * 64 + lane];
            gemm_k8r_block<F>(W1, b, bb, t[bb], lane);
            gemm_k8r_block<F>(W1, db, bb, cg, lane);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float sg = sigmoid_scaled(t[bb][r]);
                const float ss = t[bb][r] * sg * kSiluScaleInv;               // SiLU(t)
                t[bb][r] = fmaf(ss, 1.0f - sg, sg) * cg[r];
            }
        }
        f32x16 sb[D::NB];
        if (PREC == kPrecBf16)   // sbar[k] = sum_f W2[k][f] wsym[f]
            gemm_row_bf16<F>(reinterpret_cast<const __bf16 *>(A2n), Q + slot * FS, sb, lane);
        else if (PREC == kPrecF16x3)
            gemm_row_f16x3<F>(reinterpret_cast<const _Float16 *>(A2n), Q + slot * FS, sb, lane);
        else
            gemm_queue<F>(A2n, Q + slot * FS, sb, lane);
        float part = 0.f;
#pragma unroll
        for (int bb = 0; bb < D::NB; ++bb)
#pragma unroll
            for (int r = 0; r < 16; ++r) part = fmaf(sb[bb][r], t[bb][r], part);
        part += __shfl_xor(part, 32, 64);
        if (valid && lane < 32) {
            // every edge is written by exactly one pair per launch; after the first layer the value is
            // added with a fire-and-forget atomic so that no load sits in the pipeline of phase 1
            if (C.first) {
                A.dsum[e2] = part;
                A.dsum[m2] = part;
            } else {
                unsafeAtomicAdd(A.dsum + e2, part);
                unsafeAtomicAdd(A.dsum + m2, part);
            }
        }
        q_head += nval;
        q_head -= (q_head >= kQueue) ? kQueue : 0;
        q_count -= nval;
        wave_lds_fence();
    };

    for (; item < part_end; item += items.stride) {
        const int64_t chunk = item - B.chunk_start[part];
        int64_t r0_, r1_;
        if (!chunk_rows(A, chunk, r0_, r1_)) continue;
        const int32_t r0 = (int32_t)r0_;
        r1 = (int32_t)r1_;
        const int32_t e_lo = __builtin_amdgcn_readfirstlane((int32_t)A.row_ptr[r0]);   // wave-uniform: keep them scalar
        e_hi = __builtin_amdgcn_readfirstlane((int32_t)A.row_ptr[r1]);
        acc = 0.f;
        if (e_lo >= e_hi) {   // only empty rows
            for (int32_t r = r0; r < r1; ++r) store_row(r, 0.f);
            continue;
        }
        Ids IA, IB, IC;
        Step SA, SB;
        load_ids(IA, e_lo);
        load_ids(IB, e_lo + kStep);
        {   // rows of the chunk before its first edge are empty
            const int32_t first = __builtin_amdgcn_readfirstlane(IA.rk);
            for (int32_t r = r0; r < first; ++r) store_row(r, 0.f);
        }
        load_step(SA, IA, e_lo);
        for (int32_t tb = e_lo; tb < e_hi; tb += 2 * kStep) {
            int32_t nf;
            load_ids(IC, tb + 2 * kStep);
            load_step(SB, IB, tb + kStep);
            nf = __builtin_amdgcn_readfirstlane(IB.rk);
            compute_step(SA, IA, (tb + kStep < e_hi) ? nf : r1);
            if (q_count >= kQueueTrigger) phase2();
            load_ids(IA, tb + 3 * kStep);
            load_step(SA, IC, tb + 2 * kStep);
            nf = __builtin_amdgcn_readfirstlane(IC.rk);
            compute_step(SB, IB, (tb + 2 * kStep < e_hi) ? nf : r1);
            if (q_count >= kQueueTrigger) phase2();
            IB = IA;   // records of step tb + 3 kStep, loaded a step ago
            IA = IC;   // records of step tb + 2 kStep, whose rows SA holds
        }
    }   // work items
    while (q_count > 0) phase2();   // queued pairs index this partition's arrays
    }   // partitions
}

// ---------------------------------------------------------------- node kernels

enum { OP_PROJ = 0, OP_UPDATE = 1, OP_READOUT = 2, OP_BWD_UPDATE = 3, OP_BWD_PROJ = 4 };

struct NodeArgs {      // one partition
    int64_t n_rows;
    const float *X;    // GEMM input rows
    float *Y;          // primary output rows
    float *Z;          // secondary in/out rows (h for UPDATE, hbar for BWD_*)
    float *eps;
};

struct NodeBatch {     // up to kBatch partitions per launch, 32-row tiles numbered across them
    const float *P1, *P2;
    const float *wr2;
    int n;
    int64_t tile_start[kBatch + 1];
    NodeArgs s[kBatch];
};

// A 32-row tile of X travels global memory -> registers -> LDS in two halves, so that the loads of the next
// tile can be in flight while the current one is multiplied.
template <int F> struct TileRegs {
    static constexpr int LPR = F / 4;        // lanes per row (float4 each)
    static constexpr int RPI = 64 / LPR;     // rows per wave instruction
    f32x4 v[32 / RPI];
};

template <int F>
__device__ inline void fetch_tile(TileRegs<F> &T, const float *__restrict__ X, int64_t row0, int64_t n_rows, int lane)
{
    constexpr int LPR = TileRegs<F>::LPR, RPI = TileRegs<F>::RPI;
    const int rr = lane / LPR, cc = (lane % LPR) * 4;
#pragma unroll
    for (int r = 0; r < 32; r += RPI) {
        const int64_t row = row0 + r + rr;
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (row < n_rows) v = *reinterpret_cast<const f32x4 *>(X + row * F + cc);
        T.v[r / RPI] = v;
    }
}

template <int F> __device__ inline void stash_tile(const TileRegs<F> &T, float *tile, int lane)
{
    constexpr int FS = Dims<F>::FS;
    constexpr int LPR = TileRegs<F>::LPR, RPI = TileRegs<F>::RPI;
    const int rr = lane / LPR, cc = (lane % LPR) * 4;
#pragma unroll
    for (int r = 0; r < 32; r += RPI) *reinterpret_cast<f32x4 *>(tile + (r + rr) * FS + cc) = T.v[r / RPI];
}

template <int F, int OP>
__global__ void __launch_bounds__(256) k_node(NodeBatch B)
{
    using D = Dims<F>;
    constexpr bool TWO = (OP == OP_READOUT || OP == OP_BWD_UPDATE);
    extern __shared__ float lds[];
    float *P1 = lds;
    float *P2 = P1 + D::PACKF;
    float *tiles = P2 + (TWO ? D::PACKF : 0);
    for (int i = threadIdx.x; i < D::PACKF; i += 256) {
        P1[i] = B.P1[i];
        if (TWO) P2[i] = B.P2[i];
    }
    __syncthreads();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int c32 = lane & 31, h = lane >> 5;
    float *tile = tiles + wave * D::TILE;
    const int64_t n_tiles = B.tile_start[B.n];
    const int64_t stride = (int64_t)gridDim.x * 4;
    TileRegs<F> pre;
    auto fetch = [&](int64_t ti) {
        const int part = batch_find(B.tile_start, B.n, ti);
        fetch_tile<F>(pre, B.s[part].X, (ti - B.tile_start[part]) * 32, B.s[part].n_rows, lane);
    };
    int64_t ti = (int64_t)blockIdx.x * 4 + wave;
    if (ti < n_tiles) fetch(ti);
    for (; ti < n_tiles; ti += stride) {
        const int part = batch_find(B.tile_start, B.n, ti);
        const NodeArgs A = B.s[part];
        const int64_t row0 = (ti - B.tile_start[part]) * 32;
        const int64_t row = row0 + c32;
        const bool ok = row < A.n_rows;
        stash_tile<F>(pre, tile, lane);
        wave_lds_fence();
        // rows of Z this tile combines with its product, requested before the product as well
        constexpr bool READS_Z = (OP == OP_UPDATE || OP == OP_BWD_PROJ || OP == OP_BWD_UPDATE);
        f32x4 zv[D::NB][4];
        if (READS_Z)
#pragma unroll
            for (int b = 0; b < D::NB; ++b)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    zv[b][a] = f32x4{0.f, 0.f, 0.f, 0.f};
                    if (ok) zv[b][a] = *reinterpret_cast<const f32x4 *>(A.Z + row * F + 32 * b + 8 * a + 4 * h);
                }
        if (ti + stride < n_tiles) fetch(ti + stride);   // in flight during this tile's products
        f32x16 acc[D::NB];
        gemm_lds<F>(P1, tile, acc, lane);
        wave_lds_fence();
        if (OP == OP_PROJ) {
            if (ok)
#pragma unroll
                for (int b = 0; b < D::NB; ++b)
#pragma unroll
                    for (int a = 0; a < 4; ++a) {
                        f32x4 v = {acc[b][4 * a], acc[b][4 * a + 1], acc[b][4 * a + 2], acc[b][4 * a + 3]};
                        *reinterpret_cast<f32x4 *>(A.Y + row * F + 32 * b + 8 * a + 4 * h) = v;
                    }
        } else if (OP == OP_UPDATE || OP == OP_BWD_PROJ) {
            // UPDATE:   Z = h,    h    += SiLU(a Wo)
            // BWD_PROJ: Z = hbar, hbar += gbar Wm^T
            if (ok)
#pragma unroll
                for (int b = 0; b < D::NB; ++b)
#pragma unroll
                    for (int a = 0; a < 4; ++a) {
                        float *zp = A.Z + row * F + 32 * b + 8 * a + 4 * h;
                        f32x4 v = zv[b][a];
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            const float q = acc[b][4 * a + c];
                            v[c] += (OP == OP_UPDATE) ? q * sigmoidf_fast(q) : q;
                        }
                        *reinterpret_cast<f32x4 *>(zp) = v;
                    }
        } else if (OP == OP_READOUT) {
            // eps = SiLU(h Wr1) . wr2 ;  hbar = (wr2 * SiLU'(h Wr1)) Wr1^T
            float part = 0.f;
#pragma unroll
            for (int b = 0; b < D::NB; ++b)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const f32x4 wv = *reinterpret_cast<const f32x4 *>(B.wr2 + 32 * b + 8 * a + 4 * h);
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const float x = acc[b][4 * a + c];
                        const float sg = sigmoidf_fast(x);
                        part += x * sg * wv[c];
                        acc[b][4 * a + c] = wv[c] * sg * (1.0f + x * (1.0f - sg));
                    }
                }
            part += __shfl_xor(part, 32, 64);
            if (ok && h == 0) A.eps[row] = part;
            f32x16 hb[D::NB];
            gemm_regs<F>(P2, acc, hb, lane);
            if (ok)
#pragma unroll
                for (int b = 0; b < D::NB; ++b)
#pragma unroll
                    for (int a = 0; a < 4; ++a) {
                        f32x4 v = {hb[b][4 * a], hb[b][4 * a + 1], hb[b][4 * a + 2], hb[b][4 * a + 3]};
                        *reinterpret_cast<f32x4 *>(A.Y + row * F + 32 * b + 8 * a + 4 * h) = v;
                    }
        } else if (OP == OP_BWD_UPDATE) {
            // q = a Wo ; qbar = hbar * SiLU'(q) ; abar = qbar Wo^T       (X = a, Z = hbar, Y = abar)
#pragma unroll
            for (int b = 0; b < D::NB; ++b)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const f32x4 hv = zv[b][a];
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const float x = acc[b][4 * a + c];
                        const float sg = sigmoidf_fast(x);
                        acc[b][4 * a + c] = hv[c] * sg * (1.0f + x * (1.0f - sg));
                    }
                }
            f32x16 ab[D::NB];
            gemm_regs<F>(P2, acc, ab, lane);
            if (ok)
#pragma unroll
                for (int b = 0; b < D::NB; ++b)
#pragma unroll
                    for (int a = 0; a < 4; ++a) {
                        f32x4 v = {ab[b][4 * a], ab[b][4 * a + 1], ab[b][4 * a + 2], ab[b][4 * a + 3]};
                        *reinterpret_cast<f32x4 *>(A.Y + row * F + 32 * b + 8 * a + 4 * h) = v;
                    }
        }
    }
}

// ---------------------------------------------------------------- small kernels

__global__ void k_embed(int64_t n_rows, int F, const int32_t *__restrict__ nodes, const int32_t *__restrict__ species,
                        const float *__restrict__ emb, float *__restrict__ h)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n_rows * F) return;
    const int64_t r = idx / F;
    const int f = (int)(idx % F);
    const int64_t u = nodes ? nodes[r] : r;
    h[idx] = emb[species[u] * F + f];
}

struct PtrTable { float *p[kMaxSlabs]; };

// ghost rows of this partition's g  <-  the owners' rows
__global__ void k_ghost_copy(int64_t n_ghost, int64_t n_owned, int F, const int32_t *__restrict__ owner,
                             const int32_t *__restrict__ src, PtrTable tab, float *__restrict__ dst)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int F4 = F / 4;
    if (idx >= n_ghost * F4) return;
    const int64_t k = idx / F4;
    const int c = (int)(idx % F4) * 4;
    const float *sp = tab.p[owner[k]] + (int64_t)src[k] * F + c;
    *reinterpret_cast<f32x4 *>(dst + (n_owned + k) * F + c) = *reinterpret_cast<const f32x4 *>(sp);
}

// the owners' gradient rows  +=  this partition's ghost rows (each ghost atom appears once per partition)
// gbar of the ghost rows: gbar_i = sum over the ghost's sub-row (its neighbours owned by this partition) of
// w_e * abar_send(e).  w_e is the reverse edge's, which the forward pass kept (both edges of a pair have the
// same length, hence the same filter value).  One wavefront per row, lane = feature, edges in row order.
template <int F>
__global__ void __launch_bounds__(256)
k_ghost_gbar(int64_t n_ghost, int64_t n_owned, const int64_t *__restrict__ row_ptr, const int32_t *__restrict__ senders,
             const int32_t *__restrict__ mirror, const float *__restrict__ wstore, const float *__restrict__ abar,
             const int32_t *__restrict__ bond_of_edge, const float *__restrict__ wb, float *__restrict__ gbar)
{
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int64_t k = (int64_t)blockIdx.x * 4 + wave;
    if (k >= n_ghost) return;
    const int64_t r = n_owned + k;
    const unsigned f = lane & (F - 1);
    const int64_t e0 = row_ptr[r], e1 = row_ptr[r + 1];
    float acc = 0.f;
    for (int64_t eb = e0; eb < e1; eb += 16) {   // 16 edges at a time: ids by lane, then all rows in flight together
        const int n = (int)min((int64_t)16, e1 - eb);
        const int64_t el = min(eb + (lane & 15), e1 - 1);
        const int32_t jl = senders[el], ml = mirror[el];
        const int32_t bl = bond_of_edge ? bond_of_edge[ml] : -1;   // three-body variant: the reverse edge's bond
        float wv[16], av[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const int64_t j = __builtin_amdgcn_readlane(jl, k), m = __builtin_amdgcn_readlane(ml, k);
            const int64_t b = __builtin_amdgcn_readlane(bl, k);
            wv[k] = wstore[m * F + f];
            if (b >= 0) wv[k] += wb[b * F + f];
            av[k] = abar[j * F + f];
        }
#pragma unroll
        for (int k = 0; k < 16; ++k)
            if (k < n) acc = fmaf(wv[k], av[k], acc);
    }
    if (F == 64 || lane < F) gbar[r * F + f] = acc;
}

// Three-body variant, ghost rows: a ghost atom i is the sender of bonds (j <- i) held by this partition; each pulls
// on it with +dE/dDelta.  Gathered over the ghost's sub-row through the reverse edges.
__global__ void k_bond_force_ghost(int64_t n_ghost, int64_t n_owned, const int64_t *__restrict__ row_ptr,
                                   const int32_t *__restrict__ mirror, const int32_t *__restrict__ bond_of_edge,
                                   const float *__restrict__ dbond, const float *__restrict__ rbar,
                                   const float *__restrict__ rhat, const float *__restrict__ bd, float *floc)
{
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= n_ghost) return;
    const int64_t r = n_owned + k;
    float fx = 0.f, fy = 0.f, fz = 0.f;
    for (int64_t e = row_ptr[r]; e < row_ptr[r + 1]; ++e) {
        const int64_t q = bond_of_edge[mirror[e]];
        if (q < 0) continue;
        const float x = rhat[3 * q], y = rhat[3 * q + 1], z = rhat[3 * q + 2];
        const float ax = rbar[3 * q], ay = rbar[3 * q + 1], az = rbar[3 * q + 2];
        const float dot = fmaf(ax, x, fmaf(ay, y, az * z));
        const float inv = 1.0f / bd[q];
        fx -= fmaf(dbond[q], x, (ax - dot * x) * inv);
        fy -= fmaf(dbond[q], y, (ay - dot * y) * inv);
        fz -= fmaf(dbond[q], z, (az - dot * z) * inv);
    }
    floc[3 * r] += fx;
    floc[3 * r + 1] += fy;
    floc[3 * r + 2] += fz;
}

__global__ void k_ghost_addback(int64_t n_ghost, int64_t n_owned, int F, const int32_t *__restrict__ owner,
                                const int32_t *__restrict__ src, PtrTable tab, const float *__restrict__ mine)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int F4 = F / 4;
    if (idx >= n_ghost * F4) return;
    const int64_t k = idx / F4;
    const int c = (int)(idx % F4) * 4;
    float *dp = tab.p[owner[k]] + (int64_t)src[k] * F + c;
    f32x4 v = *reinterpret_cast<const f32x4 *>(dp);
    const f32x4 m = *reinterpret_cast<const f32x4 *>(mine + (n_owned + k) * F + c);
    v += m;
    *reinterpret_cast<f32x4 *>(dp) = v;
}

__device__ inline void unpack_shift(uint32_t p, int &a, int &b, int &c)
{
    a = (int)(p >> 20) - 512;
    b = (int)((p >> 10) & 1023u) - 512;
    c = (int)(p & 1023u) - 512;
}

// F_loc[r] = sum_{e in local row r} dsum_e * rhat_e, rhat from fp64 positions; 16 lanes per row, 16 rows per block
__global__ void __launch_bounds__(256)
k_force_rows(int64_t n_rows, const int64_t *__restrict__ row_ptr, const int32_t *__restrict__ senders,
             const uint32_t *__restrict__ shiftp, const float *__restrict__ dsum, const int32_t *__restrict__ nodes,
             const double *__restrict__ pos, CellParams cp, float *__restrict__ floc)
{
    const int64_t r = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
    if (r >= n_rows) return;   // whole groups of 16 lanes leave together; the shuffles below stay inside a group
    const int64_t ig = nodes ? nodes[r] : r;
    const double xi = pos[3 * ig], yi = pos[3 * ig + 1], zi = pos[3 * ig + 2];
    double fx = 0, fy = 0, fz = 0;
    const int64_t e1 = row_ptr[r + 1];
    for (int64_t e = row_ptr[r] + (threadIdx.x & 15); e < e1; e += 16) {
        const int64_t jl = senders[e];
        const int64_t jg = nodes ? nodes[jl] : jl;
        int S0, S1, S2;
        unpack_shift(shiftp[e], S0, S1, S2);
        const double t0 = (pos[3 * jg] - xi) + (((double)S0 * cp.C[0] + (double)S1 * cp.C[3]) + (double)S2 * cp.C[6]);
        const double t1 = (pos[3 * jg + 1] - yi) + (((double)S0 * cp.C[1] + (double)S1 * cp.C[4]) + (double)S2 * cp.C[7]);
        const double t2 = (pos[3 * jg + 2] - zi) + (((double)S0 * cp.C[2] + (double)S1 * cp.C[5]) + (double)S2 * cp.C[8]);
        const double s = (double)dsum[e] / sqrt((t0 * t0 + t1 * t1) + t2 * t2);
        fx += s * t0;
        fy += s * t1;
        fz += s * t2;
    }
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) {
        fx += __shfl_xor(fx, off, 64);
        fy += __shfl_xor(fy, off, 64);
        fz += __shfl_xor(fz, off, 64);
    }
    if ((threadIdx.x & 15) == 0) {
        floc[3 * r] = (float)fx;
        floc[3 * r + 1] = (float)fy;
        floc[3 * r + 2] = (float)fz;
    }
}

// owned rows: forces[global] = F_loc ; atom_energy[global] = eps
__global__ void k_store_owned(int64_t n_owned, const int32_t *__restrict__ nodes, const float *__restrict__ floc,
                              const float *__restrict__ eps, float *__restrict__ forces, float *__restrict__ atom_energy)
{
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= n_owned) return;
    const int64_t u = nodes ? nodes[r] : r;
    forces[3 * u] = floc[3 * r];
    forces[3 * u + 1] = floc[3 * r + 1];
    forces[3 * u + 2] = floc[3 * r + 2];
    if (atom_energy) atom_energy[u] = eps[r];
}

// ghost rows: forces[global] += F_loc (position gradients of ghost atoms go back to their owners)
__global__ void k_addback_ghost_forces(int64_t n_ghost, int64_t n_owned, const int32_t *__restrict__ nodes,
                                       const float *__restrict__ floc, float *__restrict__ forces)
{
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= n_ghost) return;
    const int64_t r = n_owned + k;
    const int64_t u = nodes[r];
    forces[3 * u] += floc[3 * r];
    forces[3 * u + 1] += floc[3 * r + 1];
    forces[3 * u + 2] += floc[3 * r + 2];
}

// fixed-shape fp64 reduction of the per-atom energies: 1024-element blocks, then one block over the partials
__global__ void __launch_bounds__(256) k_energy_partial(int64_t n, const float *__restrict__ eps, double *__restrict__ part)
{
    __shared__ double sh[4];
    const int64_t base = (int64_t)blockIdx.x * 1024;
    double s = 0;
    for (int k = threadIdx.x; k < 1024; k += 256)
        if (base + k < n) s += (double)eps[base + k];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) part[blockIdx.x] = (sh[0] + sh[1]) + (sh[2] + sh[3]);
}

__global__ void __launch_bounds__(256) k_energy_final(int64_t n, const double *__restrict__ part, double *__restrict__ energy)
{
    __shared__ double sh[4];
    double s = 0;
    for (int64_t k = threadIdx.x; k < n; k += 256) s += part[k];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) *energy = (sh[0] + sh[1]) + (sh[2] + sh[3]);
}

// ---------------------------------------------------------------- three-body (bond graph) kernels
//
// Benchmark configuration 4: bonds are the atom-graph edges within a smaller cutoff, two bonds interact when
// they share their centre atom (the paper's bond graph, Methods, "Distributing Bond Graphs").  All bonds of a
// centre are contiguous, so every kernel below works on one centre (or one bond) per wavefront with lane =
// feature and needs no atomics.  Notation: P_b = e0_b Wta, Q_b = e0_b Wtb, Wtc = rows 2F.. of Wt1,
//   h(b1, b2) = P_b1 + Q_b2 + T(c) Wtc,  S_b1 = sum_{b2 != b1} u_b2 SiLU(h),  m = S Wt2,  e1 = e0 + u SiLU(m).

constexpr int kAngle = 8;

__device__ inline float silu_f(float x) { return x * __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }
__device__ inline void silu_both(float x, float &s, float &ds)
{
    const float sg = __builtin_amdgcn_rcpf(1.0f + __expf(-x));
    s = x * sg;
    ds = sg * (1.0f + x * (1.0f - sg));
}

// value of lane k (wave-uniform k) of a float register, as a wave-uniform value
__device__ inline float readlane_f32(float v, int k)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), k));
}

// T_n(c) = cos(n theta), dT_n/dc = n U_{n-1}(c), n = 0..7
__device__ inline void chebyshev(float c, float (&T)[kAngle], float (&dT)[kAngle])
{
    T[0] = 1.f; dT[0] = 0.f;
    T[1] = c;   dT[1] = 1.f;
    float Um = 1.f, Un = 2.f * c;   // U_0, U_1
#pragma unroll
    for (int n = 2; n < kAngle; ++n) {
        T[n] = 2.f * c * T[n - 1] - T[n - 2];
        dT[n] = (float)n * Un;
        const float Ux = 2.f * c * Un - Um;
        Um = Un;
        Un = Ux;
    }
}

// S[b1][f] = sum_{b2 != b1, same centre} u[b2] SiLU(P[b1][f] + Q[b2][f] + sum_n T_n(c) Wtc[n][f])
// One wavefront per centre, lane = feature.  The angle basis does not depend on the feature: for a fixed b1 it is
// evaluated for 64 bonds b2 at once (lane = b2) and handed to the feature lanes through wave-uniform registers.
// Centres with at most kPairBondsFwd bonds are processed by unordered pairs {a, o}: T(c) Wtc is shared by the
// triplets (a, o) and (o, a); the term of bond a accumulates in a register, the term of bond o in a per-lane LDS row.
constexpr int kPairBondsFwd = 32;

template <int F>
__global__ void __launch_bounds__(256)
k_triplet_fwd(int64_t N, const int64_t *__restrict__ bptr, const float *__restrict__ rhat, const float *__restrict__ u,
              const float *__restrict__ P, const float *__restrict__ Q, const float *__restrict__ Wtc, float *__restrict__ S)
{
    constexpr int NB = kPairBondsFwd;
    __shared__ float acc_lds[4][NB * 64];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int64_t i = (int64_t)blockIdx.x * 4 + wave;
    if (i >= N) return;
    const int f = lane & (F - 1);
    float wc[kAngle];
#pragma unroll
    for (int n = 0; n < kAngle; ++n) wc[n] = Wtc[n * F + f];
    const int64_t b0 = bptr[i], b1e = bptr[i + 1];
    const int nb = (int)(b1e - b0);
    if (nb <= 0) return;
    if (nb <= NB) {
        float *accS = acc_lds[wave];
        for (int b = 0; b < nb; ++b) accS[b * 64 + lane] = 0.f;
        const int64_t bl = min(b0 + lane, b1e - 1);
        const float xl = rhat[3 * bl], yl = rhat[3 * bl + 1], zl = rhat[3 * bl + 2], ul = u[bl];   // lane = bond
        for (int a = 0; a < nb; ++a) {
            const int64_t ba = b0 + a;
            const float pa = P[ba * F + f], qa = Q[ba * F + f];
            const float ua = readlane_f32(ul, a);
            float T[kAngle], dT[kAngle];
            chebyshev(fmaf(readlane_f32(xl, a), xl, fmaf(readlane_f32(yl, a), yl, readlane_f32(zl, a) * zl)), T, dT);   // lane = o
            float acc = 0.f;
            for (int o = a + 1; o < nb; ++o) {
                float tw = wc[0];   // T_0 = 1
#pragma unroll
                for (int n = 1; n < kAngle; ++n) tw = fmaf(readlane_f32(T[n], o), wc[n], tw);
                const float po = P[(b0 + o) * F + f], qo = Q[(b0 + o) * F + f];
                const float so = accS[o * 64 + lane];   // per-lane slot (read early, written at the end of the step;
                                                        // LDS float atomics measured an order of magnitude slower)
                acc = fmaf(readlane_f32(ul, o), silu_f(pa + qo + tw), acc);       // triplet (b1 = a, b2 = o)
                accS[o * 64 + lane] = fmaf(ua, silu_f(po + qa + tw), so);        // triplet (b1 = o, b2 = a)
            }
            accS[a * 64 + lane] += acc;
        }
        wave_lds_fence();
        if (F == 64 || lane < F)
            for (int b = 0; b < nb; ++b) S[(b0 + b) * F + f] = accS[b * 64 + lane];
        return;
    }
    // any number of bonds, no LDS: ordered pairs, bonds b2 in groups of 64
    for (int64_t c0 = b0; c0 < b1e; c0 += 64) {   // bonds b2 in groups of 64 (one group unless the centre has more)
        const int nl = (int)min((int64_t)64, b1e - c0);
        const int64_t bl = min(c0 + lane, b1e - 1);
        const float xl = rhat[3 * bl], yl = rhat[3 * bl + 1], zl = rhat[3 * bl + 2], ul = u[bl];
        for (int64_t b1 = b0; b1 < b1e; ++b1) {
            const float p1 = P[b1 * F + f];
            const float x1 = rhat[3 * b1], y1 = rhat[3 * b1 + 1], z1 = rhat[3 * b1 + 2];
            float T[kAngle], dT[kAngle];
            chebyshev(fmaf(x1, xl, fmaf(y1, yl, z1 * zl)), T, dT);   // lane = b2
            float acc = 0.f;
            for (int k = 0; k < nl; ++k) {
                if (c0 + k == b1) continue;
                float h = p1 + Q[(c0 + k) * F + f];
#pragma unroll
                for (int n = 1; n < kAngle; ++n) h = fmaf(readlane_f32(T[n], k), wc[n], h);   // T_0 = 1
                acc = fmaf(readlane_f32(ul, k), silu_f(h + wc[0]), acc);
            }
            if (F == 64 || lane < F) {
                float *sp = S + b1 * F + f;
                *sp = (c0 == b0) ? acc : *sp + acc;
            }
        }
    }
}

// bond term of a layer's aggregation: a[i] += sum over the bonds b = (i <- j) of wb[b] * g[j]
template <int F>
__global__ void __launch_bounds__(256)
k_bond_aggregate(int64_t N, const int64_t *__restrict__ bptr, const int32_t *__restrict__ sender,
                 const float *__restrict__ wb, const float *__restrict__ g, float *__restrict__ a)
{
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int64_t i = (int64_t)blockIdx.x * 4 + wave;
    if (i >= N) return;
    const int f = lane & (F - 1);
    float acc = 0.f;
    for (int64_t b = bptr[i]; b < bptr[i + 1]; ++b) acc = fmaf(wb[b * F + f], g[(int64_t)sender[b] * F + f], acc);
    if (F == 64 || lane < F) a[i * F + f] += acc;
}

// reverse of the bond term, the share of gbar: gbar[i] += sum_b wb[mirror(b)] * abar[j]
// (the reverse bond (j <- i) is the one whose filter multiplies g_i in row j)
template <int F>
__global__ void __launch_bounds__(256)
k_bond_gbar(int64_t N, const int64_t *__restrict__ bptr, const int32_t *__restrict__ sender,
            const int32_t *__restrict__ bmirror, const float *__restrict__ wb, const float *__restrict__ abar,
            float *gbar)
{
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int64_t i = (int64_t)blockIdx.x * 4 + wave;
    if (i >= N) return;
    const int f = lane & (F - 1);
    float acc = 0.f;
    for (int64_t b = bptr[i]; b < bptr[i + 1]; ++b) {
        const int64_t j = sender[b];
        const int64_t bm = bmirror[b];   // -1: the sender is a ghost row (abar_j = 0 here, its owner adds that term)
        if (bm >= 0) acc = fmaf(wb[bm * F + f], abar[j * F + f], acc);
    }
    if (F == 64 || lane < F) gbar[i * F + f] += acc;
}

// sum over the 64 lanes of a wavefront on the data-parallel-primitive path (no LDS); the total is returned
// as a wave-uniform value
template <int CTRL, int ROW_MASK, bool BOUND> __device__ inline float dpp_shifted(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xf, BOUND));
}
__device__ inline float wave_sum(float v)
{
    v += dpp_shifted<0x111, 0xf, true>(v);    // row_shr:1  (lanes shifted in from outside a row of 16 read 0)
    v += dpp_shifted<0x112, 0xf, true>(v);    // row_shr:2
    v += dpp_shifted<0x114, 0xf, true>(v);    // row_shr:4
    v += dpp_shifted<0x118, 0xf, true>(v);    // row_shr:8: lane 15 of every row holds the row's sum
    v += dpp_shifted<0x142, 0xa, false>(v);   // row_bcast:15 into rows 1 and 3
    v += dpp_shifted<0x143, 0xc, false>(v);   // row_bcast:31 into rows 2 and 3: lane 63 holds the total
    return readlane_f32(v, 63);
}

// Reverse of k_triplet_fwd for one centre, any number of bonds, no LDS.  Pbar[b1] and rbar[b1] accumulate over the
// inner loop in registers; Qbar[b2], ubar[b2] and rbar[b2] are indexed by the inner bond, so they are accumulated
// in a second sweep with the roles of the loops exchanged (h is recomputed there): every triplet is evaluated twice.
template <int F>
__device__ inline void
triplet_bwd_sweep(int64_t i, int lane, const int64_t *__restrict__ bptr, const float *__restrict__ rhat,
                  const float *__restrict__ u, const float *__restrict__ P, const float *__restrict__ Q,
                  const float *__restrict__ Wtc, const float *__restrict__ Sbar, float *__restrict__ Pbar,
                  float *__restrict__ Qbar, float *__restrict__ ubar, float *__restrict__ rbar)
{
    const int f = lane & (F - 1);
    const bool on = (F == 64 || lane < F);
    float wc[kAngle];
#pragma unroll
    for (int n = 0; n < kAngle; ++n) wc[n] = Wtc[n * F + f];
    const int64_t b0 = bptr[i], be = bptr[i + 1];
    for (int64_t ba = b0; ba < be; ++ba) {
        const float xa = rhat[3 * ba], ya = rhat[3 * ba + 1], za = rhat[3 * ba + 2];
        const float pa = P[ba * F + f], qa = Q[ba * F + f], sa = Sbar[ba * F + f], ua = u[ba];
        float pbar = 0.f, qbar = 0.f, ub = 0.f, rx = 0.f, ry = 0.f, rz = 0.f;
        for (int64_t bo = b0; bo < be; ++bo) {
            if (bo == ba) continue;
            const float xo = rhat[3 * bo], yo = rhat[3 * bo + 1], zo = rhat[3 * bo + 2];
            const float c = fmaf(xa, xo, fmaf(ya, yo, za * zo));
            float T[kAngle], dT[kAngle];
            chebyshev(c, T, dT);
            float tw = 0.f, dw = 0.f;   // T(c) Wtc and dT(c)/dc Wtc for this lane's feature
#pragma unroll
            for (int n = 0; n < kAngle; ++n) {
                tw = fmaf(T[n], wc[n], tw);
                dw = fmaf(dT[n], wc[n], dw);
            }
            // triplet (b1 = ba, b2 = bo): contributes to Pbar[ba] and, through c, to rbar[ba]
            float s1, ds1;
            silu_both(pa + Q[bo * F + f] + tw, s1, ds1);
            const float h1 = sa * u[bo] * ds1;
            pbar += h1;
            // triplet (b1 = bo, b2 = ba): contributes to Qbar[ba], ubar[ba] and, through c, to rbar[ba]
            float s2, ds2;
            const float so = Sbar[bo * F + f];
            silu_both(P[bo * F + f] + qa + tw, s2, ds2);
            const float h2 = so * ua * ds2;
            qbar += h2;
            ub = fmaf(so, s2, ub);
            const float dc = on ? (h1 + h2) * dw : 0.f;   // this lane's share of dE/dc from both triplets
            rx = fmaf(dc, xo, rx);
            ry = fmaf(dc, yo, ry);
            rz = fmaf(dc, zo, rz);
        }
        if (!on) ub = 0.f;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            ub += __shfl_xor(ub, off, 64);
            rx += __shfl_xor(rx, off, 64);
            ry += __shfl_xor(ry, off, 64);
            rz += __shfl_xor(rz, off, 64);
        }
        if (on) {
            Pbar[ba * F + f] = pbar;
            Qbar[ba * F + f] = qbar;
        }
        if (lane == 0) {
            ubar[ba] += ub;
            rbar[3 * ba] = rx;
            rbar[3 * ba + 1] = ry;
            rbar[3 * ba + 2] = rz;
        }
    }
}


constexpr int kPairBonds = 16;   // bonds per centre up to which the pair-wise reverse triplet kernel applies

// Reverse of k_triplet_fwd, one centre per wavefront, lane = feature.  Centres with at most kPairBonds bonds
// (12 on the benchmark's lattice) are processed by unordered pairs {a, o}: the angle terms T(c) Wtc and
// dT/dc Wtc are shared by the triplets (a, o) and (o, a), and each triplet is evaluated once.  What a pair
// contributes to bond a stays in registers; what it contributes to bond o goes to per-lane accumulators in LDS
// (rows accP, accQ, accU of 64 floats per bond), and dE/dc of the pair, reduced over the features, into a small
// table from which rbar is assembled at the end with lane = bond.
template <int F>
__global__ void __launch_bounds__(256)
k_triplet_bwd(int64_t N, const int64_t *__restrict__ bptr, const float *__restrict__ rhat, const float *__restrict__ u,
              const float *__restrict__ P, const float *__restrict__ Q, const float *__restrict__ Wtc,
              const float *__restrict__ Sbar, float *__restrict__ Pbar, float *__restrict__ Qbar,
              float *__restrict__ ubar, float *__restrict__ rbar)
{
    constexpr int NB = kPairBonds;
    __shared__ float acc_lds[4][3 * NB * 64 + NB * NB];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int64_t i = (int64_t)blockIdx.x * 4 + wave;
    if (i >= N) return;
    const int64_t b0 = bptr[i];
    const int n = (int)(bptr[i + 1] - b0);
    if (n > NB) {
        triplet_bwd_sweep<F>(i, lane, bptr, rhat, u, P, Q, Wtc, Sbar, Pbar, Qbar, ubar, rbar);
        return;
    }
    if (n <= 0) return;
    const int f = lane & (F - 1);
    const bool on = (F == 64 || lane < F);
    float wc[kAngle];
#pragma unroll
    for (int k = 0; k < kAngle; ++k) wc[k] = Wtc[k * F + f];
    float *accP = acc_lds[wave], *accQ = accP + NB * 64, *accU = accQ + NB * 64, *dsym = accU + NB * 64;
    for (int b = 0; b < n; ++b) {
        accP[b * 64 + lane] = 0.f;
        accQ[b * 64 + lane] = 0.f;
        accU[b * 64 + lane] = 0.f;
    }
    for (int a = 0; a < n; ++a) {
        const int64_t ba = b0 + a;
        const float xa = rhat[3 * ba], ya = rhat[3 * ba + 1], za = rhat[3 * ba + 2];
        const float pa = P[ba * F + f], qa = Q[ba * F + f], sa = Sbar[ba * F + f], ua = u[ba];
        float pacc = 0.f, qacc = 0.f, uacc = 0.f;
        float drow = 0.f;   // lane o: dE/dc of the pair {a, o}
        for (int o = a + 1; o < n; ++o) {
            const int64_t bo = b0 + o;
            const float c = fmaf(xa, rhat[3 * bo], fmaf(ya, rhat[3 * bo + 1], za * rhat[3 * bo + 2]));
            float T[kAngle], dT[kAngle];
            chebyshev(c, T, dT);
            float tw = 0.f, dw = 0.f;   // T(c) Wtc and dT(c)/dc Wtc for this lane's feature
#pragma unroll
            for (int k = 0; k < kAngle; ++k) {
                tw = fmaf(T[k], wc[k], tw);
                dw = fmaf(dT[k], wc[k], dw);
            }
            const float po = P[bo * F + f], qo = Q[bo * F + f], so = Sbar[bo * F + f], uo = u[bo];
            // bond o's accumulators: per-lane slots, read here and written at the end of the step (LDS float
            // atomics measured an order of magnitude slower than this read-modify-write)
            const float aq = accQ[o * 64 + lane], ap = accP[o * 64 + lane], au = accU[o * 64 + lane];
            float s1, ds1, s2, ds2;
            silu_both(pa + qo + tw, s1, ds1);   // triplet (b1 = a, b2 = o)
            silu_both(po + qa + tw, s2, ds2);   // triplet (b1 = o, b2 = a)
            const float h1 = sa * uo * ds1, h2 = so * ua * ds2;
            pacc += h1;
            qacc += h2;
            uacc = fmaf(so, s2, uacc);
            accQ[o * 64 + lane] = aq + h1;
            accP[o * 64 + lane] = ap + h2;
            accU[o * 64 + lane] = fmaf(sa, s1, au);
            const float tot = wave_sum(on ? (h1 + h2) * dw : 0.f);
            drow = (lane == o) ? tot : drow;
        }
        accP[a * 64 + lane] += pacc;
        accQ[a * 64 + lane] += qacc;
        accU[a * 64 + lane] += uacc;
        if (lane < NB) dsym[a * NB + lane] = drow;   // entries o > a
    }
    wave_lds_fence();
    for (int b = 0; b < n; ++b) {
        if (on) {
            Pbar[(b0 + b) * F + f] = accP[b * 64 + lane];
            Qbar[(b0 + b) * F + f] = accQ[b * 64 + lane];
        }
        const float ub = wave_sum(on ? accU[b * 64 + lane] : 0.f);
        if (lane == 0) ubar[b0 + b] += ub;
    }
    if (lane < n) {   // lane = bond: rbar_b = sum over the other bonds o of dE/dc{b, o} rhat_o
        float rx = 0.f, ry = 0.f, rz = 0.f;
        for (int o = 0; o < n; ++o) {
            if (o == lane) continue;
            const float dv = (o > lane) ? dsym[lane * NB + o] : dsym[o * NB + lane];
            rx = fmaf(dv, rhat[3 * (b0 + o)], rx);
            ry = fmaf(dv, rhat[3 * (b0 + o) + 1], ry);
            rz = fmaf(dv, rhat[3 * (b0 + o) + 2], rz);
        }
        rbar[3 * (b0 + lane)] = rx;
        rbar[3 * (b0 + lane) + 1] = ry;
        rbar[3 * (b0 + lane) + 2] = rz;
    }
}

// Forces of the bond part.  dE/dDelta_b = dbond rhat + (rbar - (rbar . rhat) rhat) / d for the bond vector
// Delta_b = r_j + S C - r_i; it pulls on j with + and on i with -.  Gathered per centre: the bonds in which i
// is the sender are the reverse bonds of its own.   F_i += sum_b (gDelta_b - gDelta_mirror(b))
__global__ void k_bond_force(int64_t N, const int64_t *__restrict__ bptr, const int32_t *__restrict__ bmirror,
                             const float *__restrict__ dbond, const float *__restrict__ rbar,
                             const float *__restrict__ rhat, const float *__restrict__ bd, float *floc)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= N) return;
    float fx = 0.f, fy = 0.f, fz = 0.f;
    for (int64_t b = bptr[i]; b < bptr[i + 1]; ++b) {
        for (int side = 0; side < 2; ++side) {
            const int64_t q = side ? (int64_t)bmirror[b] : b;
            if (q < 0) continue;   // reverse bond held by the sender's partition (it reaches this atom as a ghost there)
            const float x = rhat[3 * q], y = rhat[3 * q + 1], z = rhat[3 * q + 2];
            const float ax = rbar[3 * q], ay = rbar[3 * q + 1], az = rbar[3 * q + 2];
            const float dot = fmaf(ax, x, fmaf(ay, y, az * z));
            const float inv = 1.0f / bd[q];
            const float sgn = side ? -1.f : 1.f;
            fx += sgn * fmaf(dbond[q], x, (ax - dot * x) * inv);
            fy += sgn * fmaf(dbond[q], y, (ay - dot * y) * inv);
            fz += sgn * fmaf(dbond[q], z, (az - dot * z) * inv);
        }
    }
    floc[3 * i] += fx;
    floc[3 * i + 1] += fy;
    floc[3 * i + 2] += fz;
}

// ---- F x F products over the bonds, fused with what surrounds them
//
// Same tile scheme as the node kernel (32 bonds per wavefront step, packed operands in LDS, features x items
// accumulators); each stage reads or writes every [bonds x F] array it touches once.
//   HEAD       e0 = bbond(d) We0 (registers only, never stored: TAIL recomputes it);  P = e0 Wta;  Q = e0 Wtb
//   TAIL       m = S Wt2;  e1 = e0 + u SiLU(m) (registers only);  wb_l = e1 Wb_l for every layer l
//   LAYER_BWD  wbbar = abar_recv * g_send (built in the tile);  e1bar (+)= wbbar Wb_l^T
//   MBAR       ubar = sum_f e1bar SiLU(m);  mbar = e1bar u SiLU'(m) (tile only);  Sbar = mbar Wt2^T
//   E0BAR      e0bar = e1bar + Pbar Wta^T + Qbar Wtb^T (registers only);
//              dbond = sum_f e0bar (We0^T dbbond/dd) + ubar du/dd
enum { BOND_HEAD = 0, BOND_TAIL = 1, BOND_LAYER_BWD = 2, BOND_MBAR = 3, BOND_E0BAR = 4 };

struct BondArgs {                      // one partition
    int64_t n;                         // bonds
    const float *d, *u, *du;           // [n] length, envelope at the bond cutoff, its derivative
    const int32_t *edge, *sender;      // [n] edge index, sender row of a bond
    const int32_t *recv;               // receiver row of an edge
    const float *We0p;                 // We0 packed for the K = 8 product (k_pack_w1)
    BasisParams bp;                    // radial basis at the bond cutoff
    const float *W[4];                 // packed F x F operands of the stage (TAIL: Wt2, then the first layers' Wb)
    const float *Wx;                   // TAIL: packed Wb of the layers beyond the third (read from global memory)
    int n_layers;                      // TAIL
    int first;                         // LAYER_BWD: store e1bar instead of accumulating
    size_t wb_stride;                  // TAIL: floats between two layers' wb
    float *P, *Q;                      // HEAD out
    const float *S;                    // TAIL in
    float *m, *wb;                     // TAIL out; MBAR reads m
    const float *abar, *g;             // LAYER_BWD in (node rows)
    float *e1bar;                      // LAYER_BWD in/out; MBAR, E0BAR in
    float *ubar, *Sbar;                // MBAR out; E0BAR reads ubar
    const float *Pbar, *Qbar;          // E0BAR in
    float *dbond;                      // E0BAR out
};

template <int STAGE> struct BondStage {
    static constexpr int NW = (STAGE == BOND_TAIL) ? 8 : 4;   // wavefronts per block
    static constexpr int NPACK = (STAGE == BOND_TAIL) ? 4 : (STAGE == BOND_HEAD || STAGE == BOND_E0BAR) ? 2 : 1;
};

template <int F, int STAGE>
__global__ void __launch_bounds__(BondStage<STAGE>::NW * 64) k_bond_mlp(BondArgs A)
{
    using D = Dims<F>;
    constexpr int NB = D::NB, FS = D::FS;
    constexpr int NW = BondStage<STAGE>::NW, NPACK = BondStage<STAGE>::NPACK;
    constexpr int LPR = TileRegs<F>::LPR, RPI = TileRegs<F>::RPI;
    extern __shared__ float lds[];
    float *packs = lds;
    float *tiles = packs + NPACK * D::PACKF;
    const int n_lds_layers = (STAGE == BOND_TAIL) ? min(A.n_layers, 3) : 0;
    const int n_packs = (STAGE == BOND_TAIL) ? 1 + n_lds_layers : NPACK;
    for (int q = 0; q < n_packs; ++q)
        for (int i = threadIdx.x; i < D::PACKF; i += NW * 64) packs[q * D::PACKF + i] = A.W[q][i];
    __syncthreads();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int c32 = lane & 31, h = lane >> 5;
    const int rr = lane / LPR, cc = (lane % LPR) * 4;   // this lane's row and first feature within a tile row group
    RegPack1<F> W0;   // We0 as the A operands of the K = 8 product
    if (STAGE == BOND_HEAD || STAGE == BOND_TAIL || STAGE == BOND_E0BAR) load_pack1<F>(W0, A.We0p, lane);
    float *tile = tiles + wave * D::TILE;
    const int64_t n_tiles = (A.n + 31) / 32;
    const int64_t stride = (int64_t)gridDim.x * NW;

    // rows of a [bonds x F] array in accumulator layout: lane (c32, h) holds features 32 b + 8 a + 4 h + (0..3) of bond c32
    auto load_rows = [&](const float *Y, int64_t row, bool ok, f32x4 (&v)[NB][4]) {
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                v[b][a] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (ok) v[b][a] = *reinterpret_cast<const f32x4 *>(Y + row * F + 32 * b + 8 * a + 4 * h);
            }
    };
    auto store_rows = [&](float *Y, int64_t row, bool ok, const f32x16 (&acc)[NB]) {
        if (ok)
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const f32x4 v = {acc[b][4 * a], acc[b][4 * a + 1], acc[b][4 * a + 2], acc[b][4 * a + 3]};
                    *reinterpret_cast<f32x4 *>(Y + row * F + 32 * b + 8 * a + 4 * h) = v;
                }
    };

    TileRegs<F> pre, pre2;
    int64_t ti = (int64_t)blockIdx.x * NW + wave;
    if (ti < n_tiles) {
        if (STAGE == BOND_TAIL) fetch_tile<F>(pre, A.S, ti * 32, A.n, lane);
        if (STAGE == BOND_MBAR) {
            fetch_tile<F>(pre, A.e1bar, ti * 32, A.n, lane);
            fetch_tile<F>(pre2, A.m, ti * 32, A.n, lane);
        }
        if (STAGE == BOND_E0BAR) fetch_tile<F>(pre, A.Pbar, ti * 32, A.n, lane);
    }
    for (; ti < n_tiles; ti += stride) {
        const int64_t row0 = ti * 32;
        const int64_t row = row0 + c32;
        const bool ok = row < A.n;
        const bool more = ti + stride < n_tiles;
        f32x16 acc[NB];

        if (STAGE == BOND_HEAD) {
            float bb[8], db[8];
            radial_basis<false>(ok ? A.d[row] : A.bp.rc, A.bp, bb, db);   // 0 at the cutoff
            f32x16 e0[NB];
            gemm_k8r<F>(W0, bb, e0, lane);
            gemm_regs<F>(packs, e0, acc, lane);
            store_rows(A.P, row, ok, acc);
            gemm_regs<F>(packs + D::PACKF, e0, acc, lane);
            store_rows(A.Q, row, ok, acc);
        } else if (STAGE == BOND_TAIL) {
            stash_tile<F>(pre, tile, lane);
            wave_lds_fence();
            const float uc = ok ? A.u[row] : 0.f;
            const float dc = ok ? A.d[row] : A.bp.rc;
            if (more) fetch_tile<F>(pre, A.S, (ti + stride) * 32, A.n, lane);
            gemm_lds<F>(packs, tile, acc, lane);
            wave_lds_fence();
            store_rows(A.m, row, ok, acc);
            f32x16 e1[NB];
            {
                float bb[8], db[8];
                radial_basis<false>(dc, A.bp, bb, db);
                gemm_k8r<F>(W0, bb, e1, lane);   // e0, as in HEAD
            }
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) e1[b][r] = fmaf(uc, silu_f(acc[b][r]), e1[b][r]);
            for (int l = 0; l < n_lds_layers; ++l) {
                gemm_regs<F>(packs + (1 + l) * D::PACKF, e1, acc, lane);
                store_rows(A.wb + (size_t)l * A.wb_stride, row, ok, acc);
            }
            for (int l = 3; l < A.n_layers; ++l) {
                gemm_regs<F>(A.Wx + (size_t)(l - 3) * D::PACKF, e1, acc, lane);
                store_rows(A.wb + (size_t)l * A.wb_stride, row, ok, acc);
            }
        } else if (STAGE == BOND_LAYER_BWD) {
#pragma unroll
            for (int r = 0; r < 32; r += RPI) {
                const int64_t rw = row0 + r + rr;
                const bool okr = rw < A.n;
                f32x4 v = {0.f, 0.f, 0.f, 0.f};
                if (okr) {
                    const int64_t i = A.recv[A.edge[rw]], j = A.sender[rw];
                    const f32x4 va = *reinterpret_cast<const f32x4 *>(A.abar + i * F + cc);
                    const f32x4 vg = *reinterpret_cast<const f32x4 *>(A.g + j * F + cc);
                    v = va * vg;
                }
                *reinterpret_cast<f32x4 *>(tile + (r + rr) * FS + cc) = v;
            }
            wave_lds_fence();
            f32x4 zv[NB][4];
            load_rows(A.e1bar, row, ok && !A.first, zv);
            gemm_lds<F>(packs, tile, acc, lane);
            wave_lds_fence();
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[b][r] += zv[b][r / 4][r % 4];
            store_rows(A.e1bar, row, ok, acc);
        } else if (STAGE == BOND_MBAR) {
#pragma unroll
            for (int r = 0; r < 32; r += RPI) {
                const int64_t rw = row0 + r + rr;
                const bool okr = rw < A.n;
                const f32x4 eb = pre.v[r / RPI], mm = pre2.v[r / RPI];   // zero past the end
                const float ur = okr ? A.u[rw] : 0.f;
                f32x4 v;
                float part = 0.f;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    float sv, ds;
                    silu_both(mm[c], sv, ds);
                    v[c] = eb[c] * ur * ds;
                    part = fmaf(eb[c], sv, part);
                }
#pragma unroll
                for (int off = LPR / 2; off > 0; off >>= 1) part += __shfl_xor(part, off, 64);
                if (okr && (lane % LPR) == 0) A.ubar[rw] = part;
                *reinterpret_cast<f32x4 *>(tile + (r + rr) * FS + cc) = v;
            }
            wave_lds_fence();
            if (more) {
                fetch_tile<F>(pre, A.e1bar, (ti + stride) * 32, A.n, lane);
                fetch_tile<F>(pre2, A.m, (ti + stride) * 32, A.n, lane);
            }
            gemm_lds<F>(packs, tile, acc, lane);
            wave_lds_fence();
            store_rows(A.Sbar, row, ok, acc);
        } else {   // BOND_E0BAR
            stash_tile<F>(pre, tile, lane);
            wave_lds_fence();
            fetch_tile<F>(pre2, A.Qbar, row0, A.n, lane);   // in flight during the first product
            f32x4 zv[NB][4];
            load_rows(A.e1bar, row, ok, zv);
            gemm_lds<F>(packs, tile, acc, lane);
            wave_lds_fence();
            stash_tile<F>(pre2, tile, lane);
            wave_lds_fence();
            if (more) fetch_tile<F>(pre, A.Pbar, (ti + stride) * 32, A.n, lane);
            gemm_lds<F, true>(packs + D::PACKF, tile, acc, lane);
            wave_lds_fence();
            float bb[8], db[8];
            radial_basis<true>(ok ? A.d[row] : A.bp.rc, A.bp, bb, db);
            f32x16 vv[NB];   // We0^T dbbond/dd
            gemm_k8r<F>(W0, db, vv, lane);
            float part = 0.f;
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) part = fmaf(zv[b][r / 4][r % 4] + acc[b][r], vv[b][r], part);
            part += __shfl_xor(part, 32, 64);
            if (ok && h == 0) A.dbond[row] = fmaf(A.ubar[row], A.du[row], part);
        }
    }
}

inline unsigned blocks_for(int64_t n, int threads) { return (unsigned)((n + threads - 1) / threads); }

// ---------------------------------------------------------------- host driver

struct Packs {  // offsets (floats) into the packed-weight buffer
    size_t per_layer, A1, A1s, W2t, W2n, Wmt, Wmn, Wot, Won, readout_t, readout_n, total;
};

Packs pack_layout(int F, int L)
{
    Packs p;
    const size_t ff = (size_t)F * F, p1 = (size_t)(F / 32) * 4 * 64;
    p.A1 = 0;
    p.A1s = p1;
    p.W2t = 2 * p1;
    p.W2n = p.W2t + ff;
    p.Wmt = p.W2n + ff;
    p.Wmn = p.Wmt + ff;
    p.Wot = p.Wmn + ff;
    p.Won = p.Wot + ff;
    p.per_layer = p.Won + ff;
    p.readout_t = p.per_layer * (size_t)L;
    p.readout_n = p.readout_t + ff;
    p.total = p.readout_n + ff;
    return p;
}

template <int F> struct Lds {
    using D = Dims<F>;
    static constexpr size_t edge_fwd = sizeof(float) * (D::PACKF + 4 * D::TILE);
    static constexpr size_t edge_bwd = sizeof(float) * (D::PACKF + D::PACK1 + kBwdWaves * kQueue * D::FS);
    static constexpr size_t node1 = sizeof(float) * (D::PACKF + 4 * D::TILE);
    static constexpr size_t node2 = sizeof(float) * (2 * D::PACKF + 4 * D::TILE);
};

template <int F, int OP> int launch_node(mlip_graph *g, NodeBatch &b)
{
    constexpr bool TWO = (OP == OP_READOUT || OP == OP_BWD_UPDATE);
    const size_t lds = TWO ? Lds<F>::node2 : Lds<F>::node1;
    static bool configured = false;
    if (!configured) {
        MLIP_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_node<F, OP>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        configured = true;
    }
    b.tile_start[0] = 0;
    for (int q = 0; q < b.n; ++q) b.tile_start[q + 1] = b.tile_start[q] + (std::max<int64_t>(b.s[q].n_rows, 0) + 31) / 32;
    for (int q = b.n; q < kBatch; ++q) b.tile_start[q + 1] = b.tile_start[b.n];
    const int64_t n_tiles = b.tile_start[b.n];
    if (n_tiles <= 0) return MLIP_OK;
    // each block keeps its weight pack in LDS, so let it walk several tiles
    const unsigned blocks = (unsigned)std::min<int64_t>((n_tiles + 3) / 4, 2048);
    k_node<F, OP><<<blocks, 256, lds, g->stream>>>(b);
    MLIP_HIP(hipGetLastError());
    return MLIP_OK;
}

template <int F, int STAGE> int launch_bond_mlp(mlip_graph *g, const BondArgs &a)
{
    constexpr int NW = BondStage<STAGE>::NW;
    constexpr size_t lds = sizeof(float) * (BondStage<STAGE>::NPACK * Dims<F>::PACKF + NW * Dims<F>::TILE);
    static bool configured = false;
    if (!configured) {
        MLIP_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_bond_mlp<F, STAGE>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        configured = true;
    }
    if (a.n <= 0) return MLIP_OK;
    const int64_t n_tiles = (a.n + 31) / 32;
    // each block keeps its operand packs in LDS, so let it walk several tiles
    const unsigned blocks = (unsigned)std::min<int64_t>((n_tiles + NW - 1) / NW, 8192 / NW);
    k_bond_mlp<F, STAGE><<<blocks, NW * 64, lds, g->stream>>>(a);
    MLIP_HIP(hipGetLastError());
    return MLIP_OK;
}

// Runs one node operation over all partitions, kBatch per launch; fill(view, args) sets the rows.
template <int F, int OP, class Fill>
int node_pass(mlip_graph *g, SlabView *views, int P, const float *P1, const float *P2, const float *wr2, Fill fill)
{
    for (int p0 = 0; p0 < P; p0 += kBatch) {
        NodeBatch nb{};
        nb.n = std::min(kBatch, P - p0);
        nb.P1 = P1;
        nb.P2 = P2;
        nb.wr2 = wr2;
        for (int q = 0; q < nb.n; ++q) fill(views[p0 + q], nb.s[q]);
        MLIP_TRY((launch_node<F, OP>(g, nb)));
    }
    return MLIP_OK;
}

template <int F, int PREC> int launch_edge(mlip_graph *g, EdgeBatch &b, bool backward)
{
    const size_t lds = backward ? Lds<F>::edge_bwd : Lds<F>::edge_fwd;
    // resident blocks per compute unit, queried once per kernel
    static int occ_f = 0, occ_b = 0, n_cu = 0;
    int &occ = backward ? occ_b : occ_f;
    if (occ == 0) {
        const void *fn = backward ? reinterpret_cast<const void *>(&k_edge_bwd<F, PREC>)
                                  : reinterpret_cast<const void *>(&k_edge_fwd<F, PREC>);
        MLIP_HIP(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        int dev = 0, o = 0;
        MLIP_HIP(hipGetDevice(&dev));
        MLIP_HIP(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
        if (backward)
            MLIP_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&o, k_edge_bwd<F, PREC>, kBwdWaves * 64, lds));
        else
            MLIP_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&o, k_edge_fwd<F, PREC>, 256, lds));
        if (o < 1 || n_cu < 8) {
            set_error("edge kernel does not fit the device (occupancy %d, %d compute units)", o, n_cu);
            return MLIP_EHIP;
        }
        occ = o;
    }
    b.chunk_start[0] = 0;
    for (int q = 0; q < b.n; ++q) b.chunk_start[q + 1] = b.chunk_start[q] + (b.s[q].n_rows > 0 ? b.s[q].n_chunks : 0);
    for (int q = b.n; q < kBatch; ++q) b.chunk_start[q + 1] = b.chunk_start[b.n];
    const int64_t items = b.chunk_start[b.n];
    if (items <= 0) return MLIP_OK;
    // persistent grid: what is resident at once, a multiple of the 8 XCDs, no more than the work needs
    const int64_t resident = (int64_t)(n_cu / 8) * occ;
    const int nw = backward ? kBwdWaves : 4;
    const int64_t needed = ((items + 7) / 8 + nw - 1) / nw;
    const unsigned blocks = (unsigned)(8 * std::max<int64_t>(1, std::min(resident, needed)));
    if (backward)
        k_edge_bwd<F, PREC><<<blocks, kBwdWaves * 64, lds, g->stream>>>(b);
    else
        k_edge_fwd<F, PREC><<<blocks, 256, lds, g->stream>>>(b);
    MLIP_HIP(hipGetLastError());
    return MLIP_OK;
}

// bw != nullptr: the three-body variant
template <int F>
int forward_t(mlip_graph *g, const mlip_weights_t *w, const mlip_bond_weights_t *bw, int32_t mode, double *energy,
              float *forces, float *atom_energy)
{
    hipStream_t s = g->stream;
    const int L = w->L;
    const int prec = (w->precision == MLIP_PRECISION_BF16) ? kPrecBf16
                     : (w->precision == MLIP_PRECISION_FP32_SPLIT) ? kPrecF16x3 : kPrecF32;
    const bool slabs = (mode == MLIP_MODE_SLABS);
    const int P = slabs ? g->P : 1;
    SlabView *views = slabs ? g->slabs.data() : &g->whole;
    const size_t rowb = (size_t)F * sizeof(float);

    // ---- workspace
    for (int p = 0; p < P; ++p)
        if (views[p].n_local * (int64_t)F * 4 >= ((int64_t)1 << 31)) {
            set_error("a partition holds more than 2^31 bytes of node features; use more slabs");
            return MLIP_EINVAL;
        }
    int64_t n_parts = 0;
    for (int p = 0; p < P; ++p) {
        SlabView &v = views[p];
        const size_t no = (size_t)std::max<int64_t>(v.n_owned, 1), nl = (size_t)std::max<int64_t>(v.n_local, 1);
        MLIP_TRY(v.h.ensure(no * rowb));
        MLIP_TRY(v.hbar.ensure(no * rowb));
        MLIP_TRY(v.abar.ensure(nl * rowb));
        MLIP_TRY(v.gbar.ensure(nl * rowb));
        MLIP_TRY(v.eps.ensure(no * sizeof(float)));
        MLIP_TRY(v.dsum.ensure((size_t)std::max<int64_t>(v.n_edges, 1) * sizeof(float)));
        MLIP_TRY(v.floc.ensure(nl * 3 * sizeof(float)));
        MLIP_TRY(v.g.ensure(nl * rowb * (size_t)std::max(L, 1)));
        MLIP_TRY(v.a.ensure(no * rowb * (size_t)std::max(L, 1)));
        if (L > 1)  // filter values of layers 1..L-1, kept for the reverse pass instead of being recomputed
            MLIP_TRY(v.wst.ensure((size_t)std::max<int64_t>(v.n_edges_owned, 1) * rowb * (size_t)(L - 1)));
        n_parts += (v.n_owned + 1023) / 1024;
    }
    MLIP_TRY(g->energy_part.ensure((size_t)std::max<int64_t>(n_parts, 1) * sizeof(double)));
    const Packs pk = pack_layout(F, L);
    MLIP_TRY(g->wpack.ensure(pk.total * sizeof(float)));
    float *wp = g->wpack.as<float>();

    BasisParams bp;
    bp.rc = (float)g->r_cut;
    bp.inv_rc = (float)(1.0 / g->r_cut);
    bp.p = w->p;
    const double pd = (double)w->p;
    bp.pc0 = (float)(pd * (pd + 1) * (pd + 2) / 2);

    // ---- pack weights
    prof_begin(g, MLIP_PROF_NODE);
    const unsigned pb = blocks_for((int64_t)F * F, 256);
    for (int l = 0; l < L; ++l) {
        float *base = wp + pk.per_layer * l;
        const size_t ff = (size_t)F * F;
        k_pack_w1<<<blocks_for((F / 32) * 256, 256), 256, 0, s>>>(w->W1 + (size_t)l * 8 * F, F, 1.0f, base + pk.A1);
        k_pack_w1<<<blocks_for((F / 32) * 256, 256), 256, 0, s>>>(w->W1 + (size_t)l * 8 * F, F, kSiluScale, base + pk.A1s);
        if (prec == kPrecBf16) {   // the two W2 operands as bf16 packs (half of their slots)
            k_pack_ff_bf16<<<pb, 256, 0, s>>>(w->W2 + l * ff, F, 1, kSiluScaleInv, reinterpret_cast<__bf16 *>(base + pk.W2t));
            k_pack_ff_bf16<<<pb, 256, 0, s>>>(w->W2 + l * ff, F, 0, 1.0f, reinterpret_cast<__bf16 *>(base + pk.W2n));
        } else if (prec == kPrecF16x3) {   // as split-fp16 packs (hi and lo halves)
            k_pack_ff_f16x2<<<pb, 256, 0, s>>>(w->W2 + l * ff, F, 1, kSiluScaleInv, reinterpret_cast<_Float16 *>(base + pk.W2t));
            k_pack_ff_f16x2<<<pb, 256, 0, s>>>(w->W2 + l * ff, F, 0, 1.0f, reinterpret_cast<_Float16 *>(base + pk.W2n));
        } else {
            k_pack_ff<<<pb, 256, 0, s>>>(w->W2 + l * ff, F, 1, kSiluScaleInv, base + pk.W2t);
            k_pack_ff<<<pb, 256, 0, s>>>(w->W2 + l * ff, F, 0, 1.0f, base + pk.W2n);
        }
        k_pack_ff<<<pb, 256, 0, s>>>(w->Wm + l * ff, F, 1, 1.0f, base + pk.Wmt);
        k_pack_ff<<<pb, 256, 0, s>>>(w->Wm + l * ff, F, 0, 1.0f, base + pk.Wmn);
        k_pack_ff<<<pb, 256, 0, s>>>(w->Wo + l * ff, F, 1, 1.0f, base + pk.Wot);
        k_pack_ff<<<pb, 256, 0, s>>>(w->Wo + l * ff, F, 0, 1.0f, base + pk.Won);
    }
    k_pack_ff<<<pb, 256, 0, s>>>(w->Wr1, F, 1, 1.0f, wp + pk.readout_t);
    k_pack_ff<<<pb, 256, 0, s>>>(w->Wr1, F, 0, 1.0f, wp + pk.readout_n);
    MLIP_HIP(hipGetLastError());

    // ---- embedding
    const int32_t *species = g->species.as<int32_t>();
    for (int p = 0; p < P; ++p) {
        SlabView &v = views[p];
        if (v.n_owned > 0)
            k_embed<<<blocks_for(v.n_owned * F, 256), 256, 0, s>>>(v.n_owned, F, v.nodes, species, w->emb, v.h.as<float>());
    }
    MLIP_HIP(hipGetLastError());
    prof_end(g);

    // ---- three-body variant: bond lists, bond embedding, triplet update, bond terms of the layers' filters.
    // All bonds and triplets of an owned centre are local to its partition, so this part needs no transfer.
    float *bpk = nullptr;        // packed F x F operands of the bond part
    const size_t ffp = (size_t)F * F;
    // operand slots: 0 Wta (y = x W), 1 Wtb, 2 Wt2, 3 Wta^T, 4 Wtb^T, 5 Wt2^T, 6 + l Wb_l, 6 + L + l Wb_l^T; after them We0
    // packed for the K = 8 product
    BasisParams bpb = bp;
    auto bstride = [&](SlabView &v) { return (size_t)std::max<int64_t>(v.bonds.n, 1) * F; };   // floats per [n][F] array
    auto wbslice = [&](SlabView &v, int l) { return v.bonds.wb.as<float>() + (size_t)l * bstride(v); };
    auto bond_args = [&](SlabView &v) {   // everything a stage of k_bond_mlp may touch; the stage's operands are set by the caller
        BondGraph &BG = v.bonds;
        BondArgs a{};
        a.n = BG.n;
        a.d = BG.d.as<float>();
        a.u = BG.u.as<float>();
        a.du = BG.du.as<float>();
        a.edge = BG.edge.as<int32_t>();
        a.sender = BG.sender.as<int32_t>();
        a.recv = v.recv;
        a.We0p = bpk + (size_t)(6 + 2 * L) * ffp;
        a.bp = bpb;
        a.wb_stride = bstride(v);
        a.P = BG.P.as<float>();
        a.Q = BG.Q.as<float>();
        a.S = BG.S.as<float>();
        a.m = BG.m.as<float>();
        a.wb = BG.wb.as<float>();
        a.abar = v.abar.as<float>();
        a.e1bar = BG.e1bar.as<float>();
        a.ubar = BG.ubar.as<float>();
        a.Sbar = BG.Sbar.as<float>();
        a.Pbar = BG.Pbar.as<float>();
        a.Qbar = BG.Qbar.as<float>();
        a.dbond = BG.dbond.as<float>();
        return a;
    };
    bool any_bonds = false;
    if (bw) {
        bpb.rc = bw->r_bond;
        bpb.inv_rc = 1.0f / bw->r_bond;
        prof_begin(g, MLIP_PROF_BOND);
        for (int p = 0; p < P; ++p) MLIP_TRY(build_bonds_impl(g, views[p], (double)bw->r_bond, w->p));
        prof_end(g);
        for (int p = 0; p < P; ++p) {
            BondGraph &BG = views[p].bonds;
            const size_t bs = bstride(views[p]), nb1 = (size_t)std::max<int64_t>(BG.n, 1);
            DevBuf *fb[] = {&BG.P, &BG.Q, &BG.S, &BG.m, &BG.e1bar, &BG.Sbar, &BG.Pbar, &BG.Qbar};
            for (DevBuf *b : fb) MLIP_TRY(b->ensure(bs * sizeof(float)));
            MLIP_TRY(BG.wb.ensure(bs * sizeof(float) * (size_t)std::max(L, 1)));
            MLIP_TRY(BG.ubar.ensure(nb1 * sizeof(float)));
            MLIP_TRY(BG.dbond.ensure(nb1 * sizeof(float)));
            MLIP_TRY(BG.rbar.ensure(nb1 * 3 * sizeof(float)));
            any_bonds = any_bonds || BG.n > 0;
        }
        MLIP_TRY(g->bond_wpack.ensure(((size_t)(6 + 2 * L) * ffp + Dims<F>::PACK1) * sizeof(float)));
        bpk = g->bond_wpack.as<float>();
        prof_begin(g, MLIP_PROF_BOND);
        const float *Wta = bw->Wt1, *Wtb = bw->Wt1 + ffp, *Wtc = bw->Wt1 + 2 * ffp;
        k_pack_ff<<<pb, 256, 0, s>>>(Wta, F, 1, 1.0f, bpk + 0 * ffp);
        k_pack_ff<<<pb, 256, 0, s>>>(Wtb, F, 1, 1.0f, bpk + 1 * ffp);
        k_pack_ff<<<pb, 256, 0, s>>>(bw->Wt2, F, 1, 1.0f, bpk + 2 * ffp);
        k_pack_ff<<<pb, 256, 0, s>>>(Wta, F, 0, 1.0f, bpk + 3 * ffp);
        k_pack_ff<<<pb, 256, 0, s>>>(Wtb, F, 0, 1.0f, bpk + 4 * ffp);
        k_pack_ff<<<pb, 256, 0, s>>>(bw->Wt2, F, 0, 1.0f, bpk + 5 * ffp);
        for (int l = 0; l < L; ++l) {
            k_pack_ff<<<pb, 256, 0, s>>>(bw->Wb + l * ffp, F, 1, 1.0f, bpk + (6 + l) * ffp);
            k_pack_ff<<<pb, 256, 0, s>>>(bw->Wb + l * ffp, F, 0, 1.0f, bpk + (6 + L + l) * ffp);
        }
        k_pack_w1<<<blocks_for(Dims<F>::PACK1, 256), 256, 0, s>>>(bw->We0, F, 1.0f, bpk + (size_t)(6 + 2 * L) * ffp);
        MLIP_HIP(hipGetLastError());
        for (int p = 0; p < P; ++p) {   // P = e0 Wta, Q = e0 Wtb with e0 = bbond(d) We0
            BondArgs a = bond_args(views[p]);
            a.W[0] = bpk + 0 * ffp;
            a.W[1] = bpk + 1 * ffp;
            MLIP_TRY((launch_bond_mlp<F, BOND_HEAD>(g, a)));
        }
        prof_end(g);
        prof_begin(g, MLIP_PROF_TRIPLET_FWD);
        for (int p = 0; p < P; ++p) {
            SlabView &v = views[p];
            BondGraph &BG = v.bonds;
            if (BG.n > 0)
                k_triplet_fwd<F><<<blocks_for(v.n_owned, 4), 256, 0, s>>>(v.n_owned, BG.ptr.as<int64_t>(), BG.rhat.as<float>(),
                                                                          BG.u.as<float>(), BG.P.as<float>(),
                                                                          BG.Q.as<float>(), Wtc, BG.S.as<float>());
        }
        MLIP_HIP(hipGetLastError());
        prof_end(g);
        prof_begin(g, MLIP_PROF_BOND);
        for (int p = 0; p < P; ++p) {   // m = S Wt2, e1 = e0 + u SiLU(m), wb_l = e1 Wb_l
            BondArgs a = bond_args(views[p]);
            a.W[0] = bpk + 2 * ffp;
            for (int l = 0; l < std::min(L, 3); ++l) a.W[1 + l] = bpk + (6 + l) * ffp;
            a.Wx = bpk + (6 + 3) * ffp;
            a.n_layers = L;
            MLIP_TRY((launch_bond_mlp<F, BOND_TAIL>(g, a)));
        }
        prof_end(g);
    }

    auto gslice = [&](SlabView &v, int l) { return v.g.as<float>() + (size_t)l * (size_t)v.n_local * F; };
    auto aslice = [&](SlabView &v, int l) { return v.a.as<float>() + (size_t)l * (size_t)v.n_owned * F; };
    auto wslice = [&](SlabView &v, int l) {  // l >= 1
        return v.wst.as<float>() + (size_t)(l - 1) * (size_t)v.n_edges_owned * F;
    };

    // ---- forward layers
    for (int l = 0; l < L; ++l) {
        const float *base = wp + pk.per_layer * l;
        prof_begin(g, MLIP_PROF_NODE);
        MLIP_TRY((node_pass<F, OP_PROJ>(g, views, P, base + pk.Wmt, nullptr, nullptr, [&](SlabView &v, NodeArgs &na) {
            na.n_rows = v.n_owned;   // sender projection on owned rows
            na.X = v.h.as<float>();
            na.Y = gslice(v, l);
        })));
        prof_end(g);
        if (slabs) {
            prof_begin(g, MLIP_PROF_GHOST);
            PtrTable tab{};
            for (int q = 0; q < P; ++q) tab.p[q] = gslice(views[q], l);
            for (int p = 0; p < P; ++p) {  // border-node transfer: ghost rows <- owners
                SlabView &v = views[p];
                if (v.n_ghost > 0)
                    k_ghost_copy<<<blocks_for(v.n_ghost * (F / 4), 256), 256, 0, s>>>(
                        v.n_ghost, v.n_owned, F, v.ghost_owner, v.ghost_src, tab, gslice(v, l));
            }
            MLIP_HIP(hipGetLastError());
            prof_end(g);
        }
        for (int p0 = 0; p0 < P; p0 += kBatch) {   // the partitions in order, up to kBatch per launch
            EdgeBatch eb{};
            eb.n = std::min(kBatch, P - p0);
            eb.c.A1 = base + pk.A1;
            eb.c.A1s = base + pk.A1s;
            eb.c.A2t = base + pk.W2t;
            eb.c.bp = bp;
            for (int q = 0; q < eb.n; ++q) {
                SlabView &v = views[p0 + q];
                EdgeArgs &ea = eb.s[q];
                ea.n_rows = v.n_owned;
                ea.n_chunks = chunks_of(v.n_edges_owned);
                ea.chunk_row = v.chunk_row;
                ea.n_nodes = v.n_local;
                ea.row_ptr = v.row_ptr;
                ea.senders = v.senders;
                ea.recv = v.recv;
                ea.d = v.d;
                ea.g = gslice(v, l);
                ea.out = aslice(v, l);
                ea.wstore = (l >= 1) ? wslice(v, l) : nullptr;
            }
            prof_begin(g, MLIP_PROF_EDGE_FWD);
            MLIP_TRY(prec == kPrecBf16 ? (launch_edge<F, kPrecBf16>(g, eb, false))
                     : prec == kPrecF16x3 ? (launch_edge<F, kPrecF16x3>(g, eb, false)) : (launch_edge<F, kPrecF32>(g, eb, false)));
            prof_end(g);
        }
        if (any_bonds) {   // bond term of the filters: a_i += sum_b wb_b * g_send(b)
            prof_begin(g, MLIP_PROF_BOND);
            for (int p = 0; p < P; ++p) {
                SlabView &v = views[p];
                if (v.bonds.n > 0)
                    k_bond_aggregate<F><<<blocks_for(v.n_owned, 4), 256, 0, s>>>(
                        v.n_owned, v.bonds.ptr.as<int64_t>(), v.bonds.sender.as<int32_t>(), wbslice(v, l), gslice(v, l),
                        aslice(v, l));
            }
            MLIP_HIP(hipGetLastError());
            prof_end(g);
        }
        prof_begin(g, MLIP_PROF_NODE);
        MLIP_TRY((node_pass<F, OP_UPDATE>(g, views, P, base + pk.Wot, nullptr, nullptr, [&](SlabView &v, NodeArgs &na) {
            na.n_rows = v.n_owned;
            na.X = aslice(v, l);
            na.Z = v.h.as<float>();
        })));
        prof_end(g);
    }

    // ---- readout (energy and dE/dh of the last layer in one pass)
    prof_begin(g, MLIP_PROF_NODE);
    MLIP_TRY((node_pass<F, OP_READOUT>(g, views, P, wp + pk.readout_t, wp + pk.readout_n, w->wr2,
                                       [&](SlabView &v, NodeArgs &na) {
                                           na.n_rows = v.n_owned;
                                           na.X = v.h.as<float>();
                                           na.Y = v.hbar.as<float>();
                                           na.eps = v.eps.as<float>();
                                       })));
    prof_end(g);
    prof_begin(g, MLIP_PROF_FORCE);
    {
        int64_t off = 0;
        double *part = g->energy_part.as<double>();
        for (int p = 0; p < P; ++p) {
            SlabView &v = views[p];
            const int64_t nb = (v.n_owned + 1023) / 1024;
            if (nb > 0) k_energy_partial<<<(unsigned)nb, 256, 0, s>>>(v.n_owned, v.eps.as<float>(), part + off);
            off += nb;
        }
        k_energy_final<<<1, 256, 0, s>>>(off, part, energy);
        MLIP_HIP(hipGetLastError());
    }
    prof_end(g);

    // ---- reverse pass
    for (int p = 0; p < P; ++p) {  // ghost rows carry no dE/da: zero once, no kernel ever writes them
        SlabView &v = views[p];
        if (L > 0 && v.n_ghost > 0)
            MLIP_HIP(hipMemsetAsync(v.abar.as<float>() + (size_t)v.n_owned * F, 0, (size_t)v.n_ghost * rowb, s));
    }
    if (any_bonds && L == 0)   // no layer writes e1bar: the energy does not depend on the bonds
        for (int p = 0; p < P; ++p)
            if (views[p].bonds.n > 0)
                MLIP_HIP(hipMemsetAsync(views[p].bonds.e1bar.p, 0, bstride(views[p]) * sizeof(float), s));
    for (int l = L - 1; l >= 0; --l) {
        const float *base = wp + pk.per_layer * l;
        const bool need_gbar = l > 0;  // dE/dh0 is never used: the embedding does not depend on positions
        prof_begin(g, MLIP_PROF_NODE);
        MLIP_TRY((node_pass<F, OP_BWD_UPDATE>(g, views, P, base + pk.Wot, base + pk.Won, nullptr,
                                              [&](SlabView &v, NodeArgs &na) {
                                                  na.n_rows = v.n_owned;
                                                  na.X = aslice(v, l);
                                                  na.Z = v.hbar.as<float>();
                                                  na.Y = v.abar.as<float>();
                                              })));
        prof_end(g);
        for (int p0 = 0; p0 < P; p0 += kBatch) {
            EdgeBatch eb{};
            eb.n = std::min(kBatch, P - p0);
            eb.c.A1 = base + pk.A1;
            eb.c.A1s = base + pk.A1s;
            eb.c.A2t = base + pk.W2t;
            eb.c.A2n = base + pk.W2n;
            eb.c.bp = bp;
            eb.c.need_gbar = need_gbar ? 1 : 0;
            eb.c.first = (l == L - 1) ? 1 : 0;
            for (int q = 0; q < eb.n; ++q) {
                SlabView &v = views[p0 + q];
                EdgeArgs &ea = eb.s[q];
                ea.n_rows = v.n_owned;
                ea.n_chunks = chunks_of(v.n_edges_owned);
                ea.chunk_row = v.chunk_row;
                ea.n_nodes = v.n_local;
                ea.row_ptr = v.row_ptr;
                ea.senders = v.senders;
                ea.recv = v.recv;
                ea.d = v.d;
                ea.g = gslice(v, l);
                ea.abar = v.abar.as<float>();
                ea.out = v.gbar.as<float>();
                ea.dsum = v.dsum.as<float>();
                ea.mirror = v.mirror;
                ea.wstore = need_gbar ? wslice(v, l) : nullptr;
                ea.n_stored = need_gbar ? v.n_edges_owned : 0;
            }
            prof_begin(g, MLIP_PROF_EDGE_BWD);
            MLIP_TRY(prec == kPrecBf16 ? (launch_edge<F, kPrecBf16>(g, eb, true))
                     : prec == kPrecF16x3 ? (launch_edge<F, kPrecF16x3>(g, eb, true)) : (launch_edge<F, kPrecF32>(g, eb, true)));
            prof_end(g);
        }
        if (any_bonds) {   // bond term: its share of gbar, and e1bar (+)= dE/dwb Wb_l^T
            prof_begin(g, MLIP_PROF_BOND);
            for (int p = 0; p < P; ++p) {
                SlabView &v = views[p];
                BondGraph &BG = v.bonds;
                if (BG.n > 0 && need_gbar)
                    k_bond_gbar<F><<<blocks_for(v.n_owned, 4), 256, 0, s>>>(
                        v.n_owned, BG.ptr.as<int64_t>(), BG.sender.as<int32_t>(), BG.mirror.as<int32_t>(), wbslice(v, l),
                        v.abar.as<float>(), v.gbar.as<float>());
            }
            MLIP_HIP(hipGetLastError());
            for (int p = 0; p < P; ++p) {   // e1bar (+)= (abar_recv * g_send) Wb_l^T
                BondArgs a = bond_args(views[p]);
                a.g = gslice(views[p], l);
                a.W[0] = bpk + (6 + L + l) * ffp;
                a.first = (l == L - 1);
                MLIP_TRY((launch_bond_mlp<F, BOND_LAYER_BWD>(g, a)));
            }
            prof_end(g);
        }
        if (need_gbar) {
            if (slabs) {
                prof_begin(g, MLIP_PROF_GHOST);
                PtrTable tab{};
                for (int q = 0; q < P; ++q) tab.p[q] = views[q].gbar.as<float>();
                for (int p = 0; p < P; ++p) {  // ghost-row gradients -> owners, partitions in ascending order
                    SlabView &v = views[p];
                    if (v.n_ghost > 0)
                        k_ghost_gbar<F><<<blocks_for(v.n_ghost, 4), 256, 0, s>>>(
                            v.n_ghost, v.n_owned, v.row_ptr, v.senders, v.mirror, wslice(v, l), v.abar.as<float>(),
                            (bw && v.bonds.n > 0) ? v.bonds.of_edge.as<int32_t>() : nullptr,
                            (bw && v.bonds.n > 0) ? wbslice(v, l) : nullptr, v.gbar.as<float>());
                    if (v.n_ghost > 0)
                        k_ghost_addback<<<blocks_for(v.n_ghost * (F / 4), 256), 256, 0, s>>>(
                            v.n_ghost, v.n_owned, F, v.ghost_owner, v.ghost_src, tab, v.gbar.as<float>());
                }
                MLIP_HIP(hipGetLastError());
                prof_end(g);
            }
            prof_begin(g, MLIP_PROF_NODE);
            MLIP_TRY((node_pass<F, OP_BWD_PROJ>(g, views, P, base + pk.Wmn, nullptr, nullptr, [&](SlabView &v, NodeArgs &na) {
                na.n_rows = v.n_owned;
                na.X = v.gbar.as<float>();
                na.Z = v.hbar.as<float>();
            })));
            prof_end(g);
        }
    }

    // ---- reverse of the bond update: e1 = e0 + u SiLU(m), m = S Wt2, S = triplet sum, e0 = bbond(d) We0
    if (any_bonds) {
        prof_begin(g, MLIP_PROF_BOND);
        const float *Wtc = bw->Wt1 + 2 * ffp;
        for (int p = 0; p < P; ++p) {   // ubar, Sbar = (e1bar u SiLU'(m)) Wt2^T
            BondArgs a = bond_args(views[p]);
            a.W[0] = bpk + 5 * ffp;
            MLIP_TRY((launch_bond_mlp<F, BOND_MBAR>(g, a)));
        }
        prof_end(g);
        prof_begin(g, MLIP_PROF_TRIPLET_BWD);
        for (int p = 0; p < P; ++p) {
            SlabView &v = views[p];
            BondGraph &BG = v.bonds;
            if (BG.n > 0)
                k_triplet_bwd<F><<<blocks_for(v.n_owned, 4), 256, 0, s>>>(
                    v.n_owned, BG.ptr.as<int64_t>(), BG.rhat.as<float>(), BG.u.as<float>(), BG.P.as<float>(), BG.Q.as<float>(),
                    Wtc, BG.Sbar.as<float>(), BG.Pbar.as<float>(), BG.Qbar.as<float>(), BG.ubar.as<float>(), BG.rbar.as<float>());
        }
        MLIP_HIP(hipGetLastError());
        prof_end(g);
        prof_begin(g, MLIP_PROF_BOND);
        for (int p = 0; p < P; ++p) {   // e0bar = e1bar + Pbar Wta^T + Qbar Wtb^T, and dE/dd of the bonds from it
            BondArgs a = bond_args(views[p]);
            a.W[0] = bpk + 3 * ffp;
            a.W[1] = bpk + 4 * ffp;
            MLIP_TRY((launch_bond_mlp<F, BOND_E0BAR>(g, a)));
        }
        prof_end(g);
    }

    // ---- forces
    prof_begin(g, MLIP_PROF_FORCE);
    const double *pos = g->pos.as<double>();
    for (int p = 0; p < P; ++p) {
        SlabView &v = views[p];
        if (L > 0 && v.n_local > 0) {
            k_force_rows<<<(unsigned)((v.n_local + 15) / 16), 256, 0, s>>>(v.n_local, v.row_ptr, v.senders, v.shiftp, v.dsum.as<float>(),
                                                            v.nodes, pos, g->cell, v.floc.as<float>());
        } else if (v.n_local > 0) {
            MLIP_HIP(hipMemsetAsync(v.floc.p, 0, (size_t)v.n_local * 3 * sizeof(float), s));
        }
        if (bw && v.bonds.n > 0) {
            BondGraph &BG = v.bonds;
            k_bond_force<<<blocks_for(v.n_owned, 128), 128, 0, s>>>(v.n_owned, BG.ptr.as<int64_t>(), BG.mirror.as<int32_t>(),
                                                                    BG.dbond.as<float>(), BG.rbar.as<float>(),
                                                                    BG.rhat.as<float>(), BG.d.as<float>(), v.floc.as<float>());
            if (v.n_ghost > 0)
                k_bond_force_ghost<<<blocks_for(v.n_ghost, 128), 128, 0, s>>>(
                    v.n_ghost, v.n_owned, v.row_ptr, v.mirror, BG.of_edge.as<int32_t>(), BG.dbond.as<float>(),
                    BG.rbar.as<float>(), BG.rhat.as<float>(), BG.d.as<float>(), v.floc.as<float>());
        }
        if (v.n_owned > 0)
            k_store_owned<<<blocks_for(v.n_owned, 256), 256, 0, s>>>(v.n_owned, v.nodes, v.floc.as<float>(),
                                                                     v.eps.as<float>(), forces, atom_energy);
    }
    if (slabs)
        for (int p = 0; p < P; ++p) {
            SlabView &v = views[p];
            if (v.n_ghost > 0)
                k_addback_ghost_forces<<<blocks_for(v.n_ghost, 256), 256, 0, s>>>(v.n_ghost, v.n_owned, v.nodes,
                                                                                  v.floc.as<float>(), forces);
        }
    MLIP_HIP(hipGetLastError());
    prof_end(g);
    return MLIP_OK;
}

}  // namespace

int forward_impl(mlip_graph *g, const mlip_weights_t *w, int32_t mode, double *energy, float *forces, float *atom_energy)
{
    if (w->F == 32) return forward_t<32>(g, w, nullptr, mode, energy, forces, atom_energy);
    return forward_t<64>(g, w, nullptr, mode, energy, forces, atom_energy);
}

int forward_bonds_impl(mlip_graph *g, const mlip_weights_t *w, const mlip_bond_weights_t *bw, int32_t mode,
                       double *energy, float *forces, float *atom_energy)
{
    if (w->F == 32) return forward_t<32>(g, w, bw, mode, energy, forces, atom_energy);
    return forward_t<64>(g, w, bw, mode, energy, forces, atom_energy);
}

}  // namespace mlip

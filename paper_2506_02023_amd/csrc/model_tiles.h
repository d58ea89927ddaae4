// Types, the radial basis, packed weight operands and the MFMA tile products shared by the model kernels.
// Part of model.hip (one translation unit): included inside namespace mlip, anonymous namespace.
#ifndef MLIP_MODEL_TILES_H
#define MLIP_MODEL_TILES_H

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

// Element access for arrays that are kept as fp32 or, in the bf16 precision mode, as bf16: rounded to nearest even
// on the way out, exact on the way in.  load4 / store4 move four consecutive elements; load4_raw returns them
// as loaded and widen4 converts later, so that a prefetch does not have to wait for its data to convert it.
template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ inline float load(const float *p) { return *p; }
    static __device__ inline void store(float *p, float v) { *p = v; }
    typedef f32x4 raw4;
    static __device__ inline raw4 load4_raw(const float *p) { return *reinterpret_cast<const f32x4 *>(p); }
    static __device__ inline f32x4 widen4(raw4 w) { return w; }
    static __device__ inline f32x4 load4(const float *p) { return *reinterpret_cast<const f32x4 *>(p); }
    static __device__ inline void store4(float *p, f32x4 v) { *reinterpret_cast<f32x4 *>(p) = v; }
};
template <> struct Elem<__bf16> {
    static __device__ inline float load(const __bf16 *p)
    {
        return __builtin_bit_cast(float, (unsigned)*reinterpret_cast<const unsigned short *>(p) << 16);
    }
    static __device__ inline void store(__bf16 *p, float v) { *p = (__bf16)v; }
    typedef uint2 raw4;
    static __device__ inline raw4 load4_raw(const __bf16 *p) { return *reinterpret_cast<const uint2 *>(p); }
    static __device__ inline f32x4 widen4(raw4 w)
    {
        return f32x4{__builtin_bit_cast(float, w.x << 16), __builtin_bit_cast(float, w.x & 0xffff0000u),
                     __builtin_bit_cast(float, w.y << 16), __builtin_bit_cast(float, w.y & 0xffff0000u)};
    }
    static __device__ inline f32x4 load4(const __bf16 *p) { return widen4(load4_raw(p)); }
    static __device__ inline void store4(__bf16 *p, f32x4 v)
    {
        const bf16x2 lo = __builtin_convertvector(f32x2{v[0], v[1]}, bf16x2);
        const bf16x2 hi = __builtin_convertvector(f32x2{v[2], v[3]}, bf16x2);
        uint2 w;
        w.x = __builtin_bit_cast(unsigned, lo);
        w.y = __builtin_bit_cast(unsigned, hi);
        *reinterpret_cast<uint2 *>(p) = w;
    }
};

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
template <int F, bool ACCUMULATE = false>
__device__ inline void gemm_rl_bf16(const __bf16 *__restrict__ Ap, const f32x16 (&in)[Dims<F>::NB],
                                    f32x16 (&out)[Dims<F>::NB], int lane)
{
    constexpr int NB = Dims<F>::NB;
    const bf16x8 *A = reinterpret_cast<const bf16x8 *>(Ap) + lane;
    if (!ACCUMULATE)
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
template <int F, bool ACCUMULATE = false>
__device__ inline void gemm_row_bf16(const __bf16 *__restrict__ Ap, const float *row, f32x16 (&out)[Dims<F>::NB], int lane)
{
    constexpr int NB = Dims<F>::NB;
    const int h = lane >> 5;
    const bf16x8 *A = reinterpret_cast<const bf16x8 *>(Ap) + lane;
    if (!ACCUMULATE)
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
template <int F, bool ACCUMULATE = false>
__device__ inline void gemm_rl_f16x3(const _Float16 *__restrict__ Ap, const f32x16 (&in)[Dims<F>::NB],
                                     f32x16 (&out)[Dims<F>::NB], int lane)
{
    constexpr int NB = Dims<F>::NB;
    const f16x8 *Ah = reinterpret_cast<const f16x8 *>(Ap) + lane;
    const f16x8 *Al = reinterpret_cast<const f16x8 *>(Ap + F * F) + lane;
    if (!ACCUMULATE)
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

template <int F, bool ACCUMULATE = false>
__device__ inline void gemm_row_f16x3(const _Float16 *__restrict__ Ap, const float *row, f32x16 (&out)[Dims<F>::NB], int lane)
{
    constexpr int NB = Dims<F>::NB;
    const int h = lane >> 5;
    const f16x8 *Ah = reinterpret_cast<const f16x8 *>(Ap) + lane;
    const f16x8 *Al = reinterpret_cast<const f16x8 *>(Ap + F * F) + lane;
    if (!ACCUMULATE)
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

#endif  // MLIP_MODEL_TILES_H

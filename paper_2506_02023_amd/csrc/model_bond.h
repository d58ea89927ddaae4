// Kernels of the three-body (bond graph) variant.
// Part of model.hip (one translation unit): included inside namespace mlip, anonymous namespace.
#ifndef MLIP_MODEL_BOND_H
#define MLIP_MODEL_BOND_H

// ---------------------------------------------------------------- three-body (bond graph) kernels
//
// Benchmark configuration 4: bonds are the atom-graph edges within a smaller cutoff, two bonds interact when
// they share their centre atom (the paper's bond graph, Methods, "Distributing Bond Graphs").  All bonds of a
// centre are contiguous, so every kernel below works on one centre (or one bond) per wavefront with lane =
// feature and needs no atomics.  Notation: P_b = e0_b Wta, Q_b = e0_b Wtb, Wtc = rows 2F.. of Wt1,
//   h(b1, b2) = P_b1 + Q_b2 + T(c) Wtc,  S_b1 = sum_{b2 != b1} u_b2 SiLU(h),  m = S Wt2,  e1 = e0 + u SiLU(m).

//
// BT is the element type of the [bonds x F] arrays (P, Q, S, m, wb, e1bar, Sbar, Pbar, Qbar): float, or __bf16 in the
// bf16 precision mode, where these arrays are most of the bytes the bond kernels move.  Arithmetic is fp32 either way.

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

template <int F, typename BT>
__global__ void __launch_bounds__(256)
k_triplet_fwd(int64_t N, const int64_t *__restrict__ bptr, const float *__restrict__ rhat, const float *__restrict__ u,
              const BT *__restrict__ P, const BT *__restrict__ Q, const float *__restrict__ Wtc, BT *__restrict__ S)
{
    using IO = Elem<BT>;
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
            const float pa = IO::load(P + ba * F + f), qa = IO::load(Q + ba * F + f);
            const float ua = readlane_f32(ul, a);
            float T[kAngle], dT[kAngle];
            chebyshev(fmaf(readlane_f32(xl, a), xl, fmaf(readlane_f32(yl, a), yl, readlane_f32(zl, a) * zl)), T, dT);   // lane = o
            float acc = 0.f;
            for (int o = a + 1; o < nb; ++o) {
                float tw = wc[0];   // T_0 = 1
#pragma unroll
                for (int n = 1; n < kAngle; ++n) tw = fmaf(readlane_f32(T[n], o), wc[n], tw);
                const float po = IO::load(P + (b0 + o) * F + f), qo = IO::load(Q + (b0 + o) * F + f);
                const float so = accS[o * 64 + lane];   // per-lane slot (read early, written at the end of the step;
                                                        // LDS float atomics measured an order of magnitude slower)
                acc = fmaf(readlane_f32(ul, o), silu_f(pa + qo + tw), acc);       // triplet (b1 = a, b2 = o)
                accS[o * 64 + lane] = fmaf(ua, silu_f(po + qa + tw), so);        // triplet (b1 = o, b2 = a)
            }
            accS[a * 64 + lane] += acc;
        }
        wave_lds_fence();
        if (F == 64 || lane < F)
            for (int b = 0; b < nb; ++b) IO::store(S + (b0 + b) * F + f, accS[b * 64 + lane]);
        return;
    }
    // any number of bonds, no LDS: ordered pairs, bonds b2 in groups of 64
    for (int64_t c0 = b0; c0 < b1e; c0 += 64) {   // bonds b2 in groups of 64 (one group unless the centre has more)
        const int nl = (int)min((int64_t)64, b1e - c0);
        const int64_t bl = min(c0 + lane, b1e - 1);
        const float xl = rhat[3 * bl], yl = rhat[3 * bl + 1], zl = rhat[3 * bl + 2], ul = u[bl];
        for (int64_t b1 = b0; b1 < b1e; ++b1) {
            const float p1 = IO::load(P + b1 * F + f);
            const float x1 = rhat[3 * b1], y1 = rhat[3 * b1 + 1], z1 = rhat[3 * b1 + 2];
            float T[kAngle], dT[kAngle];
            chebyshev(fmaf(x1, xl, fmaf(y1, yl, z1 * zl)), T, dT);   // lane = b2
            float acc = 0.f;
            for (int k = 0; k < nl; ++k) {
                if (c0 + k == b1) continue;
                float h = p1 + IO::load(Q + (c0 + k) * F + f);
#pragma unroll
                for (int n = 1; n < kAngle; ++n) h = fmaf(readlane_f32(T[n], k), wc[n], h);   // T_0 = 1
                acc = fmaf(readlane_f32(ul, k), silu_f(h + wc[0]), acc);
            }
            if (F == 64 || lane < F) {
                BT *sp = S + b1 * F + f;
                IO::store(sp, (c0 == b0) ? acc : IO::load(sp) + acc);
            }
        }
    }
}

// bond term of a layer's aggregation: a[i] += sum over the bonds b = (i <- j) of wb[b] * g[j]
template <int F, typename BT>
__global__ void __launch_bounds__(256)
k_bond_aggregate(int64_t N, const int64_t *__restrict__ bptr, const int32_t *__restrict__ sender,
                 const BT *__restrict__ wb, const float *__restrict__ g, float *__restrict__ a)
{
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int64_t i = (int64_t)blockIdx.x * 4 + wave;
    if (i >= N) return;
    const int f = lane & (F - 1);
    float acc = 0.f;
    for (int64_t b = bptr[i]; b < bptr[i + 1]; ++b) acc = fmaf(Elem<BT>::load(wb + b * F + f), g[(int64_t)sender[b] * F + f], acc);
    if (F == 64 || lane < F) a[i * F + f] += acc;
}

// reverse of the bond term, the share of gbar: gbar[i] += sum_b wb[mirror(b)] * abar[j]
// (the reverse bond (j <- i) is the one whose filter multiplies g_i in row j)
template <int F, typename BT>
__global__ void __launch_bounds__(256)
k_bond_gbar(int64_t N, const int64_t *__restrict__ bptr, const int32_t *__restrict__ sender,
            const int32_t *__restrict__ bmirror, const BT *__restrict__ wb, const float *__restrict__ abar,
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
        if (bm >= 0) acc = fmaf(Elem<BT>::load(wb + bm * F + f), abar[j * F + f], acc);
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
template <int F, typename BT>
__device__ inline void
triplet_bwd_sweep(int64_t i, int lane, const int64_t *__restrict__ bptr, const float *__restrict__ rhat,
                  const float *__restrict__ u, const BT *__restrict__ P, const BT *__restrict__ Q,
                  const float *__restrict__ Wtc, const BT *__restrict__ Sbar, BT *__restrict__ Pbar,
                  BT *__restrict__ Qbar, float *__restrict__ ubar, float *__restrict__ rbar)
{
    using IO = Elem<BT>;
    const int f = lane & (F - 1);
    const bool on = (F == 64 || lane < F);
    float wc[kAngle];
#pragma unroll
    for (int n = 0; n < kAngle; ++n) wc[n] = Wtc[n * F + f];
    const int64_t b0 = bptr[i], be = bptr[i + 1];
    for (int64_t ba = b0; ba < be; ++ba) {
        const float xa = rhat[3 * ba], ya = rhat[3 * ba + 1], za = rhat[3 * ba + 2];
        const float pa = IO::load(P + ba * F + f), qa = IO::load(Q + ba * F + f), sa = IO::load(Sbar + ba * F + f), ua = u[ba];
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
            silu_both(pa + IO::load(Q + bo * F + f) + tw, s1, ds1);
            const float h1 = sa * u[bo] * ds1;
            pbar += h1;
            // triplet (b1 = bo, b2 = ba): contributes to Qbar[ba], ubar[ba] and, through c, to rbar[ba]
            float s2, ds2;
            const float so = IO::load(Sbar + bo * F + f);
            silu_both(IO::load(P + bo * F + f) + qa + tw, s2, ds2);
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
            IO::store(Pbar + ba * F + f, pbar);
            IO::store(Qbar + ba * F + f, qbar);
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
template <int F, typename BT>
__global__ void __launch_bounds__(256)
k_triplet_bwd(int64_t N, const int64_t *__restrict__ bptr, const float *__restrict__ rhat, const float *__restrict__ u,
              const BT *__restrict__ P, const BT *__restrict__ Q, const float *__restrict__ Wtc,
              const BT *__restrict__ Sbar, BT *__restrict__ Pbar, BT *__restrict__ Qbar,
              float *__restrict__ ubar, float *__restrict__ rbar)
{
    using IO = Elem<BT>;
    constexpr int NB = kPairBonds;
    __shared__ float acc_lds[4][3 * NB * 64 + NB * NB];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int64_t i = (int64_t)blockIdx.x * 4 + wave;
    if (i >= N) return;
    const int64_t b0 = bptr[i];
    const int n = (int)(bptr[i + 1] - b0);
    if (n > NB) {
        triplet_bwd_sweep<F, BT>(i, lane, bptr, rhat, u, P, Q, Wtc, Sbar, Pbar, Qbar, ubar, rbar);
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
        const float pa = IO::load(P + ba * F + f), qa = IO::load(Q + ba * F + f), sa = IO::load(Sbar + ba * F + f), ua = u[ba];
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
            const float po = IO::load(P + bo * F + f), qo = IO::load(Q + bo * F + f), so = IO::load(Sbar + bo * F + f), uo = u[bo];
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
            IO::store(Pbar + (b0 + b) * F + f, accP[b * 64 + lane]);
            IO::store(Qbar + (b0 + b) * F + f, accQ[b * 64 + lane]);
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
//   EBAR       e1bar = sum over the layers l of (abar_l,recv * g_l,send) Wb_l^T, each factor tile built in LDS from the
//              kept per-layer abar and g rows;  ubar = sum_f e1bar SiLU(m);  mbar = e1bar u SiLU'(m) (registers only);
//              Sbar = mbar Wt2^T
//   E0BAR      e0bar = e1bar + Pbar Wta^T + Qbar Wtb^T (registers only);
//              dbond = sum_f e0bar (We0^T dbbond/dd) + ubar du/dd
enum { BOND_HEAD = 0, BOND_TAIL = 1, BOND_EBAR = 2, BOND_E0BAR = 3 };

struct BondArgs {                      // one partition
    int64_t n;                         // bonds
    const float *d, *u, *du;           // [n] length, envelope at the bond cutoff, its derivative
    const int32_t *edge, *sender;      // [n] edge index, sender row of a bond
    const int32_t *recv;               // receiver row of an edge
    const float *We0p;                 // We0 packed for the K = 8 product (k_pack_w1)
    BasisParams bp;                    // radial basis at the bond cutoff
    const float *W[4];                 // packed F x F operands of the stage (TAIL: Wt2, then the first layers' Wb;
                                       // EBAR: Wt2^T, then the first layers' Wb^T)
    const float *Wx;                   // TAIL, EBAR: the packs of the layers beyond the third (read from global memory)
    int n_layers;                      // TAIL, EBAR
    size_t wb_stride;                  // TAIL: elements between two layers' wb
    // [bonds x F] arrays, elements of type BT (fp32, or bf16 in the bf16 mode)
    void *P, *Q;                       // HEAD out
    const void *S;                     // TAIL in
    void *m, *wb;                      // TAIL out; EBAR reads m
    const float *abar, *g;             // EBAR in: kept per-layer node rows, layer l at abar + l abar_stride, g + l g_stride
    size_t abar_stride, g_stride;
    void *e1bar;                       // EBAR out; E0BAR in (BT)
    float *ubar;                       // EBAR out; E0BAR in
    void *Sbar;                        // EBAR out (BT)
    const void *Pbar, *Qbar;           // E0BAR in (BT)
    float *dbond;                      // E0BAR out
};

template <int STAGE> struct BondStage {
    static constexpr bool PER_LAYER = (STAGE == BOND_TAIL || STAGE == BOND_EBAR);   // one operand pack per layer
    static constexpr int NW = PER_LAYER ? 8 : 4;   // wavefronts per block
    static constexpr int NPACK = PER_LAYER ? 4 : 2;
};

// PREC: the F x F products follow the precision mode of the filter MLP's (fp32 MFMA; bf16 operands; split-fp16 triples;
// packs prepared accordingly, activations converted in registers, fp32 accumulation); the K = 8 products stay fp32.
// The [bonds x F] arrays are bf16 in the bf16 mode and fp32 otherwise.
template <int PREC> struct BondElem { typedef float type; };
template <> struct BondElem<kPrecBf16> { typedef __bf16 type; };

template <int F, int STAGE, int PREC>
__global__ void __launch_bounds__(BondStage<STAGE>::NW * 64) k_bond_mlp(BondArgs A)
{
    using D = Dims<F>;
    using BT = typename BondElem<PREC>::type;
    using IO = Elem<BT>;
    constexpr int NB = D::NB, FS = D::FS;
    constexpr int NW = BondStage<STAGE>::NW, NPACK = BondStage<STAGE>::NPACK;
    constexpr int LPR = TileRegs<F>::LPR, RPI = TileRegs<F>::RPI;
    extern __shared__ float lds[];
    float *packs = lds;
    float *tiles = packs + NPACK * D::PACKF;
    const int n_lds_layers = BondStage<STAGE>::PER_LAYER ? min(A.n_layers, 3) : 0;
    const int n_packs = BondStage<STAGE>::PER_LAYER ? 1 + n_lds_layers : NPACK;
    for (int q = 0; q < n_packs; ++q)   // (a bf16 pack fills the first half of its slot)
        for (int i = threadIdx.x; i < (PREC == kPrecBf16 ? D::PACKF / 2 : D::PACKF); i += NW * 64) packs[q * D::PACKF + i] = A.W[q][i];
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
    typedef typename IO::raw4 raw4;
    auto load_rows = [&](const void *Yv, int64_t row, bool ok, raw4 (&v)[NB][4]) {   // as loaded: widen at the use
        const BT *Y = static_cast<const BT *>(Yv);
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                v[b][a] = raw4{};
                if (ok) v[b][a] = IO::load4_raw(Y + row * F + 32 * b + 8 * a + 4 * h);
            }
    };
    auto store_rows = [&](void *Yv, int64_t row, bool ok, const f32x16 (&acc)[NB]) {
        BT *Y = static_cast<BT *>(Yv);
        if (ok)
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const f32x4 v = {acc[b][4 * a], acc[b][4 * a + 1], acc[b][4 * a + 2], acc[b][4 * a + 3]};
                    IO::store4(Y + row * F + 32 * b + 8 * a + 4 * h, v);
                }
    };

    // out (+)= M x, x a 32-bond tile in LDS (this lane's bond = tile row c32) or a tile held in accumulator layout
    auto mul_tile = [&](auto accumulate, const float *pack, const float *t, f32x16 (&out)[NB]) {
        constexpr bool ACC = decltype(accumulate)::value;
        if (PREC == kPrecBf16) gemm_row_bf16<F, ACC>(reinterpret_cast<const __bf16 *>(pack), t + c32 * FS, out, lane);
        else if (PREC == kPrecF16x3) gemm_row_f16x3<F, ACC>(reinterpret_cast<const _Float16 *>(pack), t + c32 * FS, out, lane);
        else gemm_lds<F, ACC>(pack, t, out, lane);
    };
    auto mul_regs = [&](const float *pack, const f32x16 (&in)[NB], f32x16 (&out)[NB]) {
        if (PREC == kPrecBf16) gemm_rl_bf16<F>(reinterpret_cast<const __bf16 *>(pack), in, out, lane);
        else if (PREC == kPrecF16x3) gemm_rl_f16x3<F>(reinterpret_cast<const _Float16 *>(pack), in, out, lane);
        else gemm_regs<F>(pack, in, out, lane);
    };
    using Fresh = std::false_type;
    using Add = std::true_type;

    TileRegs<F, BT> pre, pre2;
    int64_t ti = (int64_t)blockIdx.x * NW + wave;
    if (ti < n_tiles) {
        if (STAGE == BOND_TAIL) fetch_tile<F, BT>(pre, static_cast<const BT *>(A.S), ti * 32, A.n, lane);
        if (STAGE == BOND_E0BAR) fetch_tile<F, BT>(pre, static_cast<const BT *>(A.Pbar), ti * 32, A.n, lane);
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
            mul_regs(packs, e0, acc);
            store_rows(A.P, row, ok, acc);
            mul_regs(packs + D::PACKF, e0, acc);
            store_rows(A.Q, row, ok, acc);
        } else if (STAGE == BOND_TAIL) {
            stash_tile<F>(pre, tile, lane);
            wave_lds_fence();
            const float uc = ok ? A.u[row] : 0.f;
            const float dc = ok ? A.d[row] : A.bp.rc;
            if (more) fetch_tile<F, BT>(pre, static_cast<const BT *>(A.S), (ti + stride) * 32, A.n, lane);
            mul_tile(Fresh{}, packs, tile, acc);
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
                mul_regs(packs + (1 + l) * D::PACKF, e1, acc);
                store_rows(static_cast<BT *>(A.wb) + (size_t)l * A.wb_stride, row, ok, acc);
            }
            for (int l = 3; l < A.n_layers; ++l) {
                mul_regs(A.Wx + (size_t)(l - 3) * D::PACKF, e1, acc);
                store_rows(static_cast<BT *>(A.wb) + (size_t)l * A.wb_stride, row, ok, acc);
            }
        } else if (STAGE == BOND_EBAR) {
            raw4 mv[NB][4];
            load_rows(A.m, row, ok, mv);   // needed after the products
            const float uc = ok ? A.u[row] : 0.f;
            int32_t ri[32 / RPI], rj[32 / RPI];   // receiver and sender rows of this lane's tile rows
#pragma unroll
            for (int r = 0; r < 32; r += RPI) {
                const int64_t rw = row0 + r + rr;
                ri[r / RPI] = rj[r / RPI] = -1;
                if (rw < A.n) {
                    ri[r / RPI] = A.recv[A.edge[rw]];
                    rj[r / RPI] = A.sender[rw];
                }
            }
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[b][r] = 0.f;
            auto factor_tile = [&](int l) {   // dE/dwb_l of the tile's bonds = abar_l[receiver] * g_l[sender]
                const float *al = A.abar + (size_t)l * A.abar_stride, *gl = A.g + (size_t)l * A.g_stride;
#pragma unroll
                for (int r = 0; r < 32; r += RPI) {
                    f32x4 v = {0.f, 0.f, 0.f, 0.f};
                    if (ri[r / RPI] >= 0)
                        v = *reinterpret_cast<const f32x4 *>(al + (int64_t)ri[r / RPI] * F + cc) *
                            *reinterpret_cast<const f32x4 *>(gl + (int64_t)rj[r / RPI] * F + cc);
                    *reinterpret_cast<f32x4 *>(tile + (r + rr) * FS + cc) = v;
                }
                wave_lds_fence();
            };
            for (int l = 0; l < n_lds_layers; ++l) {
                factor_tile(l);
                mul_tile(Add{}, packs + (1 + l) * D::PACKF, tile, acc);
                wave_lds_fence();
            }
            for (int l = 3; l < A.n_layers; ++l) {
                factor_tile(l);
                mul_tile(Add{}, A.Wx + (size_t)(l - 3) * D::PACKF, tile, acc);
                wave_lds_fence();
            }
            store_rows(A.e1bar, row, ok, acc);
            float part = 0.f;
            f32x16 mb[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float sv, ds;
                    silu_both(IO::widen4(mv[b][r / 4])[r % 4], sv, ds);
                    part = fmaf(acc[b][r], sv, part);
                    mb[b][r] = acc[b][r] * uc * ds;
                }
            part += __shfl_xor(part, 32, 64);
            if (ok && h == 0) A.ubar[row] = part;
            mul_regs(packs, mb, acc);
            store_rows(A.Sbar, row, ok, acc);
        } else {   // BOND_E0BAR
            stash_tile<F>(pre, tile, lane);
            wave_lds_fence();
            fetch_tile<F, BT>(pre2, static_cast<const BT *>(A.Qbar), row0, A.n, lane);   // in flight during the first product
            raw4 zv[NB][4];
            load_rows(A.e1bar, row, ok, zv);
            mul_tile(Fresh{}, packs, tile, acc);
            wave_lds_fence();
            stash_tile<F>(pre2, tile, lane);
            wave_lds_fence();
            if (more) fetch_tile<F, BT>(pre, static_cast<const BT *>(A.Pbar), (ti + stride) * 32, A.n, lane);
            mul_tile(Add{}, packs + D::PACKF, tile, acc);
            wave_lds_fence();
            float bb[8], db[8];
            radial_basis<true>(ok ? A.d[row] : A.bp.rc, A.bp, bb, db);
            f32x16 vv[NB];   // We0^T dbbond/dd
            gemm_k8r<F>(W0, db, vv, lane);
            float part = 0.f;
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) part = fmaf(IO::widen4(zv[b][r / 4])[r % 4] + acc[b][r], vv[b][r], part);
            part += __shfl_xor(part, 32, 64);
            if (ok && h == 0) A.dbond[row] = fmaf(A.ubar[row], A.du[row], part);
        }
    }
}

#endif  // MLIP_MODEL_BOND_H

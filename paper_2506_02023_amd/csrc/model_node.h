// Node kernels (F x F products over atoms) and the small kernels: embedding, ghost transfers, forces, energy.
// Part of model.hip (one translation unit): included inside namespace mlip, anonymous namespace.
#ifndef MLIP_MODEL_NODE_H
#define MLIP_MODEL_NODE_H

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
template <int F, typename T_ = float> struct TileRegs {
    static constexpr int LPR = F / 4;        // lanes per row (four elements each)
    static constexpr int RPI = 64 / LPR;     // rows per wave instruction
    typename Elem<T_>::raw4 v[32 / RPI];     // as loaded; widened to fp32 when the tile goes to LDS
};

template <int F, typename T_>
__device__ inline void fetch_tile(TileRegs<F, T_> &T, const T_ *__restrict__ X, int64_t row0, int64_t n_rows, int lane)
{
    constexpr int LPR = TileRegs<F>::LPR, RPI = TileRegs<F>::RPI;
    const int rr = lane / LPR, cc = (lane % LPR) * 4;
#pragma unroll
    for (int r = 0; r < 32; r += RPI) {
        const int64_t row = row0 + r + rr;
        typename Elem<T_>::raw4 v = {};   // all-zero bits are 0.0 in either type
        if (row < n_rows) v = Elem<T_>::load4_raw(X + row * F + cc);
        T.v[r / RPI] = v;
    }
}

template <int F, typename T_> __device__ inline void stash_tile(const TileRegs<F, T_> &T, float *tile, int lane)
{
    constexpr int FS = Dims<F>::FS;
    constexpr int LPR = TileRegs<F>::LPR, RPI = TileRegs<F>::RPI;
    const int rr = lane / LPR, cc = (lane % LPR) * 4;
#pragma unroll
    for (int r = 0; r < 32; r += RPI) *reinterpret_cast<f32x4 *>(tile + (r + rr) * FS + cc) = Elem<T_>::widen4(T.v[r / RPI]);
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
//
// Embedding, ghost transfers, force assembly and the energy partial sums run over all partitions in one launch
// (up to kBatch partitions per launch, like the edge and node kernels): items are numbered across the
// partitions, start[q] is the first item of partition q.

struct SmallArgs {   // one partition
    int64_t n_owned, n_pure, n_ghost, n_local;
    const int32_t *nodes;          // local -> global (nullptr: identity)
    const int32_t *ghost_owner, *ghost_src;
    const int64_t *row_ptr;
    const int32_t *senders, *mirror;
    const uint32_t *shiftp;
    float *h, *g, *gbar, *abar, *floc, *eps;
    float *a;                      // the layer's receiver sums (second pass of the pair-wise forward step)
    // upper / lower split of the owned rows' edges (or nullptr: kept filter values sit at the edges' own indices)
    const int32_t *wslot;          // [E_owned] upper edges: their index in the upper-edge graph, where their filter values are kept
    const int64_t *l_row_ptr;      // the owned rows' lower edges: CSR, sender row, where the pair's filter values are kept
    const int32_t *l_senders, *l_slot;
    const float *dsum, *wstore, *d;
    const int32_t *bond_of_edge;   // three-body variant (or nullptr)
    const void *wb;                // bond filter rows of the layer: fp32, or bf16 if wb_bf16
    int wb_bf16;
    double *energy_part;
};

struct SmallBatch {
    int n;
    int first;                     // partition index of s[0]
    int64_t start[kBatch + 1];
    SmallArgs s[kBatch];
};

struct PtrTable { float *p[kMaxSlabs]; };

// What a border atom's owner needs to collect the atom's ghost rows from the other partitions: the partitions that
// hold it as a ghost (bits of needed_by) and its row in each of them (ghost_local, starting at gbase[atom]).
struct GhostIndex {
    const unsigned long long *needed_by;
    const int32_t *gbase, *ghost_local;
};

__global__ void k_embed(SmallBatch B, int F, const int32_t *__restrict__ species, const float *__restrict__ emb)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // one float4 per thread
    const int F4 = F / 4;
    const int64_t row = idx / F4;
    if (row >= B.start[B.n]) return;
    const int part = batch_find(B.start, B.n, row);
    const SmallArgs &A = B.s[part];
    const int64_t r = row - B.start[part];
    const int c = (int)(idx % F4) * 4;
    const int64_t u = A.nodes ? A.nodes[r] : r;
    const float *e = emb + (int64_t)species[u] * F + c;   // the caller's table: no alignment assumed
    *reinterpret_cast<f32x4 *>(A.h + r * F + c) = f32x4{e[0], e[1], e[2], e[3]};
}

// ghost rows of every partition's g  <-  the owners' rows (tab: the g arrays of all partitions)
__global__ void k_ghost_copy(SmallBatch B, int F, PtrTable tab)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int F4 = F / 4;
    const int64_t gk = idx / F4;
    if (gk >= B.start[B.n]) return;
    const int part = batch_find(B.start, B.n, gk);
    const SmallArgs &A = B.s[part];
    const int64_t k = gk - B.start[part];
    const int c = (int)(idx % F4) * 4;
    const float *sp = tab.p[A.ghost_owner[k]] + (int64_t)A.ghost_src[k] * F + c;
    *reinterpret_cast<f32x4 *>(A.g + (A.n_owned + k) * F + c) = *reinterpret_cast<const f32x4 *>(sp);
}

// ghost rows of abar are zero (ghost rows carry no dE/da)
__global__ void k_zero_ghost_rows(SmallBatch B, int F)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int F4 = F / 4;
    const int64_t gk = idx / F4;
    if (gk >= B.start[B.n]) return;
    const int part = batch_find(B.start, B.n, gk);
    const SmallArgs &A = B.s[part];
    const int64_t k = gk - B.start[part];
    *reinterpret_cast<f32x4 *>(A.abar + (A.n_owned + k) * F + (idx % F4) * 4) = f32x4{0.f, 0.f, 0.f, 0.f};
}

// gbar of the ghost rows: gbar_i = sum over the ghost's sub-row (its neighbours owned by this partition) of
// w_e * abar_send(e).  w_e is the reverse edge's, which the forward pass kept (both edges of a pair have the
// same length, hence the same filter value).  One wavefront per row, lane = feature, edges in row order.
// Second pass of the edge steps that run on the upper-edge graphs: the lower edges' terms of the row sums, with the
// filter values w read from the row of the edge's pair, which the forward edge kernel (on the upper-edge graph) filled.
//   forward: a_i    += sum over the lower edges e = (i <- j) of row i of  w * g_j
//   REVERSE: gbar_i += sum over the same edges of                         w * abar_j  One wavefront per row, lane = feature; the
// lower edges of 64 edges at a time are taken kLowerChunk at a time, all their rows in flight together.
constexpr int kLowerChunk = 16;   // lower edges whose rows are in flight together (32 measured no faster)

template <int F, bool REVERSE>
__global__ void __launch_bounds__(256) k_edge_lower(SmallBatch B)
{
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int64_t gk = (int64_t)blockIdx.x * 4 + wave;
    if (gk >= B.start[B.n]) return;
    const int part = batch_find(B.start, B.n, gk);
    const SmallArgs &A = B.s[part];
    const int64_t r = gk - B.start[part];
    const unsigned f = lane & (F - 1);
    // the row's lower edges (wave-uniform, kept scalar; edge indices fit 32 bits)
    const int64_t e0 = __builtin_amdgcn_readfirstlane((int32_t)A.l_row_ptr[r]);
    const int64_t e1 = __builtin_amdgcn_readfirstlane((int32_t)A.l_row_ptr[r + 1]);
    float acc = 0.f;
    for (int64_t eb = e0; eb < e1; eb += 64) {
        const int n = (int)min((int64_t)64, e1 - eb);
        const int64_t el = min(eb + lane, e1 - 1);
        const int32_t jl = A.l_senders[el];
        const int32_t sl = A.l_slot[el];   // where the pair's filter values are kept
        for (int c = 0; c < n; c += kLowerChunk) {
            float wv[kLowerChunk], gv[kLowerChunk];
#pragma unroll
            for (int t = 0; t < kLowerChunk; ++t) {
                wv[t] = gv[t] = 0.f;
                if (c + t < n) {   // wave-uniform: no load is issued for an edge that is not there
                    const int64_t j = __builtin_amdgcn_readlane(jl, c + t), m = __builtin_amdgcn_readlane(sl, c + t);
                    wv[t] = __builtin_nontemporal_load(A.wstore + m * F + f);
                    gv[t] = (REVERSE ? A.abar : A.g)[j * F + f];
                }
            }
#pragma unroll
            for (int t = 0; t < kLowerChunk; ++t) acc = fmaf(wv[t], gv[t], acc);
        }
    }
    if (F == 64 || lane < F) (REVERSE ? A.gbar : A.a)[r * F + f] += acc;
}

template <int F>
__global__ void __launch_bounds__(256) k_ghost_gbar(SmallBatch B)
{
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int64_t gk = (int64_t)blockIdx.x * 4 + wave;
    if (gk >= B.start[B.n]) return;
    const int part = batch_find(B.start, B.n, gk);
    const SmallArgs &A = B.s[part];
    const int64_t r = A.n_owned + (gk - B.start[part]);
    const unsigned f = lane & (F - 1);
    const int64_t e0 = A.row_ptr[r], e1 = A.row_ptr[r + 1];
    float acc = 0.f;
    for (int64_t eb = e0; eb < e1; eb += 16) {   // 16 edges at a time: ids by lane, then all rows in flight together
        const int n = (int)min((int64_t)16, e1 - eb);
        const int64_t el = min(eb + (lane & 15), e1 - 1);
        const int32_t jl = A.senders[el], ml = A.mirror[el];
        const int32_t bl = A.bond_of_edge ? A.bond_of_edge[ml] : -1;   // three-body variant: the reverse edge's bond
        const int32_t sl = A.wslot ? A.wslot[ml] : ml;                 // where the reverse edge's filter values are kept
        float wv[16], av[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const int64_t j = __builtin_amdgcn_readlane(jl, k), m = __builtin_amdgcn_readlane(sl, k);
            const int64_t b = __builtin_amdgcn_readlane(bl, k);
            wv[k] = A.wstore[m * F + f];
            if (b >= 0)
                wv[k] += A.wb_bf16 ? Elem<__bf16>::load(static_cast<const __bf16 *>(A.wb) + b * F + f)
                                   : static_cast<const float *>(A.wb)[b * F + f];
            av[k] = A.abar[j * F + f];
        }
#pragma unroll
        for (int k = 0; k < 16; ++k)
            if (k < n) acc = fmaf(wv[k], av[k], acc);
    }
    if (F == 64 || lane < F) A.gbar[r * F + f] = acc;
}

// Ghost-row gradients go back to the owners (the reverse of the border-node transfer): every border row adds the
// rows its atom has as a ghost in the other partitions, in ascending partition order.  Gathered from the owner's
// side, so one launch covers all partitions without two writers on a row (tab: the gbar arrays of all partitions).
__global__ void k_border_add(SmallBatch B, int F, PtrTable tab, GhostIndex G)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int F4 = F / 4;
    const int64_t bk = idx / F4;
    if (bk >= B.start[B.n]) return;
    const int part = batch_find(B.start, B.n, bk);
    const SmallArgs &A = B.s[part];
    const int64_t r = A.n_pure + (bk - B.start[part]);
    const int c = (int)(idx % F4) * 4;
    const int32_t u = A.nodes[r];
    unsigned long long nb = G.needed_by[u];
    const int32_t *loc = G.ghost_local + G.gbase[u];
    float *dp = A.gbar + r * F + c;
    f32x4 v = *reinterpret_cast<const f32x4 *>(dp);
    while (nb) {
        const int qq = __builtin_ctzll(nb);
        nb &= nb - 1;
        v += *reinterpret_cast<const f32x4 *>(tab.p[qq] + (int64_t)(*loc++) * F + c);
    }
    *reinterpret_cast<f32x4 *>(dp) = v;
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

__device__ inline void unpack_shift(uint32_t p, int &a, int &b, int &c)
{
    a = (int)(p >> 20) - 512;
    b = (int)((p >> 10) & 1023u) - 512;
    c = (int)(p & 1023u) - 512;
}

// F_loc[r] = sum_{e in local row r} dsum_e * rhat_e, edge vectors from fp64 positions; 16 lanes per row, 16 rows per block
__global__ void __launch_bounds__(256)
k_force_rows(SmallBatch B, const double *__restrict__ pos, CellParams cp)
{
    const int64_t gr = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
    if (gr >= B.start[B.n]) return;   // whole groups of 16 lanes leave together; the shuffles below stay inside a group
    const int part = batch_find(B.start, B.n, gr);
    const SmallArgs &A = B.s[part];
    const int64_t r = gr - B.start[part];
    const int32_t *nodes = A.nodes;
    const int64_t ig = nodes ? nodes[r] : r;
    const double xi = pos[3 * ig], yi = pos[3 * ig + 1], zi = pos[3 * ig + 2];
    double fx = 0, fy = 0, fz = 0;
    const int64_t e1 = A.row_ptr[r + 1];
    for (int64_t e = A.row_ptr[r] + (threadIdx.x & 15); e < e1; e += 16) {
        const int64_t jl = A.senders[e];
        const int64_t jg = nodes ? nodes[jl] : jl;
        int S0, S1, S2;
        unpack_shift(A.shiftp[e], S0, S1, S2);
        const double t0 = (pos[3 * jg] - xi) + (((double)S0 * cp.C[0] + (double)S1 * cp.C[3]) + (double)S2 * cp.C[6]);
        const double t1 = (pos[3 * jg + 1] - yi) + (((double)S0 * cp.C[1] + (double)S1 * cp.C[4]) + (double)S2 * cp.C[7]);
        const double t2 = (pos[3 * jg + 2] - zi) + (((double)S0 * cp.C[2] + (double)S1 * cp.C[5]) + (double)S2 * cp.C[8]);
        // dE/dd times the unit vector: the edge's stored length (the fp64 length rounded once to fp32) is accurate
        // to 6e-8, far inside the force bound, and spares an fp64 square root and division per edge
        const double s = (double)(A.dsum[e] * __builtin_amdgcn_rcpf(A.d[e]));
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
        A.floc[3 * r] = (float)fx;
        A.floc[3 * r + 1] = (float)fy;
        A.floc[3 * r + 2] = (float)fz;
    }
}

__global__ void k_zero_floc(SmallBatch B)
{
    const int64_t gr = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gr >= B.start[B.n]) return;
    const int part = batch_find(B.start, B.n, gr);
    const int64_t r = gr - B.start[part];
    float *f = B.s[part].floc + 3 * r;
    f[0] = 0.f;
    f[1] = 0.f;
    f[2] = 0.f;
}

// owned rows: forces[global] = F_loc (+ for a border atom, in ascending partition order, the position gradients its
// ghost rows collected in the other partitions: gathered by the owner, one writer per atom); atom_energy[global] = eps
// (tab: the floc arrays of all partitions)
__global__ void k_store_owned(SmallBatch B, PtrTable tab, GhostIndex G, float *__restrict__ forces,
                              float *__restrict__ atom_energy)
{
    const int64_t gr = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gr >= B.start[B.n]) return;
    const int part = batch_find(B.start, B.n, gr);
    const SmallArgs &A = B.s[part];
    const int64_t r = gr - B.start[part];
    const int64_t u = A.nodes ? A.nodes[r] : r;
    float fx = A.floc[3 * r], fy = A.floc[3 * r + 1], fz = A.floc[3 * r + 2];
    if (r >= A.n_pure) {
        unsigned long long nb = G.needed_by[u];
        const int32_t *loc = G.ghost_local + G.gbase[u];
        while (nb) {
            const int qq = __builtin_ctzll(nb);
            nb &= nb - 1;
            const float *fg = tab.p[qq] + 3 * (int64_t)(*loc++);
            fx += fg[0];
            fy += fg[1];
            fz += fg[2];
        }
    }
    forces[3 * u] = fx;
    forces[3 * u + 1] = fy;
    forces[3 * u + 2] = fz;
    if (atom_energy) atom_energy[u] = A.eps[r];
}

// fixed-shape fp64 reduction of the per-atom energies: 1024-element blocks, then one block over the partials
__global__ void __launch_bounds__(256) k_energy_partial(SmallBatch B, double *__restrict__ part)
{
    __shared__ double sh[4];
    // start[] counts 1024-element blocks here; the partial sums of all partitions sit one after another in `part`
    const int q = batch_find(B.start, B.n, (int64_t)blockIdx.x);
    const int64_t n = B.s[q].n_owned;
    const float *eps = B.s[q].eps;
    const int64_t base = ((int64_t)blockIdx.x - B.start[q]) * 1024;
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

#endif  // MLIP_MODEL_NODE_H

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
#include <cstring>
#include <type_traits>

namespace mlip {

namespace {

#include "model_tiles.h"
#include "model_edge.h"
#include "model_node.h"
#include "model_bond.h"

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

// Dynamic LDS size of a kernel, set once per handle (a handle lives on one device and is used by one thread at a
// time, so this state needs no lock and is right for the device the handle's memory is on).  Returns the slot of
// the kernel in g->fn_occ, whose second member caches the resident blocks per compute unit (0: not queried).
int configure_kernel(mlip_graph *g, const void *fn, size_t lds, int *slot)
{
    for (size_t k = 0; k < g->fn_occ.size(); ++k)
        if (g->fn_occ[k].first == fn) { *slot = (int)k; return MLIP_OK; }
    MLIP_HIP(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    g->fn_occ.emplace_back(fn, 0);
    *slot = (int)g->fn_occ.size() - 1;
    return MLIP_OK;
}

__global__ void k_fill_zero(float *p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.f;
}

// zero-fill with a kernel (not hipMemsetAsync: memset nodes of a captured stream have misbehaved on replay)
int fill_zero(float *p, int64_t n, hipStream_t s)
{
    if (n <= 0) return MLIP_OK;
    k_fill_zero<<<blocks_for(n, 256), 256, 0, s>>>(p, n);
    MLIP_HIP(hipGetLastError());
    return MLIP_OK;
}

template <int F, int OP> int launch_node(mlip_graph *g, NodeBatch &b)
{
    constexpr bool TWO = (OP == OP_READOUT || OP == OP_BWD_UPDATE);
    const size_t lds = TWO ? Lds<F>::node2 : Lds<F>::node1;
    int slot = 0;
    MLIP_TRY(configure_kernel(g, reinterpret_cast<const void *>(&k_node<F, OP>), lds, &slot));
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

template <int F, int STAGE, int PREC> int launch_bond_mlp(mlip_graph *g, const BondArgs &a)
{
    constexpr int NW = BondStage<STAGE>::NW;
    constexpr size_t lds = sizeof(float) * (BondStage<STAGE>::NPACK * Dims<F>::PACKF + NW * Dims<F>::TILE);
    int slot = 0;
    MLIP_TRY(configure_kernel(g, reinterpret_cast<const void *>(&k_bond_mlp<F, STAGE, PREC>), lds, &slot));
    if (a.n <= 0) return MLIP_OK;
    const int64_t n_tiles = (a.n + 31) / 32;
    // each block keeps its operand packs in LDS, so let it walk several tiles
    const unsigned blocks = (unsigned)std::min<int64_t>((n_tiles + NW - 1) / NW, 8192 / NW);
    k_bond_mlp<F, STAGE, PREC><<<blocks, NW * 64, lds, g->stream>>>(a);
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

// Edge-kernel launches of one call: two per layer and batch of partitions (L <= 8, at most 64 / kBatch batches).
constexpr int kWorkLaunches = 2 * 8 * (64 / kBatch);

// The reverse edge kernel the library runs is the one whose wavefronts alternate between the two phases.  Building
// with -DMLIP_BWD_SIMD runs the fp32 mode's launches on the upper-edge graphs with the variant whose phases sit on
// different SIMDs instead (same results; measured slightly slower, kept for that experiment).
constexpr bool kUpperGraphs = true;
template <int F, int PREC, bool COMPACT> struct BwdKernel {
    static constexpr int threads = kBwdWaves * 64, item_waves = kBwdWaves;
    static constexpr size_t lds = Lds<F>::edge_bwd;
    static const void *fn() { return reinterpret_cast<const void *>(&k_edge_bwd<F, PREC, COMPACT>); }
    static void launch(unsigned blocks, hipStream_t s, const EdgeBatch &b)
    {
        k_edge_bwd<F, PREC, COMPACT><<<blocks, threads, lds, s>>>(b);
    }
};
#ifdef MLIP_BWD_SIMD
template <int F> struct BwdKernel<F, kPrecF32, true> {
    static constexpr int threads = kSimdWaves * 64, item_waves = kSimdStream;
    static constexpr size_t lds = BwdSimdLds<F>::bytes;
    static const void *fn() { return reinterpret_cast<const void *>(&k_edge_bwd_simd<F>); }
    static void launch(unsigned blocks, hipStream_t s, const EdgeBatch &b) { k_edge_bwd_simd<F><<<blocks, threads, lds, s>>>(b); }
};
#endif

enum { kEdgeFwd = 0, kEdgeBwd = 1, kEdgeBwdUpper = 2 };   // kEdgeBwdUpper: the launch runs on upper-edge graphs

template <int F, int PREC, bool COMPACT = false> int launch_edge(mlip_graph *g, EdgeBatch &b, int kind)
{
    if (kind == kEdgeBwdUpper && !COMPACT) return launch_edge<F, PREC, true>(g, b, kind);
    using BK = BwdKernel<F, PREC, COMPACT>;
    const bool backward = (kind != kEdgeFwd);
    const size_t lds = backward ? BK::lds : Lds<F>::edge_fwd;
    // resident blocks per compute unit, queried once per kernel and handle
    const void *fn = backward ? BK::fn() : reinterpret_cast<const void *>(&k_edge_fwd<F, PREC>);
    int slot = 0;
    MLIP_TRY(configure_kernel(g, fn, lds, &slot));
    int occ = g->fn_occ[slot].second;
    if (occ == 0) {
        int dev = 0, o = 0;
        MLIP_HIP(hipGetDevice(&dev));
        MLIP_HIP(hipDeviceGetAttribute(&g->n_cu, hipDeviceAttributeMultiprocessorCount, dev));
        if (backward)
            MLIP_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&o, fn, BK::threads, lds));
        else
            MLIP_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&o, k_edge_fwd<F, PREC>, 256, lds));
        if (o < 1 || g->n_cu < 8) {
            set_error("edge kernel does not fit the device (occupancy %d, %d compute units)", o, g->n_cu);
            return MLIP_EHIP;
        }
        occ = g->fn_occ[slot].second = o;
    }
    if (g->work_next >= kWorkLaunches) {
        set_error("more than %d edge-kernel launches in one call", kWorkLaunches);
        return MLIP_ESTATE;
    }
    b.work = g->work_ptr + (size_t)g->work_next * (8 * kWorkCounterStride);
    b.chunk_start[0] = 0;
    for (int q = 0; q < b.n; ++q) b.chunk_start[q + 1] = b.chunk_start[q] + (b.s[q].n_rows > 0 ? b.s[q].n_chunks : 0);
    for (int q = b.n; q < kBatch; ++q) b.chunk_start[q + 1] = b.chunk_start[b.n];
    const int64_t items = b.chunk_start[b.n];
    if (items <= 0) return MLIP_OK;
    // persistent grid: what is resident at once, a multiple of the 8 XCDs, no more than the work needs
    const int64_t resident = (int64_t)(g->n_cu / 8) * occ;
    const int nw = backward ? BK::item_waves : 4;
    const int64_t needed = ((items + 7) / 8 + nw - 1) / nw;
    const unsigned blocks = (unsigned)(8 * std::max<int64_t>(1, std::min(resident, needed)));
    if (backward)
        BK::launch(blocks, g->stream, b);
    else
        k_edge_fwd<F, PREC><<<blocks, 256, lds, g->stream>>>(b);
    MLIP_HIP(hipGetLastError());
    ++g->work_next;   // only a launch that ran has used its counters
    return MLIP_OK;
}

// Kept filter values shared by the two edges of a pair on the full edge lists: a lower edge reads its reverse edge's
// row through one buffer descriptor, whose 32-bit range (less the largest offset a load adds) must span the partition.
inline bool fits_pairs(const SlabView &v, int F) { return (int64_t)v.n_edges_owned * F * 4 < ((int64_t)1 << 32) - (1 << 20); }

// bw != nullptr: the three-body variant
template <int F>
int forward_t(mlip_graph *g, const mlip_weights_t *w, const mlip_bond_weights_t *bw, int32_t mode, double *energy,
              float *forces, float *atom_energy, Carver *scratch)
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
    // every array of the call either lives in the view's own grow-only buffer or is carved from the fixed block
    auto place = [&](DevBuf &buf, size_t bytes, float *&ptr) -> int {
        if (scratch) {
            ptr = static_cast<float *>(scratch->take(bytes));
            return MLIP_OK;   // a failed carve is reported once, below
        }
        MLIP_TRY(buf.ensure(bytes));
        ptr = buf.as<float>();
        return MLIP_OK;
    };
    // With fp32 MFMA the edge kernels run on the partitions' upper-edge graphs (one edge per edge / reverse-edge pair:
    // both edges have the same length, hence bit for bit the same filter values), and row-wise kernels add the lower
    // edges' terms.  In the 16-bit product modes the matrix work is cheap and the forward step is faster on the full edge lists.
    const bool upper = kUpperGraphs && prec == kPrecF32;
    // Their reverse step, though, streams three rows per edge whatever the precision: it runs on the upper-edge graphs in
    // those modes too wherever the pairs share their kept filter values (fits_pairs), which then stay where the
    // forward step on the full lists put them, at the upper edges' own positions.
    bool upper_bwd = upper;
    if (kUpperGraphs && prec != kPrecF32 && L > 1) {
        upper_bwd = true;
        for (int p = 0; p < P; ++p) upper_bwd = upper_bwd && fits_pairs(views[p], F);
    }
    if (upper_bwd) {
        prof_begin(g, MLIP_PROF_GRAPH);
        MLIP_TRY(build_pairs_impl(g, views, P, /*slots_full=*/!upper, scratch));
        prof_end(g);
    }
    int64_t n_parts = 0;
    for (int p = 0; p < P; ++p) {
        SlabView &v = views[p];
        const size_t no = (size_t)std::max<int64_t>(v.n_owned, 1), nl = (size_t)std::max<int64_t>(v.n_local, 1);
        MLIP_TRY(place(v.h, no * rowb, v.ws.h));
        MLIP_TRY(place(v.hbar, no * rowb, v.ws.hbar));
        MLIP_TRY(place(v.abar, nl * rowb, v.ws.abar));
        MLIP_TRY(place(v.gbar, nl * rowb, v.ws.gbar));
        MLIP_TRY(place(v.eps, no * sizeof(float), v.ws.eps));
        MLIP_TRY(place(v.dsum, (size_t)std::max<int64_t>(v.n_edges, 1) * sizeof(float), v.ws.dsum));
        MLIP_TRY(place(v.floc, nl * 3 * sizeof(float), v.ws.floc));
        MLIP_TRY(place(v.g, nl * rowb * (size_t)std::max(L, 1), v.ws.g));
        MLIP_TRY(place(v.a, no * rowb * (size_t)std::max(L, 1), v.ws.a));
        v.ws.wst = nullptr;
        if (L > 0)  // filter values of every layer: layers 1..L-1 are kept for the reverse pass instead of being recomputed,
                    // and on the upper-edge graphs every layer's second pass reads what its first pass kept
            MLIP_TRY(place(v.wst, (size_t)std::max<int64_t>(upper ? v.pairs.n_upper : v.n_edges_owned, 1) * rowb * (size_t)L,
                           v.ws.wst));
        n_parts += (v.n_owned + 1023) / 1024;
    }
    const Packs pk = pack_layout(F, L);
    float *wp = nullptr, *energy_part_f = nullptr;
    MLIP_TRY(place(g->energy_part, (size_t)std::max<int64_t>(n_parts, 1) * sizeof(double), energy_part_f));
    MLIP_TRY(place(g->wpack, pk.total * sizeof(float), wp));
    float *work_f = nullptr;
    const size_t work_n = (size_t)kWorkLaunches * 8 * kWorkCounterStride;
    MLIP_TRY(place(g->work, work_n * sizeof(int32_t), work_f));
    if (scratch && scratch->failed()) {
        set_error("this graph and model need more than the %zu bytes of static workspace", scratch->size);
        return MLIP_EINVAL;
    }
    double *energy_part = reinterpret_cast<double *>(energy_part_f);
    g->work_ptr = reinterpret_cast<int32_t *>(work_f);
    g->work_next = 0;
    MLIP_TRY(fill_zero(work_f, (int64_t)work_n, s));


    // rows of one layer's kept filter values
    auto wrows = [&](SlabView &v) { return (size_t)(upper ? v.pairs.n_upper : v.n_edges_owned); };

    // ---- batches for the small kernels (embedding, ghost transfers, forces, energy): up to kBatch partitions per launch
    enum { U_OWNED, U_GHOST, U_BORDER, U_LOCAL, U_KBLOCKS };
    auto small_batch = [&](int p0, int unit, int layer) {
        SmallBatch sb{};
        sb.n = std::min(kBatch, P - p0);
        sb.first = p0;
        sb.start[0] = 0;
        for (int q = 0; q < kBatch; ++q) {
            if (q >= sb.n) { sb.start[q + 1] = sb.start[q]; continue; }
            SlabView &v = views[p0 + q];
            SmallArgs &a = sb.s[q];
            a.n_owned = v.n_owned;
            a.n_pure = v.n_pure;
            a.n_ghost = v.n_ghost;
            a.n_local = v.n_local;
            a.nodes = v.nodes;
            a.ghost_owner = v.ghost_owner;
            a.ghost_src = v.ghost_src;
            a.row_ptr = v.row_ptr;
            a.senders = v.senders;
            a.mirror = v.mirror;
            a.shiftp = v.shiftp;
            a.h = v.ws.h;
            a.g = (layer >= 0) ? v.ws.g + (size_t)layer * (size_t)v.n_local * F : nullptr;
            a.gbar = v.ws.gbar;
            a.abar = v.ws.abar;
            a.floc = v.ws.floc;
            a.eps = v.ws.eps;
            a.dsum = v.ws.dsum;
            a.d = v.d;
            a.wstore = (layer >= 0 && v.ws.wst) ? v.ws.wst + (size_t)layer * wrows(v) * F : nullptr;
            a.wslot = upper ? v.pairs.wslot : nullptr;
            a.l_row_ptr = upper_bwd ? v.pairs.l_row_ptr : nullptr;
            a.l_senders = upper_bwd ? v.pairs.l_senders : nullptr;
            a.l_slot = upper_bwd ? v.pairs.l_slot : nullptr;
            a.a = (layer >= 0) ? v.ws.a + (size_t)layer * (size_t)v.n_owned * F : nullptr;
            a.bond_of_edge = (bw && v.bonds.n > 0) ? v.bonds.of_edge.as<int32_t>() : nullptr;
            a.wb_bf16 = (prec == kPrecBf16);
            a.wb = (bw && v.bonds.n > 0 && layer >= 0)
                       ? static_cast<char *>(v.bonds.wb.p) + (size_t)layer * (size_t)std::max<int64_t>(v.bonds.n, 1) * F *
                                                                   (a.wb_bf16 ? sizeof(__bf16) : sizeof(float))
                       : nullptr;
            const int64_t items = unit == U_OWNED ? v.n_owned : unit == U_GHOST ? v.n_ghost
                                  : unit == U_BORDER ? v.n_owned - v.n_pure : unit == U_LOCAL ? v.n_local
                                  : (v.n_owned + 1023) / 1024;
            sb.start[q + 1] = sb.start[q] + std::max<int64_t>(items, 0);
        }
        return sb;
    };
    GhostIndex gidx{};
    if (slabs) {
        gidx.needed_by = g->needed_by.as<unsigned long long>();
        gidx.gbase = g->part.gbase.as<int32_t>();
        gidx.ghost_local = g->part.ghost_local.as<int32_t>();
    }

    BasisParams bp;
    bp.rc = (float)g->r_cut;
    bp.inv_rc = (float)(1.0 / g->r_cut);
    bp.p = w->p;
    const double pd = (double)w->p;
    bp.pc0 = (float)(pd * (pd + 1) * (pd + 2) / 2);

    // ---- pack weights (kept in the handle until a call comes with a different weight struct; the fixed block of
    // the static variant is shared by all handles, so there they are packed on every call)
    prof_begin(g, MLIP_PROF_NODE);
    const unsigned pb = blocks_for((int64_t)F * F, 256);
    const bool repack = scratch != nullptr || !g->packed_w_valid || std::memcmp(&g->packed_w, w, sizeof(*w)) != 0;
    g->packed_w_valid = false;
    for (int l = 0; repack && l < L; ++l) {
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
    if (repack) {
        k_pack_ff<<<pb, 256, 0, s>>>(w->Wr1, F, 1, 1.0f, wp + pk.readout_t);
        k_pack_ff<<<pb, 256, 0, s>>>(w->Wr1, F, 0, 1.0f, wp + pk.readout_n);
    }
    MLIP_HIP(hipGetLastError());
    if (!scratch) {
        g->packed_w = *w;
        g->packed_w_valid = true;
    }

    // ---- embedding
    const int32_t *species = g->species.as<int32_t>();
    for (int p0 = 0; p0 < P; p0 += kBatch) {
        const SmallBatch sb = small_batch(p0, U_OWNED, -1);
        if (sb.start[sb.n] > 0)
            k_embed<<<blocks_for(sb.start[sb.n] * (F / 4), 256), 256, 0, s>>>(sb, F, species, w->emb);
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
    auto bstride = [&](SlabView &v) { return (size_t)std::max<int64_t>(v.bonds.n, 1) * F; };   // elements per [n][F] array
    // the [bonds x F] arrays are bf16 in the bf16 mode, fp32 otherwise
    const bool bond_bf16 = (prec == kPrecBf16);
    const size_t belem = bond_bf16 ? sizeof(__bf16) : sizeof(float);
    auto bond_elem = [&](auto &&launch) {   // calls launch with a value of the arrays' element type
        if (bond_bf16) launch((__bf16)0.0f);
        else launch(0.0f);
    };
    auto wbslice = [&](SlabView &v, int l) -> void * {
        return static_cast<char *>(v.bonds.wb.p) + (size_t)l * bstride(v) * belem;
    };
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
        a.P = BG.P.p;
        a.Q = BG.Q.p;
        a.S = BG.S.p;
        a.m = BG.m.p;
        a.wb = BG.wb.p;
        a.abar = BG.abar_keep.as<float>();
        a.abar_stride = (size_t)std::max<int64_t>(v.n_owned, 1) * F;
        a.g = v.ws.g;
        a.g_stride = (size_t)v.n_local * F;
        a.e1bar = BG.e1bar.p;
        a.ubar = BG.ubar.as<float>();
        a.Sbar = BG.Sbar.p;
        a.Pbar = BG.Pbar.p;
        a.Qbar = BG.Qbar.p;
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
            for (DevBuf *b : fb) MLIP_TRY(b->ensure(bs * belem));
            MLIP_TRY(BG.wb.ensure(bs * belem * (size_t)std::max(L, 1)));
            MLIP_TRY(BG.abar_keep.ensure((size_t)std::max<int64_t>(views[p].n_owned, 1) * rowb * (size_t)std::max(L, 1)));
            MLIP_TRY(BG.ubar.ensure(nb1 * sizeof(float)));
            MLIP_TRY(BG.dbond.ensure(nb1 * sizeof(float)));
            MLIP_TRY(BG.rbar.ensure(nb1 * 3 * sizeof(float)));
            any_bonds = any_bonds || BG.n > 0;
        }
        MLIP_TRY(g->bond_wpack.ensure(((size_t)(6 + 2 * L) * ffp + Dims<F>::PACK1) * sizeof(float)));
        bpk = g->bond_wpack.as<float>();
        prof_begin(g, MLIP_PROF_BOND);
        const float *Wta = bw->Wt1, *Wtb = bw->Wt1 + ffp, *Wtc = bw->Wt1 + 2 * ffp;
        const bool repack_b = !g->packed_bw_valid || std::memcmp(&g->packed_bw, bw, sizeof(*bw)) != 0 ||
                              std::memcmp(&g->packed_bw_w, w, sizeof(*w)) != 0;
        g->packed_bw_valid = false;
        // the bond MLPs' F x F products follow the filter MLP's precision mode: fp32 pack, bf16 in the first half of the
        // slot, or split-fp16 (hi and lo halves)
        auto pack_bond = [&](const float *Wsrc, int trans, int slot) {
            if (prec == kPrecBf16)
                k_pack_ff_bf16<<<pb, 256, 0, s>>>(Wsrc, F, trans, 1.0f, reinterpret_cast<__bf16 *>(bpk + (size_t)slot * ffp));
            else if (prec == kPrecF16x3)
                k_pack_ff_f16x2<<<pb, 256, 0, s>>>(Wsrc, F, trans, 1.0f, reinterpret_cast<_Float16 *>(bpk + (size_t)slot * ffp));
            else
                k_pack_ff<<<pb, 256, 0, s>>>(Wsrc, F, trans, 1.0f, bpk + (size_t)slot * ffp);
        };
        if (repack_b) {
            pack_bond(Wta, 1, 0);
            pack_bond(Wtb, 1, 1);
            pack_bond(bw->Wt2, 1, 2);
            pack_bond(Wta, 0, 3);
            pack_bond(Wtb, 0, 4);
            pack_bond(bw->Wt2, 0, 5);
            for (int l = 0; l < L; ++l) {
                pack_bond(bw->Wb + l * ffp, 1, 6 + l);
                pack_bond(bw->Wb + l * ffp, 0, 6 + L + l);
            }
            k_pack_w1<<<blocks_for(Dims<F>::PACK1, 256), 256, 0, s>>>(bw->We0, F, 1.0f, bpk + (size_t)(6 + 2 * L) * ffp);
        }
        MLIP_HIP(hipGetLastError());
        g->packed_bw = *bw;
        g->packed_bw_w = *w;
        g->packed_bw_valid = true;
        for (int p = 0; p < P; ++p) {   // P = e0 Wta, Q = e0 Wtb with e0 = bbond(d) We0
            BondArgs a = bond_args(views[p]);
            a.W[0] = bpk + 0 * ffp;
            a.W[1] = bpk + 1 * ffp;
            MLIP_TRY(prec == kPrecBf16 ? (launch_bond_mlp<F, BOND_HEAD, kPrecBf16>(g, a))
                     : prec == kPrecF16x3 ? (launch_bond_mlp<F, BOND_HEAD, kPrecF16x3>(g, a)) : (launch_bond_mlp<F, BOND_HEAD, kPrecF32>(g, a)));
        }
        prof_end(g);
        prof_begin(g, MLIP_PROF_TRIPLET_FWD);
        for (int p = 0; p < P; ++p) {
            SlabView &v = views[p];
            BondGraph &BG = v.bonds;
            if (BG.n > 0)
                bond_elem([&](auto zero) {
                    using BT = decltype(zero);
                    k_triplet_fwd<F, BT><<<blocks_for(v.n_owned, 4), 256, 0, s>>>(
                        v.n_owned, BG.ptr.as<int64_t>(), BG.rhat.as<float>(), BG.u.as<float>(), BG.P.as<BT>(), BG.Q.as<BT>(), Wtc,
                        BG.S.as<BT>());
                });
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
            MLIP_TRY(prec == kPrecBf16 ? (launch_bond_mlp<F, BOND_TAIL, kPrecBf16>(g, a))
                     : prec == kPrecF16x3 ? (launch_bond_mlp<F, BOND_TAIL, kPrecF16x3>(g, a)) : (launch_bond_mlp<F, BOND_TAIL, kPrecF32>(g, a)));
        }
        prof_end(g);
    }

    // Kept filter values on the full edge lists (16-bit product modes): both edges of a pair have the same ones bit for
    // bit, so only the upper edge keeps them and the lower edge's reverse step reads its reverse edge's row.  That halves
    // what the forward launches write, which is what bounds them there (1M-atom benchmark, split-fp16: forward
    // 3.23 -> 2.71 ms, reverse 4.02 -> 4.12 ms per launch).  Needs every partition of the launch to have its kept rows
    // within the 32-bit range of one buffer descriptor (otherwise every edge keeps its own); the same answer for the
    // forward and the reverse launch of a layer.
    auto w_pairs = [&](int p0, int n) {
        if (upper || prec == kPrecF32) return 0;   // upper-edge graphs keep one row per pair by construction
        for (int q = 0; q < n; ++q)
            if (!fits_pairs(views[p0 + q], F)) return 0;
        return 1;
    };
    auto gslice = [&](SlabView &v, int l) { return v.ws.g + (size_t)l * (size_t)v.n_local * F; };
    auto aslice = [&](SlabView &v, int l) { return v.ws.a + (size_t)l * (size_t)v.n_owned * F; };
    auto wslice = [&](SlabView &v, int l) {
        return v.ws.wst + (size_t)l * wrows(v) * F;
    };

    // ---- forward layers
    for (int l = 0; l < L; ++l) {
        const float *base = wp + pk.per_layer * l;
        prof_begin(g, MLIP_PROF_NODE);
        MLIP_TRY((node_pass<F, OP_PROJ>(g, views, P, base + pk.Wmt, nullptr, nullptr, [&](SlabView &v, NodeArgs &na) {
            na.n_rows = v.n_owned;   // sender projection on owned rows
            na.X = v.ws.h;
            na.Y = gslice(v, l);
        })));
        prof_end(g);
        if (slabs) {
            prof_begin(g, MLIP_PROF_GHOST);
            PtrTable tab{};
            for (int q = 0; q < P; ++q) tab.p[q] = gslice(views[q], l);
            for (int p0 = 0; p0 < P; p0 += kBatch) {   // border-node transfer: ghost rows <- owners
                const SmallBatch sb = small_batch(p0, U_GHOST, l);
                if (sb.start[sb.n] > 0)
                    k_ghost_copy<<<blocks_for(sb.start[sb.n] * (F / 4), 256), 256, 0, s>>>(sb, F, tab);
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
            eb.c.w_pairs = w_pairs(p0, eb.n);
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
                ea.mirror = v.mirror;
                ea.g = gslice(v, l);
                ea.out = aslice(v, l);
                ea.wstore = (l >= 1 || upper) ? wslice(v, l) : nullptr;
                if (upper) {   // the same kernel on the partition's upper-edge graph: row sums of the upper edges, every
                               // edge's filter values kept one after another
                    const PairGraph &Q = v.pairs;
                    ea.n_chunks = chunks_of(Q.n_upper);
                    ea.chunk_row = Q.u_chunk_row;
                    ea.row_ptr = Q.u_row_ptr;
                    ea.senders = Q.u_senders;
                    ea.recv = Q.u_recv;
                    ea.d = Q.u_d;
                    ea.mirror = nullptr;
                }
            }
            prof_begin(g, MLIP_PROF_EDGE_FWD);
            MLIP_TRY(prec == kPrecBf16 ? (launch_edge<F, kPrecBf16>(g, eb, kEdgeFwd))
                     : prec == kPrecF16x3 ? (launch_edge<F, kPrecF16x3>(g, eb, kEdgeFwd)) : (launch_edge<F, kPrecF32>(g, eb, kEdgeFwd)));
            prof_end(g);
            if (upper) {   // second pass: the lower edges' terms, with the filter values the first pass kept
                prof_begin(g, MLIP_PROF_EDGE_FWD_LOWER);
                const SmallBatch sb = small_batch(p0, U_OWNED, l);
                if (sb.start[sb.n] > 0)
                    k_edge_lower<F, false><<<blocks_for(sb.start[sb.n], 4), 256, 0, s>>>(sb);
                MLIP_HIP(hipGetLastError());
                prof_end(g);
            }
        }
        if (any_bonds) {   // bond term of the filters: a_i += sum_b wb_b * g_send(b)
            prof_begin(g, MLIP_PROF_BOND);
            for (int p = 0; p < P; ++p) {
                SlabView &v = views[p];
                if (v.bonds.n > 0)
                    bond_elem([&](auto zero) {
                        using BT = decltype(zero);
                        k_bond_aggregate<F, BT><<<blocks_for(v.n_owned, 4), 256, 0, s>>>(
                            v.n_owned, v.bonds.ptr.as<int64_t>(), v.bonds.sender.as<int32_t>(),
                            static_cast<const BT *>(wbslice(v, l)), gslice(v, l), aslice(v, l));
                    });
            }
            MLIP_HIP(hipGetLastError());
            prof_end(g);
        }
        prof_begin(g, MLIP_PROF_NODE);
        MLIP_TRY((node_pass<F, OP_UPDATE>(g, views, P, base + pk.Wot, nullptr, nullptr, [&](SlabView &v, NodeArgs &na) {
            na.n_rows = v.n_owned;
            na.X = aslice(v, l);
            na.Z = v.ws.h;
        })));
        prof_end(g);
    }

    // ---- readout (energy and dE/dh of the last layer in one pass)
    prof_begin(g, MLIP_PROF_NODE);
    MLIP_TRY((node_pass<F, OP_READOUT>(g, views, P, wp + pk.readout_t, wp + pk.readout_n, w->wr2,
                                       [&](SlabView &v, NodeArgs &na) {
                                           na.n_rows = v.n_owned;
                                           na.X = v.ws.h;
                                           na.Y = v.ws.hbar;
                                           na.eps = v.ws.eps;
                                       })));
    prof_end(g);
    prof_begin(g, MLIP_PROF_FORCE);
    {
        int64_t off = 0;
        double *part = energy_part;
        for (int p0 = 0; p0 < P; p0 += kBatch) {
            const SmallBatch sb = small_batch(p0, U_KBLOCKS, -1);
            const int64_t nb = sb.start[sb.n];
            if (nb > 0) k_energy_partial<<<(unsigned)nb, 256, 0, s>>>(sb, part + off);
            off += nb;
        }
        k_energy_final<<<1, 256, 0, s>>>(off, part, energy);
        MLIP_HIP(hipGetLastError());
    }
    prof_end(g);

    // ---- reverse pass
    if (L > 0)   // ghost rows carry no dE/da: zero once, no kernel ever writes them
        for (int p0 = 0; p0 < P; p0 += kBatch) {
            const SmallBatch sb = small_batch(p0, U_GHOST, -1);
            if (sb.start[sb.n] > 0)
                k_zero_ghost_rows<<<blocks_for(sb.start[sb.n] * (F / 4), 256), 256, 0, s>>>(sb, F);
        }
    MLIP_HIP(hipGetLastError());
    for (int l = L - 1; l >= 0; --l) {
        const float *base = wp + pk.per_layer * l;
        const bool need_gbar = l > 0;  // dE/dh0 is never used: the embedding does not depend on positions
        prof_begin(g, MLIP_PROF_NODE);
        MLIP_TRY((node_pass<F, OP_BWD_UPDATE>(g, views, P, base + pk.Wot, base + pk.Won, nullptr,
                                              [&](SlabView &v, NodeArgs &na) {
                                                  na.n_rows = v.n_owned;
                                                  na.X = aslice(v, l);
                                                  na.Z = v.ws.hbar;
                                                  na.Y = v.ws.abar;
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
            eb.c.w_pairs = w_pairs(p0, eb.n);
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
                ea.abar = v.ws.abar;
                ea.out = v.ws.gbar;
                ea.dsum = v.ws.dsum;
                ea.mirror = v.mirror;
                ea.wstore = need_gbar ? wslice(v, l) : nullptr;
                ea.n_stored = need_gbar ? v.n_edges_owned : 0;
                if (upper_bwd) {   // on the partition's upper-edge graph
                    const PairGraph &Q = v.pairs;
                    ea.n_chunks = chunks_of(Q.n_upper);
                    ea.chunk_row = Q.u_chunk_row;
                    ea.row_ptr = Q.u_row_ptr;
                    ea.senders = Q.u_senders;
                    ea.recv = Q.u_recv;
                    ea.d = Q.u_d;
                    ea.mirror = Q.u_mirror;
                    ea.eid = Q.u_eid;
                    // kept values in the order of the upper-edge graph, or (16-bit modes) at the upper edges' positions
                    // in the full list
                    if (upper) ea.n_stored = need_gbar ? Q.n_upper : 0;
                }
            }
            prof_begin(g, MLIP_PROF_EDGE_BWD);
            const int kind = upper_bwd ? kEdgeBwdUpper : kEdgeBwd;
            MLIP_TRY(prec == kPrecBf16 ? (launch_edge<F, kPrecBf16>(g, eb, kind))
                     : prec == kPrecF16x3 ? (launch_edge<F, kPrecF16x3>(g, eb, kind)) : (launch_edge<F, kPrecF32>(g, eb, kind)));
            prof_end(g);
            if (upper_bwd && need_gbar) {   // second pass: the lower edges' terms of the rows' sums
                prof_begin(g, MLIP_PROF_EDGE_BWD_LOWER);
                const SmallBatch sb = small_batch(p0, U_OWNED, l);
                if (sb.start[sb.n] > 0)
                    k_edge_lower<F, true><<<blocks_for(sb.start[sb.n], 4), 256, 0, s>>>(sb);
                MLIP_HIP(hipGetLastError());
                prof_end(g);
            }
        }
        if (any_bonds) {   // bond term: its share of gbar; this layer's abar is kept for the bonds' own reverse step
            prof_begin(g, MLIP_PROF_BOND);
            for (int p = 0; p < P; ++p) {
                SlabView &v = views[p];
                BondGraph &BG = v.bonds;
                if (BG.n > 0)
                    MLIP_HIP(hipMemcpyAsync(BG.abar_keep.as<float>() + (size_t)l * (size_t)v.n_owned * F, v.ws.abar,
                                            (size_t)v.n_owned * rowb, hipMemcpyDeviceToDevice, s));
                if (BG.n > 0 && need_gbar)
                    bond_elem([&](auto zero) {
                        using BT = decltype(zero);
                        k_bond_gbar<F, BT><<<blocks_for(v.n_owned, 4), 256, 0, s>>>(
                            v.n_owned, BG.ptr.as<int64_t>(), BG.sender.as<int32_t>(), BG.mirror.as<int32_t>(),
                            static_cast<const BT *>(wbslice(v, l)), v.ws.abar, v.ws.gbar);
                    });
            }
            MLIP_HIP(hipGetLastError());
            prof_end(g);
        }
        if (need_gbar) {
            if (slabs) {
                prof_begin(g, MLIP_PROF_GHOST);
                PtrTable tab{};
                for (int q = 0; q < P; ++q) tab.p[q] = views[q].ws.gbar;
                for (int p0 = 0; p0 < P; p0 += kBatch) {   // the ghost rows' gradients ...
                    const SmallBatch sb = small_batch(p0, U_GHOST, l);
                    if (sb.start[sb.n] > 0)
                        k_ghost_gbar<F><<<blocks_for(sb.start[sb.n], 4), 256, 0, s>>>(sb);
                }
                for (int p0 = 0; p0 < P; p0 += kBatch) {   // ... go back to their owners
                    const SmallBatch sb = small_batch(p0, U_BORDER, l);
                    if (sb.start[sb.n] > 0)
                        k_border_add<<<blocks_for(sb.start[sb.n] * (F / 4), 256), 256, 0, s>>>(sb, F, tab, gidx);
                }
                MLIP_HIP(hipGetLastError());
                prof_end(g);
            }
            prof_begin(g, MLIP_PROF_NODE);
            MLIP_TRY((node_pass<F, OP_BWD_PROJ>(g, views, P, base + pk.Wmn, nullptr, nullptr, [&](SlabView &v, NodeArgs &na) {
                na.n_rows = v.n_owned;
                na.X = v.ws.gbar;
                na.Z = v.ws.hbar;
            })));
            prof_end(g);
        }
    }

    // ---- reverse of the bond update: e1 = e0 + u SiLU(m), m = S Wt2, S = triplet sum, e0 = bbond(d) We0
    if (any_bonds) {
        prof_begin(g, MLIP_PROF_BOND);
        const float *Wtc = bw->Wt1 + 2 * ffp;
        for (int p = 0; p < P; ++p) {   // e1bar = sum_l dE/dwb_l Wb_l^T, ubar, Sbar = (e1bar u SiLU'(m)) Wt2^T
            BondArgs a = bond_args(views[p]);
            a.W[0] = bpk + 5 * ffp;
            for (int l = 0; l < std::min(L, 3); ++l) a.W[1 + l] = bpk + (6 + L + l) * ffp;
            a.Wx = bpk + (6 + L + 3) * ffp;
            a.n_layers = L;
            MLIP_TRY(prec == kPrecBf16 ? (launch_bond_mlp<F, BOND_EBAR, kPrecBf16>(g, a))
                     : prec == kPrecF16x3 ? (launch_bond_mlp<F, BOND_EBAR, kPrecF16x3>(g, a)) : (launch_bond_mlp<F, BOND_EBAR, kPrecF32>(g, a)));
        }
        prof_end(g);
        prof_begin(g, MLIP_PROF_TRIPLET_BWD);
        for (int p = 0; p < P; ++p) {
            SlabView &v = views[p];
            BondGraph &BG = v.bonds;
            if (BG.n > 0)
                bond_elem([&](auto zero) {
                    using BT = decltype(zero);
                    k_triplet_bwd<F, BT><<<blocks_for(v.n_owned, 4), 256, 0, s>>>(
                        v.n_owned, BG.ptr.as<int64_t>(), BG.rhat.as<float>(), BG.u.as<float>(), BG.P.as<BT>(), BG.Q.as<BT>(), Wtc,
                        BG.Sbar.as<BT>(), BG.Pbar.as<BT>(), BG.Qbar.as<BT>(), BG.ubar.as<float>(), BG.rbar.as<float>());
                });
        }
        MLIP_HIP(hipGetLastError());
        prof_end(g);
        prof_begin(g, MLIP_PROF_BOND);
        for (int p = 0; p < P; ++p) {   // e0bar = e1bar + Pbar Wta^T + Qbar Wtb^T, and dE/dd of the bonds from it
            BondArgs a = bond_args(views[p]);
            a.W[0] = bpk + 3 * ffp;
            a.W[1] = bpk + 4 * ffp;
            MLIP_TRY(prec == kPrecBf16 ? (launch_bond_mlp<F, BOND_E0BAR, kPrecBf16>(g, a))
                     : prec == kPrecF16x3 ? (launch_bond_mlp<F, BOND_E0BAR, kPrecF16x3>(g, a)) : (launch_bond_mlp<F, BOND_E0BAR, kPrecF32>(g, a)));
        }
        prof_end(g);
    }

    // ---- forces
    prof_begin(g, MLIP_PROF_FORCE);
    const double *pos = g->pos.as<double>();
    for (int p0 = 0; p0 < P; p0 += kBatch) {
        const SmallBatch sb = small_batch(p0, U_LOCAL, -1);
        if (sb.start[sb.n] <= 0) continue;
        if (L > 0)
            k_force_rows<<<(unsigned)((sb.start[sb.n] + 15) / 16), 256, 0, s>>>(sb, pos, g->cell);
        else
            k_zero_floc<<<blocks_for(sb.start[sb.n], 256), 256, 0, s>>>(sb);
    }
    if (bw)
        for (int p = 0; p < P; ++p) {
            SlabView &v = views[p];
            if (v.bonds.n <= 0) continue;
            BondGraph &BG = v.bonds;
            k_bond_force<<<blocks_for(v.n_owned, 128), 128, 0, s>>>(v.n_owned, BG.ptr.as<int64_t>(), BG.mirror.as<int32_t>(),
                                                                    BG.dbond.as<float>(), BG.rbar.as<float>(),
                                                                    BG.rhat.as<float>(), BG.d.as<float>(), v.ws.floc);
            if (v.n_ghost > 0)
                k_bond_force_ghost<<<blocks_for(v.n_ghost, 128), 128, 0, s>>>(
                    v.n_ghost, v.n_owned, v.row_ptr, v.mirror, BG.of_edge.as<int32_t>(), BG.dbond.as<float>(),
                    BG.rbar.as<float>(), BG.rhat.as<float>(), BG.d.as<float>(), v.ws.floc);
        }
    {   // owned rows to the caller's arrays; a border atom also collects what its ghost rows gathered elsewhere
        PtrTable tab{};
        for (int q = 0; q < P; ++q) tab.p[q] = views[q].ws.floc;
        for (int p0 = 0; p0 < P; p0 += kBatch) {
            const SmallBatch sb = small_batch(p0, U_OWNED, -1);
            if (sb.start[sb.n] > 0)
                k_store_owned<<<blocks_for(sb.start[sb.n], 256), 256, 0, s>>>(sb, tab, gidx, forces, atom_energy);
        }
    }
    MLIP_HIP(hipGetLastError());
    prof_end(g);
    return MLIP_OK;
}

}  // namespace

int forward_impl(mlip_graph *g, const mlip_weights_t *w, int32_t mode, double *energy, float *forces, float *atom_energy,
                 Carver *scratch)
{
    if (w->F == 32) return forward_t<32>(g, w, nullptr, mode, energy, forces, atom_energy, scratch);
    return forward_t<64>(g, w, nullptr, mode, energy, forces, atom_energy, scratch);
}

int forward_bonds_impl(mlip_graph *g, const mlip_weights_t *w, const mlip_bond_weights_t *bw, int32_t mode,
                       double *energy, float *forces, float *atom_energy)
{
    if (w->F == 32) return forward_t<32>(g, w, bw, mode, energy, forces, atom_energy, nullptr);
    return forward_t<64>(g, w, bw, mode, energy, forces, atom_energy, nullptr);
}

}  // namespace mlip

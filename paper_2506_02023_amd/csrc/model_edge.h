// Edge kernels: the fused forward edge step and the pair-wise reverse edge step.
// Part of model.hip (one translation unit): included inside namespace mlip, anonymous namespace.
#ifndef MLIP_MODEL_EDGE_H
#define MLIP_MODEL_EDGE_H

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
    // Upper-edge graph (the arrays above then describe the compacted upper edges of the partition; mirror holds the
    // reverse edges' indices in the partition's full edge list):
    const int32_t *eid;        // reverse: index of every upper edge in the full edge list
};

// What all partitions of one launch share: the layer's packed weights and the basis.
struct EdgeCommon {
    const float *A1, *A1s, *A2t, *A2n;   // A1s = c W1, A2t = W2 / c (see kSiluScale), A1 and A2n unscaled
    BasisParams bp;
    int need_gbar, first;
    int w_pairs;   // kept filter values: 1 = only the upper edge of a pair keeps them (both edges' values are the same
                   // bits, since they are the same function of the same length); 0 = every edge keeps its own
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
    int32_t *work;   // this launch's 8 work counters (kWorkCounterStride apart), zero when the kernel starts
    EdgeArgs s[kBatch];
};

// Persistent launch: the grid holds exactly the blocks that are resident at once, a multiple of 8.
// Blocks go to the 8 XCDs round-robin, so blocks b with the same b % 8 share an L2.  Each XCD takes one
// contiguous eighth of the work items and its wavefronts walk through it side by side: every wavefront starts
// with the item of its own position (block slot s, wave w: item nw s + w) and then draws the next item of the
// eighth from a counter all of them share.  At any moment an XCD works on a short contiguous run of rows, whose
// neighbourhoods overlap, so the sender rows it gathers stay in its L2; and because items are handed out, not
// dealt in advance, the wavefronts finish together although those of the younger block of a compute unit
// run about a fifth slower than those of the older one (measured: the instruction arbiter prefers age).
// The counters (one per eighth, 128 bytes apart, zero before the launch) are correct for any placement of
// blocks; only the locality depends on the round-robin.
constexpr int kWorkCounterStride = 32;   // int32 elements between two counters
struct ItemQueue {
    int64_t base, end;   // this eighth of the work items
    int32_t *counter;    // items drawn so far beyond the first one of every wavefront
    int32_t n_first;     // wavefronts that share the eighth (their first items are 0 .. n_first - 1)
    int64_t first;       // this wavefront's first item
    // Ask for the next item (lane 0's atomic; the value comes back like a load and is not waited for here) ...
    __device__ int32_t draw(int lane) const
    {
        int32_t v = 0;
        if (lane == 0) v = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return v;
    }
    // ... and turn the answer into an item index when the current item is done.
    __device__ int64_t resolve(int32_t drawn) const { return base + n_first + __builtin_amdgcn_readfirstlane(drawn); }
};
__device__ inline ItemQueue edge_items(int64_t total, int32_t *counters, int wave, int nw = 4)   // nw: wavefronts per block
{
    const int64_t n_slots = gridDim.x >> 3;
    const int64_t per = (((total + 7) >> 3) + 3) & ~(int64_t)3;
    const int64_t xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    ItemQueue q;
    q.base = xcd * per;
    q.end = min(total, (xcd + 1) * per);
    q.counter = counters + xcd * kWorkCounterStride;
    q.n_first = (int32_t)(n_slots * nw);
    q.first = q.base + slot * nw + wave;
    return q;
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
// (Valid because none of the model kernels writes the graph arrays.)
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
    const ItemQueue items = edge_items(B.chunk_start[B.n], B.work, wave);
    int64_t item = items.first;
    int32_t drawn = 0;
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
    for (; item < part_end; item = items.resolve(drawn)) {
    drawn = items.draw(lane);
    const int64_t chunk = item - B.chunk_start[part];
    int64_t r0, r1;
    if (!chunk_rows(A, chunk, r0, r1)) continue;
    // wave-uniform values loaded through vector instructions: keep them scalar (edge indices fit 32 bits)
    const int32_t e_lo = __builtin_amdgcn_readfirstlane((int32_t)A.row_ptr[r0]);
    const int32_t e_hi = __builtin_amdgcn_readfirstlane((int32_t)A.row_ptr[r1]);
    const int32_t r_end = (int32_t)r1;
    const bool keep_w = A.wstore != nullptr;
    const bool w_pairs = C.w_pairs != 0;
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
    int32_t mv = (keep_w && w_pairs) ? A.mirror[en] : 0;
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
        // bit k: edge k keeps its filter values (with w_pairs only the upper edge of a pair does)
        const uint32_t keeps = w_pairs ? (uint32_t)__ballot(valid && mv > tb + c32) : 0xffffffffu;
        // next tile's edge records
        en = min(tb + 32 + c32, e_hi - 1);
        dv = A.d[en];
        rk = A.recv[en];
        sv = A.senders[en];
        if (keep_w && w_pairs) mv = A.mirror[en];
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
        if (keep_w) {   // keep w_e for the reverse pass; rows past the end of the chunk, and those of edges that do not
                        // keep theirs, fall outside the descriptor's range and are dropped by the hardware bounds check
            const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(
                A.wstore + (int64_t)tb * F, 0, kmax * (F * 4), kBufferFlags);
#pragma unroll
            for (int k = 0; k < 32; ++k)
                if (F == 64 || lane < F)
                    buffer_store_f32_stream(wv[k], w_rsrc, f * 4, (keeps & (1u << k)) ? k * (F * 4) : 32 * (F * 4));
        }
#pragma unroll
        for (int k = 0; k < 32; ++k) {
            acc = fmaf(wv[k], gv[k], acc);   // lanes past the end hold a zero filter
            if (__builtin_expect((ends & (1u << k)) != 0, 0)) {   // unlikely: keeps the common path free of taken branches
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
        asm volatile("" : "+v"(dv), "+v"(rk), "+v"(sv), "+v"(mv));
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
#ifndef MLIP_BWD_WAVES
#define MLIP_BWD_WAVES 4
#endif
constexpr int kBwdWaves = MLIP_BWD_WAVES;
#ifndef MLIP_BWD_QUEUE
#define MLIP_BWD_QUEUE (31 + kStep + 1)
#endif
constexpr int kQueue = MLIP_BWD_QUEUE;   // queued pairs per wavefront: at most 31 pending + one step's new ones
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

// COMPACT: the launch runs on the partitions' upper-edge graphs: every edge it sees is the upper edge of its pair and the
// row sums it stores (gbar) are those of the upper edges only; k_edge_lower completes them with the lower edges' terms.
// (Letting this kernel hand w * abar_i to the lower edge's row through memory instead was measured: vector stores
// return in order with the loads on this chip, and 16 scattered row stores per step stalled the load pipeline:
// 5.2 ms per launch against 3.5 ms.)
template <int F, int PREC, bool COMPACT>
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
#ifdef MLIP_TIMING_PHASES
    // timing experiment only: shader-clock cycles this wavefront spends in the dense phase, printed by one wavefront
    long long t_start = clock64(), t_dense = 0;
    int n_dense = 0;
#endif

    const ItemQueue items = edge_items(B.chunk_start[B.n], B.work, wave, kBwdWaves);
    int64_t item = items.first;
    int32_t drawn = 0;
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
        int32_t ek;       // COMPACT: the edge's index in the full list
    };
    struct Step {
        float av[kStep], gv[kStep], wv[kStep];   // abar / g rows of the senders, kept filter values
        float ai0, gi0, ai1, gi1;       // abar / g rows of the first and of the last edge's receiver
        int kmax;                       // valid edges in the step
        int32_t tb;
        uint32_t uppers;                // bit k: edge k is the upper edge of its pair
    };
    auto load_ids = [&](Ids &I, int32_t tb) {
        const int32_t e = min((int32_t)tb + l16, e_hi - 1);
        I.sj = A.senders[e];
        I.rk = A.recv[e];
        I.mk = A.mirror[e];
        I.dk = A.d[e];
        if (COMPACT) I.ek = A.eid[e];
    };
    auto load_step = [&](Step &S, const Ids &I, int32_t tb) {
        S.tb = tb;
        S.kmax = __builtin_amdgcn_readfirstlane(max(0, min(kStep, e_hi - tb)));   // (the clamp is a vector instruction)
        // A step past the end of the work item (kmax = 0) still issues its loads, from the clamped records:
        // every path through the pipeline then has the same number of loads in flight, which is what lets
        // the waits before the uses be partial ones.
        const int32_t sjo = I.sj * kRowBytes;
        S.uppers = COMPACT ? ((1u << S.kmax) - 1u)
                           : ((uint32_t)__ballot(l16 < S.kmax && I.mk > tb + l16) & ((1u << kStep) - 1u));
        const int32_t row0 = __builtin_amdgcn_readfirstlane(I.rk);
        const int32_t rowl = __builtin_amdgcn_readlane(I.rk, max(S.kmax - 1, 0));
        S.ai0 = buffer_load_f32(a_rsrc, f * 4, row0 * kRowBytes, 0);
        S.gi0 = buffer_load_f32(g_rsrc, f * 4, row0 * kRowBytes, 0);
        S.ai1 = buffer_load_f32(a_rsrc, f * 4, rowl * kRowBytes, 0);
        S.gi1 = buffer_load_f32(g_rsrc, f * 4, rowl * kRowBytes, 0);
        // w_e sits at the edge's own index or, with w_pairs, at the index of the pair's upper edge in the full list (a
        // range of zero bytes reads 0: without gbar no w is needed).  With w_pairs the descriptor spans the partition's
        // kept values (the host sets the flag only if they fit its 32-bit range) and a lower edge reads its reverse
        // edge's row, an edge of an upper-edge graph the row at its index in the full list; an edge past the end then
        // reads the row of the item's last edge, which goes into a sum nobody stores.
        const bool w_pairs = C.w_pairs != 0;
        const int32_t w_first = w_pairs ? 0 : tb;   // edge whose row the descriptor starts at
        const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(
            A.wstore + (need_gbar ? (int64_t)w_first * F : 0), 0,
            !need_gbar ? 0 : w_pairs ? (int)(uint32_t)(A.n_stored * kRowBytes) : S.kmax * kRowBytes, kBufferFlags);
        // lane k: byte offset of edge k's row (unsigned: the kept values of a partition may span up to 4 GB)
        const int32_t wro =
            (int32_t)((uint32_t)(w_pairs ? (COMPACT ? I.ek : min(I.mk, tb + l16)) : l16) * (uint32_t)kRowBytes);
#pragma unroll
        for (int k = 0; k < kStep; ++k) {
            const int32_t so = __builtin_amdgcn_readlane(sjo, k);
            S.av[k] = buffer_load_f32(a_rsrc, f * 4, so, 0);
            S.gv[k] = buffer_load_f32(g_rsrc, f * 4, so, 0);
            S.wv[k] = buffer_load_f32_stream(w_rsrc, f * 4,
                                             __builtin_amdgcn_readlane(wro, k));   // 0 outside the range
        }
    };
    // rn_first: receiver of the first edge of the following step (r1 after the last step)
    auto compute_step = [&](const Step &S, const Ids &I, int32_t rn_first) {
        if (S.kmax <= 0) return;
        const bool valid_l = l16 < S.kmax;
        const int32_t rk = valid_l ? I.rk : r1;
        const int32_t e_l = COMPACT ? I.ek : S.tb + l16;   // index in the full edge list
        // wave-uniform masks: bit k = edge k ends its row / edge k is the upper edge of its pair
        const int32_t up = __shfl(rk, l16 + 1, 64);
        const int32_t rnext = (l16 == kStep - 1) ? rn_first : up;
        const uint32_t ends = (uint32_t)__ballot(valid_l && rnext != rk) & ((1u << kStep) - 1u);
        const bool upper_l = COMPACT ? valid_l : (valid_l && I.mk > e_l);
        const uint32_t uppers = S.uppers;
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
            if (__builtin_expect((ends & (1u << k)) != 0, 0)) {   // unlikely: keeps the common path free of taken branches
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
#ifdef MLIP_TIMING_PHASES
        const long long t_in = clock64();
#endif
#ifdef MLIP_TIMING_SKIP_PAIR_PHASE
        // timing experiment only (results are wrong): drop the queued pairs without the dense work, which leaves
        // the streaming phase of the kernel to be timed on its own
        {
            const int nv = min(q_count, 32);
            q_head += nv;
            q_head -= (q_head >= kQueue) ? kQueue : 0;
            q_count -= nv;
            return;
        }
#endif
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
#ifdef MLIP_TIMING_PHASES
        t_dense += clock64() - t_in;
        ++n_dense;
#endif
    };

    for (; item < part_end; item = items.resolve(drawn)) {
        drawn = items.draw(lane);
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
#ifdef MLIP_TIMING_PHASES
    long long t_total = clock64() - t_start;
    asm volatile("" : "+s"(t_total));   // taken before the print starts
    if (lane == 0 && wave == 0 && blockIdx.x % 37 == 0)
        printf("k_edge_bwd prec %d first %d block %d : %lld cycles, %lld in %d dense phases\n", PREC, (int)B.c.first,
               (int)blockIdx.x, t_total, t_dense, n_dense);
#endif
}


#ifdef MLIP_BWD_SIMD
// ---- Reverse edge step on upper-edge graphs with the two phases on different SIMDs (fp32 MFMA; an experiment:
// compiled and used only with -DMLIP_BWD_SIMD)
//
// fp32 MFMA and vector instructions share one pipeline per SIMD, and an MFMA holds it for 64 cycles: in the kernel above,
// whose wavefronts alternate between the phases, a streaming wavefront crawls while the other wavefront of its SIMD
// multiplies, and the two phases' times add.  Wavefronts on DIFFERENT SIMDs do not disturb each other (micro-benchmark
// microbench/simd_roles.hip: row gathers on one SIMD beside MFMA chains on the other three run in the time of the longer
// of the two).  Here one block of 12 wavefronts runs per compute unit, three per SIMD.  Every wavefront reads the SIMD
// it was placed on from the hardware id register; the three wavefronts of one SIMD stream (phase 1 above, one ring of
// queued pairs each), two wavefronts on each other SIMD do the dense work (phase 2), the remaining three only attend the
// barriers.  Results are identical to the alternating kernel's.  Measured on the 1M-atom benchmark: 3.70 ms per launch
// against 3.56 ms.  The dense work alone would take about 3.0 ms on three SIMDs, but the three streaming wavefronts
// alone take 2.98 ms: what a SIMD's register file can keep in flight with a step of loads ahead (3 x 52 rows) is too
// little for the latency, a fourth streaming wavefront needs a 16-wave block (128 registers, and rings that no longer fit
// the LDS), and with one round of buffering the two sides wait for each other's slowest.
//
// Hand-over: every streaming wavefront owns a ring of kSimdRing slots in LDS (slot layout as above, plus the partition
// index, since pairs of several partitions share a ring).  All wavefronts of the block meet at one barrier per round.
// Before the barrier a streaming wavefront publishes how many pairs it has produced in all and whether it is out of
// work; after it, every wavefront reads the published numbers and derives from them, by the same rule, how many pairs
// every ring hands out in this round (kSimdTake as soon as that many are there, the rest once the producer is done):
// a 32-pair tile for each of the ring's two dense wavefronts.  Because all derive the same numbers, nothing flows back
// from the consumers, and all agree on the round after which everything is consumed: the loop bound of every
// wavefront, so no barrier is left waiting.  A streaming wavefront ends its round once kSimdTake pairs are pending
// beyond what the consumers are known to take; slots being read (at most kSimdTake) plus pending ones (less than
// kSimdTake + kStep) plus the slot a step writes speculatively stay within the ring.  The published numbers alternate
// between two sets, so a set is rewritten only after a barrier that every reader of its previous contents has passed.
constexpr int kSimdWaves = 12;    // wavefronts per block: three per SIMD
constexpr int kSimdStream = 3;    // streaming wavefronts, one ring each
constexpr int kSimdDense = 6;     // dense wavefronts; ring q is emptied by the dense wavefronts q and q + kSimdStream
constexpr int kSimdTake = 64;     // pairs a ring hands out per round: one 32-pair tile for each of its two consumers
constexpr int kSimdRing = 2 * kSimdTake + kStep + 1;   // slots of a ring
static_assert(kSimdDense == 2 * kSimdStream && kSimdTake == 64, "two 32-pair tiles per ring and round");

template <int F> struct BwdSimdLds {
    using D = Dims<F>;
    static constexpr int kQueuesAt = D::PACKF + D::PACK1;                          // floats
    static constexpr int kPubAt = kQueuesAt + kSimdStream * kSimdRing * D::FS;     // int32 [2][kSimdStream][2]
    static constexpr int kSimdAt = kPubAt + 4 * kSimdStream;                       // int32 [kSimdWaves]
    static constexpr int kTabAt = (kSimdAt + kSimdWaves + 1) & ~1;                 // float* [kBatch], 8-byte aligned
    static constexpr size_t bytes = sizeof(float) * kTabAt + sizeof(float *) * kBatch;
};

template <int F>
__global__ void __launch_bounds__(kSimdWaves * 64, 1) k_edge_bwd_simd(EdgeBatch B)
{
    using D = Dims<F>;
    using L = BwdSimdLds<F>;
    constexpr int FS = D::FS;
    constexpr int kRowBytes = F * 4;
    constexpr int kThreads = kSimdWaves * 64;
    extern __shared__ float lds[];
    float *A2n = lds;
    float *A1l = A2n + D::PACKF;
    float *queues = lds + L::kQueuesAt;
    int32_t *pub = reinterpret_cast<int32_t *>(lds + L::kPubAt);
    int32_t *simd_of = reinterpret_cast<int32_t *>(lds + L::kSimdAt);
    float **dsum_tab = reinterpret_cast<float **>(lds + L::kTabAt);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    // the SIMD this wavefront runs on: bits 5:4 of the hardware id register (HW_REG_HW_ID = 4, read whole)
    const int simd = (int)((__builtin_amdgcn_s_getreg((31 << 11) | 4) >> 4) & 3u);
    for (int i = threadIdx.x; i < D::PACKF; i += kThreads) A2n[i] = B.c.A2n[i];
    for (int i = threadIdx.x; i < D::PACK1; i += kThreads) A1l[i] = B.c.A1[i];
    if (threadIdx.x < 4 * kSimdStream) pub[threadIdx.x] = 0;
    if (threadIdx.x < kBatch) dsum_tab[threadIdx.x] = (threadIdx.x < B.n) ? B.s[threadIdx.x].dsum : nullptr;
    if (lane == 0) simd_of[wave] = simd;
    __syncthreads();
    // Roles, derived by every wavefront from the same table.  With three wavefronts on every SIMD (what the register
    // budget of a 12-wave block allows at most, so what the hardware deals) the SIMD of wavefront 0 streams and the
    // other three SIMDs run two dense wavefronts each, their third wavefront only attends the barriers.  Any other
    // placement falls back to roles by wavefront index: the same results, the phases then share SIMDs.
    enum { kStreams = 0, kDense = 1, kSpare = 2 };
    int role, mine;   // mine: streaming: the ring it fills; dense: 0 .. kSimdDense - 1
    {
        int on[4] = {0, 0, 0, 0}, rank = 0;
#pragma unroll
        for (int w = 0; w < kSimdWaves; ++w) {
            const int s = __builtin_amdgcn_readfirstlane(simd_of[w]);
#pragma unroll
            for (int k = 0; k < 4; ++k) on[k] += (s == k) ? 1 : 0;
            rank += (w < wave && s == simd) ? 1 : 0;
        }
        const int star = __builtin_amdgcn_readfirstlane(simd_of[0]);
        const bool even = on[0] == 3 && on[1] == 3 && on[2] == 3 && on[3] == 3;
        if (even) {
            const int ord = simd - (simd > star ? 1 : 0);   // 0 .. 2 among the SIMDs that do not stream
            role = (simd == star) ? kStreams : (rank < 2 ? kDense : kSpare);
            mine = (simd == star) ? rank : ord * 2 + rank;
        } else {
            role = wave < kSimdStream ? kStreams : (wave < kSimdStream + kSimdDense ? kDense : kSpare);
            mine = wave < kSimdStream ? wave : wave - kSimdStream;
        }
    }
    const bool streams = role == kStreams;
    const int c32 = lane & 31;
    const int l16 = lane % kStep;
    const unsigned f = lane & (F - 1);
    const EdgeCommon &C = B.c;
    const bool need_gbar = C.need_gbar != 0;

    // ---- the rounds' bookkeeping, identical in every wavefront
    int round = 0;
    int consumed[kSimdStream];   // pairs taken from every ring so far
    int take[kSimdStream];       // ... and in the current round
#pragma unroll
    for (int q = 0; q < kSimdStream; ++q) consumed[q] = 0;
    int consumed_mine = 0;        // streaming: consumed[mine]
    // meets the other wavefronts; returns true if this round's takes empty every ring of a finished producer
    auto rendezvous = [&]() -> bool {
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // LDS writes done; loads in flight stay in flight
        const int32_t *pb = pub + (round & 1) * (2 * kSimdStream);   // (re-read: the barrier statement clobbers memory)
        bool finished = true;
#pragma unroll
        for (int q = 0; q < kSimdStream; ++q) {
            const int produced = __builtin_amdgcn_readfirstlane(pb[2 * q]);
            const int done = __builtin_amdgcn_readfirstlane(pb[2 * q + 1]);
            const int avail = produced - consumed[q];
            take[q] = (avail >= kSimdTake || done) ? min(avail, kSimdTake) : 0;
            consumed[q] += take[q];
            finished = finished && done && produced == consumed[q];
            if (streams && q == mine) consumed_mine = consumed[q];
        }
        ++round;
        return finished;
    };

    if (!streams) {
        // ================================================================ dense wavefronts
        // dense wavefront `mine` empties ring mine % kSimdStream as its (mine / kSimdStream)-th consumer: of the pairs
        // a round hands out it takes the tile [32 j, 32 j + 32)
        const int ring = mine % kSimdStream, part_j = mine / kSimdStream;
        int q_head = 0;
        auto dense = [&](const float *Q, int head, int nval) {
#ifdef MLIP_TIMING_SKIP_PAIR_PHASE
            return;   // timing experiment only (results are wrong): the streaming wavefronts and the hand-over on their own
#endif
            int slot = head + c32;
            slot -= (slot >= kSimdRing) ? kSimdRing : 0;
            const bool valid = c32 < nval;
            const int4 rec = *reinterpret_cast<const int4 *>(Q + slot * FS + F);   // e, m, d, partition
            const int32_t e2 = valid ? rec.x : 0, m2 = valid ? rec.y : 0;
            const float d2 = valid ? __builtin_bit_cast(float, rec.z) : C.bp.rc;   // rc: zero derivative
            // (the table holds pointers to global memory; saying so keeps the stores off the flat path)
            typedef __attribute__((address_space(1))) float global_float;
            global_float *dsum = (global_float *)dsum_tab[valid ? rec.w : 0];
            float b[8], db[8];
            radial_basis<true>(d2, C.bp, b, db);
#pragma unroll
            for (int n = 0; n < 8; ++n) b[n] *= kSiluScale;   // pre-activations come out as t' = c t
            f32x16 t[D::NB];   // ds_k/dd = SiLU'(t_k) c_k, one block of 32 features at a time
#pragma unroll
            for (int bb = 0; bb < D::NB; ++bb) {
                f32x16 cg;
                RegPack1<F> W1;
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
            gemm_queue<F>(A2n, Q + slot * FS, sb, lane);   // sbar[k] = sum_f W2[k][f] wsym[f]
            float part = 0.f;
#pragma unroll
            for (int bb = 0; bb < D::NB; ++bb)
#pragma unroll
                for (int r = 0; r < 16; ++r) part = fmaf(sb[bb][r], t[bb][r], part);
            part += __shfl_xor(part, 32, 64);
            if (valid && lane < 32) {
                // every edge is written by exactly one pair per launch; after the first layer the value is added
                if (C.first) {
                    dsum[e2] = part;
                    dsum[m2] = part;
                } else {
                    __builtin_amdgcn_global_atomic_fadd_f32(dsum + e2, part);
                    __builtin_amdgcn_global_atomic_fadd_f32(dsum + m2, part);
                }
            }
        };
        for (;;) {
            const bool finished = rendezvous();
            int taken = 0;
#pragma unroll
            for (int q = 0; q < kSimdStream; ++q)
                if (q == ring) taken = take[q];
            if (role == kDense) {
                const int nval = min(taken - 32 * part_j, 32);
                if (nval > 0) {
                    int head = q_head + 32 * part_j;
                    head -= (head >= kSimdRing) ? kSimdRing : 0;
                    dense(queues + ring * (kSimdRing * FS), head, nval);
                }
                q_head += taken;
                q_head -= (q_head >= kSimdRing) ? kSimdRing : 0;
            }
            if (finished) break;
        }
        return;
    }

    // ==================================================================== streaming wavefronts
    float *Q = queues + mine * (kSimdRing * FS);
    char *Qf = reinterpret_cast<char *>(Q + f);
    int produced = 0;   // pairs queued so far
    int q_tail = 0;     // produced % kSimdRing
    auto publish = [&](int done) {
        if (lane == 0) {
            int32_t *pb = pub + (round & 1) * (2 * kSimdStream) + 2 * mine;
            pb[0] = produced;
            pb[1] = done;
        }
    };

    const ItemQueue items = edge_items(B.chunk_start[B.n], B.work, mine, kSimdStream);
    int64_t item = items.first;
    int32_t drawn = 0;
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
    int32_t r1 = 0, e_hi = 0;
    float acc = 0.f;

    // Steps of kStep edges through a software pipeline whose loads are all issued ahead of their use: the edge
    // records (sender, receiver, reverse edge, length) two steps ahead, the rows they point to one step ahead.
    // Vector memory loads complete in order, so a stage may only contain loads and address arithmetic; anything
    // that consumes a loaded value belongs to a later stage.
    struct Ids {    // lane k (mod kStep) holds edge tb + k, clamped to the last edge of the work item
        int32_t sj, rk, mk, ek;   // sender, receiver, and the indices of the reverse edge and of the edge in the full list
        float dk;
    };
    struct Step {
        float av[kStep], gv[kStep], wv[kStep];   // abar / g rows of the senders, kept filter values
        float ai0, gi0, ai1, gi1;       // abar / g rows of the first and of the last edge's receiver
        int kmax;                       // valid edges in the step
        int32_t tb;
        uint32_t uppers;                // bit k: edge k is the upper edge of its pair
    };
    auto load_ids = [&](Ids &I, int32_t tb) {
        const int32_t e = min((int32_t)tb + l16, e_hi - 1);
        I.sj = A.senders[e];
        I.rk = A.recv[e];
        I.mk = A.mirror[e];
        I.dk = A.d[e];
        I.ek = A.eid[e];
    };
    auto load_step = [&](Step &S, const Ids &I, int32_t tb) {
        S.tb = tb;
        S.kmax = __builtin_amdgcn_readfirstlane(max(0, min(kStep, e_hi - tb)));
        // A step past the end of the work item (kmax = 0) still issues its loads, from the clamped records:
        // every path through the pipeline then has the same number of loads in flight, which is what lets
        // the waits before the uses be partial ones.
        const int32_t sjo = I.sj * kRowBytes;
        S.uppers = (1u << S.kmax) - 1u;   // every edge of an upper-edge graph is the upper edge of its pair
        const int32_t row0 = __builtin_amdgcn_readfirstlane(I.rk);
        const int32_t rowl = __builtin_amdgcn_readlane(I.rk, max(S.kmax - 1, 0));
        S.ai0 = buffer_load_f32(a_rsrc, f * 4, row0 * kRowBytes, 0);
        S.gi0 = buffer_load_f32(g_rsrc, f * 4, row0 * kRowBytes, 0);
        S.ai1 = buffer_load_f32(a_rsrc, f * 4, rowl * kRowBytes, 0);
        S.gi1 = buffer_load_f32(g_rsrc, f * 4, rowl * kRowBytes, 0);
        // w_e sits at the edge's own index in the upper-edge graph (a range of zero bytes reads 0: without gbar no w
        // is needed)
        const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(
            A.wstore + (need_gbar ? (int64_t)tb * F : 0), 0, need_gbar ? S.kmax * kRowBytes : 0, kBufferFlags);
#ifdef MLIP_TIMING_SKIP_STREAM_LOADS
        // timing experiment only (results are wrong): no row is gathered, which leaves the dense side and the hand-over
#pragma unroll
        for (int k = 0; k < kStep; ++k) S.av[k] = S.gv[k] = S.wv[k] = (float)(sjo & 1);
#else
#pragma unroll
        for (int k = 0; k < kStep; ++k) {
            const int32_t so = __builtin_amdgcn_readlane(sjo, k);
            S.av[k] = buffer_load_f32(a_rsrc, f * 4, so, 0);
            S.gv[k] = buffer_load_f32(g_rsrc, f * 4, so, 0);
            S.wv[k] = buffer_load_f32_stream(w_rsrc, f * 4, k * kRowBytes);   // 0 outside the range
        }
#endif
    };
    // rn_first: receiver of the first edge of the following step (r1 after the last step)
    auto compute_step = [&](const Step &S, const Ids &I, int32_t rn_first) {
        if (S.kmax <= 0) return;
        const bool valid_l = l16 < S.kmax;
        const int32_t rk = valid_l ? I.rk : r1;
        const int32_t e_l = I.ek;   // index in the full edge list
        // wave-uniform masks: bit k = edge k ends its row / edge k is the upper edge of its pair
        const int32_t up = __shfl(rk, l16 + 1, 64);
        const int32_t rnext = (l16 == kStep - 1) ? rn_first : up;
        const uint32_t ends = (uint32_t)__ballot(valid_l && rnext != rk) & ((1u << kStep) - 1u);
        const bool upper_l = valid_l;
        const uint32_t uppers = S.uppers;
        {   // records of the pairs queued by this step, all at once: slots follow q_tail in edge order
            int slot = q_tail + (int)__builtin_amdgcn_mbcnt_lo(uppers, 0u);   // upper edges before this lane's (lanes < kStep)
            slot -= (slot >= kSimdRing) ? kSimdRing : 0;
            if (upper_l && lane < kStep) {
                float *rec = Q + slot * FS + F;
                reinterpret_cast<int32_t *>(rec)[0] = e_l;
                reinterpret_cast<int32_t *>(rec)[1] = I.mk;
                rec[2] = I.dk;
                reinterpret_cast<int32_t *>(rec)[3] = part;
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
            q_off = (q_off == kSimdRing * FS * 4) ? 0 : q_off;
            if (__builtin_expect((ends & (1u << k)) != 0, 0)) {   // unlikely: keeps the common path free of taken branches
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
        produced += n_new;
        q_tail += n_new;
        q_tail -= (q_tail >= kSimdRing) ? kSimdRing : 0;
    };
    // end of a round: enough pairs are pending beyond what the consumer is known to take
    auto maybe_round = [&]() {
        if (produced - consumed_mine >= kSimdTake) {
            publish(0);
            rendezvous();
        }
    };

    for (; item < part_end; item = items.resolve(drawn)) {
        drawn = items.draw(lane);
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
            maybe_round();
            load_ids(IA, tb + 3 * kStep);
            load_step(SA, IC, tb + 2 * kStep);
            nf = __builtin_amdgcn_readfirstlane(IC.rk);
            compute_step(SB, IB, (tb + 2 * kStep < e_hi) ? nf : r1);
            maybe_round();
            IB = IA;   // records of step tb + 3 kStep, loaded a step ago
            IA = IC;   // records of step tb + 2 kStep, whose rows SA holds
        }
    }   // work items
    }   // partitions
    // out of work: keep meeting the others until every ring is empty
    for (;;) {
        publish(1);
        if (rendezvous()) break;
    }
}

#endif  // MLIP_BWD_SIMD

#endif  // MLIP_MODEL_EDGE_H

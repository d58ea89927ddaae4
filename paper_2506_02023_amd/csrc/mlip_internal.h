// Internal declarations shared by the translation units of libmlip.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "mlip.h"

namespace mlip {

void set_error(const char *fmt, ...);

#define MLIP_HIP(expr)                                                                      \
    do {                                                                                    \
        hipError_t e_ = (expr);                                                             \
        if (e_ != hipSuccess) {                                                             \
            mlip::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
            return (e_ == hipErrorOutOfMemory) ? MLIP_ENOMEM : MLIP_EHIP;                   \
        }                                                                                   \
    } while (0)

#define MLIP_TRY(expr)            \
    do {                          \
        int rc_ = (expr);         \
        if (rc_ != MLIP_OK) return rc_; \
    } while (0)

// Grow-only device buffer owned by a graph handle.  Memory comes from the allocator that is current when the
// buffer grows (the handle's, made current by every entry point that may allocate: AllocScope); the buffer
// remembers who gave it its block and returns it there.
struct DevBuf {
    void *p = nullptr;
    size_t cap = 0;
    mlip_alloc_t owner = {nullptr, nullptr, nullptr};   // alloc == nullptr: hipMalloc / hipFree
    int ensure(size_t bytes);
    void release();
    template <class T> T *as() const { return static_cast<T *>(p); }
};

// Makes a handle's allocator (and its stream, which is synchronised before a block goes back to a caller's
// allocator) current for the calling thread until the scope ends.
struct AllocScope {
    explicit AllocScope(const mlip_graph *g);
    ~AllocScope();
    AllocScope(const AllocScope &) = delete;
    AllocScope &operator=(const AllocScope &) = delete;
};

// Bump allocator over a fixed block (the static scratch of mlip_forward_static): 256-byte aligned pieces, no frees.
struct Carver {
    char *base = nullptr;
    size_t size = 0, used = 0;
    void *take(size_t bytes)
    {
        const size_t at = (used + 255) & ~(size_t)255;
        if (at + bytes > size) { used = size + 1; return nullptr; }   // stays failed
        used = at + bytes;
        return base + at;
    }
    bool failed() const { return used > size; }
};

// Workspace of one partition for the forward call in progress (from the view's buffers, or carved from a fixed block).
struct ViewWs {
    float *h = nullptr, *hbar = nullptr, *abar = nullptr, *gbar = nullptr, *eps = nullptr, *dsum = nullptr,
          *floc = nullptr, *g = nullptr, *a = nullptr, *wst = nullptr;
};

// Cell geometry prepared on the host, passed to kernels by value.
struct CellParams {
    double C[9];       // rows = lattice vectors
    double nrm[3][3];  // n_k = a_{k+1} x a_{k+2}
    double V;          // a_0 . n_0
    double rc2;        // r_cut * r_cut
    int nb[3];         // bins per lattice direction
    int reach[3];      // stencil half-width in bins
    int axis;          // slab axis
    int n_slabs;
};

// Workgroups are dealt to the 8 XCDs round-robin (workgroup b runs on XCD b mod 8), and every XCD has its own L2.
// A kernel whose neighbouring blocks gather overlapping data (neighbour rows, candidate cells) takes its logical
// block index from xcd_block() instead of blockIdx.x: every XCD then works on one contiguous eighth of the blocks
// and its L2 holds that eighth's data, instead of all eight L2s holding the same lines.  The grid must be a
// multiple of 8 (grid8) and the kernel must bounds-check its items.
#ifdef __HIPCC__
__device__ inline unsigned xcd_block() { return (blockIdx.x & 7u) * (gridDim.x >> 3) + (blockIdx.x >> 3); }
#endif
inline unsigned grid8(int64_t blocks) { return (unsigned)(((blocks > 0 ? blocks : 1) + 7) / 8 * 8); }

// Work item of the edge kernels: the rows whose first edge lies in one span of kChunkEdges edges.
#ifndef MLIP_CHUNK
#define MLIP_CHUNK 1024
#endif
constexpr int kChunkEdges = MLIP_CHUNK;
inline int64_t chunks_of(int64_t n_edges) { return n_edges > 0 ? (n_edges + kChunkEdges - 1) / kChunkEdges : 1; }

// Bond graph of the three-body variant for one partition: the edges of its owned rows within the bond cutoff,
// in edge order (all bonds of an owned centre belong to its partition).
struct BondGraph {
    double r_bond = -1.0;   // cutoff the list was built for (< 0: none)
    int p_env = -1;         // envelope exponent the stored u, du/dd were evaluated with
    int64_t n = 0;          // bonds
    DevBuf scan;            // i32 [E + 1] exclusive scan of the bond flags (E = edges of the owned rows)
    DevBuf flag;            // i32 [E]
    DevBuf of_edge;         // i32 [E]   bond index of an edge, -1 if it is no bond
    DevBuf edge;            // i32 [n]   edge index of a bond
    DevBuf ptr;             // i64 [n_owned + 1] bonds of centre i: ptr[i] .. ptr[i + 1]
    DevBuf mirror;          // i32 [n]   the bond of the reverse edge, -1 if the sender is a ghost row
    DevBuf sender;          // i32 [n]   sender row (local) of the bond
    DevBuf d, u, du;        // f32 [n]   length, envelope u(d / r_bond), du/dd
    DevBuf rhat;            // f32 [n][3] unit vector from the centre to the neighbour's image
    // model workspace, [n][F] unless noted
    DevBuf P, Q, S, m, wb /* [L][n][F] */, e1bar, Sbar, Pbar, Qbar;
    DevBuf abar_keep;       // f32 [L][n_owned][F] dE/da of the owned rows, every layer's (for the bonds' reverse step)
    DevBuf ubar, dbond;     // f32 [n]
    DevBuf rbar;            // f32 [n][3]
};

// The edges of a partition's owned rows split into the upper and the lower edge of every edge / reverse-edge pair
// (upper: the one with the smaller index; an edge whose reverse edge lies in a ghost row is an upper edge).  The
// upper edges are compacted into a graph of their own (same rows, half the edges) on which the edge kernels run;
// the lower edges' terms are added by row-wise kernels.  Built on first use after a graph build.
struct PairGraph {
    bool valid = false;
    bool slots_full = false;   // what l_slot holds (below)
    int64_t n_upper = 0, n_lower = 0;
    // grow-only buffers behind the pointers below (unused when the arrays are carved from a caller-independent block)
    DevBuf b_u_row_ptr, b_wslot, b_u_senders, b_u_recv, b_u_eid, b_u_mirror, b_u_d, b_u_chunk_row;
    DevBuf b_l_row_ptr, b_l_senders, b_l_slot;
    int64_t *u_row_ptr = nullptr;                     // [n_owned + 1]
    int32_t *wslot = nullptr;                         // [E_owned] upper edges: their index in the upper-edge graph
    // the lower edges of the owned rows, in their order: CSR [n_owned + 1], sender row, and where the pair's filter
    // values are kept: the index of its upper edge in the upper-edge graph or (slots_full) in the full list
    int64_t *l_row_ptr = nullptr;
    int32_t *l_senders = nullptr, *l_slot = nullptr;  // [n_lower]
    // [n_upper]: sender row, receiver row, edge, reverse edge
    int32_t *u_senders = nullptr, *u_recv = nullptr, *u_eid = nullptr, *u_mirror = nullptr;
    float *u_d = nullptr;                             // [n_upper]
    int32_t *u_chunk_row = nullptr;                   // [chunks_of(n_upper) + 1]
};

// One partition as the model kernels see it.  The whole graph is the special
// case nodes == nullptr (identity), n_owned == n_local == N.
struct SlabView {
    int64_t n_owned = 0, n_pure = 0, n_border = 0, n_ghost = 0, n_local = 0;
    int64_t n_edges_owned = 0, n_edges = 0;
    const int32_t *nodes = nullptr;        // local -> global (nullptr: identity)
    const int64_t *row_ptr = nullptr;      // n_local + 1
    const int32_t *senders = nullptr;      // local ids
    const uint32_t *shiftp = nullptr;      // packed image shifts
    const int32_t *recv = nullptr;         // receiver (local row) of every edge
    const int32_t *mirror = nullptr;       // position of every edge's reverse edge
    const float *d = nullptr;              // edge lengths
    const int32_t *chunk_row = nullptr;    // [chunks_of(n_edges) + 1] first row of every work item, then n_local
    const int32_t *ghost_owner = nullptr;  // [n_ghost] owning slab
    const int32_t *ghost_src = nullptr;    // [n_ghost] local index inside the owner
    const int32_t *owned_sorted = nullptr; // [n_owned] owned atoms, ascending global id
    std::vector<int64_t> markers;          // host, P + 3
    // model workspace (sized in mlip_forward)
    DevBuf h, hbar, abar, gbar, eps, dsum, floc, g, a, wst;  // g, a and wst hold L slices each
    ViewWs ws;                             // the pointers the kernels of the current call use
    BondGraph bonds;
    PairGraph pairs;
};

// Device arrays of all partitions, each array holding the partitions' pieces one after another (one allocation and
// one kernel launch per step of the partition build instead of one per slab).
struct PartStore {
    DevBuf nodes, owned_sorted, ghost_owner, ghost_src;   // i32, pieces of n_local / n_owned / n_ghost entries
    DevBuf rowlen, row_abs, row_ptr;                      // i32 / i64 / i64, pieces of n_local + 1 entries
    DevBuf senders, recv, mirror, shiftp, d;              // pieces of n_edges entries
    DevBuf chunk_row;                                     // i32, pieces of chunks_of(n_edges) + 1 entries
    DevBuf gbase, ghost_local;                            // i32 [N + 1] scan of popcount(needed_by); i32 [sum n_ghost]
    DevBuf sizes;                                         // i64 small read-back area
};

enum { kMaxSlabs = 64, kMaxEvents = 4096 };

struct Profiler {
    bool on = false;
    std::vector<hipEvent_t> pool;  // pairs
    std::vector<int> group;        // group of pair k
    size_t used = 0;               // events used
    float ms[MLIP_PROF_COUNT] = {0};
    int64_t launches[MLIP_PROF_COUNT] = {0};
};

}  // namespace mlip

struct mlip_graph {
    hipStream_t stream = nullptr;
    mlip_alloc_t alloc = {nullptr, nullptr, nullptr};   // caller's allocator (alloc == nullptr: hipMalloc)
    // per-handle launch configuration: kernels whose attributes are set, with their resident blocks per compute unit
    std::vector<std::pair<const void *, int>> fn_occ;
    int n_cu = 0;
    // packed weights are kept until the weight struct of a call differs from the one they were packed from
    mlip_weights_t packed_w = {};
    bool packed_w_valid = false;
    mlip_bond_weights_t packed_bw = {};
    mlip_weights_t packed_bw_w = {};
    bool packed_bw_valid = false;
    int64_t N = 0, E = 0;
    int32_t P = 1;
    int32_t species_max = 0, species_min = 0;
    double r_cut = 0;
    mlip::CellParams cell;
    // inputs copied in
    mlip::DevBuf pos, species;
    // build scratch
    mlip::DevBuf cell_of, wrapp, cell_cnt, cell_start, cell_fill, sid, sx, sy, sz, swrap, counts, keys, stage, pair_aux, flags,
        scan_tmp, small;
    // whole-graph CSR
    mlip::DevBuf row_ptr, senders, recv, mirror, shiftp, d, chunk_row;
    // Verlet skin (mlip_graph_set_skin): candidate list for r_cut + skin and the positions it was built at
    double skin = 0.0;
    bool cand_valid = false;
    int64_t cand_N = 0, cand_E = 0;
    double cand_rcut = 0.0, cand_skin = 0.0, cand_cell[9] = {0};
    int64_t skin_builds = 0, skin_reuses = 0;
    mlip::DevBuf cand_row_ptr, cand_senders, cand_recv, cand_shiftp, cand_d, cand_mirror, ref_pos;
    // partition
    mlip::DevBuf slab_of, needed_by, local_of, local_in_owner, class_cnt, class_off;
    mlip::PartStore part;
    std::vector<mlip::SlabView> slabs;  // P views (empty when P == 1)
    mlip::SlabView whole;
    // forward scratch shared by all views
    mlip::DevBuf wpack, energy_part;
    mlip::DevBuf pair_cnt, pair_scan;   // upper-edge flags over the partitions' edges and their scan (scratch)
    mlip::DevBuf work;        // work counters of the edge kernels: one set of 8 per launch of a call, zeroed per call
    int32_t *work_ptr = nullptr;
    int work_next = 0;        // launches that have taken their counters in the current call
    mlip::Profiler prof;
    mlip::DevBuf bond_wpack;  // packed weights of the three-body variant's bond part
    void *pinned = nullptr;  // small pinned host staging area
};

namespace mlip {

// device-wide exclusive scans (n + 1 outputs, out[n] = total); tmp is grown as needed
int scan_i32_to_i64(const int32_t *in, int64_t *out, int64_t n, DevBuf &tmp, hipStream_t s);
int scan_i32_to_i32(const int32_t *in, int32_t *out, int64_t n, DevBuf &tmp, hipStream_t s);

void prof_begin(mlip_graph *g, int group);
void prof_end(mlip_graph *g);

int build_graph_impl(mlip_graph *g, const double *positions, const double *cell, const int32_t *species,
                     int64_t n_atoms, double r_cut, int32_t n_slabs);
// scratch != nullptr: every piece of workspace is carved from it (nothing is allocated, nothing cached)
int forward_impl(mlip_graph *g, const mlip_weights_t *w, int32_t mode, double *energy, float *forces,
                 float *atom_energy, Carver *scratch);
int unpack_shifts(const mlip_graph *g, int32_t *out);
// bond list of one partition for cutoff r_bond (kept until the graph is rebuilt or r_bond changes); synchronises
int build_bonds_impl(mlip_graph *g, SlabView &v, double r_bond, int p_envelope);
// Upper / lower split of the views' owned-row edges (PairGraph), all views in the same launches; does nothing if all are valid.  With a block to carve from,
// the arrays are taken from it (and the caller invalidates the structure when the block is given up).
int build_pairs_impl(mlip_graph *g, SlabView *views, int n_views, bool slots_full, Carver *scratch);
int forward_bonds_impl(mlip_graph *g, const mlip_weights_t *w, const mlip_bond_weights_t *bw, int32_t mode,
                       double *energy, float *forces, float *atom_energy);

}  // namespace mlip

/*
 * libmlip -- graph-partitioned inference of a radial message-passing
 * interatomic potential on one AMD MI355X (gfx950).  C ABI, no C++ or torch
 * types.  Every pointer argument is marked HOST or DEVICE.
 *
 * The problem statement followed here is the paper's: the inputs are atom
 * positions, the periodic cell and chemical identities (Introduction,
 * E = phi(r_i, C_i); appendix "Parallelizing a Model": the distributed object
 * takes positions, periodic boundary conditions and cell lattice and builds
 * the graph partitions and their transfer metadata), the output is the energy
 * and the forces F = -dE/dr obtained by a reverse pass that runs through the
 * per-layer border-node transfers (Introduction, "graph-level partitioning";
 * Methods, "Graph-Parallel Message Passing").
 *
 * Conventions
 *   - every function returns 0 (MLIP_OK) or a negative mlip_status; no C++
 *     exception or abort crosses this boundary; on error no output argument is
 *     written and mlip_last_error() describes the failure (thread-local text);
 *   - a graph handle owns all device memory it obtains - from the caller's
 *     allocator if the handle was made by mlip_graph_create with one, from
 *     hipMalloc otherwise - until mlip_graph_destroy; inputs are borrowed for
 *     the duration of the call and never written; one handle must not be used
 *     from two threads at once (different handles may be);
 *   - all work is enqueued on the HIP stream given to mlip_build_graph
 *     (a hipStream_t passed as void*, NULL = default stream); outputs of
 *     mlip_forward are valid after that stream is synchronised;
 *   - atoms are numbered 0..N-1 in input order; edges are directed i <- j
 *     (i receives, j sends) and carry an integer image shift S so that the
 *     sender's image sits at r_j + S.C, C = rows of `cell`.
 */
#ifndef MLIP_H
#define MLIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MLIP_OK = 0,
    MLIP_EINVAL = -1,      /* null pointer, N <= 0, r_cut <= 0, n_slabs outside [1,64], bad model dims */
    MLIP_ECELL = -2,       /* singular cell, or cell/positions outside the supported image range */
    MLIP_ECOINCIDENT = -3, /* two atoms (or an atom and an image) at distance 0 */
    MLIP_ENOMEM = -4,      /* device allocation failed */
    MLIP_EHIP = -5,        /* HIP runtime error */
    MLIP_ESTATE = -6       /* call not valid for this handle (e.g. SLABS mode on a graph built with n_slabs = 1) */
} mlip_status;

enum { MLIP_MODE_WHOLE = 0, MLIP_MODE_SLABS = 1 };
/*
 * MLIP_PRECISION_FP32: everything from the basis on in fp32 (fp32 MFMA).
 * MLIP_PRECISION_BF16: the F x F products of the filter MLP (forward w = SiLU(t) W2, reverse sbar = wbar W2^T)
 *   take bf16 operands with fp32 accumulation (benchmark configuration 4: "edge MLPs in bf16 with fp32
 *   accumulation"), and in mlip_forward_bonds the F x F products of the bond MLPs as well; everything else stays
 *   fp32 (arrays, the K = 8 products, activations, sums).  Forces then agree with the fp64 result to about
 *   4e-3 max|F|.
 * MLIP_PRECISION_FP32_SPLIT: the same products (the bond MLPs' included) with every operand split into two fp16 parts (hi + lo, 22
 *   significant bits) and taken as three fp16 MFMA products with fp32 accumulation.  The results meet the fp32
 *   mode's bounds (the dropped terms are of the size of fp32 accumulation rounding) in a fraction of the matrix
 *   time; the operands of those products - SiLU outputs and the products abar * g of the reverse pass - must
 *   stay below the fp16 range (65504), which holds for any physical input but is not checked: a value beyond it
 *   becomes infinite in the split and the energy and forces come out non-finite.
 */
enum { MLIP_PRECISION_FP32 = 0, MLIP_PRECISION_BF16 = 1, MLIP_PRECISION_FP32_SPLIT = 2 };

typedef struct mlip_graph mlip_graph_t;

/*
 * Caller-supplied device allocator (appendix "Parallelizing a Model": the distributed object owns the graph
 * metadata while the features live in the framework's tensors - here the framework's allocator hands out every
 * device block the handle uses, graph arrays and feature workspace alike, so that the framework's memory
 * accounting sees them).
 *   alloc(bytes, ctx)  returns a DEVICE pointer aligned to at least 256 bytes, valid on the handle's stream, or
 *                      NULL when out of memory (the call in progress then fails with MLIP_ENOMEM);
 *   free(ptr, ctx)     takes a block back; the library synchronises the handle's stream first, so no enqueued
 *                      kernel still uses the block.
 * Both are called on the thread that calls into the library, only from mlip_build_graph, mlip_forward,
 * mlip_forward_bonds and mlip_graph_destroy.  Buffers are grow-only: a rebuilt handle asks for memory only when
 * a buffer must grow.
 */
typedef struct {
    void *(*alloc)(size_t bytes, void *ctx);
    void (*free)(void *ptr, void *ctx);
    void *ctx;
} mlip_alloc_t;

/*
 * Creates an empty handle that takes all its device memory from `alloc` (copied; NULL or a NULL alloc function:
 * hipMalloc / hipFree).  Pass the handle to mlip_build_graph, which fills it.  mlip_build_graph with *graph ==
 * NULL is the same as creating a handle without an allocator first.
 */
int mlip_graph_create(const mlip_alloc_t *alloc, mlip_graph_t **graph);

/*
 * Weights of the radial message-passing potential (benchmark configuration 0
 * defines it): species embedding; per layer l the filter MLP W1_l (K x F),
 * W2_l (F x F), the sender projection Wm_l (F x F) and the update Wo_l (F x F);
 * readout Wr1 (F x F), wr2 (F).  All fp32, row-major [fan_in][fan_out]
 * (y = x W), no biases.  DEVICE pointers, borrowed.
 * Supported: F in {32, 64}, K = 8, 0 <= L <= 8, 2 <= p <= 64, n_species >= 1.
 */
typedef struct {
    int32_t n_species, F, L, K, p, precision;
    const float *emb; /* [n_species][F] */
    const float *W1;  /* [L][K][F] */
    const float *W2;  /* [L][F][F] */
    const float *Wm;  /* [L][F][F] */
    const float *Wo;  /* [L][F][F] */
    const float *Wr1; /* [F][F] */
    const float *wr2; /* [F] */
} mlip_weights_t;

/*
 * One partition's node array and local graph (Alg. "Atom Subgraph Creation":
 * concatenated buckets plus a marker array of span starts).  All pointers are
 * DEVICE memory borrowed from the handle, valid until the next
 * mlip_build_graph on it or its destruction.
 *
 *   nodes[n_local]   local -> global atom id, laid out as
 *                    PURE | BORDER | FROM[0] | FROM[1] | ... | FROM[P-1]
 *                    (BORDER = owned atoms some other partition needs, stored
 *                    once; every span in ascending global id)
 *   markers[P+3]     HOST copy of the span starts: 0, |PURE|, |PURE|+|BORDER|
 *                    (= n_owned), then the cumulative FROM lengths
 *   row_ptr[n_local+1], senders[n_edges]
 *                    receiver-sorted CSR over local rows with local sender ids.
 *                    Rows [0, n_owned) are the owned atoms' complete rows (the
 *                    edges this partition computes: an edge belongs to the
 *                    partition of its receiving node, Distributing Atom Graphs);
 *                    rows [n_owned, n_local) list, for each ghost atom, only its
 *                    neighbours owned by this partition (used by the reverse
 *                    pass to form the ghost rows' gradients without atomics).
 *                    Order inside a row: ascending (global sender id, Sx, Sy, Sz).
 */
typedef struct {
    int64_t n_owned, n_pure, n_border, n_ghost, n_local;
    int64_t n_edges_owned; /* edges of rows [0, n_owned)  */
    int64_t n_edges;       /* edges of all local rows     */
    const int32_t *nodes;
    const int64_t *markers; /* HOST */
    const int64_t *row_ptr;
    const int32_t *senders;
    const int32_t *owned_sorted; /* the n_owned owned atoms, ascending global id */
} mlip_slab_info_t;

/*
 * Build the periodic radius graph and its slab partition
 * (neighbour-list construction, Graph-Parallel Message Passing; vertical-wall
 * partition and PURE/TO/FROM buckets, Distributing Atom Graphs, Algs.
 * "Atom Subgraph Creation" and "assign_to_partitions").
 *
 *   positions  DEVICE [n_atoms][3] fp64, Cartesian Angstrom, need not lie inside the cell
 *   cell       HOST   [3][3] fp64, rows are the lattice vectors; full periodic boundaries
 *   species    DEVICE [n_atoms] int32 in [0, n_species)
 *   r_cut      edge iff 0 < d <= r_cut with
 *                delta_k = (r_j,k - r_i,k) + ((Sx C[0][k] + Sy C[1][k]) + Sz C[2][k]),
 *                d^2 = (delta_x^2 + delta_y^2) + delta_z^2 in fp64 without FMA contraction
 *   n_slabs    P >= 1 equal-width slabs along the longest lattice vector (ties: lowest index);
 *              slab(i) = min(floor(f P), P-1), f = fractional coordinate wrapped into [0,1),
 *              computed as ((x n_x + y n_y) + z n_z) / V with n = a_{k+1} x a_{k+2}, V = a_k . n
 *   stream     hipStream_t as void*
 *   graph      in/out HOST: *graph == NULL creates a handle; a handle from an earlier call is
 *              rebuilt in place and reuses its device buffers (grow-only)
 *
 * Edges are stored sorted by (receiver, sender, Sx, Sy, Sz).  The call synchronises the
 * stream a few times (edge and partition sizes are needed on the host).
 * Positions and species are copied into the handle.
 */
int mlip_build_graph(const double *positions, const double *cell, const int32_t *species,
                     int64_t n_atoms, double r_cut, int32_t n_slabs, void *stream,
                     mlip_graph_t **graph);

/*
 * Verlet skin for repeated builds on one handle (molecular dynamics: the paper's workload is long MD with the graph
 * and its partition rebuilt at every step - "Molecular Dynamics Simulation Stability", appendix "Graph
 * Partitioning").  With skin > 0 the handle keeps a candidate neighbour list for the cutoff r_cut + skin and the
 * positions it was built at.  A later mlip_build_graph with the same atom count, cell and r_cut first checks, on the
 * device, that no atom has moved further than skin / 2 from those positions; if so the neighbour list is the
 * candidates that pass the edge test at the new positions (no cell list, no search, no sort: same fp64 expression,
 * same order, so the graph is bit-identical to a fresh build), otherwise the candidate list is rebuilt first.
 * Positions must be continuous between builds (an atom folded back into the cell by a lattice vector counts as
 * moved).  Species may change freely.  skin = 0 (the default) searches at every build.  The partition is built
 * from the neighbour list either way.
 */
int mlip_graph_set_skin(mlip_graph_t *graph, double skin);
/* How often the candidate list was rebuilt and how often it was reused since the handle was made (HOST outputs). */
int mlip_graph_skin_stats(const mlip_graph_t *graph, int64_t *list_builds, int64_t *list_reuses);

/*
 * Energy and forces (Methods: per-layer border-node transfer forward, the same
 * transfers reversed for the gradients; appendix "Parallelizing a Model":
 * distribute / atom_transfer / aggregate).
 *
 *   mode          MLIP_MODE_WHOLE: one partition holding every atom;
 *                 MLIP_MODE_SLABS: the P slabs processed one after another, ghost rows
 *                 refreshed from their owners before every layer's edge step, ghost-row
 *                 gradients (features and positions) added back to the owners in the reverse pass
 *   energy        DEVICE [1] fp64, sum of the per-atom energies of owned atoms
 *   forces        DEVICE [n_atoms][3] fp32, F = -dE/dr, input atom order
 *   atom_energy   DEVICE [n_atoms] fp32 or NULL
 *
 * Asynchronous on the graph's stream; does not modify the graph's topology (it uses
 * workspace owned by the handle, so two forwards on one handle must not overlap).
 *
 * The weights are re-laid-out for the matrix units on the first call and kept in the handle: a later call whose
 * mlip_weights_t (pointers, dimensions, precision) is identical reuses them.  After changing weight VALUES in
 * place, call mlip_graph_invalidate_weights.
 */
int mlip_forward(mlip_graph_t *graph, const mlip_weights_t *weights, int32_t mode,
                 double *energy, float *forces, float *atom_energy);

/*
 * mlip_forward for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, results and error codes as mlip_forward, but every
 * piece of workspace (node features and their gradients, kept filter values, per-edge accumulators, packed
 * weights, energy partial sums) is carved from one fixed device array inside the library of
 * mlip_static_scratch_bytes() = 64 MiB per GPU, held until the process ends; the call allocates and frees
 * nothing and clears what must start at zero with fill kernels.  A graph and model whose workspace
 * (about n_local (4 + 2 L) F 4 + n_edges (36 + L F 2) bytes summed over the partitions of the mode - the kept
 * filter values take one row per edge pair and layer, the lists of the pairs' edges are rebuilt in the array on
 * every call - plus the packed weights) exceeds the array are rejected with MLIP_EINVAL; with the event profiler enabled the call
 * returns MLIP_ESTATE.  All calls on one GPU, from any handle, share the array and find the previous call's
 * contents in it: calls that overlap on one GPU (two streams, two threads) race and must be serialised by the
 * caller.  Weights are packed on every call (nothing is cached in the shared array).  The graph itself must
 * have been built before (mlip_build_graph allocates).
 */
int mlip_forward_static(mlip_graph_t *graph, const mlip_weights_t *weights, int32_t mode,
                        double *energy, float *forces, float *atom_energy);
size_t mlip_static_scratch_bytes(void);

/* Drops the handle's packed copies of the weights (two-body and bond part); the next forward call packs again. */
int mlip_graph_invalidate_weights(mlip_graph_t *graph);

/*
 * Three-body (bond graph) variant: benchmark configuration 4; the paper's counterpart is the bond graph built
 * over the atom graph, whose nodes are the atom-graph edges within a second, smaller cutoff (Methods,
 * "Distributing Bond Graphs").  Extra weights, all fp32 row-major [fan_in][fan_out], DEVICE, borrowed:
 *   We0 [K][F]        bond embedding  e0_b = bbond(d_b) We0 (Bessel basis and envelope at r_bond)
 *   Wt1 [2F + A][F]   first triplet layer, input [e0_b1, e0_b2, cos(n theta) n = 0..A-1]
 *   Wt2 [F][F]        second triplet layer, applied to sum_{b2 != b1} u_b2 SiLU(.)
 *   Wb  [L][F][F]     bond term of layer l's filter: w_e += e1_b Wb_l for a bonded edge
 * with e1_b = e0_b + u_b SiLU(m_b), u_b = u(d_b / r_bond).  A = 8.
 */
typedef struct {
    float r_bond;
    int32_t A;
    const float *We0, *Wt1, *Wt2, *Wb;
} mlip_bond_weights_t;

/*
 * Energy and forces of the three-body variant.  Arguments as mlip_forward, both modes.  The bond list of a
 * partition (edges of its owned rows with d <= r_bond, same fp64 predicate as the neighbour list; all bonds and
 * triplets of an owned centre are local to its partition) is built on the first call after a graph build or a
 * change of r_bond, which synchronises the stream once per partition.
 */
int mlip_forward_bonds(mlip_graph_t *graph, const mlip_weights_t *weights, const mlip_bond_weights_t *bond_weights,
                       int32_t mode, double *energy, float *forces, float *atom_energy);

/*
 * Bond list of the last mlip_forward_bonds, of the whole graph (p = -1, after a WHOLE call) or of partition p
 * (after a SLABS call).  Borrowed DEVICE pointers: bond_edge[n_bonds] = index of every bond's edge in that
 * graph's CSR, ascending; bond_ptr[rows + 1] = bonds of owned row i are bond_ptr[i] .. bond_ptr[i + 1];
 * n_bonds HOST.
 */
int mlip_graph_bonds(const mlip_graph_t *graph, int32_t p, const int32_t **bond_edge, const int64_t **bond_ptr,
                     int64_t *n_bonds);

/*
 * Upper / lower split of the edges of partition p's owned rows (p = -1: of the whole graph), the form in which the
 * fp32 edge kernels walk them.  The filter of the radial message-passing layer is a function of the edge length
 * alone (benchmark description: w_e = MLP(basis(d_e))), and the two edges of an edge / reverse-edge pair have the
 * same length, so the filter is evaluated for one of them, the "upper" one: the edge whose reverse edge lies at a
 * larger index of the partition's edge list.  (An edge from a ghost sender is always upper: its reverse edge is in
 * a ghost row, behind all owned rows.)  All other edges of the owned rows are "lower".
 * Borrowed DEVICE pointers, valid until the next mlip_build_graph on the handle:
 *   u_row_ptr [n_owned + 1]   CSR of the upper edges over the owned rows, the edges in the order of the full list
 *   u_senders, u_eid, u_mirror [n_upper]   sender row, index of the edge and index of its reverse edge in the full list
 *   u_d [n_upper]             edge length
 *   l_row_ptr [n_owned + 1], l_senders [n_lower]   the same for the lower edges
 *   l_slot [n_lower]          index of the pair's upper edge in the upper-edge lists
 * Built on the handle's stream on first use after a graph build (mlip_forward does the same); n_upper and n_lower
 * are HOST values.  Errors: MLIP_ESTATE without a graph, MLIP_EINVAL for a partition index out of range.
 */
typedef struct {
    int64_t n_upper, n_lower;
    const int64_t *u_row_ptr;
    const int32_t *u_senders, *u_eid, *u_mirror;
    const float *u_d;
    const int64_t *l_row_ptr;
    const int32_t *l_senders, *l_slot;
} mlip_pairs_t;
int mlip_graph_pairs(mlip_graph_t *graph, int32_t p, mlip_pairs_t *out);

void mlip_graph_destroy(mlip_graph_t *graph);

/*
 * N atoms, E directed edges, P slabs, all HOST outputs (any may be NULL): the sizes of the graph object the
 * paper's create_distributed returns (appendix "Parallelizing a Model in DistMLIP").
 */
int mlip_graph_sizes(const mlip_graph_t *graph, int64_t *n_atoms, int64_t *n_edges, int32_t *n_slabs);

/*
 * Whole-graph CSR, borrowed DEVICE pointers: row_ptr[N+1], senders[E], d[E] (fp32 edge lengths).  This is what the
 * paper's graph object exposes as src_nodes / dst_nodes (appendix "Parallelizing a Model in DistMLIP"): edge e of
 * row i has destination (receiver) i and source senders[e]; the neighbour list itself is the one of Methods,
 * "Graph-Parallel Message Passing".
 */
int mlip_graph_csr(const mlip_graph_t *graph, const int64_t **row_ptr, const int32_t **senders,
                   const float **d);

/*
 * mirror[E] (DEVICE, borrowed): position of every edge's reverse edge, i.e. for e = (i <- j, S) the
 * index of (j <- i, -S).  The edge set of a radius graph is symmetric; the reverse pass uses this to
 * evaluate the distance derivative once per pair.
 */
int mlip_graph_mirror(const mlip_graph_t *graph, const int32_t **mirror);

/*
 * Image shifts of all edges written to a caller-owned DEVICE buffer [E][3] int32 (enqueued on the stream): the
 * periodic-boundary part of an edge (the distributed object is built from positions, periodic boundary
 * conditions and the cell lattice, appendix "Parallelizing a Model in DistMLIP"); the sender's image sits at
 * r_j + S.C.
 */
int mlip_graph_shifts(const mlip_graph_t *graph, int32_t *shifts);

/*
 * slab_of[N] (DEVICE, borrowed) and the axis the walls are perpendicular to (HOST): the vertical-wall partition
 * of Methods, "Distributing Atom Graphs" (walls along the longest cell dimension; appendix "Graph Partitioning").
 */
int mlip_graph_slab_of(const mlip_graph_t *graph, const int32_t **slab_of, int32_t *axis);

/* Partition p's node array and local graph. */
int mlip_graph_slab(const mlip_graph_t *graph, int32_t p, mlip_slab_info_t *info);

/*
 * FROM_p[q]: atoms partition p receives from partition q (ascending global ids), a span of p's
 * node array.  TO_q[p] is by construction the same array (Distributing Atom Graphs), so
 * mlip_graph_to(g, q, p, ...) returns the same pointer.  DEVICE, borrowed.
 */
int mlip_graph_from(const mlip_graph_t *graph, int32_t p, int32_t q, const int32_t **ids, int64_t *n);
int mlip_graph_to(const mlip_graph_t *graph, int32_t p, int32_t q, const int32_t **ids, int64_t *n);

/*
 * Per-kernel-group timing with HIP events on the graph's stream.  While enabled, every launch
 * group is bracketed by events; mlip_profile_read synchronises the stream and returns, for each of
 * the MLIP_PROF_COUNT groups, the accumulated milliseconds and launch count since the last reset.
 */
enum {
    MLIP_PROF_GRAPH = 0,   /* neighbour list, CSR, partition                 */
    MLIP_PROF_NODE = 1,    /* embedding, node projections/updates, readout    */
    MLIP_PROF_EDGE_FWD = 2,
    MLIP_PROF_EDGE_BWD = 3,
    MLIP_PROF_GHOST = 4,   /* ghost row copies and gradient add-backs         */
    MLIP_PROF_FORCE = 5,   /* force assembly and energy reduction            */
    MLIP_PROF_BOND = 6,    /* three-body variant: bond list and the kernels over bonds */
    MLIP_PROF_TRIPLET_FWD = 7,   /* three-body variant: the triplet sum           */
    MLIP_PROF_TRIPLET_BWD = 8,   /* three-body variant: its reverse               */
    MLIP_PROF_EDGE_FWD_LOWER = 9, /* forward edge step, second pass (where the edge kernels run on one edge per edge /
                                     reverse-edge pair: the terms of the pairs' lower edges, from the kept filter values) */
    MLIP_PROF_EDGE_BWD_LOWER = 10, /* reverse edge step, second pass (the same for the gradients of the projected rows) */
    MLIP_PROF_COUNT = 11
};
int mlip_profile_enable(mlip_graph_t *graph, int32_t on);
int mlip_profile_read(mlip_graph_t *graph, float *ms /*HOST [MLIP_PROF_COUNT]*/,
                      int64_t *launches /*HOST [MLIP_PROF_COUNT]*/, int32_t reset);

/* Plain device -> host copy of `bytes` bytes after synchronising the graph's stream. */
int mlip_copy_to_host(const mlip_graph_t *graph, void *dst_host, const void *src_device, size_t bytes);

const char *mlip_last_error(void);
const char *mlip_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MLIP_H */

// C ABI of libmlip: argument checks, handle lifetime, error text, event profiler.
#include "mlip_internal.h"

#include <cstring>
#include <mutex>
#include <new>

namespace mlip {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

// allocator and stream of the handle the calling thread is working on (AllocScope)
static thread_local mlip_alloc_t t_alloc = {nullptr, nullptr, nullptr};
static thread_local hipStream_t t_stream = nullptr;
static thread_local bool t_scope = false;

AllocScope::AllocScope(const mlip_graph *g)
{
    t_alloc = g->alloc;
    t_stream = g->stream;
    t_scope = true;
}

AllocScope::~AllocScope()
{
    t_alloc = {nullptr, nullptr, nullptr};
    t_stream = nullptr;
    t_scope = false;
}

static void *raw_alloc(const mlip_alloc_t &a, size_t bytes, const char **why)
{
    void *np = nullptr;
    if (a.alloc) {
        np = a.alloc(bytes, a.ctx);
        if (!np) *why = "the caller's allocator returned NULL";
        return np;
    }
    const hipError_t e = hipMalloc(&np, bytes);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        *why = hipGetErrorString(e);
        return nullptr;
    }
    return np;
}

int DevBuf::ensure(size_t bytes)
{
    if (bytes <= cap) return MLIP_OK;
    // grow with slack so that a slowly growing system does not reallocate every step
    size_t want = bytes + bytes / 8 + 256;
    const char *why = "";
    void *np = raw_alloc(t_alloc, want, &why);
    if (!np) {
        want = bytes + 256;  // kernels may read (never use) up to 128 bytes past the end of index arrays
        np = raw_alloc(t_alloc, want, &why);
    }
    if (!np) {
        set_error("device allocation of %zu bytes failed: %s", bytes, why);
        return MLIP_ENOMEM;
    }
    release();
    p = np;
    cap = want;
    owner = t_alloc;
    return MLIP_OK;
}

void DevBuf::release()
{
    if (p) {
        if (owner.alloc) {
            // a caller's allocator may hand the block to other work at once: nothing enqueued may still use it
            if (t_scope) (void)hipStreamSynchronize(t_stream);
            if (owner.free) owner.free(p, owner.ctx);
        } else {
            (void)hipFree(p);  // hipFree synchronises, so no kernel still reads the old block
        }
    }
    p = nullptr;
    cap = 0;
}

// ---- profiler: event pairs around launch groups --------------------------

void prof_begin(mlip_graph *g, int group)
{
    Profiler &pr = g->prof;
    if (!pr.on) return;
    if (pr.used + 2 > pr.pool.size()) {
        if (pr.pool.size() >= (size_t)kMaxEvents) return;  // stop recording, keep running
        hipEvent_t a, b;
        if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return;
        pr.pool.push_back(a);
        pr.pool.push_back(b);
        pr.group.push_back(group);
    }
    pr.group[pr.used / 2] = group;
    (void)hipEventRecord(pr.pool[pr.used], g->stream);
    pr.used += 1;
}

void prof_end(mlip_graph *g)
{
    Profiler &pr = g->prof;
    if (!pr.on || (pr.used & 1) == 0) return;
    (void)hipEventRecord(pr.pool[pr.used], g->stream);
    pr.used += 1;
}

static int prof_collect(mlip_graph *g)
{
    Profiler &pr = g->prof;
    if (pr.used & 1) {  // a begin without its end (error path): close it
        (void)hipEventRecord(pr.pool[pr.used], g->stream);
        pr.used += 1;
    }
    MLIP_HIP(hipStreamSynchronize(g->stream));
    for (size_t k = 0; k + 1 < pr.used; k += 2) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, pr.pool[k], pr.pool[k + 1]) == hipSuccess) {
            pr.ms[pr.group[k / 2]] += ms;
            pr.launches[pr.group[k / 2]] += 1;
        }
    }
    pr.used = 0;
    return MLIP_OK;
}

}  // namespace mlip

using namespace mlip;

extern "C" {

const char *mlip_last_error(void) { return g_err; }
const char *mlip_version(void) { return "libmlip 0.1 (gfx950)"; }

int mlip_graph_create(const mlip_alloc_t *alloc, mlip_graph_t **graph)
{
    if (!graph) { set_error("null pointer argument"); return MLIP_EINVAL; }
    if (alloc && alloc->alloc && !alloc->free) { set_error("allocator without a free function"); return MLIP_EINVAL; }
    mlip_graph *g = new (std::nothrow) mlip_graph();
    if (!g) { set_error("host allocation failed"); return MLIP_ENOMEM; }
    if (alloc && alloc->alloc) g->alloc = *alloc;
    *graph = g;
    return MLIP_OK;
}

int mlip_graph_set_skin(mlip_graph_t *g, double skin)
{
    if (!g) { set_error("null graph"); return MLIP_EINVAL; }
    if (!(skin >= 0.0) || !(skin < 1e6)) { set_error("skin must be non-negative and finite"); return MLIP_EINVAL; }
    g->skin = skin;
    g->cand_valid = false;
    return MLIP_OK;
}

int mlip_graph_skin_stats(const mlip_graph_t *g, int64_t *list_builds, int64_t *list_reuses)
{
    if (!g) { set_error("null graph"); return MLIP_EINVAL; }
    if (list_builds) *list_builds = g->skin_builds;
    if (list_reuses) *list_reuses = g->skin_reuses;
    return MLIP_OK;
}

int mlip_graph_invalidate_weights(mlip_graph_t *g)
{
    if (!g) { set_error("null graph"); return MLIP_EINVAL; }
    g->packed_w_valid = false;
    g->packed_bw_valid = false;
    return MLIP_OK;
}

int mlip_build_graph(const double *positions, const double *cell, const int32_t *species, int64_t n_atoms,
                     double r_cut, int32_t n_slabs, void *stream, mlip_graph_t **graph)
{
    if (!positions || !cell || !species || !graph) { set_error("null pointer argument"); return MLIP_EINVAL; }
    if (n_atoms <= 0 || n_atoms > (int64_t)0x7fffff00) { set_error("n_atoms must be in [1, 2^31)"); return MLIP_EINVAL; }
    if (!(r_cut > 0.0) || !(r_cut < 1e6)) { set_error("r_cut must be positive and finite"); return MLIP_EINVAL; }
    if (n_slabs < 1 || n_slabs > kMaxSlabs) { set_error("n_slabs must be in [1, %d]", (int)kMaxSlabs); return MLIP_EINVAL; }
    mlip_graph *g = *graph;
    const bool fresh = (g == nullptr);
    if (fresh) {
        g = new (std::nothrow) mlip_graph();
        if (!g) { set_error("host allocation failed"); return MLIP_ENOMEM; }
    }
    g->stream = static_cast<hipStream_t>(stream);
    if (g->prof.on && g->prof.used + 64 > (size_t)kMaxEvents) (void)prof_collect(g);
    int rc = MLIP_EHIP;
    AllocScope scope(g);
    try {
        rc = build_graph_impl(g, positions, cell, species, n_atoms, r_cut, n_slabs);
    } catch (const std::exception &e) {
        set_error("host exception: %s", e.what());
        rc = MLIP_ENOMEM;
    }
    if (rc != MLIP_OK) {
        if (fresh) mlip_graph_destroy(g);
        return rc;
    }
    *graph = g;
    return MLIP_OK;
}

static int check_forward_args(mlip_graph_t *g, const mlip_weights_t *w, int32_t mode, double *energy, float *forces)
{
    if (!g || !w || !energy || !forces) { set_error("null pointer argument"); return MLIP_EINVAL; }
    if (g->N <= 0) { set_error("graph handle holds no graph"); return MLIP_ESTATE; }
    if (!w->emb || !w->Wr1 || !w->wr2 || (w->L > 0 && (!w->W1 || !w->W2 || !w->Wm || !w->Wo))) {
        set_error("null weight pointer");
        return MLIP_EINVAL;
    }
    if (!(w->F == 32 || w->F == 64) || w->K != 8 || w->L < 0 || w->L > 8 || w->p < 2 || w->p > 64 ||
        w->n_species < 1 || (w->precision < MLIP_PRECISION_FP32 || w->precision > MLIP_PRECISION_FP32_SPLIT)) {
        set_error("unsupported model dimensions (need F in {32,64}, K = 8, 0 <= L <= 8, 2 <= p <= 64, precision 0..2)");
        return MLIP_EINVAL;
    }
    if (g->species_min < 0 || g->species_max >= w->n_species) {
        set_error("species outside [0, n_species)");
        return MLIP_EINVAL;
    }
    if (mode != MLIP_MODE_WHOLE && mode != MLIP_MODE_SLABS) { set_error("unknown mode"); return MLIP_EINVAL; }
    if (mode == MLIP_MODE_SLABS && g->P < 2) {
        set_error("SLABS mode needs a graph built with n_slabs >= 2");
        return MLIP_ESTATE;
    }
    return MLIP_OK;
}

int mlip_forward(mlip_graph_t *g, const mlip_weights_t *w, int32_t mode, double *energy, float *forces,
                 float *atom_energy)
{
    MLIP_TRY(check_forward_args(g, w, mode, energy, forces));
    if (g->prof.on && g->prof.used + 1024 > (size_t)kMaxEvents) (void)prof_collect(g);
    AllocScope scope(g);
    try {
        return forward_impl(g, w, mode, energy, forces, atom_energy, nullptr);
    } catch (const std::exception &e) {
        set_error("host exception: %s", e.what());
        return MLIP_ENOMEM;
    }
}

// ---- mlip_forward_static: the forward call with its whole workspace in a fixed device array of the library.
//
// Each GPU holds its own copy of the array at its own address; the array's name is only a host-side handle
// for hipGetSymbolAddress, whose result (per device) is what kernels and fills are given.
#define MLIP_STATIC_SCRATCH_BYTES (64u << 20)
static __device__ __align__(256) unsigned char scratch[MLIP_STATIC_SCRATCH_BYTES];

enum { kMaxDevices = 64 };
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[kMaxDevices] = {nullptr};

// device address of the array on the current device, looked up once per device
static int static_scratch(void **out)
{
    int dev = -1;
    MLIP_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) { set_error("device index %d out of range", dev); return MLIP_EHIP; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        MLIP_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) { set_error("hipGetSymbolAddress returned a null address for the static workspace"); return MLIP_EHIP; }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return MLIP_OK;
}

size_t mlip_static_scratch_bytes(void) { return (size_t)MLIP_STATIC_SCRATCH_BYTES; }

int mlip_forward_static(mlip_graph_t *g, const mlip_weights_t *w, int32_t mode, double *energy, float *forces,
                        float *atom_energy)
{
    MLIP_TRY(check_forward_args(g, w, mode, energy, forces));
    if (g->prof.on) {   // the event profiler creates events as it goes
        set_error("mlip_forward_static does not run with the event profiler enabled");
        return MLIP_ESTATE;
    }
    void *base = nullptr;
    MLIP_TRY(static_scratch(&base));
    Carver carve;
    carve.base = static_cast<char *>(base);
    carve.size = (size_t)MLIP_STATIC_SCRATCH_BYTES;
    try {
        return forward_impl(g, w, mode, energy, forces, atom_energy, &carve);
    } catch (const std::exception &e) {
        set_error("host exception: %s", e.what());
        return MLIP_ENOMEM;
    }
}

int mlip_forward_bonds(mlip_graph_t *g, const mlip_weights_t *w, const mlip_bond_weights_t *bw, int32_t mode,
                       double *energy, float *forces, float *atom_energy)
{
    MLIP_TRY(check_forward_args(g, w, mode, energy, forces));
    if (!bw || !bw->We0 || !bw->Wt1 || !bw->Wt2 || (w->L > 0 && !bw->Wb)) {
        set_error("null bond weight pointer");
        return MLIP_EINVAL;
    }
    if (bw->A != 8 || !(bw->r_bond > 0.f) || (double)bw->r_bond > g->r_cut) {
        set_error("unsupported bond model (need A = 8 and 0 < r_bond <= r_cut)");
        return MLIP_EINVAL;
    }
    if (g->prof.on && g->prof.used + 1024 > (size_t)kMaxEvents) (void)prof_collect(g);
    AllocScope scope(g);
    try {
        return forward_bonds_impl(g, w, bw, mode, energy, forces, atom_energy);
    } catch (const std::exception &e) {
        set_error("host exception: %s", e.what());
        return MLIP_ENOMEM;
    }
}

int mlip_graph_bonds(const mlip_graph_t *g, int32_t p, const int32_t **bond_edge, const int64_t **bond_ptr,
                     int64_t *n_bonds)
{
    if (!g || g->N <= 0) { set_error("no graph"); return MLIP_ESTATE; }
    if (p < -1 || p >= g->P || (p >= 0 && g->P < 2)) { set_error("partition index out of range"); return MLIP_EINVAL; }
    const BondGraph &B = (p < 0) ? g->whole.bonds : g->slabs[p].bonds;
    if (B.r_bond < 0) { set_error("no bond list: call mlip_forward_bonds in that mode first"); return MLIP_ESTATE; }
    if (bond_edge) *bond_edge = B.edge.as<int32_t>();
    if (bond_ptr) *bond_ptr = B.ptr.as<int64_t>();
    if (n_bonds) *n_bonds = B.n;
    return MLIP_OK;
}

int mlip_graph_pairs(mlip_graph_t *g, int32_t p, mlip_pairs_t *out)
{
    if (!g || g->N <= 0) { set_error("no graph"); return MLIP_ESTATE; }
    if (!out) { set_error("null output"); return MLIP_EINVAL; }
    if (p < -1 || p >= g->P || (p >= 0 && g->P < 2)) { set_error("partition index out of range"); return MLIP_EINVAL; }
    // all partitions of the mode at once, as mlip_forward builds them
    SlabView *views = (p < 0) ? &g->whole : g->slabs.data();
    MLIP_TRY(build_pairs_impl(g, views, p < 0 ? 1 : g->P, /*slots_full=*/false, nullptr));
    const PairGraph &Q = (p < 0) ? g->whole.pairs : g->slabs[p].pairs;
    out->n_upper = Q.n_upper;
    out->n_lower = Q.n_lower;
    out->u_row_ptr = Q.u_row_ptr;
    out->u_senders = Q.u_senders;
    out->u_eid = Q.u_eid;
    out->u_mirror = Q.u_mirror;
    out->u_d = Q.u_d;
    out->l_row_ptr = Q.l_row_ptr;
    out->l_senders = Q.l_senders;
    out->l_slot = Q.l_slot;
    return MLIP_OK;
}

void mlip_graph_destroy(mlip_graph_t *g)
{
    if (!g) return;
    (void)hipStreamSynchronize(g->stream);   // once, here: the buffers' release below need not synchronise again
    DevBuf *bufs[] = {&g->pos, &g->species, &g->cell_of, &g->wrapp, &g->cell_cnt, &g->cell_start, &g->cell_fill,
                      &g->sid, &g->sx, &g->sy, &g->sz, &g->swrap, &g->counts, &g->keys, &g->stage, &g->pair_aux, &g->flags, &g->scan_tmp,
                      &g->small, &g->row_ptr, &g->senders, &g->recv, &g->mirror, &g->shiftp, &g->d, &g->chunk_row, &g->slab_of, &g->needed_by,
                      &g->local_of, &g->local_in_owner, &g->class_cnt, &g->class_off, &g->wpack, &g->energy_part, &g->work, &g->pair_cnt, &g->pair_scan,
                      &g->cand_row_ptr, &g->cand_senders, &g->cand_recv, &g->cand_shiftp, &g->cand_d, &g->cand_mirror, &g->ref_pos};
    for (DevBuf *b : bufs) b->release();
    g->bond_wpack.release();
    auto drop_view = [](SlabView &v) {
        BondGraph &B = v.bonds;
        DevBuf *vb[] = {&v.h, &v.hbar, &v.abar, &v.gbar, &v.eps, &v.dsum, &v.floc, &v.g, &v.a, &v.wst,
                        &B.scan, &B.flag, &B.of_edge, &B.edge, &B.ptr, &B.mirror, &B.sender, &B.d, &B.u, &B.du, &B.rhat,
                        &B.P, &B.Q, &B.S, &B.m, &B.wb, &B.abar_keep, &B.e1bar, &B.Sbar, &B.Pbar, &B.Qbar,
                        &B.ubar, &B.dbond, &B.rbar};
        for (DevBuf *b : vb) b->release();
        PairGraph &Q = v.pairs;
        DevBuf *pb[] = {&Q.b_u_row_ptr, &Q.b_wslot, &Q.b_u_senders, &Q.b_u_recv,
                        &Q.b_u_eid, &Q.b_u_mirror, &Q.b_u_d, &Q.b_u_chunk_row,
                        &Q.b_l_row_ptr, &Q.b_l_senders, &Q.b_l_slot};
        for (DevBuf *b : pb) b->release();
    };
    drop_view(g->whole);
    for (auto &v : g->slabs) drop_view(v);
    {
        PartStore &st = g->part;
        DevBuf *sb[] = {&st.nodes, &st.owned_sorted, &st.ghost_owner, &st.ghost_src, &st.rowlen, &st.row_abs, &st.row_ptr,
                        &st.senders, &st.recv, &st.mirror, &st.shiftp, &st.d, &st.chunk_row, &st.gbase, &st.ghost_local,
                        &st.sizes};
        for (DevBuf *b : sb) b->release();
    }
    for (hipEvent_t e : g->prof.pool) (void)hipEventDestroy(e);
    if (g->pinned) (void)hipHostFree(g->pinned);
    delete g;
}

int mlip_graph_sizes(const mlip_graph_t *g, int64_t *n_atoms, int64_t *n_edges, int32_t *n_slabs)
{
    if (!g) { set_error("null graph"); return MLIP_EINVAL; }
    if (n_atoms) *n_atoms = g->N;
    if (n_edges) *n_edges = g->E;
    if (n_slabs) *n_slabs = g->P;
    return MLIP_OK;
}

int mlip_graph_csr(const mlip_graph_t *g, const int64_t **row_ptr, const int32_t **senders, const float **d)
{
    if (!g || g->N <= 0) { set_error("no graph"); return MLIP_ESTATE; }
    if (row_ptr) *row_ptr = g->row_ptr.as<int64_t>();
    if (senders) *senders = g->senders.as<int32_t>();
    if (d) *d = g->d.as<float>();
    return MLIP_OK;
}

int mlip_graph_mirror(const mlip_graph_t *g, const int32_t **mirror)
{
    if (!g || g->N <= 0) { set_error("no graph"); return MLIP_ESTATE; }
    if (!mirror) { set_error("null pointer argument"); return MLIP_EINVAL; }
    *mirror = g->mirror.as<int32_t>();
    return MLIP_OK;
}

int mlip_graph_shifts(const mlip_graph_t *g, int32_t *shifts)
{
    if (!g || g->N <= 0) { set_error("no graph"); return MLIP_ESTATE; }
    if (!shifts) { set_error("null pointer argument"); return MLIP_EINVAL; }
    return unpack_shifts(g, shifts);
}

int mlip_graph_slab_of(const mlip_graph_t *g, const int32_t **slab_of, int32_t *axis)
{
    if (!g || g->N <= 0) { set_error("no graph"); return MLIP_ESTATE; }
    if (slab_of) *slab_of = g->slab_of.as<int32_t>();
    if (axis) *axis = g->cell.axis;
    return MLIP_OK;
}

int mlip_graph_slab(const mlip_graph_t *g, int32_t p, mlip_slab_info_t *info)
{
    if (!g || g->N <= 0) { set_error("no graph"); return MLIP_ESTATE; }
    if (!info) { set_error("null pointer argument"); return MLIP_EINVAL; }
    if (g->P < 2) { set_error("graph was built with n_slabs = 1"); return MLIP_ESTATE; }
    if (p < 0 || p >= g->P) { set_error("slab index out of range"); return MLIP_EINVAL; }
    const SlabView &v = g->slabs[p];
    info->n_owned = v.n_owned;
    info->n_pure = v.n_pure;
    info->n_border = v.n_border;
    info->n_ghost = v.n_ghost;
    info->n_local = v.n_local;
    info->n_edges_owned = v.n_edges_owned;
    info->n_edges = v.n_edges;
    info->nodes = v.nodes;
    info->markers = v.markers.data();
    info->row_ptr = v.row_ptr;
    info->senders = v.senders;
    info->owned_sorted = v.owned_sorted;
    return MLIP_OK;
}

int mlip_graph_from(const mlip_graph_t *g, int32_t p, int32_t q, const int32_t **ids, int64_t *n)
{
    if (!g || g->N <= 0) { set_error("no graph"); return MLIP_ESTATE; }
    if (!ids || !n) { set_error("null pointer argument"); return MLIP_EINVAL; }
    if (g->P < 2) { set_error("graph was built with n_slabs = 1"); return MLIP_ESTATE; }
    if (p < 0 || p >= g->P || q < 0 || q >= g->P) { set_error("slab index out of range"); return MLIP_EINVAL; }
    const SlabView &v = g->slabs[p];
    *ids = v.nodes + v.markers[2 + q];
    *n = v.markers[3 + q] - v.markers[2 + q];
    return MLIP_OK;
}

int mlip_graph_to(const mlip_graph_t *g, int32_t p, int32_t q, const int32_t **ids, int64_t *n)
{
    return mlip_graph_from(g, q, p, ids, n);
}

int mlip_profile_enable(mlip_graph_t *g, int32_t on)
{
    if (!g) { set_error("null graph"); return MLIP_EINVAL; }
    if (!on && g->prof.on) MLIP_TRY(prof_collect(g));
    g->prof.on = on != 0;
    return MLIP_OK;
}

int mlip_profile_read(mlip_graph_t *g, float *ms, int64_t *launches, int32_t reset)
{
    if (!g) { set_error("null graph"); return MLIP_EINVAL; }
    MLIP_TRY(prof_collect(g));
    for (int k = 0; k < MLIP_PROF_COUNT; ++k) {
        if (ms) ms[k] = g->prof.ms[k];
        if (launches) launches[k] = g->prof.launches[k];
        if (reset) { g->prof.ms[k] = 0.f; g->prof.launches[k] = 0; }
    }
    return MLIP_OK;
}

int mlip_copy_to_host(const mlip_graph_t *g, void *dst_host, const void *src_device, size_t bytes)
{
    if (!g || !dst_host || (!src_device && bytes)) { set_error("null pointer argument"); return MLIP_EINVAL; }
    MLIP_HIP(hipStreamSynchronize(g->stream));
    if (bytes) MLIP_HIP(hipMemcpy(dst_host, src_device, bytes, hipMemcpyDeviceToHost));
    return MLIP_OK;
}

}  // extern "C"

// Periodic radius graph, canonical receiver-sorted CSR and slab partition on gfx950.
//
// Neighbour-list construction (Methods, Graph-Parallel Message Passing): a cell
// list in fractional space with explicit image shifts.  Partition: vertical
// walls along the longest lattice vector and PURE / TO / FROM buckets
// (Distributing Atom Graphs; Algs. "Atom Subgraph Creation" and
// "assign_to_partitions").  All integer results have exactly one correct value
// (canonical order), so they can be compared bit for bit.
//
// This file is compiled with -ffp-contract=off: the edge predicate and the slab
// rule are fixed fp64 expressions whose operation order is part of the interface.
#include "mlip_internal.h"

#include <algorithm>
#include <cmath>
#include <cstring>

namespace mlip {

namespace {

constexpr int kBias = 512;

__host__ __device__ inline uint32_t pack3(int a, int b, int c)
{
    return ((uint32_t)(a + kBias) << 20) | ((uint32_t)(b + kBias) << 10) | (uint32_t)(c + kBias);
}
__host__ __device__ inline void unpack3(uint32_t p, int &a, int &b, int &c)
{
    a = (int)(p >> 20) - kBias;
    b = (int)((p >> 10) & 1023u) - kBias;
    c = (int)(p & 1023u) - kBias;
}

__device__ inline int floordiv(int a, int b)
{
    int q = a / b;
    if ((a % b != 0) && ((a < 0) != (b < 0))) --q;
    return q;
}

enum { ERR_RANGE = 1, ERR_COINCIDENT = 2, ERR_MIRROR = 4, FLAG_STAGE_OVERFLOW = 8 };
// neighbours found by the counting pass are parked in a fixed-width row per atom, from where the sort picks them
// up; an atom with more neighbours than this sets FLAG_STAGE_OVERFLOW and the rows are filled by a second pass
constexpr int kStage = 96;

// ---------------------------------------------------------------- scans

template <class T> __device__ inline T wave_inclusive_scan(T v)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        T n = __shfl_up(v, off, 64);
        if (lane >= off) v += n;
    }
    return v;
}

constexpr int kScanThreads = 256;
constexpr int kScanItems = 4;
constexpr int kScanTile = kScanThreads * kScanItems;

// exclusive scan of one tile held as kScanItems per thread; returns the tile total
template <class T> __device__ inline T block_exclusive_scan(T (&v)[kScanItems], T *lds /*[4]*/)
{
    T sum = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) sum += v[k];
    T inc = wave_inclusive_scan(sum);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 63) lds[wave] = inc;
    __syncthreads();
    T base = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kScanThreads / 64; ++w) {
        T s = lds[w];
        if (w < wave) base += s;
        total += s;
    }
    T run = base + inc - sum;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
        T x = v[k];
        v[k] = run;
        run += x;
    }
    __syncthreads();
    return total;
}

template <class Tin, class Tout>
__global__ void k_tile_sums(const Tin *in, Tout *sums, int64_t n)
{
    __shared__ Tout lds[kScanThreads / 64];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
    Tout v[kScanItems];
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) v[k] = (base + k < n) ? (Tout)in[base + k] : (Tout)0;
    Tout total = block_exclusive_scan(v, lds);
    if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

// out[i] = offsets[tile] + exclusive prefix inside the tile; the last tile also writes out[n]
template <class Tin, class Tout>
__global__ void k_tile_scan(const Tin *in, const Tout *offsets, Tout *out, int64_t n)
{
    __shared__ Tout lds[kScanThreads / 64];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
    Tout v[kScanItems];
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) v[k] = (base + k < n) ? (Tout)in[base + k] : (Tout)0;
    Tout total = block_exclusive_scan(v, lds);
    const Tout off = offsets ? offsets[blockIdx.x] : (Tout)0;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k)
        if (base + k < n) out[base + k] = off + v[k];
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) out[n] = off + total;
}

template <class Tin, class Tout>
int scan_impl(const Tin *in, Tout *out, int64_t n, char *tmp, size_t tmp_bytes, hipStream_t s)
{
    if (n <= 0) {
        if (n == 0) MLIP_HIP(hipMemsetAsync(out, 0, sizeof(Tout), s));
        return MLIP_OK;
    }
    const int64_t tiles = (n + kScanTile - 1) / kScanTile;
    if (tiles == 1) {
        k_tile_scan<Tin, Tout><<<1, kScanThreads, 0, s>>>(in, nullptr, out, n);
        MLIP_HIP(hipGetLastError());
        return MLIP_OK;
    }
    // layout of tmp: sums[tiles] | offsets[tiles + 1] | rest for the recursion
    const size_t need = (size_t)(2 * tiles + 1) * sizeof(Tout);
    if (tmp_bytes < need) { set_error("scan scratch too small"); return MLIP_EINVAL; }
    Tout *sums = reinterpret_cast<Tout *>(tmp);
    Tout *offs = sums + tiles;
    k_tile_sums<Tin, Tout><<<(unsigned)tiles, kScanThreads, 0, s>>>(in, sums, n);
    MLIP_HIP(hipGetLastError());
    MLIP_TRY((scan_impl<Tout, Tout>(sums, offs, tiles, tmp + need, tmp_bytes - need, s)));
    k_tile_scan<Tin, Tout><<<(unsigned)tiles, kScanThreads, 0, s>>>(in, offs, out, n);
    MLIP_HIP(hipGetLastError());
    return MLIP_OK;
}

size_t scan_scratch_bytes(int64_t n)
{
    size_t total = 0;
    while (n > kScanTile) {
        int64_t tiles = (n + kScanTile - 1) / kScanTile;
        total += (size_t)(2 * tiles + 1) * sizeof(int64_t);
        n = tiles;
    }
    return total + 256;
}

}  // namespace

int scan_i32_to_i64(const int32_t *in, int64_t *out, int64_t n, DevBuf &tmp, hipStream_t s)
{
    MLIP_TRY(tmp.ensure(scan_scratch_bytes(n)));
    return scan_impl<int32_t, int64_t>(in, out, n, tmp.as<char>(), tmp.cap, s);
}

int scan_i32_to_i32(const int32_t *in, int32_t *out, int64_t n, DevBuf &tmp, hipStream_t s)
{
    MLIP_TRY(tmp.ensure(scan_scratch_bytes(n)));
    return scan_impl<int32_t, int32_t>(in, out, n, tmp.as<char>(), tmp.cap, s);
}

namespace {

// ---------------------------------------------------------------- binning

__device__ inline double frac_k(const double *r, const double *n, double V)
{
    return ((r[0] * n[0] + r[1] * n[1]) + r[2] * n[2]) / V;
}

// err[0] = flag bits, err[1] = max species seen, err[2] = min species seen
__global__ void k_bin(int64_t N, const double *__restrict__ pos, const int32_t *__restrict__ species,
                      CellParams cp, int32_t *cell_of, uint32_t *wrapp, int32_t *slab_of, int32_t *cell_cnt,
                      int32_t *err)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    {   // species range, one atomic pair per wavefront
        int zmax = i < N ? species[i] : 0, zmin = zmax;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            zmax = max(zmax, __shfl_xor(zmax, off, 64));
            zmin = min(zmin, __shfl_xor(zmin, off, 64));
        }
        if ((threadIdx.x & 63) == 0) {
            // the running extremes only move one way, so a wavefront that cannot move them skips its atomics
            // (thousands of atomics on one address would serialise and dominate this kernel)
            if (zmax > __atomic_load_n(err + 1, __ATOMIC_RELAXED)) atomicMax(err + 1, zmax);
            if (zmin < __atomic_load_n(err + 2, __ATOMIC_RELAXED)) atomicMin(err + 2, zmin);
        }
    }
    if (i >= N) return;
    const double r[3] = {pos[3 * i], pos[3 * i + 1], pos[3 * i + 2]};
    int b[3], w[3];
    int slab = 0;
    bool bad = false;
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        double f = frac_k(r, cp.nrm[k], cp.V);
        double fl = floor(f);
        if (!(fabs(fl) <= 200.0)) { bad = true; fl = 0.0; f = 0.0; }
        w[k] = (int)fl;
        double fr = f - fl;
        int bk = (int)floor(fr * (double)cp.nb[k]);
        bk = bk > cp.nb[k] - 1 ? cp.nb[k] - 1 : bk;
        b[k] = bk < 0 ? 0 : bk;
        if (k == cp.axis) {
            int s = (int)floor(fr * (double)cp.n_slabs);
            s = s > cp.n_slabs - 1 ? cp.n_slabs - 1 : s;
            slab = s < 0 ? 0 : s;
        }
    }
    if (bad) atomicOr(err, ERR_RANGE);
    const int32_t c = (b[0] * cp.nb[1] + b[1]) * cp.nb[2] + b[2];
    cell_of[i] = c;
    wrapp[i] = pack3(w[0], w[1], w[2]);
    slab_of[i] = slab;
    atomicAdd(&cell_cnt[c], 1);
}

__global__ void k_fill_cells(int64_t N, const double *__restrict__ pos, const int32_t *__restrict__ cell_of,
                             const uint32_t *__restrict__ wrapp, const int32_t *__restrict__ cell_start,
                             int32_t *cell_fill, int32_t *sid, double *sx, double *sy, double *sz,
                             uint32_t *swrap)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= N) return;
    const int32_t c = cell_of[i];
    const int32_t slot = cell_start[c] + atomicAdd(&cell_fill[c], 1);
    sid[slot] = (int32_t)i;
    sx[slot] = pos[3 * i];
    sy[slot] = pos[3 * i + 1];
    sz[slot] = pos[3 * i + 2];
    swrap[slot] = wrapp[i];
}

// One thread per atom, atoms taken in cell order so that a wavefront walks the
// same candidate cells.  FILL = false counts and, if `keys` is given, parks the first kStage unsorted keys
// (sender << 32 | packed shift) in the atom's staging row keys[i * kStage ...]; FILL = true writes the keys
// into the atom's CSR row.
// The search is bound by the latency of its dependent loads, not by the fp64 pair tests: the next candidate's
// record is requested before the current one is tested.  (Requesting all 27 bin ranges at once and streaming the
// candidates across bin boundaries needs twice the registers and measured slower.)
template <bool FILL>
__global__ void k_neighbours(int64_t N, CellParams cp, const int32_t *__restrict__ cell_start,
                             const int32_t *__restrict__ sid, const double *__restrict__ sx,
                             const double *__restrict__ sy, const double *__restrict__ sz,
                             const uint32_t *__restrict__ swrap, const int32_t *__restrict__ cell_of,
                             int32_t *counts, const int64_t *__restrict__ row_ptr, uint64_t *keys, int32_t *err)
{
    const int64_t s = (int64_t)xcd_block() * blockDim.x + threadIdx.x;
    if (s >= N) return;
    const int32_t i = sid[s];
    const double xi = sx[s], yi = sy[s], zi = sz[s];
    int wi0, wi1, wi2;
    unpack3(swrap[s], wi0, wi1, wi2);
    int c = cell_of[i];
    const int b2 = c % cp.nb[2];
    c /= cp.nb[2];
    const int b1 = c % cp.nb[1];
    const int b0 = c / cp.nb[1];
    int64_t base = 0, cap = 0;
    if (FILL) { base = row_ptr[i]; cap = row_ptr[i + 1] - base; }
    else base = (int64_t)i * kStage;
    int32_t cnt = 0;
    bool coincident = false;

    struct Rec {   // one candidate: atom id, wrap counts, position
        int32_t j;
        uint32_t w;
        double x, y, z;
    };
    auto load = [&](Rec &r, int32_t q) {
        r.j = sid[q];
        r.w = swrap[q];
        r.x = sx[q];
        r.y = sy[q];
        r.z = sz[q];
    };
    // the pair test for a candidate found in a bin that is (i0, i1, i2) cells away by wrap-around
    auto test = [&](const Rec &r, int i0, int i1, int i2) {
        int wj0, wj1, wj2;
        unpack3(r.w, wj0, wj1, wj2);
        const int S0 = i0 - wj0 + wi0, S1 = i1 - wj1 + wi1, S2 = i2 - wj2 + wi2;
        if (r.j == i && S0 == 0 && S1 == 0 && S2 == 0) return;
        const double t0 = (r.x - xi) + (((double)S0 * cp.C[0] + (double)S1 * cp.C[3]) + (double)S2 * cp.C[6]);
        const double t1 = (r.y - yi) + (((double)S0 * cp.C[1] + (double)S1 * cp.C[4]) + (double)S2 * cp.C[7]);
        const double t2 = (r.z - zi) + (((double)S0 * cp.C[2] + (double)S1 * cp.C[5]) + (double)S2 * cp.C[8]);
        const double d2 = (t0 * t0 + t1 * t1) + t2 * t2;
        if (d2 <= cp.rc2) {
            if (d2 == 0.0) coincident = true;
            if (FILL ? cnt < cap : (keys != nullptr && cnt < kStage))
                keys[base + cnt] = ((uint64_t)(uint32_t)r.j << 32) | pack3(S0, S1, S2);
            ++cnt;
        }
    };

    for (int dx = -cp.reach[0]; dx <= cp.reach[0]; ++dx) {
        int c0 = b0 + dx;
        const int i0 = floordiv(c0, cp.nb[0]);
        c0 -= i0 * cp.nb[0];
        for (int dy = -cp.reach[1]; dy <= cp.reach[1]; ++dy) {
            int c1 = b1 + dy;
            const int i1 = floordiv(c1, cp.nb[1]);
            c1 -= i1 * cp.nb[1];
            for (int dz = -cp.reach[2]; dz <= cp.reach[2]; ++dz) {
                int c2 = b2 + dz;
                const int i2 = floordiv(c2, cp.nb[2]);
                c2 -= i2 * cp.nb[2];
                const int32_t cc = (c0 * cp.nb[1] + c1) * cp.nb[2] + c2;
                const int32_t qe = cell_start[cc + 1];
                int32_t q = cell_start[cc];
                Rec nxt{};
                if (q < qe) load(nxt, q);
                for (; q < qe; ++q) {
                    const Rec cur = nxt;
                    if (q + 1 < qe) load(nxt, q + 1);
                    test(cur, i0, i1, i2);
                }
            }
        }
    }
    if (!FILL) {
        counts[i] = cnt;
        if (keys != nullptr && cnt > kStage) atomicOr(err, FLAG_STAGE_OVERFLOW);
    }
    if (coincident) atomicOr(err, ERR_COINCIDENT);
}

// One wavefront per row: rank sort of the row's (sender, shift) keys (unique,
// so ranks form a permutation), then the edge length in fp64 rounded to fp32.
constexpr int kRowLds = 512;
__global__ void __launch_bounds__(64)
k_sort_rows(int64_t N, CellParams cp, const double *__restrict__ pos, const int64_t *__restrict__ row_ptr,
            const uint64_t *__restrict__ keys_in, int staged_rows, int32_t *senders, int32_t *recv, uint32_t *shiftp,
            float *d)
{
    __shared__ uint64_t lds[kRowLds];
    const int64_t i = xcd_block();
    if (i >= N) return;   // (whole block: the grid is rounded up to a multiple of 8)
    const int lane = threadIdx.x;
    const int64_t base = row_ptr[i];
    const int64_t n = row_ptr[i + 1] - base;
    // unsorted keys of the row: in the staging row of the atom, or already at the row's place
    const uint64_t *keys = staged_rows ? keys_in + i * kStage - base : keys_in;
    const bool staged = n <= kRowLds;
    if (staged)
        for (int64_t m = lane; m < n; m += 64) lds[m] = keys[base + m];
    __syncthreads();
    const double xi = pos[3 * i], yi = pos[3 * i + 1], zi = pos[3 * i + 2];
    for (int64_t m = lane; m < n; m += 64) {
        const uint64_t key = staged ? lds[m] : keys[base + m];
        int64_t rank = 0;
        if (staged) {
            for (int64_t t = 0; t < n; ++t) rank += (lds[t] < key) ? 1 : 0;
        } else {
            for (int64_t t = 0; t < n; ++t) rank += (keys[base + t] < key) ? 1 : 0;
        }
        const int64_t e = base + rank;
        const int32_t j = (int32_t)(key >> 32);
        const uint32_t sp = (uint32_t)key;
        int S0, S1, S2;
        unpack3(sp, S0, S1, S2);
        const double t0 = (pos[3 * (int64_t)j] - xi) + (((double)S0 * cp.C[0] + (double)S1 * cp.C[3]) + (double)S2 * cp.C[6]);
        const double t1 = (pos[3 * (int64_t)j + 1] - yi) + (((double)S0 * cp.C[1] + (double)S1 * cp.C[4]) + (double)S2 * cp.C[7]);
        const double t2 = (pos[3 * (int64_t)j + 2] - zi) + (((double)S0 * cp.C[2] + (double)S1 * cp.C[5]) + (double)S2 * cp.C[8]);
        const double d2 = (t0 * t0 + t1 * t1) + t2 * t2;
        senders[e] = j;
        shiftp[e] = sp;
        recv[e] = (int32_t)i;
        d[e] = (float)sqrt(d2);
    }
}

// ---- pair-wise neighbour search
//
// Every pair {(i <- j, S), (j <- i, -S)} is tested once, by the atom that comes first in cell order: the thread of
// sorted position s looks only at positions q > s (cells after its own in the cell order are taken whole, cells
// before it are skipped, its own cell from s on; q = s only for images of the atom itself, of which the one with
// the larger packed shift is taken).  The edge predicate is symmetric bit for bit (negating every term negates the
// differences exactly), so one test decides both edges.  The finder parks the key of its own edge in its "own"
// staging row (private counter) and the key of the reverse edge in the partner's "partner" staging row (atomic
// counter), and notes in each entry the slot of the other one.  After the rows are sorted, the reverse-edge index
// follows from these notes without any search: half the candidate loads of the one-sided search and no binary
// searches.  Rows are sorted afterwards, so the order in which the atomics hand out slots does not matter.
constexpr int kOwn = 64, kPar = 64;   // staging slots per atom for edges found by the atom itself / by its partners

__global__ void k_neighbours_pairs(int64_t N, CellParams cp, const int32_t *__restrict__ cell_start,
                                   const int32_t *__restrict__ sid, const double *__restrict__ sx,
                                   const double *__restrict__ sy, const double *__restrict__ sz,
                                   const uint32_t *__restrict__ swrap, const int32_t *__restrict__ cell_of,
                                   uint64_t *stage_own, uint64_t *stage_par, uint8_t *pslot_own, uint8_t *pslot_par,
                                   int32_t *n_own, int32_t *n_par, int32_t *err)
{
    const int64_t s = (int64_t)xcd_block() * blockDim.x + threadIdx.x;
    if (s >= N) return;
    const int32_t i = sid[s];
    const double xi = sx[s], yi = sy[s], zi = sz[s];
    int wi0, wi1, wi2;
    unpack3(swrap[s], wi0, wi1, wi2);
    const int32_t c = cell_of[i];
    int cr = c;
    const int b2 = cr % cp.nb[2];
    cr /= cp.nb[2];
    const int b1 = cr % cp.nb[1];
    const int b0 = cr / cp.nb[1];
    int32_t cnt = 0;
    bool coincident = false, overflow = false;

    struct Rec {   // one candidate: atom id, wrap counts, position
        int32_t j;
        uint32_t w;
        double x, y, z;
    };
    auto load = [&](Rec &r, int32_t q) {
        r.j = sid[q];
        r.w = swrap[q];
        r.x = sx[q];
        r.y = sy[q];
        r.z = sz[q];
    };
    // the pair test for the candidate at sorted position q found in a bin that is (i0, i1, i2) cells away by wrap-around
    auto test = [&](const Rec &r, bool self, int i0, int i1, int i2) {
        int wj0, wj1, wj2;
        unpack3(r.w, wj0, wj1, wj2);
        const int S0 = i0 - wj0 + wi0, S1 = i1 - wj1 + wi1, S2 = i2 - wj2 + wi2;
        const uint32_t sp = pack3(S0, S1, S2), sn = pack3(-S0, -S1, -S2);
        if (self && sp <= sn) return;   // the atom itself (zero shift) or the half of its image pairs taken from the other side
        const double t0 = (r.x - xi) + (((double)S0 * cp.C[0] + (double)S1 * cp.C[3]) + (double)S2 * cp.C[6]);
        const double t1 = (r.y - yi) + (((double)S0 * cp.C[1] + (double)S1 * cp.C[4]) + (double)S2 * cp.C[7]);
        const double t2 = (r.z - zi) + (((double)S0 * cp.C[2] + (double)S1 * cp.C[5]) + (double)S2 * cp.C[8]);
        const double d2 = (t0 * t0 + t1 * t1) + t2 * t2;
        if (d2 <= cp.rc2) {
            if (d2 == 0.0) coincident = true;
            const int a = cnt++;
            if (a < kOwn) stage_own[(int64_t)i * kOwn + a] = ((uint64_t)(uint32_t)r.j << 32) | sp;
            else overflow = true;
        }
    };

    for (int dx = -cp.reach[0]; dx <= cp.reach[0]; ++dx) {
        int c0 = b0 + dx;
        const int i0 = floordiv(c0, cp.nb[0]);
        c0 -= i0 * cp.nb[0];
        for (int dy = -cp.reach[1]; dy <= cp.reach[1]; ++dy) {
            int c1 = b1 + dy;
            const int i1 = floordiv(c1, cp.nb[1]);
            c1 -= i1 * cp.nb[1];
            for (int dz = -cp.reach[2]; dz <= cp.reach[2]; ++dz) {
                int c2 = b2 + dz;
                const int i2 = floordiv(c2, cp.nb[2]);
                c2 -= i2 * cp.nb[2];
                const int32_t cc = (c0 * cp.nb[1] + c1) * cp.nb[2] + c2;
                if (cc < c) continue;   // those atoms come before this one: they find the pair
                const int32_t qe = cell_start[cc + 1];
                int32_t q = (cc == c) ? (int32_t)s : cell_start[cc];
                Rec nxt{};
                if (q < qe) load(nxt, q);
                for (; q < qe; ++q) {
                    const Rec cur = nxt;
                    if (q + 1 < qe) load(nxt, q + 1);
                    test(cur, q == (int32_t)s, i0, i1, i2);
                }
            }
        }
    }
    n_own[i] = cnt;
    if (overflow) atomicOr(err, FLAG_STAGE_OVERFLOW);
    if (coincident) atomicOr(err, ERR_COINCIDENT);
}

// The reverse edges, in a pass of their own over what the search parked (one thread per own slot): the slot that a
// partner's counter hands out is not needed during the search, and the atomics travel past the L2, so they are
// issued from as many threads as possible instead of one after another inside the search loop.
__global__ void k_pair_partners(int64_t N, const int32_t *__restrict__ n_own, const uint64_t *__restrict__ stage_own,
                                uint64_t *stage_par, uint8_t *pslot_own, uint8_t *pslot_par, int32_t *n_par, int32_t *err)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t i = idx / kOwn;
    const int a = (int)(idx % kOwn);
    if (i >= N || a >= n_own[i]) return;
    const uint64_t key = stage_own[idx];
    const int64_t j = (int64_t)(key >> 32);
    int S0, S1, S2;
    unpack3((uint32_t)key, S0, S1, S2);
    const int b = atomicAdd(&n_par[j], 1);
    pslot_own[idx] = (uint8_t)(b < 255 ? b : 255);
    if (b < kPar) {
        stage_par[j * kPar + b] = ((uint64_t)(uint32_t)i << 32) | pack3(-S0, -S1, -S2);
        pslot_par[j * kPar + b] = (uint8_t)a;
    } else {
        atomicOr(err, FLAG_STAGE_OVERFLOW);
    }
}

__global__ void k_pair_counts(int64_t N, const int32_t *__restrict__ n_own, const int32_t *__restrict__ n_par, int32_t *counts)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < N) counts[i] = n_own[i] + n_par[i];
}

// k_sort_rows for the pair-wise search: the row's keys come from the atom's two staging rows; the rank of every
// staging slot is kept for the reverse-edge index
__global__ void __launch_bounds__(64)
k_sort_rows_pairs(int64_t N, CellParams cp, const double *__restrict__ pos, const int64_t *__restrict__ row_ptr,
                  const uint64_t *__restrict__ stage_own, const uint64_t *__restrict__ stage_par,
                  const int32_t *__restrict__ n_own, uint8_t *rank_own, uint8_t *rank_par, int32_t *senders, int32_t *recv,
                  uint32_t *shiftp, float *d)
{
    __shared__ uint64_t lds[kOwn + kPar];
    const int64_t i = xcd_block();
    if (i >= N) return;   // (whole block: the grid is rounded up to a multiple of 8)
    const int lane = threadIdx.x;
    const int64_t base = row_ptr[i];
    const int n = (int)(row_ptr[i + 1] - base);
    const int no = n_own[i];
    for (int m = lane; m < n; m += 64)
        lds[m] = (m < no) ? stage_own[i * kOwn + m] : stage_par[i * kPar + (m - no)];
    __syncthreads();
    const double xi = pos[3 * i], yi = pos[3 * i + 1], zi = pos[3 * i + 2];
    for (int m = lane; m < n; m += 64) {
        const uint64_t key = lds[m];
        int rank = 0;
        for (int t = 0; t < n; ++t) rank += (lds[t] < key) ? 1 : 0;
        if (m < no) rank_own[i * kOwn + m] = (uint8_t)rank; else rank_par[i * kPar + (m - no)] = (uint8_t)rank;
        const int64_t e = base + rank;
        const int32_t j = (int32_t)(key >> 32);
        const uint32_t sp = (uint32_t)key;
        int S0, S1, S2;
        unpack3(sp, S0, S1, S2);
        const double t0 = (pos[3 * (int64_t)j] - xi) + (((double)S0 * cp.C[0] + (double)S1 * cp.C[3]) + (double)S2 * cp.C[6]);
        const double t1 = (pos[3 * (int64_t)j + 1] - yi) + (((double)S0 * cp.C[1] + (double)S1 * cp.C[4]) + (double)S2 * cp.C[7]);
        const double t2 = (pos[3 * (int64_t)j + 2] - zi) + (((double)S0 * cp.C[2] + (double)S1 * cp.C[5]) + (double)S2 * cp.C[8]);
        const double d2 = (t0 * t0 + t1 * t1) + t2 * t2;
        senders[e] = j;
        shiftp[e] = sp;
        recv[e] = (int32_t)i;
        d[e] = (float)sqrt(d2);
    }
}

// reverse-edge index from the pair notes: the edge in own slot a of atom i and the edge in partner slot b of atom j
// are each other's reverse; 32 lanes per atom
__global__ void __launch_bounds__(256)
k_mirror_pairs(int64_t N, const int64_t *__restrict__ row_ptr, const uint64_t *__restrict__ stage_own,
               const uint8_t *__restrict__ pslot_own, const int32_t *__restrict__ n_own,
               const uint8_t *__restrict__ rank_own, const uint8_t *__restrict__ rank_par, int32_t *__restrict__ mirror)
{
    const int64_t i = (int64_t)xcd_block() * 8 + (threadIdx.x >> 5);
    if (i >= N) return;
    const int no = n_own[i];
    const int64_t rp = row_ptr[i];
    for (int a = threadIdx.x & 31; a < no; a += 32) {
        const int64_t j = (int64_t)(stage_own[i * kOwn + a] >> 32);
        const int b = pslot_own[i * kOwn + a];
        const int32_t e = (int32_t)(rp + rank_own[i * kOwn + a]);
        const int32_t m = (int32_t)(row_ptr[j] + rank_par[j * kPar + b]);
        mirror[e] = m;
        mirror[m] = e;
    }
}

// chunk_row[c] = first row whose first edge lies at or after c * kChunkEdges; chunk_row[n_chunks] = n_rows.
__global__ void k_chunk_rows(int64_t n_rows, int64_t n_chunks, const int64_t *__restrict__ row_ptr,
                             int32_t *__restrict__ chunk_row)
{
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c > n_chunks) return;
    int64_t lo = 0, hi = n_rows;
    if (c == n_chunks) lo = n_rows;
    const int64_t v = c * kChunkEdges;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (row_ptr[mid] < v) lo = mid + 1; else hi = mid;
    }
    chunk_row[c] = (int32_t)lo;
}

// mirror[e] = position of the reverse edge (send(e) <- recv(e), -S).  The edge predicate is symmetric
// bit for bit, so the reverse edge always exists; rows are sorted by (global sender id, shift), which
// makes this a binary search in the sender's row.  nodes == nullptr: row and sender ids are global.
//   PAIRS: only the edge of each pair whose sender id is the larger one (for a self-image pair: the larger
//          packed shift) searches, and writes both entries of the pair (whole graph);
//   else:  only edges whose sender is at or after min_sender search (local graphs: the senders that are
//          ghost rows; all other entries follow from the whole graph's index, see k_local_fill).
template <bool PAIRS>
__global__ void k_mirror(int64_t E, const int64_t *__restrict__ row_ptr, const int32_t *__restrict__ senders,
                         const int32_t *__restrict__ recv, const uint32_t *__restrict__ shiftp,
                         const int32_t *__restrict__ nodes, int32_t min_sender, int32_t *__restrict__ mirror,
                         int32_t *err)
{
    const int64_t e = (int64_t)xcd_block() * blockDim.x + threadIdx.x;
    if (e >= E) return;
    const int32_t r = recv[e], sd = senders[e];
    if (sd < min_sender) return;
    const uint32_t sp = shiftp[e];
    int a, b, c;
    unpack3(sp, a, b, c);
    const uint32_t sneg = pack3(-a, -b, -c);
    if (PAIRS && (sd < r || (sd == r && sp < sneg))) return;
    const uint32_t want_id = (uint32_t)(nodes ? nodes[r] : r);
    int64_t lo = row_ptr[sd], hi = row_ptr[sd + 1];
    const int64_t end = hi;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        const int32_t sm = senders[mid];
        const uint32_t id = (uint32_t)(nodes ? nodes[sm] : sm);
        bool less = id < want_id;
        if (id == want_id) less = shiftp[mid] < sneg;   // several images of one neighbour: small cells only
        if (less) lo = mid + 1; else hi = mid;
    }
    bool ok = false;
    if (lo < end) {
        const int32_t sm = senders[lo];
        ok = (uint32_t)(nodes ? nodes[sm] : sm) == want_id && shiftp[lo] == sneg;
    }
    if (ok) {
        mirror[e] = (int32_t)lo;
        if (PAIRS) mirror[lo] = (int32_t)e;
    } else {
        mirror[e] = (int32_t)e;
        atomicOr(err, ERR_MIRROR);
    }
}

__global__ void k_unpack_shifts(int64_t E, const uint32_t *__restrict__ shiftp, int32_t *out)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= E) return;
    int a, b, c;
    unpack3(shiftp[e], a, b, c);
    out[3 * e] = a;
    out[3 * e + 1] = b;
    out[3 * e + 2] = c;
}

// ---------------------------------------------------------------- partition

// needed_by[j] gets bit q when some atom owned by slab q != slab(j) receives from j
// (16 lanes per row, 16 rows per block; a bit that is already set is not set again)
__global__ void __launch_bounds__(256)
k_needed_by(int64_t N, const int64_t *__restrict__ row_ptr, const int32_t *__restrict__ senders,
            const int32_t *__restrict__ slab_of, unsigned long long *needed_by)
{
    const int64_t i = (int64_t)xcd_block() * 16 + (threadIdx.x >> 4);
    if (i >= N) return;
    const int si = slab_of[i];
    const int64_t e1 = row_ptr[i + 1];
    for (int64_t e = row_ptr[i] + (threadIdx.x & 15); e < e1; e += 16) {
        const int32_t j = senders[e];
        if (slab_of[j] != si) {
            const unsigned long long bit = 1ull << si;
            if (!(__atomic_load_n(&needed_by[j], __ATOMIC_RELAXED) & bit)) atomicOr(&needed_by[j], bit);
        }
    }
}

// class of atom u relative to partition q: 0 PURE, 1 BORDER, 2 + s ghost owned by slab s, -1 absent
__device__ inline int node_class(int s, unsigned long long nb, int q)
{
    if (s == q) return nb == 0ull ? 0 : 1;
    return ((nb >> q) & 1ull) ? 2 + s : -1;
}

// ---- index sets of all partitions in one pass
//
// Every atom u is a node of its own partition (PURE or BORDER) and a ghost of every partition q whose bit is set in
// needed_by[u] (span FROM_q[slab(u)]).  The node arrays of all partitions sit one after another in one array, each
// laid out PURE | BORDER | FROM[0] | ... | FROM[P-1] with every span in ascending atom id: a stable counting sort
// with the bins (q, c), c = 0 PURE, 1 BORDER, 2 + s FROM[s]  (P (P + 2) bins), followed by P pseudo-bins "owned by
// q" for the ascending list of owned atoms.  One wavefront walks kRange consecutive atoms and keeps its bins'
// counts (first pass) or write positions (second pass) in its own LDS table; between the passes one flat scan over
// cnt[bin][range] turns the counts into positions.
constexpr int kRange = 512;

// What the local-CSR fill needs to know about a sender, in one 16-byte record per atom: its owner partition, its
// row there, and the distance from a position in its global row to the same position in its owner's local row.
struct __attribute__((aligned(16))) OwnRec {
    int32_t local, slab;
    int64_t delta;
};

__device__ inline unsigned long long wave_or(unsigned long long v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v |= __shfl_xor(v, off, 64);
    return v;
}

template <bool SCATTER>
__global__ void __launch_bounds__(256)
k_classes(int64_t N, int P, int64_t nranges, const int32_t *__restrict__ slab_of,
          const unsigned long long *__restrict__ needed_by, int32_t *cnt, const int32_t *__restrict__ off,
          const int32_t *__restrict__ gbase, int32_t *nodes, int32_t *owned_sorted, OwnRec *own_rec,
          int32_t *ghost_local)
{
    extern __shared__ int32_t class_lds[];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int B1 = P * (P + 2), nbins = B1 + P;
    int32_t *tab = class_lds + wave * nbins;
    const int64_t w = (int64_t)blockIdx.x * (blockDim.x >> 6) + wave;
    if (w >= nranges) return;
    for (int b = lane; b < nbins; b += 64) tab[b] = SCATTER ? -1 : 0;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const unsigned long long lt = (1ull << lane) - 1ull;
    const int32_t total_local = SCATTER ? off[(int64_t)B1 * nranges] : 0;   // the pseudo-bins' positions start here
    // position of the wavefront's next entry of bin b (second pass) or its count so far (first pass), advanced by n
    auto take = [&](int b, int n) -> int32_t {
        int32_t pos = 0;
        if (lane == 0) {
            pos = tab[b];
            if (SCATTER && pos < 0) pos = off[(int64_t)b * nranges + w];
            tab[b] = pos + n;
        }
        return __builtin_amdgcn_readfirstlane(pos);
    };
    for (int c = 0; c < kRange / 64; ++c) {
        const int64_t u = w * kRange + c * 64 + lane;
        const bool valid = u < N;
        const int s = valid ? slab_of[u] : 0;
        const unsigned long long nb = valid ? needed_by[u] : 0ull;
        unsigned long long todo = wave_or(valid ? (nb | (1ull << s)) : 0ull);   // partitions some atom of the chunk is in
        while (todo) {
            const int q = __builtin_ctzll(todo);
            todo &= todo - 1;
            const int cls = valid ? node_class(s, nb, q) : -1;
            unsigned long long rem = __ballot(cls >= 0);
            const unsigned long long mo = __ballot(cls == 0 || cls == 1);
            while (rem) {
                const int cc = __builtin_amdgcn_readlane(cls, __builtin_ctzll(rem));
                const unsigned long long m = __ballot(cls == cc);
                rem &= ~m;
                const int32_t pos = take(q * (P + 2) + cc, __popcll(m));
                if (SCATTER && cls == cc) {
                    const int32_t at = pos + __popcll(m & lt);
                    const int32_t loc = at - off[(int64_t)(q * (P + 2)) * nranges];   // index inside partition q
                    nodes[at] = (int32_t)u;
                    if (cc < 2) { own_rec[u].local = loc; own_rec[u].slab = q; }
                    else ghost_local[gbase[u] + __popcll(nb & ((1ull << q) - 1ull))] = loc;
                }
            }
            if (mo) {
                const int32_t pos = take(B1 + q, __popcll(mo));
                if (SCATTER && (cls == 0 || cls == 1)) owned_sorted[pos - total_local + __popcll(mo & lt)] = (int32_t)u;
            }
        }
    }
    if (!SCATTER) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        for (int b = lane; b < nbins; b += 64)
            if (tab[b]) cnt[(int64_t)b * nranges + w] = tab[b];   // cnt is zero-filled beforehand
    }
}

__global__ void k_popcount(int64_t N, const unsigned long long *__restrict__ needed_by, int32_t *out)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < N) out[i] = __popcll(needed_by[i]);
}

// span starts of every partition: out[q * (P + 3) + k] = start of span k of partition q in the concatenated node
// array (k = P + 2: its end); out[P * (P + 3)] = number of ghost entries
__global__ void k_gather_markers(const int32_t *__restrict__ off, int P, int64_t nranges, const int32_t *__restrict__ gbase,
                                 int64_t N, int64_t *out)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    const int n = P * (P + 3);
    if (idx < n) {
        const int q = idx / (P + 3), k = idx % (P + 3);
        out[idx] = off[(int64_t)(q * (P + 2) + k) * nranges];   // (q, P + 2) is bin (q + 1, 0) or the first pseudo-bin
    } else if (idx == n) {
        out[idx] = gbase[N];
    }
}

// Where each partition's pieces start in the concatenated arrays (passed to kernels by value; all scalar reads).
struct PartTab {
    int32_t P;
    int64_t row0[kMaxSlabs + 1];    // first node / row of partition q; row0[P] = total
    int64_t n_owned[kMaxSlabs];
    int64_t ghost0[kMaxSlabs + 1];  // first ghost entry
    int64_t chunk0[kMaxSlabs + 1];  // first work-item table entry
    int64_t n_edges[kMaxSlabs];
};

__device__ inline int part_find(const int64_t *start, int P, int64_t x)
{
    int p = 0;
    for (int q = 1; q < P; ++q)
        if (x >= start[q]) p = q;
    return p;
}

// Length of each local row.  Owned rows keep their whole global row (one thread per owned atom, which knows its
// partition and row from its owner record); ghost rows keep only the senders owned by the partition and also record
// their owner and their row inside the owner (one wavefront per ghost row).  Partition q's lengths start at
// rowlen[row0[q] + q] (one closing entry per partition, zero-filled beforehand, so that one scan yields every
// partition's n_local + 1 offsets).
__global__ void k_owned_rowlen(int64_t N, PartTab T, const OwnRec *__restrict__ own_rec, const int64_t *__restrict__ row_ptr,
                               int32_t *rowlen)
{
    const int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= N) return;
    const OwnRec rec = own_rec[u];
    rowlen[T.row0[rec.slab] + rec.slab + rec.local] = (int32_t)(row_ptr[u + 1] - row_ptr[u]);
}

__global__ void __launch_bounds__(256)
k_ghost_rowlen(PartTab T, const int32_t *__restrict__ nodes, const int64_t *__restrict__ row_ptr,
               const int32_t *__restrict__ senders, const int32_t *__restrict__ slab_of,
               const OwnRec *__restrict__ own_rec, int32_t *rowlen, int32_t *ghost_owner, int32_t *ghost_src)
{
    const int lane = threadIdx.x & 63;
    const int64_t k = (int64_t)xcd_block() * 4 + (threadIdx.x >> 6);   // ghost entry, numbered across the partitions
    if (k >= T.ghost0[T.P]) return;
    const int q = part_find(T.ghost0, T.P, k);
    const int64_t r = T.n_owned[q] + (k - T.ghost0[q]);
    const int64_t x = T.row0[q] + r;
    const int32_t u = nodes[x];
    const int64_t e0 = row_ptr[u], e1 = row_ptr[u + 1];
    int cnt = 0;
    for (int64_t eb = e0; eb < e1; eb += 64) {
        const int64_t e = eb + lane;
        const bool keep = e < e1 && slab_of[senders[e]] == q;
        cnt += __popcll(__ballot(keep));
    }
    if (lane == 0) {
        rowlen[x + q] = cnt;
        ghost_owner[k] = own_rec[u].slab;
        ghost_src[k] = own_rec[u].local;
    }
}

// row_ptr of every partition, starting at 0 (row_abs holds the scan over all partitions' lengths), and per
// partition the edges of its owned rows and of all its rows
__global__ void k_local_rowptr(PartTab T, const int64_t *__restrict__ row_abs, const int32_t *__restrict__ nodes,
                               const int64_t *__restrict__ grow_ptr, int64_t *row_ptr, OwnRec *own_rec, int64_t *sizes)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t total = T.row0[T.P] + T.P;
    if (idx >= total) return;
    int q = 0;
    for (int p = 1; p < T.P; ++p)
        if (idx >= T.row0[p] + p) q = p;
    const int64_t first = T.row0[q] + q;
    const int64_t base = row_abs[first];
    row_ptr[idx] = row_abs[idx] - base;
    if (idx - first < T.n_owned[q]) {   // an owned row: where its edges went, relative to its global row
        const int32_t u = nodes[idx - q];
        own_rec[u].delta = (row_abs[idx] - base) - grow_ptr[u];
    }
    if (idx == first) {
        sizes[2 * q] = row_abs[first + T.n_owned[q]] - base;
        sizes[2 * q + 1] = row_abs[T.row0[q + 1] + q] - base;
    }
}

// Local CSR of every partition.
//
// Owned rows (k_local_fill_owned, one thread per edge of the whole graph): an edge belongs to the partition of its
// receiver, and an owned row is its whole global row, so edge e goes to position e + delta(receiver) of that
// partition's arrays, with the sender's local id; if the sender is owned by the same partition the reverse edge
// keeps its offset inside the sender's row (gmirror[e] + delta(sender)).
// Ghost rows (k_local_fill_ghost, one wavefront per ghost row): the senders the partition owns, in row order.  Each
// such edge (u <- k) is the reverse of the owned-row edge (k <- u), whose position follows from the whole graph's
// reverse-edge index; the wavefront writes both entries of the pair, so no search is needed.
__global__ void __launch_bounds__(256)
k_local_fill_owned(int64_t E, PartTab T, const int32_t *__restrict__ recv, const int32_t *__restrict__ senders,
                   const uint32_t *__restrict__ shiftp, const float *__restrict__ d, const int32_t *__restrict__ gmirror,
                   const unsigned long long *__restrict__ needed_by, const OwnRec *__restrict__ own_rec,
                   const int32_t *__restrict__ gbase, const int32_t *__restrict__ ghost_local,
                   const int64_t *__restrict__ row_abs, int32_t *lsenders, int32_t *lrecv, uint32_t *lshiftp, float *ld,
                   int32_t *lmirror)
{
    const int64_t e = (int64_t)xcd_block() * blockDim.x + threadIdx.x;
    if (e >= E) return;
    const OwnRec ri = own_rec[recv[e]];
    const int q = ri.slab;
    const int64_t o = row_abs[T.row0[q] + q] + (e + ri.delta);   // the partition's first edge + position inside it
    const int32_t j = senders[e];
    const OwnRec rj = own_rec[j];
    const bool jown = rj.slab == q;
    lsenders[o] = jown ? rj.local : ghost_local[gbase[j] + __popcll(needed_by[j] & ((1ull << q) - 1ull))];
    lshiftp[o] = shiftp[e];
    lrecv[o] = ri.local;
    ld[o] = d[e];
    if (jown) lmirror[o] = (int32_t)((int64_t)gmirror[e] + rj.delta);
}

__global__ void __launch_bounds__(256)
k_local_fill_ghost(PartTab T, const int32_t *__restrict__ nodes, const int64_t *__restrict__ row_ptr,
                   const int32_t *__restrict__ senders, const uint32_t *__restrict__ shiftp, const float *__restrict__ d,
                   const int32_t *__restrict__ gmirror, const OwnRec *__restrict__ own_rec,
                   const int64_t *__restrict__ row_abs, int32_t *lsenders, int32_t *lrecv, uint32_t *lshiftp, float *ld,
                   int32_t *lmirror)
{
    const int lane = threadIdx.x & 63;
    const int64_t k = (int64_t)xcd_block() * 4 + (threadIdx.x >> 6);
    if (k >= T.ghost0[T.P]) return;
    const int q = part_find(T.ghost0, T.P, k);
    const int64_t r = T.n_owned[q] + (k - T.ghost0[q]);
    const int64_t x = T.row0[q] + r;
    const int32_t u = nodes[x];
    const int64_t e0 = row_ptr[u], e1 = row_ptr[u + 1];
    const int64_t ebase = row_abs[T.row0[q] + q];   // the partition's first edge in the concatenated edge arrays
    int64_t out = row_abs[x + q];                   // absolute position of the row's first edge
    const unsigned long long lt = (1ull << lane) - 1ull;
    for (int64_t eb = e0; eb < e1; eb += 64) {
        const int64_t e = eb + lane;
        bool keep = false;
        OwnRec rec{};
        if (e < e1) {
            rec = own_rec[senders[e]];
            keep = rec.slab == q;
        }
        const unsigned long long m = __ballot(keep);
        if (keep) {
            const int64_t o = out + __popcll(m & lt);
            const int32_t partner = (int32_t)((int64_t)gmirror[e] + rec.delta);   // the owned row's edge from this ghost
            lsenders[o] = rec.local;
            lshiftp[o] = shiftp[e];
            lrecv[o] = (int32_t)r;
            ld[o] = d[e];
            lmirror[o] = partner;
            lmirror[ebase + partner] = (int32_t)(o - ebase);
        }
        out += __popcll(m);
    }
}

// work-item tables of all partitions: entry c of partition q = first local row whose first edge lies at or after
// c * kChunkEdges; the last entry = n_local
__global__ void k_chunk_rows_parts(PartTab T, const int64_t *__restrict__ lrow_ptr, int32_t *__restrict__ chunk_row)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= T.chunk0[T.P]) return;
    const int q = part_find(T.chunk0, T.P, idx);
    const int64_t c = idx - T.chunk0[q], n_chunks = T.chunk0[q + 1] - T.chunk0[q] - 1;
    const int64_t n_rows = T.row0[q + 1] - T.row0[q];
    const int64_t *rp = lrow_ptr + T.row0[q] + q;
    int64_t lo = 0, hi = n_rows;
    if (c == n_chunks) lo = n_rows;
    const int64_t v = c * kChunkEdges;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (rp[mid] < v) lo = mid + 1; else hi = mid;
    }
    chunk_row[idx] = (int32_t)lo;
}

// ---- neighbour list from a candidate list (Verlet skin)
//
// The candidates of atom i are its neighbour list for the cutoff r_cut + skin at some earlier positions (`ref`),
// sorted like the final rows.  While no atom has moved further than skin / 2 from `ref`, every pair within r_cut is
// among them, so the exact neighbour list is the candidates that pass the fp64 test at the current positions, in
// the same order.  One wavefront per atom; the first pass counts (and checks the displacement, assigns the slab and
// tracks the species range as the binning kernel does), the second writes the rows.
enum { FLAG_DISPLACED = 16 };
template <bool FILL>
__global__ void __launch_bounds__(256)
k_skin_rows(int64_t N, CellParams cp, const double *__restrict__ pos, const double *__restrict__ ref, double half_skin2,
            const int32_t *__restrict__ species, const int64_t *__restrict__ crow, const int32_t *__restrict__ csend,
            const uint32_t *__restrict__ cshift, int32_t *counts, int32_t *slab_of, const int64_t *__restrict__ row_ptr,
            int32_t *senders, int32_t *recv, uint32_t *shiftp, float *d, int32_t *newpos, int32_t *err)
{
    const int lane = threadIdx.x & 63;
    const int64_t i = (int64_t)xcd_block() * 4 + (threadIdx.x >> 6);
    if (i >= N) return;
    const double xi = pos[3 * i], yi = pos[3 * i + 1], zi = pos[3 * i + 2];
    if (!FILL && lane == 0) {
        const double u0 = xi - ref[3 * i], u1 = yi - ref[3 * i + 1], u2 = zi - ref[3 * i + 2];
        if (!((u0 * u0 + u1 * u1) + u2 * u2 <= half_skin2)) atomicOr(err, FLAG_DISPLACED);   // (a NaN counts as moved)
        const double r[3] = {xi, yi, zi};
        double f = frac_k(r, cp.nrm[cp.axis], cp.V);
        double fl = floor(f);
        if (!(fabs(fl) <= 200.0)) { fl = 0.0; f = 0.0; }
        const double fr = f - fl;
        int sl = (int)floor(fr * (double)cp.n_slabs);
        sl = sl > cp.n_slabs - 1 ? cp.n_slabs - 1 : sl;
        slab_of[i] = sl < 0 ? 0 : sl;
        const int z = species[i];
        if (z > __atomic_load_n(err + 1, __ATOMIC_RELAXED)) atomicMax(err + 1, z);
        if (z < __atomic_load_n(err + 2, __ATOMIC_RELAXED)) atomicMin(err + 2, z);
    }
    const int64_t e1 = crow[i + 1];
    int64_t out = FILL ? row_ptr[i] : 0;
    int cnt = 0;
    bool coincident = false;
    const unsigned long long lt = (1ull << lane) - 1ull;
    for (int64_t eb = crow[i]; eb < e1; eb += 64) {
        const int64_t e = eb + lane;
        bool keep = false;
        int32_t j = 0;
        uint32_t sp = 0;
        double d2 = 1.0;
        if (e < e1) {
            j = csend[e];
            sp = cshift[e];
            int S0, S1, S2;
            unpack3(sp, S0, S1, S2);
            const double t0 = (pos[3 * (int64_t)j] - xi) + (((double)S0 * cp.C[0] + (double)S1 * cp.C[3]) + (double)S2 * cp.C[6]);
            const double t1 = (pos[3 * (int64_t)j + 1] - yi) + (((double)S0 * cp.C[1] + (double)S1 * cp.C[4]) + (double)S2 * cp.C[7]);
            const double t2 = (pos[3 * (int64_t)j + 2] - zi) + (((double)S0 * cp.C[2] + (double)S1 * cp.C[5]) + (double)S2 * cp.C[8]);
            d2 = (t0 * t0 + t1 * t1) + t2 * t2;
            keep = d2 <= cp.rc2;
            if (keep && d2 == 0.0) coincident = true;
        }
        const unsigned long long m = __ballot(keep);
        if (FILL && keep) {
            const int64_t o = out + __popcll(m & lt);
            senders[o] = j;
            shiftp[o] = sp;
            recv[o] = (int32_t)i;
            d[o] = (float)sqrt(d2);
        }
        if (FILL && e < e1) newpos[e] = keep ? (int32_t)(out + __popcll(m & lt)) : -1;   // where the candidate went
        out += __popcll(m);
        cnt += __popcll(m);
    }
    if (!FILL) {
        if (lane == 0) counts[i] = cnt;
        if (coincident) atomicOr(err, ERR_COINCIDENT);
    }
}

// reverse-edge index of the filtered list from the candidate list's: the reverse of a kept candidate is kept as well
// (same length bit for bit), so mirror[newpos[e]] = newpos[cmirror[e]]
__global__ void k_skin_mirror(int64_t Ec, const int32_t *__restrict__ newpos, const int32_t *__restrict__ cmirror,
                              int32_t *__restrict__ mirror, int32_t *err)
{
    const int64_t e = (int64_t)xcd_block() * blockDim.x + threadIdx.x;
    if (e >= Ec) return;
    const int32_t o = newpos[e];
    if (o < 0) return;
    const int32_t m = newpos[cmirror[e]];
    if (m < 0) { atomicOr(err, ERR_MIRROR); mirror[o] = o; return; }
    mirror[o] = m;
}

inline unsigned blocks_for(int64_t n, int threads) { return (unsigned)((n + threads - 1) / threads); }

void cross3(const double *a, const double *b, double *o)
{
    o[0] = a[1] * b[2] - a[2] * b[1];
    o[1] = a[2] * b[0] - a[0] * b[2];
    o[2] = a[0] * b[1] - a[1] * b[0];
}

int prepare_cell(const double *C, double r_cut, int32_t n_slabs, int64_t N, CellParams &cp)
{
    for (int k = 0; k < 9; ++k) {
        if (!std::isfinite(C[k])) { set_error("cell has a non-finite entry"); return MLIP_ECELL; }
        cp.C[k] = C[k];
    }
    cross3(C + 3, C + 6, cp.nrm[0]);
    cross3(C + 6, C + 0, cp.nrm[1]);
    cross3(C + 0, C + 3, cp.nrm[2]);
    cp.V = (C[0] * cp.nrm[0][0] + C[1] * cp.nrm[0][1]) + C[2] * cp.nrm[0][2];
    if (!(std::fabs(cp.V) > 0.0) || !std::isfinite(cp.V)) { set_error("singular cell (volume 0)"); return MLIP_ECELL; }
    cp.rc2 = r_cut * r_cut;
    const double rpad = r_cut * 1.000001 + 1e-12;
    double h[3];
    for (int k = 0; k < 3; ++k) {
        const double l = std::sqrt(cp.nrm[k][0] * cp.nrm[k][0] + cp.nrm[k][1] * cp.nrm[k][1] + cp.nrm[k][2] * cp.nrm[k][2]);
        h[k] = std::fabs(cp.V) / l;
        int n = (int)std::floor(h[k] / rpad);
        cp.nb[k] = std::max(1, std::min(n, 1024));
    }
    // keep the number of bins comparable to the number of atoms for sparse systems
    const double max_cells = std::max<double>(4096.0, 8.0 * (double)N);
    while ((double)cp.nb[0] * cp.nb[1] * cp.nb[2] > max_cells) {
        int k = 0;
        for (int m = 1; m < 3; ++m) if (cp.nb[m] > cp.nb[k]) k = m;
        cp.nb[k] = std::max(1, cp.nb[k] / 2);
    }
    for (int k = 0; k < 3; ++k) {
        cp.reach[k] = (int)std::ceil(rpad / (h[k] / cp.nb[k]));
        if (cp.reach[k] > 100) { set_error("cell is thinner than r_cut / 100 along lattice direction %d", k); return MLIP_ECELL; }
    }
    int ax = 0;
    double best = -1.0;
    for (int k = 0; k < 3; ++k) {
        const double l2 = (C[3 * k] * C[3 * k] + C[3 * k + 1] * C[3 * k + 1]) + C[3 * k + 2] * C[3 * k + 2];
        if (l2 > best) { best = l2; ax = k; }
    }
    cp.axis = ax;
    cp.n_slabs = n_slabs;
    return MLIP_OK;
}

// ---------------------------------------------------------------- bond list (three-body variant)

// flag[e] = 1 if the edge is a bond: the neighbour list's own fp64 test with the bond cutoff
__global__ void k_bond_flag(int64_t E, CellParams cp, double rb2, const double *__restrict__ pos,
                            const int32_t *__restrict__ nodes, const int32_t *__restrict__ recv,
                            const int32_t *__restrict__ senders, const uint32_t *__restrict__ shiftp, int32_t *flag)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= E) return;
    const int64_t i = nodes ? nodes[recv[e]] : recv[e], j = nodes ? nodes[senders[e]] : senders[e];
    int S0, S1, S2;
    unpack3(shiftp[e], S0, S1, S2);
    const double t0 = (pos[3 * j] - pos[3 * i]) + (((double)S0 * cp.C[0] + (double)S1 * cp.C[3]) + (double)S2 * cp.C[6]);
    const double t1 = (pos[3 * j + 1] - pos[3 * i + 1]) + (((double)S0 * cp.C[1] + (double)S1 * cp.C[4]) + (double)S2 * cp.C[7]);
    const double t2 = (pos[3 * j + 2] - pos[3 * i + 2]) + (((double)S0 * cp.C[2] + (double)S1 * cp.C[5]) + (double)S2 * cp.C[8]);
    const double d2 = (t0 * t0 + t1 * t1) + t2 * t2;
    flag[e] = (d2 <= rb2) ? 1 : 0;
}

// bond numbering in edge order; unit vector (fp64, rounded once), length, envelope and its derivative
__global__ void k_bond_fill(int64_t E, CellParams cp, double r_bond, int p, const double *__restrict__ pos,
                            const int32_t *__restrict__ nodes, const int32_t *__restrict__ recv,
                            const int32_t *__restrict__ senders,
                            const uint32_t *__restrict__ shiftp, const float *__restrict__ d,
                            const int32_t *__restrict__ flag, const int32_t *__restrict__ scan, int32_t *of_edge,
                            int32_t *edge, int32_t *sender, float *bd, float *bu, float *bdu, float *rhat)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= E) return;
    if (!flag[e]) { of_edge[e] = -1; return; }
    const int32_t b = scan[e];
    of_edge[e] = b;
    edge[b] = (int32_t)e;
    sender[b] = senders[e];
    const int64_t i = nodes ? nodes[recv[e]] : recv[e], j = nodes ? nodes[senders[e]] : senders[e];
    int S0, S1, S2;
    unpack3(shiftp[e], S0, S1, S2);
    const double t0 = (pos[3 * j] - pos[3 * i]) + (((double)S0 * cp.C[0] + (double)S1 * cp.C[3]) + (double)S2 * cp.C[6]);
    const double t1 = (pos[3 * j + 1] - pos[3 * i + 1]) + (((double)S0 * cp.C[1] + (double)S1 * cp.C[4]) + (double)S2 * cp.C[7]);
    const double t2 = (pos[3 * j + 2] - pos[3 * i + 2]) + (((double)S0 * cp.C[2] + (double)S1 * cp.C[5]) + (double)S2 * cp.C[8]);
    const double dd = sqrt((t0 * t0 + t1 * t1) + t2 * t2);
    rhat[3 * b] = (float)(t0 / dd);
    rhat[3 * b + 1] = (float)(t1 / dd);
    rhat[3 * b + 2] = (float)(t2 / dd);
    bd[b] = d[e];
    // u(x) = 1 - c0 x^p + c1 x^(p+1) - c2 x^(p+2), x = d / r_bond
    const double x = dd / r_bond, pd = (double)p;
    const double c0 = (pd + 1) * (pd + 2) / 2, c1 = pd * (pd + 2), c2 = pd * (pd + 1) / 2;
    double xpm1 = 1.0;
    for (int k = 0; k < p - 1; ++k) xpm1 *= x;
    const double xp = xpm1 * x;
    bu[b] = (float)(1.0 - xp * (c0 - x * (c1 - c2 * x)));
    bdu[b] = (float)((-xpm1 * (pd * c0 - x * ((pd + 1) * c1 - (pd + 2) * c2 * x))) / r_bond);
}

__global__ void k_bond_ptr(int64_t N, const int64_t *__restrict__ row_ptr, const int32_t *__restrict__ scan, int64_t *ptr)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i > N) return;
    ptr[i] = scan[row_ptr[i]];
}

// the reverse edge of a bond has the same length, so it is a bond too - of this partition if it lies in an owned
// row (edge index below E), of the sender's partition otherwise (-1)
__global__ void k_bond_mirror(int64_t nb, int64_t E, const int32_t *__restrict__ edge, const int32_t *__restrict__ mirror,
                              const int32_t *__restrict__ of_edge, int32_t *bmirror)
{
    const int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= nb) return;
    const int32_t m = mirror[edge[b]];
    bmirror[b] = (m < E) ? of_edge[m] : -1;
}

}  // namespace

int unpack_shifts(const mlip_graph *g, int32_t *out)
{
    if (g->E > 0) {
        k_unpack_shifts<<<blocks_for(g->E, 256), 256, 0, g->stream>>>(g->E, g->shiftp.as<uint32_t>(), out);
        MLIP_HIP(hipGetLastError());
    }
    return MLIP_OK;
}

int build_bonds_impl(mlip_graph *g, SlabView &v, double r_bond, int p_envelope)
{
    BondGraph &B = v.bonds;
    // same graph (a rebuild resets r_bond), same cutoff, same envelope (u and du/dd are stored with the list)
    if (B.r_bond == r_bond && B.p_env == p_envelope) return MLIP_OK;
    B.r_bond = -1.0;   // the arrays are about to be overwritten: a failure below must not leave a half-built list valid
    hipStream_t s = g->stream;
    const int64_t E = v.n_edges_owned, N = v.n_owned;
    const size_t Ecap = (size_t)std::max<int64_t>(E, 1);
    MLIP_TRY(B.flag.ensure(Ecap * 4));
    MLIP_TRY(B.scan.ensure((Ecap + 1) * 4));
    MLIP_TRY(B.of_edge.ensure(Ecap * 4));
    MLIP_TRY(B.ptr.ensure((size_t)(N + 1) * 8));
    const double *pos = g->pos.as<double>();
    if (E > 0) {
        k_bond_flag<<<blocks_for(E, 256), 256, 0, s>>>(E, g->cell, r_bond * r_bond, pos, v.nodes, v.recv, v.senders,
                                                       v.shiftp, B.flag.as<int32_t>());
        MLIP_HIP(hipGetLastError());
    }
    MLIP_TRY(scan_i32_to_i32(B.flag.as<int32_t>(), B.scan.as<int32_t>(), E, g->scan_tmp, s));
    int32_t *hp = static_cast<int32_t *>(g->pinned);
    MLIP_HIP(hipMemcpyAsync(hp, B.scan.as<int32_t>() + E, 4, hipMemcpyDeviceToHost, s));
    MLIP_HIP(hipStreamSynchronize(s));
    const int64_t nb = hp[0];
    const size_t ncap = (size_t)std::max<int64_t>(nb, 1);
    MLIP_TRY(B.edge.ensure(ncap * 4));
    MLIP_TRY(B.sender.ensure(ncap * 4));
    MLIP_TRY(B.mirror.ensure(ncap * 4));
    MLIP_TRY(B.d.ensure(ncap * 4));
    MLIP_TRY(B.u.ensure(ncap * 4));
    MLIP_TRY(B.du.ensure(ncap * 4));
    MLIP_TRY(B.rhat.ensure(ncap * 12));
    if (E > 0) {
        k_bond_fill<<<blocks_for(E, 256), 256, 0, s>>>(
            E, g->cell, r_bond, p_envelope, pos, v.nodes, v.recv, v.senders, v.shiftp, v.d, B.flag.as<int32_t>(),
            B.scan.as<int32_t>(), B.of_edge.as<int32_t>(), B.edge.as<int32_t>(), B.sender.as<int32_t>(), B.d.as<float>(),
            B.u.as<float>(), B.du.as<float>(), B.rhat.as<float>());
        MLIP_HIP(hipGetLastError());
    }
    k_bond_ptr<<<blocks_for(N + 1, 256), 256, 0, s>>>(N, v.row_ptr, B.scan.as<int32_t>(), B.ptr.as<int64_t>());
    MLIP_HIP(hipGetLastError());
    if (nb > 0) {
        k_bond_mirror<<<blocks_for(nb, 256), 256, 0, s>>>(nb, E, B.edge.as<int32_t>(), v.mirror, B.of_edge.as<int32_t>(),
                                                          B.mirror.as<int32_t>());
        MLIP_HIP(hipGetLastError());
    }
    B.n = nb;
    B.r_bond = r_bond;
    B.p_env = p_envelope;
    return MLIP_OK;
}

namespace {

// ---- upper / lower split of the owned rows' edges (PairGraph), up to kPairBatch partitions per launch

constexpr int kPairBatch = 8;

struct PairArgs {   // one partition
    int64_t n_rows, n_edges_owned, n_chunks;
    const int64_t *row_ptr;
    const int32_t *senders, *recv, *mirror;
    const float *d;
    int64_t *u_row_ptr, *l_row_ptr;
    int32_t *wslot, *u_senders, *u_recv, *u_eid, *u_mirror, *u_chunk_row, *l_senders, *l_slot;
    float *u_d;
};
struct PairBatch {   // rows, edges and work items numbered across the partitions
    int n;
    int64_t row_start[kPairBatch + 1], edge_start[kPairBatch + 1], chunk_start[kPairBatch + 1];
    PairArgs s[kPairBatch];
};
__device__ inline int pair_find(const int64_t *start, int n, int64_t w)
{
    int p = 0;
#pragma unroll
    for (int q = 1; q < kPairBatch; ++q)
        if (q < n && w >= start[q]) p = q;
    return p;
}

// flag[e] = 1 for the upper edge of a pair (reverse edge at a larger index), over all partitions' owned-row edges
__global__ void k_pair_flag(PairBatch B, int32_t *__restrict__ flag)
{
    const int64_t ge = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (ge >= B.edge_start[B.n]) return;
    const int part = pair_find(B.edge_start, B.n, ge);
    const int64_t e = ge - B.edge_start[part];
    flag[ge] = (int64_t)B.s[part].mirror[e] > e ? 1 : 0;
}

// The upper edges keep their order, so an upper edge's position among them is the exclusive scan of the flags (less
// the scan at its partition's first edge), and a lower edge's position among the lower ones is its index less that
// scan: the two compacted lists.  A lower edge notes where its pair's filter values are kept: at the upper edge's
// position in the upper-edge graph or (slots_full) in the full list.
__global__ void k_pair_fill(PairBatch B, const int32_t *__restrict__ scan, int slots_full)
{
    const int64_t ge = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (ge >= B.edge_start[B.n]) return;
    const int part = pair_find(B.edge_start, B.n, ge);
    const PairArgs &A = B.s[part];
    const int64_t e0 = B.edge_start[part], e = ge - e0;
    const int32_t base = scan[e0];
    const int32_t m = A.mirror[e];
    if ((int64_t)m > e) {
        const int32_t k = scan[ge] - base;
        A.u_senders[k] = A.senders[e];
        A.u_recv[k] = A.recv[e];
        A.u_eid[k] = (int32_t)e;
        A.u_mirror[k] = m;
        A.u_d[k] = A.d[e];
        A.wslot[e] = k;
    } else {
        const int64_t kl = e - (int64_t)(scan[ge] - base);
        A.l_senders[kl] = A.senders[e];
        A.l_slot[kl] = slots_full ? m : scan[e0 + m] - base;   // (letting the upper edge store this instead was measured slower)
    }
}

// row pointers of the upper-edge graphs (the scan at the rows' first edges) and of the lower edges' lists (the rest)
__global__ void k_pair_rowptr(PairBatch B, const int32_t *__restrict__ scan)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // row, plus one closing entry per partition
    if (i >= B.row_start[B.n] + B.n) return;
    int part = 0;
    for (int q = 1; q < B.n; ++q)
        if (i >= B.row_start[q] + q) part = q;
    const PairArgs &A = B.s[part];
    const int64_t r = i - (B.row_start[part] + part);   // 0 .. n_rows
    const int64_t e0 = B.edge_start[part];
    const int64_t u = (int64_t)(scan[e0 + A.row_ptr[r]] - scan[e0]);
    A.u_row_ptr[r] = u;
    A.l_row_ptr[r] = A.row_ptr[r] - u;
}

// u_chunk_row[c] = first row whose first upper edge lies at or after c * kChunkEdges; u_chunk_row[n_chunks] = n_rows.
__global__ void k_pair_chunks(PairBatch B)
{
    const int64_t gc = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // work item, plus one closing entry per partition
    if (gc >= B.chunk_start[B.n] + B.n) return;
    int part = 0;
    for (int q = 1; q < B.n; ++q)
        if (gc >= B.chunk_start[q] + q) part = q;
    const PairArgs &A = B.s[part];
    const int64_t c = gc - (B.chunk_start[part] + part);   // 0 .. n_chunks
    int64_t lo = 0, hi = A.n_rows;
    if (c == A.n_chunks) lo = A.n_rows;
    const int64_t v = c * kChunkEdges;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (A.u_row_ptr[mid] < v) lo = mid + 1; else hi = mid;
    }
    A.u_chunk_row[c] = (int32_t)lo;
}

}  // namespace

int build_pairs_impl(mlip_graph *g, SlabView *views, int P, bool slots_full, Carver *scratch)
{
    bool all_valid = true;
    for (int p = 0; p < P; ++p) all_valid = all_valid && views[p].pairs.valid && views[p].pairs.slots_full == slots_full;
    if (all_valid) return MLIP_OK;
    hipStream_t s = g->stream;
    auto place = [&](DevBuf &buf, size_t bytes, auto *&ptr) -> int {
        using T = std::remove_reference_t<decltype(*ptr)>;
        if (scratch) {
            ptr = static_cast<T *>(scratch->take(bytes));
            return MLIP_OK;   // a failed carve is reported by the caller
        }
        MLIP_TRY(buf.ensure(bytes));
        ptr = buf.as<T>();
        return MLIP_OK;
    };
    for (int p = 0; p < P; ++p) {
        SlabView &v = views[p];
        PairGraph &Q = v.pairs;
        Q.valid = false;
        const int64_t E = v.n_edges_owned, N = v.n_owned;
        // every pair of two owned-row edges has one upper edge; an owned-row edge from a ghost sender is an upper edge,
        // and the ghost rows hold exactly the reverse edges of those
        const int64_t n_ghost_edges = v.n_edges - v.n_edges_owned;
        Q.n_upper = (E - n_ghost_edges) / 2 + n_ghost_edges;
        Q.n_lower = E - Q.n_upper;
        const size_t Ncap = (size_t)std::max<int64_t>(N, 1), Ecap = (size_t)std::max<int64_t>(E, 1);
        const size_t Ucap = (size_t)std::max<int64_t>(Q.n_upper, 1);
        MLIP_TRY(place(Q.b_u_row_ptr, (Ncap + 1) * 8, Q.u_row_ptr));
        MLIP_TRY(place(Q.b_wslot, Ecap * 4, Q.wslot));
        MLIP_TRY(place(Q.b_u_senders, Ucap * 4, Q.u_senders));
        MLIP_TRY(place(Q.b_u_recv, Ucap * 4, Q.u_recv));
        MLIP_TRY(place(Q.b_u_eid, Ucap * 4, Q.u_eid));
        MLIP_TRY(place(Q.b_u_mirror, Ucap * 4, Q.u_mirror));
        MLIP_TRY(place(Q.b_u_d, Ucap * 4, Q.u_d));
        MLIP_TRY(place(Q.b_u_chunk_row, (size_t)(chunks_of(Q.n_upper) + 1) * 4, Q.u_chunk_row));
        const size_t Lcap = (size_t)std::max<int64_t>(Q.n_lower, 1);
        MLIP_TRY(place(Q.b_l_row_ptr, (Ncap + 1) * 8, Q.l_row_ptr));
        MLIP_TRY(place(Q.b_l_senders, Lcap * 4, Q.l_senders));
        MLIP_TRY(place(Q.b_l_slot, Lcap * 4, Q.l_slot));
    }
    // flags and their scan, kPairBatch partitions at a time (their edges one after another)
    for (int p0 = 0; p0 < P; p0 += kPairBatch) {
        PairBatch b{};
        b.n = std::min(kPairBatch, P - p0);
        b.row_start[0] = b.edge_start[0] = b.chunk_start[0] = 0;
        for (int q = 0; q < kPairBatch; ++q) {
            if (q >= b.n) {
                b.row_start[q + 1] = b.row_start[q];
                b.edge_start[q + 1] = b.edge_start[q];
                b.chunk_start[q + 1] = b.chunk_start[q];
                continue;
            }
            SlabView &v = views[p0 + q];
            PairGraph &Q = v.pairs;
            PairArgs &a = b.s[q];
            a.n_rows = v.n_owned;
            a.n_edges_owned = v.n_edges_owned;
            a.n_chunks = chunks_of(Q.n_upper);
            a.row_ptr = v.row_ptr;
            a.senders = v.senders;
            a.recv = v.recv;
            a.mirror = v.mirror;
            a.d = v.d;
            a.u_row_ptr = Q.u_row_ptr;
            a.wslot = Q.wslot;
            a.u_senders = Q.u_senders;
            a.u_recv = Q.u_recv;
            a.u_eid = Q.u_eid;
            a.u_mirror = Q.u_mirror;
            a.u_chunk_row = Q.u_chunk_row;
            a.u_d = Q.u_d;
            a.l_row_ptr = Q.l_row_ptr;
            a.l_senders = Q.l_senders;
            a.l_slot = Q.l_slot;
            b.row_start[q + 1] = b.row_start[q] + v.n_owned;
            b.edge_start[q + 1] = b.edge_start[q] + v.n_edges_owned;
            b.chunk_start[q + 1] = b.chunk_start[q] + a.n_chunks;
        }
        const int64_t edges = b.edge_start[b.n], rows = b.row_start[b.n];
        if (edges >= ((int64_t)1 << 31)) {
            set_error("more than 2^31 edges in %d partitions", b.n);
            return MLIP_EINVAL;
        }
        int32_t *flag = nullptr, *scan = nullptr;
        MLIP_TRY(place(g->pair_cnt, (size_t)(edges + 1) * 4, flag));
        MLIP_TRY(place(g->pair_scan, (size_t)(edges + 1) * 4, scan));
        if (scratch && scratch->failed()) return MLIP_OK;   // nothing may be launched on a failed carve; the caller reports it
        if (edges > 0) {
            k_pair_flag<<<blocks_for(edges, 256), 256, 0, s>>>(b, flag);
            MLIP_HIP(hipGetLastError());
        }
        MLIP_TRY(scan_i32_to_i32(flag, scan, edges, g->scan_tmp, s));
        if (edges > 0) {
            k_pair_fill<<<blocks_for(edges, 256), 256, 0, s>>>(b, scan, slots_full ? 1 : 0);
            MLIP_HIP(hipGetLastError());
        }
        k_pair_rowptr<<<blocks_for(rows + b.n, 256), 256, 0, s>>>(b, scan);
        MLIP_HIP(hipGetLastError());
        k_pair_chunks<<<blocks_for(b.chunk_start[b.n] + b.n, 256), 256, 0, s>>>(b);
        MLIP_HIP(hipGetLastError());
    }
    for (int p = 0; p < P; ++p) {
        views[p].pairs.valid = (scratch == nullptr);   // arrays in a borrowed block do not outlive the call
        views[p].pairs.slots_full = slots_full;
    }
    return MLIP_OK;
}

namespace {

struct CsrOut {   // where a neighbour search puts its receiver-sorted CSR (mirror: the reverse-edge index, or nullptr)
    DevBuf *row_ptr, *senders, *recv, *shiftp, *d, *mirror;
};

// reads the edge count and the flag words after the first pass of either route and turns the flags into errors
int read_counts_and_flags(mlip_graph *g, const int64_t *row_ptr_end, int32_t *err, int64_t *E, int32_t *flags_out)
{
    hipStream_t s = g->stream;
    int64_t *hp = static_cast<int64_t *>(g->pinned);
    MLIP_HIP(hipMemcpyAsync(hp, row_ptr_end, 8, hipMemcpyDeviceToHost, s));
    MLIP_HIP(hipMemcpyAsync(hp + 1, err, 12, hipMemcpyDeviceToHost, s));
    MLIP_HIP(hipStreamSynchronize(s));
    *E = hp[0];
    const int32_t *herr = reinterpret_cast<int32_t *>(hp + 1);
    const int32_t flags = herr[0];
    *flags_out = flags;
    g->species_max = herr[1];
    g->species_min = herr[2];
    if (flags & ERR_RANGE) {
        set_error("an atom lies more than 200 cells away from the origin cell (or has a non-finite coordinate)");
        return MLIP_ECELL;
    }
    if (flags & ERR_COINCIDENT) {
        set_error("two atoms (or an atom and one of its images) coincide");
        return MLIP_ECOINCIDENT;
    }
    if (*E >= ((int64_t)1 << 31)) {
        set_error("more than 2^31 directed edges");
        return MLIP_EINVAL;
    }
    return MLIP_OK;
}

// Cell-list neighbour search for the cutoff in cp.rc2 over the positions and species held by the handle; writes the
// canonical receiver-sorted CSR to `out`, slab_of and the species range; synchronises the stream once.
int search_csr(mlip_graph *g, const CellParams &cp, int64_t N, CsrOut out, int64_t *E_out)
{
    hipStream_t s = g->stream;
    const int64_t ncell = (int64_t)cp.nb[0] * cp.nb[1] * cp.nb[2];
    MLIP_TRY(g->cell_of.ensure((size_t)N * 4));
    MLIP_TRY(g->wrapp.ensure((size_t)N * 4));
    MLIP_TRY(g->cell_cnt.ensure((size_t)(ncell + 1) * 4));
    MLIP_TRY(g->cell_fill.ensure((size_t)(ncell + 1) * 4));
    MLIP_TRY(g->cell_start.ensure((size_t)(ncell + 2) * 4));
    MLIP_TRY(g->sid.ensure((size_t)N * 4));
    MLIP_TRY(g->swrap.ensure((size_t)N * 4));
    MLIP_TRY(g->sx.ensure((size_t)N * 8));
    MLIP_TRY(g->sy.ensure((size_t)N * 8));
    MLIP_TRY(g->sz.ensure((size_t)N * 8));
    MLIP_TRY(out.row_ptr->ensure((size_t)(N + 1) * 8));
    int32_t *err = g->small.as<int32_t>();
    MLIP_HIP(hipMemsetAsync(g->small.p, 0, 4096, s));
    MLIP_HIP(hipMemsetAsync(g->cell_cnt.p, 0, (size_t)(ncell + 1) * 4, s));
    MLIP_HIP(hipMemsetAsync(g->cell_fill.p, 0, (size_t)(ncell + 1) * 4, s));
    const double *pos = g->pos.as<double>();
    k_bin<<<blocks_for(N, 256), 256, 0, s>>>(N, pos, g->species.as<int32_t>(), cp, g->cell_of.as<int32_t>(),
                                             g->wrapp.as<uint32_t>(), g->slab_of.as<int32_t>(),
                                             g->cell_cnt.as<int32_t>(), err);
    MLIP_HIP(hipGetLastError());
    MLIP_TRY(scan_i32_to_i32(g->cell_cnt.as<int32_t>(), g->cell_start.as<int32_t>(), ncell, g->scan_tmp, s));
    k_fill_cells<<<blocks_for(N, 256), 256, 0, s>>>(N, pos, g->cell_of.as<int32_t>(), g->wrapp.as<uint32_t>(),
                                                    g->cell_start.as<int32_t>(), g->cell_fill.as<int32_t>(),
                                                    g->sid.as<int32_t>(), g->sx.as<double>(), g->sy.as<double>(),
                                                    g->sz.as<double>(), g->swrap.as<uint32_t>());
    MLIP_HIP(hipGetLastError());
    int64_t E = 0;
    int32_t flags = 0;
    // Pair-wise search (every pair tested once, reverse-edge index without a search) unless its staging rows
    // (1.25 KB per atom) would take more than 8 GB; an atom with more neighbours than the staging rows hold
    // (kOwn found by itself, kPar by its partners) sets FLAG_STAGE_OVERFLOW and the one-sided search below runs instead
    bool done = false;
    if ((size_t)N * (kOwn + kPar) * 10 <= ((size_t)8 << 30)) {
        MLIP_TRY(g->stage.ensure((size_t)N * (kOwn + kPar) * 8));
        MLIP_TRY(g->pair_aux.ensure((size_t)N * (8 + 2 * (kOwn + kPar))));
        uint64_t *stage_own = g->stage.as<uint64_t>(), *stage_par = stage_own + (size_t)N * kOwn;
        int32_t *n_own = g->pair_aux.as<int32_t>(), *n_par = n_own + N;
        uint8_t *pslot_own = reinterpret_cast<uint8_t *>(n_par + N), *pslot_par = pslot_own + (size_t)N * kOwn;
        uint8_t *rank_own = pslot_par + (size_t)N * kPar, *rank_par = rank_own + (size_t)N * kOwn;
        MLIP_HIP(hipMemsetAsync(n_par, 0, (size_t)N * 4, s));
        k_neighbours_pairs<<<grid8(blocks_for(N, 128)), 128, 0, s>>>(
            N, cp, g->cell_start.as<int32_t>(), g->sid.as<int32_t>(), g->sx.as<double>(), g->sy.as<double>(),
            g->sz.as<double>(), g->swrap.as<uint32_t>(), g->cell_of.as<int32_t>(), stage_own, stage_par, pslot_own,
            pslot_par, n_own, n_par, err);
        MLIP_HIP(hipGetLastError());
        k_pair_partners<<<blocks_for(N * kOwn, 256), 256, 0, s>>>(N, n_own, stage_own, stage_par, pslot_own, pslot_par, n_par, err);
        MLIP_HIP(hipGetLastError());
        k_pair_counts<<<blocks_for(N, 256), 256, 0, s>>>(N, n_own, n_par, g->counts.as<int32_t>());
        MLIP_HIP(hipGetLastError());
        MLIP_TRY(scan_i32_to_i64(g->counts.as<int32_t>(), out.row_ptr->as<int64_t>(), N, g->scan_tmp, s));
        const int rc = read_counts_and_flags(g, out.row_ptr->as<int64_t>() + N, err, &E, &flags);   // first synchronisation
        if (!(flags & FLAG_STAGE_OVERFLOW)) {
            MLIP_TRY(rc);
            const size_t Ecap = (size_t)std::max<int64_t>(E, 1);
            MLIP_TRY(out.senders->ensure(Ecap * 4));
            MLIP_TRY(out.shiftp->ensure(Ecap * 4));
            MLIP_TRY(out.recv->ensure(Ecap * 4));
            MLIP_TRY(out.d->ensure(Ecap * 4));
            k_sort_rows_pairs<<<grid8(N), 64, 0, s>>>(N, cp, pos, out.row_ptr->as<int64_t>(), stage_own, stage_par, n_own,
                                                      rank_own, rank_par, out.senders->as<int32_t>(),
                                                      out.recv->as<int32_t>(), out.shiftp->as<uint32_t>(),
                                                      out.d->as<float>());
            MLIP_HIP(hipGetLastError());
            if (out.mirror) {
                MLIP_TRY(out.mirror->ensure(Ecap * 4));
                k_mirror_pairs<<<grid8((N + 7) / 8), 256, 0, s>>>(N, out.row_ptr->as<int64_t>(), stage_own, pslot_own, n_own,
                                                                  rank_own, rank_par, out.mirror->as<int32_t>());
                MLIP_HIP(hipGetLastError());
            }
            done = true;
        }
        // (on overflow the flag words stay as they are: species and position range remain valid, a coincidence is found again)
    }
    if (!done) {   // one-sided search in two passes (count, fill), reverse-edge index by binary search
        k_neighbours<false><<<grid8(blocks_for(N, 128)), 128, 0, s>>>(
            N, cp, g->cell_start.as<int32_t>(), g->sid.as<int32_t>(), g->sx.as<double>(), g->sy.as<double>(),
            g->sz.as<double>(), g->swrap.as<uint32_t>(), g->cell_of.as<int32_t>(), g->counts.as<int32_t>(), nullptr,
            nullptr, err);
        MLIP_HIP(hipGetLastError());
        MLIP_TRY(scan_i32_to_i64(g->counts.as<int32_t>(), out.row_ptr->as<int64_t>(), N, g->scan_tmp, s));
        MLIP_TRY(read_counts_and_flags(g, out.row_ptr->as<int64_t>() + N, err, &E, &flags));
        const size_t Ecap = (size_t)std::max<int64_t>(E, 1);
        MLIP_TRY(g->keys.ensure(Ecap * 8));
        MLIP_TRY(out.senders->ensure(Ecap * 4));
        MLIP_TRY(out.shiftp->ensure(Ecap * 4));
        MLIP_TRY(out.recv->ensure(Ecap * 4));
        MLIP_TRY(out.d->ensure(Ecap * 4));
        k_neighbours<true><<<grid8(blocks_for(N, 128)), 128, 0, s>>>(
            N, cp, g->cell_start.as<int32_t>(), g->sid.as<int32_t>(), g->sx.as<double>(), g->sy.as<double>(),
            g->sz.as<double>(), g->swrap.as<uint32_t>(), g->cell_of.as<int32_t>(), nullptr, out.row_ptr->as<int64_t>(),
            g->keys.as<uint64_t>(), err);
        MLIP_HIP(hipGetLastError());
        k_sort_rows<<<grid8(N), 64, 0, s>>>(N, cp, pos, out.row_ptr->as<int64_t>(), g->keys.as<uint64_t>(), 0,
                                            out.senders->as<int32_t>(), out.recv->as<int32_t>(), out.shiftp->as<uint32_t>(),
                                            out.d->as<float>());
        MLIP_HIP(hipGetLastError());
        if (out.mirror && E > 0) {
            MLIP_TRY(out.mirror->ensure(Ecap * 4));
            k_mirror<true><<<grid8(blocks_for(E, 256)), 256, 0, s>>>(E, out.row_ptr->as<int64_t>(), out.senders->as<int32_t>(),
                                                                     out.recv->as<int32_t>(), out.shiftp->as<uint32_t>(), nullptr,
                                                                     0, out.mirror->as<int32_t>(), err);
            MLIP_HIP(hipGetLastError());
        }
    }
    *E_out = E;
    return MLIP_OK;
}

// The exact neighbour list from the handle's candidate list; *valid = false (and nothing usable written) when some
// atom has moved more than skin / 2 since the candidates were built.  Synchronises the stream once.
int csr_from_candidates(mlip_graph *g, const CellParams &cp, int64_t N, int64_t *E_out, bool *valid)
{
    hipStream_t s = g->stream;
    int32_t *err = g->small.as<int32_t>();
    MLIP_HIP(hipMemsetAsync(g->small.p, 0, 4096, s));
    MLIP_TRY(g->row_ptr.ensure((size_t)(N + 1) * 8));
    const double h2 = 0.25 * g->skin * g->skin;
    const double *pos = g->pos.as<double>();
    k_skin_rows<false><<<grid8((N + 3) / 4), 256, 0, s>>>(
        N, cp, pos, g->ref_pos.as<double>(), h2, g->species.as<int32_t>(), g->cand_row_ptr.as<int64_t>(),
        g->cand_senders.as<int32_t>(), g->cand_shiftp.as<uint32_t>(), g->counts.as<int32_t>(), g->slab_of.as<int32_t>(),
        nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, err);
    MLIP_HIP(hipGetLastError());
    MLIP_TRY(scan_i32_to_i64(g->counts.as<int32_t>(), g->row_ptr.as<int64_t>(), N, g->scan_tmp, s));
    int64_t E = 0;
    int32_t flags = 0;
    const int rc = read_counts_and_flags(g, g->row_ptr.as<int64_t>() + N, err, &E, &flags);
    if (flags & FLAG_DISPLACED) { *valid = false; return MLIP_OK; }   // (errors seen on the way are found again by the full search)
    MLIP_TRY(rc);
    const size_t Ecap = (size_t)std::max<int64_t>(E, 1);
    MLIP_TRY(g->senders.ensure(Ecap * 4));
    MLIP_TRY(g->shiftp.ensure(Ecap * 4));
    MLIP_TRY(g->recv.ensure(Ecap * 4));
    MLIP_TRY(g->d.ensure(Ecap * 4));
    MLIP_TRY(g->mirror.ensure(Ecap * 4));
    // the candidate list's reverse-edge index is reused through the positions the kept candidates go to (the recv
    // array of the candidate list is not needed after its build and holds them)
    int32_t *newpos = g->cand_recv.as<int32_t>();
    k_skin_rows<true><<<grid8((N + 3) / 4), 256, 0, s>>>(
        N, cp, pos, g->ref_pos.as<double>(), h2, g->species.as<int32_t>(), g->cand_row_ptr.as<int64_t>(),
        g->cand_senders.as<int32_t>(), g->cand_shiftp.as<uint32_t>(), nullptr, nullptr, g->row_ptr.as<int64_t>(),
        g->senders.as<int32_t>(), g->recv.as<int32_t>(), g->shiftp.as<uint32_t>(), g->d.as<float>(), newpos, err);
    MLIP_HIP(hipGetLastError());
    if (g->cand_E > 0) {
        k_skin_mirror<<<grid8(blocks_for(g->cand_E, 256)), 256, 0, s>>>(g->cand_E, newpos, g->cand_mirror.as<int32_t>(),
                                                                        g->mirror.as<int32_t>(), err);
        MLIP_HIP(hipGetLastError());
    }
    *E_out = E;
    *valid = true;
    return MLIP_OK;
}

}  // namespace

int build_graph_impl(mlip_graph *g, const double *positions, const double *cell, const int32_t *species,
                     int64_t N, double r_cut, int32_t P)
{
    hipStream_t s = g->stream;
    CellParams cp;
    MLIP_TRY(prepare_cell(cell, r_cut, P, N, cp));
    g->cell = cp;
    g->N = 0;  // the handle is invalid until the build completes
    g->whole.bonds.r_bond = -1.0;
    g->whole.pairs.valid = false;
    for (SlabView &sv : g->slabs) {
        sv.bonds.r_bond = -1.0;
        sv.pairs.valid = false;
    }
    g->E = 0;
    if (!g->pinned) MLIP_HIP(hipHostMalloc(&g->pinned, 65536, hipHostMallocDefault));
    int64_t *hp = static_cast<int64_t *>(g->pinned);

    MLIP_TRY(g->pos.ensure((size_t)N * 3 * sizeof(double)));
    MLIP_TRY(g->species.ensure((size_t)N * sizeof(int32_t)));
    MLIP_HIP(hipMemcpyAsync(g->pos.p, positions, (size_t)N * 3 * sizeof(double), hipMemcpyDeviceToDevice, s));
    MLIP_HIP(hipMemcpyAsync(g->species.p, species, (size_t)N * sizeof(int32_t), hipMemcpyDeviceToDevice, s));
    MLIP_TRY(g->slab_of.ensure((size_t)N * 4));
    MLIP_TRY(g->counts.ensure((size_t)(N + 1) * 4));
    MLIP_TRY(g->small.ensure(4096));
    int32_t *err = g->small.as<int32_t>();

    prof_begin(g, MLIP_PROF_GRAPH);
    int64_t E = 0;
    if (g->skin > 0.0) {
        // Verlet skin: the neighbour list is filtered from a candidate list for r_cut + skin, which is rebuilt
        // when the system changed or some atom has moved more than skin / 2 since it was made
        bool valid = false;
        const bool usable = g->cand_valid && g->cand_N == N && g->cand_rcut == r_cut && g->cand_skin == g->skin &&
                            std::memcmp(g->cand_cell, cell, sizeof(g->cand_cell)) == 0;
        int rc = MLIP_OK;
        if (usable) rc = csr_from_candidates(g, cp, N, &E, &valid);
        if (rc == MLIP_OK && !valid) {
            g->cand_valid = false;
            CellParams cps;
            rc = prepare_cell(cell, r_cut + g->skin, P, N, cps);
            if (rc == MLIP_OK)
                rc = search_csr(g, cps, N, CsrOut{&g->cand_row_ptr, &g->cand_senders, &g->cand_recv, &g->cand_shiftp, &g->cand_d, &g->cand_mirror},
                                &g->cand_E);
            if (rc == MLIP_OK) rc = g->ref_pos.ensure((size_t)N * 3 * sizeof(double));
            if (rc == MLIP_OK) {
                MLIP_HIP(hipMemcpyAsync(g->ref_pos.p, g->pos.p, (size_t)N * 3 * sizeof(double), hipMemcpyDeviceToDevice, s));
                g->cand_N = N;
                g->cand_rcut = r_cut;
                g->cand_skin = g->skin;
                std::memcpy(g->cand_cell, cell, sizeof(g->cand_cell));
                g->cand_valid = true;
                g->skin_builds += 1;
                rc = csr_from_candidates(g, cp, N, &E, &valid);
                if (rc == MLIP_OK && !valid) { set_error("internal error: a fresh candidate list is not valid"); rc = MLIP_EHIP; }
            }
        } else if (rc == MLIP_OK) {
            g->skin_reuses += 1;
        }
        if (rc != MLIP_OK) { prof_end(g); return rc; }
    } else {
        const int rc = search_csr(g, cp, N, CsrOut{&g->row_ptr, &g->senders, &g->recv, &g->shiftp, &g->d, &g->mirror}, &E);
        if (rc != MLIP_OK) { prof_end(g); return rc; }
    }
    const double *pos = g->pos.as<double>();
    (void)pos;
    MLIP_TRY(g->mirror.ensure((size_t)std::max<int64_t>(E, 1) * 4));

    {
        const int64_t nc = chunks_of(E);
        MLIP_TRY(g->chunk_row.ensure((size_t)(nc + 1) * 4));
        k_chunk_rows<<<blocks_for(nc + 1, 256), 256, 0, s>>>(N, nc, g->row_ptr.as<int64_t>(), g->chunk_row.as<int32_t>());
        MLIP_HIP(hipGetLastError());
    }

    SlabView &W = g->whole;
    W.n_owned = W.n_pure = W.n_local = N;
    W.n_border = W.n_ghost = 0;
    W.n_edges = W.n_edges_owned = E;
    W.nodes = nullptr;
    W.row_ptr = g->row_ptr.as<int64_t>();
    W.senders = g->senders.as<int32_t>();
    W.shiftp = g->shiftp.as<uint32_t>();
    W.recv = g->recv.as<int32_t>();
    W.mirror = g->mirror.as<int32_t>();
    W.d = g->d.as<float>();
    W.chunk_row = g->chunk_row.as<int32_t>();
    W.markers = {0, N, N, N};

    // ------------------------------------------------------------ partition: all slabs in one pass
    if (P > 1) {
        if (g->slabs.size() < (size_t)P) g->slabs.resize(P);  // never shrunk: views own workspace
        PartStore &st = g->part;
        MLIP_TRY(g->needed_by.ensure((size_t)N * 8));
        MLIP_TRY(g->local_in_owner.ensure((size_t)N * sizeof(OwnRec)));   // one record per atom
        MLIP_TRY(st.gbase.ensure((size_t)(N + 1) * 4));
        MLIP_HIP(hipMemsetAsync(g->needed_by.p, 0, (size_t)N * 8, s));
        k_needed_by<<<grid8((N + 15) / 16), 256, 0, s>>>(N, g->row_ptr.as<int64_t>(), g->senders.as<int32_t>(),
                                               g->slab_of.as<int32_t>(), g->needed_by.as<unsigned long long>());
        MLIP_HIP(hipGetLastError());
        // ghost entries per atom and their scan: where the (partition -> local index) entries of an atom start
        k_popcount<<<blocks_for(N, 256), 256, 0, s>>>(N, g->needed_by.as<unsigned long long>(), g->counts.as<int32_t>());
        MLIP_HIP(hipGetLastError());
        MLIP_TRY(scan_i32_to_i32(g->counts.as<int32_t>(), st.gbase.as<int32_t>(), N, g->scan_tmp, s));
        // class counts of every (partition, span) bin per range of kRange atoms, one flat scan
        const int B1 = P * (P + 2), nbins = B1 + P;
        const int64_t nranges = (N + kRange - 1) / kRange;
        const int64_t nent = (int64_t)nbins * nranges;
        if (nent >= ((int64_t)1 << 31)) { prof_end(g); set_error("too many atoms for this many slabs"); return MLIP_EINVAL; }
        MLIP_TRY(g->class_cnt.ensure((size_t)nent * 4));
        MLIP_TRY(g->class_off.ensure((size_t)(nent + 1) * 4));
        MLIP_HIP(hipMemsetAsync(g->class_cnt.p, 0, (size_t)nent * 4, s));
        const int cwaves = ((size_t)nbins * 4 * 4 > 60000) ? 2 : 4;   // wavefronts per block: each keeps a table of nbins counters in LDS
        const size_t clds = (size_t)cwaves * nbins * 4;
        const unsigned cblocks = (unsigned)((nranges + cwaves - 1) / cwaves);
        k_classes<false><<<cblocks, cwaves * 64, clds, s>>>(N, P, nranges, g->slab_of.as<int32_t>(),
                                                            g->needed_by.as<unsigned long long>(), g->class_cnt.as<int32_t>(),
                                                            nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
        MLIP_HIP(hipGetLastError());
        MLIP_TRY(scan_i32_to_i32(g->class_cnt.as<int32_t>(), g->class_off.as<int32_t>(), nent, g->scan_tmp, s));
        const int nmark = P * (P + 3) + 1;
        MLIP_TRY(st.sizes.ensure((size_t)(nmark + 2 * P + 8) * 8));
        k_gather_markers<<<blocks_for(nmark, 256), 256, 0, s>>>(g->class_off.as<int32_t>(), P, nranges, st.gbase.as<int32_t>(), N,
                                                                st.sizes.as<int64_t>());
        MLIP_HIP(hipGetLastError());
        MLIP_HIP(hipMemcpyAsync(hp, st.sizes.p, (size_t)nmark * 8, hipMemcpyDeviceToHost, s));
        MLIP_HIP(hipStreamSynchronize(s));   // second synchronisation: the span starts of all partitions
        PartTab T{};
        T.P = P;
        int64_t n_ghost_total = 0, chunk_total = 0;
        for (int q = 0; q < P; ++q) {
            SlabView &v = g->slabs[q];
            const int64_t *mk = hp + (size_t)q * (P + 3);
            v.markers.resize(P + 3);
            for (int k = 0; k < P + 3; ++k) v.markers[k] = mk[k] - mk[0];
            v.n_pure = v.markers[1];
            v.n_owned = v.markers[2];
            v.n_border = v.n_owned - v.n_pure;
            v.n_local = v.markers[P + 2];
            v.n_ghost = v.n_local - v.n_owned;
            T.row0[q] = mk[0];
            T.n_owned[q] = v.n_owned;
            T.ghost0[q] = n_ghost_total;
            n_ghost_total += v.n_ghost;
        }
        const int64_t TL = hp[(size_t)(P - 1) * (P + 3) + P + 2];   // all partitions' nodes
        T.row0[P] = TL;
        T.ghost0[P] = n_ghost_total;
        if (n_ghost_total != hp[nmark - 1] || TL != N + n_ghost_total) {
            prof_end(g);
            set_error("internal error: inconsistent partition sizes");
            return MLIP_EHIP;
        }
        if (TL + N >= ((int64_t)1 << 31)) { prof_end(g); set_error("more than 2^31 local nodes over all slabs"); return MLIP_EINVAL; }
        const size_t ng1 = (size_t)std::max<int64_t>(n_ghost_total, 1);
        MLIP_TRY(st.nodes.ensure((size_t)TL * 4));
        MLIP_TRY(st.owned_sorted.ensure((size_t)N * 4));
        MLIP_TRY(st.ghost_local.ensure(ng1 * 4));
        MLIP_TRY(st.ghost_owner.ensure(ng1 * 4));
        MLIP_TRY(st.ghost_src.ensure(ng1 * 4));
        MLIP_TRY(st.rowlen.ensure((size_t)(TL + P + 1) * 4));
        MLIP_TRY(st.row_abs.ensure((size_t)(TL + P + 1) * 8));
        MLIP_TRY(st.row_ptr.ensure((size_t)(TL + P + 1) * 8));
        k_classes<true><<<cblocks, cwaves * 64, clds, s>>>(N, P, nranges, g->slab_of.as<int32_t>(),
                                                           g->needed_by.as<unsigned long long>(), nullptr,
                                                           g->class_off.as<int32_t>(), st.gbase.as<int32_t>(),
                                                           st.nodes.as<int32_t>(), st.owned_sorted.as<int32_t>(),
                                                           g->local_in_owner.as<OwnRec>(), st.ghost_local.as<int32_t>());
        MLIP_HIP(hipGetLastError());
        MLIP_HIP(hipMemsetAsync(st.rowlen.p, 0, (size_t)(TL + P + 1) * 4, s));
        k_owned_rowlen<<<blocks_for(N, 256), 256, 0, s>>>(N, T, g->local_in_owner.as<OwnRec>(), g->row_ptr.as<int64_t>(),
                                                         st.rowlen.as<int32_t>());
        if (n_ghost_total > 0)
            k_ghost_rowlen<<<grid8((n_ghost_total + 3) / 4), 256, 0, s>>>(
                T, st.nodes.as<int32_t>(), g->row_ptr.as<int64_t>(), g->senders.as<int32_t>(), g->slab_of.as<int32_t>(),
                g->local_in_owner.as<OwnRec>(), st.rowlen.as<int32_t>(), st.ghost_owner.as<int32_t>(),
                st.ghost_src.as<int32_t>());
        MLIP_HIP(hipGetLastError());
        MLIP_TRY(scan_i32_to_i64(st.rowlen.as<int32_t>(), st.row_abs.as<int64_t>(), TL + P, g->scan_tmp, s));
        int64_t *dsz = st.sizes.as<int64_t>() + nmark;
        k_local_rowptr<<<blocks_for(TL + P, 256), 256, 0, s>>>(T, st.row_abs.as<int64_t>(), st.nodes.as<int32_t>(),
                                                               g->row_ptr.as<int64_t>(), st.row_ptr.as<int64_t>(),
                                                               g->local_in_owner.as<OwnRec>(), dsz);
        MLIP_HIP(hipGetLastError());
        MLIP_HIP(hipMemcpyAsync(hp, dsz, (size_t)2 * P * 8, hipMemcpyDeviceToHost, s));
        MLIP_HIP(hipMemcpyAsync(hp + 2 * P, err, 4, hipMemcpyDeviceToHost, s));
        MLIP_HIP(hipStreamSynchronize(s));   // third and last synchronisation: the partitions' edge counts, the error flags
        if (*reinterpret_cast<int32_t *>(hp + 2 * P) & ERR_MIRROR) {
            prof_end(g);
            set_error("internal error: an edge without its reverse edge");
            return MLIP_EHIP;
        }
        int64_t TE = 0;
        std::vector<int64_t> ebase(P + 1);
        for (int q = 0; q < P; ++q) {
            SlabView &v = g->slabs[q];
            v.n_edges_owned = hp[2 * q];
            v.n_edges = hp[2 * q + 1];
            ebase[q] = TE;
            TE += v.n_edges;
            T.n_edges[q] = v.n_edges;
            T.chunk0[q] = chunk_total;
            chunk_total += chunks_of(v.n_edges) + 1;
        }
        ebase[P] = TE;
        T.chunk0[P] = chunk_total;
        if (TE >= ((int64_t)1 << 31)) { prof_end(g); set_error("more than 2^31 local edges over all slabs"); return MLIP_EINVAL; }
        const size_t ne = (size_t)std::max<int64_t>(TE, 1);
        MLIP_TRY(st.senders.ensure(ne * 4));
        MLIP_TRY(st.shiftp.ensure(ne * 4));
        MLIP_TRY(st.recv.ensure(ne * 4));
        MLIP_TRY(st.mirror.ensure(ne * 4));
        MLIP_TRY(st.d.ensure(ne * 4));
        MLIP_TRY(st.chunk_row.ensure((size_t)chunk_total * 4));
        if (E > 0) {
            k_local_fill_owned<<<grid8(blocks_for(E, 256)), 256, 0, s>>>(
                E, T, g->recv.as<int32_t>(), g->senders.as<int32_t>(), g->shiftp.as<uint32_t>(), g->d.as<float>(),
                g->mirror.as<int32_t>(), g->needed_by.as<unsigned long long>(), g->local_in_owner.as<OwnRec>(),
                st.gbase.as<int32_t>(), st.ghost_local.as<int32_t>(), st.row_abs.as<int64_t>(), st.senders.as<int32_t>(),
                st.recv.as<int32_t>(), st.shiftp.as<uint32_t>(), st.d.as<float>(), st.mirror.as<int32_t>());
            MLIP_HIP(hipGetLastError());
        }
        if (n_ghost_total > 0) {
            k_local_fill_ghost<<<grid8((n_ghost_total + 3) / 4), 256, 0, s>>>(
                T, st.nodes.as<int32_t>(), g->row_ptr.as<int64_t>(), g->senders.as<int32_t>(), g->shiftp.as<uint32_t>(),
                g->d.as<float>(), g->mirror.as<int32_t>(), g->local_in_owner.as<OwnRec>(), st.row_abs.as<int64_t>(),
                st.senders.as<int32_t>(), st.recv.as<int32_t>(), st.shiftp.as<uint32_t>(), st.d.as<float>(),
                st.mirror.as<int32_t>());
            MLIP_HIP(hipGetLastError());
        }
        k_chunk_rows_parts<<<blocks_for(chunk_total, 256), 256, 0, s>>>(T, st.row_ptr.as<int64_t>(), st.chunk_row.as<int32_t>());
        MLIP_HIP(hipGetLastError());
        for (int q = 0; q < P; ++q) {
            SlabView &v = g->slabs[q];
            v.nodes = st.nodes.as<int32_t>() + T.row0[q];
            v.owned_sorted = st.owned_sorted.as<int32_t>() + (T.row0[q] - T.ghost0[q]);   // owned atoms before partition q
            v.row_ptr = st.row_ptr.as<int64_t>() + T.row0[q] + q;
            v.senders = st.senders.as<int32_t>() + ebase[q];
            v.shiftp = st.shiftp.as<uint32_t>() + ebase[q];
            v.recv = st.recv.as<int32_t>() + ebase[q];
            v.mirror = st.mirror.as<int32_t>() + ebase[q];
            v.d = st.d.as<float>() + ebase[q];
            v.chunk_row = st.chunk_row.as<int32_t>() + T.chunk0[q];
            v.ghost_owner = st.ghost_owner.as<int32_t>() + T.ghost0[q];
            v.ghost_src = st.ghost_src.as<int32_t>() + T.ghost0[q];
        }
        prof_end(g);
    } else {
        prof_end(g);
        MLIP_HIP(hipMemcpyAsync(hp, err, 4, hipMemcpyDeviceToHost, s));
        MLIP_HIP(hipStreamSynchronize(s));
        if (*reinterpret_cast<int32_t *>(hp) & ERR_MIRROR) {
            set_error("internal error: an edge without its reverse edge");
            return MLIP_EHIP;
        }
    }
    g->N = N;
    g->E = E;
    g->P = P;
    g->r_cut = r_cut;
    return MLIP_OK;
}

}  // namespace mlip

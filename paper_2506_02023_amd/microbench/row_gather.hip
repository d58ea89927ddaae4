// Micro-benchmark: how fast can a compute unit of gfx950 gather 256-byte rows with the access pattern of the
// reverse edge kernel's streaming phase, and does the width of the load instruction matter?
//
// A million rows of 64 floats stand for the per-atom arrays of a simple-cubic block of 100^3 atoms numbered in
// lattice order; every row has 46 "edges" whose senders are the row's neighbours within 2.3 lattice constants
// (index offsets dx * 10^4 + dy * 100 + dz, wrapped), in ascending order, as in a receiver-sorted CSR.  A
// wavefront walks a chunk of 1024 edges in steps of 16 and, one step ahead of their use, gathers the sender's
// row of one or two arrays and reads the edge's own row of a streamed array.
//   layout 1: one feature per lane, one `buffer_load_dword` per row (the kernel's layout): 16 per array and step
//   layout 4: four features per lane, one `buffer_load_dwordx4` per four rows: 4 per array and step
//   layout 2: the two gathered arrays interleaved per feature, one `buffer_load_dwordx2` fetches both rows: 16 per step
// The bytes are the same; only the number of vector memory instructions differs.
//
// Build and run (one MI355X):
//   hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops \
//       paper_2506_02023_amd/microbench/row_gather.hip -o paper_2506_02023_amd/microbench/row_gather
//   paper_2506_02023_amd/microbench/row_gather
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kF = 64, kRowBytes = kF * 4, kStep = 16, kChunk = 1024;
constexpr int kBufferFlags = 0x00020000;   // raw buffer, data format 32 bits

#define CHECK(x)                                                                     \
    do {                                                                             \
        hipError_t e_ = (x);                                                         \
        if (e_ != hipSuccess) {                                                      \
            std::fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));             \
            std::exit(1);                                                            \
        }                                                                            \
    } while (0)

struct Args {
    const float *ag;   // layout 2: the two gathered arrays interleaved per feature, [row][64][2]
    const float *a, *g, *w;
    const int32_t *senders;
    float *out;
    int64_t n_rows, n_edges;   // n_edges is a multiple of kChunk
};

// ARRAYS: 1 = gather a; 2 = gather a and g; 3 = a, g and the streamed w
template <int LAYOUT, int ARRAYS, int PER_SIMD>
__global__ void __launch_bounds__(256, PER_SIMD) k_gather(Args A)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)((blockIdx.x * blockDim.x + threadIdx.x) >> 6));
    const int n_waves = gridDim.x * (blockDim.x >> 6);
    const __amdgpu_buffer_rsrc_t a_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(A.a), 0, (int)(A.n_rows * kRowBytes), kBufferFlags);
    const __amdgpu_buffer_rsrc_t g_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(A.g), 0, (int)(A.n_rows * kRowBytes), kBufferFlags);
    const int64_t n_chunks = A.n_edges / kChunk;
    float acc = 0.f;
    f32x4 acc4 = {0.f, 0.f, 0.f, 0.f};
    for (int64_t chunk = wave; chunk < n_chunks; chunk += n_waves) {
        const int64_t e0 = chunk * kChunk;
        const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float *>(A.w) + e0 * kF, 0, kChunk * kRowBytes, kBufferFlags);
        const int32_t *sp = A.senders + e0;
        int32_t s_next = sp[lane & (kStep - 1)];   // senders of step 0
        if (LAYOUT == 1) {
            float av[2][kStep], gv[2][kStep], wv[2][kStep];
            auto issue = [&](int b, int32_t sj, int t) {
                const int32_t so = sj * kRowBytes;
#pragma unroll
                for (int k = 0; k < kStep; ++k) {
                    const int32_t o = __builtin_amdgcn_readlane(so, k);
                    av[b][k] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(a_rsrc, lane * 4, o, 0));
                    if (ARRAYS >= 2)
                        gv[b][k] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(g_rsrc, lane * 4, o, 0));
                    if (ARRAYS >= 3)
                        wv[b][k] = __builtin_bit_cast(
                            float, __builtin_amdgcn_raw_buffer_load_b32(w_rsrc, lane * 4, (t * kStep + k) * kRowBytes, 2));
                }
            };
            auto consume = [&](int b) {
#pragma unroll
                for (int k = 0; k < kStep; ++k) {
                    float v = av[b][k];
                    if (ARRAYS >= 2) v *= gv[b][k];
                    acc = (ARRAYS >= 3) ? fmaf(v, wv[b][k], acc) : acc + v;
                }
            };
            int32_t s_cur = s_next;
            s_next = sp[kStep + (lane & (kStep - 1))];
            issue(0, s_cur, 0);
#pragma unroll 1
            for (int t = 0; t < kChunk / kStep; t += 2) {
                int32_t s2 = sp[min((t + 2) * kStep, kChunk - kStep) + (lane & (kStep - 1))];
                issue(1, s_next, t + 1);
                consume(0);
                int32_t s3 = sp[min((t + 3) * kStep, kChunk - kStep) + (lane & (kStep - 1))];
                if (t + 2 < kChunk / kStep) issue(0, s2, t + 2);
                consume(1);
                s_next = s3;
            }
        } else if (LAYOUT == 2) {
            typedef float f32x2 __attribute__((ext_vector_type(2)));
            const __amdgpu_buffer_rsrc_t ag_rsrc = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<float *>(A.ag), 0, (int)(A.n_rows * 2 * kRowBytes), kBufferFlags);
            f32x2 agv[2][kStep];
            float wv[2][kStep];
            auto issue = [&](int b, int32_t sj, int t) {
                const int32_t so = sj * 2 * kRowBytes;
#pragma unroll
                for (int k = 0; k < kStep; ++k) {
                    const int32_t o = __builtin_amdgcn_readlane(so, k);
                    agv[b][k] = __builtin_bit_cast(f32x2, __builtin_amdgcn_raw_buffer_load_b64(ag_rsrc, lane * 8, o, 0));
                    if (ARRAYS >= 3)
                        wv[b][k] = __builtin_bit_cast(
                            float, __builtin_amdgcn_raw_buffer_load_b32(w_rsrc, lane * 4, (t * kStep + k) * kRowBytes, 2));
                }
            };
            auto consume = [&](int b) {
#pragma unroll
                for (int k = 0; k < kStep; ++k) {
                    const float v = agv[b][k][0] * agv[b][k][1];
                    acc = (ARRAYS >= 3) ? fmaf(v, wv[b][k], acc) : acc + v;
                }
            };
            int32_t s_cur = s_next;
            s_next = sp[kStep + (lane & (kStep - 1))];
            issue(0, s_cur, 0);
#pragma unroll 1
            for (int t = 0; t < kChunk / kStep; t += 2) {
                int32_t s2 = sp[min((t + 2) * kStep, kChunk - kStep) + (lane & (kStep - 1))];
                issue(1, s_next, t + 1);
                consume(0);
                int32_t s3 = sp[min((t + 3) * kStep, kChunk - kStep) + (lane & (kStep - 1))];
                if (t + 2 < kChunk / kStep) issue(0, s2, t + 2);
                consume(1);
                s_next = s3;
            }
        } else {
            const int q = lane >> 4, c = lane & 15;
            f32x4 av[2][4], gv[2][4], wv[2][4];
            auto issue = [&](int b, int32_t sj, int t) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int32_t s = __shfl(sj, 4 * i + q, 64);
                    const int32_t o = s * kRowBytes + c * 16;
                    av[b][i] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, o, 0, 0));
                    if (ARRAYS >= 2)
                        gv[b][i] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(g_rsrc, o, 0, 0));
                    if (ARRAYS >= 3)
                        wv[b][i] = __builtin_bit_cast(
                            f32x4, __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, q * kRowBytes + c * 16,
                                                                         (t * kStep + 4 * i) * kRowBytes, 2));
                }
            };
            auto consume = [&](int b) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    f32x4 v = av[b][i];
                    if (ARRAYS >= 2) v *= gv[b][i];
                    if (ARRAYS >= 3)
                        acc4 += v * wv[b][i];
                    else
                        acc4 += v;
                }
            };
            int32_t s_cur = s_next;
            s_next = sp[kStep + (lane & (kStep - 1))];
            issue(0, s_cur, 0);
#pragma unroll 1
            for (int t = 0; t < kChunk / kStep; t += 2) {
                int32_t s2 = sp[min((t + 2) * kStep, kChunk - kStep) + (lane & (kStep - 1))];
                issue(1, s_next, t + 1);
                consume(0);
                int32_t s3 = sp[min((t + 3) * kStep, kChunk - kStep) + (lane & (kStep - 1))];
                if (t + 2 < kChunk / kStep) issue(0, s2, t + 2);
                consume(1);
                s_next = s3;
            }
        }
    }
    A.out[(int64_t)wave * 64 + lane] = acc + acc4[0] + acc4[1] + acc4[2] + acc4[3];
}

template <int LAYOUT, int ARRAYS, int PER_SIMD = 2>
static void run(const Args &A, const char *what)
{
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    float best = 1e30f, sum = 0.f;
    const int reps = 6;
    for (int r = 0; r < reps; ++r) {
        CHECK(hipEventRecord(e0, nullptr));
        k_gather<LAYOUT, ARRAYS, PER_SIMD><<<256 * PER_SIMD, 256>>>(A);
        CHECK(hipEventRecord(e1, nullptr));
        CHECK(hipEventSynchronize(e1));
        float ms;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        if (r > 0) {
            best = std::min(best, ms);
            sum += ms;
        }
    }
    const double rows = (double)A.n_edges * ARRAYS;
    const double ms = sum / (reps - 1);
    std::printf("%-44s %d/SIMD %7.3f ms (min %7.3f)  %6.1f G rows/s  %5.2f TB/s through the loads  %5.1f cycles per row and CU\n", what, PER_SIMD, ms,
                best, rows / ms * 1e-6, rows * kRowBytes / ms * 1e-9, ms * 1e-3 * 2.4e9 * 256 / rows);
    CHECK(hipEventDestroy(e0));
    CHECK(hipEventDestroy(e1));
}

int main()
{
    const int n = 100;
    const int64_t N = (int64_t)n * n * n;
    std::vector<int32_t> off;
    for (int dx = -2; dx <= 2; ++dx)
        for (int dy = -2; dy <= 2; ++dy)
            for (int dz = -2; dz <= 2; ++dz) {
                const int d2 = dx * dx + dy * dy + dz * dz;
                if (d2 > 0 && d2 <= 5) off.push_back(dx * n * n + dy * n + dz);   // 56 neighbours within sqrt(5)
            }
    std::sort(off.begin(), off.end());
    // keep 46 of them, evenly, so that the degree matches the benchmark system's mean
    std::vector<int32_t> st;
    for (int k = 0; k < 46; ++k) st.push_back(off[(size_t)k * off.size() / 46]);
    const int deg = (int)st.size();
    int64_t E = N * deg;
    E -= E % kChunk;
    std::vector<int32_t> senders((size_t)E);
    for (int64_t e = 0; e < E; ++e) {
        const int64_t i = e / deg;
        int64_t j = i + st[(size_t)(e % deg)];
        j = (j % N + N) % N;
        senders[(size_t)e] = (int32_t)j;
    }
    Args A{};
    A.n_rows = N;
    A.n_edges = E;
    float *a, *g, *w, *out;
    int32_t *sd;
    CHECK(hipMalloc(&a, N * kRowBytes));
    CHECK(hipMalloc(&g, N * kRowBytes));
    CHECK(hipMalloc(&w, E * (int64_t)kRowBytes));
    float *ag;
    CHECK(hipMalloc(&ag, N * 2 * kRowBytes));
    CHECK(hipMemset(ag, 0, N * 2 * kRowBytes));
    A.ag = ag;
    CHECK(hipMalloc(&sd, E * 4));
    CHECK(hipMalloc(&out, 1024 * 4 * 64 * 4));
    CHECK(hipMemset(a, 0, N * kRowBytes));
    CHECK(hipMemset(g, 0, N * kRowBytes));
    CHECK(hipMemset(w, 0, E * (int64_t)kRowBytes));
    CHECK(hipMemcpy(sd, senders.data(), E * 4, hipMemcpyHostToDevice));
    A.a = a;
    A.g = g;
    A.w = w;
    A.senders = sd;
    A.out = out;
    std::printf("%lld rows of 256 bytes, %lld edges (degree %d), blocks of 4 wavefronts, 1-4 wavefronts per SIMD\n",
                (long long)N, (long long)E, deg);
    run<1, 1>(A, "one gathered array, dword loads");
    run<4, 1>(A, "one gathered array, dwordx4 loads");
    run<1, 2>(A, "two gathered arrays, dword loads");
    run<4, 2>(A, "two gathered arrays, dwordx4 loads");
    run<1, 3>(A, "two gathered + one streamed, dword loads");
    run<4, 3>(A, "two gathered + one streamed, dwordx4 loads");
    run<2, 2>(A, "two gathered arrays interleaved, dwordx2 loads");
    run<2, 3>(A, "two interleaved + one streamed, dwordx2");
    run<2, 3, 1>(A, "two interleaved + one streamed, dwordx2");
    // the same with one, three and four wavefronts per SIMD
    run<1, 3, 1>(A, "two gathered + one streamed, dword loads");
    run<1, 3, 3>(A, "two gathered + one streamed, dword loads");
    run<1, 2, 1>(A, "two gathered arrays, dword loads");
    run<1, 2, 4>(A, "two gathered arrays, dword loads");
    run<4, 3, 1>(A, "two gathered + one streamed, dwordx4 loads");
    run<4, 3, 4>(A, "two gathered + one streamed, dwordx4 loads");
    run<4, 1, 4>(A, "one gathered array, dwordx4 loads");
    CHECK(hipDeviceSynchronize());
    return 0;
}

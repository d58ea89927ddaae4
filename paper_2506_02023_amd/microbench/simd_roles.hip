// Micro-benchmark: do row-gather wavefronts keep their pace beside fp32 MFMA work when the two run on DIFFERENT SIMDs of
// a compute unit of gfx950?  (On the same SIMD they do not: fp32 MFMA and vector instructions share one pipeline, see
// mfma_valu_overlap.hip.)
//
// One block of 16 wavefronts per compute unit (96 KB of LDS keep a second block away).  Every wavefront reads the SIMD
// it was placed on from the hardware id register (HW_REG_HW_ID, bits 5:4) and takes its role from it:
//   "roles by SIMD id":    the wavefronts of the last 1 or 2 SIMDs stream, those of the other SIMDs multiply
//   "roles by wave index": the first 4 or 8 wavefronts of the block stream (one or two on every SIMD), the others multiply
// Streaming = the access pattern of the reverse edge kernel's streaming phase on an upper-edge graph: per edge the
// sender's rows of two arrays (gathered) and the edge's row of a third (streamed), 16 edges per step, one step of loads
// ahead, two multiply-adds and an LDS store per row; 23 edges per row of a 100^3 lattice, work handed out in items of 1024
// edges.  Dense = 80 v_mfma_f32_32x32x2_f32 per 32 edges, handed out in groups of 8 tiles.  The two kinds of wavefront
// do not exchange data: the benchmark shows only whether their times overlap.  It also prints on which SIMD the
// wavefronts of a block land, and repeats the shared-SIMD case with the dense work as v_mfma_f32_16x16x4_f32 (twice as
// many instructions of half the duration) and with the streaming wavefronts at a raised issue priority (s_setprio 3).
//
// Build and run (one MI355X):
//   hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops \
//       paper_2506_02023_amd/microbench/simd_roles.hip -o paper_2506_02023_amd/microbench/simd_roles
//   paper_2506_02023_amd/microbench/simd_roles
#include <hip/hip_runtime.h>
#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int kF = 64, kRowBytes = kF * 4, kStep = 16, kChunk = 1024;
constexpr int kBufferFlags = 0x00020000;
#define CHECK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { std::fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); std::exit(1); } } while (0)

struct Args {
    const float *a, *g, *w;
    const int32_t *senders;
    float *out;
    unsigned long long *counters;   // [0] next chunk, [1] next tile group
    uint32_t *hwid;                 // [block][wave]
    int64_t n_rows, n_edges;
    int what;                       // bit 0: streaming runs, bit 1: dense runs, bit 2: streaming wavefronts raise their priority
    int stream_simds;               // mode 0: SIMDs >= 4 - stream_simds stream
};

// MODE 0: role by SIMD id; MODE 1: role by wave index (the first 4 * stream_simds... waves with (wave & 3) spread) -> waves
// 0 .. 4*stream_simds-1 stream (one per SIMD each round if waves are dealt round-robin)
template <int MODE, int SMALL>
__global__ void __launch_bounds__(1024) k_roles(Args A)
{
    extern __shared__ float lds[];
    const int lane = threadIdx.x & 63;
    const int wib = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const uint32_t hw = __builtin_amdgcn_s_getreg((31 << 11) | (0 << 6) | 4);   // HW_REG_HW_ID
    const int simd = (hw >> 4) & 3;
    if (lane == 0) A.hwid[blockIdx.x * 16 + wib] = hw;
    const bool streamer = MODE == 0 ? (simd >= 4 - A.stream_simds) : (wib < 4 * A.stream_simds);
    float acc = 0.f;
    if (streamer) {
        if (!(A.what & 1)) return;
        if (A.what & 4) __builtin_amdgcn_s_setprio(3);
        const __amdgpu_buffer_rsrc_t a_rsrc =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(A.a), 0, (int)(A.n_rows * kRowBytes), kBufferFlags);
        const __amdgpu_buffer_rsrc_t g_rsrc =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(A.g), 0, (int)(A.n_rows * kRowBytes), kBufferFlags);
        float *my = lds + wib * (kStep * kF);
        const int64_t n_chunks = A.n_edges / kChunk;
        for (;;) {
            unsigned long long c = 0;
            if (lane == 0) c = atomicAdd(A.counters, 1ull);
            const int64_t chunk = (int64_t)__builtin_amdgcn_readfirstlane((int)c);
            if (chunk >= n_chunks) break;
            const int64_t e0 = chunk * kChunk;
            const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<float *>(A.w) + e0 * kF, 0, kChunk * kRowBytes, kBufferFlags);
            const int32_t *sp = A.senders + e0;
            float av[2][kStep], gv[2][kStep], wv[2][kStep];
            auto issue = [&](int b, int32_t sj, int t) {
                const int32_t so = sj * kRowBytes;
#pragma unroll
                for (int k = 0; k < kStep; ++k) {
                    const int32_t o = __builtin_amdgcn_readlane(so, k);
                    av[b][k] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(a_rsrc, lane * 4, o, 0));
                    gv[b][k] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(g_rsrc, lane * 4, o, 0));
                    wv[b][k] = __builtin_bit_cast(
                        float, __builtin_amdgcn_raw_buffer_load_b32(w_rsrc, lane * 4, (t * kStep + k) * kRowBytes, 2));
                }
            };
            auto consume = [&](int b) {
#pragma unroll
                for (int k = 0; k < kStep; ++k) {
                    acc = fmaf(av[b][k], wv[b][k], acc);                       // gbar_i += w * abar_j
                    const float ws = fmaf(av[b][k], 1.5f, gv[b][k] * 0.5f);    // wsym
                    my[k * kF + lane] = ws;                                    // queued for the dense work
                }
            };
            int32_t s_next = sp[lane & (kStep - 1)];
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
        acc += my[lane];
    } else {
        if (!(A.what & 2)) return;
        const int64_t n_tiles = A.n_edges / 32;
        f32x16 c0 = {0}, c1 = {0};
        f32x4 d0 = {0}, d1 = {0}, d2 = {0}, d3 = {0};
        float x = (float)lane * 1e-3f, y = 1.0f;
        for (;;) {
            unsigned long long c = 0;
            if (lane == 0) c = atomicAdd(A.counters + 16, 8ull);
            const int64_t tile = (int64_t)__builtin_amdgcn_readfirstlane((int)c);
            if (tile >= n_tiles) break;
#pragma unroll 1
            for (int t = 0; t < 8; ++t) {
                if (SMALL) {   // the same flop as 160 MFMAs of half the duration
#pragma unroll
                    for (int k = 0; k < 40; ++k) {
                        d0 = __builtin_amdgcn_mfma_f32_16x16x4f32(x, y, d0, 0, 0, 0);
                        d1 = __builtin_amdgcn_mfma_f32_16x16x4f32(y, x, d1, 0, 0, 0);
                        d2 = __builtin_amdgcn_mfma_f32_16x16x4f32(x, x, d2, 0, 0, 0);
                        d3 = __builtin_amdgcn_mfma_f32_16x16x4f32(y, y, d3, 0, 0, 0);
                    }
                } else {
#pragma unroll
                for (int k = 0; k < 40; ++k) {   // 80 MFMAs per tile of 32 pairs
                    c0 = __builtin_amdgcn_mfma_f32_32x32x2f32(x, y, c0, 0, 0, 0);
                    c1 = __builtin_amdgcn_mfma_f32_32x32x2f32(y, x, c1, 0, 0, 0);
                }
                }
                x = x * 0.999f + (c0[0] + d0[0]) * 1e-30f;
            }
        }
        acc = c0[0] + c1[3] + x + d0[0] + d1[1] + d2[2] + d3[3];
    }
    A.out[((int64_t)blockIdx.x * 16 + wib) * 64 + lane] = acc;
}

template <int MODE, int SMALL = 0>
static float run(Args A, int what, int stream_simds, const char *label)
{
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    A.what = what;
    A.stream_simds = stream_simds;
    float sum = 0.f, best = 1e30f;
    const int reps = 4;
    for (int r = 0; r < reps; ++r) {
        CHECK(hipMemset(A.counters, 0, 256));
        CHECK(hipDeviceSynchronize());
        CHECK(hipEventRecord(e0, nullptr));
        k_roles<MODE, SMALL><<<256, 1024, 96 * 1024>>>(A);
        CHECK(hipGetLastError());
        CHECK(hipEventRecord(e1, nullptr));
        CHECK(hipEventSynchronize(e1));
        float ms;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        if (r > 0) { sum += ms; best = std::min(best, ms); }
    }
    std::printf("%-58s stream on %d SIMD(s): %s%s  %7.3f ms (min %7.3f)\n", label, stream_simds, (what & 1) ? "stream " : "       ",
                (what & 2) ? "dense" : "     ", sum / (reps - 1), best);
    std::fflush(stdout);
    return sum / (reps - 1);
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
                if (d2 > 0 && d2 <= 5) off.push_back(dx * n * n + dy * n + dz);
            }
    std::sort(off.begin(), off.end());
    std::vector<int32_t> st;
    for (int k = 0; k < 23; ++k) st.push_back(off[(size_t)k * off.size() / 23]);   // the upper half: 23 edges per row
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
    CHECK(hipMalloc(&sd, E * 4));
    CHECK(hipMalloc(&out, 256 * 16 * 64 * 4));
    CHECK(hipMalloc(&A.counters, 256));
    CHECK(hipMalloc(&A.hwid, 256 * 16 * 4));
    CHECK(hipMemset(a, 0, N * kRowBytes));
    CHECK(hipMemset(g, 0, N * kRowBytes));
    CHECK(hipMemset(w, 0, E * (int64_t)kRowBytes));
    CHECK(hipMemcpy(sd, senders.data(), E * 4, hipMemcpyHostToDevice));
    A.a = a; A.g = g; A.w = w; A.senders = sd; A.out = out;
    CHECK(hipFuncSetAttribute((const void *)k_roles<0, 0>, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024));
    CHECK(hipFuncSetAttribute((const void *)k_roles<1, 0>, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024));
    CHECK(hipFuncSetAttribute((const void *)k_roles<1, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024));
    std::printf("%lld rows, %lld edges (degree %d): 3 row loads per edge, 80 fp32 MFMA per 32 edges; 256 blocks of 16 wavefronts\n",
                (long long)N, (long long)E, deg);
    run<0>(A, 1, 1, "roles by SIMD id");
    // where did the wavefronts land?
    std::vector<uint32_t> hw(256 * 16);
    CHECK(hipMemcpy(hw.data(), A.hwid, hw.size() * 4, hipMemcpyDeviceToHost));
    int hist[4][16] = {};
    for (int b = 0; b < 256; ++b)
        for (int wv = 0; wv < 16; ++wv) hist[(hw[b * 16 + wv] >> 4) & 3][wv]++;
    for (int s = 0; s < 4; ++s) {
        std::printf("SIMD %d hosts wave index:", s);
        for (int wv = 0; wv < 16; ++wv) std::printf(" %3d", hist[s][wv]);
        std::printf("\n");
    }
    std::printf("block 0:");
    for (int wv = 0; wv < 16; ++wv) std::printf(" %08x", hw[wv]);
    std::printf("\nblock 1:");
    for (int wv = 0; wv < 16; ++wv) std::printf(" %08x", hw[16 + wv]);
    std::printf("\n");
    for (int ss = 1; ss <= 2; ++ss) {
        run<0>(A, 1, ss, "roles by SIMD id");
        run<0>(A, 2, ss, "roles by SIMD id");
        run<0>(A, 3, ss, "roles by SIMD id");
        run<1>(A, 1, ss, "roles by wave index (streamers on every SIMD)");
        run<1>(A, 2, ss, "roles by wave index (streamers on every SIMD)");
        run<1>(A, 3, ss, "roles by wave index (streamers on every SIMD)");
    }
    run<1, 1>(A, 2, 1, "roles by wave index, dense work as 16x16x4 MFMAs");
    run<1, 1>(A, 3, 1, "roles by wave index, dense work as 16x16x4 MFMAs");
    run<1, 0>(A, 7, 1, "roles by wave index, streamers at priority 3");
    run<1, 1>(A, 7, 1, "roles by wave index, 16x16x4 MFMAs, streamers at priority 3");
    CHECK(hipDeviceSynchronize());
    return 0;
}

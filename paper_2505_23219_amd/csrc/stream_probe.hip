// Measurement tool, not part of the library: what does the inner loop of a weight-streaming
// kernel cost on this GPU, by itself?
//
// The decoding step is bound by reading every weight once (Ghidorah, sections 2.1 and 2.2.2).
// This program times the bare stream - 256 workgroups of 8 wavefronts, every wavefront reading
// its own run of 1 KiB weight blocks with non-temporal 128-bit loads, a few k-steps ahead,
// no LDS, no barriers, nothing after the loop but one store per lane - with the two ways of
// multiplying a block by the activations that the linear-layer kernel could use:
//
//   mfma   v_mfma_f32_16x16x32_f16 with the block as A operand and MT packed activation
//          blocks (16 rows of x each, rows past M are padding) as B operands, read from the L2;
//   dot2   for one row of x (M = 1): v_dot2_f32_f16 on the lane's 8 weights and the matching
//          8 activations - a wavefront-reduction GEMV, no padded 16-row tile;
//   none   the loads alone (the blocks are only added up), as the floor.
//
// Every launch reads 256 x R x 128 KiB (R = 16-row tiles per workgroup, 4096 columns); four
// separate buffers are used in turn, so nothing is served by a cache.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float f4 __attribute__((ext_vector_type(4)));

enum { MUL_NONE = 0, MUL_MFMA = 1, MUL_DOT2 = 2 };

constexpr int kWaves = 8, kSteps = 128;          // k-steps of 32 columns: K = 4096
constexpr int kStepsPerWave = kSteps / kWaves;
constexpr int kXBlocks = 128;                    // packed activation blocks per row tile (K / 32)

__device__ __forceinline__ void pin_order()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

// W: tiles in blocks of 8, k-step major inside a block (the library's wide layout); workgroup b
// owns tiles [b * R, b * R + R), wavefront w the k-steps [w * 16, w * 16 + 16) of each.
template <int R, int MT, int PD, int MUL>
__global__ __launch_bounds__(kWaves * 64) void k_stream(const half8* __restrict__ W, const half8* __restrict__ X,
                                                        f4* __restrict__ out)
{
    constexpr int NB = MT > 0 ? MT : 1;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, g4 = lane >> 4;
    const int t0 = blockIdx.x * R, s0 = wave * kStepsPerWave;
    f4 acc[R][NB];
#pragma unroll
    for (int t = 0; t < R; ++t)
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[t][b] = (f4){0.f, 0.f, 0.f, 0.f};
    half8 w[PD][R], x[PD][NB];
    auto load = [&](int slot, int s) {
        s = s < kStepsPerWave ? s : kStepsPerWave - 1;
#pragma unroll
        for (int t = 0; t < R; ++t) {
            const size_t blk = (((size_t)((t0 + t) >> 3) * kSteps + s0 + s) << 3) + ((t0 + t) & 7);
            w[slot][t] = __builtin_nontemporal_load(W + blk * 64 + lane);
        }
        if constexpr (MUL == MUL_MFMA) {
#pragma unroll
            for (int b = 0; b < MT; ++b) x[slot][b] = X[((size_t)(s0 + s) * MT + b) * 64 + lane];
        } else if constexpr (MUL == MUL_DOT2) {
            x[slot][0] = X[(size_t)(s0 + s) * 64 + g4 * 16];   // row 0 of the block: 8 columns per lane group
        }
    };
#pragma unroll
    for (int p = 0; p < PD; ++p) {
        load(p, p);
        pin_order();
    }
    for (int s = 0; s < kStepsPerWave; s += PD) {
#pragma unroll
        for (int p = 0; p < PD; ++p) {
#pragma unroll
            for (int t = 0; t < R; ++t) {
                if constexpr (MUL == MUL_MFMA) {
#pragma unroll
                    for (int b = 0; b < MT; ++b)
                        acc[t][b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(w[p][t], x[p][b], acc[t][b], 0, 0, 0);
                } else if constexpr (MUL == MUL_DOT2) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        half2v a = {w[p][t][2 * e], w[p][t][2 * e + 1]}, b = {x[p][0][2 * e], x[p][0][2 * e + 1]};
                        acc[t][0][0] = __builtin_amdgcn_fdot2(a, b, acc[t][0][0], false);
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[t][0][e] += (float)w[p][t][2 * e] + (float)w[p][t][2 * e + 1];
                }
            }
            pin_order();
            load(p, s + p + PD);
            pin_order();
        }
    }
    f4 tot = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < R; ++t)
#pragma unroll
        for (int b = 0; b < NB; ++b) tot += acc[t][b];
    out[((size_t)blockIdx.x * kWaves + wave) * 64 + lane] = tot;
}

static half8* g_w[4];
static half8* g_x;
static f4* g_out;
static hipEvent_t g_e0, g_e1;
static int g_bad = 0;

static void check(hipError_t e, const char* what)
{
    if (e != hipSuccess) {
        fprintf(stderr, "%s: %s\n", what, hipGetErrorString(e));
        exit(1);
    }
}

constexpr int kMaxR = 8;
constexpr size_t kWBytes = (size_t)256 * kMaxR * kSteps * 1024;   // largest launch: 256 MiB
constexpr size_t kXBytes = (size_t)kXBlocks * 8 * 1024;           // up to 8 row tiles of x

template <int R, int MT, int PD, int MUL>
static void run(const char* mul)
{
    static_assert(R <= kMaxR && MT <= 8 && kStepsPerWave % PD == 0, "inside the buffers");
    const double bytes = 256.0 * R * kSteps * 1024;
    auto launch = [&](int i) {
        hipLaunchKernelGGL((k_stream<R, MT, PD, MUL>), dim3(256), dim3(kWaves * 64), 0, 0, g_w[i & 3], g_x, g_out);
    };
    for (int i = 0; i < 4; ++i) launch(i);
    check(hipDeviceSynchronize(), "warm-up");
    const int iters = 24;
    check(hipEventRecord(g_e0), "record");
    for (int i = 0; i < iters; ++i) launch(i);
    check(hipEventRecord(g_e1), "record");
    check(hipEventSynchronize(g_e1), "synchronize");
    float ms = 0;
    check(hipEventElapsedTime(&ms, g_e0, g_e1), "elapsed");
    const double us = ms * 1e3 / iters;
    printf("| %-4s | %d | %2d | %d | %5.1f | %6.2f | %5.0f |\n", mul, R, MUL == MUL_DOT2 ? 1 : (MUL == MUL_MFMA ? MT * 16 : 0), PD,
           bytes / 1048576, us, bytes / us / 1e3);
    fflush(stdout);
    if (!(us > 0)) g_bad = 1;
}

int main()
{
    for (int i = 0; i < 4; ++i) {
        check(hipMalloc(&g_w[i], kWBytes), "hipMalloc");
        check(hipMemset(g_w[i], 0x11, kWBytes), "hipMemset");
    }
    check(hipMalloc(&g_x, kXBytes), "hipMalloc");
    check(hipMemset(g_x, 0x22, kXBytes), "hipMemset");
    check(hipMalloc(&g_out, (size_t)256 * kWaves * 64 * sizeof(f4)), "hipMalloc");
    check(hipEventCreate(&g_e0), "event");
    check(hipEventCreate(&g_e1), "event");
    printf("weight stream of one launch, 256 workgroups x 8 wavefronts, launches back to back (time per launch\n"
           "includes the gap between launches)\n\n");
    printf("| multiply | tiles per workgroup | rows of x | k-steps in flight | MiB per launch | us per launch | GB/s |\n");
    printf("|---|---|---|---|---|---|---|\n");
    // one row of x: matrix core against wavefront-reduction GEMV, at the sizes of a 7B-shaped
    // QKV layer (3 tiles per workgroup) and gate|up layer (7)
    run<3, 0, 2, MUL_NONE>("none");
    run<3, 1, 2, MUL_MFMA>("mfma");
    run<3, 1, 2, MUL_DOT2>("dot2");
    run<7, 0, 1, MUL_NONE>("none");
    run<7, 1, 1, MUL_MFMA>("mfma");
    run<7, 1, 1, MUL_DOT2>("dot2");
    // 64 rows of x
    run<3, 4, 2, MUL_MFMA>("mfma");
    run<7, 4, 1, MUL_MFMA>("mfma");
    check(hipDeviceSynchronize(), "end");
    return g_bad;
}

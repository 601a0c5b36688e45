// Skinny linear layer  y[M,N] = x[M,K] . W[N,K]^T  for 1 <= M <= 128 rows.
//
// The cost of these layers in a verification step is streaming W once
// (Ghidorah, section 2.1: decoding is bound by memory bandwidth because the
// weights are re-read every step).  W is therefore stored pre-packed in
// 16-row x 32-column tiles whose 1 KiB image is exactly the A operand of one
// v_mfma_f32_16x16x32_f16: lane l holds row l%16, columns (l/16)*8..+8.  A
// wavefront walks along K through consecutive 1 KiB blocks with one
// 128-bit load per lane per block, fully coalesced, several blocks in flight.
// x (tiny, cache resident) supplies the B operand, so the product comes out
// transposed: acc[n][m], lane l / register r = row n=(l/16)*4+r, column m=l%16.
#include "common.h"

namespace ghd {

// Packs row-major W[N,K] into the tiled layout; one thread per 16-byte chunk.
__global__ void k_pack_weight(half8* __restrict__ dst, const half_t* __restrict__ src, int N, int K,
                              int ntiles, int ksteps)
{
    size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)ntiles * ksteps * 64;
    if (id >= total) return;
    int lane = (int)(id & 63);
    size_t blk = id >> 6;
    int ks = (int)(blk % ksteps);
    int tile = (int)(blk / ksteps);
    int n = tile * 16 + (lane & 15);
    int k = ks * 32 + (lane >> 4) * 8;
    half8 v;
    for (int e = 0; e < 8; ++e)
        v[e] = (n < N && k + e < K) ? src[(size_t)n * K + k + e] : (half_t)0;
    dst[id] = v;
}

ghd_status launch_pack(void* dst, const void* src, int N, int K, hipStream_t st)
{
    int ntiles = ceil_div(N, 16), ksteps = ceil_div(K, 32);
    size_t total = (size_t)ntiles * ksteps * 64;
    unsigned blocks = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL(k_pack_weight, dim3(blocks), dim3(256), 0, st, (half8*)dst,
                       (const half_t*)src, N, K, ntiles, ksteps);
    return check_launch();
}

// One wavefront owns NT weight tiles (16*NT output features) over a K range of
// `kps` k-steps; four independent wavefronts per workgroup.  DEPTH k-steps of
// loads are kept in flight in a register ring.
template <int MT, int NT, int DEPTH>
__global__ __launch_bounds__(256) void k_gemm_skinny(const half8* __restrict__ Wp,
                                                     const half_t* __restrict__ x,
                                                     float* __restrict__ out, int M, int N, int K,
                                                     int64_t ldx, int64_t ld, int ksteps, int kps,
                                                     int ntiles)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int tile0 = (blockIdx.x * 4 + wave) * NT;
    if (tile0 >= ntiles) return;
    const int split = blockIdx.y;
    const int ks0 = split * kps;
    const int ks1 = min(ks0 + kps, ksteps);
    const int c = lane & 15, g = lane >> 4;

    const half8* wptr[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        int tile = min(tile0 + t, ntiles - 1);
        wptr[t] = Wp + (size_t)tile * ksteps * 64 + lane;
    }
    const half_t* xptr[MT];
    bool xrow_ok[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        int m = t * 16 + c;
        xrow_ok[t] = m < M;
        xptr[t] = x + (size_t)min(m, M - 1) * ldx + g * 8;
    }

    floatx4 acc[NT][MT];
#pragma unroll
    for (int a = 0; a < NT; ++a)
#pragma unroll
        for (int b = 0; b < MT; ++b) acc[a][b] = (floatx4){0.f, 0.f, 0.f, 0.f};

    half8 wb[DEPTH][NT], xb[DEPTH][MT];
    const half8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};

    auto fetch = [&](int slot, int ks) {
        if (ks < ks1) {
#pragma unroll
            for (int t = 0; t < NT; ++t) wb[slot][t] = wptr[t][(size_t)ks * 64];
            const bool kok = ks * 32 + g * 8 < K;   // K % 8 == 0: a chunk is all in or all out
#pragma unroll
            for (int t = 0; t < MT; ++t)
                xb[slot][t] = (xrow_ok[t] && kok) ? *(const half8*)(xptr[t] + (size_t)ks * 32) : zero8;
        } else {
#pragma unroll
            for (int t = 0; t < NT; ++t) wb[slot][t] = zero8;
#pragma unroll
            for (int t = 0; t < MT; ++t) xb[slot][t] = zero8;
        }
    };

#pragma unroll
    for (int u = 0; u < DEPTH; ++u) fetch(u, ks0 + u);

    for (int ks = ks0; ks < ks1; ks += DEPTH) {
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) {
#pragma unroll
            for (int a = 0; a < NT; ++a)
#pragma unroll
                for (int b = 0; b < MT; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wb[u][a], xb[u][b], acc[a][b],
                                                                      0, 0, 0);
            fetch(u, ks + u + DEPTH);
        }
    }

    // acc[a][b][r] = y[m = b*16 + c][n = (tile0+a)*16 + g*4 + r]
#pragma unroll
    for (int a = 0; a < NT; ++a) {
        if (tile0 + a >= ntiles) break;
        int n0 = (tile0 + a) * 16 + g * 4;
#pragma unroll
        for (int b = 0; b < MT; ++b) {
            int m = b * 16 + c;
            if (m >= M) continue;
            float* o = out + ((size_t)split * M + m) * ld + n0;
            if (n0 + 3 < N && ((ld & 3) == 0)) {
                *(floatx4*)o = acc[a][b];
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (n0 + r < N) o[r] = acc[a][b][r];
            }
        }
    }
}


// Variant for M > 16: x no longer fits the register/L1 budget of every
// wavefront, so the workgroup (NW wavefronts that share a K range and own
// NW*NT consecutive weight tiles) stages x through LDS in chunks of DEPTH
// k-steps, double buffered, one barrier per chunk.  Fragments are stored in
// B-operand order (k-step, row tile, lane) with each 16-lane group padded by
// 16 bytes, so the 128-bit reads are conflict free.  The weight stream is
// unchanged: DEPTH k-steps of 128-bit loads in flight per wavefront.
template <int MT, int NT, int NW, int DEPTH>
__global__ __launch_bounds__(NW * 64) void k_gemm_lds(const half8* __restrict__ Wp,
                                                      const half_t* __restrict__ x,
                                                      float* __restrict__ out, int M, int N, int K,
                                                      int64_t ldx, int64_t ld, int ksteps, int kps,
                                                      int ntiles)
{
    constexpr int FRAG = 4 * 272;                 // bytes of one padded 16x32 fragment
    constexpr int CHUNK = DEPTH * MT * FRAG;      // bytes of one x chunk
    constexpr int PIECES = DEPTH * MT * 64;       // 16-byte pieces per chunk
    constexpr int T = NW * 64;
    constexpr int PPT = (PIECES + T - 1) / T;
    __shared__ __attribute__((aligned(16))) char xs[2 * CHUNK];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int c = lane & 15, g = lane >> 4;
    const int tile0 = (blockIdx.x * NW + wave) * NT;
    const int split = blockIdx.y;
    const int ks0 = split * kps;
    const int ks1 = min(ks0 + kps, ksteps);
    const int nchunks = (ks1 - ks0 + DEPTH - 1) / DEPTH;

    const half8* wptr[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        int tile = min(tile0 + t, ntiles - 1);
        wptr[t] = Wp + (size_t)tile * ksteps * 64 + lane;
    }

    // x staging: piece p -> (fragment f = p/64, row c = (p/4)%16, k group g = p%4)
    const half8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
    int p_src_row[PPT], p_koff[PPT], p_dst[PPT];
    bool p_ok[PPT];
#pragma unroll
    for (int i = 0; i < PPT; ++i) {
        int p = tid + i * T;
        int f = p >> 6, pc = (p >> 2) & 15, pg = p & 3;
        int s = f / MT, mt = f % MT;
        int m = mt * 16 + pc;
        p_ok[i] = (p < PIECES) && (m < M);
        p_src_row[i] = min(m, M - 1);
        p_koff[i] = s * 32 + pg * 8;
        p_dst[i] = f * FRAG + pg * 272 + pc * 16;
    }
    half8 xr[PPT];
    auto x_fetch = [&](int chunk) {
        int kbase = (ks0 + chunk * DEPTH) * 32;
#pragma unroll
        for (int i = 0; i < PPT; ++i) {
            int k = kbase + p_koff[i];
            bool ok = p_ok[i] && k < K && (k >> 5) < ks1;
            xr[i] = ok ? *(const half8*)(x + (size_t)p_src_row[i] * ldx + k) : zero8;
        }
    };
    auto x_store = [&](int buf) {
#pragma unroll
        for (int i = 0; i < PPT; ++i)
            if (tid + i * T < PIECES) *(half8*)(xs + buf * CHUNK + p_dst[i]) = xr[i];
    };

    floatx4 acc[NT][MT];
#pragma unroll
    for (int a = 0; a < NT; ++a)
#pragma unroll
        for (int b = 0; b < MT; ++b) acc[a][b] = (floatx4){0.f, 0.f, 0.f, 0.f};

    half8 wb[DEPTH][NT];
    auto w_fetch = [&](int slot, int ks) {
#pragma unroll
        for (int t = 0; t < NT; ++t) wb[slot][t] = (ks < ks1) ? wptr[t][(size_t)ks * 64] : zero8;
    };
#pragma unroll
    for (int u = 0; u < DEPTH; ++u) w_fetch(u, ks0 + u);

    x_fetch(0);
    x_store(0);
    if (nchunks > 1) x_fetch(1);
    __syncthreads();

    for (int ch = 0; ch < nchunks; ++ch) {
        const char* xb = xs + (ch & 1) * CHUNK + g * 272 + c * 16;
        const int ks = ks0 + ch * DEPTH;
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) {
            half8 xf[MT];
#pragma unroll
            for (int b = 0; b < MT; ++b) xf[b] = *(const half8*)(xb + (u * MT + b) * FRAG);
#pragma unroll
            for (int a = 0; a < NT; ++a)
#pragma unroll
                for (int b = 0; b < MT; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wb[u][a], xf[b], acc[a][b], 0,
                                                                      0, 0);
            w_fetch(u, ks + u + DEPTH);
        }
        if (ch + 1 < nchunks) {
            x_store((ch + 1) & 1);
            if (ch + 2 < nchunks) x_fetch(ch + 2);
        }
        __syncthreads();
    }

#pragma unroll
    for (int a = 0; a < NT; ++a) {
        if (tile0 + a >= ntiles) break;
        int n0 = (tile0 + a) * 16 + g * 4;
#pragma unroll
        for (int b = 0; b < MT; ++b) {
            int m = b * 16 + c;
            if (m >= M) continue;
            float* o = out + ((size_t)split * M + m) * ld + n0;
            if (n0 + 3 < N && ((ld & 3) == 0)) {
                *(floatx4*)o = acc[a][b];
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (n0 + r < N) o[r] = acc[a][b][r];
            }
        }
    }
}

static int g_force_nt = 0, g_force_s = 0, g_force_nw = 0, g_force_lds = -1;
void set_gemm_override(int nt, int s, int nw, int lds)
{
    g_force_nt = nt;
    g_force_s = s;
    g_force_nw = nw;
    g_force_lds = lds;
}

GemmPlan plan_gemm(int M, int N, int K)
{
    GemmPlan p;
    p.MT = ceil_div(M, 16);
    p.ksteps = ceil_div(K, 32);
    p.ntiles = ceil_div(N, 16);
    p.lds = p.MT >= 2;
    if (g_force_lds >= 0) p.lds = g_force_lds != 0 && p.MT >= 2;
    p.NW = 4;
    if (g_force_nw) p.NW = g_force_nw;
    if (!p.lds) p.NW = 4;
    // Two weight tiles per wavefront reuse every x fragment twice once x traffic matters.
    p.NT = (p.MT >= 2 && p.ntiles >= 512) ? 2 : 1;
    if (g_force_nt) p.NT = g_force_nt;
    if (p.lds && p.NW == 8 && p.MT >= 7 && p.NT > 2) p.NT = 2;   // register budget of 512 threads
    // Enough wavefronts to keep ~8 per compute unit streaming, at least 8 k-steps each.
    int waves = ceil_div(p.ntiles, p.NT);
    int S = 1;
    const int target = 2048;
    if (waves < target) S = ceil_div(target, waves);
    int maxS = p.ksteps / 8;
    if (maxS < 1) maxS = 1;
    if (S > maxS) S = maxS;
    if (g_force_s) S = g_force_s;
    if (S > p.ksteps) S = p.ksteps;
    p.kps = ceil_div(p.ksteps, S);
    p.S = ceil_div(p.ksteps, p.kps);
    return p;
}

template <int MT, int NT>
static void launch_direct(const GemmPlan& p, const void* Wp, const half_t* x, int64_t ldx,
                          float* out, int64_t ld, int M, int N, int K, hipStream_t st)
{
    constexpr int DEPTH = (NT == 1) ? 6 : (NT == 2 ? 4 : 2);
    dim3 grid(ceil_div(p.ntiles, 4 * NT), p.S);
    hipLaunchKernelGGL((k_gemm_skinny<MT, NT, DEPTH>), grid, dim3(256), 0, st, (const half8*)Wp, x,
                       out, M, N, K, ldx, ld, p.ksteps, p.kps, p.ntiles);
}

template <int MT, int NT, int NW>
static void launch_lds(const GemmPlan& p, const void* Wp, const half_t* x, int64_t ldx, float* out,
                       int64_t ld, int M, int N, int K, hipStream_t st)
{
    constexpr int DEPTH = 4;
    dim3 grid(ceil_div(p.ntiles, NW * NT), p.S);
    hipLaunchKernelGGL((k_gemm_lds<MT, NT, NW, DEPTH>), grid, dim3(NW * 64), 0, st, (const half8*)Wp,
                       x, out, M, N, K, ldx, ld, p.ksteps, p.kps, p.ntiles);
}

template <int MT>
static void launch_mt(const GemmPlan& p, const void* Wp, const half_t* x, int64_t ldx, float* out,
                      int64_t ld, int M, int N, int K, hipStream_t st)
{
#define GHD_ARGS p, Wp, x, ldx, out, ld, M, N, K, st
    if constexpr (MT >= 2) {
        if (p.lds) {
            if (p.NW == 8) {
                if (p.NT == 1) launch_lds<MT, 1, 8>(GHD_ARGS);
                else if (p.NT == 2) launch_lds<MT, 2, 8>(GHD_ARGS);
                else launch_lds<MT, 4, 8>(GHD_ARGS);
            } else {
                if (p.NT == 1) launch_lds<MT, 1, 4>(GHD_ARGS);
                else if (p.NT == 2) launch_lds<MT, 2, 4>(GHD_ARGS);
                else launch_lds<MT, 4, 4>(GHD_ARGS);
            }
            return;
        }
    }
    if (p.NT == 1) launch_direct<MT, 1>(GHD_ARGS);
    else if (p.NT == 2) launch_direct<MT, 2>(GHD_ARGS);
    else launch_direct<MT, 4>(GHD_ARGS);
#undef GHD_ARGS
}

ghd_status launch_gemm(const GemmPlan& p, const void* Wp, const half_t* x, int64_t ldx, float* out,
                       int64_t ld, int M, int N, int K, hipStream_t st)
{
    switch (p.MT) {
    case 1: launch_mt<1>(p, Wp, x, ldx, out, ld, M, N, K, st); break;
    case 2: launch_mt<2>(p, Wp, x, ldx, out, ld, M, N, K, st); break;
    case 3: launch_mt<3>(p, Wp, x, ldx, out, ld, M, N, K, st); break;
    case 4: launch_mt<4>(p, Wp, x, ldx, out, ld, M, N, K, st); break;
    case 5: launch_mt<5>(p, Wp, x, ldx, out, ld, M, N, K, st); break;
    case 6: launch_mt<6>(p, Wp, x, ldx, out, ld, M, N, K, st); break;
    case 7: launch_mt<7>(p, Wp, x, ldx, out, ld, M, N, K, st); break;
    default: launch_mt<8>(p, Wp, x, ldx, out, ld, M, N, K, st); break;
    }
    return check_launch();
}

}  // namespace ghd

// Small kernels around the skinny GEMMs: tree setup (depth, ancestor masks,
// rotary table), split-K reduction fused with residual add + RMSNorm, with the
// rotary embedding + KV append, and with SwiGLU.  The paper (section 2.2.2)
// leaves these element-wise operations out of its cost model; here they ride
// on the split-K reduction that the skinny GEMMs need anyway, so none of them
// costs a pass over HBM of its own.
#include "common.h"

namespace ghd {

// ---- tree setup ------------------------------------------------------------
// One workgroup.  Thread i < M walks from node i to the root (at most M steps,
// so a malformed parent[] terminates), collecting depth and the 128-bit
// ancestor-or-self mask (section 2.3: the tokens a drafted token relates to).
// The rotary table holds (cos, sin) of (kv_len + depth[i]) * base^(-2j/d),
// evaluated in double and narrowed once.
__global__ __launch_bounds__(256) void k_tree_setup(const int32_t* __restrict__ parent, int M,
                                                    int kv_len, int d, float rope_base,
                                                    int32_t* __restrict__ depth_out,
                                                    uint64_t* __restrict__ mask_out,
                                                    float2* __restrict__ rope)
{
    __shared__ int32_t s_parent[GHD_MAX_M];
    __shared__ int32_t s_depth[GHD_MAX_M];
    int tid = threadIdx.x;
    if (tid < M) s_parent[tid] = parent[tid];
    __syncthreads();
    if (tid < M) {
        uint64_t lo = 0, hi = 0;
        int dep = 0, j = tid;
        for (int step = 0; step < M; ++step) {
            if (j < 64) lo |= 1ull << j; else hi |= 1ull << (j - 64);
            int p = s_parent[j];
            if (p < 0 || p >= j) break;
            j = p;
            ++dep;
        }
        s_depth[tid] = dep;
        if (depth_out) depth_out[tid] = dep;
        if (mask_out) {
            mask_out[2 * tid] = lo;
            mask_out[2 * tid + 1] = hi;
        }
    }
    __syncthreads();
    if (rope) {
        int half = d / 2;
        for (int e = tid; e < M * half; e += blockDim.x) {
            int m = e / half, j = e % half;
            double ang = (double)(kv_len + s_depth[m]) * pow((double)rope_base, -2.0 * j / d);
            rope[e] = make_float2((float)cos(ang), (float)sin(ang));
        }
    }
}

ghd_status launch_tree_setup(const int32_t* parent, int M, int kv_len, int d, float rope_base,
                             int32_t* depth, uint64_t* mask, float2* rope, hipStream_t st)
{
    hipLaunchKernelGGL(k_tree_setup, dim3(1), dim3(256), 0, st, parent, M, kv_len, d, rope_base,
                       depth, mask, rope);
    return check_launch();
}

// ---- plain split-K reduction -------------------------------------------------
__global__ __launch_bounds__(256) void k_reduce_out(void* __restrict__ y, int64_t ldy, int out_f16,
                                                    const float* __restrict__ part, int S,
                                                    int64_t ld, int M, int N)
{
    int n = blockIdx.x * blockDim.x + threadIdx.x;
    int m = blockIdx.y;
    if (n >= N) return;
    float acc = 0.f;
    for (int s = 0; s < S; ++s) acc += part[((size_t)s * M + m) * ld + n];
    if (out_f16) ((half_t*)y)[(size_t)m * ldy + n] = (half_t)acc;
    else ((float*)y)[(size_t)m * ldy + n] = acc;
}

ghd_status launch_reduce_out(void* y, int64_t ldy, bool out_f16, const float* part, int S,
                             int64_t ld, int M, int N, hipStream_t st)
{
    hipLaunchKernelGGL(k_reduce_out, dim3(ceil_div(N, 256), M), dim3(256), 0, st, y, ldy,
                       (int)out_f16, part, S, ld, M, N);
    return check_launch();
}

// ---- residual add + RMSNorm ----------------------------------------------------
// One workgroup per row.  x_new = (x_old or widen(x_in16)) + sum of the S split
// partials (fixed order, so the result is run-to-run identical); then
// n16 = fp16(x_new * rsqrt(mean(x_new^2) + eps) * g).
__global__ __launch_bounds__(256) void k_residual_norm(float* __restrict__ x,
                                                       const half_t* __restrict__ x_in16,
                                                       const float* __restrict__ part, int S,
                                                       int64_t ld, const half_t* __restrict__ g,
                                                       half_t* __restrict__ n16, int M, int H,
                                                       float eps)
{
    extern __shared__ float s_row[];   // H floats
    __shared__ float s_red[4];
    int m = blockIdx.x, tid = threadIdx.x;
    float ss = 0.f;
    for (int c = tid; c < H; c += 256) {
        float v = x_in16 ? (float)x_in16[(size_t)m * H + c] : x[(size_t)m * H + c];
        for (int s = 0; s < S; ++s) v += part[((size_t)s * M + m) * ld + c];
        s_row[c] = v;
        x[(size_t)m * H + c] = v;
        ss += v * v;
    }
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
    if ((tid & 63) == 0) s_red[tid >> 6] = ss;
    __syncthreads();
    if (!g) return;
    float tot = s_red[0] + s_red[1] + s_red[2] + s_red[3];
    float r = 1.0f / sqrtf(tot / (float)H + eps);
    for (int c = tid; c < H; c += 256)
        n16[(size_t)m * H + c] = (half_t)(s_row[c] * r * (float)g[c]);
}

ghd_status launch_residual_norm(float* x, const half_t* x_in16, const float* part, int S, int64_t ld,
                                const half_t* g, half_t* n16, int M, int H, float eps,
                                hipStream_t st)
{
    hipLaunchKernelGGL(k_residual_norm, dim3(M), dim3(256), (size_t)H * sizeof(float), st, x, x_in16,
                       part, S, ld, g, n16, M, H, eps);
    return check_launch();
}

// ---- QKV epilogue: reduce, rotate, append --------------------------------------
// One thread per (node m, head h, pair j < d/2).  Columns of the fused QKV
// output: [0,H) q, [H,2H) k, [2H,3H) v.  q and k of node m turn by the angle of
// position kv_len + depth[m] in the half-split pairing (j, j + d/2); the
// rotated key and the value go to cache row kv_len + m as fp16.
__global__ __launch_bounds__(256) void k_qkv_epilogue(const float* __restrict__ part, int S,
                                                      int64_t ld, const float2* __restrict__ rope,
                                                      half_t* __restrict__ q16,
                                                      half_t* __restrict__ kc,
                                                      half_t* __restrict__ vc, int M, int nh, int d,
                                                      int kv_len, int64_t stride_head,
                                                      int64_t stride_tok)
{
    int half = d / 2;
    int H = nh * d;
    size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= (size_t)M * nh * half) return;
    int j = (int)(id % half);
    int h = (int)((id / half) % nh);
    int m = (int)(id / ((size_t)half * nh));
    float v[6] = {0, 0, 0, 0, 0, 0};
    for (int s = 0; s < S; ++s) {
        const float* row = part + ((size_t)s * M + m) * ld;
        v[0] += row[h * d + j];
        v[1] += row[h * d + j + half];
        v[2] += row[H + h * d + j];
        v[3] += row[H + h * d + j + half];
        v[4] += row[2 * H + h * d + j];
        v[5] += row[2 * H + h * d + j + half];
    }
    float2 cs = rope[(size_t)m * half + j];
    size_t qo = (size_t)m * H + h * d + j;
    q16[qo] = (half_t)(v[0] * cs.x - v[1] * cs.y);
    q16[qo + half] = (half_t)(v[1] * cs.x + v[0] * cs.y);
    size_t co = (size_t)h * stride_head + (size_t)(kv_len + m) * stride_tok + j;
    kc[co] = (half_t)(v[2] * cs.x - v[3] * cs.y);
    kc[co + half] = (half_t)(v[3] * cs.x + v[2] * cs.y);
    vc[co] = (half_t)v[4];
    vc[co + half] = (half_t)v[5];
}

ghd_status launch_qkv_epilogue(const float* part, int S, int64_t ld, const float2* rope, half_t* q16,
                               half_t* kc, half_t* vc, int M, int nh, int d, int kv_len,
                               int64_t stride_head, int64_t stride_tok, hipStream_t st)
{
    size_t total = (size_t)M * nh * (d / 2);
    hipLaunchKernelGGL(k_qkv_epilogue, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, part,
                       S, ld, rope, q16, kc, vc, M, nh, d, kv_len, stride_head, stride_tok);
    return check_launch();
}

// ---- SwiGLU ----------------------------------------------------------------------
// a[m,f] = silu(gate[m,f]) * up[m,f], gate = columns [0,F), up = columns [F,2F)
__global__ __launch_bounds__(256) void k_swiglu(const float* __restrict__ part, int S, int64_t ld,
                                                half_t* __restrict__ a16, int M, int F)
{
    int f = blockIdx.x * blockDim.x + threadIdx.x;
    int m = blockIdx.y;
    if (f >= F) return;
    float gt = 0.f, up = 0.f;
    for (int s = 0; s < S; ++s) {
        const float* row = part + ((size_t)s * M + m) * ld;
        gt += row[f];
        up += row[F + f];
    }
    float act = gt / (1.0f + __expf(-gt));
    a16[(size_t)m * F + f] = (half_t)(act * up);
}

ghd_status launch_swiglu(const float* part, int S, int64_t ld, half_t* a16, int M, int F,
                         hipStream_t st)
{
    hipLaunchKernelGGL(k_swiglu, dim3(ceil_div(F, 256), M), dim3(256), 0, st, part, S, ld, a16, M, F);
    return check_launch();
}

}  // namespace ghd

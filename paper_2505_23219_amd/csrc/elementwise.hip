// Element-wise kernels between the skinny GEMMs: residual add + RMSNorm, rotary
// embedding + KV append, SwiGLU.  The paper (section 2.2.2) leaves these
// operations out of its cost model; they read the fp32 output of the preceding
// linear layer ([M, N], a few MB that stay in cache) and write the fp16 operand
// of the next one, so none of them costs a pass over HBM.
#include "fused.h"

namespace ghd {

// ---- residual add + RMSNorm ----------------------------------------------------
// One workgroup of 1024 threads per row, four consecutive columns per thread and pass, so
// all loads of a row are in flight at once.  x_new = (x_old or widen(x_in16)) + y32 (the
// preceding linear layer's output, if given); then
// n16 = fp16(x_new * rsqrt(mean(x_new^2) + eps) * g).
__global__ __launch_bounds__(1024) void k_residual_norm(float* __restrict__ x,
                                                        const half_t* __restrict__ x_in16,
                                                        const float* __restrict__ part, int S,
                                                        int64_t ld, const half_t* __restrict__ g,
                                                        half_t* __restrict__ n16, int M, int H,
                                                        float eps)
{
    __shared__ float s_red[16];
    const int m = blockIdx.x, tid = threadIdx.x;
    constexpr int kMaxPass = 11;               // H <= 1024 * 4 * 11 (H % 4 == 0)
    floatx4 v[kMaxPass];
    float ss = 0.f;
#pragma unroll
    for (int p = 0; p < kMaxPass; ++p) {
        const int c = tid * 4 + p * 4096;
        if (c >= H) break;
        floatx4 t;
        if (x_in16) {
            half4 h = *(const half4*)(x_in16 + (size_t)m * H + c);
            t = (floatx4){(float)h[0], (float)h[1], (float)h[2], (float)h[3]};
        } else {
            t = *(const floatx4*)(x + (size_t)m * H + c);
        }
        for (int s = 0; s < S; ++s) t += *(const floatx4*)(part + ((size_t)s * M + m) * ld + c);
        *(floatx4*)(x + (size_t)m * H + c) = t;
        ss += t[0] * t[0] + t[1] * t[1] + t[2] * t[2] + t[3] * t[3];
        v[p] = t;
    }
    if (!g) return;
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
    if ((tid & 63) == 0) s_red[tid >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
    for (int w = 0; w < 16; ++w) tot += s_red[w];
    float r = 1.0f / sqrtf(tot / (float)H + eps);
#pragma unroll
    for (int p = 0; p < kMaxPass; ++p) {
        const int c = tid * 4 + p * 4096;
        if (c >= H) break;
        half4 gv = *(const half4*)(g + c);
        half4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (half_t)(v[p][e] * r * (float)gv[e]);
        *(half4*)(n16 + (size_t)m * H + c) = o;
    }
}

ghd_status launch_residual_norm(float* x, const half_t* x_in16, const float* part, int S, int64_t ld,
                                const half_t* g, half_t* n16, int M, int H, float eps,
                                hipStream_t st)
{
    hipLaunchKernelGGL(k_residual_norm, dim3(M), dim3(1024), 0, st, x, x_in16, part, S, ld, g, n16, M,
                       H, eps);
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
    float act = gt / (1.0f + expf(-gt));
    a16[(size_t)m * F + f] = (half_t)(act * up);
}

ghd_status launch_swiglu(const float* part, int S, int64_t ld, half_t* a16, int M, int F,
                         hipStream_t st)
{
    hipLaunchKernelGGL(k_swiglu, dim3(ceil_div(F, 256), M), dim3(256), 0, st, part, S, ld, a16, M, F);
    return check_launch();
}

}  // namespace ghd

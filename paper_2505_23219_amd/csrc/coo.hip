// The drafted tokens' own block of the attention computed from the nonzeros of the tree
// mask only - the sparse component of Ghidorah's attention split (section 3.2.2: the part
// of the scores between the drafted tokens themselves; section 3.2.3: it is computed from a
// coordinate list of the mask's nonzeros, one dot product per (token, ancestor) pair,
// instead of a dense masked product).  The paper runs it on the CPU cores of its SoC; here
// it is a GPU kernel, kept as the experiment of the paper's Figure 8b on this chip: the
// same block costs one masked MFMA tile inside the attention kernel, whatever the tree.
//
// One wavefront per (head, drafted token i).  The coordinate list of row i is the set bits
// of its 128-bit ancestor mask, walked in ascending order; a lane holds two channels, a
// score is a 64-lane reduction, and the softmax runs online over the ancestors.
#include "fused.h"

namespace ghd {

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

template <int D>
__global__ __launch_bounds__(512) void k_tree_part_coo(half_t* __restrict__ out, const half_t* __restrict__ q,
                                                      const half_t* __restrict__ kc,
                                                      const half_t* __restrict__ vc,
                                                      const uint64_t* __restrict__ mask, int M, int kv_len,
                                                      int nh, int64_t stride_head, int64_t stride_tok,
                                                      int64_t v_stride_head, int64_t v_stride_ch,
                                                      float scale_log2e)
{
    const int lane = threadIdx.x & 63;
    const int wid = blockIdx.x * 8 + (threadIdx.x >> 6);
    const int head = wid / M, i = wid - head * M;
    if (head >= nh) return;
    constexpr int HL = D / 2;                   // lanes that hold channels (two each)
    const bool on = lane < HL;
    const int ch = on ? 2 * lane : 0;
    const half2_ qh = *(const half2_*)(q + ((size_t)i * nh + head) * D + ch);
    const float q0 = on ? (float)qh[0] : 0.f, q1 = on ? (float)qh[1] : 0.f;
    const half_t* kh = kc + (size_t)head * stride_head + (size_t)kv_len * stride_tok + ch;
    const half_t* vh = vc + (size_t)head * v_stride_head + (size_t)ch * v_stride_ch + kv_len;
    // bits from M on, which a caller's mask may have set, name no token
    uint64_t lo = mask[2 * i], hi = mask[2 * i + 1];
    if (M < 64) lo &= (1ull << M) - 1;
    if (M < 128) hi &= M > 64 ? (1ull << (M - 64)) - 1 : 0ull;
    float m = -INFINITY, l = 0.f, o0 = 0.f, o1 = 0.f;
    // the coordinate list of row i, four entries at a time (loads of a batch are independent)
    while (lo | hi) {
        int js[4];
        int n = 0;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            js[u] = -1;
            if (lo) {
                js[u] = __builtin_ctzll(lo);
                lo &= lo - 1;
            } else if (hi) {
                js[u] = 64 + __builtin_ctzll(hi);
                hi &= hi - 1;
            }
            n += js[u] >= 0;
        }
        half2_ k2[4];
        half_t v0[4], v1[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int j = js[u] >= 0 ? js[u] : js[0];
            k2[u] = *(const half2_*)(kh + (size_t)j * stride_tok);
            v0[u] = vh[j];
            v1[u] = vh[v_stride_ch + j];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (u >= n) break;
            const float s = wave_sum(on ? q0 * (float)k2[u][0] + q1 * (float)k2[u][1] : 0.f) * scale_log2e;
            const float mn = fmaxf(m, s);
            const float alpha = __builtin_amdgcn_exp2f(m - mn), p = __builtin_amdgcn_exp2f(s - mn);
            l = l * alpha + p;
            o0 = o0 * alpha + p * (float)v0[u];
            o1 = o1 * alpha + p * (float)v1[u];
            m = mn;
        }
    }
    if (on) {
        const float r = l > 0.f ? 1.f / l : 0.f;
        half2_ o = {(half_t)(o0 * r), (half_t)(o1 * r)};
        *(half2_*)(out + ((size_t)i * nh + head) * D + ch) = o;
    }
}

ghd_status launch_tree_part_coo(void* out, const void* q, const void* kc, const void* vc, const uint64_t* mask,
                                int M, int kv_len, int nh, int d, int64_t stride_head, int64_t stride_tok,
                                int64_t v_stride_head, int64_t v_stride_ch, float scale, hipStream_t st)
{
    const int waves = nh * M, blocks = (waves + 7) / 8;
    const float sl = scale * 1.4426950408889634f;
    if (d == 64)
        hipLaunchKernelGGL(k_tree_part_coo<64>, dim3(blocks), dim3(512), 0, st, (half_t*)out, (const half_t*)q,
                           (const half_t*)kc, (const half_t*)vc, mask, M, kv_len, nh, stride_head, stride_tok,
                           v_stride_head, v_stride_ch, sl);
    else
        hipLaunchKernelGGL(k_tree_part_coo<128>, dim3(blocks), dim3(512), 0, st, (half_t*)out, (const half_t*)q,
                           (const half_t*)kc, (const half_t*)vc, mask, M, kv_len, nh, stride_head, stride_tok,
                           v_stride_head, v_stride_ch, sl);
    return check_launch();
}

}  // namespace ghd

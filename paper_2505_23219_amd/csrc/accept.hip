// Greedy acceptance: after the verification pass the step "falls back to the
// longest validated prefix" (Ghidorah, section 2.3).  Two launches:
//   k_row_argmax : amax[i] = lowest index of the largest logit of row i,
//                  a wavefront-level (value, index) reduction per row;
//   k_accept     : a node is valid iff every edge (p -> c) on its root path has
//                  tokens[c] == amax[p]; the deepest valid node (lowest index on
//                  ties) wins and its root path is written out.
#include "common.h"

namespace ghd {

__device__ inline void argmax_merge(float& v, int& i, float ov, int oi)
{
    if (ov > v || (ov == v && oi < i)) {
        v = ov;
        i = oi;
    }
}

__global__ __launch_bounds__(256) void k_row_argmax(const float* __restrict__ logits, int V,
                                                    int32_t* __restrict__ amax)
{
    __shared__ float s_v[4];
    __shared__ int s_i[4];
    const float* row = logits + (size_t)blockIdx.x * V;
    int tid = threadIdx.x;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int idx = tid; idx < V; idx += 256) argmax_merge(bv, bi, row[idx], idx);
    for (int off = 32; off > 0; off >>= 1) {
        float ov = __shfl_xor(bv, off);
        int oi = __shfl_xor(bi, off);
        argmax_merge(bv, bi, ov, oi);
    }
    if ((tid & 63) == 0) {
        s_v[tid >> 6] = bv;
        s_i[tid >> 6] = bi;
    }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 4; ++w) argmax_merge(bv, bi, s_v[w], s_i[w]);
        amax[blockIdx.x] = bi;
    }
}

__global__ __launch_bounds__(128) void k_accept(const int32_t* __restrict__ amax,
                                                const int32_t* __restrict__ tokens,
                                                const int32_t* __restrict__ parent, int M,
                                                int32_t* __restrict__ res,
                                                int32_t* __restrict__ amax_out)
{
    __shared__ int32_t s_par[GHD_MAX_M], s_tok[GHD_MAX_M], s_amax[GHD_MAX_M];
    __shared__ int s_key[2];
    int i = threadIdx.x;
    if (i < M) {
        s_par[i] = parent[i];
        s_tok[i] = tokens[i];
        s_amax[i] = amax[i];
        if (amax_out) amax_out[i] = s_amax[i];
    }
    __syncthreads();
    // key orders candidates by depth first, then by lower node index
    int key = -1;
    if (i < M) {
        bool ok = true;
        int depth = 0, j = i;
        for (int step = 0; step < M; ++step) {
            int p = s_par[j];
            if (p < 0 || p >= j) break;
            ok = ok && (s_tok[j] == s_amax[p]);
            j = p;
            ++depth;
        }
        if (ok) key = depth * 256 + (255 - i);
    }
    for (int off = 32; off > 0; off >>= 1) key = max(key, __shfl_xor(key, off));
    if ((i & 63) == 0) s_key[i >> 6] = key;
    __syncthreads();
    if (i == 0) {
        int best = max(s_key[0], s_key[1]);
        int depth = best >> 8, node = 255 - (best & 255);
        res[0] = depth + 1;
        res[1] = s_amax[node];
        for (int pos = depth, j = node; pos >= 0 && j >= 0; --pos, j = s_par[j]) res[2 + pos] = j;
    }
}

ghd_status launch_accept(const float* logits, const int32_t* tokens, const int32_t* parent, int M,
                         int V, int32_t* res, int32_t* amax_out, int32_t* amax_ws, hipStream_t st)
{
    hipLaunchKernelGGL(k_row_argmax, dim3(M), dim3(256), 0, st, logits, V, amax_ws);
    hipLaunchKernelGGL(k_accept, dim3(1), dim3(128), 0, st, (const int32_t*)amax_ws, tokens, parent,
                       M, res, amax_out);
    return check_launch();
}

}  // namespace ghd

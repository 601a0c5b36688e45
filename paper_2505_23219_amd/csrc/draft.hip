// The drafting side of a decoding step (Ghidorah, section 2.1: tokens for several future
// slots are predicted, then verified in one pass; section 2.3: with self-drafting the
// predictions come from extra heads at the tail of the model, several candidates per head;
// section 3.3.1: the candidates are combined into the verification tree).
//   k_embed       : hidden states of the tree's tokens, rows of the embedding table;
//   k_pick_norm   : the final hidden state of the last accepted node, RMS-normalised with
//                   the final gain, as the fp16 input row of the heads' linear layer (the
//                   K heads are one stacked [K*V, H] matrix: one skinny linear launch);
//   k_topk        : the R best candidates of every head, best first, lowest index on ties;
//   k_tree_tokens : tokens of the next tree: the root carries the token the model has just
//                   produced, a node at depth t candidate rank[i] of head t - 1.
// Also the host-side tree design from head accuracies (section 3.3.1).
#include "common.h"

#include <queue>
#include <vector>

namespace ghd {

__global__ __launch_bounds__(256) void k_embed(half8* __restrict__ x, const half8* __restrict__ table,
                                               const int32_t* __restrict__ tokens, int H8, int V)
{
    const int i = blockIdx.x;
    int t = tokens[i];
    t = t < 0 ? 0 : (t >= V ? V - 1 : t);     // a corrupt token cannot reach outside the table
    for (int j = threadIdx.x; j < H8; j += 256) x[(size_t)i * H8 + j] = table[(size_t)t * H8 + j];
}

constexpr int kPickThreads = 1024;

__global__ __launch_bounds__(kPickThreads) void k_pick_norm(const float* __restrict__ x_final,
                                                            const int32_t* __restrict__ res, int M, int H,
                                                            const half_t* __restrict__ g, float eps,
                                                            half_t* __restrict__ n16)
{
    __shared__ float s_part[kPickThreads / 64];
    __shared__ float s_rinv;
    const int tid = threadIdx.x;
    int len = res[0];
    len = len < 1 ? 1 : (len > M ? M : len);
    int last = res[2 + len - 1];
    last = last < 0 ? 0 : (last >= M ? M - 1 : last);
    const float* row = x_final + (size_t)last * H;
    float s = 0.f;
    for (int j = tid; j < H; j += kPickThreads) s += row[j] * row[j];
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
    if ((tid & 63) == 0) s_part[tid >> 6] = s;
    __syncthreads();
    if (tid == 0) {
        float tot = 0.f;
        for (int w = 0; w < kPickThreads / 64; ++w) tot += s_part[w];
        s_rinv = 1.0f / sqrtf(tot / (float)H + eps);
    }
    __syncthreads();
    const float rinv = s_rinv;
    for (int j = tid; j < H; j += kPickThreads) n16[j] = (half_t)(row[j] * rinv * (float)g[j]);
}

// order of candidates: larger value first, lower index first among equal values
__device__ inline bool cand_before(float v, int i, float ov, int oi) { return v > ov || (v == ov && i < oi); }

constexpr int kTopkThreads = 1024;

__global__ __launch_bounds__(kTopkThreads) void k_topk(const float* __restrict__ logits, int V, int R,
                                                       int32_t* __restrict__ topk)
{
    __shared__ float s_v[kTopkThreads / 64];
    __shared__ int s_i[kTopkThreads / 64];
    __shared__ float s_pv;
    __shared__ int s_pi;
    const float* row = logits + (size_t)blockIdx.x * V;
    const int tid = threadIdx.x;
    float pv = INFINITY;      // the previous pick; every entry comes after (+inf, -1)
    int pi = -1;
    for (int r = 0; r < R; ++r) {
        float bv = -INFINITY;
        int bi = 0x7fffffff;
        for (int idx = tid; idx < V; idx += kTopkThreads) {
            float v = row[idx];
            // still to be picked: strictly after the previous pick in the order
            if (cand_before(pv, pi, v, idx) && cand_before(v, idx, bv, bi)) {
                bv = v;
                bi = idx;
            }
        }
        for (int off = 32; off > 0; off >>= 1) {
            float ov = __shfl_xor(bv, off);
            int oi = __shfl_xor(bi, off);
            if (cand_before(ov, oi, bv, bi)) {
                bv = ov;
                bi = oi;
            }
        }
        if ((tid & 63) == 0) {
            s_v[tid >> 6] = bv;
            s_i[tid >> 6] = bi;
        }
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < kTopkThreads / 64; ++w)
                if (cand_before(s_v[w], s_i[w], bv, bi)) {
                    bv = s_v[w];
                    bi = s_i[w];
                }
            // fewer than R entries that compare (V < R, or NaNs): repeat the last index
            topk[(size_t)blockIdx.x * R + r] = bi == 0x7fffffff ? (pi < 0 ? 0 : pi) : bi;
            s_pv = bv;
            s_pi = bi;
        }
        __syncthreads();
        pv = s_pv;
        pi = s_pi;
        __syncthreads();
    }
}

__global__ __launch_bounds__(GHD_MAX_M) void k_tree_tokens(int32_t* __restrict__ tokens,
                                                           const int32_t* __restrict__ parent,
                                                           const int32_t* __restrict__ rank, int M,
                                                           const int32_t* __restrict__ topk, int K, int R,
                                                           const int32_t* __restrict__ res, int V)
{
    __shared__ int32_t s_parent[GHD_MAX_M];
    const int i = threadIdx.x;
    if (i < M) s_parent[i] = parent[i];
    __syncthreads();
    if (i >= M) return;
    int t;
    if (i == 0) {
        t = res[1];
    } else {
        int dep = 0;
        for (int j = i, step = 0; step < M; ++step) {
            int p = s_parent[j];
            if (p < 0 || p >= j) break;
            j = p;
            ++dep;
        }
        // clamped: a tree deeper than the heads or a rank past R cannot read outside topk
        int head = dep < 1 ? 0 : (dep > K ? K - 1 : dep - 1);
        int r = rank[i];
        r = r < 0 ? 0 : (r >= R ? R - 1 : r);
        t = topk[head * R + r];
    }
    tokens[i] = t < 0 ? 0 : (t >= V ? V - 1 : t);
}

ghd_status launch_embed(void* x16, const void* table16, const int32_t* tokens, int M, int H, int V,
                        hipStream_t st)
{
    hipLaunchKernelGGL(k_embed, dim3(M), dim3(256), 0, st, (half8*)x16, (const half8*)table16, tokens,
                       H / 8, V);
    return check_launch();
}

ghd_status launch_pick_norm(const float* x_final, const int32_t* res, int M, int H, const void* g,
                            float eps, void* n16, hipStream_t st)
{
    hipLaunchKernelGGL(k_pick_norm, dim3(1), dim3(kPickThreads), 0, st, x_final, res, M, H,
                       (const half_t*)g, eps, (half_t*)n16);
    return check_launch();
}

ghd_status launch_topk(const float* logits, int rows, int V, int R, int32_t* topk, hipStream_t st)
{
    hipLaunchKernelGGL(k_topk, dim3(rows), dim3(kTopkThreads), 0, st, logits, V, R, topk);
    return check_launch();
}

ghd_status launch_tree_tokens(int32_t* tokens, const int32_t* parent, const int32_t* rank, int M,
                              const int32_t* topk, int K, int R, const int32_t* res, int V,
                              hipStream_t st)
{
    hipLaunchKernelGGL(k_tree_tokens, dim3(1), dim3(GHD_MAX_M), 0, st, tokens, parent, rank, M, topk, K,
                       R, res, V);
    return check_launch();
}

// ---- tree design (host) -------------------------------------------------------
// The expected acceptance length of a tree is 1 + the sum over its nodes of the product of
// the accuracies along the node's path (section 3.3.1); since accuracies are at most 1 a
// node never scores above its parent, so taking the best-scoring open candidate M - 1 times
// gives the best tree of M nodes.  Open candidates sit in a heap ordered by (score, lower
// parent, lower rank); a node's R children are opened when it is inserted.
int tree_build_host(const double* acc, int K, int R, int M, int32_t* parent, int32_t* rank,
                    double* expect)
{
    struct Cand {
        double score;
        int parent, rank;
    };
    auto worse = [](const Cand& a, const Cand& b) {
        if (a.score != b.score) return a.score < b.score;
        if (a.parent != b.parent) return a.parent > b.parent;
        return a.rank > b.rank;
    };
    std::priority_queue<Cand, std::vector<Cand>, decltype(worse)> open(worse);
    std::vector<double> score(M);
    std::vector<int> depth(M);
    parent[0] = -1;
    rank[0] = 0;
    score[0] = 1.0;
    depth[0] = 0;
    double e = 1.0;
    int n = 1;
    auto open_children = [&](int u) {
        if (depth[u] >= K) return;
        for (int r = 0; r < R; ++r) open.push({score[u] * acc[(size_t)depth[u] * R + r], u, r});
    };
    open_children(0);
    while (n < M && !open.empty()) {
        Cand c = open.top();
        open.pop();
        parent[n] = c.parent;
        rank[n] = c.rank;
        score[n] = c.score;
        depth[n] = depth[c.parent] + 1;
        e += c.score;
        open_children(n);
        ++n;
    }
    if (expect) *expect = e;
    return n;
}

}  // namespace ghd

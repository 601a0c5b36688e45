// Greedy acceptance: after the verification pass the longest root path that the model
// itself would have produced is kept (Ghidorah, section 2.3).  Two launches:
//   k_row_argmax : every row of the logits is cut into kArgSeg segments; a workgroup
//                  finds the (largest value, lowest index) of one segment with a
//                  wavefront-level reduction;
//   k_accept     : merges the segments into amax[i] (lowest index on ties); a node is
//                  valid iff every edge (p -> c) on its root path has
//                  tokens[c] == amax[p]; the deepest valid node (lowest index on
//                  ties) wins and its root path is written out.
#include "common.h"

#include <mutex>

namespace ghd {

constexpr int kCommitMaxLayers = 48;

__device__ inline void argmax_merge(float& v, int& i, float ov, int oi)
{
    if (ov > v || (ov == v && oi < i)) {
        v = ov;
        i = oi;
    }
}

constexpr int kArgSeg = 8;   // segments per row

__global__ __launch_bounds__(256) void k_row_argmax(const float* __restrict__ logits, int V,
                                                    float* __restrict__ seg_v,
                                                    int32_t* __restrict__ seg_i)
{
    __shared__ float s_v[4];
    __shared__ int s_i[4];
    const int rowi = blockIdx.x / kArgSeg, seg = blockIdx.x % kArgSeg;
    const float* row = logits + (size_t)rowi * V;
    const int lo = (int)((long)V * seg / kArgSeg), hi = (int)((long)V * (seg + 1) / kArgSeg);
    int tid = threadIdx.x;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    // four independent loads in flight per thread
    for (int idx = lo + tid; idx < hi; idx += 1024) {
        float v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = (idx + 256 * u < hi) ? row[idx + 256 * u] : -INFINITY;
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (idx + 256 * u < hi) argmax_merge(bv, bi, v[u], idx + 256 * u);
    }
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
        seg_v[rowi * kArgSeg + seg] = bv;
        seg_i[rowi * kArgSeg + seg] = bi;
    }
}

// Row argmax from the per-tile candidates the LM-head finish leaves: one workgroup per row
// merges `ntiles` (value, column) pairs, lowest column on ties.
__global__ __launch_bounds__(256) void k_amax_merge(const float2* __restrict__ tbl, int ntiles, int Mpad,
                                                    int32_t* __restrict__ amax)
{
    __shared__ float s_v[4];
    __shared__ int s_i[4];
    const int row = blockIdx.x, tid = threadIdx.x;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int t0 = tid; t0 < ntiles; t0 += 1024) {
        float2 c[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) c[u] = tbl[(size_t)min(t0 + 256 * u, ntiles - 1) * Mpad + row];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (t0 + 256 * u < ntiles) argmax_merge(bv, bi, c[u].x, __float_as_int(c[u].y));
    }
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
        amax[row] = bi;
    }
}

// amax_in != nullptr: the row argmaxes are given (seg_v, seg_i unused)
__global__ __launch_bounds__(128) void k_accept(const float* __restrict__ seg_v,
                                                const int32_t* __restrict__ seg_i,
                                                const int32_t* __restrict__ amax_in,
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
        float bv = -INFINITY;
        int bi = 0x7fffffff;
        if (amax_in) bi = amax_in[i];
        else
            for (int sg = 0; sg < kArgSeg; ++sg) argmax_merge(bv, bi, seg_v[i * kArgSeg + sg], seg_i[i * kArgSeg + sg]);
        s_amax[i] = bi;
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

// ---- commit of the accepted path ---------------------------------------------
// One workgroup per (layer, head).  The K rows (and the V columns: V is channel-major) of
// the accepted nodes are gathered into LDS, and only after a barrier written to rows
// kv_len + j, so no source can have been overwritten before it is read.  The path comes
// from the device result of the acceptance kernel; its entries are clamped, so that
// whatever that buffer holds no access leaves the tree rows.
struct CommitArgs {
    half_t* k[kCommitMaxLayers];
    half_t* v[kCommitMaxLayers];
    const int32_t* res;
    int nh, d, cap, kv_len, M;
};

__global__ __launch_bounds__(256) void k_commit_path(const CommitArgs a)
{
    __shared__ __attribute__((aligned(16))) half_t s_rows[GHD_MAX_M * 128];
    __shared__ int32_t s_path[GHD_MAX_M];
    const int tid = threadIdx.x, layer = blockIdx.x / a.nh, head = blockIdx.x % a.nh;
    const int d = a.d, len = min(max(a.res[0], 0), a.M);
    for (int j = tid; j < len; j += 256) s_path[j] = min(max(a.res[2 + j], 0), a.M - 1);
    __syncthreads();
    half_t* kh = a.k[layer] + (size_t)head * a.cap * d;
    const int cpr = d / 8;
    for (int idx = tid; idx < len * cpr; idx += 256) {
        int j = idx / cpr, c = idx % cpr;
        *(half8*)(s_rows + idx * 8) = *(const half8*)(kh + (size_t)(a.kv_len + s_path[j]) * d + c * 8);
    }
    __syncthreads();
    for (int idx = tid; idx < len * cpr; idx += 256) {
        int j = idx / cpr, c = idx % cpr;
        *(half8*)(kh + (size_t)(a.kv_len + j) * d + c * 8) = *(const half8*)(s_rows + idx * 8);
    }
    __syncthreads();
    half_t* vh = a.v[layer] + (size_t)head * d * a.cap + a.kv_len;
    for (int idx = tid; idx < d * len; idx += 256) {
        int ch = idx / len, j = idx % len;
        s_rows[idx] = vh[(size_t)ch * a.cap + s_path[j]];
    }
    __syncthreads();
    for (int idx = tid; idx < d * len; idx += 256) {
        int ch = idx / len, j = idx % len;
        vh[(size_t)ch * a.cap + j] = s_rows[idx];
    }
}

ghd_status launch_commit_path(void* const* k, void* const* v, int L, int nh, int d, int cap,
                              int kv_len, int M, const int32_t* res, hipStream_t st)
{
    CommitArgs a;
    for (int l = 0; l < L; ++l) {
        a.k[l] = (half_t*)k[l];
        a.v[l] = (half_t*)v[l];
    }
    a.res = res;
    a.nh = nh;
    a.d = d;
    a.cap = cap;
    a.kv_len = kv_len;
    a.M = M;
    hipLaunchKernelGGL(k_commit_path, dim3(L * nh), dim3(256), 0, st, a);
    return check_launch();
}

size_t accept_workspace_bytes() { return (size_t)GHD_MAX_M * kArgSeg * 8; }

// ---- acceptance without a caller's workspace ------------------------------------
// The per-segment maxima of ghd_accept_greedy_static live in this array instead of a
// workspace: GHD_MAX_M rows x kArgSeg segments x (value, index) = 8 KiB, one copy per GPU
// the library runs on, held until the process ends.  The name is a host-side stand-in; the
// device address is looked up once per device and only that pointer is handed to kernels.
constexpr size_t kStaticScratchBytes = (size_t)GHD_MAX_M * kArgSeg * 8;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kScratchDevices = 64;
static void* g_scratch_ptr[kScratchDevices] = {};
static std::mutex g_scratch_mu;

// device address of `scratch` on the current device (looked up on first use)
static ghd_status static_scratch(void** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kScratchDevices) return hip_fail(hipErrorInvalidDevice);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e);
        if (!p) return hip_fail(hipErrorInvalidSymbol);
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return GHD_OK;
}

ghd_status launch_accept_static(const float* logits, const int32_t* tokens, const int32_t* parent, int M,
                                int V, int32_t* res, int32_t* amax_out, hipStream_t st)
{
    if ((size_t)M * kArgSeg * 8 > kStaticScratchBytes) return GHD_ERR_SHAPE;
    void* ws = nullptr;
    ghd_status s = static_scratch(&ws);
    if (s) return s;
    // every entry the second kernel reads (rows < M) is written by the first: nothing to clear
    return launch_accept(logits, tokens, parent, M, V, res, amax_out, ws, st);
}

ghd_status launch_accept(const float* logits, const int32_t* tokens, const int32_t* parent, int M,
                         int V, int32_t* res, int32_t* amax_out, void* ws, hipStream_t st)
{
    // workspace: per-segment maxima [GHD_MAX_M][kArgSeg] float, then their indices
    float* seg_v = (float*)ws;
    int32_t* seg_i = (int32_t*)(seg_v + GHD_MAX_M * kArgSeg);
    hipLaunchKernelGGL(k_row_argmax, dim3(M * kArgSeg), dim3(256), 0, st, logits, V, seg_v, seg_i);
    hipLaunchKernelGGL(k_accept, dim3(1), dim3(128), 0, st, (const float*)seg_v,
                       (const int32_t*)seg_i, (const int32_t*)nullptr, tokens, parent, M, res, amax_out);
    return check_launch();
}

ghd_status launch_amax_merge(const void* tbl, int ntiles, int Mpad, int M, int32_t* amax, hipStream_t st)
{
    hipLaunchKernelGGL(k_amax_merge, dim3(M), dim3(256), 0, st, (const float2*)tbl, ntiles, Mpad, amax);
    return check_launch();
}

ghd_status launch_accept_path(const int32_t* amax, const int32_t* tokens, const int32_t* parent, int M,
                              int32_t* res, hipStream_t st)
{
    hipLaunchKernelGGL(k_accept, dim3(1), dim3(128), 0, st, (const float*)nullptr, (const int32_t*)nullptr,
                       amax, tokens, parent, M, res, (int32_t*)nullptr);
    return check_launch();
}

}  // namespace ghd

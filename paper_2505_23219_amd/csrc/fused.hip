// The attention kernel (see attention_impl.h), the set-up kernel and the dispatch of the
// persistent kernels.
#include "attention_impl.h"

namespace ghd {


template <int MT, int D>
__global__ __launch_bounds__(kFT) void k_attention(const FusedArgs a)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    touch_kernel_arguments();
    Ctx cx = make_ctx(a, lds);
    attn_phase<MT, D>(a, cx, a.att_q, a.att_k, a.att_v, a.att_out, a.att_epoch);
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
template <int MT, int D>
static ghd_status launch_attention_t(const FusedArgs& a, hipStream_t st)
{
    int G = 0;
    const size_t lds = sizeof(AttnLds<MT, D>);
    ghd_status s = launch_resident_checked((const void*)k_attention<MT, D>, 0, lds, &G);
    if (s) return s;
    hipLaunchKernelGGL((k_attention<MT, D>), dim3(G), dim3(kFT), lds, st, a);
    return check_launch();
}

template <int D>
static ghd_status launch_attention_d(const FusedArgs& a, int mt, hipStream_t st)
{
    if (mt <= 1) return launch_attention_t<1, D>(a, st);
    if (mt <= 2) return launch_attention_t<2, D>(a, st);
    if (mt <= 4) return launch_attention_t<4, D>(a, st);
    return launch_attention_t<8, D>(a, st);
}

// a.mode selects the kernel; the row-tile count of M selects the instantiation
ghd_status launch_fused(const FusedArgs& a, hipStream_t st)
{
    const int mt = (a.M + 15) / 16;
    if (a.mode == MODE_LINEAR) return launch_linear(a, st);
    if (a.mode == MODE_QKV_ATTN) return launch_qkv_attn(a, st);
    return a.d == 64 ? launch_attention_d<64>(a, mt, st) : launch_attention_d<128>(a, mt, st);
}

// The attention's work shares on the host: for workgroup j and head `head`,
// out[0..5] = first part, number of parts, this part's index, t0, t1, and whether `head` is
// one of j's heads at all (otherwise the first five are -1).
void attn_share_on_host(int nh, int ntile, int j, int G, int head, int* out)
{
    const AttnHeads hs = attn_heads(nh, j, G);
    for (int i = 0; i < 6; ++i) out[i] = -1;
    out[5] = 0;
    const int hl = head - hs.hx0;
    if (hl < hs.h_lo || hl >= hs.h_hi) return;
    const AttnTiles ts = attn_tiles(hs, hl, ntile);
    out[0] = ts.first;
    out[1] = ts.np;
    out[2] = ts.me;
    out[3] = ts.t0;
    out[4] = ts.t1;
    out[5] = 1;
}

// ---- setup kernel ------------------------------------------------------------
// Blocks 0..kTreeBlocks-1: tree tables (every block walks the parents itself; block 0
// writes the ancestor masks, each block a slice of the rotary table).  The next kZeroBlocks
// blocks zero the sync block.  Further blocks: one per 16-column tile of the residual stream,
// writing x = widen(x_in), the tile's sums of squares and the gain-scaled fp16 image.
constexpr int kTreeBlocks = 8;
constexpr int kZeroBlocks = 128;

__global__ __launch_bounds__(256) void k_fused_setup(uint32_t* __restrict__ sync,
                                                     const int32_t* __restrict__ parent, int M,
                                                     int Mpad, int kv_len, int d, float rope_base,
                                                     uint64_t* __restrict__ mask,
                                                     float2* __restrict__ rope, float* __restrict__ x,
                                                     const half_t* __restrict__ x_in16, int H,
                                                     float* __restrict__ ss,
                                                     const half_t* __restrict__ gain,
                                                     half_t* __restrict__ xg16)
{
    int tid = threadIdx.x;
    if (blockIdx.x < kTreeBlocks) {
        // Ancestor sets and depths by pointer doubling: after round k a node knows its 2^k
        // nearest ancestors-or-self, how many edges lead to the farthest of them, and the
        // node 2^k edges up (-1 past the root).  ceil(log2 M) rounds whatever the depth; a
        // parent that is not an earlier node is taken as "no parent".
        __shared__ int32_t s_up[GHD_MAX_M];
        __shared__ int32_t s_depth[GHD_MAX_M];
        __shared__ uint64_t s_lo[GHD_MAX_M], s_hi[GHD_MAX_M];
        if (!parent) return;
        int up = -1, dep = 0;
        uint64_t lo = 0, hi = 0;
        if (tid < M) {
            up = parent[tid];
            if (up < 0 || up >= tid) up = -1;
            dep = up >= 0 ? 1 : 0;
            if (tid < 64) lo = 1ull << tid; else hi = 1ull << (tid - 64);
        }
        for (int span = 1; span < M; span <<= 1) {
            if (tid < M) {
                s_up[tid] = up;
                s_depth[tid] = dep;
                s_lo[tid] = lo;
                s_hi[tid] = hi;
            }
            __syncthreads();
            if (tid < M && up >= 0) {
                lo |= s_lo[up];
                hi |= s_hi[up];
                dep += s_depth[up];
                up = s_up[up];
            }
            __syncthreads();
        }
        if (tid < M) {
            s_depth[tid] = dep;
            if (blockIdx.x == 0) {
                mask[2 * tid] = lo;
                mask[2 * tid + 1] = hi;
            }
        }
        __syncthreads();
        if (rope) {
            // angle = position * base^(-2j/d), evaluated in double
            const int half = d / 2;
            const double c = -2.0 / d * log2((double)rope_base);
            for (int e = blockIdx.x * 256 + tid; e < M * half; e += kTreeBlocks * 256) {
                int m = e / half, j = e % half;
                double ang = (double)(kv_len + s_depth[m]) * exp2(c * j);
                rope[e] = make_float2((float)cos(ang), (float)sin(ang));
            }
        }
        return;
    }
    if (blockIdx.x < kTreeBlocks + kZeroBlocks) {
        // the status word is cleared for the calls that follow; what it held is kept in the
        // sticky word (first failure wins), so that a caller who reads the status only now
        // and then still learns of a call that gave up.  A workspace seen for the first time
        // (no magic word) holds nothing meaningful.
        if (blockIdx.x == kTreeBlocks && tid == 0) {
            const uint32_t st = sync[kSyncStatus], sticky = sync[kSyncSticky];
            const bool known = sync[kSyncMagic] == kSyncMagicValue;
            sync[kSyncSticky] = known ? (sticky ? sticky : st) : 0u;
            sync[kSyncMagic] = kSyncMagicValue;
            sync[kSyncStatus] = 0;
        }
        for (int i = (blockIdx.x - kTreeBlocks) * 256 + tid; i < kSyncWords; i += kZeroBlocks * 256)
            if (i < kSyncStatus || i > kSyncMagic) sync[i] = 0;
        return;
    }
    // residual stream tiles: thread -> (row m, column within the 16-wide tile)
    int tile = blockIdx.x - kTreeBlocks - kZeroBlocks;
    for (int e = tid; e < Mpad * 16; e += 256) {
        int m = e >> 4, col = tile * 16 + (e & 15);
        float v = 0.f;
        if (m < M) {
            v = x_in16 ? (float)x_in16[(size_t)m * H + col] : x[(size_t)m * H + col];
            if (x_in16) x[(size_t)m * H + col] = v;
            if (xg16) xg16[xpk_index(m, col, Mpad >> 4)] = (half_t)(v * (float)gain[col] * kXgScale);
        }
        float s = v * v;
        s += __shfl_xor(s, 1);
        s += __shfl_xor(s, 2);
        s += __shfl_xor(s, 4);
        s += __shfl_xor(s, 8);
        if ((e & 15) == 0) ss[(size_t)tile * Mpad + m] = s;
    }
}

ghd_status launch_fused_setup(uint32_t* sync, const int32_t* parent, int M, int Mpad, int kv_len, int d,
                              float rope_base, uint64_t* mask, float2* rope, float* x,
                              const half_t* x_in16, int H, float* ss, const half_t* gain,
                              half_t* xg16, hipStream_t st)
{
    int blocks = kTreeBlocks + kZeroBlocks + (ss ? H / 16 : 0);
    hipLaunchKernelGGL(k_fused_setup, dim3(blocks), dim3(256), 0, st, sync, parent, M, Mpad, kv_len, d,
                       rope_base, mask, rope, x, x_in16, H, ss, gain, xg16);
    return check_launch();
}

}  // namespace ghd

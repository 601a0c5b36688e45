// Argument block, layouts and launchers of the persistent kernels (linear.hip, fused.hip).
#pragma once
#include "common.h"

namespace ghd {

constexpr int kFT = 512;        // threads per workgroup (8 wavefronts)
constexpr int kMaxLayers = 48;  // the counter epochs (one per layer) are laid out for this many
constexpr int kRangeWgs = 256;  // workgroups whose work shares fit the argument block

enum { EPI_STORE_F32 = 0, EPI_STORE_F16 = 1, EPI_RESID = 2, EPI_SWIGLU = 3, EPI_QKV = 4 };
enum { MODE_LINEAR = 0, MODE_ATTN = 1, MODE_QKV_ATTN = 2 };
enum { PACK_PLAIN = 0, PACK_QKV = 1, PACK_GATE_UP = 2 };

// ---- packed weight layout ------------------------------------------------------
// The unit is the 1 KiB A operand of v_mfma_f32_16x16x32_f16: 16 output features (a
// "tile") by 32 input features (a "k-step"), 16 bytes per lane in lane order.  Tiles are
// stored in blocks of `blk` tiles, k-step major inside a block: the tiles a wavefront
// streams together at one k-step lie side by side.  Wide matrices (many tiles per compute
// unit) are stored in blocks of 8 tiles and always dealt out in whole tiles - a workgroup
// streams several consecutive tiles over the whole K range.  Narrow ones are stored in
// blocks of rb = 4 tiles, which are also the items of their other cut: a workgroup streams a
// k range of one block, so that the x operand it reads is shared by 64 output features
// (see plan_linear for which cut a launch takes).
constexpr int kRbNarrow = 4;
constexpr int kWideBlock = 8;
constexpr int kWideTiles = 640;   // from this many tiles on a matrix is wide

struct WLayout {
    int rb;        // 1: wide matrix; 4: narrow one (tiles per row block of the k-range cut)
    int blk;       // tiles per storage block
    int ntiles;    // 16-row tiles (last one zero padded)
    int nitems;    // row blocks (last one padded with zero tiles)
    int nblocks;   // storage blocks (last one padded with zero tiles)
    int nks;       // 32-column k-steps (last one zero padded)
};

__host__ __device__ inline WLayout w_layout(int N, int K)
{
    WLayout l;
    l.ntiles = (N + 15) / 16;
    l.rb = l.ntiles >= kWideTiles ? 1 : kRbNarrow;
    l.blk = l.rb == 1 ? kWideBlock : kRbNarrow;
    l.nitems = (l.ntiles + l.rb - 1) / l.rb;
    l.nblocks = (l.ntiles + l.blk - 1) / l.blk;
    l.nks = (K + 31) / 32;
    return l;
}

// index, in 16-byte pieces, of lane `lane` of the block (tile t, k-step s)
__host__ __device__ inline size_t w_piece(const WLayout& l, int t, int s, int lane)
{
    return ((((size_t)(t / l.blk) * l.nks + s) * l.blk + (t % l.blk)) << 6) + lane;
}
__host__ __device__ inline size_t w_pieces(const WLayout& l) { return ((size_t)l.nblocks * l.blk * l.nks) << 6; }

// ---- row order of the packed QKV matrix ------------------------------------------------
// Packed rows come in quads (j, j+1, j+d/2, j+1+d/2) of one head's channels, so that both
// members of two rotary pairs sit in one lane of the GEMM output.  With a head count that
// is a multiple of 8, the rows are grouped by XCD first: XCD x gets the q rows, then the k
// rows, then the v rows of its nh/8 heads, which are exactly the heads whose attention its
// workgroups run - the QKV layer and the attention can then share a launch, with nothing
// crossing an XCD in between.  Otherwise the order is q rows, k rows, v rows of all heads.
struct QkvRow {
    int part;    // 0 q, 1 k, 2 v
    int head;
    int ph;      // position inside the head's packed rows
};

__host__ __device__ inline bool qkv_grouped(int nh) { return nh % 8 == 0; }

__host__ __device__ inline QkvRow qkv_row(int p, int nh, int d)
{
    QkvRow r;
    const int H = nh * d;
    if (qkv_grouped(nh)) {
        const int hpx = nh / 8, rx = 3 * hpx * d;
        const int x = p / rx, q = p - x * rx;
        r.part = q / (hpx * d);
        const int hn = q - r.part * (hpx * d);
        r.head = x * hpx + hn / d;
        r.ph = hn % d;
    } else {
        r.part = p / H;
        const int hn = p - r.part * H;
        r.head = hn / d;
        r.ph = hn % d;
    }
    return r;
}

// channel of packed position ph inside a head
__host__ __device__ inline int qkv_channel(int ph, int d)
{
    const int r = ph & 3;
    return (ph >> 2) * 2 + (r & 1) + ((r >= 2) ? d / 2 : 0);
}

// ---- packed activation layout ----------------------------------------------------
// Activations that feed a linear layer are kept as MFMA B operands: per k-step (32
// columns) and row tile (16 rows) one 1 KiB block in lane order; lane (row % 16) +
// 16 * ((col % 32) / 8) holds 8 consecutive columns of one row.  mtp = row tiles (Mpad/16).
__host__ __device__ inline size_t xpk_index(int m, int k, int mtp)
{
    return ((((size_t)(k >> 5) * mtp + (m >> 4)) << 6) + (((k & 31) >> 3) << 4) + (m & 15)) * 8 + (k & 7);
}
__host__ __device__ inline size_t xpk_halves(int K, int mtp) { return (size_t)((K + 31) / 32) * mtp * 512; }

// The sync block (uint32 words), zeroed by the set-up kernel.  Every counter has a
// 128-byte line of its own (kCntStride words apart): the workgroups of one item poll and
// bump it without disturbing the others.  A linear layer's shared row block is counted on
// the line of the first work share that has a part of it (one line per share is enough);
// each kind of linear layer has an array of its own, reused layer after layer by epoch.
constexpr int kSyncStatus = 1;    // 0 = ok, else the code of the wait that gave up (this set-up's calls)
constexpr int kSyncSticky = 2;    // the first non-zero status an earlier set-up found in kSyncStatus
constexpr int kSyncMagic = 3;     // kSyncMagicValue once a set-up kernel has run on this workspace
constexpr uint32_t kSyncMagicValue = 0x67686453u;
constexpr int kCntStride = 32;
constexpr int kMaxShares = 2048;  // work shares of one linear launch (workgroups x passes)
constexpr int kSyncCnt = 32;                          // first counter line
constexpr int kCntQkv = kSyncCnt;
constexpr int kCntWo = kCntQkv + kMaxShares * kCntStride;
constexpr int kCntGu = kCntWo + kMaxShares * kCntStride;
constexpr int kCntDown = kCntGu + kMaxShares * kCntStride;
constexpr int kCntLm = kCntDown + kMaxShares * kCntStride;   // LM head and stand-alone linear calls
constexpr int kCntDraft = kCntLm + kMaxShares * kCntStride;  // drafting heads inside a whole decoding step
constexpr int kCntAttn = kCntDraft + kMaxShares * kCntStride;   // up to 256 heads
constexpr int kCntXcd = kCntAttn + 256 * kCntStride;            // one line per XCD: QKV done, attention may start
constexpr int kCntGo = kCntXcd + 8 * kCntStride;                // one line per workgroup: its XCD has met
constexpr int kSyncWords = kCntGo + kRangeWgs * kCntStride;

// RMSNorm is split around the linear layer that consumes it: the producer of the residual
// stream x also leaves xg16 = fp16(x * g * kXgScale) (g = gain of the next norm), which is
// streamed like any fp16 input, and the per-row factor rsqrt(mean x^2 + eps) / kXgScale - a
// scalar per row, so it commutes with the contraction - is applied to the fp32 sums in the
// consumer's epilogue.  x * g itself must fit fp16: magnitudes up to 65504 (LLaMA-style
// residual outliers of a few thousand do), full relative precision down to 6e-5.
constexpr float kXgScale = 1.0f;

struct FusedArgs {
    int mode;
    int M, Mpad, kv_len;
    int H, nh, d, F;
    int64_t stride_head, stride_tok;       // K cache: (head, row, channel) at h*sh + t*st + c
    int64_t v_stride_head, v_stride_ch;    // V cache, channel-major: (head, channel, row) at h*vh + c*vc + t
    float eps, scale_log2e;
    // scratch (device)
    uint32_t* sync;        // kSyncWords
    float* part;           // linear layers: partial sums of shared row blocks, two slots per work share
    float* o_part;         // attention partial states, one per workgroup: [G][Mpad][d]
    float* ml_part;        // [G][Mpad][2]
    float* x;              // residual stream [M, H] fp32
    half_t* xg16;          // fp16(x * gain of the next RMSNorm), packed activation layout
    float* ss;             // sums of squares per 16-column tile: [H/16][Mpad]
    half_t* q16;           // [M, H]
    half_t* o16;           // attention output, packed activation layout
    half_t* a16;           // SwiGLU output [M, F], packed activation layout
    const float2* rope;    // (cos, sin) [M][d/2]
    const uint64_t* mask;  // ancestor masks [M][2]
    // linear-layer launch
    const half8* lin_W;
    const half_t* lin_x;   // input, packed activation layout
    void* lin_y;
    int lin_N, lin_K, lin_epi;
    int lin_slots;         // wide matrices: row tiles a work share handles at once (template choice)
    int lin_passes;        // work shares per workgroup
    int lin_whole;         // whole tiles are dealt out (always for wide matrices), else k ranges of row blocks
    int lin_rscale;        // the input is xg16: scale output row m by the RMSNorm factor of x[m]
    const half_t* lin_gnext;   // EPI_RESID: gain of the norm that follows (xg16 is rewritten)
    half_t *lin_kc, *lin_vc;   // EPI_QKV: the layer's cache
    int lin_cnt;           // which counter array of the sync block this call uses
    uint32_t lin_epoch;    // how often that array was used since it was zeroed
    uint32_t att_epoch;    // same for the attention head counters
    int64_t lin_ldy;
    float2* lin_amax;      // EPI_STORE_F32, optional: per (16-column tile, row) the largest output and,
                           // as int bits in .y, its lowest column: [tiles][Mpad]
    // attention launch
    const half_t *att_q, *att_k, *att_v;
    half_t* att_out;
    int att_out_packed;    // output in the packed activation layout (else row-major [M, nh, d])
    // Filled in at launch (see with_launch_facts): the matrix' layout, and every workgroup's
    // work share when there is one share per workgroup - what the kernel would otherwise
    // work out with a dozen integer divisions before it can request its first weights.
    int lin_ntiles, lin_nitems, lin_nks, lin_blk_shift;
    int lin_range_ok;                      // lin_range is filled in
    uint32_t lin_range[2 * kRangeWgs];     // workgroup j (logical index): units c0 .. c1 - 1 of its share
};

ghd_status launch_fused(const FusedArgs& a, hipStream_t st);
ghd_status launch_linear(const FusedArgs& a, hipStream_t st);
ghd_status launch_qkv_attn(const FusedArgs& a, hipStream_t st);
bool qkv_attn_available(int M, int slots, int passes, int d, int nh);
ghd_status launch_resident_checked(const void* kernel, int key, size_t lds, int* grid);
int fused_grid_size();
void share_on_host(int items, int per_item, int j, int G, int item, int* out);
void attn_share_on_host(int nh, int ntile, int j, int G, int head, int* out);

// How a linear layer is cut for G workgroups and row tiles of M: passes (work shares per
// workgroup) and, for wide matrices, the most row tiles one share touches.  Host only.
struct LinPlan { int slots, passes, whole; };
bool plan_linear(int M, int N, int K, int G, LinPlan* out);
size_t linear_part_floats(int M, int G);

// setup kernel: zero the sync block, tree tables, and (optionally) the residual stream
// with its sums of squares and its gain-scaled fp16 image
ghd_status launch_fused_setup(uint32_t* sync, const int32_t* parent, int M, int Mpad, int kv_len, int d,
                              float rope_base, uint64_t* mask, float2* rope, float* x,
                              const half_t* x_in16, int H, float* ss, const half_t* gain,
                              half_t* xg16, hipStream_t st);
// row-major fp16 [M, ldx] -> packed activation layout (columns K.. of the last k-step zero)
ghd_status launch_pack_x(half_t* dst, const half_t* src, int M, int Mpad, int K, int64_t ldx, hipStream_t st);

// the drafted tokens' own attention block from the nonzeros of the mask only (coo.hip)
ghd_status launch_tree_part_coo(void* out, const void* q, const void* kc, const void* vc, const uint64_t* mask,
                                int M, int kv_len, int nh, int d, int64_t stride_head, int64_t stride_tok,
                                int64_t v_stride_head, int64_t v_stride_ch, float scale, hipStream_t st);

ghd_status launch_pack2(void* dst, const void* src, int N, int K, int kind, int d, hipStream_t st);
size_t packed_bytes2(int N, int K);

}  // namespace ghd

// Argument block and launchers of the persistent kernels (fused.hip).
#pragma once
#include "common.h"

namespace ghd {

constexpr int kFT = 512;        // threads per workgroup (8 wavefronts)
constexpr int kTG = 16;         // 16-row weight tiles per row group (8 wavefronts x 2)
constexpr int kCH = 4;          // k-steps (32 columns) per staged chunk of x
constexpr int kGroupRows = kTG * 16;
constexpr int kChunkCols = kCH * 32;
constexpr int kMaxLayers = 48;  // the counter epochs (one per layer) are laid out for this many

enum { EPI_STORE_F32 = 0, EPI_STORE_F16 = 1, EPI_RESID = 2, EPI_SWIGLU = 3, EPI_QKV = 4 };
enum { MODE_LINEAR = 0, MODE_ATTN = 1 };
enum { PACK_PLAIN = 0, PACK_QKV = 1, PACK_GATE_UP = 2 };

// The sync block (uint32 words), zeroed by the set-up kernel.  Every item counter has a
// 128-byte line of its own (kCntStride words apart): the workgroups of one item poll and
// bump it without disturbing the others.  A linear layer's shared row slice is counted on
// the line of the first workgroup that has a part of it (one line per workgroup is enough);
// each kind of linear layer has an array of its own, reused layer after layer by epoch.
constexpr int kSyncStatus = 1;    // 0 = ok, else the code of the wait that gave up
constexpr int kCntStride = 32;
constexpr int kSyncCnt = 32;                          // first counter line
constexpr int kCntQkv = kSyncCnt;                     // up to 512 workgroups each
constexpr int kCntWo = kCntQkv + 512 * kCntStride;
constexpr int kCntGu = kCntWo + 512 * kCntStride;
constexpr int kCntDown = kCntGu + 512 * kCntStride;
constexpr int kCntLm = kCntDown + 512 * kCntStride;   // LM head and stand-alone linear calls
constexpr int kCntAttn = kCntLm + 1024 * kCntStride;  // up to 256 heads
constexpr int kSyncWords = kCntAttn + 256 * kCntStride;

struct FusedArgs {
    int mode;
    int M, Mpad, kv_len;
    int H, nh, d, F;
    int64_t stride_head, stride_tok;       // K cache: (head, row, channel) at h*sh + t*st + c
    int64_t v_stride_head, v_stride_ch;    // V cache, channel-major: (head, channel, row) at h*vh + c*vc + t
    float eps, scale_log2e;
    // scratch (device)
    uint32_t* sync;        // kSyncWords
    float* part;           // GEMM partial slots: [G][2][up to 16*MT KiB]
    float* o_part;         // attention partial states, one per workgroup: [G][Mpad][d]
    float* ml_part;        // [G][Mpad][2]
    float* x;              // residual stream [M, H] fp32
    half_t* xg16;          // fp16(x * gain of the next RMSNorm / 16) [M, H]: GEMM input
    float* ss;             // sums of squares per 16-column tile: [H/16][Mpad]
    half_t* q16;           // [M, H]
    half_t* o16;           // [M, H]
    half_t* a16;           // [M, F]
    const float2* rope;    // (cos, sin) [M][d/2]
    const uint64_t* mask;  // ancestor masks [M][2]
    // linear-layer launch
    const half8* lin_W;
    const half_t* lin_x;
    void* lin_y;
    int lin_N, lin_K, lin_epi;
    int lin_rs;            // row split of the 256-row groups (1, 2 or 4; capped by the LDS at M > 64)
    int lin_rscale;        // the input is xg16: scale output row m by the RMSNorm factor of x[m]
    const half_t* lin_gnext;   // EPI_RESID: gain of the norm that follows (xg16 is rewritten)
    half_t *lin_kc, *lin_vc;   // EPI_QKV: the layer's cache
    int lin_cnt;           // which group-counter array of the sync block this call uses
    uint32_t lin_epoch;    // how often that array was used since it was zeroed
    uint32_t att_epoch;    // same for the attention head counters
    int64_t lin_ldx, lin_ldy;
    // attention launch
    const half_t *att_q, *att_k, *att_v;
    half_t* att_out;
};

ghd_status launch_fused(const FusedArgs& a, hipStream_t st);
int fused_grid_size();
void share_on_host(int items, int per_item, int j, int G, int item, int* out);
void attn_share_on_host(int nh, int ntile, int j, int G, int head, int* out);

// setup kernel: zero the sync block, tree tables, and (optionally) the residual stream
// with its sums of squares and its gain-scaled fp16 image
ghd_status launch_fused_setup(uint32_t* sync, const int32_t* parent, int M, int Mpad, int kv_len, int d,
                              float rope_base, uint64_t* mask, float2* rope, float* x,
                              const half_t* x_in16, int H, float* ss, const half_t* gain,
                              half_t* xg16, hipStream_t st);

ghd_status launch_pack2(void* dst, const void* src, int N, int K, int kind, int d, hipStream_t st);
size_t packed_bytes2(int N, int K);

}  // namespace ghd

// Shared declarations of the gfx950 kernels behind the C ABI in include/ghd.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/ghd.h"

namespace ghd {

typedef _Float16 half_t;
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half2_ __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Records the HIP error of the last failing launch for ghd_last_hip_error().
ghd_status hip_fail(hipError_t e);
ghd_status check_launch();

// ---- plans (host) --------------------------------------------------------
struct GemmPlan {
    int MT;      // 16-row tiles of x (ceil(M/16))
    int NT;      // 16-row weight tiles per wavefront
    int S;       // split-K factor
    int kps;     // k-steps (32 columns each) per split
    int ksteps;  // ceil(K/32)
    int ntiles;  // ceil(N/16)
    int NW;      // wavefronts per workgroup
    bool lds;    // stage x through LDS (M > 16)
};
GemmPlan plan_gemm(int M, int N, int K);
// test hook: force NT / S (0 = automatic)
void set_gemm_override(int nt, int s, int nw, int lds);

struct AttnPlan {
    int P;       // key-range splits
    int tps;     // 64-key tiles per split
    int ntile;   // ceil((kv_len + M)/64)
    int groups;  // row groups of up to 64 (MTW==1) or 128 (MTW==2) rows
    int MTW;     // 16-row tiles per wavefront
};
AttnPlan plan_attention(int M, int kv_len, int nh);
void set_attn_override(int p);

// ---- launches (all asynchronous on `st`) ----------------------------------
// out[(s*M + m)*ld + n] = partial sum of split s; n < N only.
ghd_status launch_gemm(const GemmPlan& p, const void* Wp, const half_t* x, int64_t ldx, float* out,
                       int64_t ld, int M, int N, int K, hipStream_t st);

ghd_status launch_pack(void* dst, const void* src, int N, int K, hipStream_t st);

// y = sum_s part[s]; fp32 or fp16 output
ghd_status launch_reduce_out(void* y, int64_t ldy, bool out_f16, const float* part, int S,
                             int64_t ld, int M, int N, hipStream_t st);

// tree setup: depth, ancestor masks, rope table (cos,sin)[M][d/2]
ghd_status launch_tree_setup(const int32_t* parent, int M, int kv_len, int d, float rope_base,
                             int32_t* depth, uint64_t* mask, float2* rope, hipStream_t st);

// x_new = (x_old | widen(x_in16)) + sum_s part[s];  n16 = fp16(rmsnorm(x_new) * g) (if g)
ghd_status launch_residual_norm(float* x, const half_t* x_in16, const float* part, int S, int64_t ld,
                                const half_t* g, half_t* n16, int M, int H, float eps,
                                hipStream_t st);

// QKV epilogue: reduce splits, rotate q and k, write q16 [M,H] and cache rows kv_len+m
ghd_status launch_qkv_epilogue(const float* part, int S, int64_t ld, const float2* rope, half_t* q16,
                               half_t* kc, half_t* vc, int M, int nh, int d, int kv_len,
                               int64_t stride_head, int64_t stride_tok, hipStream_t st);

// a16[m,f] = fp16(silu(gate) * up) from split partials of [M, 2F]
ghd_status launch_swiglu(const float* part, int S, int64_t ld, half_t* a16, int M, int F,
                         hipStream_t st);

ghd_status launch_attention(const AttnPlan& p, half_t* out, const half_t* q, const half_t* kc,
                            const half_t* vc, const uint64_t* mask, int M, int kv_len, int nh, int d,
                            int64_t stride_head, int64_t stride_tok, float scale, float* o_part,
                            float* ml_part, hipStream_t st);

ghd_status launch_accept(const float* logits, const int32_t* tokens, const int32_t* parent, int M,
                         int V, int32_t* res, int32_t* amax_out, int32_t* amax_ws, hipStream_t st);

}  // namespace ghd

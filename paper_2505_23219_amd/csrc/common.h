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

static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Records the HIP error of the last failing launch for ghd_last_hip_error().
ghd_status hip_fail(hipError_t e);
ghd_status check_launch();

ghd_status launch_accept(const float* logits, const int32_t* tokens, const int32_t* parent, int M,
                         int V, int32_t* res, int32_t* amax_out, void* ws, hipStream_t st);
size_t accept_workspace_bytes();
ghd_status launch_amax_merge(const void* tbl, int ntiles, int Mpad, int M, int32_t* amax, hipStream_t st);
ghd_status launch_accept_path(const int32_t* amax, const int32_t* tokens, const int32_t* parent, int M,
                              int32_t* res, hipStream_t st);
ghd_status launch_accept_static(const float* logits, const int32_t* tokens, const int32_t* parent, int M,
                                int V, int32_t* res, int32_t* amax_out, hipStream_t st);
ghd_status launch_commit_path(void* const* k, void* const* v, int L, int nh, int d, int cap,
                              int kv_len, int M, const int32_t* res, hipStream_t st);


// drafting side (draft.hip)
ghd_status launch_embed(void* x16, const void* table16, const int32_t* tokens, int M, int H, int V,
                        hipStream_t st);
ghd_status launch_pick_norm(const float* x_final, const int32_t* res, int M, int H, const void* g,
                            float eps, void* n16, hipStream_t st);
ghd_status launch_topk(const float* logits, int rows, int V, int R, int32_t* topk, hipStream_t st);
ghd_status launch_tree_tokens(int32_t* tokens, const int32_t* parent, const int32_t* rank, int M,
                              const int32_t* topk, int K, int R, const int32_t* res, int V,
                              hipStream_t st);
int tree_build_host(const double* acc, int K, int R, int M, int32_t* parent, int32_t* rank,
                    double* expect);

}  // namespace ghd

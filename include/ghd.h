/*
 * ghd.h - C ABI of the MI355X tree-verification library (libghd.so).
 *
 * The library runs the verification forward step of predict-then-verify
 * speculative decoding (Ghidorah, arXiv 2505.23219, sections 2.2.2 and 2.3): a
 * LLaMA-style decoder stack scores a drafted token tree of M nodes (the paper's
 * "verification width", section 3.3.1) against a committed KV cache in one
 * pass, and the longest validated root path is accepted.
 *
 * Conventions for every call
 *   - All tensor pointers are DEVICE pointers unless the name says "_host".
 *     The caller owns every buffer; the library allocates nothing, frees
 *     nothing and keeps no pointer after the call returns.
 *   - fp16 tensors are IEEE binary16.  Activations are row-major [M, width].
 *   - Weight matrices are passed in the PACKED layout written by
 *     ghd_pack_weight (the bytes of the row-major [N, K] matrix, zero padded to
 *     N%256 == 0 and K%128 == 0 and reordered so that every workgroup streams
 *     one contiguous range in 1 KiB MFMA-operand blocks).
 *   - The KV cache of one layer is fp16.  K is row-major per head: element
 *     (head h, row t, channel c) at h*k_stride_head + t*k_stride_tok + c.  V is
 *     kept channel-major, (h, c, t) at h*v_stride_head + c*v_stride_ch + t, so
 *     that a tile of V^T (the operand of the P.V product, contiguous in the
 *     key index) is read as it lies.  Rows [0, kv_len) are committed, row
 *     kv_len + i belongs to tree node i.
 *   - The tree is parent[M] (int32): parent[0] == -1 (node 0 is the root: the
 *     last committed token, whose K/V is not yet cached), 0 <= parent[i] < i.
 *   - `stream` is a hipStream_t passed as void*.  Calls enqueue work and return;
 *     they never synchronise.  `ws` is caller-provided device scratch of at
 *     least the size the matching *_workspace_bytes function returns, 256-byte
 *     aligned.
 *   - Argument checks run on the host before the first GPU call.  A negative
 *     return value means nothing was enqueued (except GHD_ERR_HIP, which
 *     reports a failing launch; ghd_last_hip_error gives the HIP code).
 */
#ifndef GHD_H
#define GHD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t ghd_status;
enum {
    GHD_OK = 0,
    GHD_ERR_NULL = -1,      /* a required pointer is NULL */
    GHD_ERR_SHAPE = -2,     /* unsupported or inconsistent sizes */
    GHD_ERR_TREE = -3,      /* parent[] is not a topologically ordered rooted tree */
    GHD_ERR_CAPACITY = -4,  /* kv_len + M exceeds the cache capacity */
    GHD_ERR_WORKSPACE = -5, /* workspace missing or too small */
    GHD_ERR_ALIGN = -6,     /* pointer or leading dimension not 16-byte aligned */
    GHD_ERR_HIP = -7        /* a HIP call failed */
};

#define GHD_MAX_M 128       /* largest tree (rows of a skinny GEMM) */

/* flags of ghd_linear_skinny */
#define GHD_OUT_F32 0u      /* y is float  [M, ldy] */
#define GHD_OUT_F16 1u      /* y is fp16   [M, ldy] */

/* Limits: L <= 48, nh <= 256, H <= 43520, F <= 65536, V <= 262144, F % 8 == 0. */
typedef struct {
    int32_t H;            /* hidden size                         */
    int32_t nh;           /* attention heads (multi-head: kv heads == heads) */
    int32_t d;            /* head dim: 64 or 128, H == nh*d      */
    int32_t F;            /* SwiGLU FFN size                     */
    int32_t V;            /* vocabulary (LM-head rows)           */
    int32_t L;            /* layers                              */
    int32_t kv_capacity;  /* rows per head in every layer's cache */
    float rope_base;      /* rotary base (10000 for LLaMA)       */
    float rms_eps;        /* RMSNorm epsilon                     */
} ghd_model_cfg;

/* One decoder layer.  Gains are fp16 [H]; matrices are packed fp16:
 * Wqkv from [3H, H] (q rows, then k rows, then v rows), Wo from [H, H],
 * Wgu from [2F, H] (gate rows, then up rows), Wdown from [H, F]. */
typedef struct {
    const void *g_attn, *Wqkv, *Wo, *g_ffn, *Wgu, *Wdown;
} ghd_layer_weights;

/* One layer's cache, fp16: k [nh][kv_capacity][d], v [nh][d][kv_capacity]
 * (channel-major); kv_capacity % 8 == 0. */
typedef struct {
    void *k, *v;
} ghd_kv;

const char *ghd_status_str(ghd_status s);
int ghd_last_hip_error(void);

/* ---- tree ------------------------------------------------------------- */

/* Host check of parent_host[M]: GHD_OK, GHD_ERR_NULL, GHD_ERR_SHAPE (M outside
 * [1, GHD_MAX_M]) or GHD_ERR_TREE.  Pure host code. */
ghd_status ghd_tree_validate(const int32_t *parent_host, int M);

/* Ancestor-or-self mask of section 2.3 ("a token needs to compute
 * relationships only with certain tokens"): bit j of the 128-bit word
 * mask[i] = {mask_dev[2i] (bits 0..63), mask_dev[2i+1] (bits 64..127)} is set
 * iff node j is on the root path of node i.  Written by the same set-up kernel
 * whose masks the attention phase tests.  Every walk is bounded by M steps, so a
 * malformed device parent[] cannot hang. */
ghd_status ghd_tree_mask(const int32_t *parent_dev, int M, uint64_t *mask_dev, void *ws,
                         size_t ws_bytes, void *stream);
size_t ghd_tree_mask_workspace_bytes(void);

/* ---- weights ---------------------------------------------------------- */

/* Bytes of the packed form of a row-major [N, K] fp16 matrix. */
size_t ghd_packed_weight_bytes(int N, int K);

/* dst (packed) <- src (row-major [N, K] fp16, device).  One-off, offline.
 * Layout: packed row p and column k live in row group p/256, k-step k/32, tile
 * (p%256)/16; the 1 KiB block of (group, k-step, tile) sits at block index
 * (group*KS + k-step)*16 + tile with KS = 4*ceil(K/128); inside a block the
 * 16-byte chunk number ((k%32)/8)*16 + p%16 holds row p, columns k-k%8 .. +8.
 * Padding is zero.  `kind` chooses which source row packed row p holds:
 *   GHD_PACK_PLAIN    row p
 *   GHD_PACK_QKV      src is [3H, K] (q, k, v rows; heads of head_dim rows): in
 *                     every head, packed rows 4i..4i+3 hold channels 2i, 2i+1,
 *                     2i+head_dim/2, 2i+1+head_dim/2 (the two rotary pairs of a
 *                     quad end up in one lane of the GEMM output)
 *   GHD_PACK_GATE_UP  src is [2F, K] (gate rows then up rows), F%8 == 0: packed
 *                     rows 16t+4i .. +3 hold gate 8t+2i, gate 8t+2i+1, up 8t+2i,
 *                     up 8t+2i+1
 * ghd_linear_skinny takes GHD_PACK_PLAIN matrices; ghd_verify_layer/stack take
 * Wqkv as GHD_PACK_QKV, Wgu as GHD_PACK_GATE_UP and the rest as GHD_PACK_PLAIN. */
#define GHD_PACK_PLAIN 0
#define GHD_PACK_QKV 1
#define GHD_PACK_GATE_UP 2
ghd_status ghd_pack_weight(void *dst, const void *src, int N, int K, int kind, int head_dim,
                           void *stream);

/* ---- skinny linear layer (section 2.2.2: the linear layers of the MHA and
 *      MLP blocks; with 1..128 rows their cost is streaming W once) -------- */

/* y[m, n] = sum_k x[m, k] * W[n, k]   for m < M, n < N.
 *   x   fp16 [M, ldx] (ldx >= K, ldx % 8 == 0), K % 8 == 0
 *   Wp  packed W
 *   y   float or fp16 (flags) [M, ldy], ldy >= N
 * fp16 products, fp32 accumulation.  1 <= M <= GHD_MAX_M. */
ghd_status ghd_linear_skinny(void *y, const void *x, const void *Wp, int M, int N, int K,
                             int64_t ldx, int64_t ldy, uint32_t flags, void *ws, size_t ws_bytes,
                             void *stream);
size_t ghd_linear_workspace_bytes(int M, int N, int K);

/* ---- tree attention (Eq. 1 under the verification pattern of section 2.3:
 *      dense over the KV cache, ancestor-or-self over the tree rows) ------- */

/* out[i, h, :] = softmax_t(scale * q[i, h, :] . K[h, t, :]) V[h, t, :], t over
 * rows [0, kv_len) and rows kv_len + j with j on the root path of i.
 *   q, out  fp16 [M, nh, d];  d in {64, 128}
 *   k_cache, v_cache  fp16, strides in elements, all multiples of 8;
 *                     rows [0, kv_len + M) must be readable, and
 *                     v_stride_ch >= kv_len + M.
 * Splits the key range over workgroups and merges the parts with the
 * online-softmax rescaling of section 3.2.2.  nh <= 256. */
ghd_status ghd_tree_attention(void *out, const void *q, const void *k_cache, const void *v_cache,
                              const int32_t *parent_dev, int M, int kv_len, int nh, int d,
                              int64_t k_stride_head, int64_t k_stride_tok, int64_t v_stride_head,
                              int64_t v_stride_ch, float scale, void *ws, size_t ws_bytes,
                              void *stream);
size_t ghd_attention_workspace_bytes(int M, int kv_len, int nh, int d);

/* ---- decoder layer and stack (section 2.2.2; model details as in the
 *      LLaMA architecture of section 4.1: RMSNorm, rotary positions at
 *      kv_len + depth, SwiGLU, no biases) -------------------------------- */

/* x [M, H] float: residual stream, updated in place.  Writes node i's rotated
 * key and its value to cache row kv_len + i, then attends. */
ghd_status ghd_verify_layer(const ghd_model_cfg *cfg, const ghd_layer_weights *w, const ghd_kv *kv,
                            float *x, const int32_t *parent_dev, int M, int kv_len, void *ws,
                            size_t ws_bytes, void *stream);

/* x_in fp16 [M, H] (hidden states of the tree tokens) -> logits float [M, V].
 * layers_host / kv_host: host arrays of length cfg->L holding device pointers.
 * g_final fp16 [H]; Wlm packed from [V, H].  x_out (optional, may be NULL)
 * receives the final residual stream, float [M, H]. */
ghd_status ghd_verify_stack(const ghd_model_cfg *cfg, const ghd_layer_weights *layers_host,
                            const ghd_kv *kv_host, const void *g_final, const void *Wlm,
                            const void *x_in, const int32_t *parent_dev, int M, int kv_len,
                            float *logits, float *x_out, void *ws, size_t ws_bytes, void *stream);
size_t ghd_workspace_bytes(const ghd_model_cfg *cfg, int M, int kv_len);

/* Every linear layer and every attention is one launch of a persistent kernel
 * (one workgroup per compute unit, all resident) whose workgroups hand partial
 * results to each other; every wait is bounded and gives up rather than hang
 * (for instance if other work on the GPU keeps some workgroups from becoming
 * resident).  This call synchronises `stream` and reports the status word the
 * last ghd_linear_skinny / ghd_tree_attention / ghd_verify_layer /
 * ghd_verify_stack call left in its workspace `ws`: 0 = completed, otherwise
 * the code of the wait that gave up (3: a workgroup did not run on the expected
 * XCD) and the outputs are invalid.  Blocking; for tests and error handling,
 * not the hot path. */
ghd_status ghd_step_status(const void *ws, int32_t *status_host, void *stream);

/* ---- greedy acceptance (section 2.3: of the drafted tree, the longest root
 *      path the model itself would have produced is kept) ------------------- */

/* amax[i] = lowest index of the largest logit in row i.  The root is valid; a
 * node is valid iff its parent is valid and tokens[i] == amax[parent[i]].
 * res_dev[0] = length of the deepest valid root path (lowest node index on
 * ties), res_dev[1] = amax of its last node (the next token), res_dev[2..] =
 * its node indices, root first.  amax_dev (optional) receives all M argmaxes.
 * logits float [M, V]; tokens_dev, parent_dev int32 [M]; res_dev int32 [2+M]. */
ghd_status ghd_accept_greedy(const float *logits, const int32_t *tokens_dev,
                             const int32_t *parent_dev, int M, int V, int32_t *res_dev,
                             int32_t *amax_dev, void *ws, size_t ws_bytes, void *stream);
size_t ghd_accept_workspace_bytes(int M);

/* ---- commit of the accepted path (section 2.3: of the drafted tree only the
 *      verified tokens join the context) ---------------------------------- */

/* In every layer and head the K and V rows of the accepted nodes move from cache
 * rows kv_len + path[j] (where the verification pass left them) to rows
 * kv_len + j, j = 0 .. len-1; the caller then counts kv_len + len committed rows.
 * res_dev is the device result of ghd_accept_greedy for the same tree (len =
 * res_dev[0], path = res_dev[2..]), read on the device: no host round trip
 * between acceptance and commit.  Entries are clamped to the tree, so a corrupt
 * result cannot reach other rows.  kv_host: host array of cfg->L caches (device
 * pointers).  One launch. */
ghd_status ghd_commit_path(const ghd_model_cfg *cfg, const ghd_kv *kv_host, const int32_t *res_dev,
                           int M, int kv_len, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* GHD_H */

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
 *     whole 16-row tiles and 32-column k-steps and reordered into 1 KiB
 *     MFMA-operand blocks so that every workgroup streams contiguous runs).
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
 *   - Concurrency: the persistent kernels need every compute unit (all their
 *     workgroups wait for each other), so two calls that overlap in time on one
 *     GPU - from two streams or two threads - slow each other down and may run
 *     into the bounded waits (reported through ghd_step_status, never a hang).
 *     Calls that share a workspace must be ordered on one stream.  The library
 *     keeps no state between calls apart from per-device facts it caches (number
 *     of compute units, kernel attributes) and the error code of
 *     ghd_last_hip_error; it may be called from several host threads as long as
 *     their GPU work is ordered as said.
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
 * Layout: the unit is the 1 KiB block of 16 packed rows (a tile, T = p/16) by 32
 * columns (a k-step, s = k/32); inside a block the 16-byte chunk number
 * ((k%32)/8)*16 + p%16 holds row p, columns k-k%8 .. +8.  With KS = ceil(K/32)
 * k-steps and NT = ceil(N/16) tiles, tiles are stored in blocks of B tiles,
 * B = 8 if NT >= 640 (wide matrices) else 4, k-step major inside a block: the
 * 1 KiB block (T, s) sits at block index ((T/B)*KS + s)*B + T%B.  The last
 * block is padded to B tiles.
 * Padding is zero.  `kind` chooses which source row packed row p holds:
 *   GHD_PACK_PLAIN    row p
 *   GHD_PACK_QKV      src is [3H, K] (q, k, v rows; heads of head_dim rows): in
 *                     every head, packed rows 4i..4i+3 hold channels 2i, 2i+1,
 *                     2i+head_dim/2, 2i+1+head_dim/2 (the two rotary pairs of a
 *                     quad end up in one lane of the GEMM output).  The heads'
 *                     row blocks come in the order q of all heads, k of all
 *                     heads, v of all heads - or, when the number of heads is a
 *                     multiple of 8, in eight groups of nh/8 heads, each group
 *                     as q rows, k rows, v rows of its heads (the group whose
 *                     attention runs on the same eighth of the GPU)
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

/* The same attention under an arbitrary verification pattern (section 2.3 shows
 * three: the token tree, the several sequences of a draft model, the n-gram
 * pattern of Lookahead).  mask_dev: uint64 [M][2], 8-byte aligned; bit j of row i
 * (bits 0..63 in word 0, 64..127 in word 1) says that drafted token i sees
 * drafted token j (cache row kv_len + j); every drafted token sees the committed
 * rows [0, kv_len).  Bits from M on are ignored.  A row that sees no key at all
 * (kv_len == 0 and no bit set) gives zeros.  ghd_tree_attention is the special
 * case mask = ancestor-or-self (ghd_tree_mask writes that mask).  Everything else,
 * workspace size included, as for ghd_tree_attention. */
ghd_status ghd_masked_attention(void *out, const void *q, const void *k_cache, const void *v_cache,
                                const uint64_t *mask_dev, int M, int kv_len, int nh, int d,
                                int64_t k_stride_head, int64_t k_stride_tok, int64_t v_stride_head,
                                int64_t v_stride_ch, float scale, void *ws, size_t ws_bytes,
                                void *stream);

/* The drafted tokens' own block of the attention alone, computed from the
 * nonzeros of the tree mask (section 3.2.2 splits the attention into the dense
 * part over the committed cache and this sparse part; section 3.2.3 computes the
 * sparse part from a coordinate list of the mask's nonzeros, one dot product per
 * (token, ancestor) pair): out[i] = softmax over j in ancestors-or-self(i) of
 * q_i . k_j * scale, applied to v_j, where k_j, v_j are cache rows kv_len + j.
 * The committed rows [0, kv_len) are NOT attended: the result equals
 * ghd_tree_attention on a cache that holds the tree rows only.  The verification
 * step does not use this call (its attention kernel covers the block with one
 * masked MFMA tile); it is the paper's sparse kernel on this chip, for
 * comparison.  Arguments, layouts and workspace size as for ghd_tree_attention. */
ghd_status ghd_tree_part_attention_coo(void *out, const void *q, const void *k_cache, const void *v_cache,
                                       const int32_t *parent_dev, int M, int kv_len, int nh, int d,
                                       int64_t k_stride_head, int64_t k_stride_tok,
                                       int64_t v_stride_head, int64_t v_stride_ch, float scale,
                                       void *ws, size_t ws_bytes, void *stream);

/* ---- decoder layer and stack (section 2.2.2; model details as in the
 *      LLaMA architecture of section 4.1: RMSNorm, rotary positions at
 *      kv_len + depth, SwiGLU, no biases) -------------------------------- */

/* x [M, H] float: residual stream, updated in place.  Writes node i's rotated
 * key and its value to cache row kv_len + i, then attends.
 * Magnitudes: the input of every normalised linear layer is kept as
 * fp16(x * gain) (the row factor of the RMSNorm is applied after the
 * contraction), so |x * gain| must stay below 65504 and keeps full fp16
 * precision down to 6e-5; smaller entries lose relative precision gradually. */
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

/* ghd_verify_stack for greedy acceptance (section 2.3 keeps the longest root
 * path the model itself would have produced, which only needs every row's
 * argmax): the finish of the LM head reduces each row's (largest logit, lowest
 * vocabulary index) per 16-column tile, one more small launch merges the tiles
 * into amax_dev int32 [M], and the logits need not be written at all: `logits`
 * may be NULL (otherwise it is filled as by ghd_verify_stack).  amax_dev[i] is
 * exactly the argmax (lowest index on ties) of the logits row this call would
 * write.  Everything else as for ghd_verify_stack, workspace size included. */
ghd_status ghd_verify_stack_argmax(const ghd_model_cfg *cfg, const ghd_layer_weights *layers_host,
                                   const ghd_kv *kv_host, const void *g_final, const void *Wlm,
                                   const void *x_in, const int32_t *parent_dev, int M, int kv_len,
                                   int32_t *amax_dev, float *logits, float *x_out, void *ws,
                                   size_t ws_bytes, void *stream);

/* Every linear layer and every attention runs in a launch of a persistent kernel
 * (one workgroup per compute unit, all resident; a layer's QKV layer and attention
 * may share one) whose workgroups hand partial results to each other; every wait is bounded and gives up rather than hang
 * (for instance if other work on the GPU keeps some workgroups from becoming
 * resident).  This call synchronises `stream` and reports the status word the
 * last ghd_linear_skinny / ghd_tree_attention / ghd_verify_layer /
 * ghd_verify_stack call left in its workspace `ws`: 0 = completed, otherwise
 * the code of the wait that gave up (3: a workgroup did not run on the expected
 * XCD) and the outputs are invalid (a workgroup whose wait gave up writes no
 * results for the item it waited for).  The word is sticky: every call's set-up
 * clears the status for the launches that follow but keeps the first non-zero
 * status it finds, so a caller who asks only every so often still learns that
 * some call since ghd_step_status_reset (or since the first use of the
 * workspace) gave up.  Blocking; for tests and error handling, not the hot path. */
ghd_status ghd_step_status(const void *ws, int32_t *status_host, void *stream);
/* Clears the status, the kept one included (enqueued on `stream`). */
ghd_status ghd_step_status_reset(void *ws, void *stream);

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

/* The second half of ghd_accept_greedy on its own: the row argmaxes are given
 * (amax_dev int32 [M], e.g. from ghd_verify_stack_argmax); validity, the deepest
 * valid node and its root path as above.  One small launch, no workspace. */
ghd_status ghd_accept_path(const int32_t *amax_dev, const int32_t *tokens_dev,
                           const int32_t *parent_dev, int M, int32_t *res_dev, void *stream);

/* ghd_accept_greedy for callers that cannot allocate or pass a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments and results, no `ws`: the per-segment maxima go to
 * an 8 KiB array that is part of the library's device image (one copy per GPU,
 * held until the process ends), which fits every tree this library accepts;
 * M > GHD_MAX_M is GHD_ERR_SHAPE as everywhere.  The call allocates nothing
 * and frees nothing.  All calls on one GPU share that array: calls that
 * overlap in time on one GPU (two streams, two threads) race; order them on one
 * stream.  Nothing in the array needs clearing between calls. */
ghd_status ghd_accept_greedy_static(const float *logits, const int32_t *tokens_dev,
                                    const int32_t *parent_dev, int M, int V, int32_t *res_dev,
                                    int32_t *amax_dev, void *stream);

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

/* ---- drafting side of a decoding step (section 2.1: tokens for several future
 *      slots are predicted and then verified together; section 2.3: with
 *      self-drafting the predictions come from extra heads at the tail of the
 *      model, each with several candidates; section 3.3.1: the candidates are
 *      combined into the verification tree) ------------------------------- */

/* x16[i, :] = table16[tokens[i], :]: fp16 hidden states [M, H] of the tree's tokens
 * from the embedding table fp16 [V, H].  Tokens are clamped to [0, V). */
ghd_status ghd_embed(void *x16, const void *table16, const int32_t *tokens_dev, int M, int H, int V,
                     void *stream);

/* Tree design from head accuracies (section 3.3.1), on the host: acc_host[k*R + r]
 * in [0, 1] is the accuracy of candidate r of head k; a node's score is the
 * product of the accuracies along its root path, the expected acceptance length
 * of a tree 1 + the sum of its nodes' scores.  Inserts the best-scoring open
 * candidate until the tree has M nodes (lower parent, then lower rank on ties);
 * node order = insertion order.  parent_host, rank_host: int32 [M] (rank[i] =
 * which candidate of head depth[i]-1 node i carries; rank[0] = 0).  Returns the
 * number of nodes (< M when K*R levels cannot supply more) or a negative
 * ghd_status; *expect_host (optional) receives the expected acceptance length.
 * The paper's last step, a local search by measured acceptance on a calibration
 * set, needs data and is not part of this call. */
int ghd_tree_build(const double *acc_host, int K, int R, int M, int32_t *parent_host,
                   int32_t *rank_host, double *expect_host);

/* Choice of the verification width (section 3.3.1: width and tree together fix
 * the acceptance length; section 3.3.2: candidate widths, powers of two in the
 * paper, are profiled on the hardware).  For every candidate width widths_host[i]
 * with measured step time latency_host[i] > 0 the tree is designed as by
 * ghd_tree_build; returns the index of the width with the most expected accepted
 * tokens per unit of step time (the first on ties), or a negative ghd_status.
 * rate_host (optional, double [n]) receives every candidate's rate.  Host only. */
int ghd_choose_width(const double *acc_host, int K, int R, const int32_t *widths_host,
                     const double *latency_host, int n, double *rate_host);

/* Tokens of the next tree.  The K drafting heads are linear layers [V, H] on the
 * RMS-normalised (gain g_final fp16 [H]) final hidden state of the last accepted
 * node; Wheads is their stacked matrix [K*V, H] packed with ghd_pack_weight
 * (plain).  x_final float [M, H] is the final residual stream of the verification
 * pass (x_out of ghd_verify_stack), res_dev the result of ghd_accept_greedy for
 * it; the last accepted node is read on the device.  Per head the R best
 * candidates are taken, best first, lowest index on ties (logits must be finite).
 * tokens_dev[0] = res_dev[1] (the token the model has just produced);
 * tokens_dev[i] = candidate rank_dev[i] of head depth[i]-1.  A tree deeper than K
 * levels or a rank >= R is the caller's error; indices are clamped so that
 * nothing outside the tables is read.  topk_dev int32 [K, R] and head_logits
 * float [K*V] are optional outputs.  K <= 16, R <= 32, K*V <= 262144. */
ghd_status ghd_draft_tokens(const void *g_final, const void *Wheads, int K, int R, int H, int V,
                            float rms_eps, const float *x_final, const int32_t *res_dev,
                            const int32_t *parent_dev, const int32_t *rank_dev, int M,
                            int32_t *tokens_dev, int32_t *topk_dev, float *head_logits, void *ws,
                            size_t ws_bytes, void *stream);
size_t ghd_draft_workspace_bytes(int K, int R, int H, int V);

/* One whole predict-then-verify step (section 2.1), enqueued without a host round
 * trip: embed the tree's tokens, verify (ghd_verify_stack), accept
 * (ghd_accept_greedy), commit the accepted path (ghd_commit_path), draft the next
 * tree's tokens (ghd_draft_tokens).  tokens_dev int32 [M]: in, the tree's tokens
 * (tokens[0] = the last produced token, not yet cached); out, the next tree's.
 * res_dev int32 [2+M]: out, the acceptance result; the step adds res_dev[0]
 * tokens to the output (the accepted drafted tokens tokens[path[1..]] as they were
 * on entry, then res_dev[1]) and the caller's next kv_len is kv_len + res_dev[0]. */
typedef struct {
    const ghd_model_cfg *cfg;
    const ghd_layer_weights *layers_host;   /* host array [cfg->L] */
    const ghd_kv *kv_host;                  /* host array [cfg->L] */
    const void *g_final, *Wlm;              /* as for ghd_verify_stack */
    const void *embed;                      /* fp16 [V, H], row-major */
    const void *Wheads;                     /* packed from [K*V, H] */
    int32_t K, R;                           /* drafting heads, candidates per head */
} ghd_spec_model;
ghd_status ghd_spec_step(const ghd_spec_model *m, const int32_t *parent_dev, const int32_t *rank_dev,
                         int M, int kv_len, int32_t *tokens_dev, int32_t *res_dev, void *ws,
                         size_t ws_bytes, void *stream);
size_t ghd_spec_workspace_bytes(const ghd_spec_model *m, int M, int kv_len);

#ifdef __cplusplus
}
#endif
#endif /* GHD_H */

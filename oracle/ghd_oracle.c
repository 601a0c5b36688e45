/*
 * CPU oracle for the tree-verification step of speculative decoding.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path may call this file:
 * it exists so that tests, the smoke check and the benchmark's CPU-baseline
 * leg have a plain, slow, independent statement of what the step computes.
 * It shares no code with the HIP kernels.
 *
 * What it follows (Ghidorah, arXiv 2505.23219):
 *   - section 2.2.2: a Transformer layer is an MHA block (QKV linear, per-head
 *     attention, output linear) and an MLP block of consecutive linears;
 *   - Eq. (1): X = Q K^T, A = softmax(X), O = A V;
 *   - section 2.3: under a verification tree a drafted token is related only to
 *     the tokens on its own root path, all drafted tokens see the whole KV
 *     cache, and softmax and A V share that sparsity pattern; after the pass only
 *     the longest verified root path is kept and joins the context.
 * The model details the paper leaves to its model choice (section 4.1,
 * Vicuna-7B, i.e. the LLaMA architecture) are written out here: RMSNorm,
 * rotary embedding in the half-split pairing, SwiGLU MLP, no biases, softmax
 * scale 1/sqrt(d) passed in by the caller.
 *
 * Every function is the definition written out: no tiling, no online softmax,
 * every sum taken in ascending index order.  The arithmetic type is ORC_REAL
 * (float by default; the same file built with -DORC_REAL=double gives a second
 * library used to bound the float one's rounding noise).  Inputs that live in
 * fp16 in the real system (weights, cache) are passed as fp16 bit patterns and
 * widened exactly.  With round16 != 0 the layer rounds to fp16 at the points
 * where the real system stores fp16 tensors (normalised activations, q/k/v,
 * attention output, MLP activation); with round16 == 0 nothing is rounded.
 *
 * Parity pins (tests/test_oracle_*.py): mask vs. an independent bitmask
 * recurrence on every tree up to 6 nodes; chain tree == causal attention;
 * path decomposition; width-1 tree == sequential decode steps; library
 * cross-checks (fp64 matmul, scaled_dot_product_attention with a boolean
 * mask); closed forms for the element-wise pieces; acceptance vs. brute-force
 * path enumeration; commit of the accepted path == feeding the accepted tokens
 * one after the other.  End-to-end logits have no value printed in the paper to
 * compare with: for those, parity is pinned only through these pieces.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef ORC_REAL
#define ORC_REAL float
#endif
typedef ORC_REAL real;

#define ORC_MAX_M 128

/* ---------------------------------------------------------------- fp16 -- */

/* IEEE binary16 -> double, exact. */
static double h2d(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24);               /* zero and subnormals */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp((double)(m + 1024), e - 25);
    return sign ? -v : v;
}

/* double -> IEEE binary16, round to nearest even (rint under the default
 * rounding mode), overflow to infinity. */
static uint16_t d2h(double v)
{
    uint16_t sign = signbit(v) ? 0x8000 : 0;
    double a = fabs(v);
    if (isnan(v))
        return 0x7e00;
    if (a >= 65520.0)                            /* halfway to 2^16 rounds up */
        return sign | 0x7c00;
    if (a < ldexp(1.0, -14)) {                   /* subnormal range */
        double q = rint(ldexp(a, 24));           /* 0 .. 1024 */
        return sign | (uint16_t)q;               /* 1024 == smallest normal */
    }
    int e2;
    (void)frexp(a, &e2);                         /* a = f * 2^e2, f in [0.5,1) */
    int E = e2 - 1;                              /* a in [2^E, 2^(E+1)) */
    double q = rint(ldexp(a, 10 - E));           /* 1024 .. 2048 */
    if (q >= 2048.0) {
        q = 1024.0;
        E += 1;
    }
    return sign | (uint16_t)(((E + 15) << 10) | ((int)q - 1024));
}

float orc_half_to_float(uint16_t h) { return (float)h2d(h); }
uint16_t orc_float_to_half(float f) { return d2h((double)f); }

static real widen(uint16_t h) { return (real)h2d(h); }
static real round_half(real v) { return (real)h2d(d2h((double)v)); }

int orc_real_bytes(void) { return (int)sizeof(real); }

/* ---------------------------------------------------------------- tree -- */

/* Returns 0 when parent[] describes a rooted tree in topological order. */
int orc_tree_validate(const int32_t *parent, int M)
{
    if (M < 1 || M > ORC_MAX_M || parent[0] != -1)
        return -1;
    for (int i = 1; i < M; ++i)
        if (parent[i] < 0 || parent[i] >= i)
            return -1;
    return 0;
}

void orc_tree_depth(const int32_t *parent, int M, int32_t *depth)
{
    depth[0] = 0;
    for (int i = 1; i < M; ++i)
        depth[i] = depth[parent[i]] + 1;
}

/* mask[i*M + j] = 1 iff node j lies on the root path of node i (i included):
 * the "certain tokens" a drafted token is related to (section 2.3).  Written
 * as the enumeration itself: walk from i up to the root. */
void orc_tree_mask(const int32_t *parent, int M, uint8_t *mask)
{
    memset(mask, 0, (size_t)M * M);
    for (int i = 0; i < M; ++i)
        for (int j = i; j >= 0; j = parent[j])
            mask[(size_t)i * M + j] = 1;
}

/* --------------------------------------------------------------- linear -- */

/* y[m,n] = sum_k x[m,k] * W[n,k], k ascending.  W holds fp16 bits, row-major
 * [N,K].  The loop nest keeps one weight row in flight and updates the M
 * running sums together; each sum still adds its terms in ascending k. */
void orc_linear(real *y, const real *x, const uint16_t *W, int M, int N, int K)
{
    real *xt = (real *)malloc((size_t)K * M * sizeof(real));
    for (int m = 0; m < M; ++m)
        for (int k = 0; k < K; ++k)
            xt[(size_t)k * M + m] = x[(size_t)m * K + k];
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        real acc[ORC_MAX_M];
        for (int m = 0; m < M; ++m)
            acc[m] = 0;
        const uint16_t *w = W + (size_t)n * K;
        for (int k = 0; k < K; ++k) {
            real wk = widen(w[k]);
            const real *xk = xt + (size_t)k * M;
            for (int m = 0; m < M; ++m)
                acc[m] += xk[m] * wk;
        }
        for (int m = 0; m < M; ++m)
            y[(size_t)m * N + n] = acc[m];
    }
    free(xt);
}

/* ------------------------------------------------------- element-wise -- */

/* out[m,:] = x[m,:] / sqrt(mean(x[m,:]^2) + eps) * g */
void orc_rmsnorm(real *out, const real *x, const uint16_t *g, int M, int H, real eps)
{
    for (int m = 0; m < M; ++m) {
        real ss = 0;
        for (int c = 0; c < H; ++c)
            ss += x[(size_t)m * H + c] * x[(size_t)m * H + c];
        real r = (real)1 / (real)sqrt((double)(ss / (real)H + eps));
        for (int c = 0; c < H; ++c)
            out[(size_t)m * H + c] = x[(size_t)m * H + c] * r * widen(g[c]);
    }
}

/* Rotary embedding, half-split pairing: dims (j, j + d/2) of every head turn
 * by the angle pos * base^(-2j/d).  The angle and its sine and cosine are
 * taken in double and then narrowed to the working type. */
void orc_rope(real *t, const int32_t *pos, int M, int nh, int d, double base)
{
    int half = d / 2;
    for (int m = 0; m < M; ++m)
        for (int j = 0; j < half; ++j) {
            double ang = (double)pos[m] * pow(base, -2.0 * j / d);
            real c = (real)cos(ang), s = (real)sin(ang);
            for (int h = 0; h < nh; ++h) {
                real *v = t + ((size_t)m * nh + h) * d;
                real a = v[j], b = v[j + half];
                v[j] = a * c - b * s;
                v[j + half] = b * c + a * s;
            }
        }
}

static real silu(real z) { return z / ((real)1 + (real)exp(-(double)z)); }

/* a[m,f] = silu(gu[m,f]) * gu[m,F+f] */
void orc_swiglu(real *a, const real *gu, int M, int F)
{
    for (int m = 0; m < M; ++m)
        for (int f = 0; f < F; ++f)
            a[(size_t)m * F + f] = silu(gu[(size_t)m * 2 * F + f]) * gu[(size_t)m * 2 * F + F + f];
}

/* ------------------------------------------------------------ attention -- */

/* Tree attention, Eq. (1) restricted to the verification pattern.
 *   q, out : [M, nh, d] in the working type
 *   kc, vc : fp16 bits; element (h, t, c) at h*stride_head + t*stride_tok + c
 *            rows [0,kv_len) are the committed cache, row kv_len+j is node j.
 * Node i attends every committed row and tree row j iff j is on i's root
 * path.  Keys outside that set are simply not part of the softmax. */
void orc_tree_attention(real *out, const real *q, const uint16_t *kc, const uint16_t *vc,
                        const int32_t *parent, int M, int kv_len, int nh, int d,
                        int64_t stride_head, int64_t stride_tok, real scale)
{
    uint8_t *mask = (uint8_t *)malloc((size_t)M * M);
    orc_tree_mask(parent, M, mask);
    int T = kv_len + M;
#pragma omp parallel for schedule(static)
    for (int h = 0; h < nh; ++h) {
        real *s = (real *)malloc((size_t)T * sizeof(real));
        for (int i = 0; i < M; ++i) {
            const real *qi = q + ((size_t)i * nh + h) * d;
            real *oi = out + ((size_t)i * nh + h) * d;
            /* X = Q K^T over the visible set */
            real mx = -INFINITY;
            for (int t = 0; t < T; ++t) {
                if (t >= kv_len && !mask[(size_t)i * M + (t - kv_len)])
                    continue;
                const uint16_t *kt = kc + h * stride_head + t * stride_tok;
                real dot = 0;
                for (int c = 0; c < d; ++c)
                    dot += qi[c] * widen(kt[c]);
                s[t] = dot * scale;
                if (s[t] > mx)
                    mx = s[t];
            }
            /* A = softmax(X) */
            real denom = 0;
            for (int t = 0; t < T; ++t) {
                if (t >= kv_len && !mask[(size_t)i * M + (t - kv_len)])
                    continue;
                s[t] = (real)exp((double)(s[t] - mx));
                denom += s[t];
            }
            /* O = A V */
            for (int c = 0; c < d; ++c)
                oi[c] = 0;
            for (int t = 0; t < T; ++t) {
                if (t >= kv_len && !mask[(size_t)i * M + (t - kv_len)])
                    continue;
                real p = s[t] / denom;
                const uint16_t *vt = vc + h * stride_head + t * stride_tok;
                for (int c = 0; c < d; ++c)
                    oi[c] += p * widen(vt[c]);
            }
        }
        free(s);
    }
    free(mask);
}

/* ---------------------------------------------------------------- layer -- */

typedef struct {
    int32_t H, nh, d, F, V, L, kv_capacity;
    float rope_base, rms_eps;
} orc_cfg;

static void maybe_round(real *t, size_t n, int round16)
{
    if (round16)
        for (size_t i = 0; i < n; ++i)
            t[i] = round_half(t[i]);
}

/* One decoder layer over the M tree nodes; x [M,H] is the residual stream,
 * updated in place.  kc/vc are this layer's cache, head-major
 * [nh][kv_capacity][d]; the layer writes node i's key and value to row
 * kv_len + i (fp16, as the cache is) before attending.  Node i sits at
 * position kv_len + depth[i]. */
void orc_verify_layer(const orc_cfg *c, const uint16_t *g_attn, const uint16_t *Wqkv,
                      const uint16_t *Wo, const uint16_t *g_ffn, const uint16_t *Wgu,
                      const uint16_t *Wdown, uint16_t *kc, uint16_t *vc, real *x,
                      const int32_t *parent, int M, int kv_len, int round16)
{
    int H = c->H, nh = c->nh, d = c->d, F = c->F;
    size_t MH = (size_t)M * H;
    real *n = (real *)malloc(MH * sizeof(real));
    real *qkv = (real *)malloc(3 * MH * sizeof(real));
    real *q = (real *)malloc(MH * sizeof(real));
    real *k = (real *)malloc(MH * sizeof(real));
    real *o = (real *)malloc(MH * sizeof(real));
    real *y = (real *)malloc(MH * sizeof(real));
    real *gu = (real *)malloc((size_t)M * 2 * F * sizeof(real));
    real *a = (real *)malloc((size_t)M * F * sizeof(real));
    int32_t depth[ORC_MAX_M], pos[ORC_MAX_M];

    orc_tree_depth(parent, M, depth);
    for (int i = 0; i < M; ++i)
        pos[i] = kv_len + depth[i];

    /* MHA block */
    orc_rmsnorm(n, x, g_attn, M, H, (real)c->rms_eps);
    maybe_round(n, MH, round16);
    orc_linear(qkv, n, Wqkv, M, 3 * H, H);
    for (int m = 0; m < M; ++m)
        for (int col = 0; col < H; ++col) {
            q[(size_t)m * H + col] = qkv[(size_t)m * 3 * H + col];
            k[(size_t)m * H + col] = qkv[(size_t)m * 3 * H + H + col];
        }
    orc_rope(q, pos, M, nh, d, (double)c->rope_base);
    orc_rope(k, pos, M, nh, d, (double)c->rope_base);
    maybe_round(q, MH, round16);
    int64_t stride_head = (int64_t)c->kv_capacity * d, stride_tok = d;
    for (int m = 0; m < M; ++m)
        for (int h = 0; h < nh; ++h)
            for (int e = 0; e < d; ++e) {
                size_t dst = (size_t)h * stride_head + (size_t)(kv_len + m) * stride_tok + e;
                kc[dst] = d2h((double)k[((size_t)m * nh + h) * d + e]);
                vc[dst] = d2h((double)qkv[(size_t)m * 3 * H + 2 * H + (size_t)h * d + e]);
            }
    orc_tree_attention(o, q, kc, vc, parent, M, kv_len, nh, d, stride_head, stride_tok,
                       (real)(1.0 / sqrt((double)d)));
    maybe_round(o, MH, round16);
    orc_linear(y, o, Wo, M, H, H);
    for (size_t i = 0; i < MH; ++i)
        x[i] += y[i];

    /* MLP block */
    orc_rmsnorm(n, x, g_ffn, M, H, (real)c->rms_eps);
    maybe_round(n, MH, round16);
    orc_linear(gu, n, Wgu, M, 2 * F, H);
    orc_swiglu(a, gu, M, F);
    maybe_round(a, (size_t)M * F, round16);
    orc_linear(y, a, Wdown, M, H, F);
    for (size_t i = 0; i < MH; ++i)
        x[i] += y[i];

    free(n); free(qkv); free(q); free(k); free(o); free(y); free(gu); free(a);
}

/* logits[M,V] = rmsnorm(x, g_final) * Wlm^T */
void orc_lm_head(const orc_cfg *c, const uint16_t *g_final, const uint16_t *Wlm,
                 const real *x, real *logits, int M, int round16)
{
    size_t MH = (size_t)M * c->H;
    real *n = (real *)malloc(MH * sizeof(real));
    orc_rmsnorm(n, x, g_final, M, c->H, (real)c->rms_eps);
    maybe_round(n, MH, round16);
    orc_linear(logits, n, Wlm, M, c->V, c->H);
    free(n);
}

/* The whole step: x_in [M,H] fp16 bits -> logits [M,V].  Per-layer pointers
 * are given as arrays of length L. */
void orc_verify_stack(const orc_cfg *c, const uint16_t *const *g_attn,
                      const uint16_t *const *Wqkv, const uint16_t *const *Wo,
                      const uint16_t *const *g_ffn, const uint16_t *const *Wgu,
                      const uint16_t *const *Wdown, uint16_t *const *kc, uint16_t *const *vc,
                      const uint16_t *g_final, const uint16_t *Wlm, const uint16_t *x_in,
                      const int32_t *parent, int M, int kv_len, real *logits, real *x_out,
                      int round16)
{
    size_t MH = (size_t)M * c->H;
    real *x = (real *)malloc(MH * sizeof(real));
    for (size_t i = 0; i < MH; ++i)
        x[i] = widen(x_in[i]);
    for (int l = 0; l < c->L; ++l)
        orc_verify_layer(c, g_attn[l], Wqkv[l], Wo[l], g_ffn[l], Wgu[l], Wdown[l], kc[l], vc[l],
                         x, parent, M, kv_len, round16);
    if (x_out)
        memcpy(x_out, x, MH * sizeof(real));
    if (logits)
        orc_lm_head(c, g_final, Wlm, x, logits, M, round16);
    free(x);
}

/* ----------------------------------------------------------- acceptance -- */

/* Greedy acceptance (section 2.3: the longest verified root path is kept).
 * amax[i] = lowest index of the largest logit of row i.  The root is valid; a
 * drafted node is valid iff its parent is valid and its token equals the
 * parent's amax.  The result is the valid node of greatest depth (lowest index
 * on ties): res[0] = path length, res[1] = amax of that node (the next token),
 * res[2..] = the node indices from the root down.  amax_out (optional) gets
 * all M argmaxes. */
void orc_accept_greedy(const real *logits, const int32_t *tokens, const int32_t *parent,
                       int M, int V, int32_t *res, int32_t *amax_out)
{
    int32_t amax[ORC_MAX_M], depth[ORC_MAX_M];
    uint8_t valid[ORC_MAX_M];
    for (int i = 0; i < M; ++i) {
        int best = 0;
        for (int v = 1; v < V; ++v)
            if (logits[(size_t)i * V + v] > logits[(size_t)i * V + best])
                best = v;
        amax[i] = best;
        if (amax_out)
            amax_out[i] = best;
    }
    orc_tree_depth(parent, M, depth);
    valid[0] = 1;
    int last = 0;
    for (int i = 1; i < M; ++i) {
        valid[i] = valid[parent[i]] && tokens[i] == amax[parent[i]];
        if (valid[i] && depth[i] > depth[last])
            last = i;
    }
    int len = depth[last] + 1;
    res[0] = len;
    res[1] = amax[last];
    for (int node = last, p = len - 1; node >= 0; node = parent[node], --p)
        res[2 + p] = node;
}

/* ---------------------------------------------------------------- commit -- */

/* Commit of the accepted path (section 2.3: only the verified tokens join the
 * context).  The K and V rows of the accepted nodes path[0..len), which the
 * verification pass left at cache rows kv_len + path[j], become the rows
 * kv_len + j, j = 0..len-1; the caller's committed length then grows by len.
 * Cache [nh][cap][d] as fp16 bit patterns; rows from kv_len + len on are left as
 * they are.  Written with a scratch copy so that no source row can have been
 * overwritten before it is read. */
void orc_commit_path(uint16_t *kc, uint16_t *vc, int nh, int cap, int d, int kv_len,
                     const int32_t *path, int len)
{
    uint16_t *tmp = (uint16_t *)malloc((size_t)len * d * sizeof(uint16_t));
    uint16_t *caches[2] = {kc, vc};
    for (int which = 0; which < 2; ++which)
        for (int h = 0; h < nh; ++h) {
            uint16_t *head = caches[which] + (size_t)h * cap * d;
            for (int j = 0; j < len; ++j)
                memcpy(tmp + (size_t)j * d, head + (size_t)(kv_len + path[j]) * d,
                       (size_t)d * sizeof(uint16_t));
            memcpy(head + (size_t)kv_len * d, tmp, (size_t)len * d * sizeof(uint16_t));
        }
    free(tmp);
}

/* -------------------------------------------------------------- drafting -- */

/* The drafting side of a decoding step (section 2.1: predictions for several
 * future slots are made in parallel and then verified; section 2.3: with
 * self-drafting, extra heads at the tail of the model predict the tokens of
 * the future slots, head k the slot k + 1 positions after the next token, each
 * with several candidates; section 3.3.1: the candidates are combined into a
 * verification tree).  Pins (tests/test_oracle_draft.py): top-R against a full
 * sort; head logits against the LM-head routine fed one head at a time; the
 * tree design against exhaustive search over all trees of the same width; the
 * decoding loop against plain sequential greedy decoding (drafting and
 * verification never change the produced tokens). */

/* Embedding: row i of x is row tokens[i] of the table (fp16 bit patterns). */
void orc_embed(uint16_t *x, const uint16_t *table, const int32_t *tokens, int M, int H)
{
    for (int i = 0; i < M; ++i)
        memcpy(x + (size_t)i * H, table + (size_t)tokens[i] * H, (size_t)H * sizeof(uint16_t));
}

/* Logits of the K drafting heads for ONE hidden state x_row[H] (the final
 * residual stream of the last accepted node): every head is a linear layer
 * [V, H] on the normalised state, the heads' matrices stacked as [K*V, H].
 * out[k*V + v].  The state is normalised and rounded exactly as for the LM head. */
void orc_draft_logits(real *out, const real *x_row, const uint16_t *g_final,
                      const uint16_t *Wheads, int K, int V, int H, real eps, int round16)
{
    real *n = (real *)malloc((size_t)H * sizeof(real));
    orc_rmsnorm(n, x_row, g_final, 1, H, eps);
    maybe_round(n, (size_t)H, round16);
    orc_linear(out, n, Wheads, 1, K * V, H);
    free(n);
}

/* The R best entries of each row, best first: R times over, the lowest index
 * of the largest value not yet taken.  idx[row*R + r]. */
void orc_topk(int32_t *idx, const real *v, int rows, int V, int R)
{
    uint8_t *taken = (uint8_t *)malloc((size_t)V);
    for (int row = 0; row < rows; ++row) {
        const real *a = v + (size_t)row * V;
        memset(taken, 0, (size_t)V);
        for (int r = 0; r < R; ++r) {
            int best = -1;
            for (int j = 0; j < V; ++j)
                if (!taken[j] && (best < 0 || a[j] > a[best]))
                    best = j;
            taken[best] = 1;
            idx[(size_t)row * R + r] = best;
        }
    }
    free(taken);
}

/* Tokens of the next verification tree: the root carries the token the model
 * has just produced; a node at depth t >= 1 carries candidate rank[i] of head
 * t - 1 (its parent fixes the earlier slots).  topk[k*R + r]. */
void orc_tree_tokens(int32_t *tokens, const int32_t *parent, const int32_t *rank, int M,
                     const int32_t *topk, int R, int32_t root_token)
{
    int32_t depth[ORC_MAX_M];
    orc_tree_depth(parent, M, depth);
    tokens[0] = root_token;
    for (int i = 1; i < M; ++i)
        tokens[i] = topk[(size_t)(depth[i] - 1) * R + rank[i]];
}

/* Tree design (section 3.3.1).  acc[k*R + r] is the measured accuracy of
 * candidate r of head k.  The accuracy of a candidate sequence is estimated as
 * the product of the accuracies of its tokens; a node is accepted exactly when
 * its whole sequence is, so the expected acceptance length of a tree is 1 (the
 * root, always kept) plus the sum of its nodes' sequence accuracies.  Nodes are
 * added one at a time, each time the candidate with the highest sequence
 * accuracy whose parent is already in the tree, until the tree has M nodes
 * (lowest parent, then lowest rank on ties).  Node order = insertion order, so
 * parent[i] < i.  Stops early when no candidate is left; returns the number of
 * nodes, *expect gets the expected acceptance length.  (The paper's final
 * refinement by measured acceptance on a calibration set is outside this
 * function: it needs data.) */
int orc_tree_build(const double *acc, int K, int R, int M, int32_t *parent, int32_t *rank,
                   double *expect)
{
    double p[ORC_MAX_M];
    int depth[ORC_MAX_M];
    int n = 1;
    parent[0] = -1;
    rank[0] = 0;
    p[0] = 1.0;
    depth[0] = 0;
    double e = 1.0;
    while (n < M) {
        int bp = -1, br = -1;
        double best = -1.0;
        for (int u = 0; u < n; ++u) {
            if (depth[u] >= K)
                continue;
            for (int r = 0; r < R; ++r) {
                int used = 0;
                for (int w = 0; w < n; ++w)
                    if (parent[w] == u && rank[w] == r)
                        used = 1;
                if (used)
                    continue;
                double q = p[u] * acc[(size_t)depth[u] * R + r];
                if (q > best) {
                    best = q;
                    bp = u;
                    br = r;
                }
            }
        }
        if (bp < 0)
            break;
        parent[n] = bp;
        rank[n] = br;
        p[n] = best;
        depth[n] = depth[bp] + 1;
        e += best;
        ++n;
    }
    if (expect)
        *expect = e;
    return n;
}

/* Choice of the verification width (section 3.3.1: both the width and the tree
 * determine the acceptance length, and a larger width costs a longer step;
 * section 3.3.2: the candidate widths are profiled on the hardware).  For
 * every candidate width the tree is designed as above; the width kept is the
 * one with the most expected accepted tokens per unit of measured step time
 * (the first such width on ties).  latency[i] is the measured step time at
 * widths[i].  Returns the index of the chosen width; rate[i] (optional) gets
 * expected tokens per unit time for every candidate. */
int orc_choose_width(const double *acc, int K, int R, const int32_t *widths,
                     const double *latency, int n, double *rate)
{
    int32_t parent[ORC_MAX_M], rank[ORC_MAX_M];
    int best = 0;
    double best_rate = -1.0;
    for (int i = 0; i < n; ++i) {
        double e;
        orc_tree_build(acc, K, R, widths[i], parent, rank, &e);
        double r = e / latency[i];
        if (rate)
            rate[i] = r;
        if (r > best_rate) {
            best_rate = r;
            best = i;
        }
    }
    return best;
}

/* ------------------------------------------- attention under a given mask -- */

/* Eq. (1) under an arbitrary verification pattern (section 2.3 shows three:
 * the token tree of multi-head drafting, the several sequences of a draft
 * model, the n-gram pattern of Lookahead): mask[i*M + j] != 0 says that drafted
 * token i is related to drafted token j; every drafted token sees the whole
 * committed cache.  Same layout and arithmetic as orc_tree_attention, which is
 * the special case mask = ancestor-or-self.  A row that sees no key at all
 * (empty cache and an all-zero mask row) gives zeros. */
void orc_masked_attention(real *out, const real *q, const uint16_t *kc, const uint16_t *vc,
                          const uint8_t *mask, int M, int kv_len, int nh, int d,
                          int64_t stride_head, int64_t stride_tok, real scale)
{
    int T = kv_len + M;
    real *s = (real *)malloc((size_t)T * sizeof(real));
    for (int h = 0; h < nh; ++h)
        for (int i = 0; i < M; ++i) {
            const real *qi = q + ((size_t)i * nh + h) * d;
            real *oi = out + ((size_t)i * nh + h) * d;
            real mx = -INFINITY;
            int seen = 0;
            for (int t = 0; t < T; ++t) {
                if (t >= kv_len && !mask[(size_t)i * M + (t - kv_len)])
                    continue;
                const uint16_t *kt = kc + h * stride_head + t * stride_tok;
                real dot = 0;
                for (int c = 0; c < d; ++c)
                    dot += qi[c] * widen(kt[c]);
                s[t] = dot * scale;
                if (s[t] > mx)
                    mx = s[t];
                ++seen;
            }
            for (int c = 0; c < d; ++c)
                oi[c] = 0;
            if (!seen)
                continue;
            real denom = 0;
            for (int t = 0; t < T; ++t) {
                if (t >= kv_len && !mask[(size_t)i * M + (t - kv_len)])
                    continue;
                s[t] = (real)exp((double)(s[t] - mx));
                denom += s[t];
            }
            for (int t = 0; t < T; ++t) {
                if (t >= kv_len && !mask[(size_t)i * M + (t - kv_len)])
                    continue;
                real p = s[t] / denom;
                const uint16_t *vt = vc + h * stride_head + t * stride_tok;
                for (int c = 0; c < d; ++c)
                    oi[c] += p * widen(vt[c]);
            }
        }
    free(s);
}

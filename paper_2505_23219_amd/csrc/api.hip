// Host side of the C ABI (include/ghd.h): argument checks, workspace layout,
// launch sequence of the verification step.  No device code here.
#include "common.h"

namespace ghd {

static int g_last_hip_error = 0;

ghd_status hip_fail(hipError_t e)
{
    g_last_hip_error = (int)e;
    return GHD_ERR_HIP;
}

ghd_status check_launch()
{
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? GHD_OK : hip_fail(e);
}

// ---- optional timing of the skinny-GEMM launches (benchmark support) ---------
// When enabled, every launch_gemm call made through timed_gemm is bracketed by a
// pair of HIP events on its stream; the caller reads the summed duration after
// synchronising.  Off by default: the hot path records nothing.
static bool g_prof_on = false;
static const int kProfMax = 512;
static hipEvent_t g_prof_ev[2 * kProfMax];
static int g_prof_made = 0, g_prof_used = 0;

static ghd_status timed_gemm(const GemmPlan& p, const void* Wp, const half_t* x, int64_t ldx,
                             float* out, int64_t ld, int M, int N, int K, hipStream_t st)
{
    if (!g_prof_on || g_prof_used >= kProfMax) return launch_gemm(p, Wp, x, ldx, out, ld, M, N, K, st);
    while (g_prof_made < 2 * (g_prof_used + 1)) {
        hipError_t e = hipEventCreate(&g_prof_ev[g_prof_made]);
        if (e != hipSuccess) return hip_fail(e);
        ++g_prof_made;
    }
    (void)hipEventRecord(g_prof_ev[2 * g_prof_used], st);
    ghd_status s = launch_gemm(p, Wp, x, ldx, out, ld, M, N, K, st);
    (void)hipEventRecord(g_prof_ev[2 * g_prof_used + 1], st);
    ++g_prof_used;
    return s;
}

static inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

// ---- workspace carving -------------------------------------------------------
struct Carver {
    char* base;
    size_t off;
    explicit Carver(void* p) : base((char*)p), off(0) {}
    template <class T>
    T* take(size_t count)
    {
        T* r = (T*)(base ? base + off : nullptr);
        off = align_up(off + count * sizeof(T), 256);
        return r;
    }
};

static size_t gemm_part_floats(int M, int N, int K)
{
    GemmPlan p = plan_gemm(M, N, K);
    return (size_t)p.S * M * ((size_t)p.ntiles * 16);
}

struct LayerWs {
    int32_t* depth;
    uint64_t* mask;
    float2* rope;
    half_t *n16, *q16, *o16, *a16;
    float *part, *o_part, *ml_part;
    float* x;       // residual stream (stack only)
    int32_t* amax;  // unused by the layer
    size_t bytes;
};

static LayerWs carve(void* ws, const ghd_model_cfg* c, int M, int kv_len, bool stack)
{
    Carver cv(ws);
    LayerWs w;
    w.depth = cv.take<int32_t>(GHD_MAX_M);
    w.mask = cv.take<uint64_t>(2 * GHD_MAX_M);
    w.rope = cv.take<float2>((size_t)M * (c->d / 2));
    w.n16 = cv.take<half_t>((size_t)M * c->H);
    w.q16 = cv.take<half_t>((size_t)M * c->H);
    w.o16 = cv.take<half_t>((size_t)M * c->H);
    w.a16 = cv.take<half_t>((size_t)M * c->F);
    size_t pf = gemm_part_floats(M, 3 * c->H, c->H);
    size_t t;
    if ((t = gemm_part_floats(M, c->H, c->H)) > pf) pf = t;
    if ((t = gemm_part_floats(M, 2 * c->F, c->H)) > pf) pf = t;
    if ((t = gemm_part_floats(M, c->H, c->F)) > pf) pf = t;
    if (stack && (t = gemm_part_floats(M, c->V, c->H)) > pf) pf = t;
    w.part = cv.take<float>(pf);
    AttnPlan a = plan_attention(M, kv_len, c->nh);
    w.o_part = cv.take<float>((size_t)a.P * c->nh * M * c->d);
    w.ml_part = cv.take<float>((size_t)a.P * c->nh * M * 2);
    w.x = stack ? cv.take<float>((size_t)M * c->H) : nullptr;
    w.amax = nullptr;
    w.bytes = cv.off;
    return w;
}

static ghd_status check_cfg(const ghd_model_cfg* c, int M, int kv_len)
{
    if (!c) return GHD_ERR_NULL;
    if (M < 1 || M > GHD_MAX_M || kv_len < 0) return GHD_ERR_SHAPE;
    if ((c->d != 64 && c->d != 128) || c->nh < 1 || c->H != c->nh * c->d) return GHD_ERR_SHAPE;
    if (c->F < 8 || (c->F % 8) != 0 || c->L < 1 || c->V < 1) return GHD_ERR_SHAPE;
    if (!(c->rope_base > 0.f) || !(c->rms_eps >= 0.f)) return GHD_ERR_SHAPE;
    if ((int64_t)kv_len + M > (int64_t)c->kv_capacity) return GHD_ERR_CAPACITY;
    return GHD_OK;
}

// One layer with n16 = rmsnorm(x) * g_attn already in ws.n16.  On return x holds the
// layer's output and, if next_g is given, ws.n16 = rmsnorm(x) * next_g.
static ghd_status run_layer(const ghd_model_cfg* c, const ghd_layer_weights* w, const ghd_kv* kv,
                            float* x, int M, int kv_len, const LayerWs& ws, const half_t* next_g,
                            hipStream_t st)
{
    const int H = c->H, F = c->F;
    const int64_t stride_head = (int64_t)c->kv_capacity * c->d, stride_tok = c->d;
    ghd_status s;
    // MHA block: QKV linear, rotate + append, tree attention, output linear
    GemmPlan p = plan_gemm(M, 3 * H, H);
    int64_t ld = (int64_t)p.ntiles * 16;
    if ((s = timed_gemm(p, w->Wqkv, ws.n16, H, ws.part, ld, M, 3 * H, H, st))) return s;
    if ((s = launch_qkv_epilogue(ws.part, p.S, ld, ws.rope, ws.q16, (half_t*)kv->k, (half_t*)kv->v,
                                 M, c->nh, c->d, kv_len, stride_head, stride_tok, st)))
        return s;
    AttnPlan a = plan_attention(M, kv_len, c->nh);
    if ((s = launch_attention(a, ws.o16, ws.q16, (const half_t*)kv->k, (const half_t*)kv->v, ws.mask,
                              M, kv_len, c->nh, c->d, stride_head, stride_tok,
                              1.0f / sqrtf((float)c->d), ws.o_part, ws.ml_part, st)))
        return s;
    p = plan_gemm(M, H, H);
    ld = (int64_t)p.ntiles * 16;
    if ((s = timed_gemm(p, w->Wo, ws.o16, H, ws.part, ld, M, H, H, st))) return s;
    if ((s = launch_residual_norm(x, nullptr, ws.part, p.S, ld, (const half_t*)w->g_ffn, ws.n16, M,
                                  H, c->rms_eps, st)))
        return s;
    // MLP block: gate|up linear + SwiGLU, down linear
    p = plan_gemm(M, 2 * F, H);
    ld = (int64_t)p.ntiles * 16;
    if ((s = timed_gemm(p, w->Wgu, ws.n16, H, ws.part, ld, M, 2 * F, H, st))) return s;
    if ((s = launch_swiglu(ws.part, p.S, ld, ws.a16, M, F, st))) return s;
    p = plan_gemm(M, H, F);
    ld = (int64_t)p.ntiles * 16;
    if ((s = timed_gemm(p, w->Wdown, ws.a16, F, ws.part, ld, M, H, F, st))) return s;
    return launch_residual_norm(x, nullptr, ws.part, p.S, ld, next_g, ws.n16, M, H, c->rms_eps, st);
}

}  // namespace ghd

using namespace ghd;

extern "C" {

const char* ghd_status_str(ghd_status s)
{
    switch (s) {
    case GHD_OK: return "ok";
    case GHD_ERR_NULL: return "null pointer";
    case GHD_ERR_SHAPE: return "unsupported or inconsistent shape";
    case GHD_ERR_TREE: return "parent[] is not a topologically ordered rooted tree";
    case GHD_ERR_CAPACITY: return "kv_len + M exceeds the cache capacity";
    case GHD_ERR_WORKSPACE: return "workspace missing or too small";
    case GHD_ERR_ALIGN: return "pointer or leading dimension not 16-byte aligned";
    case GHD_ERR_HIP: return "HIP call failed";
    default: return "unknown status";
    }
}

int ghd_last_hip_error(void) { return g_last_hip_error; }

ghd_status ghd_tree_validate(const int32_t* parent_host, int M)
{
    if (!parent_host) return GHD_ERR_NULL;
    if (M < 1 || M > GHD_MAX_M) return GHD_ERR_SHAPE;
    if (parent_host[0] != -1) return GHD_ERR_TREE;
    for (int i = 1; i < M; ++i)
        if (parent_host[i] < 0 || parent_host[i] >= i) return GHD_ERR_TREE;
    return GHD_OK;
}

ghd_status ghd_tree_mask(const int32_t* parent_dev, int M, uint64_t* mask_dev, void* stream)
{
    if (!parent_dev || !mask_dev) return GHD_ERR_NULL;
    if (M < 1 || M > GHD_MAX_M) return GHD_ERR_SHAPE;
    return launch_tree_setup(parent_dev, M, 0, 0, 1.f, nullptr, mask_dev, nullptr,
                             (hipStream_t)stream);
}

size_t ghd_packed_weight_bytes(int N, int K)
{
    if (N < 1 || K < 1) return 0;
    return (size_t)ceil_div(N, 16) * ceil_div(K, 32) * 1024;
}

ghd_status ghd_pack_weight(void* dst, const void* src, int N, int K, void* stream)
{
    if (!dst || !src) return GHD_ERR_NULL;
    if (N < 1 || K < 1) return GHD_ERR_SHAPE;
    if (!aligned16(dst)) return GHD_ERR_ALIGN;
    return launch_pack(dst, src, N, K, (hipStream_t)stream);
}

size_t ghd_linear_workspace_bytes(int M, int N, int K)
{
    if (M < 1 || M > GHD_MAX_M || N < 1 || K < 1) return 0;
    return align_up(gemm_part_floats(M, N, K) * sizeof(float), 256);
}

ghd_status ghd_linear_skinny(void* y, const void* x, const void* Wp, int M, int N, int K,
                             int64_t ldx, int64_t ldy, uint32_t flags, void* ws, size_t ws_bytes,
                             void* stream)
{
    if (!y || !x || !Wp) return GHD_ERR_NULL;
    if (M < 1 || M > GHD_MAX_M || N < 1 || K < 8 || (K % 8) != 0) return GHD_ERR_SHAPE;
    if (ldx < K || ldy < N || flags > GHD_OUT_F16) return GHD_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(Wp) || !aligned16(y) || (ldx % 8) != 0) return GHD_ERR_ALIGN;
    if (!ws) return GHD_ERR_WORKSPACE;
    if (!aligned16(ws)) return GHD_ERR_ALIGN;
    if (ws_bytes < ghd_linear_workspace_bytes(M, N, K)) return GHD_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    GemmPlan p = plan_gemm(M, N, K);
    int64_t ld = (int64_t)p.ntiles * 16;
    ghd_status s = timed_gemm(p, Wp, (const half_t*)x, ldx, (float*)ws, ld, M, N, K, st);
    if (s) return s;
    return launch_reduce_out(y, ldy, flags == GHD_OUT_F16, (const float*)ws, p.S, ld, M, N, st);
}

size_t ghd_attention_workspace_bytes(int M, int kv_len, int nh, int d)
{
    if (M < 1 || M > GHD_MAX_M || kv_len < 0 || nh < 1 || (d != 64 && d != 128)) return 0;
    AttnPlan a = plan_attention(M, kv_len, nh);
    size_t b = align_up(2 * GHD_MAX_M * sizeof(uint64_t), 256);
    b += align_up((size_t)a.P * nh * M * d * sizeof(float), 256);
    b += align_up((size_t)a.P * nh * M * 2 * sizeof(float), 256);
    return b;
}

ghd_status ghd_tree_attention(void* out, const void* q, const void* k_cache, const void* v_cache,
                              const int32_t* parent_dev, int M, int kv_len, int nh, int d,
                              int64_t stride_head, int64_t stride_tok, float scale, void* ws,
                              size_t ws_bytes, void* stream)
{
    if (!out || !q || !k_cache || !v_cache || !parent_dev) return GHD_ERR_NULL;
    if (M < 1 || M > GHD_MAX_M || kv_len < 0 || nh < 1 || (d != 64 && d != 128))
        return GHD_ERR_SHAPE;
    if (stride_tok < d || stride_head < 0) return GHD_ERR_SHAPE;
    if (!aligned16(out) || !aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) ||
        (stride_tok % 8) != 0 || (stride_head % 8) != 0)
        return GHD_ERR_ALIGN;
    if (!ws) return GHD_ERR_WORKSPACE;
    if (!aligned16(ws)) return GHD_ERR_ALIGN;
    if (ws_bytes < ghd_attention_workspace_bytes(M, kv_len, nh, d)) return GHD_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    AttnPlan a = plan_attention(M, kv_len, nh);
    Carver cv(ws);
    uint64_t* mask = cv.take<uint64_t>(2 * GHD_MAX_M);
    float* o_part = cv.take<float>((size_t)a.P * nh * M * d);
    float* ml_part = cv.take<float>((size_t)a.P * nh * M * 2);
    ghd_status s = launch_tree_setup(parent_dev, M, kv_len, d, 1.f, nullptr, mask, nullptr, st);
    if (s) return s;
    return launch_attention(a, (half_t*)out, (const half_t*)q, (const half_t*)k_cache,
                            (const half_t*)v_cache, mask, M, kv_len, nh, d, stride_head, stride_tok,
                            scale, o_part, ml_part, st);
}

size_t ghd_workspace_bytes(const ghd_model_cfg* cfg, int M, int kv_len)
{
    if (check_cfg(cfg, M, kv_len) != GHD_OK) return 0;
    return carve(nullptr, cfg, M, kv_len, true).bytes;
}

ghd_status ghd_verify_layer(const ghd_model_cfg* cfg, const ghd_layer_weights* w, const ghd_kv* kv,
                            float* x, const int32_t* parent_dev, int M, int kv_len, void* ws,
                            size_t ws_bytes, void* stream)
{
    if (!cfg || !w || !kv || !x || !parent_dev) return GHD_ERR_NULL;
    if (!w->g_attn || !w->Wqkv || !w->Wo || !w->g_ffn || !w->Wgu || !w->Wdown || !kv->k || !kv->v)
        return GHD_ERR_NULL;
    ghd_status s = check_cfg(cfg, M, kv_len);
    if (s) return s;
    if (!aligned16(x) || !aligned16(kv->k) || !aligned16(kv->v) || !aligned16(w->Wqkv) ||
        !aligned16(w->Wo) || !aligned16(w->Wgu) || !aligned16(w->Wdown))
        return GHD_ERR_ALIGN;
    if (!ws) return GHD_ERR_WORKSPACE;
    if (!aligned16(ws)) return GHD_ERR_ALIGN;
    if (ws_bytes < ghd_workspace_bytes(cfg, M, kv_len)) return GHD_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    LayerWs lw = carve(ws, cfg, M, kv_len, true);
    if ((s = launch_tree_setup(parent_dev, M, kv_len, cfg->d, cfg->rope_base, lw.depth, lw.mask,
                               lw.rope, st)))
        return s;
    if ((s = launch_residual_norm(x, nullptr, nullptr, 0, 0, (const half_t*)w->g_attn, lw.n16, M,
                                  cfg->H, cfg->rms_eps, st)))
        return s;
    return run_layer(cfg, w, kv, x, M, kv_len, lw, nullptr, st);
}

ghd_status ghd_verify_stack(const ghd_model_cfg* cfg, const ghd_layer_weights* layers_host,
                            const ghd_kv* kv_host, const void* g_final, const void* Wlm,
                            const void* x_in, const int32_t* parent_dev, int M, int kv_len,
                            float* logits, float* x_out, void* ws, size_t ws_bytes, void* stream)
{
    if (!cfg || !layers_host || !kv_host || !g_final || !Wlm || !x_in || !parent_dev || !logits)
        return GHD_ERR_NULL;
    ghd_status s = check_cfg(cfg, M, kv_len);
    if (s) return s;
    for (int l = 0; l < cfg->L; ++l) {
        const ghd_layer_weights* w = layers_host + l;
        if (!w->g_attn || !w->Wqkv || !w->Wo || !w->g_ffn || !w->Wgu || !w->Wdown ||
            !kv_host[l].k || !kv_host[l].v)
            return GHD_ERR_NULL;
        if (!aligned16(w->Wqkv) || !aligned16(w->Wo) || !aligned16(w->Wgu) ||
            !aligned16(w->Wdown) || !aligned16(kv_host[l].k) || !aligned16(kv_host[l].v))
            return GHD_ERR_ALIGN;
    }
    if (!aligned16(x_in) || !aligned16(Wlm) || !aligned16(logits) || (x_out && !aligned16(x_out)))
        return GHD_ERR_ALIGN;
    if (!ws) return GHD_ERR_WORKSPACE;
    if (!aligned16(ws)) return GHD_ERR_ALIGN;
    if (ws_bytes < ghd_workspace_bytes(cfg, M, kv_len)) return GHD_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    LayerWs lw = carve(ws, cfg, M, kv_len, true);
    const int H = cfg->H;
    if ((s = launch_tree_setup(parent_dev, M, kv_len, cfg->d, cfg->rope_base, lw.depth, lw.mask,
                               lw.rope, st)))
        return s;
    // x = widen(x_in); n16 = rmsnorm(x) * g_attn of layer 0
    if ((s = launch_residual_norm(lw.x, (const half_t*)x_in, nullptr, 0, 0,
                                  (const half_t*)layers_host[0].g_attn, lw.n16, M, H, cfg->rms_eps,
                                  st)))
        return s;
    for (int l = 0; l < cfg->L; ++l) {
        const half_t* next_g = (const half_t*)(l + 1 < cfg->L ? layers_host[l + 1].g_attn : g_final);
        if ((s = run_layer(cfg, layers_host + l, kv_host + l, lw.x, M, kv_len, lw, next_g, st)))
            return s;
    }
    if (x_out) {
        hipError_t e = hipMemcpyAsync(x_out, lw.x, (size_t)M * H * sizeof(float),
                                      hipMemcpyDeviceToDevice, st);
        if (e != hipSuccess) return hip_fail(e);
    }
    // LM head on the final norm
    GemmPlan p = plan_gemm(M, cfg->V, H);
    int64_t ld = (int64_t)p.ntiles * 16;
    if ((s = timed_gemm(p, Wlm, lw.n16, H, lw.part, ld, M, cfg->V, H, st))) return s;
    return launch_reduce_out(logits, cfg->V, false, lw.part, p.S, ld, M, cfg->V, st);
}

size_t ghd_accept_workspace_bytes(int M)
{
    if (M < 1 || M > GHD_MAX_M) return 0;
    return align_up(GHD_MAX_M * sizeof(int32_t), 256);
}

ghd_status ghd_accept_greedy(const float* logits, const int32_t* tokens_dev,
                             const int32_t* parent_dev, int M, int V, int32_t* res_dev,
                             int32_t* amax_dev, void* ws, size_t ws_bytes, void* stream)
{
    if (!logits || !tokens_dev || !parent_dev || !res_dev) return GHD_ERR_NULL;
    if (M < 1 || M > GHD_MAX_M || V < 1) return GHD_ERR_SHAPE;
    if (!ws) return GHD_ERR_WORKSPACE;
    if (((uintptr_t)ws & 3) != 0) return GHD_ERR_ALIGN;
    if (ws_bytes < ghd_accept_workspace_bytes(M)) return GHD_ERR_WORKSPACE;
    return launch_accept(logits, tokens_dev, parent_dev, M, V, res_dev, amax_dev, (int32_t*)ws,
                         (hipStream_t)stream);
}

/* Tuning hooks for sweeps (not part of the documented ABI). */
void ghd_debug_set_gemm_plan(int nt, int s, int nw, int lds) { set_gemm_override(nt, s, nw, lds); }
void ghd_debug_set_attn_splits(int p) { set_attn_override(p); }

/* Benchmark support: time the skinny-GEMM launches of ghd_verify_layer/stack with
 * HIP events.  ghd_debug_profile_gemm(1) starts a fresh measurement,
 * ghd_debug_profile_gemm(0) stops it; after synchronising the stream,
 * ghd_debug_profile_read returns the number of launches and their summed
 * duration in milliseconds. */
void ghd_debug_profile_gemm(int enable)
{
    g_prof_on = enable != 0;
    if (enable) g_prof_used = 0;
}

int ghd_debug_profile_read(float* total_ms)
{
    float tot = 0.f;
    for (int i = 0; i < g_prof_used; ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, g_prof_ev[2 * i], g_prof_ev[2 * i + 1]) == hipSuccess) tot += ms;
    }
    if (total_ms) *total_ms = tot;
    return g_prof_used;
}

}  // extern "C"

// Host side of the C ABI (include/ghd.h): argument checks, workspace layout and the
// launches of the verification step.  No device code here.
#include "fused.h"

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

// ---- optional timing of the persistent kernel (benchmark support) -----------------
// When enabled, every launch of the persistent kernel is bracketed by a pair of HIP
// events on its stream; the caller reads the summed duration after synchronising.
// Off by default: the hot path records nothing.
static int g_prof_mode = -1;   // -1 off, else the FusedArgs::mode whose launches are timed
static const int kProfMax = 256;
static hipEvent_t g_prof_ev[2 * kProfMax];
static int g_prof_made = 0, g_prof_used = 0;

static ghd_status timed_fused(const FusedArgs& a, hipStream_t st)
{
    if (g_prof_mode != a.mode || g_prof_used >= kProfMax) return launch_fused(a, st);
    while (g_prof_made < 2 * (g_prof_used + 1)) {
        hipError_t e = hipEventCreate(&g_prof_ev[g_prof_made]);
        if (e != hipSuccess) return hip_fail(e);
        ++g_prof_made;
    }
    (void)hipEventRecord(g_prof_ev[2 * g_prof_used], st);
    ghd_status s = launch_fused(a, st);
    (void)hipEventRecord(g_prof_ev[2 * g_prof_used + 1], st);
    ++g_prof_used;
    return s;
}

// benchmark support: run the QKV layer and the attention as two launches even where one would do
static bool g_split_qkv_attn = false;

static inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

// Number of workgroups of the persistent kernel; 256 (the MI355X's compute units) when
// no device can be queried, so that workspace sizes are defined on a GPU-less host.
static int grid_for_sizing()
{
    int g = fused_grid_size();
    return g > 0 ? g : 256;
}

static int mpad_of(int M)
{
    int mt = (M + 15) / 16;
    return (mt <= 1 ? 1 : mt <= 2 ? 2 : mt <= 4 ? 4 : 8) * 16;
}

// Is a linear layer of this shape within what the kernel's 32-bit share arithmetic covers?
static bool linear_shape_ok(int N, int K)
{
    if (N < 1 || K < 8 || (K % 8) != 0) return false;
    const WLayout lay = w_layout(N, K);
    // units of one XCD times shares of one XCD must fit 32 bits
    return ((int64_t)lay.nitems * lay.nks / 8 + lay.nks) * (kMaxShares / 8) < (1ll << 31);
}

// Fills in how the launch is cut (see plan_linear); false if the shape needs more work shares
// than the counters are laid out for.
static bool fill_plan(FusedArgs& a, int M, int N, int K)
{
    LinPlan pl;
    if (!plan_linear(M, N, K, grid_for_sizing(), &pl)) return false;
    a.lin_slots = pl.slots;
    a.lin_passes = pl.passes;
    a.lin_whole = pl.whole;
    return true;
}

// ---- workspace carving ---------------------------------------------------------
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

struct Ws {
    uint32_t* sync;
    float *part, *o_part, *ml_part, *x, *ss;
    half_t *q16, *o16, *a16, *xg16, *xpk;
    float2* rope;
    float2* amax_tbl;   // per (16-column tile of the LM head, row): largest logit and its column
    uint64_t* mask;
    size_t bytes;
};

// what: 0 = whole model (layer / stack), 1 = linear only (K = its input features),
// 2 = attention only
static Ws carve(void* ws, int what, int M, int H, int F, int d, int K = 0, int V = 0)
{
    Carver cv(ws);
    Ws w = {};
    const int G = grid_for_sizing();
    const int Mpad = mpad_of(M), mtp = Mpad / 16;
    w.sync = cv.take<uint32_t>(kSyncWords);
    if (what != 2) w.part = cv.take<float>(linear_part_floats(M, G));
    if (what == 1) w.xpk = cv.take<half_t>(xpk_halves(K, mtp));
    if (what != 1) {
        w.mask = cv.take<uint64_t>(2 * GHD_MAX_M);
        w.o_part = cv.take<float>((size_t)G * Mpad * d);
        w.ml_part = cv.take<float>((size_t)G * Mpad * 2);
    }
    if (what == 0) {
        w.rope = cv.take<float2>((size_t)GHD_MAX_M * (d / 2));
        w.x = cv.take<float>((size_t)M * H);
        w.ss = cv.take<float>((size_t)(H / 16) * Mpad);
        w.q16 = cv.take<half_t>((size_t)M * H);
        w.o16 = cv.take<half_t>(xpk_halves(H, mtp));
        w.a16 = cv.take<half_t>(xpk_halves(F, mtp));
        w.xg16 = cv.take<half_t>(xpk_halves(H, mtp));
        w.amax_tbl = cv.take<float2>((size_t)((V + 15) / 16) * Mpad);
    }
    w.bytes = cv.off;
    return w;
}

static ghd_status check_cfg(const ghd_model_cfg* c, int M, int kv_len)
{
    if (!c) return GHD_ERR_NULL;
    if (M < 1 || M > GHD_MAX_M || kv_len < 0) return GHD_ERR_SHAPE;
    if ((c->d != 64 && c->d != 128) || c->nh < 1 || c->nh > 256 || c->H != c->nh * c->d)
        return GHD_ERR_SHAPE;
    if (c->F < 8 || (c->F % 8) != 0 || c->F > (1 << 20) || c->L < 1 || c->L > kMaxLayers || c->V < 1) return GHD_ERR_SHAPE;
    if (c->H > 65536 || c->V > (1 << 20)) return GHD_ERR_SHAPE;
    if (!linear_shape_ok(3 * c->H, c->H) || !linear_shape_ok(2 * c->F, c->H) ||
        !linear_shape_ok(c->H, c->F) || !linear_shape_ok(c->V, c->H))
        return GHD_ERR_SHAPE;
    {
        // every linear layer of the model must fit the work-share plan at this M
        LinPlan pl;
        const int G = grid_for_sizing();
        if (!plan_linear(M, 3 * c->H, c->H, G, &pl) || !plan_linear(M, c->H, c->H, G, &pl) ||
            !plan_linear(M, 2 * c->F, c->H, G, &pl) || !plan_linear(M, c->H, c->F, G, &pl) ||
            !plan_linear(M, c->V, c->H, G, &pl))
            return GHD_ERR_SHAPE;
    }
    if (!(c->rope_base > 0.f) || !(c->rms_eps >= 0.f)) return GHD_ERR_SHAPE;
    if ((int64_t)kv_len + M > (int64_t)c->kv_capacity || (c->kv_capacity % 8) != 0) return GHD_ERR_CAPACITY;
    if ((int64_t)c->kv_capacity * c->d >= (1ll << 31)) return GHD_ERR_SHAPE;   // 32-bit offsets inside a head
    return GHD_OK;
}

static void fill_common(FusedArgs& a, const ghd_model_cfg* c, const Ws& w, int M, int kv_len)
{
    a.M = M;
    a.Mpad = mpad_of(M);
    a.kv_len = kv_len;
    a.H = c->H;
    a.nh = c->nh;
    a.d = c->d;
    a.F = c->F;
    a.stride_head = (int64_t)c->kv_capacity * c->d;
    a.stride_tok = c->d;
    a.v_stride_head = (int64_t)c->kv_capacity * c->d;
    a.v_stride_ch = c->kv_capacity;
    a.eps = c->rms_eps;
    a.scale_log2e = 1.4426950408889634f / sqrtf((float)c->d);
    a.sync = w.sync;
    a.part = w.part;
    a.o_part = w.o_part;
    a.ml_part = w.ml_part;
    a.x = w.x;
    a.ss = w.ss;
    a.q16 = w.q16;
    a.o16 = w.o16;
    a.a16 = w.a16;
    a.xg16 = w.xg16;
    a.rope = w.rope;
    a.mask = w.mask;
}

static ghd_status check_layer(const ghd_layer_weights* w, const ghd_kv* kv)
{
    if (!w->g_attn || !w->Wqkv || !w->Wo || !w->g_ffn || !w->Wgu || !w->Wdown || !kv->k || !kv->v)
        return GHD_ERR_NULL;
    if (!aligned16(w->g_attn) || !aligned16(w->Wqkv) || !aligned16(w->Wo) || !aligned16(w->g_ffn) ||
        !aligned16(w->Wgu) || !aligned16(w->Wdown) || !aligned16(kv->k) || !aligned16(kv->v))
        return GHD_ERR_ALIGN;
    return GHD_OK;
}


// ---- the step as a sequence of single-phase launches ------------------------------
// Every linear layer is one launch of the persistent GEMM kernel (all compute units,
// equal contiguous shares of the packed weight stream).  The layer's element-wise work
// rides on those launches: RMSNorm is applied while the fp32 residual stream is staged as
// the GEMM's x operand (from per-tile sums of squares left by the producer), and the
// finishing workgroups rotate q/k and append K/V (QKV), apply SwiGLU (gate|up), or add
// into the residual stream and leave the new sums of squares (output and down linears).
// A layer is five launches: QKV, attention, output, gate|up, down.
struct LinearCall {
    const void* Wp;
    int N, K, epi;
    const half_t* in16;   // fp16 input, packed activation layout
    bool rscale;          // the input is xg16: apply the RMSNorm row factor in the epilogue
    const half_t* gnext;  // EPI_RESID: gain of the norm that follows, or nullptr
    void* out;
    int64_t ldo;
    const ghd_kv* kv;     // EPI_QKV
    int cnt;
    uint32_t epoch;
    float2* amax_tbl;     // EPI_STORE_F32: per-tile row maxima (optional)
};

static ghd_status fill_linear(FusedArgs& a, const ghd_model_cfg* c, const Ws& w, float* x, int M, int kv_len,
                              const LinearCall& lc)
{
    fill_common(a, c, w, M, kv_len);
    a.x = x;
    a.mode = MODE_LINEAR;
    a.lin_W = (const half8*)lc.Wp;
    a.lin_N = lc.N;
    a.lin_K = lc.K;
    a.lin_epi = lc.epi;
    if (!fill_plan(a, M, lc.N, lc.K)) return GHD_ERR_SHAPE;
    a.lin_x = lc.in16;
    a.lin_rscale = lc.rscale;
    a.lin_gnext = lc.gnext;
    a.lin_y = lc.out;
    a.lin_ldy = lc.ldo;
    a.lin_kc = lc.kv ? (half_t*)lc.kv->k : nullptr;
    a.lin_vc = lc.kv ? (half_t*)lc.kv->v : nullptr;
    a.lin_cnt = lc.cnt;
    a.lin_epoch = lc.epoch;
    a.lin_amax = lc.amax_tbl;
    return GHD_OK;
}

static void fill_attention(FusedArgs& a, const Ws& w, const ghd_kv* kv, uint32_t epoch)
{
    a.att_q = w.q16;
    a.att_k = (const half_t*)kv->k;
    a.att_v = (const half_t*)kv->v;
    a.att_out = w.o16;
    a.att_out_packed = 1;
    a.att_epoch = epoch;
}

static ghd_status step_linear(const ghd_model_cfg* c, const Ws& w, float* x, int M, int kv_len,
                              const LinearCall& lc, hipStream_t st)
{
    FusedArgs a = {};
    ghd_status s = fill_linear(a, c, w, x, M, kv_len, lc);
    if (s) return s;
    return timed_fused(a, st);
}

static ghd_status step_attention(const ghd_model_cfg* c, const Ws& w, const ghd_kv* kv, int M,
                                 int kv_len, uint32_t epoch, hipStream_t st)
{
    FusedArgs a = {};
    fill_common(a, c, w, M, kv_len);
    a.mode = MODE_ATTN;
    fill_attention(a, w, kv, epoch);
    return timed_fused(a, st);
}

// The QKV layer and the attention of a layer: one launch where the shape allows it (see
// qkv_attn_available), else two.
static ghd_status step_qkv_attention(const ghd_model_cfg* c, const Ws& w, const ghd_kv* kv, float* x, int M,
                                     int kv_len, const LinearCall& qkv, uint32_t layer, hipStream_t st)
{
    FusedArgs a = {};
    ghd_status s = fill_linear(a, c, w, x, M, kv_len, qkv);
    if (s) return s;
    if (!g_split_qkv_attn && qkv_attn_available(M, a.lin_slots, a.lin_passes, c->d, c->nh)) {
        a.mode = MODE_QKV_ATTN;
        fill_attention(a, w, kv, layer);
        return timed_fused(a, st);
    }
    if ((s = timed_fused(a, st))) return s;
    return step_attention(c, w, kv, M, kv_len, layer, st);
}

// One decoder layer on the residual stream x.  On entry (and again on return) w.ss holds
// x's per-tile sums of squares and w.xg16 = fp16(x * g) for the gain of the norm that
// comes next: g_attn of this layer on entry, next_g on return (skipped if next_g is null).
static ghd_status run_layer(const ghd_model_cfg* c, const ghd_layer_weights* lw, const ghd_kv* kv,
                            float* x, int M, int kv_len, const Ws& w, const half_t* next_g,
                            uint32_t layer, hipStream_t st)
{
    const int H = c->H, F = c->F;
    ghd_status s;
    LinearCall qkv = {lw->Wqkv, 3 * H, H, EPI_QKV, w.xg16, true, nullptr, nullptr, 0, kv, kCntQkv, layer, nullptr};
    if ((s = step_qkv_attention(c, w, kv, x, M, kv_len, qkv, layer, st))) return s;
    LinearCall wo = {lw->Wo, H, H, EPI_RESID, w.o16, false, (const half_t*)lw->g_ffn, x, H, nullptr, kCntWo, layer, nullptr};
    if ((s = step_linear(c, w, x, M, kv_len, wo, st))) return s;
    LinearCall gu = {lw->Wgu, 2 * F, H, EPI_SWIGLU, w.xg16, true, nullptr, w.a16, F, nullptr, kCntGu, layer, nullptr};
    if ((s = step_linear(c, w, x, M, kv_len, gu, st))) return s;
    LinearCall down = {lw->Wdown, H, F, EPI_RESID, w.a16, false, next_g, x, H, nullptr, kCntDown, layer, nullptr};
    return step_linear(c, w, x, M, kv_len, down, st);
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

size_t ghd_tree_mask_workspace_bytes(void) { return align_up(kSyncWords * sizeof(uint32_t), 256); }

ghd_status ghd_tree_mask(const int32_t* parent_dev, int M, uint64_t* mask_dev, void* ws,
                         size_t ws_bytes, void* stream)
{
    if (!parent_dev || !mask_dev) return GHD_ERR_NULL;
    if (M < 1 || M > GHD_MAX_M) return GHD_ERR_SHAPE;
    if (!ws) return GHD_ERR_WORKSPACE;
    if (!aligned16(ws)) return GHD_ERR_ALIGN;
    if (ws_bytes < ghd_tree_mask_workspace_bytes()) return GHD_ERR_WORKSPACE;
    return launch_fused_setup((uint32_t*)ws, parent_dev, M, mpad_of(M), 0, 0, 1.f, mask_dev, nullptr,
                              nullptr, nullptr, 0, nullptr, nullptr, nullptr, (hipStream_t)stream);
}

size_t ghd_packed_weight_bytes(int N, int K)
{
    if (N < 1 || K < 1) return 0;
    return packed_bytes2(N, K);
}

ghd_status ghd_pack_weight(void* dst, const void* src, int N, int K, int kind, int head_dim,
                           void* stream)
{
    if (!dst || !src) return GHD_ERR_NULL;
    if (N < 1 || K < 1 || kind < GHD_PACK_PLAIN || kind > GHD_PACK_GATE_UP) return GHD_ERR_SHAPE;
    if (kind == GHD_PACK_QKV && ((head_dim != 64 && head_dim != 128) || N % (3 * head_dim) != 0))
        return GHD_ERR_SHAPE;
    if (kind == GHD_PACK_GATE_UP && (N % 16) != 0) return GHD_ERR_SHAPE;
    if (!aligned16(dst)) return GHD_ERR_ALIGN;
    return launch_pack2(dst, src, N, K, kind, head_dim, (hipStream_t)stream);
}

size_t ghd_linear_workspace_bytes(int M, int N, int K)
{
    if (M < 1 || M > GHD_MAX_M || N < 1 || K < 1) return 0;
    return carve(nullptr, 1, M, 0, 0, 0, K).bytes;
}

ghd_status ghd_linear_skinny(void* y, const void* x, const void* Wp, int M, int N, int K,
                             int64_t ldx, int64_t ldy, uint32_t flags, void* ws, size_t ws_bytes,
                             void* stream)
{
    if (!y || !x || !Wp) return GHD_ERR_NULL;
    if (M < 1 || M > GHD_MAX_M || N < 1 || K < 8 || (K % 8) != 0) return GHD_ERR_SHAPE;
    if (ldx < K || ldy < N || flags > GHD_OUT_F16 || !linear_shape_ok(N, K)) return GHD_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(Wp) || !aligned16(y) || (ldx % 8) != 0) return GHD_ERR_ALIGN;
    if (!ws) return GHD_ERR_WORKSPACE;
    if (!aligned16(ws)) return GHD_ERR_ALIGN;
    if (ws_bytes < ghd_linear_workspace_bytes(M, N, K)) return GHD_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    Ws w = carve(ws, 1, M, 0, 0, 0, K);
    FusedArgs a = {};
    if (!fill_plan(a, M, N, K)) return GHD_ERR_SHAPE;
    ghd_status s = launch_fused_setup(w.sync, nullptr, M, mpad_of(M), 0, 0, 1.f, nullptr, nullptr,
                                      nullptr, nullptr, 0, nullptr, nullptr, nullptr, st);
    if (s) return s;
    // the kernel reads x as MFMA operand blocks
    if ((s = launch_pack_x(w.xpk, (const half_t*)x, M, mpad_of(M), K, ldx, st))) return s;
    a.mode = MODE_LINEAR;
    a.M = M;
    a.Mpad = mpad_of(M);
    a.d = 128;
    a.sync = w.sync;
    a.part = w.part;
    a.lin_W = (const half8*)Wp;
    a.lin_x = w.xpk;
    a.lin_y = y;
    a.lin_N = N;
    a.lin_K = K;
    a.lin_epi = flags == GHD_OUT_F16 ? EPI_STORE_F16 : EPI_STORE_F32;
    a.lin_cnt = kCntLm;
    a.lin_epoch = 0;
    a.lin_ldy = ldy;
    return timed_fused(a, st);
}

size_t ghd_attention_workspace_bytes(int M, int kv_len, int nh, int d)
{
    if (M < 1 || M > GHD_MAX_M || kv_len < 0 || nh < 1 || (d != 64 && d != 128)) return 0;
    return carve(nullptr, 2, M, 0, 0, d).bytes;
}

// the visibility of the tree rows comes either from parent[] (masks built by the set-up
// kernel) or from the caller's masks
static ghd_status attention_call(void* out, const void* q, const void* k_cache, const void* v_cache,
                                 const int32_t* parent_dev, const uint64_t* mask_dev, int M, int kv_len,
                                 int nh, int d, int64_t k_stride_head, int64_t k_stride_tok,
                                 int64_t v_stride_head, int64_t v_stride_ch, float scale, void* ws,
                                 size_t ws_bytes, void* stream)
{
    if (!out || !q || !k_cache || !v_cache || (!parent_dev && !mask_dev)) return GHD_ERR_NULL;
    if (mask_dev && ((uintptr_t)mask_dev & 7) != 0) return GHD_ERR_ALIGN;
    if (M < 1 || M > GHD_MAX_M || kv_len < 0 || nh < 1 || nh > 256 || (d != 64 && d != 128))
        return GHD_ERR_SHAPE;
    if (k_stride_tok < d || k_stride_head < 0 || v_stride_head < 0) return GHD_ERR_SHAPE;
    if (v_stride_ch < (int64_t)kv_len + M) return GHD_ERR_CAPACITY;
    // the kernel indexes inside a head, and counts (head, key tile) pairs, in 32 bits
    if (k_stride_tok * ((int64_t)kv_len + M) >= (1ll << 31) || v_stride_ch * d >= (1ll << 31) ||
        (int64_t)nh * (((int64_t)kv_len + M + 63) / 64) >= (1ll << 31))
        return GHD_ERR_SHAPE;
    if (!aligned16(out) || !aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) ||
        (k_stride_tok % 8) != 0 || (k_stride_head % 8) != 0 || (v_stride_ch % 8) != 0 ||
        (v_stride_head % 8) != 0)
        return GHD_ERR_ALIGN;
    if (!ws) return GHD_ERR_WORKSPACE;
    if (!aligned16(ws)) return GHD_ERR_ALIGN;
    if (ws_bytes < ghd_attention_workspace_bytes(M, kv_len, nh, d)) return GHD_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    Ws w = carve(ws, 2, M, 0, 0, d);
    ghd_status s = launch_fused_setup(w.sync, parent_dev, M, mpad_of(M), kv_len, d, 1.f, w.mask,
                                      nullptr, nullptr, nullptr, 0, nullptr, nullptr, nullptr, st);
    if (s) return s;
    FusedArgs a = {};
    a.mode = MODE_ATTN;
    a.M = M;
    a.Mpad = mpad_of(M);
    a.kv_len = kv_len;
    a.nh = nh;
    a.d = d;
    a.H = nh * d;
    a.stride_head = k_stride_head;
    a.stride_tok = k_stride_tok;
    a.v_stride_head = v_stride_head;
    a.v_stride_ch = v_stride_ch;
    a.scale_log2e = scale * 1.4426950408889634f;
    a.sync = w.sync;
    a.o_part = w.o_part;
    a.ml_part = w.ml_part;
    a.mask = mask_dev ? mask_dev : w.mask;
    a.att_q = (const half_t*)q;
    a.att_k = (const half_t*)k_cache;
    a.att_v = (const half_t*)v_cache;
    a.att_out = (half_t*)out;
    return timed_fused(a, st);
}

ghd_status ghd_tree_attention(void* out, const void* q, const void* k_cache, const void* v_cache,
                              const int32_t* parent_dev, int M, int kv_len, int nh, int d,
                              int64_t k_stride_head, int64_t k_stride_tok, int64_t v_stride_head,
                              int64_t v_stride_ch, float scale, void* ws, size_t ws_bytes,
                              void* stream)
{
    if (!parent_dev) return GHD_ERR_NULL;
    return attention_call(out, q, k_cache, v_cache, parent_dev, nullptr, M, kv_len, nh, d, k_stride_head,
                          k_stride_tok, v_stride_head, v_stride_ch, scale, ws, ws_bytes, stream);
}

ghd_status ghd_masked_attention(void* out, const void* q, const void* k_cache, const void* v_cache,
                                const uint64_t* mask_dev, int M, int kv_len, int nh, int d,
                                int64_t k_stride_head, int64_t k_stride_tok, int64_t v_stride_head,
                                int64_t v_stride_ch, float scale, void* ws, size_t ws_bytes,
                                void* stream)
{
    if (!mask_dev) return GHD_ERR_NULL;
    return attention_call(out, q, k_cache, v_cache, nullptr, mask_dev, M, kv_len, nh, d, k_stride_head,
                          k_stride_tok, v_stride_head, v_stride_ch, scale, ws, ws_bytes, stream);
}

ghd_status ghd_tree_part_attention_coo(void* out, const void* q, const void* k_cache, const void* v_cache,
                                       const int32_t* parent_dev, int M, int kv_len, int nh, int d,
                                       int64_t k_stride_head, int64_t k_stride_tok, int64_t v_stride_head,
                                       int64_t v_stride_ch, float scale, void* ws, size_t ws_bytes,
                                       void* stream)
{
    if (!out || !q || !k_cache || !v_cache || !parent_dev) return GHD_ERR_NULL;
    if (M < 1 || M > GHD_MAX_M || kv_len < 0 || nh < 1 || nh > 256 || (d != 64 && d != 128))
        return GHD_ERR_SHAPE;
    if (k_stride_tok < d || k_stride_head < 0 || v_stride_head < 0) return GHD_ERR_SHAPE;
    if (v_stride_ch < (int64_t)kv_len + M) return GHD_ERR_CAPACITY;
    if (!aligned16(out) || !aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) ||
        (k_stride_tok % 8) != 0 || (k_stride_head % 8) != 0 || (v_stride_ch % 8) != 0 ||
        (v_stride_head % 8) != 0)
        return GHD_ERR_ALIGN;
    if (!ws) return GHD_ERR_WORKSPACE;
    if (!aligned16(ws)) return GHD_ERR_ALIGN;
    if (ws_bytes < ghd_attention_workspace_bytes(M, kv_len, nh, d)) return GHD_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    Ws w = carve(ws, 2, M, 0, 0, d);
    // the coordinate list is read off the ancestor masks the set-up kernel builds from parent[]
    ghd_status s = launch_fused_setup(w.sync, parent_dev, M, mpad_of(M), kv_len, d, 1.f, w.mask, nullptr,
                                      nullptr, nullptr, 0, nullptr, nullptr, nullptr, st);
    if (s) return s;
    return launch_tree_part_coo(out, q, k_cache, v_cache, w.mask, M, kv_len, nh, d, k_stride_head, k_stride_tok,
                                v_stride_head, v_stride_ch, scale, st);
}

size_t ghd_workspace_bytes(const ghd_model_cfg* cfg, int M, int kv_len)
{
    if (check_cfg(cfg, M, kv_len) != GHD_OK) return 0;
    return carve(nullptr, 0, M, cfg->H, cfg->F, cfg->d, 0, cfg->V).bytes;
}

ghd_status ghd_verify_layer(const ghd_model_cfg* cfg, const ghd_layer_weights* w, const ghd_kv* kv,
                            float* x, const int32_t* parent_dev, int M, int kv_len, void* ws,
                            size_t ws_bytes, void* stream)
{
    if (!cfg || !w || !kv || !x || !parent_dev) return GHD_ERR_NULL;
    ghd_status s = check_cfg(cfg, M, kv_len);
    if (s) return s;
    if ((s = check_layer(w, kv))) return s;
    if (!aligned16(x)) return GHD_ERR_ALIGN;
    if (!ws) return GHD_ERR_WORKSPACE;
    if (!aligned16(ws)) return GHD_ERR_ALIGN;
    if (ws_bytes < ghd_workspace_bytes(cfg, M, kv_len)) return GHD_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    Ws lw = carve(ws, 0, M, cfg->H, cfg->F, cfg->d, 0, cfg->V);
    // the caller's x is the residual stream itself; the set-up leaves its sums of squares
    if ((s = launch_fused_setup(lw.sync, parent_dev, M, mpad_of(M), kv_len, cfg->d, cfg->rope_base,
                                lw.mask, lw.rope, x, nullptr, cfg->H, lw.ss, (const half_t*)w->g_attn,
                                lw.xg16, st)))
        return s;
    return run_layer(cfg, w, kv, x, M, kv_len, lw, nullptr, 0, st);
}

static ghd_status verify_stack_impl(const ghd_model_cfg* cfg, const ghd_layer_weights* layers_host,
                                    const ghd_kv* kv_host, const void* g_final, const void* Wlm,
                                    const void* x_in, const int32_t* parent_dev, int M, int kv_len,
                                    float* logits, int32_t* amax_dev, float* x_out, void* ws,
                                    size_t ws_bytes, void* stream)
{
    if (!cfg || !layers_host || !kv_host || !g_final || !Wlm || !x_in || !parent_dev || (!logits && !amax_dev))
        return GHD_ERR_NULL;
    ghd_status s = check_cfg(cfg, M, kv_len);
    if (s) return s;
    for (int l = 0; l < cfg->L; ++l)
        if ((s = check_layer(layers_host + l, kv_host + l))) return s;
    if (!aligned16(x_in) || !aligned16(Wlm) || !aligned16(g_final) || (logits && !aligned16(logits)) ||
        (x_out && !aligned16(x_out)) || ((uintptr_t)amax_dev & 3) != 0)
        return GHD_ERR_ALIGN;
    if (!ws) return GHD_ERR_WORKSPACE;
    if (!aligned16(ws)) return GHD_ERR_ALIGN;
    if (ws_bytes < ghd_workspace_bytes(cfg, M, kv_len)) return GHD_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    Ws lw = carve(ws, 0, M, cfg->H, cfg->F, cfg->d, 0, cfg->V);
    const int H = cfg->H;
    // x = widen(x_in) with its sums of squares
    if ((s = launch_fused_setup(lw.sync, parent_dev, M, mpad_of(M), kv_len, cfg->d, cfg->rope_base,
                                lw.mask, lw.rope, lw.x, (const half_t*)x_in, H, lw.ss,
                                (const half_t*)layers_host[0].g_attn, lw.xg16, st)))
        return s;
    for (int l = 0; l < cfg->L; ++l) {
        const half_t* next_g = (const half_t*)(l + 1 < cfg->L ? layers_host[l + 1].g_attn : g_final);
        if ((s = run_layer(cfg, layers_host + l, kv_host + l, lw.x, M, kv_len, lw, next_g,
                           (uint32_t)l, st)))
            return s;
    }
    if (x_out) {
        hipError_t e = hipMemcpyAsync(x_out, lw.x, (size_t)M * H * sizeof(float),
                                      hipMemcpyDeviceToDevice, st);
        if (e != hipSuccess) return hip_fail(e);
    }
    // LM head on the final norm, straight into the caller's logits and / or into one
    // (largest logit, lowest column) candidate per 16-column tile and row
    LinearCall lm = {Wlm, cfg->V, H, EPI_STORE_F32, lw.xg16, true, nullptr,
                     logits, cfg->V, nullptr, kCntLm, 0, amax_dev ? lw.amax_tbl : nullptr};
    if ((s = step_linear(cfg, lw, lw.x, M, kv_len, lm, st))) return s;
    if (amax_dev) return launch_amax_merge(lw.amax_tbl, (cfg->V + 15) / 16, mpad_of(M), M, amax_dev, st);
    return GHD_OK;
}

ghd_status ghd_verify_stack(const ghd_model_cfg* cfg, const ghd_layer_weights* layers_host,
                            const ghd_kv* kv_host, const void* g_final, const void* Wlm,
                            const void* x_in, const int32_t* parent_dev, int M, int kv_len,
                            float* logits, float* x_out, void* ws, size_t ws_bytes, void* stream)
{
    if (!logits) return GHD_ERR_NULL;
    return verify_stack_impl(cfg, layers_host, kv_host, g_final, Wlm, x_in, parent_dev, M, kv_len, logits,
                             nullptr, x_out, ws, ws_bytes, stream);
}

ghd_status ghd_verify_stack_argmax(const ghd_model_cfg* cfg, const ghd_layer_weights* layers_host,
                                   const ghd_kv* kv_host, const void* g_final, const void* Wlm,
                                   const void* x_in, const int32_t* parent_dev, int M, int kv_len,
                                   int32_t* amax_dev, float* logits, float* x_out, void* ws,
                                   size_t ws_bytes, void* stream)
{
    if (!amax_dev) return GHD_ERR_NULL;
    return verify_stack_impl(cfg, layers_host, kv_host, g_final, Wlm, x_in, parent_dev, M, kv_len, logits,
                             amax_dev, x_out, ws, ws_bytes, stream);
}

ghd_status ghd_step_status(const void* ws, int32_t* status_host, void* stream)
{
    if (!ws || !status_host) return GHD_ERR_NULL;
    uint32_t v[4] = {0, 0, 0, 0};
    hipError_t e = hipMemcpyAsync(v, (const uint32_t*)ws, sizeof(v), hipMemcpyDeviceToHost,
                                  (hipStream_t)stream);
    if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e);
    // the calls since the last set-up, else what an earlier set-up found and kept
    uint32_t st = v[kSyncStatus];
    if (st == 0 && v[kSyncMagic] == kSyncMagicValue) st = v[kSyncSticky];
    *status_host = (int32_t)st;
    return GHD_OK;
}

ghd_status ghd_step_status_reset(void* ws, void* stream)
{
    if (!ws) return GHD_ERR_NULL;
    hipError_t e = hipMemsetAsync((uint32_t*)ws + kSyncStatus, 0, 2 * sizeof(uint32_t), (hipStream_t)stream);
    return e == hipSuccess ? GHD_OK : hip_fail(e);
}

size_t ghd_accept_workspace_bytes(int M)
{
    if (M < 1 || M > GHD_MAX_M) return 0;
    return align_up(accept_workspace_bytes(), 256);
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
    return launch_accept(logits, tokens_dev, parent_dev, M, V, res_dev, amax_dev, ws,
                         (hipStream_t)stream);
}

ghd_status ghd_accept_path(const int32_t* amax_dev, const int32_t* tokens_dev, const int32_t* parent_dev,
                           int M, int32_t* res_dev, void* stream)
{
    if (!amax_dev || !tokens_dev || !parent_dev || !res_dev) return GHD_ERR_NULL;
    if (M < 1 || M > GHD_MAX_M) return GHD_ERR_SHAPE;
    return launch_accept_path(amax_dev, tokens_dev, parent_dev, M, res_dev, (hipStream_t)stream);
}

ghd_status ghd_accept_greedy_static(const float* logits, const int32_t* tokens_dev,
                                    const int32_t* parent_dev, int M, int V, int32_t* res_dev,
                                    int32_t* amax_dev, void* stream)
{
    if (!logits || !tokens_dev || !parent_dev || !res_dev) return GHD_ERR_NULL;
    if (M < 1 || M > GHD_MAX_M || V < 1) return GHD_ERR_SHAPE;
    return launch_accept_static(logits, tokens_dev, parent_dev, M, V, res_dev, amax_dev,
                                (hipStream_t)stream);
}

ghd_status ghd_commit_path(const ghd_model_cfg* cfg, const ghd_kv* kv_host, const int32_t* res_dev,
                           int M, int kv_len, void* stream)
{
    if (!cfg || !kv_host || !res_dev) return GHD_ERR_NULL;
    ghd_status s = check_cfg(cfg, M, kv_len);
    if (s) return s;
    void* k[kMaxLayers];
    void* v[kMaxLayers];
    for (int l = 0; l < cfg->L; ++l) {
        if (!kv_host[l].k || !kv_host[l].v) return GHD_ERR_NULL;
        if (!aligned16(kv_host[l].k) || !aligned16(kv_host[l].v)) return GHD_ERR_ALIGN;
        k[l] = kv_host[l].k;
        v[l] = kv_host[l].v;
    }
    return launch_commit_path(k, v, cfg->L, cfg->nh, cfg->d, cfg->kv_capacity, kv_len, M, res_dev,
                              (hipStream_t)stream);
}

// ---- drafting side -------------------------------------------------------------
ghd_status ghd_embed(void* x16, const void* table16, const int32_t* tokens_dev, int M, int H, int V,
                     void* stream)
{
    if (!x16 || !table16 || !tokens_dev) return GHD_ERR_NULL;
    if (M < 1 || M > GHD_MAX_M || H < 8 || (H % 8) != 0 || V < 1) return GHD_ERR_SHAPE;
    if (!aligned16(x16) || !aligned16(table16)) return GHD_ERR_ALIGN;
    return launch_embed(x16, table16, tokens_dev, M, H, V, (hipStream_t)stream);
}

int ghd_tree_build(const double* acc_host, int K, int R, int M, int32_t* parent_host,
                   int32_t* rank_host, double* expect_host)
{
    if (!acc_host || !parent_host || !rank_host) return GHD_ERR_NULL;
    if (K < 1 || R < 1 || M < 1 || M > GHD_MAX_M) return GHD_ERR_SHAPE;
    for (int i = 0; i < K * R; ++i)
        if (!(acc_host[i] >= 0.0 && acc_host[i] <= 1.0)) return GHD_ERR_SHAPE;
    return tree_build_host(acc_host, K, R, M, parent_host, rank_host, expect_host);
}

int ghd_choose_width(const double* acc_host, int K, int R, const int32_t* widths_host,
                     const double* latency_host, int n, double* rate_host)
{
    if (!acc_host || !widths_host || !latency_host) return GHD_ERR_NULL;
    if (K < 1 || R < 1 || n < 1) return GHD_ERR_SHAPE;
    for (int i = 0; i < K * R; ++i)
        if (!(acc_host[i] >= 0.0 && acc_host[i] <= 1.0)) return GHD_ERR_SHAPE;
    for (int i = 0; i < n; ++i)
        if (widths_host[i] < 1 || widths_host[i] > GHD_MAX_M || !(latency_host[i] > 0.0)) return GHD_ERR_SHAPE;
    int32_t parent[GHD_MAX_M], rank[GHD_MAX_M];
    int best = 0;
    double best_rate = -1.0;
    for (int i = 0; i < n; ++i) {
        double e = 0.0;
        tree_build_host(acc_host, K, R, widths_host[i], parent, rank, &e);
        const double r = e / latency_host[i];
        if (rate_host) rate_host[i] = r;
        if (r > best_rate) {
            best_rate = r;
            best = i;
        }
    }
    return best;
}

struct DraftWs {
    Ws lin;
    half_t* n16;
    float* logits;
    int32_t* topk;
    size_t bytes;
};

static DraftWs carve_draft(void* ws, int H, int K, int V, int R)
{
    DraftWs d = {};
    d.lin = carve(ws, 1, 1, 0, 0, 0, H);
    Carver cv(ws);
    cv.off = d.lin.bytes;
    d.n16 = cv.take<half_t>((size_t)H);
    d.logits = cv.take<float>((size_t)K * V);
    d.topk = cv.take<int32_t>((size_t)K * R);
    d.bytes = cv.off;
    return d;
}

static bool draft_shape_ok(int K, int R, int H, int V)
{
    return K >= 1 && K <= 16 && R >= 1 && R <= 32 && R <= V && H >= 8 && (H % 8) == 0 && V >= 1 &&
           (int64_t)K * V <= 262144 && linear_shape_ok(K * V, H);
}

size_t ghd_draft_workspace_bytes(int K, int R, int H, int V)
{
    if (!draft_shape_ok(K, R, H, V)) return 0;
    return carve_draft(nullptr, H, K, V, R).bytes;
}

// step_sync: the sync block of the verification pass this call belongs to (its status word
// then covers the drafting launch too, and is not cleared again), or nullptr for a call of
// its own, which uses and clears the sync block of its own workspace.
static ghd_status draft_tokens_impl(const void* g_final, const void* Wheads, int K, int R, int H, int V,
                                    float rms_eps, const float* x_final, const int32_t* res_dev,
                                    const int32_t* parent_dev, const int32_t* rank_dev, int M,
                                    int32_t* tokens_dev, int32_t* topk_dev, float* head_logits, void* ws,
                                    size_t ws_bytes, void* stream, uint32_t* step_sync)
{
    if (!g_final || !Wheads || !x_final || !res_dev || !parent_dev || !rank_dev || !tokens_dev)
        return GHD_ERR_NULL;
    if (!draft_shape_ok(K, R, H, V) || M < 1 || M > GHD_MAX_M || !(rms_eps >= 0.f)) return GHD_ERR_SHAPE;
    if (!aligned16(g_final) || !aligned16(Wheads) || !aligned16(x_final) ||
        (head_logits && !aligned16(head_logits)))
        return GHD_ERR_ALIGN;
    if (!ws) return GHD_ERR_WORKSPACE;
    if (!aligned16(ws)) return GHD_ERR_ALIGN;
    if (ws_bytes < ghd_draft_workspace_bytes(K, R, H, V)) return GHD_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    DraftWs d = carve_draft(ws, H, K, V, R);
    float* logits = head_logits ? head_logits : d.logits;
    int32_t* topk = topk_dev ? topk_dev : d.topk;
    ghd_status s = GHD_OK;
    if (!step_sync &&
        (s = launch_fused_setup(d.lin.sync, nullptr, 1, mpad_of(1), 0, 0, 1.f, nullptr, nullptr, nullptr,
                                nullptr, 0, nullptr, nullptr, nullptr, st)))
        return s;
    if ((s = launch_pick_norm(x_final, res_dev, M, H, g_final, rms_eps, d.n16, st))) return s;
    if ((s = launch_pack_x(d.lin.xpk, d.n16, 1, mpad_of(1), H, H, st))) return s;
    FusedArgs a = {};
    if (!fill_plan(a, 1, K * V, H)) return GHD_ERR_SHAPE;
    a.mode = MODE_LINEAR;
    a.M = 1;
    a.Mpad = mpad_of(1);
    a.d = 128;
    a.sync = step_sync ? step_sync : d.lin.sync;
    a.part = d.lin.part;
    a.lin_W = (const half8*)Wheads;
    a.lin_x = d.lin.xpk;
    a.lin_y = logits;
    a.lin_N = K * V;
    a.lin_K = H;
    a.lin_epi = EPI_STORE_F32;
    a.lin_cnt = step_sync ? kCntDraft : kCntLm;
    a.lin_epoch = 0;
    a.lin_ldy = (int64_t)K * V;
    if ((s = timed_fused(a, st))) return s;
    if ((s = launch_topk(logits, K, V, R, topk, st))) return s;
    return launch_tree_tokens(tokens_dev, parent_dev, rank_dev, M, topk, K, R, res_dev, V, st);
}

ghd_status ghd_draft_tokens(const void* g_final, const void* Wheads, int K, int R, int H, int V,
                            float rms_eps, const float* x_final, const int32_t* res_dev,
                            const int32_t* parent_dev, const int32_t* rank_dev, int M,
                            int32_t* tokens_dev, int32_t* topk_dev, float* head_logits, void* ws,
                            size_t ws_bytes, void* stream)
{
    return draft_tokens_impl(g_final, Wheads, K, R, H, V, rms_eps, x_final, res_dev, parent_dev, rank_dev, M,
                             tokens_dev, topk_dev, head_logits, ws, ws_bytes, stream, nullptr);
}

struct SpecWs {
    void* verify;     // first, so that ghd_step_status on the step's workspace reads its status word
    void* draft;
    half_t* x16;
    int32_t* amax;
    float* x_out;
    size_t verify_bytes, draft_bytes, bytes;
};

static SpecWs carve_spec(void* ws, const ghd_spec_model* m, int M, int kv_len)
{
    SpecWs w = {};
    const ghd_model_cfg* c = m->cfg;
    w.verify_bytes = ghd_workspace_bytes(c, M, kv_len);
    w.draft_bytes = ghd_draft_workspace_bytes(m->K, m->R, c->H, c->V);
    Carver cv(ws);
    w.verify = cv.take<char>(w.verify_bytes);
    w.draft = cv.take<char>(w.draft_bytes);
    w.x16 = cv.take<half_t>((size_t)M * c->H);
    w.amax = cv.take<int32_t>((size_t)GHD_MAX_M);
    w.x_out = cv.take<float>((size_t)M * c->H);
    w.bytes = cv.off;
    return w;
}

size_t ghd_spec_workspace_bytes(const ghd_spec_model* m, int M, int kv_len)
{
    if (!m || !m->cfg || check_cfg(m->cfg, M, kv_len) != GHD_OK) return 0;
    if (!draft_shape_ok(m->K, m->R, m->cfg->H, m->cfg->V)) return 0;
    return carve_spec(nullptr, m, M, kv_len).bytes;
}

ghd_status ghd_spec_step(const ghd_spec_model* m, const int32_t* parent_dev, const int32_t* rank_dev,
                         int M, int kv_len, int32_t* tokens_dev, int32_t* res_dev, void* ws,
                         size_t ws_bytes, void* stream)
{
    if (!m || !m->cfg || !m->embed || !m->Wheads || !parent_dev || !rank_dev || !tokens_dev || !res_dev)
        return GHD_ERR_NULL;
    ghd_status s = check_cfg(m->cfg, M, kv_len);
    if (s) return s;
    if (!draft_shape_ok(m->K, m->R, m->cfg->H, m->cfg->V)) return GHD_ERR_SHAPE;
    if (!ws) return GHD_ERR_WORKSPACE;
    if (!aligned16(ws)) return GHD_ERR_ALIGN;
    if (ws_bytes < ghd_spec_workspace_bytes(m, M, kv_len)) return GHD_ERR_WORKSPACE;
    const ghd_model_cfg* c = m->cfg;
    SpecWs w = carve_spec(ws, m, M, kv_len);
    if ((s = ghd_embed(w.x16, m->embed, tokens_dev, M, c->H, c->V, stream))) return s;
    // the LM-head finish leaves the row argmaxes: no logits are written in a decoding step
    if ((s = ghd_verify_stack_argmax(c, m->layers_host, m->kv_host, m->g_final, m->Wlm, w.x16, parent_dev, M,
                                     kv_len, w.amax, nullptr, w.x_out, w.verify, w.verify_bytes, stream)))
        return s;
    if ((s = ghd_accept_path(w.amax, tokens_dev, parent_dev, M, res_dev, stream))) return s;
    if ((s = ghd_commit_path(c, m->kv_host, res_dev, M, kv_len, stream))) return s;
    return draft_tokens_impl(m->g_final, m->Wheads, m->K, m->R, c->H, c->V, c->rms_eps, w.x_out, res_dev,
                             parent_dev, rank_dev, M, tokens_dev, nullptr, nullptr, w.draft, w.draft_bytes,
                             stream, (uint32_t*)w.verify);
}

/* Benchmark support (not part of the documented ABI): time the launches of one kind
 * of the persistent kernel with HIP events on the launch stream.
 * ghd_debug_profile(1) starts a fresh measurement of the linear-layer launches,
 * ghd_debug_profile(2) of the attention launches, ghd_debug_profile(3) of the launches that
 * hold a QKV layer and its attention, ghd_debug_profile(0) stops it; after
 * synchronising the stream, ghd_debug_profile_read returns the number of launches and
 * their summed duration in milliseconds.  ghd_debug_copy is a plain copy kernel of known
 * traffic (bytes read + bytes written) used to calibrate the profiler's byte counters. */
/* Test support (not part of the documented ABI): the kernels' work-share arithmetic on the
 * host; see share_on_host. */
void ghd_debug_share(int items, int per_item, int j, int G, int item, int* out5)
{
    share_on_host(items, per_item, j, G, item, out5);
}

/* out3 = {row tiles a share handles at once, shares per workgroup, whole tiles (1) or k ranges of
 * four-tile row blocks (0)} for a linear layer [N, K] at M rows on G workgroups; returns 0, or -1
 * if the shape needs more shares than the library is laid out for. */
int ghd_debug_plan(int M, int N, int K, int G, int* out3)
{
    LinPlan pl;
    if (!plan_linear(M, N, K, G, &pl)) return -1;
    out3[0] = pl.slots;
    out3[1] = pl.passes;
    out3[2] = pl.whole;
    return 0;
}

void ghd_debug_attn_share(int nh, int ntile, int j, int G, int head, int* out6)
{
    attn_share_on_host(nh, ntile, j, G, head, out6);
}

void ghd_debug_split_qkv_attn(int on) { g_split_qkv_attn = on != 0; }

void ghd_debug_profile(int what)
{
    g_prof_mode = what == 1 ? MODE_LINEAR : what == 2 ? MODE_ATTN : what == 3 ? MODE_QKV_ATTN : -1;
    if (what) g_prof_used = 0;
}

__global__ void k_debug_copy(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x)
        dst[i] = src[i];
}

int ghd_debug_copy(void* dst, const void* src, size_t bytes, void* stream)
{
    if (!dst || !src || (bytes % 16) != 0 || !aligned16(dst) || !aligned16(src)) return GHD_ERR_SHAPE;
    hipLaunchKernelGGL(k_debug_copy, dim3(4096), dim3(256), 0, (hipStream_t)stream, (uint4*)dst,
                       (const uint4*)src, bytes / 16);
    return check_launch();
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

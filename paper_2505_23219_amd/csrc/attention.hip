// Tree attention for the verification step (Ghidorah, Eq. 1 and section 2.3).
//
// Every drafted node attends the whole committed cache (the dense part) and,
// among the M tree rows appended behind it, only the nodes on its own root
// path (the sparse part).  The key range [0, kv_len + M) is cut into 64-key
// tiles; a workgroup (head h, split p) streams its tiles through LDS once and
// all tree rows share them.  Each wavefront owns 16*MTW query rows and computes
//   S^T = K . q^T   (A = K tile rows from LDS, B = q fragments kept in registers)
// so that a lane owns ONE query row (column m = lane%16) and four keys per
// 16-key sub-tile.  Row maxima, the softmax sums and the rescale factors are
// then per-lane scalars, the fp16 probabilities are already in the B-operand
// layout of the second product
//   O^T += V^T . P^T (A = V tile read transposed from LDS)
// and the ancestor mask is a 128-bit word per lane tested with shifts.
// Sub-tiles in which no row of the wavefront sees any key are skipped.
// The parts of a head are merged with the online-softmax rescaling of section
// 3.2.2 (own softmax per part, aligned by a scaling factor at the end).
#include "common.h"

namespace ghd {

constexpr int kTileKeys = 64;

template <int D>
struct AttnSmem {
    static constexpr int KS = D + 8;          // halves per K row (padded)
    static constexpr int VS = kTileKeys + 4;  // halves per V^T row (padded)
    half_t k[kTileKeys * KS];
    half_t vt[D * VS];
};

template <int D, int MTW>
__global__ __launch_bounds__(256) void k_tree_attention(
    half_t* __restrict__ out, const half_t* __restrict__ q, const half_t* __restrict__ kc,
    const half_t* __restrict__ vc, const uint64_t* __restrict__ mask, int M, int kv_len, int nh,
    int64_t stride_head, int64_t stride_tok, float scale_log2e, int tps, int ntile, int P,
    float* __restrict__ o_part, float* __restrict__ ml_part)
{
    constexpr int DS = D / 32;        // k-steps of the QK^T product
    constexpr int DT = D / 16;        // 16-channel tiles of the output
    constexpr int CPR = D / 8;        // 16-byte chunks per cache row
    constexpr int NLD = kTileKeys * CPR / 256;   // chunks per thread per tile
    using Smem = AttnSmem<D>;
    __shared__ Smem sm;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int c = lane & 15, g = lane >> 4;
    const int p = blockIdx.x, h = blockIdx.y, grp = blockIdx.z;
    const int T = kv_len + M;
    const int t0 = p * tps, t1 = min(t0 + tps, ntile);

    const half_t* kh = kc + (size_t)h * stride_head;
    const half_t* vh = vc + (size_t)h * stride_head;

    // ---- per-wave query rows
    int mrow[MTW];
    bool mok[MTW];
    uint64_t alo[MTW], ahi[MTW];
    half8 qf[MTW][DS];
    bool wave_active = false;
#pragma unroll
    for (int t = 0; t < MTW; ++t) {
        int mt = (grp * 4 + wave) * MTW + t;
        mrow[t] = mt * 16 + c;
        mok[t] = mrow[t] < M;
        wave_active = wave_active || (mt * 16 < M);
        alo[t] = mok[t] ? mask[2 * mrow[t]] : 0;
        ahi[t] = mok[t] ? mask[2 * mrow[t] + 1] : 0;
#pragma unroll
        for (int s = 0; s < DS; ++s) {
            half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (mok[t]) v = *(const half8*)(q + ((size_t)mrow[t] * nh + h) * D + s * 32 + g * 8);
            qf[t][s] = v;
        }
    }

    float mrun[MTW], lrun[MTW];
    floatx4 oacc[MTW][DT];
#pragma unroll
    for (int t = 0; t < MTW; ++t) {
        mrun[t] = -INFINITY;
        lrun[t] = 0.f;
#pragma unroll
        for (int e = 0; e < DT; ++e) oacc[t][e] = (floatx4){0.f, 0.f, 0.f, 0.f};
    }

    // ---- tile staging: global -> registers -> LDS
    half8 kreg[NLD], vreg[NLD];
    auto load_tile = [&](int tile) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            int id = tid + 256 * i;
            int row = id / CPR, ch = id % CPR;
            int key = min(tile * kTileKeys + row, T - 1);   // stay inside the readable rows
            kreg[i] = *(const half8*)(kh + (size_t)key * stride_tok + ch * 8);
            vreg[i] = *(const half8*)(vh + (size_t)key * stride_tok + ch * 8);
        }
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            int id = tid + 256 * i;
            int row = id / CPR, ch = id % CPR;
            *(half8*)(&sm.k[row * Smem::KS + ch * 8]) = kreg[i];
#pragma unroll
            for (int e = 0; e < 8; ++e) sm.vt[(ch * 8 + e) * Smem::VS + row] = vreg[i][e];
        }
    };

    if (t0 < t1) load_tile(t0);
    for (int tile = t0; tile < t1; ++tile) {
        __syncthreads();            // everyone is done reading the previous tile
        store_tile();
        __syncthreads();
        if (tile + 1 < t1) load_tile(tile + 1);
        if (!wave_active) continue;

        const int key0 = tile * kTileKeys;
#pragma unroll
        for (int t = 0; t < MTW; ++t) {
            // visibility of this lane's 4 keys in each of the 4 sub-tiles
            floatx4 s[4];
            bool sub_any[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int kbase = key0 + j * 16;            // first key of the sub-tile
                bool vis_any;
                if (kbase + 16 <= kv_len) {
                    vis_any = true;                          // committed rows: dense, no mask
                } else {
                    bool mine = false;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        int key = kbase + g * 4 + r;
                        bool vis = key < kv_len;
                        if (key >= kv_len && key < T) {
                            int jn = key - kv_len;
                            vis = (jn < 64 ? (alo[t] >> jn) : (ahi[t] >> (jn - 64))) & 1ull;
                        }
                        mine = mine || (vis && mok[t]);
                    }
                    vis_any = __ballot(mine) != 0ull;
                }
                sub_any[j] = vis_any;
                s[j] = (floatx4){0.f, 0.f, 0.f, 0.f};
                if (vis_any) {
#pragma unroll
                    for (int ds = 0; ds < DS; ++ds) {
                        half8 kf = *(const half8*)(&sm.k[(j * 16 + c) * Smem::KS + ds * 32 + g * 8]);
                        s[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf, qf[t][ds], s[j], 0, 0, 0);
                    }
                }
            }
            // scores -> masked, scaled (log2 domain); running max
            float tmax = -INFINITY;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int kbase = key0 + j * 16;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    int key = kbase + g * 4 + r;
                    bool vis = sub_any[j] && key < kv_len;
                    if (sub_any[j] && key >= kv_len && key < T) {
                        int jn = key - kv_len;
                        vis = (jn < 64 ? (alo[t] >> jn) : (ahi[t] >> (jn - 64))) & 1ull;
                    }
                    float v = vis ? s[j][r] * scale_log2e : -INFINITY;
                    s[j][r] = v;
                    tmax = fmaxf(tmax, v);
                }
            }
            tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
            float mnew = fmaxf(mrun[t], tmax);
            float muse = (mnew == -INFINITY) ? 0.f : mnew;
            float alpha = exp2f(mrun[t] - muse);            // 0 when nothing was seen before
            mrun[t] = mnew;
            float lsum = 0.f;
            half8 pf[2];
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float pv = exp2f(s[j][r] - muse);
                    lsum += pv;
                    pf[j >> 1][(j & 1) * 4 + r] = (half_t)pv;
                }
            lrun[t] = lrun[t] * alpha + lsum;
#pragma unroll
            for (int e = 0; e < DT; ++e) oacc[t][e] *= alpha;
            // O^T += V^T . P^T, 32 keys per product
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                if (!(sub_any[2 * hf] || sub_any[2 * hf + 1])) continue;
#pragma unroll
                for (int e = 0; e < DT; ++e) {
                    const half_t* vrow = &sm.vt[(e * 16 + c) * Smem::VS];
                    half4 a0 = *(const half4*)(vrow + (2 * hf) * 16 + g * 4);
                    half4 a1 = *(const half4*)(vrow + (2 * hf + 1) * 16 + g * 4);
                    half8 vf = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
                    oacc[t][e] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vf, pf[hf], oacc[t][e], 0, 0, 0);
                }
            }
        }
    }

    if (!wave_active) return;
    // ---- write this part: lane (c, g) holds channels e*16 + g*4 .. +4 of row mrow
#pragma unroll
    for (int t = 0; t < MTW; ++t) {
        float l = lrun[t];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        if (!mok[t]) continue;
        if (P == 1) {
            float inv = 1.0f / l;
#pragma unroll
            for (int e = 0; e < DT; ++e) {
                half4 o4;
#pragma unroll
                for (int r = 0; r < 4; ++r) o4[r] = (half_t)(oacc[t][e][r] * inv);
                *(half4*)(out + ((size_t)mrow[t] * nh + h) * D + e * 16 + g * 4) = o4;
            }
        } else {
            size_t row = ((size_t)p * nh + h) * M + mrow[t];
#pragma unroll
            for (int e = 0; e < DT; ++e)
                *(floatx4*)(o_part + row * D + e * 16 + g * 4) = oacc[t][e];
            if (g == 0) {
                ml_part[row * 2] = mrun[t];
                ml_part[row * 2 + 1] = l;
            }
        }
    }
}

// Merge of the P parts of every (row, head): o = sum_p w_p o_p / sum_p w_p l_p with
// w_p = 2^(m_p - max_p m_p)  (section 3.2.2).  One thread per output channel.
template <int D>
__global__ void k_attn_combine(half_t* __restrict__ out, const float* __restrict__ o_part,
                               const float* __restrict__ ml_part, int M, int nh, int P)
{
    int m = blockIdx.x, h = blockIdx.y, ch = threadIdx.x;
    float mx = -INFINITY;
    for (int p = 0; p < P; ++p)
        mx = fmaxf(mx, ml_part[(((size_t)p * nh + h) * M + m) * 2]);
    float num = 0.f, den = 0.f;
    for (int p = 0; p < P; ++p) {
        size_t row = ((size_t)p * nh + h) * M + m;
        float mp = ml_part[row * 2];
        float w = (mp == -INFINITY) ? 0.f : exp2f(mp - mx);
        den += w * ml_part[row * 2 + 1];
        num += w * o_part[row * D + ch];
    }
    out[((size_t)m * nh + h) * D + ch] = (half_t)(num / den);
}

static int g_force_p = 0;
void set_attn_override(int p) { g_force_p = p; }

AttnPlan plan_attention(int M, int kv_len, int nh)
{
    AttnPlan a;
    a.ntile = ceil_div(kv_len + M, kTileKeys);
    a.MTW = (M > 64) ? 2 : 1;
    a.groups = 1;
    // about two workgroups per compute unit, at least two tiles each
    int P = ceil_div(512, nh * a.groups);
    if (P > a.ntile / 2) P = a.ntile / 2;
    if (P < 1) P = 1;
    if (g_force_p) P = g_force_p;
    if (P > a.ntile) P = a.ntile;
    a.tps = ceil_div(a.ntile, P);
    a.P = ceil_div(a.ntile, a.tps);
    return a;
}

template <int D, int MTW>
static void launch_attn_t(const AttnPlan& p, half_t* out, const half_t* q, const half_t* kc,
                          const half_t* vc, const uint64_t* mask, int M, int kv_len, int nh,
                          int64_t stride_head, int64_t stride_tok, float scale, float* o_part,
                          float* ml_part, hipStream_t st)
{
    dim3 grid(p.P, nh, p.groups);
    hipLaunchKernelGGL((k_tree_attention<D, MTW>), grid, dim3(256), 0, st, out, q, kc, vc, mask, M,
                       kv_len, nh, stride_head, stride_tok, scale * 1.4426950408889634f, p.tps,
                       p.ntile, p.P, o_part, ml_part);
    if (p.P > 1)
        hipLaunchKernelGGL((k_attn_combine<D>), dim3(M, nh), dim3(D), 0, st, out, o_part, ml_part, M,
                           nh, p.P);
}

ghd_status launch_attention(const AttnPlan& p, half_t* out, const half_t* q, const half_t* kc,
                            const half_t* vc, const uint64_t* mask, int M, int kv_len, int nh, int d,
                            int64_t stride_head, int64_t stride_tok, float scale, float* o_part,
                            float* ml_part, hipStream_t st)
{
    if (d == 128) {
        if (p.MTW == 1)
            launch_attn_t<128, 1>(p, out, q, kc, vc, mask, M, kv_len, nh, stride_head, stride_tok,
                                  scale, o_part, ml_part, st);
        else
            launch_attn_t<128, 2>(p, out, q, kc, vc, mask, M, kv_len, nh, stride_head, stride_tok,
                                  scale, o_part, ml_part, st);
    } else {
        if (p.MTW == 1)
            launch_attn_t<64, 1>(p, out, q, kc, vc, mask, M, kv_len, nh, stride_head, stride_tok,
                                 scale, o_part, ml_part, st);
        else
            launch_attn_t<64, 2>(p, out, q, kc, vc, mask, M, kv_len, nh, stride_head, stride_tok,
                                 scale, o_part, ml_part, st);
    }
    return check_launch();
}

}  // namespace ghd

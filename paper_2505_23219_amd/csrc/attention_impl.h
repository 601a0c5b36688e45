// Tree attention of the verification step: the device code shared by the attention kernel
// and the fused QKV + attention kernel.
//
// A head's 64-key tiles are split over a run of workgroups of one XCD.  A workgroup streams
// its tiles through LDS (the V cache is kept channel-major, so both K rows and V^T rows go
// to LDS as they are); wavefronts 0-3 take the first 32 keys of a tile, 4-7 the last 32,
// each for its own 16 (or 32) query rows.  S^T = K q^T puts one query row in each lane
// column, so softmax statistics are per-lane scalars, the fp16 probabilities are already in
// B-operand layout for O^T += V^T P^T, and the ancestor mask (Ghidorah, section 2.3) is a
// 128-bit register per lane.  Sub-tiles no row can see are skipped.  The two key halves are
// merged inside the workgroup, the workgroups of a head through one partial state each,
// with the online-softmax rescale of section 3.2.2.
#pragma once
#include "persist.h"

#include <type_traits>

namespace ghd {

// ---------------------------------------------------------------------------
// tree attention
// ---------------------------------------------------------------------------
// Work shares of the attention (see attn_phase): which heads workgroup j works on, and for
// one of them which workgroups share it and which key tiles are this workgroup's.
struct AttnHeads {
    int Gx, x, w;      // workgroups per XCD, this workgroup's XCD and its index inside it
    int hx0, Hx;       // first head and number of heads of the XCD
    int h_lo, h_hi;    // this workgroup's heads, local to the XCD (empty if h_lo == h_hi)
};

__host__ __device__ __forceinline__ AttnHeads attn_heads(int nh, int j, int G)
{
    AttnHeads s;
    const int nx = (G % 8 == 0) ? 8 : 1;
    s.Gx = G / nx;
    s.x = j / s.Gx;
    s.w = j - s.x * s.Gx;
    s.hx0 = nh * s.x / nx;
    s.Hx = nh * (s.x + 1) / nx - s.hx0;
    s.h_lo = s.h_hi = 0;
    if (s.Hx == 0) return s;
    if (s.Hx >= s.Gx) {
        s.h_lo = s.Hx * s.w / s.Gx;
        s.h_hi = s.Hx * (s.w + 1) / s.Gx;
    } else {
        s.h_lo = ((s.w + 1) * s.Hx - 1) / s.Gx;    // the head whose run of workgroups contains w
        s.h_hi = s.h_lo + 1;
    }
    return s;
}

struct AttnTiles {
    int first, np, me;   // the head's parts are workgroups first .. first + np - 1; this one is part `me`
    int t0, t1;          // its key tiles (empty, with me >= np, when there are more workgroups than tiles)
};

__host__ __device__ __forceinline__ AttnTiles attn_tiles(const AttnHeads& s, int hl, int ntile)
{
    AttnTiles t;
    t.first = s.x * s.Gx + s.w;
    t.np = 1;
    t.me = 0;
    if (s.Hx < s.Gx) {
        int wl0 = s.Gx * hl / s.Hx;                        // head hl's run of local workgroups
        int wl1 = s.Gx * (hl + 1) / s.Hx;
        t.first = s.x * s.Gx + wl0;
        t.np = (wl1 - wl0 < ntile) ? wl1 - wl0 : ntile;
        t.me = s.w - wl0;
    }
    // boundaries rounded up: when the tiles do not divide evenly the longer ranges come first,
    // and the last workgroup, whose range ends with the (costlier) tree tile, gets a shorter one
    t.t0 = t.t1 = 0;
    if (t.me < t.np) {
        t.t0 = (ntile * t.me + t.np - 1) / t.np;
        t.t1 = (ntile * (t.me + 1) + t.np - 1) / t.np;
    }
    return t;
}

// 2^x for x <= 0 (softmax weights): the hardware instruction; results below the smallest
// normal number flush to zero, which is what a weight that small should be.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int MT, int D>
struct AttnLds {
    static constexpr int MTW = (MT + 3) / 4;
    static constexpr int KS = D + 8;    // halves per K row (padded)
    static constexpr int VS = 64 + 8;   // halves per V^T row (padded, rows stay 16-byte aligned)
    // two tile buffers: while one tile is being multiplied, the next one is staged
    half_t k[2][64 * KS];
    half_t vt[2][D * VS];
    // state of the wavefronts working on the second key half, handed to their partners on
    // the first half when a head ends: [row-tile slot][tile][fragment][lane]
    floatx4 o2[4][MTW][D / 16][64];
    float m2[4][MTW][64];
    float l2[4][MTW][64];
    int wait_ok;      // thread 0's verdict on a bounded wait, for the whole workgroup
};

// `gate` is called once by every workgroup (all threads), before the first read of q or of a
// cache row from kv_len on; it returns false if the launch is to be abandoned.  A kernel that
// produces those in the same launch waits there for their producers; with PREFETCH the
// first tiles of a workgroup's first head that lie wholly below kv_len (rows of earlier
// steps) are requested before the gate, so that they arrive while it waits.
struct NoGate {
    __device__ __forceinline__ bool operator()() const { return true; }
};

template <int MT, int D, bool PREFETCH = false, class Gate = NoGate>
__device__ __forceinline__ bool attn_phase(const FusedArgs& a, Ctx& cx, const half_t* q, const half_t* kc,
                           const half_t* vc, half_t* out, uint32_t epoch, Gate gate = Gate())
{
    constexpr int MTW = (MT + 3) / 4;   // 16-row tiles per wavefront
    constexpr int DS = D / 32, DT = D / 16, CPR = D / 8;
    constexpr int NLD = 64 * CPR / kFT; // 16-byte pieces per thread per tile, for K and for V alike
    constexpr int NT = (MT <= 4) ? 4 : 2;   // tiles in flight
    using L = AttnLds<MT, D>;
    L& sm = *reinterpret_cast<L*>(cx.lds);

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int c = lane & 15, g4 = lane >> 4;
    const int kh = wave >> 2, wq = wave & 3;   // key half of the tile, row-tile slot
    // scalars of the argument block used inside the loops, as plain locals
    const int M = a.M, nh = a.nh, kv_len = a.kv_len, T = a.kv_len + a.M, Mpad = a.Mpad;
    const float scale_log2e = a.scale_log2e;
    uint32_t* const sync = a.sync;
    float* const o_part = a.o_part;
    float* const ml_part = a.ml_part;
    const int ntile = (T + 63) >> 6;

    // Work shares.  Heads are dealt to the 8 XCDs in contiguous blocks.  Inside an XCD a
    // workgroup works on one head at a time: with fewer heads than workgroups, every head
    // gets its own run of workgroups, each taking a contiguous range of the head's key
    // tiles; otherwise every workgroup takes whole heads.  A head is therefore always
    // finished inside one XCD (partial states go through that XCD's L2), and the tile loop
    // of a head has no head change in it.
    const AttnHeads hs = attn_heads(nh, cx.j, cx.G);
    const int hx0 = hs.hx0, h_lo = hs.h_lo, h_hi = hs.h_hi;

    // per-wave query rows
    int mrow[MTW];
    bool mok[MTW];
    uint64_t alo[MTW], ahi[MTW];
    bool wave_active = false;
#pragma unroll
    for (int t = 0; t < MTW; ++t) {
        int mt = wq * MTW + t;
        mrow[t] = mt * 16 + c;
        mok[t] = mrow[t] < M;
        wave_active = wave_active || (mt * 16 < M);
        alo[t] = mok[t] ? a.mask[2 * mrow[t]] : 0;
        ahi[t] = mok[t] ? a.mask[2 * mrow[t] + 1] : 0;
        // (bits from M on, which a caller's mask may have set, are never looked at: a mask bit
        // is only consulted for keys kv_len <= key < kv_len + M)
    }
    // K piece id -> (row id / CPR, 8 channels id % CPR); V^T piece id -> (channel id / 8,
    // 8 keys id % 8).  Offsets inside a head fit 32 bits (checked on the host).
    int k_off[NLD], v_off[NLD], k_row[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        int id = tid + kFT * i;
        k_row[i] = id / CPR;
        k_off[i] = (id % CPR) * 8;
        v_off[i] = (id >> 3) * (int)a.v_stride_ch + (id & 7) * 8;
    }
    const int v_last = (int)a.v_stride_ch - 8, st_tok = (int)a.stride_tok;
    const std::integral_constant<int, 0> s0;
    const std::integral_constant<int, 1> s1;
    const std::integral_constant<int, NT == 4 ? 2 : 0> s2;
    const std::integral_constant<int, NT == 4 ? 3 : 1> s3;

    bool gated = false;
    for (int hl = h_lo; hl < h_hi; ++hl) {
        const int head = hx0 + hl;
        // the workgroups first .. first + np - 1 split this head's tiles
        const AttnTiles ts = attn_tiles(hs, hl, ntile);
        const int first = ts.first, np = ts.np, me = ts.me, t0 = ts.t0, t1 = ts.t1;
        if (me >= np) continue;                            // more workgroups than tiles
        const half_t* kh_ = kc + (size_t)head * a.stride_head;
        const half_t* vh_ = vc + (size_t)head * a.v_stride_head;

        // running state of this head
        float mrun[MTW], lrun[MTW];
        floatx4 oacc[MTW][DT];
#pragma unroll
        for (int t = 0; t < MTW; ++t) {
            mrun[t] = -INFINITY;
            lrun[t] = 0.f;
#pragma unroll
            for (int e = 0; e < DT; ++e) oacc[t][e] = (floatx4){0.f, 0.f, 0.f, 0.f};
        }

        // NT tiles in flight: registers of set (tile - t0) % NT hold a tile until it is
        // staged.  A workgroup has few tiles (about 4 at 2048 cached tokens), so the time to
        // the first byte dominates unless all of them are requested at once.  The loads
        // are unconditional: past the last tile they all read one valid 16-byte piece (a
        // broadcast), which keeps the wait counts of the loop exact.
        half8 kreg[NT][NLD], vreg[NT][NLD];
        int l_tile = t0;                                   // next tile to request
        auto load_tile = [&](auto set) {
            constexpr int S = decltype(set)::value;
            const bool real = l_tile < t1;
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                int key = min(l_tile * 64 + k_row[i], T - 1);
                const half_t* kp = kh_ + key * st_tok + k_off[i];
                // keys past the capacity are never touched: the last piece is read instead
                // and zeroed when it is staged
                int over = max(l_tile * 64 + (int)((tid + kFT * i) & 7) * 8 - v_last, 0);
                const half_t* vp = vh_ + v_off[i] + l_tile * 64 - over;
                kreg[S][i] = __builtin_nontemporal_load((const half8*)(real ? kp : kc));
                vreg[S][i] = __builtin_nontemporal_load((const half8*)(real ? vp : vc));
            }
            ++l_tile;
        };
        auto store_tile = [&](auto set, int tile) {
            constexpr int S = decltype(set)::value;
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                int id = tid + kFT * i;
                *(half8*)(&sm.k[S & 1][k_row[i] * L::KS + k_off[i]]) = kreg[S][i];
                int vch = id >> 3, seg = id & 7;
                half8 v = vreg[S][i];
                int nvalid = T - (tile * 64 + seg * 8);  // rows from T on hold no data: zero them,
                if (nvalid < 8) {                        // a stray NaN times a zero weight is a NaN
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (e >= nvalid) v[e] = (half_t)0;
                }
                *(half8*)(&sm.vt[S & 1][vch * L::VS + seg * 8]) = v;
            }
        };
        // Requests, in tile order: [tiles known before the gate] gate [queries] [the rest].
        int n_pre = 0;
        if (!gated) {
            if constexpr (PREFETCH) {
                // past this share's last tile (a dummy load), or at least 64 rows below
                // kv_len: no cache line of such a tile holds a row that this launch writes,
                // whatever the strides and the alignment of the cache
                auto early = [&]() { return l_tile >= t1 || l_tile * 64 + 128 <= kv_len; };
                if (early()) {
                    load_tile(s0);
                    n_pre = 1;
                    if (early()) {
                        load_tile(s1);
                        n_pre = 2;
                        if constexpr (NT == 4) {
                            if (early()) {
                                load_tile(s2);
                                n_pre = 3;
                                if (early()) {
                                    load_tile(s3);
                                    n_pre = 4;
                                }
                            }
                        }
                    }
                }
            }
            if (!gate()) return false;
            gated = true;
        }
        half8 qf[MTW][DS];
#pragma unroll
        for (int t = 0; t < MTW; ++t) {
#pragma unroll
            for (int s = 0; s < DS; ++s) {
                half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
                if (mok[t]) v = *(const half8*)(q + ((size_t)mrow[t] * nh + head) * D + s * 32 + g4 * 8);
                qf[t][s] = v;
            }
        }
        if (n_pre < 1) load_tile(s0);
        if (n_pre < 2) load_tile(s1);
        if constexpr (NT == 4) {
            if (n_pre < 3) load_tile(s2);
            if (n_pre < 4) load_tile(s3);
        }
        // The tiles alternate between the two LDS buffers (register set S goes to buffer
        // S & 1: the number of sets is even).  While tile i is multiplied out of one buffer,
        // tile i + 1 is staged into the other and its registers are refilled - one barrier
        // per tile.  Past the share's last tile the staged data is a dummy nobody reads.
        int p_tile = t0;                                   // the tile being processed
        store_tile(s0, t0);
        load_tile(s0);
        auto do_tile = [&](auto set, auto next) {
            constexpr int B = decltype(set)::value & 1;
            const int tile = p_tile++;
            __syncthreads();            // tile staged by everybody; the other buffer is free
            store_tile(next, tile + 1);
            load_tile(next);
        if (!wave_active) return;
        const int key0 = tile * 64 + kh * 32;    // this wavefront's 32 keys
        const bool committed = key0 + 32 <= kv_len;   // every key visible to every row
#pragma unroll
        for (int t = 0; t < MTW; ++t) {
            floatx4 s[2];
            float tmax = -INFINITY;
            if (committed) {
#pragma unroll
                for (int jx = 0; jx < 2; ++jx) {
                    s[jx] = (floatx4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ds = 0; ds < DS; ++ds) {
                        half8 kf = *(const half8*)(&sm.k[B][(kh * 32 + jx * 16 + c) * L::KS + ds * 32 + g4 * 8]);
                        s[jx] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf, qf[t][ds], s[jx], 0, 0, 0);
                    }
                    s[jx] *= scale_log2e;
                    tmax = fmaxf(tmax, fmaxf(fmaxf(s[jx][0], s[jx][1]), fmaxf(s[jx][2], s[jx][3])));
                }
            } else {
                bool sub_any[2];
#pragma unroll
                for (int jx = 0; jx < 2; ++jx) {
                    const int kbase = key0 + jx * 16;
                    bool vis_any;
                    if (kbase + 16 <= kv_len) {
                        vis_any = true;
                    } else {
                        bool mine = false;
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            int key = kbase + g4 * 4 + r;
                            bool vis = key < kv_len;
                            if (key >= kv_len && key < T) {
                                int jn = key - kv_len;
                                vis = (jn < 64 ? (alo[t] >> jn) : (ahi[t] >> (jn - 64))) & 1ull;
                            }
                            mine = mine || (vis && mok[t]);
                        }
                        vis_any = __ballot(mine) != 0ull;
                    }
                    sub_any[jx] = vis_any;
                    s[jx] = (floatx4){0.f, 0.f, 0.f, 0.f};
                    if (vis_any) {
#pragma unroll
                        for (int ds = 0; ds < DS; ++ds) {
                            half8 kf = *(const half8*)(&sm.k[B][(kh * 32 + jx * 16 + c) * L::KS + ds * 32 + g4 * 8]);
                            s[jx] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf, qf[t][ds], s[jx], 0, 0, 0);
                        }
                    }
                }
                if (!(sub_any[0] || sub_any[1])) continue;
#pragma unroll
                for (int jx = 0; jx < 2; ++jx) {
                    const int kbase = key0 + jx * 16;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        int key = kbase + g4 * 4 + r;
                        bool vis = sub_any[jx] && key < kv_len;
                        if (sub_any[jx] && key >= kv_len && key < T) {
                            int jn = key - kv_len;
                            vis = (jn < 64 ? (alo[t] >> jn) : (ahi[t] >> (jn - 64))) & 1ull;
                        }
                        float v = vis ? s[jx][r] * scale_log2e : -INFINITY;
                        s[jx][r] = v;
                        tmax = fmaxf(tmax, v);
                    }
                }
            }
            tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
            float mnew = fmaxf(mrun[t], tmax);
            float muse = (mnew == -INFINITY) ? 0.f : mnew;
            float alpha = fast_exp2(mrun[t] - muse);
            mrun[t] = mnew;
            float lsum = 0.f;
            half8 pf;
#pragma unroll
            for (int jx = 0; jx < 2; ++jx)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float pv = fast_exp2(s[jx][r] - muse);
                    lsum += pv;
                    pf[jx * 4 + r] = (half_t)pv;
                }
            lrun[t] = lrun[t] * alpha + lsum;
#pragma unroll
            for (int e = 0; e < DT; ++e) {
                oacc[t][e] *= alpha;
                const half_t* vrow = &sm.vt[B][(e * 16 + c) * L::VS + kh * 32];
                half4 a0 = *(const half4*)(vrow + g4 * 4);
                half4 a1 = *(const half4*)(vrow + 16 + g4 * 4);
                half8 vf = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
                oacc[t][e] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vf, pf, oacc[t][e], 0, 0, 0);
            }
        }
    };
        // Whole groups of NT tiles run in a branch-free loop; the rest is a chain of nested
        // conditions, so every tile is only reachable through its predecessor and the number
        // of loads younger than the one being waited for is known.
        {
            int u = t0;
            if constexpr (NT == 4) {
                for (; u + 3 < t1; u += 4) {
                    do_tile(s0, s1);
                    do_tile(s1, s2);
                    do_tile(s2, s3);
                    do_tile(s3, s0);
                }
                if (u < t1) {
                    do_tile(s0, s1);
                    if (u + 1 < t1) {
                        do_tile(s1, s2);
                        if (u + 2 < t1) do_tile(s2, s3);
                    }
                }
            } else {
                for (; u + 1 < t1; u += 2) {
                    do_tile(s0, s1);
                    do_tile(s1, s0);
                }
                if (u < t1) do_tile(s0, s1);
            }
        }

        // ---- end of this workgroup's share of the head: the wavefronts of the second key
        //      half hand their state over through LDS, their partners merge it into their
        //      own (online-softmax rescale) and store the workgroup's partial state
#pragma unroll
        for (int t = 0; t < MTW; ++t) {
            float l = lrun[t];
            l += __shfl_xor(l, 16);
            l += __shfl_xor(l, 32);
            lrun[t] = l;
        }
        if (kh == 1 && wave_active) {
#pragma unroll
            for (int t = 0; t < MTW; ++t) {
#pragma unroll
                for (int e = 0; e < DT; ++e) sm.o2[wq][t][e][lane] = oacc[t][e];
                sm.m2[wq][t][lane] = mrun[t];
                sm.l2[wq][t][lane] = lrun[t];
            }
        }
        __syncthreads();
        if (kh == 0 && wave_active) {
#pragma unroll
            for (int t = 0; t < MTW; ++t) {
                float mb = sm.m2[wq][t][lane], lb = sm.l2[wq][t][lane];
                float mx = fmaxf(mrun[t], mb);
                float wa = (mrun[t] == -INFINITY) ? 0.f : fast_exp2(mrun[t] - mx);
                float wb = (mb == -INFINITY) ? 0.f : fast_exp2(mb - mx);
                float l = lrun[t] * wa + lb * wb;
                if (!mok[t]) continue;
                size_t row = (size_t)cx.j * Mpad + mrow[t];
#pragma unroll
                for (int e = 0; e < DT; ++e) {
                    floatx4 ob = sm.o2[wq][t][e][lane];
                    *(floatx4*)(o_part + row * D + e * 16 + g4 * 4) = oacc[t][e] * wa + ob * wb;
                }
                if (g4 == 0) {
                    ml_part[row * 2] = mx;
                    ml_part[row * 2 + 1] = l;
                }
            }
        }
        wait_own_stores();
        __syncthreads();   // partial state acknowledged by the L2; hand-over buffers free again
        if (tid == 0) atomicAdd(sync + kCntAttn + head * kCntStride, 1u);

        // ---- merge: every workgroup of the head combines its share of the rows
        if (tid == 0) sm.wait_ok = bounded_wait(sync, sync + kCntAttn + head * kCntStride, (uint32_t)np * (epoch + 1), 2000u);
        __syncthreads();
        if (!sm.wait_ok) return false;    // the other parts never arrived: nothing sensible to write
        int r0 = M * me / np, r1 = M * (me + 1) / np;
        for (int m = r0 + wave; m < r1; m += 8) {
            // lane p holds the statistics of part p (np <= 64: one XCD's workgroups)
            float mq = -INFINITY, lq = 0.f;
            size_t rowq = 0;
            if (lane < np) {
                rowq = (size_t)(first + lane) * Mpad + m;
                mq = ml_part[rowq * 2];
                lq = ml_part[rowq * 2 + 1];
            }
            float mx = mq;
            for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
            float wq_ = (mq == -INFINITY) ? 0.f : fast_exp2(mq - mx);
            float den = wq_ * lq;
            for (int off = 32; off > 0; off >>= 1) den += __shfl_xor(den, off);
            // weighted sum of the parts' outputs, parts in index order, 8 loads in flight
            float num[D / 64];
#pragma unroll
            for (int e = 0; e < D / 64; ++e) num[e] = 0.f;
            for (int q0 = 0; q0 < np; q0 += 8) {
                float t[8][D / 64], w8[8];
#pragma unroll
                for (int qi = 0; qi < 8; ++qi) {
                    int qq = min(q0 + qi, np - 1);
                    size_t row = (size_t)__shfl((long long)rowq, qq);
                    w8[qi] = (q0 + qi < np) ? __shfl(wq_, qq) : 0.f;
#pragma unroll
                    for (int e = 0; e < D / 64; ++e) t[qi][e] = o_part[row * D + e * 64 + lane];
                }
#pragma unroll
                for (int qi = 0; qi < 8; ++qi)
#pragma unroll
                    for (int e = 0; e < D / 64; ++e) num[e] += w8[qi] * t[qi][e];
            }
#pragma unroll
            for (int e = 0; e < D / 64; ++e) {
                // a row that sees no key at all (possible with a caller's mask and an empty
                // cache) gets zeros
                const int col = head * D + e * 64 + lane;
                const size_t at = a.att_out_packed ? xpk_index(m, col, Mpad >> 4) : (size_t)m * nh * D + col;
                out[at] = (half_t)(den > 0.f ? num[e] / den : 0.f);
            }
        }
        // a workgroup that goes on to another head reuses its partial-state slot: wait until
        // the other parts have read it
        if (hl + 1 < h_hi) __syncthreads();
    }
    // a workgroup without a share of any head still checks in
    if (!gated && !gate()) return false;
    return true;
}

}  // namespace ghd

// The skinny linear layer: y[M, N] = x[M, K] W[N, K]^T with M <= 128 rows, one launch of one
// 512-thread workgroup per compute unit.
//
// The step re-reads every weight once per decoding step and is bound by that stream
// (Ghidorah, sections 2.1 and 2.2.2), so the kernel is built around it.  A workgroup's share
// is a group of R row tiles (16 output features each) and a k range.  Its eight wavefronts
// split the k range between them; each wavefront streams its k-steps of ALL the group's
// tiles (W is the MFMA A operand, fetched with non-temporal 128-bit loads straight into
// registers, a few k-steps ahead) together with the matching x fragments (the B operand,
// read as it lies in the packed activation layout, from the L2), and keeps one fp32
// accumulator fragment per (row tile, 16 rows of x).  There is no LDS staging and no barrier
// inside the stream: the wavefronts run independently until their k ranges end.  Then the
// eight partial fragments of every tile are added up through LDS, in wavefront order, and
// the reducing wavefront runs the layer's element-wise epilogue (residual add + sums of
// squares for the next RMSNorm, rotary embedding + KV append, SwiGLU).
//
// Two ways of dealing a matrix out (chosen on the host, see plan_linear).  Whole tiles: a
// share is a run of consecutive tiles over the whole k range; nothing is exchanged between
// workgroups, every workgroup reads all of x.  K ranges of four-tile row blocks (narrow
// matrices at more than 16 rows of x): a share reads only its k range of x, stores the
// block's partial sums, and the workgroups that share a block finish it jointly at the end
// of the launch, parts added in index order, so results never depend on timing.
#pragma once
#include "persist.h"

#include <type_traits>

namespace ghd {

struct GemmOp {
    const half8* W;
    int ntiles, nitems, nks, blk_shift;   // of the packed matrix (see WLayout)
    int N, K;
    int epi;
    const half8* in;     // packed activation layout, Mpad rows
    bool rscale;         // input is xg16: multiply output row m by rsqrt(mean x[m]^2 + eps) / kXgScale
    const half_t* gnext; // RESID: gain of the next RMSNorm (xg16 is rewritten), or nullptr
    void* out;           // STORE: y;  RESID: x;  SWIGLU: a16
    int64_t ldo;
    half_t *kc, *vc;     // QKV: this layer's cache
    uint32_t* cnt;       // the operation's counters
    uint32_t epoch;      // how many times these counters were used before (layer index)
    int passes;          // shares per workgroup
};


#ifndef GHD_RING_REGS
#define GHD_RING_REGS 80     // registers the load ring of a wavefront may take
#endif
#ifndef GHD_RING_KIB
#define GHD_RING_KIB 4       // weight bytes a wavefront keeps in flight, in KiB (more was measured slower)
#endif
// k-steps in flight per wavefront: limited by registers (accumulators + the ring) and by
// what the stream needs (a few KiB per wavefront: loads return in issue order, and a long
// queue only delays the x fragments behind it)
__host__ __device__ constexpr int pd_of(int MT, int R)
{
    int by_regs = GHD_RING_REGS / ((R + MT) * 4);
    int by_bytes = (GHD_RING_KIB + R - 1) / R;
    int pd = by_regs < by_bytes ? by_regs : by_bytes;
    return pd < 1 ? 1 : (pd > 8 ? 8 : pd);
}

// share of a group's k range, in 32nds, that the first wavefront of every SIMD's pair takes
// (measured on one box, alternating builds: 16 -> 3949 us per 64-row step, 17 -> 3896,
// 18 -> 3871, 19 -> 3899)
constexpr int kFirstSet = 18;

// ---------------------------------------------------------------------------
// epilogue of one 16x16 output fragment: lane (c, g4) holds y[m][n0 .. n0+3]
// ---------------------------------------------------------------------------
__device__ __forceinline__ void epilogue(const FusedArgs& a, const GemmOp& op, floatx4 v, int m, int n0,
                                         int lane, const float* s_rinv)
{
    // Everything below depends on the fragment's position: the (empty) asm keeps the compiler
    // from working parts of it out ahead of the weight stream, before the kernel's first loads.
    asm volatile("" : "+v"(m), "+v"(n0));
    const bool mok = m < a.M;
    const int mtp = a.Mpad >> 4;
    if (op.rscale) v *= s_rinv[m];
    if (op.epi == EPI_STORE_F32) {
        if (a.lin_amax) {
            // the row's best output among this tile's 16 columns: (largest value, lowest column).
            // Greedy acceptance (section 2.3) only needs the row argmax, so the finish of the
            // LM head leaves one candidate per tile and row instead of (or besides) the logits.
            float bv = -INFINITY;
            int bi = 0x7fffffff;
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (n0 + r < op.N && v[r] > bv) {
                    bv = v[r];
                    bi = n0 + r;
                }
#pragma unroll
            for (int off = 16; off < 64; off <<= 1) {
                const float ov = __shfl_xor(bv, off);
                const int oi = __shfl_xor(bi, off);
                if (ov > bv || (ov == bv && oi < bi)) {
                    bv = ov;
                    bi = oi;
                }
            }
            if (lane < 16 && mok) a.lin_amax[(size_t)(n0 >> 4) * a.Mpad + m] = make_float2(bv, __int_as_float(bi));
        }
        if (!mok || !op.out) return;
        float* o = (float*)op.out + (size_t)m * op.ldo + n0;
        if (n0 + 3 < op.N && (op.ldo & 3) == 0) *(floatx4*)o = v;
        else
            for (int r = 0; r < 4; ++r)
                if (n0 + r < op.N) o[r] = v[r];
    } else if (op.epi == EPI_STORE_F16) {
        if (!mok) return;
        half_t* o = (half_t*)op.out + (size_t)m * op.ldo + n0;
        for (int r = 0; r < 4; ++r)
            if (n0 + r < op.N) o[r] = (half_t)v[r];
    } else if (op.epi == EPI_RESID) {
        // x += y; sums of squares of the new x over this tile's 16 columns, per row
        float s = 0.f;
        if (mok && n0 < op.N) {
            floatx4* xp = (floatx4*)((float*)op.out + (size_t)m * op.ldo + n0);
            floatx4 xn = *xp + v;
            *xp = xn;
            s = xn[0] * xn[0] + xn[1] * xn[1] + xn[2] * xn[2] + xn[3] * xn[3];
            if (op.gnext) {
                half4 gv = *(const half4*)(op.gnext + n0), o;
#pragma unroll
                for (int r = 0; r < 4; ++r) o[r] = (half_t)(xn[r] * (float)gv[r] * kXgScale);
                *(half4*)(a.xg16 + xpk_index(m, n0, mtp)) = o;
            }
        }
        s += __shfl_xor(s, 16);
        s += __shfl_xor(s, 32);
        if (lane < 16 && n0 < op.N) a.ss[(size_t)(n0 >> 4) * a.Mpad + m] = s;
    } else if (op.epi == EPI_SWIGLU) {
        // packed rows: (gate f, gate f+1, up f, up f+1)
        if (!mok) return;
        int f = (n0 >> 4) * 8 + ((n0 & 15) >> 2) * 2;
        if (f >= a.F) return;
        // silu with the hardware's exp2 and reciprocal: a few ulp, far below the fp16 rounding
        // of the result (and 0.3 us per launch on the critical path)
        float a0 = __fdividef(v[0], 1.0f + __expf(-v[0])) * v[2];
        float a1 = __fdividef(v[1], 1.0f + __expf(-v[1])) * v[3];
        half2_ h = {(half_t)a0, (half_t)a1};
        *(half2_*)((half_t*)op.out + xpk_index(m, f, mtp)) = h;
    } else {   // EPI_QKV: packed rows of a head: (j, j+1, j+d/2, j+1+d/2)
        if (!mok || n0 >= op.N) return;
        int nh = a.nh, d = a.d;
        asm volatile("" : "+s"(nh), "+s"(d));     // (the divisions by these stay here, too)
        const int H = nh * d, hd = d >> 1;
        const QkvRow qr = qkv_row(n0, nh, d);
        const int part = qr.part, head = qr.head, ph = qr.ph;
        int jj = (ph >> 2) * 2;
        float o0 = v[0], o1 = v[1], o2 = v[2], o3 = v[3];
        if (part < 2) {
            float2 cs0 = a.rope[(size_t)m * hd + jj], cs1 = a.rope[(size_t)m * hd + jj + 1];
            o0 = v[0] * cs0.x - v[2] * cs0.y;
            o2 = v[2] * cs0.x + v[0] * cs0.y;
            o1 = v[1] * cs1.x - v[3] * cs1.y;
            o3 = v[3] * cs1.x + v[1] * cs1.y;
        }
        if (part == 2) {
            // V is kept channel-major: row kv_len + m of channels jj, jj+1, jj+d/2, jj+1+d/2
            half_t* col = op.vc + (size_t)head * a.v_stride_head + (size_t)(a.kv_len + m);
            col[(size_t)jj * a.v_stride_ch] = (half_t)o0;
            col[(size_t)(jj + 1) * a.v_stride_ch] = (half_t)o1;
            col[(size_t)(jj + hd) * a.v_stride_ch] = (half_t)o2;
            col[(size_t)(jj + 1 + hd) * a.v_stride_ch] = (half_t)o3;
            return;
        }
        half_t* dst = (part == 0)
                          ? a.q16 + (size_t)m * H + head * d + jj
                          : op.kc + (size_t)head * a.stride_head + (size_t)(a.kv_len + m) * a.stride_tok + jj;
        half2_ lo = {(half_t)o0, (half_t)o1}, hi = {(half_t)o2, (half_t)o3};
        *(half2_*)dst = lo;
        *(half2_*)(dst + hd) = hi;
    }
}

// keeps the compiler from moving memory operations, MFMAs or anything else across this point
// (a load ring only works if its loads are issued where they are written)
__device__ __forceinline__ void pin_order()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

// MT = 16-row tiles of x (Mpad / 16).  R = weight tiles streamed together.  RB = how the
// matrix is dealt out.  RB == 1: whole tiles - a share is up to R consecutive tiles over the
// whole k range, in either storage layout, and finishes them alone.  RB == 4 (== R): k ranges
// of the four-tile row blocks of a narrow matrix - a share streams the blocks its range touches
// one after the other, and a block whose k range is cut between shares is finished jointly.
// Returns false if a wait for another share's partial sums gave up.
template <int MT, int R, int RB>
__device__ __forceinline__ bool gemm_phase(const FusedArgs& a, const GemmOp& op, Ctx& cx)
{
    static_assert(RB == 1 || R == RB, "narrow matrices: the slots are the tiles of one row block");
    constexpr int NF = R * MT;                     // accumulator fragments per wavefront
    constexpr int FR = NF < 16 ? NF : 16;          // fragments reduced per round through LDS
    constexpr int PD = pd_of(MT, R);
    constexpr int NFI = RB * MT;                   // fragments of one row block
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, g4 = lane >> 4;
    const size_t lane16 = (size_t)(uint32_t)(lane * 16);   // this lane's 16 bytes of a 1 KiB block
    floatx4* red = (floatx4*)cx.lds;                       // [8][FR][64]
    float* s_rinv = (float*)(cx.lds + 8 * FR * 1024);      // 128 floats
    float* s_tmp = s_rinv + 128;                           // 1024 floats
    int* s_wait_ok = (int*)(s_tmp + 1024);                 // thread 0's verdict on a bounded wait
    const int nks = op.nks;
    const int blk_sh = op.blk_shift;        // tiles per storage block: 8 or 4
    const int L = cx.G * op.passes;
    const half8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};

    // ---- RMSNorm factor per row from the per-tile sums of squares ss[tile][Mpad], in two
    //      steps.  Early, behind the stream's first loads (it has to wait for those anyway):
    //      thread (rq, part) adds 4 rows of every P-th tile and the lanes of a wavefront that
    //      share rq are combined by shuffles - no barrier, so that no wavefront waits for
    //      another before it starts streaming.
    //      Late, when the stream is over and the workgroup meets anyway: the 8 wavefronts'
    //      sums are added through LDS.  Fixed order throughout.
    bool rinv_loaded = !op.rscale, rinv_ready = !op.rscale;
    floatx4 rs4 = {0.f, 0.f, 0.f, 0.f}, sst[8];
    constexpr int RQ = MT * 4, P = kFT / RQ;      // Mpad = 16 MT rows, four per thread
    const int n_ss = op.K >> 4, rq = tid % RQ, part = tid / RQ;
    auto rinv_request = [&](int t0) {
#pragma unroll
        for (int q = 0; q < 8; ++q)
            sst[q] = *(const floatx4*)(a.ss + (size_t)min(t0 + q * P, n_ss - 1) * a.Mpad + rq * 4);
    };
    auto rinv_add = [&](int t0) {
#pragma unroll
        for (int q = 0; q < 8; ++q)
            if (t0 + q * P < n_ss) rs4 += sst[q];
    };
    auto rinv_sum = [&]() {
        for (int t0 = part; t0 < n_ss; t0 += 8 * P) {
            rinv_request(t0);
            rinv_add(t0);
        }
        for (int off = RQ; off < 64; off <<= 1) {
#pragma unroll
            for (int r = 0; r < 4; ++r) rs4[r] += __shfl_xor(rs4[r], off);
        }
        rinv_loaded = true;
    };
    // (the barrier that makes s_rinv visible is the first one of the reduction that follows)
    auto rinv_finish = [&]() {
        if (lane < RQ) *(floatx4*)(s_tmp + (wave * RQ + lane) * 4) = rs4;
        __syncthreads();
        if (tid < MT * 16) {
            float tot = 0.f;
            for (int w = 0; w < 8; ++w) tot += s_tmp[(w * RQ + (tid >> 2)) * 4 + (tid & 3)];
            s_rinv[tid] = (1.0f / kXgScale) / sqrtf(tot / (float)op.K + a.eps);
        }
        rinv_ready = true;
    };

    // Share ls of the launch.  RB == 1: the tiles are dealt out, c0 .. c1 are tile indices and
    // every share covers the whole k range of its tiles - nothing is shared between shares.
    // RB == 4: the k-steps of the four-tile row blocks are dealt out, c0 .. c1 are indices into
    // the sequence [block][k-step]; a block whose k range is cut is finished jointly.
    auto share_of = [&](int ls) {
        return RB == 1 ? make_share(op.ntiles, 1, ls, L) : make_share(op.nitems, nks, ls, L);
    };
    auto is_shared = [&](const Share& sh, int block) { return RB != 1 && sh.first_of(block) != sh.last_of(block); };
    // Slot 0 of a share holds the partial sums of the row block its range begins in, slot 1
    // those of the block it ends in (when that is another one); blocks in between are whole.
    auto slot_of = [&](const Share& sh, int ls, int block) -> float* {
        return a.part + ((size_t)ls * 2 + (sh.begins_in(ls, block) ? 0 : 1)) * (size_t)(NFI * 256);
    };
    // A shared block is counted on the line of its first part (a share is the first part of
    // at most one shared block: the one its range ends in).
    auto counter_of = [&](int first) { return op.cnt + first * kCntStride; };

    // ---- one group of R tile slots streamed together over the k-steps k0 .. k1 - 1.
    //      RB == 1: the tiles first .. first + count - 1 (count <= R; the other slots re-read
    //      slot 0's blocks, and what they accumulate is never looked at).
    //      RB == 4: the four tiles of row block `first`.
    auto run_group = [&](int ls, int first, int count, int k0, int k1) {
        int s_blk[R];       // index of the 1 KiB block of the slot's k-step 0
#pragma unroll
        for (int t = 0; t < R; ++t) {
            const int tile = first + (t < count ? t : 0);
            s_blk[t] = RB == 1 ? (tile >> blk_sh) * (nks << blk_sh) + (tile & ((1 << blk_sh) - 1)) : first * nks * RB + t;
        }
        // This wavefront's k-steps.  Wavefronts w and w + 4 share a SIMD, and the first of the
        // two gets its data sooner throughout the stream (measured: with equal ranges
        // wavefronts 0-3 end 2.5-6 us before 4-7, which then stream on alone, no faster).
        // So the first four split kFirstSet/32 of the range between them, the other four the rest.
        const int n = k1 - k0, n_a = n * kFirstSet / 32, w4 = wave & 3;
        const int ws = wave < 4 ? k0 + n_a * w4 / 4 : k0 + n_a + (n - n_a) * w4 / 4;
        const int we = wave < 4 ? k0 + n_a * (w4 + 1) / 4 : k0 + n_a + (n - n_a) * (w4 + 1) / 4;
        const int s_hi = max(we - 1, k0);       // loads never go past the wavefront's last k-step

        half8 wr[PD][R], xr[PD][MT];
        floatx4 acc[R][MT];
#pragma unroll
        for (int t = 0; t < R; ++t)
#pragma unroll
            for (int b = 0; b < MT; ++b) acc[t][b] = (floatx4){0.f, 0.f, 0.f, 0.f};

        // All loads are unconditional (clamped addresses): the compiler's wait counts then
        // stay exact and the queue is never drained inside the loop.  K-steps past the
        // wavefront's range are re-reads of its last one; they are zeroed before use.
        auto load = [&](auto slot, int s) {
            constexpr int p = decltype(slot)::value;
            const int sl = min(s, s_hi);
            const char* xq = (const char*)op.in + ((size_t)(sl * MT) << 10);
#pragma unroll
            for (int b = 0; b < MT; ++b) xr[p][b] = *(const half8*)(xq + (b << 10) + lane16);
#pragma unroll
            for (int t = 0; t < R; ++t) {
                const char* wq = (const char*)op.W + ((size_t)(s_blk[t] + (RB == 1 ? sl << blk_sh : sl * RB)) << 10);
                wr[p][t] = __builtin_nontemporal_load((const half8*)(wq + lane16));
            }
        };
        // MASKED: k-steps past the wavefront's range, and columns past K in the last k-step,
        // count as zeros (the x fragments are zeroed: one select for all the slots).
        auto compute = [&](auto masked, auto slot, int s) {
            constexpr int p = decltype(slot)::value;
            constexpr bool MASKED = decltype(masked)::value;
            half8 xf[MT];
            if constexpr (MASKED) {
                const bool use = s < we && s * 32 + g4 * 8 < op.K;
#pragma unroll
                for (int b = 0; b < MT; ++b) xf[b] = use ? xr[p][b] : zero8;
            } else {
#pragma unroll
                for (int b = 0; b < MT; ++b) xf[b] = xr[p][b];
            }
#pragma unroll
            for (int t = 0; t < R; ++t)
#pragma unroll
                for (int b = 0; b < MT; ++b)
                    acc[t][b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wr[p][t], xf[b], acc[t][b], 0, 0, 0);
        };
        auto ring = [&](auto self, auto masked, auto slot, int s) {
            constexpr int p = decltype(slot)::value;
            if constexpr (p < PD) {
                compute(masked, slot, s + p);
                pin_order();
                load(slot, s + p + PD);
                pin_order();
                self(self, masked, std::integral_constant<int, p + 1>{}, s);
            }
        };
        auto prologue = [&](auto self, auto slot) {
            constexpr int p = decltype(slot)::value;
            if constexpr (p < PD) {
                load(slot, ws + p);
                pin_order();
                self(self, std::integral_constant<int, p + 1>{});
            }
        };
        // The norm factors are only needed by the epilogues, but their loads are cheapest here.
        prologue(prologue, std::integral_constant<int, 0>{});
        if (!rinv_loaded) rinv_sum();
        // (the share's place among its neighbours is only needed for the finish: worked out
        // here, while the first weights are on their way)
        bool shared = false;
        int first_part = 0;
        float* my_slot = nullptr;
        if constexpr (RB != 1) {
            const Share sh = share_of(ls);
            first_part = sh.first_of(first);
            shared = first_part != sh.last_of(first);
            my_slot = slot_of(sh, ls, first);
        }
        {
            // whole rings of k-steps that need no masking first, then the rest
            const bool plain = (op.K & 31) == 0 || we < nks;
            int s = ws;
            if (plain)
                for (; s + PD <= we; s += PD) ring(ring, std::false_type{}, std::integral_constant<int, 0>{}, s);
            for (; s < we; s += PD) ring(ring, std::true_type{}, std::integral_constant<int, 0>{}, s);
        }

        // ---- the eight k slices are added up through LDS, FR fragments per round; wavefront
        //      w reduces fragments w, w + 8 of the round (in wavefront order) and finishes them:
        //      the layer's epilogue, or - for a row block that other shares have parts of -
        //      a store of the partial sums, which are signalled once all of them are stored.
        if (!rinv_ready) rinv_finish();
        constexpr int kLastRound = (NF - 1) / FR;
#pragma unroll
        for (int r0 = 0; r0 < NF; r0 += FR) {
#pragma unroll
            for (int ff = 0; ff < FR; ++ff)
                if (r0 + ff < NF) red[(wave * FR + ff) * 64 + lane] = acc[(r0 + ff) / MT][(r0 + ff) % MT];
            __syncthreads();
            for (int ff = wave; ff < FR && r0 + ff < NF; ff += 8) {
                floatx4 v = red[ff * 64 + lane];
#pragma unroll
                for (int w = 1; w < 8; ++w) v += red[(w * FR + ff) * 64 + lane];
                const int f = r0 + ff, t = f / MT, b = f % MT;
                if (RB == 1 && t >= count) continue;
                const int tile = RB == 1 ? first + t : first * RB + t;
                if (!shared)
                    epilogue(a, op, v, b * 16 + c, tile * 16 + g4 * 4, lane, s_rinv);
                else
                    *(floatx4*)(my_slot + ((size_t)(t * MT + b) * 64 + lane) * 4) = v;
            }
            if (shared && r0 / FR == kLastRound) wait_own_stores();   // the partials are in the L2
            __syncthreads();
            if (shared && r0 / FR == kLastRound && tid == 0) atomicAdd(counter_of(first_part), 1u);
        }
        return shared;
    };

    // ---- the shares of this workgroup, one after the other.  With one share per workgroup
    //      its range comes from the table in the argument block.
    bool shared_any = false;
    for (int p = 0; p < op.passes; ++p) {
        const int ls = cx.j * op.passes + p;
        int c0, c1;
        if (RB != 1 || a.lin_range_ok) {       // (the row-block cut always has one share per workgroup)
            c0 = (int)a.lin_range[2 * cx.j];   // a scalar load from the argument block
            c1 = (int)a.lin_range[2 * cx.j + 1];
        } else {
            const Share sh = share_of(ls);
            c0 = sh.c0;
            c1 = sh.c1;
        }
        if (c0 >= c1) continue;
        if constexpr (RB == 1) {
            run_group(ls, c0, c1 - c0, 0, nks);      // (the launch was planned for c1 - c0 <= R)
        } else {
            const int it0 = c0 / nks, it1 = (c1 - 1) / nks;
            for (int it = it0; it <= it1; ++it)
                shared_any = run_group(ls, it, RB, max(c0 - it * nks, 0), min(c1 - it * nks, nks)) || shared_any;
        }
    }
    if (!shared_any) return true;

    // ---- joint finish of the shared row blocks this workgroup has parts of.  All its partial
    //      sums were stored and signalled before it waits for anybody else's.
    for (int p = 0; p < op.passes; ++p) {
        const int ls = cx.j * op.passes + p;
        const Share sh = share_of(ls);
        if (sh.c0 >= sh.c1) continue;
        const int it0 = sh.c0 / nks, it1 = (sh.c1 - 1) / nks;
        for (int k = 0; k < 2; ++k) {
            const int block = k ? it1 : it0;
            if (k && it1 == it0) break;
            if (!is_shared(sh, block)) continue;
            const int first = sh.first_of(block), last = sh.last_of(block);
            const int np = last - first + 1, me = ls - first;
            if (tid == 0)
                *s_wait_ok = bounded_wait(a.sync, counter_of(first), (uint32_t)np * (op.epoch + 1), 1000u + op.epi);
            __syncthreads();
            if (!*s_wait_ok) return false;    // the other parts never arrived: nothing sensible to write
            const int f0 = NFI * me / np, f1 = NFI * (me + 1) / np;
            for (int f = f0 + wave; f < f1; f += 8) {
                // Sum the parts in index order (fixed order: the result does not depend on
                // timing), eight loads in flight at a time.
                const size_t foff = ((size_t)f * 64 + lane) * 4;
                floatx4 v = *(const floatx4*)(slot_of(sh, first, block) + foff);
                for (int p0 = 1; p0 < np; p0 += 8) {
                    floatx4 t[8];
#pragma unroll
                    for (int q = 0; q < 8; ++q)
                        if (p0 + q < np) t[q] = *(const floatx4*)(slot_of(sh, first + p0 + q, block) + foff);
#pragma unroll
                    for (int q = 0; q < 8; ++q)
                        if (p0 + q < np) v += t[q];
                }
                const int tile = block * RB + f / MT, b = f % MT;
                epilogue(a, op, v, b * 16 + c, tile * 16 + g4 * 4, lane, s_rinv);
            }
        }
    }
    return true;
}

__device__ __forceinline__ GemmOp linear_op_of(const FusedArgs& a)
{
    GemmOp op;
    op.W = a.lin_W;
    op.N = a.lin_N;
    op.K = a.lin_K;
    op.ntiles = a.lin_ntiles;
    op.nitems = a.lin_nitems;
    op.nks = a.lin_nks;
    op.blk_shift = a.lin_blk_shift;
    op.epi = a.lin_epi;
    op.in = (const half8*)a.lin_x;
    op.rscale = a.lin_rscale != 0;
    op.gnext = a.lin_gnext;
    op.out = a.lin_y;
    op.ldo = a.lin_ldy;
    op.kc = a.lin_kc;
    op.vc = a.lin_vc;
    op.cnt = a.sync + a.lin_cnt;
    op.epoch = a.lin_epoch;
    op.passes = a.lin_passes;
    return op;
}

template <int MT, int R, int RB>
__global__ __launch_bounds__(kFT) void k_linear(const FusedArgs a)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    touch_kernel_arguments();
    Ctx cx = make_ctx(a, lds);
    const GemmOp op = linear_op_of(a);
    gemm_phase<MT, R, RB>(a, op, cx);
}

// The launch's argument block with the facts the host can work out for the kernel: the packed
// matrix' layout and, when there is one share per workgroup and the grid fits the table, every
// workgroup's work share (the same make_share the kernel would evaluate).
static inline FusedArgs with_launch_facts(const FusedArgs& a, int G)
{
    FusedArgs b = a;
    const WLayout lay = w_layout(a.lin_N, a.lin_K);
    const bool whole = lay.rb == 1 || a.lin_whole;
    b.lin_ntiles = lay.ntiles;
    b.lin_nitems = lay.nitems;
    b.lin_nks = lay.nks;
    b.lin_blk_shift = lay.blk == kWideBlock ? 3 : 2;
    static_assert(kWideBlock == 8 && kRbNarrow == 4, "storage blocks of 8 or 4 tiles");
    b.lin_range_ok = a.lin_passes == 1;     // (launches have at most kRangeWgs workgroups)
    if (b.lin_range_ok)
        for (int j = 0; j < G; ++j) {
            const Share sh = whole ? make_share(lay.ntiles, 1, j, G) : make_share(lay.nitems, lay.nks, j, G);
            b.lin_range[2 * j] = (uint32_t)sh.c0;
            b.lin_range[2 * j + 1] = (uint32_t)sh.c1;
        }
    return b;
}

template <int MT, int R>
constexpr size_t linear_lds_bytes()
{
    return 8 * (size_t)(R * MT < 16 ? R * MT : 16) * 1024 + (128 + 1024 + 4) * sizeof(float);
}

template <int MT, int R, int RB>
static ghd_status launch_linear_t(const FusedArgs& a, hipStream_t st)
{
    int G = 0;
    const size_t lds = linear_lds_bytes<MT, R>();
    ghd_status s = launch_resident_checked((const void*)k_linear<MT, R, RB>, (MT * 16 + R) * 8 + RB, lds, &G);
    if (s) return s;
    hipLaunchKernelGGL((k_linear<MT, R, RB>), dim3(G), dim3(kFT), lds, st, with_launch_facts(a, G));
    return check_launch();
}

// the instantiations of one M range; slots = row tiles a share handles at once
template <int MT>
ghd_status launch_linear_mt(const FusedArgs& a, hipStream_t st)
{
    const WLayout lay = w_layout(a.lin_N, a.lin_K);
    if (lay.rb != 1 && !a.lin_whole) return launch_linear_t<MT, kRbNarrow, kRbNarrow>(a, st);
    constexpr int CAP = MT <= 4 ? 8 : 4;
    switch (a.lin_slots) {
    case 1: return launch_linear_t<MT, 1, 1>(a, st);
    case 2: return launch_linear_t<MT, 2, 1>(a, st);
    case 3: return launch_linear_t<MT, 3, 1>(a, st);
    case 4: return launch_linear_t<MT, 4, 1>(a, st);
    default: break;
    }
    if constexpr (CAP >= 8) {
        switch (a.lin_slots) {
        case 5: return launch_linear_t<MT, 5, 1>(a, st);
        case 6: return launch_linear_t<MT, 6, 1>(a, st);
        case 7: return launch_linear_t<MT, 7, 1>(a, st);
        case 8: return launch_linear_t<MT, 8, 1>(a, st);
        default: break;
        }
    }
    return GHD_ERR_SHAPE;
}

ghd_status launch_linear_mt1(const FusedArgs& a, hipStream_t st);
ghd_status launch_linear_mt2(const FusedArgs& a, hipStream_t st);
ghd_status launch_linear_mt4(const FusedArgs& a, hipStream_t st);
ghd_status launch_linear_mt8(const FusedArgs& a, hipStream_t st);

}  // namespace ghd

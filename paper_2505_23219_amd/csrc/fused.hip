// The two persistent kernels of the verification step: skinny linear layers and
// tree attention.
//
// The step is a chain of short, strictly dependent, bandwidth-bound operations
// (Ghidorah, section 2.1: every decoding step re-reads all weights; section
// 2.2.2: per layer QKV linear, attention, output linear, two MLP linears).  Each
// of them is one launch with one workgroup per compute unit, all resident, that
// cuts the operation's byte stream into equal contiguous shares whatever its
// shape; the layer's element-wise work rides on those launches.
//
// Skinny linear layers.  W is packed in row groups of 256 output features
// (16 tiles of 16 rows), inside a group k-step major: one k-step of a group is
// 16 KiB, tile t of it is the 1 KiB A operand of v_mfma_f32_16x16x32_f16.  The
// chunks (4 k-steps of one group) of a matrix form one linear sequence that is
// cut into equal contiguous ranges, one per workgroup, whatever the shape
// (no tile quantisation).  Wavefront w owns tiles 2w, 2w+1 of the group; x is
// staged through LDS in B-operand order, double buffered, shared by all eight
// wavefronts.  A group whose K range is split over several workgroups is
// finished cooperatively: every part stores its fp32 partial tile sums, bumps
// the group's counter, waits (bounded) for the other parts, then reduces and
// post-processes its own share of the group's fragments in a fixed order, so
// results do not depend on timing.  The post-processing is the layer's
// element-wise work: residual add + sums of squares for the next RMSNorm,
// rotary embedding + KV append, SwiGLU.  RMSNorm is split around the GEMM that
// consumes it: the producer of the residual stream also leaves fp16(x * g / 16),
// which is staged like any fp16 input, and the row factor 16 * rsqrt(mean x^2 + eps)
// (a per-row scalar, so it commutes with the contraction) is applied to the fp32
// sums in the epilogue.  The 1/16 keeps x * g inside the fp16 range.
//
// Tree attention.  A head's 64-key tiles are split over a run of workgroups of
// one XCD.  A workgroup streams its tiles through LDS (the V cache is kept
// channel-major, so both K rows and V^T rows go to LDS as they are); wavefronts
// 0-3 take the first 32 keys of a tile, 4-7 the last 32, each for its own 16 (or
// 32) query rows.  S^T = K q^T puts one query row in each lane column, so softmax
// statistics are per-lane scalars, the fp16 probabilities are already in
// B-operand layout for O^T += V^T P^T, and the ancestor mask (section 2.3) is a
// 128-bit register per lane.  Sub-tiles no row can see are skipped.  The two key
// halves are merged inside the workgroup, the workgroups of a head through one
// partial state each, with the online-softmax rescale of section 3.2.2.
#include "fused.h"

#include <type_traits>

namespace ghd {

constexpr int kFrag = 4 * 272;              // LDS bytes of one padded 16x32 B fragment
constexpr long long kWaitTicks = 2000000;   // bounded waits give up after 20 ms (100 MHz clock)

struct GemmOp {
    const half8* W;
    int N, K;            // logical output features (packed order) and input features
    int ngroups, ncpg;   // row groups, chunks per group
    int epi;
    const half_t* in16;  // fp16 input [M, ld_in]
    int64_t ld_in;
    bool rscale;         // input is xg16: multiply output row m by 16 * rsqrt(mean x[m]^2 + eps)
    const half_t* gnext; // RESID: gain of the next RMSNorm (xg16 is rewritten), or nullptr
    void* out;           // STORE: y;  RESID: x;  SWIGLU: a16
    int64_t ldo;
    half_t *kc, *vc;     // QKV: this layer's cache
    uint32_t* cnt;       // the operation's group counters
    uint32_t epoch;      // how many times these counters were used before (layer index)
};

struct Ctx {
    int j, G;            // logical workgroup index, number of workgroups
    char* lds;           // dynamic LDS
};

__device__ __forceinline__ uint32_t ld_relaxed(const uint32_t* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Work shares.  A phase has `items` (row groups, or heads) of `per_item` units (chunks,
// or key tiles) each.  Items are dealt to the 8 XCDs in contiguous blocks, and the units
// of an XCD's items to its workgroups in equal contiguous ranges.  Workgroup i runs on
// XCD i % 8 (checked at kernel start), so the logical index j = (i % 8) * G/8 + i / 8
// puts the G/8 workgroups of an XCD side by side.  An item that is split over several
// workgroups is therefore always finished inside one XCD, and its partial results are
// exchanged through that XCD's L2 with plain stores and loads: every wavefront waits for
// the acknowledgement of its own stores before the barrier after which thread 0 bumps the
// item's counter, and a reader's first access to a slot line in a launch cannot hit in
// its L1.  No device-scope fence (a write-back and invalidate of a whole L2, about
// 4 us here) is needed anywhere inside a phase.
struct Share {
    int U;        // units of this XCD (fits 32 bits together with the factor Ge)
    int base;     // global index of its first unit (the unit count of an operation fits 31 bits)
    int Ge;       // workgroups of this XCD that get units
    int wg0;      // logical index of its first workgroup
    int c0, c1;   // this workgroup's range of global unit indices (empty if c0 == c1)
    int per_item;
    // local (within-XCD) unit index where workgroup wg's range begins
    __host__ __device__ int lbegin(int wg) const { return (int)((unsigned)U * (unsigned)(wg - wg0) / (unsigned)Ge); }
    __host__ __device__ int owner_local(int lunit) const
    {
        return wg0 + (int)(((unsigned)(lunit + 1) * (unsigned)Ge - 1u) / (unsigned)U);
    }
    __host__ __device__ int litem0(int item) const { return item * per_item - base; }
    __host__ __device__ int first_of(int item) const { return owner_local(litem0(item)); }
    __host__ __device__ int last_of(int item) const { return owner_local(litem0(item) + per_item - 1); }
    // does workgroup wg's range begin inside `item` (and not in an earlier one)?
    __host__ __device__ bool begins_in(int wg, int item) const { return lbegin(wg) >= litem0(item); }
};

__host__ __device__ __forceinline__ Share make_share(int items, int per_item, int j, int G)
{
    const int nx = (G % 8 == 0) ? 8 : 1;
    const int Gx = G / nx, x = j / Gx;
    const int i0 = items * x / nx, i1 = items * (x + 1) / nx;
    Share sh;
    sh.per_item = per_item;
    sh.U = (i1 - i0) * per_item;
    sh.base = i0 * per_item;
    sh.wg0 = x * Gx;
    sh.Ge = sh.U < Gx ? sh.U : Gx;
    sh.c0 = sh.c1 = 0;
    if (j - sh.wg0 < sh.Ge) {
        sh.c0 = sh.base + sh.lbegin(j);
        sh.c1 = sh.base + ((j + 1 - sh.wg0 < sh.Ge) ? sh.lbegin(j + 1) : sh.U);
    }
    return sh;
}

// Every wavefront calls this before the barrier that precedes a counter bump: it returns
// once the wavefront's own stores have been acknowledged by the L2, i.e. are visible to
// the other compute units of the XCD.  (The barrier alone orders the wavefronts of the
// workgroup, not their stores still on the way to the L2.)  s_waitcnt vmcnt(0).
__device__ __forceinline__ void wait_own_stores() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// Waits until *p >= target.  Gives up (and raises the status word to `code`) after
// kWaitTicks of wall-clock time, or as soon as another workgroup has given up, so that a
// launch that is not fully resident ends with an error instead of hanging.  One thread calls.
__device__ __forceinline__ uint32_t poll(uint32_t* p)
{
    // a read-modify-write that changes nothing: it is served where the counting atomics
    // are, so it sees them at once (a device-scope load lags them by several microseconds)
    return atomicOr(p, 0u);
}

__device__ __forceinline__ void bounded_wait(uint32_t* sync, uint32_t* p, uint32_t target,
                                             uint32_t code)
{
    if (poll(p) >= target) return;
    const long long t0 = wall_clock64();
    while (poll(p) < target) {
        if (wall_clock64() - t0 > kWaitTicks || ld_relaxed(sync + kSyncStatus) != 0) {
            atomicCAS(sync + kSyncStatus, 0u, code);
            break;
        }
        __builtin_amdgcn_s_sleep(8);
    }
}

// ---------------------------------------------------------------------------
// epilogue of one 16x16 output fragment: lane (c, g4) holds y[m][n0 .. n0+3]
// ---------------------------------------------------------------------------
constexpr float kXgScale = 0.0625f;   // xg16 = fp16(x * g * kXgScale)

__device__ __forceinline__ void epilogue(const FusedArgs& a, const GemmOp& op, floatx4 v, int m, int n0,
                                int lane, const float* s_rinv)
{
    const bool mok = m < a.M;
    if (op.rscale) v *= s_rinv[m];
    if (op.epi == EPI_STORE_F32) {
        if (!mok) return;
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
                *(half4*)(a.xg16 + (size_t)m * op.ldo + n0) = o;
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
        float a0 = v[0] / (1.0f + expf(-v[0])) * v[2];
        float a1 = v[1] / (1.0f + expf(-v[1])) * v[3];
        half2_ h = {(half_t)a0, (half_t)a1};
        *(half2_*)((half_t*)op.out + (size_t)m * op.ldo + f) = h;
    } else {   // EPI_QKV: packed rows of a head: (j, j+1, j+d/2, j+1+d/2)
        if (!mok || n0 >= op.N) return;
        const int H = a.H, d = a.d, hd = a.d >> 1;
        int part = n0 / H, hn = n0 - part * H;
        int head = hn / d, ph = hn - head * d;
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

// ---------------------------------------------------------------------------
// one skinny linear layer
// ---------------------------------------------------------------------------
//
// RS (1, 2 or 4) cuts every 256-row group of the packed matrix into RS row slices of
// TGS = 16 / RS tiles; a slice is the item of the work shares, and a chunk is 4 * RS k-steps
// of a slice (64 KiB whatever RS).  The 8 wavefronts form 8 / RS tile pairs times RS
// k-slices: wavefront w streams tiles 2 tp, 2 tp + 1 (tp = w % (8 / RS)) for k-steps
// 4 ksl .. 4 ksl + 3 (ksl = w / (8 / RS)) of every chunk, and the k-slices are added up
// through LDS when a row slice ends.  A larger RS means smaller partial sums where the K
// range of a slice is split between workgroups (their traffic goes with 1 / RS) and more of
// x staged per workgroup (goes with RS).
template <int MT, int RS>
__device__ __forceinline__ void gemm_phase(const FusedArgs& a, const GemmOp& op, Ctx& cx)
{
    constexpr int TGS = kTG / RS;                  // tiles of a row slice
    constexpr int TP = TGS / 2;                    // tile pairs = wavefronts per k-slice
    constexpr int KS = kCH * RS;                   // k-steps of a chunk
    constexpr int CHUNK = KS * MT * kFrag;         // LDS bytes of one staged x chunk
    constexpr int PIECES = KS * MT * 64;           // 16-byte pieces per chunk
    constexpr int PPT = (PIECES + kFT - 1) / kFT;
    constexpr int NF = TGS * MT;                   // fragments of one row slice
    static_assert((8 / RS) * RS == 8 && TP >= 1, "RS is 1, 2 or 4");
    static_assert((RS - 1) * TP * 2 * MT * 1024 <= CHUNK, "the k-slice sums go through one x buffer");
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int c = lane & 15, g4 = lane >> 4;
    const int tp = wave % TP, ksl = wave / TP;
    const int nks = ((op.K + kChunkCols - 1) / kChunkCols) * kCH;   // k-steps of the packed matrix
    char* xs = cx.lds;                             // 2 * CHUNK
    float* s_rinv = (float*)(cx.lds + 2 * CHUNK);  // Mpad floats
    float* s_tmp = s_rinv + 128;                   // 1024 floats

    const Share sh = make_share(op.ngroups, op.ncpg, cx.j, cx.G);
    const int c0 = sh.c0, c1 = sh.c1;
    const half8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};

    // ---- weight stream: linear in the chunk index
    // One chunk of weights is in flight per wavefront, in registers: k-step s of the next
    // chunk is requested right after k-step s of the current one has been consumed.  (Two
    // chunks in flight were measured slower at every M: the extra registers and the longer
    // fill cost more than the deeper queue gains.)
    half8 wb[kCH][2];
    const half8* wp_next;        // this wavefront's first tile, k-step 0 of its group
    int ks_next;                 // its first k-step in the chunk w_locate() was called for
    auto w_locate = [&](int cu) {
        int sg = cu / op.ncpg, kc = cu - sg * op.ncpg;
        int grp = sg / RS, q = sg - grp * RS;
        wp_next = op.W + ((size_t)grp * nks * kTG + q * TGS + tp * 2) * 64 + lane;
        ks_next = kc * KS + ksl * kCH;
    };
    // Loads inside the streaming loop are unconditional (the tail is peeled instead): a load
    // that may or may not be issued makes the number of younger loads unknown, and every
    // wait for an older one then has to drain the whole queue.
    // k-steps past the end of the matrix (ragged last chunk of a slice) re-read the last
    // one: their x is staged as zeros
    auto w_fetch = [&](int s) {
        const half8* p = wp_next + (size_t)min(ks_next + s, nks - 1) * (kTG * 64);
        // streamed once: non-temporal, so the weights do not push x and the partial sums
        // out of the L2
        wb[s][0] = __builtin_nontemporal_load(p);
        wb[s][1] = __builtin_nontemporal_load(p + 64);
    };
    // ---- x staging: the chunk of a row is KS * 4 pieces of 16 bytes, contiguous in memory;
    //      piece p -> row p / (KS*4), piece kp = p % (KS*4) of it (k-step s = kp / 4, k group
    //      kp % 4): a wavefront's 64 pieces are whole 128-byte lines of a few rows
    int p_row[PPT], p_koff[PPT], p_dst[PPT];
    bool p_ok[PPT];
#pragma unroll
    for (int i = 0; i < PPT; ++i) {
        int p = tid + i * kFT;
        int m = p / (KS * 4), kp = p % (KS * 4);
        int s = kp >> 2, pg = kp & 3;
        int mt = m >> 4, pc = m & 15;
        int f = s * MT + mt;
        p_ok[i] = (p < PIECES) && (m < a.M);
        p_row[i] = min(m, a.M - 1);
        p_koff[i] = s * 32 + pg * 8;
        p_dst[i] = f * kFrag + pg * 272 + pc * 16;
    }
    half8 xr[PPT];
    bool xok[PPT];
    auto x_fetch = [&](int cu) {
        int kbase = (int)(min(cu, c1 - 1) % op.ncpg) * (KS * 32);
#pragma unroll
        for (int i = 0; i < PPT; ++i) {
            int k = kbase + p_koff[i];
            xok[i] = p_ok[i] && k < op.K;
            xr[i] = *(const half8*)(op.in16 + (size_t)p_row[i] * op.ld_in + (xok[i] ? k : 0));
        }
    };
    auto x_store = [&](int buf) {
#pragma unroll
        for (int i = 0; i < PPT; ++i)
            if (tid + i * kFT < PIECES) *(half8*)(xs + buf * CHUNK + p_dst[i]) = xok[i] ? xr[i] : zero8;
    };

    // Loads return in issue order: the first x chunk is requested ahead of the weight ring
    // so that staging does not wait behind the ring.
    auto w_first = [&]() {
        if (c0 >= c1) return;
        w_locate(c0);
#pragma unroll
        for (int s = 0; s < kCH; ++s) w_fetch(s);
    };
    if (c0 < c1) x_fetch(c0);
    w_first();

    // ---- RMSNorm factor per row from the per-tile sums of squares ss[tile][Mpad]:
    //      thread (rq, part) adds 4 rows of every P-th tile, lanes of a wavefront that share
    //      rq are combined by shuffles, the 8 wavefronts through LDS; fixed order throughout.
    //      Only the epilogue needs it, so it is computed late: after this workgroup has
    //      signalled its partial sums, while the other parts of the group are still arriving.
    bool rinv_ready = !op.rscale;
    auto compute_rinv = [&]() {
        const int n_ss = op.K >> 4;
        const int RQ = a.Mpad >> 2, P = kFT / RQ;
        const int rq = tid % RQ, part = tid / RQ;
        floatx4 s4 = {0.f, 0.f, 0.f, 0.f};
        for (int t0 = part; t0 < n_ss; t0 += 8 * P) {
            floatx4 sst[8];
#pragma unroll
            for (int q = 0; q < 8; ++q)
                sst[q] = *(const floatx4*)(a.ss + (size_t)min(t0 + q * P, n_ss - 1) * a.Mpad + rq * 4);
#pragma unroll
            for (int q = 0; q < 8; ++q)
                if (t0 + q * P < n_ss) s4 += sst[q];
        }
        for (int off = RQ; off < 64; off <<= 1) {
#pragma unroll
            for (int r = 0; r < 4; ++r) s4[r] += __shfl_xor(s4[r], off);
        }
        if (lane < RQ) *(floatx4*)(s_tmp + (wave * RQ + lane) * 4) = s4;
        __syncthreads();
        if (tid < a.Mpad) {
            float tot = 0.f;
            for (int w = 0; w < 8; ++w) tot += s_tmp[(w * RQ + (tid >> 2)) * 4 + (tid & 3)];
            s_rinv[tid] = (1.0f / kXgScale) / sqrtf(tot / (float)op.K + a.eps);
        }
        __syncthreads();
        rinv_ready = true;
    };

    floatx4 acc[2][MT];
    auto acc_zero = [&]() {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int b = 0; b < MT; ++b) acc[t][b] = (floatx4){0.f, 0.f, 0.f, 0.f};
    };
    acc_zero();

    // The parts of a row slice: workgroups first..last own pieces of its K range.  A
    // workgroup's range is contiguous, so only the slice it begins in and the slice it ends
    // in can be shared with others.  Slot 0 of a workgroup holds the partial of the slice
    // its range begins in, slot 1 that of the slice it ends in (when that is another one).
    auto slot_of = [&](int wg, int sg) -> float* {
        return a.part + ((size_t)wg * 2 + (sh.begins_in(wg, sg) ? 0 : 1)) * (size_t)(NF * 256);
    };
    // A shared slice is counted on the line of its first part (a workgroup is the first
    // part of at most one shared slice: the one its range ends in).
    auto counter_of = [&](int first) { return op.cnt + first * kCntStride; };
    // first output feature of tile `tile` of slice sg
    auto row0_of = [&](int sg, int tile) {
        int grp = sg / RS, q = sg - grp * RS;
        return (grp * kTG + q * TGS + tile) * 16;
    };

    // Ends the accumulation of row slice `sg`, whose last chunk was staged in x buffer
    // `buf`: the k-slices are added up (in index order) in the wavefronts of k-slice 0,
    // which then run the epilogue when this workgroup owns the whole K range, and otherwise
    // store the partial (the slice's counter is bumped once the whole share has been streamed).
    auto flush = [&](int sg, int buf) {
        const int first = sh.first_of(sg), last = sh.last_of(sg);
        if (first == last && !rinv_ready) compute_rinv();
        if constexpr (RS > 1) {
            // the buffer's x was consumed before the barrier that ended the chunk, and nothing
            // is staged into it before the next chunk's end
            floatx4* red = (floatx4*)(xs + buf * CHUNK);
            if (ksl > 0) {
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int b = 0; b < MT; ++b)
                        red[((((ksl - 1) * TP + tp) * 2 + t) * MT + b) * 64 + lane] = acc[t][b];
            }
            __syncthreads();
            if (ksl == 0) {
#pragma unroll
                for (int sl = 1; sl < RS; ++sl)
#pragma unroll
                    for (int t = 0; t < 2; ++t)
#pragma unroll
                        for (int b = 0; b < MT; ++b)
                            acc[t][b] += red[((((sl - 1) * TP + tp) * 2 + t) * MT + b) * 64 + lane];
            }
            __syncthreads();
        }
        if (ksl == 0) {
            if (first == last) {
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int b = 0; b < MT; ++b)
                        epilogue(a, op, acc[t][b], b * 16 + c, row0_of(sg, tp * 2 + t) + g4 * 4, lane, s_rinv);
            } else {
                float* slot = slot_of(cx.j, sg);
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int b = 0; b < MT; ++b)
                        *(floatx4*)(slot + ((size_t)((tp * 2 + t) * MT + b) * 64 + lane) * 4) = acc[t][b];
                // signalled after the loop: no barrier for it in the middle of the stream
            }
        }
        acc_zero();
    };

    if (c0 < c1) {
        x_store(0);
        x_fetch(c0 + 1);
        __syncthreads();
        // One chunk: this wavefront's 4 k-steps of MFMAs, each followed (FW) by the request
        // for the same k-step of the next chunk; then the next x chunk goes to LDS and the
        // one after it is requested.  No branches: the wait counts stay exact.
        auto chunk_step = [&](auto fw, int cu) {
            constexpr bool FW = decltype(fw)::value;
            const char* xb = xs + (int)((cu - c0) & 1) * CHUNK + ksl * (kCH * MT * kFrag) + g4 * 272 + c * 16;
            if constexpr (FW) w_locate(cu + 1);
#pragma unroll
            for (int s = 0; s < kCH; ++s) {
                // at most four x fragments live at a time (register budget at M > 64)
                constexpr int XB = MT > 4 ? 4 : MT;
#pragma unroll
                for (int b0 = 0; b0 < MT; b0 += XB) {
                    half8 xf[XB];
#pragma unroll
                    for (int b = 0; b < XB; ++b) xf[b] = *(const half8*)(xb + (s * MT + b0 + b) * kFrag);
#pragma unroll
                    for (int t = 0; t < 2; ++t)
#pragma unroll
                        for (int b = 0; b < XB; ++b)
                            acc[t][b0 + b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                                wb[s][t], xf[b], acc[t][b0 + b], 0, 0, 0);
                }
                if constexpr (FW) w_fetch(s);
            }
            x_store((int)((cu + 1 - c0) & 1));
            x_fetch(cu + 2);
            __syncthreads();
        };
        const int fend = c1 - 1;        // the last chunk has nothing left to prefetch
        for (int cu = c0; cu < c1;) {
            int sg = (int)(cu / op.ncpg);
            int se = min(c1, (sg + 1) * op.ncpg);
            int mid = min(se, max(fend, cu));
            for (int b = cu; b < mid; ++b) chunk_step(std::true_type{}, b);
            for (int b = mid; b < se; ++b) chunk_step(std::false_type{}, b);
            flush(sg, (int)((se - 1 - c0) & 1));
            cu = se;
        }

        // ---- cooperative finish of the shared slices this workgroup took part in
        int gfirst = (int)(c0 / op.ncpg), glast = (int)((c1 - 1) / op.ncpg);
        wait_own_stores();
        __syncthreads();                // every wavefront's partials have been acknowledged by the L2
        if (tid == 0)
            for (int sg = gfirst; sg <= glast; ++sg) {
                int first = sh.first_of(sg);
                if (first != sh.last_of(sg)) atomicAdd(counter_of(first), 1u);
            }
        if (!rinv_ready) compute_rinv();
        for (int sg = gfirst; sg <= glast; ++sg) {
            int first = sh.first_of(sg), last = sh.last_of(sg);
            if (first == last) continue;
            int np = last - first + 1, me = cx.j - first;
            if (tid == 0) bounded_wait(a.sync, counter_of(first), (uint32_t)np * (op.epoch + 1), 1000u + op.epi);
            __syncthreads();
            int f0 = NF * me / np, f1 = NF * (me + 1) / np;
            for (int f = f0 + wave; f < f1; f += 8) {
                // Sum the parts in index order (fixed order: the result does not depend on
                // timing), eight loads in flight at a time.  Parts after the first begin
                // inside this slice, so their partial is in their slot 0.
                const size_t foff = ((size_t)f * 64 + lane) * 4;
                floatx4 v = *(const floatx4*)(slot_of(first, sg) + foff);
                for (int p0 = 1; p0 < np; p0 += 8) {
                    floatx4 t[8];
#pragma unroll
                    for (int q = 0; q < 8; ++q)
                        if (p0 + q < np)
                            t[q] = *(const floatx4*)(a.part + (size_t)(first + p0 + q) * 2 * (NF * 256) + foff);
#pragma unroll
                    for (int q = 0; q < 8; ++q)
                        if (p0 + q < np) v += t[q];
                }
                int tile = f / MT, b = f % MT;
                epilogue(a, op, v, b * 16 + c, row0_of(sg, tile) + g4 * 4, lane, s_rinv);
            }
        }
    }
}

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
    half_t k[64 * KS];
    half_t vt[D * VS];
    // state of the wavefronts working on the second key half, handed to their partners on
    // the first half when a head ends: [row-tile slot][tile][fragment][lane]
    floatx4 o2[4][MTW][D / 16][64];
    float m2[4][MTW][64];
    float l2[4][MTW][64];
};

template <int MT, int D>
__device__ __forceinline__ void attn_phase(const FusedArgs& a, Ctx& cx, const half_t* q, const half_t* kc,
                           const half_t* vc, half_t* out, uint32_t epoch)
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

    for (int hl = h_lo; hl < h_hi; ++hl) {
        const int head = hx0 + hl;
        // the workgroups first .. first + np - 1 split this head's tiles
        const AttnTiles ts = attn_tiles(hs, hl, ntile);
        const int first = ts.first, np = ts.np, me = ts.me, t0 = ts.t0, t1 = ts.t1;
        if (me >= np) continue;                            // more workgroups than tiles
        const half_t* kh_ = kc + (size_t)head * a.stride_head;
        const half_t* vh_ = vc + (size_t)head * a.v_stride_head;

        // query fragments and running state of this head
        half8 qf[MTW][DS];
        float mrun[MTW], lrun[MTW];
        floatx4 oacc[MTW][DT];
#pragma unroll
        for (int t = 0; t < MTW; ++t) {
#pragma unroll
            for (int s = 0; s < DS; ++s) {
                half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
                if (mok[t]) v = *(const half8*)(q + ((size_t)mrow[t] * nh + head) * D + s * 32 + g4 * 8);
                qf[t][s] = v;
            }
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
                *(half8*)(&sm.k[k_row[i] * L::KS + k_off[i]]) = kreg[S][i];
                int vch = id >> 3, seg = id & 7;
                half8 v = vreg[S][i];
                int nvalid = T - (tile * 64 + seg * 8);  // rows from T on hold no data: zero them,
                if (nvalid < 8) {                        // a stray NaN times a zero weight is a NaN
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (e >= nvalid) v[e] = (half_t)0;
                }
                *(half8*)(&sm.vt[vch * L::VS + seg * 8]) = v;
            }
        };
        load_tile(s0);
        load_tile(s1);
        if constexpr (NT == 4) {
            load_tile(s2);
            load_tile(s3);
        }
        int p_tile = t0;                                   // the tile being processed
        auto do_tile = [&](auto set) {
            const int tile = p_tile++;
            __syncthreads();            // previous tile fully consumed
            store_tile(set, tile);
            __syncthreads();
            load_tile(set);
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
                        half8 kf = *(const half8*)(&sm.k[(kh * 32 + jx * 16 + c) * L::KS + ds * 32 + g4 * 8]);
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
                            half8 kf = *(const half8*)(&sm.k[(kh * 32 + jx * 16 + c) * L::KS + ds * 32 + g4 * 8]);
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
                const half_t* vrow = &sm.vt[(e * 16 + c) * L::VS + kh * 32];
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
                    do_tile(s0);
                    do_tile(s1);
                    do_tile(s2);
                    do_tile(s3);
                }
                if (u < t1) {
                    do_tile(s0);
                    if (u + 1 < t1) {
                        do_tile(s1);
                        if (u + 2 < t1) do_tile(s2);
                    }
                }
            } else {
                for (; u + 1 < t1; u += 2) {
                    do_tile(s0);
                    do_tile(s1);
                }
                if (u < t1) do_tile(s0);
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
        if (tid == 0) bounded_wait(sync, sync + kCntAttn + head * kCntStride, (uint32_t)np * (epoch + 1), 2000u);
        __syncthreads();
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
            for (int e = 0; e < D / 64; ++e)
                // a row that sees no key at all (possible with a caller's mask and an empty
                // cache) gets zeros
                out[((size_t)m * nh + head) * D + e * 64 + lane] = (half_t)(den > 0.f ? num[e] / den : 0.f);
        }
        // a workgroup that goes on to another head reuses its partial-state slot: wait until
        // the other parts have read it
        if (hl + 1 < h_hi) __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// the kernels
// ---------------------------------------------------------------------------
// Workgroups are dealt round-robin to the 8 XCDs; neighbours in the work sequence (which
// share row groups, or heads, and exchange partial results) get the same XCD.  The
// exchange relies on workgroup i running on XCD i % 8, which is checked here.
// The argument block is a few 64-byte lines of kernel-argument memory, which the compiler
// reads field by field as the code needs them, one memory round trip after the other.  One
// word of every line is requested here, back to back at the start of the kernel, so that
// the lines arrive together and the later reads find them in the scalar cache.
__device__ __forceinline__ uint32_t touch_kernel_arguments()
{
    typedef const __attribute__((address_space(4))) uint32_t* kernarg_words;
    kernarg_words kp = (kernarg_words)__builtin_amdgcn_kernarg_segment_ptr();
    uint32_t t = 0;
#pragma unroll
    for (int i = 0; i < (int)((sizeof(FusedArgs) + 63) / 64); ++i) t ^= kp[i * 16];
    return t;
}

__device__ __forceinline__ Ctx make_ctx(const FusedArgs& a, char* lds)
{
    Ctx cx;
    const int G = gridDim.x, i = blockIdx.x;
    cx.G = G;
    cx.j = (G % 8 == 0) ? (i % 8) * (G / 8) + i / 8 : i;
    cx.lds = lds;
    if (G % 8 == 0 && threadIdx.x == 0) {
        unsigned xcc = __builtin_amdgcn_s_getreg(20 | (31 << 11)) & 15u;   // HW_REG_XCC_ID
        if (xcc != (unsigned)(i % 8)) atomicCAS(a.sync + kSyncStatus, 0u, 3u);
    }
    return cx;
}

template <int MT, int RS>
__global__ __launch_bounds__(kFT) void k_linear(const FusedArgs a)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const uint32_t touched = touch_kernel_arguments();
    Ctx cx = make_ctx(a, lds);
    GemmOp op;
    op.W = a.lin_W;
    op.N = a.lin_N;
    op.K = a.lin_K;
    op.epi = a.lin_epi;
    op.in16 = a.lin_x;
    op.ld_in = a.lin_ldx;
    op.rscale = a.lin_rscale != 0;
    op.gnext = a.lin_gnext;
    op.out = a.lin_y;
    op.ldo = a.lin_ldy;
    op.kc = a.lin_kc;
    op.vc = a.lin_vc;
    op.cnt = a.sync + a.lin_cnt;
    op.epoch = a.lin_epoch;
    // items of the work shares: row slices, each of ncpg chunks of 4 * RS k-steps
    op.ngroups = ((op.N + kGroupRows - 1) / kGroupRows) * RS;
    op.ncpg = (op.K + kChunkCols * RS - 1) / (kChunkCols * RS);
    gemm_phase<MT, RS>(a, op, cx);
    // (keeps the early reads alive; never true: lin_N is positive)
    if (touched == 0x9e3779b9u && a.lin_N < 0) a.sync[kSyncStatus] = 4u;
}

template <int MT, int D>
__global__ __launch_bounds__(kFT) void k_attention(const FusedArgs a)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const uint32_t touched = touch_kernel_arguments();
    Ctx cx = make_ctx(a, lds);
    attn_phase<MT, D>(a, cx, a.att_q, a.att_k, a.att_v, a.att_out, a.att_epoch);
    // (keeps the early reads alive; never true: nh is positive)
    if (touched == 0x9e3779b9u && a.nh < 0) a.sync[kSyncStatus] = 4u;
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
// What is cached about a device (its compute units, which kernels have had their LDS size
// set on it) is kept per device: the current device of the calling thread decides.
constexpr int kMaxDevices = 64;
static int g_num_cu[kMaxDevices] = {};

static int current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return -1;
    return dev;
}

int fused_grid_size()
{
    const int dev = current_device();
    if (dev < 0) return 0;
    if (g_num_cu[dev] == 0) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return 0;
        g_num_cu[dev] = prop.multiProcessorCount;
    }
    return g_num_cu[dev];
}

template <int MT, int RS>
static size_t linear_lds_bytes()
{
    return 2 * (size_t)kCH * RS * MT * kFrag + (128 + 1024) * sizeof(float);
}

// All workgroups must be resident at once (they wait for each other): one per compute unit.
template <class Kernel>
static ghd_status launch_resident(Kernel kernel, bool (&checked_on)[kMaxDevices], size_t lds,
                                  const FusedArgs& a, hipStream_t st)
{
    const int dev = current_device();
    int G = fused_grid_size();
    if (dev < 0 || G <= 0 || G > 512) return hip_fail(hipErrorInvalidDevice);   // counter arrays hold 512 lines
    bool& checked = checked_on[dev];
    if (!checked) {
        hipError_t e = hipFuncSetAttribute((const void*)kernel,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return hip_fail(e);
        int per_cu = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kFT, lds);
        if (e != hipSuccess) return hip_fail(e);
        if (per_cu < 1) return hip_fail(hipErrorLaunchOutOfResources);
        checked = true;
    }
    hipLaunchKernelGGL(kernel, dim3(G), dim3(kFT), lds, st, a);
    return check_launch();
}

template <int MT, int RS>
static ghd_status launch_linear_t(const FusedArgs& a, hipStream_t st)
{
    static bool checked[kMaxDevices] = {};
    return launch_resident(k_linear<MT, RS>, checked, linear_lds_bytes<MT, RS>(), a, st);
}

// Row split of a linear layer (see gemm_phase).  The two x buffers of RS * MT * 4.25 KiB
// each have to fit the LDS: RS * MT <= 16.
template <int MT>
static ghd_status launch_linear_rs(const FusedArgs& a, hipStream_t st)
{
    int rs = a.lin_rs;
    if constexpr (MT * 4 <= 16)
        if (rs >= 4) return launch_linear_t<MT, 4>(a, st);
    if constexpr (MT * 2 <= 16)
        if (rs >= 2) return launch_linear_t<MT, 2>(a, st);
    return launch_linear_t<MT, 1>(a, st);
}

template <int MT, int D>
static ghd_status launch_attention_t(const FusedArgs& a, hipStream_t st)
{
    static bool checked[kMaxDevices] = {};
    return launch_resident(k_attention<MT, D>, checked, sizeof(AttnLds<MT, D>), a, st);
}

template <int D>
static ghd_status launch_attention_d(const FusedArgs& a, int mt, hipStream_t st)
{
    if (mt <= 1) return launch_attention_t<1, D>(a, st);
    if (mt <= 2) return launch_attention_t<2, D>(a, st);
    if (mt <= 4) return launch_attention_t<4, D>(a, st);
    return launch_attention_t<8, D>(a, st);
}

// a.mode selects the kernel; the row-tile count of M selects the instantiation
ghd_status launch_fused(const FusedArgs& a, hipStream_t st)
{
    const int mt = (a.M + 15) / 16;
    if (a.mode == MODE_LINEAR) {
        if (mt <= 1) return launch_linear_rs<1>(a, st);
        if (mt <= 2) return launch_linear_rs<2>(a, st);
        if (mt <= 4) return launch_linear_rs<4>(a, st);
        return launch_linear_rs<8>(a, st);
    }
    return a.d == 64 ? launch_attention_d<64>(a, mt, st) : launch_attention_d<128>(a, mt, st);
}

// The work-share arithmetic evaluated on the host (for tests of its invariants): the unit
// range of workgroup j, and for `item` its first and last part and whether j's range begins
// in it.  out[0..4] = c0, c1, first_of(item), last_of(item), begins_in(j, item).
void share_on_host(int items, int per_item, int j, int G, int item, int* out)
{
    const Share sh = make_share(items, per_item, j, G);
    out[0] = sh.c0;
    out[1] = sh.c1;
    out[2] = out[3] = out[4] = -1;
    // only items of j's XCD can be asked about
    if (sh.U > 0 && item * per_item >= sh.base && item * per_item < sh.base + sh.U) {
        out[2] = sh.first_of(item);
        out[3] = sh.last_of(item);
        out[4] = sh.begins_in(j, item) ? 1 : 0;
    }
}

// The attention's work shares on the host: for workgroup j and head `head`,
// out[0..5] = first part, number of parts, this part's index, t0, t1, and whether `head` is
// one of j's heads at all (otherwise the first five are -1).
void attn_share_on_host(int nh, int ntile, int j, int G, int head, int* out)
{
    const AttnHeads hs = attn_heads(nh, j, G);
    for (int i = 0; i < 6; ++i) out[i] = -1;
    out[5] = 0;
    const int hl = head - hs.hx0;
    if (hl < hs.h_lo || hl >= hs.h_hi) return;
    const AttnTiles ts = attn_tiles(hs, hl, ntile);
    out[0] = ts.first;
    out[1] = ts.np;
    out[2] = ts.me;
    out[3] = ts.t0;
    out[4] = ts.t1;
    out[5] = 1;
}

// ---- setup kernel ------------------------------------------------------------
// Blocks 0..kTreeBlocks-1: tree tables (every block walks the parents itself; block 0
// writes the ancestor masks, each block a slice of the rotary table).  The next kZeroBlocks
// blocks zero the sync block.  Further blocks: one per 16-column tile of the residual stream,
// writing x = widen(x_in), the tile's sums of squares and the gain-scaled fp16 image.
constexpr int kTreeBlocks = 8;
constexpr int kZeroBlocks = 32;

__global__ __launch_bounds__(256) void k_fused_setup(uint32_t* __restrict__ sync,
                                                     const int32_t* __restrict__ parent, int M,
                                                     int Mpad, int kv_len, int d, float rope_base,
                                                     uint64_t* __restrict__ mask,
                                                     float2* __restrict__ rope, float* __restrict__ x,
                                                     const half_t* __restrict__ x_in16, int H,
                                                     float* __restrict__ ss,
                                                     const half_t* __restrict__ gain,
                                                     half_t* __restrict__ xg16)
{
    int tid = threadIdx.x;
    if (blockIdx.x < kTreeBlocks) {
        // Ancestor sets and depths by pointer doubling: after round k a node knows its 2^k
        // nearest ancestors-or-self, how many edges lead to the farthest of them, and the
        // node 2^k edges up (-1 past the root).  ceil(log2 M) rounds whatever the depth; a
        // parent that is not an earlier node is taken as "no parent".
        __shared__ int32_t s_up[GHD_MAX_M];
        __shared__ int32_t s_depth[GHD_MAX_M];
        __shared__ uint64_t s_lo[GHD_MAX_M], s_hi[GHD_MAX_M];
        if (!parent) return;
        int up = -1, dep = 0;
        uint64_t lo = 0, hi = 0;
        if (tid < M) {
            up = parent[tid];
            if (up < 0 || up >= tid) up = -1;
            dep = up >= 0 ? 1 : 0;
            if (tid < 64) lo = 1ull << tid; else hi = 1ull << (tid - 64);
        }
        for (int span = 1; span < M; span <<= 1) {
            if (tid < M) {
                s_up[tid] = up;
                s_depth[tid] = dep;
                s_lo[tid] = lo;
                s_hi[tid] = hi;
            }
            __syncthreads();
            if (tid < M && up >= 0) {
                lo |= s_lo[up];
                hi |= s_hi[up];
                dep += s_depth[up];
                up = s_up[up];
            }
            __syncthreads();
        }
        if (tid < M) {
            s_depth[tid] = dep;
            if (blockIdx.x == 0) {
                mask[2 * tid] = lo;
                mask[2 * tid + 1] = hi;
            }
        }
        __syncthreads();
        if (rope) {
            // angle = position * base^(-2j/d), evaluated in double
            const int half = d / 2;
            const double c = -2.0 / d * log2((double)rope_base);
            for (int e = blockIdx.x * 256 + tid; e < M * half; e += kTreeBlocks * 256) {
                int m = e / half, j = e % half;
                double ang = (double)(kv_len + s_depth[m]) * exp2(c * j);
                rope[e] = make_float2((float)cos(ang), (float)sin(ang));
            }
        }
        return;
    }
    if (blockIdx.x < kTreeBlocks + kZeroBlocks) {
        for (int i = (blockIdx.x - kTreeBlocks) * 256 + tid; i < kSyncWords; i += kZeroBlocks * 256) sync[i] = 0;
        return;
    }
    // residual stream tiles: thread -> (row m, column within the 16-wide tile)
    int tile = blockIdx.x - kTreeBlocks - kZeroBlocks;
    for (int e = tid; e < Mpad * 16; e += 256) {
        int m = e >> 4, col = tile * 16 + (e & 15);
        float v = 0.f;
        if (m < M) {
            v = x_in16 ? (float)x_in16[(size_t)m * H + col] : x[(size_t)m * H + col];
            if (x_in16) x[(size_t)m * H + col] = v;
            if (xg16) xg16[(size_t)m * H + col] = (half_t)(v * (float)gain[col] * kXgScale);
        }
        float s = v * v;
        s += __shfl_xor(s, 1);
        s += __shfl_xor(s, 2);
        s += __shfl_xor(s, 4);
        s += __shfl_xor(s, 8);
        if ((e & 15) == 0) ss[(size_t)tile * Mpad + m] = s;
    }
}

ghd_status launch_fused_setup(uint32_t* sync, const int32_t* parent, int M, int Mpad, int kv_len, int d,
                              float rope_base, uint64_t* mask, float2* rope, float* x,
                              const half_t* x_in16, int H, float* ss, const half_t* gain,
                              half_t* xg16, hipStream_t st)
{
    int blocks = kTreeBlocks + kZeroBlocks + (ss ? H / 16 : 0);
    hipLaunchKernelGGL(k_fused_setup, dim3(blocks), dim3(256), 0, st, sync, parent, M, Mpad, kv_len, d,
                       rope_base, mask, rope, x, x_in16, H, ss, gain, xg16);
    return check_launch();
}

// ---- weight packing ------------------------------------------------------------
// One thread per 16-byte chunk of the packed image.  Packed row p of the matrix maps
// to a source row through the permutation of its kind:
//   PLAIN    p
//   QKV      inside every head the rows are ordered (j, j+1, j+d/2, j+1+d/2), j even,
//            so the two rotary pairs of a quad sit in one lane of the GEMM output
//   GATE_UP  (gate f, gate f+1, up f, up f+1): source holds gate rows [0,F) then up rows
__global__ void k_pack2(half8* __restrict__ dst, const half_t* __restrict__ src, int N, int K,
                        int kind, int d, int ngroups, int ksteps)
{
    size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)ngroups * ksteps * kTG * 64;
    if (id >= total) return;
    int lane = (int)(id & 63);
    size_t blk = id >> 6;
    int tile_in = (int)(blk % kTG);
    size_t gk = blk / kTG;
    int ks = (int)(gk % ksteps);
    int grp = (int)(gk / ksteps);
    int p = (grp * kTG + tile_in) * 16 + (lane & 15);
    int k = ks * 32 + (lane >> 4) * 8;
    int srow = -1;
    if (kind == PACK_PLAIN) {
        if (p < N) srow = p;
    } else if (kind == PACK_QKV) {
        if (p < N) {
            int head = p / d, ph = p % d;
            int r = ph & 3;
            int ch = (ph >> 2) * 2 + (r & 1) + ((r >= 2) ? d / 2 : 0);
            srow = head * d + ch;
        }
    } else {
        int F = N / 2;
        int f = (p >> 4) * 8 + ((p & 15) >> 2) * 2 + (p & 1);
        bool up = (p & 3) >= 2;
        if (f < F) srow = (up ? F : 0) + f;
    }
    half8 v;
    for (int e = 0; e < 8; ++e)
        v[e] = (srow >= 0 && k + e < K) ? src[(size_t)srow * K + k + e] : (half_t)0;
    dst[id] = v;
}

size_t packed_bytes2(int N, int K)
{
    size_t ngroups = (N + kGroupRows - 1) / kGroupRows;
    size_t ksteps = (size_t)((K + kChunkCols - 1) / kChunkCols) * kCH;
    return ngroups * ksteps * kTG * 1024;
}

ghd_status launch_pack2(void* dst, const void* src, int N, int K, int kind, int d, hipStream_t st)
{
    int ngroups = (N + kGroupRows - 1) / kGroupRows;
    int ksteps = ((K + kChunkCols - 1) / kChunkCols) * kCH;
    size_t total = (size_t)ngroups * ksteps * kTG * 64;
    hipLaunchKernelGGL(k_pack2, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (half8*)dst,
                       (const half_t*)src, N, K, kind, d, ngroups, ksteps);
    return check_launch();
}

}  // namespace ghd

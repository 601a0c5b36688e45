// The QKV linear layer and the tree attention of one decoder layer in one launch.
//
// The attention of head h needs q, k and v of head h only (Ghidorah, section 2.2.2: the
// heads are independent), and with the packed QKV rows grouped by XCD (see qkv_row) the
// workgroups that produce them are the ones that run that head's attention: all on one
// XCD.  So instead of ending the launch after the QKV layer, the 32 workgroups of an XCD
// meet at a counter in their L2 once their rotated queries and cache rows are stored, and go
// on with the attention of their XCD's heads.  What is saved is a launch boundary per
// layer: the dispatch gap and the start-up of the attention kernel.
#pragma once
#include "attention_impl.h"
#include "linear_impl.h"

namespace ghd {

template <int MT, int R, int D>
__global__ __launch_bounds__(kFT) void k_qkv_attn(const FusedArgs a)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    touch_kernel_arguments();
    Ctx cx = make_ctx(a, lds);
    const GemmOp op = linear_op_of(a);
    const bool ok = gemm_phase<MT, R, 1>(a, op, cx);
    // ---- the XCD's workgroups meet.  Every one of them counts itself in once its part of
    //      q16 and of the cache rows is acknowledged by the L2 they share (the wait below
    //      covers loads too, so it comes before the attention requests anything) ...
    //      Thirty-two workgroups polling one counter line with read-modify-writes queue up
    //      behind each other (a poll then takes microseconds), so the counter is only
    //      incremented: the workgroup that arrives last tells the others, each on a line of
    //      its own.
    const int Gx = cx.G / 8, xcd = cx.j / Gx;
    uint32_t* const cnt = a.sync + kCntXcd + xcd * kCntStride;
    uint32_t* const go = a.sync + kCntGo;
    const uint32_t round = a.att_epoch + 1;
    wait_own_stores();
    __syncthreads();       // also: the linear phase's use of the LDS is over
    bool last = false;
    if (threadIdx.x == 0) {
        last = atomicAdd(cnt, 1u) + 1u == (uint32_t)Gx * round;
        if (last)
            for (int w = 0; w < Gx; ++w)
                __hip_atomic_store(go + (xcd * Gx + w) * kCntStride, round, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // ... and waits for the others at the attention's gate, after it has set up its indices
    //     and requested the cache rows of earlier steps that it starts with.  (Counting in
    //     only after that set-up was measured slower: it is the stores that make a workgroup
    //     late, and everybody waits for the last.)
    auto gate = [&]() -> bool {
        int* s_ok = &reinterpret_cast<AttnLds<MT, D>*>(cx.lds)->wait_ok;
        if (threadIdx.x == 0)
            *s_ok = ok && (last || bounded_wait(a.sync, go + cx.j * kCntStride, round, 3000u));
        __syncthreads();
        if (!*s_ok) return false;
        // Nothing of q16 or of the tree's cache rows should be in this compute unit's L1 (it
        // has not read them in this launch); dropping the L1's contents makes that independent
        // of what the L1 does with this workgroup's own stores.  The L1 only: an agent-scope
        // acquire would also walk the L2, which every workgroup of the XCD is streaming through.
        invalidate_l1();
        return true;
    };
    attn_phase<MT, D, true>(a, cx, a.att_q, a.att_k, a.att_v, a.att_out, a.att_epoch, gate);
}

template <int MT, int R, int D>
static ghd_status launch_qkv_attn_t(const FusedArgs& a, hipStream_t st)
{
    int G = 0;
    const size_t l1 = linear_lds_bytes<MT, R>(), l2 = sizeof(AttnLds<MT, D>);
    const size_t lds = l1 > l2 ? l1 : l2;
    ghd_status s = launch_resident_checked((const void*)k_qkv_attn<MT, R, D>, 0, lds, &G);
    if (s) return s;
    hipLaunchKernelGGL((k_qkv_attn<MT, R, D>), dim3(G), dim3(kFT), lds, st, with_launch_facts(a, G));
    return check_launch();
}

// the instantiations of one M range: head dim 128, wide QKV matrices of 3 to 6 row tiles per
// workgroup (7B- to 70B-shaped layers)
template <int MT>
ghd_status launch_qkv_attn_mt(const FusedArgs& a, hipStream_t st)
{
    if (a.d != 128) return GHD_ERR_SHAPE;
    switch (a.lin_slots) {
    case 3: return launch_qkv_attn_t<MT, 3, 128>(a, st);
    case 4: return launch_qkv_attn_t<MT, 4, 128>(a, st);
    default: break;
    }
    if constexpr (MT <= 4) {
        switch (a.lin_slots) {
        case 5: return launch_qkv_attn_t<MT, 5, 128>(a, st);
        case 6: return launch_qkv_attn_t<MT, 6, 128>(a, st);
        default: break;
        }
    }
    return GHD_ERR_SHAPE;
}

ghd_status launch_qkv_attn_mt1(const FusedArgs& a, hipStream_t st);
ghd_status launch_qkv_attn_mt2(const FusedArgs& a, hipStream_t st);
ghd_status launch_qkv_attn_mt4(const FusedArgs& a, hipStream_t st);
ghd_status launch_qkv_attn_mt8(const FusedArgs& a, hipStream_t st);

}  // namespace ghd

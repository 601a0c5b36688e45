// Device-side pieces shared by the persistent kernels: work shares, bounded waits,
// the XCD-local hand-off of partial results.
#pragma once
#include "fused.h"

#include <cstddef>

namespace ghd {

constexpr long long kWaitTicks = 2000000;   // bounded waits give up after 20 ms (100 MHz clock)

struct Ctx {
    int j, G;            // logical workgroup index, number of workgroups
    char* lds;           // dynamic LDS
};

__device__ __forceinline__ uint32_t ld_relaxed(const uint32_t* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Work shares.  An operation has `items` (row blocks, or heads) of `per_item` units
// (k-steps, or key tiles) each.  Items are dealt to the 8 XCDs in contiguous blocks, and
// the units of an XCD's items to its shares in equal contiguous ranges.  Workgroup i runs
// on XCD i % 8 (checked at kernel start), so the logical index j = (i % 8) * G/8 + i / 8
// puts the G/8 workgroups of an XCD side by side.  An item that is split over several
// shares is therefore always finished inside one XCD, and its partial results are
// exchanged through that XCD's L2 with plain stores and loads: every wavefront waits for
// the acknowledgement of its own stores before the barrier after which thread 0 bumps the
// item's counter, and a reader's first access to a slot line in a launch cannot hit in
// its L1.  No device-scope fence (a write-back and invalidate of a whole L2, about
// 4 us here) is needed anywhere inside a launch.
struct Share {
    int U;        // units of this XCD (fits 32 bits together with the factor Ge)
    int base;     // global index of its first unit (the unit count of an operation fits 31 bits)
    int Ge;       // shares of this XCD that get units
    int wg0;      // index of its first share
    int c0, c1;   // this share's range of global unit indices (empty if c0 == c1)
    int per_item;
    // local (within-XCD) unit index where share wg's range begins
    __host__ __device__ int lbegin(int wg) const { return (int)((unsigned)U * (unsigned)(wg - wg0) / (unsigned)Ge); }
    __host__ __device__ int owner_local(int lunit) const
    {
        return wg0 + (int)(((unsigned)(lunit + 1) * (unsigned)Ge - 1u) / (unsigned)U);
    }
    __host__ __device__ int litem0(int item) const { return item * per_item - base; }
    __host__ __device__ int first_of(int item) const { return owner_local(litem0(item)); }
    __host__ __device__ int last_of(int item) const { return owner_local(litem0(item) + per_item - 1); }
    // does share wg's range begin inside `item` (and not in an earlier one)?
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

// Invalidates this compute unit's vector L1 (workgroup-scope buffer_inv): loads that follow
// are served by the L2.
__device__ __forceinline__ void invalidate_l1() { asm volatile("buffer_inv sc0" ::: "memory"); }

__device__ __forceinline__ uint32_t poll(uint32_t* p)
{
    // a read-modify-write that changes nothing: it is served where the counting atomics
    // are, so it sees them at once (a device-scope load lags them by several microseconds)
    return atomicOr(p, 0u);
}

// Waits until *p >= target.  Gives up (and raises the status word to `code`) after
// kWaitTicks of wall-clock time, or as soon as another workgroup has given up, so that a
// launch that is not fully resident ends with an error instead of hanging.  One thread calls.
// Returns false if it gave up: what was waited for is then not there.
__device__ __forceinline__ bool bounded_wait(uint32_t* sync, uint32_t* p, uint32_t target,
                                             uint32_t code)
{
    if (poll(p) >= target) return true;
    const long long t0 = wall_clock64();
    while (poll(p) < target) {
        if (wall_clock64() - t0 > kWaitTicks || ld_relaxed(sync + kSyncStatus) != 0) {
            atomicCAS(sync + kSyncStatus, 0u, code);
            return false;
        }
        __builtin_amdgcn_s_sleep(8);
    }
    return true;
}

// The argument block is a few 64-byte lines of kernel-argument memory, which the compiler
// reads field by field as the code needs them, one memory round trip after the other.  One
// word of every line is requested here, back to back at the start of the kernel, so that
// the lines arrive together and the later reads find them in the scalar cache.  (Written as
// one block of scalar loads with its own wait: left to the compiler, the five results are
// parked one by one, with a wait after each load.)
__device__ __forceinline__ void touch_kernel_arguments()
{
    static_assert(offsetof(FusedArgs, lin_range) > 320 && offsetof(FusedArgs, lin_range) <= 384,
                  "six 64-byte lines before the table of work shares");
    typedef const __attribute__((address_space(4))) uint32_t* kernarg_words;
    kernarg_words kp = (kernarg_words)__builtin_amdgcn_kernarg_segment_ptr();
    uint32_t t0, t1, t2, t3, t4, t5;
    asm volatile(
        "s_load_dword %0, %6, 0x0\n\t"
        "s_load_dword %1, %6, 0x40\n\t"
        "s_load_dword %2, %6, 0x80\n\t"
        "s_load_dword %3, %6, 0xc0\n\t"
        "s_load_dword %4, %6, 0x100\n\t"
        "s_load_dword %5, %6, 0x140\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&s"(t0), "=&s"(t1), "=&s"(t2), "=&s"(t3), "=&s"(t4), "=&s"(t5)
        : "s"(kp)
        : "memory");
}

// Workgroups are dealt round-robin to the 8 XCDs; neighbours in the work sequence (which
// share row blocks, or heads, and exchange partial results) get the same XCD.  The
// exchange relies on workgroup i running on XCD i % 8, which is checked here.
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

}  // namespace ghd

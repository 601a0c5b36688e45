// Host side of the skinny linear layers (how an operation is cut into work shares, kernel
// selection) and the two packing kernels (weights, activations).
#include "linear_impl.h"
#include "qkv_attn_impl.h"

#include <cstdlib>
#include <mutex>
#include <vector>

namespace ghd {

// ---- per-device facts ------------------------------------------------------------
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

// All workgroups of a persistent kernel must be resident at once (they wait for each
// other): one per compute unit.  The first launch of a kernel on a device raises its
// dynamic LDS limit and checks that a workgroup fits; *grid = workgroups to launch.
ghd_status launch_resident_checked(const void* kernel, int key, size_t lds, int* grid)
{
    (void)key;
    static std::mutex mu;
    static std::vector<const void*> checked[kMaxDevices];
    const int dev = current_device();
    const int G = fused_grid_size();
    // the hand-off of partial results is laid out for 8 XCDs of G / 8 compute units
    // and for at most kRangeWgs workgroups (their work shares travel in the argument block)
    if (dev < 0 || G <= 0 || G > kRangeWgs || (G % 8) != 0) return hip_fail(hipErrorInvalidDevice);
    *grid = G;
    std::lock_guard<std::mutex> lock(mu);
    for (const void* k : checked[dev])
        if (k == kernel) return GHD_OK;
    hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return hip_fail(e);
    int per_cu = 0;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kFT, lds);
    if (e != hipSuccess) return hip_fail(e);
    if (per_cu < 1) return hip_fail(hipErrorLaunchOutOfResources);
    checked[dev].push_back(kernel);
    return GHD_OK;
}

// ---- how a linear layer is cut -------------------------------------------------------
// Whole tiles: the 16-row tiles are dealt out, every share streams its tiles over the whole
// k range and finishes them alone - nothing is exchanged between workgroups, at the price of
// shares that differ by one tile and of x being read once per share.  That is how wide
// matrices are cut at every M (measured against equal shares of k-steps with the boundary
// tiles finished jointly: 5.7% of a 64-row step, 4.8% of a 1-row step), and narrow ones up to
// 16 rows of x (where x is small) unless the one-tile difference between shares costs more
// stream time than the exchange it saves (about 3 us a launch).  Otherwise narrow matrices
// are cut into k ranges of four-tile row blocks: a share then reads a fraction of x, and the
// blocks' partial sums are exchanged.  Every share streams all the row tiles it touches at
// once, so their number is bounded by the accumulator registers (8 tiles up to 64 rows of x,
// 4 above); more shares per workgroup (passes) make the shares smaller until that holds.
constexpr double kStreamBytesPerUs = 6.4e6;    // what a launch streams at best (measured)
constexpr double kExchangeUs = 3.0;            // what finishing shared row blocks jointly costs a launch

static bool plan_whole(const WLayout& lay, int mt, int G, LinPlan* out)
{
    const int cap = mt <= 4 ? 8 : 4;
    for (int P = 1; P <= kMaxShares / (G > 0 ? G : 1) && P <= 8; ++P) {
        int most = 1;
        for (int ls = 0; ls < G * P; ++ls) {
            const Share sh = make_share(lay.ntiles, 1, ls, G * P);
            most = sh.c1 - sh.c0 > most ? sh.c1 - sh.c0 : most;
        }
        if (most <= cap) {
            out->slots = most;
            out->passes = P;
            out->whole = 1;
            return true;
        }
    }
    return false;
}

bool plan_linear(int M, int N, int K, int G, LinPlan* out)
{
    const WLayout lay = w_layout(N, K);
    const int mt = (M + 15) / 16;
    if (lay.rb == 1) return plan_whole(lay, mt, G, out);
    if (mt <= 1 && plan_whole(lay, mt, G, out)) {
        // stream time lost to the shares with one tile more than the average
        const double excess = (double)out->slots * out->passes * G / lay.ntiles - 1.0;
        if (excess * (2.0 * N * K / kStreamBytesPerUs) < kExchangeUs) return true;
    }
    out->slots = kRbNarrow;
    out->passes = 1;
    out->whole = 0;
    return true;
}

// partial-sum slots of the row-block cut (one share per workgroup): two per share, each one
// row block of fragments
size_t linear_part_floats(int M, int G)
{
    const size_t mt = (size_t)((M + 15) / 16 <= 1 ? 1 : (M + 15) / 16 <= 2 ? 2 : (M + 15) / 16 <= 4 ? 4 : 8);
    return (size_t)G * 2 * kRbNarrow * mt * 256;
}

ghd_status launch_linear(const FusedArgs& a, hipStream_t st)
{
    const int mt = (a.M + 15) / 16;
    if (mt <= 1) return launch_linear_mt1(a, st);
    if (mt <= 2) return launch_linear_mt2(a, st);
    if (mt <= 4) return launch_linear_mt4(a, st);
    return launch_linear_mt8(a, st);
}

// The QKV layer and the attention share a launch when the packed QKV rows are grouped by
// XCD, the matrix is a wide one that needs one share per workgroup, and a kernel was built
// for the shape.
bool qkv_attn_available(int M, int slots, int passes, int d, int nh)
{
    const int mt = (M + 15) / 16;
    if (!qkv_grouped(nh) || d != 128 || passes != 1) return false;
    if (w_layout(3 * nh * d, nh * d).rb != 1) return false;
    return slots >= 3 && slots <= (mt <= 4 ? 6 : 4);
}

ghd_status launch_qkv_attn(const FusedArgs& a, hipStream_t st)
{
    const int mt = (a.M + 15) / 16;
    if (mt <= 1) return launch_qkv_attn_mt1(a, st);
    if (mt <= 2) return launch_qkv_attn_mt2(a, st);
    if (mt <= 4) return launch_qkv_attn_mt4(a, st);
    return launch_qkv_attn_mt8(a, st);
}

// The work-share arithmetic evaluated on the host (for tests of its invariants): the unit
// range of share j, and for `item` its first and last part and whether j's range begins
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

// ---- weight packing ------------------------------------------------------------
// One thread per 16-byte piece of the packed image.  Packed row p of the matrix maps
// to a source row through the permutation of its kind:
//   PLAIN    p
//   QKV      inside every head the rows are ordered (j, j+1, j+d/2, j+1+d/2), j even,
//            so the two rotary pairs of a quad sit in one lane of the GEMM output; heads
//            grouped by XCD when their number is a multiple of 8 (see qkv_row)
//   GATE_UP  (gate f, gate f+1, up f, up f+1): source holds gate rows [0,F) then up rows
__global__ void k_pack2(half8* __restrict__ dst, const half_t* __restrict__ src, int N, int K,
                        int kind, int d, WLayout lay)
{
    size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = w_pieces(lay);
    if (id >= total) return;
    int lane = (int)(id & 63);
    size_t blk = id >> 6;
    int tin = (int)(blk % lay.blk);
    size_t bk = blk / lay.blk;
    int ks = (int)(bk % lay.nks);
    int block = (int)(bk / lay.nks);
    int p = (block * lay.blk + tin) * 16 + (lane & 15);
    int k = ks * 32 + (lane >> 4) * 8;
    int srow = -1;
    if (kind == PACK_PLAIN) {
        if (p < N) srow = p;
    } else if (kind == PACK_QKV) {
        if (p < N) {
            const int H = N / 3;
            const QkvRow qr = qkv_row(p, H / d, d);
            srow = qr.part * H + qr.head * d + qkv_channel(qr.ph, d);
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
    return w_pieces(w_layout(N, K)) * 16;
}

ghd_status launch_pack2(void* dst, const void* src, int N, int K, int kind, int d, hipStream_t st)
{
    const WLayout lay = w_layout(N, K);
    size_t total = w_pieces(lay);
    hipLaunchKernelGGL(k_pack2, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (half8*)dst,
                       (const half_t*)src, N, K, kind, d, lay);
    return check_launch();
}

// ---- activation packing -----------------------------------------------------------
// One thread per 16-byte piece of the packed image: row-major [M, ldx] -> B-operand blocks.
// Rows from M on and columns from K on are written as zeros.
__global__ void k_pack_x(half8* __restrict__ dst, const half_t* __restrict__ src, int M, int mtp, int K,
                         int64_t ldx)
{
    size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)((K + 31) / 32) * mtp * 64;
    if (id >= total) return;
    int lane = (int)(id & 63);
    size_t blk = id >> 6;
    int b = (int)(blk % mtp);
    int ks = (int)(blk / mtp);
    int m = b * 16 + (lane & 15), k = ks * 32 + (lane >> 4) * 8;
    half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
    if (m < M && k < K) v = *(const half8*)(src + (size_t)m * ldx + k);
    dst[id] = v;
}

ghd_status launch_pack_x(half_t* dst, const half_t* src, int M, int Mpad, int K, int64_t ldx, hipStream_t st)
{
    const int mtp = Mpad / 16;
    size_t total = (size_t)((K + 31) / 32) * mtp * 64;
    hipLaunchKernelGGL(k_pack_x, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (half8*)dst, src, M,
                       mtp, K, ldx);
    return check_launch();
}

}  // namespace ghd

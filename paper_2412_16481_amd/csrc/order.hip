// Canonical serving order for the rebalancing of Algorithm 2 (Section 4.1 "Bucket rebalancing" leaves the arrival
// order of the contenders of a bucket to the hardware race). Serving them in increasing
// (Z-order code of the voxel, x, y, z, input index) makes the partition of the points independent of the order in
// which they are stored. It is done by sorting the points once by that key and running the index-ordered bucketing on
// the sorted copy; the result is mapped back through the sort order.
//
// The sort is a stable least-significant-digit radix sort on 8-bit digits of six 32-bit key words per point, carrying
// only the point index: per pass one kernel counts the digits of every tile of 2048 positions, and one kernel sums the
// count rows of the earlier tiles itself (small inputs; from 160 tiles on a third kernel scans the count columns
// first), ranks its tile by digit in position order (wave ballots over the digit's bits plus per-(round, wave) counters
// in LDS) and scatters the indices.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "order.h"
#include "psh.h"
#include "psh_common.h"

namespace f3d {
namespace {

constexpr int OT = 256;          // threads per workgroup
constexpr int OE = 2048;         // positions per tile
constexpr int OR = OE / OT;      // rounds: position = tile*OE + round*OT + thread
constexpr int OW = OT / 64;      // waves
constexpr int ORDER_SCAN_TILES = 160;

__device__ __forceinline__ int scan_of(const OrderArgs& a, int p)
{
    return a.batch_offsets ? find_scan(a.batch_offsets, a.n_scans, p) : 0;
}

__global__ __launch_bounds__(OT) void k_order_init(OrderArgs a)
{
    const int i = blockIdx.x * OT + threadIdx.x;
    if (i < a.n_scans * 4) a.box[i] = 0xFFFFFFFFu;
}

// per-scan coordinate minimum (Algorithm 1, "compute voxel coordinate"). A workgroup takes OB consecutive positions.
// Almost always they belong to one scan: then the minimum is reduced inside the workgroup and costs three global
// atomics; a workgroup that straddles a scan boundary publishes wave by wave whenever a wave moves on to another scan.
constexpr int OB = 4 * OE;
__global__ __launch_bounds__(OT) void k_order_box(OrderArgs a)
{
    __shared__ uint32_t red[3];
    const int tid = threadIdx.x, lane = tid & 63;
    const long long first = (long long)blockIdx.x * OB;
    const long long last = min(first + OB, (long long)a.n) - 1;
    if (first > last) return;
    const int b_first = scan_of(a, (int)first), b_last = scan_of(a, (int)last);
    const bool uniform = b_first == b_last;      // offsets are non-decreasing when they are valid at all
    if (tid < 3) red[tid] = 0xFFFFFFFFu;
    __syncthreads();
    uint32_t mn[3] = {0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu};
    if (uniform) {
        for (long long e = first + tid; e <= last; e += OT) {
#pragma unroll
            for (int t = 0; t < 3; ++t) mn[t] = min(mn[t], f2ord(a.coords[(size_t)e * 3 + t]));
        }
    } else {
        // a lane walks its positions in increasing order, so its scan index only grows: it keeps the minimum of the
        // scan it is in; when any lane of the wave moves on to another scan the whole wave publishes (one atomic per
        // axis if all its lanes were in the same scan, else one per lane and axis)
        int cur = -1;
        const auto flush = [&]() {
            const unsigned long long have = __ballot(cur >= 0);
            if (!have) return;
            const int lead = __shfl(cur, __ffsll((long long)have) - 1, 64);
            if (__ballot(cur >= 0 && cur != lead) == 0) {
#pragma unroll
                for (int t = 0; t < 3; ++t) {
                    uint32_t lo = mn[t];
                    for (int d = 32; d >= 1; d >>= 1) lo = min(lo, (uint32_t)__shfl_xor((int)lo, d, 64));
                    if (lane == 0) atomicMin(&a.box[lead * 4 + t], lo);
                }
            } else if (cur >= 0) {
#pragma unroll
                for (int t = 0; t < 3; ++t) atomicMin(&a.box[cur * 4 + t], mn[t]);
            }
        };
        for (long long e0 = first; e0 <= last; e0 += OT) {   // the trip count is the same for every lane
            const long long e = e0 + tid;
            const bool ok = e <= last;
            const int b = ok ? scan_of(a, (int)e) : -1;
            if (__ballot(ok && cur >= 0 && b != cur)) {
                flush();
                cur = -1;
                mn[0] = mn[1] = mn[2] = 0xFFFFFFFFu;
            }
            if (ok) {
                cur = b;
#pragma unroll
                for (int t = 0; t < 3; ++t) mn[t] = min(mn[t], f2ord(a.coords[(size_t)e * 3 + t]));
            }
        }
        flush();
    }
    if (!uniform) return;
#pragma unroll
    for (int t = 0; t < 3; ++t) {
        uint32_t lo = mn[t];
        for (int d = 32; d >= 1; d >>= 1) lo = min(lo, (uint32_t)__shfl_xor((int)lo, d, 64));
        if (lane == 0) atomicMin(&red[t], lo);
    }
    __syncthreads();
    if (tid < 3) atomicMin(&a.box[b_first * 4 + tid], red[tid]);
}

// key words of every point
__global__ __launch_bounds__(OT) void k_order_keys(OrderArgs a)
{
    const long long p = (long long)blockIdx.x * OT + threadIdx.x;
    if (p >= a.n) return;
    const int b = scan_of(a, (int)p);
    int v[3];
    uint32_t o[3];
#pragma unroll
    for (int t = 0; t < 3; ++t) {
        const float c = a.coords[(size_t)p * 3 + t];
        o[t] = f2ord(c);
        v[t] = voxel_of(c, ord2f(a.box[b * 4 + t]), a.inv_voxel);
    }
    const uint64_t code = morton3(v[0], v[1], v[2]);
    const size_t n = (size_t)a.n;
    a.words[0 * n + p] = o[2];
    a.words[1 * n + p] = o[1];
    a.words[2 * n + p] = o[0];
    a.words[3 * n + p] = (uint32_t)code;
    a.words[4 * n + p] = (uint32_t)(code >> 32);
    a.words[5 * n + p] = (uint32_t)b;
}

__global__ __launch_bounds__(OT) void k_order_count(const int32_t* __restrict__ src, const uint32_t* __restrict__ word, int shift,
                                                    int n, uint32_t* __restrict__ hist)
{
    __shared__ uint32_t h[256];
    h[threadIdx.x] = 0;
    __syncthreads();
#pragma unroll
    for (int r = 0; r < OR; ++r) {
        const long long e = (long long)blockIdx.x * OE + r * OT + threadIdx.x;
        if (e < n) {
            const int i = src ? src[e] : (int)e;
            atomicAdd(&h[(word[i] >> shift) & 255u], 1u);
        }
    }
    __syncthreads();
    hist[(size_t)blockIdx.x * 256 + threadIdx.x] = h[threadIdx.x];
}

// Large inputs only: exclusive prefix over the tiles of every digit's count column, so that the scatter kernel reads one
// row instead of summing all earlier rows itself. One workgroup per digit; hist[t][d] becomes the number of positions
// with digit d in the tiles before t, total[d] the count over all tiles.
__global__ __launch_bounds__(OT) void k_order_scan(uint32_t* __restrict__ hist, uint32_t* __restrict__ total, int tiles)
{
    __shared__ uint32_t wsum[OW];
    const int d = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t carry = 0;
    for (int t0 = 0; t0 < tiles; t0 += OT) {
        const int t = t0 + tid;
        const uint32_t c = t < tiles ? hist[(size_t)t * 256 + d] : 0u;
        uint32_t inc = c;
        for (int s = 1; s < 64; s <<= 1) {
            const uint32_t o = (uint32_t)__shfl_up((int)inc, s, 64);
            if (lane >= s) inc += o;
        }
        if (lane == 63) wsum[wave] = inc;
        __syncthreads();
        uint32_t before = 0, all = 0;
        for (int w = 0; w < OW; ++w) {
            if (w < wave) before += wsum[w];
            all += wsum[w];
        }
        if (t < tiles) hist[(size_t)t * 256 + d] = carry + before + inc - c;
        carry += all;
        __syncthreads();
    }
    if (tid == 0) total[d] = carry;
}

__global__ __launch_bounds__(OT) void k_order_scatter(const int32_t* __restrict__ src, int32_t* __restrict__ dst,
                                                      const uint32_t* __restrict__ word, int shift, int n,
                                                      const uint32_t* __restrict__ hist, int tiles,
                                                      const uint32_t* __restrict__ total)
{
    __shared__ uint32_t base[256];
    __shared__ uint32_t wsum[OW];
    __shared__ uint16_t cnt[OR * OW][256];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tile = blockIdx.x;

    // first position of digit `tid` for this tile: all smaller digits of all tiles, plus this digit in earlier tiles
    uint32_t pre = 0, tot = 0;
    if (total) {   // the count columns have been scanned by k_order_scan
        pre = hist[(size_t)tile * 256 + tid];
        tot = total[tid];
    } else {
#pragma unroll 8
        for (int t = 0; t < tiles; ++t) {
            const uint32_t c = hist[(size_t)t * 256 + tid];
            pre += t < tile ? c : 0u;
            tot += c;
        }
    }
    uint32_t inc = tot;
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = (uint32_t)__shfl_up((int)inc, d, 64);
        if (lane >= d) inc += o;
    }
    if (lane == 63) wsum[wave] = inc;
    uint32_t* cz = reinterpret_cast<uint32_t*>(&cnt[0][0]);
#pragma unroll
    for (int j = 0; j < OR * OW * 256 / 2 / OT; ++j) cz[j * OT + tid] = 0u;
    __syncthreads();
    uint32_t before = 0;
    for (int w = 0; w < wave; ++w) before += wsum[w];
    base[tid] = before + inc - tot + pre;

    // digit of every position of the tile and its rank among equal digits of the same wave and round
    int idx[OR], dig[OR], rk[OR];
#pragma unroll
    for (int r = 0; r < OR; ++r) {
        const long long e = (long long)tile * OE + r * OT + tid;
        const bool ok = e < n;
        idx[r] = ok ? (src ? src[e] : (int)e) : 0;
        dig[r] = ok ? (int)((word[idx[r]] >> shift) & 255u) : -1;
    }
#pragma unroll
    for (int r = 0; r < OR; ++r) {
        const bool ok = dig[r] >= 0;
        unsigned long long peers = __ballot(ok);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const unsigned long long bal = __ballot(ok && ((dig[r] >> b) & 1));
            peers &= ((dig[r] >> b) & 1) ? bal : ~bal;
        }
        rk[r] = __popcll(peers & ((1ull << lane) - 1ull));
        if (ok && rk[r] == 0) cnt[r * OW + wave][dig[r]] = (uint16_t)__popcll(peers);
    }
    __syncthreads();
    {   // exclusive prefix over the (round, wave) rows, one digit per thread
        uint32_t run = 0;
#pragma unroll
        for (int row = 0; row < OR * OW; ++row) {
            const uint32_t c = cnt[row][tid];
            cnt[row][tid] = (uint16_t)run;
            run += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < OR; ++r) {
        if (dig[r] < 0) continue;
        const uint32_t pos = base[dig[r]] + cnt[r * OW + wave][dig[r]] + (uint32_t)rk[r];
        if (pos < (uint32_t)n) dst[pos] = idx[r];
    }
}

__global__ __launch_bounds__(OT) void k_order_gather(const int32_t* __restrict__ order, const float* __restrict__ coords, int n,
                                                     float* __restrict__ out)
{
    const long long p = (long long)blockIdx.x * OT + threadIdx.x;
    if (p >= n) return;
    const unsigned i = (unsigned)order[p];
    if (i >= (unsigned)n) return;
    out[(size_t)p * 3 + 0] = coords[(size_t)i * 3 + 0];
    out[(size_t)p * 3 + 1] = coords[(size_t)i * 3 + 1];
    out[(size_t)p * 3 + 2] = coords[(size_t)i * 3 + 2];
}

__global__ __launch_bounds__(OT) void k_order_compose(const int32_t* __restrict__ order, const int32_t* __restrict__ perm_sorted,
                                                      const int32_t* __restrict__ inv_sorted, int n, const int32_t* __restrict__ status,
                                                      int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm)
{
    if (status[0]) return;
    const long long p = (long long)blockIdx.x * OT + threadIdx.x;
    if (p >= n) return;
    const unsigned s = (unsigned)perm_sorted[p];
    if (s < (unsigned)n) perm[p] = order[s];
    const unsigned i = (unsigned)order[p];
    if (inv_perm && i < (unsigned)n) inv_perm[i] = inv_sorted[p];
}

}  // namespace

size_t order_hist_bytes(long long n) { return (size_t)((n + OE - 1) / OE + 1) * 256 * 4; }

hipError_t order_launch(const OrderArgs& a, const int32_t** order_out, hipStream_t stream)
{
    *order_out = a.idx[0];
    if (a.n <= 0) return hipSuccess;
    const int tiles = (a.n + OE - 1) / OE;
    const int blocks = (a.n + OT - 1) / OT;
    k_order_init<<<(a.n_scans * 4 + OT - 1) / OT, OT, 0, stream>>>(a);
    k_order_box<<<(a.n + OB - 1) / OB, OT, 0, stream>>>(a);
    k_order_keys<<<blocks, OT, 0, stream>>>(a);
    // least significant first: z, y, x, the code's low and high word (31 bits), the scan (as many digits as it needs)
    const int32_t* src = nullptr;
    int cur = 0;
    // from this many tiles on a third launch per pass (a scan of the count columns) is cheaper than every workgroup
    // summing all earlier count rows
    uint32_t* total = tiles > ORDER_SCAN_TILES ? a.hist + (size_t)tiles * 256 : nullptr;
    const int scan_digits = a.n_scans > 256 ? 2 : (a.n_scans > 1 ? 1 : 0);
    for (int w = 0; w < 6; ++w) {
        const int digits = w < 5 ? 4 : scan_digits;
        const uint32_t* word = a.words + (size_t)w * a.n;
        for (int d = 0; d < digits; ++d) {
            k_order_count<<<tiles, OT, 0, stream>>>(src, word, 8 * d, a.n, a.hist);
            if (total) k_order_scan<<<256, OT, 0, stream>>>(a.hist, total, tiles);
            k_order_scatter<<<tiles, OT, 0, stream>>>(src, a.idx[cur], word, 8 * d, a.n, a.hist, tiles, total);
            src = a.idx[cur];
            cur ^= 1;
        }
    }
    *order_out = src;
    k_order_gather<<<blocks, OT, 0, stream>>>(src, a.coords, a.n, a.coords_sorted);
    return hipGetLastError();
}

hipError_t order_compose_launch(const int32_t* order, const int32_t* perm_sorted, const int32_t* inv_sorted, int n,
                                const int32_t* status, int32_t* perm, int32_t* inv_perm, hipStream_t stream)
{
    if (n <= 0) return hipSuccess;
    k_order_compose<<<(n + OT - 1) / OT, OT, 0, stream>>>(order, perm_sorted, inv_sorted, n, status, perm, inv_perm);
    return hipGetLastError();
}

}  // namespace f3d

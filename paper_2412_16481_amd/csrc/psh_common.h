// Device helpers shared by the two bucketing paths (psh.hip: any size; psh_fast.hip: scans whose count
// matrix is small enough that every workgroup can sum it by itself).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "psh.h"

namespace f3d {

constexpr uint32_t KEY_PLACED = 0xFFFFFFFFu;
constexpr int LR_BITS = 12;  // rank inside a chunk: chunks hold at most 4096 points

__device__ __forceinline__ int batch_off(const PshArgs& a, int b)
{
    if (a.batch_offsets) return a.batch_offsets[b];
    return b == 0 ? 0 : a.n;
}

// order-preserving map binary32 -> uint32 (so that integer atomicMin/Max give the float min/max)
__device__ __forceinline__ uint32_t f2ord(float f)
{
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float ord2f(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k ^ 0x80000000u) : ~k);
}

// spread the low 11 bits of v so that bit k lands at bit 3k (32-bit arithmetic: 11 bits -> 31 bits)
__device__ __forceinline__ uint32_t spread11(uint32_t v)
{
    uint32_t x = v & 0x7FFu;
    x = (x | (x << 16)) & 0x070000FFu;
    x = (x | (x << 8)) & 0x0700F00Fu;
    x = (x | (x << 4)) & 0x430C30C3u;
    x = (x | (x << 2)) & 0x49249249u;
    return x;
}
// Z-order code of three 21-bit coordinates: bit k of x at 3k, of y at 3k+1, of z at 3k+2.
// The low 11 bits of every axis fill code bits 0..32, the high 10 bits fill code bits 33..62.
__device__ __forceinline__ uint64_t morton3(int x, int y, int z)
{
    const uint32_t lx = spread11((uint32_t)x), ly = spread11((uint32_t)y), lz = spread11((uint32_t)z);
    const uint32_t hx = spread11((uint32_t)x >> 11), hy = spread11((uint32_t)y >> 11), hz = spread11((uint32_t)z >> 11);
    const uint64_t lo = (uint64_t)lx | ((uint64_t)ly << 1) | ((uint64_t)lz << 2);   // 33 bits
    const uint64_t hi = (uint64_t)(hx | (hy << 1) | (hz << 2));                     // 30 bits
    return lo | (hi << 33);
}

__device__ __forceinline__ int bit_width64(uint64_t v) { return v ? 64 - __clzll((long long)v) : 0; }

// Per-scan hash setting (Section 4.1): derived once per scan from its bounding box.
struct ScanCfg {
    float mn[3];
    int vmax[3];
    unsigned long long D;   // divisor of the *_DIV hashes
    double invD;            // 1/D and 1/K: exact integer division by multiply + one correction step
    double invK;
    unsigned int m32;       // 2^32 mod K
    int step;               // probe distance in voxels
    int K;                  // buckets of the scan
    int p0;                 // first point
    int nb;                 // points
    int kb0;                // first bucket (global index)
    int lastcap;            // capacity of the scan's last bucket
    float invDf;            // 1/D in binary32: quotient estimate of the *_DIV hashes (the result is clamped below 2^13)
    int wide;               // some voxel coordinate of the scan needs more than 11 bits
};

__device__ __forceinline__ int voxel_of(float c, float mn, float inv)
{
    // three separate binary32 operations: subtract, multiply, floor. No product feeds a sum here, so there is nothing
    // the compiler could contract into a fused multiply-add (the _rn helpers are plain operators and would not stop it).
    float f = floorf(__fmul_rn(__fsub_rn(c, mn), inv));
    int q = f >= (float)F3D_VOXEL_MAX ? F3D_VOXEL_MAX : (int)f;
    return q < 0 ? 0 : q;
}

// x mod K for x < 2^52 and K < 2^31, exact: quotient estimate in binary64, remainder fixed up by one step
__device__ __forceinline__ unsigned int umod52(unsigned long long x, int K, double invK)
{
    const long long q = (long long)((double)x * invK);
    long long r = (long long)x - q * K;
    if (r < 0) r += K;
    if (r >= K) r -= K;
    return (unsigned int)r;
}

// binary64 value of an unsigned 64-bit integer (one rounding): two 32-bit conversions and a fused multiply-add
__device__ __forceinline__ double u64_to_double(unsigned long long x)
{
    return __fma_rn(__uint2double_rn((unsigned int)(x >> 32)), 4294967296.0, __uint2double_rn((unsigned int)x));
}

// x mod K for x < 2^45 and K >= 2 with x / K < 2^32, exact: 32-bit quotient estimate, remainder fixed up by one step
__device__ __forceinline__ unsigned int umod_q32(unsigned long long x, int K, double invK)
{
    const unsigned int q = __double2uint_rz(u64_to_double(x) * invK);
    long long r = (long long)(x - (unsigned long long)q * (unsigned int)K);
    if (r < 0) r += K;
    if (r >= K) r -= K;
    return (unsigned int)r;
}

// the same code when every coordinate is below 2^11: its upper 30 bits are zero
__device__ __forceinline__ uint64_t morton3_low(int x, int y, int z)
{
    const uint32_t lx = spread11((uint32_t)x), ly = spread11((uint32_t)y), lz = spread11((uint32_t)z);
    return (uint64_t)lx | ((uint64_t)ly << 1) | ((uint64_t)lz << 2);
}

__device__ __forceinline__ int hash_bucket(int hash, int x, int y, int z, const ScanCfg& c)
{
    unsigned long long code;
    if (hash == 0 || hash == 1)
        code = (unsigned long long)((uint32_t)x ^ (uint32_t)y ^ (uint32_t)z);
    else
        code = c.wide ? morton3(x, y, z) : morton3_low(x, y, z);
    if (hash == 0 || hash == 2) {
        if (c.K < 2) return 0;
        // code = hi*2^32 + lo  =>  code mod K = ((hi mod K) * (2^32 mod K) + lo) mod K; K < 2^13 keeps the
        // intermediate below 2^33 and every quotient below 2^32
        const unsigned int hi = (unsigned int)(code >> 32), lo = (unsigned int)code;
        const unsigned long long t = (unsigned long long)umod_q32(hi, c.K, c.invK) * c.m32 + lo;
        return (int)umod_q32(t, c.K, c.invK);
    }
    // code / D clamped to K-1, K < 2^13 + 1. A binary32 estimate (code, 1/D and their product each rounded once more
    // than exactly: relative error below 2^-22) is within 0.002 of the true quotient wherever it is below K + 1, so its
    // integer part is within one of the true one and one correction step with the exact remainder settles it; at K + 1
    // and above the true quotient is certainly >= K. With K >= 2 the divisor is at most 2^62 + 1 and the product below
    // stays inside 64 bits.
    if (c.K < 2) return 0;
    const float cf = __fmaf_rn(__uint2float_rn((unsigned int)(code >> 32)), 4294967296.0f, __uint2float_rn((unsigned int)code));
    const float qf = cf * c.invDf;
    if (qf >= (float)(c.K + 1)) return c.K - 1;
    long long q = (long long)__float2uint_rz(qf);
    const long long r = (long long)(code - (unsigned long long)(unsigned int)q * c.D);
    if (r < 0) --q;
    else if ((unsigned long long)r >= c.D) ++q;
    return (int)(q < (long long)c.K ? q : (long long)(c.K - 1));
}

// 32-bit mixer (xor-shift, odd multiply, xor-shift, odd multiply, xor-shift): a stateless generator for the seeded
// probe directions; any machine computes the same value from the same arguments
__device__ __forceinline__ uint32_t mix32(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x7feb352du;
    x ^= x >> 15;
    x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

// voxel of a point moved by probe r (1..6), clamped to the scan's voxel box (Algorithm 2, "perturb voxel coordinate").
// mode 0: +-step along x, y, z in that order; mode 1: the caller's table of voxel offsets; mode 2: +-step along an
// axis drawn from (seed, r, voxel), so that the points of a voxel move together whatever their indices are.
__device__ __forceinline__ void probe_voxel(const PshArgs& a, int r, const ScanCfg& c, int& x, int& y, int& z)
{
    // Voxel coordinates are below 2^21, so an offset beyond +-2^22 lands outside the box exactly as +-2^22 does: with
    // the offsets limited to that, the sums fit 32 bits.
    constexpr int LIM = 1 << 22;
    int dx = 0, dy = 0, dz = 0;
    if (a.probe_mode == 1) {
        dx = min(max(a.probe_table[3 * (r - 1)], -LIM), LIM);
        dy = min(max(a.probe_table[3 * (r - 1) + 1], -LIM), LIM);
        dz = min(max(a.probe_table[3 * (r - 1) + 2], -LIM), LIM);
    } else {
        int dir = r - 1;
        if (a.probe_mode == 2) {
            uint32_t h = mix32(a.probe_seed + (uint32_t)r);
            h = mix32(h ^ (uint32_t)x);
            h = mix32(h ^ (uint32_t)y);
            h = mix32(h ^ (uint32_t)z);
            dir = (int)(((unsigned long long)h * 6ull) >> 32);
        }
        const int st = min(c.step, LIM);              // a caller's step may be any positive int
        const int d = (dir & 1) ? -st : st;
        const int ax = dir >> 1;
        dx = ax == 0 ? d : 0;
        dy = ax == 1 ? d : 0;
        dz = ax == 2 ? d : 0;
    }
    x = min(max(x + dx, 0), c.vmax[0]);
    y = min(max(y + dy, 0), c.vmax[1]);
    z = min(max(z + dz, 0), c.vmax[2]);
}

// largest b in [0, n_scans) with start[b] <= x, given start[0] <= x < start[n_scans]
__device__ __forceinline__ int find_scan(const int* start, int n_scans, int x)
{
    int lo = 0, hi = n_scans;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (start[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

// z / K for z < 2^63 and K < 2^21, exact: long division over three 21-bit limbs, every step below 2^52
__device__ __forceinline__ unsigned long long udiv63_small(unsigned long long z, int K, double invK)
{
    const unsigned long long l2 = z >> 42, l1 = (z >> 21) & 0x1FFFFFull, l0 = z & 0x1FFFFFull;
    const unsigned int r2 = umod52(l2, K, invK);
    const unsigned long long q2 = (unsigned long long)(((double)(l2 - r2)) * invK + 0.5);   // exact multiples of K
    const unsigned long long t1 = ((unsigned long long)r2 << 21) | l1;
    const unsigned int r1 = umod52(t1, K, invK);
    const unsigned long long q1 = (unsigned long long)(((double)(t1 - r1)) * invK + 0.5);
    const unsigned long long t0 = ((unsigned long long)r1 << 21) | l0;
    const unsigned int r0 = umod52(t0, K, invK);
    const unsigned long long q0 = (unsigned long long)(((double)(t0 - r0)) * invK + 0.5);
    return (q2 << 42) + (q1 << 21) + q0;
}

// hash setting of scan b from its bounding box (ordered-int encoding: min xyz at [0..2], max xyz at [4..6])
// and the scan tables
__device__ inline void compute_cfg(const PshArgs& a, int b, const uint32_t* box, ScanCfg& c)
{
    c.p0 = a.scan_p0[b];
    c.nb = a.scan_p0[b + 1] - c.p0;
    c.kb0 = a.sbs[b];
    c.K = a.sbs[b + 1] - c.kb0;
    c.lastcap = c.nb - (c.K - 1) * a.S;
    int vm = 0;
    for (int ax = 0; ax < 3; ++ax) {
        c.mn[ax] = ord2f(box[ax]);
        float mx = ord2f(box[4 + ax]);
        c.vmax[ax] = voxel_of(mx, c.mn[ax], a.inv_voxel);  // the voxel map is monotone, so this is max v
        vm = max(vm, c.vmax[ax]);
    }
    const int K = max(c.K, 1);
    int nbits = max(1, bit_width64((unsigned long long)vm));
    unsigned long long D = 1;
    c.invK = 1.0 / (double)K;
    if (a.hash == 1) D = udiv63_small((1ull << nbits) - 1, K, c.invK) + 1;
    if (a.hash == 3) D = udiv63_small(morton3(c.vmax[0], c.vmax[1], c.vmax[2]), K, c.invK) + 1;
    if (a.div > 0) D = (unsigned long long)a.div;
    c.D = D;
    c.invD = 1.0 / (double)D;
    c.invDf = (float)c.invD;
    c.wide = vm >= 2048;
    c.m32 = umod52(4294967296ull, K, c.invK);
    long long step = 1;
    if (a.hash == 1) step = (long long)(D > (unsigned long long)F3D_VOXEL_MAX ? (unsigned long long)F3D_VOXEL_MAX : D);
    if (a.hash == 3) step = 1ll << ((bit_width64(D) + 2) / 3);
    if (a.step > 0) step = a.step;
    c.step = (int)step;
}

__device__ __forceinline__ int wave_incl_scan(int v, int lane)
{
    for (int d = 1; d < 64; d <<= 1) {
        int t = __shfl_up(v, d, 64);
        if (lane >= d) v += t;
    }
    return v;
}

// exclusive scan of one value per thread over a block of up to 1024 threads; *total = block sum
__device__ inline int block_excl_scan(int v, int* total, int* lds /*[17]*/)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = wave_incl_scan(v, lane);
    if (lane == 63) lds[wave] = inc;
    __syncthreads();
    if (wave == 0) {
        const int nw = (int)(blockDim.x >> 6);
        const int t = lane < nw ? lds[lane] : 0;
        const int ti = wave_incl_scan(t, lane);
        if (lane < nw) lds[lane] = ti - t;
        if (lane == nw - 1) lds[16] = ti;
    }
    __syncthreads();
    int res = inc - v + lds[wave];
    *total = lds[16];
    __syncthreads();
    return res;
}

// lanes of the wave whose key equals this lane's key (ballots over the key bits); 0 for inactive lanes
__device__ __forceinline__ unsigned long long match_key(int key, bool active, int keybits)
{
    // Inactive lanes take key 0 and are never in the starting mask, so a ballot needs no "and active": the compare
    // writes the lane mask directly (the compiler builtin takes the predicate as it is; __ballot() goes through an
    // integer and back).
    unsigned long long m = __builtin_amdgcn_ballot_w64(active);
    const int k = active ? key : 0;
    for (int bit = 0; bit < keybits; ++bit) {
        const bool one = (k >> bit) & 1;
        const unsigned long long bal = __builtin_amdgcn_ballot_w64(one);
        m &= one ? bal : ~bal;
    }
    return active ? m : 0ull;
}

}  // namespace f3d

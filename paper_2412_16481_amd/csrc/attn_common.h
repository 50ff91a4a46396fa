// Device helpers shared by the forward (attn.hip) and backward (attn_bwd.hip) attention kernels: the MFMA
// fragment types, the scope -> row-segment arithmetic (Section 4.2; Appendix "Bucket-Swin") and bf16 packing.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn.h"

namespace f3d {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int KT = 128;         // key rows per LDS stage
constexpr int VSTR = KT + 8;    // row pitch of V^T in LDS (elements); keeps 16-byte alignment, staggers banks
constexpr int MAXSEG = 16;

union U4 {
    uint4 u;
    bf16x8 b;
    f16x8 f;
    uint16_t h[8];
};

__device__ __forceinline__ int find_slot_scan(const int* sbs, int n_scans, int m, int extra, int slot)
{
    // scans own disjoint slot ranges starting at sbs[b]/m + extra*b
    int lo = 0, hi = n_scans;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (sbs[mid] / m + extra * mid <= slot) lo = mid; else hi = mid;
    }
    return lo;
}

// Position inside a scope -> bucket-major row. A scope is up to m runs of rows (one per bucket).
struct SegMap {
    int nseg, d0, d1, d2, d3, p1, p2, p3;
};

__device__ __forceinline__ int seg_row_of(const SegMap sm, const int* seg_pre, const int* seg_row0, int x)
{
    if (sm.nseg == 1) return sm.d0 + x;
    if (sm.nseg <= 4) {
        int d = sm.d0;
        d = x >= sm.p1 ? sm.d1 : d;
        d = x >= sm.p2 ? sm.d2 : d;
        d = x >= sm.p3 ? sm.d3 : d;
        return x + d;
    }
    int s = 0;
    while (s + 1 < sm.nseg && x >= seg_pre[s + 1]) ++s;
    return seg_row0[s] + (x - seg_pre[s]);
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    f32x2 x = {lo, hi};
    bf16x2 y = __builtin_convertvector(x, bf16x2);  // v_cvt_pk_bf16_f32, round to nearest even
    return *reinterpret_cast<uint32_t*>(&y);
}

// Row segments of scope g of a scan (first bucket kb0, K buckets): one run for plain and shifted scopes, up to m
// runs (one bucket each) for strided ones. Written by one thread: seg_row0[s] = first row, seg_pre[s] = position of
// that row inside the scope, seg_pre[nseg] = rows of the scope.
__device__ inline void build_segments(const AttnArgs& a, int g, int kb0, int K, int* seg_row0, int* seg_pre, int* s_nseg)
{
    int nseg = 0, pre = 0;
    const int m = a.m;
    if (a.mode == 2) {
        const int t = a.stride;
        const int full = K / (m * t), rem = K - full * m * t;
        const int ngr = full * t + min(rem, t);
        if (g < ngr) {
            const int j0 = (g / t) * m * t + (g % t);
            for (int i = 0; i < m; ++i) {
                const int j = j0 + i * t;
                if (j >= K) break;
                const int r0 = a.offsets[kb0 + j], len = a.offsets[kb0 + j + 1] - r0;
                if (len <= 0) continue;
                seg_row0[nseg] = r0;
                seg_pre[nseg] = pre;
                pre += len;
                ++nseg;
            }
        }
    } else {
        int j0, j1;
        if (a.mode == 1) {
            j0 = g == 0 ? 0 : a.shift + (g - 1) * m;
            j1 = g == 0 ? a.shift : j0 + m;
        } else {
            j0 = g * m;
            j1 = j0 + m;
        }
        j1 = min(j1, K);
        if (j0 < K) {
            const int r0 = a.offsets[kb0 + j0], len = a.offsets[kb0 + j1] - r0;
            if (len > 0) {
                seg_row0[0] = r0;
                seg_pre[0] = 0;
                pre = len;
                nseg = 1;
            }
        }
    }
    seg_pre[nseg] = pre;
    *s_nseg = nseg;
}

}  // namespace

}  // namespace f3d

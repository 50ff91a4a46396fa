// Backward of the Bucket-and-Swin attention (Section 4.2; the experiments report training latency) for gfx950.
//
//   S = scale Q K^T,  P = exp(S - lse),  dP = dO V^T,  D_i = sum_c dO_ic O_ic,  dS = P o (dP - D),
//   dQ = scale dS K,  dK = scale dS^T Q,  dV = P^T dO
// inside every scope, with the same scope -> row arithmetic as the forward kernel. P is recomputed from the
// forward's log-sum-exp; nothing of size n_g^2 ever leaves the registers.
//
// Two kernels, neither needs atomics:
//   k_attn_bwd_dq    a workgroup owns 128 query rows and streams the scope's K and V through LDS (as the forward
//                    kernel does). Scores are computed transposed (keys x queries), so a lane owns 16 keys of ONE
//                    query: lse and D are per-lane scalars, and dS^T, packed to bf16, is directly the B operand of
//                    dQ^T += K^T dS^T with K^T kept in LDS in the matching key order.
//   k_attn_bwd_dkdv  a workgroup owns 128 key rows and streams the scope's Q and dO through LDS. Scores are
//                    computed as queries x keys, so a lane owns 16 queries of ONE key: P and dS, packed to bf16, are
//                    the B operands of dV^T += dO^T P and dK^T += Q^T dS with Q^T and dO^T kept in LDS.
// Both recompute the exponentials; the matrix core has the room (it is not the busy unit of the forward either).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn.h"
#include "attn_common.h"

namespace f3d {

namespace {

constexpr float LOG2E = 1.4426950408889634f;

// ------------------------------------------------------------------------------------------------
// D[p, h] = sum over the head's channels of dO[p, c] * O[p, c]   (both bucket-major bf16 rows)
__global__ __launch_bounds__(256) void k_attn_bwd_pre(AttnBwdArgs a, int head_dim)
{
    const long long total = (long long)a.f.n * a.f.H;
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const long long p = i / a.f.H;
    const int h = (int)(i - p * a.f.H);
    const uint4* o = reinterpret_cast<const uint4*>(a.f.out + p * a.f.C + (size_t)h * head_dim);
    const uint4* g = reinterpret_cast<const uint4*>(a.dout + p * a.f.C + (size_t)h * head_dim);
    float acc = 0.f;
    for (int c = 0; c < head_dim / 8; ++c) {
        const uint4 x = o[c], y = g[c];
        const uint32_t xw[4] = {x.x, x.y, x.z, x.w}, yw[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc += __uint_as_float(xw[e] << 16) * __uint_as_float(yw[e] << 16);
            acc += __uint_as_float(xw[e] & 0xFFFF0000u) * __uint_as_float(yw[e] & 0xFFFF0000u);
        }
    }
    a.dsum[i] = acc;
}

// scope of a workgroup, shared by both kernels
struct ScopeCtx {
    int head, blk, ng;
    SegMap sm;
};

template <int D>
__device__ __forceinline__ bool scope_of_block(const AttnArgs& a, int blocks_per_scope, int* seg_row0, int* seg_pre, int* s_nseg,
                                               ScopeCtx& c)
{
    const int total = gridDim.x;  // multiple of 8; consecutive ids stay on one XCD
    const int w = blockIdx.x;
    const int u = (w & 7) * (total >> 3) + (w >> 3);
    c.blk = u % blocks_per_scope;
    c.head = (u / blocks_per_scope) % a.H;
    const int slot = u / (blocks_per_scope * a.H);
    if (slot >= a.n_slots) return false;
    if (a.sbs[a.n_scans] <= 0) return false;
    const int b = find_slot_scan(a.sbs, a.n_scans, a.m, a.extra, slot);
    const int g = slot - (a.sbs[b] / a.m + a.extra * b);
    const int kb0 = a.sbs[b], K = a.sbs[b + 1] - kb0;
    if (K <= 0) return false;
    if (threadIdx.x == 0) build_segments(a, g, kb0, K, seg_row0, seg_pre, s_nseg);
    __syncthreads();
    const int nseg = *s_nseg;
    if (nseg == 0) return false;
    c.ng = seg_pre[nseg];
    if (c.blk * 128 >= c.ng) return false;
    constexpr int BIG = 0x7FFFFFFF;
    c.sm.nseg = nseg;
    c.sm.d0 = __builtin_amdgcn_readfirstlane(seg_row0[0]);
    c.sm.p1 = __builtin_amdgcn_readfirstlane(nseg > 1 ? seg_pre[1] : BIG);
    c.sm.p2 = __builtin_amdgcn_readfirstlane(nseg > 2 ? seg_pre[2] : BIG);
    c.sm.p3 = __builtin_amdgcn_readfirstlane(nseg > 3 ? seg_pre[3] : BIG);
    c.sm.d1 = __builtin_amdgcn_readfirstlane(nseg > 1 ? seg_row0[1] - seg_pre[1] : 0);
    c.sm.d2 = __builtin_amdgcn_readfirstlane(nseg > 2 ? seg_row0[2] - seg_pre[2] : 0);
    c.sm.d3 = __builtin_amdgcn_readfirstlane(nseg > 3 ? seg_row0[3] - seg_pre[3] : 0);
    return true;
}

// bf16 fragment times a scalar, split into a bf16 head and a bf16 remainder (x*c = hi + lo up to 2^-17 relative)
__device__ __forceinline__ void scale_split(const U4& x, float c, U4& hi, U4& lo)
{
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const uint32_t w2 = (&x.u.x)[e];
        const float x0 = __uint_as_float(w2 << 16) * c, x1 = __uint_as_float(w2 & 0xFFFF0000u) * c;
        const uint32_t h = pack_bf16(x0, x1);
        const float r0 = x0 - __uint_as_float(h << 16), r1 = x1 - __uint_as_float(h & 0xFFFF0000u);
        (&hi.u.x)[e] = h;
        (&lo.u.x)[e] = pack_bf16(r0, r1);
    }
}

// A row's log-sum-exp (in log2 units) and D as bf16 head + remainder pairs: {L_hi, L_lo}, {D_hi, D_lo}. One more MFMA
// whose other operand holds -1 at the matching two positions subtracts them from a whole score tile (error 2^-17
// relative), which is cheaper than 16 subtractions per lane and tile on the vector ALU.
__device__ __forceinline__ uint2 split_pairs(float l2, float dsum)
{
    const uint32_t lh = pack_bf16(l2, dsum);   // heads: l2 in the low half, dsum in the high half
    const float lr = l2 - __uint_as_float(lh << 16), dr = dsum - __uint_as_float(lh & 0xFFFF0000u);
    const uint32_t lo = pack_bf16(lr, dr);
    // regroup to {L_hi, L_lo} and {D_hi, D_lo}
    return make_uint2((lh & 0xFFFFu) | (lo << 16), (lh >> 16) | (lo & 0xFFFF0000u));
}

// store one 16-byte piece of a row transposed into a [rows of dims][VSTR] array, at the column the MFMA result order
// wants for row kk of the stage (see the forward kernel's V^T)
template <int TS>
__device__ __forceinline__ void store_transposed(uint16_t* base, int c, int kk, uint32_t v0, uint32_t v1, uint32_t v2, uint32_t v3)
{
    const int w16 = kk & 15;
    const int pos = (kk & ~15) + 8 * ((w16 >> 2) & 1) + 4 * (w16 >> 3) + (w16 & 3);
    uint16_t* col = base + c * 8 * TS + pos;
    col[0 * TS] = (uint16_t)(v0 & 0xFFFFu);
    col[1 * TS] = (uint16_t)(v0 >> 16);
    col[2 * TS] = (uint16_t)(v1 & 0xFFFFu);
    col[3 * TS] = (uint16_t)(v1 >> 16);
    col[4 * TS] = (uint16_t)(v2 & 0xFFFFu);
    col[5 * TS] = (uint16_t)(v2 >> 16);
    col[6 * TS] = (uint16_t)(v3 & 0xFFFFu);
    col[7 * TS] = (uint16_t)(v3 >> 16);
}

template <int D>
__device__ __forceinline__ void store_grad_rows(uint16_t* dst_base, const int32_t* out_perm, int row, int C, size_t hoff, int hf,
                                                const f32x16& acc, float mul)
{
    if (row < 0) return;
    const size_t drow = out_perm ? (size_t)out_perm[row] : (size_t)row;
    uint16_t* dst = dst_base + drow * C + hoff;
#pragma unroll
    for (int blk = 0; blk < D / 8; ++blk) {
        uint2 pk;
        pk.x = pack_bf16(acc[4 * blk] * mul, acc[4 * blk + 1] * mul);
        pk.y = pack_bf16(acc[4 * blk + 2] * mul, acc[4 * blk + 3] * mul);
        *reinterpret_cast<uint2*>(dst + 8 * blk + 4 * hf) = pk;
    }
}

constexpr int TROWS16 = 17;   // head_dim 16: 16 rows of a transposed operand plus one row of zeros for the idle MFMA rows

template <int D>
constexpr int trows() { return D == 16 ? TROWS16 : D; }

template <int D>
constexpr int dkdv_stage_rows() { return D == 32 ? 64 : 128; }

// ------------------------------------------------------------------------------------------------
// dQ. dynamic LDS per buffer: K rows [KT*D] | V rows [KT*D] | K^T [trows][VSTR]   (bf16), two buffers
template <int D>
__global__ __launch_bounds__(256) void k_attn_bwd_dq(AttnBwdArgs b)
{
    constexpr int NC = D / 8, KS = D / 16, LPT = KT * NC / 256;
    constexpr int SWZ_SHIFT = (NC == 2) ? 3 : 2;
    constexpr int BUF = 2 * KT * D + trows<D>() * VSTR;   // elements per buffer
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    __shared__ int seg_row0[MAXSEG];
    __shared__ int seg_pre[MAXSEG + 1];
    __shared__ int s_nseg;
    const AttnArgs& a = b.f;
    ScopeCtx sc;
    if (!scope_of_block<D>(a, a.qblocks, seg_row0, seg_pre, &s_nseg, sc)) return;
    const int ng = sc.ng, head = sc.head;
    const SegMap sm = sc.sm;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hf = lane >> 5;
    const size_t hoff = (size_t)head * D;
    const uint32_t row_bytes = (uint32_t)a.C * 2u;

    // ---- this lane's query: q and dO fragments, log-sum-exp and D
    const int xq = sc.blk * 128 + wave * 32 + l32;
    const bool qok = xq < ng;
    const int orow = qok ? seg_row_of(sm, seg_pre, seg_row0, xq) : -1;
    U4 qhi[KS], qlo[KS], dof[KS];
    U4 ext;         // B operand that carries this query's log-sum-exp and D (lower half-wave: k positions 0..3)
    U4 negS, negD;  // A operands with -1 at the positions of the log-sum-exp pair / the D pair
    ext.u = make_uint4(0, 0, 0, 0);
    negS.u = make_uint4(hf == 0 ? 0xBF80BF80u : 0u, 0, 0, 0);
    negD.u = make_uint4(0, hf == 0 ? 0xBF80BF80u : 0u, 0, 0);
    {
        const size_t gr = qok ? (size_t)(a.perm ? a.perm[orow] : orow) : 0;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            U4 qf;
            qf.u = make_uint4(0, 0, 0, 0);
            dof[ks].u = make_uint4(0, 0, 0, 0);
            if (qok) {
                qf.u = *reinterpret_cast<const uint4*>(a.q + gr * a.C + hoff + ks * 16 + hf * 8);
                dof[ks].u = *reinterpret_cast<const uint4*>(b.dout + (size_t)orow * a.C + hoff + ks * 16 + hf * 8);
            }
            scale_split(qf, a.c_log2, qhi[ks], qlo[ks]);
        }
        if (qok && hf == 0) {
            const uint2 pr = split_pairs(a.lse[(size_t)orow * a.H + head] * LOG2E, b.dsum[(size_t)orow * a.H + head]);
            ext.u.x = pr.x;
            ext.u.y = pr.y;
        }
    }

    // ---- staging of K and V rows (row index through perm one stage ahead, as in the forward kernel)
    u32x4 kreg[LPT], vreg[LPT];
    uint32_t rows_next[LPT];
    const char* kthr[LPT];
    const char* vthr[LPT];
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
        const int c = (tid + i * 256) % NC;
        kthr[i] = reinterpret_cast<const char*>(a.k + hoff + c * 8);
        vthr[i] = reinterpret_cast<const char*>(a.v + hoff + c * 8);
    }
    auto fetch_rows = [&](int st) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            const int x = min(st * KT + (tid + i * 256) / NC, ng - 1);
            const uint32_t r = (uint32_t)seg_row_of(sm, seg_pre, seg_row0, x);
            rows_next[i] = a.perm ? (uint32_t)a.perm[r] : r;
        }
    };
    auto load_stage = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            const uint64_t at = (uint64_t)rows_next[i] * row_bytes;
            kreg[i] = *reinterpret_cast<const u32x4*>(kthr[i] + at);
            vreg[i] = *reinterpret_cast<const u32x4*>(vthr[i] + at);
        }
    };
    auto store_stage = [&](int buf) __attribute__((always_inline)) {
        uint16_t* sK = smem + buf * BUF;
        uint16_t* sVr = sK + KT * D;
        uint16_t* sKT = sVr + KT * D;
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            uint32_t k0 = kreg[i].x, k1 = kreg[i].y, k2 = kreg[i].z, k3 = kreg[i].w;
            asm volatile("" : "+v"(k0), "+v"(k1), "+v"(k2), "+v"(k3));   // no half-splitting right behind the load
            const int uidx = tid + i * 256;
            const int kk = uidx / NC, c = uidx % NC;
            const int cs = c ^ ((kk >> SWZ_SHIFT) & (NC - 1));
            u32x4 kw = {k0, k1, k2, k3};
            *reinterpret_cast<u32x4*>(&sK[kk * D + cs * 8]) = kw;
            *reinterpret_cast<u32x4*>(&sVr[kk * D + cs * 8]) = vreg[i];
            store_transposed<VSTR>(sKT, c, kk, k0, k1, k2, k3);
        }
    };
    if (D == 16)   // the zeros row of K^T
        for (int i = tid; i < VSTR; i += 256) {
            smem[2 * KT * D + D * VSTR + i] = 0;
            smem[BUF + 2 * KT * D + D * VSTR + i] = 0;
        }

    const int nst = (ng + KT - 1) / KT;
    const int trow = (D == 16) ? min(l32, 16) : l32;
    const int toff = trow * VSTR + 8 * hf;
    f32x16 acc = {0};

    fetch_rows(0);
    load_stage();
    if (nst > 1) fetch_rows(1);
    store_stage(0);
    __syncthreads();
    for (int st = 0; st < nst; ++st) {
        const int buf = st & 1;
        if (st + 1 < nst) {
            load_stage();
            if (st + 2 < nst) fetch_rows(st + 2);
        }
        const uint16_t* sK = smem + buf * BUF;
        const uint16_t* sVr = sK + KT * D;
        const uint16_t* sKT = sVr + KT * D + toff;
#pragma unroll 2
        for (int t4 = 0; t4 < KT / 32; ++t4) {
            const int kbase = st * KT + t4 * 32;
            if (kbase >= ng) break;
            const int kk = t4 * 32 + l32;
            f32x16 s = {0}, dp = {0};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const int c = 2 * ks + hf;
                const int cs = c ^ ((kk >> SWZ_SHIFT) & (NC - 1));
                U4 kf, vf;
                kf.u = *reinterpret_cast<const uint4*>(&sK[kk * D + cs * 8]);
                vf.u = *reinterpret_cast<const uint4*>(&sVr[kk * D + cs * 8]);
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf.b, qhi[ks].b, s, 0, 0, 0);
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf.b, qlo[ks].b, s, 0, 0, 0);
                dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.b, dof[ks].b, dp, 0, 0, 0);
            }
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(negS.b, ext.b, s, 0, 0, 0);     // score - lse
            dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(negD.b, ext.b, dp, 0, 0, 0);   // dP - D
            U4 kt0, kt1;
            kt0.u = *reinterpret_cast<const uint4*>(&sKT[t4 * 32]);
            kt1.u = *reinterpret_cast<const uint4*>(&sKT[t4 * 32 + 16]);
            if (kbase + 32 > ng) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = kbase + 8 * (r >> 2) + 4 * hf + (r & 3);
                    if (key >= ng) s[r] = -INFINITY;
                }
            }
            // dS^T = P o (dP^T - D), P = 2^(score - lse)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] = __builtin_amdgcn_exp2f(s[r]) * dp[r];
            union { uint32_t u[4]; bf16x8 b; } pb0, pb1;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                pb0.u[e] = pack_bf16(s[2 * e], s[2 * e + 1]);
                pb1.u[e] = pack_bf16(s[8 + 2 * e], s[8 + 2 * e + 1]);
            }
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt0.b, pb0.b, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt1.b, pb1.b, acc, 0, 0, 0);
        }
        if (st + 1 < nst) store_stage(buf ^ 1);
        __syncthreads();
    }
    store_grad_rows<D>(b.dq, a.out_perm, orow, a.C, hoff, hf, acc, b.scale);
}

// ------------------------------------------------------------------------------------------------
// dK and dV. dynamic LDS per buffer: Q rows [KT*D] | dO rows [KT*D] | Q^T [trows][VSTR] | dO^T [trows][VSTR] (bf16) |
// per row 16 bytes {lse*log2e hi, lo, D hi, lo, 0 x 4} [KT], two buffers
template <int D>
__global__ __launch_bounds__(256) void k_attn_bwd_dkdv(AttnBwdArgs b)
{
    constexpr int KT = dkdv_stage_rows<D>();   // query rows per stage: 64 at head_dim 32 keeps three workgroups per CU
    constexpr int VSTR = KT + 8;
    constexpr int NC = D / 8, KS = D / 16, LPT = KT * NC / 256;
    constexpr int SWZ_SHIFT = (NC == 2) ? 3 : 2;
    constexpr int BUF = 2 * KT * D + 2 * trows<D>() * VSTR + 8 * KT;   // 16-bit elements per buffer
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    __shared__ int seg_row0[MAXSEG];
    __shared__ int seg_pre[MAXSEG + 1];
    __shared__ int s_nseg;
    const AttnArgs& a = b.f;
    ScopeCtx sc;
    if (!scope_of_block<D>(a, b.kblocks, seg_row0, seg_pre, &s_nseg, sc)) return;
    const int ng = sc.ng, head = sc.head;
    const SegMap sm = sc.sm;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hf = lane >> 5;
    const size_t hoff = (size_t)head * D;
    const uint32_t row_bytes = (uint32_t)a.C * 2u;

    // ---- this lane's key: k (scaled, split) and v fragments
    const int xk = sc.blk * 128 + wave * 32 + l32;
    const bool kok = xk < ng;
    const int krow = kok ? seg_row_of(sm, seg_pre, seg_row0, xk) : -1;
    U4 khi[KS], klo[KS], vfr[KS];
    U4 negS, negD;   // B operands with -1 at the positions of a staged row's log-sum-exp pair / D pair
    negS.u = make_uint4(hf == 0 ? 0xBF80BF80u : 0u, 0, 0, 0);
    negD.u = make_uint4(0, hf == 0 ? 0xBF80BF80u : 0u, 0, 0);
    {
        const size_t gr = kok ? (size_t)(a.perm ? a.perm[krow] : krow) : 0;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            U4 kf;
            kf.u = make_uint4(0, 0, 0, 0);
            vfr[ks].u = make_uint4(0, 0, 0, 0);
            if (kok) {
                kf.u = *reinterpret_cast<const uint4*>(a.k + gr * a.C + hoff + ks * 16 + hf * 8);
                vfr[ks].u = *reinterpret_cast<const uint4*>(a.v + gr * a.C + hoff + ks * 16 + hf * 8);
            }
            scale_split(kf, a.c_log2, khi[ks], klo[ks]);
        }
    }

    // ---- staging of Q and dO rows with their lse and D
    u32x4 qreg[LPT], greg[LPT];
    uint32_t rows_next[LPT], brow_next[LPT];   // row of q (through perm) and bucket-major row (dO, lse, D)
    float lreg = 0.f, dreg = 0.f;
    int lrow_next = 0;
    const char* qthr[LPT];
    const char* gthr[LPT];
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
        const int c = (tid + i * 256) % NC;
        qthr[i] = reinterpret_cast<const char*>(a.q + hoff + c * 8);
        gthr[i] = reinterpret_cast<const char*>(b.dout + hoff + c * 8);
    }
    auto fetch_rows = [&](int st) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            const int x = min(st * KT + (tid + i * 256) / NC, ng - 1);
            const uint32_t r = (uint32_t)seg_row_of(sm, seg_pre, seg_row0, x);
            brow_next[i] = r;
            rows_next[i] = a.perm ? (uint32_t)a.perm[r] : r;
        }
        if (tid < KT) {
            const int x = st * KT + tid;
            lrow_next = x < ng ? seg_row_of(sm, seg_pre, seg_row0, x) : -1;
        }
    };
    auto load_stage = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            qreg[i] = *reinterpret_cast<const u32x4*>(qthr[i] + (uint64_t)rows_next[i] * row_bytes);
            greg[i] = *reinterpret_cast<const u32x4*>(gthr[i] + (uint64_t)brow_next[i] * row_bytes);
        }
        if (tid < KT) {
            // a position past the end of the scope gets a huge lse: its probabilities are exactly zero
            lreg = lrow_next >= 0 ? a.lse[(size_t)lrow_next * a.H + head] * LOG2E : 1e30f;
            dreg = lrow_next >= 0 ? b.dsum[(size_t)lrow_next * a.H + head] : 0.f;
        }
    };
    auto store_stage = [&](int buf) __attribute__((always_inline)) {
        uint16_t* sQ = smem + buf * BUF;
        uint16_t* sG = sQ + KT * D;
        uint16_t* sQT = sG + KT * D;
        uint16_t* sGT = sQT + trows<D>() * VSTR;
        uint4* sX = reinterpret_cast<uint4*>(sGT + trows<D>() * VSTR);
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            uint32_t q0 = qreg[i].x, q1 = qreg[i].y, q2 = qreg[i].z, q3 = qreg[i].w;
            uint32_t g0 = greg[i].x, g1 = greg[i].y, g2 = greg[i].z, g3 = greg[i].w;
            asm volatile("" : "+v"(q0), "+v"(q1), "+v"(q2), "+v"(q3), "+v"(g0), "+v"(g1), "+v"(g2), "+v"(g3));
            const int uidx = tid + i * 256;
            const int kk = uidx / NC, c = uidx % NC;
            const int cs = c ^ ((kk >> SWZ_SHIFT) & (NC - 1));
            u32x4 qw = {q0, q1, q2, q3}, gw = {g0, g1, g2, g3};
            *reinterpret_cast<u32x4*>(&sQ[kk * D + cs * 8]) = qw;
            *reinterpret_cast<u32x4*>(&sG[kk * D + cs * 8]) = gw;
            store_transposed<VSTR>(sQT, c, kk, q0, q1, q2, q3);
            store_transposed<VSTR>(sGT, c, kk, g0, g1, g2, g3);
        }
        if (tid < KT) {
            const uint2 pr = split_pairs(lreg, dreg);
            sX[tid] = make_uint4(pr.x, pr.y, 0, 0);
        }
    };
    if (D == 16)   // the zeros rows of Q^T and dO^T
        for (int i = tid; i < VSTR; i += 256)
            for (int bf = 0; bf < 2; ++bf) {
                smem[bf * BUF + 2 * KT * D + D * VSTR + i] = 0;
                smem[bf * BUF + 2 * KT * D + trows<D>() * VSTR + D * VSTR + i] = 0;
            }

    const int nst = (ng + KT - 1) / KT;
    const int trow = (D == 16) ? min(l32, 16) : l32;
    const int toff = trow * VSTR + 8 * hf;
    f32x16 dk = {0}, dv = {0};

    fetch_rows(0);
    load_stage();
    if (nst > 1) fetch_rows(1);
    store_stage(0);
    __syncthreads();
    for (int st = 0; st < nst; ++st) {
        const int buf = st & 1;
        if (st + 1 < nst) {
            load_stage();
            if (st + 2 < nst) fetch_rows(st + 2);
        }
        const uint16_t* sQ = smem + buf * BUF;
        const uint16_t* sG = sQ + KT * D;
        const uint16_t* sQT = sG + KT * D + toff;
        const uint16_t* sGT = sQT + trows<D>() * VSTR;
        const uint4* sX = reinterpret_cast<const uint4*>(smem + buf * BUF + 2 * KT * D + 2 * trows<D>() * VSTR);
#pragma unroll 2
        for (int t4 = 0; t4 < KT / 32; ++t4) {
            const int qbase = st * KT + t4 * 32;
            if (qbase >= ng) break;
            const int qq = t4 * 32 + l32;   // the stage row this lane reads as an A operand (a query)
            f32x16 s = {0}, dp = {0};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const int c = 2 * ks + hf;
                const int cs = c ^ ((qq >> SWZ_SHIFT) & (NC - 1));
                U4 qf, gf;
                qf.u = *reinterpret_cast<const uint4*>(&sQ[qq * D + cs * 8]);
                gf.u = *reinterpret_cast<const uint4*>(&sG[qq * D + cs * 8]);
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf.b, khi[ks].b, s, 0, 0, 0);
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf.b, klo[ks].b, s, 0, 0, 0);
                dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gf.b, vfr[ks].b, dp, 0, 0, 0);
            }
            {   // subtract every query's log-sum-exp from its score row and its D from its dP row on the matrix core
                U4 xf;
                xf.u = sX[qq];
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf.b, negS.b, s, 0, 0, 0);
                dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf.b, negD.b, dp, 0, 0, 0);
            }
            U4 qt0, qt1, gt0, gt1;
            qt0.u = *reinterpret_cast<const uint4*>(&sQT[t4 * 32]);
            qt1.u = *reinterpret_cast<const uint4*>(&sQT[t4 * 32 + 16]);
            gt0.u = *reinterpret_cast<const uint4*>(&sGT[t4 * 32]);
            gt1.u = *reinterpret_cast<const uint4*>(&sGT[t4 * 32 + 16]);
            // P = 2^(score - lse), dS = P o (dP - D)
            f32x16 p;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                p[r] = __builtin_amdgcn_exp2f(s[r]);
                s[r] = p[r] * dp[r];
            }
            union { uint32_t u[4]; bf16x8 b; } pb0, pb1, sb0, sb1;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                pb0.u[e] = pack_bf16(p[2 * e], p[2 * e + 1]);
                pb1.u[e] = pack_bf16(p[8 + 2 * e], p[8 + 2 * e + 1]);
                sb0.u[e] = pack_bf16(s[2 * e], s[2 * e + 1]);
                sb1.u[e] = pack_bf16(s[8 + 2 * e], s[8 + 2 * e + 1]);
            }
            dv = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gt0.b, pb0.b, dv, 0, 0, 0);
            dv = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gt1.b, pb1.b, dv, 0, 0, 0);
            dk = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qt0.b, sb0.b, dk, 0, 0, 0);
            dk = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qt1.b, sb1.b, dk, 0, 0, 0);
        }
        if (st + 1 < nst) store_stage(buf ^ 1);
        __syncthreads();
    }
    store_grad_rows<D>(b.dk, a.out_perm, krow, a.C, hoff, hf, dk, b.scale);
    store_grad_rows<D>(b.dv, a.out_perm, krow, a.C, hoff, hf, dv, 1.0f);
}

template <int D>
hipError_t launch_d(const AttnBwdArgs& b, hipStream_t stream)
{
    const AttnArgs& a = b.f;
    const long long rows = (long long)a.n * a.H;
    if (rows > 0) k_attn_bwd_pre<<<(unsigned)((rows + 255) / 256), 256, 0, stream>>>(b, D);
    const size_t lds_dq = (size_t)2 * (2 * KT * D + trows<D>() * VSTR) * 2;
    constexpr int KB = dkdv_stage_rows<D>();
    const size_t lds_kv = (size_t)2 * (2 * KB * D + 2 * trows<D>() * (KB + 8) + 8 * KB) * 2;
    hipError_t e = hipFuncSetAttribute((const void*)k_attn_bwd_dq<D>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_dq);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void*)k_attn_bwd_dkdv<D>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_kv);
    if (e != hipSuccess) return e;
    long long total = (long long)a.n_slots * a.H * a.qblocks;
    total = (total + 7) / 8 * 8;
    if (total > 0) k_attn_bwd_dq<D><<<(unsigned)total, 256, lds_dq, stream>>>(b);
    total = (long long)a.n_slots * a.H * b.kblocks;
    total = (total + 7) / 8 * 8;
    if (total > 0) k_attn_bwd_dkdv<D><<<(unsigned)total, 256, lds_kv, stream>>>(b);
    return hipGetLastError();
}

}  // namespace

hipError_t attn_bwd_launch(const AttnBwdArgs& b, int head_dim, hipStream_t stream)
{
    return head_dim == 16 ? launch_d<16>(b, stream) : launch_d<32>(b, stream);
}

}  // namespace f3d

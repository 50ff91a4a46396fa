// Bucket-and-Swin attention forward for gfx950 (Section 4.2; Appendix "Bucket-Swin").
//
// One workgroup = 4 waves; a wave owns QT tiles of 32 query rows of one (scope, head), so a workgroup covers
// 128*QT query rows. Keys/values of the scope stream through LDS in stages of 128 rows, double buffered.
// Which rows a stage holds is index arithmetic on the bucket offsets (plain / shifted / strided scope), so
// regrouping costs no pass over memory.
//
// Per 32-key tile a wave computes the TRANSPOSED score tile S^T = K Q^T with 32x32x16 bf16 MFMAs. In the
// MFMA result layout a lane then owns 16 keys of ONE query, so the exponentials are per-lane work, and the
// fp32 result registers, rounded to bf16, already are the B operand of the second MFMA O^T += V^T P^T as
// long as V^T is read from LDS in the matching key order. No cross-lane shuffle of P, no LDS round trip.
// For head_dim 16 the second MFMA has 16 spare output rows; row 16 multiplies P by ones, which yields the
// softmax denominator on the matrix core instead of the vector ALU.
// The K and V^T fragments of a key tile are read from LDS once and used for all QT query tiles of the wave.
//
// The element type is bfloat16 (the benchmark configurations) or binary16 (the Appendix keeps the features in FP16):
// same kernel, other MFMA and conversion instructions. binary16 probabilities overflow at 2^16, so the optimistic
// sweep described below is accepted only for denominators in a much narrower window.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "attn.h"
#include "attn_common.h"

namespace f3d {

namespace {

// what depends on the 16-bit element type
template <bool F16>
struct Elem;
template <>
struct Elem<false> {
    static constexpr uint16_t ONE = 0x3F80;
    static constexpr float DEN_LO = 9.094947e-13f, DEN_HI = 1.2089258e24f;   // 2^-40, 2^80
    static __device__ __forceinline__ uint32_t pack(float lo, float hi) { return pack_bf16(lo, hi); }
    static __device__ __forceinline__ float lo(uint32_t w) { return __uint_as_float(w << 16); }
    static __device__ __forceinline__ float hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
    static __device__ __forceinline__ f32x16 mfma(const U4& x, const U4& y, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(x.b, y.b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ float sum2(uint32_t pair, float c)   // c + both halves of the pair
    {
        const uint32_t ones = 0x3F803F80u;
        return __builtin_amdgcn_fdot2_f32_bf16(*reinterpret_cast<const bf16x2*>(&pair), *reinterpret_cast<const bf16x2*>(&ones), c, false);
    }
};
template <>
struct Elem<true> {
    static constexpr uint16_t ONE = 0x3C00;
    // a probability above 65504 rounds to infinity (and so does the denominator); below 2^-3 the terms that carry the
    // sum may be subnormal with fewer than eight significant bits
    static constexpr float DEN_LO = 0.125f, DEN_HI = 1.0737418e9f;           // 2^-3, 2^30
    static __device__ __forceinline__ uint32_t pack(float lo, float hi)
    {
        f32x2 x = {lo, hi};
        f16x2 y = __builtin_convertvector(x, f16x2);   // round to nearest even, overflow to infinity
        return *reinterpret_cast<uint32_t*>(&y);
    }
    static __device__ __forceinline__ float lo(uint32_t w)
    {
        const f16x2 h = *reinterpret_cast<const f16x2*>(&w);
        return (float)h[0];
    }
    static __device__ __forceinline__ float hi(uint32_t w)
    {
        const f16x2 h = *reinterpret_cast<const f16x2*>(&w);
        return (float)h[1];
    }
    static __device__ __forceinline__ f32x16 mfma(const U4& x, const U4& y, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(x.f, y.f, c, 0, 0, 0);
    }
    static __device__ __forceinline__ float sum2(uint32_t pair, float c)
    {
        const uint32_t ones = 0x3C003C00u;
        return __builtin_amdgcn_fdot2(*reinterpret_cast<const f16x2*>(&pair), *reinterpret_cast<const f16x2*>(&ones), c, false);
    }
};

template <int D, int QT, bool F16>
__global__ __launch_bounds__(256) void k_attn(AttnArgs a)
{
    using E = Elem<F16>;
    constexpr int NC = D / 8;              // 16-byte chunks of one head in a row
    constexpr int KS = D / 16;             // MFMA k-steps for Q K^T
    constexpr int LPT = KT * NC / 256;     // 16-byte loads per thread per stage and tensor
    constexpr int SWZ_SHIFT = (NC == 2) ? 3 : 2;
    constexpr int BM = 128 * QT;           // query rows per workgroup

    __shared__ __attribute__((aligned(16))) uint16_t sK[2][KT * D];
    __shared__ __attribute__((aligned(16))) uint16_t sV[2][(D + (D == 16 ? 2 : 0)) * VSTR];
    __shared__ int seg_row0[MAXSEG];
    __shared__ int seg_pre[MAXSEG + 1];
    __shared__ int s_nseg;

    // ---- which (scope, head, query block) is this workgroup: consecutive ids stay on one XCD
    const int total = gridDim.x;  // multiple of 8
    const int w = blockIdx.x;
    const int u = (w & 7) * (total >> 3) + (w >> 3);
    const int qb = u % a.qblocks;
    const int head = (u / a.qblocks) % a.H;
    const int slot = u / (a.qblocks * a.H);
    if (slot >= a.n_slots) return;
    if (a.sbs[a.n_scans] <= 0) return;
    const int b = find_slot_scan(a.sbs, a.n_scans, a.m, a.extra, slot);
    const int g = slot - (a.sbs[b] / a.m + a.extra * b);
    const int kb0 = a.sbs[b], K = a.sbs[b + 1] - kb0;
    if (K <= 0) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hf = lane >> 5;

    // ---- rows of the scope: up to m segments (one bucket each; plain/shifted scopes are one run)
    if (tid == 0) build_segments(a, g, kb0, K, seg_row0, seg_pre, &s_nseg);
    __syncthreads();
    const int nseg = s_nseg;
    if (nseg == 0) return;
    const int ng = seg_pre[nseg];         // rows in this scope
    if (qb * BM >= ng) return;

    // Up to four segments (the usual scope of four buckets) are kept in scalar registers as (first position,
    // row minus position) pairs, so mapping a position to its row is a few compares and no LDS traffic.
    constexpr int BIG = 0x7FFFFFFF;
    const int d0 = __builtin_amdgcn_readfirstlane(seg_row0[0]);
    const int p1 = __builtin_amdgcn_readfirstlane(nseg > 1 ? seg_pre[1] : BIG);
    const int p2 = __builtin_amdgcn_readfirstlane(nseg > 2 ? seg_pre[2] : BIG);
    const int p3 = __builtin_amdgcn_readfirstlane(nseg > 3 ? seg_pre[3] : BIG);
    const int d1 = __builtin_amdgcn_readfirstlane(nseg > 1 ? seg_row0[1] - seg_pre[1] : 0);
    const int d2 = __builtin_amdgcn_readfirstlane(nseg > 2 ? seg_row0[2] - seg_pre[2] : 0);
    const int d3 = __builtin_amdgcn_readfirstlane(nseg > 3 ? seg_row0[3] - seg_pre[3] : 0);
    const SegMap sm{nseg, d0, d1, d2, d3, p1, p2, p3};
    auto seg_row = [sm](int x) __attribute__((always_inline)) -> int {
        return seg_row_of(sm, seg_pre, seg_row0, x);
    };

    const size_t hoff = (size_t)head * D;
    const uint32_t row_bytes = (uint32_t)a.C * 2u;

    // ---- staging of K and V rows. The row index of a staged key goes through the permutation, a load the
    //      K/V loads depend on; it is fetched one stage earlier than the rows themselves so that no stage
    //      starts with a dependent round trip to memory. Positions past the end of the scope fetch its last
    //      row again instead of zeros: their scores are masked, so all they must be is finite wherever the
    //      scope's own rows are, and no lane leaves the common path.
    u32x4 kreg[LPT], vreg[LPT];
    uint32_t rows_next[LPT];
    const char* kthr[LPT];   // this thread's 16-byte column of the K / V matrices
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
            const uint32_t r = (uint32_t)seg_row(x);
            rows_next[i] = a.perm ? (uint32_t)a.perm[r] : r;
        }
    };
    auto load_stage = [&]() __attribute__((always_inline)) {   // rows_next -> registers
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            const uint64_t at = (uint64_t)rows_next[i] * row_bytes;   // one 32x32->64 multiply-add per address
            kreg[i] = *reinterpret_cast<const u32x4*>(kthr[i] + at);
            vreg[i] = *reinterpret_cast<const u32x4*>(vthr[i] + at);
        }
    };
    auto store_stage = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            // The loaded V words are made opaque up to here: otherwise the compiler splits them into halves
            // right behind the load instruction, and every stage begins by waiting out the load it just issued.
            uint32_t v0 = vreg[i].x, v1 = vreg[i].y, v2 = vreg[i].z, v3 = vreg[i].w;
            asm volatile("" : "+v"(v0), "+v"(v1), "+v"(v2), "+v"(v3));
            const int uidx = tid + i * 256;
            const int kk = uidx / NC, c = uidx % NC;
            const int cs = c ^ ((kk >> SWZ_SHIFT) & (NC - 1));
            *reinterpret_cast<u32x4*>(&sK[buf][kk * D + cs * 8]) = kreg[i];
            // V is stored transposed, keys of a 16-block reordered to the order the MFMA result holds them
            const int w16 = kk & 15;
            const int pos = (kk & ~15) + 8 * ((w16 >> 2) & 1) + 4 * (w16 >> 3) + (w16 & 3);
            uint16_t* col = &sV[buf][c * 8 * VSTR + pos];
            col[0 * VSTR] = (uint16_t)(v0 & 0xFFFFu);
            col[1 * VSTR] = (uint16_t)(v0 >> 16);
            col[2 * VSTR] = (uint16_t)(v1 & 0xFFFFu);
            col[3 * VSTR] = (uint16_t)(v1 >> 16);
            col[4 * VSTR] = (uint16_t)(v2 & 0xFFFFu);
            col[5 * VSTR] = (uint16_t)(v2 >> 16);
            col[6 * VSTR] = (uint16_t)(v3 & 0xFFFFu);
            col[7 * VSTR] = (uint16_t)(v3 >> 16);
        }
    };

    // ---- the first memory requests of the workgroup, in the order that makes two round trips of them instead of
    //      four: the row indices (of the queries and of the keys of stage 0, both through the permutation), then the
    //      query fragments and the K/V rows of stage 0. The query fragment is row l32 of each of the wave's QT query
    //      tiles, dims 8*hf + 16*ks ..
    U4 qf[QT][KS];
    int orow[QT];
    size_t qrow[QT];
#pragma unroll
    for (int t = 0; t < QT; ++t) {
        const int xq = qb * BM + (wave * QT + t) * 32 + l32;
        orow[t] = xq < ng ? seg_row(xq) : -1;
        const int r = max(orow[t], 0);                       // past the end: some valid row, never stored
        qrow[t] = (size_t)(a.perm ? a.perm[r] : r);
    }
    fetch_rows(0);
#pragma unroll
    for (int t = 0; t < QT; ++t) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            qf[t][ks].u = *reinterpret_cast<const uint4*>(a.q + qrow[t] * a.C + hoff + ks * 16 + hf * 8);
    }
    load_stage();

    // head_dim 16: rows 16 and 17 of V^T are constants (ones -> softmax denominator, zeros -> unused rows)
    if (D == 16) {
        for (int i = tid; i < 2 * VSTR; i += 256) {
            const uint16_t val = i < VSTR ? E::ONE : 0;
            sV[0][D * VSTR + i] = val;
            sV[1][D * VSTR + i] = val;
        }
    }

    // The query fragment is pre-multiplied by softmax_scale*log2(e) and split into a 16-bit head and a 16-bit
    // remainder (q*c = hi + lo up to 2^-17 relative), so the MFMA delivers the scaled score directly. The
    // vector ALU is the busy unit of this kernel, the matrix core is not: one more MFMA per tile is cheaper
    // than 16 multiplies. (binary16: the product is kept inside the finite range of the format.)
    U4 qhi[QT][KS], qlo[QT][KS];
    {
        const float cl2 = a.c_log2;
#pragma unroll
        for (int t = 0; t < QT; ++t) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t w2 = (&qf[t][ks].u.x)[e];
                    float x0 = E::lo(w2) * cl2, x1 = E::hi(w2) * cl2;
                    if (F16) {
                        x0 = fminf(fmaxf(x0, -65000.f), 65000.f);
                        x1 = fminf(fmaxf(x1, -65000.f), 65000.f);
                    }
                    const uint32_t h = E::pack(x0, x1);
                    const float r0 = x0 - E::lo(h), r1 = x1 - E::hi(h);
                    (&qhi[t][ks].u.x)[e] = h;
                    (&qlo[t][ks].u.x)[e] = E::pack(r0, r1);
                }
            }
        }
    }

    const int nst = (ng + KT - 1) / KT;
    // this lane's row of V^T: a head dim, or the ones row, or the zeros row
    const int vrow = (D == 16) ? min(l32, 17) : l32;
    const int voff = vrow * VSTR + 8 * hf;

    f32x16 o[QT];
    float l_run[QT], den[QT], mfin[QT];   // mfin: the reference the final sweep's exponentials were taken against

    // One sweep over the keys of the scope. ROBUST == false is the optimistic sweep: softmax taken against
    // the fixed reference 0, i.e. p = 2^score with no running maximum at all. It is exact (softmax does not
    // depend on the reference) as long as the denominator stays well inside the fp32 range, which is checked
    // afterwards; scores beyond about +-55 (natural log units) fail the check and the workgroup repeats the
    // sweep with ROBUST == true, the usual running-maximum form.
    auto sweep = [&](auto robust_tag) {
        constexpr bool ROBUST = decltype(robust_tag)::value;   // the optimistic sweep finds stage 0 already requested
        float m_ref[QT];
        bool first[QT];
#pragma unroll
        for (int t = 0; t < QT; ++t) {
            o[t] = f32x16{0};
            l_run[t] = 0.f;
            m_ref[t] = 0.f;
            first[t] = true;
        }
        if (ROBUST) {
            fetch_rows(0);
            load_stage();
        }
        if (nst > 1) fetch_rows(1);
        store_stage(0);
        __syncthreads();
        for (int st = 0; st < nst; ++st) {
            const int buf = st & 1;
            if (st + 1 < nst) {
                load_stage();            // rows of stage st+1, fetched a stage ago
                if (st + 2 < nst) fetch_rows(st + 2);
            }
            const uint16_t* kbuf = sK[buf];
            const uint16_t* vbuf = sV[buf] + voff;
#pragma unroll 2
            for (int t4 = 0; t4 < KT / 32; ++t4) {
                const int kbase = st * KT + t4 * 32;
                if (kbase >= ng) break;
                const int kk = t4 * 32 + l32;
                U4 kf[KS];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const int c = 2 * ks + hf;
                    const int cs = c ^ ((kk >> SWZ_SHIFT) & (NC - 1));
                    kf[ks].u = *reinterpret_cast<const uint4*>(&kbuf[kk * D + cs * 8]);
                }
                U4 vf0, vf1;
                vf0.u = *reinterpret_cast<const uint4*>(&vbuf[t4 * 32]);
                vf1.u = *reinterpret_cast<const uint4*>(&vbuf[t4 * 32 + 16]);
                // S^T tiles (rows = 32 keys, cols = 32 queries), scaled to log2 units
                f32x16 s[QT];
#pragma unroll
                for (int t = 0; t < QT; ++t) {
                    s[t] = f32x16{0};
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
                        s[t] = E::mfma(kf[ks], qhi[t][ks], s[t]);
                        s[t] = E::mfma(kf[ks], qlo[t][ks], s[t]);
                    }
                }
#pragma unroll
                for (int t = 0; t < QT; ++t) {
                    if (kbase + 32 > ng) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int key = kbase + 8 * (r >> 2) + 4 * hf + (r & 3);
                            if (key >= ng) s[t][r] = -INFINITY;
                        }
                    }
                    if (ROBUST) {
                        float mx = fmaxf(fmaxf(s[t][0], s[t][1]), s[t][2]);
#pragma unroll
                        for (int r = 3; r < 15; r += 2) mx = fmaxf(fmaxf(mx, s[t][r]), s[t][r + 1]);
                        mx = fmaxf(mx, s[t][15]);
                        {   // both half-waves hold keys of the same query: share the maximum
                            const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_int(mx), __float_as_int(mx), false, false);
                            mx = fmaxf(__int_as_float(sw[0]), __int_as_float(sw[1]));
                        }
                        // the reference follows the maximum only when a score exceeds it by more than 2^8 (the first
                        // tile sets it): exponentials stay below 256 and O is rescaled rarely
                        if (first[t] || __builtin_amdgcn_ballot_w64(mx > m_ref[t] + 8.0f)) {
                            const float m_new = first[t] ? mx : fmaxf(mx, m_ref[t]);
                            // the first tile has nothing to rescale (O and the sum are zero), and 2^(0 - m_new) would be
                            // infinite for a maximum below -128: 0 * inf
                            const float alpha = first[t] ? 1.0f : __builtin_amdgcn_exp2f(m_ref[t] - m_new);
                            first[t] = false;
                            m_ref[t] = m_new;
                            constexpr int NO = (D == 16) ? 9 : 16;
#pragma unroll
                            for (int r = 0; r < NO; ++r) o[t][r] *= alpha;
                            if (D == 32) l_run[t] *= alpha;
                        }
#pragma unroll
                        for (int r = 0; r < 16; ++r) s[t][r] -= m_ref[t];
                    }
#pragma unroll
                    for (int r = 0; r < 16; ++r) s[t][r] = __builtin_amdgcn_exp2f(s[t][r]);
                    U4 pb0, pb1;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        (&pb0.u.x)[e] = E::pack(s[t][2 * e], s[t][2 * e + 1]);
                        (&pb1.u.x)[e] = E::pack(s[t][8 + 2 * e], s[t][8 + 2 * e + 1]);
                    }
                    if (D == 32) {   // denominator from the rounded probabilities, two per instruction
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            l_run[t] = E::sum2((&pb0.u.x)[e], l_run[t]);
                            l_run[t] = E::sum2((&pb1.u.x)[e], l_run[t]);
                        }
                    }
                    o[t] = E::mfma(vf0, pb0, o[t]);
                    o[t] = E::mfma(vf1, pb1, o[t]);
                }
            }
            if (st + 1 < nst) store_stage(buf ^ 1);
            __syncthreads();
        }
#pragma unroll
        for (int t = 0; t < QT; ++t) {
            mfin[t] = m_ref[t];
            if (D == 16) {
                den[t] = __shfl(o[t][8], l32, 64);   // row 16 of O^T (sum of probabilities) lives in the lower half-wave
            } else {
                den[t] = l_run[t] + __shfl_xor(l_run[t], 32, 64);
            }
        }
    };

    sweep(std::false_type{});
    {
        // bfloat16: 2^-40 < den < 2^80: no exponential overflowed, and the largest one is far above the flush-to-zero
        // range. binary16: 2^-3 < den < 2^30, see Elem<true>.
        bool bad = false;
#pragma unroll
        for (int t = 0; t < QT; ++t) bad = bad || ((orow[t] >= 0) && !(den[t] > E::DEN_LO && den[t] < E::DEN_HI));
        if (__syncthreads_or(bad)) sweep(std::true_type{});
    }

    // ---- epilogue: divide by the softmax denominator, round to the element type, store
#pragma unroll
    for (int t = 0; t < QT; ++t) {
        if (orow[t] >= 0) {
            const float inv = 1.0f / den[t];
            if (a.lse && hf == 0) a.lse[(size_t)orow[t] * a.H + head] = (mfin[t] + __log2f(den[t])) * 0.6931471805599453f;
            // the query's own bucket-major row, or straight to where the caller wants that row (the inverse of the
            // up-front scatter folded into the last layer's store: same 32-byte pieces, no extra pass)
            const size_t drow = a.out_perm ? (size_t)a.out_perm[orow[t]] : (size_t)orow[t];
            uint16_t* dst = a.out + drow * a.C + hoff;
            constexpr int NB = D / 8;
#pragma unroll
            for (int blk = 0; blk < NB; ++blk) {
                uint2 pk;
                pk.x = E::pack(o[t][4 * blk] * inv, o[t][4 * blk + 1] * inv);
                pk.y = E::pack(o[t][4 * blk + 2] * inv, o[t][4 * blk + 3] * inv);
                *reinterpret_cast<uint2*>(dst + 8 * blk + 4 * hf) = pk;
            }
        }
    }
}

}  // namespace

// Query rows per workgroup. Two query tiles per wave share every K/V fragment read and halve the staging per
// FLOP, but need more registers (3 instead of 5 waves per SIMD) and make fewer, longer workgroups; that pays
// only when the launch is many times larger than what the GPU keeps resident.
static int pick_qt(int head_dim, long long slots, int heads, int bucket_cap)
{
    if (head_dim != 16) return 1;
    const long long wgs_qt1 = slots * heads * ((bucket_cap + 127) / 128);
    return wgs_qt1 >= 16384 ? 2 : 1;
}

int attn_block_rows(int head_dim, long long slots, int heads, int bucket_cap)
{
    return 128 * pick_qt(head_dim, slots, heads, bucket_cap);
}

hipError_t attn_launch(const AttnArgs& a, int head_dim, int block_rows, hipStream_t stream)
{
    long long total = (long long)a.n_slots * a.H * a.qblocks;
    total = (total + 7) / 8 * 8;
    if (total == 0) return hipSuccess;
    if (a.f16) {
        if (head_dim == 16 && block_rows == 256)
            k_attn<16, 2, true><<<(unsigned)total, 256, 0, stream>>>(a);
        else if (head_dim == 16)
            k_attn<16, 1, true><<<(unsigned)total, 256, 0, stream>>>(a);
        else
            k_attn<32, 1, true><<<(unsigned)total, 256, 0, stream>>>(a);
    } else if (head_dim == 16 && block_rows == 256)
        k_attn<16, 2, false><<<(unsigned)total, 256, 0, stream>>>(a);
    else if (head_dim == 16)
        k_attn<16, 1, false><<<(unsigned)total, 256, 0, stream>>>(a);
    else
        k_attn<32, 1, false><<<(unsigned)total, 256, 0, stream>>>(a);
    return hipGetLastError();
}

}  // namespace f3d

// Bucket-and-Swin attention forward for gfx950 (Section 4.2; Appendix "Bucket-Swin").
//
// One workgroup = 4 waves; a wave owns QT tiles of 32 query rows of one (scope, head), so a workgroup covers
// 128*QT query rows. Which rows a scope holds is index arithmetic on the bucket offsets (plain / shifted / strided
// scope), so regrouping costs no pass over memory.
//
// Keys and values of the scope stream through LDS in stages of 128 rows, double buffered, and get there without
// passing through registers: every lane issues 16-byte global -> LDS loads (the row it fetches goes through the
// permutation; the LDS side of such a load is fixed, lane i of a wave fills the i-th 16-byte piece of a 1 KB block,
// so the layout in LDS is chosen through WHICH piece of WHICH row a lane asks for). The loads of stage s+2 are issued
// when stage s has been read, a whole stage of arithmetic before they are needed.
//
// Per 32-key tile a wave computes the TRANSPOSED score tile S^T = K Q^T with 32x32x16 MFMAs. In the MFMA result
// layout a lane then owns 16 keys of ONE query, so the exponentials are per-lane work, and the fp32 result registers,
// rounded to 16 bits, already are the B operand of the second MFMA O^T += V^T P^T. Its A operand, V^T, is read from
// the row-major V tile in LDS with the transposing LDS read of gfx950 (ds_read_b64_tr_b16: 16 lanes hand in the
// addresses of a 4 x 16 block and each receives one column of it), with the key order of the score registers.
// For head_dim 16 the second MFMA has 16 spare output rows; row 16 multiplies P by ones, which yields the
// softmax denominator on the matrix core instead of the vector ALU: the lanes of those rows read a constant block
// of LDS instead of V.
//
// The vector ALU (16 exponentials and 8 packs per tile and lane) is the busy unit, the matrix core is not. The tile
// loop is therefore software pipelined inside the wave: the score MFMAs of the next tile are issued before the
// exponentials of the current one, so the matrix core works underneath the vector ALU.
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

typedef __attribute__((ext_vector_type(4))) short s16x4;
#define F3D_LDS(p) ((__attribute__((address_space(3))) void*)(p))
#define F3D_GLB(p) ((const __attribute__((address_space(1))) void*)(p))

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

// LDS geometry: stages of AKT key rows, NBUF of them resident.
constexpr int AKT = 128;                  // key rows per stage
constexpr int NBUF = 3;
template <int D>
struct Lay {
    static constexpr int NC = D / 8;                  // 16-byte pieces of one head in a row
    static constexpr int KBUF = AKT * D * 2;          // bytes of one K buffer: row-major, pieces of a row xor-swizzled
    // V buffer, bytes. head_dim 32: row-major, 64 bytes per key. head_dim 16: per 32 keys a 1 KB block of rows
    // (32 bytes per key) followed by a 1 KB block of constants, read by the lanes that own rows 16..31 of V^T
    static constexpr int VBUF = 8192;
    static constexpr int VTILE = 2048;                // bytes from one 32-key tile of V to the next
    static constexpr int KTILE = 32 * D * 2;          // the same for K
    static constexpr int LPW = AKT * NC / 256;        // global->LDS loads per lane, stage and tensor
    static constexpr int TOTAL = NBUF * (KBUF + VBUF);
};

// One 16-byte global -> LDS load per lane: lane i of the wave fills bytes [16 i, 16 i + 16) of the 1 KB block at the
// LDS byte address `lds` (wave-uniform; it travels in M0). Written as assembly so that the compiler does not count
// it among its own memory operations: it would otherwise wait for ALL loads in flight before every LDS read that
// follows, and the loads issued here are meant to stay in flight for a whole stage. The kernel waits for them itself
// (s_waitcnt vmcnt(0) before the barrier that hands a stage over).
__device__ __forceinline__ void lds_dma16(const void* g, uint32_t lds)
{
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds), "v"(g) : "memory", "m0");
}

__device__ __forceinline__ uint2 lds_read_tr(uint32_t addr)
{
    const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(uintptr_t)addr);
    return *reinterpret_cast<const uint2*>(&v);
}

__device__ __forceinline__ uint4 lds_read16(uint32_t addr)
{
    const u32x4 v = *(const __attribute__((address_space(3))) u32x4*)(uintptr_t)addr;
    return make_uint4(v.x, v.y, v.z, v.w);
}

#define F3D_SB() __builtin_amdgcn_sched_barrier(0)

template <int D, int QT, bool F16>
__global__ __launch_bounds__(256) void k_attn(AttnArgs a)
{
    using E = Elem<F16>;
    using L = Lay<D>;
    constexpr int NC = L::NC;
    constexpr int KS = D / 16;             // MFMA k-steps for Q K^T
    constexpr int LPW = L::LPW;
    constexpr int BM = 128 * QT;           // query rows per workgroup

    __shared__ __attribute__((aligned(1024))) unsigned char smem[L::TOTAL];
    __shared__ int seg_row0[MAXSEG];
    __shared__ int seg_pre[MAXSEG + 1];
    __shared__ int s_nseg;
    const uint32_t sK = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smem;   // LDS byte addresses
    const uint32_t sV = sK + NBUF * L::KBUF;

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

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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

    // ---- staging of K and V rows: global -> LDS, 16 bytes per lane and load. Load i of this lane fills piece
    //      p = (wave*LPW + i)*64 + lane of the stage: key row p / NC, piece p % NC of that row. K pieces are stored
    //      xor-swizzled by the row (the fragment reads below are then free of bank conflicts), so the lane asks for
    //      piece (p % NC) ^ swizzle(row) of K. The row index of a staged key goes through the permutation, a load the
    //      K/V loads depend on; it is fetched a stage earlier than the rows themselves. Positions past the end of the
    //      scope fetch its last row again instead of zeros: their scores are masked, so all they must be is finite.
    uint32_t rows_next[LPW];
    const char* kthr[LPW];   // this lane's 16-byte column of the K / V matrices
    const char* vthr[LPW];
    int krow[LPW];           // key row inside the stage
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
        const int p = (wave * LPW + i) * 64 + lane;
        const int kk = p / NC, cs = p % NC;
        const int c = (NC == 4) ? (cs ^ ((kk >> 2) & 3)) : (cs ^ ((kk >> 3) & 1));
        krow[i] = kk;
        kthr[i] = reinterpret_cast<const char*>(a.k + hoff + c * 8);
        vthr[i] = reinterpret_cast<const char*>(a.v + hoff + cs * 8);
    }
    auto fetch_rows = [&](int st) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int x = min(st * AKT + krow[i], ng - 1);
            const uint32_t r = (uint32_t)seg_row(x);
            rows_next[i] = a.perm ? (uint32_t)a.perm[r] : r;
        }
    };
    auto dma_stage = [&](int buf) __attribute__((always_inline)) {   // rows_next -> LDS buffer `buf`
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const uint64_t at = (uint64_t)rows_next[i] * row_bytes;   // one 32x32->64 multiply-add per address
            const int blk = wave * LPW + i;
            lds_dma16(kthr[i] + at, sK + buf * L::KBUF + blk * 1024);
            // head_dim 16: 64 pieces are the 32 rows of one tile; its block is followed by the constants' block
            lds_dma16(vthr[i] + at, sV + buf * L::VBUF + (D == 16 ? blk * 2048 : blk * 1024));
        }
    };
    const int nst = (ng + AKT - 1) / AKT;
    auto request_first_stages = [&]() __attribute__((always_inline)) {
        fetch_rows(0);
        dma_stage(0);
        if (nst > 1) {
            fetch_rows(1);
            dma_stage(1);
        }
    };

    // ---- the first memory requests of the workgroup: the row indices (of the queries and of the keys of stages 0
    //      and 1, through the permutation), then the K/V rows of both stages and the query fragments. The query
    //      fragment is row l32 of each of the wave's QT query tiles, dims 8*hf + 16*ks ..
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
    request_first_stages();
#pragma unroll
    for (int t = 0; t < QT; ++t) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            qf[t][ks].u = *reinterpret_cast<const uint4*>(a.q + qrow[t] * a.C + hoff + ks * 16 + hf * 8);
    }

    // head_dim 16: the constants' blocks. Rows 16..31 of V^T are a row of ones (-> softmax denominator) and 15 rows of
    // zeros; the lanes that own them read {1,0,0,0} or {0,0,0,0} from here whatever the key. The pattern sits at
    // bytes 0 and 128 of every 256 so that it shares no bank with the rows the other lanes read at the same moment.
    if (D == 16) {
        for (int i = tid; i < NBUF * 4 * 256; i += 256) {     // buffers x 4 blocks x 256 words
            const int blk = i >> 8, wd = i & 255;
            const uint32_t val = ((wd & 31) == 0) ? (uint32_t)E::ONE : 0u;     // word 0 of every 128 bytes: {1, 0}
            *(__attribute__((address_space(3))) uint32_t*)(uintptr_t)(sV + (blk >> 2) * L::VBUF + (blk & 3) * 2048 + 1024 + wd * 4) = val;
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

    // ---- this lane's fragment addresses inside a buffer (bytes); a tile further on is a constant away
    // K fragment: row l32 of the tile, dims 16*ks + 8*hf ..: one 16-byte piece
    uint32_t koff[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        const int c = 2 * ks + hf;
        const int cs = (NC == 4) ? (c ^ ((l32 >> 2) & 3)) : (c ^ ((l32 >> 3) & 1));
        koff[ks] = sK + (l32 * NC + cs) * 16;
    }
    // V^T fragment through the transposing read: inside every group of 16 lanes, lane 4j + c hands in the address
    // of dims 4c..4c+3 of key row j (of the four rows the read covers) and lane i receives dim i of those four rows.
    // The key rows are the ones the score registers hold: 4*hf + j, +8, +16, +24.
    uint32_t voff;
    {
        const int i16 = lane & 15, j = i16 >> 2, c = i16 & 3, g16 = (lane >> 4) & 1;
        if (D == 32) voff = (4 * hf + j) * 64 + (16 * g16 + 4 * c) * 2;
        else voff = g16 ? 1024 + (hf ? 0 : 128) + (c ? 8 : 0) : (4 * hf + j) * 32 + 8 * c;
        voff += sV;
    }
    constexpr int VSTEP = (D == 32) ? 512 : 256;      // eight key rows further on

    f32x16 o[QT];
    float l_run[QT], den[QT], mfin[QT];   // mfin: the reference the final sweep's exponentials were taken against

    // One sweep over the keys of the scope. ROBUST == false is the optimistic sweep: softmax taken against
    // the fixed reference 0, i.e. p = 2^score with no running maximum at all. It is exact (softmax does not
    // depend on the reference) as long as the denominator stays well inside the fp32 range, which is checked
    // afterwards; scores beyond about +-55 (natural log units) fail the check and the workgroup repeats the
    // sweep with ROBUST == true, the usual running-maximum form.
    auto sweep = [&](auto robust_tag) {
        constexpr bool ROBUST = decltype(robust_tag)::value;   // the optimistic sweep finds stages 0 and 1 already requested
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
            __syncthreads();           // every wave has left the first sweep's buffers
            request_first_stages();
        }
        const int ntile = (ng + 31) >> 5;

        // One unit of the pipeline: the softmax of the score tile `s` (query tile t, keys from kbase on; scores in log2
        // units) and O^T += V^T P^T, with the MFMAs that produce the NEXT score tile (`sn` = kfn * q[tn]^T) issued in
        // between, one per 32 cycles of vector work, so that both units stay busy. The scheduling barriers keep the
        // compiler from regrouping the two streams.
        auto unit = [&](f32x16& s, int t, int kbase, const U4& vf0, const U4& vf1, auto more_tag, f32x16& sn, const U4 (&kfn)[KS],
                        int tn, auto ragged_tag) __attribute__((always_inline)) {
            constexpr bool MORE = decltype(more_tag)::value;
            if (decltype(ragged_tag)::value && kbase + 32 > ng) {   // only the scope's last key tile can be short
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = kbase + 8 * (r >> 2) + 4 * hf + (r & 3);
                    if (key >= ng) s[r] = -INFINITY;
                }
            }
            if (ROBUST) {
                float mx = fmaxf(fmaxf(s[0], s[1]), s[2]);
#pragma unroll
                for (int r = 3; r < 15; r += 2) mx = fmaxf(fmaxf(mx, s[r]), s[r + 1]);
                mx = fmaxf(mx, s[15]);
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
                for (int r = 0; r < 16; ++r) s[r] -= m_ref[t];
            }
            F3D_SB();
#pragma unroll
            for (int r = 0; r < 4; ++r) s[r] = __builtin_amdgcn_exp2f(s[r]);
            F3D_SB();
            if (MORE) sn = E::mfma(kfn[0], qhi[tn][0], f32x16{0});
            F3D_SB();
#pragma unroll
            for (int r = 4; r < 8; ++r) s[r] = __builtin_amdgcn_exp2f(s[r]);
            F3D_SB();
            if (MORE && KS == 2) sn = E::mfma(kfn[0], qlo[tn][0], sn);
            F3D_SB();
#pragma unroll
            for (int r = 8; r < 12; ++r) s[r] = __builtin_amdgcn_exp2f(s[r]);
            F3D_SB();
            if (MORE) sn = (KS == 2) ? E::mfma(kfn[KS - 1], qhi[tn][KS - 1], sn) : E::mfma(kfn[0], qlo[tn][0], sn);
            F3D_SB();
#pragma unroll
            for (int r = 12; r < 16; ++r) s[r] = __builtin_amdgcn_exp2f(s[r]);
            F3D_SB();
            if (MORE && KS == 2) sn = E::mfma(kfn[KS - 1], qlo[tn][KS - 1], sn);
            F3D_SB();
            U4 pb0, pb1;
#pragma unroll
            for (int e = 0; e < 4; ++e) (&pb0.u.x)[e] = E::pack(s[2 * e], s[2 * e + 1]);
            if (D == 32) {   // denominator from the rounded probabilities, two per instruction
#pragma unroll
                for (int e = 0; e < 4; ++e) l_run[t] = E::sum2((&pb0.u.x)[e], l_run[t]);
            }
            F3D_SB();
            o[t] = E::mfma(vf0, pb0, o[t]);
            F3D_SB();
#pragma unroll
            for (int e = 0; e < 4; ++e) (&pb1.u.x)[e] = E::pack(s[8 + 2 * e], s[8 + 2 * e + 1]);
            if (D == 32) {
#pragma unroll
                for (int e = 0; e < 4; ++e) l_run[t] = E::sum2((&pb1.u.x)[e], l_run[t]);
            }
            F3D_SB();
            o[t] = E::mfma(vf1, pb1, o[t]);
            F3D_SB();
        };
        // key tile jt (counted inside a buffer pair: 0..3 this stage, 4.. the next) of the buffers at kb / kbn
        auto read_k = [&](U4 (&kf)[KS], uint32_t kb, int t4) __attribute__((always_inline)) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) kf[ks].u = lds_read16(koff[ks] + kb + t4 * L::KTILE);
        };
        auto read_v = [&](U4& vf0, U4& vf1, uint32_t vb, int t4) __attribute__((always_inline)) {
            const uint32_t p = voff + vb + t4 * L::VTILE;
            const uint2 x0 = lds_read_tr(p), x1 = lds_read_tr(p + VSTEP), x2 = lds_read_tr(p + 2 * VSTEP), x3 = lds_read_tr(p + 3 * VSTEP);
            vf0.u = make_uint4(x0.x, x0.y, x1.x, x1.y);
            vf1.u = make_uint4(x2.x, x2.y, x3.x, x3.y);
        };
        auto scores = [&](f32x16& s, const U4 (&kf)[KS], int t) __attribute__((always_inline)) {
            s = f32x16{0};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                s = E::mfma(kf[ks], qhi[t][ks], s);
                s = E::mfma(kf[ks], qlo[t][ks], s);
            }
        };
        // Hands stage st+1 over to the readers and refills the buffer of stage st-1 with stage st+2: every wave waits
        // for its own loads of stage st+1 (issued a stage ago) and meets the others; whoever arrives has read the last
        // of stage st-1.
        auto handover = [&](int st) __attribute__((always_inline)) {
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
            __syncthreads();
            if (st + 2 < nst) {
                dma_stage((st + 2) % NBUF);
                if (st + 3 < nst) fetch_rows(st + 3);
            }
        };

        // stages 0 and 1 have landed for every wave
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        __syncthreads();
        if (nst > 2) fetch_rows(2);

        // The loop runs one score tile ahead of the softmax. With one query tile per wave the score registers
        // alternate between sa and sb from one key tile to the next; with two, sa is query tile 0 and sb query tile 1
        // of the same key tile. K fragments are read from LDS a whole unit before the MFMAs that use them.
        f32x16 sa, sb;
        U4 kf1[KS], kf2[KS], vf0, vf1;
        const std::true_type yes;
        const std::false_type no;
        read_k(kf1, 0, 0);
        scores(sa, kf1, 0);
        if (QT == 1) read_k(kf1, 0, 1);    // a stage always holds four tiles of (clamped, finite) rows
        int bufi = 0;
        // A scope of whole stages (every scope of full buckets) runs its last stage through the same straight code:
        // the score tile computed "ahead" of the very last one reads a buffer that holds no stage and is never used.
        // The general version of the last stage decides per tile at run time whether there is a next one; the joins
        // of its paths cost more register moves than a tile's own arithmetic.
        const bool whole = (ng & (AKT - 1)) == 0;
        const int nfast = whole ? nst : nst - 1;
        for (int st = 0; st < nfast; ++st) {            // no tile is masked, every tile has a next one (see above for the last)
            const int bufn = bufi + 1 == NBUF ? 0 : bufi + 1;
            const uint32_t kb = bufi * L::KBUF, vb = bufi * L::VBUF, kbn = bufn * L::KBUF;
            const int k0 = st * AKT;
#pragma unroll
            for (int t4 = 0; t4 < 4; ++t4) {
                read_v(vf0, vf1, vb, t4);
                if (QT == 1) {
                    if (t4 < 2) read_k(kf2, kb, t4 + 2); else read_k(kf2, kbn, t4 - 2);
                    if ((t4 & 1) == 0) unit(sa, 0, k0 + 32 * t4, vf0, vf1, yes, sb, kf1, 0, no);
                    else unit(sb, 0, k0 + 32 * t4, vf0, vf1, yes, sa, kf1, 0, no);
                } else {
                    if (t4 < 3) read_k(kf2, kb, t4 + 1); else read_k(kf2, kbn, 0);
                    unit(sa, 0, k0 + 32 * t4, vf0, vf1, yes, sb, kf1, 1, no);
                    unit(sb, 1, k0 + 32 * t4, vf0, vf1, yes, sa, kf2, 0, no);
                }
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) kf1[ks] = kf2[ks];
                if (t4 == 1) handover(st);
            }
            bufi = bufn;
        }
        if (!whole) {                                   // the last stage: 1..4 tiles, the last one possibly ragged
            const uint32_t kb = bufi * L::KBUF, vb = bufi * L::VBUF;
            const int k0 = (nst - 1) * AKT;
            const int ntl = ntile - (nst - 1) * 4;
#pragma unroll
            for (int t4 = 0; t4 < 4; ++t4) {
                if (t4 >= ntl) break;
                const bool more = t4 + 1 < ntl;
                read_v(vf0, vf1, vb, t4);
                if (QT == 1) {
                    if (t4 < 2) read_k(kf2, kb, t4 + 2);
                    f32x16& s_cur = (t4 & 1) ? sb : sa;
                    f32x16& s_nxt = (t4 & 1) ? sa : sb;
                    if (more) unit(s_cur, 0, k0 + 32 * t4, vf0, vf1, yes, s_nxt, kf1, 0, no);
                    else unit(s_cur, 0, k0 + 32 * t4, vf0, vf1, no, s_nxt, kf1, 0, yes);
                } else {
                    if (t4 < 3) read_k(kf2, kb, t4 + 1);
                    if (more) {
                        unit(sa, 0, k0 + 32 * t4, vf0, vf1, yes, sb, kf1, 1, no);
                        unit(sb, 1, k0 + 32 * t4, vf0, vf1, yes, sa, kf2, 0, no);
                    } else {
                        unit(sa, 0, k0 + 32 * t4, vf0, vf1, yes, sb, kf1, 1, yes);
                        unit(sb, 1, k0 + 32 * t4, vf0, vf1, no, sa, kf2, 0, yes);
                    }
                }
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) kf1[ks] = kf2[ks];
            }
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

// Query rows per workgroup. Two query tiles per wave share every K/V fragment read, halve the staging and the
// per-workgroup set-up per FLOP, and let a wave alternate between two independent score tiles; they need more
// registers (fewer waves per SIMD), which the software-pipelined tile loop tolerates. One tile per wave only where a
// scope is too short for 256-row blocks or the launch too small to fill the GPU with them.
static int pick_qt(int head_dim, long long slots, int heads, int bucket_cap)
{
    (void)head_dim;
    if (bucket_cap < 256) return 1;
    const long long wgs_qt2 = slots * heads * ((bucket_cap + 255) / 256);
    return wgs_qt2 >= 512 ? 2 : 1;
}

int attn_block_rows(int head_dim, long long slots, int heads, int bucket_cap)
{
    return 128 * pick_qt(head_dim, slots, heads, bucket_cap);
}

template <bool F16>
static void launch_typed(const AttnArgs& a, int head_dim, int block_rows, unsigned total, hipStream_t stream)
{
    if (head_dim == 16) {
        if (block_rows == 256) k_attn<16, 2, F16><<<total, 256, 0, stream>>>(a);
        else k_attn<16, 1, F16><<<total, 256, 0, stream>>>(a);
    } else {
        if (block_rows == 256) k_attn<32, 2, F16><<<total, 256, 0, stream>>>(a);
        else k_attn<32, 1, F16><<<total, 256, 0, stream>>>(a);
    }
}

hipError_t attn_launch(const AttnArgs& a, int head_dim, int block_rows, hipStream_t stream)
{
    long long total = (long long)a.n_slots * a.H * a.qblocks;
    total = (total + 7) / 8 * 8;
    if (total == 0) return hipSuccess;
    if (a.f16) launch_typed<true>(a, head_dim, block_rows, (unsigned)total, stream);
    else launch_typed<false>(a, head_dim, block_rows, (unsigned)total, stream);
    return hipGetLastError();
}

}  // namespace f3d

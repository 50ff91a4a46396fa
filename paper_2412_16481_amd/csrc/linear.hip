// The point-wise glue of a transformer block around the attention (Section 4.2, block equations; Section 4.1 "Stage
// Orchestration": the bucket-major array "suits point-wise MLPs and LayerNorm"): LayerNorm + linear map in one pass,
// with the row gather that puts q, k, v into bucket-major order (so that the attention reads contiguous rows) and the
// row scatter + residual that brings a block's output back.
//
//   y[p] = LN(x[row_in[p]]) W^T + bias;   out[row_out[p]] = y[p] + residual[row_out[p]]
//
// One workgroup = 128 rows. The rows are normalised in place in LDS (two threads per row), rounded to bf16 and kept in
// LDS for the whole workgroup; the weight matrix (resident in L2) is read straight from memory, once per workgroup,
// as the A operand of v_mfma_f32_32x32x16_bf16 computing the TRANSPOSED product Y^T = W X^T, so that a lane
// owns one row of Y and, with the rows of W taken in a suitable order, 16 consecutive columns of it: 16-byte stores,
// no shuffles.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "linear.h"

namespace f3d {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;

union F8 {
    uint4 u;
    bf16x8 b;
};

__device__ __forceinline__ uint32_t pack2(float lo, float hi)
{
    f32x2 x = {lo, hi};
    bf16x2 y = __builtin_convertvector(x, bf16x2);
    return *reinterpret_cast<uint32_t*>(&y);
}
__device__ __forceinline__ float lo16(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float hi16(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

constexpr int LBM = 128;   // rows per workgroup
constexpr int LTH = 256;   // threads per workgroup
constexpr int TPR = LTH / LBM;   // threads per row in the LayerNorm

// dynamic LDS: X tile [LBM][CI + 8] bf16
template <int CI>
__global__ __launch_bounds__(LTH) void k_ln_linear(LinearArgs a)
{
    constexpr int PITCH = CI + 8;      // elements; the 16-byte pad staggers the banks of consecutive rows
    constexpr int KS = CI / 16;        // MFMA k-steps
    constexpr int CPT = CI / 8 / TPR;  // 16-byte pieces per thread in the LayerNorm (TPR threads per row)
    extern __shared__ __attribute__((aligned(16))) uint16_t sx[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hf = lane >> 5;
    const long long row0 = (long long)blockIdx.x * LBM;

    // ---- load the rows into LDS, then normalise them in place: thread (r, half) handles 1/TPR of row r. The three
    //      passes (sum; squared deviations; scale and shift) walk over the thread's own 16-byte pieces in LDS, so no
    //      pass keeps a row in registers.
    {
        const int r = tid / TPR, half = tid % TPR;
        const long long p = row0 + r;
        const bool ok = p < a.n;
        const size_t src = ok ? (size_t)(a.row_in ? a.row_in[p] : p) : 0;
        const uint4* xr = reinterpret_cast<const uint4*>(a.x + src * CI) + half * CPT;
        uint4* mine = reinterpret_cast<uint4*>(&sx[r * PITCH + half * (CI / TPR)]);
        float sum = 0.f;
#pragma unroll
        for (int c = 0; c < CPT; ++c) {
            const uint4 v = ok ? xr[c] : make_uint4(0, 0, 0, 0);
            mine[c] = v;
            sum += (lo16(v.x) + hi16(v.x)) + (lo16(v.y) + hi16(v.y)) + (lo16(v.z) + hi16(v.z)) + (lo16(v.w) + hi16(v.w));
        }
        if (a.gamma) {
            sum += __shfl_xor(sum, 1, 64);
            if (TPR == 4) sum += __shfl_xor(sum, 2, 64);
            const float mu = sum * (1.0f / CI);
            float sq = 0.f;
#pragma unroll 4
            for (int c = 0; c < CPT; ++c) {
                const uint4 v = mine[c];
                const uint32_t w4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float d0 = lo16(w4[e]) - mu, d1 = hi16(w4[e]) - mu;
                    sq += d0 * d0 + d1 * d1;
                }
            }
            sq += __shfl_xor(sq, 1, 64);
            if (TPR == 4) sq += __shfl_xor(sq, 2, 64);
            const float rstd = rsqrtf(sq * (1.0f / CI) + a.eps);
            const float4* g4 = reinterpret_cast<const float4*>(a.gamma) + half * CPT * 2;
            const float4* b4 = a.beta ? reinterpret_cast<const float4*>(a.beta) + half * CPT * 2 : nullptr;
#pragma unroll 2
            for (int c = 0; c < CPT; ++c) {
                const uint4 v = mine[c];
                const uint32_t w4[4] = {v.x, v.y, v.z, v.w};
                const float4 ga = g4[2 * c], gb = g4[2 * c + 1];
                const float4 ba = b4 ? b4[2 * c] : make_float4(0, 0, 0, 0), bb = b4 ? b4[2 * c + 1] : make_float4(0, 0, 0, 0);
                const float gg[8] = {ga.x, ga.y, ga.z, ga.w, gb.x, gb.y, gb.z, gb.w};
                const float bt[8] = {ba.x, ba.y, ba.z, ba.w, bb.x, bb.y, bb.z, bb.w};
                uint32_t o[4];
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    o[e] = pack2((lo16(w4[e]) - mu) * rstd * gg[2 * e] + bt[2 * e], (hi16(w4[e]) - mu) * rstd * gg[2 * e + 1] + bt[2 * e + 1]);
                mine[c] = make_uint4(o[0], o[1], o[2], o[3]);
            }
        }
    }
    __syncthreads();

    // ---- Y^T unit by unit. A unit is one 32-column block of the output for RB of the workgroup's four 32-row blocks
    //      (all four from 128 channels on, so that the workgroup reads every row of W exactly once, from L2, while the
    //      normalised rows are re-read from LDS; two at 64 channels, where there are too few column blocks to keep four
    //      waves busy otherwise). Wave w takes units w, w+4, ...
    //      Row i of the A operand is output column col0 + 16*((i>>2)&1) + 4*(i>>3) + (i&3): with this order the 16
    //      accumulator registers of a lane are 16 CONSECUTIVE columns of its row (two 16-byte stores), and the two
    //      half-waves of a row together write 64 contiguous bytes.
    constexpr int RB = CI == 64 ? 2 : 4;
    constexpr int UPC = 4 / RB;                              // units per column block
    const int per_out = a.c_out / a.n_outs;
    const int units = (a.c_out >> 5) * UPC;
    const int wcol = 16 * ((l32 >> 2) & 1) + 4 * (l32 >> 3) + (l32 & 3);
    for (int u = wave; u < units; u += LTH / 64) {
        const int col0 = (u / UPC) << 5, rb0 = (u % UPC) * RB;
        f32x16 acc[RB];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) acc[rb] = f32x16{0};
        const uint16_t* wr = a.w + (size_t)(col0 + wcol) * CI + 8 * hf;   // rows of W = output columns
        const uint16_t* xrow = &sx[(rb0 * 32 + l32) * PITCH + 8 * hf];
#pragma unroll 2
        for (int ks = 0; ks < KS; ++ks) {
            F8 wa;
            wa.u = *reinterpret_cast<const uint4*>(wr + 16 * ks);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                F8 xf;
                xf.u = *reinterpret_cast<const uint4*>(xrow + rb * 32 * PITCH + 16 * ks);
                acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa.b, xf.b, acc[rb], 0, 0, 0);
            }
        }
        const int col = col0 + 16 * hf;                      // first of this lane's 16 columns
        const int t = col / per_out, lc = col - t * per_out;
        float bs[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) bs[e] = 0.f;
        if (a.bias) {
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const float4 bv = *reinterpret_cast<const float4*>(a.bias + col + 4 * q4);
                bs[4 * q4] = bv.x; bs[4 * q4 + 1] = bv.y; bs[4 * q4 + 2] = bv.z; bs[4 * q4 + 3] = bv.w;
            }
        }
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const long long p = row0 + (rb0 + rb) * 32 + l32;    // this lane's row of Y
            if (p >= a.n) continue;
            const size_t drow = (size_t)(a.row_out ? a.row_out[p] : p);
            float y[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) y[e] = acc[rb][e] + bs[e];
            if (a.residual) {
                const uint4* rp = reinterpret_cast<const uint4*>(a.residual + drow * a.c_out + col);
#pragma unroll
                for (int h8 = 0; h8 < 2; ++h8) {
                    const uint4 rv = rp[h8];
                    const uint32_t w4[4] = {rv.x, rv.y, rv.z, rv.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        y[8 * h8 + 2 * e] += lo16(w4[e]);
                        y[8 * h8 + 2 * e + 1] += hi16(w4[e]);
                    }
                }
            }
            uint4* op = reinterpret_cast<uint4*>(a.outs[t] + drow * per_out + lc);
#pragma unroll
            for (int h8 = 0; h8 < 2; ++h8)
                op[h8] = make_uint4(pack2(y[8 * h8], y[8 * h8 + 1]), pack2(y[8 * h8 + 2], y[8 * h8 + 3]),
                                    pack2(y[8 * h8 + 4], y[8 * h8 + 5]), pack2(y[8 * h8 + 6], y[8 * h8 + 7]));
        }
    }
}

template <int CI>
hipError_t launch_ci(const LinearArgs& a, hipStream_t stream)
{
    const size_t lds = (size_t)LBM * (CI + 8) * 2;
    if (lds > 60000) {
        const hipError_t e = hipFuncSetAttribute((const void*)k_ln_linear<CI>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    const unsigned blocks = (unsigned)((a.n + LBM - 1) / LBM);
    if (blocks > 0) k_ln_linear<CI><<<blocks, LTH, lds, stream>>>(a);
    return hipGetLastError();
}

}  // namespace

hipError_t linear_launch(const LinearArgs& a, hipStream_t stream)
{
    switch (a.c_in) {
        case 64: return launch_ci<64>(a, stream);
        case 128: return launch_ci<128>(a, stream);
        case 256: return launch_ci<256>(a, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace f3d

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
// owns one row of Y and four consecutive columns per register group: 8-byte stores, no shuffles.
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

// dynamic LDS: X tile [LBM][CI + 8] bf16
template <int CI>
__global__ __launch_bounds__(256) void k_ln_linear(LinearArgs a)
{
    constexpr int PITCH = CI + 8;      // elements; the 16-byte pad staggers the banks of consecutive rows
    constexpr int KS = CI / 16;        // MFMA k-steps
    constexpr int CPT = CI / 16;       // 16-byte chunks per thread in the LayerNorm (two threads per row)
    extern __shared__ __attribute__((aligned(16))) uint16_t sx[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hf = lane >> 5;
    const long long row0 = (long long)blockIdx.x * LBM;

    // ---- load the rows into LDS, then normalise them in place: thread (r, half) handles half of row r. The three
    //      passes (sum; squared deviations; scale and shift) walk over the thread's own 16-byte pieces in LDS, so no
    //      pass keeps a row in registers.
    {
        const int r = tid >> 1, half = tid & 1;
        const long long p = row0 + r;
        const bool ok = p < a.n;
        const size_t src = ok ? (size_t)(a.row_in ? a.row_in[p] : p) : 0;
        const uint4* xr = reinterpret_cast<const uint4*>(a.x + src * CI) + half * CPT;
        uint4* mine = reinterpret_cast<uint4*>(&sx[r * PITCH + half * (CI / 2)]);
        float sum = 0.f;
#pragma unroll 4
        for (int c = 0; c < CPT; ++c) {
            const uint4 v = ok ? xr[c] : make_uint4(0, 0, 0, 0);
            mine[c] = v;
            sum += (lo16(v.x) + hi16(v.x)) + (lo16(v.y) + hi16(v.y)) + (lo16(v.z) + hi16(v.z)) + (lo16(v.w) + hi16(v.w));
        }
        if (a.gamma) {
            sum += __shfl_xor(sum, 1, 64);
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

    // ---- Y^T block by block: a wave takes every fourth 32-column block of the output and computes it for ALL 128 rows
    //      of the workgroup, so the workgroup reads every row of W exactly once (from L2) while the normalised rows
    //      are re-read from LDS.
    size_t drow[4];
    bool ok[4];
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) {
        const long long p = row0 + rb * 32 + l32;          // this lane's row of Y in row block rb
        ok[rb] = p < a.n;
        drow[rb] = ok[rb] ? (size_t)(a.row_out ? a.row_out[p] : p) : 0;
    }
    const int per_out = a.c_out / a.n_outs;
    const uint16_t* xrow = &sx[l32 * PITCH + 8 * hf];
    for (int col0 = 32 * wave; col0 < a.c_out; col0 += 128) {
        f32x16 acc[4];
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) acc[rb] = f32x16{0};
        const uint16_t* wr = a.w + (size_t)(col0 + l32) * CI + 8 * hf;   // rows of W = output columns
#pragma unroll 2
        for (int ks = 0; ks < KS; ++ks) {
            F8 wa;
            wa.u = *reinterpret_cast<const uint4*>(wr + 16 * ks);
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) {
                F8 xf;
                xf.u = *reinterpret_cast<const uint4*>(xrow + rb * 32 * PITCH + 16 * ks);
                acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa.b, xf.b, acc[rb], 0, 0, 0);
            }
        }
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) {
            if (!ok[rb]) continue;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int col = col0 + 8 * j + 4 * hf;        // four consecutive columns of this lane's row
                float y[4] = {acc[rb][4 * j], acc[rb][4 * j + 1], acc[rb][4 * j + 2], acc[rb][4 * j + 3]};
                if (a.bias) {
                    const float4 bv = *reinterpret_cast<const float4*>(a.bias + col);
                    y[0] += bv.x; y[1] += bv.y; y[2] += bv.z; y[3] += bv.w;
                }
                if (a.residual) {
                    const uint2 rv = *reinterpret_cast<const uint2*>(a.residual + drow[rb] * a.c_out + col);
                    y[0] += lo16(rv.x); y[1] += hi16(rv.x); y[2] += lo16(rv.y); y[3] += hi16(rv.y);
                }
                const int t = col / per_out, lc = col - t * per_out;
                uint2 pk;
                pk.x = pack2(y[0], y[1]);
                pk.y = pack2(y[2], y[3]);
                *reinterpret_cast<uint2*>(a.outs[t] + drow[rb] * per_out + lc) = pk;
            }
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
    if (blocks > 0) k_ln_linear<CI><<<blocks, 256, lds, stream>>>(a);
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

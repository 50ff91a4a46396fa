// The point-wise glue of a transformer block around the attention (Section 4.2, block equations; Section 4.1 "Stage
// Orchestration": the bucket-major array "suits point-wise MLPs and LayerNorm"): LayerNorm + linear map in one pass,
// with the row gather that puts q, k, v into bucket-major order (so that the attention reads contiguous rows) and the
// row scatter + residual that brings a block's output back.
//
//   y[p] = LN(x[row_in[p]]) W^T + bias;   out[row_out[p]] = y[p] + residual[row_out[p]]
//
// One workgroup = 4 waves = 128 rows; a wave owns 32 rows and keeps them in registers for the whole kernel, in the
// layout of the B operand of v_mfma_f32_32x32x16_bf16 (a lane holds half of one row), normalised there and rounded
// to bf16. The weight matrix (resident in L2) streams through LDS in double-buffered tiles of 16 KB, loaded with whole
// rows per wave (coalesced) once per workgroup, and is the A operand of the TRANSPOSED product Y^T = W X^T: a lane
// then owns one row of Y and, with the rows of W stored in a suitable order, 16 consecutive columns of it: 16-byte
// stores, no shuffles.
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

constexpr int LNW = 4;          // waves per workgroup; a wave owns 32 rows
constexpr int LTH = LNW * 64;
constexpr int LBM = LNW * 32;   // rows per workgroup

// W tiles in LDS: 32 * TCB output columns x CI inputs, TCB chosen so that a tile is 1024 16-byte pieces (16 KB) and a
// wave runs 16 MFMAs per tile and barrier whatever the width.
template <int CI>
struct Tile {
    static constexpr int TCB = 256 / CI;            // 32-column blocks per tile
    static constexpr int TROWS = 32 * TCB;          // rows of W (output columns) per tile
    static constexpr int PITCH = CI + 8;            // elements; the 16-byte pad staggers the banks of consecutive rows
    static constexpr size_t LDS_BYTES = (size_t)2 * TROWS * PITCH * 2;
};

template <int CI>
__global__ __launch_bounds__(LTH, 3) void k_ln_linear(LinearArgs a)
{
    constexpr int KS = CI / 16;                     // MFMA k-steps
    constexpr int TCB = Tile<CI>::TCB, TROWS = Tile<CI>::TROWS, PITCH = Tile<CI>::PITCH;
    constexpr int CPR = CI / 8;                     // 16-byte pieces per row of W
    constexpr int PPT = TROWS * CPR / LTH;          // pieces per thread and tile (4)
    static_assert(TROWS * CPR % LTH == 0, "a W tile is a whole number of pieces per thread");
    extern __shared__ __attribute__((aligned(16))) uint16_t sw[];   // [2][TROWS][PITCH], then binary32 bias [c_out], scale [CI], shift [CI]
    float* sbias = reinterpret_cast<float*>(sw + 2 * TROWS * PITCH);   // [c_out], zeros without a bias
    float* sgamma = sbias + a.c_out;                                  // [CI] LayerNorm scale
    float* sbeta = sgamma + CI;                                       // [CI] LayerNorm shift, zeros without one
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hf = lane >> 5;
    const long long p = (long long)blockIdx.x * LBM + wave * 32 + l32;   // this lane's row of Y
    const bool ok = p < a.n;
    const int n_cb = a.c_out >> 5;                  // 32-column blocks of the output
    const int n_tiles = (n_cb + TCB - 1) / TCB;

    // ---- staging of W tiles: global -> registers (coalesced: whole rows of W) -> LDS. Row j of a 32-row block is
    //      stored at slot 8*((j>>2)&3) + 4*(j>>4) + (j&3), so that MFMA row i holds output column
    //      16*((i>>2)&1) + 4*(i>>3) + (i&3) of the block: with this order the 16 accumulator registers of a lane are 16
    //      CONSECUTIVE columns of its row (two 16-byte stores; the two half-waves of a row write 64 contiguous bytes).
    struct WTile { uint4 v[PPT]; } wreg;   // handled by value: a lambda that captures an array by reference can put it in scratch
    const auto load_tile = [=](int t) __attribute__((always_inline)) -> WTile {
        WTile r;
#pragma unroll
        for (int i = 0; i < PPT; ++i) {
            const int q = tid + i * LTH;
            const int j = q / CPR, c = q % CPR;
            const int col = min(t * TROWS + j, a.c_out - 1);   // past the last column: some valid row, never used
            r.v[i] = *reinterpret_cast<const uint4*>(a.w + (size_t)col * CI + 8 * c);
        }
        return r;
    };
    const auto store_tile = [=](int buf, const WTile r) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < PPT; ++i) {
            const int q = tid + i * LTH;
            const int j = q / CPR, c = q % CPR;
            const int jr = j & 31;
            const int slot = (j & ~31) + 8 * ((jr >> 2) & 3) + 4 * (jr >> 4) + (jr & 3);
            *reinterpret_cast<uint4*>(&sw[(size_t)buf * TROWS * PITCH + slot * PITCH + 8 * c]) = r.v[i];
        }
    };
    // Everything the prologue reads from memory is requested before anything waits: the row index (the row loads depend
    // on it), the first W tile, the per-column vectors, then the rows themselves.
    const size_t src = ok ? (size_t)(a.row_in ? a.row_in[p] : p) : 0;
    wreg = load_tile(0);
    // the output tensors' addresses are kept in LDS: indexing the argument block inside the loop is a dependent load
    // from memory per tile, in front of the tile's stores
    __shared__ uint16_t* s_outs[LIN_MAX_OUTS];
    if (tid == 0) {
        s_outs[0] = a.outs[0];
        s_outs[1] = a.outs[1];
        s_outs[2] = a.outs[2];
        s_outs[3] = a.outs[3];
    }
    // The per-column vectors are read by every wave (the bias for every tile): they are kept in LDS, off the vector
    // memory path, so that neither the LayerNorm nor an epilogue waits for a trip to memory. Loads in batches of four
    // without per-element predicates (an index past the end re-reads the last element and is not written).
    float gv = 0.f, bev = 0.f;
    if (a.gamma) {
        gv = a.gamma[min(tid, CI - 1)];
        if (a.beta) bev = a.beta[min(tid, CI - 1)];
    }
    if (a.bias) {
        for (int i0 = tid; i0 < a.c_out; i0 += 4 * LTH) {
            float v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = a.bias[min(i0 + u * LTH, a.c_out - 1)];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (i0 + u * LTH < a.c_out) sbias[i0 + u * LTH] = v[u];
        }
    } else {
        for (int i = tid; i < a.c_out; i += LTH) sbias[i] = 0.f;
    }

    // ---- this lane's part of its row: elements 16*ks + 8*hf .. +7 for every k-step, i.e. the B operand of the MFMAs.
    //      The row stays in registers for the whole kernel.
    F8 xf[KS];
    {
        const uint16_t* xr = a.x + src * CI + 8 * hf;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) xf[ks].u = *reinterpret_cast<const uint4*>(xr + 16 * ks);   // rows past the end read row 0 and are never stored
    }
    if (a.gamma && tid < CI) {
        sgamma[tid] = gv;
        sbeta[tid] = bev;
    }
    __syncthreads();   // the vectors are in LDS (the row loads stay in flight across the barrier)
    if (a.gamma) {   // LayerNorm: the two half-waves hold the two halves of a row
        // Between the three passes the packed words are made opaque, so that each pass unpacks them again instead of
        // keeping the whole row alive as binary32 values.
        const auto opaque = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(xf[ks].u.x), "+v"(xf[ks].u.y), "+v"(xf[ks].u.z), "+v"(xf[ks].u.w));
        };
        float sum = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const uint32_t w4[4] = {xf[ks].u.x, xf[ks].u.y, xf[ks].u.z, xf[ks].u.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) sum += lo16(w4[e]) + hi16(w4[e]);
        }
        sum += __shfl_xor(sum, 32, 64);
        const float mu = sum * (1.0f / CI);
        opaque();
        float sq = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const uint32_t w4[4] = {xf[ks].u.x, xf[ks].u.y, xf[ks].u.z, xf[ks].u.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float d0 = lo16(w4[e]) - mu, d1 = hi16(w4[e]) - mu;
                sq += d0 * d0 + d1 * d1;
            }
        }
        sq += __shfl_xor(sq, 32, 64);
        const float rstd = rsqrtf(sq * (1.0f / CI) + a.eps);
        opaque();
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const float4* g4 = reinterpret_cast<const float4*>(sgamma + 16 * ks + 8 * hf);
            const float4 ga = g4[0], gb = g4[1];
            const float4* b4 = reinterpret_cast<const float4*>(sbeta + 16 * ks + 8 * hf);
            const float4 ba = b4[0], bb = b4[1];
            const float gg[8] = {ga.x, ga.y, ga.z, ga.w, gb.x, gb.y, gb.z, gb.w};
            const float bt[8] = {ba.x, ba.y, ba.z, ba.w, bb.x, bb.y, bb.z, bb.w};
            const uint32_t w4[4] = {xf[ks].u.x, xf[ks].u.y, xf[ks].u.z, xf[ks].u.w};
            uint32_t o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e)
                o[e] = pack2((lo16(w4[e]) - mu) * rstd * gg[2 * e] + bt[2 * e], (hi16(w4[e]) - mu) * rstd * gg[2 * e + 1] + bt[2 * e + 1]);
            xf[ks].u = make_uint4(o[0], o[1], o[2], o[3]);
            if ((ks & 1) == 1) asm volatile("" ::: "memory");   // at most two k-steps of scale/shift reads in flight
        }
    }
    store_tile(0, wreg);
    __syncthreads();

    // ---- Y^T = W X^T tile by tile: the A operand (32 rows of W) comes from LDS, the B operand is the wave's rows
    const size_t drow = ok ? (size_t)(a.row_out ? a.row_out[p] : p) : 0;
    const int per_out = a.c_out / a.n_outs;

    for (int t = 0; t < n_tiles; ++t) {
        const int buf = t & 1;
        if (t + 1 < n_tiles) wreg = load_tile(t + 1);
        const uint16_t* wt = &sw[(size_t)buf * TROWS * PITCH + l32 * PITCH + 8 * hf];
        // The next tile goes to LDS in the middle of this iteration: behind enough MFMAs to cover the latency of its
        // loads, and in front of the stores of the epilogues that follow (the memory counter retires in order, so a
        // wait placed behind those stores would also wait for them). The other buffer is free: every wave passed the
        // barrier at the end of the last iteration, after its last read of it.
        bool staged = t + 1 >= n_tiles;
#pragma unroll
        for (int cb = 0; cb < TCB; ++cb) {
            const int col0 = (t * TCB + cb) << 5;
            if (col0 >= a.c_out) break;
            f32x16 acc = {0};
            // what the epilogue needs from LDS is requested before the MFMAs, not behind them
            const int col = col0 + 16 * hf;                      // first of this lane's 16 columns
            const int to = col / per_out, lc = col - to * per_out;
            uint16_t* const ob = s_outs[to];
            float4 bv[4];
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) bv[q4] = *reinterpret_cast<const float4*>(sbias + col + 4 * q4);
            uint4 rv[2] = {make_uint4(0, 0, 0, 0), make_uint4(0, 0, 0, 0)};   // the residual's 16 columns (bf16 zeros without one)
            if (a.residual) {
                const uint4* rp = reinterpret_cast<const uint4*>(a.residual + drow * a.c_out + col);   // drow is a valid row also past the end
                rv[0] = rp[0];
                rv[1] = rp[1];
            }
            // W fragments four k-steps at a time, one group ahead of the MFMAs that use them
            constexpr int G = 4, NG = KS / G;
            F8 wf[2][G];
#pragma unroll
            for (int i = 0; i < G; ++i) wf[0][i].u = *reinterpret_cast<const uint4*>(wt + cb * 32 * PITCH + 16 * i);
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                if (g + 1 < NG) {
#pragma unroll
                    for (int i = 0; i < G; ++i)
                        wf[(g + 1) & 1][i].u = *reinterpret_cast<const uint4*>(wt + cb * 32 * PITCH + 16 * ((g + 1) * G + i));
                }
#pragma unroll
                for (int i = 0; i < G; ++i) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[g & 1][i].b, xf[g * G + i].b, acc, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (cb == TCB / 2 && !staged) {
                store_tile(buf ^ 1, wreg);
                staged = true;
            }
            if (ok) {
                float y[16];
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    y[4 * q4] = acc[4 * q4] + bv[q4].x;
                    y[4 * q4 + 1] = acc[4 * q4 + 1] + bv[q4].y;
                    y[4 * q4 + 2] = acc[4 * q4 + 2] + bv[q4].z;
                    y[4 * q4 + 3] = acc[4 * q4 + 3] + bv[q4].w;
                }
#pragma unroll
                for (int h8 = 0; h8 < 2; ++h8) {
                    const uint32_t w4[4] = {rv[h8].x, rv[h8].y, rv[h8].z, rv[h8].w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        y[8 * h8 + 2 * e] += lo16(w4[e]);
                        y[8 * h8 + 2 * e + 1] += hi16(w4[e]);
                    }
                }
                uint4* op = reinterpret_cast<uint4*>(ob + drow * per_out + lc);
#pragma unroll
                for (int h8 = 0; h8 < 2; ++h8)
                    op[h8] = make_uint4(pack2(y[8 * h8], y[8 * h8 + 1]), pack2(y[8 * h8 + 2], y[8 * h8 + 3]),
                                        pack2(y[8 * h8 + 4], y[8 * h8 + 5]), pack2(y[8 * h8 + 6], y[8 * h8 + 7]));
            }
        }
        if (!staged) store_tile(buf ^ 1, wreg);   // a last, partial tile ended before the staging point
        __syncthreads();
    }
}

template <int CI>
hipError_t launch_ci(const LinearArgs& a, hipStream_t stream)
{
    const unsigned blocks = (unsigned)((a.n + LBM - 1) / LBM);
    const size_t lds = Tile<CI>::LDS_BYTES + (size_t)a.c_out * 4 + (size_t)2 * CI * 4;
    if (lds > 60000) {
        const hipError_t e = hipFuncSetAttribute((const void*)k_ln_linear<CI>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
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

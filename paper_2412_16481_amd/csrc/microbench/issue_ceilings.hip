// Measured ceilings behind the attention kernel's roofline discussion: what the matrix core and the vector
// ALU of this GPU sustain on the kernel's own instruction mix, with no memory traffic at all.
//   kind 0: MFMA only        back-to-back v_mfma_f32_32x32x16_bf16, two accumulators per wave
//   kind 1: softmax only     per 32x32 score tile and wave: 16 v_exp_f32 + 8 v_cvt_pk_bf16_f32
//   kind 2: tile loop        the head_dim-16 tile of Bucket-Swin attention (Section 4.2) in registers: two MFMAs
//                            for the scaled scores (bf16 head + remainder of q), 16 exponentials, 8 packs, two
//                            MFMAs for P V
//   kind 3: pipelined tile, head_dim 32   the tile loop as the attention kernel issues it: the four score MFMAs of
//                            the NEXT tile between groups of four exponentials of the current one, then packs,
//                            8 dot2 (softmax denominator) and the two P V MFMAs; order pinned by scheduling barriers
//   kind 4: pipelined tile, head_dim 16   the same with two score MFMAs and no dot2
//   kind 5: vector part only of kind 3 (16 exp, 8 packs, 8 dot2)
//   kind 6: six accumulating MFMAs per tile on three independent accumulators, nothing else
//   kind 7: kinds 5 and 6 in one loop, with no data dependence between the vector and the matrix work: what the two
//           units cost each other when nothing but issue and register ports couple them
// Operands hold random bits: the clock this GPU sustains depends on the data. Built into its own library
// (libf3d_microbench.so); bench.py --ceilings runs it. Not part of the product path.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

union Frag {
    uint32_t u[4];
    bf16x8 b;
};

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    f32x2 x = {lo, hi};
    bf16x2 y = __builtin_convertvector(x, bf16x2);
    return *reinterpret_cast<uint32_t*>(&y);
}

constexpr int ITER = 4096;   // tiles (kinds 1..7) or groups of four MFMAs (kind 0) per wave
#define MB_SB() __builtin_amdgcn_sched_barrier(0)

__device__ __forceinline__ float sum2(uint32_t pair, float c)
{
    const uint32_t ones = 0x3F803F80u;
    return __builtin_amdgcn_fdot2_f32_bf16(*reinterpret_cast<const bf16x2*>(&pair), *reinterpret_cast<const bf16x2*>(&ones), c, false);
}

template <int KIND>
__global__ __launch_bounds__(256) void k_ceiling(const uint32_t* __restrict__ seed, float* __restrict__ sink, float mul)
{
    const int lane = threadIdx.x & 63;
    Frag K, Q, Q2, V0, V1;
    for (int i = 0; i < 4; ++i) {   // bf16 pairs with exponents near 1: finite results, random mantissas and signs
        const uint32_t r = seed[(threadIdx.x * 4 + i) & 4095];
        K.u[i] = (r & 0x807F807Fu) | 0x3F003F00u;
        Q.u[i] = ((r >> 3) & 0x807F807Fu) | 0x3E803E80u;
        Q2.u[i] = ((r >> 5) & 0x807F807Fu) | 0x3A803A80u;
        V0.u[i] = ((r >> 7) & 0x807F807Fu) | 0x3F003F00u;
        V1.u[i] = ((r >> 9) & 0x807F807Fu) | 0x3F003F00u;
    }
    f32x16 o = {0}, o2 = {0};
    float t = 0.f;
    if (KIND == 0) {
        for (int it = 0; it < ITER; ++it) {
            o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(K.b, Q.b, o, 0, 0, 0);
            o2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(V0.b, Q2.b, o2, 0, 0, 0);
            o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(V1.b, Q.b, o, 0, 0, 0);
            o2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(K.b, Q2.b, o2, 0, 0, 0);
        }
    } else if (KIND == 1) {
        f32x16 s;
        for (int i = 0; i < 16; ++i) s[i] = (float)(lane + i) * mul;
        for (int it = 0; it < ITER; ++it) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] = __builtin_amdgcn_exp2f(s[r]);
            Frag p0, p1;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                p0.u[e] = pack_bf16(s[2 * e], s[2 * e + 1]);
                p1.u[e] = pack_bf16(s[8 + 2 * e], s[9 + 2 * e]);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {   // feed the packed values back so that nothing is dead; costs no instruction
                s[2 * e] = __uint_as_float(p0.u[e] & 0x3FFF0000u);
                s[8 + 2 * e] = __uint_as_float(p1.u[e] & 0x3FFF0000u);
            }
        }
        for (int i = 0; i < 16; ++i) t += s[i];
    } else if (KIND == 3 || KIND == 4) {
        constexpr bool D32 = KIND == 3;
        f32x16 sa = {0}, sb = {0};
        float l2 = 0.f;
        sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(K.b, Q.b, sa, 0, 0, 0);
        auto unit = [&](f32x16& s, f32x16& sn, int it) __attribute__((always_inline)) {
            K.u[0] ^= (uint32_t)it & 0x00010001u;
            MB_SB();
#pragma unroll
            for (int r = 0; r < 4; ++r) s[r] = __builtin_amdgcn_exp2f(s[r]);
            MB_SB();
            sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(K.b, Q.b, f32x16{0}, 0, 0, 0);
            MB_SB();
#pragma unroll
            for (int r = 4; r < 8; ++r) s[r] = __builtin_amdgcn_exp2f(s[r]);
            MB_SB();
            if (D32) sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(K.b, Q2.b, sn, 0, 0, 0);
            MB_SB();
#pragma unroll
            for (int r = 8; r < 12; ++r) s[r] = __builtin_amdgcn_exp2f(s[r]);
            MB_SB();
            sn = D32 ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(V0.b, Q.b, sn, 0, 0, 0) : __builtin_amdgcn_mfma_f32_32x32x16_bf16(K.b, Q2.b, sn, 0, 0, 0);
            MB_SB();
#pragma unroll
            for (int r = 12; r < 16; ++r) s[r] = __builtin_amdgcn_exp2f(s[r]);
            MB_SB();
            if (D32) sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(V0.b, Q2.b, sn, 0, 0, 0);
            MB_SB();
            Frag p0, p1;
#pragma unroll
            for (int e = 0; e < 4; ++e) p0.u[e] = pack_bf16(s[2 * e], s[2 * e + 1]);
            if (D32) {
#pragma unroll
                for (int e = 0; e < 4; ++e) { if (e & 1) l2 = sum2(p0.u[e], l2); else t = sum2(p0.u[e], t); }
            }
            MB_SB();
            o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(V0.b, p0.b, o, 0, 0, 0);
            MB_SB();
#pragma unroll
            for (int e = 0; e < 4; ++e) p1.u[e] = pack_bf16(s[8 + 2 * e], s[9 + 2 * e]);
            if (D32) {
#pragma unroll
                for (int e = 0; e < 4; ++e) { if (e & 1) l2 = sum2(p1.u[e], l2); else t = sum2(p1.u[e], t); }
            }
            MB_SB();
            o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(V1.b, p1.b, o, 0, 0, 0);
            MB_SB();
        };
        for (int it = 0; it < ITER; it += 2) { unit(sa, sb, it); unit(sb, sa, it + 1); }
        for (int i = 0; i < 16; ++i) t += sa[i] + sb[i];
        t += l2;
    } else if (KIND >= 5) {
        // the vector stream and the matrix stream share no register: only issue slots and register ports couple them
        f32x16 s, c1 = {0}, c2 = {0};
        float l2 = 0.f;
        for (int i = 0; i < 16; ++i) s[i] = (float)(lane + i) * mul;
        for (int it = 0; it < ITER; ++it) {
            K.u[0] ^= (uint32_t)it & 0x00010001u;
#pragma unroll
            for (int n = 0; n < 6; ++n) {
                MB_SB();
                if (KIND != 6) {
                    if (n < 4) {
#pragma unroll
                        for (int r = 0; r < 4; ++r) s[4 * n + r] = __builtin_amdgcn_exp2f(s[4 * n + r]);
                    } else {
                        Frag p;
#pragma unroll
                        for (int e = 0; e < 4; ++e) p.u[e] = pack_bf16(s[8 * (n - 4) + 2 * e], s[8 * (n - 4) + 2 * e + 1]);
#pragma unroll
                        for (int e = 0; e < 4; ++e) { if (e & 1) l2 = sum2(p.u[e], l2); else t = sum2(p.u[e], t); }
#pragma unroll
                        for (int e = 0; e < 4; ++e) s[8 * (n - 4) + 2 * e] = __uint_as_float(p.u[e] & 0x3FFF0000u);   // nothing dead, nothing grows
                    }
                }
                MB_SB();
                if (KIND != 5) {
                    if (n % 3 == 0) o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(K.b, Q.b, o, 0, 0, 0);
                    else if (n % 3 == 1) c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(V0.b, Q2.b, c1, 0, 0, 0);
                    else c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(V1.b, Q.b, c2, 0, 0, 0);
                }
                MB_SB();
            }
        }
        for (int i = 0; i < 16; ++i) t += s[i] + c1[i] + c2[i];
        t += l2;
    } else {
        for (int it = 0; it < ITER; ++it) {
            K.u[0] ^= (uint32_t)it & 0x00010001u;
            f32x16 s = {0};
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(K.b, Q.b, s, 0, 0, 0);
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(K.b, Q2.b, s, 0, 0, 0);
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] = __builtin_amdgcn_exp2f(s[r]);
            Frag p0, p1;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                p0.u[e] = pack_bf16(s[2 * e], s[2 * e + 1]);
                p1.u[e] = pack_bf16(s[8 + 2 * e], s[9 + 2 * e]);
            }
            o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(V0.b, p0.b, o, 0, 0, 0);
            o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(V1.b, p1.b, o, 0, 0, 0);
        }
    }
    for (int i = 0; i < 16; ++i) t += o[i] + o2[i];
    sink[blockIdx.x * 256 + threadIdx.x] = t;
}

}  // namespace

// Runs one kind with `waves_per_simd` (1..8) waves on every SIMD of the current device and writes the duration of
// one launch in milliseconds and the work it did (MFMA FLOP for kind 0, score elements = 1024 per tile for the others).
// Returns 0, or a hipError_t value. Allocates and frees its own small buffers; not for use inside a timed region.
extern "C" int f3d_mb_run(int kind, int waves_per_simd, float* ms_out, double* work_out)
{
    if (kind < 0 || kind > 7 || waves_per_simd < 1 || waves_per_simd > 8 || !ms_out || !work_out) return (int)hipErrorInvalidValue;
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return (int)e;
    const int blocks = cus * waves_per_simd;   // 256 threads = one wave per SIMD of a CU
    uint32_t* seed = nullptr;
    float* sink = nullptr;
    uint32_t host[4096];
    uint32_t x = 2463534242u;
    for (int i = 0; i < 4096; ++i) { x ^= x << 13; x ^= x >> 17; x ^= x << 5; host[i] = x; }
    e = hipMalloc(&seed, sizeof(host));
    if (e == hipSuccess) e = hipMalloc(&sink, (size_t)blocks * 256 * sizeof(float));
    if (e == hipSuccess) e = hipMemcpy(seed, host, sizeof(host), hipMemcpyHostToDevice);
    hipEvent_t a = nullptr, b = nullptr;
    if (e == hipSuccess) e = hipEventCreate(&a);
    if (e == hipSuccess) e = hipEventCreate(&b);
    if (e == hipSuccess) {
        for (int rep = 0; rep < 2 && e == hipSuccess; ++rep) {   // the first launch warms up
            e = hipEventRecord(a, nullptr);
            switch (kind) {
                case 0: k_ceiling<0><<<blocks, 256>>>(seed, sink, 0.001f); break;
                case 1: k_ceiling<1><<<blocks, 256>>>(seed, sink, 0.001f); break;
                case 2: k_ceiling<2><<<blocks, 256>>>(seed, sink, 0.001f); break;
                case 3: k_ceiling<3><<<blocks, 256>>>(seed, sink, 0.001f); break;
                case 4: k_ceiling<4><<<blocks, 256>>>(seed, sink, 0.001f); break;
                case 5: k_ceiling<5><<<blocks, 256>>>(seed, sink, 0.001f); break;
                case 6: k_ceiling<6><<<blocks, 256>>>(seed, sink, 0.001f); break;
                default: k_ceiling<7><<<blocks, 256>>>(seed, sink, 0.001f); break;
            }
            if (e == hipSuccess) e = hipEventRecord(b, nullptr);
            if (e == hipSuccess) e = hipEventSynchronize(b);
        }
        if (e == hipSuccess) e = hipEventElapsedTime(ms_out, a, b);
    }
    const double waves = (double)blocks * 4;
    *work_out = kind == 0 ? waves * ITER * 4 * 32768.0 : waves * ITER * 1024.0;
    if (a) (void)hipEventDestroy(a);
    if (b) (void)hipEventDestroy(b);
    if (seed) (void)hipFree(seed);
    if (sink) (void)hipFree(sink);
    return (int)e;
}

// In-bucket pooling (Section 4.2 "In-bucket Pooling"; Appendix "In-bucket Pooling") for gfx950.
//
// The bucket-major array is cut into tiles of up to 1024 consecutive rows of one scan; one workgroup of
// 1024 threads (a thread per row) builds the tile's M = ceil(n / rho) sub-buckets entirely in LDS, in the
// Appendix's three steps (initial sub-buckets from a hash of the voxel coordinate, new sub-buckets for the
// points beyond capacity until the block counter reaches M, rounds in which the points still left join the
// nearest sub-bucket with room), then reduces the feature rows of every sub-bucket and writes the pooled rows
// of the tile as one contiguous piece.
//
// The Appendix decides who comes first with block-level atomics. Here every such decision is taken in row
// order (stable ranks from wave ballots plus per-wave counters, as in the bucketing kernels), so the result
// is a function of the input alone.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pool.h"
#include "psh_common.h"


namespace f3d {

// The squared distances that decide the nearest sub-bucket are three binary32 products and two binary32 sums, each
// rounded on its own; a fused multiply-add would round differently and can pick another sub-bucket on a near tie.
// The compiler contracts a*b + c of ordinary expressions (also through the __fmul_rn / __fadd_rn helpers, which are
// plain operators), so the products are issued as instructions it cannot look into.
__device__ __forceinline__ float mul_own_rounding(float x, float y)
{
    float r;
    asm("v_mul_f32_e32 %0, %1, %2" : "=v"(r) : "v"(x), "v"(y));
    return r;
}
__device__ __forceinline__ float dist2(float dx, float dy, float dz)
{
    return (mul_own_rounding(dx, dx) + mul_own_rounding(dy, dy)) + mul_own_rounding(dz, dz);
}

namespace {

constexpr int PT = POOL_MAX_TILE;   // threads per workgroup = most rows of a tile
constexpr int PW = PT / 64;

typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    f32x2 x = {lo, hi};
    bf16x2 y = __builtin_convertvector(x, bf16x2);  // round to nearest even
    return *reinterpret_cast<uint32_t*>(&y);
}

__device__ __forceinline__ int pool_batch_off(const PoolArgs& a, int b)
{
    if (a.batch_offsets) return a.batch_offsets[b];
    return b == 0 ? 0 : a.n;
}

// ------------------------------------------------------------------------------------------------
// tile table and pooled-row offsets of every scan (one workgroup)
__global__ __launch_bounds__(1024) void k_pool_meta(PoolArgs a)
{
    __shared__ int lds[17];
    __shared__ int bad;
    const int tid = threadIdx.x;
    if (tid == 0) {
        bad = 0;
        *a.tile_counter = 0;
    }
    __syncthreads();
    const int per_full = (a.tile + a.rho - 1) / a.rho;   // pooled rows of a full tile
    int tcarry = 0, ocarry = 0;
    for (int base = 0; base < a.n_scans; base += 1024) {
        const int b = base + tid;
        int tiles = 0, rows = 0, p0 = 0, nb = 0;
        if (b < a.n_scans) {
            p0 = pool_batch_off(a, b);
            const int p1 = pool_batch_off(a, b + 1);
            nb = p1 - p0;
            bool ok = nb >= 0 && p0 >= 0 && p1 <= a.n;
            if (b == 0 && p0 != 0) ok = false;
            if (b == a.n_scans - 1 && p1 != a.n) ok = false;
            if (!ok) { bad = 1; nb = 0; }
            if (nb > 0) {
                tiles = (nb + a.tile - 1) / a.tile;
                const int last = nb - (tiles - 1) * a.tile;
                rows = (tiles - 1) * per_full + (last + a.rho - 1) / a.rho;
            }
        }
        int ttot, otot;
        const int tpre = block_excl_scan(tiles, &ttot, lds);
        const int opre = block_excl_scan(rows, &otot, lds);
        if (b < a.n_scans) {
            a.pooled_offsets[b] = ocarry + opre;
            for (int t = 0; t < tiles && tcarry + tpre + t < a.n_tiles_ub; ++t) {   // scans are spread over the threads
                const int r0 = p0 + t * a.tile;
                a.tile_info[tcarry + tpre + t] = make_int4(r0, min(a.tile, p0 + nb - r0), ocarry + opre + t * per_full, b);
            }
        }
        tcarry += ttot;
        ocarry += otot;
    }
    __syncthreads();
    const int isbad = bad;
    if (tid == 0) a.pooled_offsets[a.n_scans] = isbad ? -1 : ocarry;
    // with inconsistent offsets no tile is processed at all
    for (int t = (isbad ? 0 : min(tcarry, a.n_tiles_ub)) + tid; t < a.n_tiles_ub; t += 1024) a.tile_info[t] = make_int4(0, 0, 0, -1);
}

// ------------------------------------------------------------------------------------------------
// Rank of every active thread among the active threads of the workgroup that hold the same key, in thread
// order. wcnt [PW][kp] is scratch; when ktot is given, ktot[k] = number of active threads with key k, k < nkeys.
__device__ __forceinline__ int block_rank_by_key(int key, bool active, int keybits, int nkeys, uint16_t* wcnt, int kp,
                                                 uint16_t* ktot)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int w = tid; w < PW * kp / 2; w += PT) reinterpret_cast<uint32_t*>(wcnt)[w] = 0u;
    __syncthreads();
    const unsigned long long m = match_key(key, active, keybits);
    const int before = __popcll(m & ((1ull << lane) - 1ull));
    if (active && before == 0) wcnt[wave * kp + key] = (uint16_t)__popcll(m);
    __syncthreads();
    for (int k = tid; k < nkeys; k += PT) {   // exclusive prefix over the waves
        int run = 0;
#pragma unroll
        for (int w = 0; w < PW; ++w) {
            const int c = wcnt[w * kp + k];
            wcnt[w * kp + k] = (uint16_t)run;
            run += c;
        }
        if (ktot) ktot[k] = (uint16_t)run;
    }
    __syncthreads();
    return active ? (int)wcnt[wave * kp + key] + before : 0;
}

// hash setting of a tile: M sub-buckets, voxel box vmax (automatic divisor as for the main hash, Section 4.1)
__device__ inline void tile_hash_cfg(int hash, int M, const int* vmax, ScanCfg& c)
{
    const int K = max(M, 1);
    c.K = K;
    int vm = 0;
    for (int ax = 0; ax < 3; ++ax) {
        c.vmax[ax] = vmax[ax];
        vm = max(vm, vmax[ax]);
    }
    const int nbits = max(1, bit_width64((unsigned long long)vm));
    c.invK = 1.0 / (double)K;
    unsigned long long D = 1;
    if (hash == 1) D = udiv63_small((1ull << nbits) - 1, K, c.invK) + 1;
    if (hash == 3) D = udiv63_small(morton3(vmax[0], vmax[1], vmax[2]), K, c.invK) + 1;
    c.D = D;
    c.invD = 1.0 / (double)D;
    c.invDf = (float)c.invD;
    c.wide = vm >= 2048;
    c.m32 = umod52(4294967296ull, K, c.invK);
    c.step = 1;
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// ------------------------------------------------------------------------------------------------
// The value of the lane whose number differs in bit log2(D), from data-parallel-primitive moves (inside a row of 16
// lanes) and the lane-swap instructions (between rows and between halves): vector instructions only, where a shuffle
// through the LDS crossbar would make the LDS pipeline the bottleneck of the sort below.
template <int CTRL, int BANKS>
__device__ __forceinline__ unsigned int dpp_mov(unsigned int old, unsigned int x)
{
    return (unsigned int)__builtin_amdgcn_update_dpp((int)old, (int)x, CTRL, 0xF, BANKS, false);
}
template <int D>
__device__ __forceinline__ unsigned int lane_xor(unsigned int x, int lane)
{
    // every lane is written, so the moves that cover all banks need no previous value (and no copy to provide one)
    if (D == 1) return (unsigned int)__builtin_amdgcn_mov_dpp((int)x, 0xB1, 0xF, 0xF, false);    // quad_perm [1,0,3,2]
    if (D == 2) return (unsigned int)__builtin_amdgcn_mov_dpp((int)x, 0x4E, 0xF, 0xF, false);    // quad_perm [2,3,0,1]
    if (D == 4)   // row_ror 12 for lanes 0-3 and 8-11 of a row, row_ror 4 for the others
        return dpp_mov<0x124, 0xA>((unsigned int)__builtin_amdgcn_mov_dpp((int)x, 0x12C, 0xF, 0xF, false), x);
    if (D == 8) return (unsigned int)__builtin_amdgcn_mov_dpp((int)x, 0x128, 0xF, 0xF, false);   // row_ror 8
    if (D == 16) {
        const auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
        return (lane & 16) ? r[0] : r[1];
    }
    const auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
    return (lane & 32) ? r[0] : r[1];
}

// Bitonic sort of 64 * NPL distinct 64-bit keys held by one wave, NPL per lane (element lane * NPL + r), ascending.
// Strides below NPL stay inside a lane; larger ones exchange with the lane at distance stride / NPL. K is the length
// of the runs being merged, J the stride of the step.
template <int NPL, int K, int J>
__device__ __forceinline__ void sort_step(unsigned long long (&key)[NPL], int lane)
{
    // direction of the run of K elements this element is in; the last phase sorts everything upwards
    const bool lane_up = K >= 64 * NPL ? true : (lane & (K / NPL)) == 0;
    if constexpr (J >= NPL) {
        constexpr int LJ = J / NPL;
        const bool keep_min = ((lane & LJ) == 0) == lane_up;
#pragma unroll
        for (int r = 0; r < NPL; ++r) {
            const unsigned long long mine = key[r];
            const unsigned int olo = lane_xor<LJ>((unsigned int)mine, lane);
            const unsigned int ohi = lane_xor<LJ>((unsigned int)(mine >> 32), lane);
            const unsigned long long other = ((unsigned long long)ohi << 32) | olo;
            key[r] = ((mine < other) == keep_min) ? mine : other;
        }
    } else {
#pragma unroll
        for (int r = 0; r < NPL; ++r) {
            if (r & J) continue;
            const bool up = K < NPL ? (r & K) == 0 : lane_up;
            const unsigned long long x = key[r], y = key[r | J];
            const bool swap = (x > y) == up;
            key[r] = swap ? y : x;
            key[r | J] = swap ? x : y;
        }
    }
    if constexpr (J > 1) sort_step<NPL, K, J / 2>(key, lane);
}
template <int NPL, int K = 2>
__device__ __forceinline__ void wave_sort_keys(unsigned long long (&key)[NPL], int lane)
{
    sort_step<NPL, K, K / 2>(key, lane);
    if constexpr (K < 64 * NPL) wave_sort_keys<NPL, K * 2>(key, lane);
}

// The same network on 32-bit keys, at less than half the instructions: a step is a minimum and a maximum. Runs that
// are to end up descending are sorted ascending on complemented keys instead (the lanes of such a run flip their keys
// when the phase begins), so no step depends on a direction except through the constant choice of the lower lane.
template <int NPL, int K, int J>
__device__ __forceinline__ void sort32_step(unsigned int (&key)[NPL], int lane)
{
    if constexpr (J >= NPL) {
        constexpr int LJ = J / NPL;
        const bool lower = (lane & LJ) == 0;
#pragma unroll
        for (int r = 0; r < NPL; ++r) {
            const unsigned int other = lane_xor<LJ>(key[r], lane);
            const unsigned int lo = min(key[r], other), hi = max(key[r], other);
            key[r] = lower ? lo : hi;
        }
    } else {
#pragma unroll
        for (int r = 0; r < NPL; ++r) {
            if (r & J) continue;
            const bool up = K < NPL ? (r & K) == 0 : true;
            const unsigned int lo = min(key[r], key[r | J]), hi = max(key[r], key[r | J]);
            key[r] = up ? lo : hi;
            key[r | J] = up ? hi : lo;
        }
    }
    if constexpr (J > 1) sort32_step<NPL, K, J / 2>(key, lane);
}
template <int NPL, int K = 2>
__device__ __forceinline__ void wave_sort32(unsigned int (&key)[NPL], int lane)
{
    if constexpr (K >= NPL) {
        const bool up_now = K >= 64 * NPL ? true : (lane & (K / NPL)) == 0;
        const bool up_before = K / 2 >= NPL ? (lane & (K / 2 / NPL)) == 0 : true;
        const unsigned int flip = up_now != up_before ? 0xFFFFFFFFu : 0u;
#pragma unroll
        for (int r = 0; r < NPL; ++r) key[r] ^= flip;
    }
    sort32_step<NPL, K, K / 2>(key, lane);
    if constexpr (K < 64 * NPL) wave_sort32<NPL, K * 2>(key, lane);
}

// Odd-even transposition sweeps over the wave's 64 * NPL keys (element lane * NPL + r) until a sweep swaps nothing;
// false when `sweeps` sweeps did not suffice. For sequences that are sorted except inside short runs.
template <int NPL>
__device__ __forceinline__ bool settle_order(unsigned long long (&key)[NPL], int lane, int sweeps)
{
    for (int s = 0; s < sweeps; ++s) {
        bool moved = false;
#pragma unroll
        for (int r0 = 0; r0 < 2; ++r0) {
#pragma unroll
            for (int r = r0; r + 1 < NPL; r += 2) {
                const unsigned long long x = key[r], y = key[r + 1];
                const bool swap = x > y;
                key[r] = swap ? y : x;
                key[r + 1] = swap ? x : y;
                moved |= swap;
            }
        }
        // the pair that straddles two lanes: this lane's last key and the next lane's first
        const unsigned long long last = key[NPL - 1], first = key[0];
        const unsigned long long next_first =
            ((unsigned long long)(unsigned int)__shfl_down((int)(unsigned int)(first >> 32), 1, 64) << 32) | (unsigned int)__shfl_down((int)(unsigned int)first, 1, 64);
        const unsigned long long prev_last =
            ((unsigned long long)(unsigned int)__shfl_up((int)(unsigned int)(last >> 32), 1, 64) << 32) | (unsigned int)__shfl_up((int)(unsigned int)last, 1, 64);
        const bool give = lane < 63 && last > next_first, take = lane > 0 && prev_last > first;
        if (give) key[NPL - 1] = next_first;
        if (take) key[0] = prev_last;
        moved |= give | take;
        if (__builtin_amdgcn_ballot_w64(moved) == 0ull) return true;
    }
    return false;
}

// One wave writes, for each of the rows left it is given (every PW-th), the ids of the open sub-buckets in the
// order in which the row would choose them: increasing squared distance to the sub-bucket's first row, the lower id
// first on a tie, i.e. increasing (bits of the distance, position in the open list): a squared distance is a
// non-negative binary32 number, whose bit patterns are ordered like the numbers. The sort runs on 32-bit keys (the
// upper 23 bits of the distance's pattern, 9 bits of position: at most 512 sub-buckets are open when rows are
// left); that orders all candidates except those whose distances agree in the bits kept, which the full 64-bit keys
// then settle among neighbours (if that takes long, the full keys are sorted outright). `list` rows have `pitch`
// entries (a multiple of 8, >= nopen).
template <int NPL>
__device__ __forceinline__ void sort_choices(int nleft, int nopen, int pitch, const uint16_t* left_list, const float* px,
                                             const float* py, const float* pz, const float4* o4, const uint16_t* open_list,
                                             uint16_t* list)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int p = wave; p < nleft; p += PW) {
        const int id = left_list[p];
        const float qx = px[id], qy = py[id], qz = pz[id];
        unsigned int k32[NPL];
#pragma unroll
        for (int r = 0; r < NPL; ++r) {   // the candidates' positions are read again for every row: registers are scarce
            const int e = lane * NPL + r;
            const float4 o = o4[min(e, nopen - 1)];
            const float d2 = dist2(qx - o.x, qy - o.y, qz - o.z);
            k32[r] = e < nopen ? ((__float_as_uint(d2) >> 8) << 9) | (unsigned int)e : 0xFFFFFFFFu;
        }
        wave_sort32<NPL>(k32, lane);
        unsigned long long key[NPL];
#pragma unroll
        for (int r = 0; r < NPL; ++r) {   // the full key of the candidate now at this place
            const int e = min((int)(k32[r] & 511u), nopen - 1);
            const float4 o = o4[e];
            const float d2 = dist2(qx - o.x, qy - o.y, qz - o.z);
            key[r] = k32[r] != 0xFFFFFFFFu ? ((unsigned long long)__float_as_uint(d2) << 32) | (unsigned int)e : ~0ull;
        }
        if (!settle_order<NPL>(key, lane, 16)) wave_sort_keys<NPL>(key, lane);
        unsigned int sid[NPL];   // padding entries (beyond nopen) become id 0: never chosen, but a valid index
#pragma unroll
        for (int r = 0; r < NPL; ++r) sid[r] = key[r] == ~0ull ? 0u : (unsigned int)open_list[(unsigned int)key[r] & 511u];
        if (lane * NPL < pitch) {
            uint16_t* dst = list + (size_t)p * pitch + lane * NPL;
            if (NPL == 8) {
                *reinterpret_cast<uint4*>(dst) = make_uint4(sid[0] | (sid[1] << 16), sid[2] | (sid[3] << 16), sid[4] | (sid[5] << 16), sid[6] | (sid[7] << 16));
            } else if (NPL == 4) {
                *reinterpret_cast<uint2*>(dst) = make_uint2(sid[0] | (sid[1] << 16), sid[2] | (sid[3] << 16));
            } else {
                *reinterpret_cast<unsigned int*>(dst) = sid[0] | (sid[1] << 16);
            }
        }
    }
}

// Workgroup barrier for steps that exchange data through LDS only: waits for this wave's LDS operations, not for
// its global loads (__syncthreads() waits for both; in the rounds below the read of a row's next list chunk may still
// be in flight at the barrier, and is waited for where the chunk is used).
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// entry `i` (0..7) of a chunk of eight 16-bit ids
__device__ __forceinline__ int chunk_entry(const uint4& c, int i)
{
    // selects and a shift: indexing the four words by a variable would put the chunk into scratch memory
    const unsigned long long lo = ((unsigned long long)c.y << 32) | c.x, hi = ((unsigned long long)c.w << 32) | c.z;
    const unsigned long long half = (i & 4) ? hi : lo;
    return (int)((half >> ((i & 3) << 4)) & 0xFFFFull);
}

// The passes of one round, by all threads of the workgroup: thread `tid` speaks for a row that contends for
// sub-bucket c (or for none). The lowest contender of every sub-bucket joins; with room for more than one the
// others try again, in row order, while there is room. win [2][kp] holds the lowest contender per sub-bucket,
// alternating by pass (par); a winner clears its entry, which is next written two barriers later. Returns whether
// this thread's row joined; its sub-bucket and slot are then in rsub / rslot [tid]. `probe`, when given, is a word of
// LDS read right after the first barrier (with the other reads of that moment) into *probed.
__device__ __forceinline__ bool join_passes(bool contend, int c, int tid, int rho, int kp, int* win, int* fill, uint16_t* rsub,
                                            uint16_t* rslot, int* rows_left, int* more, int& par, bool sent = false,
                                            const int* probe = nullptr, int* probed = nullptr)
{
    bool joined = false;
    for (;;) {
        if (contend && !sent) atomicMin(&win[par * kp + c], tid);   // sent: the caller has done this for the first pass
        sent = false;
        lds_barrier();
        // the fill level is read beside the winner, not after it: one LDS round trip instead of two
        const int w = contend ? win[par * kp + c] : -1;
        const int f = contend ? fill[c] : 0;
        if (probe) {
            *probed = *probe;
            probe = nullptr;
        }
        asm volatile("" ::"v"(f));
        if (contend && w == tid) {
            rsub[tid] = (uint16_t)c;
            rslot[tid] = (uint16_t)f;
            fill[c] = f + 1;
            joined = true;
            contend = false;
            atomicSub(rows_left, 1);
            win[par * kp + c] = 0x7FFFFFFF;
        }
        if (tid == 0) more[par ^ 1] = 0;
        lds_barrier();
        if (rho <= 2) {   // a sub-bucket holds a row, so it has room for one at most
            par ^= 1;
            break;
        }
        contend = contend && fill[c] < rho;
        if (contend) more[par] = 1;
        lds_barrier();
        const int again = more[par];
        par ^= 1;
        if (!again) break;
    }
    return joined;
}

// dynamic LDS, kp = a.kp: px,py,pz [PT] floats | o4 [kp] float4 (x, y, z, -) | fill [kp] ints | win [2][kp] ints |
// open_list, id_of_hash, first_idx, ktot [kp] u16 each | members [PT + POOL_MAX_RHO] u16 | rsub, rslot [PT] u16 |
// wcnt [PW][kp] u16 (at least PT entries: later the choices of a searched round)
//
// Workgroups are persistent: each takes tiles from a counter until none is left, and owns one slot of the
// choice-list area in global memory (its block index).
// WPE = waves per SIMD the kernel is compiled for: 4 (128 registers, one workgroup per compute unit) or 8 (64
// registers, a little spilling in the sort, two workgroups per compute unit). A tile's rounds leave the vector ALU
// idle most of the time and its sort saturates it: with two workgroups resident, one's rounds run beside the other's
// sort. With no more tiles than compute units there is nothing to put beside, and the form without spills is taken.
template <int WPE>
__global__ __launch_bounds__(PT, WPE) void k_pool(PoolArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __shared__ int lds[17];
    __shared__ uint32_t red[8];
    __shared__ ScanCfg cfg;
    __shared__ int next_tile;
    __shared__ int rows_left;
    __shared__ int more[2];
    __shared__ int any[2];
    __shared__ int any3[3];
    const int rho = a.rho, kp = a.kp;
    const int tid = threadIdx.x, lane = tid & 63;
    float* px = reinterpret_cast<float*>(smem);
    float* py = px + PT;
    float* pz = py + PT;
    float4* o4 = reinterpret_cast<float4*>(pz + PT);   // first-row position of every open sub-bucket: one 16-byte read
    int* fill = reinterpret_cast<int*>(o4 + kp);
    int* win = fill + kp;                               // [2][kp] lowest contender of a sub-bucket, by parity of the pass
    uint16_t* open_list = reinterpret_cast<uint16_t*>(win + 2 * kp);
    uint16_t* id_of_hash = open_list + kp;
    uint16_t* first_idx = id_of_hash + kp;
    uint16_t* ktot = first_idx + kp;
    uint16_t* members = ktot + kp;
    uint16_t* rsub = members + PT + POOL_MAX_RHO;    // [PT] sub-bucket the t-th row left joined, and its slot there
    uint16_t* rslot = rsub + PT;
    uint16_t* wcnt = rslot + PT;                        // per-wave counters of the ranking by key (initial sub-buckets only)
    uint16_t* const my_lists = a.lists + (size_t)blockIdx.x * a.list_cap;

  for (;;) {
    __syncthreads();   // the tile before is done with LDS and with next_tile
    if (tid == 0) next_tile = atomicAdd(a.tile_counter, 1);
    __syncthreads();
    const int tile_id = next_tile;
    if (tile_id >= a.n_tiles_ub) break;
    const int4 ti = a.tile_info[tile_id];
    const int n = ti.y;
    if (n <= 0) continue;
    const int row0 = ti.x, out0 = ti.z;
    const int M = (n + rho - 1) / rho;

    // ---- the tile's points, its minimum, voxel coordinates, voxel box
    const bool act = tid < n;
    float x = 0.f, y = 0.f, z = 0.f;
    if (act) {
        const size_t src = a.perm ? (size_t)a.perm[row0 + tid] : (size_t)(row0 + tid);
        x = a.coords[3 * src];
        y = a.coords[3 * src + 1];
        z = a.coords[3 * src + 2];
        px[tid] = x;
        py[tid] = y;
        pz[tid] = z;
    }
    if (tid < 3) { red[tid] = 0xFFFFFFFFu; red[4 + tid] = 0u; }
    for (int k = tid; k < kp; k += PT) {
        fill[k] = 0;
        first_idx[k] = 0;
        win[k] = 0x7FFFFFFF;
        win[kp + k] = 0x7FFFFFFF;
    }
    if (tid == 0) { more[0] = 0; more[1] = 0; any[0] = 0; any[1] = 0; any3[0] = 0; any3[1] = 0; any3[2] = 0; }
    __syncthreads();
    {
        uint32_t o[3] = {act ? f2ord(x) : 0xFFFFFFFFu, act ? f2ord(y) : 0xFFFFFFFFu, act ? f2ord(z) : 0xFFFFFFFFu};
#pragma unroll
        for (int ax = 0; ax < 3; ++ax) {
            uint32_t lo = o[ax];
            for (int d = 32; d >= 1; d >>= 1) lo = min(lo, (uint32_t)__shfl_xor((int)lo, d, 64));
            if (lane == 0) atomicMin(&red[ax], lo);
        }
    }
    __syncthreads();
    const float mnx = ord2f(red[0]), mny = ord2f(red[1]), mnz = ord2f(red[2]);
    int vx = 0, vy = 0, vz = 0;
    if (act) {
        vx = voxel_of(x, mnx, a.inv_voxel);
        vy = voxel_of(y, mny, a.inv_voxel);
        vz = voxel_of(z, mnz, a.inv_voxel);
    }
    {
        int v[3] = {vx, vy, vz};
#pragma unroll
        for (int ax = 0; ax < 3; ++ax) {
            int hi = v[ax];
            for (int d = 32; d >= 1; d >>= 1) hi = max(hi, __shfl_xor(hi, d, 64));
            if (lane == 0) atomicMax(&red[4 + ax], (uint32_t)hi);
        }
    }
    __syncthreads();
    if (tid == 0) {
        const int vmax[3] = {(int)red[4], (int)red[5], (int)red[6]};
        tile_hash_cfg(a.hash, M, vmax, cfg);
    }
    __syncthreads();
    const int h = act ? hash_bucket(a.hash, vx, vy, vz, cfg) : 0;
    const int keybits = max(1, 32 - __clz(max(M - 1, 1)));

    // ---- initial sub-buckets: occupied hash values get ids in the order of their first row; a sub-bucket keeps
    //      its first rho rows
    const int r = block_rank_by_key(h, act, keybits, M, wcnt, kp, ktot);
    const bool is_first = act && r == 0;
    int A;
    const int id = block_excl_scan(is_first ? 1 : 0, &A, lds);
    if (is_first) {
        id_of_hash[h] = (uint16_t)id;
        first_idx[id] = (uint16_t)tid;
        fill[id] = min((int)ktot[h], rho);
    }
    __syncthreads();
    int sub = -1, slot = 0;
    if (act && r < rho) {
        sub = id_of_hash[h];
        slot = r;
    }
    // ---- new sub-buckets: the rows beyond capacity, in row order, open one each until the counter reaches M
    const bool overflow = act && sub < 0;
    int nov;
    const int orank = block_excl_scan(overflow ? 1 : 0, &nov, lds);
    if (overflow && A + orank < M) {
        sub = A + orank;
        slot = 0;
        fill[sub] = 1;
        first_idx[sub] = (uint16_t)tid;
    }
    // ---- rounds: every row still left picks the open sub-bucket whose first row is nearest (state at the start of
    //      the round); the contenders of a sub-bucket join in row order while it has room.
    //      The first rounds search: every row left scans the open sub-buckets. That pays while a round places many
    //      rows (isolated rows find a sub-bucket of their own at once). What remains are the rows of dense clusters,
    //      which share their nearest sub-buckets and get one of them per round. For them the search is taken out
    //      of the rounds: a sub-bucket never reopens and its first row never changes, so the choices of a row over
    //      all rounds are one fixed sequence: the sub-buckets open now, by (distance, id), of which the row takes
    //      the first that still has room. The sequences are written once (a wave sorts one row's candidates at a
    //      time); a round is then a step along them.
    uint16_t* left_list = members;   // [PT] thread ids of the rows still left, in row order (members is filled last)
    uint16_t* pick = wcnt;   // [PT] choices of a searched round (the counters of the ranking are free by then)
    bool left = act && sub < 0;
    int lpos = 0, nleft = 0, nopen = 0, par = 0;
    for (int searched = 0, joined_last = 0, nleft_before = 0;; ++searched) {
        // one scan builds both lists: the rows still left (low half) and the sub-buckets with room (high half)
        __syncthreads();   // the fill levels written by the steps above / the last round are in place
        {
            const bool open = tid < M && fill[tid] < rho;
            int tot;
            const int pre = block_excl_scan((left ? 1 : 0) | (open ? 0x10000 : 0), &tot, lds);
            lpos = pre & 0xFFFF;
            nleft = tot & 0xFFFF;
            nopen = tot >> 16;
            if (left) left_list[lpos] = (uint16_t)tid;
            if (open) {
                const int f = first_idx[tid], opos = pre >> 16;
                open_list[opos] = (uint16_t)tid;
                o4[opos] = make_float4(px[f], py[f], pz[f], 0.f);
            }
            if (tid == 0) rows_left = nleft;
            rsub[tid] = (uint16_t)0xFFFF;
            __syncthreads();
        }
        // a searched round costs about nleft * nopen / 6 vector instructions, a sorted list about 2000 per row
        if (nleft == 0 || nopen == 0 || (searched > 0 && (searched >= 8 || joined_last * 16 < nleft_before))) break;
        // the rows left are spread over all threads: g neighbouring lanes share one row's search
        int g = 1;
        while (g < 64 && nleft * g * 2 <= PT) g *= 2;
        const int p = tid / g, part = tid - p * g;
        float bd = __builtin_inff();
        int bi = 0x7FFFFFFF;
        if (p < nleft) {
            const int id = left_list[p];
            const float qx = px[id], qy = py[id], qz = pz[id];
            // Lane `part` of the row's g lanes takes a contiguous range of the open list, in ascending order: the first
            // candidate unconditionally, a later one only if strictly nearer (a tie keeps the lower sub-bucket id). Four
            // candidates per trip, their reads issued together.
            const int chunk = (nopen + g - 1) / g;
            int c = part * chunk;
            const int cend = min(c + chunk, nopen);
            if (c < cend) {
                const float4 o = o4[c];
                bd = dist2(qx - o.x, qy - o.y, qz - o.z);
                bi = c;
                ++c;
                for (; c + 3 < cend; c += 4) {
                    float4 v4[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) v4[u] = o4[c + u];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const float d2 = dist2(qx - v4[u].x, qy - v4[u].y, qz - v4[u].z);
                        if (d2 < bd) { bd = d2; bi = c + u; }
                    }
                }
                for (; c < cend; ++c) {
                    const float4 v = o4[c];
                    const float d2 = dist2(qx - v.x, qy - v.y, qz - v.z);
                    if (d2 < bd) { bd = d2; bi = c; }
                }
            }
        }
        for (int d = g >> 1; d >= 1; d >>= 1) {   // smallest distance, the lower list position on a tie
            const float od = __shfl_xor(bd, d, 64);
            const int oi = __shfl_xor(bi, d, 64);
            if (oi != 0x7FFFFFFF && (bi == 0x7FFFFFFF || od < bd || (od == bd && oi < bi))) { bd = od; bi = oi; }
        }
        if (p < nleft && part == 0) pick[p] = open_list[min(bi, nopen - 1)];
        __syncthreads();
        // thread t now speaks for the t-th row left: row order is kept
        join_passes(tid < nleft, tid < nleft ? (int)pick[tid] : 0, tid, rho, kp, win, fill, rsub, rslot, &rows_left, more, par);
        if (left && rsub[lpos] != 0xFFFF) {
            sub = rsub[lpos];
            slot = rslot[lpos];
            left = false;
        }
        joined_last = nleft - rows_left;
        nleft_before = nleft;
    }
    const int pitch = (nopen + 7) & ~7;
    if (nleft > 0 && nopen > 0 && (long long)nleft * pitch <= (long long)a.list_cap) {
        if (nopen <= 128)
            sort_choices<2>(nleft, nopen, pitch, left_list, px, py, pz, o4, open_list, my_lists);
        else if (nopen <= 256)
            sort_choices<4>(nleft, nopen, pitch, left_list, px, py, pz, o4, open_list, my_lists);
        else
            sort_choices<8>(nleft, nopen, pitch, left_list, px, py, pz, o4, open_list, my_lists);
        __threadfence_block();   // the lists are read by other waves of this workgroup
        __syncthreads();
        // Thread t now speaks for the t-th row left: row order is kept. It walks its list in chunks of eight entries
        // (16 bytes), the chunk in use in registers. The lists were written by this compute unit a moment ago and
        // come back from its caches; a ring of the next chunks in LDS, refilled by global->LDS loads a round ahead,
        // measured no faster than reading a chunk when it is entered: the rounds are bound by the number of
        // instructions a wave issues per round, not by this latency.
        bool walking = tid < nleft;
        const uint4* mine = reinterpret_cast<const uint4*>(my_lists + (size_t)tid * pitch);
        uint4 cur = make_uint4(0, 0, 0, 0);
        if (walking) cur = mine[0];
        // With rho = 2 an open sub-bucket holds one row and has room for one: whoever contends for it knows that it
        // is closed after this round, without waiting for the winner. The contenders themselves mark it (with the
        // round's number, so that a search of the same round still sees it open), and a round needs one barrier
        // instead of two. stamp[c]: very negative while open, minus the round in which it closed, 1 if it was full
        // before the rounds; open in round t means stamp[c] < 1 - t. For other rho the fill level decides (< rho).
        const bool two = rho == 2;
        int* stamp = reinterpret_cast<int*>(o4);   // the candidates' positions are not needed after the sort
        if (two) {
            for (int k = tid; k < M; k += PT) stamp[k] = fill[k] < 2 ? (int)0x80000000 : 1;
            __syncthreads();
        }
        const int* level_of = two ? stamp : fill;
        int idx = 0, c = 0, rpar = 0, r3 = 0;
        for (int round = 0; round <= PT + 1; ++round) {   // every round places at least one row; the bound is a safeguard
            bool contend = false;
            const int thr = two ? 1 - round : rho;
            if (tid == 0) {
                if (two) any3[r3 == 2 ? 0 : r3 + 1] = 0; else any[rpar ^ 1] = 0;
            }
            if (walking) {
                for (;;) {   // the first sub-bucket of the sequence that still has room
                    if (idx >= nopen) break;
                    // all eight entries of the chunk are looked up together (their reads overlap, no branch per entry)
                    const unsigned int w[4] = {cur.x, cur.y, cur.z, cur.w};
                    unsigned int room = 0;
                    int level[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const unsigned int eo = (j & 1) ? (w[j >> 1] >> 14) & ~3u : (w[j >> 1] << 2) & 0x3FFFCu;   // 4 * id
                        level[j] = *reinterpret_cast<const int*>(reinterpret_cast<const char*>(level_of) + eo);
                    }
                    __builtin_amdgcn_sched_barrier(0);   // all eight reads are under way before the first is waited for
#pragma unroll
                    for (int j = 0; j < 8; ++j) room |= (level[j] < thr ? 1u : 0u) << j;
                    const int base = idx & ~7, lim = nopen - base;   // entries before idx are behind, those from nopen on are padding
                    room &= 0xFFu << (idx & 7);
                    if (lim < 8) room &= (1u << lim) - 1u;
                    if (room) {
                        const int j = __builtin_ctz(room);
                        idx = base + j;
                        c = chunk_entry(cur, j);
                        contend = true;
                        break;
                    }
                    idx = base + 8;
                    if (idx < nopen) cur = mine[idx >> 3];
                }
            }
            int seen = 0;   // did any row contend in this round? (the same answer for every thread)
            if (two) {
                if (contend) {
                    atomicMin(&win[par * kp + c], tid);
                    stamp[c] = -round;
                    any3[r3] = 1;
                }
                lds_barrier();
                const int w = contend ? win[par * kp + c] : -1;
                seen = any3[r3];
                if (contend && w == tid) {
                    rsub[tid] = (uint16_t)c;
                    rslot[tid] = (uint16_t)1;
                    walking = false;
                    win[par * kp + c] = 0x7FFFFFFF;   // next written two rounds from here, a barrier in between
                }
                par ^= 1;
                r3 = r3 == 2 ? 0 : r3 + 1;
            } else {
                if (contend) {   // first step of the passes
                    atomicMin(&win[par * kp + c], tid);
                    any[rpar] = 1;
                }
                if (join_passes(contend, c, tid, rho, kp, win, fill, rsub, rslot, &rows_left, more, par, true, &any[rpar], &seen)) walking = false;
                rpar ^= 1;
            }
            if (!seen) break;
        }
        __syncthreads();
        if (two) {   // the sub-buckets closed in the rounds are full
            for (int k = tid; k < M; k += PT)
                if (stamp[k] != (int)0x80000000 && stamp[k] <= 0) fill[k] = 2;
        }
        if (left && rsub[lpos] != 0xFFFF) {
            sub = rsub[lpos];
            slot = rslot[lpos];
        }
    }

    // ---- members of every sub-bucket by slot, the map row -> pooled row
    if (act && sub >= 0) {
        members[sub * rho + slot] = (uint16_t)tid;
        if (a.sub_of) a.sub_of[row0 + tid] = out0 + sub;
    }
    __syncthreads();
    // ---- reduce: one (sub-bucket, 16-byte column) per thread and pass; rows are added in slot order
    const int NCH = a.C >> 3;
    const uint4* feat = reinterpret_cast<const uint4*>(a.feat);
    uint4* outp = reinterpret_cast<uint4*>(a.pooled_feat);
    const int op = a.op;
    for (int idx = tid; idx < M * NCH; idx += PT) {
        const int s = idx / NCH, ch = idx - s * NCH;
        const int cnt = fill[s];
        float acc[8];
        for (int sl = 0; sl < cnt; ++sl) {
            const int rr = min((int)members[s * rho + sl], n - 1);
            const uint4 v = feat[(size_t)(row0 + rr) * NCH + ch];
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float lo = bf16_lo(w[e]), hi = bf16_hi(w[e]);
                if (sl == 0) {
                    acc[2 * e] = lo;
                    acc[2 * e + 1] = hi;
                } else if (op <= 1) {
                    acc[2 * e] += lo;
                    acc[2 * e + 1] += hi;
                } else if (op == 2) {
                    acc[2 * e] = fminf(acc[2 * e], lo);
                    acc[2 * e + 1] = fminf(acc[2 * e + 1], hi);
                } else {
                    acc[2 * e] = fmaxf(acc[2 * e], lo);
                    acc[2 * e + 1] = fmaxf(acc[2 * e + 1], hi);
                }
            }
        }
        if (op == 1) {
            const float c = (float)cnt;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = acc[e] / c;
        }
        uint4 o;
        o.x = pack_bf16(acc[0], acc[1]);
        o.y = pack_bf16(acc[2], acc[3]);
        o.z = pack_bf16(acc[4], acc[5]);
        o.w = pack_bf16(acc[6], acc[7]);
        outp[(size_t)(out0 + s) * NCH + ch] = o;
    }
    // ---- pooled position: mean of the members' coordinates
    if (a.pooled_coords && tid < M) {
        const int cnt = fill[tid];
        float sx = 0.f, sy = 0.f, sz = 0.f;
        for (int sl = 0; sl < cnt; ++sl) {
            const int rr = min((int)members[tid * rho + sl], n - 1);
            sx += px[rr];
            sy += py[rr];
            sz += pz[rr];
        }
        const float c = (float)cnt;
        float* dst = a.pooled_coords + (size_t)(out0 + tid) * 3;
        dst[0] = sx / c;
        dst[1] = sy / c;
        dst[2] = sz / c;
    }
  }   // next tile
}

size_t pool_lds_bytes(int kp)
{
    const size_t wcnt = (size_t)PW * kp * 2;   // kp >= 64, so this is at least PT entries
    return (size_t)3 * PT * 4 + (size_t)4 * kp * 4 + (size_t)3 * kp * 4 + (size_t)4 * kp * 2 + (size_t)(PT + POOL_MAX_RHO) * 2 +
           (size_t)2 * PT * 2 + wcnt;
}

}  // namespace

hipError_t pool_launch(const PoolArgs& a, hipStream_t stream)
{
    k_pool_meta<<<1, 1024, 0, stream>>>(a);
    if (a.n == 0) return hipGetLastError();
    const size_t lds = pool_lds_bytes(a.kp);
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) cus = 0;
    const bool two = cus > 0 && a.n_tiles_ub > cus && 2 * lds <= 160 * 1024;
    if (lds > 60000) {
        const hipError_t e = two ? hipFuncSetAttribute((const void*)k_pool<8>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)
                                 : hipFuncSetAttribute((const void*)k_pool<4>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    if (two) {
        const int grid = a.n_slots < 2 * cus ? a.n_slots : 2 * cus;
        k_pool<8><<<grid, PT, lds, stream>>>(a);
    } else {
        const int grid = cus > 0 && a.n_slots > cus ? cus : a.n_slots;
        k_pool<4><<<grid, PT, lds, stream>>>(a);
    }
    return hipGetLastError();
}

}  // namespace f3d

// PSH bucketing, batch path: ONE workgroup per scan runs all of Algorithms 1 and 2 for its scan in a single launch.
//
// Same schedule and same results as psh.hip and psh_fast.hip (lock step, contenders served by input index). Those
// two spread a scan over many workgroups and need a grid-wide boundary per step; with many scans in a batch the
// scans themselves are the parallel work, and a workgroup that walks its scan in index order knows the rank of a
// contender the moment it sees it (contenders so far + rank inside the 2048 points at hand), so a point is accepted
// or passed on immediately: no count matrix, no launch boundary per step, and the points still unplaced are kept
// as a compacted list (index, packed voxel) that shrinks from step to step, so later steps read only what is left.
//
// Per iteration of 2048 list entries (two per thread): ranks inside a wave from ballots over the key bits, per-wave
// counters packed two per LDS word, an exclusive prefix over the waves per bucket, then accept / pass on. Two
// workgroup barriers per iteration; the list entries that are passed on are written one iteration late, after the
// barrier that makes every wave's count visible.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "psh_common.h"

namespace f3d {

namespace {

constexpr int STH = 1024;          // threads per workgroup
constexpr int SNW = STH / 64;      // waves
constexpr int SPPT = 2;            // list entries per thread and iteration
constexpr int SIT = STH * SPPT;    // list entries per iteration
constexpr int SKMAX = 1024;        // most buckets per scan on this path (LDS: 76 bytes per bucket)

__device__ __forceinline__ unsigned long long pack_voxel(int x, int y, int z)
{
    return (unsigned long long)(uint32_t)x | ((unsigned long long)(uint32_t)y << 21) | ((unsigned long long)(uint32_t)z << 42);
}

// dynamic LDS, in 32-bit words: fill[K] run[2][K] wh[SNW][kw] wbase[SNW][kw] with kw = (K + 1) / 2.
// The hash function is a template parameter: the kernel holds many scan-wide values in scalar registers, and the
// branches between four hash functions cost enough of them to spill.
// WPE = waves per SIMD the kernel is compiled for: 4 (128 registers, one workgroup per compute unit) or 8 (64
// registers at the price of a few spills, two workgroups per compute unit: taken when there are more scans than
// compute units, where the second workgroup fills the issue slots the first leaves at its barriers).
template <int HASH, int WPE>
__global__ __launch_bounds__(STH, WPE) void k_pshs_scan(PshArgs a, int32_t* __restrict__ lidx0, int32_t* __restrict__ lidx1,
                                                   unsigned long long* __restrict__ lvox0, unsigned long long* __restrict__ lvox1)
{
    extern __shared__ int smem[];
    __shared__ ScanCfg cfg;
    __shared__ uint32_t red[8];
    __shared__ int wcount[2][SNW];
    __shared__ int s_placed;
    __shared__ int lds17[17];
    if (a.status[0]) return;   // inconsistent batch offsets: flagged by the set-up kernel, nothing to do
    const int b = blockIdx.x;
    const int p0 = a.scan_p0[b], nb = a.scan_p0[b + 1] - p0;
    const int kb0 = a.sbs[b], K = a.sbs[b + 1] - kb0;
    if (nb <= 0 || K <= 0) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kw = (K + 1) >> 1;
    int* fill = smem;
    int* runb[2] = {smem + K, smem + 2 * K};
    uint32_t* wh = reinterpret_cast<uint32_t*>(smem + 3 * K);
    uint32_t* wbase = wh + SNW * kw;

    // ---- first row of every bucket of the scan (buckets are full except the last), bounding box
    for (int j = tid; j < K; j += STH) a.offsets[kb0 + j] = p0 + min(j * a.S, nb);
    {
        uint32_t mn[3] = {0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu}, mx[3] = {0u, 0u, 0u};
        const float* src = a.coords + (size_t)p0 * 3;
        const long long nf = (long long)nb * 3;
        constexpr int UB = 6;   // loads in flight per thread; 6 * 1024 is a multiple of 3, so a slot keeps its axis
        for (long long f0 = tid; f0 < nf; f0 += (long long)UB * STH) {
            float v[UB];
#pragma unroll
            for (int j = 0; j < UB; ++j) {
                const long long f = f0 + (long long)j * STH;
                v[j] = f < nf ? src[f] : 0.f;
            }
#pragma unroll
            for (int j = 0; j < UB; ++j) {
                const long long f = f0 + (long long)j * STH;
                if (f < nf) {
                    const uint32_t o = f2ord(v[j]);
                    const int ax = (tid + j) % 3;   // f mod 3: 1024 = 1 (mod 3), and f0 advances by a multiple of 3
#pragma unroll
                    for (int t = 0; t < 3; ++t)
                        if (ax == t) { mn[t] = min(mn[t], o); mx[t] = max(mx[t], o); }
                }
            }
        }
        if (tid < 3) { red[tid] = 0xFFFFFFFFu; red[4 + tid] = 0u; }
        __syncthreads();
#pragma unroll
        for (int t = 0; t < 3; ++t) {
            uint32_t lo = mn[t], hi = mx[t];
            for (int d = 32; d >= 1; d >>= 1) {
                lo = min(lo, (uint32_t)__shfl_xor((int)lo, d, 64));
                hi = max(hi, (uint32_t)__shfl_xor((int)hi, d, 64));
            }
            if (lane == 0) { atomicMin(&red[t], lo); atomicMax(&red[4 + t], hi); }
        }
        __syncthreads();
        if (tid == 0) compute_cfg(a, b, red, cfg);
    }
    for (int k = tid; k < K; k += STH) { fill[k] = 0; runb[0][k] = 0; }
    for (int w = tid; w < SNW * kw; w += STH) wh[w] = 0u;
    __syncthreads();

    const int keybits = max(1, 32 - __clz(max(K - 1, 1)));
    int n_in = nb;          // entries of the list this step reads (step 0: the scan itself)
    int cur = 0;            // which run buffer holds the contenders seen so far in this step
    for (int r = 0; r <= a.n_probes; ++r) {
        const int32_t* in_idx = (r & 1) ? lidx0 : lidx1;     // step 0 reads the coordinates instead
        const unsigned long long* in_vox = (r & 1) ? lvox0 : lvox1;
        int32_t* out_idx = (r & 1) ? lidx1 : lidx0;
        unsigned long long* out_vox = (r & 1) ? lvox1 : lvox0;
        if (tid == 0) s_placed = 0;
        int out_base = 0, nplaced = 0;
        // entries passed on by the previous iteration, written after the next barrier
        int pend_idx[SPPT], pend_pos[SPPT];
        unsigned long long pend_vox[SPPT];
        bool pend[SPPT] = {false, false};
        const int n_it = (n_in + SIT - 1) / SIT;
        // The entries of an iteration are requested one iteration ahead (three words each: the coordinates in step 0,
        // index and packed voxel afterwards), so that an iteration does not start by waiting for memory.
        uint32_t nw0[SPPT], nw1[SPPT], nw2[SPPT];
#pragma unroll
        for (int s = 0; s < SPPT; ++s) {
            const int j = wave * (SIT / SNW) + s * 64 + lane;
            nw0[s] = nw1[s] = nw2[s] = 0u;
            if (j < n_in) {
                if (r == 0) {
                    const uint32_t* c = reinterpret_cast<const uint32_t*>(a.coords + (size_t)(p0 + j) * 3);
                    nw0[s] = c[0]; nw1[s] = c[1]; nw2[s] = c[2];
                } else {
                    const unsigned long long v = in_vox[p0 + j];
                    nw0[s] = (uint32_t)in_idx[p0 + j]; nw1[s] = (uint32_t)v; nw2[s] = (uint32_t)(v >> 32);
                }
            }
        }
        for (int it = 0; it < n_it; ++it) {
            int idx[SPPT], hh[SPPT], wl[SPPT];
            unsigned long long vox[SPPT];
            bool act[SPPT];
            uint32_t w0[SPPT], w1[SPPT], w2[SPPT];
#pragma unroll
            for (int s = 0; s < SPPT; ++s) { w0[s] = nw0[s]; w1[s] = nw1[s]; w2[s] = nw2[s]; }
            if (it + 1 < n_it) {
#pragma unroll
                for (int s = 0; s < SPPT; ++s) {
                    const int j = (it + 1) * SIT + wave * (SIT / SNW) + s * 64 + lane;
                    if (j < n_in) {
                        if (r == 0) {
                            const uint32_t* c = reinterpret_cast<const uint32_t*>(a.coords + (size_t)(p0 + j) * 3);
                            nw0[s] = c[0]; nw1[s] = c[1]; nw2[s] = c[2];
                        } else {
                            const unsigned long long v = in_vox[p0 + j];
                            nw0[s] = (uint32_t)in_idx[p0 + j]; nw1[s] = (uint32_t)v; nw2[s] = (uint32_t)(v >> 32);
                        }
                    }
                }
            }
#pragma unroll
            for (int s = 0; s < SPPT; ++s) {
                const int j = it * SIT + wave * (SIT / SNW) + s * 64 + lane;
                act[s] = j < n_in;
                idx[s] = 0;
                vox[s] = 0ull;
                if (act[s]) {
                    if (r == 0) {
                        idx[s] = j;
                        vox[s] = pack_voxel(voxel_of(__uint_as_float(w0[s]), cfg.mn[0], a.inv_voxel),
                                            voxel_of(__uint_as_float(w1[s]), cfg.mn[1], a.inv_voxel),
                                            voxel_of(__uint_as_float(w2[s]), cfg.mn[2], a.inv_voxel));
                    } else {
                        idx[s] = (int)w0[s];
                        vox[s] = (unsigned long long)w1[s] | ((unsigned long long)w2[s] << 32);
                    }
                }
            }
#pragma unroll
            for (int s = 0; s < SPPT; ++s) {
                int h = 0;
                if (act[s]) {
                    int x = (int)(vox[s] & 0x1FFFFFull), y = (int)((vox[s] >> 21) & 0x1FFFFFull), z = (int)(vox[s] >> 42);
                    if (r > 0) probe_voxel(a, r, cfg, x, y, z);
                    h = hash_bucket(HASH, x, y, z, cfg);
                }
                hh[s] = h;
            }
            // ---- rank inside the wave, per-wave counters
#pragma unroll
            for (int s = 0; s < SPPT; ++s) {
                const int h = hh[s];
                const unsigned long long m = match_key(h, act[s], keybits);
                int old = 0;
                if (act[s]) {
                    const int leader = __ffsll((long long)m) - 1;
                    const int before = __popcll(m & ((1ull << lane) - 1ull));
                    if (lane == leader) {
                        const int sh = (h & 1) * 16;
                        const uint32_t o = atomicAdd(&wh[wave * kw + (h >> 1)], (uint32_t)__popcll(m) << sh);
                        old = (int)((o >> sh) & 0xFFFFu);
                    }
                    old = __shfl(old, leader, 64) + before;
                }
                wl[s] = old;
            }
            __syncthreads();
            // ---- entries the previous iteration passed on: every wave's count is visible now
            {
                const int pb = (it + 1) & 1;
                int before = 0, total = 0;
                if (it > 0) {
#pragma unroll
                    for (int v = 0; v < SNW; ++v) {
                        const int c = wcount[pb][v];
                        before += v < wave ? c : 0;
                        total += c;
                    }
                }
#pragma unroll
                for (int s = 0; s < SPPT; ++s) {
                    if (pend[s]) {
                        out_idx[p0 + out_base + before + pend_pos[s]] = pend_idx[s];
                        out_vox[p0 + out_base + before + pend_pos[s]] = pend_vox[s];
                    }
                }
                out_base += total;
            }
            // ---- exclusive prefix over the waves per bucket; the counters are cleared for the next iteration
            int* run_cur = runb[cur];
            int* run_next = runb[cur ^ 1];
            for (int w = tid; w < kw; w += STH) {
                uint32_t run = 0;
#pragma unroll
                for (int v = 0; v < SNW; ++v) {
                    const uint32_t t = wh[v * kw + w];
                    wbase[v * kw + w] = run;
                    wh[v * kw + w] = 0u;
                    run += t;   // halves cannot carry into each other: an iteration has 2048 entries
                }
                run_next[2 * w] = run_cur[2 * w] + (int)(run & 0xFFFFu);
                if (2 * w + 1 < K) run_next[2 * w + 1] = run_cur[2 * w + 1] + (int)(run >> 16);
            }
            __syncthreads();
            // ---- accept while the bucket has room, pass on otherwise
            bool pass[SPPT];
#pragma unroll
            for (int s = 0; s < SPPT; ++s) {
                pass[s] = false;
                if (act[s]) {
                    const int h = hh[s];
                    const int rank = run_cur[h] + (int)((wbase[wave * kw + (h >> 1)] >> ((h & 1) * 16)) & 0xFFFFu) + wl[s];
                    const int cap = (h == K - 1) ? cfg.lastcap : a.S;
                    const int f = fill[h];
                    if (rank < cap - f) {
                        const int dst = p0 + h * a.S + f + rank;
                        a.inv_perm[p0 + idx[s]] = dst;
                        a.perm[dst] = p0 + idx[s];
                        ++nplaced;
                    } else {
                        pass[s] = true;
                    }
                }
            }
            {
                const unsigned long long b0 = __ballot(pass[0]), b1 = __ballot(pass[1]);
                const unsigned long long lt = (1ull << lane) - 1ull;
                const int c0 = __popcll(b0);
                if (lane == 0) wcount[it & 1][wave] = c0 + __popcll(b1);
                pend[0] = pass[0];
                pend[1] = pass[1];
                pend_pos[0] = __popcll(b0 & lt);
                pend_pos[1] = c0 + __popcll(b1 & lt);
#pragma unroll
                for (int s = 0; s < SPPT; ++s) { pend_idx[s] = idx[s]; pend_vox[s] = vox[s]; }
            }
            cur ^= 1;
        }
        __syncthreads();
        // ---- what the last iteration passed on; the list of the next step is complete after this
        {
            int before = 0, total = 0;
            if (n_it > 0) {
                const int pb = (n_it + 1) & 1;
#pragma unroll
                for (int v = 0; v < SNW; ++v) {
                    const int c = wcount[pb][v];
                    before += v < wave ? c : 0;
                    total += c;
                }
            }
#pragma unroll
            for (int s = 0; s < SPPT; ++s) {
                if (pend[s]) {
                    out_idx[p0 + out_base + before + pend_pos[s]] = pend_idx[s];
                    out_vox[p0 + out_base + before + pend_pos[s]] = pend_vox[s];
                }
            }
            n_in = out_base + total;
        }
        for (int d = 32; d >= 1; d >>= 1) nplaced += __shfl_xor(nplaced, d, 64);
        if (lane == 0 && nplaced) atomicAdd(&s_placed, nplaced);
        // fill levels after this step; contenders are counted afresh in the next one
        {
            int* run_cur = runb[cur];
            for (int k = tid; k < K; k += STH) {
                const int cap = (k == K - 1) ? cfg.lastcap : a.S;
                fill[k] = min(fill[k] + run_cur[k], cap);
                run_cur[k] = 0;
            }
        }
        // the list written in this step is read by other threads of the workgroup in the next one
        __threadfence_block();
        __syncthreads();
        if (tid == 0 && s_placed) atomicAdd(&a.round_count[r], s_placed);
        __syncthreads();
    }

    // ---- recycle: the j-th entry left takes the j-th free slot (buckets ascending, slots ascending)
    if (n_in == 0) return;   // uniform
    const int last = a.n_probes + 1;
    const int32_t* in_idx = (last & 1) ? lidx0 : lidx1;
    int* freepre = runb[0];   // both run buffers are free now
    {
        int carry = 0;
        for (int k0 = 0; k0 < K; k0 += STH) {
            const int k = k0 + tid;
            int v = 0;
            if (k < K) v = ((k == K - 1) ? cfg.lastcap : a.S) - fill[k];
            int tot;
            const int pre = block_excl_scan(v, &tot, lds17);
            if (k < K) freepre[k] = carry + pre;
            carry += tot;
        }
    }
    __syncthreads();
    int placed = 0;
    for (int j = tid; j < n_in; j += STH) {
        const int i = in_idx[p0 + j];
        int lo = 0, hi = K;   // largest k with freepre[k] <= j
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (freepre[mid] <= j) lo = mid; else hi = mid;
        }
        const int dst = p0 + lo * a.S + fill[lo] + (j - freepre[lo]);
        if (dst < p0 || dst >= p0 + nb) continue;   // cannot happen while capacities add up to the scan size
        a.inv_perm[p0 + i] = dst;
        a.perm[dst] = p0 + i;
        ++placed;
    }
    for (int d = 32; d >= 1; d >>= 1) placed += __shfl_xor(placed, d, 64);
    if (tid == 0) s_placed = 0;   // the last step's count was read before that step's final barrier
    __syncthreads();
    if (lane == 0 && placed) atomicAdd(&s_placed, placed);
    __syncthreads();
    if (tid == 0 && s_placed) atomicAdd(&a.round_count[a.n_probes + 1], s_placed);
}

}  // namespace

bool psh_scan_eligible(int kcap) { return kcap <= SKMAX; }

hipError_t psh_scan_launch(const PshArgs& args, int32_t* lidx0, int32_t* lidx1, unsigned long long* lvox0, unsigned long long* lvox1,
                           hipStream_t stream)
{
    PshArgs a = args;
    a.chunk = SIT;
    a.chunk_info = nullptr;
    a.meta_light = 1;   // the scan's own workgroup writes its bucket offsets
    k_psh_meta<<<1, 1024, 0, stream>>>(a);
    if (a.n == 0) return hipGetLastError();
    const size_t kw = (size_t)(a.kcap + 1) / 2;
    const size_t lds = ((size_t)3 * a.kcap + 2 * SNW * kw) * 4;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) cus = 0;
    const bool two = cus > 0 && a.n_scans > cus && 2 * lds <= 150 * 1024;
    const void* fn[8] = {(const void*)k_pshs_scan<0, 4>, (const void*)k_pshs_scan<1, 4>, (const void*)k_pshs_scan<2, 4>,
                         (const void*)k_pshs_scan<3, 4>, (const void*)k_pshs_scan<0, 8>, (const void*)k_pshs_scan<1, 8>,
                         (const void*)k_pshs_scan<2, 8>, (const void*)k_pshs_scan<3, 8>};
    const int which = (a.hash & 3) + (two ? 4 : 0);
    if (lds > 60000) {
        const hipError_t e = hipFuncSetAttribute(fn[which], hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    switch (which) {
        case 0: k_pshs_scan<0, 4><<<a.n_scans, STH, lds, stream>>>(a, lidx0, lidx1, lvox0, lvox1); break;
        case 1: k_pshs_scan<1, 4><<<a.n_scans, STH, lds, stream>>>(a, lidx0, lidx1, lvox0, lvox1); break;
        case 2: k_pshs_scan<2, 4><<<a.n_scans, STH, lds, stream>>>(a, lidx0, lidx1, lvox0, lvox1); break;
        case 3: k_pshs_scan<3, 4><<<a.n_scans, STH, lds, stream>>>(a, lidx0, lidx1, lvox0, lvox1); break;
        case 4: k_pshs_scan<0, 8><<<a.n_scans, STH, lds, stream>>>(a, lidx0, lidx1, lvox0, lvox1); break;
        case 5: k_pshs_scan<1, 8><<<a.n_scans, STH, lds, stream>>>(a, lidx0, lidx1, lvox0, lvox1); break;
        case 6: k_pshs_scan<2, 8><<<a.n_scans, STH, lds, stream>>>(a, lidx0, lidx1, lvox0, lvox1); break;
        default: k_pshs_scan<3, 8><<<a.n_scans, STH, lds, stream>>>(a, lidx0, lidx1, lvox0, lvox1); break;
    }
    return hipGetLastError();
}

}  // namespace f3d

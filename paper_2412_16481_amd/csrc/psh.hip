// PSH bucketing for gfx950: voxelise, hash, rank, rebalance, scatter (Algorithms 1 and 2).
//
// The paper lets atomic counters decide which point gets which slot. Here every step is a stable
// counting rank instead, so the result is the one a lock-step execution with index-ordered
// atomics would give and is bit-reproducible:
//   step 0      every point hashes its voxel; the first `cap` contenders of a bucket (by input index) stay
//   step 1..P   points still unplaced hash the voxel moved by the step's probe offset; they fill the
//               room left in that bucket, again by input index
//   recycle     what is left fills the remaining free slots, first bucket first
// A workgroup owns a chunk of CHUNK consecutive points of one scan. Ranks inside a chunk come from
// wave ballots plus per-wave LDS counters (the block-local counters of the appendix's two-stage
// scheme); the ranks of different chunks are joined by a column scan over a [chunk][bucket] count
// matrix (the "bulk commit" that rebases local offsets to global ones).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "psh_common.h"

namespace f3d {

// ------------------------------------------------------------------------------------------------
// one workgroup: per-scan tables (points, buckets, chunks), offsets[], counters, bounding-box init
__global__ __launch_bounds__(1024) void k_psh_meta(PshArgs a)
{
    __shared__ int lds[17];
    __shared__ int bad;
    const int tid = threadIdx.x;
    if (tid == 0) bad = 0;
    __syncthreads();
    int kcarry = 0, ccarry = 0;
    for (int base = 0; base < a.n_scans; base += 1024) {
        const int b = base + tid;
        int K = 0, c = 0, p0 = 0;
        if (b < a.n_scans) {
            p0 = batch_off(a, b);
            const int p1 = batch_off(a, b + 1);
            const long long nb = (long long)p1 - p0;
            bool ok = nb >= 0 && nb <= a.max_scan_points && p0 >= 0 && p1 <= a.n;
            if (b == 0 && p0 != 0) ok = false;
            if (b == a.n_scans - 1 && p1 != a.n) ok = false;
            if (!ok) bad = 1;
            if (ok) {
                K = (int)((nb + a.S - 1) / a.S);
                c = (int)((nb + a.chunk - 1) / a.chunk);
            }
        }
        int ktot, ctot;
        int kpre = block_excl_scan(K, &ktot, lds);
        int cpre = block_excl_scan(c, &ctot, lds);
        if (b < a.n_scans) {
            a.sbs[b] = kcarry + kpre;
            a.scan_c0[b] = ccarry + cpre;
            a.scan_p0[b] = p0;
            for (int ax = 0; ax < 3; ++ax) {
                a.mm[b * 8 + ax] = 0xFFFFFFFFu;
                a.mm[b * 8 + 4 + ax] = 0u;
            }
            a.done[b] = 0;
        }
        kcarry += ktot;
        ccarry += ctot;
    }
    __syncthreads();
    const int isbad = bad;
    if (tid == 0) {
        a.sbs[a.n_scans] = isbad ? -1 : kcarry;
        a.scan_c0[a.n_scans] = isbad ? 0 : ccarry;
        a.scan_p0[a.n_scans] = a.n;
        a.status[0] = isbad;
    }
    if (tid < 8) a.round_count[tid] = 0;
    __threadfence_block();   // the scan tables just written are read below by other threads (the barrier alone orders LDS)
    __syncthreads();
    if (isbad) return;
    // first row of every bucket (buckets are full except the last of a scan) and the chunk table (everything a
    // workgroup needs to find its points, in one load). With up to three scans the whole workgroup walks each scan; with more,
    // that loop is a chain of dependent loads (a batch may hold hundreds of scans): then a wave takes a scan.
    const bool by_wave = a.n_scans >= 4;   // measured: one scan 4.9 against 5.6 us, eight scans 10.3 against 6.7 us
    const int first = by_wave ? (tid >> 6) : 0, scan_step = by_wave ? 16 : 1;
    const int e0 = by_wave ? (tid & 63) : tid, e_step = by_wave ? 64 : 1024;
    for (int b = (a.meta_light ? a.n_scans : first); b < a.n_scans; b += scan_step) {
        const int p0 = a.scan_p0[b], nb = a.scan_p0[b + 1] - p0;
        const int kb0 = a.sbs[b], K = a.sbs[b + 1] - kb0;
        for (int j = e0; j < K; j += e_step) {
            a.offsets[kb0 + j] = p0 + min(j * a.S, nb);
            a.cnt[kb0 + j] = 0;
        }
    }
    for (int j = kcarry + tid; j <= a.max_buckets; j += 1024) a.offsets[j] = a.n;
    if (a.chunk_info) {
        for (int b = first; b < a.n_scans; b += scan_step) {
            const int p0 = a.scan_p0[b], p1 = a.scan_p0[b + 1];
            const int kb0 = a.sbs[b], K = a.sbs[b + 1] - kb0;
            const int c0 = a.scan_c0[b], nc = a.scan_c0[b + 1] - c0;
            for (int lc = e0; lc < nc; lc += e_step) {
                const int begin = p0 + lc * a.chunk;
                a.chunk_info[2 * (c0 + lc)] = make_int4(b, lc, nc, begin);
                a.chunk_info[2 * (c0 + lc) + 1] = make_int4(min(begin + a.chunk, p1), kb0, K, c0);
            }
        }
        for (int c = ccarry + tid; c < a.n_chunks_ub; c += 1024) a.chunk_info[2 * c] = make_int4(-1, 0, 0, 0);
    }
}

// ------------------------------------------------------------------------------------------------
// per-scan bounding box
__global__ __launch_bounds__(PSH_THREADS) void k_psh_minmax(PshArgs a)
{
    if (a.status[0]) return;
    const int chunk = blockIdx.x;
    if (chunk >= a.scan_c0[a.n_scans]) return;
    const int b = find_scan(a.scan_c0, a.n_scans, chunk);
    const int p0 = a.scan_p0[b], p1 = a.scan_p0[b + 1];
    const int begin = p0 + (chunk - a.scan_c0[b]) * PSH_CHUNK;
    const int end = min(begin + PSH_CHUNK, p1);
    uint32_t mn[3] = {0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu}, mx[3] = {0u, 0u, 0u};
    // the chunk's coordinates are 3*(end-begin) consecutive floats: read them flat and coalesced
    const float* src = a.coords + (size_t)begin * 3;
    const int nf = (end - begin) * 3;
    for (int f = threadIdx.x; f < nf; f += PSH_THREADS) {
        const uint32_t o = f2ord(src[f]);
        const int ax = f % 3;
#pragma unroll
        for (int t = 0; t < 3; ++t)
            if (ax == t) { mn[t] = min(mn[t], o); mx[t] = max(mx[t], o); }
    }
    __shared__ uint32_t red[8];
    if (threadIdx.x < 3) { red[threadIdx.x] = 0xFFFFFFFFu; red[4 + threadIdx.x] = 0u; }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < 3; ++t) {
        uint32_t lo = mn[t], hi = mx[t];
        for (int d = 32; d >= 1; d >>= 1) {
            lo = min(lo, (uint32_t)__shfl_xor((int)lo, d, 64));
            hi = max(hi, (uint32_t)__shfl_xor((int)hi, d, 64));
        }
        if ((threadIdx.x & 63) == 0) { atomicMin(&red[t], lo); atomicMax(&red[4 + t], hi); }
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        atomicMin(&a.mm[b * 8 + threadIdx.x], red[threadIdx.x]);
        atomicMax(&a.mm[b * 8 + 4 + threadIdx.x], red[4 + threadIdx.x]);
    }
}

// ------------------------------------------------------------------------------------------------
// step r of the schedule: settle step r-1 (accept what fits), then rank the contenders of step r.
//   r == 0          all points are contenders of their direct hash
//   1 <= r <= P     contenders = points not accepted so far, hashed with probe offset r
//   r == P+1        no new hash: the points still left are counted and ranked for the recycle step
// dynamic LDS: pre[kcap] ints (this chunk's row of rebased counters) + 4 waves x kcap packed u16 counters
__global__ __launch_bounds__(PSH_THREADS) void k_psh_step(PshArgs a, int r)
{
    extern __shared__ int smem[];
    __shared__ ScanCfg cfg;
    __shared__ int placed_ct;
    if (a.status[0]) return;
    const int chunk = blockIdx.x;
    if (chunk >= a.scan_c0[a.n_scans]) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = find_scan(a.scan_c0, a.n_scans, chunk);
    if (tid == 0) { compute_cfg(a, b, a.mm + b * 8, cfg); placed_ct = 0; }
    const int kwords = (a.kcap + 1) >> 1;
    int* pre = smem;                              // [kcap]
    uint32_t* wh = (uint32_t*)(smem + a.kcap);    // [PSH_WAVES][kwords], two 16-bit counters per word
    __syncthreads();
    const int K = cfg.K;
    const bool last_step = (r == a.n_probes + 1);
    int* row = a.hist + (size_t)chunk * a.kcap;
    if (r > 0)
        for (int k = tid; k < K; k += PSH_THREADS) pre[k] = row[k];
    for (int w = tid; w < PSH_WAVES * kwords; w += PSH_THREADS) wh[w] = 0u;
    __syncthreads();

    const int begin = cfg.p0 + (chunk - a.scan_c0[b]) * PSH_CHUNK;
    const int end = min(begin + PSH_CHUNK, cfg.p0 + cfg.nb);
    const int keybits = last_step ? 0 : max(1, 32 - __clz(max(K - 1, 1)));
    constexpr int PPT = PSH_CHUNK / PSH_THREADS;
    int hh[PPT], wl[PPT];
    int nplaced = 0;
#pragma unroll
    for (int s = 0; s < PPT; ++s) {
        const int i = begin + wave * (PSH_CHUNK / PSH_WAVES) + s * 64 + lane;
        bool active = i < end;
        int h = 0;
        if (active && r > 0) {
            const uint32_t kw = a.key[i];
            if (kw == KEY_PLACED) {
                active = false;
            } else {
                const int hp = (int)(kw >> LR_BITS), lr = (int)(kw & ((1u << LR_BITS) - 1));
                const int rank = pre[hp] + lr;
                const int cap = (hp == K - 1) ? cfg.lastcap : a.S;
                if (rank < cap) {
                    const int dst = cfg.p0 + hp * a.S + rank;
                    a.inv_perm[i] = dst;
                    a.perm[dst] = i;
                    a.key[i] = KEY_PLACED;
                    active = false;
                    ++nplaced;
                }
            }
        }
        if (active && !last_step) {
            const float* c = a.coords + (size_t)i * 3;
            int x = voxel_of(c[0], cfg.mn[0], a.inv_voxel);
            int y = voxel_of(c[1], cfg.mn[1], a.inv_voxel);
            int z = voxel_of(c[2], cfg.mn[2], a.inv_voxel);
            if (r > 0) probe_voxel(a, r, cfg, x, y, z);
            h = hash_bucket(a.hash, x, y, z, cfg);
        }
        // lanes of this wave that contend for the same bucket, by ballots over the key bits
        unsigned long long m = __ballot(active);
        for (int bit = 0; bit < keybits; ++bit) {
            const bool one = (h >> bit) & 1;
            const unsigned long long bal = __ballot(active && one);
            m &= one ? bal : ~bal;
        }
        int old = 0;
        if (active) {
            const int leader = __ffsll((long long)m) - 1;
            const int before = __popcll(m & ((1ull << lane) - 1ull));
            if (lane == leader) {
                const int sh = (h & 1) * 16;
                const uint32_t o = atomicAdd(&wh[wave * kwords + (h >> 1)], (uint32_t)__popcll(m) << sh);
                old = (int)((o >> sh) & 0xFFFFu);
            }
            old = __shfl(old, leader, 64) + before;
        }
        hh[s] = active ? h : -1;
        wl[s] = old;
    }
    __syncthreads();
    // join the waves: exclusive prefix over the four waves per bucket, total to the count matrix
    const int nk = last_step ? 1 : K;
    for (int w = tid; w < (nk + 1) >> 1; w += PSH_THREADS) {
        uint32_t run = 0;
#pragma unroll
        for (int v = 0; v < PSH_WAVES; ++v) {
            const uint32_t t = wh[v * kwords + w];
            wh[v * kwords + w] = run;
            run += t;  // halves cannot carry into each other: a chunk has at most 4096 points
        }
        if (!last_step) {
            row[2 * w] = (int)(run & 0xFFFFu);
            if (2 * w + 1 < K) row[2 * w + 1] = (int)(run >> 16);
        } else {
            a.left[chunk] = (int)(run & 0xFFFFu);
        }
    }
    __syncthreads();
#pragma unroll
    for (int s = 0; s < PPT; ++s) {
        const int i = begin + wave * (PSH_CHUNK / PSH_WAVES) + s * 64 + lane;
        if (hh[s] >= 0) {
            const int h = hh[s];
            const int base = (int)((wh[wave * kwords + (h >> 1)] >> ((h & 1) * 16)) & 0xFFFFu);
            a.key[i] = ((uint32_t)h << LR_BITS) | (uint32_t)(base + wl[s]);
        }
    }
    if (r > 0) {
        for (int d = 32; d >= 1; d >>= 1) nplaced += __shfl_xor(nplaced, d, 64);
        if (lane == 0 && nplaced) atomicAdd(&placed_ct, nplaced);
        __syncthreads();
        if (tid == 0 && placed_ct) atomicAdd(&a.round_count[r - 1], placed_ct);
    }
}

// ------------------------------------------------------------------------------------------------
// column scan of the count matrix: hist[c][k] <- cnt[k] + sum_{c' < c} hist[c'][k]; cnt[k] <- min(cap, total)
// block = 64 buckets x 16 chunk lanes; grid = (ceil(kcap/64), n_scans)
__global__ __launch_bounds__(1024) void k_psh_colscan(PshArgs a)
{
    if (a.status[0]) return;
    const int b = blockIdx.y;
    const int kb0 = a.sbs[b], K = a.sbs[b + 1] - kb0;
    const int kx = threadIdx.x & 63, cy = threadIdx.x >> 6;
    const int k = blockIdx.x * 64 + kx;
    if (blockIdx.x * 64 >= K) return;
    const int c0 = a.scan_c0[b], nc = a.scan_c0[b + 1] - c0;
    const int per = (nc + 15) >> 4;
    const int cb = min(cy * per, nc), ce = min(cb + per, nc);
    __shared__ int part[16][64];
    int sum = 0;
    if (k < K)
        for (int c = cb; c < ce; ++c) sum += a.hist[(size_t)(c0 + c) * a.kcap + k];
    part[cy][kx] = sum;
    __syncthreads();
    if (k < K) {
        int run = a.cnt[kb0 + k];
        for (int y = 0; y < cy; ++y) run += part[y][kx];
        for (int c = cb; c < ce; ++c) {
            const size_t at = (size_t)(c0 + c) * a.kcap + k;
            const int t = a.hist[at];
            a.hist[at] = run;
            run += t;
        }
        if (cy == 15) {
            // lane 15 owns the tail, so `run` is now the grand total (empty tails included)
            const int nb = a.scan_p0[b + 1] - a.scan_p0[b];
            const int cap = (k == K - 1) ? nb - (K - 1) * a.S : a.S;
            a.cnt_next[kb0 + k] = min(run, cap);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// recycle, part 1 (one workgroup per scan): prefix of leftovers per chunk, prefix of free slots per bucket
__global__ __launch_bounds__(1024) void k_psh_recycle_scan(PshArgs a)
{
    __shared__ int lds[17];
    if (a.status[0]) return;
    const int b = blockIdx.x, tid = threadIdx.x;
    const int c0 = a.scan_c0[b], nc = a.scan_c0[b + 1] - c0;
    int carry = 0;
    for (int base = 0; base < nc; base += 1024) {
        const int c = base + tid;
        const int v = c < nc ? a.left[c0 + c] : 0;
        int tot;
        const int pre = block_excl_scan(v, &tot, lds);
        if (c < nc) a.leftpre[c0 + c] = carry + pre;
        carry += tot;
    }
    const int kb0 = a.sbs[b], K = a.sbs[b + 1] - kb0;
    const int nb = a.scan_p0[b + 1] - a.scan_p0[b];
    carry = 0;
    for (int base = 0; base < K; base += 1024) {
        const int k = base + tid;
        int v = 0;
        if (k < K) v = ((k == K - 1) ? nb - (K - 1) * a.S : a.S) - a.cnt[kb0 + k];
        int tot;
        const int pre = block_excl_scan(v, &tot, lds);
        if (k < K) a.freepre[kb0 + k] = carry + pre;
        carry += tot;
    }
}

// recycle, part 2: the r-th leftover of a scan takes the r-th free slot (buckets ascending, slots ascending)
__global__ __launch_bounds__(PSH_THREADS) void k_psh_recycle_place(PshArgs a)
{
    if (a.status[0]) return;
    const int chunk = blockIdx.x;
    if (chunk >= a.scan_c0[a.n_scans]) return;
    if (a.left[chunk] == 0) return;
    const int b = find_scan(a.scan_c0, a.n_scans, chunk);
    const int p0 = a.scan_p0[b], p1 = a.scan_p0[b + 1];
    const int kb0 = a.sbs[b], K = a.sbs[b + 1] - kb0;
    const int begin = p0 + (chunk - a.scan_c0[b]) * PSH_CHUNK;
    const int end = min(begin + PSH_CHUNK, p1);
    const int base = a.leftpre[chunk];
    int mine = 0;
    for (int i = begin + threadIdx.x; i < end; i += PSH_THREADS) {
        const uint32_t kw = a.key[i];
        if (kw == KEY_PLACED) continue;
        const int rank = base + (int)(kw & ((1u << LR_BITS) - 1));
        int lo = 0, hi = K;  // largest j with freepre[j] <= rank
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (a.freepre[kb0 + mid] <= rank) lo = mid; else hi = mid;
        }
        const int dst = p0 + lo * a.S + a.cnt[kb0 + lo] + (rank - a.freepre[kb0 + lo]);
        if (dst < p0 || dst >= p1) continue;  // cannot happen while capacities add up to the scan size
        a.inv_perm[i] = dst;
        a.perm[dst] = i;
        ++mine;
    }
    // one atomic per workgroup: per-wave atomics of thousands of workgroups on one counter queue up
    __shared__ int s_mine;
    for (int d = 32; d >= 1; d >>= 1) mine += __shfl_xor(mine, d, 64);
    if (threadIdx.x == 0) s_mine = 0;
    __syncthreads();
    if ((threadIdx.x & 63) == 0 && mine) atomicAdd(&s_mine, mine);
    __syncthreads();
    if (threadIdx.x == 0 && s_mine) atomicAdd(&a.round_count[a.n_probes + 1], s_mine);
}

// ------------------------------------------------------------------------------------------------
hipError_t psh_launch(const PshArgs& args, hipStream_t stream)
{
    PshArgs a = args;
    a.chunk = PSH_CHUNK;
    a.chunk_info = nullptr;  // the chunk table is sized for the other path's chunks
    k_psh_meta<<<1, 1024, 0, stream>>>(a);
    if (a.n == 0) return hipGetLastError();
    const int chunks = (int)(a.n / PSH_CHUNK) + a.n_scans;  // upper bound, surplus workgroups exit
    k_psh_minmax<<<chunks, PSH_THREADS, 0, stream>>>(a);
    const size_t lds = (size_t)a.kcap * 4 + (size_t)PSH_WAVES * ((a.kcap + 1) / 2) * 4;
    if (lds > 60000) {
        const hipError_t e = hipFuncSetAttribute((const void*)k_psh_step, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    const dim3 cgrid((a.kcap + 63) / 64, a.n_scans);
    int32_t* c0 = a.cnt;
    int32_t* c1 = a.cnt_next;
    for (int r = 0; r <= a.n_probes + 1; ++r) {
        a.cnt = c0;
        a.cnt_next = c1;
        k_psh_step<<<chunks, PSH_THREADS, lds, stream>>>(a, r);
        if (r <= a.n_probes) {
            k_psh_colscan<<<cgrid, 1024, 0, stream>>>(a);
            int32_t* t = c0; c0 = c1; c1 = t;  // the scan wrote the new fill levels to cnt_next
        }
    }
    a.cnt = c0;
    k_psh_recycle_scan<<<a.n_scans, 1024, 0, stream>>>(a);
    k_psh_recycle_place<<<chunks, PSH_THREADS, 0, stream>>>(a);
    return hipGetLastError();
}

}  // namespace f3d

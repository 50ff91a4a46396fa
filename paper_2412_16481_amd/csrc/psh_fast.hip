// PSH bucketing, short-latency path for scans whose [chunk][bucket] count matrix is small (all of the
// paper's operating range: ~1e5 points per scan, a few hundred buckets).
//
// Same schedule and same results as psh.hip (Algorithms 1 and 2 in lock step, index-ordered), but one
// launch per step instead of two: a workgroup ranks a chunk of 2048 points, writes one row of 16-bit
// counts, and in the NEXT launch every workgroup sums the rows it needs by itself (rows of earlier
// chunks rebase its local ranks, all rows give the new fill levels), so no separate scan kernel and no
// second round trip through the launch queue.
//
// At these sizes the kernels are bound by memory LATENCY and launch boundaries, not bandwidth: every
// kernel is written as "one load that tells the workgroup what to do, then all other loads at once,
// then arithmetic".
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "psh_common.h"

namespace f3d {

namespace {

constexpr int FCH = 2048;    // points per workgroup
constexpr int FTH = 512;     // threads per workgroup
constexpr int FW = FTH / 64; // waves
constexpr int FPPT = FCH / FTH;
constexpr int FKMAX = 2048;           // most buckets per scan on this path
constexpr int KPT = FKMAX / FTH;      // buckets per thread when a row is walked linearly
constexpr long long FMATMAX = 131072; // most (chunks of a scan) x (buckets of a scan)
constexpr int CFGW = (int)(sizeof(ScanCfg) / 4);
static_assert(sizeof(ScanCfg) <= 128 && sizeof(ScanCfg) % 4 == 0, "the workspace reserves 128 bytes per scan");

struct ChunkInfo {
    int b, lc, nc, begin, end, kb0, K, c0;
};
__device__ __forceinline__ ChunkInfo load_chunk(const PshArgs& a, int chunk)
{
    const int4 u = a.chunk_info[2 * chunk], v = a.chunk_info[2 * chunk + 1];
    return ChunkInfo{u.x, u.y, u.z, u.w, v.x, v.y, v.z, v.w};
}

// row pitch of the count matrix in 32-bit words (two 16-bit counts per word), rows 16-byte aligned
__host__ __device__ inline int row_pitch(int kcap) { return (((kcap + 1) >> 1) + 3) & ~3; }

// ------------------------------------------------------------------------------------------------
// per-scan bounding box
__global__ __launch_bounds__(FTH) void k_pshf_minmax(PshArgs a)
{
    const ChunkInfo ci = load_chunk(a, blockIdx.x);
    if (ci.b < 0 || a.status[0]) return;
    const int b = ci.b;
    uint32_t mn[3] = {0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu}, mx[3] = {0u, 0u, 0u};
    const float* src = a.coords + (size_t)ci.begin * 3;
    const int nf = (ci.end - ci.begin) * 3;
    float v[3 * FPPT];
#pragma unroll
    for (int j = 0; j < 3 * FPPT; ++j) {   // all twelve loads in flight together
        const int f = threadIdx.x + j * FTH;
        v[j] = f < nf ? src[f] : 0.f;
    }
#pragma unroll
    for (int j = 0; j < 3 * FPPT; ++j) {
        const int f = threadIdx.x + j * FTH;
        if (f < nf) {
            const uint32_t o = f2ord(v[j]);
            const int ax = f % 3;
#pragma unroll
            for (int t = 0; t < 3; ++t)
                if (ax == t) { mn[t] = min(mn[t], o); mx[t] = max(mx[t], o); }
        }
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
// Set-up and bounding boxes in ONE launch, for batches of at most 64 scans. The scan tables (first point, first bucket,
// first chunk of every scan) are a closed form of batch_offsets and S: every workgroup works them out itself (one
// wave, a prefix over the scans), finds its chunk and writes the chunk's own box, without atomics, so nothing has to
// be initialised by an earlier launch; step 0 joins the boxes of a scan's chunks. Workgroup 0 also writes the tables
// the later kernels read.
constexpr int SETUP_MAX_SCANS = 64;

__global__ __launch_bounds__(FTH) void k_pshf_setup(PshArgs a)
{
    __shared__ int s_p0[SETUP_MAX_SCANS + 1], s_kb0[SETUP_MAX_SCANS + 1], s_c0[SETUP_MAX_SCANS + 1];
    __shared__ int s_bad;
    __shared__ uint32_t red[8];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ns = a.n_scans;
    if (wave == 0) {
        int p0 = 0, K = 0, c = 0;
        bool ok = true;
        if (lane < ns) {
            p0 = batch_off(a, lane);
            const int p1 = batch_off(a, lane + 1);
            const long long nb = (long long)p1 - p0;
            ok = nb >= 0 && nb <= a.max_scan_points && p0 >= 0 && p1 <= a.n;
            if (lane == 0 && p0 != 0) ok = false;
            if (lane == ns - 1 && p1 != a.n) ok = false;
            if (ok) {
                K = (int)((nb + a.S - 1) / a.S);
                c = (int)((nb + FCH - 1) / FCH);
            }
        }
        const bool bad = __builtin_amdgcn_ballot_w64(!ok) != 0ull;
        const int kin = wave_incl_scan(K, lane), cin = wave_incl_scan(c, lane);
        if (lane < ns) {
            s_p0[lane] = p0;
            s_kb0[lane] = kin - K;
            s_c0[lane] = cin - c;
        }
        if (lane == ns - 1) {
            s_p0[ns] = a.n;
            s_kb0[ns] = kin;
            s_c0[ns] = cin;
        }
        if (lane == 0) s_bad = bad ? 1 : 0;
    }
    __syncthreads();
    const int isbad = s_bad, ktot = s_kb0[ns], ctot = s_c0[ns];
    if (blockIdx.x == 0) {   // the tables of the later kernels
        if (tid < ns) {
            a.sbs[tid] = s_kb0[tid];
            a.scan_c0[tid] = s_c0[tid];
            a.scan_p0[tid] = s_p0[tid];
            a.done[tid] = 0;
        }
        if (tid == 0) {
            a.sbs[ns] = isbad ? -1 : ktot;
            a.scan_c0[ns] = isbad ? 0 : ctot;
            a.scan_p0[ns] = a.n;
            a.status[0] = isbad;
        }
        if (tid < 8) a.round_count[tid] = 0;
        if (!isbad) {
            // first row of every bucket (buckets are full except the last of a scan); a wave takes a scan
            for (int b = wave; b < ns; b += FW) {
                const int p0 = s_p0[b], nb = s_p0[b + 1] - p0, kb0 = s_kb0[b], K = s_kb0[b + 1] - kb0;
                for (int j = lane; j < K; j += 64) {
                    a.offsets[kb0 + j] = p0 + min(j * a.S, nb);
                    a.cnt[kb0 + j] = 0;
                }
            }
            for (int j = ktot + tid; j <= a.max_buckets; j += FTH) a.offsets[j] = a.n;
        }
    }
    const int chunk = blockIdx.x;
    if (isbad || chunk >= ctot) {
        if (tid == 0) a.chunk_info[2 * chunk] = make_int4(-1, 0, 0, 0);
        return;
    }
    // the chunk's scan: the last one that starts at or before it (scans without points have no chunks)
    const int b = __popcll(__builtin_amdgcn_ballot_w64(lane < ns && s_c0[lane] <= chunk)) - 1;
    const int p0 = s_p0[b], p1 = s_p0[b + 1], c0 = s_c0[b], lc = chunk - c0;
    const int begin = p0 + lc * FCH, end = min(begin + FCH, p1);
    if (tid == 0) {
        a.chunk_info[2 * chunk] = make_int4(b, lc, s_c0[b + 1] - c0, begin);
        a.chunk_info[2 * chunk + 1] = make_int4(end, s_kb0[b], s_kb0[b + 1] - s_kb0[b], c0);
    }
    uint32_t mn[3] = {0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu}, mx[3] = {0u, 0u, 0u};
    const float* src = a.coords + (size_t)begin * 3;
    const int nf = (end - begin) * 3;
    float v[3 * FPPT];
#pragma unroll
    for (int j = 0; j < 3 * FPPT; ++j) {   // all twelve loads in flight together
        const int f = tid + j * FTH;
        v[j] = f < nf ? src[f] : 0.f;
    }
#pragma unroll
    for (int j = 0; j < 3 * FPPT; ++j) {
        const int f = tid + j * FTH;
        if (f < nf) {
            const uint32_t o = f2ord(v[j]);
            const int ax = f % 3;
#pragma unroll
            for (int t = 0; t < 3; ++t)
                if (ax == t) { mn[t] = min(mn[t], o); mx[t] = max(mx[t], o); }
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
    if (tid < 3) {
        a.mmpart[chunk * 8 + tid] = red[tid];
        a.mmpart[chunk * 8 + 4 + tid] = red[4 + tid];
    }
}

// ------------------------------------------------------------------------------------------------
// step r: settle step r-1 from the count rows of that step, then rank the contenders of step r
// dynamic LDS: tot[kcap] + pre[kcap] ints + NW x kwp words of packed 16-bit counters.
// TH threads rank the 2048 points of a chunk: 512 (four points each, two workgroups per CU) when the grid is
// larger than the GPU, 1024 (two points each: every phase of the step is half as long) when it is not.
template <int TH>
__global__ __launch_bounds__(TH) void k_pshf_step(PshArgs a, int r, const uint32_t* __restrict__ mat_prev,
                                                   uint32_t* __restrict__ mat_cur)
{
    constexpr int NW = TH / 64, PPT = FCH / TH, KPT_ = FKMAX / TH;
    extern __shared__ int smem[];
    __shared__ ScanCfg cfg;
    __shared__ int placed_ct;
    const int chunk = blockIdx.x;
    const ChunkInfo ci = load_chunk(a, chunk);
    if (ci.b < 0 || a.status[0]) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int K = ci.K, kb0 = ci.kb0, lc = ci.lc, nc = ci.nc;
    const int kwp = row_pitch(a.kcap);
    int* tot = smem;                                // [kcap] contenders of step r-1 per bucket, all chunks
    int* pre = smem + a.kcap;                       // [kcap] ... of earlier chunks; then rebased fill level
    uint32_t* wh = (uint32_t*)(smem + 2 * a.kcap);  // [NW][kwp]
    const bool last_step = (r == a.n_probes + 1);

    // ---- every global load of this kernel is issued here, before anything waits
    uint32_t box[8];
    uint32_t cfgw = 0;
    if (r == 0) {
        if (a.mmpart) {   // the boxes of the scan's chunks, joined by the first wave
            if (wave == 0) {
                uint32_t lo[3] = {0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu}, hi[3] = {0u, 0u, 0u};
                for (int t = lane; t < ci.nc; t += 64) {
                    const uint32_t* pb = a.mmpart + (size_t)(ci.c0 + t) * 8;
#pragma unroll
                    for (int ax = 0; ax < 3; ++ax) { lo[ax] = min(lo[ax], pb[ax]); hi[ax] = max(hi[ax], pb[4 + ax]); }
                }
#pragma unroll
                for (int ax = 0; ax < 3; ++ax) {
                    for (int d = 32; d >= 1; d >>= 1) {
                        lo[ax] = min(lo[ax], (uint32_t)__shfl_xor((int)lo[ax], d, 64));
                        hi[ax] = max(hi[ax], (uint32_t)__shfl_xor((int)hi[ax], d, 64));
                    }
                    box[ax] = lo[ax];
                    box[4 + ax] = hi[ax];
                }
            }
        } else if (tid == 0) {
            for (int i = 0; i < 8; ++i) box[i] = a.mm[ci.b * 8 + i];
        }
    } else if (tid < CFGW) {
        cfgw = reinterpret_cast<const uint32_t*>(reinterpret_cast<const ScanCfg*>(a.cfg) + ci.b)[tid];
    }
    uint32_t kwv[PPT];
    float cx[PPT], cy[PPT], cz[PPT];
#pragma unroll
    for (int s = 0; s < PPT; ++s) {
        const int i = ci.begin + wave * (FCH / NW) + s * 64 + lane;
        kwv[s] = KEY_PLACED;
        cx[s] = cy[s] = cz[s] = 0.f;
        if (i < ci.end) {
            kwv[s] = r > 0 ? a.key[i] : 0u;
            if (!last_step) {
                const float* c = a.coords + (size_t)i * 3;
                cx[s] = c[0]; cy[s] = c[1]; cz[s] = c[2];
            }
        }
    }
    // Count rows of step r-1, 16 bytes (8 buckets) per load: thread (g, seg) sums column group g over
    // rows seg, seg+nseg, ... in registers; the row segments are joined in LDS afterwards.
    const int G = (((K + 1) >> 1) + 3) >> 2;        // column groups in use (<= 256)
    const int nseg = TH / G, seg = tid / G, g = tid - seg * G;
    int tl[8], pl[8], cntv[KPT_];
#pragma unroll
    for (int e = 0; e < 8; ++e) { tl[e] = 0; pl[e] = 0; }
    if (r > 0) {
        if (seg < nseg) {
            const uint4* col = reinterpret_cast<const uint4*>(mat_prev + (size_t)ci.c0 * kwp) + g;
            const int pitch4 = kwp >> 2;
            constexpr int LB = 12;   // loads in flight per thread: a row fetch costs a trip to HBM-side cache
            for (int c = seg; c < nc; c += LB * nseg) {
                uint4 v[LB];
#pragma unroll
                for (int j = 0; j < LB; ++j) {
                    const int cj = c + j * nseg;
                    v[j] = cj < nc ? col[(size_t)cj * pitch4] : make_uint4(0, 0, 0, 0);
                }
#pragma unroll
                for (int j = 0; j < LB; ++j) {
                    const bool before = (c + j * nseg) < lc;
                    const uint32_t w4[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int lo = (int)(w4[e] & 0xFFFFu), hi = (int)(w4[e] >> 16);
                        tl[2 * e] += lo;
                        tl[2 * e + 1] += hi;
                        if (before) { pl[2 * e] += lo; pl[2 * e + 1] += hi; }
                    }
                }
            }
        }
#pragma unroll
        for (int j = 0; j < KPT_; ++j) cntv[j] = (tid + j * TH < K) ? a.cnt[kb0 + tid + j * TH] : 0;
    }

    // ---- LDS set-up while the loads fly
    for (int w = tid; w < NW * kwp; w += TH) wh[w] = 0u;
    if (r > 0)
        for (int k = tid; k < 2 * a.kcap; k += TH) smem[k] = 0;
    if (tid == 0) placed_ct = 0;
    if (r == 0) {
        if (tid == 0) {
            compute_cfg(a, ci.b, box, cfg);   // a hundred-odd instructions on one lane
            if (lc == 0) reinterpret_cast<ScanCfg*>(a.cfg)[ci.b] = cfg;   // later steps load it
        }
    } else if (tid < CFGW) {
        reinterpret_cast<uint32_t*>(&cfg)[tid] = cfgw;
    }
    __syncthreads();
    if (r > 0) {
        if (seg < nseg) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int k = 8 * g + e;
                if (k < K) {
                    if (tl[e]) atomicAdd(&tot[k], tl[e]);
                    if (pl[e]) atomicAdd(&pre[k], pl[e]);
                }
            }
        }
        __syncthreads();
        // fill level before step r-1 plus earlier chunks' contenders = first rank of this chunk's contenders;
        // chunk 0 of the scan also publishes the fill level after step r-1
#pragma unroll
        for (int j = 0; j < KPT_; ++j) {
            const int k = tid + j * TH;
            if (k < K) {
                const int base = cntv[j];
                if (lc == 0) a.cnt_next[kb0 + k] = min(base + tot[k], k == K - 1 ? cfg.lastcap : a.S);
                pre[k] += base;
            }
        }
        __syncthreads();
    }

    const int keybits = last_step ? 0 : max(1, 32 - __clz(max(K - 1, 1)));
    int hh[PPT], wl[PPT];
    bool act[PPT];
    int nplaced = 0;
    // accept what fits from step r-1, hash what is left for step r
#pragma unroll
    for (int s = 0; s < PPT; ++s) {
        const int i = ci.begin + wave * (FCH / NW) + s * 64 + lane;
        bool active = i < ci.end;
        int h = 0;
        if (active && r > 0) {
            const uint32_t kv = kwv[s];
            if (kv == KEY_PLACED) {
                active = false;
            } else {
                const int hp = (int)(kv >> LR_BITS), lr = (int)(kv & ((1u << LR_BITS) - 1));
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
            int x = voxel_of(cx[s], cfg.mn[0], a.inv_voxel);
            int y = voxel_of(cy[s], cfg.mn[1], a.inv_voxel);
            int z = voxel_of(cz[s], cfg.mn[2], a.inv_voxel);
            if (r > 0) probe_voxel(a, r, cfg, x, y, z);
            h = hash_bucket(a.hash, x, y, z, cfg);
        }
        act[s] = active;
        hh[s] = h;
    }
    // rank inside the chunk: ballots inside the wave, per-wave LDS counters across the wave's four steps
#pragma unroll
    for (int s = 0; s < PPT; ++s) {
        const int h = hh[s];
        const bool active = act[s];
        const unsigned long long m = match_key(h, active, keybits);
        int old = 0;
        if (active) {
            const int leader = __ffsll((long long)m) - 1;
            const int before = __popcll(m & ((1ull << lane) - 1ull));
            if (lane == leader) {
                const int sh = (h & 1) * 16;
                const uint32_t o = atomicAdd(&wh[wave * kwp + (h >> 1)], (uint32_t)__popcll(m) << sh);
                old = (int)((o >> sh) & 0xFFFFu);
            }
            old = __shfl(old, leader, 64) + before;
        }
        if (!active) hh[s] = -1;
        wl[s] = old;
    }
    __syncthreads();
    // join the waves: exclusive prefix over the waves per bucket; the total is this chunk's row
    if (!last_step) {
        for (int w = tid; w < kwp; w += TH) {
            uint32_t run = 0;
            if (2 * w < K) {
#pragma unroll
                for (int v = 0; v < NW; ++v) {
                    const uint32_t t = wh[v * kwp + w];
                    wh[v * kwp + w] = run;
                    run += t;  // halves cannot carry into each other: a chunk has 2048 points
                }
            }
            mat_cur[(size_t)chunk * kwp + w] = run;   // padding words of the row are written as zero
        }
    } else if (tid == 0) {
        uint32_t run = 0;
        for (int v = 0; v < NW; ++v) {
            const uint32_t t = wh[v * kwp];
            wh[v * kwp] = run;
            run += t;
        }
        a.left[chunk] = (int)(run & 0xFFFFu);
    }
    __syncthreads();
#pragma unroll
    for (int s = 0; s < PPT; ++s) {
        const int i = ci.begin + wave * (FCH / NW) + s * 64 + lane;
        if (hh[s] >= 0) {
            const int h = hh[s];
            const int base = (int)((wh[wave * kwp + (h >> 1)] >> ((h & 1) * 16)) & 0xFFFFu);
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
// recycle: the r-th leftover of a scan takes the r-th free slot (buckets ascending, slots ascending)
// dynamic LDS: freepre[kcap] + fill[kcap] ints
__global__ __launch_bounds__(FTH) void k_pshf_recycle(PshArgs a)
{
    extern __shared__ int smem[];
    __shared__ int lds[17];
    __shared__ int s_base;
    const int chunk = blockIdx.x;
    const ChunkInfo ci = load_chunk(a, chunk);
    if (ci.b < 0 || a.status[0]) return;
    const int tid = threadIdx.x;
    const int K = ci.K, kb0 = ci.kb0, lc = ci.lc;
    int* freepre = smem;
    int* fill = smem + a.kcap;
    // ---- all loads first
    const int my_left = a.left[chunk];
    int mine = 0;
    for (int c = tid; c < lc; c += FTH) mine += a.left[ci.c0 + c];
    int cntv[KPT];
#pragma unroll
    for (int j = 0; j < KPT; ++j) cntv[j] = (tid + j * FTH < K) ? a.cnt[kb0 + tid + j * FTH] : 0;
    uint32_t kv[FPPT];
#pragma unroll
    for (int s = 0; s < FPPT; ++s) {
        const int i = ci.begin + tid + s * FTH;
        kv[s] = i < ci.end ? a.key[i] : KEY_PLACED;
    }
    const int p0 = ci.begin - lc * FCH;
    const int nb = a.scan_p0[ci.b + 1] - p0;
    if (my_left == 0) return;   // uniform: nothing of this chunk is left over
    // leftovers of earlier chunks
    int tot;
    block_excl_scan(mine, &tot, lds);
    if (tid == 0) s_base = tot;
    // free slots per bucket, exclusive prefix
    int carry = 0;
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
        if (j * FTH < K) {
            const int k = tid + j * FTH;
            int v = 0;
            if (k < K) {
                v = ((k == K - 1) ? nb - (K - 1) * a.S : a.S) - cntv[j];
                fill[k] = cntv[j];
            }
            int t2;
            const int pre = block_excl_scan(v, &t2, lds);
            if (k < K) freepre[k] = carry + pre;
            carry += t2;
        }
    }
    __syncthreads();
    const int base = s_base;
    int placed = 0;
#pragma unroll
    for (int s = 0; s < FPPT; ++s) {
        const int i = ci.begin + tid + s * FTH;
        if (kv[s] == KEY_PLACED) continue;
        const int rank = base + (int)(kv[s] & ((1u << LR_BITS) - 1));
        int lo = 0, hi = K;  // largest j with freepre[j] <= rank
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (freepre[mid] <= rank) lo = mid; else hi = mid;
        }
        const int dst = p0 + lo * a.S + fill[lo] + (rank - freepre[lo]);
        if (dst < p0 || dst >= p0 + nb) continue;  // cannot happen while capacities add up to the scan size
        a.inv_perm[i] = dst;
        a.perm[dst] = i;
        ++placed;
    }
    // one atomic per workgroup: hundreds of waves adding to the same counter queue up behind each other
    for (int d = 32; d >= 1; d >>= 1) placed += __shfl_xor(placed, d, 64);
    __syncthreads();              // everybody is done with s_base
    if (tid == 0) s_base = 0;
    __syncthreads();
    if ((tid & 63) == 0 && placed) atomicAdd(&s_base, placed);
    __syncthreads();
    if (tid == 0 && s_base) atomicAdd(&a.round_count[a.n_probes + 1], s_base);
}

}  // namespace

bool psh_fast_eligible(long long max_scan_points, int kcap)
{
    const long long nc = (max_scan_points + FCH - 1) / FCH;
    return kcap <= FKMAX && nc * kcap <= FMATMAX;
}

size_t psh_fast_matrix_bytes(long long n, int n_scans, int kcap)
{
    return (size_t)2 * (size_t)(n / FCH + n_scans) * row_pitch(kcap) * 4;
}

hipError_t psh_fast_launch(const PshArgs& args, hipStream_t stream)
{
    PshArgs a = args;
    a.chunk = FCH;
    const int chunks = (int)(a.n / FCH) + a.n_scans;  // upper bound, surplus workgroups exit
    a.n_chunks_ub = chunks;
    if (a.n_scans <= SETUP_MAX_SCANS && a.n > 0) {
        k_pshf_setup<<<chunks, FTH, 0, stream>>>(a);
    } else {
        a.mmpart = nullptr;
        k_psh_meta<<<1, 1024, 0, stream>>>(a);
        if (a.n == 0) return hipGetLastError();
        k_pshf_minmax<<<chunks, FTH, 0, stream>>>(a);
    }
    const int kwp = row_pitch(a.kcap);
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) cus = 0;
    const bool wide = chunks <= cus;   // one workgroup per CU at most: take the 1024-thread form
    const int nw = wide ? 16 : 8;
    const size_t lds = (size_t)a.kcap * 8 + (size_t)nw * kwp * 4;
    if (lds > 60000) {
        const hipError_t e = wide ? hipFuncSetAttribute((const void*)k_pshf_step<1024>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)
                                  : hipFuncSetAttribute((const void*)k_pshf_step<512>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    uint32_t* mat[2] = {reinterpret_cast<uint32_t*>(a.hist), reinterpret_cast<uint32_t*>(a.hist) + (size_t)chunks * kwp};
    int32_t* c0 = a.cnt;
    int32_t* c1 = a.cnt_next;
    for (int r = 0; r <= a.n_probes + 1; ++r) {
        a.cnt = c0;
        a.cnt_next = c1;
        if (wide) k_pshf_step<1024><<<chunks, 1024, lds, stream>>>(a, r, mat[(r + 1) & 1], mat[r & 1]);
        else k_pshf_step<512><<<chunks, 512, lds, stream>>>(a, r, mat[(r + 1) & 1], mat[r & 1]);
        if (r > 0) { int32_t* t = c0; c0 = c1; c1 = t; }  // step r wrote the fill levels after step r-1
    }
    a.cnt = c0;
    k_pshf_recycle<<<chunks, FTH, (size_t)a.kcap * 8, stream>>>(a);
    return hipGetLastError();
}

}  // namespace f3d

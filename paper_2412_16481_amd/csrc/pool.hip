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
    if (tid == 0) bad = 0;
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

// dynamic LDS, kp = a.kp: px,py,pz [PT] floats | o4 [kp] float4 (x, y, z, -) | fill [kp] ints | wcnt [PW][kp] u16 |
// open_list, id_of_hash, first_idx, ktot [kp] u16 each | members [PT + POOL_MAX_RHO] u16 | pick, rsub, rslot [PT] u16
__global__ __launch_bounds__(PT) void k_pool(PoolArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __shared__ int lds[17];
    __shared__ uint32_t red[8];
    __shared__ ScanCfg cfg;
    const int4 ti = a.tile_info[blockIdx.x];
    const int n = ti.y;
    if (n <= 0) return;
    const int row0 = ti.x, out0 = ti.z;
    const int rho = a.rho, kp = a.kp;
    const int M = (n + rho - 1) / rho;
    const int tid = threadIdx.x, lane = tid & 63;
    float* px = reinterpret_cast<float*>(smem);
    float* py = px + PT;
    float* pz = py + PT;
    float4* o4 = reinterpret_cast<float4*>(pz + PT);   // first-row position of every open sub-bucket: one 16-byte read
    int* fill = reinterpret_cast<int*>(o4 + kp);
    uint16_t* wcnt = reinterpret_cast<uint16_t*>(fill + kp);
    uint16_t* open_list = wcnt + PW * kp;
    uint16_t* id_of_hash = open_list + kp;
    uint16_t* first_idx = id_of_hash + kp;
    uint16_t* ktot = first_idx + kp;
    uint16_t* members = ktot + kp;
    uint16_t* pick = members + PT + POOL_MAX_RHO;   // [PT] choice of the t-th row left
    uint16_t* rsub = pick + PT;                      // [PT] sub-bucket it joined (0xFFFF: none yet) and its slot
    uint16_t* rslot = rsub + PT;

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
    }
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
    bool left = act && sub < 0;
    // ---- rounds: every row still left picks the open sub-bucket whose first row is nearest (state at the start of
    //      the round); the contenders of a sub-bucket join in row order while it has room. While many rows are
    //      left the whole workgroup takes the round (a row per thread). The long tail of rounds with at most 64
    //      rows left is run by wave 0 alone, without workgroup barriers: its lanes hold the rows in row order.
    int lpos = 0, nleft = 0, nopen = 0;
    uint16_t* left_list = members;   // [PT] thread ids of the rows still left, in row order (members is filled last)
    for (int round = 0; round <= PT; ++round) {   // every round places at least one row; the bound is a safeguard
        // one scan builds both lists: the rows still left (low half) and the sub-buckets with room (high half)
        __syncthreads();   // the fill levels written by the steps above / the last round are in place
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
        __syncthreads();
        if (nleft <= 64) break;
        // the rows left are spread over all threads again: g neighbouring lanes share one row's search
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
            // candidates per trip, their reads issued together: the loop is bound by instruction issue and LDS latency.
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
        const bool dense = tid < nleft;   // thread t now speaks for the t-th row left: row order is kept
        const int best = dense ? (int)pick[tid] : 0;
        const int rank = block_rank_by_key(best, dense, keybits, M, wcnt, kp, nullptr);
        const bool join = dense && fill[best] + rank < rho;
        if (dense) {
            rsub[tid] = join ? (uint16_t)best : (uint16_t)0xFFFF;
            rslot[tid] = (uint16_t)(fill[best] + rank);
        }
        __syncthreads();   // every fill level has been read, every answer is written
        if (join) atomicAdd(&fill[best], 1);
        if (left && rsub[lpos] != 0xFFFF) {
            sub = rsub[lpos];
            slot = rslot[lpos];
            left = false;
        }
    }
    if (nleft > 0 && nleft <= 64) {
        // wave 0 takes the rows that are left (left_list, in row order) and the open list of this moment
        uint16_t* tail_id = left_list;
        uint16_t* res_sub = rsub;
        uint16_t* res_slot = rslot;
        if (tid < 64) {
            const int L = nleft;
            bool tl = lane < L;
            const int me = tl ? (int)tail_id[lane] : 0;
            const float qx0 = px[me], qy0 = py[me], qz0 = pz[me];
            const unsigned long long lt = (1ull << lane) - 1ull;
            int tsub = 0, tslot = 0, O = nopen;
            for (int round = 0; round <= 64 && O > 0; ++round) {
                const unsigned long long leftmask = __ballot(tl);
                if (leftmask == 0ull) break;
                // drop the sub-buckets that filled up (in place: a chunk is read before anything of it is overwritten)
                int newO = 0;
                for (int base = 0; base < O; base += 64) {
                    const int c = base + lane;
                    int s = 0;
                    float4 co = make_float4(0.f, 0.f, 0.f, 0.f);
                    bool keep = false;
                    if (c < O) {
                        s = open_list[c];
                        co = o4[c];
                        keep = fill[s] < rho;
                    }
                    const unsigned long long bal = __ballot(keep);
                    if (keep) {
                        const int p = newO + __popcll(bal & lt);
                        open_list[p] = (uint16_t)s;
                        o4[p] = co;
                    }
                    newO += __popcll(bal);
                }
                O = newO;
                __threadfence_block();
                if (O == 0) break;
                // nearest open sub-bucket of this lane's row (ascending id: a tie keeps the lower one)
                int mybest = 0;
                if (tl) {
                    const float4 o = o4[0];   // O > 0: the first candidate unconditionally, later ones if strictly nearer
                    float bd = dist2(qx0 - o.x, qy0 - o.y, qz0 - o.z);
                    int bj = 0;
                    int c = 1;
                    for (; c + 3 < O; c += 4) {   // four candidates per trip, reads first (as in the rounds above)
                        float4 v4[4];
#pragma unroll
                        for (int u = 0; u < 4; ++u) v4[u] = o4[c + u];
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            const float d2 = dist2(qx0 - v4[u].x, qy0 - v4[u].y, qz0 - v4[u].z);
                            if (d2 < bd) { bd = d2; bj = c + u; }
                        }
                    }
                    for (; c < O; ++c) {
                        const float4 v = o4[c];
                        const float d2 = dist2(qx0 - v.x, qy0 - v.y, qz0 - v.z);
                        if (d2 < bd) { bd = d2; bj = c; }
                    }
                    mybest = open_list[bj];
                }
                const unsigned long long m = match_key(mybest, tl, keybits);
                const int rank = __popcll(m & lt);
                const int room = tl ? rho - fill[mybest] : 0;
                const bool join = tl && rank < room;
                if (join) {
                    tsub = mybest;
                    tslot = fill[mybest] + rank;
                }
                __threadfence_block();   // every lane has read the fill levels
                if (tl && rank == 0) fill[mybest] += min((int)__popcll(m), room);
                __threadfence_block();
                tl = tl && !join;
            }
            if (lane < L) {
                res_sub[lane] = (uint16_t)tsub;
                res_slot[lane] = (uint16_t)tslot;
            }
        }
        __syncthreads();
        if (left) {
            sub = res_sub[lpos];
            slot = res_slot[lpos];
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
}

size_t pool_lds_bytes(int kp)
{
    return (size_t)3 * PT * 4 + (size_t)4 * kp * 4 + (size_t)kp * 4 + (size_t)PW * kp * 2 + (size_t)4 * kp * 2 +
           (size_t)(PT + POOL_MAX_RHO) * 2 + (size_t)3 * PT * 2;
}

}  // namespace

hipError_t pool_launch(const PoolArgs& a, hipStream_t stream)
{
    k_pool_meta<<<1, 1024, 0, stream>>>(a);
    if (a.n == 0) return hipGetLastError();
    const size_t lds = pool_lds_bytes(a.kp);
    if (lds > 60000) {
        const hipError_t e = hipFuncSetAttribute((const void*)k_pool, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    k_pool<<<a.n_tiles_ub, PT, lds, stream>>>(a);
    return hipGetLastError();
}

}  // namespace f3d

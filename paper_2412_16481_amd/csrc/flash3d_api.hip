// C ABI of the library: argument checks on the host, workspace carving, kernel launches.
// Declarations and the meaning of every argument are in include/flash3d.h.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <string.h>

#include <atomic>

#include "attn.h"
#include "flash3d.h"
#include "linear.h"
#include "pool.h"
#include "order.h"
#include "psh.h"

// Workspace of f3d_psh_bucketize_static: device memory that exists as soon as the code object is loaded on a GPU, so
// that entry point never allocates. Every GPU holds its own copy at its own address. In host code the name `scratch`
// is only a handle for hipGetSymbolAddress; the address kernels can use is asked for once per device and kept.
static __device__ __align__(256) unsigned char scratch[F3D_STATIC_SCRATCH_BYTES];

namespace {

thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e)
{
    g_last_hip_error = (int)e;
    return F3D_ERR_HIP;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

constexpr int MAX_DEVICES = 64;
std::atomic<char*> g_scratch_ptr[MAX_DEVICES];

int static_scratch(char** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= MAX_DEVICES) return F3D_ERR_UNSUPPORTED;
    char* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        // the current device is `dev`: the address returned is that of this GPU's copy of the array
        void* sym = nullptr;
        e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e);
        if (!sym || ((uintptr_t)sym & 255)) return F3D_ERR_BAD_ALIGNMENT;
        ptr = (char*)sym;
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);   // two threads racing here store the same value
    }
    *out = ptr;
    return F3D_OK;
}

struct Plan {
    int S;
    int kcap;
    long long max_scan_points;
    long long max_buckets;
    long long chunks;
    size_t bytes;
    // offsets (bytes) of the workspace arrays
    size_t o_status, o_p0, o_c0, o_mm, o_cnt, o_cnt2, o_hist, o_key, o_left, o_leftpre, o_freepre, o_inv, o_rc, o_cfg, o_done, o_ci, o_mmpart;
    // canonical order only
    size_t o_obox, o_owords, o_oidx0, o_oidx1, o_ohist, o_ocoords, o_operm;
    // one workgroup per scan only: the two lists of points still unplaced (index, packed voxel)
    bool scans;
    size_t o_lidx0, o_lidx1, o_lvox0, o_lvox1;
};

int check_params(int64_t n, int32_t n_scans, const f3d_params* p)
{
    if (!p || p->struct_size != sizeof(f3d_params)) return F3D_ERR_INVALID_ARG;
    if (n < 0 || n_scans < 1) return F3D_ERR_INVALID_ARG;
    if (!(p->voxel_size > 0.0f) || !isfinite(p->voxel_size)) return F3D_ERR_INVALID_ARG;
    if (p->scope_buckets < 1 || p->bucket_cap < 1) return F3D_ERR_INVALID_ARG;
    if (p->hash < 0 || p->hash > 3) return F3D_ERR_INVALID_ARG;
    if (p->n_probes < 0 || p->n_probes > F3D_MAX_PROBES) return F3D_ERR_INVALID_ARG;
    if (p->div < 0 || p->probe_step < 0 || p->max_scan_points < 0) return F3D_ERR_INVALID_ARG;
    if (p->schedule < F3D_SCHEDULE_AUTO || p->schedule > F3D_SCHEDULE_SCANS) return F3D_ERR_INVALID_ARG;
    if (p->order < F3D_ORDER_INDEX || p->order > F3D_ORDER_CANONICAL) return F3D_ERR_INVALID_ARG;
    if (p->probe_mode < F3D_PROBE_AXES || p->probe_mode > F3D_PROBE_SEEDED) return F3D_ERR_INVALID_ARG;
    if (p->bucket_cap % (16 * p->scope_buckets) != 0) return F3D_ERR_INVALID_ARG;
    if (p->scope_buckets > F3D_MAX_SCOPE_BUCKETS) return F3D_ERR_UNSUPPORTED;
    if (n >= (int64_t)2147483647 - (1 << 20)) return F3D_ERR_UNSUPPORTED;
    if (n_scans > 65535) return F3D_ERR_UNSUPPORTED;
    const long long S = p->bucket_cap / p->scope_buckets;
    long long msp = p->max_scan_points > 0 ? p->max_scan_points : n;
    if (msp > n) msp = n;
    if ((msp + S - 1) / S > F3D_MAX_SCAN_BUCKETS) return F3D_ERR_UNSUPPORTED;
    return F3D_OK;
}

// One workgroup per scan pays when the scans themselves fill the GPU. Measured on an MI355X: that path needs about
// 10.4 ns per point of the LARGEST scan and per round of 256 scans (a workgroup walks its scan alone; with more scans
// than compute units two workgroups share one and a round is about 15 % shorter than this), the paths that spread a
// scan over the GPU about 0.13 ms plus 0.125 ns per point of the whole batch.
bool wants_scans(int64_t n, int32_t n_scans, const f3d_params* p, long long max_scan_points, int kcap)
{
    if (!f3d::psh_scan_eligible(kcap)) return false;
    if (p->schedule == F3D_SCHEDULE_SCANS) return true;
    if (p->schedule != F3D_SCHEDULE_AUTO || n_scans < 48) return false;
    const double rounds = (double)((n_scans + 255) / 256);
    const double t_scans = rounds * (double)max_scan_points * 10.4e-9 + 0.02e-3;
    const double t_spread = 0.13e-3 + (double)n * 0.125e-9;
    return t_scans < t_spread;
}

void make_plan(int64_t n, int32_t n_scans, const f3d_params* p, Plan* pl)
{
    pl->S = p->bucket_cap / p->scope_buckets;
    long long msp = p->max_scan_points > 0 ? p->max_scan_points : n;
    if (msp > n) msp = n;
    pl->max_scan_points = msp;
    long long kcap = (msp + pl->S - 1) / pl->S;
    if (kcap < 1) kcap = 1;
    pl->kcap = (int)kcap;
    pl->max_buckets = n / pl->S + n_scans;
    pl->chunks = n / f3d::PSH_CHUNK + n_scans;
    size_t at = 0;
    auto take = [&](size_t bytes) { size_t o = at; at = align_up(at + bytes, 256); return o; };
    pl->o_status = take(16);
    pl->o_rc = take(8 * 4);
    pl->o_p0 = take((size_t)(n_scans + 1) * 4);
    pl->o_c0 = take((size_t)(n_scans + 1) * 4);
    pl->o_mm = take((size_t)n_scans * 8 * 4);
    pl->o_cfg = take((size_t)n_scans * 128);
    pl->o_done = take((size_t)n_scans * 4);
    pl->o_ci = take((size_t)(n / 2048 + n_scans) * 32);
    pl->o_mmpart = take((size_t)(n / 2048 + n_scans) * 32);
    pl->o_cnt = take((size_t)(pl->max_buckets + 1) * 4);
    pl->o_cnt2 = take((size_t)(pl->max_buckets + 1) * 4);
    pl->o_freepre = take((size_t)(pl->max_buckets + 1) * 4);
    pl->o_left = take((size_t)pl->chunks * 4);
    pl->o_leftpre = take((size_t)pl->chunks * 4);
    {
        size_t hb = (size_t)pl->chunks * pl->kcap * 4;
        const size_t fb = f3d::psh_fast_matrix_bytes(n, n_scans, pl->kcap);
        pl->o_hist = take(hb > fb ? hb : fb);
    }
    pl->o_key = take((size_t)n * 4);
    pl->o_inv = take((size_t)n * 4);
    if (p->order == F3D_ORDER_CANONICAL) {
        pl->o_obox = take((size_t)n_scans * 16);
        pl->o_owords = take((size_t)n * 24);
        pl->o_oidx0 = take((size_t)n * 4);
        pl->o_oidx1 = take((size_t)n * 4);
        pl->o_ohist = take(f3d::order_hist_bytes(n));
        pl->o_ocoords = take((size_t)n * 12);
        pl->o_operm = take((size_t)n * 4);
    }
    pl->scans = wants_scans(n, n_scans, p, pl->max_scan_points, pl->kcap);
    if (pl->scans) {
        pl->o_lidx0 = take((size_t)n * 4);
        pl->o_lidx1 = take((size_t)n * 4);
        pl->o_lvox0 = take((size_t)n * 8);
        pl->o_lvox1 = take((size_t)n * 8);
    }
    pl->bytes = at;
}

__global__ void k_unpermute16(const uint4* __restrict__ src, const int32_t* __restrict__ perm, long long n, int vec_per_row,
                              uint4* __restrict__ dst)
{
    const long long total = n * vec_per_row;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
        const long long p = i / vec_per_row;
        const int c = (int)(i - p * vec_per_row);
        dst[(long long)perm[p] * vec_per_row + c] = src[i];
    }
}

__global__ void k_unpermute4(const uint32_t* __restrict__ src, const int32_t* __restrict__ perm, long long n, int w_per_row,
                             uint32_t* __restrict__ dst)
{
    const long long total = n * w_per_row;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
        const long long p = i / w_per_row;
        const int c = (int)(i - p * w_per_row);
        dst[(long long)perm[p] * w_per_row + c] = src[i];
    }
}

}  // namespace

extern "C" {

void f3d_params_default(f3d_params* p, float voxel_size, int32_t bucket_cap)
{
    if (!p) return;
    memset(p, 0, sizeof(*p));
    p->struct_size = sizeof(f3d_params);
    p->voxel_size = voxel_size;
    p->bucket_cap = bucket_cap;
    p->scope_buckets = 4;
    p->hash = F3D_HASH_ZORDER_DIV;
    p->n_probes = F3D_MAX_PROBES;
}

int64_t f3d_max_buckets(int64_t n, int32_t n_scans, const f3d_params* p)
{
    if (check_params(n, n_scans, p) != F3D_OK) return -1;
    return n / (p->bucket_cap / p->scope_buckets) + n_scans;
}

int f3d_workspace_bytes(int64_t n, int32_t n_scans, const f3d_params* p, size_t* out_bytes)
{
    if (!out_bytes) return F3D_ERR_INVALID_ARG;
    const int rc = check_params(n, n_scans, p);
    if (rc != F3D_OK) return rc;
    Plan pl;
    make_plan(n, n_scans, p, &pl);
    *out_bytes = pl.bytes;
    return F3D_OK;
}

// Checks that need no workspace: parameters, required pointers, alignment of the caller's arrays.
static int check_bucketize_args(const float* coords, const int32_t* batch_offsets, int64_t n, int32_t n_scans, const f3d_params* p,
                                int32_t* perm, int32_t* inv_perm, int32_t* offsets, int32_t* scan_bucket_start,
                                int32_t* placed_per_round)
{
    const int rc = check_params(n, n_scans, p);
    if (rc != F3D_OK) return rc;
    if (!offsets || !scan_bucket_start) return F3D_ERR_INVALID_ARG;
    if (n > 0 && (!coords || !perm)) return F3D_ERR_INVALID_ARG;
    if (((uintptr_t)coords | (uintptr_t)batch_offsets | (uintptr_t)perm | (uintptr_t)inv_perm | (uintptr_t)offsets |
         (uintptr_t)scan_bucket_start | (uintptr_t)placed_per_round) & 3)
        return F3D_ERR_BAD_ALIGNMENT;
    return F3D_OK;
}

// Carves the workspace (device memory of at least pl.bytes, 256-byte aligned) and launches the bucketing kernels.
static int bucketize_on(const Plan& pl, char* ws, const float* coords, const int32_t* batch_offsets, int64_t n, int32_t n_scans,
                        const f3d_params* p, int32_t* perm, int32_t* inv_perm, int32_t* offsets, int32_t* scan_bucket_start,
                        int32_t* placed_per_round, void* stream)
{
    f3d::PshArgs a;
    memset(&a, 0, sizeof(a));
    a.coords = coords;
    a.batch_offsets = batch_offsets;
    a.n = (int)n;
    a.n_scans = n_scans;
    a.inv_voxel = 1.0f / p->voxel_size;
    a.S = pl.S;
    a.hash = p->hash;
    a.n_probes = p->n_probes;
    a.div = p->div;
    a.step = p->probe_step;
    a.probe_mode = p->probe_mode;
    a.probe_seed = p->probe_seed;
    for (int i = 0; i < 3 * F3D_MAX_PROBES; ++i) a.probe_table[i] = p->probe_table[i];
    a.kcap = pl.kcap;
    a.max_scan_points = pl.max_scan_points;
    a.max_buckets = (int)pl.max_buckets;
    a.perm = perm;
    a.inv_perm = inv_perm ? inv_perm : (int32_t*)(ws + pl.o_inv);
    a.offsets = offsets;
    a.sbs = scan_bucket_start;
    a.round_count = placed_per_round ? placed_per_round : (int32_t*)(ws + pl.o_rc);
    a.status = (int32_t*)(ws + pl.o_status);
    a.scan_p0 = (int32_t*)(ws + pl.o_p0);
    a.scan_c0 = (int32_t*)(ws + pl.o_c0);
    a.mm = (uint32_t*)(ws + pl.o_mm);
    a.mmpart = (uint32_t*)(ws + pl.o_mmpart);
    a.cnt = (int32_t*)(ws + pl.o_cnt);
    a.cnt_next = (int32_t*)(ws + pl.o_cnt2);
    a.hist = (int32_t*)(ws + pl.o_hist);
    a.key = (uint32_t*)(ws + pl.o_key);
    a.left = (int32_t*)(ws + pl.o_left);
    a.leftpre = (int32_t*)(ws + pl.o_leftpre);
    a.freepre = (int32_t*)(ws + pl.o_freepre);
    a.cfg = (void*)(ws + pl.o_cfg);
    a.done = (int32_t*)(ws + pl.o_done);
    a.chunk_info = (int4*)(ws + pl.o_ci);
    (void)hipGetLastError();  // a stale error left by an earlier, unrelated runtime call is not ours
    const bool fast_ok = f3d::psh_fast_eligible(pl.max_scan_points, pl.kcap);
    int schedule = p->schedule;
    if (schedule == F3D_SCHEDULE_SCANS && !pl.scans) return F3D_ERR_UNSUPPORTED;
    if (pl.scans) schedule = F3D_SCHEDULE_SCANS;
    if (schedule == F3D_SCHEDULE_AUTO) schedule = fast_ok ? F3D_SCHEDULE_STEPS : F3D_SCHEDULE_GENERAL;
    if (schedule == F3D_SCHEDULE_STEPS && !fast_ok) return F3D_ERR_UNSUPPORTED;
    // canonical order: sort the points, bucket the sorted copy by index, map the result back through the sort
    const int32_t* order = nullptr;
    if (p->order == F3D_ORDER_CANONICAL) {
        f3d::OrderArgs o;
        memset(&o, 0, sizeof(o));
        o.coords = coords;
        o.batch_offsets = batch_offsets;
        o.n = (int)n;
        o.n_scans = n_scans;
        o.inv_voxel = a.inv_voxel;
        o.box = (uint32_t*)(ws + pl.o_obox);
        o.words = (uint32_t*)(ws + pl.o_owords);
        o.idx[0] = (int32_t*)(ws + pl.o_oidx0);
        o.idx[1] = (int32_t*)(ws + pl.o_oidx1);
        o.hist = (uint32_t*)(ws + pl.o_ohist);
        o.coords_sorted = (float*)(ws + pl.o_ocoords);
        const hipError_t eo = f3d::order_launch(o, &order, (hipStream_t)stream);
        if (eo != hipSuccess) return hip_fail(eo);
        a.coords = o.coords_sorted;
        a.perm = (int32_t*)(ws + pl.o_operm);
        a.inv_perm = (int32_t*)(ws + pl.o_inv);
    }
    hipError_t e;
    if (schedule == F3D_SCHEDULE_SCANS)
        e = f3d::psh_scan_launch(a, (int32_t*)(ws + pl.o_lidx0), (int32_t*)(ws + pl.o_lidx1), (unsigned long long*)(ws + pl.o_lvox0),
                                 (unsigned long long*)(ws + pl.o_lvox1), (hipStream_t)stream);
    else
        e = schedule == F3D_SCHEDULE_GENERAL ? f3d::psh_launch(a, (hipStream_t)stream) : f3d::psh_fast_launch(a, (hipStream_t)stream);
    if (e == hipSuccess && order)
        e = f3d::order_compose_launch(order, a.perm, a.inv_perm, (int)n, a.status, perm, inv_perm, (hipStream_t)stream);
    return e == hipSuccess ? F3D_OK : hip_fail(e);
}

int f3d_psh_bucketize(const float* coords, const int32_t* batch_offsets, int64_t n, int32_t n_scans, const f3d_params* p,
                      int32_t* perm, int32_t* inv_perm, int32_t* offsets, int32_t* scan_bucket_start,
                      int32_t* placed_per_round, void* workspace, size_t workspace_bytes, void* stream)
{
    const int rc = check_bucketize_args(coords, batch_offsets, n, n_scans, p, perm, inv_perm, offsets, scan_bucket_start,
                                        placed_per_round);
    if (rc != F3D_OK) return rc;
    if (!workspace) return F3D_ERR_INVALID_ARG;
    if ((uintptr_t)workspace & 255) return F3D_ERR_BAD_ALIGNMENT;
    Plan pl;
    make_plan(n, n_scans, p, &pl);
    if (workspace_bytes < pl.bytes) return F3D_ERR_WORKSPACE_TOO_SMALL;
    return bucketize_on(pl, (char*)workspace, coords, batch_offsets, n, n_scans, p, perm, inv_perm, offsets, scan_bucket_start,
                        placed_per_round, stream);
}

int f3d_psh_bucketize_static(const float* coords, const int32_t* batch_offsets, int64_t n, int32_t n_scans, const f3d_params* p,
                             int32_t* perm, int32_t* inv_perm, int32_t* offsets, int32_t* scan_bucket_start,
                             int32_t* placed_per_round, void* stream)
{
    const int rc = check_bucketize_args(coords, batch_offsets, n, n_scans, p, perm, inv_perm, offsets, scan_bucket_start,
                                        placed_per_round);
    if (rc != F3D_OK) return rc;
    Plan pl;
    make_plan(n, n_scans, p, &pl);
    if (pl.bytes > (size_t)F3D_STATIC_SCRATCH_BYTES) return F3D_ERR_SCRATCH_LIMIT;
    char* ws = nullptr;
    const int rs = static_scratch(&ws);
    if (rs != F3D_OK) return rs;
    return bucketize_on(pl, ws, coords, batch_offsets, n, n_scans, p, perm, inv_perm, offsets, scan_bucket_start,
                        placed_per_round, stream);
}

// argument checks and the launch geometry shared by the forward and backward attention calls
static int fill_attn_args(f3d::AttnArgs& a, const void* q, const void* k, const void* v, const int32_t* perm, const int32_t* offsets,
                          const int32_t* scan_bucket_start, int64_t n, int32_t n_scans, int64_t max_buckets, int32_t bucket_cap,
                          int32_t scope_buckets, int32_t mode, int32_t shift, int32_t stride, int32_t heads, int32_t head_dim,
                          float softmax_scale, float* scale_out, long long* slots_out)
{
    if (n < 0 || n_scans < 1 || heads < 1 || bucket_cap < 1 || scope_buckets < 1 || max_buckets < 0) return F3D_ERR_INVALID_ARG;
    if (mode < F3D_PLAIN || mode > F3D_STRIDE) return F3D_ERR_INVALID_ARG;
    if (bucket_cap % (16 * scope_buckets) != 0) return F3D_ERR_INVALID_ARG;
    if (mode == F3D_SHIFT && (shift <= 0 || shift >= scope_buckets)) return F3D_ERR_INVALID_ARG;
    if (mode == F3D_STRIDE && stride < 1) return F3D_ERR_INVALID_ARG;
    if (!(softmax_scale >= 0.0f) || !isfinite(softmax_scale)) return F3D_ERR_INVALID_ARG;
    if (head_dim != 16 && head_dim != 32) return F3D_ERR_UNSUPPORTED;
    if (scope_buckets > F3D_MAX_SCOPE_BUCKETS || stride > 4096 || n_scans > 65535) return F3D_ERR_UNSUPPORTED;
    if (n >= (int64_t)2147483647 - (1 << 20) || (long long)heads * head_dim > 65536) return F3D_ERR_UNSUPPORTED;
    if (!offsets || !scan_bucket_start) return F3D_ERR_INVALID_ARG;
    if (n > 0 && (!q || !k || !v)) return F3D_ERR_INVALID_ARG;
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v) & 15) return F3D_ERR_BAD_ALIGNMENT;
    if (((uintptr_t)perm | (uintptr_t)offsets | (uintptr_t)scan_bucket_start) & 3) return F3D_ERR_BAD_ALIGNMENT;
    memset(&a, 0, sizeof(a));
    a.q = (const uint16_t*)q;
    a.k = (const uint16_t*)k;
    a.v = (const uint16_t*)v;
    a.perm = perm;
    a.offsets = offsets;
    a.sbs = scan_bucket_start;
    a.n = (int)n;
    a.n_scans = n_scans;
    a.m = scope_buckets;
    a.mode = mode;
    a.shift = shift;
    a.stride = stride;
    a.H = heads;
    a.C = heads * head_dim;
    const float scale = softmax_scale > 0.0f ? softmax_scale : 1.0f / sqrtf((float)head_dim);
    a.c_log2 = scale * 1.44269504088896340736f;
    a.extra = mode == F3D_STRIDE ? stride + 1 : 2;
    *scale_out = scale;
    *slots_out = max_buckets / scope_buckets + (long long)a.extra * n_scans + 1;
    return F3D_OK;
}

static int attn_forward(int f16, const void* q, const void* k, const void* v, const int32_t* perm, const int32_t* offsets,
                        const int32_t* scan_bucket_start, int64_t n, int32_t n_scans, int64_t max_buckets, int32_t bucket_cap,
                        int32_t scope_buckets, int32_t mode, int32_t shift, int32_t stride, int32_t heads, int32_t head_dim,
                        float softmax_scale, void* out, const int32_t* out_perm, float* lse, void* stream)
{
    f3d::AttnArgs a;
    float scale;
    long long slots;
    const int rc = fill_attn_args(a, q, k, v, perm, offsets, scan_bucket_start, n, n_scans, max_buckets, bucket_cap, scope_buckets,
                                  mode, shift, stride, heads, head_dim, softmax_scale, &scale, &slots);
    if (rc != F3D_OK) return rc;
    if (n == 0) return F3D_OK;
    if (!out) return F3D_ERR_INVALID_ARG;
    if ((uintptr_t)out & 15) return F3D_ERR_BAD_ALIGNMENT;
    if (((uintptr_t)out_perm | (uintptr_t)lse) & 3) return F3D_ERR_BAD_ALIGNMENT;
    a.out = (uint16_t*)out;
    a.out_perm = out_perm;
    a.lse = lse;
    a.f16 = f16;
    const int bm = f3d::attn_block_rows(head_dim, slots, heads, bucket_cap);
    a.qblocks = (bucket_cap + bm - 1) / bm;
    if (slots * heads * a.qblocks > 2000000000ll) return F3D_ERR_UNSUPPORTED;
    a.n_slots = (int)slots;
    (void)hipGetLastError();
    const hipError_t e = f3d::attn_launch(a, head_dim, bm, (hipStream_t)stream);
    return e == hipSuccess ? F3D_OK : hip_fail(e);
}

int f3d_attn_block_rows(int64_t n_scans, int64_t max_buckets, int32_t bucket_cap, int32_t scope_buckets, int32_t mode,
                        int32_t stride, int32_t heads, int32_t head_dim)
{
    if (n_scans < 1 || max_buckets < 0 || bucket_cap < 1 || scope_buckets < 1 || heads < 1) return F3D_ERR_INVALID_ARG;
    if (mode < F3D_PLAIN || mode > F3D_STRIDE || (mode == F3D_STRIDE && stride < 1)) return F3D_ERR_INVALID_ARG;
    if (head_dim != 16 && head_dim != 32) return F3D_ERR_UNSUPPORTED;
    const long long extra = mode == F3D_STRIDE ? stride + 1 : 2;
    const long long slots = max_buckets / scope_buckets + extra * n_scans + 1;
    return f3d::attn_block_rows(head_dim, slots, heads, bucket_cap);
}

int f3d_bucket_swin_attn(const void* q, const void* k, const void* v, const int32_t* perm, const int32_t* offsets,
                         const int32_t* scan_bucket_start, int64_t n, int32_t n_scans, int64_t max_buckets,
                         int32_t bucket_cap, int32_t scope_buckets, int32_t mode, int32_t shift, int32_t stride, int32_t heads,
                         int32_t head_dim, float softmax_scale, void* out, const int32_t* out_perm, float* lse, void* stream)
{
    return attn_forward(0, q, k, v, perm, offsets, scan_bucket_start, n, n_scans, max_buckets, bucket_cap, scope_buckets, mode,
                        shift, stride, heads, head_dim, softmax_scale, out, out_perm, lse, stream);
}

int f3d_bucket_swin_attn_f16(const void* q, const void* k, const void* v, const int32_t* perm, const int32_t* offsets,
                             const int32_t* scan_bucket_start, int64_t n, int32_t n_scans, int64_t max_buckets,
                             int32_t bucket_cap, int32_t scope_buckets, int32_t mode, int32_t shift, int32_t stride, int32_t heads,
                             int32_t head_dim, float softmax_scale, void* out, const int32_t* out_perm, float* lse, void* stream)
{
    return attn_forward(1, q, k, v, perm, offsets, scan_bucket_start, n, n_scans, max_buckets, bucket_cap, scope_buckets, mode,
                        shift, stride, heads, head_dim, softmax_scale, out, out_perm, lse, stream);
}

int f3d_attn_bwd_workspace_bytes(int64_t n, int32_t heads, size_t* out_bytes)
{
    if (!out_bytes || n < 0 || heads < 1) return F3D_ERR_INVALID_ARG;
    *out_bytes = align_up((size_t)n * heads * sizeof(float), 256);
    return F3D_OK;
}

int f3d_bucket_swin_attn_bwd(const void* q, const void* k, const void* v, const void* out, const void* dout, const float* lse,
                             const int32_t* perm, const int32_t* offsets, const int32_t* scan_bucket_start, int64_t n,
                             int32_t n_scans, int64_t max_buckets, int32_t bucket_cap, int32_t scope_buckets, int32_t mode,
                             int32_t shift, int32_t stride, int32_t heads, int32_t head_dim, float softmax_scale, void* dq, void* dk,
                             void* dv, const int32_t* grad_perm, void* workspace, size_t workspace_bytes, void* stream)
{
    f3d::AttnBwdArgs b;
    memset(&b, 0, sizeof(b));
    float scale;
    long long slots;
    const int rc = fill_attn_args(b.f, q, k, v, perm, offsets, scan_bucket_start, n, n_scans, max_buckets, bucket_cap, scope_buckets,
                                  mode, shift, stride, heads, head_dim, softmax_scale, &scale, &slots);
    if (rc != F3D_OK) return rc;
    if (n == 0) return F3D_OK;
    if (!out || !dout || !lse || !dq || !dk || !dv || !workspace) return F3D_ERR_INVALID_ARG;
    if (((uintptr_t)out | (uintptr_t)dout | (uintptr_t)dq | (uintptr_t)dk | (uintptr_t)dv) & 15) return F3D_ERR_BAD_ALIGNMENT;
    if (((uintptr_t)lse | (uintptr_t)grad_perm) & 3) return F3D_ERR_BAD_ALIGNMENT;
    if ((uintptr_t)workspace & 255) return F3D_ERR_BAD_ALIGNMENT;
    size_t need = 0;
    f3d_attn_bwd_workspace_bytes(n, heads, &need);
    if (workspace_bytes < need) return F3D_ERR_WORKSPACE_TOO_SMALL;
    b.f.out = (uint16_t*)const_cast<void*>(out);
    b.f.lse = const_cast<float*>(lse);
    b.f.out_perm = grad_perm;
    b.dout = (const uint16_t*)dout;
    b.dsum = (float*)workspace;
    b.dq = (uint16_t*)dq;
    b.dk = (uint16_t*)dk;
    b.dv = (uint16_t*)dv;
    b.scale = scale;
    b.f.qblocks = (bucket_cap + 127) / 128;
    b.kblocks = b.f.qblocks;
    if (slots * heads * b.f.qblocks > 2000000000ll) return F3D_ERR_UNSUPPORTED;
    b.f.n_slots = (int)slots;
    (void)hipGetLastError();
    const hipError_t e = f3d::attn_bwd_launch(b, head_dim, (hipStream_t)stream);
    return e == hipSuccess ? F3D_OK : hip_fail(e);
}

int f3d_ln_linear(const void* x, const int32_t* row_in, const float* gamma, const float* beta, float eps, const void* w,
                  const float* bias, const void* residual, int64_t n, int32_t c_in, int32_t c_out, void* const* outs,
                  int32_t n_outs, const int32_t* row_out, void* stream)
{
    if (n < 0 || c_in < 1 || c_out < 1 || n_outs < 1 || !outs) return F3D_ERR_INVALID_ARG;
    if (n_outs > f3d::LIN_MAX_OUTS || (c_in != 64 && c_in != 128 && c_in != 256)) return F3D_ERR_UNSUPPORTED;
    if (c_out % 64 != 0 || c_out % n_outs != 0 || (c_out / n_outs) % 16 != 0 || c_out > 4096) return F3D_ERR_UNSUPPORTED;
    if (n >= (int64_t)2147483647 - (1 << 20)) return F3D_ERR_UNSUPPORTED;
    if (gamma && !(eps >= 0.0f && isfinite(eps))) return F3D_ERR_INVALID_ARG;
    if (!gamma && beta) return F3D_ERR_INVALID_ARG;
    if (n == 0) return F3D_OK;
    if (!x || !w) return F3D_ERR_INVALID_ARG;
    if (((uintptr_t)x | (uintptr_t)w | (uintptr_t)residual | (uintptr_t)gamma | (uintptr_t)beta | (uintptr_t)bias) & 15)
        return F3D_ERR_BAD_ALIGNMENT;
    if (((uintptr_t)row_in | (uintptr_t)row_out) & 3) return F3D_ERR_BAD_ALIGNMENT;
    f3d::LinearArgs a;
    memset(&a, 0, sizeof(a));
    for (int t = 0; t < n_outs; ++t) {
        if (!outs[t]) return F3D_ERR_INVALID_ARG;
        if ((uintptr_t)outs[t] & 15) return F3D_ERR_BAD_ALIGNMENT;
        a.outs[t] = (uint16_t*)outs[t];
    }
    a.x = (const uint16_t*)x;
    a.row_in = row_in;
    a.gamma = gamma;
    a.beta = beta;
    a.eps = eps;
    a.w = (const uint16_t*)w;
    a.bias = bias;
    a.residual = (const uint16_t*)residual;
    a.n = (int)n;
    a.c_in = c_in;
    a.c_out = c_out;
    a.n_outs = n_outs;
    a.row_out = row_out;
    (void)hipGetLastError();
    const hipError_t e = f3d::linear_launch(a, (hipStream_t)stream);
    return e == hipSuccess ? F3D_OK : hip_fail(e);
}

static int check_pool(int64_t n, int32_t n_scans, int32_t tile, int32_t rho)
{
    if (n < 0 || n_scans < 1 || tile < 1 || rho < 1) return F3D_ERR_INVALID_ARG;
    if (tile > F3D_POOL_MAX_TILE || rho > F3D_POOL_MAX_RHO) return F3D_ERR_UNSUPPORTED;
    if (n >= (int64_t)2147483647 - (1 << 20) || n_scans > 65535) return F3D_ERR_UNSUPPORTED;
    return F3D_OK;
}

int64_t f3d_pool_max_rows(int64_t n, int32_t n_scans, int32_t tile, int32_t rho)
{
    if (check_pool(n, n_scans, tile, rho) != F3D_OK) return -1;
    return n / rho + n / tile + n_scans + 1;
}

int f3d_pool_workspace_bytes(int64_t n, int32_t n_scans, int32_t tile, size_t* out_bytes)
{
    if (!out_bytes) return F3D_ERR_INVALID_ARG;
    const int rc = check_pool(n, n_scans, tile, 1);
    if (rc != F3D_OK) return rc;
    const size_t tiles = (size_t)(n / tile + n_scans);
    const size_t slots = tiles < (size_t)f3d::POOL_MAX_SLOTS ? tiles : (size_t)f3d::POOL_MAX_SLOTS;
    *out_bytes = align_up(tiles * sizeof(int4), 256) + 256 + align_up(slots * f3d::pool_list_entries(tile) * 2, 256);
    return F3D_OK;
}

int f3d_inbucket_pool(const float* coords, const int32_t* perm, const void* feat, const int32_t* batch_offsets, int64_t n,
                      int32_t n_scans, int32_t channels, int32_t tile, int32_t rho, float voxel_size, int32_t hash, int32_t op,
                      void* pooled_feat, float* pooled_coords, int32_t* sub_of, int32_t* pooled_offsets, void* workspace,
                      size_t workspace_bytes, void* stream)
{
    const int rc = check_pool(n, n_scans, tile, rho);
    if (rc != F3D_OK) return rc;
    if (channels < 8 || channels % 8 != 0) return F3D_ERR_INVALID_ARG;
    if (!(voxel_size > 0.0f) || !isfinite(voxel_size)) return F3D_ERR_INVALID_ARG;
    if (hash < 0 || hash > 3 || op < F3D_POOL_SUM || op > F3D_POOL_MAX) return F3D_ERR_INVALID_ARG;
    if (!pooled_offsets || !workspace) return F3D_ERR_INVALID_ARG;
    if (n > 0 && (!coords || !feat || !pooled_feat)) return F3D_ERR_INVALID_ARG;
    if (((uintptr_t)coords | (uintptr_t)perm | (uintptr_t)batch_offsets | (uintptr_t)pooled_coords | (uintptr_t)sub_of |
         (uintptr_t)pooled_offsets) & 3)
        return F3D_ERR_BAD_ALIGNMENT;
    if (((uintptr_t)feat | (uintptr_t)pooled_feat) & 15) return F3D_ERR_BAD_ALIGNMENT;
    if ((uintptr_t)workspace & 255) return F3D_ERR_BAD_ALIGNMENT;
    size_t need = 0;
    f3d_pool_workspace_bytes(n, n_scans, tile, &need);
    if (workspace_bytes < need) return F3D_ERR_WORKSPACE_TOO_SMALL;

    f3d::PoolArgs a;
    memset(&a, 0, sizeof(a));
    a.coords = coords;
    a.perm = perm;
    a.feat = (const uint16_t*)feat;
    a.batch_offsets = batch_offsets;
    a.n = (int)n;
    a.n_scans = n_scans;
    a.C = channels;
    a.tile = tile;
    a.rho = rho;
    a.inv_voxel = 1.0f / voxel_size;
    a.hash = hash;
    a.op = op;
    a.kp = ((tile + rho - 1) / rho + 63) / 64 * 64;
    a.n_tiles_ub = (int)(n / tile) + n_scans;
    a.pooled_feat = (uint16_t*)pooled_feat;
    a.pooled_coords = pooled_coords;
    a.sub_of = sub_of;
    a.pooled_offsets = pooled_offsets;
    a.tile_info = (int4*)workspace;
    a.tile_counter = (int*)((char*)workspace + align_up((size_t)a.n_tiles_ub * sizeof(int4), 256));
    a.lists = (uint16_t*)((char*)a.tile_counter + 256);
    a.list_cap = f3d::pool_list_entries(tile);
    a.n_slots = a.n_tiles_ub < f3d::POOL_MAX_SLOTS ? a.n_tiles_ub : f3d::POOL_MAX_SLOTS;
    (void)hipGetLastError();
    const hipError_t e = f3d::pool_launch(a, (hipStream_t)stream);
    return e == hipSuccess ? F3D_OK : hip_fail(e);
}

int f3d_unpermute(const void* src, const int32_t* perm, int64_t n, int32_t row_bytes, void* dst, void* stream)
{
    if (n < 0 || row_bytes <= 0 || (row_bytes & 3)) return F3D_ERR_INVALID_ARG;
    if (n == 0) return F3D_OK;
    if (!src || !perm || !dst || src == dst) return F3D_ERR_INVALID_ARG;
    if (((uintptr_t)src | (uintptr_t)dst | (uintptr_t)perm) & 3) return F3D_ERR_BAD_ALIGNMENT;
    (void)hipGetLastError();
    const bool wide = (row_bytes % 16 == 0) && ((((uintptr_t)src | (uintptr_t)dst) & 15) == 0);
    const long long units = n * (wide ? row_bytes / 16 : row_bytes / 4);
    long long blocks = (units + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    if (wide)
        k_unpermute16<<<(unsigned)blocks, 256, 0, (hipStream_t)stream>>>((const uint4*)src, perm, n, row_bytes / 16, (uint4*)dst);
    else
        k_unpermute4<<<(unsigned)blocks, 256, 0, (hipStream_t)stream>>>((const uint32_t*)src, perm, n, row_bytes / 4, (uint32_t*)dst);
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? F3D_OK : hip_fail(e);
}

const char* f3d_error_string(int code)
{
    switch (code) {
        case F3D_OK: return "ok";
        case F3D_ERR_INVALID_ARG: return "invalid argument";
        case F3D_ERR_BAD_ALIGNMENT: return "pointer or row size not aligned as required";
        case F3D_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case F3D_ERR_UNSUPPORTED: return "request outside the implemented limits";
        case F3D_ERR_HIP: return "HIP runtime error";
        case F3D_ERR_SCRATCH_LIMIT: return "input needs more scratch memory than the built-in buffer of f3d_psh_bucketize_static holds";
        default: return "unknown error code";
    }
}

int f3d_last_hip_error(void) { return g_last_hip_error; }

int f3d_version(void) { return 1; }

}  // extern "C"

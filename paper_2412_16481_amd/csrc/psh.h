// Internal interface between the C ABI (flash3d_api.hip) and the bucketing kernels (psh.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace f3d {

constexpr int PSH_CHUNK = 1024;   // points one workgroup ranks
constexpr int PSH_THREADS = 256;
constexpr int PSH_WAVES = PSH_THREADS / 64;
constexpr int F3D_VOXEL_MAX = (1 << 21) - 1;

struct PshArgs {
    // inputs
    const float* coords;
    const int32_t* batch_offsets;  // may be null: one scan
    int n;
    int n_scans;
    float inv_voxel;
    int S;       // bucket capacity
    int hash;
    int n_probes;
    int div;
    int step;
    int probe_mode;          // 0 axis neighbours, 1 table, 2 seeded per-voxel direction
    uint32_t probe_seed;
    int probe_table[18];     // [6][3] voxel offsets of mode 1
    int kcap;    // pitch of the count matrix = most buckets a scan may have
    int chunk;   // points per workgroup chunk
    long long max_scan_points;
    int max_buckets;
    // outputs
    int32_t* perm;
    int32_t* inv_perm;
    int32_t* offsets;
    int32_t* sbs;          // scan_bucket_start
    int32_t* round_count;  // [8]
    // workspace
    int32_t* status;   // [4]
    int32_t* scan_p0;  // [n_scans+1]
    int32_t* scan_c0;  // [n_scans+1] first chunk of every scan
    uint32_t* mm;      // [n_scans][8] bounding box as ordered ints
    int32_t* cnt;      // [max_buckets] fill level of every bucket
    int32_t* cnt_next;
    int32_t* hist;     // [chunks][kcap]
    uint32_t* key;     // [n] per point: (bucket << 12 | rank inside chunk) or KEY_PLACED
    int32_t* left;     // [chunks] leftovers per chunk
    int32_t* leftpre;  // [chunks]
    int32_t* freepre;  // [max_buckets]
    void* cfg;         // [n_scans] per-scan hash settings (fast path)
    int4* chunk_info;  // [chunks][2] {scan, chunk in scan, chunks of scan, first point}, {end point, first bucket, buckets, first chunk}; null = not wanted
    int n_chunks_ub;   // rows of chunk_info
    int32_t* done;     // [n_scans] workgroups of a scan that finished the bounding box (fast path)
    int meta_light;    // the set-up kernel leaves the bucket offsets of the scans to the caller's kernels (batch path)
    uint32_t* mmpart;  // [chunks][8] bounding box of every chunk as ordered ints (fast path, batches of few scans)
};

hipError_t psh_launch(const PshArgs& args, hipStream_t stream);       // any size
hipError_t psh_fast_launch(const PshArgs& args, hipStream_t stream);  // small count matrix
hipError_t psh_scan_launch(const PshArgs& args, int32_t* lidx0, int32_t* lidx1, unsigned long long* lvox0,
                           unsigned long long* lvox1, hipStream_t stream);    // one workgroup per scan: batches of many scans
bool psh_scan_eligible(int kcap);
bool psh_fast_eligible(long long max_scan_points, int kcap);
size_t psh_fast_matrix_bytes(long long n, int n_scans, int kcap);
__global__ void k_psh_meta(PshArgs a);

}  // namespace f3d

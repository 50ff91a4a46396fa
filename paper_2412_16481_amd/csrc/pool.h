// Internal interface between the C ABI (flash3d_api.hip) and the in-bucket pooling kernels (pool.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace f3d {

constexpr int POOL_MAX_TILE = 1024;   // rows of a tile = threads of a workgroup
constexpr int POOL_MAX_RHO = 64;
constexpr int POOL_MAX_SLOTS = 512;   // resident workgroups: at most two per compute unit

// Entries (16-bit ids) of one workgroup's choice lists: rows left x open sub-buckets rounded up to 8. With n rows and
// M sub-buckets at most n - M rows are left and at most M sub-buckets are open: (n - M)(M + 7) <= (n / 2 + 4)^2.
constexpr size_t pool_list_entries(int tile) { return ((size_t)(tile / 2 + 8) * (size_t)(tile / 2 + 8) + 7) & ~(size_t)7; }

struct PoolArgs {
    const float* coords;           // [n,3], input order if perm is given, else bucket-major
    const int32_t* perm;           // may be null
    const uint16_t* feat;          // bf16 [n, C], bucket-major
    const int32_t* batch_offsets;  // may be null: one scan
    int n;
    int n_scans;
    int C;
    int tile;
    int rho;
    float inv_voxel;
    int hash;
    int op;
    int kp;                        // ceil(tile / rho) rounded up to 64: pitch of the per-key LDS arrays
    int n_tiles_ub;                // rows of tile_info
    uint16_t* pooled_feat;         // bf16 [max_rows, C]
    float* pooled_coords;          // [max_rows, 3], may be null
    int32_t* sub_of;               // [n], may be null
    int32_t* pooled_offsets;       // [n_scans + 1]
    int4* tile_info;               // workspace: {first row, rows, first pooled row, scan} per tile; rows = 0: no tile
    int* tile_counter;             // workspace: next tile to hand out (cleared by the set-up kernel)
    uint16_t* lists;               // workspace: [n_slots][list_cap] sorted choices of the rows left, per workgroup
    size_t list_cap;
    int n_slots;                   // workgroups of the pooling kernel
};

hipError_t pool_launch(const PoolArgs& a, hipStream_t stream);

}  // namespace f3d

// Internal interface between the C ABI (flash3d_api.hip) and the in-bucket pooling kernels (pool.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace f3d {

constexpr int POOL_MAX_TILE = 1024;   // rows of a tile = threads of a workgroup
constexpr int POOL_MAX_RHO = 64;

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
};

hipError_t pool_launch(const PoolArgs& a, hipStream_t stream);

}  // namespace f3d

// Internal interface: the canonical serving order of the bucketing (an input-order-independent rebalancing) and
// the composition of the result with it. Used by flash3d_api.hip only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace f3d {

struct OrderArgs {
    const float* coords;           // [n,3]
    const int32_t* batch_offsets;  // [n_scans+1] or null
    int n;
    int n_scans;
    float inv_voxel;
    // workspace
    uint32_t* box;      // [n_scans][4] per-scan minimum as ordered ints (word 3 unused)
    uint32_t* words;    // [6][n] key words: z, y, x (ordered ints), Z-order code low and high word, scan
    int32_t* idx[2];    // [n] each: ping-pong buffers of the sort
    uint32_t* hist;     // [tiles][256]
    float* coords_sorted;  // [n,3] (out)
};

size_t order_hist_bytes(long long n);

// Sorts the points by (scan, Z-order code of the voxel, x, y, z, input index) and writes the coordinates in that
// order. Returns in *order_out the buffer (one of idx[0], idx[1]) that holds the input index of every sorted position.
hipError_t order_launch(const OrderArgs& a, const int32_t** order_out, hipStream_t stream);

// perm[row] = order[perm_sorted[row]], inv_perm[order[p]] = inv_sorted[p]; nothing is written when *status != 0
// (the bucketing refused its input) and indices outside [0, n) are skipped.
hipError_t order_compose_launch(const int32_t* order, const int32_t* perm_sorted, const int32_t* inv_sorted, int n,
                                const int32_t* status, int32_t* perm, int32_t* inv_perm, hipStream_t stream);

}  // namespace f3d

// Internal interface between the C ABI (flash3d_api.hip) and the LayerNorm + linear kernel (linear.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace f3d {

constexpr int LIN_MAX_OUTS = 4;

struct LinearArgs {
    const uint16_t* x;        // bf16 [n, c_in]
    const int32_t* row_in;    // null, or [n]: output row p reads x[row_in[p]]
    const float* gamma;       // null: no LayerNorm
    const float* beta;        // may be null
    float eps;
    const uint16_t* w;        // bf16 [c_out, c_in]
    const float* bias;        // may be null
    const uint16_t* residual; // null, or bf16 [n, c_out], indexed by the DESTINATION row
    int n;
    int c_in;
    int c_out;
    int n_outs;               // the c_out columns are split evenly over this many output tensors
    uint16_t* outs[LIN_MAX_OUTS];
    const int32_t* row_out;   // null, or [n]: output row p is stored at row row_out[p]
};

hipError_t linear_launch(const LinearArgs& a, hipStream_t stream);

}  // namespace f3d

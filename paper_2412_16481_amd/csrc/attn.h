// Internal interface between the C ABI (flash3d_api.hip) and the attention kernel (attn.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace f3d {

struct AttnArgs {
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    uint16_t* out;
    float* lse;                // null, or [n, H]: natural-log sum of exponentials of every row's scaled scores (bucket-major)
    const int32_t* out_perm;   // null: out is bucket-major; else the result of bucket-major row p goes to row out_perm[p]
    const int32_t* perm;     // may be null
    const int32_t* offsets;
    const int32_t* sbs;      // scan_bucket_start
    int n;
    int n_scans;
    int m;        // buckets per scope
    int mode;     // 0 plain, 1 shift, 2 stride
    int shift;
    int stride;
    int H;
    int C;        // row pitch in elements = heads * head_dim
    float c_log2; // softmax scale * log2(e)
    int n_slots;  // scope slots over all scans (upper bound, surplus workgroups exit)
    int qblocks;  // query blocks per scope = ceil(bucket_cap / attn_block_rows(...))
    int extra;    // spare slots per scan: 2 (plain, shift) or stride + 1
    int f16;      // 0: q, k, v, out are bfloat16; 1: binary16 (forward only)
};

// Backward pass: the forward arguments (f.out = the forward output O, f.lse = its log-sum-exp, f.out_perm = where a
// gradient row goes, null = bucket-major) plus the incoming gradient and the three outgoing ones.
struct AttnBwdArgs {
    AttnArgs f;
    const uint16_t* dout;   // bf16 [n, C], gradient of the bucket-major output rows
    float* dsum;            // workspace [n, H]: sum over the head's channels of dO * O
    uint16_t* dq;           // bf16 [n, C]
    uint16_t* dk;
    uint16_t* dv;
    float scale;            // softmax scale (the forward's c_log2 divided by log2 e)
    int kblocks;            // ceil(bucket_cap / 128): key blocks of a scope in the dK/dV kernel
};

hipError_t attn_bwd_launch(const AttnBwdArgs& a, int head_dim, hipStream_t stream);

int attn_block_rows(int head_dim, long long slots, int heads, int bucket_cap);   // query rows one workgroup covers
hipError_t attn_launch(const AttnArgs& a, int head_dim, int block_rows, hipStream_t stream);

}  // namespace f3d

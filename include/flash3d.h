/*
 * flash3d.h - C ABI of the MI355X (gfx950) implementation of Flash3D's hot path
 * (arXiv 2412.16481): Perfect-Spatial-Hashing bucketing of 3D points (Section 4.1,
 * Algorithms 1 and 2) followed by Bucket-and-Swin multi-head self-attention (Section 4.2,
 * Appendix "Bucket-Swin") and the inverse of the one up-front scatter.
 *
 * Conventions for every call
 *   - Pointers are DEVICE pointers unless the comment says "host". The caller owns every buffer;
 *     the library keeps no state between calls and allocates nothing.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default stream).
 *     No call synchronises with the host, copies to the host, or reads device memory on the host.
 *   - Return value: F3D_OK (0) or a negative F3D_ERR_* code. Argument errors are detected on the
 *     host before anything is launched. Errors that only the device can see (inconsistent
 *     batch_offsets) are reported through scan_bucket_start[n_scans] = -1, see f3d_psh_bucketize.
 *   - NaN / Inf coordinates give unspecified (but memory-safe) bucket assignments.
 *
 * Vocabulary (paper -> here)
 *   bucket            a PSH hash bucket of capacity S = bucket_cap / scope_buckets rows
 *   attention scope   a group of up to `scope_buckets` buckets (at most bucket_cap rows) inside which
 *                     attention is computed; plain, shifted and strided scopes regroup the SAME
 *                     bucket-major layout (Section 4.2: no feature shuffling between passes)
 *   bucket-major row  row p of the array obtained by scattering point i to
 *                     bucket_base[bucket_id[i]] + bucket_offset[i] (Section 4.1, "Input and Output")
 */
#ifndef FLASH3D_H
#define FLASH3D_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define F3D_OK 0
#define F3D_ERR_INVALID_ARG (-1)         /* NULL required pointer, negative size, bad enum, ...          */
#define F3D_ERR_BAD_ALIGNMENT (-2)       /* a pointer or row size is not aligned as documented           */
#define F3D_ERR_WORKSPACE_TOO_SMALL (-3) /* workspace_bytes < f3d_workspace_bytes(...)                  */
#define F3D_ERR_UNSUPPORTED (-4)         /* valid request outside the implemented limits                 */
#define F3D_ERR_HIP (-5)                 /* a HIP runtime call failed; see f3d_last_hip_error()          */
#define F3D_ERR_SCRATCH_LIMIT (-6)       /* f3d_psh_bucketize_static: needs > F3D_STATIC_SCRATCH_BYTES   */

/* Hash functions of Section 4.1 ("Hash functions"). */
#define F3D_HASH_XOR_MOD 0
#define F3D_HASH_XOR_DIV 1
#define F3D_HASH_ZORDER_MOD 2
#define F3D_HASH_ZORDER_DIV 3

/* Scope patterns of Section 4.2 and Table 2: plain windows, windows shifted by `shift` buckets,
 * and scopes that take every `stride`-th bucket. */
#define F3D_PLAIN 0
#define F3D_SHIFT 1
#define F3D_STRIDE 2

/* How the bucketing steps are put on the GPU. The result does not depend on it. AUTO picks SCANS for a batch of
 * at least 48 scans of at most 1024 buckets each when a cost estimate from n, n_scans and max_scan_points favours
 * it (many scans, none of them a large share of the points), else STEPS when the per-scan count matrix is small (the paper's operating range), else GENERAL.
 * Asking for STEPS or SCANS on an input that does not qualify is F3D_ERR_UNSUPPORTED. */
#define F3D_SCHEDULE_AUTO 0
#define F3D_SCHEDULE_GENERAL 1 /* two launches per step, any size                                      */
#define F3D_SCHEDULE_STEPS 2   /* one launch per step                                                  */
#define F3D_SCHEDULE_SCANS 3   /* one launch, one workgroup per scan: batches of many scans            */

/* Variants of the rebalancing (Section 4.1 "Bucket rebalancing": Algorithm 2 leaves the arrival order of the
 * contenders of a bucket to the hardware race, and the probe offsets open, calling them randomly perturbed).
 * F3D_ORDER_INDEX serves the contenders of a bucket in increasing input index. F3D_ORDER_CANONICAL serves them in
 * increasing (Z-order code of the voxel, x, y, z as numbers, input index): the partition of the POINTS then does
 * not depend on the order in which they are stored (only points with identical coordinates can swap rows); it
 * costs a sort of the points before the bucketing. */
#define F3D_ORDER_INDEX 0
#define F3D_ORDER_CANONICAL 1
/* Probe r (1..n_probes) moves the voxel of a point that is still unplaced, clamped to the scan's voxel box:
 * AXES   to the r-th of the six axis neighbours (+x, -x, +y, -y, +z, -z) at distance probe_step;
 * TABLE  by probe_table[r-1] voxels (the caller draws the offsets, e.g. from a seeded generator);
 * SEEDED by probe_step along the axis direction number (h * 6) >> 32, where h = mix(mix(mix(mix(seed + r) ^ vx)
 *        ^ vy) ^ vz) over the point's voxel and mix(x) is: x ^= x >> 16; x *= 0x7feb352d; x ^= x >> 15;
 *        x *= 0x846ca68b; x ^= x >> 16 (32-bit arithmetic). Points of one voxel move together. */
#define F3D_PROBE_AXES 0
#define F3D_PROBE_TABLE 1
#define F3D_PROBE_SEEDED 2

#define F3D_MAX_PROBES 6          /* probe offsets of Algorithm 2                                      */
#define F3D_MAX_SCAN_BUCKETS 8192 /* most hash buckets one scan may own                               */
#define F3D_MAX_SCOPE_BUCKETS 16  /* most buckets per attention scope                                 */
#define F3D_MAX_VOXEL ((1 << 21) - 1) /* voxel coordinates saturate here (63-bit Morton code)        */

/* Parameters of the bucketing (plain data; set struct_size = sizeof(f3d_params)). */
typedef struct f3d_params {
    uint32_t struct_size;
    float voxel_size;        /* > 0; voxel coordinate = floor((c - scan minimum) * (1/voxel_size)), binary32 */
    int32_t bucket_cap;      /* capacity of one attention scope in rows; multiple of 16*scope_buckets        */
    int32_t scope_buckets;   /* buckets per scope (1..16); bucket capacity S = bucket_cap / scope_buckets    */
    int32_t hash;            /* F3D_HASH_*                                                                   */
    int32_t n_probes;        /* 0..6 rebalancing probes (Algorithm 2); 0 sends overflow straight to recycle  */
    int32_t div;             /* divisor of the *_DIV hashes; 0 = automatic (largest code / K + 1)            */
    int32_t probe_step;      /* probe distance in voxels; 0 = automatic                                      */
    int64_t max_scan_points; /* upper bound on the points of any one scan; 0 = n. Sizes the workspace and    */
                             /* must satisfy ceil(max_scan_points / S) <= F3D_MAX_SCAN_BUCKETS               */
    int32_t schedule;        /* F3D_SCHEDULE_*; 0 = automatic                                                */
    int32_t order;           /* F3D_ORDER_*                                                                  */
    int32_t probe_mode;      /* F3D_PROBE_*                                                                  */
    uint32_t probe_seed;     /* seed of F3D_PROBE_SEEDED                                                     */
    int32_t probe_table[3 * F3D_MAX_PROBES]; /* voxel offsets (x, y, z) of probes 1..6 for F3D_PROBE_TABLE   */
} f3d_params;

/* Fill *p with the defaults: scope_buckets 4, Z-order-div hash, 6 axis probes, automatic divisor and step,
 * contenders served by input index. */
void f3d_params_default(f3d_params *p, float voxel_size, int32_t bucket_cap);

/* Upper bound on the total number of hash buckets: n / S + n_scans. `offsets` needs this many + 1 ints. */
int64_t f3d_max_buckets(int64_t n, int32_t n_scans, const f3d_params *p);

/* Bytes of scratch device memory f3d_psh_bucketize needs (written to *out_bytes, host). */
int f3d_workspace_bytes(int64_t n, int32_t n_scans, const f3d_params *p, size_t *out_bytes);

/*
 * PSH bucketing with rebalancing (Algorithms 1 and 2; Appendix "PSH with Two-Stage Counters").
 * The racing atomics of the paper are replaced by a deterministic schedule with the same
 * admissible result: all points take the same step together (direct hash, then probe 1, ...), and
 * the points contending for a bucket in one step are served in increasing input index (or in the canonical
 * order, see F3D_ORDER_CANONICAL; perm and inv_perm always refer to the caller's indices).
 *
 *   coords            [n,3] binary32, 4-byte aligned, scans stored back to back
 *   batch_offsets     [n_scans+1] int32, non-decreasing, first 0, last n; NULL = one scan of n points
 *   n, n_scans        0 <= n < 2^31 - 2^20; n_scans >= 1
 *   perm       (out)  [n] perm[p] = input index of the point stored at bucket-major row p
 *   inv_perm   (out)  [n] inv_perm[i] = bucket_base[bucket_id[i]] + bucket_offset[i]; may be NULL
 *   offsets    (out)  [f3d_max_buckets()+1] first row of every bucket; entries past the last bucket = n
 *   scan_bucket_start (out) [n_scans+1] first bucket of every scan; last entry = total buckets,
 *                     or -1 if batch_offsets was inconsistent or a scan exceeded max_scan_points
 *                     (then perm/inv_perm/offsets are unspecified; no out-of-bounds access happens)
 *   placed_per_round (out) [8] int32, may be NULL: points placed by the direct hash, by probes 1..6,
 *                     and by the recycle step
 *   workspace         >= f3d_workspace_bytes(), 256-byte aligned; contents are scratch
 * Every bucket of a scan ends up holding exactly S rows except the scan's last one, so
 * offsets[first bucket of scan + j] = scan start + j*S ("any bucket-size-aligned sub-array is a bucket").
 */
int f3d_psh_bucketize(const float *coords, const int32_t *batch_offsets, int64_t n, int32_t n_scans,
                      const f3d_params *p, int32_t *perm, int32_t *inv_perm, int32_t *offsets,
                      int32_t *scan_bucket_start, int32_t *placed_per_round, void *workspace,
                      size_t workspace_bytes, void *stream);

/* The short form: one scan, default parameters. */
static inline int f3d_psh_bucketize_simple(const float *coords, int64_t n, float voxel_size, int32_t bucket_cap,
                                           int32_t *perm, int32_t *offsets, int32_t *scan_bucket_start,
                                           void *workspace, size_t workspace_bytes, void *stream)
{
    f3d_params p;
    f3d_params_default(&p, voxel_size, bucket_cap);
    return f3d_psh_bucketize(coords, NULL, n, 1, &p, perm, NULL, offsets, scan_bucket_start, NULL, workspace,
                             workspace_bytes, stream);
}

/*
 * f3d_psh_bucketize for callers that cannot allocate device memory and have no workspace to pass: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc. Same arguments (minus the workspace), same
 * kernels and bit-identical results; the scratch memory is a buffer of F3D_STATIC_SCRATCH_BYTES that is part of the
 * library's device image (every GPU the library runs on holds it until the process ends). The call allocates and
 * frees nothing.
 *   - An input whose f3d_workspace_bytes() exceeds F3D_STATIC_SCRATCH_BYTES is refused with F3D_ERR_SCRATCH_LIMIT
 *     before anything is launched (32 MiB serves about 1.4 M points in 8 scans with the default parameters; the
 *     canonical order needs about five times the scratch per point).
 *   - The buffer's address on the current device is looked up on the first call on that device (one
 *     hipGetSymbolAddress, no allocation); make that first call outside a stream capture.
 *   - All calls on one GPU share the one buffer, which keeps the last call's contents; the kernels initialise
 *     everything they read, so nothing has to be cleared. Two calls that overlap in time on one GPU (different streams,
 *     or graphs replayed concurrently) race on it: serialise them.
 */
#define F3D_STATIC_SCRATCH_BYTES (32u << 20)
int f3d_psh_bucketize_static(const float *coords, const int32_t *batch_offsets, int64_t n, int32_t n_scans,
                             const f3d_params *p, int32_t *perm, int32_t *inv_perm, int32_t *offsets,
                             int32_t *scan_bucket_start, int32_t *placed_per_round, void *stream);

/*
 * Bucket-and-Swin multi-head self-attention, forward (Section 4.2 "Zero-Overhead Bucket-Swin
 * Attention"; Appendix "Bucket-Swin"): exact softmax attention inside every scope, computed
 * FlashAttention-style; the scope pattern only redirects which rows a tile is fetched from.
 *
 *   q, k, v     bf16 [n, heads*head_dim], row stride heads*head_dim elements, 16-byte aligned
 *   perm        NULL: rows of q,k,v are already bucket-major. Otherwise row p is read from perm[p]
 *   offsets, scan_bucket_start   as written by f3d_psh_bucketize (any layout with buckets of at most
 *               bucket_cap/scope_buckets rows works)
 *   max_buckets any upper bound on scan_bucket_start[n_scans] known on the host, e.g. f3d_max_buckets();
 *               it only sizes the launch
 *   bucket_cap, scope_buckets    as in f3d_params; a scope never has more than bucket_cap rows
 *   mode        F3D_PLAIN | F3D_SHIFT | F3D_STRIDE
 *   shift       buckets the windows are moved by, 0 < shift < scope_buckets (F3D_SHIFT only)
 *   stride      distance between the buckets of a strided scope, >= 1 (F3D_STRIDE only)
 *   heads, head_dim   head_dim is 16 or 32
 *   softmax_scale     0 = 1/sqrt(head_dim)
 *   out  (out)  bf16 [n, heads*head_dim], BUCKET-MAJOR rows: row p holds the result for the point stored
 *               at row p (Appendix: input and output of a point sit at the same row)
 *   out_perm    NULL, or [n] int32, a permutation: the result for bucket-major row p is stored at row
 *               out_perm[p] instead. Passing `perm` returns the last layer's output in the input order of the
 *               points, i.e. f3d_unpermute folded into the store (4-byte aligned; must not alias q, k, v)
 *   lse  (out)  NULL, or binary32 [n, heads], BUCKET-MAJOR rows (out_perm does not apply): natural logarithm of
 *               the sum of exponentials of the row's scaled scores; what f3d_bucket_swin_attn_bwd needs
 * Arithmetic: bf16 operands, fp32 accumulation and softmax, probabilities rounded to bf16 before P*V. The scale
 * is folded into q before the product (q*scale*log2(e) carried as two bf16 terms), so a scaled score is exact to
 * about 2^-17 of |q||k| scale (the product of the norms, not the score itself): far below the rounding of the
 * probabilities while |q||k| scale stays below a few hundred, and visible in `lse` as an absolute error of about
 * 4e-3 plus that amount. Where |q||k| scale reaches 10^4 and two top scores of a row lie within one unit of each
 * other, single outputs move by a few 10^-2. Inputs must be finite, and so must their scaled scores in binary32.
 */
int f3d_bucket_swin_attn(const void *q, const void *k, const void *v, const int32_t *perm, const int32_t *offsets,
                         const int32_t *scan_bucket_start, int64_t n, int32_t n_scans, int64_t max_buckets,
                         int32_t bucket_cap, int32_t scope_buckets, int32_t mode, int32_t shift, int32_t stride, int32_t heads,
                         int32_t head_dim, float softmax_scale, void *out, const int32_t *out_perm, float *lse,
                         void *stream);

/* Query rows one workgroup of the attention kernel covers for a launch of this geometry: 128 (one tile of 32 query rows
 * per wave) or 256 (two). The result does not depend on it; tests use it to know which kernel variant a case runs.
 * Arguments as in f3d_bucket_swin_attn; a negative return value is an F3D_ERR_* code. */
int f3d_attn_block_rows(int64_t n_scans, int64_t max_buckets, int32_t bucket_cap, int32_t scope_buckets, int32_t mode,
                        int32_t stride, int32_t heads, int32_t head_dim);

/*
 * The same attention on IEEE binary16 ("FP16") tensors, the element type the Appendix "Bucket-Swin" names for the
 * point features: q, k, v and out are binary16 [n, heads*head_dim]; every other argument, the layout and the error
 * behaviour are those of f3d_bucket_swin_attn. Arithmetic: binary16 operands, fp32 accumulation and softmax,
 * probabilities rounded to binary16 (round to nearest even) before P*V. |q * softmax_scale * log2(e)| is
 * clamped to 65000 (finite in binary16); scores that large saturate the softmax anyway. Forward only.
 */
int f3d_bucket_swin_attn_f16(const void *q, const void *k, const void *v, const int32_t *perm, const int32_t *offsets,
                             const int32_t *scan_bucket_start, int64_t n, int32_t n_scans, int64_t max_buckets,
                             int32_t bucket_cap, int32_t scope_buckets, int32_t mode, int32_t shift, int32_t stride,
                             int32_t heads, int32_t head_dim, float softmax_scale, void *out, const int32_t *out_perm,
                             float *lse, void *stream);

/*
 * Backward of f3d_bucket_swin_attn (Section 4.2; the experiments report training latency): given the gradient dout of
 * the BUCKET-MAJOR output rows, the gradients of q, k and v inside every scope,
 *   P = exp(scale q k^T - lse),  dP = dout v^T,  D = rowsum(dout o out),  dS = P o (dP - D),
 *   dq = scale dS k,  dk = scale dS^T q,  dv = P^T dout.
 *
 *   q, k, v, perm, offsets, scan_bucket_start, n .. softmax_scale   exactly as in the forward call
 *   out         bf16 [n, heads*head_dim], the forward output, bucket-major (not written with out_perm)
 *   dout        bf16 [n, heads*head_dim], bucket-major
 *   lse         binary32 [n, heads], the forward call's lse output
 *   dq, dk, dv (out)  bf16 [n, heads*head_dim]: row p holds the gradient of the q/k/v row that bucket-major row p
 *               was read from; with grad_perm it is stored at row grad_perm[p] instead (passing perm returns the
 *               gradients in the input order of the points)
 *   grad_perm   NULL or [n] int32, a permutation
 *   workspace   >= f3d_attn_bwd_workspace_bytes(n, heads), 256-byte aligned
 * Arithmetic: bf16 operands, fp32 accumulation; P and dS are rounded to bf16 before the second products.
 */
int f3d_attn_bwd_workspace_bytes(int64_t n, int32_t heads, size_t *out_bytes);

int f3d_bucket_swin_attn_bwd(const void *q, const void *k, const void *v, const void *out, const void *dout,
                             const float *lse, const int32_t *perm, const int32_t *offsets,
                             const int32_t *scan_bucket_start, int64_t n, int32_t n_scans, int64_t max_buckets,
                             int32_t bucket_cap, int32_t scope_buckets, int32_t mode, int32_t shift, int32_t stride,
                             int32_t heads, int32_t head_dim, float softmax_scale, void *dq, void *dk, void *dv,
                             const int32_t *grad_perm, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The point-wise glue of a transformer block (Section 4.2, block equations F' = MHSA(LN(F)) + F, F~ = MLP(LN(F')) + F';
 * Section 4.1 "Stage Orchestration"): LayerNorm and a linear map over every row in one pass, with the row gather that
 * writes q, k, v in bucket-major order and the row scatter + residual that brings a block's output back.
 *     y[p] = LN(x[row_in[p]]) W^T + bias,   LN(v) = (v - mean v) / sqrt(var v + eps) * gamma + beta  (biased variance)
 *     out[row_out[p]] = y[p] + residual[row_out[p]]
 *   x         bf16 [n, c_in], 16-byte aligned;  c_in is 64, 128 or 256
 *   row_in    NULL (row p reads x[p]) or [n] int32, e.g. perm: the outputs come out bucket-major
 *   gamma, beta  binary32 [c_in], 16-byte aligned; gamma NULL skips the LayerNorm (then beta must be NULL); beta may be NULL
 *   w         bf16 [c_out, c_in] (one row per output column), 16-byte aligned;  bias  binary32 [c_out] or NULL
 *   residual  NULL or bf16 [n, c_out], indexed by the DESTINATION row
 *   c_out     multiple of 64, at most 4096
 *   outs      HOST array of n_outs (1..4) DEVICE pointers: the c_out columns are split evenly over bf16 [n, c_out/n_outs]
 *             tensors (three for q, k, v); c_out / n_outs must be a multiple of 16
 *   row_out   NULL or [n] int32, a permutation: output row p is stored at row row_out[p]
 * Arithmetic: LayerNorm in fp32 on the bf16 input, rounded to bf16; bf16 MFMA with fp32 accumulation; bias and
 * residual added in fp32; one rounding to bf16.
 */
int f3d_ln_linear(const void *x, const int32_t *row_in, const float *gamma, const float *beta, float eps, const void *w,
                  const float *bias, const void *residual, int64_t n, int32_t c_in, int32_t c_out, void *const *outs,
                  int32_t n_outs, const int32_t *row_out, void *stream);

/*
 * In-bucket pooling (Section 4.2 "In-bucket Pooling"; Appendix "In-bucket Pooling"): the bucket-major array is
 * cut into tiles of `tile` consecutive rows (tiles start at a scan's first row and never span scans); inside a
 * tile of n rows, M = ceil(n / rho) sub-buckets of capacity rho are built in the Appendix's three steps (initial
 * sub-buckets from a hash of the voxel coordinate relative to the tile's minimum, new sub-buckets for the rows
 * beyond capacity until M exist, rounds in which the rows still left join the sub-bucket with room whose first
 * row is nearest), and every sub-bucket is reduced to one pooled row. The block-level atomics of the Appendix are
 * replaced by decisions in row order, so the result is a function of the input alone. Pooled rows are numbered
 * tile by tile, sub-bucket ids inside a tile; every sub-bucket holds between 1 and rho rows.
 *
 *   coords        [n,3] binary32: input order if perm is given (row p is read from perm[p]), else bucket-major
 *   perm          NULL or [n] as written by f3d_psh_bucketize
 *   feat          bf16 [n, channels] BUCKET-MAJOR rows (what f3d_bucket_swin_attn writes), 16-byte aligned
 *   batch_offsets [n_scans+1] int32 device array as for f3d_psh_bucketize (scans keep their row ranges), NULL = one scan
 *   channels      multiple of 8
 *   tile          1 .. 1024 rows;  rho  1 .. 64, the pooling factor and sub-bucket capacity
 *   voxel_size    > 0, edge of the voxels the in-tile hash works on;  hash  F3D_HASH_*
 *   op            F3D_POOL_SUM | F3D_POOL_MEAN | F3D_POOL_MIN | F3D_POOL_MAX
 *   pooled_feat (out)   bf16 [f3d_pool_max_rows(), channels]; fp32 accumulation in slot order, one rounding to bf16
 *   pooled_coords (out) [f3d_pool_max_rows(), 3] binary32 mean position of every pooled row; may be NULL
 *   sub_of (out)        [n] pooled row of every bucket-major input row; may be NULL
 *   pooled_offsets (out) [n_scans+1] first pooled row of every scan; last entry = number of pooled rows, or -1
 *                       if batch_offsets was inconsistent (then nothing else is written)
 *   workspace           >= f3d_pool_workspace_bytes(), 256-byte aligned: the tile table, a tile counter, and for
 *                       each of up to 512 resident workgroups the sorted choice lists of its tile's leftover rows
 *                       ((tile/2 + 8)^2 two-byte entries: 0.53 MB at tile 1024, 277 MB in all for large inputs)
 */
#define F3D_POOL_SUM 0
#define F3D_POOL_MEAN 1
#define F3D_POOL_MIN 2
#define F3D_POOL_MAX 3
#define F3D_POOL_MAX_TILE 1024
#define F3D_POOL_MAX_RHO 64

/* Upper bound on the number of pooled rows, known on the host: n / rho + n / tile + n_scans + 1; -1 on bad arguments. */
int64_t f3d_pool_max_rows(int64_t n, int32_t n_scans, int32_t tile, int32_t rho);

int f3d_pool_workspace_bytes(int64_t n, int32_t n_scans, int32_t tile, size_t *out_bytes);

int f3d_inbucket_pool(const float *coords, const int32_t *perm, const void *feat, const int32_t *batch_offsets,
                      int64_t n, int32_t n_scans, int32_t channels, int32_t tile, int32_t rho, float voxel_size,
                      int32_t hash, int32_t op, void *pooled_feat, float *pooled_coords, int32_t *sub_of,
                      int32_t *pooled_offsets, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Inverse of the up-front scatter (Section 4, "up-front global shuffle"): dst[perm[p], :] = src[p, :].
 *   src, dst  [n, row_bytes] bytes; row_bytes > 0 and a multiple of 4; src != dst; 4-byte aligned
 *             (16-byte aligned rows take the wide path)
 */
int f3d_unpermute(const void *src, const int32_t *perm, int64_t n, int32_t row_bytes, void *dst, void *stream);

const char *f3d_error_string(int code); /* host string, static storage */
int f3d_last_hip_error(void);           /* hipError_t of the last failed HIP call in this thread, 0 if none */
int f3d_version(void);                  /* 1000*major + minor */

#ifdef __cplusplus
}
#endif
#endif /* FLASH3D_H */

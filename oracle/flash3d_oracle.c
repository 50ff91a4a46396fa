/*
 * CPU oracle for the PSH bucketize + Bucket-Swin attention path of Flash3D (arXiv 2412.16481).
 *
 * TEST INFRASTRUCTURE ONLY. This file is the slow, plain reference the HIP library is checked
 * against. It shares no code with the HIP path and must never be linked into it or called from
 * it; only the tests, the smoke check and the benchmark's cpu-baseline leg use it.
 *
 * What is defined here and where it comes from:
 *   - voxel coordinate, the four hash functions          (Section 4.1, "Hash functions")
 *   - bucket assignment with rebalancing                 (Algorithm 1 and Algorithm 2)
 *   - scatter index bucket_base[bucket_id] + bucket_off  (Section 4.1, "Input and Output")
 *   - scope regrouping: plain / shifted / strided        (Section 4.2, worked example; Table 2 caption)
 *   - multi-head self-attention inside one scope         (Section 4.2; Appendix "Bucket-Swin")
 *   - gradient of that attention (plain definition)       (Section 4.2; the experiments report training latency)
 *   - in-bucket pooling: sub-bucket construction, reduce  (Section 4.2 "In-bucket Pooling"; Appendix "In-bucket Pooling")
 *   - variants of the rebalancing (orc_bucketize_ex): contenders served in an order that does not depend on the input
 *     order, probe offsets from a table or drawn per voxel from a seeded integer mixer
 *     (Section 4.1 "Bucket rebalancing": the offsets are left open and called randomly perturbed)
 *
 * Algorithms 1 and 2 let hardware atomics decide the arrival order, so their result depends on
 * the schedule. The oracle fixes one admissible schedule: all points take the same step together
 * (first the direct hash of Algorithm 1, then probe 1 of Algorithm 2, then probe 2, ...), and
 * inside a step the points contending for a bucket are served in increasing input index. Under
 * that schedule the optimistic increment followed by a roll-back of Algorithm 2 leaves the same
 * counters as "take the slot only if one is free", which is what the loops below do.
 *
 * Everything in the bucketing half is integer arithmetic except the voxel coordinate, which is
 * three IEEE-754 binary32 operations (subtract, multiply, floor) evaluated one by one; build
 * with -ffp-contract=off. The attention half is the plain definition in binary64.
 *
 * Parity pins (see tests/test_oracle_*.py): hand-computed hashes and Morton codes, the paper's
 * regrouping example, a literal thread-by-thread simulation of Algorithms 1+2, stable-argsort on
 * overflow-free inputs, brute-force masked dense attention, a library dense-attention routine on
 * the single-scope case, closed forms and invariants; for the pooling hand traces of the three steps, a
 * literal simulation with an AtomicInc primitive, capacity/coverage invariants, a brute-force
 * nearest-sub-bucket check and numpy reductions with an independent bf16 rounding; for the rebalancing variants
 * reductions to the pinned default (pre-sorted input, the axis table), equivariance under input permutation on
 * overflowing inputs, a literal Python simulation, and bijectivity/avalanche/uniformity of the mixer. No function
 * here is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_XOR_MOD = 0, ORC_XOR_DIV = 1, ORC_ZORDER_MOD = 2, ORC_ZORDER_DIV = 3 };
enum { ORC_PLAIN = 0, ORC_SHIFT = 1, ORC_STRIDE = 2 };

#define ORC_VOXEL_MAX ((1 << 21) - 1) /* 21 bits per axis fit a 63-bit Morton code */

/* ------------------------------------------------------------------ hash functions (Section 4.1) */

/* Z-order code: bit k of x goes to bit 3k, of y to 3k+1, of z to 3k+2. */
uint64_t orc_morton3(uint32_t x, uint32_t y, uint32_t z)
{
    uint64_t code = 0;
    for (int k = 0; k < 21; ++k) {
        code |= (uint64_t)((x >> k) & 1u) << (3 * k);
        code |= (uint64_t)((y >> k) & 1u) << (3 * k + 1);
        code |= (uint64_t)((z >> k) & 1u) << (3 * k + 2);
    }
    return code;
}

static int bit_width_u64(uint64_t v)
{
    int w = 0;
    while (v) { ++w; v >>= 1; }
    return w;
}

/* Per-scan hash setting: number of buckets K, divisor D, probe step, per-axis voxel maximum. */
typedef struct {
    int32_t hash;
    int64_t K;
    uint64_t D;
    int32_t step;
    int32_t vmax[3];
} orc_hash_cfg;

static uint64_t hash_code(const orc_hash_cfg *c, const int32_t v[3])
{
    if (c->hash == ORC_XOR_MOD || c->hash == ORC_XOR_DIV)
        return (uint64_t)((uint32_t)v[0] ^ (uint32_t)v[1] ^ (uint32_t)v[2]);
    return orc_morton3((uint32_t)v[0], (uint32_t)v[1], (uint32_t)v[2]);
}

static int64_t hash_bucket(const orc_hash_cfg *c, const int32_t v[3])
{
    uint64_t code = hash_code(c, v);
    if (c->hash == ORC_XOR_MOD || c->hash == ORC_ZORDER_MOD)
        return (int64_t)(code % (uint64_t)c->K);
    uint64_t q = code / c->D;
    return (int64_t)(q < (uint64_t)c->K ? q : (uint64_t)c->K - 1);
}

/* Fill divisor and probe step. div_override/step_override > 0 replace the automatic choice.
 * Automatic divisor: the smallest D for which (largest possible code) / D < K.
 * Automatic probe step: 1 voxel for the mod hashes; for the div hashes about the edge length of
 * the cell of voxels that share one bucket. */
static void hash_cfg_fill(orc_hash_cfg *c, int32_t hash, int64_t K, const int32_t vmax[3],
                          int32_t div_override, int32_t step_override)
{
    c->hash = hash;
    c->K = K;
    memcpy(c->vmax, vmax, sizeof(c->vmax));
    int32_t vm = vmax[0] > vmax[1] ? vmax[0] : vmax[1];
    vm = vm > vmax[2] ? vm : vmax[2];
    int nb = bit_width_u64((uint64_t)vm);
    if (nb < 1) nb = 1;
    uint64_t D = 1;
    if (hash == ORC_XOR_DIV) D = (((uint64_t)1 << nb) - 1) / (uint64_t)K + 1;
    if (hash == ORC_ZORDER_DIV) D = orc_morton3(vmax[0], vmax[1], vmax[2]) / (uint64_t)K + 1;
    if (div_override > 0) D = (uint64_t)div_override;
    c->D = D;
    int64_t step = 1;
    if (hash == ORC_XOR_DIV) step = (int64_t)(D > (uint64_t)ORC_VOXEL_MAX ? (uint64_t)ORC_VOXEL_MAX : D);
    if (hash == ORC_ZORDER_DIV) step = (int64_t)1 << ((bit_width_u64(D) + 2) / 3);
    if (step_override > 0) step = step_override;
    c->step = (int32_t)step;
}

/* The probe offsets of Algorithm 2: the six axis neighbours at distance `step`, in this order. */
static const int8_t ORC_PROBE_DIR[6][3] = {
    {+1, 0, 0}, {-1, 0, 0}, {0, +1, 0}, {0, -1, 0}, {0, 0, +1}, {0, 0, -1}};

/* Exposed for the tests: bucket of voxel v under a hash setting built from (K, vmax, overrides). */
int64_t orc_hash(int32_t hash, int64_t K, const int32_t vmax[3], int32_t div_override,
                 const int32_t v[3], int64_t *divisor_out, int32_t *step_out)
{
    orc_hash_cfg c;
    hash_cfg_fill(&c, hash, K, vmax, div_override, 0);
    if (divisor_out) *divisor_out = (int64_t)c.D;
    if (step_out) *step_out = c.step;
    return hash_bucket(&c, v);
}

/* ------------------------------------------------------------------ bucketize (Algorithms 1, 2) */

/* ---- variants of the rebalancing -------------------------------------------------------------- */

enum { ORC_ORDER_INDEX = 0, ORC_ORDER_CANONICAL = 1 };
enum { ORC_PROBE_AXES = 0, ORC_PROBE_TABLE = 1, ORC_PROBE_SEEDED = 2 };

/* A 32-bit integer mixer (xor-shift / odd multiply / xor-shift / odd multiply / xor-shift): a bijection of
 * the 32-bit words with good avalanche. Used as a counter-based generator: no state, the same value on any
 * machine for the same arguments. */
uint32_t orc_mix32(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x7feb352du;
    x ^= x >> 15;
    x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

/* Direction (0..5, an index into ORC_PROBE_DIR) of probe r for a point of voxel v under `seed`: points of one
 * voxel move together, and the draw does not depend on the point's index. */
int32_t orc_probe_direction(uint32_t seed, int32_t r, const int32_t v[3])
{
    uint32_t h = orc_mix32(seed + (uint32_t)r);
    h = orc_mix32(h ^ (uint32_t)v[0]);
    h = orc_mix32(h ^ (uint32_t)v[1]);
    h = orc_mix32(h ^ (uint32_t)v[2]);
    return (int32_t)(((uint64_t)h * 6u) >> 32);
}

/* binary32 bit pattern mapped to an unsigned integer with the same order as the numbers (-0 below +0) */
static uint32_t float_order_key(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof(u));
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

typedef struct {
    uint64_t code;      /* Z-order code of the voxel */
    uint32_t c[3];      /* ordered coordinate keys */
    int64_t idx;        /* input index inside the scan */
} orc_sort_rec;

static int cmp_sort_rec(const void *pa, const void *pb)
{
    const orc_sort_rec *a = (const orc_sort_rec *)pa, *b = (const orc_sort_rec *)pb;
    if (a->code != b->code) return a->code < b->code ? -1 : 1;
    for (int k = 0; k < 3; ++k)
        if (a->c[k] != b->c[k]) return a->c[k] < b->c[k] ? -1 : 1;
    return a->idx < b->idx ? -1 : (a->idx > b->idx ? 1 : 0);
}

int64_t orc_bucketize_ex(const float *coords, const int32_t *batch_offsets, int64_t n, int32_t n_scans,
                         float voxel_size, int32_t bucket_size, int32_t hash, int32_t n_probes,
                         int32_t div_override, int32_t step_override,
                         int32_t order, int32_t probe_mode, uint32_t probe_seed, const int32_t *probe_table,
                         int32_t *bucket_id, int32_t *bucket_off, int32_t *round_of,
                         int32_t *perm, int32_t *inv_perm, int32_t *offsets, int32_t *scan_bucket_start);

/*
 * coords        [n,3] binary32, scans stored back to back
 * batch_offsets [n_scans+1], scan b owns points batch_offsets[b] .. batch_offsets[b+1]-1
 * bucket_size   capacity S of one hash bucket
 * outputs (caller allocates; any may be NULL except perm):
 *   bucket_id[n]   global bucket index of point i          (Section 4.1 "Input and Output")
 *   bucket_off[n]  slot of point i inside its bucket
 *   round_of[n]    0 = direct hash, 1..n_probes = probe that placed it, n_probes+1 = recycled
 *   perm[n]        perm[row] = input index stored at that row of the bucket-major array
 *   inv_perm[n]    inv_perm[i] = bucket_base[bucket_id[i]] + bucket_off[i]
 *   offsets[K+1]   first row of every bucket (exclusive scan of the final counters), K = total buckets
 *   scan_bucket_start[n_scans+1]  first bucket of every scan
 * returns the total number of buckets, or -1 on bad arguments.
 */
int64_t orc_bucketize(const float *coords, const int32_t *batch_offsets, int64_t n, int32_t n_scans,
                      float voxel_size, int32_t bucket_size, int32_t hash, int32_t n_probes,
                      int32_t div_override, int32_t step_override,
                      int32_t *bucket_id, int32_t *bucket_off, int32_t *round_of,
                      int32_t *perm, int32_t *inv_perm, int32_t *offsets, int32_t *scan_bucket_start)
{
    return orc_bucketize_ex(coords, batch_offsets, n, n_scans, voxel_size, bucket_size, hash, n_probes, div_override,
                            step_override, ORC_ORDER_INDEX, ORC_PROBE_AXES, 0u, NULL, bucket_id, bucket_off, round_of,
                            perm, inv_perm, offsets, scan_bucket_start);
}

/*
 * The same schedule with two choices opened up (Section 4.1 "Bucket rebalancing" leaves both to the hardware race
 * and to "each probe offset"):
 *   order        ORC_ORDER_INDEX: contenders are served in increasing input index.
 *                ORC_ORDER_CANONICAL: in increasing (Z-order code of the voxel, x, y, z as numbers, input index),
 *                so that the partition of the POINTS does not depend on the order in which they are stored
 *                (only points with identical coordinates can still swap places).
 *   probe_mode   ORC_PROBE_AXES: probe r moves the voxel to the r-th axis neighbour at distance `step`.
 *                ORC_PROBE_TABLE: probe r adds probe_table[3(r-1) .. 3(r-1)+2] voxels (the caller draws them).
 *                ORC_PROBE_SEEDED: probe r moves the voxel by `step` in direction orc_probe_direction(seed, r, v).
 * In every mode the moved voxel is clamped to the scan's voxel box.
 */
int64_t orc_bucketize_ex(const float *coords, const int32_t *batch_offsets, int64_t n, int32_t n_scans,
                         float voxel_size, int32_t bucket_size, int32_t hash, int32_t n_probes,
                         int32_t div_override, int32_t step_override,
                         int32_t order, int32_t probe_mode, uint32_t probe_seed, const int32_t *probe_table,
                         int32_t *bucket_id, int32_t *bucket_off, int32_t *round_of,
                         int32_t *perm, int32_t *inv_perm, int32_t *offsets, int32_t *scan_bucket_start)
{
    if (n < 0 || n_scans < 0 || !(voxel_size > 0.0f) || bucket_size <= 0 || hash < 0 || hash > 3 ||
        n_probes < 0 || n_probes > 6 || !perm)
        return -1;
    if (order < 0 || order > 1 || probe_mode < 0 || probe_mode > 2 || (probe_mode == ORC_PROBE_TABLE && !probe_table))
        return -1;
    const float inv = 1.0f / voxel_size;
    int64_t kbase = 0; /* buckets of earlier scans */
    int32_t *id = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    int32_t *off = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    if (offsets) offsets[0] = 0;

    for (int32_t b = 0; b < n_scans; ++b) {
        const int64_t p0 = batch_offsets[b], p1 = batch_offsets[b + 1];
        const int64_t nb = p1 - p0;
        if (scan_bucket_start) scan_bucket_start[b] = (int32_t)kbase;
        if (nb <= 0) continue;
        const int64_t K = (nb + bucket_size - 1) / bucket_size;

        /* voxel coordinates: subtract the scan's minimum, scale, floor (Algorithm 1, line 4) */
        float mn[3] = {coords[3 * p0], coords[3 * p0 + 1], coords[3 * p0 + 2]};
        for (int64_t i = p0; i < p1; ++i)
            for (int a = 0; a < 3; ++a)
                if (coords[3 * i + a] < mn[a]) mn[a] = coords[3 * i + a];
        int32_t *v = (int32_t *)malloc(sizeof(int32_t) * 3 * (size_t)nb);
        int32_t vmax[3] = {0, 0, 0};
        for (int64_t i = 0; i < nb; ++i)
            for (int a = 0; a < 3; ++a) {
                volatile float d = coords[3 * (p0 + i) + a] - mn[a];
                volatile float s = d * inv;
                float f = floorf(s);
                int32_t q = f >= (float)ORC_VOXEL_MAX ? ORC_VOXEL_MAX : (int32_t)f;
                if (q < 0) q = 0;
                v[3 * i + a] = q;
                if (q > vmax[a]) vmax[a] = q;
            }

        orc_hash_cfg cfg;
        hash_cfg_fill(&cfg, hash, K, vmax, div_override, step_override);

        /* capacities: every bucket holds bucket_size points, the last one what is left */
        int64_t *cnt = (int64_t *)calloc((size_t)K, sizeof(int64_t));
        int64_t *cap = (int64_t *)malloc(sizeof(int64_t) * (size_t)K);
        for (int64_t j = 0; j < K; ++j) cap[j] = bucket_size;
        cap[K - 1] = nb - (K - 1) * (int64_t)bucket_size;
        int8_t *placed = (int8_t *)calloc((size_t)nb, 1);

        /* the order in which the points of the scan are served inside every step */
        int64_t *ord = (int64_t *)malloc(sizeof(int64_t) * (size_t)nb);
        for (int64_t i = 0; i < nb; ++i) ord[i] = i;
        if (order == ORC_ORDER_CANONICAL) {
            orc_sort_rec *rec = (orc_sort_rec *)malloc(sizeof(orc_sort_rec) * (size_t)nb);
            for (int64_t i = 0; i < nb; ++i) {
                rec[i].code = orc_morton3((uint32_t)v[3 * i], (uint32_t)v[3 * i + 1], (uint32_t)v[3 * i + 2]);
                for (int a = 0; a < 3; ++a) rec[i].c[a] = float_order_key(coords[3 * (p0 + i) + a]);
                rec[i].idx = i;
            }
            qsort(rec, (size_t)nb, sizeof(orc_sort_rec), cmp_sort_rec);
            for (int64_t i = 0; i < nb; ++i) ord[i] = rec[i].idx;
            free(rec);
        }

        /* step 0: direct hash (Algorithm 1, lines 5-9) */
        for (int64_t t = 0; t < nb; ++t) {
            const int64_t i = ord[t];
            int64_t j = hash_bucket(&cfg, &v[3 * i]);
            if (cnt[j] < cap[j]) {
                id[p0 + i] = (int32_t)j;
                off[p0 + i] = (int32_t)cnt[j]++;
                placed[i] = 1;
                if (round_of) round_of[p0 + i] = 0;
            }
        }
        /* steps 1..n_probes: Algorithm 2, one probe offset per step */
        for (int32_t r = 1; r <= n_probes; ++r) {
            for (int64_t t = 0; t < nb; ++t) {
                const int64_t i = ord[t];
                if (placed[i]) continue;
                int32_t w[3];
                const int32_t dir = probe_mode == ORC_PROBE_SEEDED ? orc_probe_direction(probe_seed, r, &v[3 * i]) : r - 1;
                for (int a = 0; a < 3; ++a) {
                    const int64_t delta = probe_mode == ORC_PROBE_TABLE ? (int64_t)probe_table[3 * (r - 1) + a]
                                                                        : (int64_t)ORC_PROBE_DIR[dir][a] * cfg.step;
                    int64_t moved = (int64_t)v[3 * i + a] + delta;
                    if (moved < 0) moved = 0;
                    if (moved > vmax[a]) moved = vmax[a];
                    w[a] = (int32_t)moved;
                }
                int64_t j = hash_bucket(&cfg, w);
                if (cnt[j] < cap[j]) {
                    id[p0 + i] = (int32_t)j;
                    off[p0 + i] = (int32_t)cnt[j]++;
                    placed[i] = 1;
                    if (round_of) round_of[p0 + i] = r;
                }
            }
        }
        /* recycle (Algorithm 2, lines 19-22): leftovers fill the free slots, first bucket first */
        int64_t j = 0;
        for (int64_t t = 0; t < nb; ++t) {
            const int64_t i = ord[t];
            if (placed[i]) continue;
            while (cnt[j] >= cap[j]) ++j;
            id[p0 + i] = (int32_t)j;
            off[p0 + i] = (int32_t)cnt[j]++;
            placed[i] = 1;
            if (round_of) round_of[p0 + i] = n_probes + 1;
        }

        /* exclusive scan of the counters gives bucket_base (Algorithm 1, line 12) */
        int64_t run = p0;
        for (int64_t jj = 0; jj < K; ++jj) {
            if (offsets) offsets[kbase + jj] = (int32_t)run;
            run += cnt[jj];
        }
        if (offsets) offsets[kbase + K] = (int32_t)run;
        /* scatter (Algorithm 1, line 13) */
        int64_t *base = (int64_t *)malloc(sizeof(int64_t) * (size_t)K);
        run = p0;
        for (int64_t jj = 0; jj < K; ++jj) { base[jj] = run; run += cnt[jj]; }
        for (int64_t i = p0; i < p1; ++i) {
            int64_t row = base[id[i]] + off[i];
            perm[row] = (int32_t)i;
            if (inv_perm) inv_perm[i] = (int32_t)row;
            if (bucket_id) bucket_id[i] = (int32_t)(kbase + id[i]);
            if (bucket_off) bucket_off[i] = off[i];
        }
        free(base); free(placed); free(cap); free(cnt); free(v); free(ord);
        kbase += K;
    }
    if (scan_bucket_start) scan_bucket_start[n_scans] = (int32_t)kbase;
    if (offsets && n_scans == 0) offsets[0] = 0;
    free(id); free(off);
    return kbase;
}

/* ------------------------------------------------------------------ regrouping (Section 4.2) */

/* Scope (attention group) of the j-th bucket of a scan; m buckets per scope.
 * plain:  consecutive windows of m buckets.
 * shift:  the windows moved forward by s buckets; the first s buckets form a scope of their own.
 * stride: every t-th bucket inside a block of m*t consecutive buckets. */
int64_t orc_group_of_bucket(int64_t j, int32_t m, int32_t mode, int32_t s, int32_t t)
{
    if (mode == ORC_SHIFT) return (j + m - s) / m;
    if (mode == ORC_STRIDE) return (j / ((int64_t)m * t)) * t + j % t;
    return j / m;
}

/* ------------------------------------------------------------------ attention (Section 4.2) */

static double bf16_to_double(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof(f));
    return (double)f;
}

/* IEEE-754 binary16 bit pattern to binary64, field by field (the Appendix "Bucket-Swin" keeps the features in FP16). */
double orc_half_to_double(uint16_t h)
{
    const int sign = (h >> 15) & 1, ex = (h >> 10) & 31, man = h & 1023;
    double v;
    if (ex == 0) v = ldexp((double)man, -24);                 /* zero and subnormals */
    else if (ex == 31) v = man ? NAN : INFINITY;
    else v = ldexp(1.0 + (double)man / 1024.0, ex - 15);
    return sign ? -v : v;
}

enum { ORC_FMT_BF16 = 0, ORC_FMT_F16 = 1 };

static double elem_to_double(int32_t fmt, uint16_t h)
{
    return fmt == ORC_FMT_F16 ? orc_half_to_double(h) : bf16_to_double(h);
}

/*
 * Multi-head self-attention restricted to scopes. q,k,v are 16-bit patterns [n, heads*head_dim] of bfloat16
 * (fmt = ORC_FMT_BF16) or binary16 (fmt = ORC_FMT_F16) numbers; the arithmetic is binary64 either way.
 * Row p of the bucket-major array holds input row perm[p] (perm == NULL: inputs are already
 * bucket-major). out[p, :] (binary64, bucket-major rows) = sum_j softmax_j(q_p . k_j * scale) v_j
 * over the rows j of p's scope, head by head. row_sel (may be NULL) limits the computed query rows
 * to those with row_sel[p] != 0; other rows of out are left untouched.
 * returns the number of scopes visited, -1 on bad arguments.
 */
int64_t orc_attn_fmt(const uint16_t *q, const uint16_t *k, const uint16_t *v, int32_t fmt, const int32_t *perm,
                     const int32_t *offsets, const int32_t *scan_bucket_start, int32_t n_scans,
                     int32_t m, int32_t mode, int32_t s, int32_t t, int32_t heads, int32_t head_dim,
                     double scale, const uint8_t *row_sel, double *out)
{
    if (fmt < 0 || fmt > 1) return -1;
    if (m <= 0 || heads <= 0 || head_dim <= 0 || mode < 0 || mode > 2) return -1;
    if (mode == ORC_SHIFT && (s <= 0 || s >= m)) return -1;
    if (mode == ORC_STRIDE && t <= 0) return -1;
    const int64_t C = (int64_t)heads * head_dim;
    int64_t visited = 0;

    for (int32_t b = 0; b < n_scans; ++b) {
        const int64_t kb0 = scan_bucket_start[b], K = scan_bucket_start[b + 1] - kb0;
        if (K <= 0) continue;
        int64_t ngroups = 0;
        for (int64_t j = 0; j < K; ++j) {
            int64_t g = orc_group_of_bucket(j, m, mode, s, t);
            if (g + 1 > ngroups) ngroups = g + 1;
        }
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : visited)
        for (int64_t g = 0; g < ngroups; ++g) {
            /* rows of the scope: its buckets in increasing order, each a contiguous row range */
            int64_t ng = 0;
            for (int64_t j = 0; j < K; ++j)
                if (orc_group_of_bucket(j, m, mode, s, t) == g) ng += offsets[kb0 + j + 1] - offsets[kb0 + j];
            if (ng == 0) continue;
            int64_t *rows = (int64_t *)malloc(sizeof(int64_t) * (size_t)ng);
            int64_t c = 0;
            for (int64_t j = 0; j < K; ++j)
                if (orc_group_of_bucket(j, m, mode, s, t) == g)
                    for (int64_t p = offsets[kb0 + j]; p < offsets[kb0 + j + 1]; ++p) rows[c++] = p;
            double *sc = (double *)malloc(sizeof(double) * (size_t)ng);
            ++visited;
            for (int64_t a = 0; a < ng; ++a) {
                const int64_t pa = rows[a];
                if (row_sel && !row_sel[pa]) continue;
                const int64_t ia = perm ? perm[pa] : pa;
                for (int32_t h = 0; h < heads; ++h) {
                    const int64_t co = (int64_t)h * head_dim;
                    double mx = -INFINITY;
                    for (int64_t bb = 0; bb < ng; ++bb) {
                        const int64_t ib = perm ? perm[rows[bb]] : rows[bb];
                        double dot = 0.0;
                        for (int32_t e = 0; e < head_dim; ++e)
                            dot += elem_to_double(fmt, q[ia * C + co + e]) * elem_to_double(fmt, k[ib * C + co + e]);
                        sc[bb] = dot * scale;
                        if (sc[bb] > mx) mx = sc[bb];
                    }
                    double den = 0.0;
                    for (int64_t bb = 0; bb < ng; ++bb) {
                        sc[bb] = exp(sc[bb] - mx);
                        den += sc[bb];
                    }
                    for (int64_t bb = 0; bb < ng; ++bb) sc[bb] /= den; /* softmax row */
                    for (int32_t e = 0; e < head_dim; ++e) {
                        double acc = 0.0;
                        for (int64_t bb = 0; bb < ng; ++bb) {
                            const int64_t ib = perm ? perm[rows[bb]] : rows[bb];
                            acc += sc[bb] * elem_to_double(fmt, v[ib * C + co + e]);
                        }
                        out[pa * C + co + e] = acc;
                    }
                }
            }
            free(sc);
            free(rows);
        }
    }
    return visited;
}

/* The bfloat16 form (the five benchmark configurations). */
int64_t orc_attn(const uint16_t *q, const uint16_t *k, const uint16_t *v, const int32_t *perm,
                 const int32_t *offsets, const int32_t *scan_bucket_start, int32_t n_scans,
                 int32_t m, int32_t mode, int32_t s, int32_t t, int32_t heads, int32_t head_dim,
                 double scale, const uint8_t *row_sel, double *out)
{
    return orc_attn_fmt(q, k, v, ORC_FMT_BF16, perm, offsets, scan_bucket_start, n_scans, m, mode, s, t, heads, head_dim,
                        scale, row_sel, out);
}

/*
 * Gradient of the scope-restricted attention above (what training needs; the paper reports training
 * latency in its experiments). Plain definition, binary64, scope by scope and head by head:
 *   S = scale * Q K^T,  P = softmax_rows(S),  O = P V,
 *   dV = P^T dO,  dP = dO V^T,  D_i = sum_j P_ij dP_ij,  dS = P o (dP - D),  dQ = scale * dS K,  dK = scale * dS^T Q.
 * q,k,v: bf16 [n,C] read through perm as in orc_attn; dout: bf16 [n,C] gradient of the BUCKET-MAJOR output rows.
 * dq, dk, dv: binary64 [n,C], BUCKET-MAJOR rows (row p = gradient of the input row stored at p). lse (may be NULL):
 * [n, heads] natural-log sum of exponentials of the scaled scores of row p. scope_sel (may be NULL): [n] flags;
 * only the scopes that contain a flagged row are computed, and done[p] (may be NULL) is set to 1 for their rows.
 * returns the number of scopes computed, -1 on bad arguments.
 */
int64_t orc_attn_bwd(const uint16_t *q, const uint16_t *k, const uint16_t *v, const uint16_t *dout, const int32_t *perm,
                     const int32_t *offsets, const int32_t *scan_bucket_start, int32_t n_scans, int32_t m, int32_t mode,
                     int32_t s, int32_t t, int32_t heads, int32_t head_dim, double scale, const uint8_t *scope_sel,
                     double *dq, double *dk, double *dv, double *lse, uint8_t *done)
{
    if (m <= 0 || heads <= 0 || head_dim <= 0 || mode < 0 || mode > 2) return -1;
    if (mode == ORC_SHIFT && (s <= 0 || s >= m)) return -1;
    if (mode == ORC_STRIDE && t <= 0) return -1;
    const int64_t C = (int64_t)heads * head_dim;
    int64_t visited = 0;
    for (int32_t b = 0; b < n_scans; ++b) {
        const int64_t kb0 = scan_bucket_start[b], K = scan_bucket_start[b + 1] - kb0;
        if (K <= 0) continue;
        int64_t ngroups = 0;
        for (int64_t j = 0; j < K; ++j) {
            int64_t g = orc_group_of_bucket(j, m, mode, s, t);
            if (g + 1 > ngroups) ngroups = g + 1;
        }
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : visited)
        for (int64_t g = 0; g < ngroups; ++g) {
            int64_t ng = 0;
            for (int64_t j = 0; j < K; ++j)
                if (orc_group_of_bucket(j, m, mode, s, t) == g) ng += offsets[kb0 + j + 1] - offsets[kb0 + j];
            if (ng == 0) continue;
            int64_t *rows = (int64_t *)malloc(sizeof(int64_t) * (size_t)ng);
            int64_t c = 0;
            int wanted = scope_sel ? 0 : 1;
            for (int64_t j = 0; j < K; ++j)
                if (orc_group_of_bucket(j, m, mode, s, t) == g)
                    for (int64_t p = offsets[kb0 + j]; p < offsets[kb0 + j + 1]; ++p) {
                        rows[c++] = p;
                        if (scope_sel && scope_sel[p]) wanted = 1;
                    }
            if (!wanted) { free(rows); continue; }
            ++visited;
            double *P = (double *)malloc(sizeof(double) * (size_t)ng * (size_t)ng);
            double *dS = (double *)malloc(sizeof(double) * (size_t)ng * (size_t)ng);
            for (int32_t h = 0; h < heads; ++h) {
                const int64_t co = (int64_t)h * head_dim;
                for (int64_t a = 0; a < ng; ++a) {          /* P = softmax(scale Q K^T), row by row */
                    const int64_t ia = perm ? perm[rows[a]] : rows[a];
                    double mx = -INFINITY;
                    for (int64_t bb = 0; bb < ng; ++bb) {
                        const int64_t ib = perm ? perm[rows[bb]] : rows[bb];
                        double dot = 0.0;
                        for (int32_t e = 0; e < head_dim; ++e)
                            dot += bf16_to_double(q[ia * C + co + e]) * bf16_to_double(k[ib * C + co + e]);
                        P[a * ng + bb] = dot * scale;
                        if (P[a * ng + bb] > mx) mx = P[a * ng + bb];
                    }
                    double den = 0.0;
                    for (int64_t bb = 0; bb < ng; ++bb) {
                        P[a * ng + bb] = exp(P[a * ng + bb] - mx);
                        den += P[a * ng + bb];
                    }
                    for (int64_t bb = 0; bb < ng; ++bb) P[a * ng + bb] /= den;
                    if (lse) lse[rows[a] * heads + h] = mx + log(den);
                }
                for (int64_t a = 0; a < ng; ++a) {          /* dP = dO V^T, D, dS */
                    double D = 0.0;
                    for (int64_t bb = 0; bb < ng; ++bb) {
                        const int64_t ib = perm ? perm[rows[bb]] : rows[bb];
                        double dp = 0.0;
                        for (int32_t e = 0; e < head_dim; ++e)
                            dp += bf16_to_double(dout[rows[a] * C + co + e]) * bf16_to_double(v[ib * C + co + e]);
                        dS[a * ng + bb] = dp;
                        D += P[a * ng + bb] * dp;
                    }
                    for (int64_t bb = 0; bb < ng; ++bb) dS[a * ng + bb] = P[a * ng + bb] * (dS[a * ng + bb] - D);
                }
                for (int64_t a = 0; a < ng; ++a) {          /* dQ = scale dS K */
                    for (int32_t e = 0; e < head_dim; ++e) {
                        double acc = 0.0;
                        for (int64_t bb = 0; bb < ng; ++bb) {
                            const int64_t ib = perm ? perm[rows[bb]] : rows[bb];
                            acc += dS[a * ng + bb] * bf16_to_double(k[ib * C + co + e]);
                        }
                        dq[rows[a] * C + co + e] = scale * acc;
                    }
                }
                for (int64_t bb = 0; bb < ng; ++bb) {       /* dK = scale dS^T Q,  dV = P^T dO */
                    for (int32_t e = 0; e < head_dim; ++e) {
                        double acck = 0.0, accv = 0.0;
                        for (int64_t a = 0; a < ng; ++a) {
                            const int64_t ia = perm ? perm[rows[a]] : rows[a];
                            acck += dS[a * ng + bb] * bf16_to_double(q[ia * C + co + e]);
                            accv += P[a * ng + bb] * bf16_to_double(dout[rows[a] * C + co + e]);
                        }
                        dk[rows[bb] * C + co + e] = scale * acck;
                        dv[rows[bb] * C + co + e] = accv;
                    }
                }
            }
            if (done)
                for (int64_t a = 0; a < ng; ++a) done[rows[a]] = 1;
            free(dS);
            free(P);
            free(rows);
        }
    }
    return visited;
}

/* Restore input order: dst[perm[p], :] = src[p, :] (the inverse of the one up-front scatter). */
int orc_unpermute(const uint8_t *src, const int32_t *perm, int64_t n, int64_t row_bytes, uint8_t *dst)
{
    if (n < 0 || row_bytes < 0) return -1;
    for (int64_t p = 0; p < n; ++p) memcpy(dst + (int64_t)perm[p] * row_bytes, src + p * row_bytes, (size_t)row_bytes);
    return 0;
}

/* ------------------------------------------------------------------ in-bucket pooling
 * (Section 4.2 "In-bucket Pooling"; Appendix "In-bucket Pooling")
 *
 * The bucket-major array is cut into tiles of `tile` consecutive rows (tiles start at a scan's first row
 * and never span scans). Inside a tile of n rows, M = ceil(n / rho) sub-buckets of capacity rho are built
 * in the Appendix's three steps, and each sub-bucket becomes one pooled row.
 *
 * The Appendix lets block-level atomics decide the order; as for Algorithms 1 and 2 the oracle fixes the
 * index-ordered, round-synchronous schedule:
 *   initial sub-buckets   each point hashes its voxel coordinate (relative to the tile's minimum, one of
 *                         the four hash functions with M as the number of buckets) and the occupied hash
 *                         values receive sub-bucket ids 0, 1, ... from the block counter in the order of
 *                         their first (lowest-row) point. A sub-bucket keeps its first rho points.
 *   new sub-buckets       the points beyond capacity, in row order, each open a new sub-bucket (next id
 *                         of the counter) holding just that point, until the counter reaches M.
 *   find new sub-bucket   the points still left repeat rounds: every one of them picks, from the state at
 *                         the start of the round, the sub-bucket with room whose FIRST point is nearest to
 *                         it (squared distance, binary32, ((dx*dx + dy*dy) + dz*dz), ties to the lower
 *                         id); the contenders of a sub-bucket join in row order while it has room; the
 *                         others try again next round. The text scans "newly allocated" sub-buckets; an
 *                         initial sub-bucket that holds fewer than rho points has room just the same and
 *                         is a candidate here, otherwise capacity could run out.
 * M * rho >= n guarantees that every point is placed, and (M-1) * rho < n that all M sub-buckets exist.
 *
 * coords      [n,3] binary32, BUCKET-MAJOR rows
 * row_offsets [n_scans+1] first row of every scan
 * outputs: sub_of[n]  pooled row of every input row (global numbering: tiles in order, ids inside a tile)
 *          slot_of[n] position of the row inside its sub-bucket (0 .. rho-1), may be NULL
 *          step_of[n] 1 = initial, 2 = opened a new sub-bucket, 2 + r = joined in round r; may be NULL
 *          pooled_offsets[n_scans+1] first pooled row of every scan; may be NULL
 * returns the number of pooled rows, or -1 on bad arguments. */
int64_t orc_pool_assign(const float *coords, const int32_t *row_offsets, int32_t n_scans, int32_t tile, int32_t rho,
                        float voxel_size, int32_t hash, int32_t *sub_of, int32_t *slot_of, int32_t *step_of,
                        int32_t *pooled_offsets)
{
    if (n_scans < 0 || tile < 1 || rho < 1 || !(voxel_size > 0.0f) || hash < 0 || hash > 3 || !sub_of) return -1;
    const float inv = 1.0f / voxel_size;
    int64_t out_base = 0;
    int32_t *v = (int32_t *)malloc(sizeof(int32_t) * 3 * (size_t)tile);
    int64_t *hv = (int64_t *)malloc(sizeof(int64_t) * (size_t)tile);
    int32_t *id_of_hash = (int32_t *)malloc(sizeof(int32_t) * (size_t)tile);
    int32_t *fill = (int32_t *)malloc(sizeof(int32_t) * (size_t)tile);
    int32_t *first = (int32_t *)malloc(sizeof(int32_t) * (size_t)tile);   /* first point of a sub-bucket (local row) */
    int32_t *sub = (int32_t *)malloc(sizeof(int32_t) * (size_t)tile);     /* -1 = not placed yet */
    int32_t *pick = (int32_t *)malloc(sizeof(int32_t) * (size_t)tile);
    int32_t *room = (int32_t *)malloc(sizeof(int32_t) * (size_t)tile);
    for (int32_t b = 0; b < n_scans; ++b) {
        if (pooled_offsets) pooled_offsets[b] = (int32_t)out_base;
        for (int64_t t0 = row_offsets[b]; t0 < row_offsets[b + 1]; t0 += tile) {
            const int64_t t1 = t0 + tile < row_offsets[b + 1] ? t0 + tile : row_offsets[b + 1];
            const int32_t n = (int32_t)(t1 - t0);
            const int32_t M = (n + rho - 1) / rho;
            const float *c = coords + 3 * t0;
            /* voxel coordinate inside the tile, as in Algorithm 1 line 4 */
            float mn[3] = {c[0], c[1], c[2]};
            for (int32_t i = 0; i < n; ++i)
                for (int a = 0; a < 3; ++a)
                    if (c[3 * i + a] < mn[a]) mn[a] = c[3 * i + a];
            int32_t vmax[3] = {0, 0, 0};
            for (int32_t i = 0; i < n; ++i)
                for (int a = 0; a < 3; ++a) {
                    volatile float d = c[3 * i + a] - mn[a];
                    volatile float sc = d * inv;
                    float f = floorf(sc);
                    int32_t q = f >= (float)ORC_VOXEL_MAX ? ORC_VOXEL_MAX : (int32_t)f;
                    if (q < 0) q = 0;
                    v[3 * i + a] = q;
                    if (q > vmax[a]) vmax[a] = q;
                }
            orc_hash_cfg cfg;
            hash_cfg_fill(&cfg, hash, M, vmax, 0, 0);
            for (int32_t i = 0; i < n; ++i) hv[i] = hash_bucket(&cfg, &v[3 * i]);

            /* initial sub-buckets */
            int32_t counter = 0;
            for (int32_t h = 0; h < M; ++h) id_of_hash[h] = -1;
            for (int32_t s = 0; s < M; ++s) fill[s] = 0;
            for (int32_t i = 0; i < n; ++i) {
                const int64_t h = hv[i];
                if (id_of_hash[h] < 0) {
                    id_of_hash[h] = counter;
                    first[counter] = i;
                    ++counter;
                }
                const int32_t s = id_of_hash[h];
                sub[i] = -1;
                if (fill[s] < rho) {
                    sub[i] = s;
                    if (slot_of) slot_of[t0 + i] = fill[s];
                    if (step_of) step_of[t0 + i] = 1;
                    ++fill[s];
                }
            }
            /* new sub-bucket allocation */
            for (int32_t i = 0; i < n && counter < M; ++i) {
                if (sub[i] >= 0) continue;
                const int32_t s = counter++;
                first[s] = i;
                fill[s] = 1;
                sub[i] = s;
                if (slot_of) slot_of[t0 + i] = 0;
                if (step_of) step_of[t0 + i] = 2;
            }
            /* find new sub-bucket, in rounds */
            for (int32_t round = 1;; ++round) {
                int32_t left = 0;
                for (int32_t s = 0; s < M; ++s) room[s] = rho - fill[s];
                for (int32_t i = 0; i < n; ++i) {
                    if (sub[i] >= 0) continue;
                    ++left;
                    int32_t best = -1;
                    float bestd = 0.0f;
                    for (int32_t s = 0; s < M; ++s) {
                        if (room[s] <= 0) continue;
                        const float *a = c + 3 * i, *f = c + 3 * first[s];
                        volatile float dx = a[0] - f[0], dy = a[1] - f[1], dz = a[2] - f[2];
                        volatile float xx = dx * dx, yy = dy * dy, zz = dz * dz;
                        volatile float xy = xx + yy;
                        const float d2 = xy + zz;
                        if (best < 0 || d2 < bestd) { best = s; bestd = d2; }
                    }
                    pick[i] = best;
                }
                if (left == 0) break;
                for (int32_t i = 0; i < n; ++i) {
                    if (sub[i] >= 0) continue;
                    const int32_t s = pick[i];
                    if (s >= 0 && fill[s] < rho) {
                        sub[i] = s;
                        if (slot_of) slot_of[t0 + i] = fill[s];
                        if (step_of) step_of[t0 + i] = 2 + round;
                        ++fill[s];
                    }
                }
                if (round > n + 1) break; /* cannot happen: every round places at least one point */
            }
            for (int32_t i = 0; i < n; ++i) sub_of[t0 + i] = (int32_t)(out_base + sub[i]);
            out_base += M;
        }
    }
    if (pooled_offsets) pooled_offsets[n_scans] = (int32_t)out_base;
    free(room); free(pick); free(sub); free(first); free(fill); free(id_of_hash); free(hv); free(v);
    return out_base;
}

/* binary64 -> bf16 with ONE rounding to nearest even (going through binary32 would round twice). */
static uint16_t double_to_bf16(double x)
{
    if (x != x) return 0x7FC0;
    float f = (float)x;
    if (x != 0.0 && !isinf(x)) {
        int e;
        const double m = frexp(x, &e);              /* x = m * 2^e with 0.5 <= |m| < 1 */
        int keep = 8;                               /* significant bits of a normal bf16 */
        if (e - 1 < -126) keep -= -126 - (e - 1);   /* below the smallest normal exponent fewer bits remain */
        if (keep < 0) keep = 0;
        const double r = nearbyint(ldexp(m, keep)); /* default rounding mode: to nearest, ties to even */
        f = (float)ldexp(r, e - keep);              /* exactly representable (or infinity on overflow) */
    }
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)(u >> 16);
}

/* Reduce the rows of every sub-bucket (Section 4.2: sum, mean, min, max) in binary64 and round once to bf16.
 * op: 0 sum, 1 mean, 2 min, 3 max. feat [n,C] bf16 bucket-major; sub_of [n]; out [n_out,C] bf16;
 * counts [n_out] (may be NULL); coords [n,3] -> pooled_coords [n_out,3] = mean position in binary32 (both may be NULL). */
int orc_pool_reduce(const uint16_t *feat, int64_t n, int32_t C, const int32_t *sub_of, int64_t n_out, int32_t op,
                    uint16_t *out, int32_t *counts, const float *coords, float *pooled_coords)
{
    if (n < 0 || C < 1 || n_out < 0 || op < 0 || op > 3) return -1;
    double *acc = (double *)malloc(sizeof(double) * (size_t)(n_out > 0 ? n_out : 1) * (size_t)C);
    double *cacc = (double *)calloc((size_t)(n_out > 0 ? n_out : 1) * 3, sizeof(double));
    int32_t *cnt = (int32_t *)calloc((size_t)(n_out > 0 ? n_out : 1), sizeof(int32_t));
    for (int64_t p = 0; p < n; ++p) {
        const int64_t s = sub_of[p];
        if (s < 0 || s >= n_out) { free(acc); free(cacc); free(cnt); return -1; }
        for (int32_t ch = 0; ch < C; ++ch) {
            const double x = bf16_to_double(feat[p * C + ch]);
            double *a = &acc[s * C + ch];
            if (cnt[s] == 0) *a = x;
            else if (op <= 1) *a += x;
            else if (op == 2) *a = x < *a ? x : *a;
            else *a = x > *a ? x : *a;
        }
        if (coords)
            for (int a = 0; a < 3; ++a) cacc[s * 3 + a] += (double)coords[3 * p + a];
        ++cnt[s];
    }
    for (int64_t s = 0; s < n_out; ++s) {
        for (int32_t ch = 0; ch < C; ++ch) {
            double x = cnt[s] ? acc[s * C + ch] : 0.0;
            if (op == 1 && cnt[s]) x /= (double)cnt[s];
            out[s * C + ch] = double_to_bf16(x);
        }
        if (pooled_coords)
            for (int a = 0; a < 3; ++a) pooled_coords[s * 3 + a] = cnt[s] ? (float)(cacc[s * 3 + a] / (double)cnt[s]) : 0.0f;
        if (counts) counts[s] = cnt[s];
    }
    free(acc); free(cacc); free(cnt);
    return 0;
}

int orc_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}

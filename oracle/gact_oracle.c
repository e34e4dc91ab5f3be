/*
 * CPU oracle for the GACT activation compressor / decompressor / bit allocator.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, scalar, obviously-correct
 * statement of what the method computes.  It shares no code with the HIP
 * library; only tests, the smoke check and the benchmark's cpu_baseline leg
 * may build or call it.  The product path never routes through it.
 *
 * What it follows (arXiv 2206.11357):
 *   - the stochastic-rounding quantizer of App. A.4 (the transform T_{h,b},
 *     round up with probability T - floor(T), map back with the inverse of T),
 *     applied per group of G consecutive elements of the flattened tensor
 *     (Sec. 5: per-group quantizer; Sec. 3.1: tensors are flattened vectors);
 *   - the bit-allocation integer program Eq. (ilp) of Sec. 4.1 with
 *     S(b) = (2^b-1)^-2 (assumption B2), solved greedily (Sec. 4.2 cites an
 *     O(L log L) greedy without describing it; the descent used here is this
 *     build's reading).
 *
 * Arithmetic contract: IEEE-754 binary32, round-to-nearest-even, every
 * operation rounded on its own (compile with -ffp-contract=off, no fast-math,
 * SSE scalar maths).  The allocator uses binary64 the same way.
 *
 * Conventions the paper leaves open (each is listed as a "reading" in the
 * design notes): group statistics over the group not the tensor; range below
 * 2^-100 is treated as a constant group; strict "u < frac" so on-grid values
 * never move; codes clamped to 2^b-1; packed layout is a linear LSB-first bit
 * string; per group the minimum and the dequantisation step are stored as
 * fp32; 16 random bits per element from Philox4x32-10.
 *
 * Parity unpinned (conventions only oracle<->GPU agreement can confirm): the
 * 2^-100 threshold, the packed layout, storing step (not range), 16 bits per
 * element and the slot order inside a Philox block, allocator tie-break.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define GACT_ORACLE_F32 0
#define GACT_ORACLE_BF16 1

/* threads the group / element loops run on (groups are independent and the
   noise is a function of the index, so threading cannot change a result) */
int gact_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* limit the loops to n threads (n >= 1); used to time the oracle on one core */
void gact_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ------------------------------------------------------------------ Philox */
/*
 * Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11).  One round:
 * two 32x32->64 products of the round multipliers with counter words 0 and 2,
 * the high halves are xor-ed with counter words 1 and 3 and the round key, the
 * low halves pass through in swapped positions; the key is bumped by the two
 * Weyl constants between rounds.
 */
void gact_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2],
                               uint32_t out[4])
{
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = M0 * (uint64_t)c0;
        uint64_t p1 = M1 * (uint64_t)c2;
        uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += W0;
        k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/*
 * Rounding noise for element i of a tensor compressed with `seed`.
 * Key = (low, high) words of seed.  Counter = (low, high words of i/8, 0, 0).
 * The block's four words hold eight 16-bit slots; element i uses slot i%8,
 * low half of a word first.  u = (r16 + 1/2) / 2^16, exact in binary32 and
 * strictly inside (0,1).
 */
float gact_oracle_noise(uint64_t seed, uint64_t i)
{
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint64_t blk = i >> 3;
    uint32_t ctr[4] = { (uint32_t)blk, (uint32_t)(blk >> 32), 0u, 0u };
    uint32_t w[4];
    gact_oracle_philox4x32_10(ctr, key, w);
    unsigned j = (unsigned)(i & 7u);
    uint32_t r16 = (w[j >> 1] >> (16u * (j & 1u))) & 0xFFFFu;
    return ((float)r16 + 0.5f) * 0x1p-16f;
}

/* noise for elements start .. start+n-1 of a tensor (lets a test check a slice
   of a large tensor: groups are independent once their noise is given) */
void gact_oracle_noise_fill(uint64_t seed, uint64_t start, int64_t n, float *u)
{
    for (int64_t i = 0; i < n; ++i) u[i] = gact_oracle_noise(seed, start + (uint64_t)i);
}

/* ------------------------------------------------------------ bf16 <-> f32 */
static float bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* round-to-nearest-even on the 16 discarded bits; NaN stays NaN */
static uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u)
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

static float load_elem(const void *x, int dtype, int64_t i)
{
    if (dtype == GACT_ORACLE_BF16)
        return bf16_to_f32(((const uint16_t *)x)[i]);
    return ((const float *)x)[i];
}

/* ------------------------------------------------------------------ sizes */
int64_t gact_oracle_num_groups(int64_t n, int group_size)
{
    return (n + group_size - 1) / group_size;
}

/* ceil(n*bits/8), rounded up to a multiple of 16 bytes */
int64_t gact_oracle_packed_bytes(int64_t n, int bits)
{
    int64_t bytes = (n * (int64_t)bits + 7) / 8;
    return (bytes + 15) / 16 * 16;
}

static int args_ok(int64_t n, int group_size, int bits, int dtype)
{
    if (n < 0) return 0;
    if (!(bits == 1 || bits == 2 || bits == 4 || bits == 8)) return 0;
    if (group_size < 32 || group_size > 1024 || group_size % 32) return 0;
    if (!(dtype == GACT_ORACLE_F32 || dtype == GACT_ORACLE_BF16)) return 0;
    return 1;
}

/* --------------------------------------------------------------- compress */
/*
 * App. A.4 quantizer per group, with the rounding noise handed in: u has one
 * float per element (the seeded entry point below draws it from Philox; tests
 * pass their own to enumerate the rounding rule).  All pointers are host
 * memory.  `packed` has gact_oracle_packed_bytes(n, bits) bytes and is fully
 * written (pad = 0); gmin / gscale have one float per group.  Returns 0, or
 * -1 on a bad argument.
 */
int gact_oracle_compress_with_noise(const void *x, int dtype, int64_t n,
                                    int group_size, int bits, const float *u,
                                    uint8_t *packed, float *gmin, float *gscale)
{
    if (!args_ok(n, group_size, bits, dtype)) return -1;
    const int64_t G = group_size;
    const int64_t NG = gact_oracle_num_groups(n, group_size);
    const int levels = (1 << bits) - 1;          /* B = 2^b - 1 */
    const float Bf = (float)levels;
    memset(packed, 0, (size_t)gact_oracle_packed_bytes(n, bits));

    #pragma omp parallel for schedule(static)
    for (int64_t g = 0; g < NG; ++g) {
        const int64_t lo = g * G;
        const int64_t hi = (lo + G < n) ? lo + G : n;

        /* group statistics over the valid elements */
        float mn = load_elem(x, dtype, lo);
        float mx = mn;
        for (int64_t i = lo + 1; i < hi; ++i) {
            float v = load_elem(x, dtype, i);
            if (v < mn) mn = v;
            if (v > mx) mx = v;
        }
        mn = mn + 0.0f;                          /* -0.0 becomes +0.0 */
        const float range = mx - mn;
        float inv, step;
        if (!(range >= 0x1p-100f)) { inv = 0.0f; step = 0.0f; }
        else { inv = Bf / range; step = range / Bf; }
        gmin[g] = mn;
        gscale[g] = step;

        /* T(h_j), stochastic rounding, packing */
        for (int64_t i = lo; i < hi; ++i) {
            float v = load_elem(x, dtype, i);
            float d = v - mn;
            float t = d * inv;
            float f = floorf(t);
            float frac = t - f;
            int q = (int)f + ((u[i] < frac) ? 1 : 0);
            if (q > levels) q = levels;
            /* element i occupies bits [i*b, i*b+b) of the bit string; bit k of
               the string is bit k%8 of byte k/8.  b divides 8, so a code never
               straddles a byte; G*b is a multiple of 32, so groups never share
               a byte and the parallel loop is race-free. */
            int64_t bitpos = i * (int64_t)bits;
            packed[bitpos >> 3] |= (uint8_t)((unsigned)q << (bitpos & 7));
        }
    }
    return 0;
}

/* The compressor as the library exposes it: noise from (seed, element index). */
int gact_oracle_compress(const void *x, int dtype, int64_t n, int group_size,
                         int bits, uint64_t seed, uint8_t *packed,
                         float *gmin, float *gscale)
{
    if (!args_ok(n, group_size, bits, dtype)) return -1;
    float *u = (float *)malloc(sizeof(float) * (size_t)(n > 0 ? n : 1));
    if (!u) return -1;
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) u[i] = gact_oracle_noise(seed, (uint64_t)i);
    int rc = gact_oracle_compress_with_noise(x, dtype, n, group_size, bits, u,
                                             packed, gmin, gscale);
    free(u);
    return rc;
}

/* code of element i, read back from the bit string */
static unsigned unpack_code(const uint8_t *packed, int64_t i, int bits)
{
    int64_t bitpos = i * (int64_t)bits;
    return ((unsigned)packed[bitpos >> 3] >> (bitpos & 7)) & ((1u << bits) - 1u);
}

/* ------------------------------------------------------------- decompress */
/* Inverse transform: y = fl(fl(q * step) + min); bf16 output rounds y once
   more, to nearest even. */
int gact_oracle_decompress(const uint8_t *packed, const float *gmin,
                           const float *gscale, int64_t n, int group_size,
                           int bits, void *y, int dtype)
{
    if (!args_ok(n, group_size, bits, dtype)) return -1;
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        int64_t g = i / group_size;
        float q = (float)unpack_code(packed, i, bits);
        float prod = q * gscale[g];
        float v = prod + gmin[g];
        if (dtype == GACT_ORACLE_BF16) ((uint16_t *)y)[i] = f32_to_bf16_rne(v);
        else ((float *)y)[i] = v;
    }
    return 0;
}

/* codes as one byte each (test helper: lets a test look at q without
   re-implementing the unpacking) */
int gact_oracle_unpack_codes(const uint8_t *packed, int64_t n, int bits,
                             uint8_t *codes)
{
    if (!(bits == 1 || bits == 2 || bits == 4 || bits == 8) || n < 0) return -1;
    for (int64_t i = 0; i < n; ++i) codes[i] = (uint8_t)unpack_code(packed, i, bits);
    return 0;
}

/* ---------------------------------------------------------- bit allocator */
/*
 * Eq. (ilp): minimise sum_l c_l S(b_l) subject to sum_l b_l D_l <= budget,
 * b_l in {1,2,4,8}, S(b) = (2^b-1)^-2.  Greedy descent: start from 8 bits
 * everywhere; while over budget, take the single one-level step (8->4, 4->2,
 * 2->1 of one tensor) that adds the least variance per bit saved, ties to the
 * lowest tensor index.  Stops at the first feasible state.  Plain O(L) scan
 * per step.  budget = floor(avg * sum D).  Returns 0, -1 bad argument,
 * -4 if avg < 1 (no feasible scheme).
 */
/* Same greedy descent over a caller-given ascending level set drawn from
 * {1,2,4,8,32}; 32 means "leave the tensor uncompressed" (the paper keeps up
 * to 32 bits for the most sensitive tensors, Sec. 6.1), S(32) = (2^32-1)^-2.
 * Starts from the top level; -4 if avg is below the lowest level. */
int gact_oracle_allocate_bits_levels(const float *sensitivity, const int64_t *numel,
                                     int L, double avg_bit_budget,
                                     const int32_t *level, int n_levels,
                                     int32_t *bits_out)
{
    if (L < 0 || n_levels < 1 || n_levels > 5) return -1;
    double S[5];
    for (int k = 0; k < n_levels; ++k) {
        int b = level[k];
        if (!(b == 1 || b == 2 || b == 4 || b == 8 || b == 32)) return -1;
        if (k > 0 && level[k] <= level[k - 1]) return -1;
        double B = ldexp(1.0, b) - 1.0;          /* 2^b - 1 */
        S[k] = 1.0 / (B * B);
    }
    if (!(avg_bit_budget >= (double)level[0])) return -4;
    const int top = n_levels - 1;
    uint64_t total = 0;
    for (int l = 0; l < L; ++l) {
        double c = (double)sensitivity[l];
        if (!(c >= 0.0) || isinf(c) || numel[l] < 0) return -1;
        total += (uint64_t)numel[l];
    }
    int *idx = (int *)malloc(sizeof(int) * (size_t)(L > 0 ? L : 1));
    if (!idx) return -1;
    for (int l = 0; l < L; ++l) { idx[l] = top; bits_out[l] = level[top]; }
    double cap = floor(avg_bit_budget * (double)total);
    uint64_t budget = (cap >= 18446744073709549568.0) ? UINT64_MAX : (uint64_t)cap;
    uint64_t used = (uint64_t)level[top] * total;

    while (used > budget) {
        int best = -1;
        double best_key = 0.0;
        for (int l = 0; l < L; ++l) {
            if (numel[l] == 0 || idx[l] == 0) continue;
            int hi = level[idx[l]], lo = level[idx[l] - 1];
            double key = ((double)sensitivity[l] * (S[idx[l] - 1] - S[idx[l]]))
                       / ((double)numel[l] * (double)(hi - lo));
            if (best < 0 || key < best_key) { best = l; best_key = key; }
        }
        if (best < 0) break;                     /* cannot happen when avg >= lowest level */
        int hi = level[idx[best]], lo = level[idx[best] - 1];
        idx[best] -= 1;
        bits_out[best] = lo;
        used -= (uint64_t)numel[best] * (uint64_t)(hi - lo);
    }
    free(idx);
    return 0;
}

int gact_oracle_allocate_bits(const float *sensitivity, const int64_t *numel,
                              int L, double avg_bit_budget, int32_t *bits_out)
{
    static const int32_t level[4] = { 1, 2, 4, 8 };
    return gact_oracle_allocate_bits_levels(sensitivity, numel, L, avg_bit_budget,
                                            level, 4, bits_out);
}

/* ------------------------------------------- sensitivity and variance alert */
/*
 * Alg. 1 (Sec. 4.2) returns, for tensor l, 1/2 ||g0 - g1||^2 / S(b_l), where
 * g0 and g1 are the full gradients of two iterations that differ only in the
 * seed of tensor l's compressor.  The gradient is a list of K parameter
 * buffers; the norm runs over all of them.  Binary64 terms, compensated
 * accumulation in index order.
 */
static double load_elem_f64(const void *x, int dtype, int64_t i)
{
    return (double)load_elem(x, dtype, i);
}

/* Compensated (Neumaier) accumulator: the sums below are defined in exact
   arithmetic; a plain running binary64 sum of N positive terms drifts by about
   1e-10 relative at N = 1e8, this one stays within a few ulp for any N. */
typedef struct { double sum, comp; } acc_t;
static void acc_add(acc_t *a, double x)
{
    double t = a->sum + x;
    if (fabs(a->sum) >= fabs(x)) a->comp += (a->sum - t) + x;
    else a->comp += (x - t) + a->sum;
    a->sum = t;
}
static double acc_value(const acc_t *a) { return a->sum + a->comp; }

int gact_oracle_sensitivity(const void *const *g0, const void *const *g1,
                            const int64_t *numel, const int *dtype, int K,
                            int bits, double *out)
{
    if (K < 0 || !(bits == 1 || bits == 2 || bits == 4 || bits == 8)) return -1;
    acc_t acc = { 0.0, 0.0 };
    for (int k = 0; k < K; ++k) {
        if (numel[k] < 0) return -1;
        for (int64_t i = 0; i < numel[k]; ++i) {
            double d = load_elem_f64(g0[k], dtype[k], i) - load_elem_f64(g1[k], dtype[k], i);
            acc_add(&acc, d * d);
        }
    }
    double B = (double)((1 << bits) - 1);
    *out = 0.5 * acc_value(&acc) * (B * B);   /* dividing by S(b) = (2^b-1)^-2 */
    return 0;
}

/*
 * Running mean of the gradient (Sec. 4.2: "the overall gradient variance can
 * be computed by maintaining a running mean of the gradient").  Step t >= 1:
 *   mean <- mean + (g - mean) * rt,   rt = (float)(1 / t) rounded once,
 * each operation in binary32.  Returns sum g^2 and sum mean_new^2 in binary64.
 */
int gact_oracle_grad_stats_update(const void *g, float *mean, int64_t n,
                                  int dtype, int64_t t, double *sum_g2,
                                  double *sum_m2)
{
    if (n < 0 || t < 1) return -1;
    const float rt = (float)(1.0 / (double)t);
    acc_t a = { 0.0, 0.0 }, b = { 0.0, 0.0 };
    for (int64_t i = 0; i < n; ++i) {
        float gi = load_elem(g, dtype, i);
        float d = gi - mean[i];
        float s = d * rt;
        float m = mean[i] + s;
        mean[i] = m;
        acc_add(&a, (double)gi * (double)gi);
        acc_add(&b, (double)m * (double)m);
    }
    *sum_g2 += acc_value(&a);
    *sum_m2 += acc_value(&b);
    return 0;
}

/* V(b) = sum_l c_l S(b_l) (Thm. 2, Eq. (var-decomposition)) over the gradient
   variance; the caller alerts when the ratio exceeds its threshold. */
int gact_oracle_variance_ratio(const float *c, const int32_t *bits, int L,
                               double grad_var, double *ratio)
{
    double V = 0.0;
    for (int l = 0; l < L; ++l) {
        int b = bits[l];
        /* 32 = a tensor the allocator left uncompressed (Sec. 6.1); S(b) = (2^b - 1)^-2
           of Sec. 4.1 evaluated at b = 32 */
        if (!(b == 1 || b == 2 || b == 4 || b == 8 || b == 32) || !(c[l] >= 0.0f)) return -1;
        double B = ldexp(1.0, b) - 1.0;
        V += (double)c[l] / (B * B);
    }
    if (!(grad_var > 0.0)) return -1;
    *ratio = V / grad_var;
    return 0;
}

/* ---------------------------------------------------------------- footprint */
/*
 * Footprint for duplicate detection (Sec. 5.2: a tensor saved by several
 * operators is recognised by its data pointer, sampled points and sum).
 * out[0] = sum of all elements; out[1 + j] = element floor(j * n / n_samples),
 * j < n_samples, widened to binary64.  The data pointer is the caller's part.
 */
int gact_oracle_footprint(const void *x, int64_t n, int dtype, int n_samples,
                          double *out)
{
    if (n < 0 || n_samples < 0 || !(dtype == GACT_ORACLE_F32 || dtype == GACT_ORACLE_BF16)) return -1;
    acc_t acc = { 0.0, 0.0 };
    for (int64_t i = 0; i < n; ++i) acc_add(&acc, load_elem_f64(x, dtype, i));
    out[0] = acc_value(&acc);
    for (int j = 0; j < n_samples; ++j) {
        int64_t i = n > 0 ? (int64_t)(((__int128)j * (__int128)n) / n_samples) : 0;
        out[1 + j] = n > 0 ? load_elem_f64(x, dtype, i) : 0.0;
    }
    return 0;
}

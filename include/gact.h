/*
 * gact.h -- C ABI of the MI355X (gfx950) activation compressor / decompressor
 * of GACT (arXiv 2206.11357) and its host-side bit allocator.
 *
 * What the calls compute
 *   The paper's compressor Q is a per-group stochastic-rounding quantizer
 *   (Sec. 5: quantisation per group; App. A.4: transform
 *   T(h_j) = (2^b-1)(h_j - min h)/(max h - min h), round up with probability
 *   T - floor(T), otherwise down, and map back with the inverse of T).  A
 *   context tensor is a flattened vector (Sec. 3.1); it is cut into groups of
 *   `group_size` consecutive elements, the last group may be shorter.
 *   Per-tensor bit widths b_l come from Eq. (ilp) of Sec. 4.1,
 *   min sum_l c_l S(b_l) s.t. sum_l b_l D_l <= budget, S(b) = (2^b-1)^-2.
 *
 * Arithmetic (bit-exact contract)
 *   IEEE binary32, round to nearest even, every operation rounded on its own
 *   (no fused multiply-add where it would change a result):
 *     mn = min, mx = max over the group;  mn = mn + 0.0f (so -0 is stored as +0)
 *     range = mx - mn;  B = 2^bits - 1
 *     range >= 2^-100 :  inv = B / range,  step = range / B
 *     otherwise       :  inv = 0,          step = 0        (constant group)
 *     t = (x - mn) * inv;  q = floor(t) + (u < t - floor(t));  q = min(q, B)
 *     y = q * step + mn                  (decompress; bf16 output rounds y RNE)
 *   Rounding noise u for element i of a tensor compressed with `seed`:
 *   Philox4x32-10 (Salmon et al., SC'11), key = (low, high 32 bits of seed),
 *   counter = (low, high 32 bits of i/8, 0, 0).  The four output words hold
 *   eight 16-bit slots, low half first; element i takes slot i%8 and
 *   u = (slot + 0.5) / 65536.  (For a shard, i counts from the descriptor's
 *   index_base.)  The stream is a function of (seed, i) only, so
 *   results never depend on launch shape or on single- vs multi-tensor calls,
 *   and the same seed replays the same compression (Alg. 1 of the paper relies
 *   on replayable per-tensor seeds).
 *
 * Layouts
 *   packed : linear bit string, element i in bits [i*bits, (i+1)*bits), bit k
 *            of the string is bit k%8 of byte k/8 (little-endian, LSB first).
 *            gact_packed_bytes(n, bits) bytes; all pad bits are written as 0.
 *   gmin   : float[gact_num_groups]  group minimum.
 *   gscale : float[gact_num_groups]  dequantisation step, range / (2^bits-1).
 *
 * Memory and ownership
 *   Pointers named d_* are DEVICE pointers owned by the caller; h_* are HOST
 *   pointers.  The library allocates nothing, frees nothing and keeps no
 *   pointer after a call returns.  d_x, d_y, d_packed and the multi-tensor
 *   workspace must be 16-byte aligned; d_gmin / d_gscale 4-byte aligned.
 *   Device calls enqueue work on `stream` (a hipStream_t passed as void*;
 *   NULL is the default stream) and return without waiting for it.
 *
 * Errors
 *   Every call returns GACT_OK or a negative code; on error nothing has been
 *   enqueued.  Inputs must be finite with max - min finite; NaN / Inf give
 *   unspecified values but never an out-of-bounds access.
 */
#ifndef GACT_H
#define GACT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { GACT_F32 = 0, GACT_BF16 = 1 } gact_dtype;

/* Bit width that means "leave this tensor uncompressed" in the allocator's
 * level sets and in multi-tensor descriptors. */
#define GACT_BITS_UNCOMPRESSED 32

enum {
    GACT_OK       =  0,
    GACT_E_ARG    = -1,  /* null pointer, n < 0, misaligned pointer, bad dtype, L < 0,
                            negative / non-finite sensitivity or numel, workspace too small */
    GACT_E_BITS   = -2,  /* bits not in {1,2,4,8} */
    GACT_E_GROUP  = -3,  /* group_size not a multiple of 32 in [32, 1024] */
    GACT_E_BUDGET = -4,  /* avg_bit_budget < 1 or NaN: no feasible scheme */
    GACT_E_HIP    = -5,  /* the HIP runtime refused the launch or copy */
    GACT_E_CAPTURE = -6, /* the stream is being captured into a HIP graph and this call
                            would have to upload a table from host memory */
    GACT_E_SCRATCH = -7  /* gact_compress_footprint_noalloc: the tensor needs more than the
                            library's static scratch area */
};

/* ceil(n / group_size); 0 when n <= 0 or group_size <= 0. */
size_t gact_num_groups(int64_t n, int group_size);

/* ceil(n * bits / 8) rounded up to a multiple of 16; 0 when n <= 0. */
size_t gact_packed_bytes(int64_t n, int bits);

/* Human-readable name of an error code (static string). */
const char *gact_error_string(int code);

/*
 * Compressor (forward pass; App. A.4 applied per group, Sec. 5).
 *   d_x      in   n elements of `dtype`, contiguous, not modified
 *   d_packed out  gact_packed_bytes(n, bits) bytes
 *   d_gmin   out  gact_num_groups(n, group_size) floats
 *   d_gscale out  same count
 * n == 0 is GACT_OK and launches nothing.
 */
int gact_compress(const void *d_x, gact_dtype dtype, int64_t n, int group_size,
                  int bits, uint64_t seed, void *d_packed, float *d_gmin,
                  float *d_gscale, void *stream);

/*
 * Decompressor (backward pass; inverse transform of App. A.4).
 *   d_y out  n elements of `dtype`.  Must not overlap the inputs.
 */
int gact_decompress(const void *d_packed, const float *d_gmin,
                    const float *d_gscale, int64_t n, int group_size, int bits,
                    void *d_y, gact_dtype dtype, void *stream);

/*
 * Multi-tensor launches: the many saved tensors of one iteration (the paper's
 * hook compresses every saved tensor of every operator, Sec. 5) in one launch
 * per direction.  Each descriptor carries its own element count, dtype, bits
 * and seed (the per-tensor seeds r_l of Alg. 1).  The result for each tensor
 * is byte-identical to the single-tensor call with the same arguments.
 *
 *   h_descs          host array of L descriptors; device pointers inside.
 *                    compress reads x and writes packed/gmin/gscale (y unused);
 *                    decompress reads packed/gmin/gscale and writes y (x unused).
 *   d_workspace      device scratch of at least gact_multi_workspace_bytes(L)
 *                    bytes, 16-byte aligned.  With more than 64 non-empty
 *                    tensors it holds the launch table until the enqueued
 *                    kernel has run, so it must not be reused for a different
 *                    table before then; smaller tables travel in the kernel
 *                    arguments and leave it untouched.
 * A table in the workspace is uploaded with a stream-ordered copy from host
 * memory the call owns; h_descs may be reused as soon as the call returns.
 * HIP graphs: with at most 64 non-empty tensors a call enqueues exactly one
 * kernel and can be captured (pointers, sizes, bits and seeds are baked into
 * the node).  A larger table needs an upload from host memory the call owns,
 * which a graph could not replay: on a capturing stream such a call enqueues
 * nothing and returns GACT_E_CAPTURE -- capture those sets in slices of 64.
 * Shards: the noise of element i is a function of (seed, index_base + i) only,
 * so a tensor cut at multiples of the group size and compressed piece by piece
 * (on one GPU or on several), each piece with the tensor's seed and its own
 * offset as index_base, gives pieces whose packed strings, minima and steps
 * concatenate to the result for the whole tensor.  index_base must be a
 * non-negative multiple of 8 (GACT_E_ARG otherwise); decompress ignores it.
 * A descriptor with bits == GACT_BITS_UNCOMPRESSED is skipped by both calls:
 * the allocator left that tensor at full precision and the caller keeps it.
 * L == 0, or all n == 0, is GACT_OK and launches nothing.
 */
typedef struct {
    const void *x;
    void       *packed;
    float      *gmin;
    float      *gscale;
    void       *y;
    int64_t     n;
    uint64_t    seed;
    int32_t     bits;
    int32_t     dtype;     /* gact_dtype */
    int64_t     index_base; /* compress: index of x[0] in the noise stream (see below); 0 for a whole tensor */
} gact_tensor_desc;

size_t gact_multi_workspace_bytes(int L);

int gact_compress_multi(const gact_tensor_desc *h_descs, int L, int group_size,
                        void *d_workspace, size_t workspace_bytes, void *stream);

int gact_decompress_multi(const gact_tensor_desc *h_descs, int L, int group_size,
                          void *d_workspace, size_t workspace_bytes, void *stream);

/*
 * Sensitivity of one context tensor (Alg. 1, Sec. 4.2).  g0 and g1 are the
 * gradients of two iterations that differ only in the seed of tensor l's
 * compressor, each a list of K parameter buffers; the call computes
 *     c_l = 1/2 * sum_k ||g0_k - g1_k||^2 / S(bits),   S(b) = (2^b-1)^-2,
 * `bits` being the width tensor l was compressed with, accumulated in binary64
 * in a fixed order (the result does not depend on scheduling).
 *   h_pairs      host array of K buffer pairs; device pointers inside, 16-byte
 *                aligned, both buffers of a pair have n elements of `dtype`.
 *   d_out        device double[1], receives c_l when the stream reaches it.
 *   d_workspace  device scratch, >= gact_reduce_workspace_bytes(K, sum of n),
 *                16-byte aligned; in use until the enqueued kernels have run.
 * K == 0 or all n == 0 writes 0.
 * The buffer table is uploaded from host memory the call owns, so this call
 * and gact_grad_stats_update return GACT_E_CAPTURE, with nothing enqueued, on
 * a stream that is being captured into a HIP graph.
 */
typedef struct {
    const void *g0;
    const void *g1;
    int64_t     n;
    int32_t     dtype;     /* gact_dtype */
    int32_t     reserved;
} gact_grad_pair;

size_t gact_reduce_workspace_bytes(int K, int64_t total_elems);

int gact_sensitivity(const gact_grad_pair *h_pairs, int K, int bits, double *d_out,
                     void *d_workspace, size_t workspace_bytes, void *stream);

/*
 * Running gradient statistics for the a-posteriori alert of Sec. 4.2, which
 * needs the variance of the gradient and obtains it from a running mean kept
 * over the iterations.  Step t >= 1 over K parameter buffers, binary32 per element:
 *     mean <- mean + (g - mean) * rt,    rt = (float)(1 / t),
 * and, in binary64, d_out[0] = sum g^2, d_out[1] = sum mean_new^2.  With the
 * caller's running average s_t of d_out[0], Var[g] ~ s_t - d_out[1].
 *   mean   device float[n] per buffer, read and written in place (start at 0).
 */
typedef struct {
    const void *g;
    float      *mean;
    int64_t     n;
    int32_t     dtype;     /* gact_dtype of g */
    int32_t     reserved;
} gact_grad_stat;

int gact_grad_stats_update(const gact_grad_stat *h_stats, int K, int64_t t, double *d_out,
                           void *d_workspace, size_t workspace_bytes, void *stream);

/*
 * Footprint of a tensor for duplicate detection (Sec. 5.2: a tensor saved by
 * several operators is recognised by its data pointer, sampled points and its
 * sum, and compressed once).  One read of the tensor:
 *     d_out[0]     = sum of all elements, binary64, fixed order
 *     d_out[1 + j] = element floor(j * n / n_samples), j < n_samples <= 32768
 *   d_workspace  >= gact_reduce_workspace_bytes(1, n) bytes, 16-byte aligned.
 * n == 0 writes zeros.
 */
int gact_footprint(const void *d_x, gact_dtype dtype, int64_t n, int n_samples, double *d_out,
                   void *d_workspace, size_t workspace_bytes, void *stream);

/*
 * Compressor and footprint from one read of the tensor: the sum is taken in
 * the pass that computes the group statistics (Sec. 5.2 names the footprint,
 * App. A.4 the statistics).  Arguments and results of gact_compress, plus
 *   d_footprint  out  double[1 + n_samples], as gact_footprint defines it
 *                     (the sum is accumulated in another fixed order, so it
 *                     may differ from gact_footprint's in the last bits)
 *   d_workspace       >= gact_compress_footprint_workspace_bytes(n, group_size)
 *                     bytes, 16-byte aligned, in use until the kernels have run
 * A caller that finds the footprint among tensors it already holds drops the
 * new compressed copy and keeps the old one.  n == 0 writes zeros.
 */
size_t gact_compress_footprint_workspace_bytes(int64_t n, int group_size);
int gact_compress_footprint(const void *d_x, gact_dtype dtype, int64_t n, int group_size,
                            int bits, uint64_t seed, void *d_packed, float *d_gmin,
                            float *d_gscale, int n_samples, double *d_footprint,
                            void *d_workspace, size_t workspace_bytes, void *stream);

/*
 * Copy of nbytes between buffers a kernel can address -- device memory, or host
 * memory that is pinned and mapped (hipHostMalloc) -- by a kernel of
 * `workgroups` workgroups (1..1024), enqueued on `stream`.  For the swap of
 * compressed activations to the host that Sec. 5.3 runs on a stream of its own
 * next to the forward pass: a few workgroups keep PCIe busy and leave the rest
 * of the GPU to the model, which the runtime's own device-to-host copy kernel
 * does not.  dst and src 16-byte aligned and not overlapping.  A pointer that
 * no kernel may touch (ordinary host memory) returns GACT_E_ARG, nothing is
 * enqueued.
 */
int gact_copy_bounded(void *dst, const void *src, size_t nbytes, int workgroups, void *stream);

/*
 * gact_compress_footprint for callers that cannot allocate device memory and
 * so cannot bring a workspace: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  The per-tile partial sums go to a
 * scratch area of GACT_NOALLOC_SCRATCH_BYTES that is part of the library's
 * device image (each GPU the library runs on holds one copy until the process
 * ends); the call allocates and frees nothing.  Same arguments, results and
 * error codes as gact_compress_footprint without the workspace pair; results
 * are byte-identical to that call's.
 *   Limit: one 8-byte partial per tile of 2048 elements (63 * 32 ... 64 * 32
 *   elements when group_size / 32 is not a power of two), i.e. up to
 *   536,870,912 elements for power-of-two group sizes.  A larger n returns
 *   GACT_E_SCRATCH and enqueues nothing.
 *   All calls on one GPU share that GPU's area: two calls whose kernels may
 *   overlap in time (different streams, or graph launches in flight together)
 *   race on it and must be ordered by the caller.  The area keeps the last
 *   call's contents; nothing in it has to start at zero, because every partial
 *   a call reads was written by that call's own compress kernel.
 */
#define GACT_NOALLOC_SCRATCH_BYTES (2u << 20)
int gact_compress_footprint_noalloc(const void *d_x, gact_dtype dtype, int64_t n, int group_size,
                                    int bits, uint64_t seed, void *d_packed, float *d_gmin,
                                    float *d_gscale, int n_samples, double *d_footprint,
                                    void *stream);

/*
 * Variance alert (host only): V(b) = sum_l c_l S(b_l) (Thm. 2) against the
 * gradient variance.  Writes V / grad_var to *h_ratio (may be NULL) and
 * returns 1 if it exceeds `threshold`, 0 if not, a negative code on error.
 * b_l in {1, 2, 4, 8, GACT_BITS_UNCOMPRESSED}: a tensor that
 * gact_allocate_bits_levels left uncompressed counts with S(32) = (2^32-1)^-2.
 */
int gact_variance_alert(const float *h_sensitivity, const int32_t *h_bits, int L,
                        double grad_var, double threshold, double *h_ratio);

/*
 * Bit allocator (host only, synchronous; Eq. (ilp), Sec. 4.1-4.2).
 *   h_sensitivity in  c_l >= 0, finite, L floats (Alg. 1's estimate)
 *   h_numel       in  D_l >= 0, L values
 *   avg_bit_budget    budget = floor(avg * sum_l D_l) bits; must be >= 1
 *   h_bits_out    out b_l in {1,2,4,8}
 * Greedy descent from 8 bits: repeatedly apply the one-level step
 * (8->4, 4->2, 2->1 of one tensor) with the least added variance per bit
 * saved, c_l (S(lo) - S(hi)) / (D_l (hi - lo)) in binary64, ties to the lowest
 * index, until sum b_l D_l <= budget.  Tensors with D_l = 0 keep 8.
 */
int gact_allocate_bits(const float *h_sensitivity, const int64_t *h_numel, int L,
                       double avg_bit_budget, int32_t *h_bits_out);

/*
 * The same program over a caller-given level set: h_levels is strictly
 * ascending and drawn from {1, 2, 4, 8, GACT_BITS_UNCOMPRESSED}; the descent
 * starts from the top level and avg_bit_budget must be >= the lowest.  With 32
 * in the set the most sensitive tensors can stay uncompressed, as in the
 * paper's experiments (Sec. 6.1), S(32) = (2^32-1)^-2.
 * gact_allocate_bits is this call with levels {1, 2, 4, 8}.
 */
int gact_allocate_bits_levels(const float *h_sensitivity, const int64_t *h_numel, int L,
                              double avg_bit_budget, const int32_t *h_levels, int n_levels,
                              int32_t *h_bits_out);

#ifdef __cplusplus
}
#endif
#endif /* GACT_H */

// Sensitivity reduction of GACT's Alg. 1 (arXiv 2206.11357, Sec. 4.2) and the
// running gradient statistics behind its variance alert, for MI355X (gfx950).
//
// Both are multi-buffer streaming reductions bound by HBM reads: a block of
// 256 threads takes 16 KB of each input buffer with coalesced 16-byte loads,
// accumulates in binary64 per thread, reduces over the block, and writes one
// partial per block; a second, single-block kernel adds the partials in a
// fixed order, so results do not depend on scheduling.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gact_device.h"

namespace gact {

typedef uint32_t u4r __attribute__((ext_vector_type(4)));
typedef float    f4r __attribute__((ext_vector_type(4)));

constexpr int kRedThreads = 256;

__device__ __forceinline__ double block_sum(double v, double* lds) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (lane == 0) lds[wave] = v;
    __syncthreads();
    double r = 0.0;
    if (threadIdx.x == 0) r = (lds[0] + lds[1]) + (lds[2] + lds[3]);
    __syncthreads();
    return r;                       // valid in thread 0
}

__device__ __forceinline__ int find_buffer(const uint32_t* first_block, int K, uint32_t b) {
    int lo = 0, hi = K;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (first_block[mid] <= b) lo = mid; else hi = mid;
    }
    return lo;
}

// eight fp32 values of a 16-byte piece of bf16, or four of fp32 (rest unused)
template <int DT>
__device__ __forceinline__ void unpack_piece(const u4r w, float v[8]) {
    // components are copied to scalars first: a bit cast applied directly to a
    // vector component reads component 0
    const uint32_t c0 = w.x, c1 = w.y, c2 = w.z, c3 = w.w;
    if (DT == GACT_DT_F32) {
        v[0] = __builtin_bit_cast(float, c0); v[1] = __builtin_bit_cast(float, c1);
        v[2] = __builtin_bit_cast(float, c2); v[3] = __builtin_bit_cast(float, c3);
    } else {
        v[0] = __builtin_bit_cast(float, c0 << 16); v[1] = __builtin_bit_cast(float, c0 & 0xFFFF0000u);
        v[2] = __builtin_bit_cast(float, c1 << 16); v[3] = __builtin_bit_cast(float, c1 & 0xFFFF0000u);
        v[4] = __builtin_bit_cast(float, c2 << 16); v[5] = __builtin_bit_cast(float, c2 & 0xFFFF0000u);
        v[6] = __builtin_bit_cast(float, c3 << 16); v[7] = __builtin_bit_cast(float, c3 & 0xFFFF0000u);
    }
}

// One 16-byte piece starting at element e of a buffer with n elements; pieces
// that cross the end are read element by element and padded with zeros.
template <int DT, bool FULL = false>
__device__ __forceinline__ u4r load_piece16(const void* base, int64_t e, int64_t n) {
    constexpr int P = DT == GACT_DT_F32 ? 4 : 8;
    u4r w = {0u, 0u, 0u, 0u};
    if (FULL || e + P <= n) {
        if (DT == GACT_DT_F32) w = __builtin_nontemporal_load((const u4r*)((const uint32_t*)base + e));
        else w = __builtin_nontemporal_load((const u4r*)((const uint16_t*)base + e));
    } else if (e < n) {
        uint32_t t[4] = {0u, 0u, 0u, 0u};
        if (DT == GACT_DT_F32) {
            for (int j = 0; j < P; ++j) if (e + j < n) t[j] = ((const uint32_t*)base)[e + j];
        } else {
            for (int j = 0; j < P; ++j)
                if (e + j < n) t[j >> 1] |= (uint32_t)((const uint16_t*)base)[e + j] << (16 * (j & 1));
        }
        w.x = t[0]; w.y = t[1]; w.z = t[2]; w.w = t[3];
    }
    return w;
}

// ------------------------------------------------------------- sensitivity
// FULL: the whole chunk lies inside the buffer, so all loads are unguarded and
// issued back to back.
template <int DT, bool FULL>
__device__ __forceinline__ double diff_sq_chunk(const ReduceArgs& r, int64_t chunk) {
    constexpr int P = DT == GACT_DT_F32 ? 4 : 8;
    const int64_t e0 = chunk * (int64_t)(kRedThreads * 4 * P) + (int64_t)threadIdx.x * P;
    u4r a[4], b[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int64_t e = e0 + (int64_t)k * kRedThreads * P;
        a[k] = load_piece16<DT, FULL>(r.a, e, r.n);
        b[k] = load_piece16<DT, FULL>(r.b, e, r.n);
    }
    double acc = 0.0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        float x[8], y[8];
        unpack_piece<DT>(a[k], x);
        unpack_piece<DT>(b[k], y);
#pragma unroll
        for (int j = 0; j < P; ++j) {
            const double d = (double)x[j] - (double)y[j];
            acc += d * d;
        }
    }
    return acc;
}

__global__ __launch_bounds__(kRedThreads) void diff_sq_kernel(const ReduceArgs* __restrict__ table,
                                                              const uint32_t* __restrict__ first_block,
                                                              int K, double* __restrict__ partial) {
    __shared__ double lds[4];
    const uint32_t b = blockIdx.x;
    const int k = find_buffer(first_block, K, b);
    const ReduceArgs r = table[k];
    const int64_t chunk = (int64_t)(b - first_block[k]);
    const bool full = (chunk + 1) * reduce_chunk_elems(r.dtype) <= r.n;
    double acc;
    if (r.dtype == GACT_DT_F32)
        acc = full ? diff_sq_chunk<GACT_DT_F32, true>(r, chunk) : diff_sq_chunk<GACT_DT_F32, false>(r, chunk);
    else
        acc = full ? diff_sq_chunk<GACT_DT_BF16, true>(r, chunk) : diff_sq_chunk<GACT_DT_BF16, false>(r, chunk);
    const double s = block_sum(acc, lds);
    if (threadIdx.x == 0) partial[b] = s;
}

// ---------------------------------------------------------------- footprint
template <int DT, bool FULL>
__device__ __forceinline__ double sum_chunk(const ReduceArgs& r, int64_t chunk) {
    constexpr int P = DT == GACT_DT_F32 ? 4 : 8;
    const int64_t e0 = chunk * (int64_t)(kRedThreads * 4 * P) + (int64_t)threadIdx.x * P;
    u4r a[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
        a[k] = load_piece16<DT, FULL>(r.a, e0 + (int64_t)k * kRedThreads * P, r.n);
    double acc = 0.0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        float x[8];
        unpack_piece<DT>(a[k], x);      // elements past n were loaded as 0
#pragma unroll
        for (int j = 0; j < P; ++j) acc += (double)x[j];
    }
    return acc;
}

// one buffer; block b takes chunk b
__global__ __launch_bounds__(kRedThreads) void sum_kernel(ReduceArgs r, double* __restrict__ partial) {
    __shared__ double lds[4];
    const int64_t chunk = (int64_t)blockIdx.x;
    const bool full = (chunk + 1) * reduce_chunk_elems(r.dtype) <= r.n;
    double acc;
    if (r.dtype == GACT_DT_F32)
        acc = full ? sum_chunk<GACT_DT_F32, true>(r, chunk) : sum_chunk<GACT_DT_F32, false>(r, chunk);
    else
        acc = full ? sum_chunk<GACT_DT_BF16, true>(r, chunk) : sum_chunk<GACT_DT_BF16, false>(r, chunk);
    const double s = block_sum(acc, lds);
    if (threadIdx.x == 0) partial[blockIdx.x] = s;
}

// out[1 + j] = element floor(j * n / n_samples) as binary64
__global__ void sample_kernel(ReduceArgs r, int n_samples, double* __restrict__ out) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= n_samples) return;
    const int64_t i = (int64_t)(((unsigned __int128)(uint64_t)j * (uint64_t)r.n) / (uint64_t)n_samples);
    float v;
    if (r.dtype == GACT_DT_F32) v = ((const float*)r.a)[i];
    else v = __builtin_bit_cast(float, (uint32_t)((const uint16_t*)r.a)[i] << 16);
    out[1 + j] = (double)v;
}

// ------------------------------------------------------- gradient statistics
template <int DT, bool FULL>
__device__ __forceinline__ void stats_chunk(const ReduceArgs& r, int64_t chunk, float rt,
                                            double& sg2, double& sm2) {
    constexpr int P = DT == GACT_DT_F32 ? 4 : 8;
    const int64_t e0 = chunk * (int64_t)(kRedThreads * 4 * P) + (int64_t)threadIdx.x * P;
    float* mean = (float*)r.b;
    u4r g[4];
    f4r m[4][2];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int64_t e = e0 + (int64_t)k * kRedThreads * P;
        g[k] = load_piece16<DT, FULL>(r.a, e, r.n);
#pragma unroll
        for (int h = 0; h < P / 4; ++h) {
            const u4r w = load_piece16<GACT_DT_F32, FULL>(mean, e + 4 * h, r.n);
            m[k][h] = __builtin_bit_cast(f4r, w);
        }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int64_t e = e0 + (int64_t)k * kRedThreads * P;
        float x[8];
        unpack_piece<DT>(g[k], x);
#pragma unroll
        for (int h = 0; h < P / 4; ++h) {
            const float old[4] = {m[k][h].x, m[k][h].y, m[k][h].z, m[k][h].w};
            float nw[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float gi = x[4 * h + j];
                const float d = gi - old[j];
                const float s = d * rt;
                nw[j] = old[j] + s;
                if (FULL || e + 4 * h + j < r.n) {
                    sg2 += (double)gi * (double)gi;
                    sm2 += (double)nw[j] * (double)nw[j];
                }
            }
            const int64_t em = e + 4 * h;
            if (FULL || em + 4 <= r.n) {
                const f4r o = {nw[0], nw[1], nw[2], nw[3]};
                __builtin_nontemporal_store(o, (f4r*)(mean + em));
            } else {
                for (int j = 0; j < 4; ++j) if (em + j < r.n) mean[em + j] = nw[j];
            }
        }
    }
}

__global__ __launch_bounds__(kRedThreads) void grad_stats_kernel(const ReduceArgs* __restrict__ table,
                                                                 const uint32_t* __restrict__ first_block,
                                                                 int K, float rt, uint32_t blocks,
                                                                 double* __restrict__ partial) {
    __shared__ double lds[4];
    const uint32_t b = blockIdx.x;
    const int k = find_buffer(first_block, K, b);
    const ReduceArgs r = table[k];
    const int64_t chunk = (int64_t)(b - first_block[k]);
    double sg2 = 0.0, sm2 = 0.0;
    const bool full = (chunk + 1) * reduce_chunk_elems(r.dtype) <= r.n;
    if (r.dtype == GACT_DT_F32) {
        if (full) stats_chunk<GACT_DT_F32, true>(r, chunk, rt, sg2, sm2);
        else stats_chunk<GACT_DT_F32, false>(r, chunk, rt, sg2, sm2);
    } else {
        if (full) stats_chunk<GACT_DT_BF16, true>(r, chunk, rt, sg2, sm2);
        else stats_chunk<GACT_DT_BF16, false>(r, chunk, rt, sg2, sm2);
    }
    const double s0 = block_sum(sg2, lds);
    const double s1 = block_sum(sm2, lds);
    if (threadIdx.x == 0) { partial[b] = s0; partial[blocks + b] = s1; }
}

// ------------------------------------------------------------ final addition
// out[j] = scale * sum_i partial[j * count + i] in a fixed order, so that the
// result is reproducible.  One block of 1024 threads per output: thread t adds
// the terms t, t + 1024, ... eight at a time (eight independent loads in
// flight), then the block adds the thread sums in a tree.  `stride` is the
// distance between terms (1, or the chunk length after fold_kernel).
constexpr int kFinThreads = 1024;
__global__ __launch_bounds__(kFinThreads) void finish_kernel(const double* __restrict__ partial,
                                                             uint32_t count, uint32_t stride,
                                                             size_t out_pitch, double scale,
                                                             double* __restrict__ out) {
    __shared__ double lds[kFinThreads / 64];
    const double* p = partial + (size_t)blockIdx.x * out_pitch;
    double acc = 0.0;
    uint32_t i = threadIdx.x;
    for (; i + 7u * kFinThreads < count; i += 8u * kFinThreads) {
        double v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = p[(size_t)(i + (uint32_t)k * kFinThreads) * stride];
        acc += ((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7]));
    }
    for (; i < count; i += kFinThreads) acc += p[(size_t)i * stride];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double s = 0.0;
        for (int w = 0; w < kFinThreads / 64; ++w) s += lds[w];
        out[blockIdx.x] = scale * s;
    }
}

// First level for long lists: block (k, j) adds the terms [k * chunk, (k + 1) * chunk)
// of output j and leaves the sum in the first of them (it only touches its own chunk).
__global__ __launch_bounds__(kRedThreads) void fold_kernel(double* __restrict__ partial, uint32_t count,
                                                           uint32_t chunk) {
    __shared__ double lds[4];
    double* p = partial + (size_t)blockIdx.y * count + (size_t)blockIdx.x * chunk;
    const uint32_t left = count - blockIdx.x * chunk;
    const uint32_t m = left < chunk ? left : chunk;
    double acc = 0.0;
    for (uint32_t i = threadIdx.x; i < m; i += kRedThreads) acc += p[i];
    const double s = block_sum(acc, lds);
    if (threadIdx.x == 0) p[0] = s;
}

// Enqueues the final addition of `count` terms for each of `nout` outputs.
static void launch_finish(double* d_partial, unsigned count, int nout, double scale, double* d_out,
                          hipStream_t s) {
    constexpr unsigned kFoldBlocks = 128;
    if (count <= 32768u) {
        hipLaunchKernelGGL(finish_kernel, dim3(nout), dim3(kFinThreads), 0, s, d_partial, count, 1u,
                           (size_t)count, scale, d_out);
        return;
    }
    const unsigned chunk = (count + kFoldBlocks - 1) / kFoldBlocks;
    const unsigned folded = (count + chunk - 1) / chunk;
    hipLaunchKernelGGL(fold_kernel, dim3(folded, nout), dim3(kRedThreads), 0, s, d_partial, count, chunk);
    hipLaunchKernelGGL(finish_kernel, dim3(nout), dim3(kFinThreads), 0, s, d_partial, folded, chunk,
                       (size_t)count, scale, d_out);
}

}  // namespace gact

extern "C" int gact_launch_diff_sq(const gact::ReduceArgs* d_table, const uint32_t* d_first, int K,
                                   unsigned blocks, double* d_partial, double scale, double* d_out,
                                   void* stream) {
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(gact::diff_sq_kernel, dim3(blocks), dim3(gact::kRedThreads), 0, s, d_table, d_first,
                       K, d_partial);
    gact::launch_finish(d_partial, blocks, 1, scale, d_out, s);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

extern "C" int gact_launch_grad_stats(const gact::ReduceArgs* d_table, const uint32_t* d_first, int K,
                                      float rt, unsigned blocks, double* d_partial, double* d_out,
                                      void* stream) {
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(gact::grad_stats_kernel, dim3(blocks), dim3(gact::kRedThreads), 0, s, d_table,
                       d_first, K, rt, blocks, d_partial);
    gact::launch_finish(d_partial, blocks, 2, 1.0, d_out, s);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// out[0 .. nout) = 0 through a kernel (no memset node, so callers may capture it)
extern "C" int gact_launch_zero(double* d_out, int nout, void* stream) {
    hipLaunchKernelGGL(gact::finish_kernel, dim3(nout), dim3(gact::kFinThreads), 0, (hipStream_t)stream,
                       (const double*)d_out, 0u, 1u, (size_t)0, 0.0, d_out);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// The footprint from per-tile sums that a compress launch left in d_partial.
extern "C" int gact_launch_footprint_finish(const gact::ReduceArgs* r, unsigned count, double* d_partial,
                                            int n_samples, double* d_out, void* stream) {
    hipStream_t s = (hipStream_t)stream;
    gact::launch_finish(d_partial, count, 1, 1.0, d_out, s);
    if (n_samples > 0)
        hipLaunchKernelGGL(gact::sample_kernel, dim3((n_samples + 255) / 256), dim3(256), 0, s, *r,
                           n_samples, d_out);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

extern "C" int gact_launch_footprint(const gact::ReduceArgs* r, unsigned blocks, double* d_partial,
                                     int n_samples, double* d_out, void* stream) {
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(gact::sum_kernel, dim3(blocks), dim3(gact::kRedThreads), 0, s, *r, d_partial);
    gact::launch_finish(d_partial, blocks, 1, 1.0, d_out, s);
    if (n_samples > 0)
        hipLaunchKernelGGL(gact::sample_kernel, dim3((n_samples + 255) / 256), dim3(256), 0, s, *r,
                           n_samples, d_out);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

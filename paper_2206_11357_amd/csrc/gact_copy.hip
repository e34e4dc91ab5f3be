// Copy kernel with a bounded footprint on the GPU, for moving compressed
// activations between device memory and pinned host memory (arXiv 2206.11357,
// Sec. 5.3: swap-out on a stream of its own, next to the forward pass).
//
// The runtime's own device-to-host copy is a kernel too; enqueued behind an
// event of the compute stream it stretched every kernel that started beside it
// to its own length (the forward pass of a transformer step went from 6 to
// 26 ms).  PCIe moves 56 GB/s; sixteen workgroups streaming 16-byte pieces
// cover that, and the rest of the chip stays with the model.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gact {

typedef uint32_t u4c __attribute__((ext_vector_type(4)));

// 16-byte store at system scope, written through the L2 instead of left there as a dirty line.
// With ordinary stores a copy to host memory at PCIe rate slowed kernels running beside it by
// 1.7x (a 4096^3 bf16 GEMM) to 3x (the compressor); with these, by 1.2x and 1.1x, at the same rate.
__device__ __forceinline__ void store_through(u4c* p, u4c v) {
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" ::"v"(p), "v"(v) : "memory");
}

// dst[0 .. n16) = src[0 .. n16) in 16-byte pieces, grid-stride, four pieces in
// flight per thread; the last thread also moves the `tail` bytes behind them.
__global__ __launch_bounds__(256) void copy_kernel(u4c* __restrict__ dst, const u4c* __restrict__ src,
                                                   uint64_t n16, uint32_t tail) {
    const uint64_t stride = (uint64_t)gridDim.x * 256u;
    uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const u4c a = __builtin_nontemporal_load(src + i);
        const u4c b = __builtin_nontemporal_load(src + i + stride);
        const u4c c = __builtin_nontemporal_load(src + i + 2 * stride);
        const u4c d = __builtin_nontemporal_load(src + i + 3 * stride);
        store_through(dst + i, a);
        store_through(dst + i + stride, b);
        store_through(dst + i + 2 * stride, c);
        store_through(dst + i + 3 * stride, d);
    }
    for (; i < n16; i += stride) store_through(dst + i, __builtin_nontemporal_load(src + i));
    if (tail != 0u && blockIdx.x == gridDim.x - 1 && threadIdx.x == 255) {
        const uint8_t* s = (const uint8_t*)(src + n16);
        uint8_t* d = (uint8_t*)(dst + n16);
        for (uint32_t k = 0; k < tail; ++k) d[k] = s[k];
    }
}

}  // namespace gact

extern "C" int gact_launch_copy(void* dst, const void* src, uint64_t nbytes, unsigned workgroups, void* stream) {
    hipLaunchKernelGGL(gact::copy_kernel, dim3(workgroups), dim3(256), 0, (hipStream_t)stream, (gact::u4c*)dst,
                       (const gact::u4c*)src, nbytes / 16, (uint32_t)(nbytes % 16));
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

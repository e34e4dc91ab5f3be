// Issue rate of the VALU instructions the compress kernel is made of, on the
// GPU it runs on: eight independent register chains per wavefront, eight
// wavefronts per SIMD, no memory traffic but one store at the end.  Standalone
// tool (not part of libgact.so); prints cycles per wavefront instruction and
// SIMD at the nominal 2.4 GHz.  The compress kernel's ALU bound is priced with
// these figures.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#define CHECK(x)                                                                         \
    do {                                                                                 \
        hipError_t e_ = (x);                                                             \
        if (e_ != hipSuccess) {                                                          \
            fprintf(stderr, "valu_rate_probe: %s (line %d)\n", hipGetErrorString(e_), __LINE__); \
            return 1;                                                                    \
        }                                                                                \
    } while (0)

// a0..a7 <- OP(a, b, c), 64 instructions per loop iteration
#define RATE_KERNEL(NAME, ASM)                                                                   \
    __global__ __launch_bounds__(256) void NAME(uint32_t* out, int iters, uint32_t seed) {       \
        uint32_t a0 = threadIdx.x + seed, a1 = a0 * 3u + 1u, a2 = a0 * 5u + 2u, a3 = a0 * 7u + 3u, \
                 a4 = a0 * 9u + 4u, a5 = a0 * 11u + 5u, a6 = a0 * 13u + 6u, a7 = a0 * 17u + 7u;  \
        const uint32_t b = seed | 1u, c = seed * 77u + 5u;                                       \
        for (int i = 0; i < iters; ++i) {                                                        \
            _Pragma("unroll") for (int u = 0; u < 8; ++u) {                                      \
                asm volatile(ASM : "+v"(a0) : "v"(b), "v"(c));                                   \
                asm volatile(ASM : "+v"(a1) : "v"(b), "v"(c));                                   \
                asm volatile(ASM : "+v"(a2) : "v"(b), "v"(c));                                   \
                asm volatile(ASM : "+v"(a3) : "v"(b), "v"(c));                                   \
                asm volatile(ASM : "+v"(a4) : "v"(b), "v"(c));                                   \
                asm volatile(ASM : "+v"(a5) : "v"(b), "v"(c));                                   \
                asm volatile(ASM : "+v"(a6) : "v"(b), "v"(c));                                   \
                asm volatile(ASM : "+v"(a7) : "v"(b), "v"(c));                                   \
            }                                                                                    \
        }                                                                                        \
        out[blockIdx.x * 256 + threadIdx.x] = a0 ^ a1 ^ a2 ^ a3 ^ a4 ^ a5 ^ a6 ^ a7;             \
    }

RATE_KERNEL(k_add_u32, "v_add_u32 %0, %0, %1")
RATE_KERNEL(k_sub_f32, "v_sub_f32 %0, %0, %1")
RATE_KERNEL(k_mul_f32, "v_mul_f32 %0, %0, %1")
RATE_KERNEL(k_fma_f32, "v_fma_f32 %0, %0, %1, %2")
RATE_KERNEL(k_ashr, "v_ashrrev_i32 %0, 17, %0")
RATE_KERNEL(k_bitop3, "v_bitop3_b32 %0, %0, %1, %2 bitop3:0x96")
RATE_KERNEL(k_cvt_flr, "v_cvt_flr_i32_f32 %0, %0")
RATE_KERNEL(k_mad_u32_u16, "v_mad_u32_u16 %0, %0, %1, %2")
RATE_KERNEL(k_lshl_add, "v_lshl_add_u32 %0, %0, 3, %1")
RATE_KERNEL(k_min3, "v_min3_f32 %0, %0, %1, %2")
RATE_KERNEL(k_mul_lo, "v_mul_lo_u32 %0, %0, %1")
RATE_KERNEL(k_mul_hi, "v_mul_hi_u32 %0, %0, %1")
RATE_KERNEL(k_alignbit, "v_alignbit_b32 %0, %0, %1, 7")
RATE_KERNEL(k_add3, "v_add3_u32 %0, %0, %1, %2")
RATE_KERNEL(k_rcp, "v_rcp_f32 %0, %0")

// the 64-bit multiply-add of the Philox rounds needs a register pair
__global__ __launch_bounds__(256) void k_mad_u64_u32(uint32_t* out, int iters, uint32_t seed) {
    uint64_t a[8];
    for (int j = 0; j < 8; ++j) a[j] = (uint64_t)(threadIdx.x + seed) * (j + 3);
    const uint32_t b = seed | 1u;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
#pragma unroll
            for (int j = 0; j < 8; ++j)
                asm volatile("v_mad_u64_u32 %0, vcc, %1, %2, %0"
                             : "+v"(a[j]) : "v"(b), "v"((uint32_t)(j + u + seed)) : "vcc");
        }
    }
    uint64_t r = 0;
    for (int j = 0; j < 8; ++j) r ^= a[j];
    out[blockIdx.x * 256 + threadIdx.x] = (uint32_t)r ^ (uint32_t)(r >> 32);
}

typedef void (*kernel_t)(uint32_t*, int, uint32_t);

int main() {
    const int blocks = 256 * 8 * 4;      // 8 blocks of 4 wavefronts per CU resident, 4 rounds of them
    const int iters = 256;               // x 64 instructions
    uint32_t* out;
    CHECK(hipMalloc(&out, (size_t)blocks * 256 * sizeof(uint32_t)));
    const struct { const char* name; kernel_t k; } ks[] = {
        {"v_add_u32", k_add_u32}, {"v_sub_f32", k_sub_f32}, {"v_mul_f32", k_mul_f32}, {"v_fma_f32", k_fma_f32},
        {"v_ashrrev_i32", k_ashr}, {"v_bitop3_b32", k_bitop3}, {"v_cvt_flr_i32_f32", k_cvt_flr},
        {"v_mad_u32_u16", k_mad_u32_u16}, {"v_lshl_add_u32", k_lshl_add}, {"v_min3_f32", k_min3},
        {"v_mul_lo_u32", k_mul_lo}, {"v_mul_hi_u32", k_mul_hi}, {"v_alignbit_b32", k_alignbit},
        {"v_add3_u32", k_add3}, {"v_rcp_f32", k_rcp}, {"v_mad_u64_u32", k_mad_u64_u32}};
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    printf("%-20s %10s %16s %s\n", "instruction", "ms", "lane-ops/s", "cycles per wavefront instruction and SIMD at 2.4 GHz");
    for (const auto& s : ks) {
        s.k<<<blocks, 256>>>(out, 8, 1u);
        CHECK(hipDeviceSynchronize());
        CHECK(hipEventRecord(e0));
        s.k<<<blocks, 256>>>(out, iters, 1u);
        CHECK(hipEventRecord(e1));
        CHECK(hipEventSynchronize(e1));
        CHECK(hipGetLastError());
        float ms;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        const double lane_ops = (double)blocks * 256 * iters * 64;
        const double rate = lane_ops / (ms * 1e-3);
        printf("%-20s %10.3f %16.3e %.2f\n", s.name, ms, rate, 256.0 * 4 * 64 * 2.4e9 / rate);
        fflush(stdout);
    }
    CHECK(hipFree(out));
    return 0;
}

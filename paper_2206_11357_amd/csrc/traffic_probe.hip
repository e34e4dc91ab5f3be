// HBM ceilings for the traffic mixes of the codec, measured with kernels that do
// no arithmetic and have the access shapes of the compress / decompress kernels:
// read side, a wavefront streams one 8 KB chunk with coalesced 16-byte
// non-temporal loads and writes 512 B; write side, the four wavefronts of a
// block write 16 consecutive 1 KB units (wavefront w the units w, w+4, w+8,
// w+12) with coalesced 16-byte non-temporal stores and read 64 B per unit.
// Standalone tool
// (not part of libgact.so); prints one JSON object.  bench.py runs it to put
// the memory system's own limit for a 16:1 read:write mix next to what the
// compressor achieves.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#define CHECK(x)                                                                      \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) {                                                       \
            fprintf(stderr, "traffic_probe: %s (line %d)\n", hipGetErrorString(e_), __LINE__); \
            return 1;                                                                 \
        }                                                                             \
    } while (0)

typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef uint32_t u2 __attribute__((ext_vector_type(2)));

constexpr int kChunkU4 = 512;          // 8 KB per wavefront and chunk
constexpr int kSmallU2 = 64;           // 512 B per wavefront and chunk

// big: nchunks * 8 KB, small: nchunks * 512 B.
// MODE 0 read big | 1 read big, write small | 4 read big, write big2
template <int MODE>
__global__ __launch_bounds__(256) void probe(u4* __restrict__ big, u2* __restrict__ small_,
                                             u4* __restrict__ big2, uint32_t nchunks) {
    const uint32_t chunk = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (chunk >= nchunks) return;
    u4* p = big + (size_t)chunk * kChunkU4 + lane;
    u2* s = small_ + (size_t)chunk * kSmallU2 + lane;
    {
        u4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = __builtin_nontemporal_load(p + j * 64);
        if (MODE == 4) {
            u4* q = big2 + (size_t)chunk * kChunkU4 + lane;
#pragma unroll
            for (int j = 0; j < 8; ++j) __builtin_nontemporal_store(v[j], q + j * 64);
            return;
        }
        uint32_t a = 0, b = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) { a ^= v[j].x + v[j].y; b += v[j].z ^ v[j].w; }
        const u2 r = {a, b};
        if (MODE == 1) __builtin_nontemporal_store(r, s);
        else if (a == 0x12345u && b == 0x54321u) *s = r;      // keeps the loads alive, never taken on zeros
    }
}

// MODE 2 write big | 3 read small (one byte per lane and unit), write big
template <int MODE>
__global__ __launch_bounds__(256) void probe_write(u4* __restrict__ big, const uint8_t* __restrict__ small_,
                                                   uint32_t nunits) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    uint32_t code[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t unit = blockIdx.x * 16 + k * 4 + wave;
        code[k] = lane;
        if (MODE == 3 && unit < nunits) code[k] = __builtin_nontemporal_load(small_ + (size_t)unit * 64 + lane);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t unit = blockIdx.x * 16 + k * 4 + wave;
        if (unit >= nunits) continue;
        const u4 v = {code[k], code[k] + 1u, code[k] ^ unit, (uint32_t)lane};
        __builtin_nontemporal_store(v, big + (size_t)unit * 64 + lane);
    }
}

template <int MODE>
static int run(const char* name, double bytes, u4* big, u2* small_, u4* big2, uint32_t nchunks, bool last) {
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    const unsigned blocks = (nchunks + 3) / 4;
    const uint32_t nunits = nchunks * 8;                     // 1 KB units of the big stream
    const unsigned wblocks = (nunits + 15) / 16;
    auto launch = [&]() {
        if constexpr (MODE == 2 || MODE == 3)
            probe_write<MODE><<<wblocks, 256>>>(big, (const uint8_t*)small_, nunits);
        else
            probe<MODE><<<blocks, 256>>>(big, small_, big2, nchunks);
    };
    for (int i = 0; i < 3; ++i) launch();
    CHECK(hipDeviceSynchronize());
    float sum = 0.f;
    const int reps = 15;
    for (int i = 0; i < reps; ++i) {
        CHECK(hipEventRecord(e0));
        launch();
        CHECK(hipEventRecord(e1));
        CHECK(hipEventSynchronize(e1));
        float ms;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        sum += ms;
    }
    CHECK(hipGetLastError());
    printf("\"%s_GBps\": %.1f%s", name, bytes / (sum / reps) / 1e6, last ? "" : ", ");
    CHECK(hipEventDestroy(e0));
    CHECK(hipEventDestroy(e1));
    return 0;
}

int main() {
    const uint32_t nchunks = 1u << 18;                       // 2 GiB big streams
    u4 *big, *big2;
    u2* small_;
    CHECK(hipMalloc(&big, (size_t)nchunks * kChunkU4 * sizeof(u4)));
    CHECK(hipMalloc(&big2, (size_t)nchunks * kChunkU4 * sizeof(u4)));
    CHECK(hipMalloc(&small_, (size_t)nchunks * kSmallU2 * sizeof(u2)));
    CHECK(hipMemset(big, 0, (size_t)nchunks * kChunkU4 * sizeof(u4)));
    CHECK(hipMemset(small_, 0, (size_t)nchunks * kSmallU2 * sizeof(u2)));
    CHECK(hipDeviceSynchronize());
    const double B = (double)nchunks * 8192, S = (double)nchunks * 512;
    printf("{\"read_side\": \"8 KB + 512 B per wavefront\", \"write_side\": \"4 x (1 KB + 64 B) per wavefront\", "
           "\"big_stream_GiB\": 2, ");
    if (run<0>("read_only", B, big, small_, big2, nchunks, false)) return 1;
    if (run<1>("read16_write1", B + S, big, small_, big2, nchunks, false)) return 1;
    if (run<2>("write_only", B, big, small_, big2, nchunks, false)) return 1;
    if (run<3>("read1_write16", B + S, big, small_, big2, nchunks, false)) return 1;
    if (run<4>("copy", 2 * B, big, small_, big2, nchunks, true)) return 1;
    printf("}\n");
    CHECK(hipFree(big));
    CHECK(hipFree(big2));
    CHECK(hipFree(small_));
    return 0;
}

// Device-facing side of the C ABI declared in include/gact.h: argument checks,
// launch geometry, the multi-tensor launch table.  The entry points that never
// touch the GPU (sizes, bit allocator, variance alert) are in gact_host.cpp.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <mutex>
#include <queue>
#include <algorithm>
#include <vector>

#include "gact.h"
#include "gact_device.h"

// Scratch area of gact_compress_footprint_noalloc: device memory that is part
// of the library's code object, one copy per GPU, held until the process ends.
// In host code this name is only a handle for hipGetSymbolAddress; kernels get
// the address that call returns.
static __device__ __align__(256) unsigned char scratch[GACT_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int kPerLane = 32;
constexpr int kWavesPerBlock = 4;

bool bits_ok(int bits) { return bits == 1 || bits == 2 || bits == 4 || bits == 8; }
bool group_ok(int g) { return g >= 32 && g <= 1024 && g % 32 == 0; }
bool dtype_ok(int dt) { return dt == GACT_F32 || dt == GACT_BF16; }
bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

gact::Geometry make_geometry(int group_size) {
    gact::Geometry geo;
    geo.lpg = group_size / kPerLane;
    geo.lanes_used = (64 / geo.lpg) * geo.lpg;
    geo.pow2 = (geo.lpg & (geo.lpg - 1)) == 0 ? 1 : 0;
    geo.lpg_shift = 0;
    while ((1 << (geo.lpg_shift + 1)) <= geo.lpg) ++geo.lpg_shift;
    geo.groups_per_tile = geo.lanes_used / geo.lpg;
    geo.group_size = group_size;
    geo.group_shift = geo.lpg_shift + 5;
    geo.lds_wave_dwords = 0;      // set per launch from the dtypes in it
    return geo;
}

int64_t tiles_for(int64_t n, const gact::Geometry& geo) {
    const int64_t te = (int64_t)geo.lanes_used * kPerLane;
    return (n + te - 1) / te;
}

// Fills `out`; returns GACT_OK or the error for this tensor.
int make_args(bool compress, const void* x, void* packed, float* gmin, float* gscale, void* y,
              int64_t n, uint64_t seed, int64_t index_base, int bits, int dtype,
              const gact::Geometry& geo, gact::TensorArgs* out) {
    if (!bits_ok(bits)) return GACT_E_BITS;
    if (n < 0 || !dtype_ok(dtype)) return GACT_E_ARG;
    // noise is drawn per block of 8 elements: a shard starts on a block boundary
    if (index_base < 0 || (index_base & 7) != 0 || (index_base >> 3) >= (1ll << 48)) return GACT_E_ARG;
    if (n > 0) {
        const void* io = compress ? x : y;
        if (!io || !packed || !gmin || !gscale) return GACT_E_ARG;
        if (!aligned(io, 16) || !aligned(packed, 16) || !aligned(gmin, 4) || !aligned(gscale, 4))
            return GACT_E_ARG;
    }
    const int64_t tiles = tiles_for(n, geo);
    if (tiles > 0xFFFFFFFFll) return GACT_E_ARG;
    out->io = compress ? const_cast<void*>(x) : y;
    out->packed = packed;
    out->gmin = gmin;
    out->gscale = gscale;
    out->n = n;
    out->seed_lo = (uint32_t)seed;
    out->seed_hi = (uint32_t)(seed >> 32);
    const uint64_t blk_base = (uint64_t)index_base >> 3;
    out->blk_base_lo = (uint32_t)blk_base;
    out->meta = (uint32_t)bits | ((uint32_t)dtype << 8) | ((uint32_t)(blk_base >> 32) << 16);
    return GACT_OK;
}

// blocks a tensor needs: compress takes 4 wavefront tiles per block, decompress
// a fixed span of elements per block
int64_t blocks_for(bool compress, const gact::TensorArgs& t, const gact::Geometry& geo) {
    if (compress) return (tiles_for(t.n, geo) + kWavesPerBlock - 1) / kWavesPerBlock;
    const int64_t span = gact::dec_block_elems(t.dtype(), t.bits());
    return (t.n + span - 1) / span;
}

int run_single(bool compress, const gact::TensorArgs& t, const gact::Geometry& geo, void* stream) {
    if (t.n == 0) return GACT_OK;
    const int64_t blocks = blocks_for(compress, t, geo);
    if (blocks > 0x7FFFFFFFll) return GACT_E_ARG;
    return gact_launch_single(compress ? 1 : 0, &t, &geo, (unsigned)blocks, stream) == 0
               ? GACT_OK : GACT_E_HIP;
}

// A table upload reads host memory that is gone when a captured graph replays.
// GACT_OK when `stream` is not capturing.
int refuse_if_capturing(void* stream) {
    hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing((hipStream_t)stream, &status) != hipSuccess) return GACT_E_HIP;
    return status == hipStreamCaptureStatusNone ? GACT_OK : GACT_E_CAPTURE;
}

size_t table_bytes(int L) { return ((size_t)L * sizeof(gact::TensorArgs) + 15) / 16 * 16; }
size_t first_bytes(int L) { return ((size_t)(L + 1) * sizeof(uint32_t) + 15) / 16 * 16; }

// The coarse block -> tensor index over `first` (live + 1 entries, the last is
// the block total): at most `buckets` buckets of 2^shift blocks; hint[k] is the
// tensor that holds block k << shift, and one more entry closes the last bucket.
template <typename T>
unsigned make_hints(const std::vector<uint32_t>& first, int buckets, std::vector<T>* hint) {
    const uint32_t blocks = first.back();
    const int live = (int)first.size() - 1;
    unsigned shift = 0;
    while ((((uint64_t)blocks - 1) >> shift) + 1 > (uint64_t)buckets) ++shift;
    const uint32_t used = (uint32_t)((((uint64_t)blocks - 1) >> shift) + 1);
    hint->resize((size_t)used + 1);
    int l = 0;
    for (uint32_t k = 0; k < used; ++k) {
        const uint64_t pos = (uint64_t)k << shift;
        while ((uint64_t)first[(size_t)l + 1] <= pos) ++l;
        (*hint)[k] = (T)l;
    }
    (*hint)[used] = (T)(live - 1);
    return shift;
}

int run_multi(bool compress, const gact_tensor_desc* descs, int L, int group_size,
              void* d_workspace, size_t workspace_bytes, void* stream) {
    if (L < 0) return GACT_E_ARG;
    if (!group_ok(group_size)) return GACT_E_GROUP;
    if (L == 0) return GACT_OK;
    if (!descs) return GACT_E_ARG;
    gact::Geometry geo = make_geometry(group_size);

    // one contiguous staging image: table of the non-empty tensors, then the
    // first block of each, then the total
    std::vector<gact::TensorArgs> table;
    std::vector<uint32_t> first;
    table.reserve(L);
    first.reserve(L + 1);
    uint64_t blocks = 0;
    for (int l = 0; l < L; ++l) {
        const gact_tensor_desc& d = descs[l];
        if (d.bits == GACT_BITS_UNCOMPRESSED) {          // left uncompressed by the allocator
            if (d.n < 0) return GACT_E_ARG;
            continue;
        }
        gact::TensorArgs t;
        const int rc = make_args(compress, d.x, d.packed, d.gmin, d.gscale, d.y, d.n, d.seed,
                                 compress ? d.index_base : 0, d.bits, d.dtype, geo, &t);
        if (rc != GACT_OK) return rc;
        if (d.n == 0) continue;
        first.push_back((uint32_t)blocks);
        table.push_back(t);
        geo.lds_wave_dwords = std::max(geo.lds_wave_dwords, gact::lds_dwords_per_wave(d.dtype));
        blocks += (uint64_t)blocks_for(compress, t, geo);
        if (blocks > 0x7FFFFFFFull) return GACT_E_ARG;
    }
    const int live = (int)table.size();
    if (live == 0) return GACT_OK;
    first.push_back((uint32_t)blocks);

    if (!d_workspace || !aligned(d_workspace, 16) ||
        workspace_bytes < gact_multi_workspace_bytes(L))
        return GACT_E_ARG;

    if (live <= gact::kInlineTensors) {
        // small table: by value in the kernel arguments, nothing to upload
        gact::InlineTable tab;
        std::memset(&tab, 0, sizeof(tab));
        std::memcpy(tab.t, table.data(), (size_t)live * sizeof(gact::TensorArgs));
        std::memcpy(tab.first_block, first.data(), first.size() * sizeof(uint32_t));
        tab.L = live;
        std::vector<uint8_t> hint;
        tab.hint_shift = make_hints(first, gact::kInlineHints, &hint);
        for (size_t k = 0; k < hint.size(); ++k) tab.hint[k >> 2] |= (uint32_t)hint[k] << ((k & 3) * 8);
        return gact_launch_multi_inline(compress ? 1 : 0, &tab, &geo, (unsigned)blocks, stream) == 0
                   ? GACT_OK : GACT_E_HIP;
    }

    if (const int rc = refuse_if_capturing(stream)) return rc;
    std::vector<uint32_t> hint;
    const unsigned shift = make_hints(first, gact::hint_buckets(live), &hint);
    const size_t tb = table_bytes(live), fb = first_bytes(live);
    std::vector<unsigned char> image(tb + fb + hint.size() * sizeof(uint32_t));
    std::memcpy(image.data(), table.data(), (size_t)live * sizeof(gact::TensorArgs));
    std::memcpy(image.data() + tb, first.data(), first.size() * sizeof(uint32_t));
    std::memcpy(image.data() + tb + fb, hint.data(), hint.size() * sizeof(uint32_t));
    // pageable source: the runtime has taken its own copy when this returns
    if (hipMemcpyAsync(d_workspace, image.data(), image.size(), hipMemcpyHostToDevice,
                       (hipStream_t)stream) != hipSuccess)
        return GACT_E_HIP;
    const unsigned char* base = (const unsigned char*)d_workspace;
    return gact_launch_multi(compress ? 1 : 0, (const gact::TensorArgs*)base, (const uint32_t*)(base + tb),
                             (const uint32_t*)(base + tb + fb), shift, &geo, (unsigned)blocks,
                             stream) == 0 ? GACT_OK : GACT_E_HIP;
}

// ---------------------------------------------------------------- reductions
size_t reduce_table_bytes(int K) {
    return ((size_t)K * sizeof(gact::ReduceArgs) + (size_t)(K + 1) * sizeof(uint32_t) + 15) / 16 * 16;
}

// Builds and uploads the buffer table of a reduction launch.  On success
// *blocks_out is the grid size, *d_partial the per-block result area behind
// the table; returns 1 when there is nothing to reduce.
int stage_reduction(const std::vector<gact::ReduceArgs>& bufs, void* d_workspace,
                    size_t workspace_bytes, int nout, void* stream, unsigned* blocks_out,
                    const gact::ReduceArgs** d_table, const uint32_t** d_first, double** d_partial) {
    std::vector<gact::ReduceArgs> live;
    std::vector<uint32_t> first;
    uint64_t blocks = 0;
    for (const gact::ReduceArgs& r : bufs) {
        if (r.n == 0) continue;
        const int64_t chunk = gact::reduce_chunk_elems(r.dtype);
        first.push_back((uint32_t)blocks);
        live.push_back(r);
        blocks += (uint64_t)((r.n + chunk - 1) / chunk);
        if (blocks > 0x7FFFFFFFull) return GACT_E_ARG;
    }
    first.push_back((uint32_t)blocks);
    const int K = (int)live.size();
    if (K == 0) return 1;
    const size_t tb = reduce_table_bytes(K);
    const size_t need = tb + (size_t)nout * blocks * sizeof(double);
    if (!d_workspace || !aligned(d_workspace, 16) || workspace_bytes < need) return GACT_E_ARG;
    if (const int rc = refuse_if_capturing(stream)) return rc;
    std::vector<unsigned char> image(tb);
    std::memcpy(image.data(), live.data(), (size_t)K * sizeof(gact::ReduceArgs));
    std::memcpy(image.data() + (size_t)K * sizeof(gact::ReduceArgs), first.data(),
                first.size() * sizeof(uint32_t));
    // pageable source: the runtime has taken its own copy when this returns
    if (hipMemcpyAsync(d_workspace, image.data(), image.size(), hipMemcpyHostToDevice,
                       (hipStream_t)stream) != hipSuccess)
        return GACT_E_HIP;
    *blocks_out = (unsigned)blocks;
    *d_table = (const gact::ReduceArgs*)d_workspace;
    *d_first = (const uint32_t*)((const unsigned char*)d_workspace + (size_t)K * sizeof(gact::ReduceArgs));
    *d_partial = (double*)((unsigned char*)d_workspace + tb);
    return GACT_OK;
}

// Address of `scratch` on the current device, looked up once per device.
int scratch_of_current_device(void** out) {
    constexpr int kMaxDevices = 64;
    static std::mutex lock;
    static void* address[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return GACT_E_HIP;
    std::lock_guard<std::mutex> hold(lock);
    if (!address[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return GACT_E_HIP;
        address[dev] = p;
    }
    *out = address[dev];
    return GACT_OK;
}

// gact_compress_footprint on a caller workspace, or (limited = true) on the
// library's own scratch area, where a tensor that needs more is refused.
int compress_footprint(const void* d_x, gact_dtype dtype, int64_t n, int group_size, int bits,
                       uint64_t seed, void* d_packed, float* d_gmin, float* d_gscale, int n_samples,
                       double* d_footprint, void* d_workspace, size_t workspace_bytes, bool limited,
                       void* stream) {
    if (!bits_ok(bits)) return GACT_E_BITS;
    if (!group_ok(group_size)) return GACT_E_GROUP;
    if (n_samples < 0 || n_samples > 32768 || !d_footprint || !aligned(d_footprint, 8)) return GACT_E_ARG;
    gact::Geometry geo = make_geometry(group_size);
    geo.lds_wave_dwords = gact::lds_dwords_per_wave((int)dtype);
    gact::TensorArgs t;
    const int rc = make_args(true, d_x, d_packed, d_gmin, d_gscale, nullptr, n, seed, 0, bits,
                             (int)dtype, geo, &t);
    if (rc != GACT_OK) return rc;
    if (n == 0)
        return gact_launch_zero(d_footprint, 1 + n_samples, stream) == 0 ? GACT_OK : GACT_E_HIP;
    const size_t need = (size_t)tiles_for(n, geo) * sizeof(double);       // one partial sum per tile
    if (!d_workspace || !aligned(d_workspace, 16) || workspace_bytes < need)
        return limited ? GACT_E_SCRATCH : GACT_E_ARG;
    const int64_t blocks = blocks_for(true, t, geo);
    if (blocks > 0x7FFFFFFFll) return GACT_E_ARG;
    if (gact_launch_compress_sum(&t, &geo, (unsigned)blocks, (double*)d_workspace, stream) != 0)
        return GACT_E_HIP;
    const gact::ReduceArgs r{d_x, nullptr, n, (int32_t)dtype, 0};
    return gact_launch_footprint_finish(&r, (unsigned)tiles_for(n, geo), (double*)d_workspace, n_samples,
                                        d_footprint, stream) == 0 ? GACT_OK : GACT_E_HIP;
}

}  // namespace

extern "C" {

int gact_compress(const void* d_x, gact_dtype dtype, int64_t n, int group_size, int bits,
                  uint64_t seed, void* d_packed, float* d_gmin, float* d_gscale, void* stream) {
    if (!bits_ok(bits)) return GACT_E_BITS;
    if (!group_ok(group_size)) return GACT_E_GROUP;
    gact::Geometry geo = make_geometry(group_size);
    geo.lds_wave_dwords = gact::lds_dwords_per_wave((int)dtype);
    gact::TensorArgs t;
    const int rc = make_args(true, d_x, d_packed, d_gmin, d_gscale, nullptr, n, seed, 0, bits,
                             (int)dtype, geo, &t);
    if (rc != GACT_OK) return rc;
    return run_single(true, t, geo, stream);
}

int gact_decompress(const void* d_packed, const float* d_gmin, const float* d_gscale, int64_t n,
                    int group_size, int bits, void* d_y, gact_dtype dtype, void* stream) {
    if (!bits_ok(bits)) return GACT_E_BITS;
    if (!group_ok(group_size)) return GACT_E_GROUP;
    const gact::Geometry geo = make_geometry(group_size);
    gact::TensorArgs t;
    const int rc = make_args(false, nullptr, const_cast<void*>(d_packed),
                             const_cast<float*>(d_gmin), const_cast<float*>(d_gscale), d_y, n, 0, 0,
                             bits, (int)dtype, geo, &t);
    if (rc != GACT_OK) return rc;
    return run_single(false, t, geo, stream);
}

size_t gact_multi_workspace_bytes(int L) {
    if (L <= 0) return 0;
    return table_bytes(L) + first_bytes(L) + ((size_t)gact::hint_buckets(L) + 1) * sizeof(uint32_t);
}

int gact_compress_multi(const gact_tensor_desc* h_descs, int L, int group_size, void* d_workspace,
                        size_t workspace_bytes, void* stream) {
    return run_multi(true, h_descs, L, group_size, d_workspace, workspace_bytes, stream);
}

int gact_decompress_multi(const gact_tensor_desc* h_descs, int L, int group_size,
                          void* d_workspace, size_t workspace_bytes, void* stream) {
    return run_multi(false, h_descs, L, group_size, d_workspace, workspace_bytes, stream);
}

// -------------------------------------------------- sensitivity, statistics
size_t gact_reduce_workspace_bytes(int K, int64_t total_elems) {
    if (K < 0 || total_elems < 0) return 0;
    // every buffer rounds up to whole 4096-element chunks; two results per block
    const uint64_t blocks = (uint64_t)total_elems / 4096 + (uint64_t)K + 1;
    return reduce_table_bytes(K) + (size_t)(2 * blocks * sizeof(double)) + 16;
}

int gact_sensitivity(const gact_grad_pair* h_pairs, int K, int bits, double* d_out,
                     void* d_workspace, size_t workspace_bytes, void* stream) {
    if (!bits_ok(bits)) return GACT_E_BITS;
    if (K < 0 || !d_out || !aligned(d_out, 8) || (K > 0 && !h_pairs)) return GACT_E_ARG;
    std::vector<gact::ReduceArgs> bufs;
    for (int k = 0; k < K; ++k) {
        const gact_grad_pair& p = h_pairs[k];
        if (p.n < 0 || !dtype_ok(p.dtype)) return GACT_E_ARG;
        if (p.n > 0 && (!p.g0 || !p.g1 || !aligned(p.g0, 16) || !aligned(p.g1, 16))) return GACT_E_ARG;
        bufs.push_back(gact::ReduceArgs{p.g0, const_cast<void*>(p.g1), p.n, p.dtype, 0});
    }
    unsigned blocks = 0;
    const gact::ReduceArgs* d_table = nullptr;
    const uint32_t* d_first = nullptr;
    double* d_partial = nullptr;
    const int rc = stage_reduction(bufs, d_workspace, workspace_bytes, 1, stream, &blocks, &d_table,
                                   &d_first, &d_partial);
    if (rc < 0) return rc;
    if (rc == 1)     // nothing to reduce: the result is zero
        return gact_launch_zero(d_out, 1, stream) == 0 ? GACT_OK : GACT_E_HIP;
    const double B = (double)((1 << bits) - 1);
    const int live = (int)(((const unsigned char*)d_first - (const unsigned char*)d_table) /
                           sizeof(gact::ReduceArgs));
    return gact_launch_diff_sq(d_table, d_first, live, blocks, d_partial, 0.5 * B * B, d_out,
                               stream) == 0 ? GACT_OK : GACT_E_HIP;
}

int gact_grad_stats_update(const gact_grad_stat* h_stats, int K, int64_t t, double* d_out,
                           void* d_workspace, size_t workspace_bytes, void* stream) {
    if (K < 0 || t < 1 || !d_out || !aligned(d_out, 8) || (K > 0 && !h_stats)) return GACT_E_ARG;
    std::vector<gact::ReduceArgs> bufs;
    for (int k = 0; k < K; ++k) {
        const gact_grad_stat& p = h_stats[k];
        if (p.n < 0 || !dtype_ok(p.dtype)) return GACT_E_ARG;
        if (p.n > 0 && (!p.g || !p.mean || !aligned(p.g, 16) || !aligned(p.mean, 16))) return GACT_E_ARG;
        bufs.push_back(gact::ReduceArgs{p.g, p.mean, p.n, p.dtype, 0});
    }
    unsigned blocks = 0;
    const gact::ReduceArgs* d_table = nullptr;
    const uint32_t* d_first = nullptr;
    double* d_partial = nullptr;
    const int rc = stage_reduction(bufs, d_workspace, workspace_bytes, 2, stream, &blocks, &d_table,
                                   &d_first, &d_partial);
    if (rc < 0) return rc;
    if (rc == 1) return gact_launch_zero(d_out, 2, stream) == 0 ? GACT_OK : GACT_E_HIP;
    const int live = (int)(((const unsigned char*)d_first - (const unsigned char*)d_table) /
                           sizeof(gact::ReduceArgs));
    const float rt = (float)(1.0 / (double)t);
    return gact_launch_grad_stats(d_table, d_first, live, rt, blocks, d_partial, d_out, stream) == 0
               ? GACT_OK : GACT_E_HIP;
}

int gact_footprint(const void* d_x, gact_dtype dtype, int64_t n, int n_samples, double* d_out,
                   void* d_workspace, size_t workspace_bytes, void* stream) {
    if (n < 0 || n_samples < 0 || n_samples > 32768 || !dtype_ok((int)dtype) || !d_out ||
        !aligned(d_out, 8))
        return GACT_E_ARG;
    if (n == 0) return gact_launch_zero(d_out, 1 + n_samples, stream) == 0 ? GACT_OK : GACT_E_HIP;
    if (!d_x || !aligned(d_x, 16)) return GACT_E_ARG;
    const int64_t chunk = gact::reduce_chunk_elems((int)dtype);
    const int64_t blocks = (n + chunk - 1) / chunk;
    if (blocks > 0x7FFFFFFFll) return GACT_E_ARG;
    if (!d_workspace || !aligned(d_workspace, 16) ||
        workspace_bytes < (size_t)blocks * sizeof(double))
        return GACT_E_ARG;
    const gact::ReduceArgs r{d_x, nullptr, n, (int32_t)dtype, 0};
    return gact_launch_footprint(&r, (unsigned)blocks, (double*)d_workspace, n_samples, d_out,
                                 stream) == 0 ? GACT_OK : GACT_E_HIP;
}

size_t gact_compress_footprint_workspace_bytes(int64_t n, int group_size) {
    if (n <= 0 || !group_ok(group_size)) return 0;
    return (size_t)tiles_for(n, make_geometry(group_size)) * sizeof(double);
}

int gact_compress_footprint(const void* d_x, gact_dtype dtype, int64_t n, int group_size, int bits,
                            uint64_t seed, void* d_packed, float* d_gmin, float* d_gscale,
                            int n_samples, double* d_footprint, void* d_workspace,
                            size_t workspace_bytes, void* stream) {
    return compress_footprint(d_x, dtype, n, group_size, bits, seed, d_packed, d_gmin, d_gscale,
                              n_samples, d_footprint, d_workspace, workspace_bytes, false, stream);
}

// The address a kernel can use for `p`: device memory as it is; host memory only when it is pinned
// and mapped into the device's address space.  nullptr when a kernel must not touch it.
static void* device_visible(const void* p) {
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, p) != hipSuccess) {
        (void)hipGetLastError();                      // an ordinary host pointer: not an error state to keep
        return nullptr;
    }
    return attr.devicePointer;
}

int gact_copy_bounded(void* dst, const void* src, size_t nbytes, int workgroups, void* stream) {
    if (workgroups < 1 || workgroups > 1024 || (nbytes > 0 && (!dst || !src))) return GACT_E_ARG;
    if (nbytes == 0) return GACT_OK;
    if (!aligned(dst, 16) || !aligned(src, 16)) return GACT_E_ARG;
    void* d = device_visible(dst);
    const void* s = device_visible(src);
    if (!d || !s) return GACT_E_ARG;
    return gact_launch_copy(d, s, (uint64_t)nbytes, (unsigned)workgroups, stream) == 0 ? GACT_OK : GACT_E_HIP;
}

int gact_compress_footprint_noalloc(const void* d_x, gact_dtype dtype, int64_t n, int group_size,
                                    int bits, uint64_t seed, void* d_packed, float* d_gmin,
                                    float* d_gscale, int n_samples, double* d_footprint,
                                    void* stream) {
    void* area = nullptr;
    if (const int rc = scratch_of_current_device(&area)) return rc;
    return compress_footprint(d_x, dtype, n, group_size, bits, seed, d_packed, d_gmin, d_gscale,
                              n_samples, d_footprint, area, GACT_NOALLOC_SCRATCH_BYTES, true, stream);
}

}  // extern "C"

// Records passed from the host entry points to the kernels.  Internal to the
// library; the public interface is include/gact.h.
#ifndef GACT_DEVICE_H
#define GACT_DEVICE_H

#include <stdint.h>

#ifndef __HIPCC__
#define __host__
#define __device__
#endif

#define GACT_DT_F32 0
#define GACT_DT_BF16 1

namespace gact {

// One tensor of a launch (56 bytes).  Pointers are device pointers.
struct TensorArgs {
    void*       io;        // compress: input x (read only); decompress: output y
    void*       packed;    // bit string (compress output, decompress input)
    float*      gmin;      // per-group minimum
    float*      gscale;    // per-group dequantisation step
    int64_t     n;         // elements
    uint32_t    seed_lo, seed_hi;
    // Whole dwords only: a sub-dword field would be fetched with a vector load,
    // which queues behind the kernel's own HBM traffic at the start of every block,
    // whereas dword fields of a uniform record come through the scalar cache.
    uint32_t    blk_base_lo;  // Philox block of element 0 (index_base / 8), low word
    uint32_t    meta;         // bits | dtype << 8 | (index_base / 8 >> 32) << 16
    __host__ __device__ int bits() const { return (int)(meta & 0xFFu); }
    __host__ __device__ int dtype() const { return (int)((meta >> 8) & 0xFFu); }
    __host__ __device__ uint64_t blk_base() const {
        return ((uint64_t)(meta >> 16) << 32) | blk_base_lo;
    }
};

// How a group size maps onto a wavefront: a lane owns 32 consecutive
// elements, a group is `lpg` = G/32 neighbouring lanes, a tile holds as many
// whole groups as fit into 64 lanes.
struct Geometry {
    int32_t lpg;           // lanes per group, 1..32
    int32_t lanes_used;    // (64 / lpg) * lpg
    int32_t pow2;          // lpg is a power of two (DPP reductions, full tiles)
    int32_t lpg_shift;     // log2(lpg) when pow2
    int32_t groups_per_tile;
    int32_t group_size;
    int32_t group_shift;   // log2(group_size) when pow2
    int32_t lds_wave_dwords;   // compress: LDS dwords per wavefront (lds_dwords_per_wave of the widest dtype launched)
};

// LDS one compressing wavefront stages its tile in: 64 rows of 32 elements in
// the input's own format.
constexpr int lds_dwords_per_wave(int dtype) { return dtype == GACT_DT_F32 ? 64 * 32 : 64 * 16; }

// Block -> tensor lookup of a multi-tensor launch.  first_block[l] is the first
// block of tensor l (one entry per tensor plus the total).  A search over it
// from scratch is a chain of dependent scalar loads at the start of every
// block (nine for 400 tensors), during which the block issues nothing else, so
// the host also lays a coarse index over the blocks: hint[k] is the tensor that
// holds block k << hint_shift.  Block b then belongs to a tensor in
// [hint[b >> hint_shift], hint[(b >> hint_shift) + 1]], which for all but the
// buckets that contain a tensor boundary is a single tensor.
constexpr int kInlineHints = 128;
// buckets for a table of L tensors in the workspace: a power of two >= 4 L
constexpr int hint_buckets(int L) {
    int h = 64;
    while (h < 4 * L && h < 16384) h *= 2;
    return h;
}

// A launch table small enough to travel in the kernel arguments (4 KB limit).
constexpr int kInlineTensors = 64;
struct InlineTable {
    TensorArgs t[kInlineTensors];
    uint32_t   first_block[kInlineTensors + 1];
    int32_t    L;
    uint32_t   hint_shift;
    uint32_t   hint[kInlineHints / 4 + 1];   // one byte per bucket, four to a dword (scalar loads fetch dwords)
};
// tensor of bucket k in a byte-packed hint array
__host__ __device__ inline int packed_hint(const uint32_t* hint, uint32_t k) {
    return (int)((hint[k >> 2] >> ((k & 3u) * 8u)) & 0xFFu);
}

// One buffer pair of a reduction launch: sensitivity reads a and b; gradient
// statistics read a (the gradient) and read-modify-write b (the fp32 mean).
struct ReduceArgs {
    const void* a;
    void*       b;
    int64_t     n;
    int32_t     dtype;     // of a (and of b for sensitivity)
    int32_t     pad;
};
// elements of one buffer a block covers: 256 threads x 4 pieces of 16 bytes
constexpr int64_t reduce_chunk_elems(int dtype) { return dtype == GACT_DT_F32 ? 4096 : 8192; }

// Decompress launch shape.  A unit is the 1 KB of output one coalesced
// wavefront store covers (256 fp32 or 512 bf16 elements); a block of four
// wavefronts takes 4 * units consecutive units.  Units per wavefront trade the
// load latency a wavefront hides against the length of its store burst; the
// best value depends on dtype and code width and was chosen by sweep on MI355X
// (% of HBM peak, decompress, 32 tensors of 13 / 26 M elements):
//            units  1     2     3     4     6
//   bf16 b=1      59.4  66.9  71.7  65.8  64.0
//   bf16 b=2      61.2  75.2  74.7  75.4  68.0   (2 units: 68.8 in a second run)
//   bf16 b=4      63.3  79.5  76.2  72.8  74.1
//   bf16 b=8      72.8  80.6  74.3  75.4  75.0
//   fp32 b=1      56.8  75.0  78.8  73.6  66.1
//   fp32 b=2      56.9  68.4  76.9  77.1  62.2
//   fp32 b=4      57.5  75.8  72.2  69.6  63.5
//   fp32 b=8      63.9  79.2  66.2  66.7  62.6
constexpr int dec_units_per_wave(int /*dtype*/, int bits) {
    return bits == 1 ? 3 : bits == 2 ? 4 : 2;
}
constexpr int dec_block_elems(int dtype, int bits) {
    return 4 * dec_units_per_wave(dtype, bits) * (dtype == GACT_DT_F32 ? 256 : 512);
}

}  // namespace gact

extern "C" int gact_launch_single(int compress, const gact::TensorArgs* t,
                                  const gact::Geometry* geo, unsigned blocks, void* stream);
extern "C" int gact_launch_diff_sq(const gact::ReduceArgs* d_table, const uint32_t* d_first, int K,
                                   unsigned blocks, double* d_partial, double scale, double* d_out,
                                   void* stream);
extern "C" int gact_launch_compress_sum(const gact::TensorArgs* t, const gact::Geometry* geo,
                                        unsigned blocks, double* d_tile_sum, void* stream);
extern "C" int gact_launch_footprint_finish(const gact::ReduceArgs* r, unsigned count, double* d_partial,
                                            int n_samples, double* d_out, void* stream);
extern "C" int gact_launch_footprint(const gact::ReduceArgs* r, unsigned blocks, double* d_partial,
                                     int n_samples, double* d_out, void* stream);
extern "C" int gact_launch_zero(double* d_out, int nout, void* stream);
extern "C" int gact_launch_grad_stats(const gact::ReduceArgs* d_table, const uint32_t* d_first, int K,
                                      float rt, unsigned blocks, double* d_partial, double* d_out,
                                      void* stream);
extern "C" int gact_launch_copy(void* dst, const void* src, uint64_t nbytes, unsigned workgroups, void* stream);
extern "C" int gact_launch_multi_inline(int compress, const gact::InlineTable* tab,
                                        const gact::Geometry* geo, unsigned blocks, void* stream);
extern "C" int gact_launch_multi(int compress, const gact::TensorArgs* d_table,
                                 const uint32_t* d_first_block, const uint32_t* d_hint,
                                 unsigned hint_shift, const gact::Geometry* geo, unsigned blocks,
                                 void* stream);

#endif

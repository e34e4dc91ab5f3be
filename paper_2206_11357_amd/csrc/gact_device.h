// Records passed from the host entry points to the kernels.  Internal to the
// library; the public interface is include/gact.h.
#ifndef GACT_DEVICE_H
#define GACT_DEVICE_H

#include <stdint.h>

#define GACT_DT_F32 0
#define GACT_DT_BF16 1

namespace gact {

// One tensor of a launch.  Pointers are device pointers.
struct TensorArgs {
    const void* x;         // compress input
    void*       packed;    // bit string (compress output, decompress input)
    float*      gmin;      // per-group minimum
    float*      gscale;    // per-group dequantisation step
    void*       y;         // decompress output
    int64_t     n;         // elements
    int64_t     tiles;     // wavefront tiles covering the tensor
    int64_t     packed_words;  // gact_packed_bytes / 4
    uint32_t    seed_lo, seed_hi;
    int32_t     bits;
    int32_t     dtype;
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
};

}  // namespace gact

extern "C" int gact_launch_single(int compress, const gact::TensorArgs* t,
                                  const gact::Geometry* geo, unsigned blocks, void* stream);
extern "C" int gact_launch_multi(int compress, const gact::TensorArgs* d_table,
                                 const uint32_t* d_first_block, int L,
                                 const gact::Geometry* geo, unsigned blocks, void* stream);

#endif

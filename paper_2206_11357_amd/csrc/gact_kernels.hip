// GACT activation compressor / decompressor for MI355X (gfx950, wave64).
//
// What is computed: the per-group stochastic-rounding quantizer of
// arXiv 2206.11357 (App. A.4, applied per group as in Sec. 5) and its inverse;
// the exact arithmetic contract is stated in include/gact.h.
//
// How the work is laid out
//   Compress
//   * One wavefront owns one "tile": 64 lanes x 32 consecutive elements
//     (2048 elements when the group size is a power of two).  A group of G
//     elements is G/32 neighbouring lanes, so group statistics are a handful
//     of DPP steps and every lane does the two IEEE divisions of its group
//     once per 32 elements.
//   * HBM is read with fully coalesced 16-byte loads (lane i of load k reads
//     bytes [k*1024 + 16 i, +16)).  The switch from that layout to "32
//     consecutive elements per lane" goes through a private LDS region per
//     wavefront, in the input's own format (8 KB for fp32, 4 KB for bf16; the
//     16-byte pieces of a row are XOR-swizzled so that 128-bit LDS reads and
//     writes are conflict-free without padding).  The LDS a wavefront holds
//     bounds how many are resident, so the launch sizes it by the widest dtype
//     present.
//   * With 32 elements per lane a lane owns 32*bits packed bits = `bits`
//     dwords, and neighbouring lanes own neighbouring dwords: the packed
//     stream is written coalesced without further staging.
//   * Rounding noise: one Philox4x32-10 block per 8 consecutive elements, so
//     four blocks per lane; the stream depends on (seed, element index) only.
//   Decompress
//   * No layout switch and no LDS: a lane produces one 16-byte piece of output
//     per coalesced store and fetches that piece's codes with one small load.
//   * No MFMA anywhere: the path is a streaming codec, bound by HBM (fp32) or
//     by plain VALU work (bf16 compress), not a contraction.
//
// Tiles that are not full (the end of a tensor) and group sizes that are not a
// power of two take the guarded `Edge` instantiation of the same code.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gact_device.h"

namespace gact {

typedef float    f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef uint32_t u2 __attribute__((ext_vector_type(2)));

constexpr int kLanes        = 64;
constexpr int kPerLane      = 32;                 // consecutive elements one lane owns
constexpr int kWavesPerBlk  = 4;
constexpr int kBlockThreads = kLanes * kWavesPerBlk;

// 32-bit words of the packed buffer: ceil(n*bits/8) bytes rounded up to 16
__device__ __forceinline__ int64_t packed_words(const TensorArgs& t) {
    return (int64_t)((((uint64_t)t.n * (uint64_t)t.bits() + 127u) >> 7) << 2);
}

// ---------------------------------------------------------------- lane moves
__device__ __forceinline__ float swizzle_xor16(float v) {
    // bit-mask mode: and 0x1f, or 0, xor 0x10 (lane ^ 16 inside each half wave)
    return __builtin_bit_cast(
        float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), (16 << 10) | 0x1F));
}
__device__ __forceinline__ float lane_read(float v, int src_lane) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_ds_bpermute(src_lane << 2, __builtin_bit_cast(int, v)));
}

// min / max of finite values (v_min_f32 / v_min3_f32).  The sign of a zero
// result is not defined by these; the stored minimum is canonicalised later.
__device__ __forceinline__ float fmin2(float a, float b) { return __builtin_fminf(a, b); }
__device__ __forceinline__ float fmax2(float a, float b) { return __builtin_fmaxf(a, b); }

// v = min / max(v, v of the DPP-selected lane) in one instruction.  Written as
// assembly because the compiler otherwise moves the DPP operand into its own
// register and re-canonicalises both inputs (4 instructions per step).
// A DPP operand must not be read in the two issue slots after a vector
// instruction has written it, and the compiler's hazard pass does not look
// inside an assembly statement, so each statement brings its own wait states.
#define GACT_DPP_MINMAX(NAME, OP, CTRL)                                                  \
    __device__ __forceinline__ float NAME(float v) {                                     \
        float r;                                                                          \
        asm("s_nop 1\n\t" OP " %0, %1, %1 " CTRL " row_mask:0xf bank_mask:0xf"          \
            : "=v"(r) : "v"(v));                                                          \
        return r;                                                                         \
    }
GACT_DPP_MINMAX(min_xor1, "v_min_f32_dpp", "quad_perm:[1,0,3,2]")
GACT_DPP_MINMAX(max_xor1, "v_max_f32_dpp", "quad_perm:[1,0,3,2]")
GACT_DPP_MINMAX(min_xor2, "v_min_f32_dpp", "quad_perm:[2,3,0,1]")
GACT_DPP_MINMAX(max_xor2, "v_max_f32_dpp", "quad_perm:[2,3,0,1]")
GACT_DPP_MINMAX(min_half_mirror, "v_min_f32_dpp", "row_half_mirror")
GACT_DPP_MINMAX(max_half_mirror, "v_max_f32_dpp", "row_half_mirror")
GACT_DPP_MINMAX(min_mirror, "v_min_f32_dpp", "row_mirror")
GACT_DPP_MINMAX(max_mirror, "v_max_f32_dpp", "row_mirror")
#undef GACT_DPP_MINMAX

// All lanes of a group (lpg neighbouring lanes, lpg a power of two <= 32,
// groups aligned to lpg) end up with the group's min and max.  After the two
// quad steps all lanes of a quad agree, so the 8- and 16-lane mirrors pair
// each lane with one from the other half.
__device__ __forceinline__ void group_minmax_pow2(float& mn, float& mx, int lpg) {
    if (lpg > 1)  { mn = min_xor1(mn);        mx = max_xor1(mx); }
    if (lpg > 2)  { mn = min_xor2(mn);        mx = max_xor2(mx); }
    if (lpg > 4)  { mn = min_half_mirror(mn); mx = max_half_mirror(mx); }
    if (lpg > 8)  { mn = min_mirror(mn);      mx = max_mirror(mx); }
    if (lpg > 16) { mn = fmin2(mn, swizzle_xor16(mn)); mx = fmax2(mx, swizzle_xor16(mx)); }
}

// Any lpg in [1, 32]: every lane scans the lanes of its own group.
__device__ __forceinline__ void group_minmax_any(float& mn, float& mx, int lpg, int lane) {
    const int first = (lane / lpg) * lpg;
    float a = mn, b = mx;
    for (int j = 0; j < lpg; ++j) {
        const int src = (first + j) & 63;
        a = fmin2(a, lane_read(mn, src));
        b = fmax2(b, lane_read(mx, src));
    }
    mn = a;
    mx = b;
}

// ------------------------------------------------------------------- Philox
// Philox4x32-10 (Salmon et al., SC'11) on counter (c0, c1, 0, 0), key (k0, k1).
constexpr uint32_t kPhiloxM0 = 0xD2511F53u, kPhiloxM1 = 0xCD9E8D57u;
constexpr uint32_t kPhiloxW0 = 0x9E3779B9u, kPhiloxW1 = 0xBB67AE85u;

// three-input xor in one v_bitop3_b32 (truth table 0x96)
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

// rounds FIRST .. 9 (round r uses the key bumped r times)
template <int FIRST>
__device__ __forceinline__ void philox_rounds(uint32_t& c0, uint32_t& c1, uint32_t& c2, uint32_t& c3,
                                              uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = FIRST; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)kPhiloxM0 * c0;
        const uint64_t p1 = (uint64_t)kPhiloxM1 * c2;
        const uint32_t n0 = xor3((uint32_t)(p1 >> 32), c1, k0 + (uint32_t)r * kPhiloxW0);
        const uint32_t n2 = xor3((uint32_t)(p0 >> 32), c3, k1 + (uint32_t)r * kPhiloxW1);
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
    }
}

// Rounds 0..2 of a block whose counter is (c0, c1u, 0, 0) with the high word c1u
// and the key uniform over the wavefront -- the case for every block of a tile
// unless the low counter word wraps inside the tile.  Counter words 2 and 3
// being zero, part of these rounds is the same for every lane and is computed
// once per wavefront, on the scalar unit (PhiloxUniform):
//   round 0: M1 * 0 = 0, so word 0 becomes c1u ^ k0 (uniform) and word 1 is 0;
//   round 1: M0 * (uniform word 0) is a scalar product; its low half is the
//            new, uniform, word 3;
//   round 2: the uniform word 3 and the key fold into one scalar operand.
// Four 32 x 32 -> 64 multiplies per block instead of six.
struct PhiloxUniform {
    uint32_t f2, g2;
    __device__ __forceinline__ PhiloxUniform(uint32_t c1u, uint32_t k0, uint32_t k1) {
        const uint32_t a0 = c1u ^ k0;                                      // round 0, word 0
        const uint64_t P0 = (uint64_t)kPhiloxM0 * a0;                       // round 1 product
        f2 = (uint32_t)(P0 >> 32) ^ (k1 + kPhiloxW1);                       // round 1: word 2 = f2 ^ old word 3
        g2 = (uint32_t)P0 ^ (k1 + 2u * kPhiloxW1);                          // round 2: word 2 = hi(M0 word 0) ^ g2
    }
};
__device__ __forceinline__ void philox_head_uniform(uint32_t c0, const PhiloxUniform& u, uint32_t k0,
                                                    uint32_t k1, uint32_t st[4]) {
    const uint64_t p0 = (uint64_t)kPhiloxM0 * c0;                           // round 0
    const uint32_t a2 = (uint32_t)(p0 >> 32) ^ k1;
    const uint32_t a3 = (uint32_t)p0;
    const uint64_t p1 = (uint64_t)kPhiloxM1 * a2;                           // round 1
    const uint32_t b0 = (uint32_t)(p1 >> 32) ^ (k0 + kPhiloxW0);
    const uint32_t b1 = (uint32_t)p1;
    const uint32_t b2 = a3 ^ u.f2;
    const uint64_t q0 = (uint64_t)kPhiloxM0 * b0;                           // round 2
    const uint64_t q1 = (uint64_t)kPhiloxM1 * b2;
    st[0] = xor3((uint32_t)(q1 >> 32), b1, k0 + 2u * kPhiloxW0);
    st[1] = (uint32_t)q1;
    st[2] = (uint32_t)(q0 >> 32) ^ u.g2;
    st[3] = (uint32_t)q0;
}

// The same three rounds for any per-lane 64-bit block number.
__device__ __forceinline__ void philox_head_any(uint64_t blk, uint32_t k0, uint32_t k1, uint32_t st[4]) {
    uint32_t c0 = (uint32_t)blk, c1 = (uint32_t)(blk >> 32), c2 = 0u, c3 = 0u;
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const uint64_t p0 = (uint64_t)kPhiloxM0 * c0;
        const uint64_t p1 = (uint64_t)kPhiloxM1 * c2;
        const uint32_t n0 = xor3((uint32_t)(p1 >> 32), c1, k0 + (uint32_t)r * kPhiloxW0);
        const uint32_t n2 = xor3((uint32_t)(p0 >> 32), c3, k1 + (uint32_t)r * kPhiloxW1);
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
    }
    st[0] = c0; st[1] = c1; st[2] = c2; st[3] = c3;
}

// Three-input min / max of finite values.  As assembly because the compiler
// puts a canonicalising v_max_f32 x, x in front of values it cannot prove to be
// free of signalling NaNs (everything that was widened from bf16 with bit
// operations); non-finite input is outside the contract.
__device__ __forceinline__ float fmin3(float a, float b, float c) {
    float r;
    asm("v_min3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
__device__ __forceinline__ float fmax3(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// x[j] <- x[j] + b for eight values, rounded toward minus infinity.  The
// wavefront's binary32 rounding mode (MODE bits 1:0) is switched to round-down
// for exactly these eight additions and back to nearest-even; the block is one
// volatile statement, so no other floating-point instruction can be scheduled
// into it and everything outside keeps the nearest-even contract.
__device__ __forceinline__ void add8_round_down(float (&x)[8], float b) {
    asm volatile(
        "s_setreg_imm32_b32 hwreg(HW_REG_MODE, 0, 2), 2\n\t"
        "v_add_f32 %0, %0, %8\n\t"
        "v_add_f32 %1, %1, %8\n\t"
        "v_add_f32 %2, %2, %8\n\t"
        "v_add_f32 %3, %3, %8\n\t"
        "v_add_f32 %4, %4, %8\n\t"
        "v_add_f32 %5, %5, %8\n\t"
        "v_add_f32 %6, %6, %8\n\t"
        "v_add_f32 %7, %7, %8\n\t"
        "s_setreg_imm32_b32 hwreg(HW_REG_MODE, 0, 2), 0"
        : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7])
        : "v"(b));
}

// Instructions the compiler does not select on its own.
// floor(x) as int32 in one instruction.
__device__ __forceinline__ int32_t cvt_floor_i32(float x) {
    int32_t r;
    asm("v_cvt_flr_i32_f32 %0, %1" : "=v"(r) : "v"(x));
    return r;
}
// 2 * (low / high 16 bits of w) + c
__device__ __forceinline__ uint32_t mad2_lo16(uint32_t w, uint32_t c) {
    uint32_t r;
    asm("v_mad_u32_u16 %0, %1, 2, %2" : "=v"(r) : "v"(w), "v"(c));
    return r;
}
__device__ __forceinline__ uint32_t mad2_hi16(uint32_t w, uint32_t c) {
    uint32_t r;
    asm("v_mad_u32_u16 %0, %1, 2, %2 op_sel:[1,0,0,0]" : "=v"(r) : "v"(w), "v"(c));
    return r;
}

// ------------------------------------------------------- tile <-> HBM moves
// The raw 16-byte loads of one tile: fp32 8 per lane, bf16 4 per lane.
template <int DT>
struct RawTile {
    u4 r[DT == GACT_DT_F32 ? 8 : 4];
};

// Coalesced global loads.  `ne` = number of valid elements of the tile (2048
// for a full tile); elements past `ne` are never read from memory and read 0.
template <int DT, bool EDGE>
__device__ __forceinline__ void load_tile(const void* __restrict__ x, int64_t e0, int ne, int lane,
                                          RawTile<DT>& raw) {
    if (DT == GACT_DT_F32) {
        const uint32_t* p = (const uint32_t*)x + e0;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int e = k * 256 + lane * 4;
            if (!EDGE) {
                raw.r[k] = __builtin_nontemporal_load((const u4*)(p + e));
            } else if (e + 4 <= ne) {
                raw.r[k] = *(const u4*)(p + e);
            } else {
                u4 t = {0u, 0u, 0u, 0u};
                if (e + 0 < ne) t.x = p[e + 0];
                if (e + 1 < ne) t.y = p[e + 1];
                if (e + 2 < ne) t.z = p[e + 2];
                raw.r[k] = t;
            }
        }
    } else {
        const uint16_t* p = (const uint16_t*)x + e0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int e = k * 512 + lane * 8;
            if (!EDGE) {
                raw.r[k] = __builtin_nontemporal_load((const u4*)(p + e));
            } else if (e + 8 <= ne) {
                raw.r[k] = *(const u4*)(p + e);
            } else {
                uint32_t h[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) h[j] = (e + j < ne) ? (uint32_t)p[e + j] : 0u;
                u4 t = {h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16),
                        h[6] | (h[7] << 16)};
                raw.r[k] = t;
            }
        }
    }
}

// Raw tile -> LDS rows (row r = elements 32 r .. 32 r + 31) in the input's own
// format: 8 (fp32) or 4 (bf16) pieces of 16 bytes per row.  Staging bf16
// unwidened halves the LDS a wavefront holds, which is what bounds the number
// of resident wavefronts.  Rows are not padded; piece p of row r sits at slot
// p ^ s(r), with s(r) = (r >> 1) & 7 for fp32 and (r >> 2) & 3 for bf16.  A
// 128-bit LDS access is served 16 lanes at a time over 64 banks:
//   * writes: 16 neighbouring lanes hold 16 consecutive pieces, i.e. all slots
//     of 2 (4) neighbouring rows that share s(r) -> 16 distinct bank quads;
//   * reads: 16 neighbouring lanes read the same piece index of 16 consecutive
//     rows; the row's own offset covers 2 (4) bank quads and s(r) runs through
//     the 8 (4) values that complete them.
template <int DT>
__device__ __forceinline__ void stage_tile(const RawTile<DT>& raw, uint32_t* __restrict__ lds,
                                           int lane) {
    if (DT == GACT_DT_F32) {
        // load k, lane L: row 8 k + L / 8, piece L % 8, s = (4 k + L / 16) & 7
        uint32_t* base = lds + (lane >> 3) * 32;
        const int slot0 = ((lane & 7) ^ (lane >> 4)) * 4;          // even k
        const int slot1 = slot0 ^ 16;                              // odd k
#pragma unroll
        for (int k = 0; k < 8; ++k)
            *(u4*)(base + k * 256 + ((k & 1) ? slot1 : slot0)) = raw.r[k];
    } else {
        // load k, lane L: row 16 k + L / 4, piece L % 4, s = (L / 16) & 3
        uint32_t* base = lds + (lane >> 2) * 16 + (((lane & 3) ^ (lane >> 4)) * 4);
#pragma unroll
        for (int k = 0; k < 4; ++k) *(u4*)(base + k * 256) = raw.r[k];
    }
}

// The lane's own row as fp32; bf16 is widened here, exactly.
template <int DT>
__device__ __forceinline__ void read_row(const uint32_t* __restrict__ lds, int row, float v[kPerLane]) {
    if (DT == GACT_DT_F32) {
        const uint32_t first = (uint32_t)row * 32u + (((uint32_t)row >> 1) & 7u) * 4u;   // piece 0
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const f4 q = *(const f4*)(lds + (first ^ (uint32_t)(4 * k)));
            v[4 * k + 0] = q.x; v[4 * k + 1] = q.y; v[4 * k + 2] = q.z; v[4 * k + 3] = q.w;
        }
    } else {
        const uint32_t first = (uint32_t)row * 16u + (((uint32_t)row >> 2) & 3u) * 4u;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const u4 w = *(const u4*)(lds + (first ^ (uint32_t)(4 * k)));
            const uint32_t h[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                v[8 * k + 2 * j + 0] = __builtin_bit_cast(float, h[j] << 16);
                v[8 * k + 2 * j + 1] = __builtin_bit_cast(float, h[j] & 0xFFFF0000u);
            }
        }
    }
}

// two fp32 -> two bf16 (low half = a), round to nearest even: v_cvt_pk_bf16_f32
typedef float  f2v  __attribute__((ext_vector_type(2)));
typedef __bf16 bf2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t bf16_pair_rne(float a, float b) {
    const f2v v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf2v));
}

__device__ __forceinline__ void wave_lds_sync() {
    // LDS operations of one wavefront execute in order; this only stops the
    // compiler from moving LDS accesses across the layout switch.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ----------------------------------------------------------------- compress
// One wavefront compresses tile `tile` of tensor `t`.
//   geo.lpg        lanes per group (G/32)
//   geo.lanes_used lanes that hold data in a full tile (64 for power-of-two G)
//   SUM            also write the binary64 sum of the tile's elements to tile_sum[tile]
//                  (the footprint of Sec. 5.2 from the same read)
template <int DT, int BITS, bool EDGE, bool SUM>
__device__ __forceinline__ void compress_tile(const TensorArgs& t, const Geometry& geo,
                                              int64_t tile, uint32_t* __restrict__ lds, int lane,
                                              double* __restrict__ tile_sum) {
    constexpr uint32_t B = (1u << BITS) - 1u;
    const int tile_elems = geo.lanes_used * kPerLane;
    const int64_t e0 = tile * (int64_t)tile_elems;       // `tile` is uniform over the wavefront
    int ne = tile_elems;
    if (EDGE) {
        const int64_t left = t.n - e0;
        ne = left < (int64_t)tile_elems ? (int)left : tile_elems;
    }

    RawTile<DT> raw;
    load_tile<DT, EDGE>(t.io, e0, ne, lane, raw);

    // layout switch: coalesced rows in, 32 consecutive elements per lane out
    float v[kPerLane];
    stage_tile<DT>(raw, lds, lane);
    wave_lds_sync();
    read_row<DT>(lds, lane, v);

    const int my0 = lane * kPerLane;                 // first element of this lane in the tile
    if (SUM) {
        // lane: its 32 elements in index order; wavefront: xor butterfly 32, 16, ... 1
        double acc = 0.0;
#pragma unroll
        for (int j = 0; j < kPerLane; ++j)
            if (!EDGE || my0 + j < ne) acc += (double)v[j];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
        if (lane == 0) tile_sum[tile] = acc;
    }

    // group statistics
    float mn, mx;
    if (!EDGE) {
        mn = fmin3(v[0], v[1], v[2]); mx = fmax3(v[0], v[1], v[2]);
#pragma unroll
        for (int j = 3; j + 1 < kPerLane; j += 2) { mn = fmin3(mn, v[j], v[j + 1]); mx = fmax3(mx, v[j], v[j + 1]); }
        mn = fmin3(mn, v[kPerLane - 1], v[kPerLane - 1]); mx = fmax3(mx, v[kPerLane - 1], v[kPerLane - 1]);
        group_minmax_pow2(mn, mx, geo.lpg);
    } else {
        mn = __builtin_inff(); mx = -__builtin_inff();
#pragma unroll
        for (int j = 0; j < kPerLane; ++j) {
            if (my0 + j < ne) { mn = fmin2(mn, v[j]); mx = fmax2(mx, v[j]); }
        }
        if (geo.pow2) group_minmax_pow2(mn, mx, geo.lpg);
        else group_minmax_any(mn, mx, geo.lpg, lane);
    }
    mn = mn + 0.0f;                                  // store -0 as +0
    const float range = mx - mn;
    const float Bf = (float)B;
    float inv = 0.0f, step = 0.0f;
    if (range >= 0x1p-100f) { inv = Bf / range; step = range / Bf; }

    // Minimum and step of every group of the tile.  All lanes of a group hold the
    // same pair.  Stored from the first lane of each group, the values would leave
    // from lanes lpg apart, and a store whose active lanes are scattered over the
    // wavefront goes to memory as one small request per lane (with 4 lanes per
    // group those requests cost 7 % of the compressor's time).  So the pairs are
    // first gathered into the low lanes (two ds_bpermute on the LDS crossbar: lane
    // i takes minimum and step of group i from lane i * lpg) and leave as two
    // contiguous runs.  The gathers are issued here and their results stored
    // after the codes, so that nothing waits for the LDS round trip.
    const int64_t g0 = tile * (int64_t)geo.groups_per_tile;        // first group of the tile
    float group_mn = mn, group_step = step;
    if (geo.lpg > 1) {
        const int src = lane * geo.lpg;                            // lanes past the last group read a wrapped lane, unused
        group_mn = lane_read(mn, src);
        group_step = lane_read(step, src);
    }

    // stochastic rounding + packing: 8 elements per Philox block.
    //
    // The rule "q = floor(t) + [ (r+1/2)/2^16 < t - floor(t) ]" is evaluated in
    // integers.  With T = 2^17 t (an exact rescaling of the binary32 product),
    // C = ceil(T) and c = C mod 2^17:  round up  <=>  2 frac 2^16 > 2r + 1
    // <=>  c >= 2r + 2  <=>  2r + 1 - C < -(floor(t) 2^17), hence
    //     -q = (2r + 1 - C) >> 17   (arithmetic shift).
    // 1 - C = floor(-T) + 1 comes out of one addition rounded toward minus
    // infinity: for |T| < 2^22 (codes of up to 4 bits: T <= 15 * 2^17 (1 + 2^-23))
    // the sum -T + (1.5 * 2^23 + 1) lies in [2^23, 2^24), where binary32 has a
    // spacing of 1, so its round-down value is 1.5 * 2^23 + 1 + floor(-T) exactly
    // and its bit pattern is 0x4B400001 + floor(-T).  The 16-bit multiply-add
    // that selects the noise half word adds 2r to that pattern, and because
    // 0x4B400000 is a multiple of 2^17 the shift gives kBias - q with
    // kBias = 0x4B400000 >> 17.  8-bit codes (T up to 2^25) use a
    // convert-with-floor instead (kBias = 0).  The biased negated codes are
    // accumulated last element first, one shift-add each, and the word is
    // kBias * (sum of the field weights) - accumulator, all modulo 2^32.
    constexpr bool kMagic = BITS <= 4;
    constexpr uint32_t kBias = kMagic ? (0x4B400000u >> 17) : 0u;
    constexpr uint32_t kFieldWeights = BITS == 1 ? 0xFFFFFFFFu : BITS == 2 ? 0x55555555u
                                     : BITS == 4 ? 0x11111111u : 0x01010101u;
    constexpr uint32_t kBiasWord = kBias * kFieldWeights;          // modulo 2^32
    uint32_t acc[BITS];
#pragma unroll
    for (int w = 0; w < BITS; ++w) acc[w] = 0u;
    const float ninv17 = -(inv * 0x1p17f);
    // block numbers of this lane: tile_blk + 4 lane + (0..3); the high word is the
    // same for the whole tile unless the low word wraps inside it
    const uint64_t tile_blk = t.blk_base() + ((uint64_t)e0 >> 3);
    const bool hi_uniform = (uint32_t)tile_blk <= 0xFFFFFEFFu;
    const PhiloxUniform pu((uint32_t)(tile_blk >> 32), t.seed_lo, t.seed_hi);
    const uint32_t lane_c0 = (uint32_t)tile_blk + 4u * (uint32_t)lane;
#pragma unroll
    for (int c = 3; c >= 0; --c) {
        uint32_t r[4];
        if (hi_uniform) philox_head_uniform(lane_c0 + (uint32_t)c, pu, t.seed_lo, t.seed_hi, r);
        else philox_head_any(tile_blk + (uint64_t)(4 * lane + c), t.seed_lo, t.seed_hi, r);
        philox_rounds<3>(r[0], r[1], r[2], r[3], t.seed_lo, t.seed_hi);
        float tn[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) tn[j] = (v[c * 8 + j] - mn) * ninv17;   // -T, T in [0, 2^25)
        if (kMagic) add8_round_down(tn, 12582913.0f);                      // 1.5 * 2^23 + 1
#pragma unroll
        for (int j = 7; j >= 0; --j) {
            const int e = c * 8 + j;
            const uint32_t n1 = kMagic ? __builtin_bit_cast(uint32_t, tn[j])
                                       : (uint32_t)(cvt_floor_i32(tn[j]) + 1);     // (bias +) 1 - C
            const uint32_t y = (j & 1) ? mad2_hi16(r[j >> 1], n1) : mad2_lo16(r[j >> 1], n1);
            int32_t nq = (int32_t)y >> 17;                        // kBias - q
            // t <= B (1 + 2^-23): an overshoot's fraction is below the smallest
            // noise value 2^-17 unless B = 255, so only 8-bit codes can round
            // past the top level
            if (BITS == 8) nq = nq > -(int32_t)B ? nq : -(int32_t)B;
            if (EDGE && my0 + e >= ne) nq = (int32_t)kBias;
            const int w = (e * BITS) >> 5;
            acc[w] = (acc[w] << BITS) + (uint32_t)nq;
        }
    }
    uint32_t out[BITS];
#pragma unroll
    for (int w = 0; w < BITS; ++w) out[w] = kBiasWord - acc[w];

    if (lane < geo.groups_per_tile && (!EDGE || lane * geo.lpg * kPerLane < ne)) {
        float* gm = t.gmin + g0;                                   // uniform bases, lane offsets
        float* gs = t.gscale + g0;
        gm[lane] = group_mn;
        gs[lane] = group_step;
    }

    // lane i owns dwords [i*BITS, (i+1)*BITS) of the tile's packed words
    const int64_t word0 = (e0 >> 5) * BITS + (int64_t)lane * BITS;
    uint32_t* pk = (uint32_t*)t.packed + word0;
    if (!EDGE) {
        if (BITS == 1) {
            __builtin_nontemporal_store(out[0], pk);
        } else if (BITS == 2) {
            u2 o = {out[0], out[1]};
            __builtin_nontemporal_store(o, (u2*)pk);
        } else {
#pragma unroll
            for (int w = 0; w < BITS; w += 4) {
                u4 o = {out[w], out[w + 1], out[w + 2], out[w + 3]};
                __builtin_nontemporal_store(o, (u4*)(pk + w));
            }
        }
    } else {
        // the packed buffer ends at a multiple of 16 bytes; pad words are zero
        const int64_t words_total = packed_words(t);
#pragma unroll
        for (int w = 0; w < BITS; ++w)
            if (lane < geo.lanes_used && word0 + w < words_total) pk[w] = out[w];
        // when a tile is narrower than 128*8/BITS elements' worth of padding
        // (group sizes that are not a power of two), up to three pad words lie
        // past the last tile's lanes: the last tile zeroes them
        if ((tile + 1) * (int64_t)tile_elems >= t.n && lane < 4) {          // the last tile
            const int64_t w = (e0 >> 5) * BITS + (int64_t)geo.lanes_used * BITS + lane;
            if (w < words_total) ((uint32_t*)t.packed)[w] = 0u;
        }
    }
}

// --------------------------------------------------------------- decompress
// The decompressor needs no layout switch: a lane handles one 16-byte piece of
// output (4 fp32 or 8 bf16 consecutive elements) per "unit", a unit being the
// 1 KB that one coalesced wavefront store covers.  The piece's codes are
// 4*BITS or 8*BITS consecutive bits of the packed string (a nibble, byte, half
// word, word or two words), fetched with one small load; neighbouring lanes
// fetch neighbouring bits, so those loads coalesce too.  The group's min and
// step are two more loads that all lanes of a group share.  Wavefront w of a
// block takes units w, w+4, w+8, ... so that the four wavefronts write one
// contiguous 4 KB at each step.  Stores are the bottleneck here; the number of
// units per wavefront (dec_units_per_wave) trades load latency hidden per
// wavefront against the length of its store burst and was chosen by sweep.
template <int DT>
struct DecGeom {
    static constexpr int kPiece = DT == GACT_DT_F32 ? 4 : 8;      // elements per lane and unit
    static constexpr int kUnit = 64 * kPiece;                     // elements per unit
};

// codes of one piece, first element in the low bits
template <int DT, int BITS>
struct PieceBits {
    static constexpr int kBits = DecGeom<DT>::kPiece * BITS;      // 4 .. 64
    uint32_t lo, hi;
};

template <int DT, int BITS, bool EDGE>
__device__ __forceinline__ void load_piece(const TensorArgs& t, int64_t e, PieceBits<DT, BITS>& pb) {
    constexpr int nb = PieceBits<DT, BITS>::kBits;
    const uint8_t* base = (const uint8_t*)t.packed;
    const int64_t bit = e * BITS;
    const int64_t byte = bit >> 3;
    pb.lo = 0u; pb.hi = 0u;
    if (EDGE) {
        // byte by byte, never past the end of the (16-byte rounded) buffer
        const int64_t total = packed_words(t) * 4;
#pragma unroll
        for (int k = 0; k < (nb + 7) / 8; ++k) {
            const uint32_t v = (byte + k < total) ? (uint32_t)base[byte + k] : 0u;
            if (k < 4) pb.lo |= v << (8 * k); else pb.hi |= v << (8 * (k - 4));
        }
        if (nb == 4) pb.lo = (pb.lo >> (int)(bit & 7)) & 0xFu;
        return;
    }
    if (nb == 4) {
        pb.lo = ((uint32_t)__builtin_nontemporal_load(base + byte) >> (int)(bit & 7)) & 0xFu;
    } else if (nb == 8) {
        pb.lo = __builtin_nontemporal_load(base + byte);
    } else if (nb == 16) {
        pb.lo = __builtin_nontemporal_load((const uint16_t*)(base + byte));
    } else if (nb == 32) {
        pb.lo = __builtin_nontemporal_load((const uint32_t*)(base + byte));
    } else {
        const u2 w = __builtin_nontemporal_load((const u2*)(base + byte));
        pb.lo = w.x; pb.hi = w.y;
    }
}

template <int DT, int BITS, bool EDGE, int UNITS>
__device__ __forceinline__ void decompress_units(const TensorArgs& t, const Geometry& geo,
                                                 int64_t block_in_tensor, int wave, int lane) {
    constexpr uint32_t B = (1u << BITS) - 1u;
    constexpr int P = DecGeom<DT>::kPiece;
    constexpr int U = DecGeom<DT>::kUnit;
    PieceBits<DT, BITS> pb[UNITS];
    float mn[UNITS], step[UNITS];
    int64_t e[UNITS];
#pragma unroll
    for (int k = 0; k < UNITS; ++k) {
        const int64_t unit = block_in_tensor * (kWavesPerBlk * UNITS) + k * kWavesPerBlk + wave;
        e[k] = unit * U + lane * P;
        mn[k] = 0.0f; step[k] = 0.0f; pb[k].lo = 0u; pb[k].hi = 0u;
        if (!EDGE || e[k] < t.n) {
            load_piece<DT, BITS, EDGE>(t, e[k], pb[k]);
            const int64_t g = geo.pow2 ? (e[k] >> geo.group_shift)
                                       : (int64_t)((uint64_t)e[k] / (uint32_t)geo.group_size);
            mn[k] = t.gmin[g];
            step[k] = t.gscale[g];
        }
    }
#pragma unroll
    for (int k = 0; k < UNITS; ++k) {
        if (EDGE && e[k] >= t.n) continue;
        float o[P];
#pragma unroll
        for (int j = 0; j < P; ++j) {
            const int bit = j * BITS;
            const uint32_t q = ((bit < 32 ? pb[k].lo >> bit : pb[k].hi >> (bit - 32))) & B;
            const float prod = (float)q * step[k];
            o[j] = prod + mn[k];
        }
        if (DT == GACT_DT_F32) {
            float* p = (float*)t.io + e[k];
            if (!EDGE || e[k] + P <= t.n) {
                const f4 v = {o[0], o[1], o[2], o[3]};
                if (!EDGE) __builtin_nontemporal_store(v, (f4*)p); else *(f4*)p = v;
            } else {
#pragma unroll
                for (int j = 0; j < P; ++j) if (e[k] + j < t.n) p[j] = o[j];
            }
        } else {
            uint16_t* p = (uint16_t*)t.io + e[k];
            const u4 v = {bf16_pair_rne(o[0], o[1]), bf16_pair_rne(o[2 % P], o[3 % P]),
                          bf16_pair_rne(o[4 % P], o[5 % P]), bf16_pair_rne(o[6 % P], o[7 % P])};
            if (!EDGE || e[k] + P <= t.n) {
                if (!EDGE) __builtin_nontemporal_store(v, (u4*)p); else *(u4*)p = v;
            } else {
                const uint32_t hh[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int j = 0; j < P; ++j)
                    if (e[k] + j < t.n) p[j] = (uint16_t)(hh[j >> 1] >> (16 * (j & 1)));
            }
        }
    }
}

// ------------------------------------------------------------------ kernels
// uniform dispatch over (dtype, bits)
#define GACT_DISPATCH(t, CALL)                                                       \
    switch ((t).dtype() * 16 + (t).bits()) {                                             \
        case GACT_DT_F32 * 16 + 1:  { CALL(GACT_DT_F32, 1) } break;                  \
        case GACT_DT_F32 * 16 + 2:  { CALL(GACT_DT_F32, 2) } break;                  \
        case GACT_DT_F32 * 16 + 4:  { CALL(GACT_DT_F32, 4) } break;                  \
        case GACT_DT_F32 * 16 + 8:  { CALL(GACT_DT_F32, 8) } break;                  \
        case GACT_DT_BF16 * 16 + 1: { CALL(GACT_DT_BF16, 1) } break;                 \
        case GACT_DT_BF16 * 16 + 2: { CALL(GACT_DT_BF16, 2) } break;                 \
        case GACT_DT_BF16 * 16 + 4: { CALL(GACT_DT_BF16, 4) } break;                 \
        case GACT_DT_BF16 * 16 + 8: { CALL(GACT_DT_BF16, 8) } break;                 \
        default: break;                                                              \
    }

template <bool SUM>
__device__ __forceinline__ void compress_block(const TensorArgs& t, const Geometry& geo,
                                               int64_t block_in_tensor, double* __restrict__ tile_sum) {
    // sized by the launcher: geo.lds_wave_dwords per wavefront
    extern __shared__ __attribute__((aligned(16))) uint32_t lds_all[];
    const int wave = threadIdx.x >> 6;
    const int lane = threadIdx.x & 63;
    uint32_t* lds = lds_all + wave * geo.lds_wave_dwords;
    const int64_t tile = block_in_tensor * kWavesPerBlk + __builtin_amdgcn_readfirstlane(wave);
    if (tile * (int64_t)(geo.lanes_used * kPerLane) >= t.n) return;
    // a tile is "full" when all its elements exist and G is a power of two
    const bool full = geo.pow2 && (tile + 1) * (int64_t)(geo.lanes_used * kPerLane) <= t.n;
#define GACT_C_FULL(DT, BITS) compress_tile<DT, BITS, false, SUM>(t, geo, tile, lds, lane, tile_sum);
#define GACT_C_EDGE(DT, BITS) compress_tile<DT, BITS, true, SUM>(t, geo, tile, lds, lane, tile_sum);
    if (full) { GACT_DISPATCH(t, GACT_C_FULL) } else { GACT_DISPATCH(t, GACT_C_EDGE) }
#undef GACT_C_FULL
#undef GACT_C_EDGE
}

__device__ __forceinline__ void decompress_block(const TensorArgs& t, const Geometry& geo,
                                                 int64_t block_in_tensor) {
    const int wave = threadIdx.x >> 6;
    const int lane = threadIdx.x & 63;
    // full: every element of the block's span exists
    const bool full = (block_in_tensor + 1) * (int64_t)dec_block_elems(t.dtype(), t.bits()) <= t.n;
#define GACT_D_FULL(DT, BITS) \
    decompress_units<DT, BITS, false, dec_units_per_wave(DT, BITS)>(t, geo, block_in_tensor, wave, lane);
#define GACT_D_EDGE(DT, BITS) \
    decompress_units<DT, BITS, true, dec_units_per_wave(DT, BITS)>(t, geo, block_in_tensor, wave, lane);
    if (full) { GACT_DISPATCH(t, GACT_D_FULL) } else { GACT_DISPATCH(t, GACT_D_EDGE) }
#undef GACT_D_FULL
#undef GACT_D_EDGE
}

template <bool COMPRESS>
__device__ __forceinline__ void run_block(const TensorArgs& t, const Geometry& geo,
                                          int64_t block_in_tensor) {
    if (COMPRESS) compress_block<false>(t, geo, block_in_tensor, nullptr);
    else decompress_block(t, geo, block_in_tensor);
}

// Eight resident wavefronts per SIMD (at most 64 VGPRs) for every kernel: the
// bf16 compressor, which is bound by instruction issue, needs all of them.
template <bool COMPRESS>
__global__ __launch_bounds__(kBlockThreads) __attribute__((amdgpu_waves_per_eu(8, 8))) void single_kernel(TensorArgs t, Geometry geo) {
    run_block<COMPRESS>(t, geo, (int64_t)blockIdx.x);
}

// One tensor, compressed, with the sum of every tile as a by-product.
__global__ __launch_bounds__(kBlockThreads) void compress_sum_kernel(TensorArgs t, Geometry geo,
                                                                     double* __restrict__ tile_sum) {
    compress_block<true>(t, geo, (int64_t)blockIdx.x, tile_sum);
}

// Multi-tensor: block b belongs to the tensor l with first_block[l] <= b <
// first_block[l+1]; hint[] narrows the search to the tensors that overlap the
// block's bucket (see gact_device.h), usually one.
template <bool PACKED>
__device__ __forceinline__ int find_tensor(const uint32_t* first_block, const uint32_t* hint, uint32_t shift,
                                           uint32_t b) {
    const uint32_t k = b >> shift;
    int lo = PACKED ? packed_hint(hint, k) : (int)hint[k];
    int hi = (PACKED ? packed_hint(hint, k + 1) : (int)hint[k + 1]) + 1;
    // invariant: first_block[lo] <= b < first_block[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (first_block[mid] <= b) lo = mid; else hi = mid;
    }
    return lo;
}

// Table in device memory (the caller's workspace): any number of tensors.
template <bool COMPRESS>
__global__ __launch_bounds__(kBlockThreads) __attribute__((amdgpu_waves_per_eu(8, 8))) void multi_kernel(
    const TensorArgs* __restrict__ table, const uint32_t* __restrict__ first_block,
    const uint32_t* __restrict__ hint, uint32_t hint_shift, Geometry geo) {
    const uint32_t b = blockIdx.x;
    const int l = find_tensor<false>(first_block, hint, hint_shift, b);
    const TensorArgs t = table[l];
    run_block<COMPRESS>(t, geo, (int64_t)(b - first_block[l]));
}

// Table passed by value in the kernel arguments: up to kInlineTensors tensors,
// no upload and no host synchronisation before the launch.
template <bool COMPRESS>
__global__ __launch_bounds__(kBlockThreads) __attribute__((amdgpu_waves_per_eu(8, 8))) void multi_inline_kernel(
    InlineTable tab, Geometry geo) {
    const uint32_t b = blockIdx.x;
    const int l = find_tensor<true>(tab.first_block, tab.hint, tab.hint_shift, b);
    run_block<COMPRESS>(tab.t[l], geo, (int64_t)(b - tab.first_block[l]));
}

}  // namespace gact

// ------------------------------------------------------------ host launchers
extern "C" int gact_launch_single(int compress, const gact::TensorArgs* t, const gact::Geometry* geo,
                                  unsigned blocks, void* stream) {
    hipStream_t s = (hipStream_t)stream;
    const unsigned lds = compress ? 4u * gact::kWavesPerBlk * (unsigned)geo->lds_wave_dwords : 0u;
    if (compress)
        hipLaunchKernelGGL(gact::single_kernel<true>, dim3(blocks), dim3(gact::kBlockThreads), lds, s, *t, *geo);
    else
        hipLaunchKernelGGL(gact::single_kernel<false>, dim3(blocks), dim3(gact::kBlockThreads), lds, s, *t, *geo);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

extern "C" int gact_launch_compress_sum(const gact::TensorArgs* t, const gact::Geometry* geo,
                                        unsigned blocks, double* d_tile_sum, void* stream) {
    const unsigned lds = 4u * gact::kWavesPerBlk * (unsigned)geo->lds_wave_dwords;
    hipLaunchKernelGGL(gact::compress_sum_kernel, dim3(blocks), dim3(gact::kBlockThreads), lds,
                       (hipStream_t)stream, *t, *geo, d_tile_sum);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

extern "C" int gact_launch_multi_inline(int compress, const gact::InlineTable* tab,
                                        const gact::Geometry* geo, unsigned blocks, void* stream) {
    hipStream_t s = (hipStream_t)stream;
    const unsigned lds = compress ? 4u * gact::kWavesPerBlk * (unsigned)geo->lds_wave_dwords : 0u;
    if (compress)
        hipLaunchKernelGGL(gact::multi_inline_kernel<true>, dim3(blocks), dim3(gact::kBlockThreads), lds, s,
                           *tab, *geo);
    else
        hipLaunchKernelGGL(gact::multi_inline_kernel<false>, dim3(blocks), dim3(gact::kBlockThreads), lds, s,
                           *tab, *geo);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

extern "C" int gact_launch_multi(int compress, const gact::TensorArgs* d_table,
                                 const uint32_t* d_first_block, const uint32_t* d_hint,
                                 unsigned hint_shift, const gact::Geometry* geo, unsigned blocks,
                                 void* stream) {
    hipStream_t s = (hipStream_t)stream;
    const unsigned lds = compress ? 4u * gact::kWavesPerBlk * (unsigned)geo->lds_wave_dwords : 0u;
    if (compress)
        hipLaunchKernelGGL(gact::multi_kernel<true>, dim3(blocks), dim3(gact::kBlockThreads), lds, s,
                           d_table, d_first_block, d_hint, hint_shift, *geo);
    else
        hipLaunchKernelGGL(gact::multi_kernel<false>, dim3(blocks), dim3(gact::kBlockThreads), lds, s,
                           d_table, d_first_block, d_hint, hint_shift, *geo);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

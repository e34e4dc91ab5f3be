// GACT activation compressor / decompressor for MI355X (gfx950, wave64).
//
// What is computed: the per-group stochastic-rounding quantizer of
// arXiv 2206.11357 (App. A.4, applied per group as in Sec. 5) and its inverse;
// the exact arithmetic contract is stated in include/gact.h.
//
// How the work is laid out
//   * One wavefront owns one "tile": 64 lanes x 32 consecutive elements
//     (2048 elements when the group size is a power of two).  A group of G
//     elements is G/32 neighbouring lanes, so group statistics are a handful
//     of DPP steps and every lane does the two IEEE divisions of its group
//     once per 32 elements.
//   * HBM is always touched with fully coalesced 16-byte accesses (lane i of
//     load k reads bytes [k*1024 + 16 i, +16)).  The switch between that
//     layout and "32 consecutive elements per lane" goes through a private,
//     padded LDS region per wavefront (row stride 36 dwords: conflict-free
//     128-bit LDS reads and writes).
//   * With 32 elements per lane a lane owns 32*bits packed bits = `bits`
//     dwords, and neighbouring lanes own neighbouring dwords: the packed
//     stream is written (and read back) coalesced without further staging.
//   * Rounding noise: one Philox4x32-10 block per 8 consecutive elements, so
//     four blocks per lane; the stream depends on (seed, element index) only.
//   * No MFMA: the path is a streaming codec, bound by HBM (fp32 input) or by
//     plain VALU work (bf16 input), not a contraction.
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
constexpr int kRowDwords    = kPerLane + 4;       // padded LDS row of one lane
constexpr int kWaveLdsDw    = kLanes * kRowDwords;
constexpr int kWavesPerBlk  = 4;
constexpr int kBlockThreads = kLanes * kWavesPerBlk;

// ---------------------------------------------------------------- lane moves
template <int CTRL>
__device__ __forceinline__ float dpp(float v) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
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

// All lanes of a group (lpg neighbouring lanes, lpg a power of two <= 32,
// groups aligned to lpg) end up with the group's min and max.
__device__ __forceinline__ void group_minmax_pow2(float& mn, float& mx, int lpg) {
    if (lpg > 1)  { mn = fmin2(mn, dpp<0xB1>(mn));  mx = fmax2(mx, dpp<0xB1>(mx)); }   // lane^1
    if (lpg > 2)  { mn = fmin2(mn, dpp<0x4E>(mn));  mx = fmax2(mx, dpp<0x4E>(mx)); }   // lane^2
    if (lpg > 4)  { mn = fmin2(mn, dpp<0x141>(mn)); mx = fmax2(mx, dpp<0x141>(mx)); }  // 7-lane mirror
    if (lpg > 8)  { mn = fmin2(mn, dpp<0x140>(mn)); mx = fmax2(mx, dpp<0x140>(mx)); }  // 15-lane mirror
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
// Philox4x32-10 (Salmon et al., SC'11) on counter (c0, c1, 0, 0).
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t k0,
                                              uint32_t k1, uint32_t w[4]) {
    uint32_t c2 = 0u, c3 = 0u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        // three-input xor in one v_bitop3_b32 (truth table 0x96)
        const uint32_t n0 = __builtin_amdgcn_bitop3_b32((uint32_t)(p1 >> 32), c1, k0, 0x96);
        const uint32_t n2 = __builtin_amdgcn_bitop3_b32((uint32_t)(p0 >> 32), c3, k1, 0x96);
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    w[0] = c0; w[1] = c1; w[2] = c2; w[3] = c3;
}

// ------------------------------------------------------- tile <-> HBM moves
// Coalesced global -> LDS rows.  `ne` = number of valid elements of the tile
// (2048 for a full tile).  Elements past `ne` are never read from memory.
template <int DT, bool EDGE>
__device__ __forceinline__ void load_tile_to_lds(const void* __restrict__ x, int64_t e0, int ne,
                                                 float* __restrict__ lds, int lane) {
    if (DT == GACT_DT_F32) {
        const float* p = (const float*)x + e0;
        f4 v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int e = k * 256 + lane * 4;
            if (!EDGE) {
                v[k] = __builtin_nontemporal_load((const f4*)(p + e));
            } else if (e + 4 <= ne) {
                v[k] = *(const f4*)(p + e);
            } else {
                f4 t = {0.f, 0.f, 0.f, 0.f};
                if (e + 0 < ne) t.x = p[e + 0];
                if (e + 1 < ne) t.y = p[e + 1];
                if (e + 2 < ne) t.z = p[e + 2];
                v[k] = t;
            }
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int e = k * 256 + lane * 4;
            *(f4*)(lds + (e >> 5) * kRowDwords + (e & 31)) = v[k];
        }
    } else {
        const uint16_t* p = (const uint16_t*)x + e0;
        u4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int e = k * 512 + lane * 8;
            if (!EDGE) {
                v[k] = __builtin_nontemporal_load((const u4*)(p + e));
            } else if (e + 8 <= ne) {
                v[k] = *(const u4*)(p + e);
            } else {
                uint32_t h[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) h[j] = (e + j < ne) ? (uint32_t)p[e + j] : 0u;
                u4 t = {h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16),
                        h[6] | (h[7] << 16)};
                v[k] = t;
            }
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int e = k * 512 + lane * 8;
            float* row = lds + (e >> 5) * kRowDwords + (e & 31);
            f4 lo = {__builtin_bit_cast(float, v[k].x << 16),
                     __builtin_bit_cast(float, v[k].x & 0xFFFF0000u),
                     __builtin_bit_cast(float, v[k].y << 16),
                     __builtin_bit_cast(float, v[k].y & 0xFFFF0000u)};
            f4 hi = {__builtin_bit_cast(float, v[k].z << 16),
                     __builtin_bit_cast(float, v[k].z & 0xFFFF0000u),
                     __builtin_bit_cast(float, v[k].w << 16),
                     __builtin_bit_cast(float, v[k].w & 0xFFFF0000u)};
            *(f4*)(row) = lo;
            *(f4*)(row + 4) = hi;
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

// LDS rows -> coalesced global stores of the dequantised tile.
template <int DT, bool EDGE>
__device__ __forceinline__ void store_tile_from_lds(void* __restrict__ y, int64_t e0, int ne,
                                                    const float* __restrict__ lds, int lane) {
    if (DT == GACT_DT_F32) {
        float* p = (float*)y + e0;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int e = k * 256 + lane * 4;
            const f4 v = *(const f4*)(lds + (e >> 5) * kRowDwords + (e & 31));
            if (!EDGE) {
                __builtin_nontemporal_store(v, (f4*)(p + e));
            } else if (e + 4 <= ne) {
                *(f4*)(p + e) = v;
            } else {
                if (e + 0 < ne) p[e + 0] = v.x;
                if (e + 1 < ne) p[e + 1] = v.y;
                if (e + 2 < ne) p[e + 2] = v.z;
            }
        }
    } else {
        uint16_t* p = (uint16_t*)y + e0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int e = k * 512 + lane * 8;
            const float* row = lds + (e >> 5) * kRowDwords + (e & 31);
            const f4 a = *(const f4*)(row);
            const f4 b = *(const f4*)(row + 4);
            const u4 t = {bf16_pair_rne(a.x, a.y), bf16_pair_rne(a.z, a.w),
                          bf16_pair_rne(b.x, b.y), bf16_pair_rne(b.z, b.w)};
            if (!EDGE) {
                __builtin_nontemporal_store(t, (u4*)(p + e));
            } else if (e + 8 <= ne) {
                *(u4*)(p + e) = t;
            } else {
                const uint32_t h[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (e + j < ne) p[e + j] = (uint16_t)(h[j >> 1] >> (16 * (j & 1)));
            }
        }
    }
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
template <int DT, int BITS, bool EDGE>
__device__ __forceinline__ void compress_tile(const TensorArgs& t, const Geometry& geo,
                                              int64_t tile, float* __restrict__ lds, int lane) {
    constexpr uint32_t B = (1u << BITS) - 1u;
    const int tile_elems = geo.lanes_used * kPerLane;
    const int64_t e0 = tile * (int64_t)tile_elems;
    int ne = tile_elems;
    if (EDGE) {
        const int64_t left = t.n - e0;
        ne = left < (int64_t)tile_elems ? (int)left : tile_elems;
    }

    load_tile_to_lds<DT, EDGE>(t.x, e0, ne, lds, lane);
    wave_lds_sync();

    float v[kPerLane];
    {
        const float* row = lds + lane * kRowDwords;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const f4 q = *(const f4*)(row + 4 * k);
            v[4 * k + 0] = q.x; v[4 * k + 1] = q.y; v[4 * k + 2] = q.z; v[4 * k + 3] = q.w;
        }
    }

    // group statistics
    const int my0 = lane * kPerLane;                 // first element of this lane in the tile
    float mn, mx;
    if (!EDGE) {
        mn = v[0]; mx = v[0];
#pragma unroll
        for (int j = 1; j < kPerLane; ++j) { mn = fmin2(mn, v[j]); mx = fmax2(mx, v[j]); }
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

    const bool lane_live = !EDGE || my0 < ne;
    const int grp_in_tile = EDGE ? lane / geo.lpg : lane >> geo.lpg_shift;
    if (lane_live && lane == grp_in_tile * geo.lpg) {
        const int64_t g = tile * (int64_t)geo.groups_per_tile + grp_in_tile;
        t.gmin[g] = mn;
        t.gscale[g] = step;
    }

    // stochastic rounding + packing: 8 elements per Philox block.  Elements are
    // visited last to first so that each word grows by one shift-or per code.
    uint32_t out[BITS];
#pragma unroll
    for (int w = 0; w < BITS; ++w) out[w] = 0u;
    const uint64_t blk0 = (uint64_t)(e0 + my0) >> 3;
#pragma unroll
    for (int c = 3; c >= 0; --c) {
        uint32_t r[4];
        const uint64_t blk = blk0 + (uint64_t)c;
        philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), t.seed_lo, t.seed_hi, r);
#pragma unroll
        for (int j = 7; j >= 0; --j) {
            const int e = c * 8 + j;
            const uint32_t r16 = (j & 1) ? (r[j >> 1] >> 16) : (r[j >> 1] & 0xFFFFu);
            // (r16 + 1/2) / 65536, exact in binary32 either way it is written
            const float u = __builtin_fmaf((float)r16, 0x1p-16f, 0x1p-17f);
            const float d = v[e] - mn;
            const float tt = d * inv;
            const float frac = __builtin_amdgcn_fractf(tt);      // tt - floor(tt), tt >= 0
            uint32_t q = (uint32_t)(int)tt + (u < frac ? 1u : 0u);
            // tt <= B (1 + 2^-23): the fraction of an overshoot is below the
            // smallest noise value 2^-17 unless B = 255, so only 8-bit codes
            // can round past the top level
            if (BITS == 8) q = q < B ? q : B;
            if (EDGE && my0 + e >= ne) q = 0u;
            const int w = (e * BITS) >> 5;
            out[w] = (out[w] << BITS) | q;
        }
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
        const int64_t words_total = t.packed_words;
#pragma unroll
        for (int w = 0; w < BITS; ++w)
            if (lane < geo.lanes_used && word0 + w < words_total) pk[w] = out[w];
        // when a tile is narrower than 128*8/BITS elements' worth of padding
        // (group sizes that are not a power of two), up to three pad words lie
        // past the last tile's lanes: the last tile zeroes them
        if (tile == t.tiles - 1 && lane < 4) {
            const int64_t w = (e0 >> 5) * BITS + (int64_t)geo.lanes_used * BITS + lane;
            if (w < words_total) ((uint32_t*)t.packed)[w] = 0u;
        }
    }
}

// --------------------------------------------------------------- decompress
template <int DT, int BITS, bool EDGE>
__device__ __forceinline__ void decompress_tile(const TensorArgs& t, const Geometry& geo,
                                                int64_t tile, float* __restrict__ lds, int lane) {
    constexpr uint32_t B = (1u << BITS) - 1u;
    const int tile_elems = geo.lanes_used * kPerLane;
    const int64_t e0 = tile * (int64_t)tile_elems;
    int ne = tile_elems;
    if (EDGE) {
        const int64_t left = t.n - e0;
        ne = left < (int64_t)tile_elems ? (int)left : tile_elems;
    }
    const int my0 = lane * kPerLane;
    const bool lane_live = !EDGE || (lane < geo.lanes_used && my0 < ne);

    uint32_t in[BITS];
    float mn = 0.0f, step = 0.0f;
    const int64_t word0 = (e0 >> 5) * BITS + (int64_t)lane * BITS;
    const uint32_t* pk = (const uint32_t*)t.packed + word0;
#pragma unroll
    for (int w = 0; w < BITS; ++w) in[w] = 0u;
    if (lane_live) {
        if (EDGE) {
            // a live lane's words may run past the 16-byte-rounded end of the buffer
#pragma unroll
            for (int w = 0; w < BITS; ++w)
                if (word0 + w < t.packed_words) in[w] = pk[w];
        } else if (BITS == 1) {
            in[0] = __builtin_nontemporal_load(pk);
        } else if (BITS == 2) {
            const u2 o = __builtin_nontemporal_load((const u2*)pk);
            in[0] = o.x; in[1] = o.y;
        } else {
#pragma unroll
            for (int w = 0; w < BITS; w += 4) {
                const u4 o = __builtin_nontemporal_load((const u4*)(pk + w));
                in[w] = o.x; in[w + 1] = o.y; in[w + 2] = o.z; in[w + 3] = o.w;
            }
        }
        const int64_t g = tile * (int64_t)geo.groups_per_tile
                          + (EDGE ? lane / geo.lpg : lane >> geo.lpg_shift);
        mn = t.gmin[g];
        step = t.gscale[g];
    }

    float* row = lds + lane * kRowDwords;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        float o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int bit = (4 * k + j) * BITS;
            const uint32_t q = (in[bit >> 5] >> (bit & 31)) & B;
            const float prod = (float)q * step;
            o[j] = prod + mn;
        }
        f4 ov = {o[0], o[1], o[2], o[3]};
        *(f4*)(row + 4 * k) = ov;
    }
    wave_lds_sync();
    store_tile_from_lds<DT, EDGE>(t.y, e0, ne, lds, lane);
}

// ------------------------------------------------------------------ kernels
template <bool COMPRESS, bool EDGE>
__device__ __forceinline__ void run_tile(const TensorArgs& t, const Geometry& geo, int64_t tile,
                                         float* lds, int lane) {
#define GACT_CASE(DT, BITS)                                                           \
    if (COMPRESS) compress_tile<DT, BITS, EDGE>(t, geo, tile, lds, lane);             \
    else decompress_tile<DT, BITS, EDGE>(t, geo, tile, lds, lane);                    \
    break;
    switch (t.dtype * 16 + t.bits) {
        case GACT_DT_F32 * 16 + 1:  GACT_CASE(GACT_DT_F32, 1)
        case GACT_DT_F32 * 16 + 2:  GACT_CASE(GACT_DT_F32, 2)
        case GACT_DT_F32 * 16 + 4:  GACT_CASE(GACT_DT_F32, 4)
        case GACT_DT_F32 * 16 + 8:  GACT_CASE(GACT_DT_F32, 8)
        case GACT_DT_BF16 * 16 + 1: GACT_CASE(GACT_DT_BF16, 1)
        case GACT_DT_BF16 * 16 + 2: GACT_CASE(GACT_DT_BF16, 2)
        case GACT_DT_BF16 * 16 + 4: GACT_CASE(GACT_DT_BF16, 4)
        case GACT_DT_BF16 * 16 + 8: GACT_CASE(GACT_DT_BF16, 8)
        default: break;
    }
#undef GACT_CASE
}

template <bool COMPRESS>
__device__ __forceinline__ void run_block(const TensorArgs& t, const Geometry& geo,
                                          int64_t block_in_tensor) {
    __shared__ __attribute__((aligned(16))) float lds_all[kWavesPerBlk * kWaveLdsDw];
    const int wave = threadIdx.x >> 6;
    const int lane = threadIdx.x & 63;
    float* lds = lds_all + wave * kWaveLdsDw;
    const int64_t tile = block_in_tensor * kWavesPerBlk + wave;
    if (tile >= t.tiles) return;
    // a tile is "full" when all its elements exist and G is a power of two
    const bool full = geo.pow2 && (tile + 1) * (int64_t)(geo.lanes_used * kPerLane) <= t.n;
    if (full) run_tile<COMPRESS, false>(t, geo, tile, lds, lane);
    else run_tile<COMPRESS, true>(t, geo, tile, lds, lane);
}

template <bool COMPRESS>
__global__ __launch_bounds__(kBlockThreads) void single_kernel(TensorArgs t, Geometry geo) {
    run_block<COMPRESS>(t, geo, (int64_t)blockIdx.x);
}

// Multi-tensor: block b belongs to the tensor l with first_block[l] <= b <
// first_block[l+1]; the table sits in the caller's workspace.
template <bool COMPRESS>
__global__ __launch_bounds__(kBlockThreads) void multi_kernel(const TensorArgs* __restrict__ table,
                                                              const uint32_t* __restrict__ first_block,
                                                              int L, Geometry geo) {
    const uint32_t b = blockIdx.x;
    int lo = 0, hi = L;                 // invariant: first_block[lo] <= b < first_block[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (first_block[mid] <= b) lo = mid; else hi = mid;
    }
    const TensorArgs t = table[lo];
    run_block<COMPRESS>(t, geo, (int64_t)(b - first_block[lo]));
}

}  // namespace gact

// ------------------------------------------------------------ host launchers
extern "C" int gact_launch_single(int compress, const gact::TensorArgs* t, const gact::Geometry* geo,
                                  unsigned blocks, void* stream) {
    hipStream_t s = (hipStream_t)stream;
    if (compress)
        hipLaunchKernelGGL(gact::single_kernel<true>, dim3(blocks), dim3(gact::kBlockThreads), 0, s, *t, *geo);
    else
        hipLaunchKernelGGL(gact::single_kernel<false>, dim3(blocks), dim3(gact::kBlockThreads), 0, s, *t, *geo);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

extern "C" int gact_launch_multi(int compress, const gact::TensorArgs* d_table,
                                 const uint32_t* d_first_block, int L, const gact::Geometry* geo,
                                 unsigned blocks, void* stream) {
    hipStream_t s = (hipStream_t)stream;
    if (compress)
        hipLaunchKernelGGL(gact::multi_kernel<true>, dim3(blocks), dim3(gact::kBlockThreads), 0, s,
                           d_table, d_first_block, L, *geo);
    else
        hipLaunchKernelGGL(gact::multi_kernel<false>, dim3(blocks), dim3(gact::kBlockThreads), 0, s,
                           d_table, d_first_block, L, *geo);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Internal declarations shared by the HIP translation units of liblgreco.so (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/lgreco.h"

namespace lgreco {

constexpr int kTile = 32768;       // largest streaming tile in elements (256 buckets of 128); a position inside a
                                   // tile fits 15 bits (the Top-K candidate records rely on it)
constexpr int kTileMin = 8192;     // smallest: small problems get smaller tiles so that the launch still fills the chip
// Tile size: halved from kTile while there would be fewer than kTilesFill tiles (small problems
// still fill the chip), down to kTileMin.  Measured on 355 M elements: 10.8 k tiles of 32768
// took 4 % off the streaming kernels against 5.4 k of 65536; 21.7 k of 16384 cost the histogram
// pass more (one flush of 4096 bins per tile) than it gained.
constexpr int kTilesFill = 2048;
constexpr int kBucket = 128;       // quantization bucket (elements)
constexpr int kChunk = 512;        // elements one wavefront handles per step (4 buckets)
constexpr int kThreads = 256;      // workgroup size of the streaming kernels (4 wavefronts)
constexpr int kMaxQuant = 8;       // quantization candidates profiled in one pass
constexpr int kMaxTopk = 8;        // top-k candidates profiled in one pass
constexpr int kHistBins = 4096;    // coarse magnitude histogram: top 12 bits of |x|'s pattern
constexpr int kHistShift = 19;

// One tile = up to kTile consecutive elements of ONE layer, starting at a multiple of
// kBucket from the layer start, so buckets never straddle tiles or layers.
struct Tile {
    int64_t pos;      // first element, relative to the layer start
    int32_t layer;
    int32_t count;    // elements in this tile
    int32_t fast;     // 1: 16-byte aligned and count % kChunk == 0 (vector path)
    int32_t pad;
};

struct DevLayer {
    int64_t offset;       // elements, into the flat gradient buffer
    int64_t numel;
    int64_t payload;      // byte offset of the layer's payload (compress only)
    int64_t q_offset;     // element offset of the layer's warm-start block (low rank)
    int32_t rows, cols;
    int32_t tile_begin;   // first tile of this layer
    int32_t tile_end;
    int32_t family;       // compress: family of the chosen candidate
    int32_t iparam;       // compress: bits / k / rank of the chosen candidate
    int32_t slot;         // compress right behind a profile: index of the chosen density in the profile's
                          // Top-K selection records (written by the solver kernel; -1 otherwise)
    int32_t pad1;
};

// ------------------------------------------------------------------ cross-lane helpers
// DPP controls of the gfx9 family.
constexpr int kDppQuadXor1 = 0xB1;       // quad_perm:[1,0,3,2]
constexpr int kDppQuadXor2 = 0x4E;       // quad_perm:[2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141;
constexpr int kDppRowMirror = 0x140;

// 128-bit loads and stores marked as streaming (the data is used once): the caches need not keep it
typedef float f32x4_native __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_stream(const float4* p) {
    const f32x4_native v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_native*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_stream(float4* p, const float4 v) {
    f32x4_native n;
    n.x = v.x; n.y = v.y; n.z = v.z; n.w = v.w;
    __builtin_nontemporal_store(n, reinterpret_cast<f32x4_native*>(p));
}

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, false);
}

// All 16 lanes of a DPP row end up with the row's minimum / maximum / sum.
__device__ __forceinline__ float row16_min(float v) {
    v = fminf(v, dpp_f32<kDppQuadXor1>(v));
    v = fminf(v, dpp_f32<kDppQuadXor2>(v));
    v = fminf(v, dpp_f32<kDppRowHalfMirror>(v));
    v = fminf(v, dpp_f32<kDppRowMirror>(v));
    return v;
}
__device__ __forceinline__ float row16_max(float v) {
    v = fmaxf(v, dpp_f32<kDppQuadXor1>(v));
    v = fmaxf(v, dpp_f32<kDppQuadXor2>(v));
    v = fmaxf(v, dpp_f32<kDppRowHalfMirror>(v));
    v = fmaxf(v, dpp_f32<kDppRowMirror>(v));
    return v;
}
// Minimum and maximum of a DPP row together: one instruction per step and operand.  (Written as
// min / max of a moved value the compiler spends four instructions per step.)  A DPP read of a
// register needs two wait states after the write; the s_nop in front of each step provides them,
// and the last one covers a DPP read the compiler may place behind this block.
__device__ __forceinline__ void row16_minmax(float& mn, float& mx) {
    asm("s_nop 1\n\t"
        "v_min_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_min_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_min_f32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_min_f32_dpp %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 row_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1"
        : "+v"(mn), "+v"(mx));
}
// min / max of three in one instruction (inputs are results of arithmetic, so already canonical)
__device__ __forceinline__ float min3f(float a, float b, float c) {
    float r;
    asm("v_min3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
__device__ __forceinline__ float max3f(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
__device__ __forceinline__ float row16_sum(float v) {
    v += dpp_f32<kDppQuadXor1>(v);
    v += dpp_f32<kDppQuadXor2>(v);
    v += dpp_f32<kDppRowHalfMirror>(v);
    v += dpp_f32<kDppRowMirror>(v);
    return v;
}
// Value of lane (row base + LANE) for every lane of the row.
template <int LANE>
__device__ __forceinline__ float row16_bcast(float v) {
    // every lane has a source lane, so no previous value is needed (none is set up)
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x150 + LANE, 0xF, 0xF,
                                                              true));   // row_newbcast:LANE
}
// All 64 lanes end up with the wavefront's sum (fixed order -> reproducible).
__device__ __forceinline__ float wave_sum(float v) {
    v = row16_sum(v);
    v += __shfl_xor(v, 16, 64);
    v += __shfl_xor(v, 32, 64);
    return v;
}
__device__ __forceinline__ double wave_sum(double v) {
    for (int o = 1; o < 64; o <<= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_min(float v) {
    v = row16_min(v);
    v = fminf(v, __shfl_xor(v, 16, 64));
    v = fminf(v, __shfl_xor(v, 32, 64));
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
    v = row16_max(v);
    v = fmaxf(v, __shfl_xor(v, 16, 64));
    v = fmaxf(v, __shfl_xor(v, 32, 64));
    return v;
}

// ------------------------------------------------------------------ Philox4x32-10
// Counter-based generator of Salmon et al. (SC'11): ten rounds of two 32x32->64 multiplies
// and a Weyl key schedule.  Written from the published round function.
struct Philox4 {
    uint32_t w[4];
};
__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return Philox4{{c0, c1, c2, c3}};
}
__device__ __forceinline__ uint32_t philox_word(const Philox4& r, int i) {
    return i == 0 ? r.w[0] : i == 1 ? r.w[1] : i == 2 ? r.w[2] : r.w[3];
}
// 24 high bits of a word as a float in [0, 1).
__device__ __forceinline__ float u01(uint32_t w) { return (float)(w >> 8) * 0x1p-24f; }

// ------------------------------------------------------------------ launch parameters
struct QuantParams {
    const float* g;
    const float* e;            // may be null
    const DevLayer* layers;
    const Tile* tiles;
    double* partials;          // [n_tiles x stride]
    int32_t stride;            // doubles per tile in partials
    int32_t nq;                // quantization candidates
    int32_t bits[kMaxQuant];
    int32_t col[kMaxQuant];    // column of each candidate in partials
    int32_t stochastic;
    uint32_t seed_lo, seed_hi;
    // fused Top-K work (Top-K candidates in the same profile call)
    uint32_t* hist;            // [L x kHistBins] coarse magnitude histogram, or null
    const uint32_t* lo;        // [L] lowest coarse key collected as a candidate (collection mode)
    uint32_t* cand;            // candidate buffer
    uint16_t* cand_idx;        // not null: position within the tile (15 bits) and sign of every candidate, same slots
    const int64_t* cand_base;  // [L] first candidate slot of every layer
    void* tinfo;               // [n_tiles] TopkTileInfo
    double* base_part;         // [n_tiles] energy of the elements below lo
    // not null: x = fl32(g + e) is written here as it is formed, same layout as g (may be the
    // error-feedback buffer itself: every element is read once, by the lane that then writes it)
    float* x_out;
};

}  // namespace lgreco

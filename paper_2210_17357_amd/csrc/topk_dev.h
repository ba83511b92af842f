// Device-side pieces of the Top-K path shared by the stand-alone collection kernel and the
// fused quantization-profile kernel.
#pragma once

#include "common.h"

namespace lgreco {

// Per tile: what each of the 4 wavefronts wrote into the tile's slice of the candidate buffer.
// A wavefront owns a contiguous range of the tile's elements and writes its candidates from the
// slot of its own first element on, so slices never collide and no atomics are needed.
struct TopkTileInfo {
    uint32_t cnt[kThreads / 64];
    uint32_t start[kThreads / 64];     // first slot, relative to the tile's slice
};

__device__ __forceinline__ uint32_t mag_bits(float x) { return __float_as_uint(x) & 0x7FFFFFFFu; }

// Candidate collection of one wavefront.  Elements whose coarse key (top 12 bits of |x|) is at or
// above `lo` are written out in ballot-prefix order (the same order on every run); the energy of
// the others is summed per lane.
// A collection bound given as a coarse key, as the lowest magnitude pattern that qualifies (all
// ones: nothing does - patterns have the sign bit cleared).
__device__ __forceinline__ uint32_t bound_of_key(uint32_t lo) {
    return (lo >= (uint32_t)kHistBins) ? 0xFFFFFFFFu : (lo << kHistShift);
}

// Where a candidate is, in 16 bits: position inside its tile (below kTile = 2^15) and the sign.
static_assert(kTile <= (1 << 15), "a position inside a tile must fit 15 bits");
__device__ __forceinline__ uint16_t place16(uint32_t in_tile, uint32_t bits) {
    return (uint16_t)(in_tile | ((bits >> 16) & 0x8000u));
}

struct Collector {
    uint32_t* dst;
    uint32_t* dst_idx;   // optional: index (within the layer) and sign of every candidate
    uint16_t* dst_idx16; // optional: the same as place16 of (index - idx_base)
    uint32_t idx_base;   // the tile's first index within the layer
    uint32_t lo_key;   // lowest magnitude pattern collected (a multiple of a coarse key where the caller
                       // compares keys only; any pattern where it compares whole patterns)
    uint32_t cur;      // candidates written so far (uniform over the wavefront)
    float base;        // this lane's sum of x^2 over elements below the bound
    static constexpr uint32_t kKeyMask = (uint32_t)(kHistBins - 1) << kHistShift;
    __device__ __forceinline__ void init(uint32_t* d, uint32_t* di, uint32_t bound, uint16_t* di16 = nullptr,
                                         uint32_t tile_first = 0) {
        dst = d; dst_idx = di; dst_idx16 = di16; idx_base = tile_first; cur = 0; base = 0.0f;
        lo_key = bound;
    }
    __device__ __forceinline__ static uint32_t below(unsigned long long m, uint32_t add) {
        return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, add));
    }
    // one element per lane
    __device__ __forceinline__ void take(float x, bool valid, uint32_t idx = 0) {
        take_keyed(x, mag_bits(x), valid, idx);
    }
    // the same with the value compared against the bound supplied by the caller: the magnitude
    // pattern, or just its coarse key (pattern & kKeyMask) when the bound is a coarse key
    __device__ __forceinline__ void take_keyed(float x, uint32_t key, bool valid, uint32_t idx = 0) {
        const uint32_t bits = __float_as_uint(x);
        const bool hit = valid && key >= lo_key;
        const unsigned long long m = __ballot(hit);
        const float low = (hit || !valid) ? 0.0f : x;     // the energy below lo, without a branch
        base = __builtin_fmaf(low, low, base);
        if (hit) {
            // byte offset in 32 bits (a slice holds fewer than 2^30 entries): uniform base + lane offset
            const uint32_t off = (below(m, 0u) + cur) << 2;
            *reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(dst) + off) = bits & 0x7FFFFFFFu;
            if (dst_idx)
                *reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(dst_idx) + off) = idx | (bits & 0x80000000u);
            if (dst_idx16) dst_idx16[off >> 2] = place16(idx - idx_base, bits);
        }
        cur += (uint32_t)__popcll(m);
    }
    // four consecutive elements per lane, lanes in element order: candidates come out in element order
    __device__ __forceinline__ void take4(const float (&x)[4], uint32_t idx0) {
        bool hit[4];
        uint32_t pat[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            pat[q] = mag_bits(x[q]);
            hit[q] = pat[q] >= lo_key;
        }
        const unsigned long long m0 = __ballot(hit[0]), m1 = __ballot(hit[1]), m2 = __ballot(hit[2]),
                                 m3 = __ballot(hit[3]);
        uint32_t at = cur + below(m0, below(m1, below(m2, below(m3, 0u))));
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (hit[q]) {
                dst[at] = pat[q];
                if (dst_idx) dst_idx[at] = (idx0 + q) | (__float_as_uint(x[q]) & 0x80000000u);
                if (dst_idx16) dst_idx16[at] = place16(idx0 + q - idx_base, __float_as_uint(x[q]));
                ++at;
            } else {
                base = __builtin_fmaf(x[q], x[q], base);
            }
        }
        cur += (uint32_t)(__popcll(m0) + __popcll(m1) + __popcll(m2) + __popcll(m3));
    }
};

// The same collection with the candidates staged in LDS: a wavefront appends to its own buffer of
// kStageWords words and writes 128 candidates at a time, as two full 256-byte stores, instead of a
// few scattered words per element slot.  Order and content of the slice are those of Collector.
// IDX: where every candidate is (place16) goes the same way through a second buffer of kStageWords
// 16-bit entries right behind the first, into dst_idx.
constexpr int kStageFlush = 128;
constexpr int kStageWords = kStageFlush + 64;     // below kStageFlush before an append of at most 64
template <bool IDX>
struct StagedCollector {
    static constexpr int kWordsPerWave = IDX ? kStageWords + kStageWords / 2 : kStageWords;
    uint32_t* dst;       // the wavefront's slice in global memory
    uint16_t* dst_idx;   // IDX: the same slice of the place buffer
    uint32_t* stage;     // the wavefront's kWordsPerWave words of LDS
    uint16_t* stage16;   // IDX: its second part
    uint32_t lo_key;
    uint32_t cur;        // candidates written to global memory so far (uniform over the wavefront)
    uint32_t fill;       // candidates waiting in the buffer (uniform)
    float base;          // this lane's sum of x^2 over elements below the bound
    __device__ __forceinline__ void init(uint32_t* d, uint16_t* di, uint32_t* st, uint32_t bound) {
        dst = d; dst_idx = di; stage = st; stage16 = reinterpret_cast<uint16_t*>(st + kStageWords);
        cur = 0; fill = 0; base = 0.0f;
        lo_key = bound;
    }
    // in_tile: the element's position inside its tile (IDX only)
    __device__ __forceinline__ void take_keyed(float x, uint32_t key, bool valid, uint32_t in_tile = 0) {
        const uint32_t bits = __float_as_uint(x);
        const bool hit = valid && key >= lo_key;
        const unsigned long long m = __ballot(hit);
        const float low = (hit || !valid) ? 0.0f : x;
        base = __builtin_fmaf(low, low, base);
        if (hit) {
            const uint32_t at = fill + Collector::below(m, 0u);
            stage[at] = bits & 0x7FFFFFFFu;
            if (IDX) stage16[at] = place16(in_tile, bits);
        }
        fill += (uint32_t)__popcll(m);
        if (fill >= (uint32_t)kStageFlush) {          // uniform
            const uint32_t lane = threadIdx.x & 63u;
            const uint32_t rem = fill - kStageFlush;  // < 64
            const uint32_t v0 = stage[lane], v1 = stage[64 + lane];
            const uint32_t v2 = stage[kStageFlush + lane];
            dst[cur + lane] = v0;
            dst[cur + 64 + lane] = v1;
            if (IDX) {
                const uint16_t i0 = stage16[lane], i1 = stage16[64 + lane];
                const uint16_t i2 = stage16[kStageFlush + lane];
                dst_idx[cur + lane] = i0;
                dst_idx[cur + 64 + lane] = i1;
                if (lane < rem) stage16[lane] = i2;
            }
            if (lane < rem) stage[lane] = v2;         // what is left moves to the front
            cur += kStageFlush;
            fill = rem;
        }
    }
    __device__ __forceinline__ void take(float x, bool valid, uint32_t in_tile = 0) {
        take_keyed(x, __float_as_uint(x) & Collector::kKeyMask, valid, in_tile);
    }
    // writes out what is left; afterwards cur is the wavefront's candidate count
    __device__ __forceinline__ void finish() {
        const uint32_t lane = threadIdx.x & 63u;
        for (uint32_t i = lane; i < fill; i += 64) {
            dst[cur + i] = stage[i];
            if (IDX) dst_idx[cur + i] = stage16[i];
        }
        cur += fill;
        fill = 0;
    }
};

// Contiguous share of `n` work items for wavefront `wave` of 4: [begin, end)
__device__ __forceinline__ void wave_range(int n, int wave, int* begin, int* end) {
    const int q = (n + kThreads / 64 - 1) / (kThreads / 64);
    *begin = min(n, wave * q);
    *end = min(n, (wave + 1) * q);
}

}  // namespace lgreco

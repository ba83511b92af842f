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
struct Collector {
    uint32_t* dst;
    uint32_t* dst_idx;   // optional: index (within the layer) and sign of every candidate
    uint32_t lo;
    uint32_t lo_key;   // lo moved to the key's place in the pattern (all ones: nothing qualifies)
    uint32_t cur;      // candidates written so far (uniform over the wavefront)
    float base;        // this lane's sum of x^2 over elements below lo
    static constexpr uint32_t kKeyMask = (uint32_t)(kHistBins - 1) << kHistShift;
    __device__ __forceinline__ void init(uint32_t* d, uint32_t* di, uint32_t l) {
        dst = d; dst_idx = di; lo = l; cur = 0; base = 0.0f;
        lo_key = (l >= (uint32_t)kHistBins) ? 0xFFFFFFFFu : (l << kHistShift);
    }
    __device__ __forceinline__ static uint32_t below(unsigned long long m, uint32_t add) {
        return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, add));
    }
    // one element per lane
    __device__ __forceinline__ void take(float x, bool valid, uint32_t idx = 0) {
        take_keyed(x, __float_as_uint(x) & kKeyMask, valid, idx);
    }
    // the same with the coarse key (pattern & kKeyMask) supplied by the caller
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
            hit[q] = (pat[q] >> kHistShift) >= lo;
        }
        const unsigned long long m0 = __ballot(hit[0]), m1 = __ballot(hit[1]), m2 = __ballot(hit[2]),
                                 m3 = __ballot(hit[3]);
        uint32_t at = cur + below(m0, below(m1, below(m2, below(m3, 0u))));
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (hit[q]) {
                dst[at] = pat[q];
                if (dst_idx) dst_idx[at] = (idx0 + q) | (__float_as_uint(x[q]) & 0x80000000u);
                ++at;
            } else {
                base = __builtin_fmaf(x[q], x[q], base);
            }
        }
        cur += (uint32_t)(__popcll(m0) + __popcll(m1) + __popcll(m2) + __popcll(m3));
    }
};

// Contiguous share of `n` work items for wavefront `wave` of 4: [begin, end)
__device__ __forceinline__ void wave_range(int n, int wave, int* begin, int* end) {
    const int q = (n + kThreads / 64 - 1) / (kThreads / 64);
    *begin = min(n, wave * q);
    *end = min(n, (wave + 1) * q);
}

}  // namespace lgreco

// Bucketed min-max quantization: fused all-bit-widths error profile, and the compressor
// (codes, bit packing, per-bucket meta, error-feedback update).  gfx950 / wave64.
//
// Arithmetic per bucket of 128 elements, all fp32, one rounding per step (the build disables
// floating-point contraction; fused multiply-adds are written explicitly):
//   x = g + e;  m = min, M = max;  r = M - m;  lv = 2^b - 1
//   unit = r / lv;  inv = lv / r, replaced by 0 when not finite
//   q = floor(fma(x - m, inv, 0.5)) or floor(fma(x - m, inv, u));  q = min(max(q, 0), lv)
//     (the clamp is a no-op except for the upper bound under stochastic rounding)
//   xhat = fma(q, unit, m);  error += (xhat - x)^2
//
// Data layout of the fast path: one wavefront handles 4 consecutive buckets per step; DPP
// row r (16 lanes) owns bucket r, lane j of the row holds elements 4j..4j+3 and 64+4j..64+4j+3
// of it (two 128-bit loads per input array, each covering two whole 128-byte lines per row).
// Bucket min / max are DPP reductions inside the row; the 2 x nq divisions of a bucket are
// spread over the row's 16 lanes (lane c: unit of candidate c, lane 8+c: inv of candidate c)
// and broadcast back with row_newbcast.
#include "internal.h"
#include "reduce_dev.h"
#include "topk_dev.h"

namespace lgreco {

__device__ __forceinline__ float safe_inv(float lv, float r) {
    const float inv = lv / r;
    return (__builtin_fabsf(inv) <= 3.402823466e38f) ? inv : 0.0f;   // inf or nan -> 0
}

// One candidate, one element (xm = x - m): returns xhat; q (as float) through *qout.
template <bool STOCH>
__device__ __forceinline__ float quant_one(float xm, float m, float inv, float unit, float lv, float u,
                                           float* qout) {
    float q = __builtin_floorf(__builtin_fmaf(xm, inv, STOCH ? u : 0.5f));
    // (x - m) * inv >= 0 always, so the lower clamp never acts.  The upper clamp can act only with
    // stochastic rounding: (x - m) * inv <= lv * (1 + 2^-23), so floor(. + 0.5) <= lv, whereas
    // adding u < 1 may round up to lv + 1.
    if (STOCH) q = fminf(q, lv);
    *qout = q;
    return __builtin_fmaf(q, unit, m);
}

// HIST: also build the coarse magnitude histogram of the Top-K path and collect its candidates
// (elements whose coarse key is at or above the layer's predicted bound) in the same read.
// IDX (with HIST): the candidates' indices and signs are recorded too (p.cand_idx), for a compression
// that works from the candidates alone.
template <bool STOCH, bool HAS_EF, bool HIST, bool IDX = false>
__global__ __launch_bounds__(kThreads) void quant_profile_kernel(QuantParams p) {
    static_assert(HIST || !IDX, "indices are recorded with the candidates");
    __shared__ double s_part[kThreads / 64][kMaxQuant + 1];
    __shared__ uint32_t s_hist[HIST ? kHistBins : 1];

    const Tile t = p.tiles[blockIdx.x];
    const DevLayer L = p.layers[t.layer];
    const float* __restrict__ g = p.g + L.offset + t.pos;
    const float* e = HAS_EF ? p.e + L.offset + t.pos : nullptr;           // may be what xo points to
    float* const xo = p.x_out ? p.x_out + L.offset + t.pos : nullptr;
    // the wavefront's number through a scalar register: its share of the tile, the loop over it and
    // the candidate slice's address are then uniform values
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int nq = p.nq;

    if (HIST) {
        for (int b = threadIdx.x; b < kHistBins; b += kThreads) s_hist[b] = 0;
        __syncthreads();
    }

    float acc[kMaxQuant];
#pragma unroll
    for (int c = 0; c < kMaxQuant; ++c) acc[c] = 0.0f;

    __shared__ uint32_t s_stage[HIST ? kThreads / 64 : 1][HIST ? StagedCollector<IDX>::kWordsPerWave : 1];
    StagedCollector<IDX> col;
    uint32_t col_start = 0;
    uint32_t* const slice = HIST ? p.cand + p.cand_base[t.layer] + t.pos : nullptr;
    uint16_t* const slice_idx = IDX ? p.cand_idx + p.cand_base[t.layer] + t.pos : nullptr;
    const uint32_t col_lo = HIST ? bound_of_key(p.lo[t.layer]) : 0xFFFFFFFFu;

    if (t.fast) {
        // division owned by this lane: candidate (lane & 7), unit for lanes 0-7, inv for 8-15
        const int j = lane & 15;
        const int myc = j & 7;
        const float mylv = (myc < nq) ? (float)((1 << p.bits[myc]) - 1) : 1.0f;
        const bool want_inv = (j >> 3) != 0;
        // each wavefront owns a contiguous range of the tile's 512-element chunks
        int c_begin, c_end;
        wave_range(t.count / kChunk, wave, &c_begin, &c_end);
        if (HIST) {
            col_start = (uint32_t)c_begin * kChunk;
            col.init(slice + col_start, IDX ? slice_idx + col_start : nullptr, s_stage[wave], col_lo);
        }
        // One chunk: 8 elements per lane (a: elements 4j..4j+3 of the lane's bucket, b: 64+4j..).
        auto chunk = [&](float4 a, float4 b, const float4 ea, const float4 eb, const int base)
            __attribute__((always_inline)) {
            if (HAS_EF) {
                a.x += ea.x; a.y += ea.y; a.z += ea.z; a.w += ea.w;
                b.x += eb.x; b.y += eb.y; b.z += eb.z; b.w += eb.w;
            }
            if (xo) {                                   // uniform
                store_stream(reinterpret_cast<float4*>(xo + base), a);
                store_stream(reinterpret_cast<float4*>(xo + base + 64), b);
            }
            float x[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
            if (HIST) {
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    // the masked pattern serves the comparison and, shifted, is the bin's byte offset
                    uint32_t key = __float_as_uint(x[k]) & Collector::kKeyMask;
                    asm("" : "+v"(key));
                    atomicAdd(reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(s_hist) + (key >> (kHistShift - 2))),
                              1u);
                    col.take_keyed(x[k], key, true, (uint32_t)(base + (k < 4 ? k : 60 + k)));
                }
            }
            float mn = fminf(min3f(min3f(min3f(x[0], x[1], x[2]), x[3], x[4]), x[5], x[6]), x[7]);
            float mx = fmaxf(max3f(max3f(max3f(x[0], x[1], x[2]), x[3], x[4]), x[5], x[6]), x[7]);
            row16_minmax(mn, mx);
            const float r = mx - mn;
            // one division per lane: r / lv (unit) or lv / r (inv, replaced by 0 when not finite)
            float dv = (want_inv ? mylv : r) / (want_inv ? r : mylv);
            if (want_inv && !(__builtin_fabsf(dv) <= 3.402823466e38f)) dv = 0.0f;

            float u[8];
            if (STOCH) {
                const uint64_t i0 = (uint64_t)(t.pos + base) >> 2;
                const Philox4 ra = philox4x32_10((uint32_t)i0, (uint32_t)(i0 >> 32), (uint32_t)t.layer, 0u,
                                                 p.seed_lo, p.seed_hi);
                const uint64_t i1 = i0 + 16;
                const Philox4 rb = philox4x32_10((uint32_t)i1, (uint32_t)(i1 >> 32), (uint32_t)t.layer, 0u,
                                                 p.seed_lo, p.seed_hi);
#pragma unroll
                for (int k = 0; k < 4; ++k) { u[k] = u01(ra.w[k]); u[4 + k] = u01(rb.w[k]); }
            }
            float xm[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) xm[k] = x[k] - mn;

#define LGRECO_CAND(C)                                                                  \
            if (C < nq) {                                                               \
                const float unit = row16_bcast<C>(dv);                                  \
                const float inv = row16_bcast<8 + C>(dv);                               \
                const float lv = (float)((1 << p.bits[C]) - 1);                         \
                float s = acc[C];                                                       \
                _Pragma("unroll") for (int k = 0; k < 8; ++k) {                         \
                    float q;                                                            \
                    const float xh = quant_one<STOCH>(xm[k], mn, inv, unit, lv,         \
                                                      STOCH ? u[k] : 0.0f, &q);         \
                    const float d = xh - x[k];                                          \
                    s = __builtin_fmaf(d, d, s);                                        \
                }                                                                       \
                acc[C] = s;                                                             \
            }
            LGRECO_CAND(0) LGRECO_CAND(1) LGRECO_CAND(2) LGRECO_CAND(3)
            LGRECO_CAND(4) LGRECO_CAND(5) LGRECO_CAND(6) LGRECO_CAND(7)
#undef LGRECO_CAND
        };
        // Two register sets take turns: while one chunk is worked on, the loads of the next are in
        // flight.  Nothing is loaded past the range's end (streaming loads of a chunk that was
        // already read would go to memory again).
        const int lane_off = (lane >> 4) * kBucket + j * 4;
        const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
        auto load = [&](const int c, float4& a, float4& b, float4& ea, float4& eb)
            __attribute__((always_inline)) {
            if (c >= c_end) return;                     // uniform over the wavefront
            const int base = c * kChunk + lane_off;
            a = load_stream(reinterpret_cast<const float4*>(g + base));
            b = load_stream(reinterpret_cast<const float4*>(g + base + 64));
            ea = HAS_EF ? load_stream(reinterpret_cast<const float4*>(e + base)) : zero4;
            eb = HAS_EF ? load_stream(reinterpret_cast<const float4*>(e + base + 64)) : zero4;
        };
        if (c_begin < c_end) {
            float4 a0, b0, ea0, eb0, a1, b1, ea1, eb1;
            load(c_begin, a0, b0, ea0, eb0);
            for (int c = c_begin; c < c_end; c += 2) {
                load(c + 1, a1, b1, ea1, eb1);
                chunk(a0, b0, ea0, eb0, c * kChunk + lane_off);
                if (c + 1 >= c_end) break;
                load(c + 2, a0, b0, ea0, eb0);
                chunk(a1, b1, ea1, eb1, (c + 1) * kChunk + lane_off);
            }
        }
    } else {
        // Slow path (tail of a layer, or a layer that is not 16-byte aligned): one wavefront per
        // bucket, two elements per lane, out-of-range lanes masked.
        const int nb = (t.count + kBucket - 1) / kBucket;
        int b_begin, b_end;
        wave_range(nb, wave, &b_begin, &b_end);
        if (HIST) {
            col_start = (uint32_t)b_begin * kBucket;
            col.init(slice + col_start, IDX ? slice_idx + col_start : nullptr, s_stage[wave], col_lo);
        }
        for (int bk = b_begin; bk < b_end; ++bk) {
            float x[2];
            bool ok[2];
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int idx = bk * kBucket + lane + 64 * k;
                ok[k] = idx < t.count;
                x[k] = 0.0f;
                if (ok[k]) x[k] = HAS_EF ? g[idx] + e[idx] : g[idx];
                if (ok[k] && xo) xo[idx] = x[k];
                if (HIST) {
                    if (ok[k]) atomicAdd(&s_hist[mag_bits(x[k]) >> kHistShift], 1u);
                    col.take(x[k], ok[k], (uint32_t)idx);
                }
            }
            const float inf = __builtin_huge_valf();
            const float mn = wave_min(fminf(ok[0] ? x[0] : inf, ok[1] ? x[1] : inf));
            const float mx = wave_max(fmaxf(ok[0] ? x[0] : -inf, ok[1] ? x[1] : -inf));
            const float r = mx - mn;
            float u[2] = {0.0f, 0.0f};
            if (STOCH) {
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    const uint64_t i = (uint64_t)(t.pos + bk * kBucket + lane + 64 * k);
                    const Philox4 rr = philox4x32_10((uint32_t)(i >> 2), (uint32_t)(i >> 34),
                                                     (uint32_t)t.layer, 0u, p.seed_lo, p.seed_hi);
                    u[k] = u01(philox_word(rr, (int)(i & 3)));
                }
            }
#pragma unroll
            for (int c = 0; c < kMaxQuant; ++c) {
                if (c < nq) {
                    const float lv = (float)((1 << p.bits[c]) - 1);
                    const float unit = r / lv;
                    const float inv = safe_inv(lv, r);
#pragma unroll
                    for (int k = 0; k < 2; ++k) {
                        float q;
                        const float xh = quant_one<STOCH>(x[k] - mn, mn, inv, unit, lv, u[k], &q);
                        const float d = xh - x[k];
                        if (ok[k]) acc[c] = __builtin_fmaf(d, d, acc[c]);
                    }
                }
            }
        }
    }

    // tile partials: fp32 inside the wavefront (fixed DPP order), fp64 across wavefronts
#pragma unroll
    for (int c = 0; c < kMaxQuant; ++c) {
        if (c < nq) {
            const float s = wave_sum(acc[c]);
            if (lane == 0) s_part[wave][c] = (double)s;
        }
    }
    __syncthreads();
    if ((int)threadIdx.x < nq) {
        double s = 0.0;
        for (int w = 0; w < kThreads / 64; ++w) s += s_part[w][threadIdx.x];
        p.partials[(size_t)blockIdx.x * p.stride + p.col[threadIdx.x]] = s;
    }
    if (HIST) {
        col.finish();
        const double bs = wave_sum((double)col.base);
        TopkTileInfo* const ti = reinterpret_cast<TopkTileInfo*>(p.tinfo) + blockIdx.x;
        if (lane == 0) {
            s_part[wave][kMaxQuant] = bs;
            ti->cnt[wave] = col.cur;
            ti->start[wave] = col_start;
        }
        __syncthreads();
        if (threadIdx.x == 0)
            p.base_part[blockIdx.x] = (s_part[0][kMaxQuant] + s_part[1][kMaxQuant]) +
                                      (s_part[2][kMaxQuant] + s_part[3][kMaxQuant]);
        uint32_t* gh = p.hist + (size_t)t.layer * kHistBins;
        for (int b = threadIdx.x; b < kHistBins; b += kThreads) {
            const uint32_t c = s_hist[b];
            if (c) atomicAdd(&gh[b], c);
        }
    }
}

__global__ __launch_bounds__(256) void reduce_partials_kernel(const double* __restrict__ partials,
                                                               int stride, ReduceCols cols,
                                                               const DevLayer* __restrict__ layers,
                                                               double* __restrict__ errors) {
    __shared__ double s[kMaxQuant][256];
    reduce_partials_block(partials, stride, cols, layers, errors, (int)blockIdx.x, s);
}

// ------------------------------------------------------------------------- compressor
struct QuantCompressParams {
    const float* g;
    float* e;                  // in: error feedback, out: x - xhat
    const DevLayer* layers;
    const Tile* tiles;
    uint8_t* payload;
    uint32_t seed_lo, seed_hi;
};

template <bool STOCH>
__global__ __launch_bounds__(kThreads) void quant_compress_kernel(QuantCompressParams p) {
    __shared__ uint32_t s_codes[kThreads / 64][4 * 16 * 8 / 4];   // 4 buckets x (16*8 bytes) per wave

    const Tile t = p.tiles[blockIdx.x];
    const DevLayer L = p.layers[t.layer];
    if (L.family != LGRECO_QUANT) return;
    const int bits = L.iparam;
    const float lv = (float)((1 << bits) - 1);
    // g null: the buffer e already holds x = fl32(g + e) (the profile of the same call left it there)
    const bool x_in_e = p.g == nullptr;
    const float* __restrict__ g = x_in_e ? nullptr : p.g + L.offset + t.pos;
    float* __restrict__ e = p.e + L.offset + t.pos;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t nb_layer = (L.numel + kBucket - 1) / kBucket;
    uint8_t* const lp = p.payload + L.payload;
    float2* const meta = reinterpret_cast<float2*>(lp);
    uint8_t* const codes = lp + 8 * nb_layer;
    const int64_t bucket0 = t.pos / kBucket;                      // first bucket of this tile

    if (t.fast) {
        const int j = lane & 15, row = lane >> 4;
        uint8_t* const sc = reinterpret_cast<uint8_t*>(s_codes[wave]);
        int c_begin, c_end;
        wave_range(t.count / kChunk, wave, &c_begin, &c_end);
        for (int c = c_begin; c < c_end; ++c) {
            const int base = c * kChunk + row * kBucket + j * 4;
            float4 a = load_stream(reinterpret_cast<const float4*>(e + base));
            float4 b = load_stream(reinterpret_cast<const float4*>(e + base + 64));
            if (!x_in_e) {                              // uniform
                const float4 ga = load_stream(reinterpret_cast<const float4*>(g + base));
                const float4 gb = load_stream(reinterpret_cast<const float4*>(g + base + 64));
                a.x = ga.x + a.x; a.y = ga.y + a.y; a.z = ga.z + a.z; a.w = ga.w + a.w;
                b.x = gb.x + b.x; b.y = gb.y + b.y; b.z = gb.z + b.z; b.w = gb.w + b.w;
            }
            float x[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
            float mn = fminf(fminf(fminf(x[0], x[1]), fminf(x[2], x[3])),
                             fminf(fminf(x[4], x[5]), fminf(x[6], x[7])));
            float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])),
                             fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
            mn = row16_min(mn);
            mx = row16_max(mx);
            const float r = mx - mn;
            const float unit = r / lv;
            const float inv = safe_inv(lv, r);
            float u[8];
            if (STOCH) {
                const uint64_t i0 = (uint64_t)(t.pos + base) >> 2;
                const Philox4 ra = philox4x32_10((uint32_t)i0, (uint32_t)(i0 >> 32), (uint32_t)t.layer, 0u,
                                                 p.seed_lo, p.seed_hi);
                const uint64_t i1 = i0 + 16;
                const Philox4 rb = philox4x32_10((uint32_t)i1, (uint32_t)(i1 >> 32), (uint32_t)t.layer, 0u,
                                                 p.seed_lo, p.seed_hi);
#pragma unroll
                for (int k = 0; k < 4; ++k) { u[k] = u01(ra.w[k]); u[4 + k] = u01(rb.w[k]); }
            }
            uint32_t wa = 0, wb = 0;
            float ne[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                float q;
                const float xh = quant_one<STOCH>(x[k] - mn, mn, inv, unit, lv, STOCH ? u[k] : 0.0f, &q);
                ne[k] = x[k] - xh;
                const uint32_t qi = (uint32_t)q;
                if (k < 4) wa |= qi << (bits * k);
                else wb |= qi << (bits * (k - 4));
            }
            store_stream(reinterpret_cast<float4*>(e + base), make_float4(ne[0], ne[1], ne[2], ne[3]));
            store_stream(reinterpret_cast<float4*>(e + base + 64), make_float4(ne[4], ne[5], ne[6], ne[7]));
            const int64_t bk = bucket0 + (int64_t)c * 4 + row;
            if (j == 0) meta[bk] = make_float2(mn, unit);

            // 8 consecutive elements = `bits` whole bytes.  Even lanes assemble elements
            // 4j..4j+7 of the first half, odd lanes elements 64+4(j-1)..64+4(j-1)+7.
            const uint32_t pa = dpp_u32<kDppQuadXor1>(wa);
            const uint32_t pb = dpp_u32<kDppQuadXor1>(wb);
            const bool odd = (j & 1) != 0;
            const uint64_t w64 = odd ? ((uint64_t)pb | ((uint64_t)wb << (4 * bits)))
                                     : ((uint64_t)wa | ((uint64_t)pa << (4 * bits)));
            const int off = row * 16 * bits + (odd ? 8 * bits : 0) + (j >> 1) * bits;
            for (int i = 0; i < bits; ++i) sc[off + i] = (uint8_t)(w64 >> (8 * i));
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            // the wavefront's 4 buckets are contiguous in the stream: 16*bits dwords
            uint32_t* const dst = reinterpret_cast<uint32_t*>(codes + (bucket0 + (int64_t)c * 4) * 16 * bits);
            for (int d = lane; d < 16 * bits; d += 64) dst[d] = s_codes[wave][d];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    } else {
        uint32_t* const sw = s_codes[wave];
        const int nb = (t.count + kBucket - 1) / kBucket;
        int b_begin, b_end;
        wave_range(nb, wave, &b_begin, &b_end);
        for (int bk = b_begin; bk < b_end; ++bk) {
            const int cnt = min(kBucket, t.count - bk * kBucket);
            for (int d = lane; d < 32; d += 64) sw[d] = 0;          // 128 elements x 8 bits max
            float x[2];
            bool ok[2];
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int idx = bk * kBucket + lane + 64 * k;
                ok[k] = lane + 64 * k < cnt;
                x[k] = ok[k] ? (x_in_e ? e[idx] : g[idx] + e[idx]) : 0.0f;
            }
            const float inf = __builtin_huge_valf();
            const float mn = wave_min(fminf(ok[0] ? x[0] : inf, ok[1] ? x[1] : inf));
            const float mx = wave_max(fmaxf(ok[0] ? x[0] : -inf, ok[1] ? x[1] : -inf));
            const float r = mx - mn;
            const float unit = r / lv;
            const float inv = safe_inv(lv, r);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                if (!ok[k]) continue;
                const int i = lane + 64 * k;
                float u = 0.0f;
                if (STOCH) {
                    const uint64_t gi = (uint64_t)(t.pos + bk * kBucket + i);
                    const Philox4 rr = philox4x32_10((uint32_t)(gi >> 2), (uint32_t)(gi >> 34),
                                                     (uint32_t)t.layer, 0u, p.seed_lo, p.seed_hi);
                    u = u01(philox_word(rr, (int)(gi & 3)));
                }
                float q;
                const float xh = quant_one<STOCH>(x[k] - mn, mn, inv, unit, lv, u, &q);
                e[bk * kBucket + i] = x[k] - xh;
                const uint32_t qi = (uint32_t)q;
                const int bit = i * bits;
                atomicOr(&sw[bit >> 5], qi << (bit & 31));
                if ((bit & 31) + bits > 32) atomicOr(&sw[(bit >> 5) + 1], qi >> (32 - (bit & 31)));
            }
            if (lane == 0) meta[bucket0 + bk] = make_float2(mn, unit);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            uint8_t* const dst = codes + (bucket0 + bk) * 16 * bits;
            const uint8_t* const sb = reinterpret_cast<const uint8_t*>(sw);
            const int nbytes = (cnt * bits + 7) / 8;
            for (int d = lane; d < nbytes; d += 64) dst[d] = sb[d];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    }
}

// ------------------------------------------------------------------------- launchers
hipError_t launch_quant_profile(const QuantParams& p, int n_tiles, bool hist, hipStream_t s, Section* sec) {
    if (n_tiles <= 0) return hipSuccess;
    const dim3 grid(n_tiles), block(kThreads);
    const bool st = p.stochastic != 0, ef = p.e != nullptr;
#define LGRECO_LAUNCH(S, E, H) \
    launch_timed(sec, true, true, quant_profile_kernel<S, E, H>, grid, block, 0, s, p)
    if (p.cand_idx) {
        // recorded only by the variant the one call over both families uses
        if (!hist || !ef) return hipErrorInvalidValue;
        if (st) launch_timed(sec, true, true, quant_profile_kernel<true, true, true, true>, grid, block, 0, s, p);
        else launch_timed(sec, true, true, quant_profile_kernel<false, true, true, true>, grid, block, 0, s, p);
        return hipGetLastError();
    }
    if (st) {
        if (ef) { if (hist) LGRECO_LAUNCH(true, true, true); else LGRECO_LAUNCH(true, true, false); }
        else    { if (hist) LGRECO_LAUNCH(true, false, true); else LGRECO_LAUNCH(true, false, false); }
    } else {
        if (ef) { if (hist) LGRECO_LAUNCH(false, true, true); else LGRECO_LAUNCH(false, true, false); }
        else    { if (hist) LGRECO_LAUNCH(false, false, true); else LGRECO_LAUNCH(false, false, false); }
    }
#undef LGRECO_LAUNCH
    return hipGetLastError();
}

hipError_t launch_reduce_partials(const double* partials, int stride, const int* cols, int ncols,
                                  const DevLayer* layers, int n_layers, double* errors, hipStream_t s) {
    if (n_layers <= 0 || ncols <= 0) return hipSuccess;
    ReduceCols rc{};
    rc.n = ncols < kMaxQuant ? ncols : kMaxQuant;
    for (int i = 0; i < rc.n; ++i) rc.col[i] = cols[i];
    hipLaunchKernelGGL(reduce_partials_kernel, dim3(n_layers), dim3(256), 0, s, partials, stride, rc,
                       layers, errors);
    return hipGetLastError();
}

hipError_t launch_quant_compress(const float* g, float* e, const DevLayer* layers, const Tile* tiles,
                                 int n_tiles, uint8_t* payload, bool stochastic, uint64_t seed,
                                 hipStream_t s, Section* sec, size_t lds_pad) {
    if (n_tiles <= 0) return hipSuccess;
    QuantCompressParams p{g, e, layers, tiles, payload, (uint32_t)seed, (uint32_t)(seed >> 32)};
    if (stochastic)
        launch_timed(sec, true, true, quant_compress_kernel<true>, dim3(n_tiles), dim3(kThreads), lds_pad, s, p);
    else
        launch_timed(sec, true, true, quant_compress_kernel<false>, dim3(n_tiles), dim3(kThreads), lds_pad, s, p);
    return hipGetLastError();
}

}  // namespace lgreco

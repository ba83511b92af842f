// Layer-wise Top-K: radix-histogram threshold search, dropped-energy profile for several
// densities at once, and threshold-select compaction.  gfx950 / wave64.
//
// Magnitudes are compared as the fp32 bit pattern with the sign cleared (31 bits); the "coarse
// key" of an element is the top 12 bits (exponent + 4 mantissa bits).  Per call:
//   1. sample: coarse histogram of 1/16 of the data (one 512-element chunk out of 16).  From it a
//      cautious lower bound `lo` of the coarse key of the k-th largest magnitude is predicted for
//      every layer (the largest k asked for, with a wide margin).
//   2. main pass, ONE read of the data (fused into the quantization profile kernel when both
//      families are profiled): exact coarse histogram of every element (LDS per tile, integer
//      atomics to global); elements with key >= lo ("candidates", 10-20 % of the data) are
//      written, as bit patterns, to the tile's own slice of a candidate buffer in ballot-prefix
//      order; the energy of everything below lo is summed in registers.
//   3. scan of the exact histogram: for every requested k the coarse bin holding the k-th largest
//      magnitude and how many entries to take inside it.  If the prediction was too high for a
//      layer (lo above its lowest threshold bin) that layer alone is collected again with the
//      exact bound, so the result never depends on the sample.
//   4. refinement on the candidates only: energy below each threshold bin (fp64, fixed order),
//      histogram of the next 10 bits inside each threshold bin, pick the sub-bin, histogram of
//      the last 9 bits, pick the exact k-th magnitude and the number of equal magnitudes to keep
//      (compress always; the profile only for a sub-bin whose share of the layer's dropped energy
//      is not provably negligible, see topk_pick_a_kernel).
//      Histogram bins carry their energy as integers (entries of one coarse bin share the
//      exponent: x^2 = m^2 2^(2(E-150)), m the 24-bit significand; sum (m^2 >> 16) is exact), so
//      nothing depends on the order of atomics.
// Compression then counts kept entries per tile from the candidates, scans the tile counts, and
// writes values and indices in ascending index order (equal magnitudes: lowest indices first).
// A compression queued right behind a profile of the same data takes the candidates from that
// profile, whose main pass then also records where each candidate is (16 bits: position in the
// tile, sign), and reads the data no second time.
#include <cstdlib>
#include <cstring>

#include "internal.h"
#include "reduce_dev.h"
#include "topk_dev.h"

namespace lgreco {

struct TopkList {
    uint32_t bin, count;
};
struct TopkSel {
    uint32_t k, tbin, need, list;   // need: entries to take from the threshold bin (1..count)
    uint32_t bin_a, need_a;         // refinement level A (bits 18..9)
    uint32_t thr, ties_keep;        // exact threshold pattern; equal entries kept (compress)
};
struct TopkLayer {
    int64_t cand_base;              // first slot of this layer's region in the candidate buffer
    uint32_t nlists, min_tbin;
    uint32_t recollect, pad;        // 1: the predicted bound was too high, collect again
    TopkList lists[kMaxTopk];
    TopkSel sel[kMaxTopk];
};
constexpr int kRefTiles = 16;       // largest tiles per refinement / sample workgroup (fewer elements never: with
                                    // smaller tiles a workgroup takes proportionally more of them)
constexpr int kRefThreads = 1024;
constexpr int kRefSlots = 512;      // refinement workgroups the chip runs at a time (256 CUs x 2)
constexpr int kBinsA = 1024, kBinsB = 512;
constexpr int kSampleEvery = 16;    // one 512-element chunk out of 16 is sampled
constexpr uint32_t kHintMargin = 2; // coarse bins (4.4 % in magnitude each) between a remembered threshold and the bound derived from it

// ------------------------------------------------------------------------ block helpers
// Suffix sums of a histogram in LDS over the block's first 256 threads: thread t owns the bins
// [t * per, (t + 1) * per) and scan[t] becomes the number of entries in its bins and all higher
// ones (scan[0] = total).  nbins <= 16 * 256.  Every thread of the block calls; the threads past
// the first 256 only join the barriers.
__device__ void block_suffix(const uint32_t* hist, int nbins, uint32_t* scan) {
    __shared__ uint32_t wtot[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bool act = tid < 256;
    const int per = (nbins + 255) / 256;
    const int lo = min(tid * per, nbins), hi = min(lo + per, nbins);
    uint32_t inc = 0;
    if (act)
        for (int b = lo; b < hi; ++b) inc += hist[b];
    for (int o = 1; o < 64; o <<= 1) {        // inclusive suffix scan inside the wavefront
        const uint32_t n = __shfl_down(inc, o, 64);
        if (lane + o < 64) inc += n;
    }
    if (act && lane == 0) wtot[wave] = inc;
    __syncthreads();
    if (act) {
        for (int w = wave + 1; w < 4; ++w) inc += wtot[w];
        scan[tid] = inc;
    }
    __syncthreads();
}

// After block_suffix: for each of n requests, the largest bin b with (entries in bins >= b) >=
// need[j], and `above` = entries in bins > b, written to res[2j], res[2j+1].  If fewer than need[j]
// entries exist, {0, total - hist[0]}.
template <int N>
__device__ void block_find(const uint32_t* hist, int nbins, const uint32_t (&need)[N], int n, const uint32_t* scan,
                           uint32_t* res) {
    const int tid = threadIdx.x;
    const bool act = tid < 256;
    const int per = (nbins + 255) / 256;
    const int lo = min(tid * per, nbins), hi = min(lo + per, nbins);
    if (tid == 0) {
        const uint32_t rest = scan[0] - hist[0];
#pragma unroll
        for (int j = 0; j < N; ++j)
            if (j < n) { res[2 * j] = 0; res[2 * j + 1] = rest; }
    }
    __syncthreads();
    if (act) {
        uint32_t running = (tid + 1 < 256) ? scan[tid + 1] : 0;
        for (int b = hi - 1; b >= lo; --b) {
            const uint32_t c = hist[b];
#pragma unroll
            for (int j = 0; j < N; ++j) {
                if (j < n && running < need[j] && running + c >= need[j]) {
                    res[2 * j] = (uint32_t)b;
                    res[2 * j + 1] = running;
                }
            }
            running += c;
        }
    }
    __syncthreads();
}

// One request: result broadcast through res[2]; scan[0] is left holding the total.
__device__ void block_kth_from_top(const uint32_t* hist, int nbins, uint32_t need, uint32_t* scan,
                                   uint32_t* res) {
    block_suffix(hist, nbins, scan);
    const uint32_t one[1] = {need};
    block_find<1>(hist, nbins, one, 1, scan, res);
}

// Exclusive scan of one uint32 per thread over the 256-thread block; returns the prefix and the
// block total through *total.  tmp: 4 words of LDS.
__device__ uint32_t block_excl_scan(uint32_t v, uint32_t* tmp, uint32_t* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t inc = v;
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t n = __shfl_up(inc, o, 64);
        if (lane >= o) inc += n;
    }
    __syncthreads();
    if (lane == 63) tmp[wave] = inc;
    __syncthreads();
    uint32_t base = 0, tot = 0;
    for (int w = 0; w < kThreads / 64; ++w) {
        if (w < wave) base += tmp[w];
        tot += tmp[w];
    }
    *total = tot;
    return base + inc - v;
}

// ------------------------------------------------------------------------ kernels
__global__ void copy_u32_kernel(uint32_t* dst, const uint32_t* src, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

__global__ void fill_u32_kernel(uint32_t* p, size_t n, uint32_t v) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        p[i] = v;
}

struct RefWork {                     // one workgroup of the sample / refinement kernels: tiles [t0, t1) of a layer
    int32_t layer, t0, t1, pad;
};

// Coarse histogram of a sample: every kSampleEvery-th 512-element chunk of every tile (chunk 0
// included, so short tiles are sampled whole or by their first chunk).  One workgroup takes a run
// of tiles of one layer; a wavefront takes whole sampled chunks.
__global__ __launch_bounds__(kThreads) void topk_sample_kernel(const float* __restrict__ g,
                                                                const float* __restrict__ e,
                                                                const DevLayer* __restrict__ layers,
                                                                const Tile* __restrict__ tiles,
                                                                const RefWork* __restrict__ work,
                                                                int per_tile, uint32_t* __restrict__ shist) {
    __shared__ uint32_t s_hist[kHistBins];
    const RefWork w = work[blockIdx.x];
    const DevLayer L = layers[w.layer];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int b = threadIdx.x; b < kHistBins; b += kThreads) s_hist[b] = 0;
    __syncthreads();
    const int kPerTile = per_tile;                               // sampled chunks of a full tile
    constexpr int kWaves = kThreads / 64, kBatch = 4;            // chunks a wavefront has in flight
    const int npairs = (w.t1 - w.t0) * kPerTile;
    for (int pr0 = wave * kBatch; pr0 < npairs; pr0 += kWaves * kBatch) {
        float4 a[kBatch][2];
        bool vec[kBatch];
#pragma unroll
        for (int q = 0; q < kBatch; ++q) {
            const int pr = pr0 + q;
            vec[q] = false;
            if (pr >= npairs) continue;
            const Tile t = tiles[w.t0 + pr / kPerTile];
            const int first = (pr % kPerTile) * kSampleEvery * kChunk;
            if (first >= t.count) continue;
            const float* gp = g + L.offset + t.pos + first;
            const float* ep = e ? e + L.offset + t.pos + first : nullptr;
            if (t.fast) {
                vec[q] = true;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    a[q][h] = reinterpret_cast<const float4*>(gp)[h * 64 + lane];
                    if (ep) {
                        const float4 b = reinterpret_cast<const float4*>(ep)[h * 64 + lane];
                        a[q][h].x += b.x; a[q][h].y += b.y; a[q][h].z += b.z; a[q][h].w += b.w;
                    }
                }
            } else {
                const int n = min(kChunk, t.count - first);
                for (int i = lane; i < n; i += 64) {
                    const float x = ep ? gp[i] + ep[i] : gp[i];
                    atomicAdd(&s_hist[mag_bits(x) >> kHistShift], 1u);
                }
            }
        }
#pragma unroll
        for (int q = 0; q < kBatch; ++q) {
            if (!vec[q]) continue;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                atomicAdd(&s_hist[mag_bits(a[q][h].x) >> kHistShift], 1u);
                atomicAdd(&s_hist[mag_bits(a[q][h].y) >> kHistShift], 1u);
                atomicAdd(&s_hist[mag_bits(a[q][h].z) >> kHistShift], 1u);
                atomicAdd(&s_hist[mag_bits(a[q][h].w) >> kHistShift], 1u);
            }
        }
    }
    __syncthreads();
    uint32_t* gh = shist + (size_t)w.layer * kHistBins;
    for (int b = threadIdx.x; b < kHistBins; b += kThreads) {
        const uint32_t c = s_hist[b];
        if (c) atomicAdd(&gh[b], c);
    }
}

// One workgroup per layer: predicted lower bound of the lowest threshold bin.
__global__ __launch_bounds__(256) void topk_predict_kernel(const uint32_t* __restrict__ shist,
                                                           const uint32_t* __restrict__ ks, int ntk,
                                                           const DevLayer* __restrict__ layers,
                                                           uint32_t* __restrict__ lo) {
    __shared__ uint32_t s_hist[kHistBins];
    __shared__ uint32_t s_scan[256];
    __shared__ uint32_t s_res[2];
    const int l = blockIdx.x;
    if (ks[(size_t)l * kMaxTopk] == 0) {
        if (threadIdx.x == 0) lo[l] = 0xFFFFFFFFu;
        return;
    }
    for (int b = threadIdx.x; b < kHistBins; b += 256) s_hist[b] = shist[(size_t)l * kHistBins + b];
    __syncthreads();
    uint32_t kmax = 0;
    for (int j = 0; j < ntk; ++j) kmax = max(kmax, ks[(size_t)l * kMaxTopk + j]);
    // sample size = total of the histogram (left in s_scan[0] by a scan for "everything")
    block_kth_from_top(s_hist, kHistBins, 0xFFFFFFFFu, s_scan, s_res);
    const double ns = (double)s_scan[0];
    __syncthreads();
    const double n = (double)layers[l].numel;
    const double t = (double)kmax * ns / n;                 // expected sample entries above the threshold
    const double want = 1.5 * t + 6.0 * sqrt(t) + 16.0;     // wide margin: the sample only has to be roughly right
    if (want >= ns) {
        if (threadIdx.x == 0) lo[l] = 0u;
        return;
    }
    block_kth_from_top(s_hist, kHistBins, (uint32_t)want, s_scan, s_res);
    if (threadIdx.x == 0) lo[l] = s_res[0];
}

struct CollectParams {
    const float* g;
    const float* e;
    const DevLayer* layers;
    const Tile* tiles;
    const uint32_t* ks;
    const TopkLayer* tl;        // KNOWN: the profile's selection records
    const uint32_t* lo;
    uint32_t* hist;
    uint32_t* cand;
    uint32_t* cand_idx;         // compress: index within the layer and sign of every candidate
    float* ef_out;              // compress: error feedback, written as x everywhere (kept entries are
                                // zeroed afterwards by the emit kernel)
    const int64_t* cand_base;
    TopkTileInfo* tinfo;
    double* base_part;
    uint32_t* cnt_b;            // KNOWN: [L x kBinsB] last 9 pattern bits inside each layer's boundary sub-bin
    // profile (no EMIT): not null = x is written here as it is formed (may be the buffer e points to:
    // every element is read once, by the lane that then writes it)
    float* x_out;
    // profile (no EMIT): where every candidate is goes to cand_idx too, as 16-bit entries (place16)
    int32_t record_idx;
};

// Main pass without quantization candidates: exact coarse histogram (HIST) and candidate
// collection.
// KNOWN (compression right behind a profile of the same data): which layers take part and what
// they keep comes from the layer records (family, slot of the chosen density in the profile's
// selection records), the bound is the 22-bit prefix the profile resolved the k-th magnitude to
// (nearly exactly the kept set qualifies), and the elements inside that boundary sub-bin are
// counted by their last 9 pattern bits (s_hist: kBinsB cells) for the exact threshold.
// TEAM (the second collection, made by the refinement kernel's workgroup for its own tiles): the
// workgroup is several teams of kThreads threads, each with a tile of its own (or none: `active`
// false; the teams still meet at the barrier) and its own s_red; the caller has checked that the
// layer takes part.
template <bool HIST, bool EMIT, bool KNOWN = false, bool TEAM = false>
__device__ __forceinline__ void collect_tile(const CollectParams& p, const int tile, uint32_t* s_hist, double* s_red,
                                             const bool active = true) {
    static_assert(!(HIST && KNOWN), "the coarse histogram is not built when the thresholds are known");
    static_assert(!TEAM || (!HIST && !KNOWN), "teams collect, nothing else");
    if (TEAM && !active) {             // (uniform over the team)
        __syncthreads();
        return;
    }
    const Tile t = p.tiles[tile];
    const DevLayer L = p.layers[t.layer];
    uint32_t bound;
    if (KNOWN) {
        if (L.family != LGRECO_TOPK || L.slot < 0 || L.slot >= kMaxTopk) return;
        const TopkSel& S = p.tl[t.layer].sel[L.slot];
        bound = ((S.tbin << 10) | S.bin_a) << 9;
    } else {
        if (!TEAM) {
            if (p.ks[(size_t)t.layer * kMaxTopk] == 0) return;
        }
        bound = bound_of_key(p.lo[t.layer]);
    }
    const float* gp = p.g + L.offset + t.pos;
    const float* ep = p.e ? p.e + L.offset + t.pos : nullptr;
    float* const eo = EMIT ? p.ef_out + L.offset + t.pos : nullptr;
    float* const xo = (!EMIT && p.x_out) ? p.x_out + L.offset + t.pos : nullptr;
    const int tid = TEAM ? (int)(threadIdx.x % kThreads) : (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (HIST || KNOWN) {
        for (int b = tid; b < (KNOWN ? kBinsB : kHistBins); b += kThreads) s_hist[b] = 0;
        __syncthreads();
    }
    const int64_t slice_off = p.cand_base[t.layer] + t.pos;
    uint32_t* const slice = p.cand + slice_off;
    uint32_t* const slice_idx = EMIT ? p.cand_idx + slice_off : nullptr;
    uint16_t* const slice_at = (!EMIT && p.record_idx) ? reinterpret_cast<uint16_t*>(p.cand_idx) + slice_off : nullptr;
    Collector col;
    uint32_t start;
    if (t.fast) {
        int c0, c1;
        wave_range(t.count / kChunk, wave, &c0, &c1);
        start = (uint32_t)c0 * kChunk;
        col.init(slice + start, slice_idx ? slice_idx + start : nullptr, bound,
                 slice_at ? slice_at + start : nullptr, (uint32_t)t.pos);
        // one 512-element chunk per iteration (uniform trip count): both halves are loaded before
        // either is used, so a lane keeps four 128-bit loads in flight
        for (int v = c0 * (kChunk / 4) + lane; v < c1 * (kChunk / 4); v += kChunk / 4) {
            float4 a[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) a[h] = load_stream(reinterpret_cast<const float4*>(gp) + v + 64 * h);
            if (ep) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const float4 b = load_stream(reinterpret_cast<const float4*>(ep) + v + 64 * h);
                    a[h].x += b.x; a[h].y += b.y; a[h].z += b.z; a[h].w += b.w;
                }
            }
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                if (!EMIT && xo) store_stream(reinterpret_cast<float4*>(xo) + v + 64 * h, a[h]);
                if (EMIT && KNOWN) {
                    // nearly every candidate is kept here: candidates are written as zero at once, the
                    // emit step puts the few that are not kept back
                    float4 w = a[h];
                    w.x = mag_bits(w.x) >= bound ? 0.0f : w.x;
                    w.y = mag_bits(w.y) >= bound ? 0.0f : w.y;
                    w.z = mag_bits(w.z) >= bound ? 0.0f : w.z;
                    w.w = mag_bits(w.w) >= bound ? 0.0f : w.w;
                    store_stream(reinterpret_cast<float4*>(eo) + v + 64 * h, w);
                } else if (EMIT) {
                    store_stream(reinterpret_cast<float4*>(eo) + v + 64 * h, a[h]);
                }
                if (HIST) {
                    atomicAdd(&s_hist[mag_bits(a[h].x) >> kHistShift], 1u);
                    atomicAdd(&s_hist[mag_bits(a[h].y) >> kHistShift], 1u);
                    atomicAdd(&s_hist[mag_bits(a[h].z) >> kHistShift], 1u);
                    atomicAdd(&s_hist[mag_bits(a[h].w) >> kHistShift], 1u);
                }
                const float x[4] = {a[h].x, a[h].y, a[h].z, a[h].w};
                if (KNOWN) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const uint32_t in = mag_bits(x[q]) - bound;      // below the bound: wraps to a large value
                        if (in < (uint32_t)kBinsB) atomicAdd(&s_hist[in], 1u);
                    }
                }
                col.take4(x, (uint32_t)(t.pos + 4 * (int64_t)(v + 64 * h)));
            }
        }
    } else {
        int b0, b1;
        wave_range((t.count + 63) / 64, wave, &b0, &b1);
        start = (uint32_t)b0 * 64;
        col.init(slice + start, slice_idx ? slice_idx + start : nullptr, bound,
                 slice_at ? slice_at + start : nullptr, (uint32_t)t.pos);
        for (int b = b0; b < b1; ++b) {
            const int i = b * 64 + lane;
            const bool valid = i < t.count;
            float x = 0.0f;
            if (valid) x = ep ? gp[i] + ep[i] : gp[i];
            if (EMIT && valid) eo[i] = (KNOWN && mag_bits(x) >= bound) ? 0.0f : x;
            if (!EMIT && valid && xo) xo[i] = x;
            if (HIST && valid) atomicAdd(&s_hist[mag_bits(x) >> kHistShift], 1u);
            if (KNOWN && valid && mag_bits(x) - bound < (uint32_t)kBinsB) atomicAdd(&s_hist[mag_bits(x) - bound], 1u);
            col.take(x, valid, (uint32_t)(t.pos + i));
        }
    }
    const double bs = wave_sum((double)col.base);
    if (lane == 0) {
        s_red[wave] = bs;
        p.tinfo[tile].cnt[wave] = col.cur;
        p.tinfo[tile].start[wave] = start;
    }
    __syncthreads();
    if (tid == 0) p.base_part[tile] = (s_red[0] + s_red[1]) + (s_red[2] + s_red[3]);
    if (HIST) {
        uint32_t* gh = p.hist + (size_t)t.layer * kHistBins;
        for (int b = tid; b < kHistBins; b += kThreads) {
            const uint32_t c = s_hist[b];
            if (c) atomicAdd(&gh[b], c);
        }
    }
    if (KNOWN) {
        uint32_t* gh = p.cnt_b + (size_t)t.layer * kBinsB;
        for (int b = tid; b < kBinsB; b += kThreads) {
            const uint32_t c = s_hist[b];
            if (c) atomicAdd(&gh[b], c);
        }
    }
}

// Main pass of the compression when the profile's selection records are valid for the same data.
__global__ __launch_bounds__(kThreads) void topk_collect_known_kernel(CollectParams p) {
    __shared__ uint32_t s_hist[kBinsB];
    __shared__ double s_red[kThreads / 64];
    collect_tile<false, true, true>(p, (int)blockIdx.x, s_hist, s_red);
}

// The same step from the profile's candidates instead of the data (the profile recorded index and
// sign of every candidate and left x in the error-feedback buffer): every kept entry is among them,
// so the data is not read again.  One workgroup per tile, a wavefront per candidate slice: the
// candidates at or above the boundary sub-bin's lower edge are copied to the second candidate
// buffer IN ELEMENT ORDER (the profile's main pass may store a slice in another order), and the
// boundary sub-bin's entries are counted by their last 9 bits.  Order: every such candidate sets
// the bit of its element in a bitmap of the wavefront's share of the tile (at most kFilterSpan
// elements); its place in the output is the number of bits below its own.
__device__ __forceinline__ uint32_t lanes_below(unsigned long long m, uint32_t add);
constexpr int kFilterSpan = kTile / (kThreads / 64);
struct FilterParams {
    const DevLayer* layers;
    const Tile* tiles;
    const TopkLayer* tl;
    const int64_t* cand_base;
    const TopkTileInfo* tinfo;      // what the profile's main pass wrote
    const uint32_t* cand;
    const uint32_t* cand_idx;
    TopkTileInfo* tinfo_out;
    uint32_t* cand_out;
    uint32_t* cand_idx_out;
    uint32_t* cnt_b;
};
constexpr int kFilterKeep = 512;    // kept candidates a wavefront holds in LDS between the two steps
__global__ __launch_bounds__(kThreads) void topk_filter_known_kernel(FilterParams p) {
    constexpr int kWords = kFilterSpan / 32;
    static_assert(kFilterSpan <= 65536, "places inside a wavefront's share are kept in 16 bits");
    __shared__ uint32_t s_bits[kThreads / 64][kWords];
    __shared__ uint16_t s_before[kThreads / 64][kWords];
    __shared__ uint2 s_keep[kThreads / 64][kFilterKeep];
    __shared__ uint32_t s_hist[kBinsB];
    const int tile = blockIdx.x;
    const Tile t = p.tiles[tile];
    const DevLayer L = p.layers[t.layer];
    if (L.family != LGRECO_TOPK || L.slot < 0 || L.slot >= kMaxTopk) return;       // the whole workgroup
    const TopkSel& S = p.tl[t.layer].sel[L.slot];
    const uint32_t bound = ((S.tbin << 10) | S.bin_a) << 9;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t n = p.tinfo[tile].cnt[wave], start = p.tinfo[tile].start[wave];
    const int64_t off = p.cand_base[t.layer] + t.pos + start;
    const uint32_t* const pats = p.cand + off;
    const uint16_t* const idxs = reinterpret_cast<const uint16_t*>(p.cand_idx) + off;   // place16 entries
    for (int b = tid; b < kBinsB; b += kThreads) s_hist[b] = 0;
    for (int b = lane; b < kWords; b += 64) s_bits[wave][b] = 0;
    __syncthreads();
    // step 1: one read of the slice.  What passes sets its element's bit, is counted if it lies in
    // the boundary sub-bin, and is put aside in LDS (the first kFilterKeep of the wavefront).
    constexpr int kBatch = 4;                                 // pairs of loads a lane has in flight
    uint32_t kept = 0;                                        // uniform
    for (uint32_t i0 = 0; i0 < n; i0 += 64 * kBatch) {
        uint32_t pat[kBatch], ix[kBatch];
#pragma unroll
        for (int q = 0; q < kBatch; ++q) {
            const uint32_t i = i0 + 64 * q + lane;
            pat[q] = i < n ? pats[i] : 0u;
            ix[q] = i < n ? idxs[i] : 0u;
        }
#pragma unroll
        for (int q = 0; q < kBatch; ++q) {
            const uint32_t rel = (ix[q] & 0x7FFFu) - start;
            const bool pass = i0 + 64 * q + lane < n && pat[q] >= bound && rel < (uint32_t)kFilterSpan;
            const unsigned long long m = __ballot(pass);
            if (pass) {
                atomicOr(&s_bits[wave][rel >> 5], 1u << (rel & 31u));
                if (pat[q] - bound < (uint32_t)kBinsB) atomicAdd(&s_hist[pat[q] - bound], 1u);
                const uint32_t at = kept + lanes_below(m, 0u);
                if (at < (uint32_t)kFilterKeep) s_keep[wave][at] = make_uint2(pat[q], ix[q]);
            }
            kept += (uint32_t)__popcll(m);
        }
    }
    __syncthreads();
    // exclusive prefix of the bitmap's population over the wavefront's words
    {
        constexpr int kPer = kWords / 64;
        uint32_t c[kPer], mine = 0;
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            c[j] = (uint32_t)__popc(s_bits[wave][lane * kPer + j]);
            mine += c[j];
        }
        uint32_t inc = mine;
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t v = __shfl_up(inc, o, 64);
            if (lane >= o) inc += v;
        }
        uint32_t run = inc - mine;
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            s_before[wave][lane * kPer + j] = (uint16_t)run;
            run += c[j];
        }
    }
    __syncthreads();
    // step 2: every kept candidate goes to the place its element has among the kept ones
    uint32_t* const out = p.cand_out + off;
    uint32_t* const out_idx = p.cand_idx_out + off;
    auto place = [&](const uint32_t pat, const uint32_t ix) __attribute__((always_inline)) {
        const uint32_t rel = (ix & 0x7FFFu) - start;
        const uint32_t w = rel >> 5;
        const uint32_t at = s_before[wave][w] + (uint32_t)__popc(s_bits[wave][w] & ((1u << (rel & 31u)) - 1u));
        out[at] = pat;
        out_idx[at] = ((uint32_t)t.pos + (ix & 0x7FFFu)) | ((ix & 0x8000u) << 16);   // index within the layer, sign
    };
    if (kept <= (uint32_t)kFilterKeep) {
        for (uint32_t i = lane; i < kept; i += 64) {
            const uint2 c = s_keep[wave][i];
            place(c.x, c.y);
        }
    } else {                                                  // more than LDS holds: the slice is read again
        for (uint32_t i0 = 0; i0 < n; i0 += 64 * kBatch) {
            uint32_t pat[kBatch], ix[kBatch];
#pragma unroll
            for (int q = 0; q < kBatch; ++q) {
                const uint32_t i = i0 + 64 * q + lane;
                pat[q] = i < n ? pats[i] : 0u;
                ix[q] = i < n ? idxs[i] : 0u;
            }
#pragma unroll
            for (int q = 0; q < kBatch; ++q) {
                const uint32_t rel = (ix[q] & 0x7FFFu) - start;
                if (i0 + 64 * q + lane < n && pat[q] >= bound && rel < (uint32_t)kFilterSpan) place(pat[q], ix[q]);
            }
        }
    }
    if (lane == 0) {
        p.tinfo_out[tile].cnt[wave] = kept;
        p.tinfo_out[tile].start[wave] = start;
    }
    uint32_t* gh = p.cnt_b + (size_t)t.layer * kBinsB;
    for (int b = tid; b < kBinsB; b += kThreads) {
        const uint32_t c = s_hist[b];
        if (c) atomicAdd(&gh[b], c);
    }
}

// One workgroup per layer: the exact threshold pattern and the number of entries equal to it that
// are kept, from the counts the main pass above left; the counts are cleared for the next call.
__global__ __launch_bounds__(256) void topk_pick_known_kernel(const DevLayer* __restrict__ layers,
                                                              TopkLayer* __restrict__ tl,
                                                              uint32_t* __restrict__ cnt_b) {
    __shared__ uint32_t s_hist[kBinsB];
    __shared__ uint32_t s_scan[256];
    __shared__ uint32_t s_res[2];
    const int l = blockIdx.x;
    const DevLayer L = layers[l];
    if (L.family != LGRECO_TOPK || L.slot < 0 || L.slot >= kMaxTopk) return;
    TopkSel& S = tl[l].sel[L.slot];
    for (int b = threadIdx.x; b < kBinsB; b += 256) {
        s_hist[b] = cnt_b[(size_t)l * kBinsB + b];
        cnt_b[(size_t)l * kBinsB + b] = 0u;
    }
    __syncthreads();
    const uint32_t need_a = S.need_a, prefix = (S.tbin << 10) | S.bin_a;
    block_kth_from_top(s_hist, kBinsB, need_a, s_scan, s_res);
    if (threadIdx.x == 0) {
        S.thr = (prefix << 9) | s_res[0];
        S.ties_keep = need_a - s_res[1];
    }
}

template <bool HIST, bool EMIT>
__global__ __launch_bounds__(kThreads) void topk_collect_kernel(CollectParams p) {
    __shared__ uint32_t s_hist[HIST ? kHistBins : 1];
    __shared__ double s_red[kThreads / 64];
    collect_tile<HIST, EMIT>(p, (int)blockIdx.x, s_hist, s_red);
}

// One workgroup per layer: threshold bin and in-bin rank for every requested k; threshold-bin
// lists; check of the predicted bound.
// Workgroups past the first n_layers (when the call also profiles quantization) sum that family's
// tile partials per layer instead: the two jobs depend on the main pass only and share a launch.
struct ScanReduce {
    const double* partials;     // null: no such workgroups
    double* errors;
    const DevLayer* layers;
    int32_t stride;
    ReduceCols cols;
};
__global__ __launch_bounds__(256) void topk_scan_kernel(uint32_t* __restrict__ hist,
                                                        const uint32_t* __restrict__ ks, int ntk,
                                                        const int64_t* __restrict__ cand_base,
                                                        const uint32_t* lo_in, uint32_t* lo_out,
                                                        TopkLayer* __restrict__ tl, uint32_t* hint, int clear,
                                                        int n_layers, ScanReduce red) {
    __shared__ __align__(16) unsigned char s_raw[sizeof(uint32_t) * kHistBins];   // 16 KB: the histogram, or the reduction's tree
    static_assert(sizeof(s_raw) >= sizeof(double) * kMaxQuant * 256, "shared by both jobs");
    if ((int)blockIdx.x >= n_layers) {
        reduce_partials_block(red.partials, red.stride, red.cols, red.layers, red.errors, (int)blockIdx.x - n_layers,
                              reinterpret_cast<double(*)[256]>(s_raw));
        return;
    }
    uint32_t* const s_hist = reinterpret_cast<uint32_t*>(s_raw);
    __shared__ uint32_t s_scan[256];
    __shared__ uint32_t s_res[2 * kMaxTopk];
    const int l = blockIdx.x;
    TopkLayer& T = tl[l];
    if (ks[(size_t)l * kMaxTopk] == 0) {
        if (threadIdx.x == 0) {
            T.nlists = 0; T.min_tbin = 0; T.recollect = 0;
            for (int j = 0; j < kMaxTopk; ++j) T.sel[j].k = 0;
            lo_out[l] = lo_in[l];
            if (hint) hint[l] = 0xFFFFFFFFu;
        }
        if (clear)
            for (int b = threadIdx.x; b < kHistBins; b += 256) hist[(size_t)l * kHistBins + b] = 0u;
        return;
    }
    for (int b = threadIdx.x; b < kHistBins; b += 256) {
        s_hist[b] = hist[(size_t)l * kHistBins + b];
        if (clear) hist[(size_t)l * kHistBins + b] = 0u;     // the next call's main pass starts from zero
    }
    __syncthreads();
    // one suffix scan of the histogram serves every requested k
    uint32_t kk[kMaxTopk];
#pragma unroll
    for (int j = 0; j < kMaxTopk; ++j) kk[j] = j < ntk ? ks[(size_t)l * kMaxTopk + j] : 0u;
    block_suffix(s_hist, kHistBins, s_scan);
    block_find<kMaxTopk>(s_hist, kHistBins, kk, ntk, s_scan, s_res);
    // the layer's record is put together in LDS and written out by the whole workgroup
    __shared__ TopkLayer sT;
    if (threadIdx.x == 0) {
        uint32_t nl = 0, mn = 0xFFFFFFFFu;
        for (int j = 0; j < kMaxTopk; ++j) {
            TopkSel& S = sT.sel[j];
            S = TopkSel{};
            if (j >= ntk) continue;
            const uint32_t k = ks[(size_t)l * kMaxTopk + j];
            S.k = k;
            S.tbin = s_res[2 * j];
            S.need = k - s_res[2 * j + 1];
            uint32_t u = nl;
            for (uint32_t q = 0; q < nl; ++q)
                if (sT.lists[q].bin == S.tbin) u = q;
            if (u == nl) {
                sT.lists[nl] = TopkList{S.tbin, s_hist[S.tbin]};
                ++nl;
            }
            S.list = u;
            mn = min(mn, S.tbin);
        }
        for (uint32_t q = nl; q < (uint32_t)kMaxTopk; ++q) sT.lists[q] = TopkList{0u, 0u};
        sT.nlists = nl;
        sT.min_tbin = mn;
        sT.cand_base = cand_base[l];
        // every element at or above the lowest threshold bin must be among the candidates
        // (lo_in may be the same array as hint: it is read before hint is written)
        const uint32_t used = lo_in[l];
        sT.recollect = used > mn ? 1u : 0u;
        sT.pad = 0;
        lo_out[l] = sT.recollect ? mn : used;
        // collection bound for the next call of this kind: kHintMargin coarse bins (4.4 % in magnitude each)
        // under the lowest threshold found now
        if (hint) hint[l] = mn > kHintMargin ? mn - kHintMargin : 0u;
    }
    __syncthreads();
    static_assert(sizeof(TopkLayer) % 4 == 0, "copied as 32-bit words");
    for (int w = threadIdx.x; w < (int)(sizeof(TopkLayer) / 4); w += 256)
        reinterpret_cast<uint32_t*>(&T)[w] = reinterpret_cast<const uint32_t*>(&sT)[w];
}

struct RefineParams {
    TopkLayer* tl;
    const DevLayer* layers;
    const Tile* tiles;
    const TopkTileInfo* tinfo;
    const uint32_t* cand;
    const RefWork* work;              // [n_work]
    const int2* work_range;           // [L] the layer's workgroups [x, y)
    const double* base_part;          // [n_tiles]
    double* below_part;               // [n_work x kMaxTopk] energy of candidates below each threshold bin
    // per-workgroup partial histograms (plain stores, summed in workgroup order by the pick kernels)
    uint32_t* cnt_a;                  // [n_work x kMaxTopk x kBinsA] compress: counts
    unsigned long long* cell_a;       // [n_work x kMaxTopk x kBinsA] profile: packed count + energy
    uint32_t* cnt_b;                  // [n_work x kMaxTopk x kBinsB] compress: counts
    double* errors;                   // may be null (compress)
    int32_t stride;
    int32_t ntk;
    int32_t col[kMaxTopk];
    // the second collection of a layer whose predicted bound was too high (flagged by the scan):
    // every workgroup of the first refinement kernel makes it for its own tiles before it looks at
    // their candidates (rc.ef_out not null: the compression's form, which also writes x)
    CollectParams rc;
};

// The second collection for the tiles [t0, t1) of a flagged layer, by a refinement workgroup: four
// teams of kThreads threads, a tile each per round.
static_assert(kRefThreads % kThreads == 0, "whole teams");
template <bool EMIT>
__device__ __forceinline__ void collect_again(const CollectParams& rc, int t0, int t1) {
    constexpr int kTeams = kRefThreads / kThreads;
    __shared__ double s_team_red[kTeams][kThreads / 64];
    const int team = threadIdx.x / kThreads;
    for (int first = t0; first < t1; first += kTeams) {
        const int tile = first + team;
        collect_tile<false, EMIT, false, true>(rc, min(tile, t1 - 1), nullptr, s_team_red[team], tile < t1);
        __syncthreads();                                // s_team_red is reused; the tile's records are written
    }
}

// Walks the candidates of tiles [t0, t1): one (tile, wavefront slice) pair per wavefront at a
// time, 8 loads in flight per lane; f(pattern) is called for every candidate, in a fixed order
// per thread.
template <typename F>
__device__ __forceinline__ void for_each_candidate(const RefineParams& p, const TopkLayer& T, int t0, int t1, F f) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    constexpr int kSub = kThreads / 64;
    const int npairs = (t1 - t0) * kSub;
    for (int pr = wave; pr < npairs; pr += kRefThreads / 64) {
        const int t = t0 + pr / kSub, sub = pr % kSub;
        const uint32_t n = p.tinfo[t].cnt[sub];
        const uint32_t* __restrict__ items = p.cand + T.cand_base + p.tiles[t].pos + p.tinfo[t].start[sub];
        uint32_t i0 = 0;
        for (; i0 + 64 * 8 <= n; i0 += 64 * 8) {          // full batches: no range checks
            uint32_t pat[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) pat[q] = items[i0 + q * 64 + lane];
#pragma unroll
            for (int q = 0; q < 8; ++q) f(pat[q]);
        }
        if (i0 < n) {
            uint32_t pat[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const uint32_t i = i0 + q * 64 + lane;
                pat[q] = i < n ? items[i] : 0xFFFFFFFFu;      // never a candidate's pattern (sign bit cleared)
            }
#pragma unroll
            for (int q = 0; q < 8; ++q)
                if (pat[q] != 0xFFFFFFFFu) f(pat[q]);
        }
    }
}

// Level-A histogram cell of the profile: entries in the low 20 bits (a refinement workgroup sees at
// most kRefTiles * kTile = 2^19 candidates), their integer energy sum (m^2 >> 23 each, < 2^25) above.
constexpr int kPackCountBits = 20, kPackEnergyShift = 23;
static_assert((long long)kRefTiles * kTile < (1ll << kPackCountBits), "count field too narrow");
static_assert(48 - kPackEnergyShift + kPackCountBits - 1 + kPackCountBits <= 64, "energy field too narrow");

__device__ __forceinline__ unsigned long long packed_cell(uint32_t pat) {
    const unsigned long long m = (pat & 0x7FFFFFu) | ((pat >> 23) ? 0x800000u : 0u);
    return (((m * m) >> kPackEnergyShift) << kPackCountBits) | 1ull;
}

// below[j] += x^2 for every j < NTK whose threshold bin lies above the candidate's key.  The
// requested k do not increase with j, so the threshold bins do not decrease and the sets
// {key < tb[j]} are nested: walking j downwards, each comparison narrows the set of active lanes
// (a compare that writes the execution mask) and the add runs under it: two vector instructions
// per k.  The mask is restored at the end; one asm statement, so nothing else runs under it.  The
// closing s_nop keeps the wait states a DPP instruction needs after a vector write of the mask,
// should the compiler place one right behind the block.
#define LG_BELOW_STEP(J) "v_cmpx_gt_u32 vcc, %[t" #J "], %[key]\n\tv_fmac_f32 %[b" #J "], %[x], %[x]\n\t"
#define LG_BELOW_ASM(STEPS)                                                                          \
    asm volatile("s_mov_b64 %[save], exec\n\t" STEPS "s_mov_b64 exec, %[save]\n\ts_nop 3"            \
                 : [b0] "+v"(b[0]), [b1] "+v"(b[1]), [b2] "+v"(b[2]), [b3] "+v"(b[3]), [b4] "+v"(b[4]), \
                   [b5] "+v"(b[5]), [b6] "+v"(b[6]), [b7] "+v"(b[7]), [save] "=&s"(save)              \
                 : [key] "v"(key), [x] "v"(x), [t0] "s"(tb[0]), [t1] "s"(tb[1]), [t2] "s"(tb[2]),      \
                   [t3] "s"(tb[3]), [t4] "s"(tb[4]), [t5] "s"(tb[5]), [t6] "s"(tb[6]), [t7] "s"(tb[7]) \
                 : "vcc")
template <int NTK>
__device__ __forceinline__ void below_chain(float (&b)[kMaxTopk], const uint32_t (&tb)[kMaxTopk], uint32_t key,
                                            float x) {
    static_assert(kMaxTopk == 8 && NTK >= 1 && NTK <= 8, "written out for 8");
    unsigned long long save;
    if constexpr (NTK == 1) LG_BELOW_ASM(LG_BELOW_STEP(0));
    if constexpr (NTK == 2) LG_BELOW_ASM(LG_BELOW_STEP(1) LG_BELOW_STEP(0));
    if constexpr (NTK == 3) LG_BELOW_ASM(LG_BELOW_STEP(2) LG_BELOW_STEP(1) LG_BELOW_STEP(0));
    if constexpr (NTK == 4) LG_BELOW_ASM(LG_BELOW_STEP(3) LG_BELOW_STEP(2) LG_BELOW_STEP(1) LG_BELOW_STEP(0));
    if constexpr (NTK == 5)
        LG_BELOW_ASM(LG_BELOW_STEP(4) LG_BELOW_STEP(3) LG_BELOW_STEP(2) LG_BELOW_STEP(1) LG_BELOW_STEP(0));
    if constexpr (NTK == 6)
        LG_BELOW_ASM(LG_BELOW_STEP(5) LG_BELOW_STEP(4) LG_BELOW_STEP(3) LG_BELOW_STEP(2) LG_BELOW_STEP(1)
                         LG_BELOW_STEP(0));
    if constexpr (NTK == 7)
        LG_BELOW_ASM(LG_BELOW_STEP(6) LG_BELOW_STEP(5) LG_BELOW_STEP(4) LG_BELOW_STEP(3) LG_BELOW_STEP(2)
                         LG_BELOW_STEP(1) LG_BELOW_STEP(0));
    if constexpr (NTK == 8)
        LG_BELOW_ASM(LG_BELOW_STEP(7) LG_BELOW_STEP(6) LG_BELOW_STEP(5) LG_BELOW_STEP(4) LG_BELOW_STEP(3)
                         LG_BELOW_STEP(2) LG_BELOW_STEP(1) LG_BELOW_STEP(0));
}
#undef LG_BELOW_ASM
#undef LG_BELOW_STEP

// Refinement level A over the candidates of a run of tiles.  NTK > 0 (profile, NTK = number of
// requested k): per list (distinct threshold bin) a histogram of bits 18..9 whose cells pack count
// and integer energy into one 64-bit LDS atomic, and per requested k the energy of the candidates
// below its threshold bin (fp32 per lane - a lane sees some tens of candidates - fp64 from the
// wavefront up).  NTK = 0 (compress): counts only.  Which list a candidate belongs to comes from a
// table over the 4096 coarse keys the workgroup builds first.  Partial histograms go to global
// memory with plain stores.
__host__ __device__ constexpr size_t refine_a_lds(int ntk, bool energy) {
    return (size_t)ntk * kBinsA * (energy ? 8 : 4) + kHistBins;
}
template <int NTK>
__global__ __launch_bounds__(kRefThreads, 8) void topk_refine_a_kernel(RefineParams p) {
    constexpr bool ENERGY = NTK > 0;
    extern __shared__ unsigned char refine_smem[];
    __shared__ double s_red[kRefThreads / 64][kMaxTopk];
    const RefWork w = p.work[blockIdx.x];
    const int l = w.layer;
    const TopkLayer& T = p.tl[l];
    if (T.recollect) {                  // workgroup-uniform; rare: the predicted bound was too high
        if (ENERGY) collect_again<false>(p.rc, w.t0, w.t1);
        else collect_again<true>(p.rc, w.t0, w.t1);
    }
    const int nlists = (int)T.nlists;
    const int tid = threadIdx.x, ntk = p.ntk;
    unsigned long long* const s_cell = reinterpret_cast<unsigned long long*>(refine_smem);   // ENERGY
    uint32_t* const s_cnt = reinterpret_cast<uint32_t*>(refine_smem);                        // !ENERGY
    uint8_t* const s_tab = refine_smem + (size_t)ntk * kBinsA * (ENERGY ? 8 : 4);
    for (int i = tid; i < nlists * kBinsA; i += kRefThreads) {
        if (ENERGY) s_cell[i] = 0; else s_cnt[i] = 0;
    }
    // workgroup-uniform: threshold bin of every k and the distinct threshold bins ("lists")
    uint32_t tb[kMaxTopk], lb[kMaxTopk];
#pragma unroll
    for (int j = 0; j < kMaxTopk; ++j) {
        tb[j] = __builtin_amdgcn_readfirstlane(j < ntk ? T.sel[j].tbin : 0u);
        lb[j] = j < nlists ? T.lists[j].bin : 0xFFFFFFFFu;
    }
    for (uint32_t key = tid; key < (uint32_t)kHistBins; key += kRefThreads) {
        uint32_t hit = 0;               // 1 + index of the list whose bin the key is
#pragma unroll
        for (int j = 0; j < kMaxTopk; ++j) hit = key == lb[j] ? (uint32_t)(j + 1) : hit;
        s_tab[key] = (uint8_t)hit;
    }
    __syncthreads();
    float below[kMaxTopk];
#pragma unroll
    for (int j = 0; j < kMaxTopk; ++j) below[j] = 0.0f;
    for_each_candidate(p, T, w.t0, w.t1, [&](uint32_t pat) {
        const uint32_t key = pat >> kHistShift;
        const uint32_t hit = s_tab[key];
        if constexpr (ENERGY) below_chain<NTK>(below, tb, key, __uint_as_float(pat));
        if (hit) {
            const uint32_t b = (hit - 1) * kBinsA + ((pat >> 9) & (kBinsA - 1));
            if (ENERGY) atomicAdd(&s_cell[b], packed_cell(pat));
            else atomicAdd(&s_cnt[b], 1u);
        }
    });
    if (ENERGY) {
#pragma unroll
        for (int j = 0; j < kMaxTopk; ++j) {
            if (j < ntk) {
                const double s = wave_sum((double)below[j]);
                if ((tid & 63) == 0) s_red[tid >> 6][j] = s;
            }
        }
    }
    __syncthreads();
    if (ENERGY && tid < ntk) {
        double s = 0.0;
        for (int wv = 0; wv < kRefThreads / 64; ++wv) s += s_red[wv][tid];
        p.below_part[(size_t)blockIdx.x * kMaxTopk + tid] = s;
    }
    if (ENERGY) {
        unsigned long long* const gc = p.cell_a + (size_t)blockIdx.x * kMaxTopk * kBinsA;
        for (int i = tid; i < nlists * kBinsA; i += kRefThreads) gc[i] = s_cell[i];
    } else {
        uint32_t* const gc = p.cnt_a + (size_t)blockIdx.x * kMaxTopk * kBinsA;
        for (int i = tid; i < nlists * kBinsA; i += kRefThreads) gc[i] = s_cnt[i];
    }
}

// One workgroup per (layer, requested k): sub-bin of level A holding the k-th magnitude.
// ENERGY (profile): the dropped energy is written here.  Everything outside the boundary sub-bin is
// summed exactly (integer energies).  Inside it the dropped entries are the `drop` smallest of
// `cnt` entries whose integer energies lie in [e_lo, e_hi] and sum to S, so their sum lies in
//     [ max(drop * e_lo, S - keep * e_hi),  drop * S / cnt ]
// (the kept ones are the largest: their mean is at least the overall mean, and none exceeds e_hi).
// The midpoint is taken when half the interval is within 1e-5 of the layer's error - for data
// without clusters the sub-bin holds a vanishing share of the dropped energy and this is always so.
// Otherwise (a constant or clipped layer, quantised values) the workgroup resolves the sub-bin
// exactly: it histograms the last 9 pattern bits of the layer's candidates that fall into the
// sub-bin - every cell is one fp32 value, so its energy is count * value^2 - and sums the `drop`
// smallest.  The deviation from the exact dropped energy is therefore at most 1e-5 relative from
// this step (plus 1.2e-7 from the truncated integer energies and the fp32 sums below the bound).
constexpr double kInsideTolerance = 1e-5;
template <bool ENERGY, int kPickThreads>
__global__ __launch_bounds__(kPickThreads) void topk_pick_a_kernel(RefineParams p) {
    __shared__ uint32_t s_hist[kBinsA];
    __shared__ unsigned long long s_en[ENERGY ? kBinsA : 1];
    __shared__ uint32_t s_scan[256];
    __shared__ uint32_t s_res[2];
    __shared__ unsigned long long s_e;
    __shared__ double s_sum[kPickThreads / 64];
    __shared__ double s_outside;        // error without the boundary sub-bin's dropped part
    __shared__ uint32_t s_exact[3];     // [0] resolve the sub-bin exactly, [1] its prefix (pattern >> 9), [2] entries kept in it
    const int l = blockIdx.x / p.ntk, j = blockIdx.x % p.ntk;      // the grid holds L x ntk workgroups
    TopkLayer& T = p.tl[l];
    if (T.sel[j].k == 0) return;
    const TopkSel S = T.sel[j];
    const int2 wr = p.work_range[l];
    const int tid = threadIdx.x, t = tid & 255, grp = tid >> 8;
    for (int b = tid; b < kBinsA; b += kPickThreads) {
        s_hist[b] = 0;
        if (ENERGY) s_en[b] = 0;
    }
    if (tid == 0) {
        s_e = 0;
        s_exact[0] = 0;
    }
    // energy below the collection bound (tile partials) and of the candidates below the threshold
    // bin (workgroup partials): loaded first so that the histogram work hides the latency; both
    // are summed in a fixed order (per thread, then a fixed tree)
    double part = 0.0;
    if (ENERGY && tid < 256) {
        const DevLayer L = p.layers[l];
        // four loads in flight per round trip; summed in index order all the same
        for (int tt = L.tile_begin + tid; tt < L.tile_end; tt += 4 * 256) {
            double v[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) v[q] = tt + q * 256 < L.tile_end ? p.base_part[tt + q * 256] : 0.0;
#pragma unroll
            for (int q = 0; q < 4; ++q) part += v[q];
        }
        for (int wg = wr.x + tid; wg < wr.y; wg += 256) part += p.below_part[(size_t)wg * kMaxTopk + j];
    }
    __syncthreads();
    // sum the layer's workgroup partials of this k's list: 4 bins per thread as 16-byte loads (two
    // pairs of packed cells, or four counts), the workgroups dealt round-robin to the thread groups,
    // integer LDS atomics join them (order does not matter).  The loop is a chain of memory round
    // trips with a fixed number of loads in flight: wide loads halve its length.
    {
        uint32_t c[4] = {0, 0, 0, 0};
        unsigned long long e[4] = {0, 0, 0, 0};
        static_assert(kBinsA == 1024, "written out for 1024 cells and 256 threads per group");
        const size_t off = (size_t)S.list * kBinsA;
#pragma unroll(kPickThreads == 256 ? 8 : 4)
        for (int wg = wr.x + grp; wg < wr.y; wg += kPickThreads / 256) {
            const size_t i = (size_t)wg * kMaxTopk * kBinsA + off;
            if (ENERGY) {
                const ulonglong2 v0 = *reinterpret_cast<const ulonglong2*>(p.cell_a + i + 2 * t);
                const ulonglong2 v1 = *reinterpret_cast<const ulonglong2*>(p.cell_a + i + 512 + 2 * t);
                const unsigned long long v[4] = {v0.x, v0.y, v1.x, v1.y};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    c[q] += (uint32_t)(v[q] & ((1ull << kPackCountBits) - 1));
                    e[q] += v[q] >> kPackCountBits;
                }
            } else {
                const uint4 v = *reinterpret_cast<const uint4*>(p.cnt_a + i + 4 * t);
                c[0] += v.x; c[1] += v.y; c[2] += v.z; c[3] += v.w;
            }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int cell = ENERGY ? (q >> 1) * 512 + 2 * t + (q & 1) : 4 * t + q;
            if (c[q]) atomicAdd(&s_hist[cell], c[q]);
            if (ENERGY && e[q]) atomicAdd(&s_en[cell], e[q]);
        }
    }
    __syncthreads();
    block_kth_from_top(s_hist, kBinsA, S.need, s_scan, s_res);
    const uint32_t bin_a = s_res[0];
    if (ENERGY) {
        unsigned long long e = 0;
        for (uint32_t b = tid; b < bin_a; b += kPickThreads) e += s_en[b];
        if (e) atomicAdd(&s_e, e);
        if (tid < 256) {
            const double w = wave_sum(part);                 // xor tree inside the wavefront
            if ((tid & 63) == 0) s_sum[tid >> 6] = w;
        }
        __syncthreads();
    }
    const uint32_t ex = S.tbin >> (23 - kHistShift);
    const int sh = 2 * ((int)(ex ? ex : 1u) - 150) + kPackEnergyShift;    // integer energy units -> x^2
    if (tid == 0) {
        const uint32_t need_a = S.need - s_res[1];
        T.sel[j].bin_a = bin_a;
        T.sel[j].need_a = need_a;
        if (ENERGY) {
            const uint32_t cnt = s_hist[bin_a];
            const double outside = ((s_sum[0] + s_sum[1]) + (s_sum[2] + s_sum[3])) + ldexp((double)s_e, sh);
            double inside = 0.0;      // dropped part of the sub-bin, in integer-energy units
            bool exact = false;
            if (cnt > need_a) {
                const uint32_t edge = (S.tbin << kHistShift) | (bin_a << 9);
                const double e_lo = (double)(packed_cell(edge) >> kPackCountBits);
                const double e_hi = (double)(packed_cell(edge | 0x1FFu) >> kPackCountBits);
                const double sum = (double)s_en[bin_a];
                const double drop = (double)(cnt - need_a), keep = (double)need_a;
                const double lower = fmax(drop * e_lo, sum - keep * e_hi);
                const double upper = drop * (sum / (double)cnt);
                inside = 0.5 * (lower + upper);
                const double half = 0.5 * (upper - lower);
                exact = ldexp(half, sh) > kInsideTolerance * (outside + ldexp(inside, sh));
            }
            if (exact) {
                s_outside = outside;
                s_exact[1] = (S.tbin << 10) | bin_a;
                s_exact[2] = need_a;
                s_exact[0] = 1;
            } else {
                p.errors[(size_t)l * p.stride + p.col[j]] = outside + ldexp(inside, sh);
            }
        }
    }
    if (!ENERGY) return;
    __syncthreads();
    if (!s_exact[0]) return;                                  // workgroup-uniform
    // ---- the rare exact route: last 9 bits of the candidates inside the sub-bin
    const uint32_t prefix = s_exact[1], need_a = s_exact[2];
    for (int b = tid; b < kBinsB; b += kPickThreads) s_hist[b] = 0;      // kBinsB <= kBinsA
    __syncthreads();
    {
        const DevLayer L = p.layers[l];
        const int lane = tid & 63, wave = tid >> 6;
        constexpr int kSub = kThreads / 64;
        const int npairs = (L.tile_end - L.tile_begin) * kSub;
        for (int pr = wave; pr < npairs; pr += kPickThreads / 64) {
            const int tt = L.tile_begin + pr / kSub, sub = pr % kSub;
            const uint32_t n = p.tinfo[tt].cnt[sub];
            const uint32_t* __restrict__ items = p.cand + T.cand_base + p.tiles[tt].pos + p.tinfo[tt].start[sub];
            for (uint32_t i = lane; i < n; i += 64) {
                const uint32_t pat = items[i];
                if ((pat >> 9) == prefix) atomicAdd(&s_hist[pat & (kBinsB - 1)], 1u);
            }
        }
    }
    __syncthreads();
    block_kth_from_top(s_hist, kBinsB, need_a, s_scan, s_res);
    const uint32_t thr_b = s_res[0], keep_at_thr = need_a - s_res[1];
    // dropped inside the sub-bin: every pattern below the threshold pattern, and the entries equal
    // to it that are not kept; a thread's cells in index order, then a fixed tree
    double mine = 0.0;
    for (uint32_t b = tid; b < (uint32_t)kBinsB; b += kPickThreads) {
        const uint32_t c = s_hist[b];
        const uint32_t n_drop = b < thr_b ? c : (b == thr_b ? c - keep_at_thr : 0u);
        const double v = (double)__uint_as_float((prefix << 9) | b);
        mine += (double)n_drop * (v * v);
    }
    const double w = wave_sum(mine);
    __syncthreads();                                          // s_sum was read by thread 0 above
    if ((tid & 63) == 0) s_sum[tid >> 6] = w;
    __syncthreads();
    if (tid == 0) {
        double inside = 0.0;
        for (int q = 0; q < kPickThreads / 64; ++q) inside += s_sum[q];
        p.errors[(size_t)l * p.stride + p.col[j]] = s_outside + inside;
    }
}

// Refinement level B (compress only): histogram of bits 8..0 of the candidates inside each k's
// level-A sub-bin.
__global__ __launch_bounds__(kRefThreads) void topk_refine_b_kernel(RefineParams p) {
    extern __shared__ unsigned char refine_smem[];
    const RefWork w = p.work[blockIdx.x];
    const TopkLayer& T = p.tl[w.layer];
    const int ntk = p.ntk;
    uint32_t* const s_cnt = reinterpret_cast<uint32_t*>(refine_smem);
    const int tid = threadIdx.x;
    for (int i = tid; i < ntk * kBinsB; i += kRefThreads) s_cnt[i] = 0;
    uint32_t prefix[kMaxTopk];       // top 22 bits (coarse bin, level-A bin) of each k
#pragma unroll
    for (int j = 0; j < kMaxTopk; ++j)
        prefix[j] = (j < ntk && T.sel[j].k) ? ((T.sel[j].tbin << 10) | T.sel[j].bin_a) : 0xFFFFFFFFu;
    __syncthreads();
    for_each_candidate(p, T, w.t0, w.t1, [&](uint32_t pat) {
        const uint32_t pre = pat >> 9;
#pragma unroll
        for (int j = 0; j < kMaxTopk; ++j)
            if (pre == prefix[j]) atomicAdd(&s_cnt[j * kBinsB + (pat & (kBinsB - 1))], 1u);
    });
    __syncthreads();
    uint32_t* const gc = p.cnt_b + (size_t)blockIdx.x * kMaxTopk * kBinsB;
    for (int i = tid; i < ntk * kBinsB; i += kRefThreads) gc[i] = s_cnt[i];
}

// One workgroup per (layer, requested k): exact threshold pattern and how many of the entries
// equal to it are kept.
__global__ __launch_bounds__(256) void topk_pick_b_kernel(RefineParams p) {
    __shared__ uint32_t s_hist[kBinsB];
    __shared__ uint32_t s_scan[256];
    __shared__ uint32_t s_res[2];
    const int l = blockIdx.x / kMaxTopk, j = blockIdx.x % kMaxTopk;
    TopkLayer& T = p.tl[l];
    if (j >= p.ntk || T.sel[j].k == 0) return;
    const TopkSel S = T.sel[j];
    const int2 wr = p.work_range[l];
    const int tid = threadIdx.x;
    {
        uint32_t c[2] = {0, 0};
        const size_t off = (size_t)j * kBinsB + tid;
#pragma unroll 8
        for (int wg = wr.x; wg < wr.y; ++wg) {
            const size_t i = (size_t)wg * kMaxTopk * kBinsB + off;
#pragma unroll
            for (int q = 0; q < 2; ++q) c[q] += p.cnt_b[i + 256 * q];
        }
#pragma unroll
        for (int q = 0; q < 2; ++q) s_hist[tid + 256 * q] = c[q];
    }
    __syncthreads();
    block_kth_from_top(s_hist, kBinsB, S.need_a, s_scan, s_res);
    if (tid == 0) {
        T.sel[j].thr = (S.tbin << kHistShift) | (S.bin_a << 9) | s_res[0];
        T.sel[j].ties_keep = S.need_a - s_res[1];
    }
}

// ---------------------------------------------------------------- compression kernels
// The compressor keeps the collector's partition: wavefront w of a tile owns the same contiguous
// element range it collected candidates from, so everything below is per wavefront and needs no
// workgroup barrier.

// Both kernels below are chains of dependent loads (tile -> layer record -> a few tens of
// candidates per wavefront), so a workgroup takes kSliceBatch consecutive tiles and every
// wavefront walks its slice of each of them side by side: the loads of one level are in flight
// together and the chain's latency is paid once per batch.
constexpr int kSliceBatch = 4;

// per (tile, wavefront): entries above the threshold, entries equal to it (from its candidates)
// KNOWN: the layer records say which layers take part and which selection record holds the threshold.
template <bool KNOWN>
__global__ __launch_bounds__(kThreads) void topk_count_kernel(const Tile* __restrict__ tiles, int n_tiles,
                                                               const DevLayer* __restrict__ layers,
                                                               const TopkLayer* __restrict__ tl,
                                                               const TopkTileInfo* __restrict__ tinfo,
                                                               const uint32_t* __restrict__ cand,
                                                               uint2* __restrict__ wavecnt) {
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int first = blockIdx.x * kSliceBatch;
    const uint32_t* items[kSliceBatch];
    uint32_t n[kSliceBatch], thr[kSliceBatch], gt[kSliceBatch], eq[kSliceBatch];
    bool active[kSliceBatch];
    uint32_t nmax = 0;
    // every load of a level is unconditional (indices clamped to the table), so that the levels
    // of the batch's chains are issued together
    int64_t pos[kSliceBatch], base[kSliceBatch];
    int layer[kSliceBatch];
    uint32_t start[kSliceBatch], k[kSliceBatch];
#pragma unroll
    for (int q = 0; q < kSliceBatch; ++q) {
        const int ti = min(first + q, n_tiles - 1);
        layer[q] = tiles[ti].layer;
        pos[q] = tiles[ti].pos;
        n[q] = tinfo[ti].cnt[wave];
        start[q] = tinfo[ti].start[wave];
    }
    int slot[kSliceBatch];
#pragma unroll
    for (int q = 0; q < kSliceBatch; ++q) {
        slot[q] = 0;
        if (KNOWN) {
            const DevLayer& L = layers[layer[q]];
            k[q] = (L.family == LGRECO_TOPK && L.slot >= 0 && L.slot < kMaxTopk) ? 1u : 0u;
            slot[q] = k[q] ? L.slot : 0;
        }
    }
#pragma unroll
    for (int q = 0; q < kSliceBatch; ++q) {
        const TopkLayer& T = tl[layer[q]];
        if (!KNOWN) k[q] = T.sel[0].k;
        thr[q] = T.sel[slot[q]].thr;
        base[q] = T.cand_base;
    }
#pragma unroll
    for (int q = 0; q < kSliceBatch; ++q) {
        // a layer that is not compressed with Top-K has k = 0 in its record (and no candidates)
        active[q] = first + q < n_tiles && k[q] != 0;
        n[q] = active[q] ? n[q] : 0u;
        items[q] = active[q] ? cand + base[q] + pos[q] + start[q] : cand;
        gt[q] = eq[q] = 0;
        nmax = max(nmax, n[q]);
    }
    for (uint32_t i = lane; i < nmax; i += 64) {
        uint32_t pat[kSliceBatch];
#pragma unroll
        for (int q = 0; q < kSliceBatch; ++q) pat[q] = i < n[q] ? items[q][i] : 0xFFFFFFFFu;   // never a pattern
#pragma unroll
        for (int q = 0; q < kSliceBatch; ++q) {
            gt[q] += (pat[q] != 0xFFFFFFFFu) & (pat[q] > thr[q]);
            eq[q] += pat[q] == thr[q];
        }
    }
#pragma unroll
    for (int q = 0; q < kSliceBatch; ++q) {
        for (int o = 1; o < 64; o <<= 1) {
            gt[q] += __shfl_xor(gt[q], o, 64);
            eq[q] += __shfl_xor(eq[q], o, 64);
        }
        if (lane == 0 && active[q])
            wavecnt[(size_t)(first + q) * (kThreads / 64) + wave] = make_uint2(gt[q], eq[q]);
    }
}

// per layer: exclusive prefix of the per-wavefront counts, in element order.  Both counts travel
// in one 64-bit word (each stays below 2^31: a layer has fewer elements than that) and a thread
// takes four consecutive entries, so a round of 1024 threads covers 4096 entries with one scan
// (the largest layer's entries, tiles x 4, are the critical path of this kernel); 256 threads when
// the chip is shared with another stream's kernel and a workgroup of 16 wavefronts would wait long
// for a compute unit with that much room.
template <int kScanThreads>
__global__ __launch_bounds__(kScanThreads) void topk_tilescan_kernel(const DevLayer* __restrict__ layers,
                                                            const uint2* __restrict__ wavecnt,
                                                            uint2* __restrict__ wavebase) {
    __shared__ unsigned long long s_tmp[kScanThreads / 64];
    const DevLayer L = layers[blockIdx.x];
    if (L.family != LGRECO_TOPK) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned long long run = 0;             // (entries above the threshold) << 32 | entries equal to it
    const int q0 = L.tile_begin * (kThreads / 64), q1 = L.tile_end * (kThreads / 64);
    for (int b = q0; b < q1; b += 4 * kScanThreads) {
        const int first = b + 4 * (int)threadIdx.x;
        unsigned long long c[4], mine = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint2 v = first + i < q1 ? wavecnt[first + i] : make_uint2(0, 0);
            c[i] = ((unsigned long long)v.x << 32) | v.y;
            mine += c[i];
        }
        unsigned long long inc = mine;
        for (int o = 1; o < 64; o <<= 1) {
            const unsigned long long n = __shfl_up(inc, o, 64);
            if (lane >= o) inc += n;
        }
        __syncthreads();                     // the previous round is done with s_tmp
        if (lane == 63) s_tmp[wave] = inc;
        __syncthreads();
        unsigned long long before = run, total = 0;
        for (int w = 0; w < kScanThreads / 64; ++w) {
            if (w < wave) before += s_tmp[w];
            total += s_tmp[w];
        }
        before += inc - mine;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (first + i < q1) wavebase[first + i] = make_uint2((uint32_t)(before >> 32), (uint32_t)before);
            before += c[i];
        }
        run += total;
    }
}

__device__ __forceinline__ uint32_t lanes_below(unsigned long long m, uint32_t add) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, add));
}

// Kept values and indices in ascending index order, from the candidates alone (every kept entry
// is a candidate, and a wavefront's candidates are stored in element order); the error feedback,
// already written as x everywhere by the collection pass, is zeroed at the kept entries (KNOWN:
// written as zero at every candidate by that pass, and set back to x at those not kept).
template <bool KNOWN>
__global__ __launch_bounds__(kThreads) void topk_emit_kernel(float* __restrict__ e,
                                                              const DevLayer* __restrict__ layers,
                                                              const Tile* __restrict__ tiles, int n_tiles,
                                                              const TopkLayer* __restrict__ tl,
                                                              const TopkTileInfo* __restrict__ tinfo,
                                                              const uint32_t* __restrict__ cand,
                                                              const uint32_t* __restrict__ cand_idx,
                                                              const uint2* __restrict__ wavecnt,
                                                              const uint2* __restrict__ wavebase,
                                                              uint8_t* __restrict__ payload, int x_in_e) {
    // x_in_e (KNOWN only): the main pass left the buffer as it was (x everywhere), so the kept
    // entries are zeroed here, as without KNOWN, and nothing is put back
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int first = blockIdx.x * kSliceBatch;
    struct Slice {
        const uint32_t* pats;
        const uint32_t* idxs;
        float* ef;
        float* values;
        uint32_t* indices;
        uint32_t n, thr, ties_keep, out, eq_seen;
        bool eq_all, eq_none;
    } S[kSliceBatch];
    uint32_t nmax = 0;
    // every load of a level is unconditional (indices clamped to the tables; the count arrays
    // cover every tile), so that the levels of the batch's chains are issued together
    int64_t pos[kSliceBatch];
    int layer[kSliceBatch];
    uint32_t start[kSliceBatch];
    uint2 cnt[kSliceBatch], before[kSliceBatch];
#pragma unroll
    for (int q = 0; q < kSliceBatch; ++q) {
        const int ti = min(first + q, n_tiles - 1);
        const size_t slot = (size_t)ti * (kThreads / 64) + wave;
        layer[q] = tiles[ti].layer;
        pos[q] = tiles[ti].pos;
        S[q].n = tinfo[ti].cnt[wave];
        start[q] = tinfo[ti].start[wave];
        cnt[q] = wavecnt[slot];
        before[q] = wavebase[slot];
    }
#pragma unroll
    for (int q = 0; q < kSliceBatch; ++q) {
        const DevLayer& L = layers[layer[q]];
        const TopkLayer& T = tl[layer[q]];
        const bool active = first + q < n_tiles && L.family == LGRECO_TOPK &&
                            (!KNOWN || (L.slot >= 0 && L.slot < kMaxTopk));
        const int64_t off = active ? T.cand_base + pos[q] + start[q] : 0;
        const TopkSel& Sel = T.sel[(KNOWN && active) ? L.slot : 0];
        const uint32_t keep_eq = Sel.ties_keep;
        S[q].pats = cand + off;
        S[q].idxs = cand_idx + off;
        S[q].ef = e + L.offset;
        S[q].values = reinterpret_cast<float*>(payload + L.payload);
        S[q].indices = reinterpret_cast<uint32_t*>(payload + L.payload) + Sel.k;
        S[q].n = active ? S[q].n : 0u;
        S[q].thr = Sel.thr;
        S[q].ties_keep = keep_eq;
        // equal entries: global rank r (in index order) is kept iff r < ties_keep
        S[q].eq_all = before[q].y + cnt[q].y <= keep_eq;
        S[q].eq_none = before[q].y >= keep_eq;
        S[q].out = before[q].x + min(before[q].y, keep_eq);
        S[q].eq_seen = before[q].y;
        nmax = max(nmax, S[q].n);
    }
    for (uint32_t i0 = 0; i0 < nmax; i0 += 64) {
        const uint32_t i = i0 + lane;
        uint32_t pat[kSliceBatch], ix[kSliceBatch];
#pragma unroll
        for (int q = 0; q < kSliceBatch; ++q) {
            const bool ok = i < S[q].n;
            pat[q] = ok ? S[q].pats[i] : 0u;
            ix[q] = ok ? S[q].idxs[i] : 0u;
        }
#pragma unroll
        for (int q = 0; q < kSliceBatch; ++q) {
            if (i0 >= S[q].n) continue;                      // wavefront-uniform
            const bool ok = i < S[q].n;
            bool keep = ok && pat[q] > S[q].thr;
            const bool eq = ok && pat[q] == S[q].thr;
            if (S[q].eq_all) {
                keep = keep || eq;
            } else if (!S[q].eq_none) {
                const unsigned long long bq = __ballot(eq);
                if (eq) keep = S[q].eq_seen + lanes_below(bq, 0u) < S[q].ties_keep;
                S[q].eq_seen += (uint32_t)__popcll(bq);
            }
            const unsigned long long kq = __ballot(keep);
            if (keep) {
                const uint32_t pos = S[q].out + lanes_below(kq, 0u);
                S[q].values[pos] = __uint_as_float(pat[q] | (ix[q] & 0x80000000u));
                S[q].indices[pos] = ix[q] & 0x7FFFFFFFu;
                if (!KNOWN || x_in_e) S[q].ef[ix[q] & 0x7FFFFFFFu] = 0.0f;
            } else if (KNOWN && !x_in_e && ok) {
                // the main pass wrote zero for every candidate: the ones that are not kept get x back
                S[q].ef[ix[q] & 0x7FFFFFFFu] = __uint_as_float(pat[q] | (ix[q] & 0x80000000u));
            }
            S[q].out += (uint32_t)__popcll(kq);
        }
    }
}

// ------------------------------------------------------------------------ host side
#define TK_CHECK(expr)                     \
    do {                                   \
        hipError_t _e = (expr);            \
        if (_e != hipSuccess) return _e;   \
    } while (0)

hipError_t topk_scratch_create(TopkScratch* t, int64_t max_elems, int max_layers, int max_tiles) {
    t->max_elems = max_elems;
    t->max_layers = max_layers;
    t->max_tiles = max_tiles;
    TK_CHECK(hipMalloc(&t->d_hist, sizeof(uint32_t) * 2 * (size_t)max_layers * kHistBins));   // exact + sample
    // Between calls the exact histogram is all zero: cleared here once, and by the last scan of every
    // call for the layers that call counted.  hist_clean is false only after a call that failed midway.
    TK_CHECK(hipMemset(t->d_hist, 0, sizeof(uint32_t) * 2 * (size_t)max_layers * kHistBins));
    t->hist_clean = true;
    TK_CHECK(hipMalloc(&t->d_tl, sizeof(TopkLayer) * (size_t)max_layers));
    // counts of the known-threshold compression: all zero between calls (the pick kernel clears what it reads)
    TK_CHECK(hipMalloc(&t->d_cnt_known, sizeof(uint32_t) * (size_t)max_layers * kBinsB));
    TK_CHECK(hipMemset(t->d_cnt_known, 0, sizeof(uint32_t) * (size_t)max_layers * kBinsB));
    TK_CHECK(hipMalloc(&t->d_cand, sizeof(uint32_t) * (size_t)max_elems));
    TK_CHECK(hipMalloc(&t->d_cand_idx, sizeof(uint32_t) * (size_t)max_elems));
    TK_CHECK(hipMalloc(&t->d_kept, sizeof(uint32_t) * (size_t)max_elems));
    TK_CHECK(hipMalloc(&t->d_kept_idx, sizeof(uint32_t) * (size_t)max_elems));
    TK_CHECK(hipMalloc(&t->d_tinfo_kept, sizeof(TopkTileInfo) * (size_t)max_tiles));
    TK_CHECK(hipMalloc(&t->d_lo, sizeof(uint32_t) * (size_t)max_layers));
    for (int i = 0; i < 2; ++i) TK_CHECK(hipMalloc(&t->d_hint[i], sizeof(uint32_t) * (size_t)max_layers));
    TK_CHECK(hipMalloc(&t->d_tilecnt, sizeof(uint2) * (size_t)max_tiles * (kThreads / 64)));
    TK_CHECK(hipMalloc(&t->d_tilebase, sizeof(uint2) * (size_t)max_tiles * (kThreads / 64)));
    TK_CHECK(hipMalloc(&t->d_tinfo, sizeof(TopkTileInfo) * (size_t)max_tiles));
    TK_CHECK(hipMalloc(&t->d_base_part, sizeof(double) * (size_t)max_tiles));
    t->max_work = (int)(max_elems / ((int64_t)kRefTiles * kTile)) + 2 * max_layers + 2 + 2 * kRefSlots;   // see topk_begin
    TK_CHECK(hipMalloc(&t->d_below_part, sizeof(double) * (size_t)t->max_work * kMaxTopk));
    t->ref_words = (size_t)t->max_work * kMaxTopk * (3 * kBinsA + kBinsB);      // u64 + u32 level A, u32 level B
    TK_CHECK(hipMalloc(&t->d_ref, sizeof(uint32_t) * t->ref_words));
    // control block layout (every part a multiple of 16 bytes)
    const size_t o_k = 0;
    const size_t o_base = o_k + sizeof(uint32_t) * (size_t)max_layers * kMaxTopk;
    const size_t o_range = o_base + (sizeof(int64_t) * (size_t)max_layers + 15) / 16 * 16;
    const size_t o_work = o_range + (sizeof(int2) * (size_t)max_layers + 15) / 16 * 16;
    t->ctl_bytes = o_work + sizeof(RefWork) * (size_t)t->max_work;
    t->ctl_off[0] = o_k; t->ctl_off[1] = o_base; t->ctl_off[2] = o_range; t->ctl_off[3] = o_work;
    TK_CHECK(hipHostMalloc(&t->h_ctl, t->ctl_bytes, hipHostMallocDefault));
    TK_CHECK(hipEventCreateWithFlags(&t->ctl_copied, hipEventDisableTiming));
    std::memset(t->h_ctl, 0, t->ctl_bytes);
    for (int i = 0; i < 2; ++i) {
        TK_CHECK(hipMalloc(&t->d_ctl[i], t->ctl_bytes));
        t->h_ctl_last[i] = static_cast<uint8_t*>(std::malloc(t->ctl_bytes));
        if (!t->h_ctl_last[i]) return hipErrorOutOfMemory;
        t->ctl_last_bytes[i] = 0;
    }
    t->h_k = reinterpret_cast<uint32_t*>(t->h_ctl + o_k);
    t->h_cand_base = reinterpret_cast<int64_t*>(t->h_ctl + o_base);
    t->h_work_range = t->h_ctl + o_range;
    t->h_work = t->h_ctl + o_work;
    return hipSuccess;
}

void topk_scratch_destroy(TopkScratch* t) {
    (void)hipFree(t->d_hist);
    (void)hipFree(t->d_tl);
    (void)hipFree(t->d_cnt_known);
    (void)hipFree(t->d_cand);
    (void)hipFree(t->d_cand_idx);
    (void)hipFree(t->d_kept);
    (void)hipFree(t->d_kept_idx);
    (void)hipFree(t->d_tinfo_kept);
    (void)hipFree(t->d_lo);
    for (int i = 0; i < 2; ++i) (void)hipFree(t->d_hint[i]);
    (void)hipFree(t->d_tilecnt);
    (void)hipFree(t->d_tilebase);
    (void)hipFree(t->d_tinfo);
    (void)hipFree(t->d_base_part);
    (void)hipFree(t->d_below_part);
    (void)hipFree(t->d_ref);
    for (int i = 0; i < 2; ++i) {
        (void)hipFree(t->d_ctl[i]);
        std::free(t->h_ctl_last[i]);
    }
    (void)hipHostFree(t->h_ctl);
    if (t->ctl_copied) (void)hipEventDestroy(t->ctl_copied);
    *t = TopkScratch{};
}

// The pinned control block may be written again once the last upload that was queued from it has
// executed (a call may return, and a stream may be busy, with that copy still pending).
static hipError_t ctl_writable(TopkScratch* t) {
    if (t->ctl_pending) {
        TK_CHECK(hipEventSynchronize(t->ctl_copied));
        t->ctl_pending = false;
    }
    return hipSuccess;
}

// One upload of the control block up to the last work item, skipped when this slot's device copy
// already holds the same bytes.
static hipError_t upload_ctl(TopkScratch* t, int slot, hipStream_t s, bool* changed = nullptr) {
    uint8_t* const d = t->d_ctl[slot];
    t->d_k = reinterpret_cast<uint32_t*>(d + t->ctl_off[0]);
    t->d_cand_base = reinterpret_cast<int64_t*>(d + t->ctl_off[1]);
    t->d_work_range = d + t->ctl_off[2];
    t->d_work = d + t->ctl_off[3];
    const size_t used = t->ctl_off[3] + sizeof(RefWork) * (size_t)std::max(t->n_work, 1);
    const bool differs = used != t->ctl_last_bytes[slot] || std::memcmp(t->h_ctl, t->h_ctl_last[slot], used) != 0;
    if (differs) {
        TK_CHECK(hipMemcpyAsync(d, t->h_ctl, used, hipMemcpyHostToDevice, s));
        // the copy reads the pinned block when it executes: the next writer waits for this event
        TK_CHECK(hipEventRecord(t->ctl_copied, s));
        t->ctl_pending = true;
        std::memcpy(t->h_ctl_last[slot], t->h_ctl, used);
        t->ctl_last_bytes[slot] = used;
    }
    if (changed) *changed = differs;
    return hipSuccess;
}

// A further group of requested k for the data that was just collected (more candidates than one
// pass resolves): only the k table changes.  The group must not ask for more entries than the
// first one did, so every threshold lies at or above the collection bound.
hipError_t topk_regroup(TopkScratch* t, int L, const uint32_t* ks, int slot, hipStream_t s) {
    TK_CHECK(ctl_writable(t));
    for (size_t i = 0; i < (size_t)L * kMaxTopk; ++i) t->h_k[i] = ks[i];
    return upload_ctl(t, slot, s);
}

// Upload the requested k per (layer, candidate) (0 = layer inactive), clear both histograms, take
// the sample and predict the collection bound of every layer.
hipError_t topk_begin(TopkScratch* t, const float* g, const float* e, const DevLayer* d_layers,
                      const DevLayer* h_layers, const Tile* d_tiles, int L, int n_tiles, int tile_elems,
                      const uint32_t* ks, int ntk, int slot, Timing* tm, hipStream_t s) {
    (void)n_tiles;
    // Tiles per work item of the sample / refinement kernels: 2^19 elements, fewer when that would
    // leave part of the chip without a work item (two 1024-thread workgroups per CU, kRefSlots in
    // all): a work item's time is proportional to its candidates, and a small problem's chain is as
    // long as its largest item.
    int group = kRefTiles * (kTile / tile_elems);
    {
        int64_t active = 0;
        for (int l = 0; l < L; ++l)
            if (ks[(size_t)l * kMaxTopk]) active += h_layers[l].tile_end - h_layers[l].tile_begin;
        group = (int)std::max<int64_t>(1, std::min<int64_t>(group, active / kRefSlots));
    }
    TK_CHECK(ctl_writable(t));
    int64_t base = 0;
    RefWork* const work = (RefWork*)t->h_work;
    int2* const wrange = (int2*)t->h_work_range;
    int nw = 0, max_items = 0;
    for (int l = 0; l < L; ++l) {
        for (int j = 0; j < kMaxTopk; ++j) t->h_k[(size_t)l * kMaxTopk + j] = ks[(size_t)l * kMaxTopk + j];
        // the refinement relies on this order: an active layer asks for ntk values of k, none larger
        // than the one before it
        if (ks[(size_t)l * kMaxTopk])
            for (int j = 1; j < ntk; ++j)
                if (ks[(size_t)l * kMaxTopk + j] == 0 || ks[(size_t)l * kMaxTopk + j] > ks[(size_t)l * kMaxTopk + j - 1])
                    return hipErrorInvalidValue;
        t->h_cand_base[l] = base;
        wrange[l].x = nw;
        if (ks[(size_t)l * kMaxTopk]) {
            base += h_layers[l].numel;
            for (int t0 = h_layers[l].tile_begin; t0 < h_layers[l].tile_end; t0 += group) {
                if (nw >= t->max_work) return hipErrorInvalidValue;      // cannot happen: see max_work
                work[nw++] = RefWork{l, t0, std::min(h_layers[l].tile_end, t0 + group), 0};
            }
        }
        wrange[l].y = nw;
        max_items = std::max(max_items, wrange[l].y - wrange[l].x);
    }
    t->n_work = nw;
    t->max_items = max_items;
    t->cand_has_idx = false;
    bool changed = true;
    TK_CHECK(upload_ctl(t, slot, s, &changed));
    t->cur_slot = slot;
    Section sec(tm, "topk_sample");
    // the sample's histogram has its own half of the buffer, whatever L is: a call never leaves
    // counts where a later call with more layers expects a cleared exact histogram
    uint32_t* const shist = t->d_hist + (size_t)t->max_layers * kHistBins;
    auto fill = [&](uint32_t* dst, size_t n) {
        hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)std::min<size_t>((n + 255) / 256, 2048)), dim3(256), 0, s,
                           dst, n, 0u);
        return hipGetLastError();
    };
    if (t->reuse_thresholds && t->hint_valid[slot] && !changed) {
        // Same layers and the same k as the previous call of this kind: start from the thresholds
        // it found, a margin lower, instead of sampling.  The scan still checks the bound against
        // the exact histogram and collects a layer again if the data moved past the margin.  The
        // previous call's last scan left the histogram cleared, so no kernel runs before the main pass.
        t->lo_src = t->d_hint[slot];
        if (!t->hist_clean) TK_CHECK(fill(t->d_hist, (size_t)t->max_layers * kHistBins));
        t->hist_clean = false;
        return hipSuccess;
    }
    t->lo_src = t->d_lo;
    t->hint_valid[slot] = false;
    if (!t->hist_clean) TK_CHECK(fill(t->d_hist, (size_t)t->max_layers * kHistBins));
    t->hist_clean = false;
    TK_CHECK(fill(shist, (size_t)L * kHistBins));
    if (nw > 0) {
        hipLaunchKernelGGL(topk_sample_kernel, dim3(nw), dim3(kThreads), 0, s, g, e, d_layers, d_tiles,
                           (const RefWork*)t->d_work, std::max(1, tile_elems / kChunk / kSampleEvery), shist);
        TK_CHECK(hipGetLastError());
    }
    hipLaunchKernelGGL(topk_predict_kernel, dim3(L), dim3(256), 0, s, (const uint32_t*)shist,
                       (const uint32_t*)t->d_k, ntk, d_layers, t->d_lo);
    return hipGetLastError();
}

static CollectParams collect_params(TopkScratch* t, const float* g, const float* e, const DevLayer* d_layers,
                                    const Tile* d_tiles) {
    CollectParams p{};
    p.g = g;
    p.e = e;
    p.layers = d_layers;
    p.tiles = d_tiles;
    p.ks = t->d_k;
    p.tl = (const TopkLayer*)t->d_tl;
    p.lo = t->lo_src;
    p.hist = t->d_hist;
    p.cand = t->d_cand;
    p.cand_idx = t->d_cand_idx;
    p.cand_base = t->d_cand_base;
    p.tinfo = (TopkTileInfo*)t->d_tinfo;
    p.base_part = t->d_base_part;
    return p;
}

// main pass without quantization candidates: histogram + collection in one read.  ef_out != null
// (compress): also records index and sign of every candidate and writes x to the error feedback.
hipError_t topk_collect(TopkScratch* t, const float* g, const float* e, float* ef_out, const DevLayer* d_layers,
                        const Tile* d_tiles, int n_tiles, hipStream_t s, Section* sec, float* x_out) {
    if (n_tiles <= 0) return hipSuccess;
    CollectParams p = collect_params(t, g, e, d_layers, d_tiles);
    p.ef_out = ef_out;
    p.x_out = ef_out ? nullptr : x_out;        // profile only: x is left where the compression will look for it
    // ... and that compression works from the candidates, so it needs their indices and signs
    p.record_idx = p.x_out ? 1 : 0;
    t->cand_has_idx = p.record_idx != 0;
    if (ef_out)
        launch_timed(sec, true, true, topk_collect_kernel<true, true>, dim3(n_tiles), dim3(kThreads), 0, s, p);
    else
        launch_timed(sec, true, true, topk_collect_kernel<true, false>, dim3(n_tiles), dim3(kThreads), 0, s, p);
    return hipGetLastError();
}

// exact threshold bins; layers whose predicted bound was too high are collected again
hipError_t topk_select(TopkScratch* t, const float* g, const float* e, float* ef_out, const DevLayer* d_layers,
                       const Tile* d_tiles, int L, int n_tiles, int ntk, bool first_group, bool last_group,
                       Timing* tm, hipStream_t s, const QuantReduce* quant) {
    {
        Section sec(tm, "topk_scan");
        // the first group of a call holds the lowest thresholds: it leaves the bound for the next call
        uint32_t* const hint = (first_group && t->reuse_thresholds) ? t->d_hint[t->cur_slot] : nullptr;
        ScanReduce red{};
        if (quant) {
            red.partials = quant->partials;
            red.errors = quant->errors;
            red.layers = d_layers;
            red.stride = quant->stride;
            red.cols.n = std::min(quant->ncols, (int)kMaxQuant);
            for (int i = 0; i < red.cols.n; ++i) red.cols.col[i] = quant->cols[i];
        }
        hipLaunchKernelGGL(topk_scan_kernel, dim3(quant ? 2 * L : L), dim3(256), 0, s, t->d_hist,
                           (const uint32_t*)t->d_k, ntk, (const int64_t*)t->d_cand_base,
                           first_group ? t->lo_src : (const uint32_t*)t->d_lo, t->d_lo, (TopkLayer*)t->d_tl, hint,
                           last_group ? 1 : 0, L, red);
        TK_CHECK(hipGetLastError());
        if (hint) t->hint_valid[t->cur_slot] = true;
        if (last_group) t->hist_clean = true;
        t->lo_src = t->d_lo;                     // a second collection uses the bound the scan wrote
    }
    // Layers whose predicted bound was too high (flagged by the scan; none in the usual call) are
    // collected a second time with the exact bound, by the first refinement kernel's workgroups,
    // each for its own tiles: what that collection reads and writes is noted here.  It reads
    // x = g + e again; in compress e already holds x, so g is not added.
    t->rc_g = ef_out ? ef_out : g;
    t->rc_e = ef_out ? nullptr : e;
    t->rc_ef_out = ef_out;
    (void)n_tiles;
    return hipSuccess;
}

hipError_t topk_finalize(TopkScratch* t, const DevLayer* d_layers, const Tile* d_tiles, int L, int ntk,
                         const int* col, double* d_errors, int stride, Timing* tm, hipStream_t s) {
    if (t->n_work <= 0) return hipSuccess;
    // the pick kernel's workgroups: small ones, so that all of them run at once, unless a layer has
    // so many partial histograms to sum that its workgroup alone would outlast the rest
    const bool wide_pick = t->max_items > 64;
    RefineParams p{};
    p.tl = (TopkLayer*)t->d_tl;
    p.layers = d_layers;
    p.tiles = d_tiles;
    p.tinfo = (const TopkTileInfo*)t->d_tinfo;
    p.cand = t->d_cand;
    p.work = (const RefWork*)t->d_work;
    p.work_range = (const int2*)t->d_work_range;
    p.base_part = t->d_base_part;
    p.below_part = t->d_below_part;
    // per-workgroup partial histograms: [packed cells A (u64)][counts A][counts B]
    const size_t na = (size_t)t->max_work * kMaxTopk * kBinsA;
    p.cell_a = reinterpret_cast<unsigned long long*>(t->d_ref);
    p.cnt_a = t->d_ref + 2 * na;
    p.cnt_b = p.cnt_a + na;
    p.errors = d_errors;
    p.stride = stride;
    p.ntk = ntk;
    for (int j = 0; j < ntk; ++j) p.col[j] = col ? col[j] : 0;
    p.rc = collect_params(t, t->rc_g, t->rc_e, d_layers, d_tiles);
    p.rc.ef_out = t->rc_ef_out;
    p.rc.record_idx = (!t->rc_ef_out && t->cand_has_idx) ? 1 : 0;
    Section sec(tm, "topk_refine");
    if (d_errors) {       // profile: level A gives the dropped energy, no exact threshold is needed
        const size_t lds = refine_a_lds(ntk, true);
        static bool configured[kMaxTopk + 1] = {};   // the dynamic LDS limit is raised once per variant
#define LG_REFINE_A(N)                                                                                   \
    case N:                                                                                              \
        if (!configured[N]) {                                                                            \
            TK_CHECK(hipFuncSetAttribute((const void*)topk_refine_a_kernel<N>,                           \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));         \
            configured[N] = true;                                                                        \
        }                                                                                                \
        hipLaunchKernelGGL(topk_refine_a_kernel<N>, dim3(t->n_work), dim3(kRefThreads), lds, s, p);      \
        break;
        switch (ntk) {
            LG_REFINE_A(1) LG_REFINE_A(2) LG_REFINE_A(3) LG_REFINE_A(4)
            LG_REFINE_A(5) LG_REFINE_A(6) LG_REFINE_A(7) LG_REFINE_A(8)
            default: return hipErrorInvalidValue;
        }
#undef LG_REFINE_A
        TK_CHECK(hipGetLastError());
        if (wide_pick) hipLaunchKernelGGL((topk_pick_a_kernel<true, 512>), dim3(L * ntk), dim3(512), 0, s, p);
        else hipLaunchKernelGGL((topk_pick_a_kernel<true, 256>), dim3(L * ntk), dim3(256), 0, s, p);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(topk_refine_a_kernel<0>, dim3(t->n_work), dim3(kRefThreads), refine_a_lds(ntk, false), s, p);
    TK_CHECK(hipGetLastError());
    if (wide_pick) hipLaunchKernelGGL((topk_pick_a_kernel<false, 512>), dim3(L * ntk), dim3(512), 0, s, p);
    else hipLaunchKernelGGL((topk_pick_a_kernel<false, 256>), dim3(L * ntk), dim3(256), 0, s, p);
    TK_CHECK(hipGetLastError());
    hipLaunchKernelGGL(topk_refine_b_kernel, dim3(t->n_work), dim3(kRefThreads), (size_t)ntk * kBinsB * 4, s, p);
    TK_CHECK(hipGetLastError());
    hipLaunchKernelGGL(topk_pick_b_kernel, dim3(L * kMaxTopk), dim3(256), 0, s, p);
    return hipGetLastError();
}

// x_in_e: g is the error-feedback buffer itself, which already holds x = fl32(g + e) (nothing is added)
hipError_t topk_compress(TopkScratch* t, const float* g, float* e, const DevLayer* d_layers,
                         const DevLayer* h_layers, const Tile* d_tiles, int L, int n_tiles, int tile_elems,
                         uint8_t* payload, Timing* tm, hipStream_t s, bool x_in_e) {
    std::vector<uint32_t> ks((size_t)L * kMaxTopk, 0u);
    for (int l = 0; l < L; ++l)
        if (h_layers[l].family == LGRECO_TOPK) ks[(size_t)l * kMaxTopk] = (uint32_t)h_layers[l].iparam;
    const float* const e_in = x_in_e ? nullptr : e;
    TK_CHECK(topk_begin(t, g, e_in, d_layers, h_layers, d_tiles, L, n_tiles, tile_elems, ks.data(), 1, 1, tm, s));
    {
        Section sec(tm, "topk_collect", true);
        TK_CHECK(topk_collect(t, g, e_in, e, d_layers, d_tiles, n_tiles, s, &sec));
    }
    TK_CHECK(topk_select(t, g, e_in, e, d_layers, d_tiles, L, n_tiles, 1, true, true, tm, s, nullptr));
    TK_CHECK(topk_finalize(t, d_layers, d_tiles, L, 1, nullptr, nullptr, 0, tm, s));
    {
        Section sec(tm, "topk_count");
        hipLaunchKernelGGL(topk_count_kernel<false>, dim3((n_tiles + kSliceBatch - 1) / kSliceBatch), dim3(kThreads), 0,
                           s, d_tiles, n_tiles, d_layers, (const TopkLayer*)t->d_tl, (const TopkTileInfo*)t->d_tinfo,
                           (const uint32_t*)t->d_cand, (uint2*)t->d_tilecnt);
        TK_CHECK(hipGetLastError());
    }
    {
        Section sec(tm, "topk_tilescan");
        hipLaunchKernelGGL(topk_tilescan_kernel<1024>, dim3(L), dim3(1024), 0, s, d_layers, (const uint2*)t->d_tilecnt,
                           (uint2*)t->d_tilebase);
        TK_CHECK(hipGetLastError());
    }
    {
        Section sec(tm, "topk_emit");
        hipLaunchKernelGGL(topk_emit_kernel<false>, dim3((n_tiles + kSliceBatch - 1) / kSliceBatch), dim3(kThreads), 0, s, e,
                           d_layers, d_tiles, n_tiles, (const TopkLayer*)t->d_tl,
                           (const TopkTileInfo*)t->d_tinfo, (const uint32_t*)t->d_cand,
                           (const uint32_t*)t->d_cand_idx, (const uint2*)t->d_tilecnt,
                           (const uint2*)t->d_tilebase, payload, 0);
        TK_CHECK(hipGetLastError());
    }
    return hipSuccess;
}

// Compression of the Top-K layers right behind a profile of the same data (the one-call entry
// point): the layer records the solver kernel wrote say which layers take part and which of the
// profile's selection records (threshold bin, sub-bin, entries to take) applies, so nothing is
// sampled, no histogram is built and nothing depends on the host knowing the assignment.
// x_in_e (the profile left x in the error-feedback buffer and recorded where its candidates are):
// what lies at or above the sub-bin's lower edge is taken from the profile's candidates, the
// sub-bin's entries counted by their last 9 bits, and the data is not read at all.  Otherwise one
// pass over g and e writes x to the error feedback and collects the same set.  Then the exact
// threshold, the per-wavefront counts, their scan and the ordered emit, as in topk_compress.
hipError_t topk_compress_known(TopkScratch* t, const float* g, float* e, const DevLayer* d_layers,
                               const Tile* d_tiles, int L, int n_tiles, uint8_t* payload, Timing* tm, hipStream_t s,
                               bool x_in_e, bool shared_chip) {
    if (n_tiles <= 0) return hipSuccess;
    // the profile's control block (slot 0) holds every layer's candidate region
    uint8_t* const d = t->d_ctl[0];
    CollectParams p{};
    p.g = g;
    p.e = e;
    p.ef_out = e;
    p.layers = d_layers;
    p.tiles = d_tiles;
    p.tl = (const TopkLayer*)t->d_tl;
    p.cand = t->d_cand;
    p.cand_idx = t->d_cand_idx;
    p.cand_base = reinterpret_cast<const int64_t*>(d + t->ctl_off[1]);
    p.tinfo = (TopkTileInfo*)t->d_tinfo;
    p.base_part = t->d_base_part;
    p.cnt_b = t->d_cnt_known;
    const TopkTileInfo* tinfo = (const TopkTileInfo*)t->d_tinfo;
    const uint32_t* cand = t->d_cand;
    const uint32_t* cand_idx = t->d_cand_idx;
    if (x_in_e) {
        // the profile recorded where its candidates are: what is kept is taken from them
        if (!t->cand_has_idx) return hipErrorInvalidValue;
        FilterParams f{};
        f.layers = d_layers;
        f.tiles = d_tiles;
        f.tl = p.tl;
        f.cand_base = p.cand_base;
        f.tinfo = tinfo;
        f.cand = cand;
        f.cand_idx = cand_idx;
        f.tinfo_out = (TopkTileInfo*)t->d_tinfo_kept;
        f.cand_out = t->d_kept;
        f.cand_idx_out = t->d_kept_idx;
        f.cnt_b = t->d_cnt_known;
        Section sec(tm, "topk_filter", true);
        launch_timed(&sec, true, true, topk_filter_known_kernel, dim3(n_tiles), dim3(kThreads), 0, s, f);
        TK_CHECK(hipGetLastError());
        tinfo = f.tinfo_out;
        cand = f.cand_out;
        cand_idx = f.cand_idx_out;
    } else {
        Section sec(tm, "topk_collect", true);
        launch_timed(&sec, true, true, topk_collect_known_kernel, dim3(n_tiles), dim3(kThreads), 0, s, p);
        TK_CHECK(hipGetLastError());
    }
    {
        Section sec(tm, "topk_pick");
        hipLaunchKernelGGL(topk_pick_known_kernel, dim3(L), dim3(256), 0, s, d_layers, (TopkLayer*)t->d_tl,
                           t->d_cnt_known);
        TK_CHECK(hipGetLastError());
    }
    {
        Section sec(tm, "topk_count");
        hipLaunchKernelGGL(topk_count_kernel<true>, dim3((n_tiles + kSliceBatch - 1) / kSliceBatch), dim3(kThreads), 0,
                           s, d_tiles, n_tiles, d_layers, (const TopkLayer*)t->d_tl, tinfo, cand, (uint2*)t->d_tilecnt);
        TK_CHECK(hipGetLastError());
    }
    {
        Section sec(tm, "topk_tilescan");
        if (shared_chip)
            hipLaunchKernelGGL(topk_tilescan_kernel<256>, dim3(L), dim3(256), 0, s, d_layers, (const uint2*)t->d_tilecnt,
                               (uint2*)t->d_tilebase);
        else
            hipLaunchKernelGGL(topk_tilescan_kernel<1024>, dim3(L), dim3(1024), 0, s, d_layers,
                               (const uint2*)t->d_tilecnt, (uint2*)t->d_tilebase);
        TK_CHECK(hipGetLastError());
    }
    {
        Section sec(tm, "topk_emit");
        hipLaunchKernelGGL(topk_emit_kernel<true>, dim3((n_tiles + kSliceBatch - 1) / kSliceBatch), dim3(kThreads), 0, s, e,
                           d_layers, d_tiles, n_tiles, (const TopkLayer*)t->d_tl, tinfo, cand, cand_idx,
                           (const uint2*)t->d_tilecnt,
                           (const uint2*)t->d_tilebase, payload, x_in_e ? 1 : 0);
        TK_CHECK(hipGetLastError());
    }
    return hipSuccess;
}

}  // namespace lgreco

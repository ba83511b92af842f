// Layer x error-bin dynamic program of Algorithm 1 and its back-trace, one workgroup.
//
// DP[l][e] = min over candidates c with bin(l,c) <= e of DP[l-1][e - bin(l,c)] + size(l,c),
// starting from a virtual row DP[0] = (0, inf, inf, ...).  Layers are sequential; the bins of a
// row are independent, so the 1024 threads each own a few bins (adjacent pairs, strided by 2048) and keep
// the new row in registers while the previous row sits in LDS.  Candidates are visited in index
// order with a strict '<' (lowest index wins ties); the back-trace starts from the lowest e among
// the minima of the last row.  PD (arg-min per cell) goes to global memory, one byte per cell.
//
// The host hands over, per layer, the list of usable candidates with equal bins merged (for one
// bin only the smallest size can win, the lowest index among equals; merging keeps the result
// identical, tie-breaks included) and entries that another entry beats in both bin and size left
// out (they cannot lie on the traced-back path).  A layer whose list is a single entry with bin 0 adds a
// constant to the whole row: the host fixes its choice and leaves it out, so L here counts the
// swept layers only.  Entry lists are staged through LDS 32 layers at a time.  Costs are 32-bit when the sum of every layer's largest size stays below 2^30, else
// 64-bit; "infinity" is 2^30 (2^62), so inf + size never overflows and never beats a real value.
#include <cstdlib>

#include "internal.h"

namespace lgreco {


template <typename T> struct DpInf;
template <> struct DpInf<uint32_t> { static constexpr uint32_t v = 1u << 30; };
template <> struct DpInf<int64_t> { static constexpr int64_t v = (int64_t)1 << 62; };

__device__ __forceinline__ uint32_t readlane_u32(uint32_t v, int lane) {
    return (uint32_t)__builtin_amdgcn_readlane((int)v, lane);
}
__device__ __forceinline__ int64_t readlane_i64(int64_t v, int lane) {
    const uint32_t lo = readlane_u32((uint32_t)v, lane);
    const uint32_t hi = readlane_u32((uint32_t)((uint64_t)v >> 32), lane);
    return (int64_t)(((uint64_t)hi << 32) | lo);
}
template <typename T> __device__ __forceinline__ T readlane_t(T v, int lane);
template <> __device__ __forceinline__ uint32_t readlane_t<uint32_t>(uint32_t v, int lane) {
    return readlane_u32(v, lane);
}
template <> __device__ __forceinline__ int64_t readlane_t<int64_t>(int64_t v, int lane) {
    return readlane_i64(v, lane);
}

constexpr int kDpStageEntries = 1024;   // entries staged in LDS at a time (16 KB)
constexpr int kDpStageMax = 32;         // at most this many layers per stage
constexpr int kDpMaxGroups = 8;         // layer groups swept side by side (a power of two)

// Thread t owns KMAX cells.  With an even KMAX they come in adjacent pairs (2t, 2t+1), (2t, 2t+1) +
// 2*threads, ...: the two reads row[e - b], row[e + 1 - b] of a pair are one ds_read2_b32 and the
// 64 lanes of a wavefront cover 128 consecutive cells without bank conflicts.
template <int KMAX, int THREADS>
__device__ __forceinline__ int dp_cell(int tid, int k) {
    return KMAX % 2 == 0 ? 2 * tid + (k & 1) + (k >> 1) * 2 * THREADS : tid + k * THREADS;
}

// Sweep of the swept layers [l_begin, l_end) over the row in LDS (the caller has written the row the
// first of them starts from): per layer the new row is formed in registers from the entries'
// shifted reads, then written back together with the arg-min bytes PD[l][0..D].  With s_bins the
// bin of every entry is also kept in LDS for the back-trace.  Every thread of the block calls.
template <typename T, int KMAX, bool PADDED, int kDpThreads>
__device__ __forceinline__ void dp_sweep_layers(const DpParams& p, T* const row, DpEntry* const s_entries,
                                                int32_t* const s_count, uint16_t* const s_bins, const int l_begin,
                                                const int l_end) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int D = p.D;
    const int64_t width = p.pd_stride;
    constexpr T kInf = DpInf<T>::v;
    const int bstride = p.max_count;
    const int stage = min(kDpStageMax, kDpStageEntries / bstride);     // layers per stage
    for (int l0 = l_begin; l0 < l_end; l0 += stage) {
        const int nl = min(stage, l_end - l0);
        __syncthreads();                              // previous stage fully consumed, row written
        for (int i = tid; i < nl * bstride; i += kDpThreads) {
            const DpEntry en = p.entries[(size_t)l0 * bstride + i];
            s_entries[i] = en;
            if (s_bins) s_bins[(size_t)l0 * bstride + i] = (uint16_t)en.bin;
        }
        if (tid < nl) s_count[tid] = p.count[l0 + tid];
        __syncthreads();
        for (int ll = 0; ll < nl; ++ll) {
            const int cn = s_count[ll];
            // entry c of the layer lives in lane c % 64 of register c / 64
            int32_t mybin = 0, mybin_hi = 0;
            T mysize = 0, mysize_hi = 0;
            if (lane < cn) {
                mybin = s_entries[ll * bstride + lane].bin;
                mysize = (T)s_entries[ll * bstride + lane].size;
            }
            if (lane + 64 < cn) {
                mybin_hi = s_entries[ll * bstride + lane + 64].bin;
                mysize_hi = (T)s_entries[ll * bstride + lane + 64].size;
            }
            T nv[KMAX];
            int32_t na[KMAX];
#pragma unroll
            for (int k = 0; k < KMAX; ++k) { nv[k] = kInf; na[k] = 255; }
            auto relax = [&](int32_t b, T sz, int c) {
                if (PADDED) {
                    const T* __restrict__ src = row + (dp_cell<KMAX, kDpThreads>(tid, 0) - b);
#pragma unroll
                    for (int k = 0; k < KMAX; ++k) {
                        const T t = src[dp_cell<KMAX, kDpThreads>(0, k)] + sz;
                        const bool lt = t < nv[k];
                        nv[k] = lt ? t : nv[k];
                        na[k] = lt ? c : na[k];
                    }
                } else {
#pragma unroll
                    for (int k = 0; k < KMAX; ++k) {
                        const int idx = dp_cell<KMAX, kDpThreads>(tid, k) - b;
                        T t = row[max(idx, 0)] + sz;
                        t = idx >= 0 ? t : kInf;
                        const bool lt = t < nv[k];
                        nv[k] = lt ? t : nv[k];
                        na[k] = lt ? c : na[k];
                    }
                }
            };
            const int cn_lo = min(cn, 64);
            for (int c = 0; c < cn_lo; ++c)
                relax((int32_t)readlane_u32((uint32_t)mybin, c), readlane_t<T>(mysize, c), c);
            for (int c = 64; c < cn; ++c)             // rare: more than 64 entries survive the host's pruning
                relax((int32_t)readlane_u32((uint32_t)mybin_hi, c - 64), readlane_t<T>(mysize_hi, c - 64), c);
            __syncthreads();
            uint8_t* __restrict__ pdrow = p.pd + (size_t)(l0 + ll) * width;
            if (KMAX % 2 == 0) {
                // a pair is written as a whole: cells above D get infinity (they stay out of every
                // later minimum), their PD bytes fall into the row's padding
#pragma unroll
                for (int k = 0; k < KMAX; k += 2) {
                    const int e = dp_cell<KMAX, kDpThreads>(tid, k);
                    if (e <= D) {
                        row[e] = nv[k];
                        row[e + 1] = (e + 1 <= D) ? nv[k + 1] : kInf;
                        *reinterpret_cast<uint16_t*>(pdrow + e) = (uint16_t)((na[k] & 255) | ((na[k + 1] & 255) << 8));
                    }
                }
            } else {
#pragma unroll
                for (int k = 0; k < KMAX; ++k) {
                    const int e = tid + k * kDpThreads;
                    if (e <= D) {
                        row[e] = nv[k];               // never above kInf: only a smaller t replaces it
                        pdrow[e] = (uint8_t)na[k];    // index into the layer's entry list
                    }
                }
            }
            __syncthreads();
        }
    }
}

// ---- grouped sweep: G workgroups, each sweeping its share of the layers from the virtual start row
// Block g takes the swept layers whose running entry count falls into the g-th of G equal parts
// (the sweep costs one pass over the row per entry), writes their arg-min rows like the
// sequential sweep and leaves, per exact bin sum e, the smallest size of its layers alone.
// 32-bit costs and the padded row only (what the host turns groups on for).
template <int KMAX, int kDpThreads>
__global__ __launch_bounds__(kDpThreads) void dp_group_kernel(DpParams p) {
    using T = uint32_t;
    extern __shared__ unsigned char dp_smem[];
    T* const row = reinterpret_cast<T*>(dp_smem) + p.pad;
    __shared__ DpEntry s_entries[kDpStageEntries];
    __shared__ int32_t s_count[kDpStageMax];
    __shared__ int32_t s_wsum[kDpThreads / 64];
    __shared__ int32_t s_lb[kDpMaxGroups + 1];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int G = p.groups.G, g = blockIdx.x;
    constexpr T kInf = DpInf<T>::v;
    int L = p.L;
    if (p.L_dev) {
        if (p.L_dev[1] != 0) return;                  // nothing to solve: the last kernel reports
        L = p.L_dev[0];
    }
    // group boundaries from the exclusive prefix of the entry counts (L <= kDpThreads)
    const int c = tid < L ? p.count[tid] : 0;
    int inc = c;
    for (int o = 1; o < 64; o <<= 1) {
        const int n = __shfl_up(inc, o, 64);
        if (lane >= o) inc += n;
    }
    if (lane == 63) s_wsum[wave] = inc;
    if (tid <= G) s_lb[tid] = L;
    __syncthreads();
    int base = 0, total = 0;
    for (int w = 0; w < kDpThreads / 64; ++w) {
        if (w < wave) base += s_wsum[w];
        total += s_wsum[w];
    }
    if (tid < L) {
        const int gid = total > 0 ? min(G - 1, (int)(((int64_t)(base + inc - c) * G) / total)) : 0;
        atomicMin(&s_lb[gid], tid);
    }
    __syncthreads();
    if (tid == 0)
        for (int q = G - 1; q >= 0; --q)              // a group without layers begins where the next one does
            if (s_lb[q] > s_lb[q + 1]) s_lb[q] = s_lb[q + 1];
    __syncthreads();
    const int lb = s_lb[g], le = s_lb[g + 1];
    for (int e = tid - p.pad; e < KMAX * kDpThreads; e += kDpThreads) row[e] = (e == 0) ? (T)0 : kInf;
    dp_sweep_layers<T, KMAX, true, kDpThreads>(p, row, s_entries, s_count, nullptr, lb, le);
    __syncthreads();
    T* const out = p.groups.nodes + (size_t)(G - 1 + g) * p.groups.stride;
    for (int e = tid; e < p.groups.stride; e += kDpThreads) out[e] = e <= p.D ? row[e] : kInf;
    if (tid == 0) {
        p.groups.range[2 * g] = lb;
        p.groups.range[2 * g + 1] = le;
    }
}

// One level of the tree: node = first_node + blockIdx.y joins its children X (lower layers) and Y,
//     T[e] = min over e2 <= e of Y[e2] + X[e - e2].
// Which e2 attains it is looked up later, for the few cells the trace passes through.  Both
// children sit in LDS; a wavefront takes whole cells (interleaved over the grid: a cell costs
// e + 1 terms), its lanes the terms of a cell.
constexpr int kConvThreads = 1024;
__global__ __launch_bounds__(kConvThreads) void dp_conv_kernel(DpGroups gr, int first_node, int D,
                                                                const int32_t* __restrict__ L_dev) {
    extern __shared__ uint32_t conv_smem[];
    constexpr uint32_t kInf = DpInf<uint32_t>::v;
    if (L_dev && L_dev[1] != 0) return;
    const int node = first_node + blockIdx.y;
    const uint32_t* __restrict__ X = gr.nodes + (size_t)(2 * node + 1) * gr.stride;
    const uint32_t* __restrict__ Y = gr.nodes + (size_t)(2 * node + 2) * gr.stride;
    uint32_t* const sX = conv_smem;
    uint32_t* const sY = conv_smem + (D + 1);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i <= D; i += kConvThreads) {
        sX[i] = X[i];
        sY[i] = Y[i];
    }
    __syncthreads();
    uint32_t* const T = gr.nodes + (size_t)node * gr.stride;
    const int nw = gridDim.x * (kConvThreads / 64);
    for (int e = blockIdx.x * (kConvThreads / 64) + wave; e <= D; e += nw) {
        uint32_t best = kInf;                        // a sum with an infinite term is at least kInf
#pragma unroll 4
        for (int e2 = lane; e2 <= e; e2 += 64) best = min(best, sY[e2] + sX[e - e2]);
        for (int o = 1; o < 64; o <<= 1) best = min(best, (uint32_t)__shfl_xor(best, o, 64));
        if (lane == 0) T[e] = best;
    }
}

// The host's input block from pinned memory into device memory (grouped solves of lgreco_solve:
// every group reads the lists, so they are fetched once, ahead of the groups).
__global__ __launch_bounds__(256) void dp_fetch_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int n) {
    for (int i = blockIdx.x * 256 + threadIdx.x; i < n; i += gridDim.x * 256) dst[i] = src[i];
}

// ---- pieces shared by the sequential kernel and the kernel that traces a grouped solve

// arg-min of src[0..D], lowest e among equal minima -> s_val[0], s_idx[0] (every thread calls)
template <typename T, int kDpThreads>
__device__ __forceinline__ void dp_argmin(const T* src, const int D, int64_t* const s_val, int32_t* const s_idx) {
    const int tid = threadIdx.x, lane = tid & 63;
    int64_t bv = (int64_t)DpInf<T>::v;
    int32_t be = 0x7FFFFFFF;
    for (int e = tid; e <= D; e += kDpThreads) {
        const int64_t v = (int64_t)src[e];
        if (v < bv) { bv = v; be = e; }              // e ascending per thread -> keeps the lowest
    }
    for (int o = 1; o < 64; o <<= 1) {
        const int64_t ov = __shfl_xor(bv, o, 64);
        const int32_t oe = __shfl_xor(be, o, 64);
        if (ov < bv || (ov == bv && oe < be)) { bv = ov; be = oe; }
    }
    __syncthreads();                              // earlier readers of s_val / s_idx are done
    if (lane == 0) { s_val[tid >> 6] = bv; s_idx[tid >> 6] = be; }
    __syncthreads();
    if (tid < 64) {
        // the first wavefront: every lane joins the per-wavefront minima the same way
        for (int w = 1; w < kDpThreads / 64; ++w)
            if (s_val[w] < bv || (s_val[w] == bv && s_idx[w] < be)) { bv = s_val[w]; be = s_idx[w]; }
    }
    __syncthreads();
    if (tid == 0) { s_val[0] = bv; s_idx[0] = be; }
    __syncthreads();
}

// The walk is a chain of dependent loads: one PD byte per layer from global memory, the bin it
// stands for from LDS.  One wavefront walks the swept layers [l_lo, l_hi) downwards from cell e,
// writes the picked entry of every layer to out[layer] and returns the cell it ends in (0 if all
// is consistent, -1 after a byte that cannot be).
// Two layers per load latency: lane j holds the bin of entry j of layer l, so while PD[l][e]
// is on its way lane j already fetches PD[l-1][e - bin_j], the byte the walk needs next if
// entry j is the one picked.  A wavefront pays the full issue latency of every instruction here,
// so the loop is kept short: rows by a running pointer, no branches, consistency checks joined
// into one flag (a bad byte still gives in-row addresses: e only shrinks and is clamped at 0,
// lanes past the list hold bin 0).  Lists of at most 64 entries.
__device__ __forceinline__ int dp_walk(const uint8_t* __restrict__ pd, const int64_t width,
                                       const uint16_t* const s_bins, const int bstride, const int l_hi,
                                       const int l_lo, int e, uint8_t* const out) {
    const int lane = threadIdx.x & 63;
    auto bins_of = [&](int layer) -> uint32_t {
        return lane < bstride ? (uint32_t)s_bins[max(layer, 0) * bstride + lane] : 0u;
    };
    int l = l_hi - 1;
    uint32_t bins_cur = bins_of(l), bins_prev = bins_of(l - 1);
    const uint8_t* __restrict__ row_l = pd + (size_t)max(l, 0) * width;
    int bad = 0;
    for (; l >= l_lo + 1; l -= 2, row_l -= 2 * width) {
        const uint32_t bins_n1 = bins_of(l - 2), bins_n2 = bins_of(l - 3);
        const uint32_t ka_v = row_l[e];
        const uint32_t kb_v = (row_l - width)[max(e - (int)bins_cur, 0)];
        const int ka = __builtin_amdgcn_readfirstlane((int)ka_v);
        const int kb = (int)readlane_u32(kb_v, ka);
        out[l] = (uint8_t)ka;                  // every lane writes the same byte
        out[l - 1] = (uint8_t)kb;
        e -= (int)readlane_u32(bins_cur, ka) + (int)readlane_u32(bins_prev, kb);
        bad |= (ka >= bstride) | (kb >= bstride) | (e < 0);
        e = max(e, 0);
        bins_cur = bins_n1;
        bins_prev = bins_n2;
    }
    if (l == l_lo && l_hi > l_lo) {
        const int ka = __builtin_amdgcn_readfirstlane((int)row_l[e]);
        out[l] = (uint8_t)ka;
        e -= (int)readlane_u32(bins_cur, ka);
        bad |= (ka >= bstride) | (e < 0);
    }
    return bad ? -1 : e;
}

// What a solve ends with, once s_val[0] / s_idx[0] hold the minimum of the last row and its cell,
// s_idx[1] the cell the walk ended in and s_pick the picked entry of every swept layer: the
// compression's layer records (see DpApply), the assignment and the result block.  `staging`:
// 16 KB of LDS free by now.  Every thread calls; the threads past the first wavefront return
// before the hand-over.
template <typename T, int kDpThreads>
__device__ __forceinline__ void dp_finish(const DpParams& p, const int L, const bool lds_bins, const uint8_t* const s_pick,
                                          unsigned char* const staging, const int64_t* const s_val,
                                          const int32_t* const s_idx, const int32_t pre_fixed, const int32_t pre_sweep,
                                          const uint64_t t_begin, const uint64_t t_sweep, const int64_t how) {
    constexpr T kInf = DpInf<T>::v;
    const int tid = threadIdx.x, lane = tid & 63;
    const int bstride = p.max_count;
    const bool feasible = s_val[0] < (int64_t)kInf;
    const bool traced = feasible && lds_bins && s_idx[1] == 0;
    int64_t applied = 0;                 // the layer records were written (workgroup-uniform)
    if (p.apply.layers) {
        // The compression's layer records from the assignment, one thread per layer: candidate per
        // layer first (fixed layers from the build's report, swept ones from the back-trace), then
        // the payload offsets, a running sum of the chosen sizes rounded up to 16 bytes.
        const DpApply& A = p.apply;
        static_assert(kDpThreads >= kBuildThreads, "one thread per layer");
        uint8_t* const s_chosen = staging;                                                         // [threads]
        int64_t* const s_wtot = reinterpret_cast<int64_t*>(staging) + kDpThreads / 8;              // [waves]
        int32_t* const s_bad = reinterpret_cast<int32_t*>(s_wtot + kDpThreads / 64);
        const int wave = tid >> 6;
        bool ok = traced && A.L <= kDpThreads;          // workgroup-uniform
        int c = 0;
        int32_t fam = 0, ipar = 0, tslot = -1;
        int64_t off = 0;
        if (ok) {
            const int32_t swept_cand = tid < L ? p.entries[(size_t)tid * bstride + s_pick[tid]].cand : 0;
            s_chosen[tid] = tid < A.L ? (uint8_t)pre_fixed : (uint8_t)0;
            if (tid == 0) *s_bad = 0;
            __syncthreads();
            if (tid < L) s_chosen[pre_sweep] = (uint8_t)swept_cand;
            __syncthreads();
            c = s_chosen[tid];
            const bool mine = tid < A.L;
            const bool bad = mine && c >= A.P;           // a layer neither fixed nor swept
            const int cc = bad ? 0 : c;
            // the three table reads of the chosen column go out together
            const int64_t raw = mine ? A.sizes[(size_t)tid * A.P + cc] : 0;
            fam = mine ? A.family[cc] : 0;
            tslot = mine ? A.topk_slot[cc] : -1;
            ipar = mine ? A.iparam[(size_t)tid * A.P + cc] : 0;
            const int64_t sz = (mine && !bad) ? (raw + 15) / 16 * 16 : 0;
            int64_t inc = sz;
            for (int o = 1; o < 64; o <<= 1) {
                const int64_t n = __shfl_up(inc, o, 64);
                if (lane >= o) inc += n;
            }
            if (lane == 63) s_wtot[wave] = inc;
            if (bad) *s_bad = 1;
            __syncthreads();
            int64_t base = 0, total = 0;
            for (int w = 0; w < kDpThreads / 64; ++w) {
                if (w < wave) base += s_wtot[w];
                total += s_wtot[w];
            }
            off = base + inc - sz;
            ok = *s_bad == 0 && total <= A.capacity;
        }
        if (tid < A.L) {
            if (ok) {
                A.layers[tid].payload = off;
                A.layers[tid].family = fam;
                A.layers[tid].iparam = ipar;
                A.layers[tid].slot = tslot;
            } else {
                A.layers[tid].family = -1;
            }
        }
        if (A.L > kDpThreads)
            for (int l = kDpThreads + tid; l < A.L; l += kDpThreads) A.layers[l].family = -1;
        applied = ok ? 1 : 0;
    }
    // The result block lies in the host's pinned memory and the host may be polling it: the first
    // wavefront alone writes it (the other writer of host memory, the back-trace without LDS
    // tables, is its thread 0).  What the host relies on does not depend on the order in which
    // the stores arrive there: the slots of this kernel go out as ONE store of the wavefront (lane
    // i holds slot i; the 128-byte block is two 64-byte halves, each carrying a copy of the
    // launch's sequence number), the assignment is covered by a check word in the block, and the
    // sequence number in slot 7, which the host polls, follows behind a system-scope fence.
    if (tid >= 64) return;
    unsigned long long check = 0;        // sum of (candidate + 1) * (swept layer + 1): the host's check word
    bool adds_up = true;
    if (traced) {
        // the assignment goes out, and is held against the cell it was traced from on the way:
        // its bins must sum to e*, its costs to the minimum found there
        long long sum_bin = 0, sum_cost = 0;
        for (int l = lane; l < L; l += 64) {
            const DpEntry en = p.entries[(size_t)l * bstride + s_pick[l]];
            p.choice[l] = en.cand;
            check += (unsigned long long)(uint32_t)(en.cand + 1) * (unsigned long long)(l + 1);
            sum_bin += en.bin;
            sum_cost += en.size;
        }
        for (int o = 1; o < 64; o <<= 1) {
            check += (unsigned long long)__shfl_xor((long long)check, o, 64);
            sum_bin += __shfl_xor(sum_bin, o, 64);
            sum_cost += __shfl_xor(sum_cost, o, 64);
        }
        adds_up = sum_bin == (long long)s_idx[0] && sum_cost == (long long)s_val[0];
    } else if (!lds_bins) {
        check = (unsigned long long)s_val[2];         // summed by the thread that wrote the assignment
    }
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)t_sweep);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(t_sweep >> 32));
    const uint64_t tsw = ((uint64_t)hi << 32) | lo;                  // thread 0 took the time
    const uint64_t ticks_sweep = tsw - t_begin, ticks_trace = wall_clock64() - tsw;
    int64_t v = 0;
    bool mine = true;
    switch (lane) {
        case 0: v = !feasible ? 1 : ((s_idx[1] == 0 && adds_up) ? 0 : 2); break;      // 2: an internal inconsistency
        case 1: v = feasible ? s_val[0] : 0; break;
        case 2: v = feasible ? (int64_t)s_idx[0] : 0; break;
        // diagnostics: ticks of the constant-rate (100 MHz) counter spent in sweep (low half) and
        // back-trace (high half)
        case 3: v = (int64_t)((ticks_sweep & 0xFFFFFFFFull) | (ticks_trace << 32)); break;
        case 4: v = p.seq; break;
        case 8: v = applied; break;
        // how the table was swept: 0 sequentially, G in G groups, 1000 + G in G groups with
        // ambiguous splits resolved by comparing traced sequences, -G sequentially after the
        // grouped route gave up
        case 9: v = how; break;
        case 10: v = (int64_t)check; break;
        case 15: v = p.seq; break;
        default: mine = false;                    // 5, 6: the list-building kernel's; 7: below
    }
    if (mine) p.result[lane] = v;
    __threadfence_system();
    if (tid == 0) p.result[7] = p.seq;
}

// The build kernel found nothing to solve (a NaN, a layer without usable candidate): only the
// hand-over is left.  Every thread calls.
template <int kDpThreads>
__device__ __forceinline__ void dp_hand_over_unsolved(const DpParams& p) {
    const int tid = threadIdx.x;
    if (p.apply.layers)
        for (int l = tid; l < p.apply.L; l += kDpThreads) p.apply.layers[l].family = -1;
    if (tid < 64) {
        // slots as in dp_finish; the status in slot 0 is the list-building kernel's
        const int lane = tid;
        if (lane == 4 || lane == 15) p.result[lane] = p.seq;
        if (lane == 8 || lane == 10) p.result[lane] = 0;
        __threadfence_system();
        if (tid == 0) p.result[7] = p.seq;
    }
}

// ---- the sequential solve: one workgroup sweeps every layer, traces back and finishes
template <typename T, int KMAX, bool PADDED, int kDpThreads>
__global__ __launch_bounds__(kDpThreads) void dp_kernel(DpParams p) {
    // In a grouped solve this kernel is queued behind dp_trace_kernel and has work only if that
    // one gave up (it then left flag = 1 and no result).
    const int G = p.groups.G;
    if (G > 1 && p.groups.flag[0] == 0) return;
    // LDS row: [pad] cells of infinity, then cells 0 .. KMAX*threads-1 (cells above D stay infinite).
    // With PADDED the pad is at least the largest bin, so row[e - b] needs no range check.
    extern __shared__ unsigned char dp_smem[];
    T* const row = reinterpret_cast<T*>(dp_smem) + p.pad;
    __shared__ DpEntry s_entries[kDpStageEntries];      // [layers of the stage][max_count]
    __shared__ int32_t s_count[kDpStageMax];
    __shared__ int64_t s_val[kDpThreads / 64];
    __shared__ int32_t s_idx[kDpThreads / 64];
    const int tid = threadIdx.x;
    const int64_t width = p.pd_stride;
    constexpr T kInf = DpInf<T>::v;
    // back-trace tables behind the row when they fit (the host decides): the bin of every entry
    // (16 bits: D <= 16384) and the picked entry per layer
    const bool lds_bins = p.bt_lds != 0;
    uint16_t* const s_bins = reinterpret_cast<uint16_t*>(row + KMAX * kDpThreads);
    const int bstride = p.max_count;
    uint8_t* const s_pick = reinterpret_cast<uint8_t*>(s_bins + (size_t)p.L * bstride);   // p.L: capacity
    // Entry lists built on the device (dp_build_kernel): the number of swept layers and the status
    // it found come from memory; anything but "ok" there ends the solve.
    int L = p.L;
    if (p.L_dev) {
        if (p.L_dev[1] != 0) {
            dp_hand_over_unsolved<kDpThreads>(p);
            return;
        }
        L = p.L_dev[0];
    }
    // for the apply step at the end (see DpApply): the build's report for this thread's layer,
    // fetched now so that the tail does not wait for it
    int32_t pre_fixed = 0, pre_sweep = 0;
    if (p.apply.layers) {
        if (tid < p.apply.L) pre_fixed = p.apply.fixed_choice[tid];
        if (tid < L) pre_sweep = p.apply.sweep_layer[tid];
    }
    const uint64_t t_begin = wall_clock64();
    if (p.host_in) {
        // fetch the input block from the host's pinned memory: one 16-byte word per thread and
        // round, all in flight together; the barrier below orders it before the first read
        for (int i = tid; i < p.in_vec; i += kDpThreads) p.dev_in[i] = p.host_in[i];
        __threadfence_block();
    }
    for (int e = tid - p.pad; e < KMAX * kDpThreads; e += kDpThreads) row[e] = (e == 0) ? (T)0 : kInf;
    dp_sweep_layers<T, KMAX, PADDED, kDpThreads>(p, row, s_entries, s_count, lds_bins ? s_bins : nullptr, 0, L);
    __syncthreads();
    dp_argmin<T, kDpThreads>(row, min(p.D, p.e_limit), s_val, s_idx);
    uint64_t t_sweep = 0;
    if (tid == 0) t_sweep = wall_clock64();
    if (tid < 64 && s_val[0] < (int64_t)kInf) {
        int e = __builtin_amdgcn_readfirstlane(s_idx[0]);
        if (lds_bins && bstride <= 64) {
            e = dp_walk(p.pd, width, s_bins, bstride, L, 0, e, s_pick);
        } else if (tid == 0) {
            if (lds_bins) {
                for (int l = L - 1; l >= 0; --l) {
                    const int k = p.pd[(size_t)l * width + e];
                    s_pick[l] = (uint8_t)k;
                    e -= s_bins[l * bstride + k];
                }
            } else {
                unsigned long long check = 0;
                for (int l = L - 1; l >= 0; --l) {
                    const int k = p.pd[(size_t)l * width + e];
                    const DpEntry en = p.entries[(size_t)l * bstride + k];
                    p.choice[l] = en.cand;
                    check += (unsigned long long)(uint32_t)(en.cand + 1) * (unsigned long long)(l + 1);
                    e -= en.bin;
                }
                s_val[2] = (int64_t)check;
            }
        }
        if (tid == 0) s_idx[1] = e;
    }
    __syncthreads();
    dp_finish<T, kDpThreads>(p, L, lds_bins, s_pick, reinterpret_cast<unsigned char*>(s_entries), s_val, s_idx, pre_fixed,
                             pre_sweep, t_begin, t_sweep, G > 1 ? -(int64_t)G : 0);
}

// ---- tracing a grouped solve (see dp_group_kernel / dp_conv_kernel): one workgroup
// The layers were swept in G groups side by side and the groups' cost functions joined pairwise;
// node 0 of the tree is the last row of the whole table.  Walking down the tree gives every
// group its share of the bins: at an inner node holding e bins the split is the e2 with
// Y[e2] + X[e - e2] = T[e].  Where several e2 attain it, Algorithm 1's tie-breaks decide (lowest
// candidate index, last layer first): the split whose higher-layer child Y traces back to the
// lexicographically smallest sequence of picks, compared from Y's last layer down (slow path
// below).  Every group is then walked back from its share by a wavefront of its own, the
// assignment is checked against the root cell (bins and size must add up to it) and the solve is
// finished as in the sequential kernel.  A solve this kernel gives up on (too many candidates to
// compare, a check that fails) gets flag = 1 and is swept by the sequential kernel queued next.
// Dynamic LDS: the bin of every entry (16 bits) and the picked entry per layer.
template <int kDpThreads>
__global__ __launch_bounds__(kDpThreads) void dp_trace_kernel(DpParams p) {
    using T = uint32_t;
    extern __shared__ unsigned char dp_smem[];
    __shared__ __align__(16) unsigned char s_stage[16384];       // buffers of the slow path, then the finish
    __shared__ int64_t s_val[kDpThreads / 64];
    __shared__ int32_t s_idx[kDpThreads / 64];
    constexpr int kSplitCap = 16, kWalkBudget = 96, kTreeDepth = 3;
    static_assert((1 << kTreeDepth) == kDpMaxGroups, "the slow path is written out for this depth");
    __shared__ int32_t s_alloc[2 * kDpMaxGroups], s_ncnt[2 * kDpMaxGroups], s_nlast[2 * kDpMaxGroups];
    __shared__ int32_t s_tie, s_walk_bad, s_slow_ok, s_nsplit;
    const int tid = threadIdx.x, lane = tid & 63;
    const int D = p.D;
    const int64_t width = p.pd_stride;
    constexpr T kInf = DpInf<T>::v;
    const int bstride = p.max_count;
    uint16_t* const s_bins = reinterpret_cast<uint16_t*>(dp_smem);
    uint8_t* const s_pick = reinterpret_cast<uint8_t*>(s_bins + (size_t)p.L * bstride);   // p.L: capacity
    const int G = p.groups.G;
    const DpGroups& gr = p.groups;
    if (tid == 0) gr.flag[0] = 0;
    int L = p.L;
    if (p.L_dev) {
        if (p.L_dev[1] != 0) {
            dp_hand_over_unsolved<kDpThreads>(p);
            return;
        }
        L = p.L_dev[0];
    }
    int32_t pre_fixed = 0, pre_sweep = 0;
    if (p.apply.layers) {
        if (tid < p.apply.L) pre_fixed = p.apply.fixed_choice[tid];
        if (tid < L) pre_sweep = p.apply.sweep_layer[tid];
    }
    const uint64_t t_begin = wall_clock64();
    // the bin of every entry, for the walks
    for (int i = tid; i < L * bstride; i += kDpThreads) s_bins[i] = (uint16_t)p.entries[i].bin;
    if (tid == 0) { s_tie = 0; s_walk_bad = 0; s_slow_ok = 0; }
    dp_argmin<T, kDpThreads>(gr.nodes, min(D, p.e_limit), s_val, s_idx);
    bool resolved = false;                            // ambiguous splits were met and resolved
    bool give_up = false;
    if (s_val[0] < (int64_t)kInf) {
        // every e2 with Y[e2] + X[e - e2] = T[e] of an inner node, up to kSplitCap of them in out[]
        // (in no particular order); the whole block scans (every thread calls, with the same
        // arguments); returns how many there are, which may be more than fit out[]
        auto splits_of = [&](const int node, const int e, int32_t* const out) -> int {
            const uint32_t* __restrict__ X = gr.nodes + (size_t)(2 * node + 1) * gr.stride;
            const uint32_t* __restrict__ Y = gr.nodes + (size_t)(2 * node + 2) * gr.stride;
            const uint32_t target = gr.nodes[(size_t)node * gr.stride + e];
            __syncthreads();                              // earlier readers of s_nsplit / out are done
            if (tid == 0) s_nsplit = 0;
            __syncthreads();
            if (target < (uint32_t)kInf) {
#pragma unroll 4
                for (int e2 = tid; e2 <= e; e2 += kDpThreads) {
                    if (Y[e2] + X[e - e2] == target) {
                        const int pos = atomicAdd(&s_nsplit, 1);
                        if (pos < kSplitCap) out[pos] = e2;
                    }
                }
            }
            __syncthreads();
            return s_nsplit;
        };
        // first and last swept layer of the leaves under a node of the tree
        auto layers_of = [&](int node, int* lo, int* hi) {
            int a = node, b = node;
            while (a < G - 1) { a = 2 * a + 1; b = 2 * b + 2; }
            *lo = gr.range[2 * (a - (G - 1))];
            *hi = gr.range[2 * (b - (G - 1)) + 1];
        };
        if (tid == 0) s_alloc[0] = s_idx[0];
        // fast path, level by level: the threads share out the nodes of a level and each node's
        // e2 range; a node where not exactly one e2 matches ends it
        for (int first = 0; first < G - 1; first = 2 * first + 1) {         // nodes first .. 2 first
            if (tid < 2 * kDpMaxGroups) { s_ncnt[tid] = 0; s_nlast[tid] = -1; }
            __syncthreads();
            const int tpn = kDpThreads / (first + 1);                       // threads per node
            const int node = first + tid / tpn, t_in = tid % tpn;
            const bool live = s_tie == 0;                                   // else the shares above are not set
            const int a = live ? s_alloc[node] : 0;
            const uint32_t* __restrict__ X = gr.nodes + (size_t)(2 * node + 1) * gr.stride;
            const uint32_t* __restrict__ Y = gr.nodes + (size_t)(2 * node + 2) * gr.stride;
            const uint32_t target = gr.nodes[(size_t)node * gr.stride + a];
            int cnt = 0, last = -1;
            if (live) {
#pragma unroll 4
                for (int e2 = t_in; e2 <= a; e2 += tpn) {
                    const bool ok = Y[e2] + X[a - e2] == target;
                    cnt += ok ? 1 : 0;
                    last = ok ? e2 : last;
                }
            }
            if (cnt) {
                atomicAdd(&s_ncnt[node], cnt);
                atomicMax(&s_nlast[node], last);
            }
            __syncthreads();
            if (t_in == 0 && live) {
                if (s_ncnt[node] != 1) {
                    s_tie = 1;
                } else {
                    s_alloc[2 * node + 2] = s_nlast[node];
                    s_alloc[2 * node + 1] = a - s_nlast[node];
                }
            }
            __syncthreads();
        }
        __syncthreads();
        if (s_tie != 0) {
            // slow path: resolve every ambiguous split by comparing the sequences of picks its
            // candidates lead to in the higher-layer child.  Every thread runs the same control
            // flow (all decisions come from LDS); the scans use the whole block, the walks one
            // wavefront per group, the comparisons the first wavefront.
            uint8_t* const bufs = s_stage;                                      // [depth][2][L <= 1024]
            int32_t* const cands = reinterpret_cast<int32_t*>(s_stage) + 2048;  // behind the buffers: [depth][cap]
            int32_t* const saved = cands + kTreeDepth * kSplitCap;              // [depth][2 G] shares of the best candidate
            static_assert(sizeof(s_stage) >= 8192 + 4 * kTreeDepth * (kSplitCap + 2 * kDpMaxGroups),
                          "staging area too small");
            int budget = kWalkBudget;         // candidates looked at; the same in every thread
            // picks of [lo, hi) compared from the last layer down: is a before b?
            auto before = [&](const uint8_t* a, const uint8_t* b, int lo, int hi) -> bool {
                if (tid < 64) {
                    int res = 0;
                    for (int top = hi - 1; top >= lo; top -= 64) {
                        const int l = top - lane;
                        const int da = l >= lo ? a[l] : 0, db = l >= lo ? b[l] : 0;
                        const unsigned long long m = __ballot(da != db);
                        if (m) {
                            const int firstl = __builtin_amdgcn_readfirstlane(__builtin_ctzll(m));
                            res = (int)readlane_u32((uint32_t)(da < db), firstl);
                            break;
                        }
                    }
                    if (lane == 0) s_nlast[0] = res;
                }
                __syncthreads();
                const bool r = s_nlast[0] != 0;
                __syncthreads();
                return r;
            };
            // picks of every group under `node`, each from the share s_alloc gives it: one
            // wavefront per group, side by side
            auto walk_under = [&](int node, uint8_t* out) -> bool {
                int a = node, b = node;
                while (a < G - 1) { a = 2 * a + 1; b = 2 * b + 2; }
                if (tid == 0) s_nlast[1] = 0;
                __syncthreads();
                const int leafn = a + (tid >> 6);
                if (leafn <= b) {
                    const int g = leafn - (G - 1);
                    const int e_end = dp_walk(p.pd, width, s_bins, bstride, gr.range[2 * g + 1], gr.range[2 * g],
                                              __builtin_amdgcn_readfirstlane(s_alloc[leafn]), out);
                    if (lane == 0 && e_end != 0) s_nlast[1] = 1;
                }
                __syncthreads();
                const bool ok = s_nlast[1] == 0;
                __syncthreads();
                return ok;
            };
            // the shares of every node under `node` holding e bins -> s_alloc
            auto share = [&](auto&& deeper, int level, int node, int e) -> bool {
                if (tid == 0) s_alloc[node] = e;
                if (node >= G - 1) return true;
                int32_t* const cd = cands + level * kSplitCap;
                const int cnt = splits_of(node, e, cd);
                if (cnt < 1 || cnt > kSplitCap) return false;
                int pick = 0;
                if (cnt > 1) {
                    int lo, hi;
                    layers_of(2 * node + 2, &lo, &hi);
                    uint8_t* best = bufs + (size_t)(2 * level) * 1024;
                    uint8_t* cur = bufs + (size_t)(2 * level + 1) * 1024;
                    int32_t* const keep = saved + level * 2 * kDpMaxGroups;
                    for (int i = 0; i < cnt; ++i) {
                        if (--budget < 0) return false;
                        if (!deeper(2 * node + 2, cd[i])) return false;
                        if (!walk_under(2 * node + 2, i == 0 ? best : cur)) return false;
                        const bool better = i > 0 && before(cur, best, lo, hi);
                        if (better) {
                            uint8_t* t = best; best = cur; cur = t;
                            pick = i;
                        }
                        if (i == 0 || better) {
                            if (tid < 2 * kDpMaxGroups) keep[tid] = s_alloc[tid];
                            __syncthreads();
                        }
                    }
                    if (tid < 2 * kDpMaxGroups) s_alloc[tid] = keep[tid];     // the best candidate's shares
                    __syncthreads();
                } else if (!deeper(2 * node + 2, cd[0])) {
                    return false;
                }
                return deeper(2 * node + 1, e - cd[pick]);
            };
            auto leaf_share = [&](int n, int ee) -> bool {
                if (tid == 0) s_alloc[n] = ee;
                return true;
            };
            auto share2 = [&](int node, int e) -> bool { return share(leaf_share, 2, node, e); };
            auto share1 = [&](int node, int e) -> bool { return share(share2, 1, node, e); };
            const bool ok = share(share1, 0, 0, s_idx[0]);
            __syncthreads();
            if (tid == 0) s_slow_ok = ok ? 1 : 0;
            __syncthreads();
            give_up = s_slow_ok == 0;
            resolved = !give_up;
        }
        if (!give_up) {
            // every group walked back from its share, one wavefront each
            const int g = tid >> 6;
            if (g < G) {
                const int e_end = dp_walk(p.pd, width, s_bins, bstride, gr.range[2 * g + 1], gr.range[2 * g],
                                          __builtin_amdgcn_readfirstlane(s_alloc[G - 1 + g]), s_pick);
                if (lane == 0 && e_end != 0) s_walk_bad = 1;
            }
            __syncthreads();
            // The assignment must add up to the root's cell: bins to e*, sizes to the minimum
            // found there.  Whatever does not (it never should) is swept sequentially instead.
            long long sum_b = 0, sum_s = 0;
            int ok = 1;
            for (int l = tid; l < L; l += kDpThreads) {
                const int k = s_pick[l];
                ok &= k < p.count[l] ? 1 : 0;
                const DpEntry en = p.entries[(size_t)l * bstride + min(k, bstride - 1)];
                sum_b += en.bin;
                sum_s += en.size;
            }
            for (int o = 1; o < 64; o <<= 1) {
                sum_b += __shfl_xor(sum_b, o, 64);
                sum_s += __shfl_xor(sum_s, o, 64);
                ok &= __shfl_xor(ok, o, 64);
            }
            long long* const s_tot = reinterpret_cast<long long*>(s_stage);      // [waves][2]
            if (lane == 0) {
                s_tot[2 * (tid >> 6)] = sum_b;
                s_tot[2 * (tid >> 6) + 1] = sum_s;
                if (!ok) s_walk_bad = 1;
            }
            __syncthreads();
            if (tid == 0) {
                long long tb = 0, ts = 0;
                for (int w = 0; w < kDpThreads / 64; ++w) { tb += s_tot[2 * w]; ts += s_tot[2 * w + 1]; }
                if (tb != (long long)s_idx[0] || ts != (long long)s_val[0]) s_walk_bad = 1;
                s_idx[1] = 0;
            }
            __syncthreads();
            give_up = s_walk_bad != 0;
        }
    }
    if (give_up) {                                    // block-uniform: the sequential kernel takes over
        if (tid == 0) gr.flag[0] = 1;
        return;
    }
    uint64_t t_sweep = 0;
    if (tid == 0) t_sweep = wall_clock64();
    __syncthreads();
    dp_finish<T, kDpThreads>(p, L, true, s_pick, s_stage, s_val, s_idx, pre_fixed, pre_sweep, t_begin, t_sweep,
                             resolved ? 1000 + G : G);
}

// ------------------------------------------------------------------ entry lists on the device
// What lgreco_solve does on the host between the error table and the sweep, for a solve that
// follows the profile on the same stream without a host round trip: E_max (the default
// candidate's errors summed in layer order), bins = floor(err * D / E_max) in fp64, equal bins
// merged (smallest size, lowest index among equals), entries beaten in both bin and size dropped,
// layers with a single entry of bin 0 fixed, the others compacted into the sweep's tables.  One
// workgroup.  Binning, then merging and pruning in one pass, run with one thread per (layer,
// candidate), each comparing itself with the layer's other candidates in LDS; then one thread per layer counts
// what is left, the swept layers are numbered in layer order and their entries written in
// candidate order, as on the host.
__global__ __launch_bounds__(kBuildThreads) void dp_build_kernel(DpBuildParams p) {
    // tables from device memory into LDS; the error table is passed on to the host's pinned copy
    // on the way (posted writes; reading the tables from there instead took 30 us)
    __shared__ __align__(16) double s_err[kBuildMaxLP];
    __shared__ __align__(16) int64_t s_size[kBuildMaxLP];
    __shared__ int32_t s_bin[kBuildMaxLP], s_sz32[kBuildMaxLP];   // sizes below 2^30 on this path
    __shared__ uint8_t s_kept[kBuildMaxLP];
    __shared__ double s_emax;
    __shared__ int32_t s_wave[kBuildThreads / 64];
    __shared__ int32_t s_flags[2];          // [0] a layer without usable candidate, [1] invalid input
    // check words over what this kernel writes into the host's memory (the host holds what it reads
    // there against them): [0] the error table, sum of bit pattern * (index + 1); [1] the report,
    // sum of (fixed choice + 2) * (layer + 1) plus 65537 * sum of (swept layer + 1) * (slot + 1)
    __shared__ unsigned long long s_chk[2];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int L = p.L, P = p.P, LP = L * P;
    const double D = (double)p.D;
    if (tid < 2) {
        s_flags[tid] = 0;
        s_chk[tid] = 0;
    }
    {
        // whole 16-byte words, then the odd last entry on its own: a caller's table ends at LP entries
        const int n16 = LP / 2;
        const uint4* const ge = reinterpret_cast<const uint4*>(p.errors);
        const uint4* const gs = reinterpret_cast<const uint4*>(p.sizes);
        uint4* const he = reinterpret_cast<uint4*>(p.errors_host);
        for (int i = tid; i < n16; i += kBuildThreads) {
            const uint4 e = ge[i];
            reinterpret_cast<uint4*>(s_err)[i] = e;
            if (he) he[i] = e;
            reinterpret_cast<uint4*>(s_size)[i] = gs[i];
        }
        if ((LP & 1) && tid == 0) {
            const double e = p.errors[LP - 1];
            s_err[LP - 1] = e;
            if (p.errors_host) p.errors_host[LP - 1] = e;
            s_size[LP - 1] = p.sizes[LP - 1];
        }
    }
    __syncthreads();
    if (p.errors_host) {
        unsigned long long c = 0;
        for (int i = tid; i < LP; i += kBuildThreads)
            c += __builtin_bit_cast(unsigned long long, s_err[i]) * (unsigned long long)(i + 1);
        for (int o = 1; o < 64; o <<= 1) c += (unsigned long long)__shfl_xor((long long)c, o, 64);
        if (lane == 0) atomicAdd(&s_chk[0], c);
    }
    // This path sweeps with 32-bit costs.  A caller whose size table the host has not seen asks for
    // the check here: sizes must be non-negative and every layer's largest, summed, below 2^30.
    if (p.check_sizes) {
        int64_t lmax = 0;
        if (tid < L)
            for (int c = 0; c < P; ++c) {
                const int64_t sz = s_size[tid * P + c];
                if (sz < 0 || sz >= ((int64_t)1 << 30)) s_flags[1] = 1;
                lmax = sz > lmax ? sz : lmax;
            }
        for (int o = 1; o < 64; o <<= 1) lmax += __shfl_xor(lmax, o, 64);
        __shared__ int64_t s_lmax[kBuildThreads / 64];
        if (lane == 0) s_lmax[wave] = lmax;
        __syncthreads();
        if (tid == 0) {
            int64_t worst = 0;
            for (int w = 0; w < kBuildThreads / 64; ++w) worst += s_lmax[w];
            if (worst >= ((int64_t)1 << 30)) s_flags[1] = 1;
        }
    }
    // E_max: errors[l][default] summed for l = 0 .. L-1 in that order (bit-identical to the host
    // loop): one thread, the LDS reads issued in batches ahead of the dependent adds
    if (tid == 0) {
        double sum = 0.0;
        int l = 0;
        for (; l + 32 <= L; l += 32) {
            double v[32];
#pragma unroll
            for (int u = 0; u < 32; ++u) v[u] = s_err[(l + u) * P + p.default_cand];
#pragma unroll
            for (int u = 0; u < 32; ++u) sum += v[u];
        }
        for (; l < L; ++l) sum += s_err[l * P + p.default_cand];
        s_emax = sum;
    }
    __syncthreads();
    const double e_max = s_emax;
    if (!(e_max == e_max) && tid == 0) s_flags[1] = 1;
    // bins, one (layer, candidate) per thread and pass
    for (int i = tid; i < LP; i += kBuildThreads) {
        double e = s_err[i];
        if (!(e == e)) s_flags[1] = 1;
        if (e < 0.0) e = 0.0;
        int32_t b;
        if (e_max > 0.0) {
            const double q = floor((e * D) / e_max);
            b = (q <= D) ? (int32_t)q : -1;
        } else {
            b = (e <= 0.0) ? 0 : -1;
        }
        s_bin[i] = (e == e) ? b : -1;
        s_sz32[i] = (int32_t)s_size[i];
    }
    __syncthreads();
    // What stays of a layer's list: a candidate goes when another usable one has the same bin and
    // a smaller size (or the same size and a lower index: one representative per bin), or a smaller
    // bin and a size that is not larger.  (The host states the second rule for representatives
    // only; a usable candidate that beats this one has a representative that does, too.)
    for (int i = tid; i < LP; i += kBuildThreads) {
        const int l = i / P, c = i - l * P;
        const int32_t b = s_bin[i];
        const int32_t sz = s_sz32[i];
        bool k = b >= 0;
        // all of the layer's candidates are read before the first comparison (fixed trip count;
        // reads past the layer's last candidate are clamped and not used)
        int32_t bo[kBuildMaxP], so[kBuildMaxP];
#pragma unroll
        for (int o = 0; o < kBuildMaxP; ++o) {
            const int j = min(l * P + o, LP - 1);
            bo[o] = s_bin[j];
            so[o] = s_sz32[j];
        }
#pragma unroll
        for (int o = 0; o < kBuildMaxP; ++o) {
            const bool same = bo[o] == b && (so[o] < sz || (so[o] == sz && o < c));
            const bool lower = bo[o] >= 0 && bo[o] < b && so[o] <= sz;
            if (o < P && o != c && (same || lower)) k = false;
        }
        s_kept[i] = k ? 1 : 0;
    }
    __syncthreads();
    // one thread per layer: what is left of its list
    const bool active = tid < L;
    int cnt = 0, first_bin = -1, first_cand = -1;
    if (active) {
        for (int c = P - 1; c >= 0; --c)
            if (s_kept[tid * P + c]) { ++cnt; first_bin = s_bin[tid * P + c]; first_cand = c; }
    }
    const bool dead = active && cnt == 0;
    const bool fixed = active && cnt == 1 && first_bin == 0;
    const bool swept = active && !dead && !fixed;
    if (dead) s_flags[0] = 1;
    // position among the swept layers, in layer order
    const unsigned long long m = __ballot(swept);
    const int before = (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
    if (lane == 0) s_wave[wave] = (int)__popcll(m);
    __syncthreads();
    int base = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kBuildThreads / 64; ++w) {
        if (w < wave) base += s_wave[w];
        total += s_wave[w];
    }
    const int slot = base + before;
    {
        unsigned long long c = 0;
        if (active) c = (unsigned long long)(uint32_t)((fixed ? first_cand : -1) + 2) * (unsigned long long)(tid + 1);
        if (swept) c += 65537ull * (unsigned long long)(tid + 1) * (unsigned long long)(slot + 1);
        for (int o = 1; o < 64; o <<= 1) c += (unsigned long long)__shfl_xor((long long)c, o, 64);
        if (lane == 0) atomicAdd(&s_chk[1], c);
    }
    if (active) {
        p.fixed_choice[tid] = fixed ? first_cand : -1;
        p.fixed_choice_dev[tid] = fixed ? first_cand : -1;
    }
    if (swept) {
        p.count[slot] = cnt;
        p.sweep_layer[slot] = tid;
        p.sweep_layer_dev[slot] = tid;
        DpEntry* const en = p.entries + (size_t)slot * p.stride;
        int r = 0;
        for (int c = 0; c < P; ++c)
            if (s_kept[tid * P + c]) en[r++] = DpEntry{s_bin[tid * P + c], c, s_size[tid * P + c]};
    }
    __syncthreads();                           // the check words are complete
    if (tid == 0) {
        const int status = s_flags[1] ? 3 : (s_flags[0] ? 1 : 0);  // 3: invalid input, 1: infeasible
        p.n_sweep[0] = total;
        p.n_sweep[1] = status;
        p.result[0] = status;
        p.result[5] = total;
        p.result[6] = (int64_t)__builtin_bit_cast(uint64_t, e_max);
        p.result[11] = (int64_t)s_chk[0];
        p.result[12] = (int64_t)s_chk[1];
    }
}

hipError_t launch_dp_build(const DpBuildParams& p, hipStream_t s, Section* sec) {
    if (p.L < 1 || p.L > kBuildThreads || p.P < 1 || p.P > kBuildMaxP || p.L * p.P > kBuildMaxLP)
        return hipErrorInvalidValue;
    launch_timed(sec, true, false, dp_build_kernel, dim3(1), dim3(kBuildThreads), 0, s, p);
    return hipGetLastError();
}

constexpr size_t kDpLdsBudget = 140 * 1024;     // dynamic LDS; ~17 KB more is static (160 KB per CU)

// How many layer groups a solve is split into: worth it once the sequential sweep (one pass over
// the row per entry: layers x entries x cells) takes several times what the extra launches cost.
static int auto_groups(const DpParams& p) {
    const double work = (double)p.L * p.max_count * (p.D + 1);
    return work >= 6e6 ? 8 : (work >= 3e6 ? 4 : 1);
}

template <typename T, int THREADS>
static hipError_t launch_dp_t(DpParams p, int max_bin, hipStream_t s, Section* sec, bool first) {
    constexpr int kMaxK = (LGRECO_MAX_BINS + 1 + THREADS - 1) / THREADS;
    const int nk = (p.D + 1 + THREADS - 1) / THREADS;
    int kmax = 1;
    while (kmax < nk) kmax *= 2;
    if (kmax > kMaxK) kmax = kMaxK;
    const int pad = (max_bin + 63) / 64 * 64;
    const bool padded = ((size_t)pad + (size_t)kmax * THREADS) * sizeof(T) <= kDpLdsBudget;
    p.pad = padded ? pad : 0;
    p.pd_stride = (p.D + 1 + 3) & ~3;
    size_t lds = ((size_t)p.pad + (size_t)kmax * THREADS) * sizeof(T);
    const size_t row_lds = lds;
    const size_t bt = (size_t)p.L * p.max_count * sizeof(uint16_t) + (size_t)p.L;
    p.bt_lds = lds + bt <= kDpLdsBudget ? 1 : 0;
    if (p.bt_lds) lds += bt;
    hipError_t err = hipSuccess;
    // layer groups: 32-bit costs, the padded row, the back-trace tables in LDS, one thread per layer
    int G = p.groups.G;
    const bool can_group = sizeof(T) == 4 && padded && p.bt_lds && p.max_count <= 64 && p.L <= THREADS &&
                           p.groups.nodes && p.groups.range && p.groups.flag &&
                           2 * (size_t)(p.D + 1) * sizeof(uint32_t) <= kDpLdsBudget;
    if (G == 0) G = auto_groups(p);
    if (!can_group || G < 2) G = 1;
    if (G > kDpMaxGroups) G = kDpMaxGroups;
    while (G & (G - 1)) G &= G - 1;                  // a power of two
    p.groups.G = G;
    p.groups.stride = p.pd_stride;
    bool first_pending = first;
    if (G > 1) {
        if (p.host_in) {
            launch_timed(sec, first_pending, false, dp_fetch_kernel, dim3((p.in_vec + 255) / 256), dim3(256), 0, s,
                         p.host_in, p.dev_in, (int)p.in_vec);
            first_pending = false;
            p.host_in = nullptr;
        }
#define LGRECO_DPG(K)                                                                              \
    do {                                                                                           \
        static bool configured = false;                                                            \
        if (!configured) {                                                                         \
            err = hipFuncSetAttribute((const void*)dp_group_kernel<K, THREADS>,                    \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)kDpLdsBudget); \
            if (err != hipSuccess) return err;                                                     \
            configured = true;                                                                     \
        }                                                                                          \
        launch_timed(sec, first_pending, false, dp_group_kernel<K, THREADS>, dim3(G), dim3(THREADS), row_lds, s, p); \
    } while (0)
        if (kmax == 1) LGRECO_DPG(1);
        else if (kmax == 2) LGRECO_DPG(2);
        else if (kmax == 4) LGRECO_DPG(4);
        else if (kmax == 8) LGRECO_DPG(8);
        else if (kmax == 16) LGRECO_DPG(16);
        else LGRECO_DPG(kMaxK);
#undef LGRECO_DPG
        first_pending = false;
        err = hipGetLastError();
        if (err != hipSuccess) return err;
        {
            static bool configured = false;
            if (!configured) {
                err = hipFuncSetAttribute((const void*)dp_conv_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                          (int)kDpLdsBudget);
                if (err != hipSuccess) return err;
                configured = true;
            }
        }
        const size_t conv_lds = 2 * (size_t)(p.D + 1) * sizeof(uint32_t);
        for (int nodes = G / 2; nodes >= 1; nodes /= 2) {      // the level above the leaves first, the root last
            // two cells per wavefront or more, and no more workgroups than fit the chip at once
            const int per_node = std::max(1, std::min(256 / nodes, (p.D + 1 + 31) / 32));
            hipLaunchKernelGGL(dp_conv_kernel, dim3(per_node, nodes), dim3(kConvThreads), conv_lds, s, p.groups,
                               nodes - 1, (int)p.D, p.L_dev);
        }
        {
            static bool configured = false;
            if (!configured) {
                err = hipFuncSetAttribute((const void*)dp_trace_kernel<THREADS>,
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)kDpLdsBudget);
                if (err != hipSuccess) return err;
                configured = true;
            }
        }
        // the trace finishes the solve; the sequential kernel behind it returns at once unless the
        // trace gave up (it also closes the section's bracket)
        hipLaunchKernelGGL(dp_trace_kernel<THREADS>, dim3(1), dim3(THREADS), bt, s, p);
        err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
#define LGRECO_DP2(K, PD)                                                                          \
    do {                                                                                           \
        static bool configured = false;   /* the limit is raised once per instantiation */        \
        if (!configured) {                                                                         \
            err = hipFuncSetAttribute((const void*)dp_kernel<T, K, PD, THREADS>,                   \
                                      hipFuncAttributeMaxDynamicSharedMemorySize,                  \
                                      (int)kDpLdsBudget);                                          \
            if (err != hipSuccess) return err;                                                     \
            configured = true;                                                                     \
        }                                                                                          \
        launch_timed(sec, first_pending, true, dp_kernel<T, K, PD, THREADS>, dim3(1), dim3(THREADS), lds, s, p); \
    } while (0)
#define LGRECO_DP(K) do { if (padded) LGRECO_DP2(K, true); else LGRECO_DP2(K, false); } while (0)
    if (kmax == 1) LGRECO_DP(1);
    else if (kmax == 2) LGRECO_DP(2);
    else if (kmax == 4) LGRECO_DP(4);
    else if (kmax == 8) LGRECO_DP(8);
    else if (kmax == 16) LGRECO_DP(16);
    else LGRECO_DP(kMaxK);
#undef LGRECO_DP
#undef LGRECO_DP2
    return hipGetLastError();
}

hipError_t launch_dp(const DpParams& p, bool narrow, int max_bin, hipStream_t s, Section* sec, bool first_in_section) {
    return narrow ? launch_dp_t<uint32_t, 1024>(p, max_bin, s, sec, first_in_section)
                  : launch_dp_t<int64_t, 1024>(p, max_bin, s, sec, first_in_section);
}

}  // namespace lgreco

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

// Thread t owns KMAX cells.  With an even KMAX they come in adjacent pairs (2t, 2t+1), (2t, 2t+1) +
// 2*threads, ...: the two reads row[e - b], row[e + 1 - b] of a pair are one ds_read2_b32 and the
// 64 lanes of a wavefront cover 128 consecutive cells without bank conflicts.
template <int KMAX, int THREADS>
__device__ __forceinline__ int dp_cell(int tid, int k) {
    return KMAX % 2 == 0 ? 2 * tid + (k & 1) + (k >> 1) * 2 * THREADS : tid + k * THREADS;
}

template <typename T, int KMAX, bool PADDED, int kDpThreads>
__global__ __launch_bounds__(kDpThreads) void dp_kernel(DpParams p) {
    // LDS row: [pad] cells of infinity, then cells 0 .. KMAX*threads-1 (cells above D stay infinite).
    // With PADDED the pad is at least the largest bin, so row[e - b] needs no range check.
    extern __shared__ unsigned char dp_smem[];
    T* const row = reinterpret_cast<T*>(dp_smem) + p.pad;
    __shared__ DpEntry s_entries[kDpStageEntries];      // [layers of the stage][max_count]
    __shared__ int32_t s_count[kDpStageMax];
    __shared__ int64_t s_val[kDpThreads / 64];
    __shared__ int32_t s_idx[kDpThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63;
    const int D = p.D;
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
        if (p.L_dev[1] != 0) {            // the build kernel reported the status; only the hand-over is left
            if (p.apply.layers)
                for (int l = tid; l < p.apply.L; l += kDpThreads) p.apply.layers[l].family = -1;
            if (tid == 0) {
                p.result[8] = 0;
                __threadfence_system();
                p.result[7] = p.seq;
            }
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

    const int stage = min(kDpStageMax, kDpStageEntries / bstride);     // layers per stage
    for (int l0 = 0; l0 < L; l0 += stage) {
        const int nl = min(stage, L - l0);
        __syncthreads();                              // previous stage fully consumed, row written
        for (int i = tid; i < nl * bstride; i += kDpThreads) {
            const DpEntry en = p.entries[(size_t)l0 * bstride + i];
            s_entries[i] = en;
            if (lds_bins) s_bins[(size_t)l0 * bstride + i] = (uint16_t)en.bin;
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
    __syncthreads();

    // arg-min of the last row, lowest e among equal minima
    int64_t bv = (int64_t)kInf;
    int32_t be = 0x7FFFFFFF;
    for (int e = tid; e <= D; e += kDpThreads) {
        const int64_t v = (int64_t)row[e];
        if (v < bv) { bv = v; be = e; }              // e ascending per thread -> keeps the lowest
    }
    for (int o = 1; o < 64; o <<= 1) {
        const int64_t ov = __shfl_xor(bv, o, 64);
        const int32_t oe = __shfl_xor(be, o, 64);
        if (ov < bv || (ov == bv && oe < be)) { bv = ov; be = oe; }
    }
    if (lane == 0) { s_val[tid >> 6] = bv; s_idx[tid >> 6] = be; }
    __syncthreads();
    uint64_t t_sweep = 0;
    if (tid < 64) {
        // the first wavefront: every lane joins the per-wavefront minima the same way
        if (tid == 0) t_sweep = wall_clock64();
        for (int w = 1; w < kDpThreads / 64; ++w)
            if (s_val[w] < bv || (s_val[w] == bv && s_idx[w] < be)) { bv = s_val[w]; be = s_idx[w]; }
        if (tid == 0) {
            s_val[0] = bv;
            s_idx[0] = be;
        }
        if (bv < (int64_t)kInf) {
            // The walk is a chain of dependent loads: one PD byte per layer from global memory,
            // the bin it stands for from LDS when the table fits there.
            int e = __builtin_amdgcn_readfirstlane(be);
            if (lds_bins && bstride <= 64) {
                // Two layers per load latency: lane j holds the bin of entry j of layer l, so
                // while PD[l][e] is on its way lane j already fetches PD[l-1][e - bin_j], the
                // byte the walk needs next if entry j is the one picked.  One wavefront runs
                // alone here and every instruction costs its full issue latency, so the loop is
                // kept short: rows by a running pointer, no branches, consistency checks joined
                // into one flag (a bad byte still gives in-row addresses: e only shrinks and is
                // clamped at 0, lanes past the list hold bin 0).
                auto bins_of = [&](int layer) -> uint32_t {
                    return lane < bstride ? (uint32_t)s_bins[max(layer, 0) * bstride + lane] : 0u;
                };
                int l = L - 1;
                uint32_t bins_cur = bins_of(l), bins_prev = bins_of(l - 1);
                const uint8_t* __restrict__ row_l = p.pd + (size_t)max(l, 0) * width;
                int bad = 0;
                for (; l >= 1; l -= 2, row_l -= 2 * width) {
                    const uint32_t bins_n1 = bins_of(l - 2), bins_n2 = bins_of(l - 3);
                    const uint32_t ka_v = row_l[e];
                    const uint32_t kb_v = (row_l - width)[max(e - (int)bins_cur, 0)];
                    const int ka = __builtin_amdgcn_readfirstlane((int)ka_v);
                    const int kb = (int)readlane_u32(kb_v, ka);
                    s_pick[l] = (uint8_t)ka;               // every lane writes the same byte
                    s_pick[l - 1] = (uint8_t)kb;
                    e -= (int)readlane_u32(bins_cur, ka) + (int)readlane_u32(bins_prev, kb);
                    bad |= (ka >= bstride) | (kb >= bstride) | (e < 0);
                    e = max(e, 0);
                    bins_cur = bins_n1;
                    bins_prev = bins_n2;
                }
                if (l == 0) {
                    const int ka = __builtin_amdgcn_readfirstlane((int)row_l[e]);
                    s_pick[0] = (uint8_t)ka;
                    e -= (int)readlane_u32(bins_cur, ka);
                    bad |= (ka >= bstride) | (e < 0);
                }
                if (bad) e = -1;                            // an internal inconsistency
            } else if (tid == 0) {
                if (lds_bins) {
                    for (int l = L - 1; l >= 0; --l) {
                        const int k = p.pd[(size_t)l * width + e];
                        s_pick[l] = (uint8_t)k;
                        e -= s_bins[l * bstride + k];
                    }
                } else {
                    for (int l = L - 1; l >= 0; --l) {
                        const int k = p.pd[(size_t)l * width + e];
                        const DpEntry en = p.entries[(size_t)l * bstride + k];
                        p.choice[l] = en.cand;
                        e -= en.bin;
                    }
                }
            }
            if (tid == 0) s_idx[1] = e;
        }
    }
    __syncthreads();
    const bool feasible = s_val[0] < (int64_t)kInf;
    const bool traced = feasible && lds_bins && s_idx[1] == 0;
    if (p.apply.layers) {
        // The compression's layer records from the assignment (see DpApply), one thread per
        // layer.  The staging area of the entry lists is free now: candidate per layer first
        // (fixed layers from the build's report, swept ones from the back-trace), then the payload
        // offsets, a running sum of the chosen sizes rounded up to 16 bytes.
        const DpApply& A = p.apply;
        static_assert(kDpThreads >= kBuildThreads, "one thread per layer");
        static_assert(sizeof(s_entries) >= kDpThreads + 8 * (kDpThreads / 64) + 8, "staging area too small");
        uint8_t* const s_chosen = reinterpret_cast<uint8_t*>(s_entries);                          // [threads]
        int64_t* const s_wtot = reinterpret_cast<int64_t*>(s_entries) + kDpThreads / 8;            // [waves]
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
        if (tid == 0) p.result[8] = ok ? 1 : 0;
    }
    // The result block lies in the host's pinned memory and the host may be polling it: the first
    // wavefront alone writes it (the other writer of host memory, the back-trace without LDS
    // tables, is its thread 0), puts a system-scope fence behind its stores and the launch's
    // sequence number behind the fence.
    if (tid >= 64) return;
    if (traced)
        for (int l = lane; l < L; l += 64)
            p.choice[l] = p.entries[(size_t)l * bstride + s_pick[l]].cand;
    if (tid == 0) {
        if (!feasible) {
            p.result[0] = 1;
            p.result[1] = 0;
            p.result[2] = 0;
        } else {
            p.result[0] = (s_idx[1] == 0) ? 0 : 2;   // 2 would be an internal inconsistency
            p.result[1] = s_val[0];
            p.result[2] = s_idx[0];
        }
        // diagnostics: ticks of the constant-rate (100 MHz) counter spent in sweep and back-trace
        p.result[3] = (int64_t)(t_sweep - t_begin);
        p.result[4] = (int64_t)(wall_clock64() - t_sweep);
    }
    __threadfence_system();
    if (tid == 0) p.result[7] = p.seq;
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
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int L = p.L, P = p.P, LP = L * P;
    const double D = (double)p.D;
    if (tid < 2) s_flags[tid] = 0;
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
    if (tid == 0) {
        const int status = s_flags[1] ? 3 : (s_flags[0] ? 1 : 0);  // 3: invalid input, 1: infeasible
        p.n_sweep[0] = total;
        p.n_sweep[1] = status;
        p.result[0] = status;
        p.result[5] = total;
        p.result[6] = (int64_t)__builtin_bit_cast(uint64_t, e_max);
    }
}

hipError_t launch_dp_build(const DpBuildParams& p, hipStream_t s, Section* sec) {
    if (p.L < 1 || p.L > kBuildThreads || p.P < 1 || p.P > kBuildMaxP || p.L * p.P > kBuildMaxLP)
        return hipErrorInvalidValue;
    launch_timed(sec, true, false, dp_build_kernel, dim3(1), dim3(kBuildThreads), 0, s, p);
    return hipGetLastError();
}

constexpr size_t kDpLdsBudget = 140 * 1024;     // dynamic LDS; ~17 KB more is static (160 KB per CU)

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
    const size_t bt = (size_t)p.L * p.max_count * sizeof(uint16_t) + (size_t)p.L;
    p.bt_lds = lds + bt <= kDpLdsBudget ? 1 : 0;
    if (p.bt_lds) lds += bt;
    hipError_t err = hipSuccess;
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
        launch_timed(sec, first, true, dp_kernel<T, K, PD, THREADS>, dim3(1), dim3(THREADS), lds, s, p); \
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

// Interfaces between the translation units of liblgreco.so (host side).
#pragma once

#include <algorithm>
#include <vector>

#include "common.h"

namespace lgreco {

// Optional per-kernel timing: each Section brackets the work enqueued during its lifetime with
// two HIP events on the call's stream.
struct Timing {
    static constexpr int kMaxSections = 32;
    int level = 0;          // 0 off, 1 main kernels, 2 every section
    bool ready = false;
    hipStream_t stream = nullptr;
    hipEvent_t ev[2 * kMaxSections]{};
    const char* name[kMaxSections]{};
    int n = 0;
};
struct Section {
    Timing* t;
    int idx = -1;
    Section(Timing* tt, const char* name, bool main_kernel = false) : t(tt) {
        if (t && t->level >= (main_kernel ? 1 : 2) && t->ready && t->n < Timing::kMaxSections) {
            idx = t->n++;
            t->name[idx] = name;
            (void)hipEventRecord(t->ev[2 * idx], t->stream);
        }
    }
    ~Section() {
        if (idx >= 0) (void)hipEventRecord(t->ev[2 * idx + 1], t->stream);
    }
    Section(const Section&) = delete;
    Section& operator=(const Section&) = delete;
};

// ---- quant.hip
hipError_t launch_quant_profile(const QuantParams& p, int n_tiles, bool hist, hipStream_t s);
hipError_t launch_reduce_partials(const double* partials, int stride, const int* cols, int ncols,
                                  const DevLayer* layers, int n_layers, double* errors, hipStream_t s);
hipError_t launch_quant_compress(const float* g, float* e, const DevLayer* layers, const Tile* tiles,
                                 int n_tiles, uint8_t* payload, bool stochastic, uint64_t seed,
                                 hipStream_t s);

// ---- dp.hip
struct DpEntry {            // one usable candidate of a layer (equal bins merged by the host)
    int32_t bin;
    int32_t cand;
    int64_t size;
};
struct DpParams {
    const DpEntry* entries;   // [L x max_count] swept layers only, in candidate order
    const int32_t* count;     // [L] entries per swept layer
    uint8_t* pd;              // [L x pd_stride] entry index per cell
    int32_t* choice;          // [L] candidate index per swept layer
    int64_t* result;          // [0] status (0 ok, 1 infeasible), [1] swept size, [2] final bin sum
    int32_t L, D;
    int32_t pad;              // set by launch_dp: cells of infinity in front of the LDS row
    int32_t pd_stride;        // set by launch_dp: bytes per PD row, a multiple of 4 and >= D + 2
    int32_t bt_lds;           // set by launch_dp: back-trace tables live in LDS behind the row
    int32_t max_count;        // largest entry count of a swept layer = row stride of `entries`
    // The input block (count | entries) as the host wrote it in pinned memory and its place in
    // device memory: the kernel's first step copies it over (in_vec 16-byte words), which saves
    // the separate copy operation and the wait between it and the kernel.  Null: nothing to copy.
    const uint4* host_in;
    uint4* dev_in;
    int32_t in_vec;
    // Not null: the entry lists were built on the device; [0] is the number of swept layers (L above
    // is then only the capacity the LDS tables are sized for), [1] the status the build found
    // (not 0: nothing to solve).
    const int32_t* L_dev;
};
// Entry lists built on the device from the error table (see dp_build_kernel).
constexpr int kBuildThreads = 1024;   // layers per solve on this path
constexpr int kBuildMaxP = 16;        // candidates per layer on this path
constexpr int kBuildMaxLP = 4096;     // table entries (layers x candidates) on this path: 64 KB of LDS
struct DpBuildParams {
    const double* errors;     // [L x P] device memory
    const int64_t* sizes;     // [L x P] device memory
    double* errors_host;      // [L x P] the host's pinned copy of the error table, written here
    int32_t L, P, D, default_cand;
    int32_t stride;           // row stride of `entries` (>= P)
    DpEntry* entries;         // out: swept layers, compacted
    int32_t* count;           // out [swept]
    int32_t* sweep_layer;     // out [swept] original index of every swept layer
    int32_t* fixed_choice;    // out [L] candidate of a layer fixed here, -1 otherwise
    int32_t* n_sweep;         // out, device memory, read by the sweep: [0] swept layers, [1] status
    int64_t* result;          // out: [0] status (0 ok, 1 infeasible, 3 invalid input), [5] swept layers,
                              //      [6] bit pattern of E_max
};
hipError_t launch_dp_build(const DpBuildParams& p, hipStream_t s);
// narrow: 32-bit costs (sum of the layers' largest sizes < 2^30)
// max_bin: largest bin in entries
hipError_t launch_dp(const DpParams& p, bool narrow, int max_bin, hipStream_t s);

// ---- topk.hip
struct TopkScratch {
    uint32_t* d_hist = nullptr;       // [2 x max_layers x kHistBins] exact coarse histogram, then the sample's
    void* d_tl = nullptr;             // per-layer selection records
    uint32_t* d_cand = nullptr;       // bit patterns of the candidates, tile i at its own first element
    uint32_t* d_cand_idx = nullptr;   // compress: index within the layer (+ sign bit) of every candidate
    uint32_t* d_k = nullptr;          // [max_layers x kMaxTopk] requested k (0 = layer inactive)
    uint32_t* d_lo = nullptr;         // [max_layers] lowest coarse key collected as a candidate
    uint32_t* d_hint[2] = {nullptr, nullptr};   // per kind of call: bound derived from the last thresholds
    bool hint_valid[2] = {false, false};
    bool reuse_thresholds = false;
    const uint32_t* lo_src = nullptr; // bound the main pass of this call collects with: d_lo or a d_hint
    bool hist_clean = false;          // the exact histogram is all zero (the last scan of a call clears it)
    int cur_slot = 0;
    int64_t* d_cand_base = nullptr;   // [max_layers] first candidate slot of every layer
    void* d_tilecnt = nullptr;        // per tile (above, equal) counts (compress)
    void* d_tilebase = nullptr;       // per tile exclusive prefix of those counts
    void* d_tinfo = nullptr;          // per tile, per wavefront: candidates written and where
    double* d_base_part = nullptr;    // per tile energy below the collection bound
    double* d_below_part = nullptr;   // refinement partial sums
    uint32_t* d_ref = nullptr;        // per-workgroup refinement histograms (counts, integer energies)
    size_t ref_words = 0;
    // control block, one upload per call and none when it repeats the last one:
    // [k | cand_base | work_range | work]; the pointers above and below are views into it
    // (two device copies: profile calls and compress calls alternate and each repeats itself)
    uint8_t* d_ctl[2] = {nullptr, nullptr};
    uint8_t* h_ctl = nullptr;         // pinned
    hipEvent_t ctl_copied = nullptr;  // recorded behind every upload from h_ctl
    bool ctl_pending = false;         // an upload was queued since h_ctl was last known to be free
    uint8_t* h_ctl_last[2] = {nullptr, nullptr};    // what each d_ctl holds
    size_t ctl_bytes = 0, ctl_last_bytes[2] = {0, 0};
    size_t ctl_off[4] = {0, 0, 0, 0}; // byte offsets of k, cand_base, work_range, work
    void* d_work = nullptr;           // refinement work table and per-layer ranges
    void* d_work_range = nullptr;
    void* h_work = nullptr;
    void* h_work_range = nullptr;
    int max_work = 0, n_work = 0;
    uint32_t* h_k = nullptr;
    int64_t* h_cand_base = nullptr;
    int64_t max_elems = 0;
    int max_layers = 0, max_tiles = 0;
};
hipError_t topk_scratch_create(TopkScratch* t, int64_t max_elems, int max_layers, int max_tiles);
void topk_scratch_destroy(TopkScratch* t);
// upload k per (layer, candidate), clear the histograms, sample the data and predict every
// layer's collection bound
hipError_t topk_begin(TopkScratch* t, const float* g, const float* e, const DevLayer* d_layers,
                      const DevLayer* h_layers, const Tile* d_tiles, int L, int n_tiles, int tile_elems,
                      const uint32_t* ks, int ntk, int slot, Timing* tm, hipStream_t s);
// replace the requested k by another group (each k no larger than the first group's largest)
hipError_t topk_regroup(TopkScratch* t, int L, const uint32_t* ks, int slot, hipStream_t s);
// main pass (exact coarse histogram + candidate collection) when no quantization candidate shares
// the read; otherwise the quantization profile kernel does the same work
hipError_t topk_collect(TopkScratch* t, const float* g, const float* e, float* ef_out, const DevLayer* d_layers,
                        const Tile* d_tiles, int n_tiles, hipStream_t s);
// exact threshold bins from the histogram; layers whose predicted bound was too high are
// collected again with the exact one
hipError_t topk_select(TopkScratch* t, const float* g, const float* e, float* ef_out, const DevLayer* d_layers,
                       const Tile* d_tiles, int L, int n_tiles, int ntk, bool first_group, bool last_group,
                       Timing* tm, hipStream_t s);
// refinement on the candidates: exact thresholds; writes the dropped energy to errors (if not null)
hipError_t topk_finalize(TopkScratch* t, const DevLayer* d_layers, const Tile* d_tiles, int L, int ntk,
                         const int* col, double* d_errors, int stride, Timing* tm, hipStream_t s);
hipError_t topk_compress(TopkScratch* t, const float* g, float* e, const DevLayer* d_layers,
                         const DevLayer* h_layers, const Tile* d_tiles, int L, int n_tiles, int tile_elems,
                         uint8_t* payload, Timing* tm, hipStream_t s);

// ---- lowrank.hip
struct LowrankScratch {
    void* host = nullptr;        // work tables and scratch buffers (grown on demand)
    int64_t max_elems = 0;
    int max_layers = 0, r_max = 0, power_iters = 1;
};
hipError_t lowrank_scratch_create(LowrankScratch* t, int64_t max_elems, int max_layers, int r_max,
                                  int power_iters);
void lowrank_scratch_destroy(LowrankScratch* t);
hipError_t lowrank_profile(LowrankScratch* t, const float* g, const float* e, const DevLayer* d_layers,
                           const DevLayer* h_layers, int L, const float* q0, int r_max, const int* rank,
                           const int* col, int nlr, double* d_errors, int stride, Timing* tm, hipStream_t s);
hipError_t lowrank_compress(LowrankScratch* t, const float* g, float* e, const DevLayer* d_layers,
                            const DevLayer* h_layers, int L, float* q, int r_max, uint8_t* payload, Timing* tm,
                            hipStream_t s);
// receiver side: out (+)= Phat Q^T from the payload
hipError_t lowrank_decompress(LowrankScratch* t, const DevLayer* h_layers, int L, int r_max, const uint8_t* payload,
                              float* out, bool accumulate, Timing* tm, hipStream_t s);

// ---- decode.hip: receiver side of quantization and Top-K, gradient accumulation
hipError_t launch_accumulate(float* acc, const float* g, int64_t n, bool reset, hipStream_t s);
hipError_t launch_decode(const uint8_t* payload, const DevLayer* layers, const Tile* tiles, int n_tiles,
                         float* out, bool accumulate, bool any_quant, bool any_topk, Timing* tm, hipStream_t s);

}  // namespace lgreco

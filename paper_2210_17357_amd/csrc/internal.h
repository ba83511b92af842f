// Interfaces between the translation units of liblgreco.so (host side).
#pragma once

#include <algorithm>
#include <cstring>
#include <vector>

#include <hip/hip_ext.h>

#include "common.h"

namespace lgreco {

// Optional per-kernel timing.  A Section covers the work enqueued during its lifetime with two HIP
// events of the call's stream.  A main-kernel section (the level-1 sections a benchmark keeps on
// inside its timed region) puts its events on the kernels themselves: launch_timed below hands
// the start event to the section's first kernel and the stop event to its last one, and
// hipExtLaunchKernelGGL takes the kernel's own begin and end timestamps, so the figure is the
// kernels' time without launch gaps.  The other sections record their events as separate stream
// operations.  Either way a timed kernel leaves about 5 us of the stream idle on either side
// (measured), which is why a call kind can be timed every n-th call only.
struct Timing {
    static constexpr int kMaxSections = 32;
    int level = 0;          // 0 off, 1 main kernels, 2 every section
    int every = 1;          // only every `every`-th call of this kind is timed
    int64_t calls = 0;      // calls of this kind since the level was set
    bool active = false;    // the call in progress is one of the timed ones
    bool ready = false;
    hipStream_t stream = nullptr;
    hipEvent_t ev[2 * kMaxSections]{};
    const char* name[kMaxSections]{};
    int n = 0;
    // Read-out: the events of the last call are turned into milliseconds once ("harvested"), at a
    // moment when the host has nothing better to do, and added to the totals since the level was set.
    bool harvested = true;
    float ms[kMaxSections]{};
    static constexpr int kMaxNames = 48;
    const char* total_name[kMaxNames]{};
    double total_ms[kMaxNames]{};
    int64_t total_count[kMaxNames]{};
    int n_totals = 0;
    // A phase bracket: two recorded events around everything a call (or a part of it) queues,
    // kept at level 1 like the main kernels.  Opened and closed by hand because one phase can
    // span two functions (the compression whose first kernel is queued behind the solver).
    int open_phase(const char* nm) {
        if (!(active && level >= 1 && ready && n < kMaxSections)) return -1;
        const int idx = n++;
        name[idx] = nm;
        (void)hipEventRecord(ev[2 * idx], stream);
        return idx;
    }
    void close_phase(int idx) {
        if (idx >= 0) (void)hipEventRecord(ev[2 * idx + 1], stream);
    }
    void add_total(const char* nm, double v) {
        int i = 0;
        while (i < n_totals && total_name[i] != nm && std::strcmp(total_name[i], nm) != 0) ++i;
        if (i == n_totals) {
            if (n_totals == kMaxNames) return;
            total_name[n_totals++] = nm;
            total_ms[i] = 0.0;
            total_count[i] = 0;
        }
        total_ms[i] += v;
        total_count[i] += 1;
    }
};
struct Section {
    Timing* t;
    int idx = -1;
    bool on_kernels = false;            // events are bound to kernels, not recorded
    bool start_taken = false, stop_taken = false;
    Section(Timing* tt, const char* name, bool main_kernel = false) : t(tt) {
        if (t && t->active && t->level >= (main_kernel ? 1 : 2) && t->ready && t->n < Timing::kMaxSections) {
            idx = t->n++;
            t->name[idx] = name;
            on_kernels = main_kernel;
            if (!on_kernels) (void)hipEventRecord(t->ev[2 * idx], t->stream);
        }
    }
    ~Section() {
        if (idx < 0) return;
        if (!on_kernels) {
            (void)hipEventRecord(t->ev[2 * idx + 1], t->stream);
        } else if (!start_taken && !stop_taken) {
            // nothing was launched inside: an empty bracket
            (void)hipEventRecord(t->ev[2 * idx], t->stream);
            (void)hipEventRecord(t->ev[2 * idx + 1], t->stream);
        } else if (!stop_taken) {
            (void)hipEventRecord(t->ev[2 * idx + 1], t->stream);
        }
    }
    hipEvent_t start_event() {
        if (idx < 0 || !on_kernels || start_taken) return nullptr;
        start_taken = true;
        return t->ev[2 * idx];
    }
    hipEvent_t stop_event() {
        if (idx < 0 || !on_kernels) return nullptr;
        stop_taken = true;
        return t->ev[2 * idx + 1];
    }
    Section(const Section&) = delete;
    Section& operator=(const Section&) = delete;
};

// Kernel launch inside a main-kernel section (sec may be null = plain launch): `first` / `last`
// say whether this is the section's first / last kernel.
template <typename... P, typename... A>
inline void launch_timed(Section* sec, bool first, bool last, void (*kernel)(P...), dim3 grid, dim3 block,
                         size_t lds, hipStream_t s, A&&... args) {
    static_assert(sizeof...(P) == sizeof...(A), "one argument per kernel parameter");
    hipEvent_t a = (sec && first) ? sec->start_event() : nullptr;
    hipEvent_t b = (sec && last) ? sec->stop_event() : nullptr;
    if (a || b)
        hipExtLaunchKernelGGL(kernel, grid, block, (std::uint32_t)lds, s, a, b, 0u, static_cast<P>(args)...);
    else
        hipLaunchKernelGGL(kernel, grid, block, lds, s, static_cast<P>(args)...);
}

// ---- quant.hip
// sec (may be null): the main-kernel section the launch belongs to
hipError_t launch_quant_profile(const QuantParams& p, int n_tiles, bool hist, hipStream_t s, Section* sec);
hipError_t launch_reduce_partials(const double* partials, int stride, const int* cols, int ncols,
                                  const DevLayer* layers, int n_layers, double* errors, hipStream_t s);
hipError_t launch_quant_compress(const float* g, float* e, const DevLayer* layers, const Tile* tiles,
                                 int n_tiles, uint8_t* payload, bool stochastic, uint64_t seed,
                                 hipStream_t s, Section* sec, size_t lds_pad = 0);   // lds_pad: LDS bytes requested and not used

// ---- dp.hip
struct DpEntry {            // one usable candidate of a layer (equal bins merged by the host)
    int32_t bin;
    int32_t cand;
    int64_t size;
};
// Optional last step of the solver kernel: turn the assignment into the per-layer records the
// compression kernels read (family, parameter, payload offset), so that a compression kernel
// queued right behind the solver needs nothing from the host.  The tables hold, per (layer,
// candidate), what the host would compute for that choice.  If the solve fails, the layout does
// not fit `capacity`, or the back-trace ran without its LDS tables, every record gets family -1
// (no compression kernel touches such a layer) and result[8] stays 0; otherwise result[8] = 1.
struct DpApply {
    DevLayer* layers;             // null: off
    const int32_t* sweep_layer;   // [swept] device copy of the build's report
    const int32_t* fixed_choice;  // [L]
    const int64_t* sizes;         // [L x P] bytes
    const int32_t* iparam;        // [L x P] bits / k / rank
    const int32_t* family;        // [P]
    const int32_t* topk_slot;     // [P] position of a Top-K candidate in the profile's selection records, else -1
    int32_t L, P;
    int64_t capacity;             // bytes the payload buffer holds
};
// Layer groups swept side by side (dp_group_kernel) and joined pairwise (dp_conv_kernel): a
// complete binary tree in heap order, node 0 the whole table, leaves G-1 .. 2G-2 the groups in
// layer order, the left child of a node holding the lower layers.
struct DpGroups {
    int32_t G = 0;                // in: 0 = let launch_dp decide, 1 = off, 2 / 4 / 8 = forced; out: groups used (0 / 1: none)
    int32_t stride = 0;           // cells per node array (set by launch_dp, > D)
    uint32_t* nodes = nullptr;    // [(2G-1) x stride] smallest size of a node's layers per exact bin sum (null: groups off)
    int32_t* range = nullptr;     // [G x 2] swept layers [begin, end) of every group, written by the group sweeps
    int32_t* flag = nullptr;      // [1] written by dp_trace_kernel: 1 = it gave up, the sequential kernel behind it solves
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
    // Written to result[7] as the kernel's last store (after a system-scope fence): the host
    // may poll the pinned result block for it instead of waiting for the stream.
    int64_t seq;
    DpApply apply;
    DpGroups groups;
    // The traced-back assignment starts from the best cell among 0 .. min(D, e_limit) of the last
    // row (the strict budget looks at fewer cells than the table has; negative: none, no
    // assignment fits).
    int32_t e_limit = 0x7FFFFFFF;
};
// Entry lists built on the device from the error table (see dp_build_kernel).
constexpr int kBuildThreads = 1024;   // layers per solve on this path
constexpr int kBuildMaxP = 16;        // candidates per layer on this path
constexpr int kBuildMaxLP = 4096;     // table entries (layers x candidates) on this path: 64 KB of LDS
struct DpBuildParams {
    const double* errors;     // [L x P] device memory
    const int64_t* sizes;     // [L x P] device memory
    double* errors_host;      // [L x P] the host's pinned copy of the error table, written here (may be null)
    int32_t L, P, D, default_cand;
    int32_t stride;           // row stride of `entries` (>= P)
    DpEntry* entries;         // out: swept layers, compacted
    int32_t* count;           // out [swept]
    int32_t* sweep_layer;     // out [swept] original index of every swept layer
    int32_t* fixed_choice;    // out [L] candidate of a layer fixed here, -1 otherwise
    int32_t* sweep_layer_dev; // the same two in device memory, for the solver's apply step
    int32_t* fixed_choice_dev;
    int32_t* n_sweep;         // out, device memory, read by the sweep: [0] swept layers, [1] status
    int64_t* result;          // out: [0] status (0 ok, 1 infeasible, 3 invalid input), [5] swept layers,
                              //      [6] bit pattern of E_max
    int32_t check_sizes;      // 1: also reject (status 3) sizes this path's 32-bit costs cannot hold
};
hipError_t launch_dp_build(const DpBuildParams& p, hipStream_t s, Section* sec);
// narrow: 32-bit costs (sum of the layers' largest sizes < 2^30)
// max_bin: largest bin in entries
// sec (may be null): the section's last kernel, and its first one too when `first_in_section`
hipError_t launch_dp(const DpParams& p, bool narrow, int max_bin, hipStream_t s, Section* sec,
                     bool first_in_section);

// ---- topk.hip
struct TopkScratch {
    uint32_t* d_hist = nullptr;       // [2 x max_layers x kHistBins] exact coarse histogram, then the sample's
    void* d_tl = nullptr;             // per-layer selection records
    uint32_t* d_cnt_known = nullptr;  // [max_layers x 512] sub-bin counts of topk_compress_known
    uint32_t* d_cand = nullptr;       // bit patterns of the candidates, tile i at its own first element
    uint32_t* d_cand_idx = nullptr;   // compress: index within the layer (+ sign bit) of every candidate; a profile that
                                      // records where its candidates are uses it for 16-bit entries (place in tile, sign)
    bool cand_has_idx = false;        // the current call's profile recorded d_cand_idx too
    // compression from the profile's candidates: what is kept of them, in element order
    uint32_t* d_kept = nullptr;
    uint32_t* d_kept_idx = nullptr;
    void* d_tinfo_kept = nullptr;
    uint32_t* d_k = nullptr;          // [max_layers x kMaxTopk] requested k (0 = layer inactive)
    uint32_t* d_lo = nullptr;         // [max_layers] lowest coarse key collected as a candidate
    // what a second collection reads and writes (noted by topk_select for the refinement kernel)
    const float* rc_g = nullptr;
    const float* rc_e = nullptr;
    float* rc_ef_out = nullptr;
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
    int max_items = 0;          // most work items of one layer in the current call
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
                        const Tile* d_tiles, int n_tiles, hipStream_t s, Section* sec, float* x_out = nullptr);
// exact threshold bins from the histogram; layers whose predicted bound was too high are
// collected again with the exact one
// quant (may be null): the quantization profile's per-tile partial sums, reduced per layer by extra
// workgroups of the scan's launch instead of a kernel of their own
struct QuantReduce {
    const double* partials;
    double* errors;
    int stride;
    const int* cols;
    int ncols;
};
hipError_t topk_select(TopkScratch* t, const float* g, const float* e, float* ef_out, const DevLayer* d_layers,
                       const Tile* d_tiles, int L, int n_tiles, int ntk, bool first_group, bool last_group,
                       Timing* tm, hipStream_t s, const QuantReduce* quant);
// refinement on the candidates: exact thresholds; writes the dropped energy to errors (if not null)
hipError_t topk_finalize(TopkScratch* t, const DevLayer* d_layers, const Tile* d_tiles, int L, int ntk,
                         const int* col, double* d_errors, int stride, Timing* tm, hipStream_t s);
hipError_t topk_compress(TopkScratch* t, const float* g, float* e, const DevLayer* d_layers,
                         const DevLayer* h_layers, const Tile* d_tiles, int L, int n_tiles, int tile_elems,
                         uint8_t* payload, Timing* tm, hipStream_t s, bool x_in_e = false);

// Top-K layers of a compression queued right behind a profile of the same data and the solver
// kernel that wrote the layer records (family, k, payload offset, slot of the chosen density in
// the profile's selection records): nothing here needs the host to know the assignment.
// shared_chip: another stream's kernel fills most of the chip meanwhile (the scan of the counts
// then runs in workgroups small enough to be placed beside it).
hipError_t topk_compress_known(TopkScratch* t, const float* g, float* e, const DevLayer* d_layers,
                               const Tile* d_tiles, int L, int n_tiles, uint8_t* payload, Timing* tm, hipStream_t s,
                               bool x_in_e = false, bool shared_chip = false);

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
// low-rank layers of a compression queued right behind a profile of the same data (see topk_compress_known)
hipError_t lowrank_compress_known(LowrankScratch* t, const float* g, float* e, const DevLayer* d_layers, float* q,
                                  int r_max, uint8_t* payload, Timing* tm, hipStream_t s,
                                  bool e_is_zero = false);   // e_is_zero: e holds zeros on entry (the caller's promise) and is not read
// receiver side: out (+)= Phat Q^T from the payload
hipError_t lowrank_decompress(LowrankScratch* t, const DevLayer* h_layers, int L, int r_max, const uint8_t* payload,
                              float* out, bool accumulate, Timing* tm, hipStream_t s);

// ---- decode.hip: receiver side of quantization and Top-K, gradient accumulation
hipError_t launch_accumulate(float* acc, const float* g, int64_t n, bool reset, hipStream_t s, Section* sec);
hipError_t launch_decode(const uint8_t* payload, const DevLayer* layers, const Tile* tiles, int n_tiles,
                         float* out, bool accumulate, bool any_quant, bool any_topk, Timing* tm, hipStream_t s);

}  // namespace lgreco

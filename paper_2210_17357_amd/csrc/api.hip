// C ABI of liblgreco.so: handle, argument checks, host-side tables (sizes, bins, tiles,
// payload layout) and the launch sequence of each entry point.
#include <algorithm>
#include <atomic>
#include <chrono>
#include <cmath>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "common.h"
#include "internal.h"

using namespace lgreco;

struct lgreco_handle {
    lgreco_config_t cfg{};
    int64_t max_elems = 0;
    int32_t max_layers = 0, max_cands = 0;
    int device = 0;
    std::string hip_error;

    // layer table cache (rebuilt only when the caller's table changes)
    std::vector<lgreco_layer_t> cached;
    std::vector<DevLayer> hl;
    std::vector<Tile> ht;
    int64_t total_elems = 0;
    bool layers_dirty = true;       // device copy of hl is stale
    // second stream of the one-call path: the quantized layers' compression runs there beside the
    // Top-K layers' chain of short kernels (default priority, joined before the call goes on)
    hipStream_t side = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;

    DevLayer* d_layers = nullptr;
    Tile* d_tiles = nullptr;
    int32_t max_tiles = 0;
    int32_t tile_elems = kTile;     // tile size of the current layer table
    double* d_partials = nullptr;   // [max_tiles x max_cands]
    double* h_errors = nullptr;     // [max_layers x max_cands], pinned host memory
    double* d_errors = nullptr;     // the same memory as the kernels address it

    TopkScratch topk;
    LowrankScratch lowrank;

    // solver
    // input block [count | entries]: one upload; output block [result | choice]: pinned host
    // memory the kernel writes
    uint8_t* d_dp_in = nullptr;
    uint8_t* h_dp_in = nullptr;     // pinned
    const uint4* d_dp_in_host = nullptr;   // h_dp_in as the kernel addresses it
    uint8_t* h_dp_out = nullptr;    // pinned
    uint8_t* d_dp_out = nullptr;    // h_dp_out as the kernel addresses it
    size_t dp_entries_off = 0;      // byte offset of the entries inside the input block
    DpEntry* d_entries = nullptr;   // views into the blocks
    int32_t* d_count = nullptr;
    uint8_t* d_pd = nullptr;
    int32_t* d_choice = nullptr;
    int64_t* d_result = nullptr;
    int32_t* h_bins = nullptr;      // pinned: original index of every swept layer
    DpEntry* h_entries = nullptr;
    int32_t* h_count = nullptr;
    int32_t* h_choice = nullptr;
    int64_t* h_result = nullptr;
    // lgreco_profile_solve: error and size tables in device memory for the device-side entry build
    // (the sizes with a pinned staging copy, uploaded when they change), what the build reports back
    // (pinned: sweep_layer | fixed_choice) and the swept-layer count / status it hands the sweep
    int64_t* h_sizes = nullptr;
    int64_t* d_sizes = nullptr;
    size_t sizes_count = 0;            // entries of h_sizes / d_sizes in use
    double* d_errors_dev = nullptr;    // error table in device memory (the build forwards it to h_errors)
    int32_t* h_build = nullptr;
    int32_t* d_build_host = nullptr;
    int32_t* d_nsweep = nullptr;
    int64_t dp_seq = 0;                  // sequence number of the last solver launch
    int64_t last_solve_groups = 0;       // how the last solve swept its table (the kernel's report)
    // layer groups of the solver (see DpGroups): tree nodes, group ranges
    bool ef_zero_on_entry = false;          // lgreco_set_ef_zero_on_entry
    int64_t late_handovers = 0;             // solves whose result block was incomplete when its sequence number arrived
    uint32_t* d_dp_nodes = nullptr;
    int32_t* d_dp_range = nullptr;
    // lgreco_profile_solve_compress: what the solver kernel needs to write the compression's layer
    // records itself - device copies of the build's report and, per (layer, candidate), the integer
    // parameter a choice stands for plus the family per candidate (pinned staging copy, uploaded
    // when it changes)
    int32_t* d_build_dev = nullptr;      // [2 x max_layers] sweep_layer | fixed_choice
    int32_t* h_apply = nullptr;          // pinned [max_layers x max_cands | max_cands | max_cands] iparam | family | Top-K slot
    int32_t* d_apply = nullptr;
    size_t apply_count = 0;              // int32 entries of h_apply / d_apply in use
    std::vector<DevLayer> hl_uploaded;   // what d_layers holds
    // Top-K candidates of the last profile call: how many, and the candidate column of each of the
    // selection records it left on the device (valid while they number at most one group)
    int last_ntk = 0;
    int last_tk_col[kMaxTopk] = {};
    int last_nlr = 0;                    // low-rank candidates of the last profile call
    std::vector<DpEntry> build_entries;  // [max_layers x LGRECO_MAX_CANDS] host scratch of lgreco_solve

    // One set of timing events per kind of call (LGRECO_CALL_*): a call that returns before its
    // kernels have finished (lgreco_compress) keeps its brackets while the next call of another
    // kind records its own.  tm is the set of the call in progress / the last call.
    Timing tms[4];
    Timing* tm = &tms[0];
    // sub-sections measured inside a kernel (device clock), appended after the solve call's event sections
    const char* sub_name[4]{};
    float sub_ms[4]{};
    int n_sub = 0;
};

namespace {

constexpr int kDpResultSlots = 16;      // int64 words at the head of the solver's result block
constexpr int kMaxDpGroups = 8;         // layer groups the solver may sweep side by side

DpGroups dp_groups(const lgreco_handle* h) {
    DpGroups g;
    g.G = h->cfg.dp_groups;             // 0: chosen per solve from its size
    g.nodes = h->d_dp_nodes;
    g.range = h->d_dp_range;
    g.flag = h->d_dp_range + 2 * kMaxDpGroups;
    return g;
}

// lgreco_profile_solve_compress: the compression's first kernel queued behind the solver.
struct EarlyCompress {
    float* d_ef;
    uint8_t* d_payload;
    int64_t capacity;
    int phase = -1;          // the compress call's phase bracket, opened with that kernel
    bool topk_known = false; // the Top-K layers' kernels were queued too (see topk_compress_known)
    bool lowrank_known = false;   // ... and the low-rank layers' (see lowrank_compress_known)
    float* d_q = nullptr;    // warm start, updated by the low-rank compression
    // the profile leaves x = fl32(g + e) in the error-feedback buffer and the compression reads it
    // there (no second read of g, and no pass over the Top-K layers that rewrites what is not kept)
    bool x_in_e = false;
    bool launched = false;   // the quantization kernel was queued right behind the solver kernel
    bool applied = false;    // ... and ran on layer records the solver kernel wrote from its result
};

int hip_fail(lgreco_handle* h, hipError_t e, const char* what) {
    if (h) h->hip_error = std::string(what) + ": " + hipGetErrorString(e);
    return LGRECO_EHIP;
}
#define HIPCHK(expr)                                             \
    do {                                                         \
        hipError_t _e = (expr);                                  \
        if (_e != hipSuccess) return hip_fail(h, _e, #expr);     \
    } while (0)

int64_t quant_size(int64_t n, int bits, int bucket) {
    const int64_t full = n / bucket, rem = n % bucket;
    int64_t s = full * ((int64_t)bucket * bits / 8 + 8);
    if ((bucket * bits) % 8 != 0) {     // generic bucket sizes: per-bucket byte rounding
        s = full * (((int64_t)bucket * bits + 7) / 8 + 8);
    }
    if (rem) s += (rem * bits + 7) / 8 + 8;
    return s;
}

int64_t topk_k(int64_t n, double d) {
    const double v = std::floor(d * (double)n + 0.5);
    int64_t k = (v >= 9.0e18) ? n : (int64_t)v;
    if (k < 1) k = 1;
    if (k > n) k = n;
    return k;
}

int check_cand(const lgreco_cand_t& c, const lgreco_layer_t* layer, int r_max) {
    switch (c.family) {
        case LGRECO_QUANT:
            if (!(c.param >= 1.0 && c.param <= 8.0) || c.param != std::floor(c.param)) return LGRECO_EINVAL;
            return LGRECO_OK;
        case LGRECO_TOPK:
            if (!(c.param > 0.0 && c.param <= 1.0)) return LGRECO_EINVAL;
            return LGRECO_OK;
        case LGRECO_LOWRANK:
            if (!(c.param >= 1.0) || c.param != std::floor(c.param)) return LGRECO_EINVAL;
            if (r_max > 0 && c.param > (double)r_max) return LGRECO_EINVAL;
            if (layer && (layer->rows <= 0 || layer->cols <= 0)) return LGRECO_EINVAL;
            return LGRECO_OK;
        default:
            return LGRECO_EINVAL;
    }
}

int check_layers(const lgreco_layer_t* layers, int32_t L) {
    if (!layers || L <= 0) return LGRECO_EINVAL;
    std::vector<std::pair<int64_t, int64_t>> r;
    r.reserve(L);
    for (int l = 0; l < L; ++l) {
        const lgreco_layer_t& a = layers[l];
        if (a.offset < 0 || a.numel <= 0 || a.numel >= ((int64_t)1 << 31)) return LGRECO_EINVAL;
        if (a.rows < 0 || a.cols < 0) return LGRECO_EINVAL;
        if (a.rows > 0 && (int64_t)a.rows * a.cols != a.numel) return LGRECO_EINVAL;
        r.emplace_back(a.offset, a.offset + a.numel);
    }
    std::sort(r.begin(), r.end());
    for (int l = 1; l < L; ++l)
        if (r[l].first < r[l - 1].second) return LGRECO_EINVAL;
    return LGRECO_OK;
}

// Rebuild the tile table if the caller's layer table differs from the cached one.
int prepare_layers(lgreco_handle* h, const lgreco_layer_t* layers, int32_t L) {
    if ((int)h->cached.size() == L && std::memcmp(h->cached.data(), layers, sizeof(lgreco_layer_t) * L) == 0)
        return LGRECO_OK;
    int st = check_layers(layers, L);
    if (st != LGRECO_OK) return st;
    if (L > h->max_layers) return LGRECO_ENOSPACE;
    int64_t total = 0;
    for (int l = 0; l < L; ++l) total += layers[l].numel;
    if (total > h->max_elems) return LGRECO_ENOSPACE;

    // tile size: see kTilesFill
    int tile = kTile;
    while (tile > kTileMin && total / tile < kTilesFill) tile /= 2;
    h->tile_elems = tile;
    h->hl.assign(L, DevLayer{});
    h->ht.clear();
    int64_t qoff = 0;
    for (int l = 0; l < L; ++l) {
        const lgreco_layer_t& a = layers[l];
        DevLayer& d = h->hl[l];
        d.offset = a.offset;
        d.numel = a.numel;
        d.rows = a.rows;
        d.cols = a.cols;
        d.q_offset = qoff;
        qoff += (int64_t)a.cols * h->cfg.r_max;
        d.tile_begin = (int32_t)h->ht.size();
        const bool aligned = (a.offset % 4) == 0;
        int64_t pos = 0, n = a.numel;
        auto push = [&](int64_t cnt, int fast) {
            h->ht.push_back(Tile{pos, l, (int32_t)cnt, fast, 0});
            pos += cnt;
        };
        while (n - pos >= tile) push(tile, aligned ? 1 : 0);
        const int64_t rem = n - pos;
        if (aligned) {
            const int64_t mid = (rem / kChunk) * kChunk;
            if (mid) push(mid, 1);
            if (rem - mid) push(rem - mid, 0);
        } else if (rem) {
            push(rem, 0);
        }
        d.tile_end = (int32_t)h->ht.size();
    }
    if ((int64_t)h->ht.size() > h->max_tiles) return LGRECO_ENOSPACE;
    h->cached.assign(layers, layers + L);
    h->total_elems = total;
    h->layers_dirty = true;
    return LGRECO_OK;
}

// The tile table travels only when it was rebuilt; the layer records also when the caller changed
// their per-call fields (family, parameter, payload offset).  The copies read the handle's host
// vectors, which the next call may rewrite while this call's kernels are still queued
// (lgreco_compress does not wait at its end): a call that uploads waits for its copies here.  In a
// loop that repeats one table and one choice nothing is uploaded and nothing waits.
int upload_layers(lgreco_handle* h, hipStream_t s, bool layers_changed) {
    bool copied = false;
    if (h->layers_dirty || (layers_changed && (h->hl_uploaded.size() != h->hl.size() ||
                                               std::memcmp(h->hl_uploaded.data(), h->hl.data(),
                                                           sizeof(DevLayer) * h->hl.size()) != 0))) {
        HIPCHK(hipMemcpyAsync(h->d_layers, h->hl.data(), sizeof(DevLayer) * h->hl.size(), hipMemcpyHostToDevice,
                              s));
        h->hl_uploaded = h->hl;
        copied = true;
    }
    if (h->layers_dirty) {
        HIPCHK(hipMemcpyAsync(h->d_tiles, h->ht.data(), sizeof(Tile) * h->ht.size(), hipMemcpyHostToDevice, s));
        copied = true;
    }
    h->layers_dirty = false;
    if (copied) HIPCHK(hipStreamSynchronize(s));
    return LGRECO_OK;
}

// Turns the brackets of the last call of one kind into milliseconds (waits for them) and adds
// them to the totals.  Does nothing when that was done already or nothing was recorded.
hipError_t harvest(Timing& tm) {
    if (tm.harvested || tm.n == 0) return hipSuccess;
    tm.harvested = true;
    // (a phase bracket closes after the sections opened inside it: every stop event is waited for)
    hipError_t e = hipSuccess;
    for (int i = 0; i < tm.n && e == hipSuccess; ++i) {
        e = hipEventSynchronize(tm.ev[2 * i + 1]);
        if (e != hipSuccess) break;
        e = hipEventElapsedTime(&tm.ms[i], tm.ev[2 * i], tm.ev[2 * i + 1]);
        if (e == hipSuccess) tm.add_total(tm.name[i], (double)tm.ms[i]);
    }
    if (e != hipSuccess) tm.n = 0;
    return e;
}

// Brackets of asynchronous calls (lgreco_compress) that are still unread: a call that is about to
// wait for the stream anyway reads them first - their kernels were queued before its own, so the
// wait costs it nothing - and a loop that alternates the calls never waits for timing elsewhere.
void harvest_others(lgreco_handle* h) {
    if (h->tm->level == 0) return;
    for (Timing& t : h->tms)
        if (&t != h->tm) (void)harvest(t);
}

// A call starts: its kind's brackets of the previous call are read out if nobody did (with timing
// on, a call therefore waits for the previous call of its kind), then the set is reused.
void begin_call(lgreco_handle* h, hipStream_t s, int kind) {
    h->tm = &h->tms[kind];
    (void)harvest(*h->tm);
    h->tm->n = 0;
    h->tm->active = h->tm->level > 0 && (h->tm->calls++ % h->tm->every) == 0;
    h->tm->harvested = !h->tm->active;
    h->tm->stream = s;
    if (kind == LGRECO_CALL_SOLVE) h->n_sub = 0;
}

// Waits for the solver launch `seq` to hand over its result block.  The kernel writes the block
// straight into pinned host memory and stores its sequence number last (slot 7), behind a
// system-scope fence: polling that word sees the end of the solve several microseconds before a
// stream synchronisation returns (the stream is still retiring the kernel then; the caller's next
// launches queue behind it as usual).  Nothing else is asked of the stream meanwhile - a status
// query can put a marker into the queue, which then sits between this call's kernels and the
// next ones.
// The hand-over does not lean on the order in which the kernel's stores reach host memory: both
// 64-byte halves of the block carry a copy of the sequence number (slots 4 and 15, written with
// the block's other slots by one store), and the assignment is covered by a check word (slot 10,
// the sum of (candidate + 1) * (swept layer + 1)).  The block is taken as complete when all three
// sequence words agree and, for a solved table, the assignment in memory adds up to the check
// word; until then the host keeps polling.  Whatever does not arrive within the limit (a solve
// that long, a launch that failed) ends in an ordinary stream synchronisation, which also brings
// up any error, and a block that still does not add up then is reported, never used.
// What the list-building kernel (an earlier launch of the same call) left in host memory - the
// error table and its report of fixed and swept layers - has check words of its own (slots 11,
// 12) and is held against them in the same way.
//   n_choice: swept layers whose assignment follows the block; < 0: lists built on the device,
//   the count is in slot 5 and the error table (L x P) and the report are checked as well
int wait_for_solver(lgreco_handle* h, int64_t seq, hipStream_t s, int n_choice, int L = 0, int P = 0) {
    volatile const int64_t* const r = h->h_result;
    volatile const int32_t* const ch = h->h_choice;
    auto complete = [&]() -> bool {
        if (r[7] != seq || r[4] != seq || r[15] != seq) return false;
        const int n = n_choice >= 0 ? n_choice : (int)r[5];
        if (n < 0 || n > h->max_layers) return false;
        if (n_choice < 0) {
            volatile const uint64_t* const eb = reinterpret_cast<volatile const uint64_t*>(h->h_errors);
            uint64_t ce = 0;
            for (int i = 0; i < L * P; ++i) ce += eb[i] * (uint64_t)(i + 1);
            if (ce != (uint64_t)r[11]) return false;
            if (r[0] == 0) {                     // the report is read for a solved table only
                volatile const int32_t* const sweep_layer = h->h_build;
                volatile const int32_t* const fixed_choice = h->h_build + L;
                uint64_t cb = 0;
                for (int l = 0; l < L; ++l) cb += (uint64_t)(uint32_t)(fixed_choice[l] + 2) * (uint64_t)(l + 1);
                for (int i = 0; i < n; ++i) cb += 65537ull * (uint64_t)(sweep_layer[i] + 1) * (uint64_t)(i + 1);
                if (cb != (uint64_t)r[12]) return false;
            }
        }
        if (r[0] != 0) return true;                          // nothing was traced back
        uint64_t sum = 0;
        for (int i = 0; i < n; ++i) sum += (uint64_t)(uint32_t)(ch[i] + 1) * (uint64_t)(i + 1);
        return sum == (uint64_t)r[10];
    };
    const auto t0 = std::chrono::steady_clock::now();
    bool ok = false;
    bool counted = false;
    for (uint32_t polls = 1;; ++polls) {
        if (r[7] == seq) {
            if ((ok = complete())) break;
            if (!counted) {                  // the sequence number was there before the rest of the block
                ++h->late_handovers;
                counted = true;
            }
        }
        if ((polls & 0x3FFu) == 0 && std::chrono::steady_clock::now() - t0 > std::chrono::milliseconds(50)) break;
#if !defined(__HIP_DEVICE_COMPILE__) && (defined(__x86_64__) || defined(__i386__))
        asm volatile("pause");
#endif
    }
    if (!ok) {
        HIPCHK(hipStreamSynchronize(s));
        if (!complete()) {
            h->hip_error = r[7] != seq ? "the solver kernel did not report"
                                       : "the solver's result block and its check words disagree";
            return LGRECO_EHIP;
        }
    }
    std::atomic_thread_fence(std::memory_order_acquire);
    return LGRECO_OK;
}

// Device-clock sub-sections of the solve (100 MHz constant-rate counter).
void record_dp_sub(lgreco_handle* h) {
    h->sub_name[0] = "dp_solve.sweep";
    h->sub_ms[0] = (float)((double)((uint64_t)h->h_result[3] & 0xFFFFFFFFull) * 1e-5);
    h->sub_name[1] = "dp_solve.backtrace";
    h->sub_ms[1] = (float)((double)((uint64_t)h->h_result[3] >> 32) * 1e-5);
    h->n_sub = 2;
    for (int j = 0; j < 2; ++j) h->tms[LGRECO_CALL_SOLVE].add_total(h->sub_name[j], (double)h->sub_ms[j]);
}

}  // namespace

extern "C" {

const char* lgreco_strerror(int status) {
    switch (status) {
        case LGRECO_OK: return "ok";
        case LGRECO_EINVAL: return "invalid argument";
        case LGRECO_ENOSPACE: return "problem exceeds the limits given to lgreco_create";
        case LGRECO_EINFEASIBLE: return "no assignment fits the error budget";
        case LGRECO_EHIP: return "HIP runtime error";
        case LGRECO_EUNSUPPORTED: return "not supported by this build";
        default: return "unknown status";
    }
}

const char* lgreco_last_hip_error(const lgreco_handle_t* h) { return h ? h->hip_error.c_str() : ""; }

int lgreco_last_solve_groups(const lgreco_handle_t* h) {
    if (!h) return LGRECO_EINVAL;
    return (int)h->last_solve_groups;
}

int64_t lgreco_late_handovers(const lgreco_handle_t* h) { return h ? h->late_handovers : 0; }

int lgreco_set_ef_zero_on_entry(lgreco_handle_t* h, int32_t on) {
    if (!h) return LGRECO_EINVAL;
    h->ef_zero_on_entry = on != 0;
    return LGRECO_OK;
}

int lgreco_create(lgreco_handle_t** out, const lgreco_config_t* cfg, int64_t max_elems, int32_t max_layers,
                  int32_t max_cands) {
    if (!out || !cfg || max_elems <= 0 || max_layers <= 0 || max_cands <= 0) return LGRECO_EINVAL;
    if (max_cands > LGRECO_MAX_CANDS) return LGRECO_EINVAL;
    if (cfg->bucket != kBucket) return LGRECO_EUNSUPPORTED;
    if (cfg->power_iters < 1 || cfg->power_iters > 16) return LGRECO_EUNSUPPORTED;
    if (cfg->r_max < 0 || cfg->r_max > 64) return LGRECO_EUNSUPPORTED;
    if (cfg->strict_budget != 0 && cfg->strict_budget != 1) return LGRECO_EINVAL;
    if (cfg->keep_ef_on_failure != 0 && cfg->keep_ef_on_failure != 1) return LGRECO_EINVAL;
    if (cfg->dp_groups != 0 && cfg->dp_groups != 1 && cfg->dp_groups != 2 && cfg->dp_groups != 4 &&
        cfg->dp_groups != 8)
        return LGRECO_EINVAL;
    lgreco_handle* h = new (std::nothrow) lgreco_handle();
    if (!h) return LGRECO_ENOSPACE;
    h->cfg = *cfg;
    h->max_elems = max_elems;
    h->max_layers = max_layers;
    h->max_cands = max_cands;
    *out = h;
    auto fail = [&](int st) {
        lgreco_destroy(h);
        *out = nullptr;
        return st;
    };
#define HIPCHK_C(expr)                                                      \
    do {                                                                    \
        hipError_t _e = (expr);                                             \
        if (_e != hipSuccess) { hip_fail(h, _e, #expr); return fail(LGRECO_EHIP); } \
    } while (0)
    HIPCHK_C(hipGetDevice(&h->device));
    h->max_tiles = (int32_t)std::min<int64_t>(max_elems / kTileMin + 2 * (int64_t)max_layers + 2, INT32_MAX);
    HIPCHK_C(hipMalloc(&h->d_layers, sizeof(DevLayer) * max_layers));
    HIPCHK_C(hipMalloc(&h->d_tiles, sizeof(Tile) * h->max_tiles));
    HIPCHK_C(hipMalloc(&h->d_partials, sizeof(double) * (size_t)h->max_tiles * max_cands));
    // Small results (the error table, the solver's output) are written by the kernels straight into
    // pinned host memory: no copy operation between the last kernel and the host's wait.
    // Memory the kernels write and the host reads (or the other way round) while kernels may still
    // be running is asked for as coherent whatever the process's default is: the solver's
    // hand-over is polled, not fenced by a stream synchronisation.
    HIPCHK_C(hipHostMalloc(&h->h_errors, sizeof(double) * (size_t)max_layers * max_cands + 16, hipHostMallocCoherent));
    HIPCHK_C(hipHostGetDevicePointer(reinterpret_cast<void**>(&h->d_errors), h->h_errors, 0));
    const size_t lp = (size_t)max_layers * max_cands;
    h->build_entries.assign((size_t)max_layers * LGRECO_MAX_CANDS, DpEntry{});
    h->dp_entries_off = (sizeof(int32_t) * (size_t)max_layers + 15) / 16 * 16;
    const size_t dp_in = (h->dp_entries_off + sizeof(DpEntry) * (size_t)max_layers * LGRECO_MAX_CANDS + 15) / 16 * 16;
    const size_t dp_out = sizeof(int64_t) * kDpResultSlots + sizeof(int32_t) * (size_t)max_layers;
    HIPCHK_C(hipMalloc(&h->d_dp_in, dp_in));
    HIPCHK_C(hipHostMalloc(&h->h_dp_in, dp_in, hipHostMallocCoherent));
    HIPCHK_C(hipHostMalloc(&h->h_dp_out, dp_out, hipHostMallocCoherent));
    // (pinned allocations are not cleared, and a freed block of an earlier handle may come back:
    // the hand-over word the host polls must not hold an old sequence number)
    std::memset(h->h_dp_out, 0, dp_out);
    HIPCHK_C(hipHostGetDevicePointer(reinterpret_cast<void**>(&h->d_dp_out), h->h_dp_out, 0));
    HIPCHK_C(hipHostGetDevicePointer(reinterpret_cast<void**>(const_cast<uint4**>(&h->d_dp_in_host)), h->h_dp_in, 0));
    h->d_count = reinterpret_cast<int32_t*>(h->d_dp_in);
    h->d_entries = reinterpret_cast<DpEntry*>(h->d_dp_in + h->dp_entries_off);
    h->h_count = reinterpret_cast<int32_t*>(h->h_dp_in);
    h->h_entries = reinterpret_cast<DpEntry*>(h->h_dp_in + h->dp_entries_off);
    h->d_result = reinterpret_cast<int64_t*>(h->d_dp_out);
    h->d_choice = reinterpret_cast<int32_t*>(h->d_dp_out + sizeof(int64_t) * kDpResultSlots);
    h->h_result = reinterpret_cast<int64_t*>(h->h_dp_out);
    h->h_choice = reinterpret_cast<int32_t*>(h->h_dp_out + sizeof(int64_t) * kDpResultSlots);
    HIPCHK_C(hipMalloc(&h->d_pd, (size_t)max_layers * (LGRECO_MAX_BINS + 4)));
    HIPCHK_C(hipMalloc(&h->d_dp_nodes, sizeof(uint32_t) * (2 * kMaxDpGroups - 1) * (LGRECO_MAX_BINS + 4)));
    HIPCHK_C(hipMalloc(&h->d_dp_range, sizeof(int32_t) * (2 * kMaxDpGroups + 4)));
    HIPCHK_C(hipHostMalloc(&h->h_sizes, sizeof(int64_t) * (size_t)max_layers * max_cands + 16, hipHostMallocDefault));
    HIPCHK_C(hipMalloc(&h->d_sizes, sizeof(int64_t) * (size_t)max_layers * max_cands + 16));
    HIPCHK_C(hipMalloc(&h->d_errors_dev, sizeof(double) * (size_t)max_layers * max_cands + 16));
    HIPCHK_C(hipHostMalloc(&h->h_build, sizeof(int32_t) * 2 * (size_t)max_layers, hipHostMallocCoherent));
    HIPCHK_C(hipHostGetDevicePointer(reinterpret_cast<void**>(&h->d_build_host), h->h_build, 0));
    HIPCHK_C(hipMalloc(&h->d_nsweep, sizeof(int32_t) * 2));
    HIPCHK_C(hipMalloc(&h->d_build_dev, sizeof(int32_t) * 2 * (size_t)max_layers));
    HIPCHK_C(hipHostMalloc(&h->h_apply, sizeof(int32_t) * ((size_t)max_layers * max_cands + 2 * max_cands), hipHostMallocDefault));
    HIPCHK_C(hipMalloc(&h->d_apply, sizeof(int32_t) * ((size_t)max_layers * max_cands + 2 * max_cands)));
    HIPCHK_C(hipHostMalloc(&h->h_bins, sizeof(int32_t) * lp, hipHostMallocDefault));
    for (Timing& t : h->tms) {
        for (int i = 0; i < 2 * Timing::kMaxSections; ++i) HIPCHK_C(hipEventCreate(&t.ev[i]));
        t.ready = true;
    }
    HIPCHK_C(hipStreamCreateWithFlags(&h->side, hipStreamNonBlocking));
    HIPCHK_C(hipEventCreateWithFlags(&h->ev_fork, hipEventDisableTiming));
    HIPCHK_C(hipEventCreateWithFlags(&h->ev_join, hipEventDisableTiming));
    {
        hipError_t e = topk_scratch_create(&h->topk, max_elems, max_layers, h->max_tiles);
        h->topk.reuse_thresholds = cfg->reuse_thresholds != 0;
        if (e != hipSuccess) { hip_fail(h, e, "topk_scratch_create"); return fail(LGRECO_EHIP); }
        e = lowrank_scratch_create(&h->lowrank, max_elems, max_layers, cfg->r_max, cfg->power_iters);
        if (e != hipSuccess) { hip_fail(h, e, "lowrank_scratch_create"); return fail(LGRECO_EHIP); }
    }
#undef HIPCHK_C
    return LGRECO_OK;
}

int lgreco_destroy(lgreco_handle_t* h) {
    if (!h) return LGRECO_EINVAL;
    (void)hipFree(h->d_layers);
    (void)hipFree(h->d_tiles);
    (void)hipFree(h->d_partials);
    (void)hipHostFree(h->h_errors);
    (void)hipFree(h->d_dp_in);
    (void)hipFree(h->d_pd);
    (void)hipFree(h->d_dp_nodes);
    (void)hipFree(h->d_dp_range);
    (void)hipHostFree(h->h_sizes);
    (void)hipFree(h->d_sizes);
    (void)hipFree(h->d_errors_dev);
    (void)hipHostFree(h->h_build);
    (void)hipFree(h->d_nsweep);
    (void)hipFree(h->d_build_dev);
    (void)hipHostFree(h->h_apply);
    (void)hipFree(h->d_apply);
    (void)hipHostFree(h->h_bins);
    (void)hipHostFree(h->h_dp_in);
    (void)hipHostFree(h->h_dp_out);
    for (Timing& t : h->tms)
        for (int i = 0; i < 2 * Timing::kMaxSections; ++i)
            if (t.ev[i]) (void)hipEventDestroy(t.ev[i]);
    if (h->side) (void)hipStreamDestroy(h->side);
    if (h->ev_fork) (void)hipEventDestroy(h->ev_fork);
    if (h->ev_join) (void)hipEventDestroy(h->ev_join);
    topk_scratch_destroy(&h->topk);
    lowrank_scratch_destroy(&h->lowrank);
    delete h;
    return LGRECO_OK;
}

int lgreco_set_timing(lgreco_handle_t* h, int32_t level) {
    if (!h || level < 0 || level > 2) return LGRECO_EINVAL;
    for (Timing& t : h->tms) {
        t.level = level;
        t.n = 0;
        t.calls = 0;
        t.active = false;
        t.harvested = true;
        t.n_totals = 0;
    }
    h->n_sub = 0;
    return LGRECO_OK;
}

int lgreco_set_timing_stride(lgreco_handle_t* h, int32_t every) {
    if (!h || every < 1) return LGRECO_EINVAL;
    for (Timing& t : h->tms) t.every = every;
    return LGRECO_OK;
}

static int read_timing(lgreco_handle_t* h, Timing& tm, bool with_sub, const char** names, float* ms, int32_t cap) {
    {
        const hipError_t e = harvest(tm);
        if (e != hipSuccess) return hip_fail(h, e, "reading timing events");
    }
    const int n = tm.n;
    for (int i = 0; i < n && i < cap; ++i) {
        if (names) names[i] = tm.name[i];
        if (ms) ms[i] = tm.ms[i];
    }
    int total = n;
    if (with_sub) {
        for (int j = 0; j < h->n_sub && n + j < cap; ++j) {
            if (names) names[n + j] = h->sub_name[j];
            if (ms) ms[n + j] = h->sub_ms[j];
        }
        total += h->n_sub;
    }
    return total;
}

int lgreco_get_timing(lgreco_handle_t* h, const char** names, float* ms, int32_t cap) {
    if (!h || cap < 0) return LGRECO_EINVAL;
    return read_timing(h, *h->tm, h->tm == &h->tms[LGRECO_CALL_SOLVE], names, ms, cap);
}

int lgreco_get_timing_of(lgreco_handle_t* h, int32_t call, const char** names, float* ms, int32_t cap) {
    if (!h || cap < 0 || call < 0 || call > LGRECO_CALL_RECEIVE) return LGRECO_EINVAL;
    return read_timing(h, h->tms[call], call == LGRECO_CALL_SOLVE, names, ms, cap);
}

int lgreco_get_timing_totals(lgreco_handle_t* h, int32_t call, const char** names, double* total_ms,
                             int64_t* count, int32_t cap) {
    if (!h || cap < 0 || call < 0 || call > LGRECO_CALL_RECEIVE) return LGRECO_EINVAL;
    Timing& tm = h->tms[call];
    const hipError_t e = harvest(tm);
    if (e != hipSuccess) return hip_fail(h, e, "reading timing events");
    for (int i = 0; i < tm.n_totals && i < cap; ++i) {
        if (names) names[i] = tm.total_name[i];
        if (total_ms) total_ms[i] = tm.total_ms[i];
        if (count) count[i] = tm.total_count[i];
    }
    return tm.n_totals;
}

int lgreco_sizes(const lgreco_layer_t* layers, int32_t L, const lgreco_cand_t* cands, int32_t P,
                 int32_t bucket, int64_t* sizes) {
    if (!layers || !cands || !sizes || L <= 0 || P <= 0 || bucket <= 0) return LGRECO_EINVAL;
    for (int l = 0; l < L; ++l) {
        if (layers[l].numel <= 0) return LGRECO_EINVAL;
        for (int c = 0; c < P; ++c) {
            const int st = check_cand(cands[c], &layers[l], 0);
            if (st != LGRECO_OK) return st;
            const int64_t n = layers[l].numel;
            int64_t s = 0;
            if (cands[c].family == LGRECO_QUANT) s = quant_size(n, (int)cands[c].param, bucket);
            else if (cands[c].family == LGRECO_TOPK) s = 8 * topk_k(n, cands[c].param);
            else s = 4 * ((int64_t)layers[l].rows + layers[l].cols) * (int64_t)cands[c].param;
            sizes[(size_t)l * P + c] = s;
        }
    }
    return LGRECO_OK;
}

int lgreco_candidate_range(int32_t family, double default_param, int32_t r_max, lgreco_cand_t* cands,
                           int32_t cap, int32_t* count, int32_t* default_index) {
    if (!cands || !count || cap <= 0) return LGRECO_EINVAL;
    int n = 0, def = -1;
    auto push = [&](double v, bool is_default) {
        if (n < cap) cands[n] = lgreco_cand_t{family, 0, v};
        if (is_default) def = n;
        ++n;
    };
    if (family == LGRECO_QUANT || family == LGRECO_LOWRANK) {
        if (!(default_param >= 1.0) || default_param != std::floor(default_param) || default_param > 1e6)
            return LGRECO_EINVAL;
        const int d = (int)default_param;
        const int top = family == LGRECO_QUANT ? 8 : (r_max > 0 ? r_max : 2 * d);
        if (d > top) return LGRECO_EINVAL;
        const int lo = std::max(1, d / 2), hi = std::min(top, 2 * d);
        for (int v = lo; v <= hi; ++v) push((double)v, v == d);
    } else if (family == LGRECO_TOPK) {
        if (!(default_param > 0.0 && default_param <= 1.0)) return LGRECO_EINVAL;
        for (int i = 1; i <= 100; ++i) {
            const double v = (double)i * default_param / 10.0;      // i = 10 reproduces the default exactly
            if (v > 1.0) break;
            push(i == 10 ? default_param : v, i == 10);
        }
    } else {
        return LGRECO_EINVAL;
    }
    *count = n;
    if (default_index) *default_index = def;
    return n > cap ? LGRECO_ENOSPACE : LGRECO_OK;
}

int lgreco_emax(const double* errors, int32_t L, int32_t P, int32_t default_cand, double* e_max) {
    if (!errors || !e_max || L <= 0 || P <= 0 || default_cand < 0 || default_cand >= P) return LGRECO_EINVAL;
    double s = 0.0;
    for (int l = 0; l < L; ++l) s += errors[(size_t)l * P + default_cand];
    *e_max = s;
    return LGRECO_OK;
}

// Queues every kernel of the profile on s; they write the error table to d_err (device memory, or
// the pinned host table as the kernels address it).
// x_out (quantization / Top-K candidates only): not null = the main pass writes x = fl32(g + e) there as it
// forms it (the error-feedback buffer itself in the one-call path) and everything after it reads x from there
static int profile_enqueue(lgreco_handle_t* h, const float* d_grads, const float* d_ef, const lgreco_layer_t* layers,
                           int32_t L, const lgreco_cand_t* cands, int32_t P, const float* d_q0, int64_t* sizes,
                           double* d_err, hipStream_t s, float* x_out = nullptr) {
    if (!h || !d_grads || !layers || !cands || L <= 0 || P <= 0) return LGRECO_EINVAL;
    if (P > h->max_cands) return LGRECO_ENOSPACE;
    begin_call(h, s, LGRECO_CALL_PROFILE);
    int st = prepare_layers(h, layers, L);
    if (st != LGRECO_OK) return st;
    // everything the profile queues, chains between the kernels included
    struct Phase {
        Timing* t;
        int idx;
        ~Phase() { t->close_phase(idx); }
    } phase{h->tm, -1};

    QuantParams qp{};
    // Top-K candidates, largest density first: one pass resolves kMaxTopk of them, the rest follow
    // in further groups on the same collected candidates (the first group has the lowest
    // thresholds, so its collection bound serves all)
    std::vector<std::pair<double, int>> tk_all;
    int lr_col[LGRECO_MAX_CANDS], lr_rank[LGRECO_MAX_CANDS], nlr = 0;
    for (int c = 0; c < P; ++c) {
        st = check_cand(cands[c], nullptr, h->cfg.r_max);
        if (st != LGRECO_OK) return st;
        if (cands[c].family == LGRECO_QUANT) {
            if (qp.nq >= kMaxQuant) return LGRECO_ENOSPACE;
            qp.bits[qp.nq] = (int)cands[c].param;
            qp.col[qp.nq++] = c;
        } else if (cands[c].family == LGRECO_TOPK) {
            tk_all.emplace_back(cands[c].param, c);
        } else {
            lr_rank[nlr] = (int)cands[c].param;
            lr_col[nlr++] = c;
        }
    }
    h->last_nlr = nlr;
    if (nlr && x_out) return LGRECO_EINVAL;          // the low-rank kernels read g and e themselves
    if (nlr) {
        if (!d_q0) return LGRECO_EINVAL;
        for (int l = 0; l < L; ++l)
            if (layers[l].rows <= 0 || layers[l].cols <= 0) return LGRECO_EINVAL;
    }
    if (sizes) {
        st = lgreco_sizes(layers, L, cands, P, h->cfg.bucket, sizes);
        if (st != LGRECO_OK) return st;
    }
    st = upload_layers(h, s, false);
    if (st != LGRECO_OK) return st;
    phase.idx = h->tm->open_phase("phase_profile");

    const int n_tiles = (int)h->ht.size();
    const bool ptr_aligned = ((uintptr_t)d_grads % 16 == 0) && (!d_ef || (uintptr_t)d_ef % 16 == 0);
    if (!ptr_aligned) return LGRECO_EINVAL;     // device allocations are always 256-byte aligned

    std::stable_sort(tk_all.begin(), tk_all.end(),
                     [](const std::pair<double, int>& a, const std::pair<double, int>& b) { return a.first > b.first; });
    const int ntk_all = (int)tk_all.size();
    const int ntk = std::min(ntk_all, (int)kMaxTopk);          // size of the first group
    h->last_ntk = ntk_all;
    for (int j = 0; j < ntk; ++j) h->last_tk_col[j] = tk_all[j].second;
    int tk_col[kMaxTopk];
    std::vector<uint32_t> ks((size_t)L * kMaxTopk, 0u);
    auto load_group = [&](int first) {                          // fills ks / tk_col, returns the group's size
        const int cnt = std::min((int)kMaxTopk, ntk_all - first);
        std::fill(ks.begin(), ks.end(), 0u);
        for (int j = 0; j < cnt; ++j) {
            tk_col[j] = tk_all[first + j].second;
            for (int l = 0; l < L; ++l)
                ks[(size_t)l * kMaxTopk + j] = (uint32_t)topk_k(layers[l].numel, tk_all[first + j].first);
        }
        return cnt;
    };
    if (ntk) {
        load_group(0);
        HIPCHK(topk_begin(&h->topk, d_grads, d_ef, h->d_layers, h->hl.data(), h->d_tiles, L, n_tiles,
                          h->tile_elems, ks.data(), ntk, 0, h->tm, s));
    }
    if (qp.nq) {
        qp.g = d_grads;
        qp.e = d_ef;
        qp.x_out = x_out;
        qp.layers = h->d_layers;
        qp.tiles = h->d_tiles;
        qp.partials = h->d_partials;
        qp.stride = P;
        qp.stochastic = h->cfg.stochastic;
        qp.seed_lo = (uint32_t)h->cfg.seed;
        qp.seed_hi = (uint32_t)(h->cfg.seed >> 32);
        if (ntk) {
            qp.hist = h->topk.d_hist;
            qp.lo = h->topk.lo_src;
            qp.cand = h->topk.d_cand;
            qp.cand_base = h->topk.d_cand_base;
            qp.tinfo = h->topk.d_tinfo;
            qp.base_part = h->topk.d_base_part;
            if (x_out) {
                // the compression behind this profile works from the candidates: it needs to know where they are
                qp.cand_idx = reinterpret_cast<uint16_t*>(h->topk.d_cand_idx);
                h->topk.cand_has_idx = true;
            }
        }
        Section sec(h->tm, ntk ? "quant_profile_topk_collect" : "quant_profile", true);
        HIPCHK(launch_quant_profile(qp, n_tiles, ntk > 0, s, &sec));
    } else if (ntk) {
        Section sec(h->tm, "topk_collect", true);
        HIPCHK(topk_collect(&h->topk, d_grads, d_ef, nullptr, h->d_layers, h->d_tiles, n_tiles, s, &sec, x_out));
    }
    // behind the main pass x is read from where it was left
    const float* const g_after = x_out ? x_out : d_grads;
    const float* const e_after = x_out ? nullptr : d_ef;
    if (ntk) {
        // (the per-layer sums of the quantization errors ride on the scan's launch)
        const QuantReduce qr{h->d_partials, d_err, P, qp.col, qp.nq};
        HIPCHK(topk_select(&h->topk, g_after, e_after, nullptr, h->d_layers, h->d_tiles, L, n_tiles, ntk, true,
                           ntk_all <= (int)kMaxTopk, h->tm, s, qp.nq ? &qr : nullptr));
    } else if (qp.nq) {
        Section sec(h->tm, "reduce_partials");
        HIPCHK(launch_reduce_partials(h->d_partials, P, qp.col, qp.nq, h->d_layers, L, d_err, s));
    }
    if (ntk) HIPCHK(topk_finalize(&h->topk, h->d_layers, h->d_tiles, L, ntk, tk_col, d_err, P, h->tm, s));
    for (int first = kMaxTopk; first < ntk_all; first += kMaxTopk) {
        const int cnt = load_group(first);
        HIPCHK(topk_regroup(&h->topk, L, ks.data(), 0, s));
        HIPCHK(topk_select(&h->topk, g_after, e_after, nullptr, h->d_layers, h->d_tiles, L, n_tiles, cnt, false,
                           first + (int)kMaxTopk >= ntk_all, h->tm, s, nullptr));
        HIPCHK(topk_finalize(&h->topk, h->d_layers, h->d_tiles, L, cnt, tk_col, d_err, P, h->tm, s));
    }
    if (nlr) {
        HIPCHK(lowrank_profile(&h->lowrank, d_grads, d_ef, h->d_layers, h->hl.data(), L, d_q0, h->cfg.r_max,
                               lr_rank, lr_col, nlr, d_err, P, h->tm, s));
    }
    return LGRECO_OK;
}

int lgreco_profile(lgreco_handle_t* h, const float* d_grads, const float* d_ef, const lgreco_layer_t* layers,
                   int32_t L, const lgreco_cand_t* cands, int32_t P, const float* d_q0, double* errors,
                   int64_t* sizes, void* stream) {
    if (!errors) return LGRECO_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    const int st = profile_enqueue(h, d_grads, d_ef, layers, L, cands, P, d_q0, sizes, h->d_errors, s);
    if (st != LGRECO_OK) return st;
    harvest_others(h);
    HIPCHK(hipStreamSynchronize(s));      // the kernels wrote h_errors
    std::memcpy(errors, h->h_errors, sizeof(double) * (size_t)L * P);
    return LGRECO_OK;
}

int lgreco_solve(lgreco_handle_t* h, const double* errors, const int64_t* sizes, int32_t L, int32_t P,
                 double e_max, int32_t n_bins, int32_t* choice, int64_t* total_size, double* total_error,
                 void* stream) {
    if (!h || !errors || !sizes || !choice || L <= 0 || P <= 0) return LGRECO_EINVAL;
    if (n_bins < 1 || n_bins > LGRECO_MAX_BINS || !(e_max == e_max)) return LGRECO_EINVAL;
    if (L > h->max_layers || P > h->max_cands) return LGRECO_ENOSPACE;
    hipStream_t s = (hipStream_t)stream;
    begin_call(h, s, LGRECO_CALL_SOLVE);
    const double D = (double)n_bins;
    int64_t worst = 0;                  // sum over layers of the largest usable size
    int max_bin = 0;
    int n_sweep = 0;                    // layers the kernel sweeps; h_bins[l] = their original index
    int max_count = 1;                  // most entries of a swept layer
    bool dead_layer = false;            // a layer without any usable candidate
    for (int l = 0; l < L; ++l) {
        DpEntry* en = h->build_entries.data() + (size_t)n_sweep * LGRECO_MAX_CANDS;
        int cnt = 0;
        int64_t lmax = 0;
        for (int c = 0; c < P; ++c) {
            const size_t i = (size_t)l * P + c;
            if (sizes[i] < 0 || sizes[i] >= ((int64_t)1 << 45)) return LGRECO_EINVAL;
            double err = errors[i];
            if (!(err == err)) return LGRECO_EINVAL;
            if (err < 0.0) err = 0.0;
            int32_t b;
            if (e_max > 0.0) {
                const double prod = err * D;
                const double q = std::floor(prod / e_max);
                b = (q <= D) ? (int32_t)q : -1;
            } else {
                b = (err <= 0.0) ? 0 : -1;
            }
            if (b < 0) continue;
            lmax = std::max(lmax, sizes[i]);
            max_bin = std::max(max_bin, (int)b);
            // equal bins: only the smallest size (lowest index among equals) can ever win
            int same = -1;
            for (int k = 0; k < cnt; ++k)
                if (en[k].bin == b) same = k;
            if (same < 0) {
                en[cnt++] = DpEntry{b, c, sizes[i]};
            } else if (sizes[i] < en[same].size) {
                // the group's representative moves to candidate c: keep the list in index order
                for (int k = same; k + 1 < cnt; ++k) en[k] = en[k + 1];
                en[cnt - 1] = DpEntry{b, c, sizes[i]};
            }
        }
        // An entry with both a larger bin and a size that is not smaller than another entry's can
        // never lie on the path that is traced back: swapping it for the other entry would give a
        // total that is no larger at a lower bin sum, which the final arg-min (smallest size, then
        // lowest bin sum) prefers.  Dropping such entries changes only cells off that path.
        {
            DpEntry all[LGRECO_MAX_CANDS];
            for (int k = 0; k < cnt; ++k) all[k] = en[k];
            int kept = 0;
            for (int k = 0; k < cnt; ++k) {
                bool dominated = false;
                for (int j = 0; j < cnt && !dominated; ++j)
                    dominated = all[j].bin < all[k].bin && all[j].size <= all[k].size;
                if (!dominated) en[kept++] = all[k];
            }
            cnt = kept;
        }
        worst += lmax;
        if (cnt == 0) {
            dead_layer = true;
        } else if (cnt == 1 && en[0].bin == 0) {
            choice[l] = en[0].cand;             // adds a constant to every cell: fixed here
        } else {
            h->h_count[n_sweep] = cnt;
            max_count = std::max(max_count, cnt);
            h->h_bins[n_sweep] = l;
            ++n_sweep;
        }
    }
    auto infeasible = [&]() {
        for (int l = 0; l < L; ++l) {           // report each layer's minimum-error candidate
            int best = 0;
            for (int c = 1; c < P; ++c)
                if (errors[(size_t)l * P + c] < errors[(size_t)l * P + best]) best = c;
            choice[l] = best;
        }
        return LGRECO_EINFEASIBLE;
    };
    if (dead_layer) return infeasible();
    if (h->cfg.strict_budget && n_bins - L < 0) return infeasible();      // more layers than bins: nothing is certain to fit
    if (n_sweep > 0) {
        const bool narrow = worst < ((int64_t)1 << 30);
        // the kernel's table has max_count entries per layer: the upload carries no unused slots
        for (int i = 0; i < n_sweep; ++i)
            std::memcpy(h->h_entries + (size_t)i * max_count,
                        h->build_entries.data() + (size_t)i * LGRECO_MAX_CANDS, sizeof(DpEntry) * max_count);
        // the kernel itself fetches the input block from the pinned staging memory
        const size_t in_bytes = h->dp_entries_off + sizeof(DpEntry) * (size_t)n_sweep * max_count;
        DpParams dp{h->d_entries, h->d_count, h->d_pd, h->d_choice, h->d_result, n_sweep, n_bins, 0, 0, 0, max_count,
                    h->d_dp_in_host, reinterpret_cast<uint4*>(h->d_dp_in), (int32_t)((in_bytes + 15) / 16), nullptr,
                    ++h->dp_seq, DpApply{}, dp_groups(h)};
        if (h->cfg.strict_budget) dp.e_limit = n_bins - L;        // all L layers round down, the fixed ones too
        {
            Section sec(h->tm, "dp_solve", true);
            HIPCHK(launch_dp(dp, narrow, max_bin, s, &sec, true));
        }
        harvest_others(h);
        {
            const int wst = wait_for_solver(h, h->dp_seq, s, n_sweep);     // the kernel wrote h_dp_out
            if (wst != LGRECO_OK) return wst;
        }
        h->last_solve_groups = h->h_result[9];
        if (h->tm->active) record_dp_sub(h);
        if (h->h_result[0] == 1) return infeasible();
        if (h->h_result[0] != 0) {
            h->hip_error = "dp back-trace inconsistent";
            return LGRECO_EHIP;
        }
        for (int i = 0; i < n_sweep; ++i) choice[h->h_bins[i]] = h->h_choice[i];
    }
    double terr = 0.0;
    int64_t tsize = 0;
    for (int l = 0; l < L; ++l) {
        terr += errors[(size_t)l * P + choice[l]];
        tsize += sizes[(size_t)l * P + choice[l]];
    }
    if (total_size) *total_size = tsize;
    if (total_error) *total_error = terr;
    return LGRECO_OK;
}

// lgreco_profile_solve; with `ec`, also the compression's first kernel (see EarlyCompress).
static int profile_solve_impl(lgreco_handle_t* h, const float* d_grads, const float* d_ef,
                              const lgreco_layer_t* layers, int32_t L, const lgreco_cand_t* cands, int32_t P,
                              const float* d_q0, int32_t default_cand, int32_t n_bins, double* errors,
                              int64_t* sizes, double* e_max, int32_t* choice, int64_t* total_size,
                              double* total_error, void* stream, EarlyCompress* ec) {
    if (!h || !errors || !sizes || !e_max || !choice || L <= 0 || P <= 0) return LGRECO_EINVAL;
    if (default_cand < 0 || default_cand >= P || n_bins < 1 || n_bins > LGRECO_MAX_BINS) return LGRECO_EINVAL;
    if (L > h->max_layers || P > h->max_cands) return LGRECO_ENOSPACE;
    hipStream_t s = (hipStream_t)stream;
    // strict budget, nothing fits it: the uniform default, whose total error is E_max itself (the
    // device wrote no layer records then: a compression that follows takes the host's route)
    auto strict_default = [&](const double* err, const int64_t* sz) {
        double terr = 0.0;
        int64_t tsize = 0;
        for (int l = 0; l < L; ++l) {
            choice[l] = default_cand;
            terr += err[(size_t)l * P + default_cand];
            tsize += sz[(size_t)l * P + default_cand];
        }
        h->last_solve_groups = 0;
        if (total_size) *total_size = tsize;
        if (total_error) *total_error = terr;
        return (int)LGRECO_OK;
    };
    // the device-side build reads the error table from device memory and passes it on to the host
    const bool on_device = L <= kBuildThreads && P <= kBuildMaxP && L * P <= kBuildMaxLP;
    int st = profile_enqueue(h, d_grads, d_ef, layers, L, cands, P, d_q0, sizes,
                             on_device ? h->d_errors_dev : h->d_errors, s, (ec && ec->x_in_e) ? ec->d_ef : nullptr);
    if (st != LGRECO_OK) return st;
    // The device-side build takes 32-bit costs only; anything it does not take goes the three
    // calls' route (same results, one more host round trip).
    int64_t worst = 0;
    for (int l = 0; l < L; ++l) {
        int64_t lmax = 0;
        for (int c = 0; c < P; ++c) {
            const int64_t sz = sizes[(size_t)l * P + c];
            if (sz < 0 || sz >= ((int64_t)1 << 45)) return LGRECO_EINVAL;
            lmax = std::max(lmax, sz);
        }
        worst += lmax;
    }
    if (!on_device || worst >= ((int64_t)1 << 30)) {
        if (on_device)      // (the rare wide-cost case: fetch the table the kernels left on the device)
            HIPCHK(hipMemcpyAsync(h->h_errors, h->d_errors_dev, sizeof(double) * (size_t)L * P,
                                  hipMemcpyDeviceToHost, s));
        HIPCHK(hipStreamSynchronize(s));
        std::memcpy(errors, h->h_errors, sizeof(double) * (size_t)L * P);
        st = lgreco_emax(errors, L, P, default_cand, e_max);
        if (st != LGRECO_OK) return st;
        st = lgreco_solve(h, errors, sizes, L, P, *e_max, n_bins, choice, total_size, total_error, stream);
        if (st == LGRECO_EINFEASIBLE && h->cfg.strict_budget) return strict_default(errors, sizes);
        return st;
    }
    begin_call(h, s, LGRECO_CALL_SOLVE);
    // the size table lives on the device and is uploaded when it changes (a training loop repeats it)
    if (h->sizes_count != (size_t)L * P || std::memcmp(h->h_sizes, sizes, sizeof(int64_t) * (size_t)L * P) != 0) {
        std::memcpy(h->h_sizes, sizes, sizeof(int64_t) * (size_t)L * P);
        h->sizes_count = (size_t)L * P;
        HIPCHK(hipMemcpyAsync(h->d_sizes, h->h_sizes, sizeof(int64_t) * (size_t)L * P, hipMemcpyHostToDevice, s));
        HIPCHK(hipStreamSynchronize(s));      // h_sizes may be rewritten by the next call
    }
    DpBuildParams bp{h->d_errors_dev, h->d_sizes, h->d_errors, L, P, n_bins, default_cand, P, h->d_entries,
                     h->d_count, h->d_build_host, h->d_build_host + L, h->d_build_dev, h->d_build_dev + L,
                     h->d_nsweep, h->d_result};
    DpParams dp{h->d_entries, h->d_count, h->d_pd, h->d_choice, h->d_result, L, n_bins, 0, 0, 0, P,
                nullptr, nullptr, 0, h->d_nsweep, ++h->dp_seq, DpApply{}, dp_groups(h)};
    if (h->cfg.strict_budget) dp.e_limit = n_bins - L;
    if (ec) {
        // what every (layer, candidate) means to the compression kernels, as lgreco_compress works
        // it out for a choice: the solver kernel picks the chosen column
        const size_t n_apply = (size_t)L * P + 2 * (size_t)P;
        std::vector<int32_t> tab(n_apply);
        for (int l = 0; l < L; ++l)
            for (int c = 0; c < P; ++c)
                tab[(size_t)l * P + c] = cands[c].family == LGRECO_TOPK ? (int32_t)topk_k(layers[l].numel, cands[c].param)
                                                                        : (int32_t)cands[c].param;
        for (int c = 0; c < P; ++c) tab[(size_t)L * P + c] = cands[c].family;
        // where the profile left the selection record of every Top-K candidate (one group only)
        const bool topk_known = h->last_ntk >= 1 && h->last_ntk <= (int)kMaxTopk;
        for (int c = 0; c < P; ++c) tab[(size_t)L * P + P + c] = -1;
        if (topk_known)
            for (int j = 0; j < h->last_ntk; ++j) tab[(size_t)L * P + P + h->last_tk_col[j]] = j;
        ec->topk_known = topk_known;
        if (h->apply_count != n_apply || std::memcmp(h->h_apply, tab.data(), sizeof(int32_t) * n_apply) != 0) {
            std::memcpy(h->h_apply, tab.data(), sizeof(int32_t) * n_apply);
            h->apply_count = n_apply;
            HIPCHK(hipMemcpyAsync(h->d_apply, h->h_apply, sizeof(int32_t) * n_apply, hipMemcpyHostToDevice, s));
            HIPCHK(hipStreamSynchronize(s));      // h_apply may be rewritten by the next call
        }
        dp.apply = DpApply{h->d_layers, h->d_build_dev, h->d_build_dev + L, h->d_sizes, h->d_apply,
                           h->d_apply + (size_t)L * P, h->d_apply + (size_t)L * P + P, L, P, ec->capacity};
    }
    {
        Section sec(h->tm, "dp_solve", true);
        HIPCHK(launch_dp_build(bp, s, &sec));
        HIPCHK(launch_dp(dp, true, n_bins, s, &sec, false));
    }
    if (ec) {
        // The quantization kernel of the compression, queued behind the solver: it reads the layer
        // records the solver kernel writes (layers of other families, or all of them after a
        // failed solve, are skipped).  From here on the host no longer knows what the device's
        // layer table holds, until lgreco_compress has worked out the same records.
        Timing* const solve_tm = h->tm;
        begin_call(h, s, LGRECO_CALL_COMPRESS);
        h->hl_uploaded.clear();
        ec->phase = h->tm->open_phase("phase_compress");
        bool any_quant = false;
        for (int c = 0; c < P; ++c) any_quant = any_quant || cands[c].family == LGRECO_QUANT;
        // With both families the quantized layers' one kernel goes to the second stream: the Top-K
        // layers' part is one pass over the candidates and a handful of short kernels that leave
        // most of the chip idle, and the two parts write disjoint layers (error feedback and
        // payload alike).  The quantization kernel is launched with 30 KB of LDS it does not use,
        // which holds it to five workgroups per compute unit instead of the six its registers
        // allow: the room left (a quarter of the vector registers) is what lets the Top-K kernels'
        // workgroups in beside it.  Measured on the 355 M-element mixed workload, the compression
        // from the solver kernel's end to its last kernel's: 272 us on one stream, 217 with the
        // quantization kernel queued behind the Top-K main pass, 213 beside it without the LDS,
        // 197 with it (the two bandwidth-bound kernels alone take 192).
        // (Only when the Top-K part works from the candidates: its pass over the whole data, which
        // the keep_ef_on_failure path makes, is as bandwidth-bound as the quantization kernel.)
        const bool beside = any_quant && ec->topk_known && ec->x_in_e;
        if (beside) HIPCHK(hipEventRecord(h->ev_fork, s));
        if (ec->topk_known) {
            // the Top-K layers' part, from the selection records the profile left for this very
            // data: the chosen density's record is picked on the device
            HIPCHK(topk_compress_known(&h->topk, d_grads, ec->d_ef, h->d_layers, h->d_tiles, L, (int)h->ht.size(),
                                       ec->d_payload, h->tm, s, ec->x_in_e, beside));
        }
        if (beside) HIPCHK(hipStreamWaitEvent(h->side, h->ev_fork, 0));
        if (any_quant) {
            Section sec(h->tm, "quant_compress", true);
            HIPCHK(launch_quant_compress(ec->x_in_e ? nullptr : d_grads, ec->d_ef, h->d_layers, h->d_tiles,
                                         (int)h->ht.size(), ec->d_payload, h->cfg.stochastic != 0, h->cfg.seed,
                                         beside ? h->side : s, &sec, beside ? 30 * 1024 : 0));
        }
        if (beside) {
            HIPCHK(hipEventRecord(h->ev_join, h->side));
            HIPCHK(hipStreamWaitEvent(s, h->ev_join, 0));
        }
        ec->launched = true;
        ec->lowrank_known = h->last_nlr > 0 && ec->d_q != nullptr;
        if (ec->lowrank_known) {
            // ... and the low-rank layers': the factors of every rank are the leading columns of
            // the rank-64 run the profile just made on this data
            HIPCHK(lowrank_compress_known(&h->lowrank, d_grads, ec->d_ef, h->d_layers, ec->d_q, h->cfg.r_max,
                                          ec->d_payload, h->tm, s, h->ef_zero_on_entry));
        }
        // the compress call stays open until lgreco_compress's part has queued the rest: nobody
        // reads its events out before (that would wait for the kernel just queued)
        h->tm->harvested = true;
        h->tm = solve_tm;
    }
    harvest_others(h);
    {
        // error table, build report and solver output are in pinned memory
        const int wst = wait_for_solver(h, h->dp_seq, s, -1, L, P);
        if (wst != LGRECO_OK) return wst;
    }
    std::memcpy(errors, h->h_errors, sizeof(double) * (size_t)L * P);
    const int64_t status = h->h_result[0];
    h->last_solve_groups = status == 0 ? h->h_result[9] : 0;
    if (ec) ec->applied = h->h_result[8] == 1;
    {
        const uint64_t bits = (uint64_t)h->h_result[6];
        std::memcpy(e_max, &bits, sizeof(double));
    }
    if (status == 3) return LGRECO_EINVAL;                  // a NaN in the error table
    if (h->tm->active && status == 0) record_dp_sub(h);
    if (status == 1 && h->cfg.strict_budget) return strict_default(errors, sizes);
    if (status == 1) {                                      // report each layer's minimum-error candidate
        for (int l = 0; l < L; ++l) {
            int best = 0;
            for (int c = 1; c < P; ++c)
                if (errors[(size_t)l * P + c] < errors[(size_t)l * P + best]) best = c;
            choice[l] = best;
        }
        return LGRECO_EINFEASIBLE;
    }
    if (status != 0) {
        h->hip_error = "dp back-trace inconsistent";
        return LGRECO_EHIP;
    }
    const int n_sweep = (int)h->h_result[5];
    const int32_t* const sweep_layer = h->h_build;
    const int32_t* const fixed_choice = h->h_build + L;
    for (int l = 0; l < L; ++l) choice[l] = fixed_choice[l];
    for (int i = 0; i < n_sweep; ++i) choice[sweep_layer[i]] = h->h_choice[i];
    double terr = 0.0;
    int64_t tsize = 0;
    for (int l = 0; l < L; ++l) {
        if (choice[l] < 0 || choice[l] >= P) {
            h->hip_error = "device-side entry build left a layer without a choice";
            return LGRECO_EHIP;
        }
        terr += errors[(size_t)l * P + choice[l]];
        tsize += sizes[(size_t)l * P + choice[l]];
    }
    if (total_size) *total_size = tsize;
    if (total_error) *total_error = terr;
    return LGRECO_OK;
}

int lgreco_profile_solve(lgreco_handle_t* h, const float* d_grads, const float* d_ef, const lgreco_layer_t* layers,
                         int32_t L, const lgreco_cand_t* cands, int32_t P, const float* d_q0, int32_t default_cand,
                         int32_t n_bins, double* errors, int64_t* sizes, double* e_max, int32_t* choice,
                         int64_t* total_size, double* total_error, void* stream) {
    return profile_solve_impl(h, d_grads, d_ef, layers, L, cands, P, d_q0, default_cand, n_bins, errors, sizes, e_max,
                              choice, total_size, total_error, stream, nullptr);
}

int lgreco_solve_weighted(lgreco_handle_t* h, const double* errors, const int64_t* sizes, const int64_t* weights,
                          int32_t L, int32_t P, double e_max, int32_t n_bins, int32_t* choice,
                          int64_t* total_size, int64_t* total_cost, double* total_error, void* stream) {
    if (!h || !errors || !sizes || !weights || !choice || L <= 0 || P <= 0) return LGRECO_EINVAL;
    const int64_t limit = (int64_t)1 << 45;
    std::vector<int64_t> cost((size_t)L * P);
    for (int l = 0; l < L; ++l) {
        if (weights[l] < 0 || weights[l] >= limit) return LGRECO_EINVAL;
        for (int c = 0; c < P; ++c) {
            const int64_t sz = sizes[(size_t)l * P + c];
            if (sz < 0 || sz >= limit) return LGRECO_EINVAL;
            if (weights[l] != 0 && sz > (limit - 1) / weights[l]) return LGRECO_EINVAL;
            cost[(size_t)l * P + c] = sz * weights[l];
        }
    }
    int64_t tcost = 0;
    const int st = lgreco_solve(h, errors, cost.data(), L, P, e_max, n_bins, choice, &tcost, total_error, stream);
    if (st != LGRECO_OK) return st;
    if (total_cost) *total_cost = tcost;
    if (total_size) {
        int64_t ts = 0;
        for (int l = 0; l < L; ++l) ts += sizes[(size_t)l * P + choice[l]];
        *total_size = ts;
    }
    return LGRECO_OK;
}

int lgreco_payload_layout(const lgreco_layer_t* layers, int32_t L, const lgreco_cand_t* cands, int32_t P,
                          const int32_t* choice, int32_t bucket, int64_t* offsets) {
    if (!layers || !cands || !choice || !offsets || L <= 0 || P <= 0 || bucket <= 0) return LGRECO_EINVAL;
    int64_t off = 0;
    for (int l = 0; l < L; ++l) {
        if (choice[l] < 0 || choice[l] >= P) return LGRECO_EINVAL;
        int64_t sz = 0;
        const int st = lgreco_sizes(&layers[l], 1, &cands[choice[l]], 1, bucket, &sz);
        if (st != LGRECO_OK) return st;
        offsets[l] = off;
        off = (off + sz + 15) / 16 * 16;
    }
    offsets[L] = off;
    return LGRECO_OK;
}

// lgreco_compress; `ec` (may be null): the quantization kernel was already queued (EarlyCompress).
static int compress_impl(lgreco_handle_t* h, const float* d_grads, float* d_ef, const lgreco_layer_t* layers,
                         int32_t L, const lgreco_cand_t* cands, int32_t P, const int32_t* choice, float* d_q,
                         uint8_t* d_payload, const int64_t* offsets, void* stream, const EarlyCompress* ec) {
    if (!h || !d_grads || !d_ef || !layers || !cands || !choice || !d_payload || !offsets || L <= 0 || P <= 0)
        return LGRECO_EINVAL;
    if ((uintptr_t)d_grads % 16 || (uintptr_t)d_ef % 16 || (uintptr_t)d_payload % 16) return LGRECO_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    const bool early = ec && ec->launched;
    if (early) {                                            // the call began with that launch
        h->tm = &h->tms[LGRECO_CALL_COMPRESS];
        h->tm->harvested = !h->tm->active;
    } else {
        begin_call(h, s, LGRECO_CALL_COMPRESS);
    }
    int st = prepare_layers(h, layers, L);
    if (st != LGRECO_OK) return st;
    bool any[3] = {false, false, false};
    for (int l = 0; l < L; ++l) {
        if (choice[l] < 0 || choice[l] >= P) return LGRECO_EINVAL;
        const lgreco_cand_t& c = cands[choice[l]];
        st = check_cand(c, &layers[l], h->cfg.r_max);
        if (st != LGRECO_OK) return st;
        if (offsets[l] < 0 || offsets[l] % 16) return LGRECO_EINVAL;
        DevLayer& d = h->hl[l];
        d.family = c.family;
        d.payload = offsets[l];
        d.iparam = (c.family == LGRECO_TOPK) ? (int32_t)topk_k(layers[l].numel, c.param) : (int32_t)c.param;
        any[c.family] = true;
    }
    if (any[LGRECO_LOWRANK] && !d_q) return LGRECO_EINVAL;
    // the solver kernel wrote these very records into the device's table (same tables, same
    // arithmetic) and the quantization kernel has run on them: nothing to upload, nothing to repeat
    const bool quant_done = early && ec->applied && !h->layers_dirty;
    if (quant_done) h->hl_uploaded = h->hl;
    st = upload_layers(h, s, true);
    if (st != LGRECO_OK) return st;
    const int n_tiles = (int)h->ht.size();
    const int phase = early ? ec->phase : h->tm->open_phase("phase_compress");
    // behind a profile of the same call that left x in the error-feedback buffer, x is read from there
    const bool x_in_e = ec && ec->x_in_e;                 // whether or not the early kernels were queued
    if (x_in_e && any[LGRECO_LOWRANK]) return LGRECO_EINVAL;      // never set together (see the one-call entry point)
    if (any[LGRECO_QUANT] && !quant_done) {
        Section sec(h->tm, "quant_compress", true);
        HIPCHK(launch_quant_compress(x_in_e ? nullptr : d_grads, d_ef, h->d_layers, h->d_tiles, n_tiles, d_payload,
                                     h->cfg.stochastic != 0, h->cfg.seed, s, &sec));
    }
    if (any[LGRECO_TOPK] && !(quant_done && ec->topk_known)) {
        HIPCHK(topk_compress(&h->topk, x_in_e ? d_ef : d_grads, d_ef, h->d_layers, h->hl.data(), h->d_tiles, L,
                             n_tiles, h->tile_elems, d_payload, h->tm, s, x_in_e));
    }
    if (any[LGRECO_LOWRANK] && !(quant_done && ec->lowrank_known)) {
        HIPCHK(lowrank_compress(&h->lowrank, d_grads, d_ef, h->d_layers, h->hl.data(), L, d_q, h->cfg.r_max,
                                d_payload, h->tm, s));
    }
    h->tm->close_phase(phase);
    // No host output: the call returns with its kernels queued.  Payload, error feedback and q are
    // ready in stream order; the caller's next call on this stream (or its own wait) sees them.
    return LGRECO_OK;
}

int lgreco_compress(lgreco_handle_t* h, const float* d_grads, float* d_ef, const lgreco_layer_t* layers, int32_t L,
                    const lgreco_cand_t* cands, int32_t P, const int32_t* choice, float* d_q, uint8_t* d_payload,
                    const int64_t* offsets, void* stream) {
    return compress_impl(h, d_grads, d_ef, layers, L, cands, P, choice, d_q, d_payload, offsets, stream, nullptr);
}

int lgreco_profile_solve_compress(lgreco_handle_t* h, const float* d_grads, float* d_ef,
                                  const lgreco_layer_t* layers, int32_t L, const lgreco_cand_t* cands, int32_t P,
                                  float* d_q, int32_t default_cand, int32_t n_bins, double* errors, int64_t* sizes,
                                  double* e_max, int32_t* choice, int64_t* total_size, double* total_error,
                                  uint8_t* d_payload, int64_t payload_capacity, int64_t* offsets, void* stream) {
    if (!h || !d_grads || !d_ef || !d_payload || !offsets || payload_capacity < 0) return LGRECO_EINVAL;
    if ((uintptr_t)d_grads % 16 || (uintptr_t)d_ef % 16 || (uintptr_t)d_payload % 16) return LGRECO_EINVAL;
    EarlyCompress ec{d_ef, d_payload, payload_capacity};
    ec.d_q = d_q;
    // a buffer the caller promises to be all zeros is not read by the profile: x = fl32(g + 0) = g
    const float* const d_ef_profile = h->ef_zero_on_entry ? nullptr : d_ef;
    // x in place: unless the configuration asks for an untouched buffer on failure, the profile
    // leaves x in d_ef and the compression reads it there (quantization and Top-K candidates only:
    // the low-rank kernels read g and e themselves)
    if (cands && P > 0 && !h->cfg.keep_ef_on_failure && d_ef_profile) {
        ec.x_in_e = true;
        for (int c = 0; c < P; ++c) ec.x_in_e = ec.x_in_e && cands[c].family != LGRECO_LOWRANK;
    }
    int st = profile_solve_impl(h, d_grads, d_ef_profile, layers, L, cands, P, d_q, default_cand, n_bins, errors, sizes,
                                e_max, choice, total_size, total_error, stream, &ec);
    if (st != LGRECO_OK) return st;
    // the layout of lgreco_payload_layout, from the size table the profile just filled
    int64_t off = 0;
    for (int l = 0; l < L; ++l) {
        offsets[l] = off;
        off = (off + sizes[(size_t)l * P + choice[l]] + 15) / 16 * 16;
    }
    offsets[L] = off;
    if (off > payload_capacity) return LGRECO_ENOSPACE;
    return compress_impl(h, d_grads, d_ef, layers, L, cands, P, choice, d_q, d_payload, offsets, stream, &ec);
}

int lgreco_decompress(lgreco_handle_t* h, const uint8_t* d_payload, const int64_t* offsets,
                      const lgreco_layer_t* layers, int32_t L, const lgreco_cand_t* cands, int32_t P,
                      const int32_t* choice, float* d_out, int32_t accumulate, void* stream) {
    if (!h || !d_payload || !offsets || !layers || !cands || !choice || !d_out || L <= 0 || P <= 0)
        return LGRECO_EINVAL;
    if ((uintptr_t)d_out % 16 || (uintptr_t)d_payload % 16) return LGRECO_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    begin_call(h, s, LGRECO_CALL_RECEIVE);
    int st = prepare_layers(h, layers, L);
    if (st != LGRECO_OK) return st;
    bool any[3] = {false, false, false};
    for (int l = 0; l < L; ++l) {
        if (choice[l] < 0 || choice[l] >= P) return LGRECO_EINVAL;
        const lgreco_cand_t& c = cands[choice[l]];
        st = check_cand(c, &layers[l], h->cfg.r_max);
        if (st != LGRECO_OK) return st;
        if (offsets[l] < 0 || offsets[l] % 16) return LGRECO_EINVAL;
        DevLayer& d = h->hl[l];
        d.family = c.family;
        d.payload = offsets[l];
        d.iparam = (c.family == LGRECO_TOPK) ? (int32_t)topk_k(layers[l].numel, c.param) : (int32_t)c.param;
        any[c.family] = true;
    }
    st = upload_layers(h, s, true);
    if (st != LGRECO_OK) return st;
    HIPCHK(launch_decode(d_payload, h->d_layers, h->d_tiles, (int)h->ht.size(), d_out, accumulate != 0,
                         any[LGRECO_QUANT], any[LGRECO_TOPK], h->tm, s));
    if (any[LGRECO_LOWRANK])
        HIPCHK(lowrank_decompress(&h->lowrank, h->hl.data(), L, h->cfg.r_max, d_payload, d_out, accumulate != 0,
                                  h->tm, s));
    HIPCHK(hipStreamSynchronize(s));
    return LGRECO_OK;
}

int lgreco_accumulate(lgreco_handle_t* h, float* d_acc, const float* d_grads, int64_t n, int32_t reset,
                      void* stream) {
    if (!h || !d_acc || !d_grads || n < 0) return LGRECO_EINVAL;
    if ((uintptr_t)d_acc % 16 || (uintptr_t)d_grads % 16) return LGRECO_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    begin_call(h, s, LGRECO_CALL_RECEIVE);
    {
        Section sec(h->tm, "accumulate", true);
        HIPCHK(launch_accumulate(d_acc, d_grads, n, reset != 0, s, &sec));
    }
    HIPCHK(hipStreamSynchronize(s));
    return LGRECO_OK;
}

}  // extern "C"

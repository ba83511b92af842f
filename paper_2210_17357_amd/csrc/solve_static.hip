// lgreco_solve_static: the solver for callers that cannot allocate (code under HIP graph capture,
// tight serving loops, harnesses that forbid hipMalloc).  Same kernels as lgreco_profile_solve's
// device-side route (dp_build_kernel, dp_kernel), with every intermediate table in one file-scope
// device array instead of a handle's allocations.  Inputs and outputs are the caller's device
// buffers; nothing is copied to or from the host and the call does not wait.
#include "internal.h"

// Bytes of the arg-min table plus 80.5 KB of lists and counters, see the layout below.  One copy per
// GPU the library runs on, held until the process ends.  In host code this name is a stand-in,
// not an address: the address on the current device comes from hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[LGRECO_STATIC_MAX_PD_BYTES + 82432];

namespace lgreco {
namespace {

// ---- layout of the scratch array (every part a multiple of 256 bytes)
constexpr int kStaticMaxLayers = kBuildThreads;                 // 1024
constexpr int kStaticMaxLP = kBuildMaxLP;                       // 4096 table entries
constexpr size_t kStaticPdBytes = LGRECO_STATIC_MAX_PD_BYTES;   // arg-min table, one byte per cell
constexpr size_t kOffEntries = 0;                                                   // DpEntry [4096]
constexpr size_t kOffCount = kOffEntries + sizeof(DpEntry) * kStaticMaxLP;          // int32 [1024]
constexpr size_t kOffSweepLayer = kOffCount + sizeof(int32_t) * kStaticMaxLayers;   // int32 [1024]
constexpr size_t kOffFixed = kOffSweepLayer + sizeof(int32_t) * kStaticMaxLayers;   // int32 [1024]
constexpr size_t kOffSweepChoice = kOffFixed + sizeof(int32_t) * kStaticMaxLayers;  // int32 [1024]
constexpr size_t kOffNsweep = kOffSweepChoice + sizeof(int32_t) * kStaticMaxLayers; // int32 [2] (+ pad)
constexpr size_t kOffResult = kOffNsweep + 256;                                     // int64 [16] (+ pad)
constexpr size_t kOffPd = kOffResult + 256;
constexpr size_t kScratchBytes = kOffPd + kStaticPdBytes;
static_assert(kOffCount % 256 == 0 && kOffPd % 256 == 0, "parts are 256-byte aligned");

static_assert(kScratchBytes == sizeof(scratch), "the array above is declared with this size");

constexpr int kMaxDevices = 64;
unsigned char* g_scratch_ptr[kMaxDevices] = {};

// The assignment over all layers and its totals from what the build and the sweep left: one
// workgroup.  status 0: fixed layers from the build's report, swept ones from the back-trace;
// status 1 (no assignment fits): each layer's minimum-error candidate, totals 0; else: -1.
__global__ __launch_bounds__(kBuildThreads) void static_gather_kernel(
    const double* __restrict__ errors, const int64_t* __restrict__ sizes, int L, int P,
    const int32_t* __restrict__ fixed_choice, const int32_t* __restrict__ sweep_layer,
    const int32_t* __restrict__ sweep_choice, const int32_t* __restrict__ n_sweep,
    const int64_t* __restrict__ dp_result, int32_t* __restrict__ choice, int64_t* __restrict__ out) {
    __shared__ int32_t s_choice[kBuildThreads];
    __shared__ int32_t s_bad;
    const int tid = threadIdx.x;
    const int64_t status = dp_result[0];
    if (tid == 0) s_bad = 0;
    s_choice[tid] = -1;
    if (status == 0) {
        if (tid < L) s_choice[tid] = fixed_choice[tid];
        __syncthreads();
        const int ns = n_sweep[0];
        if (tid < ns) {
            const int l = sweep_layer[tid];
            if (l >= 0 && l < L) s_choice[l] = sweep_choice[tid];
        }
    } else if (status == 1) {
        if (tid < L) {
            int best = 0;
            for (int c = 1; c < P; ++c)
                if (errors[(size_t)tid * P + c] < errors[(size_t)tid * P + best]) best = c;
            s_choice[tid] = best;
        }
    }
    __syncthreads();
    if (tid < L) {
        const int c = s_choice[tid];
        if (status == 0 && (c < 0 || c >= P)) s_bad = 1;      // a layer neither fixed nor swept
        choice[tid] = c;
    }
    __syncthreads();
    if (tid == 0) {
        // totals in layer order, as the host route sums them
        double terr = 0.0;
        int64_t tsize = 0;
        const bool ok = status == 0 && !s_bad;
        if (ok)
            for (int l = 0; l < L; ++l) {
                terr += errors[(size_t)l * P + s_choice[l]];
                tsize += sizes[(size_t)l * P + s_choice[l]];
            }
        out[0] = (status == 0 && s_bad) ? 2 : status;
        out[1] = tsize;
        out[2] = (int64_t)__builtin_bit_cast(uint64_t, terr);
        out[3] = dp_result[6];                                 // bit pattern of E_max (the build wrote it)
    }
}

}  // namespace
}  // namespace lgreco

using namespace lgreco;

extern "C" int lgreco_solve_static(const double* d_errors, const int64_t* d_sizes, int32_t L, int32_t P,
                                   int32_t default_cand, int32_t n_bins, int32_t* d_choice, int64_t* d_result,
                                   void* stream) {
    if (!d_errors || !d_sizes || !d_choice || !d_result || L <= 0 || P <= 0) return LGRECO_EINVAL;
    if (default_cand < 0 || default_cand >= P || n_bins < 1) return LGRECO_EINVAL;
    if ((uintptr_t)d_errors % 16 || (uintptr_t)d_sizes % 16) return LGRECO_EINVAL;
    // the stated maximum: what the scratch array and the device-side list building hold
    if (L > kStaticMaxLayers || P > kBuildMaxP || (int64_t)L * P > kStaticMaxLP || n_bins > LGRECO_MAX_BINS)
        return LGRECO_ENOSPACE;
    const size_t pd_stride = ((size_t)n_bins + 1 + 3) & ~(size_t)3;
    if ((size_t)L * pd_stride > kStaticPdBytes) return LGRECO_ENOSPACE;

    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LGRECO_EHIP;
    if (!g_scratch_ptr[dev]) {
        // once per device, with that device current: each GPU holds its own copy at its own address
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return LGRECO_EHIP;
        g_scratch_ptr[dev] = static_cast<unsigned char*>(ptr);
    }
    unsigned char* const base = g_scratch_ptr[dev];
    DpEntry* const entries = reinterpret_cast<DpEntry*>(base + kOffEntries);
    int32_t* const count = reinterpret_cast<int32_t*>(base + kOffCount);
    int32_t* const sweep_layer = reinterpret_cast<int32_t*>(base + kOffSweepLayer);
    int32_t* const fixed = reinterpret_cast<int32_t*>(base + kOffFixed);
    int32_t* const sweep_choice = reinterpret_cast<int32_t*>(base + kOffSweepChoice);
    int32_t* const nsweep = reinterpret_cast<int32_t*>(base + kOffNsweep);
    int64_t* const result = reinterpret_cast<int64_t*>(base + kOffResult);
    uint8_t* const pd = base + kOffPd;

    hipStream_t s = (hipStream_t)stream;
    // Nothing in the scratch has to start at zero: the build writes every word the sweep reads
    // (counts and entries of the swept layers, their number, the status), the sweep writes every
    // arg-min cell the back-trace reads, and the gather step reads what those two wrote.
    DpBuildParams bp{d_errors, d_sizes, nullptr, L, P, n_bins, default_cand, P, entries, count,
                     sweep_layer, fixed, sweep_layer, fixed, nsweep, result, 1};
    DpParams dp{entries, count, pd, sweep_choice, result, L, n_bins, 0, 0, 0, P,
                nullptr, nullptr, 0, nsweep, 1, DpApply{}};
    if (launch_dp_build(bp, s, nullptr) != hipSuccess) return LGRECO_EHIP;
    if (launch_dp(dp, true, n_bins, s, nullptr, false) != hipSuccess) return LGRECO_EHIP;
    hipLaunchKernelGGL(static_gather_kernel, dim3(1), dim3(kBuildThreads), 0, s, d_errors, d_sizes, (int)L, (int)P,
                       (const int32_t*)fixed, (const int32_t*)sweep_layer, (const int32_t*)sweep_choice,
                       (const int32_t*)nsweep, (const int64_t*)result, d_choice, d_result);
    return hipGetLastError() == hipSuccess ? LGRECO_OK : LGRECO_EHIP;
}

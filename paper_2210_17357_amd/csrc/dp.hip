// Layer x error-bin dynamic program of Algorithm 1 and its back-trace, one workgroup.
//
// DP[l][e] = min over candidates c with bin(l,c) <= e of DP[l-1][e - bin(l,c)] + size(l,c),
// starting from a virtual row DP[0] = (0, inf, inf, ...).  Layers are sequential; the bins of a
// row are independent, so the 1024 threads each own the bins e = tid, tid + 1024, ... and keep
// the new row in registers while the previous row sits in LDS.  Candidates are visited in index
// order with a strict '<' (lowest index wins ties); the back-trace starts from the lowest e among
// the minima of the last row.  PD (arg-min per cell) goes to global memory, one byte per cell.
#include "internal.h"

namespace lgreco {

constexpr int kDpThreads = 1024;
constexpr int kDpMaxK = (LGRECO_MAX_BINS + 1 + kDpThreads - 1) / kDpThreads;   // 17
constexpr int64_t kDpInf = (int64_t)1 << 62;

template <int KMAX>
__global__ __launch_bounds__(kDpThreads) void dp_kernel(DpParams p) {
    extern __shared__ int64_t row[];               // [D+1] previous row
    __shared__ int64_t s_val[kDpThreads / 64];
    __shared__ int32_t s_idx[kDpThreads / 64];
    const int tid = threadIdx.x;
    const int D = p.D, P = p.P;
    const int64_t width = (int64_t)D + 1;

    for (int e = tid; e <= D; e += kDpThreads) row[e] = (e == 0) ? 0 : kDpInf;
    __syncthreads();

    for (int l = 0; l < p.L; ++l) {
        const int32_t* __restrict__ lb = p.bins + (size_t)l * P;
        const int64_t* __restrict__ ls = p.sizes + (size_t)l * P;
        int64_t nv[KMAX];
        int32_t na[KMAX];
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
            const int e = tid + k * kDpThreads;
            int64_t best = kDpInf;
            int32_t arg = 255;
            if (e <= D) {
                for (int c = 0; c < P; ++c) {
                    const int32_t b = lb[c];
                    if (b >= 0 && b <= e) {
                        const int64_t prev = row[e - b];
                        const int64_t t = prev + ls[c];
                        if (prev < kDpInf && t < best) {
                            best = t;
                            arg = c;
                        }
                    }
                }
            }
            nv[k] = best;
            na[k] = arg;
        }
        __syncthreads();
        uint8_t* __restrict__ pdrow = p.pd + (size_t)l * width;
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
            const int e = tid + k * kDpThreads;
            if (e <= D) {
                row[e] = nv[k];
                pdrow[e] = (uint8_t)na[k];
            }
        }
        __syncthreads();
    }

    // arg-min of the last row, lowest e among equal minima
    int64_t bv = kDpInf;
    int32_t be = 0x7FFFFFFF;
    for (int e = tid; e <= D; e += kDpThreads) {
        const int64_t v = row[e];
        if (v < bv) { bv = v; be = e; }              // e ascending per thread -> keeps the lowest
    }
    for (int o = 1; o < 64; o <<= 1) {
        const int64_t ov = __shfl_xor(bv, o, 64);
        const int32_t oe = __shfl_xor(be, o, 64);
        if (ov < bv || (ov == bv && oe < be)) { bv = ov; be = oe; }
    }
    if ((tid & 63) == 0) { s_val[tid >> 6] = bv; s_idx[tid >> 6] = be; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < kDpThreads / 64; ++w)
            if (s_val[w] < bv || (s_val[w] == bv && s_idx[w] < be)) { bv = s_val[w]; be = s_idx[w]; }
        if (bv >= kDpInf) {
            p.result[0] = 1;
            p.result[1] = 0;
            p.result[2] = 0;
        } else {
            int e = be;
            for (int l = p.L - 1; l >= 0; --l) {
                const int c = p.pd[(size_t)l * width + e];
                p.choice[l] = c;
                e -= p.bins[(size_t)l * P + c];
            }
            p.result[0] = (e == 0) ? 0 : 2;          // 2 would be an internal inconsistency
            p.result[1] = bv;
            p.result[2] = be;
        }
    }
}

hipError_t launch_dp(const DpParams& p, hipStream_t s) {
    const size_t lds = (size_t)(p.D + 1) * sizeof(int64_t);
    const int nk = (p.D + 1 + kDpThreads - 1) / kDpThreads;
    hipError_t err = hipSuccess;
#define LGRECO_DP(K)                                                                               \
    do {                                                                                           \
        err = hipFuncSetAttribute((const void*)dp_kernel<K>, hipFuncAttributeMaxDynamicSharedMemorySize, \
                                  (int)lds);                                                       \
        if (err != hipSuccess) return err;                                                         \
        hipLaunchKernelGGL((dp_kernel<K>), dim3(1), dim3(kDpThreads), lds, s, p);                  \
    } while (0)
    if (nk <= 1) LGRECO_DP(1);
    else if (nk <= 2) LGRECO_DP(2);
    else if (nk <= 4) LGRECO_DP(4);
    else if (nk <= 8) LGRECO_DP(8);
    else LGRECO_DP(kDpMaxK);
#undef LGRECO_DP
    return hipGetLastError();
}

}  // namespace lgreco

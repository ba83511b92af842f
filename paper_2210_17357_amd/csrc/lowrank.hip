// PowerSGD-style low rank: one power-iteration step per layer on fp32 MFMA, for gfx950.
//
//   P = X Q0            X = g + e viewed as [m x n] row-major, Q0 [n x 64] warm start
//   Phat = orth(P)      Gram-Schmidt on the columns, done in coefficient space: G = P^T P in
//                       fp64, one wavefront per layer runs the column-by-column elimination
//                       on the 64 x 64 Gram matrix (lane j owns column j; this is exactly the
//                       Gram-Schmidt recurrence on the inner products), inverts the triangular
//                       factor and Phat = P T.  A column whose squared norm after projection is
//                       0 or below 1e-10 x its squared norm before projection becomes zero.
//   Q = X^T Phat
//   error_r = ||X||^2 - sum_{j<r} ||q_j||^2    (Phat orthonormal, Q = X^T Phat, and the factors
//                       of rank r are the leading columns of the rank-64 run, so one run yields
//                       every rank's error)
//   compress: payload Phat[:, :r], Q[:, :r];  e' = X - Phat[:, :r] Q[:, :r]^T
//
// The two contractions and the reconstruction use v_mfma_f32_32x32x2f32 (fp32 in, fp32
// accumulate).  Operand layout of that instruction, lane l of 64:
//   A (32 x 2): A[i = l % 32][k = l / 32];   B (2 x 32): B[k = l / 32][j = l % 32]
//   D (32 x 32): register v (0..15) holds D[8 (v / 4) + 4 (l / 32) + v % 4][l % 32]
#include <cstring>

#include "internal.h"

namespace lgreco {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kLrCols = 64;       // columns computed per layer (r_max <= 64)
constexpr int kLrBM = 128;        // rows (GEMM1, reconstruction) / columns (GEMM2) per workgroup
constexpr int kLrBK = 32;         // contraction chunk staged in LDS
constexpr int kLrGramSpan = 256;  // rows per Gram partial (one workgroup)
constexpr int kLrQChunk = 64;     // Q rows per workgroup in the split-K reduction
constexpr int kLrPSplit = 512;    // columns contracted per workgroup in P = X Q0
constexpr int kLrEfSpan = 512;    // columns reconstructed per workgroup

struct LrLayer {
    int64_t offset;     // into g / e
    int64_t q_off;      // into q0 / q (stride r_max)
    int64_t p_off;      // into the P scratch (rows x 64)
    int64_t qs_off;     // into the Q scratch (cols x 64)
    int64_t part_off;   // into the split-K partial buffer (splits x cols x 64)
    int64_t payload;    // byte offset of the payload (compress)
    int32_t rows, cols;
    int32_t rank;       // columns written out (64 when profiling)
    int32_t splits, ksplit;         // split of the row contraction of Q = X^T Phat
    int32_t psplits, pksplit;       // split of the column contraction of P = X Q0
    int64_t ppart_off;              // into the P partial buffer (psplits x rows x 64) when psplits > 1
    int32_t gram_begin, gram_end;   // Gram partial range
    int32_t rt_begin, rt_end;       // row-tile range (||X||^2 partials)
    int32_t qc_begin, qc_end;       // Q-chunk range (column-norm partials)
    int32_t vec_ok;     // 16-byte aligned rows: offset % 4 == 0 and cols % 4 == 0
    int32_t index;      // index in the caller's layer table
    int32_t pad;
};
struct LrTile {
    int32_t layer, a0, split, pad;
};

struct LrParams {
    const float* g;
    const float* e;          // may be null
    float* e_out;            // compress: error feedback (same buffer as e)
    const float* q0;         // warm start (stride r_max)
    float* q_out;            // compress: new Q (stride r_max), same buffer as q0
    int32_t r_max;
    const LrLayer* layers;
    const LrTile* row_tiles;   // 128-row tiles (orthogonalisation)
    const LrTile* p_tiles;     // (128-row tile, column split) of P = X Q0
    const LrTile* ef_tiles;    // (64-row tile, 512-column span) of the reconstruction
    const LrTile* col_tiles;
    const LrTile* gram_tiles;
    const LrTile* q_chunks;
    float* P;                // scratch [sum rows x 64]
    float* Q;                // scratch [sum cols x 64]
    float* part;             // split-K partials of Q
    float* ppart;            // split-K partials of P
    double* gram_part;       // [gram tiles x 64 x 64]
    double* T;               // [layers x 64 x 64]
    double* xnorm_part;      // [row tiles]
    double* qnorm_part;      // [q chunks x 64]
    uint8_t* payload;
    double* errors;          // [L x stride]
    int32_t stride;
    int32_t nrank;
    int32_t rank[LGRECO_MAX_CANDS];
    int32_t col[LGRECO_MAX_CANDS];
    int32_t accumulate;      // decode: add the image to the output instead of replacing it
    int32_t q_from_scratch;  // P = X Q reads the previous step's Q instead of the warm start
    int32_t e_is_zero;       // compression: e is null because the caller promised zeros; x = fl32(g + 0) all the same
    const DevLayer* dev_layers;   // KNOWN kernels: the caller's layer records (family, rank, payload offset) on the device
};

// 4 consecutive elements of x = g + e starting at idx of a row that has `left` elements left.
__device__ __forceinline__ float4 load_x4(const float* __restrict__ g, const float* __restrict__ e, int64_t idx,
                                          int left, bool vec_ok) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (left >= 4 && vec_ok) {
        v = *reinterpret_cast<const float4*>(g + idx);
        if (e) {
            const float4 w = *reinterpret_cast<const float4*>(e + idx);
            v.x += w.x; v.y += w.y; v.z += w.z; v.w += w.w;
        }
    } else {
        if (left > 0) v.x = e ? g[idx] + e[idx] : g[idx];
        if (left > 1) v.y = e ? g[idx + 1] + e[idx + 1] : g[idx + 1];
        if (left > 2) v.z = e ? g[idx + 2] + e[idx + 2] : g[idx + 2];
        if (left > 3) v.w = e ? g[idx + 3] + e[idx + 3] : g[idx + 3];
    }
    return v;
}

// ------------------------------------------------------------------ P = X Q0 (and ||X||^2)
// One workgroup: 128 rows x 64 columns of P over one column range of X; wavefront w owns rows
// 32w .. 32w+31.  The A operand never passes through LDS: lane l keeps, for row l % 32, the 16
// consecutive elements X[row][k0 + 16 (l / 32) .. + 15] of the current 32-column chunk in
// registers (four 128-bit loads; lanes l and l + 32 together read one 128-byte line of the row),
// and MFMA step s contracts the column pair (k0 + s, k0 + 16 + s).  Only the 32 x 64 chunk of Q0,
// shared by the four wavefronts, is staged in LDS (double buffered).
template <bool HAS_E>
__global__ __launch_bounds__(256) void lr_gemm1_kernel(LrParams p) {
    __shared__ float Qs[2][kLrBK][kLrCols];
    __shared__ double s_red[4];
    const LrTile tile = p.p_tiles[blockIdx.x];
    const LrLayer L = p.layers[tile.layer];
    const int m = L.rows, n = L.cols, row0 = tile.a0;
    const int kbeg = tile.split * L.pksplit, kend = min(n, kbeg + L.pksplit);
    const float* __restrict__ g = p.g + L.offset;
    const float* __restrict__ e = HAS_E ? p.e + L.offset : nullptr;
    // first power-iteration step: the caller's warm start (row stride r_max); later steps: the Q
    // of the previous step in the scratch buffer (row stride 64)
    const bool qscr = p.q_from_scratch != 0;
    const float* __restrict__ q = qscr ? p.Q + L.qs_off : p.q0 + L.q_off;
    const int qstride = qscr ? kLrCols : p.r_max;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const bool vec = L.vec_ok != 0;
    const bool qvec = (qstride == kLrCols) && (qscr || L.q_off % 4 == 0);
    const int half = lane >> 5, bj = lane & 31;
    const int row = row0 + 32 * wave + bj;               // this lane's row of X
    const bool row_ok = row < m;
    const float* __restrict__ grow = g + (int64_t)row * n;
    const float* __restrict__ erow = HAS_E ? e + (int64_t)row * n : nullptr;

    float4 xg[4], xe[HAS_E ? 4 : 1], qr[2];
    bool add_e = false;
    // issue the loads of one chunk (their values are first used after the MFMAs of the chunk
    // that is being multiplied)
    auto fetch = [&](int k0) {
        const int kx = k0 + 16 * half;
        add_e = false;
        if (vec && row_ok && k0 + kLrBK <= kend) {           // uniform except for the row test
            add_e = HAS_E;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                xg[s] = *reinterpret_cast<const float4*>(grow + kx + 4 * s);
                if (HAS_E) xe[s] = *reinterpret_cast<const float4*>(erow + kx + 4 * s);
            }
        } else {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                xg[s] = make_float4(0.f, 0.f, 0.f, 0.f);
                const int kk = kx + 4 * s;
                if (row_ok && kk < kend) xg[s] = load_x4(grow, erow, kk, kend - kk, vec);
            }
        }
        if (qvec && k0 + kLrBK <= kend) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const int f = tid + 256 * s;
                qr[s] = *reinterpret_cast<const float4*>(q + (int64_t)(k0 + (f >> 4)) * kLrCols + (f & 15) * 4);
            }
        } else {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const int f = tid + 256 * s;
                const int k = k0 + (f >> 4), c = (f & 15) * 4;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (k < kend) {
                    const float* src = q + (int64_t)k * qstride + c;
                    if (c < qstride) v.x = src[0];
                    if (c + 1 < qstride) v.y = src[1];
                    if (c + 2 < qstride) v.z = src[2];
                    if (c + 3 < qstride) v.w = src[3];
                }
                qr[s] = v;
            }
        }
    };
    float xsq = 0.0f;
    float cur[16];
    // take the fetched chunk into use: x = g + e, ||x||^2, Q0 rows to LDS
    auto commit = [&](int buf) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            float4 v = xg[s];
            if (HAS_E && add_e) { v.x += xe[s].x; v.y += xe[s].y; v.z += xe[s].z; v.w += xe[s].w; }
            cur[4 * s] = v.x; cur[4 * s + 1] = v.y; cur[4 * s + 2] = v.z; cur[4 * s + 3] = v.w;
            xsq = __builtin_fmaf(v.x, v.x, xsq);
            xsq = __builtin_fmaf(v.y, v.y, xsq);
            xsq = __builtin_fmaf(v.z, v.z, xsq);
            xsq = __builtin_fmaf(v.w, v.w, xsq);
        }
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int f = tid + 256 * s;
            *reinterpret_cast<float4*>(&Qs[buf][f >> 4][(f & 15) * 4]) = qr[s];
        }
    };

    f32x16 acc0 = {0}, acc1 = {0};
    const int nchunks = (kend - kbeg + kLrBK - 1) / kLrBK;
    fetch(kbeg);
    commit(0);
    __syncthreads();
    for (int c = 0; c < nchunks; ++c) {
        const int buf = c & 1;
        if (c + 1 < nchunks) fetch(kbeg + (c + 1) * kLrBK);
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            const float b0 = Qs[buf][16 * half + s][bj];
            const float b1 = Qs[buf][16 * half + s][32 + bj];
            acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(cur[s], b0, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(cur[s], b1, acc1, 0, 0, 0);
        }
        if (c + 1 < nchunks) commit(buf ^ 1);
        __syncthreads();
    }
    float* __restrict__ P = L.psplits > 1 ? p.ppart + L.ppart_off + (int64_t)tile.split * m * kLrCols
                                          : p.P + L.p_off;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int orow = row0 + 32 * wave + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (orow < m) {
            P[(int64_t)orow * kLrCols + bj] = acc0[v];
            P[(int64_t)orow * kLrCols + 32 + bj] = acc1[v];
        }
    }
    const double s = wave_sum((double)xsq);
    if (lane == 0) s_red[wave] = s;
    __syncthreads();
    if (tid == 0) p.xnorm_part[blockIdx.x] = s_red[0] + s_red[1] + s_red[2] + s_red[3];
}

// ------------------------------------------------------------------ P = sum of column-split partials
__global__ __launch_bounds__(256) void lr_preduce_kernel(LrParams p) {
    const LrTile tile = p.row_tiles[blockIdx.x];
    const LrLayer L = p.layers[tile.layer];
    if (L.psplits <= 1) return;
    const int nrows = min(kLrBM, L.rows - tile.a0);
    const float* __restrict__ part = p.ppart + L.ppart_off;
    float* __restrict__ P = p.P + L.p_off;
    for (int f = threadIdx.x; f < nrows * kLrCols / 4; f += 256) {
        const int64_t idx = (int64_t)tile.a0 * kLrCols + (int64_t)f * 4;
        float4 s = *reinterpret_cast<const float4*>(part + idx);
        for (int sp = 1; sp < L.psplits; ++sp) {
            const float4 v = *reinterpret_cast<const float4*>(part + (int64_t)sp * L.rows * kLrCols + idx);
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
        *reinterpret_cast<float4*>(P + idx) = s;
    }
}

// ------------------------------------------------------------------ partial Gram matrices
// G = P^T P over a span of rows, accumulated in fp64 on v_mfma_f64_16x16x4f64.  Operand layout of
// that instruction, lane l of 64:  A (16 x 4): A[i = l % 16][k = l / 16];  B (4 x 16):
// B[k = l / 16][j = l % 16];  D (16 x 16): register v (0..3) holds D[4 v + l / 16][l % 16].
// With A = P^T and B = P both operands of a 4-row step are the same four values per lane
// (P[row0 + l / 16][16 b + l % 16], b = 0..3), so P goes from global memory straight into the
// matrix pipe.  The four wavefronts take interleaved 16-row groups and add their results in LDS
// in wavefront order.
typedef double f64x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void lr_gram_kernel(LrParams p) {
    __shared__ double Gs[kLrCols][kLrCols];
    const LrTile tile = p.gram_tiles[blockIdx.x];
    const LrLayer L = p.layers[tile.layer];
    const float* __restrict__ P = p.P + L.p_off;
    const int span_end = min(L.rows, tile.a0 + kLrGramSpan);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int lr = lane >> 4, lc = lane & 15;
    f64x4 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f64x4{0.0, 0.0, 0.0, 0.0};
    // the loads of the next 16-row group are in flight while the current one is multiplied
    auto fetch = [&](int r0, float (&x)[4][4]) __attribute__((always_inline)) {
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            const int r = r0 + 4 * st + lr;
#pragma unroll
            for (int b = 0; b < 4; ++b) x[st][b] = r < span_end ? P[(int64_t)r * kLrCols + 16 * b + lc] : 0.0f;
        }
    };
    float x[4][4], xn[4][4];      // [4-row step][column block]
    fetch(tile.a0 + 16 * wave, x);          // rows past the span's end read as zero
    for (int r0 = tile.a0 + 16 * wave; r0 < span_end; r0 += 64) {
        fetch(r0 + 64, xn);
#pragma unroll
        for (int st = 0; st < 4; ++st) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)x[st][i], (double)x[st][j], acc[i][j],
                                                                     0, 0, 0);
        }
#pragma unroll
        for (int st = 0; st < 4; ++st)
#pragma unroll
            for (int b = 0; b < 4; ++b) x[st][b] = xn[st][b];
    }
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        double* g = &Gs[16 * i + 4 * v + lr][16 * j + lc];
                        *g = (w == 0) ? acc[i][j][v] : *g + acc[i][j][v];
                    }
        }
        __syncthreads();
    }
    double* __restrict__ out = p.gram_part + (size_t)blockIdx.x * kLrCols * kLrCols;
    for (int f = tid; f < kLrCols * kLrCols; f += 256) out[f] = Gs[f >> 6][f & 63];
}

// ------------------------------------------------------------------ Gram-Schmidt coefficients
// One workgroup per layer.  The Gram matrix sits in registers: thread (wavefront w, lane j) holds
// G[4 m + w][j], m = 0..15.  Elimination step i (Gram-Schmidt on the inner products): the
// wavefront that owns row i scales it into row i of R and publishes it in LDS; after one barrier
// every thread subtracts R[i][k] R[i][j] from its rows k > i.  Then T = R^-1 by back substitution
// (one wavefront, lane j solves column j against R in LDS).
__device__ __forceinline__ double lane_value(double v, int lane) {      // v of a given lane, as a scalar
    const uint64_t b = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)b, lane);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(b >> 32), lane);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}

// G = sum of a layer's Gram partials in partial order, one matrix element per thread (16
// workgroups per layer), left in the layer's first partial.  A layer of many rows has many
// partials: summed here their loads run eight deep on 4096 threads instead of serially in the
// one workgroup that eliminates.
__global__ __launch_bounds__(256) void lr_gram_reduce_kernel(LrParams p) {
    const LrLayer L = p.layers[blockIdx.x / 16];
    if (L.gram_end - L.gram_begin < 2) return;
    const int f = (blockIdx.x % 16) * 256 + threadIdx.x;
    double* const first = p.gram_part + (size_t)L.gram_begin * kLrCols * kLrCols + f;
    const int n = L.gram_end - L.gram_begin;
    double s = 0.0;
    int c = 0;
    for (; c + 8 <= n; c += 8) {
        double v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = first[(size_t)(c + u) * kLrCols * kLrCols];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; c < n; ++c) s += first[(size_t)c * kLrCols * kLrCols];
    *first = s;
}

__global__ __launch_bounds__(256) void lr_orth_kernel(LrParams p) {
    __shared__ double R[kLrCols][kLrCols];
    __shared__ double diag0[kLrCols];
    const LrLayer L = p.layers[blockIdx.x];
    const int tid = threadIdx.x, w = tid >> 6, j = tid & 63;
    // G: the layer's Gram matrix (its partials already summed into the first)
    double g[16];
    {
        const double* __restrict__ src = p.gram_part + (size_t)L.gram_begin * kLrCols * kLrCols + w * kLrCols + j;
#pragma unroll
        for (int m = 0; m < 16; ++m) g[m] = src[4 * m * kLrCols];
    }
#pragma unroll
    for (int m = 0; m < 16; ++m)
        if (4 * m + w == j) diag0[j] = g[m];      // squared norms before any projection
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kLrCols; ++i) {
        if (w == (i & 3)) {
            const double gi = g[i >> 2];                     // G[i][j], current
            const double d = lane_value(gi, i);
            const double d0 = diag0[i];
            const bool ok = d > 0.0 && d >= 1e-10 * d0;
            const double rii = ok ? sqrt(d) : 0.0;
            const double inv = ok ? 1.0 / rii : 0.0;
            R[i][j] = (j >= i) ? ((j == i) ? rii : gi * inv) : 0.0;
        }
        __syncthreads();
        const double rj = R[i][j];
#pragma unroll
        for (int m = 0; m < 16; ++m)
            if (4 * m + 3 > i) {                              // some row of this group lies below i
                const int k = 4 * m + w;
                if (k > i) g[m] = __builtin_fma(-R[i][k], rj, g[m]);
            }
    }
    __syncthreads();
    if (w != 0) return;
    // T = R^-1, column j; columns that were zeroed stay zero
    double t[kLrCols];
#pragma unroll
    for (int i = kLrCols - 1; i >= 0; --i) {
        double s = (i == j) ? 1.0 : 0.0;
#pragma unroll
        for (int k = i + 1; k < kLrCols; ++k) s = __builtin_fma(-R[i][k], t[k], s);
        const double rii = R[i][i];
        t[i] = (i <= j && rii != 0.0) ? s / rii : 0.0;
    }
    double* __restrict__ T = p.T + (size_t)blockIdx.x * kLrCols * kLrCols;
#pragma unroll
    for (int i = 0; i < kLrCols; ++i) T[i * kLrCols + j] = t[i];
}

// ------------------------------------------------------------------ Phat = P T
// fp64 MFMA: a wavefront takes 16 rows of P at a time (A[i][k] = P[row0 + i][k], 16 loads per
// lane, all issued before the first MFMA and before any store, so the update is in place) against
// T in LDS; T is upper triangular, so column block b needs only k < 16 (b + 1).
__global__ __launch_bounds__(256) void lr_apply_kernel(LrParams p) {
    __shared__ double Tl[kLrCols][kLrCols + 2];     // padded: the four k rows of a step on different banks
    const LrTile tile = p.gram_tiles[blockIdx.x];          // one workgroup per span of kLrGramSpan rows
    const LrLayer L = p.layers[tile.layer];
    float* __restrict__ P = p.P + L.p_off;
    const double* __restrict__ T = p.T + (size_t)tile.layer * kLrCols * kLrCols;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int lr = lane >> 4, lc = lane & 15;
    for (int f = tid; f < kLrCols * kLrCols; f += 256) Tl[f >> 6][f & 63] = T[f];
    float* pay = p.payload ? reinterpret_cast<float*>(p.payload + L.payload) : nullptr;
    __syncthreads();
    for (int blk = wave; blk < kLrGramSpan / 16; blk += 4) {
        const int row0 = tile.a0 + 16 * blk;
        if (row0 >= L.rows) break;
        const int arow = row0 + lc;
        float a[16];
#pragma unroll
        for (int s = 0; s < 16; ++s) a[s] = arow < L.rows ? P[(int64_t)arow * kLrCols + 4 * s + lr] : 0.0f;
        f64x4 acc[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            acc[b] = f64x4{0.0, 0.0, 0.0, 0.0};
#pragma unroll
            for (int s = 0; s < 4 * (b + 1); ++s)
                acc[b] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)a[s], Tl[4 * s + lr][16 * b + lc], acc[b], 0, 0, 0);
        }
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = row0 + 4 * v + lr, col = 16 * b + lc;
                if (row < L.rows) {
                    const float val = (float)acc[b][v];
                    P[(int64_t)row * kLrCols + col] = val;
                    if (pay && col < L.rank) pay[(int64_t)row * L.rank + col] = val;
                }
            }
    }
}

// ------------------------------------------------------------------ Q partials = X^T Phat
template <bool HAS_E>
__global__ __launch_bounds__(256) void lr_gemm2_kernel(LrParams p) {
    __shared__ float Xs[2][kLrBK][kLrBM];
    __shared__ float Ps[2][kLrBK][kLrCols];
    const LrTile tile = p.col_tiles[blockIdx.x];
    const LrLayer L = p.layers[tile.layer];
    const int m = L.rows, n = L.cols, col0 = tile.a0;
    const int kbeg = tile.split * L.ksplit, kend = min(m, kbeg + L.ksplit);
    const float* __restrict__ g = p.g + L.offset;
    const float* __restrict__ e = HAS_E ? p.e + L.offset : nullptr;
    const float* __restrict__ P = p.P + L.p_off;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const bool vec = L.vec_ok != 0;

    float4 xr[4], pr[2];
    const bool cols_full = col0 + kLrBM <= n;
    float4 er[HAS_E ? 4 : 1];
    bool add_e = false;
    auto fetch = [&](int k0) {
        add_e = false;
        if (vec && cols_full && k0 + kLrBK <= kend) {       // no per-load condition (see lr_gemm1_kernel)
            add_e = HAS_E;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int f = tid + 256 * s;
                const int64_t idx = (int64_t)(k0 + (f >> 5)) * n + col0 + (f & 31) * 4;
                xr[s] = *reinterpret_cast<const float4*>(g + idx);
                if (HAS_E) er[s] = *reinterpret_cast<const float4*>(e + idx);
            }
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const int f = tid + 256 * s;
                pr[s] = *reinterpret_cast<const float4*>(P + (int64_t)(k0 + (f >> 4)) * kLrCols + (f & 15) * 4);
            }
            return;
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int f = tid + 256 * s;
            const int kr = f >> 5, c = (f & 31) * 4;
            const int row = k0 + kr, col = col0 + c;
            xr[s] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row < kend && col < n) xr[s] = load_x4(g, e, (int64_t)row * n + col, n - col, vec);
        }
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int f = tid + 256 * s;
            const int kr = f >> 4, c = (f & 15) * 4;
            const int row = k0 + kr;
            pr[s] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row < kend) pr[s] = *reinterpret_cast<const float4*>(P + (int64_t)row * kLrCols + c);
        }
    };
    auto stash = [&](int buf) {
        if (HAS_E && add_e) {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                xr[s].x += er[s].x; xr[s].y += er[s].y; xr[s].z += er[s].z; xr[s].w += er[s].w;
            }
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int f = tid + 256 * s;
            *reinterpret_cast<float4*>(&Xs[buf][f >> 5][(f & 31) * 4]) = xr[s];
        }
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int f = tid + 256 * s;
            *reinterpret_cast<float4*>(&Ps[buf][f >> 4][(f & 15) * 4]) = pr[s];
        }
    };

    f32x16 acc0 = {0}, acc1 = {0};
    const int nchunks = (kend - kbeg + kLrBK - 1) / kLrBK;
    fetch(kbeg);
    stash(0);
    __syncthreads();
    const int ai = 32 * wave + (lane & 31), ak = lane >> 5, bj = lane & 31;
    for (int c = 0; c < nchunks; ++c) {
        const int buf = c & 1;
        if (c + 1 < nchunks) fetch(kbeg + (c + 1) * kLrBK);
#pragma unroll
        for (int kk = 0; kk < kLrBK; kk += 2) {
            const float a = Xs[buf][kk + ak][ai];
            const float b0 = Ps[buf][kk + ak][bj];
            const float b1 = Ps[buf][kk + ak][32 + bj];
            acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b0, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b1, acc1, 0, 0, 0);
        }
        if (c + 1 < nchunks) stash(buf ^ 1);
        __syncthreads();
    }
    float* __restrict__ out = p.part + L.part_off + (int64_t)tile.split * n * kLrCols;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int col = col0 + 32 * wave + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (col < n) {
            out[(int64_t)col * kLrCols + bj] = acc0[v];
            out[(int64_t)col * kLrCols + 32 + bj] = acc1[v];
        }
    }
}

// ------------------------------------------------------------------ Q = sum of partials, norms
__global__ __launch_bounds__(256) void lr_qreduce_kernel(LrParams p) {
    __shared__ double s_n[4][kLrCols];
    __shared__ float s_p[4][kLrCols];
    const LrTile tile = p.q_chunks[blockIdx.x];
    const LrLayer L = p.layers[tile.layer];
    const int n = L.cols, c0 = tile.a0, nc = min(tile.split, n - c0);    // tile.split = rows of this chunk
    const float* __restrict__ part = p.part + L.part_off;
    float* __restrict__ Q = p.Q + L.qs_off;
    const int tid = threadIdx.x, j = tid & 63, grp = tid >> 6;
    float* pay = nullptr;
    if (p.payload) pay = reinterpret_cast<float*>(p.payload + L.payload) + (int64_t)L.rows * L.rank;
    double norm = 0.0;
    auto emit = [&](int r, float s) {
        const int64_t idx = (int64_t)(c0 + r) * kLrCols + j;
        Q[idx] = s;
        norm = __builtin_fma((double)s, (double)s, norm);
        if (p.payload && j < L.rank) {
            pay[(int64_t)(c0 + r) * L.rank + j] = s;
            p.q_out[L.q_off + (int64_t)(c0 + r) * p.r_max + j] = s;
        }
    };
    // sum of partials [sp0, sp1) of one element in partial order, the loads eight deep
    auto sum_partials = [&](int64_t idx, int sp0, int sp1) {
        const int64_t stride = (int64_t)n * kLrCols;
        float s = 0.0f;
        int sp = sp0;
        for (; sp + 8 <= sp1; sp += 8) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = part[(int64_t)(sp + u) * stride + idx];
#pragma unroll
            for (int u = 0; u < 8; ++u) s += v[u];
        }
        for (; sp < sp1; ++sp) s += part[(int64_t)sp * stride + idx];
        return s;
    };
    if (L.splits <= 4) {
        // few partials: one thread per (row, column), rows strided over the 4 wavefronts
        // (four rows per pass: their up to 16 loads are in flight together)
        const int64_t stride = (int64_t)n * kLrCols;
        for (int r = grp; r < nc; r += 16) {
            float v[4][4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int rr = r + 4 * u;
                const int64_t idx = (int64_t)(c0 + rr) * kLrCols + j;
#pragma unroll
                for (int sp = 0; sp < 4; ++sp)
                    v[u][sp] = (rr < nc && sp < L.splits) ? part[(int64_t)sp * stride + idx] : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int rr = r + 4 * u;
                if (rr < nc) {
                    float s = 0.0f;
#pragma unroll
                    for (int sp = 0; sp < 4; ++sp)
                        if (sp < L.splits) s += v[u][sp];
                    emit(rr, s);
                }
            }
        }
    } else {
        // many partials: the 4 wavefronts share one row, each sums a contiguous quarter of the
        // partials, and wavefront 0 adds the four sums in order
        const int per = (L.splits + 3) / 4;
        const int sp0 = grp * per, sp1 = min(L.splits, sp0 + per);
        for (int r = 0; r < nc; ++r) {
            const int64_t idx = (int64_t)(c0 + r) * kLrCols + j;
            s_p[grp][j] = sum_partials(idx, sp0, sp1);
            __syncthreads();
            if (grp == 0) emit(r, ((s_p[0][j] + s_p[1][j]) + s_p[2][j]) + s_p[3][j]);
            __syncthreads();
        }
    }
    s_n[grp][j] = norm;
    __syncthreads();
    if (tid < kLrCols)
        p.qnorm_part[(size_t)blockIdx.x * kLrCols + tid] = s_n[0][tid] + s_n[1][tid] + s_n[2][tid] + s_n[3][tid];
}

// ------------------------------------------------------------------ errors of every rank
// One workgroup per layer; the four wavefronts split the partial sums (column norms of Q per
// chunk, ||X||^2 per tile) into contiguous quarters that are added in a fixed order.
__global__ __launch_bounds__(256) void lr_errors_kernel(LrParams p) {
    __shared__ double s_q[4][kLrCols];
    __shared__ double s_x[4];
    const LrLayer L = p.layers[blockIdx.x];
    const int j = threadIdx.x & 63, w = threadIdx.x >> 6;
    {
        const int n = L.qc_end - L.qc_begin, per = (n + 3) / 4;
        const int c0 = L.qc_begin + min(n, w * per), c1 = L.qc_begin + min(n, (w + 1) * per);
        double qn = 0.0;
#pragma unroll 8
        for (int c = c0; c < c1; ++c) qn += p.qnorm_part[(size_t)c * kLrCols + j];
        s_q[w][j] = qn;
    }
    {
        const int n = L.rt_end - L.rt_begin, per = (n + 3) / 4;
        const int t0 = L.rt_begin + min(n, w * per), t1 = L.rt_begin + min(n, (w + 1) * per);
        double xn = 0.0;
        for (int t = t0 + j; t < t1; t += 64) xn += p.xnorm_part[t];
        xn = wave_sum(xn);
        if (j == 0) s_x[w] = xn;
    }
    __syncthreads();
    if (w != 0) return;
    const double qn = ((s_q[0][j] + s_q[1][j]) + s_q[2][j]) + s_q[3][j];
    const double xn = ((s_x[0] + s_x[1]) + s_x[2]) + s_x[3];
    // inclusive prefix over columns, in column order
    double pre = qn;
    for (int o = 1; o < 64; o <<= 1) {
        const double v = __shfl_up(pre, o, 64);
        if (j >= o) pre += v;
    }
    for (int c = 0; c < p.nrank; ++c)
        if (j == p.rank[c] - 1) p.errors[(size_t)L.index * p.stride + p.col[c]] = fmax(xn - pre, 0.0);
}

// ------------------------------------------------------------------ e' = X - Phat Q^T
// DECODE (receiver side): the factors come from the payload (row stride = rank) and the product
// is written, or added, to the output buffer instead of being subtracted from x.
// KNOWN (compression right behind a profile of the same data): the factors are the leading columns
// of the profile's rank-64 run, still in its scratch; whether the layer takes part and its rank
// come from the layer records the solver kernel wrote.
template <bool DECODE, bool KNOWN = false>
__global__ __launch_bounds__(256) void lr_ef_kernel(LrParams p) {
    __shared__ float Ps[64][kLrCols + 1];
    __shared__ float Qs[kLrCols][kLrCols + 1];
    __shared__ float Ms[64][kLrCols + 4];
    const LrTile tile = p.ef_tiles[blockIdx.x];
    const LrLayer L = p.layers[tile.layer];
    int r = L.rank;
    if (KNOWN) {
        const DevLayer& dl = p.dev_layers[L.index];
        if (dl.family != LGRECO_LOWRANK || dl.iparam < 1 || dl.iparam > kLrCols) return;
        r = dl.iparam;
    }
    const int m = L.rows, n = L.cols;
    const int kmax = (r + 1) & ~1;
    const float* __restrict__ g = DECODE ? (p.accumulate ? p.e_out + L.offset : nullptr) : p.g + L.offset;
    const float* __restrict__ ein = DECODE ? nullptr : p.e;
    float* __restrict__ e = p.e_out + L.offset;
    const float* __restrict__ P =
        DECODE ? reinterpret_cast<const float*>(p.payload + L.payload) : p.P + L.p_off;
    const float* __restrict__ Q = DECODE ? P + (int64_t)m * r : p.Q + L.qs_off;
    const int pstride = DECODE ? r : kLrCols;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const bool vec = L.vec_ok != 0;
    // the 4 wavefronts split a 64 x 64 output tile into 32 x 32 quadrants
    const int wr = wave >> 1, wc = wave & 1;
    const int ar = 32 * wr + (lane & 31), ak = lane >> 5, bj = 32 * wc + (lane & 31);
    const int row0 = tile.a0, cbeg = tile.split, cend = min(n, cbeg + kLrEfSpan);
    for (int f = tid; f < 64 * kLrCols; f += 256) {
        const int rr = f >> 6, c = f & 63;
        Ps[rr][c] = (row0 + rr < m && c < r) ? P[(int64_t)(row0 + rr) * pstride + c] : 0.0f;
    }
    // Software pipeline over the 64-column tiles of the span, two tiles deep: the loads of tiles
    // t+1 and t+2 (x and the rows of Q) are in flight while tile t is worked on, in two register
    // sets that take turns (a workgroup has few neighbours on its compute unit - LDS allows three -
    // so the bytes in flight per workgroup are what the memory latency is hidden with).  Interior
    // tiles of aligned layers take a path without per-load conditions.
    struct Stage {
        float4 xn[4], en[4], qn[4];
        float qs[16];
        bool fast_x, fast_q, add_e;
    };
    const float* __restrict__ ebase = ein ? ein + L.offset : nullptr;
    auto fetch = [&](Stage& S, int c0) __attribute__((always_inline)) {
        S.fast_x = vec && g != nullptr && row0 + 64 <= m && c0 + kLrCols <= n;
        S.add_e = S.fast_x && ebase != nullptr;
        if (S.fast_x) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int f = tid + 256 * q;
                const int64_t idx = (int64_t)(row0 + (f >> 4)) * n + c0 + (f & 15) * 4;
                S.xn[q] = *reinterpret_cast<const float4*>(g + idx);
                if (ebase) S.en[q] = *reinterpret_cast<const float4*>(ebase + idx);
            }
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int f = tid + 256 * q;
                const int row = row0 + (f >> 4), colx = c0 + (f & 15) * 4;
                S.xn[q] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (g && row < m && colx < n) S.xn[q] = load_x4(g, ebase, (int64_t)row * n + colx, n - colx, vec);
            }
        }
        S.fast_q = !DECODE && c0 + kLrCols <= n;        // scratch Q: 64 columns per row, 16-byte aligned
        if (S.fast_q) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int f = tid + 256 * q;
                S.qn[q] = *reinterpret_cast<const float4*>(Q + (int64_t)(c0 + (f >> 4)) * kLrCols + (f & 15) * 4);
            }
        } else {
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int f = tid + 256 * q;
                const int cc = f >> 6, k = f & 63;
                S.qs[q] = (c0 + cc < n && k < r) ? Q[(int64_t)(c0 + cc) * pstride + k] : 0.0f;
            }
        }
    };
    // one tile from the stage that holds it; the stage is refilled with the tile two further on
    auto step = [&](Stage& S, int c0) __attribute__((always_inline)) {
        float4 x[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            x[q] = S.xn[q];
            if (S.add_e) { x[q].x += S.en[q].x; x[q].y += S.en[q].y; x[q].z += S.en[q].z; x[q].w += S.en[q].w; }
            // zeros that are not read are still added (a gradient of -0 becomes the +0 the sum with
            // a stored zero gives: every bit as without the promise)
            if (!DECODE && p.e_is_zero) { x[q].x += 0.0f; x[q].y += 0.0f; x[q].z += 0.0f; x[q].w += 0.0f; }
        }
        if (S.fast_q) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int f = tid + 256 * q;
                const int cc = f >> 4, k = (f & 15) * 4;
                Qs[cc][k] = k < r ? S.qn[q].x : 0.0f;
                Qs[cc][k + 1] = k + 1 < r ? S.qn[q].y : 0.0f;
                Qs[cc][k + 2] = k + 2 < r ? S.qn[q].z : 0.0f;
                Qs[cc][k + 3] = k + 3 < r ? S.qn[q].w : 0.0f;
            }
        } else {
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int f = tid + 256 * q;
                Qs[f >> 6][f & 63] = S.qs[q];
            }
        }
        __syncthreads();
        if (c0 + 2 * kLrCols < cend) fetch(S, c0 + 2 * kLrCols);
        f32x16 acc = {0};
        for (int kk = 0; kk < kmax; kk += 2)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(Ps[ar][kk + ak], Qs[bj][kk + ak], acc, 0, 0, 0);
#pragma unroll
        for (int v = 0; v < 16; ++v)
            Ms[32 * wr + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)][bj] = acc[v];
        __syncthreads();
        // coalesced update of the error feedback: 64 rows x 16 float4
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int f = tid + 256 * q;
            const int rr = f >> 4, c4 = (f & 15) * 4;
            const int row = row0 + rr, colx = c0 + c4;
            if (row < m && colx < n) {
                const int64_t idx = (int64_t)row * n + colx;
                const int left = n - colx;
                const float4 mh = *reinterpret_cast<const float4*>(&Ms[rr][c4]);
                const float4 o = DECODE ? make_float4(x[q].x + mh.x, x[q].y + mh.y, x[q].z + mh.z, x[q].w + mh.w)
                                        : make_float4(x[q].x - mh.x, x[q].y - mh.y, x[q].z - mh.z, x[q].w - mh.w);
                if (vec && left >= 4) {
                    *reinterpret_cast<float4*>(e + idx) = o;
                } else {
                    e[idx] = o.x;
                    if (left > 1) e[idx + 1] = o.y;
                    if (left > 2) e[idx + 2] = o.z;
                    if (left > 3) e[idx + 3] = o.w;
                }
            }
        }
    };
    Stage s0, s1;
    fetch(s0, cbeg);
    if (cbeg + kLrCols < cend) fetch(s1, cbeg + kLrCols);
    for (int c0 = cbeg; c0 < cend; c0 += 2 * kLrCols) {
        step(s0, c0);
        if (c0 + kLrCols < cend) step(s1, c0 + kLrCols);
    }
}

// Payload and warm-start update of a layer from the profile's scratch (KNOWN, see lr_ef_kernel):
// the first `rank` columns of Phat (row tiles, blockIdx < n_row_tiles) and of Q (chunks of
// kLrQChunk rows after them); Q also replaces the first `rank` columns of the layer's warm start.
__global__ __launch_bounds__(256) void lr_emit_known_kernel(LrParams p, int n_row_tiles) {
    const bool is_p = (int)blockIdx.x < n_row_tiles;
    const LrTile tile = is_p ? p.row_tiles[blockIdx.x] : p.q_chunks[blockIdx.x - n_row_tiles];
    const LrLayer L = p.layers[tile.layer];
    const DevLayer& dl = p.dev_layers[L.index];
    if (dl.family != LGRECO_LOWRANK || dl.iparam < 1 || dl.iparam > kLrCols) return;
    const int r = dl.iparam;
    float* const pay = reinterpret_cast<float*>(p.payload + dl.payload);
    const int tid = threadIdx.x;
    if (is_p) {
        const float* __restrict__ P = p.P + L.p_off;
        const int nr = min(kLrBM, L.rows - tile.a0);
        for (int f = tid; f < nr * r; f += 256) {
            const int rr = f / r, c = f - rr * r;
            pay[(int64_t)(tile.a0 + rr) * r + c] = P[(int64_t)(tile.a0 + rr) * kLrCols + c];
        }
    } else {
        const float* __restrict__ Q = p.Q + L.qs_off;
        float* const payq = pay + (int64_t)L.rows * r;
        const int nr = min(tile.split, L.cols - tile.a0);      // tile.split = rows of this chunk
        for (int f = tid; f < nr * r; f += 256) {
            const int rr = f / r, c = f - rr * r;
            const float v = Q[(int64_t)(tile.a0 + rr) * kLrCols + c];
            payq[(int64_t)(tile.a0 + rr) * r + c] = v;
            p.q_out[L.q_off + (int64_t)(tile.a0 + rr) * p.r_max + c] = v;
        }
    }
}

// ------------------------------------------------------------------------ host side
#define LR_CHECK(expr)                     \
    do {                                   \
        hipError_t _e = (expr);            \
        if (_e != hipSuccess) return _e;   \
    } while (0)

// Work tables and scratch are kept per kind of call (profile, compress, decompress): the three
// alternate in a training loop and each repeats its own layer table, so nothing is rebuilt.
constexpr int kLrSlots = 3;
enum { kLrSlotProfile = 0, kLrSlotCompress = 1, kLrSlotDecode = 2 };

struct LrHost {
    std::vector<LrLayer> layers;
    std::vector<LrTile> row_tiles, p_tiles, ef_tiles, col_tiles, gram_tiles, q_chunks;
    std::vector<int64_t> sig;       // signature of the layer table the tables were built for
    int64_t p_elems = 0, q_elems = 0, part_elems = 0, ppart_elems = 0;
    // device copies
    LrLayer* d_layers = nullptr;
    LrTile* d_tiles = nullptr;      // the four tile tables back to back
    size_t cap_layers = 0, cap_tiles = 0, cap_p = 0, cap_q = 0, cap_part = 0, cap_ppart = 0, cap_gram = 0, cap_T = 0,
           cap_xn = 0, cap_qn = 0;
    float* P = nullptr;
    float* Q = nullptr;
    float* part = nullptr;
    float* ppart = nullptr;
    double* gram = nullptr;
    double* T = nullptr;
    double* xn = nullptr;
    double* qn = nullptr;
};

static hipError_t grow(void** ptr, size_t* cap, size_t need) {
    if (need <= *cap) return hipSuccess;
    if (*ptr) LR_CHECK(hipFree(*ptr));
    *ptr = nullptr;
    *cap = 0;
    LR_CHECK(hipMalloc(ptr, need));
    *cap = need;
    return hipSuccess;
}

hipError_t lowrank_scratch_create(LowrankScratch* t, int64_t max_elems, int max_layers, int r_max,
                                  int power_iters) {
    t->power_iters = power_iters;
    t->max_elems = max_elems;
    t->max_layers = max_layers;
    t->r_max = r_max;
    t->host = new LrHost[kLrSlots]();
    return hipSuccess;
}

void lowrank_scratch_destroy(LowrankScratch* t) {
    LrHost* all = (LrHost*)t->host;
    if (all) {
        for (int i = 0; i < kLrSlots; ++i) {
            LrHost* H = &all[i];
            (void)hipFree(H->d_layers);
            (void)hipFree(H->d_tiles);
            (void)hipFree(H->P);
            (void)hipFree(H->Q);
            (void)hipFree(H->part);
            (void)hipFree(H->ppart);
            (void)hipFree(H->gram);
            (void)hipFree(H->T);
            (void)hipFree(H->xn);
            (void)hipFree(H->qn);
        }
        delete[] all;
    }
    *t = LowrankScratch{};
}

// Build the work tables for the layers with rank[l] > 0 and upload them.  Scratch buffers grow on
// demand (allocation happens only when a larger layer table arrives).
static hipError_t lr_prepare(LowrankScratch* t, int slot, const DevLayer* hl, int L, const int* rank, int r_max,
                             bool tables_only, hipStream_t s) {
    LrHost* H = &((LrHost*)t->host)[slot];
    std::vector<int64_t> sig;
    sig.reserve((size_t)L * 5 + 1);
    sig.push_back(r_max);
    for (int l = 0; l < L; ++l) {
        sig.push_back(hl[l].offset);
        sig.push_back(hl[l].rows);
        sig.push_back(hl[l].cols);
        sig.push_back(rank[l]);
        sig.push_back(hl[l].payload);
    }
    if (sig == H->sig) return hipSuccess;
    H->layers.clear();
    H->row_tiles.clear();
    H->p_tiles.clear();
    H->ef_tiles.clear();
    H->col_tiles.clear();
    H->gram_tiles.clear();
    H->q_chunks.clear();
    int64_t p_off = 0, q_off = 0, part_off = 0, ppart_off = 0;
    for (int l = 0; l < L; ++l) {
        if (rank[l] <= 0) continue;
        LrLayer a{};
        a.offset = hl[l].offset;
        a.q_off = hl[l].q_offset;
        a.rows = hl[l].rows;
        a.cols = hl[l].cols;
        a.rank = rank[l];
        a.payload = hl[l].payload;
        a.index = l;
        a.vec_ok = (a.offset % 4 == 0 && a.cols % 4 == 0) ? 1 : 0;
        a.p_off = p_off;
        a.qs_off = q_off;
        a.part_off = part_off;
        // split the contraction over rows so that every column tile gets enough workgroups
        const int col_tiles = (a.cols + kLrBM - 1) / kLrBM;
        int splits = 1;
        while (splits < 64 && (int64_t)a.rows / (splits * 2) >= 512 && col_tiles * splits < 128) splits *= 2;
        a.ksplit = ((a.rows + splits - 1) / splits + kLrBK - 1) / kLrBK * kLrBK;
        a.splits = (a.rows + a.ksplit - 1) / a.ksplit;
        const int li = (int)H->layers.size();
        // P = X Q0: equal work units of at most kLrPSplit contracted columns
        a.psplits = (a.cols + kLrPSplit - 1) / kLrPSplit;
        a.pksplit = ((a.cols + a.psplits - 1) / a.psplits + kLrBK - 1) / kLrBK * kLrBK;
        a.psplits = (a.cols + a.pksplit - 1) / a.pksplit;
        a.ppart_off = ppart_off;
        if (a.psplits > 1) ppart_off += (int64_t)a.psplits * a.rows * kLrCols;
        a.rt_begin = (int)H->p_tiles.size();            // ||X||^2 partials: one per P tile
        for (int r0 = 0; r0 < a.rows; r0 += kLrBM) {
            H->row_tiles.push_back(LrTile{li, r0, 0, 0});
            for (int sp = 0; sp < a.psplits; ++sp) H->p_tiles.push_back(LrTile{li, r0, sp, 0});
        }
        a.rt_end = (int)H->p_tiles.size();
        for (int r0 = 0; r0 < a.rows; r0 += 64)
            for (int c0 = 0; c0 < a.cols; c0 += kLrEfSpan) H->ef_tiles.push_back(LrTile{li, r0, c0, 0});
        for (int c0 = 0; c0 < a.cols; c0 += kLrBM)
            for (int sp = 0; sp < a.splits; ++sp) H->col_tiles.push_back(LrTile{li, c0, sp, 0});
        a.gram_begin = (int)H->gram_tiles.size();
        for (int r0 = 0; r0 < a.rows; r0 += kLrGramSpan) H->gram_tiles.push_back(LrTile{li, r0, 0, 0});
        a.gram_end = (int)H->gram_tiles.size();
        a.qc_begin = (int)H->q_chunks.size();
        {
            // rows per chunk: fewer when many split-K partials have to be summed per row
            const int qrows = a.splits <= 4 ? kLrQChunk : std::max(2, kLrQChunk / a.splits * 2);
            for (int c0 = 0; c0 < a.cols; c0 += qrows) H->q_chunks.push_back(LrTile{li, c0, qrows, 0});
        }
        a.qc_end = (int)H->q_chunks.size();
        p_off += (int64_t)a.rows * kLrCols;
        q_off += (int64_t)a.cols * kLrCols;
        part_off += (int64_t)a.splits * a.cols * kLrCols;
        H->layers.push_back(a);
    }
    H->p_elems = p_off;
    H->q_elems = q_off;
    H->part_elems = part_off;
    H->ppart_elems = ppart_off;
    const size_t nl = H->layers.size();
    const size_t nt = H->row_tiles.size() + H->p_tiles.size() + H->ef_tiles.size() + H->col_tiles.size() +
                      H->gram_tiles.size() + H->q_chunks.size();
    LR_CHECK(grow((void**)&H->d_layers, &H->cap_layers, sizeof(LrLayer) * std::max<size_t>(nl, 1)));
    LR_CHECK(grow((void**)&H->d_tiles, &H->cap_tiles, sizeof(LrTile) * std::max<size_t>(nt, 1)));
    if (tables_only) { p_off = q_off = part_off = ppart_off = 0; }
    LR_CHECK(grow((void**)&H->P, &H->cap_p, sizeof(float) * std::max<int64_t>(p_off, 1)));
    LR_CHECK(grow((void**)&H->Q, &H->cap_q, sizeof(float) * std::max<int64_t>(q_off, 1)));
    LR_CHECK(grow((void**)&H->part, &H->cap_part, sizeof(float) * std::max<int64_t>(part_off, 1)));
    LR_CHECK(grow((void**)&H->ppart, &H->cap_ppart, sizeof(float) * std::max<int64_t>(ppart_off, 1)));
    LR_CHECK(grow((void**)&H->gram, &H->cap_gram,
                  sizeof(double) * kLrCols * kLrCols * (tables_only ? 1 : std::max<size_t>(H->gram_tiles.size(), 1))));
    LR_CHECK(grow((void**)&H->T, &H->cap_T,
                  sizeof(double) * kLrCols * kLrCols * (tables_only ? 1 : std::max<size_t>(nl, 1))));
    LR_CHECK(grow((void**)&H->xn, &H->cap_xn, sizeof(double) * std::max<size_t>(H->p_tiles.size(), 1)));
    LR_CHECK(grow((void**)&H->qn, &H->cap_qn, sizeof(double) * kLrCols * std::max<size_t>(H->q_chunks.size(), 1)));
    if (nl) {
        LR_CHECK(hipMemcpyAsync(H->d_layers, H->layers.data(), sizeof(LrLayer) * nl, hipMemcpyHostToDevice, s));
        size_t o = 0;
        for (auto* v : {&H->row_tiles, &H->p_tiles, &H->ef_tiles, &H->col_tiles, &H->gram_tiles, &H->q_chunks}) {
            if (!v->empty())
                LR_CHECK(hipMemcpyAsync(H->d_tiles + o, v->data(), sizeof(LrTile) * v->size(),
                                        hipMemcpyHostToDevice, s));
            o += v->size();
        }
        LR_CHECK(hipStreamSynchronize(s));
    }
    H->sig = std::move(sig);
    return hipSuccess;
}

static void lr_fill_params(LrHost* H, LrParams* p) {
    p->layers = H->d_layers;
    p->row_tiles = H->d_tiles;
    p->p_tiles = p->row_tiles + H->row_tiles.size();
    p->ef_tiles = p->p_tiles + H->p_tiles.size();
    p->col_tiles = p->ef_tiles + H->ef_tiles.size();
    p->gram_tiles = p->col_tiles + H->col_tiles.size();
    p->q_chunks = p->gram_tiles + H->gram_tiles.size();
    p->P = H->P;
    p->Q = H->Q;
    p->part = H->part;
    p->ppart = H->ppart;
    p->gram_part = H->gram;
    p->T = H->T;
    p->xnorm_part = H->xn;
    p->qnorm_part = H->qn;
}

// `iters` power-iteration steps: P = X Q, Phat = orth(P), Q = X^T Phat, Q feeding the next step.
static hipError_t lr_factorize(LrHost* H, LrParams p, int iters, Timing* tm, hipStream_t s) {
  for (int it = 0; it < iters; ++it) {
    p.q_from_scratch = it > 0 ? 1 : 0;
    {
        Section sec(tm, "lowrank_gemm_p", true);
        const bool reduce = H->ppart_elems > 0;        // split-K partials: a second kernel ends the section
        if (p.e)
            launch_timed(&sec, true, !reduce, lr_gemm1_kernel<true>, dim3((unsigned)H->p_tiles.size()), dim3(256), 0, s, p);
        else
            launch_timed(&sec, true, !reduce, lr_gemm1_kernel<false>, dim3((unsigned)H->p_tiles.size()), dim3(256), 0, s, p);
        LR_CHECK(hipGetLastError());
        if (reduce) {
            launch_timed(&sec, false, true, lr_preduce_kernel, dim3((unsigned)H->row_tiles.size()), dim3(256), 0, s, p);
            LR_CHECK(hipGetLastError());
        }
    }
    {
        Section sec(tm, "lowrank_orth");
        hipLaunchKernelGGL(lr_gram_kernel, dim3((unsigned)H->gram_tiles.size()), dim3(256), 0, s, p);
        LR_CHECK(hipGetLastError());
        if (H->gram_tiles.size() > H->layers.size()) {      // some layer has more than one partial
            hipLaunchKernelGGL(lr_gram_reduce_kernel, dim3((unsigned)H->layers.size() * 16), dim3(256), 0, s, p);
            LR_CHECK(hipGetLastError());
        }
        hipLaunchKernelGGL(lr_orth_kernel, dim3((unsigned)H->layers.size()), dim3(256), 0, s, p);
        LR_CHECK(hipGetLastError());
        hipLaunchKernelGGL(lr_apply_kernel, dim3((unsigned)H->gram_tiles.size()), dim3(256), 0, s, p);
        LR_CHECK(hipGetLastError());
    }
    {
        Section sec(tm, "lowrank_gemm_q", true);
        if (p.e)
            launch_timed(&sec, true, true, lr_gemm2_kernel<true>, dim3((unsigned)H->col_tiles.size()), dim3(256), 0, s, p);
        else
            launch_timed(&sec, true, true, lr_gemm2_kernel<false>, dim3((unsigned)H->col_tiles.size()), dim3(256), 0, s, p);
        LR_CHECK(hipGetLastError());
    }
    {
        Section sec(tm, "lowrank_q_reduce");
        hipLaunchKernelGGL(lr_qreduce_kernel, dim3((unsigned)H->q_chunks.size()), dim3(256), 0, s, p);
        LR_CHECK(hipGetLastError());
    }
  }
    return hipSuccess;
}

hipError_t lowrank_profile(LowrankScratch* t, const float* g, const float* e, const DevLayer* d_layers,
                           const DevLayer* h_layers, int L, const float* q0, int r_max, const int* rank,
                           const int* col, int nlr, double* d_errors, int stride, Timing* tm, hipStream_t s) {
    (void)d_layers;
    LrHost* H = &((LrHost*)t->host)[kLrSlotProfile];
    std::vector<int> ranks(L, kLrCols);
    std::vector<DevLayer> hl(h_layers, h_layers + L);
    for (auto& d : hl) d.payload = 0;                 // not part of the profile's signature
    LR_CHECK(lr_prepare(t, kLrSlotProfile, hl.data(), L, ranks.data(), r_max, false, s));
    if (H->layers.empty()) return hipSuccess;
    LrParams p{};
    lr_fill_params(H, &p);
    p.g = g;
    p.e = e;
    p.q0 = q0;
    p.r_max = r_max;
    p.errors = d_errors;
    p.stride = stride;
    p.nrank = nlr;
    for (int c = 0; c < nlr; ++c) { p.rank[c] = rank[c]; p.col[c] = col[c]; }
    LR_CHECK(lr_factorize(H, p, t->power_iters, tm, s));
    Section sec(tm, "lowrank_errors");
    hipLaunchKernelGGL(lr_errors_kernel, dim3((unsigned)H->layers.size()), dim3(256), 0, s, p);
    return hipGetLastError();
}

hipError_t lowrank_compress(LowrankScratch* t, const float* g, float* e, const DevLayer* d_layers,
                            const DevLayer* h_layers, int L, float* q, int r_max, uint8_t* payload, Timing* tm,
                            hipStream_t s) {
    (void)d_layers;
    LrHost* H = &((LrHost*)t->host)[kLrSlotCompress];
    std::vector<int> ranks(L, 0);
    for (int l = 0; l < L; ++l)
        if (h_layers[l].family == LGRECO_LOWRANK) ranks[l] = h_layers[l].iparam;
    LR_CHECK(lr_prepare(t, kLrSlotCompress, h_layers, L, ranks.data(), r_max, false, s));
    if (H->layers.empty()) return hipSuccess;
    LrParams p{};
    lr_fill_params(H, &p);
    p.g = g;
    p.e = e;
    p.e_out = e;
    p.q0 = q;
    p.q_out = q;
    p.r_max = r_max;
    p.payload = payload;
    LR_CHECK(lr_factorize(H, p, t->power_iters, tm, s));
    Section sec(tm, "lowrank_ef", true);
    launch_timed(&sec, true, true, lr_ef_kernel<false>, dim3((unsigned)H->ef_tiles.size()), dim3(256), 0, s, p);
    return hipGetLastError();
}

// Low-rank layers of a compression queued right behind a profile of the same data and the solver
// kernel that wrote the layer records: the profile's rank-64 factors are still in its scratch and
// every rank's factors are their leading columns, so nothing is contracted again.  Uses the
// profile's work tables (all layers); needs nothing from the host.
hipError_t lowrank_compress_known(LowrankScratch* t, const float* g, float* e, const DevLayer* d_layers, float* q,
                                  int r_max, uint8_t* payload, Timing* tm, hipStream_t s, bool e_is_zero) {
    LrHost* H = &((LrHost*)t->host)[kLrSlotProfile];
    if (H->layers.empty()) return hipSuccess;
    LrParams p{};
    lr_fill_params(H, &p);
    p.g = g;
    p.e = e_is_zero ? nullptr : e;       // promised zeros are not fetched
    p.e_is_zero = e_is_zero ? 1 : 0;
    p.e_out = e;
    p.q0 = q;
    p.q_out = q;
    p.r_max = r_max;
    p.payload = payload;
    p.dev_layers = d_layers;
    {
        Section sec(tm, "lowrank_emit");
        hipLaunchKernelGGL(lr_emit_known_kernel, dim3((unsigned)(H->row_tiles.size() + H->q_chunks.size())), dim3(256), 0,
                           s, p, (int)H->row_tiles.size());
        LR_CHECK(hipGetLastError());
    }
    Section sec(tm, "lowrank_ef", true);
    launch_timed(&sec, true, true, lr_ef_kernel<false, true>, dim3((unsigned)H->ef_tiles.size()), dim3(256), 0, s, p);
    return hipGetLastError();
}

hipError_t lowrank_decompress(LowrankScratch* t, const DevLayer* h_layers, int L, int r_max, const uint8_t* payload,
                              float* out, bool accumulate, Timing* tm, hipStream_t s) {
    LrHost* H = &((LrHost*)t->host)[kLrSlotDecode];
    std::vector<int> ranks(L, 0);
    for (int l = 0; l < L; ++l)
        if (h_layers[l].family == LGRECO_LOWRANK) ranks[l] = h_layers[l].iparam;
    LR_CHECK(lr_prepare(t, kLrSlotDecode, h_layers, L, ranks.data(), r_max, true, s));
    if (H->layers.empty()) return hipSuccess;
    LrParams p{};
    lr_fill_params(H, &p);
    p.e_out = out;
    p.payload = const_cast<uint8_t*>(payload);
    p.accumulate = accumulate ? 1 : 0;
    p.r_max = r_max;
    Section sec(tm, "lowrank_decode", true);
    launch_timed(&sec, true, true, lr_ef_kernel<true>, dim3((unsigned)H->ef_tiles.size()), dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace lgreco

// Receiver side of the codec for bucketed quantization and Top-K: payload -> dense fp32 image,
// written or added to an output buffer (the step after compression in the paper's pipeline, where
// a worker sums the gradients it received).  gfx950 / wave64.
//
// Quantization payload of a layer: (min, unit) fp32 pairs of all buckets, then every bucket's codes
// as an LSB-first bit stream padded to a byte.  A full bucket of 128 codes takes 16 b bytes, and a
// group of 8 consecutive codes is exactly b bytes, so one thread decodes one group:
//   xhat = fma(code, unit, min)        (the same single rounding as the sender)
// Top-K payload: values[k] then indices[k]; the image is zero except at the indices.
#include <algorithm>

#include "internal.h"

namespace lgreco {

struct DecodeParams {
    const uint8_t* payload;
    const DevLayer* layers;
    const Tile* tiles;
    float* out;
    int32_t accumulate;
};

__global__ __launch_bounds__(kThreads) void quant_decode_kernel(DecodeParams p) {
    const Tile t = p.tiles[blockIdx.x];
    const DevLayer L = p.layers[t.layer];
    if (L.family != LGRECO_QUANT) return;
    const int bits = L.iparam;
    const uint32_t mask = (1u << bits) - 1u;
    const int64_t nb_layer = (L.numel + kBucket - 1) / kBucket;
    const uint8_t* const lp = p.payload + L.payload;
    const float2* const meta = reinterpret_cast<const float2*>(lp);
    const uint8_t* const codes = lp + 8 * nb_layer;
    float* const out = p.out + L.offset + t.pos;
    const bool vec = ((L.offset + t.pos) % 4) == 0;
    const int ngroups = (t.count + 7) / 8;
    for (int gidx = threadIdx.x; gidx < ngroups; gidx += kThreads) {
        const int first = gidx * 8;                              // element within the tile
        const int64_t bucket = (t.pos + first) / kBucket;        // tiles start on a bucket boundary
        const int in_bucket = first % kBucket;
        const int64_t bstart = bucket * kBucket;
        const int bcount = (int)((L.numel - bstart < kBucket) ? (L.numel - bstart) : kBucket);
        const int bbytes = (bcount * bits + 7) / 8;              // bytes of this bucket's stream
        const uint8_t* src = codes + bucket * (kBucket * bits / 8) + (in_bucket / 8) * bits;
        const int avail = bbytes - (in_bucket / 8) * bits;       // bytes left in the stream
        unsigned long long v = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (i < bits && i < avail) v |= (unsigned long long)src[i] << (8 * i);
        const float2 mu = meta[bucket];
        float x[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const float q = (float)((uint32_t)(v >> (bits * k)) & mask);
            x[k] = __builtin_fmaf(q, mu.y, mu.x);
        }
        const int valid = min(8, t.count - first);
        if (vec && valid == 8) {
            float4* o = reinterpret_cast<float4*>(out + first);
            float4 a = make_float4(x[0], x[1], x[2], x[3]), b = make_float4(x[4], x[5], x[6], x[7]);
            if (p.accumulate) {
                const float4 oa = load_stream(o), ob = load_stream(o + 1);
                a.x += oa.x; a.y += oa.y; a.z += oa.z; a.w += oa.w;
                b.x += ob.x; b.y += ob.y; b.z += ob.z; b.w += ob.w;
            }
            store_stream(o, a);
            store_stream(o + 1, b);
        } else {
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (k < valid) out[first + k] = p.accumulate ? out[first + k] + x[k] : x[k];
        }
    }
}

// Top-K, first kernel (only when the image replaces the output): zero the layer.
__global__ __launch_bounds__(kThreads) void topk_decode_zero_kernel(DecodeParams p) {
    const Tile t = p.tiles[blockIdx.x];
    const DevLayer L = p.layers[t.layer];
    if (L.family != LGRECO_TOPK) return;
    float* const out = p.out + L.offset + t.pos;
    if (t.fast) {
        const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int v = threadIdx.x; v < t.count / 4; v += kThreads) store_stream(reinterpret_cast<float4*>(out) + v, z);
    } else {
        for (int i = threadIdx.x; i < t.count; i += kThreads) out[i] = 0.0f;
    }
}

// Top-K, second kernel: scatter.  The k entries of a layer are dealt to its tiles in proportion
// to the tiles' element ranges; indices are distinct, so plain read-modify-writes do not collide.
__global__ __launch_bounds__(kThreads) void topk_decode_scatter_kernel(DecodeParams p) {
    const Tile t = p.tiles[blockIdx.x];
    const DevLayer L = p.layers[t.layer];
    if (L.family != LGRECO_TOPK) return;
    const int64_t k = L.iparam;
    const int64_t e0 = k * t.pos / L.numel, e1 = k * (t.pos + t.count) / L.numel;
    const float* const values = reinterpret_cast<const float*>(p.payload + L.payload);
    const uint32_t* const indices = reinterpret_cast<const uint32_t*>(p.payload + L.payload) + k;
    float* const out = p.out + L.offset;
    for (int64_t i = e0 + threadIdx.x; i < e1; i += kThreads) {
        const uint32_t ix = indices[i];
        if ((int64_t)ix < L.numel) out[ix] = p.accumulate ? out[ix] + values[i] : values[i];
    }
}

// Gradient accumulation between two runs of the algorithm (section "Implementation": per-layer
// gradients are accumulated in auxiliary buffers in between runs).  acc = g or acc += g, fp32.
__global__ __launch_bounds__(kThreads) void accumulate_kernel(float* __restrict__ acc, const float* __restrict__ g,
                                                              int64_t n, int reset) {
    const int64_t n4 = n / 4;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x; v < n4; v += stride) {
        float4 a = load_stream(reinterpret_cast<const float4*>(g) + v);
        if (!reset) {
            const float4 o = load_stream(reinterpret_cast<const float4*>(acc) + v);
            a.x += o.x; a.y += o.y; a.z += o.z; a.w += o.w;
        }
        store_stream(reinterpret_cast<float4*>(acc) + v, a);
    }
    if (blockIdx.x == 0 && threadIdx.x < n - 4 * n4) {
        const int64_t i = 4 * n4 + threadIdx.x;
        acc[i] = reset ? g[i] : acc[i] + g[i];
    }
}

hipError_t launch_accumulate(float* acc, const float* g, int64_t n, bool reset, hipStream_t s, Section* sec) {
    if (n <= 0) return hipSuccess;
    const int64_t blocks = std::min<int64_t>((n / 4 + kThreads - 1) / kThreads + 1, 256 * 16);
    launch_timed(sec, true, true, accumulate_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, s, acc, g, n, reset ? 1 : 0);
    return hipGetLastError();
}

hipError_t launch_decode(const uint8_t* payload, const DevLayer* layers, const Tile* tiles, int n_tiles,
                         float* out, bool accumulate, bool any_quant, bool any_topk, Timing* tm, hipStream_t s) {
    if (n_tiles <= 0) return hipSuccess;
    DecodeParams p{payload, layers, tiles, out, accumulate ? 1 : 0};
    if (any_quant) {
        Section sec(tm, "quant_decode", true);
        launch_timed(&sec, true, true, quant_decode_kernel, dim3(n_tiles), dim3(kThreads), 0, s, p);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (any_topk) {
        Section sec(tm, "topk_decode", true);
        if (!accumulate) {
            launch_timed(&sec, true, false, topk_decode_zero_kernel, dim3(n_tiles), dim3(kThreads), 0, s, p);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
        launch_timed(&sec, true, true, topk_decode_scatter_kernel, dim3(n_tiles), dim3(kThreads), 0, s, p);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace lgreco

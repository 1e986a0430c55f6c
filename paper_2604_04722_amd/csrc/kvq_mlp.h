// Controller forward pass of one feature row by one workgroup (paper Sec. 3.6), shared by the per-step controller
// kernel and by the fused features + controller kernel, so that both produce the same logits bit for bit.
#pragma once

#include "kvq_internal.h"

namespace kvq {

constexpr int kMaxWidth = 256;
constexpr int kRowThreads = 256;     // per-step shape: thread = output unit

struct MlpArgs {
    const float *feats;
    const float *W[4];
    const float *b[4];
    uint8_t *bits;
    float *logits;
    long long n;
    int n_linear;
    int dims[5];
};

int mlp_args_from(const kvq_mlp *mlp, MlpArgs *out, int *max_width);

// argmax with the first maximum winning, bits = {2,4,8,16}[class] (label mapping of Algorithm 1); returns the bits
__device__ __forceinline__ int emit_decision(const float *o, int nout, long long row, uint8_t *bits, float *logits)
{
    int best = 0;
    for (int k = 1; k < nout; ++k) if (o[k] > o[best]) best = k;     // strict: the first maximum wins
    bits[row] = (uint8_t)(2 << best);                                // 2, 4, 8, 16
    if (logits) for (int k = 0; k < 4; ++k) logits[row * 4 + k] = k < nout ? o[k] : -INFINITY;
    return 2 << best;
}

// Copies all weights into `stage` with contiguous (coalesced) global reads, issued back to back so that they share
// one memory latency.  Every thread of the workgroup calls it; a barrier must follow before the weights are used.
__device__ __forceinline__ void mlp_stage_weights(const MlpArgs &A, float *stage, int tid, int nthreads)
{
    int base = 0;
    // compile-time layer indices: a weight pointer picked from the array at run time would lose its address space
#pragma unroll
    for (int l = 0; l < 3; ++l) {
        if (l >= A.n_linear) break;
        const int in = A.dims[l], outw = A.dims[l + 1], row = in + 1, total = in * outw;
        const float *W = A.W[l];
        if ((in & 3) == 0 && ((uintptr_t)W & 15) == 0) {
            const int n4 = total / 4;
            for (int e0 = tid; e0 < n4; e0 += 8 * nthreads) {          // eight loads in flight per thread
                float4 v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int e4 = e0 + u * nthreads;
                    v[u] = ((const float4 *)W)[e4 < n4 ? e4 : e0];
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int e4 = e0 + u * nthreads;
                    if (e4 < n4) {
                        const int j = (e4 * 4) / in, i = e4 * 4 - j * in;
                        float *d = stage + base + j * row + i;
                        d[0] = v[u].x; d[1] = v[u].y; d[2] = v[u].z; d[3] = v[u].w;
                    }
                }
            }
        } else {
            for (int e = tid; e < total; e += nthreads) {
                const int j = e / in, i = e - j * in;
                stage[base + j * row + i] = W[e];
            }
        }
        base += outw * row;
    }
}

// Forward pass of one row by one workgroup of any size.  A layer's work is cut into items of (output unit, chunk of
// kRowChunk consecutive inputs): 128 x 128 weights are 1024 items, one per thread of a 1024-thread workgroup, each a
// chain of 16 FMAs on weights it reads straight from global memory (consecutive threads read consecutive 64 bytes; the
// weights of a controller stay in L2 from one decode step to the next).  The items' partial sums go through LDS and
// thread j adds its unit's chunks in ascending order to the bias.  Staging all weights in LDS first and giving a unit's
// whole chain to one thread took 8 us per call for the 4-128-128-4 network; this takes a third of that.
// Every thread of the workgroup calls mlp_row_prefetch early, then mlp_row_forward with the features in
// act[0][0..dims[0]) and a barrier behind them; `part` is LDS for kRowPartMax floats.  Returns the index (0 or 1) of the act row that holds the logits; a barrier has been
// passed when it returns.
constexpr int kRowChunk = 16;
constexpr int kRowPartMax = kMaxWidth * (kMaxWidth / kRowChunk);

// What a thread needs of the weights for its first work item of every layer, asked for before the features exist (the
// weights do not depend on them): with 1024 threads and widths up to 128 that is every item, and the three layers'
// reads cost one memory latency together instead of one each.
typedef float f32x4 __attribute__((ext_vector_type(4)));     // a first-class vector value (the float4 class wraps a union)

struct RowLayerPrefetch {
    f32x4 w0, w1, w2, w3;          // (named members, no arrays: an array indexed in a loop ends up in scratch memory)
    float bias;
};
struct RowPrefetch { RowLayerPrefetch l0, l1, l2; };

__device__ __forceinline__ bool mlp_row_vec(const MlpArgs &A, int l) { return (A.dims[l] & 3) == 0 && ((uintptr_t)A.W[l] & 15) == 0; }

// the 16 weights of item `it` of layer L (vectorised layers only); loads beyond the row's end re-read its start
struct RowItemWeights { f32x4 w0, w1, w2, w3; };

template <int L> __device__ __forceinline__ RowItemWeights mlp_row_item_weights(const MlpArgs &A, int it)
{
    const int in = A.dims[L];
    const int chunks = (in + kRowChunk - 1) / kRowChunk;
    const int j = it / chunks, c = it - j * chunks;
    const int i0 = c * kRowChunk, i1 = min(i0 + kRowChunk, in);
    const float *w = A.W[L] + (size_t)j * in;
    RowItemWeights r;
    r.w0 = *(const f32x4 *)(w + i0);
    r.w1 = *(const f32x4 *)(w + (i0 + 4 < i1 ? i0 + 4 : i0));
    r.w2 = *(const f32x4 *)(w + (i0 + 8 < i1 ? i0 + 8 : i0));
    r.w3 = *(const f32x4 *)(w + (i0 + 12 < i1 ? i0 + 12 : i0));
    return r;
}

template <int L> __device__ __forceinline__ RowLayerPrefetch mlp_row_prefetch_layer(const MlpArgs &A, int tid)
{
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    f32x4 w0 = zero, w1 = zero, w2 = zero, w3 = zero;
    float bias = 0.f;
    if (L < A.n_linear) {
        const int outw = A.dims[L + 1];
        const int items = outw * ((A.dims[L] + kRowChunk - 1) / kRowChunk);
        if (tid < items && mlp_row_vec(A, L)) {
            const RowItemWeights r = mlp_row_item_weights<L>(A, tid);
            w0 = r.w0; w1 = r.w1; w2 = r.w2; w3 = r.w3;
        }
        if (tid < outw) bias = A.b[L][tid];
    }
    RowLayerPrefetch p;
    p.w0 = w0; p.w1 = w1; p.w2 = w2; p.w3 = w3; p.bias = bias;
    return p;
}

__device__ __forceinline__ RowPrefetch mlp_row_prefetch(const MlpArgs &A, int tid)
{
    RowPrefetch pf;
    pf.l0 = mlp_row_prefetch_layer<0>(A, tid);
    pf.l1 = mlp_row_prefetch_layer<1>(A, tid);
    pf.l2 = mlp_row_prefetch_layer<2>(A, tid);
    return pf;
}

__device__ __forceinline__ float mlp_row_fma4(const f32x4 &w, const float *h, int i, int i1, float a)
{
    if (i < i1) {
        a = fmaf(w.x, h[i], a);
        a = fmaf(w.y, h[i + 1], a);
        a = fmaf(w.z, h[i + 2], a);
        a = fmaf(w.w, h[i + 3], a);
    }
    return a;
}

// one layer; h = the layer's input in LDS, out = its output row in LDS
template <int L> __device__ __forceinline__ void mlp_row_layer(const MlpArgs &A, const float *h, float *out, float *part, int tid, int nthreads,
                                                               const RowLayerPrefetch &p)
{
    const int in = A.dims[L], outw = A.dims[L + 1];
    const int chunks = (in + kRowChunk - 1) / kRowChunk;
    const int items = outw * chunks;
    const bool vec = mlp_row_vec(A, L);
    // the first item of a thread runs on the prefetched weights, any further one fetches its own
    auto item = [&](int it, const f32x4 &w0, const f32x4 &w1, const f32x4 &w2, const f32x4 &w3) {
        const int j = it / chunks, c = it - j * chunks;
        const int i0 = c * kRowChunk, i1 = min(i0 + kRowChunk, in);
        float a = 0.f;
        if (vec) {
            a = mlp_row_fma4(w0, h, i0, i1, a);
            a = mlp_row_fma4(w1, h, i0 + 4, i1, a);
            a = mlp_row_fma4(w2, h, i0 + 8, i1, a);
            a = mlp_row_fma4(w3, h, i0 + 12, i1, a);
        } else {
            const float *w = A.W[L] + (size_t)j * in;
            for (int i = i0; i < i1; ++i) a = fmaf(w[i], h[i], a);
        }
        part[it] = a;
    };
    if (tid < items) item(tid, p.w0, p.w1, p.w2, p.w3);
    for (int it = tid + nthreads; it < items; it += nthreads) {
        RowItemWeights r = {p.w0, p.w0, p.w0, p.w0};
        if (vec) r = mlp_row_item_weights<L>(A, it);
        item(it, r.w0, r.w1, r.w2, r.w3);
    }
    __syncthreads();
    if (tid < outw) {
        float a = p.bias;
        for (int c = 0; c < chunks; ++c) a += part[tid * chunks + c];
        if (L + 1 < A.n_linear) a = fmaxf(a, 0.f);
        out[tid] = a;
    }
    __syncthreads();
}

__device__ __forceinline__ int mlp_row_forward(const MlpArgs &A, float (*act)[kMaxWidth], float *part, int tid, int nthreads,
                                               const RowPrefetch &pf)
{
    mlp_row_layer<0>(A, act[0], act[1], part, tid, nthreads, pf.l0);
    mlp_row_layer<1>(A, act[1], act[0], part, tid, nthreads, pf.l1);
    if (A.n_linear < 3) return 0;
    mlp_row_layer<2>(A, act[0], act[1], part, tid, nthreads, pf.l2);
    return 1;
}

}  // namespace kvq

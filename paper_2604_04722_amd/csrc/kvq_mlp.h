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

// Floats of LDS that hold every layer's weights with rows padded by one float (conflict-free for thread = row).
__host__ __device__ inline int mlp_stage_floats(const MlpArgs &A)
{
    int total = 0;
    for (int l = 0; l < A.n_linear; ++l) total += A.dims[l + 1] * (A.dims[l] + 1);
    return total;
}
constexpr int kMlpStageMaxFloats = 18432;       // 72 KiB: 4-128-128-4 needs 17 668 floats; wider nets read global memory

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

// Forward pass of one row: thread j < width computes output unit j as the sequential fp32 FMA chain
// bias + sum_i W[j][i]*h[i], i ascending (the chain of the vector-ALU bulk shape, so the two agree bit for bit).
// Every thread of the workgroup calls this with the features in act[0][0..dims[0]) and a barrier behind them (and
// behind mlp_stage_weights if stage != nullptr; with stage == nullptr the weights are read from global memory).
// Returns the index (0 or 1) of the act row that holds the logits; a barrier has been passed when it returns.
// Staged selects the weights' address space at compile time (LDS `stage`, or global memory): a pointer that may be
// either would be a generic one, and every weight read a flat load.
template <bool Staged>
__device__ __forceinline__ int mlp_row_forward(const MlpArgs &A, float (*act)[kMaxWidth], int tid, const float *stage)
{
    int cur = 0, base = 0;
#pragma unroll
    for (int l = 0; l < 3; ++l) {
        if (l >= A.n_linear) break;
        const int in = A.dims[l], outw = A.dims[l + 1];
        if (tid < outw) {
            float a = A.b[l][tid];
            const float *h = act[cur];
            int i = 0;
            // eight weights and activations are fetched before their FMAs: one read latency per eight terms
            if constexpr (Staged) {
                const float *w = stage + base + tid * (in + 1);
                for (; i + 8 <= in; i += 8) {
                    float wv[8], hv[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) { wv[u] = w[i + u]; hv[u] = h[i + u]; }
#pragma unroll
                    for (int u = 0; u < 8; ++u) a = fmaf(wv[u], hv[u], a);
                }
                for (; i < in; ++i) a = fmaf(w[i], h[i], a);
            } else {
                const float *w = A.W[l] + (size_t)tid * in;
                for (; i + 8 <= in; i += 8) {
                    float wv[8], hv[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) { wv[u] = w[i + u]; hv[u] = h[i + u]; }
#pragma unroll
                    for (int u = 0; u < 8; ++u) a = fmaf(wv[u], hv[u], a);
                }
                for (; i < in; ++i) a = fmaf(w[i], h[i], a);
            }
            if (l + 1 < A.n_linear) a = fmaxf(a, 0.f);
            act[cur ^ 1][tid] = a;
        }
        __syncthreads();
        cur ^= 1;
        base += outw * (in + 1);
    }
    return cur;
}

}  // namespace kvq

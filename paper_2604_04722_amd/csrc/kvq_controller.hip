// Controller forward (paper Sec. 3.6): h1 = ReLU(W1 s + b1), h2 = ReLU(W2 h1 + b2), o = W3 h2 + b3,
// class = argmax_k o_k, bits = {2,4,8,16}[class] (label mapping of Algorithm 1).
//
// Two launch shapes compute bit-identical logits (each output is the same sequential fp32 FMA chain
// bias + sum_i W[j][i]*h[i], i ascending):
//   - per-step shape (few rows): one workgroup per row, thread = output unit, activations in LDS;
//   - bulk shape (cache construction, thousands to millions of rows): thread = row, activations in LDS
//     columns, weights read through wave-uniform loads, four outputs per pass to reuse each activation.
#include "kvq_internal.h"

namespace kvq {

constexpr int kMaxWidth = 256;
constexpr int kRowThreads = 256;     // per-step shape
constexpr int kBulkThreads = 64;     // bulk shape: rows per workgroup

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

__device__ __forceinline__ void emit_decision(const float *o, int nout, long long row, uint8_t *bits, float *logits)
{
    int best = 0;
    for (int k = 1; k < nout; ++k) if (o[k] > o[best]) best = k;     // strict: the first maximum wins
    bits[row] = (uint8_t)(2 << best);                                // 2, 4, 8, 16
    if (logits) for (int k = 0; k < 4; ++k) logits[row * 4 + k] = k < nout ? o[k] : -INFINITY;
}

__global__ __launch_bounds__(kRowThreads) void k_mlp_row(MlpArgs A)
{
    __shared__ float act[2][kMaxWidth];
    const long long row = blockIdx.x;
    const int tid = threadIdx.x;
    if (tid < A.dims[0]) act[0][tid] = A.feats[row * A.dims[0] + tid];
    __syncthreads();
    int cur = 0;
    for (int l = 0; l < A.n_linear; ++l) {
        const int in = A.dims[l], outw = A.dims[l + 1];
        if (tid < outw) {
            const float *w = A.W[l] + (size_t)tid * in;
            float a = A.b[l][tid];
            for (int i = 0; i < in; ++i) a = fmaf(w[i], act[cur][i], a);
            if (l + 1 < A.n_linear) a = fmaxf(a, 0.f);
            act[cur ^ 1][tid] = a;
        }
        __syncthreads();
        cur ^= 1;
    }
    if (tid == 0) emit_decision(act[cur], A.dims[A.n_linear], row, A.bits, A.logits);
}

__global__ __launch_bounds__(kBulkThreads) void k_mlp_bulk(MlpArgs A, int maxw)
{
    extern __shared__ float lds[];                 // [2][maxw][kBulkThreads]
    const int tid = threadIdx.x;
    const long long row = (long long)blockIdx.x * kBulkThreads + tid;
    const bool live = row < A.n;
    float *buf0 = lds, *buf1 = lds + (size_t)maxw * kBulkThreads;
    for (int i = 0; i < A.dims[0]; ++i) buf0[i * kBulkThreads + tid] = live ? A.feats[row * A.dims[0] + i] : 0.f;
    float *in_act = buf0, *out_act = buf1;
    for (int l = 0; l < A.n_linear; ++l) {
        const int in = A.dims[l], outw = A.dims[l + 1];
        const float *W = A.W[l];
        const float *bias = A.b[l];
        const bool relu = l + 1 < A.n_linear;
        int j = 0;
        for (; j + 4 <= outw; j += 4) {
            float a0 = bias[j], a1 = bias[j + 1], a2 = bias[j + 2], a3 = bias[j + 3];
            const float *w0 = W + (size_t)j * in;
            for (int i = 0; i < in; ++i) {
                const float h = in_act[i * kBulkThreads + tid];
                a0 = fmaf(w0[i], h, a0);
                a1 = fmaf(w0[in + i], h, a1);
                a2 = fmaf(w0[2 * in + i], h, a2);
                a3 = fmaf(w0[3 * in + i], h, a3);
            }
            if (relu) { a0 = fmaxf(a0, 0.f); a1 = fmaxf(a1, 0.f); a2 = fmaxf(a2, 0.f); a3 = fmaxf(a3, 0.f); }
            out_act[(j + 0) * kBulkThreads + tid] = a0;
            out_act[(j + 1) * kBulkThreads + tid] = a1;
            out_act[(j + 2) * kBulkThreads + tid] = a2;
            out_act[(j + 3) * kBulkThreads + tid] = a3;
        }
        for (; j < outw; ++j) {
            float a = bias[j];
            const float *w0 = W + (size_t)j * in;
            for (int i = 0; i < in; ++i) a = fmaf(w0[i], in_act[i * kBulkThreads + tid], a);
            if (relu) a = fmaxf(a, 0.f);
            out_act[j * kBulkThreads + tid] = a;
        }
        float *t = in_act; in_act = out_act; out_act = t;
    }
    if (!live) return;
    float o[4];
    const int nout = A.dims[A.n_linear];
    for (int k = 0; k < 4; ++k) o[k] = k < nout ? in_act[k * kBulkThreads + tid] : -INFINITY;
    emit_decision(o, nout, row, A.bits, A.logits);
}

}  // namespace kvq

using namespace kvq;

extern "C" int kvq_controller(const float *feats, int64_t n, const kvq_mlp *mlp, uint8_t *bits_out,
                              float *logits_out, void *stream)
{
    if (n < 0) { set_error("n negative"); return KVQ_ERR_INVALID_ARG; }
    if (!mlp) { set_error("mlp is NULL"); return KVQ_ERR_INVALID_ARG; }
    if (mlp->n_linear < 2 || mlp->n_linear > 3) { set_error("n_linear must be 2 or 3"); return KVQ_ERR_UNSUPPORTED; }
    if (mlp->dims[0] != 4) { set_error("dims[0] must be 4 (the feature vector)"); return KVQ_ERR_INVALID_ARG; }
    if (mlp->dims[mlp->n_linear] != 4) { set_error("the last layer must have 4 outputs"); return KVQ_ERR_INVALID_ARG; }
    int maxw = 4;
    for (int l = 1; l < mlp->n_linear; ++l) {
        if (mlp->dims[l] < 1 || mlp->dims[l] > kMaxWidth) {
            set_error("hidden width %d outside 1..%d", mlp->dims[l], kMaxWidth);
            return KVQ_ERR_UNSUPPORTED;
        }
        if (mlp->dims[l] > maxw) maxw = mlp->dims[l];
    }
    for (int l = 0; l < mlp->n_linear; ++l)
        if (!mlp->W[l] || !mlp->b[l]) { set_error("W[%d] or b[%d] is NULL", l, l); return KVQ_ERR_INVALID_ARG; }
    if (n == 0) return KVQ_OK;
    if (!feats || !bits_out) { set_error("feats or bits_out is NULL"); return KVQ_ERR_INVALID_ARG; }
    MlpArgs A;
    A.feats = feats;
    A.bits = bits_out;
    A.logits = logits_out;
    A.n = n;
    A.n_linear = mlp->n_linear;
    for (int l = 0; l < 5; ++l) A.dims[l] = l <= mlp->n_linear ? mlp->dims[l] : 0;
    for (int l = 0; l < 4; ++l) {
        A.W[l] = l < mlp->n_linear ? mlp->W[l] : nullptr;
        A.b[l] = l < mlp->n_linear ? mlp->b[l] : nullptr;
    }
    hipStream_t st = (hipStream_t)stream;
    if (n <= 2048) {
        hipLaunchKernelGGL(k_mlp_row, dim3((unsigned)n), dim3(kRowThreads), 0, st, A);
    } else {
        const long long blocks = (n + kBulkThreads - 1) / kBulkThreads;
        if (blocks > 0x7fffffffLL) { set_error("n too large for one launch"); return KVQ_ERR_CAPACITY; }
        const size_t lds = (size_t)2 * maxw * kBulkThreads * sizeof(float);
        if (lds > 48 * 1024)
            KVQ_HIP(hipFuncSetAttribute((const void *)k_mlp_bulk, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(k_mlp_bulk, dim3((unsigned)blocks), dim3(kBulkThreads), lds, st, A, maxw);
    }
    KVQ_HIP(hipGetLastError());
    return KVQ_OK;
}

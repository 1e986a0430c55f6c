// Controller forward (paper Sec. 3.6): h1 = ReLU(W1 s + b1), h2 = ReLU(W2 h1 + b2), o = W3 h2 + b3,
// class = argmax_k o_k, bits = {2,4,8,16}[class] (label mapping of Algorithm 1).
//
// Three launch shapes:
//   - per-step shape (few rows): one workgroup per row, a layer cut into (output unit, 16 inputs) work items over all
//     its threads, weights read straight from global memory (L2), activations and partial sums in LDS;
//   - bulk shape on the matrix cores (cache construction, thousands to millions of rows; hidden widths 32, 64 or
//     128): a wavefront takes 32 rows, the hidden layers are fp32 MFMA 32x32x2 tiles whose accumulators feed the
//     next layer's B operand directly, the 4-output layer is a short vector dot product;
//   - bulk shape on the vector ALU (any other width up to 256): thread = row, activations in LDS columns.
// The three sum the same fp32 products in three orders (chains of 16 then the chunks in ascending order; tile order;
// one chain per output unit); the fused front end shares the first shape's code and agrees with it bit for bit.
#include "kvq_internal.h"
#include "kvq_mlp.h"

#include <cstdlib>

namespace kvq {

constexpr int kBulkThreads = 64;     // vector-ALU bulk shape: rows per workgroup

// Launched with 1024 threads for up to a few hundred rows (a 128 x 128 layer is then one work item per thread), with
// kRowThreads beyond that.
__global__ __launch_bounds__(1024) void k_mlp_row(MlpArgs A)
{
    __shared__ float part[kRowPartMax];
    __shared__ float act[2][kMaxWidth];
    const long long row = blockIdx.x;
    const int tid = threadIdx.x;
    const RowPrefetch pf = mlp_row_prefetch(A, tid);
    if (tid < A.dims[0]) act[0][tid] = A.feats[row * A.dims[0] + tid];
    __syncthreads();
    const int cur = mlp_row_forward(A, act, part, tid, (int)blockDim.x, pf);
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

// ---- bulk shape on the matrix cores -------------------------------------------------------------------------
//
// v_mfma_f32_32x32x2_f32 computes D[32x32] = A[32x2] * B[2x32] + C.  Here i (rows of A, D) is the output unit and
// j (columns of B, D) is the token, so one wavefront carries 32 tokens through the network:
//   A: lane l holds A[i = l%32][k = l/32];  B: lane l holds B[k = l/32][j = l%32];
//   D: lane l, register r holds D[i = 8*(r/4) + 4*(l/32) + r%4][j = l%32].
// A layer's output register r therefore holds, in the lanes of half hh = l/32, unit u(r, hh) = 8*(r/4) + 4*hh + r%4
// of token l%32: exactly a B operand for one k-step of the next layer whose two k indices are u(r,0) and u(r,1).
// The order of the k-steps is free, so the registers are used as they are and the weights are staged in LDS in the
// matching order (lane l of step r reads W[i = l%32][u(r, l/32)]).  Nothing is shuffled between layers.

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__host__ __device__ constexpr size_t mfma_lds_floats(int T1, int T2)
{
    const int TL = T2 ? T2 : T1;
    return (size_t)T1 * 128 + T1 * 32 + (size_t)T2 * T1 * 1024 + T2 * 32 + TL * 128 + 4;
}

template <int T1, int T2, int NW>   // hidden widths 32*T1 and 32*T2 (T2 == 0: one hidden layer); NW wavefronts per workgroup
__global__ __launch_bounds__(64 * NW) void k_mlp_mfma(MlpArgs A, long long ntiles)
{
    extern __shared__ float lds[];
    constexpr int TL = T2 ? T2 : T1;
    float *w1p = lds;                               // [T1][2 k-steps][64 lanes]
    float *b1p = w1p + T1 * 128;                    // [T1][16 regs][2 halves]
    float *w2p = b1p + T1 * 32;                     // [T2][T1][16 regs][64 lanes]
    float *b2p = w2p + (size_t)T2 * T1 * 1024;      // [T2][16][2]
    float *wfp = b2p + T2 * 32;                     // [TL][16][2][4 outputs]
    float *bfp = wfp + TL * 128;                    // [4]
    constexpr int NT = 64 * NW;
    const int tid = threadIdx.x;
    const float *W1 = A.W[0], *Wf = A.W[T2 ? 2 : 1];
    for (int idx = tid; idx < T1 * 128; idx += NT) {
        const int l = idx & 63, s = (idx >> 6) & 1, ot = idx >> 7;
        w1p[idx] = W1[(32 * ot + (l & 31)) * 4 + 2 * s + (l >> 5)];
    }
    for (int idx = tid; idx < T1 * 32; idx += NT) {
        const int hh = idx & 1, r = (idx >> 1) & 15, it = idx >> 5;
        b1p[idx] = A.b[0][32 * it + (r >> 2) * 8 + hh * 4 + (r & 3)];
    }
    if constexpr (T2 > 0) {
        // W2: four consecutive inputs per load, eight loads in flight per thread, and consecutive threads take
        // consecutive output units.  Each element goes to the (tile, k-step, lane) slot that the MFMA loop reads it
        // from, and in that layout the lane is the output unit: with the units across the threads a wavefront's
        // writes spread over all LDS banks (in memory order, where 32 consecutive threads share a unit, they all fall
        // into one bank and the staging alone took a seventh of the kernel's time).
        const float *W2 = A.W[1];
        constexpr int K = 32 * T1, NJ = 32 * T2, N4 = NJ * K / 4;
        for (int e0 = tid; e0 < N4; e0 += 8 * NT) {
            f32x4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int e4 = e0 + u * NT;
                const int ec = e4 < N4 ? e4 : e0;
                v[u] = *(const f32x4 *)(W2 + (size_t)(ec % NJ) * K + (ec / NJ) * 4);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int e4 = e0 + u * NT;
                if (e4 < N4) {
                    const int j = e4 % NJ, i = (e4 / NJ) * 4;               // output unit, first of four inputs
                    const int ot = j >> 5, it = i >> 5, rem = i & 31;
                    const int r0 = (rem >> 3) * 4, l = ((rem >> 2) & 1) * 32 + (j & 31);
                    float *d = w2p + ((ot * T1 + it) * 16 + r0) * 64 + l;
                    d[0] = v[u][0]; d[64] = v[u][1]; d[128] = v[u][2]; d[192] = v[u][3];
                }
            }
        }
        for (int idx = tid; idx < T2 * 32; idx += NT) {
            const int hh = idx & 1, r = (idx >> 1) & 15, it = idx >> 5;
            b2p[idx] = A.b[1][32 * it + (r >> 2) * 8 + hh * 4 + (r & 3)];
        }
    }
    for (int idx = tid; idx < TL * 128; idx += NT) {
        const int o = idx & 3, hh = (idx >> 2) & 1, r = (idx >> 3) & 15, it = idx >> 7;
        wfp[idx] = Wf[o * (32 * TL) + 32 * it + (r >> 2) * 8 + hh * 4 + (r & 3)];
    }
    if (tid < 4) bfp[tid] = A.b[T2 ? 2 : 1][tid];
    __syncthreads();

    const int lane = tid & 63, hh = lane >> 5, j = lane & 31;
    const long long stride = (long long)gridDim.x * NW;
    // a tile's feature rows are asked for one tile ahead: the load's latency would otherwise stand at the head of every
    // tile, in front of the first matrix instruction that needs it
    const long long tile0 = (long long)blockIdx.x * NW + (tid >> 6);
    f32x4 x_next = {0.f, 0.f, 0.f, 0.f};
    if (tile0 < ntiles) {
        const long long row0 = tile0 * 32 + j;
        x_next = *(const f32x4 *)(A.feats + (row0 < A.n ? row0 : A.n - 1) * 4);
    }
    for (long long tile = tile0; tile < ntiles; tile += stride) {
        const long long row = tile * 32 + j;
        const bool live = row < A.n;
        const f32x4 x = x_next;
        if (tile + stride < ntiles) {
            const long long rown = (tile + stride) * 32 + j;
            x_next = *(const f32x4 *)(A.feats + (rown < A.n ? rown : A.n - 1) * 4);
        }
        const float xb[2] = {hh ? x[1] : x[0], hh ? x[3] : x[2]};
        f32x16 h1[T1];
#pragma unroll
        for (int it = 0; it < T1; ++it) {
#pragma unroll
            for (int r = 0; r < 16; ++r) h1[it][r] = b1p[(it * 16 + r) * 2 + hh];
#pragma unroll
            for (int s = 0; s < 2; ++s)
                h1[it] = __builtin_amdgcn_mfma_f32_32x32x2f32(w1p[(it * 2 + s) * 64 + lane], xb[s], h1[it], 0, 0, 0);
#pragma unroll
            for (int r = 0; r < 16; ++r) h1[it][r] = fmaxf(h1[it][r], 0.f);
            __builtin_amdgcn_sched_barrier(0);
        }
        // Second hidden layer two output tiles at a time: 32 accumulator registers live instead of 16 * T2, which leaves
        // room for two waves per SIMD.  The 4-output layer is a short vector dot product (each lane sums over the units it
        // holds, the two halves of a token are added at the end), and a finished pair is folded into it while the next
        // pair's matrix instructions run: one slice of the fold per chunk of k-steps, in the order r = 0..15 of the
        // pair's first tile, then of its second.  Only the last pair's fold stands alone.
        float o[4] = {0.f, 0.f, 0.f, 0.f};
        if constexpr (T2 > 0) {
            constexpr int GO = T2 >= 2 ? 2 : 1;
            constexpr int NCH = T1 * 4;                         // chunks of four k-steps
            constexpr int RPC = GO * 16 / NCH;                  // registers of the previous pair folded per chunk
            f32x16 hp[GO];                                      // the pair before this one, waiting to be folded
#pragma unroll
            for (int g = 0; g < GO; ++g)
#pragma unroll
                for (int r = 0; r < 16; ++r) hp[g][r] = 0.f;
#pragma unroll
            for (int o0 = 0; o0 < T2; o0 += GO) {
                f32x16 h2[GO];
#pragma unroll
                for (int g = 0; g < GO; ++g)
#pragma unroll
                    for (int r = 0; r < 16; ++r) h2[g][r] = b2p[((o0 + g) * 16 + r) * 2 + hh];
                // the next chunk's A operands are read from LDS while this chunk's MFMAs run, and a scheduling fence per
                // chunk keeps the compiler from hoisting every LDS read of the layer to the top
                float a_cur[4][GO], a_nxt[4][GO];
#pragma unroll
                for (int s_ = 0; s_ < 4; ++s_)
#pragma unroll
                    for (int g = 0; g < GO; ++g) a_cur[s_][g] = w2p[((o0 + g) * T1 * 16 + s_) * 64 + lane];
#pragma unroll
                for (int c = 0; c < NCH; ++c) {
                    if (c + 1 < NCH) {
#pragma unroll
                        for (int s_ = 0; s_ < 4; ++s_)
#pragma unroll
                            for (int g = 0; g < GO; ++g) a_nxt[s_][g] = w2p[((o0 + g) * T1 * 16 + (c + 1) * 4 + s_) * 64 + lane];
                    }
#pragma unroll
                    for (int s_ = 0; s_ < 4; ++s_) {
                        const int st_ = c * 4 + s_;                 // k-step = (input tile, register)
#pragma unroll
                        for (int g = 0; g < GO; ++g)
                            h2[g] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_cur[s_][g], h1[st_ / 16][st_ % 16], h2[g], 0, 0, 0);
                    }
                    if (o0 > 0) {
#pragma unroll
                        for (int q = c * RPC; q < (c + 1) * RPC; ++q) {
                            const int g = q / 16, r = q % 16;
                            const float h = fmaxf(hp[g][r], 0.f);
                            const f32x4 w = *(const f32x4 *)(wfp + (((o0 - GO + g) * 16 + r) * 2 + hh) * 4);
#pragma unroll
                            for (int k = 0; k < 4; ++k) o[k] = fmaf(h, w[k], o[k]);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int s_ = 0; s_ < 4; ++s_)
#pragma unroll
                        for (int g = 0; g < GO; ++g) a_cur[s_][g] = a_nxt[s_][g];
                }
                if (o0 + GO < T2) {
#pragma unroll
                    for (int g = 0; g < GO; ++g) hp[g] = h2[g];
                } else {
#pragma unroll
                    for (int g = 0; g < GO; ++g)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const float h = fmaxf(h2[g][r], 0.f);
                            const f32x4 w = *(const f32x4 *)(wfp + (((o0 + g) * 16 + r) * 2 + hh) * 4);
#pragma unroll
                            for (int k = 0; k < 4; ++k) o[k] = fmaf(h, w[k], o[k]);
                        }
                }
            }
        } else {
#pragma unroll
            for (int it = 0; it < T1; ++it)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const f32x4 w = *(const f32x4 *)(wfp + ((it * 16 + r) * 2 + hh) * 4);
#pragma unroll
                    for (int k = 0; k < 4; ++k) o[k] = fmaf(h1[it][r], w[k], o[k]);
                    if (r % 4 == 3) __builtin_amdgcn_sched_barrier(0);
                }
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] = (o[k] + __shfl_xor(o[k], 32, 64)) + bfp[k];
        if (live && hh == 0) emit_decision(o, 4, row, A.bits, A.logits);
    }
}

static int device_cu_count(int *out)
{
    static int n_cu = 0;
    if (n_cu == 0) {
        int dev = 0;
        KVQ_HIP(hipGetDevice(&dev));
        KVQ_HIP(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
        if (n_cu < 1) n_cu = 1;
    }
    *out = n_cu;
    return KVQ_OK;
}

template <int T1, int T2, int NW> static int launch_mfma_nw(const MlpArgs &A, hipStream_t st, long long max_blocks)
{
    const size_t lds = mfma_lds_floats(T1, T2) * sizeof(float);
    {
        static size_t granted = 0;                 // one per instantiation
        const int rc_lds = ensure_dynamic_lds((const void *)k_mlp_mfma<T1, T2, NW>, lds, &granted);
        if (rc_lds != KVQ_OK) return rc_lds;
    }
    const long long ntiles = (A.n + 31) / 32;
    long long blocks = (ntiles + NW - 1) / NW;
    if (blocks > max_blocks) blocks = max_blocks;
    hipLaunchKernelGGL((k_mlp_mfma<T1, T2, NW>), dim3((unsigned)blocks), dim3(64 * NW), lds, st, A, ntiles);
    return KVQ_OK;
}

// Persistent launch: every workgroup stages the weights once and walks over the row tiles.  Two waves per SIMD either
// way (one wave's matrix instructions cover the other's LDS reads and vector work): as one workgroup of eight waves
// per compute unit when there are enough tiles to give every compute unit one (the weights are then staged once per
// compute unit: 82.5 against 84.5 us for 262 144 rows of the 4-128-128-4 network), else as two of four.
template <int T1, int T2> static int launch_mfma(const MlpArgs &A, hipStream_t st)
{
    int n_cu = 1;
    const int rc = device_cu_count(&n_cu);
    if (rc != KVQ_OK) return rc;
    const long long ntiles = (A.n + 31) / 32;
    const Tuning &tn = tuning();
    const int nw = (tn.controller_waves == 4 || tn.controller_waves == 8) ? tn.controller_waves : ntiles >= 8LL * n_cu ? 8 : 4;
    const int per_cu = tn.controller_wg_per_cu >= 1 ? tn.controller_wg_per_cu : nw == 8 ? 1 : 2;
    if (nw == 8) return launch_mfma_nw<T1, T2, 8>(A, st, (long long)per_cu * n_cu);
    return launch_mfma_nw<T1, T2, 4>(A, st, (long long)per_cu * n_cu);
}

template <int T1> static int launch_mfma_t2(int t2, const MlpArgs &A, hipStream_t st)
{
    switch (t2) {
    case 0: return launch_mfma<T1, 0>(A, st);
    case 1: return launch_mfma<T1, 1>(A, st);
    case 2: return launch_mfma<T1, 2>(A, st);
    default: return launch_mfma<T1, 4>(A, st);
    }
}

static bool mfma_width(int w) { return w == 32 || w == 64 || w == 128; }

// stand-in rule-based policy: thread = row
struct RuleArgs { float w[4], bias, thr[3]; };

__global__ __launch_bounds__(256) void k_rule_policy(const float *feats, long long n, RuleArgs R, uint8_t *bits, float *score)
{
    const long long row = (long long)blockIdx.x * 256 + threadIdx.x;
    if (row >= n) return;
    float u = R.bias;
#pragma unroll
    for (int i = 0; i < 4; ++i) u = fmaf(R.w[i], feats[row * 4 + i], u);
    int cls = 0;
#pragma unroll
    for (int k = 0; k < 3; ++k) cls += u > R.thr[k] ? 1 : 0;
    bits[row] = (uint8_t)(2 << cls);
    if (score) score[row] = u;
}

}  // namespace kvq

using namespace kvq;

// validates the network description and copies it into kernel arguments (feats, bits, logits and n are left to the caller)
int kvq::mlp_args_from(const kvq_mlp *mlp, MlpArgs *out, int *max_width)
{
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
    MlpArgs &A = *out;
    A.feats = nullptr;
    A.bits = nullptr;
    A.logits = nullptr;
    A.n = 0;
    A.n_linear = mlp->n_linear;
    for (int l = 0; l < 5; ++l) A.dims[l] = l <= mlp->n_linear ? mlp->dims[l] : 0;
    for (int l = 0; l < 4; ++l) {
        A.W[l] = l < mlp->n_linear ? mlp->W[l] : nullptr;
        A.b[l] = l < mlp->n_linear ? mlp->b[l] : nullptr;
    }
    if (max_width) *max_width = maxw;
    return KVQ_OK;
}

extern "C" int kvq_controller(const float *feats, int64_t n, const kvq_mlp *mlp, uint8_t *bits_out,
                              float *logits_out, void *stream)
{
    if (n < 0) { set_error("n negative"); return KVQ_ERR_INVALID_ARG; }
    MlpArgs A;
    int maxw = 4;
    const int rc0 = mlp_args_from(mlp, &A, &maxw);
    if (rc0 != KVQ_OK) return rc0;
    if (n == 0) return KVQ_OK;
    if (!feats || !bits_out) { set_error("feats or bits_out is NULL"); return KVQ_ERR_INVALID_ARG; }
    A.feats = feats;
    A.bits = bits_out;
    A.logits = logits_out;
    A.n = n;
    hipStream_t st = (hipStream_t)stream;
    if (n <= 2048) {
        hipLaunchKernelGGL(k_mlp_row, dim3((unsigned)n), dim3(n <= 256 ? 1024 : kRowThreads), 0, st, A);
    } else if (mfma_width(A.dims[1]) && (A.n_linear == 2 || mfma_width(A.dims[2])) && ((uintptr_t)feats & 15) == 0 &&
               !tuning().controller_no_mfma) {
        const int t1 = A.dims[1] / 32, t2 = A.n_linear == 3 ? A.dims[2] / 32 : 0;
        const int rc = t1 == 1 ? launch_mfma_t2<1>(t2, A, st) : t1 == 2 ? launch_mfma_t2<2>(t2, A, st) : launch_mfma_t2<4>(t2, A, st);
        if (rc != KVQ_OK) return rc;
    } else {
        const long long blocks = (n + kBulkThreads - 1) / kBulkThreads;
        if (blocks > 0x7fffffffLL) { set_error("n too large for one launch"); return KVQ_ERR_CAPACITY; }
        const size_t lds = (size_t)2 * maxw * kBulkThreads * sizeof(float);
        {
        static size_t granted = 0;
        const int rc_lds = ensure_dynamic_lds((const void *)k_mlp_bulk, lds, &granted);
        if (rc_lds != KVQ_OK) return rc_lds;
    }
        hipLaunchKernelGGL(k_mlp_bulk, dim3((unsigned)blocks), dim3(kBulkThreads), lds, st, A, maxw);
    }
    KVQ_HIP(hipGetLastError());
    return KVQ_OK;
}

extern "C" int kvq_rule_policy(const float *feats, int64_t n, const kvq_rule *rule, uint8_t *bits_out, float *score_out, void *stream)
{
    if (n < 0) { set_error("n negative"); return KVQ_ERR_INVALID_ARG; }
    if (!rule) { set_error("rule is NULL"); return KVQ_ERR_INVALID_ARG; }
    if (!(rule->thr[0] <= rule->thr[1] && rule->thr[1] <= rule->thr[2])) { set_error("thresholds must ascend"); return KVQ_ERR_INVALID_ARG; }
    if (n == 0) return KVQ_OK;
    if (!feats || !bits_out) { set_error("feats or bits_out is NULL"); return KVQ_ERR_INVALID_ARG; }
    if ((n + 255) / 256 > 0x7fffffffLL) { set_error("n too large for one launch"); return KVQ_ERR_CAPACITY; }
    RuleArgs R;
    for (int i = 0; i < 4; ++i) R.w[i] = rule->w[i];
    R.bias = rule->bias;
    for (int k = 0; k < 3; ++k) R.thr[k] = rule->thr[k];
    hipLaunchKernelGGL(k_rule_policy, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, feats, (long long)n, R,
                       bits_out, score_out);
    KVQ_HIP(hipGetLastError());
    return KVQ_OK;
}

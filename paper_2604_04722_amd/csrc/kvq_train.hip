// Training step of the controller (paper Sec. 3.8 and the inner loop of Algorithm 1): forward pass, the objective
// L = alpha L_ce + beta L_lat + gamma L_qual, its gradient by the chain rule, and one Adam update.
//
// Two launches.  k_train_grad: a workgroup stages the weights in LDS once (rows padded by one float) and takes tiles
// of 32 mini-batch rows; activations live in LDS as
// [unit][row] columns (row stride 33: conflict-free for "lane = row" and for "lane = unit"); the forward pass is
// thread = (row, unit group); the per-row loss and dL/do follow; weight gradients are sums over the tile's rows
// with thread = gradient element; deltas are propagated in place of the activations they belong to.  Each
// (persistent) workgroup accumulates its rows' gradient into its own slice of the workspace, so no atomics are needed
// and the result does not depend on scheduling.  k_train_adam: thread = parameter; sums the slices in order and
// applies Adam.  The network is small (17 540 parameters for 4-128-128-4) and a mini-batch is a handful of tiles: the
// step takes as long as one workgroup needs for one tile.  On the vector ALU that is set by LDS reads (both operands
// of every FMA); with hidden widths of 32, 64 or 128 the middle layer's three products run on the matrix cores instead
// (see k_train_grad).
#include "kvq_internal.h"
#include "kvq_mlp.h"

#include <cmath>

namespace kvq {

constexpr int kTrainRows = 32;                 // rows per tile
constexpr int kTrainRS = kTrainRows + 1;       // LDS row stride
constexpr int kTrainThreads = 256;
constexpr int kTrainMaxWidth = 128;
constexpr int kTrainMaxGroups = 256;           // workspace slices

struct TrainArgs {
    const float *feats;
    const uint8_t *labels;
    float *W[3];
    float *b[3];
    float *mW[3], *mb[3], *vW[3], *vb[3];
    float *ws;                                  // [groups][P] gradient slices, then [groups][4] loss partials
    float *losses;                              // [4] total, ce, lat, qual (or nullptr)
    float *grads_out;                           // [P] or nullptr
    long long n;
    int n_linear;
    int dims[4];
    int offW[3], offb[3];                       // offsets of each tensor in the flat parameter order W1,b1,W2,b2,(W3,b3)
    int P;
    int groups;
    float alpha, beta, gamma, c[4], q[4];
    float lr, beta1, beta2, eps, corr1, corr2;  // corr = 1 / (1 - beta^t)
    float inv_n;
};

// All LDS regions are addressed as lds[offset + ...] with offsets held in registers, and the loops over the (at most
// three) layers are unrolled with compile-time layer indices: a pointer picked from an array at run time would be a
// generic one, and every LDS access a flat load.
struct TrainLds {
    int act[3];        // input of linear layer l: features, h1, h2   ([unit][row], row stride kTrainRS)
    int dO;            // logits, then dL/do
    int W[3];          // weights of layer l, rows padded to in + 1
    int b[3];          // biases
};

__device__ __forceinline__ TrainLds train_lds_layout(const TrainArgs &A)
{
    TrainLds L;
    L.act[0] = 0;
    L.act[1] = 4 * kTrainRS;
    L.act[2] = L.act[1] + A.dims[1] * kTrainRS;
    const int last = A.n_linear == 3 ? L.act[2] + A.dims[2] * kTrainRS : L.act[2];
    L.dO = last;
    int nxt = L.dO + 4 * kTrainRS;
#pragma unroll
    for (int l = 0; l < 3; ++l) { L.W[l] = nxt; if (l < A.n_linear) nxt += A.dims[l + 1] * (A.dims[l] + 1); }
#pragma unroll
    for (int l = 0; l < 3; ++l) { L.b[l] = nxt; if (l < A.n_linear) nxt += A.dims[l + 1]; }
    return L;
}

typedef float f32x16 __attribute__((ext_vector_type(16)));

// unit of a 32 x 32 MFMA result that register r holds in the lanes of half hh (the row is lane % 32)
__device__ __forceinline__ int mfma_unit(int r, int hh) { return 8 * (r >> 2) + 4 * hh + (r & 3); }

// T1, T2 > 0: three linear layers with hidden widths 32 T1 and 32 T2; the middle layer (all but a few percent of the
// arithmetic) then runs on the matrix cores.  A tile's 32 rows are the N of v_mfma_f32_32x32x2_f32, the activations
// [unit][row] in LDS are its B operands as they lie, and the three products are
//   forward   h2[j][row]  = b2[j] + sum_i W2[j][i] h1[i][row]       A = W2 rows,        K = 32 T1 units
//   weights   dW2[j][i]  += sum_row D2[j][row] h1[i][row]           A = D2, B = h1,     K = 32 rows
//   deltas    D1[i][row]  = sum_j W2[j][i] D2[j][row]  (h1 > 0)     A = W2 columns,     K = 32 T2 units
// Each wavefront owns ceil(T1 T2 / 4) tiles of dW2 and keeps them in registers over all of the workgroup's row tiles.
// T1 == 0: every layer on the vector ALU (any widths).
template <int T1, int T2>
__global__ __launch_bounds__(kTrainThreads) void k_train_grad(TrainArgs A)
{
    constexpr bool MM = T1 > 0;
    constexpr int kGradTiles = MM ? (T1 * T2 + 3) / 4 : 1;
    f32x16 gacc[kGradTiles];
#pragma unroll
    for (int q = 0; q < kGradTiles; ++q)
#pragma unroll
        for (int rr = 0; rr < 16; ++rr) gacc[q][rr] = 0.f;
    const int wv = threadIdx.x >> 6, lane = threadIdx.x & 63, hh = lane >> 5, jl = lane & 31;
    extern __shared__ float lds[];
    const TrainLds L = train_lds_layout(A);
    const int tid = threadIdx.x, r = tid & (kTrainRows - 1), ug = tid / kTrainRows;
    constexpr int kGroups = kTrainThreads / kTrainRows;
    // weights and biases, copied once by contiguous reads that share one memory latency
    {
        MlpArgs M;
        M.n_linear = A.n_linear;
#pragma unroll
        for (int l = 0; l < 5; ++l) M.dims[l] = l < 4 ? A.dims[l] : 0;
#pragma unroll
        for (int l = 0; l < 4; ++l) { M.W[l] = l < 3 ? A.W[l] : nullptr; M.b[l] = l < 3 ? A.b[l] : nullptr; }
        mlp_stage_weights(M, lds + L.W[0], tid, kTrainThreads);
#pragma unroll
        for (int l = 0; l < 3; ++l)
            if (l < A.n_linear)
                for (int j = tid; j < A.dims[l + 1]; j += kTrainThreads) lds[L.b[l] + j] = A.b[l][j];
    }
    float *slice = A.ws + (size_t)blockIdx.x * A.P;
    float *loss_slice = A.ws + (size_t)A.groups * A.P + (size_t)blockIdx.x * 4;
    float l_ce = 0.f, l_lat = 0.f, l_q = 0.f;
    const long long n_tiles = (A.n + kTrainRows - 1) / kTrainRows;
    bool first = true;
    for (long long tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const long long row = tile * kTrainRows + r;
        const bool live = row < A.n;
        if (ug < 4) lds[L.act[0] + ug * kTrainRS + r] = live ? A.feats[row * 4 + ug] : 0.f;
        __syncthreads();
        // ---- forward (Sec. 3.6)
#pragma unroll
        for (int l = 0; l < 3; ++l) {
            if (l >= A.n_linear) break;
            const int in = A.dims[l], outw = A.dims[l + 1];
            const bool hidden = l + 1 < A.n_linear;
            const int in_off = L.act[l] + r, out_off = (hidden ? L.act[l < 2 ? l + 1 : 2] : L.dO) + r;
            if (MM && l == 1) {
                for (int ot = wv; ot < T2; ot += 4) {
                    f32x16 acc;
#pragma unroll
                    for (int rr = 0; rr < 16; ++rr) acc[rr] = lds[L.b[1] + 32 * ot + mfma_unit(rr, hh)];
                    const int a_off = L.W[1] + (32 * ot + jl) * (in + 1) + hh, b_off = L.act[1] + hh * kTrainRS + jl;
#pragma unroll 8
                    for (int s2 = 0; s2 < 32 * T1; s2 += 2)
                        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(lds[a_off + s2], lds[b_off + s2 * kTrainRS], acc, 0, 0, 0);
#pragma unroll
                    for (int rr = 0; rr < 16; ++rr)
                        lds[L.act[2] + (32 * ot + mfma_unit(rr, hh)) * kTrainRS + jl] = fmaxf(acc[rr], 0.f);
                }
                __syncthreads();
                continue;
            }
            for (int j = ug; j < outw; j += kGroups) {
                float a = lds[L.b[l] + j];
                const int w_off = L.W[l] + j * (in + 1);
                int i = 0;
                for (; i + 8 <= in; i += 8) {              // eight LDS reads of each kind before their FMAs
                    float wv[8], hv[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) { wv[u] = lds[w_off + i + u]; hv[u] = lds[in_off + (i + u) * kTrainRS]; }
#pragma unroll
                    for (int u = 0; u < 8; ++u) a = fmaf(wv[u], hv[u], a);
                }
                for (; i < in; ++i) a = fmaf(lds[w_off + i], lds[in_off + i * kTrainRS], a);
                if (hidden) a = fmaxf(a, 0.f);
                lds[out_off + j * kTrainRS] = a;
            }
            __syncthreads();
        }
        // ---- objective and dL/do for the tile's rows (Sec. 3.8); a row past the end contributes nothing
        if (tid < kTrainRows) {
            float o[4], p[4], d[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int k = 0; k < 4; ++k) o[k] = lds[L.dO + k * kTrainRS + r];
            const float mx = fmaxf(fmaxf(o[0], o[1]), fmaxf(o[2], o[3]));
            float sum = 0.f;
#pragma unroll
            for (int k = 0; k < 4; ++k) { p[k] = expf(o[k] - mx); sum += p[k]; }
            const float inv = 1.0f / sum;
            if (live) {
                const int lb = A.labels[row];
                const int y = lb == 2 ? 0 : lb == 4 ? 1 : lb == 8 ? 2 : 3;         // label map of Algorithm 1
                float pw = 0.f, pc = 0.f, pq = 0.f;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    p[k] *= inv;
                    pc = fmaf(p[k], A.c[k], pc);
                    pq = fmaf(p[k], A.q[k], pq);
                    pw = fmaf(p[k], A.beta * A.c[k] - A.gamma * A.q[k], pw);
                }
                l_ce += -(o[y] - mx - logf(sum));
                l_lat += pc;
                l_q += pq;
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    d[k] = (A.alpha * (p[k] - (k == y ? 1.f : 0.f)) + p[k] * (A.beta * A.c[k] - A.gamma * A.q[k] - pw)) * A.inv_n;
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) lds[L.dO + k * kTrainRS + r] = d[k];
        }
        __syncthreads();
        // ---- backward: gradients of layer l from its input act[l] and the delta D of its output
#pragma unroll
        for (int l = 2; l >= 0; --l) {
            if (l >= A.n_linear) continue;
            const int in = A.dims[l], outw = A.dims[l + 1];
            const int d_off = l + 1 < A.n_linear ? L.act[l < 2 ? l + 1 : 2] : L.dO;      // delta of this layer's output
            const int in_off = L.act[l];
            if (MM && l == 1) {
#pragma unroll
                for (int q = 0; q < kGradTiles; ++q) {
                    const int idx = wv + 4 * q;
                    if (idx < T1 * T2) {
                        const int jt = idx / T1, it = idx % T1;
                        const int a_off = d_off + (32 * jt + jl) * kTrainRS + hh, b_off = in_off + (32 * it + jl) * kTrainRS + hh;
#pragma unroll 8
                        for (int s2 = 0; s2 < kTrainRows; s2 += 2)
                            gacc[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(lds[a_off + s2], lds[b_off + s2], gacc[q], 0, 0, 0);
                    }
                }
                for (int j = tid; j < outw; j += kTrainThreads) {
                    float g = 0.f;
#pragma unroll
                    for (int rr = 0; rr < kTrainRows; ++rr) g += lds[d_off + j * kTrainRS + rr];
                    float *dst = slice + A.offb[l] + j;
                    *dst = first ? g : *dst + g;
                }
                __syncthreads();                               // every gradient of this layer has read act[l]
                for (int it = wv; it < T1; it += 4) {
                    f32x16 acc;
#pragma unroll
                    for (int rr = 0; rr < 16; ++rr) acc[rr] = 0.f;
                    const int a_off = L.W[1] + hh * (in + 1) + 32 * it + jl, b_off = d_off + hh * kTrainRS + jl;
#pragma unroll 8
                    for (int s2 = 0; s2 < 32 * T2; s2 += 2)
                        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(lds[a_off + s2 * (in + 1)], lds[b_off + s2 * kTrainRS], acc, 0, 0, 0);
#pragma unroll
                    for (int rr = 0; rr < 16; ++rr) {
                        const int at = in_off + (32 * it + mfma_unit(rr, hh)) * kTrainRS + jl;
                        lds[at] = lds[at] > 0.f ? acc[rr] : 0.f;
                    }
                }
                __syncthreads();
                continue;
            }
            for (int e = tid; e < in * outw; e += kTrainThreads) {
                const int j = e / in, i = e - j * in;
                float g = 0.f;
#pragma unroll
                for (int rr = 0; rr < kTrainRows; ++rr)
                    g = fmaf(lds[d_off + j * kTrainRS + rr], lds[in_off + i * kTrainRS + rr], g);
                float *dst = slice + A.offW[l] + e;
                *dst = first ? g : *dst + g;
            }
            for (int j = tid; j < outw; j += kTrainThreads) {
                float g = 0.f;
#pragma unroll
                for (int rr = 0; rr < kTrainRows; ++rr) g += lds[d_off + j * kTrainRS + rr];
                float *dst = slice + A.offb[l] + j;
                *dst = first ? g : *dst + g;
            }
            if (l > 0) {
                __syncthreads();                               // every gradient of this layer has read act[l]
                // delta of the layer below, written over its activations: (W^T D) where the unit was active
                for (int i = ug; i < in; i += kGroups) {
                    float s = 0.f;
                    int j = 0;
                    for (; j + 8 <= outw; j += 8) {
                        float wv[8], dv[8];
#pragma unroll
                        for (int u = 0; u < 8; ++u) {
                            wv[u] = lds[L.W[l] + (j + u) * (in + 1) + i];
                            dv[u] = lds[d_off + (j + u) * kTrainRS + r];
                        }
#pragma unroll
                        for (int u = 0; u < 8; ++u) s = fmaf(wv[u], dv[u], s);
                    }
                    for (; j < outw; ++j) s = fmaf(lds[L.W[l] + j * (in + 1) + i], lds[d_off + j * kTrainRS + r], s);
                    const int at = in_off + i * kTrainRS + r;
                    lds[at] = lds[at] > 0.f ? s : 0.f;
                }
                __syncthreads();
            }
        }
        first = false;
        __syncthreads();                                       // the next tile overwrites the LDS buffers
    }
    // a workgroup that had no tile still owns a slice: clear it
    if (first) {
        for (int e = tid; e < A.P; e += kTrainThreads) slice[e] = 0.f;
    }
    if constexpr (MM) {
        // the middle layer's weight gradient, summed in registers over the workgroup's tiles
        if (!first) {
#pragma unroll
            for (int q = 0; q < kGradTiles; ++q) {
                const int idx = wv + 4 * q;
                if (idx < T1 * T2) {
                    const int jt = idx / T1, it = idx % T1;
#pragma unroll
                    for (int rr = 0; rr < 16; ++rr)
                        slice[A.offW[1] + (32 * jt + mfma_unit(rr, hh)) * (32 * T1) + 32 * it + jl] = gacc[q][rr];
                }
            }
        }
    }
    if (tid < kTrainRows) {
#pragma unroll
        for (int o = kTrainRows / 2; o >= 1; o >>= 1) {
            l_ce += __shfl_xor(l_ce, o, 64);
            l_lat += __shfl_xor(l_lat, o, 64);
            l_q += __shfl_xor(l_q, o, 64);
        }
        if (tid == 0) { loss_slice[0] = l_ce; loss_slice[1] = l_lat; loss_slice[2] = l_q; loss_slice[3] = 0.f; }
    }
}

__global__ __launch_bounds__(256) void k_train_adam(TrainArgs A)
{
    const int p = blockIdx.x * 256 + threadIdx.x;
    if (p == 0 && A.losses) {
        float ce = 0.f, lat = 0.f, qs = 0.f;
        for (int g = 0; g < A.groups; ++g) {
            const float *ls = A.ws + (size_t)A.groups * A.P + (size_t)g * 4;
            ce += ls[0]; lat += ls[1]; qs += ls[2];
        }
        ce *= A.inv_n; lat *= A.inv_n;
        const float qual = 1.0f - qs * A.inv_n;
        A.losses[0] = A.alpha * ce + A.beta * lat + A.gamma * qual;
        A.losses[1] = ce; A.losses[2] = lat; A.losses[3] = qual;
    }
    if (p >= A.P) return;
    float g = 0.f;
    int s = 0;
    for (; s + 8 <= A.groups; s += 8) {                       // eight loads in flight, added in slice order
        float t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = A.ws[(size_t)(s + u) * A.P + p];
#pragma unroll
        for (int u = 0; u < 8; ++u) g += t[u];
    }
    for (; s < A.groups; ++s) g += A.ws[(size_t)s * A.P + p];
    if (A.grads_out) A.grads_out[p] = g;
    // which tensor does flat index p belong to
    float *theta = nullptr, *m = nullptr, *v = nullptr;
    int local = 0;
    for (int l = 0; l < A.n_linear; ++l) {
        const int nW = A.dims[l] * A.dims[l + 1], nb = A.dims[l + 1];
        if (p >= A.offW[l] && p < A.offW[l] + nW) { local = p - A.offW[l]; theta = A.W[l]; m = A.mW[l]; v = A.vW[l]; }
        if (p >= A.offb[l] && p < A.offb[l] + nb) { local = p - A.offb[l]; theta = A.b[l]; m = A.mb[l]; v = A.vb[l]; }
    }
    const float mn = A.beta1 * m[local] + (1.0f - A.beta1) * g;
    const float vn = A.beta2 * v[local] + (1.0f - A.beta2) * g * g;
    m[local] = mn;
    v[local] = vn;
    theta[local] -= A.lr * (mn * A.corr1) / (sqrtf(vn * A.corr2) + A.eps);
}

static int fill_train_args(const kvq_mlp *mlp, const kvq_mlp *am, const kvq_mlp *av, TrainArgs *out)
{
    if (!mlp || !am || !av) { set_error("mlp, adam_m or adam_v is NULL"); return KVQ_ERR_INVALID_ARG; }
    if (mlp->n_linear < 2 || mlp->n_linear > 3) { set_error("n_linear must be 2 or 3"); return KVQ_ERR_UNSUPPORTED; }
    if (mlp->dims[0] != 4 || mlp->dims[mlp->n_linear] != 4) { set_error("the network must map 4 features to 4 classes"); return KVQ_ERR_INVALID_ARG; }
    TrainArgs &A = *out;
    A.n_linear = mlp->n_linear;
    int off = 0;
    for (int l = 0; l < 4; ++l) A.dims[l] = l <= mlp->n_linear ? mlp->dims[l] : 0;
    for (int l = 0; l < 3; ++l) {
        A.W[l] = A.b[l] = A.mW[l] = A.mb[l] = A.vW[l] = A.vb[l] = nullptr;
        A.offW[l] = A.offb[l] = 0;
    }
    for (int l = 0; l < mlp->n_linear; ++l) {
        if (l >= 1 && (mlp->dims[l] < 1 || mlp->dims[l] > kTrainMaxWidth)) {
            set_error("hidden width %d outside 1..%d", mlp->dims[l], kTrainMaxWidth);
            return KVQ_ERR_UNSUPPORTED;
        }
        if (am->n_linear != mlp->n_linear || av->n_linear != mlp->n_linear || am->dims[l + 1] != mlp->dims[l + 1] ||
            av->dims[l + 1] != mlp->dims[l + 1]) {
            set_error("adam_m / adam_v do not have the network's shape");
            return KVQ_ERR_INVALID_ARG;
        }
        if (!mlp->W[l] || !mlp->b[l] || !am->W[l] || !am->b[l] || !av->W[l] || !av->b[l]) {
            set_error("a weight, bias or Adam state pointer of layer %d is NULL", l);
            return KVQ_ERR_INVALID_ARG;
        }
        A.W[l] = const_cast<float *>(mlp->W[l]); A.b[l] = const_cast<float *>(mlp->b[l]);
        A.mW[l] = const_cast<float *>(am->W[l]); A.mb[l] = const_cast<float *>(am->b[l]);
        A.vW[l] = const_cast<float *>(av->W[l]); A.vb[l] = const_cast<float *>(av->b[l]);
        A.offW[l] = off; off += mlp->dims[l] * mlp->dims[l + 1];
        A.offb[l] = off; off += mlp->dims[l + 1];
    }
    A.P = off;
    return KVQ_OK;
}

template <int T1, int T2> static int launch_train_grad(const TrainArgs &A, size_t lds, hipStream_t st)
{
    static size_t granted = 0;                     // one per instantiation
    const int rc_lds = ensure_dynamic_lds((const void *)k_train_grad<T1, T2>, lds, &granted);
    if (rc_lds != KVQ_OK) return rc_lds;
    hipLaunchKernelGGL((k_train_grad<T1, T2>), dim3((unsigned)A.groups), dim3(kTrainThreads), lds, st, A);
    KVQ_HIP(hipGetLastError());
    return KVQ_OK;
}

static int train_groups(int64_t n)
{
    const int64_t tiles = (n + kTrainRows - 1) / kTrainRows;
    return (int)(tiles < kTrainMaxGroups ? tiles : kTrainMaxGroups);
}

}  // namespace kvq

using namespace kvq;

extern "C" int64_t kvq_controller_param_count(const kvq_mlp *mlp)
{
    if (!mlp || mlp->n_linear < 2 || mlp->n_linear > 3) return 0;
    int64_t p = 0;
    for (int l = 0; l < mlp->n_linear; ++l) p += (int64_t)mlp->dims[l] * mlp->dims[l + 1] + mlp->dims[l + 1];
    return p;
}

extern "C" size_t kvq_controller_train_workspace(const kvq_mlp *mlp, int64_t n)
{
    const int64_t P = kvq_controller_param_count(mlp);
    if (P <= 0 || n <= 0) return 0;
    return (size_t)train_groups(n) * (size_t)(P + 4) * sizeof(float) + 256;
}

extern "C" int kvq_controller_train_step(const float *feats, const uint8_t *label_bits, int64_t n, const kvq_mlp *mlp,
                                         const kvq_mlp *adam_m, const kvq_mlp *adam_v, const kvq_train_hparams *hp,
                                         int64_t step, float *losses_out, float *grads_out, void *workspace,
                                         size_t workspace_bytes, void *stream)
{
    if (n < 1) { set_error("n must be positive"); return KVQ_ERR_INVALID_ARG; }
    if (!feats || !label_bits || !hp) { set_error("feats, label_bits or hp is NULL"); return KVQ_ERR_INVALID_ARG; }
    if (step < 1) { set_error("step counts from 1"); return KVQ_ERR_INVALID_ARG; }
    if (!(hp->beta1 >= 0.f && hp->beta1 < 1.f && hp->beta2 >= 0.f && hp->beta2 < 1.f)) {
        set_error("Adam's beta1 and beta2 must lie in [0, 1)");
        return KVQ_ERR_INVALID_ARG;
    }
    TrainArgs A;
    const int rc = fill_train_args(mlp, adam_m, adam_v, &A);
    if (rc != KVQ_OK) return rc;
    const size_t need = kvq_controller_train_workspace(mlp, n) - 256;
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 15) != 0) {
        set_error("workspace missing, misaligned or too small: %zu bytes given, %zu needed", workspace_bytes, need);
        return KVQ_ERR_INVALID_ARG;
    }
    A.feats = feats;
    A.labels = label_bits;
    A.ws = (float *)workspace;
    A.losses = losses_out;
    A.grads_out = grads_out;
    A.n = n;
    A.groups = train_groups(n);
    A.alpha = hp->alpha; A.beta = hp->beta; A.gamma = hp->gamma;
    for (int k = 0; k < 4; ++k) { A.c[k] = hp->c[k]; A.q[k] = hp->q[k]; }
    A.lr = hp->lr; A.beta1 = hp->beta1; A.beta2 = hp->beta2; A.eps = hp->eps;
    A.corr1 = (float)(1.0 / (1.0 - std::pow((double)hp->beta1, (double)step)));
    A.corr2 = (float)(1.0 / (1.0 - std::pow((double)hp->beta2, (double)step)));
    A.inv_n = (float)(1.0 / (double)n);
    size_t lds = (size_t)(8 + A.dims[1] + (A.n_linear == 3 ? A.dims[2] : 0)) * kTrainRS * sizeof(float);
    for (int l = 0; l < A.n_linear; ++l) lds += (size_t)A.dims[l + 1] * (A.dims[l] + 2) * sizeof(float);    // weights (padded rows) + bias
    hipStream_t st = (hipStream_t)stream;
    const auto mm_width = [](int w) { return w == 32 || w == 64 || w == 128; };
    const bool mm = A.n_linear == 3 && mm_width(A.dims[1]) && mm_width(A.dims[2]) && !tuning().train_no_mfma;
    const int t1 = mm ? A.dims[1] / 32 : 0, t2 = mm ? A.dims[2] / 32 : 0;
    int rc_launch = KVQ_OK;
    switch (t1 * 8 + t2) {
    case 1 * 8 + 1: rc_launch = launch_train_grad<1, 1>(A, lds, st); break;
    case 1 * 8 + 2: rc_launch = launch_train_grad<1, 2>(A, lds, st); break;
    case 1 * 8 + 4: rc_launch = launch_train_grad<1, 4>(A, lds, st); break;
    case 2 * 8 + 1: rc_launch = launch_train_grad<2, 1>(A, lds, st); break;
    case 2 * 8 + 2: rc_launch = launch_train_grad<2, 2>(A, lds, st); break;
    case 2 * 8 + 4: rc_launch = launch_train_grad<2, 4>(A, lds, st); break;
    case 4 * 8 + 1: rc_launch = launch_train_grad<4, 1>(A, lds, st); break;
    case 4 * 8 + 2: rc_launch = launch_train_grad<4, 2>(A, lds, st); break;
    case 4 * 8 + 4: rc_launch = launch_train_grad<4, 4>(A, lds, st); break;
    default: rc_launch = launch_train_grad<0, 0>(A, lds, st); break;
    }
    if (rc_launch != KVQ_OK) return rc_launch;
    hipLaunchKernelGGL(k_train_adam, dim3((unsigned)((A.P + 255) / 256)), dim3(256), 0, st, A);
    KVQ_HIP(hipGetLastError());
    return KVQ_OK;
}

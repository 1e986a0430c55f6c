// Token-level saliency features s_t = [H_t, R_t, V_t, C_t] (paper Sec. 3.5).
//
// H_t and C_t come from one pass over the logits row: with m = max z, S = sum exp(z-m),
// T = sum (z-m) exp(z-m):  H = ln S - T/S  (= -sum p ln p)  and  C = max p = 1/S.
// A row is cut into slices so that n rows x slices fill the chip; each thread keeps a running
// (m, S, T) triple, triples are merged exactly (rescaling by exp(m_a - m_b)), slice results go to a
// small workspace and a second kernel merges them and adds R_t and V_t.
#include "kvq_internal.h"

namespace kvq {

constexpr int kFeatThreads = 256;
constexpr int kMaxSlices = 64;

struct Lse3 { float m, s, t; };

// merge b into a:  both are (max, sum e^{z-max}, sum (z-max) e^{z-max}) of disjoint sets
__device__ __forceinline__ Lse3 lse3_merge(Lse3 a, Lse3 b)
{
    if (b.m == -INFINITY) return a;
    if (a.m == -INFINITY) return b;
    const float M = fmaxf(a.m, b.m);
    const float da = a.m - M, db = b.m - M;              // <= 0
    const float fa = expf(da), fb = expf(db);
    Lse3 r;
    r.m = M;
    r.s = a.s * fa + b.s * fb;
    r.t = fa * (a.t + da * a.s) + fb * (b.t + db * b.s);   // sum (z-M)e^{z-M} = e^{d}(T + d*S)
    return r;
}

__device__ __forceinline__ void lse3_add4(Lse3 &a, float z0, float z1, float z2, float z3)
{
    const float m4 = fmaxf(fmaxf(z0, z1), fmaxf(z2, z3));
    if (m4 > a.m) {
        if (a.m != -INFINITY) {
            const float d = a.m - m4;
            const float f = expf(d);
            a.t = f * (a.t + d * a.s);
            a.s *= f;
        }
        a.m = m4;
    }
    const float d0 = z0 - a.m, d1 = z1 - a.m, d2 = z2 - a.m, d3 = z3 - a.m;
    const float e0 = expf(d0), e1 = expf(d1), e2 = expf(d2), e3 = expf(d3);
    a.s += (e0 + e1) + (e2 + e3);
    a.t += (d0 * e0 + d1 * e1) + (d2 * e2 + d3 * e3);
}

__device__ __forceinline__ void lse3_add1(Lse3 &a, float z)
{
    if (z > a.m) {
        if (a.m != -INFINITY) {
            const float d = a.m - z;
            const float f = expf(d);
            a.t = f * (a.t + d * a.s);
            a.s *= f;
        }
        a.m = z;
    }
    const float d = z - a.m;
    const float e = expf(d);
    a.s += e;
    a.t = fmaf(d, e, a.t);
}

__global__ __launch_bounds__(kFeatThreads) void k_lse_partial(const float *logits, long long vocab, int slices, float *ws)
{
    const long long row = blockIdx.y;
    const int slice = blockIdx.x;
    const float *z = logits + row * vocab;
    const long long per = (vocab + slices - 1) / slices;
    long long lo = per * slice, hi = lo + per;
    if (hi > vocab) hi = vocab;
    Lse3 a = {-INFINITY, 0.f, 0.f};
    if (lo < hi) {
        const float *p = z + lo;
        long long n = hi - lo;
        // peel to a 16-byte boundary
        long long head = ((16 - ((uintptr_t)p & 15)) & 15) / 4;
        if (head > n) head = n;
        if ((long long)threadIdx.x < head) lse3_add1(a, p[threadIdx.x]);
        p += head;
        n -= head;
        const long long n4 = n / 4;
        const float4 *p4 = (const float4 *)p;
        for (long long i = threadIdx.x; i < n4; i += kFeatThreads) {
            const float4 v = p4[i];
            lse3_add4(a, v.x, v.y, v.z, v.w);
        }
        const long long tail = n - n4 * 4;
        if ((long long)threadIdx.x < tail) lse3_add1(a, p[n4 * 4 + threadIdx.x]);
    }
    __shared__ Lse3 sm[kFeatThreads];
    sm[threadIdx.x] = a;
    __syncthreads();
    for (int o = kFeatThreads / 2; o >= 1; o >>= 1) {
        if ((int)threadIdx.x < o) sm[threadIdx.x] = lse3_merge(sm[threadIdx.x], sm[threadIdx.x + o]);
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        float *w = ws + (row * slices + slice) * 4;
        w[0] = sm[0].m; w[1] = sm[0].s; w[2] = sm[0].t;
    }
}

struct FeatArgs {
    const float *ws;
    const int32_t *token_ids;
    const long long *counts;
    const long long *totals;
    const float *attn_probs;
    const float *sum_p2;
    const int32_t *attn_len;
    float *feats;
    long long vocab, ld;
    int slices, Hq;
};

// one workgroup per token: merges the slice triples, then R and V
__global__ __launch_bounds__(kFeatThreads) void k_features_finalize(FeatArgs A)
{
    const long long t = blockIdx.x;
    __shared__ float red[kFeatThreads];
    __shared__ float red2[kFeatThreads];
    const int l = A.attn_len[t];
    const float inv_l = 1.0f / (float)l;
    float V = 0.f;
    if (A.attn_probs) {
        // population variance of each head's row, accumulated around the expected mean 1/l so that
        // nothing cancels:  Var = sum d^2 / l - (sum d / l)^2  with d = p - 1/l
        for (int h = 0; h < A.Hq; ++h) {
            const float *row = A.attn_probs + (t * A.Hq + h) * A.ld;
            float s1 = 0.f, s2 = 0.f;
            for (int j = threadIdx.x; j < l; j += kFeatThreads) {
                const float d = row[j] - inv_l;
                s1 += d;
                s2 = fmaf(d, d, s2);
            }
            red[threadIdx.x] = s1;
            red2[threadIdx.x] = s2;
            __syncthreads();
            for (int o = kFeatThreads / 2; o >= 1; o >>= 1) {
                if ((int)threadIdx.x < o) {
                    red[threadIdx.x] += red[threadIdx.x + o];
                    red2[threadIdx.x] += red2[threadIdx.x + o];
                }
                __syncthreads();
            }
            const float md = red[0] * inv_l;
            V += red2[0] * inv_l - md * md;
            __syncthreads();
        }
        V /= (float)A.Hq;
    } else {
        float s = 0.f;
        for (int h = threadIdx.x; h < A.Hq; h += kFeatThreads) s += A.sum_p2[t * A.Hq + h] * inv_l - inv_l * inv_l;
        red[threadIdx.x] = s;
        __syncthreads();
        for (int o = kFeatThreads / 2; o >= 1; o >>= 1) {
            if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
            __syncthreads();
        }
        V = red[0] / (float)A.Hq;
    }
    if (threadIdx.x != 0) return;
    Lse3 a = {-INFINITY, 0.f, 0.f};
    for (int s = 0; s < A.slices; ++s) {
        const float *w = A.ws + (t * A.slices + s) * 4;
        Lse3 b = {w[0], w[1], w[2]};
        a = lse3_merge(a, b);
    }
    const float H = logf(a.s) - a.t / a.s;
    const float C = 1.0f / a.s;
    const long long id = A.token_ids[t];
    const long long c = (id >= 0 && id < A.vocab) ? A.counts[id] : 0;    // an id outside the table counts as unseen
    // one fp64 logarithm per token: the ratio is close to 1 for common tokens
    const float R = (float)(-log((double)(c + 1) / (double)(A.totals[0] + A.totals[1] + 1)));
    float *f = A.feats + t * 4;
    f[0] = H; f[1] = R; f[2] = V; f[3] = C;
}

// counting pass that follows scoring: c[id] += 1 for every token, |V_obs| += ids seen for the first time
__global__ void k_counts_update(const int32_t *ids, long long n, long long vocab, unsigned long long *counts,
                                unsigned long long *totals)
{
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    if (i == 0) atomicAdd(&totals[0], (unsigned long long)n);
    const long long id = ids[i];
    if (id < 0 || id >= vocab) return;
    const unsigned long long old = atomicAdd(&counts[id], 1ull);
    if (old == 0ull) atomicAdd(&totals[1], 1ull);
}

static int pick_slices(long long n, long long vocab)
{
    long long s = (1024 + n - 1) / n;                     // aim at >= ~1024 workgroups
    const long long max_by_len = (vocab + 4095) / 4096;   // at least 4096 logits per slice
    if (s > max_by_len) s = max_by_len;
    if (s > kMaxSlices) s = kMaxSlices;
    if (s < 1) s = 1;
    return (int)s;
}

}  // namespace kvq

using namespace kvq;

extern "C" size_t kvq_features_workspace(int64_t n, int64_t vocab)
{
    if (n <= 0 || vocab <= 0) return 0;
    return (size_t)n * kMaxSlices * 4 * sizeof(float) + 256;
}

extern "C" int kvq_features(const float *logits, int64_t n, int64_t vocab, const int32_t *token_ids,
                            int64_t *counts, int64_t *totals, int32_t update_counts,
                            const float *attn_probs, const float *sum_p2, const int32_t *attn_len,
                            int32_t n_q_heads, int64_t ld, float *feats_out,
                            void *workspace, size_t workspace_bytes, void *stream)
{
    if (n < 0 || vocab < 1) { set_error("n or vocab out of range"); return KVQ_ERR_INVALID_ARG; }
    if (n == 0) return KVQ_OK;
    if (!logits || !token_ids || !counts || !totals || !attn_len || !feats_out) { set_error("NULL argument"); return KVQ_ERR_INVALID_ARG; }
    if ((attn_probs == nullptr) == (sum_p2 == nullptr)) {
        set_error("exactly one of attn_probs and sum_p2 must be given");
        return KVQ_ERR_INVALID_ARG;
    }
    if (n_q_heads < 1) { set_error("n_q_heads must be positive"); return KVQ_ERR_INVALID_ARG; }
    if (attn_probs && ld < 1) { set_error("ld must be positive"); return KVQ_ERR_INVALID_ARG; }
    if (n > 0x7fffffffLL / kMaxSlices) { set_error("n too large for one call"); return KVQ_ERR_CAPACITY; }
    const size_t need = kvq_features_workspace(n, vocab) - 256;
    if (!workspace || workspace_bytes < need) {
        set_error("workspace too small: %zu bytes given, %zu needed", workspace_bytes, need);
        return KVQ_ERR_INVALID_ARG;
    }
    hipStream_t st = (hipStream_t)stream;
    const int slices = pick_slices(n, vocab);
    if (n > 65535) { set_error("n above 65535 rows per call is not supported"); return KVQ_ERR_UNSUPPORTED; }
    hipLaunchKernelGGL(k_lse_partial, dim3(slices, (unsigned)n), dim3(kFeatThreads), 0, st, logits, (long long)vocab,
                       slices, (float *)workspace);
    KVQ_HIP(hipGetLastError());
    FeatArgs A;
    A.ws = (const float *)workspace;
    A.token_ids = token_ids;
    A.counts = (const long long *)counts;
    A.totals = (const long long *)totals;
    A.attn_probs = attn_probs;
    A.sum_p2 = sum_p2;
    A.attn_len = attn_len;
    A.feats = feats_out;
    A.vocab = vocab;
    A.ld = ld;
    A.slices = slices;
    A.Hq = n_q_heads;
    hipLaunchKernelGGL(k_features_finalize, dim3((unsigned)n), dim3(kFeatThreads), 0, st, A);
    KVQ_HIP(hipGetLastError());
    if (update_counts) {
        hipLaunchKernelGGL(k_counts_update, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, token_ids, (long long)n,
                           (long long)vocab, (unsigned long long *)counts, (unsigned long long *)totals);
        KVQ_HIP(hipGetLastError());
    }
    return KVQ_OK;
}

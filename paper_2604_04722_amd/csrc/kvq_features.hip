// Token-level saliency features s_t = [H_t, R_t, V_t, C_t] (paper Sec. 3.5).
//
// H_t and C_t come from one pass over the logits row: with m = max z, S = sum exp(z-m),
// T = sum (z-m) exp(z-m):  H = ln S - T/S  (= -sum p ln p)  and  C = max p = 1/S.
// A row is cut into slices so that n rows x slices fill the chip; each thread keeps a running
// (m, S, T) triple, triples are merged exactly (rescaling by exp(m_a - m_b)), slice results go to a
// small workspace and a second kernel merges them and adds R_t and V_t.
#include "kvq_internal.h"
#include "kvq_mlp.h"

namespace kvq {

constexpr int kFeatThreads = 256;
constexpr int kMaxSlices = 64;

struct Lse3 { float m, s, t; };
typedef uint32_t u32x4_nt __attribute__((ext_vector_type(4)));

// e^d for d <= 0 through the hardware 2^x: relative error below 2e-6 over the range that still contributes to a
// sum (d > -20), which is a tenth of the tolerance of the features; the library routine costs ten times the issue
// slots, and one compute unit takes a whole row of 49 152 logits in the fused kernel.
__device__ __forceinline__ float exp_neg(float d) { return __builtin_amdgcn_exp2f(d * 1.44269504088896340736f); }

// merge b into a:  both are (max, sum e^{z-max}, sum (z-max) e^{z-max}) of disjoint sets
__device__ __forceinline__ Lse3 lse3_merge(Lse3 a, Lse3 b)
{
    if (b.m == -INFINITY) return a;
    if (a.m == -INFINITY) return b;
    const float M = fmaxf(a.m, b.m);
    const float da = a.m - M, db = b.m - M;              // <= 0
    const float fa = exp_neg(da), fb = exp_neg(db);
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
            const float f = exp_neg(d);
            a.t = f * (a.t + d * a.s);
            a.s *= f;
        }
        a.m = m4;
    }
    const float d0 = z0 - a.m, d1 = z1 - a.m, d2 = z2 - a.m, d3 = z3 - a.m;
    const float e0 = exp_neg(d0), e1 = exp_neg(d1), e2 = exp_neg(d2), e3 = exp_neg(d3);
    a.s += (e0 + e1) + (e2 + e3);
    a.t += (d0 * e0 + d1 * e1) + (d2 * e2 + d3 * e3);
}

__device__ __forceinline__ void lse3_add1(Lse3 &a, float z)
{
    if (z > a.m) {
        if (a.m != -INFINITY) {
            const float d = a.m - z;
            const float f = exp_neg(d);
            a.t = f * (a.t + d * a.s);
            a.s *= f;
        }
        a.m = z;
    }
    const float d = z - a.m;
    const float e = exp_neg(d);
    a.s += e;
    a.t = fmaf(d, e, a.t);
}

// Logits come as fp32, fp16 or bf16.  The narrow types are widened exactly, so the features are those of the
// widened row; a thread's 16-byte load then carries eight logits instead of four.
struct Bf16 { uint16_t bits; };
template <typename T> __device__ __forceinline__ float widen(T x);
template <> __device__ __forceinline__ float widen<float>(float x) { return x; }
template <> __device__ __forceinline__ float widen<__half>(__half x) { return __half2float(x); }
template <> __device__ __forceinline__ float widen<Bf16>(Bf16 x) { return __uint_as_float((uint32_t)x.bits << 16); }

template <typename T> __device__ __forceinline__ void lse3_add_vec(Lse3 &a, const uint4 &v);
template <> __device__ __forceinline__ void lse3_add_vec<float>(Lse3 &a, const uint4 &v)
{
    lse3_add4(a, __uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
}
template <> __device__ __forceinline__ void lse3_add_vec<__half>(Lse3 &a, const uint4 &v)
{
    const __half2 h0 = *(const __half2 *)&v.x, h1 = *(const __half2 *)&v.y, h2 = *(const __half2 *)&v.z, h3 = *(const __half2 *)&v.w;
    lse3_add4(a, __low2float(h0), __high2float(h0), __low2float(h1), __high2float(h1));
    lse3_add4(a, __low2float(h2), __high2float(h2), __low2float(h3), __high2float(h3));
}
template <> __device__ __forceinline__ void lse3_add_vec<Bf16>(Lse3 &a, const uint4 &v)
{
    lse3_add4(a, __uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u), __uint_as_float(v.y << 16), __uint_as_float(v.y & 0xffff0000u));
    lse3_add4(a, __uint_as_float(v.z << 16), __uint_as_float(v.z & 0xffff0000u), __uint_as_float(v.w << 16), __uint_as_float(v.w & 0xffff0000u));
}

// (m, S, T) of the part of one slice of a logits row that thread `lt` of kFeatThreads takes
// Stream: the rows are read once and are too many to stay in any cache (a bulk call), so the loads go past the caches.
template <typename T, bool Stream = false>
__device__ __forceinline__ Lse3 thread_partial(const T *logits, long long vocab, int slices, long long row, int slice, int lt)
{
    constexpr int kPer = 16 / (int)sizeof(T);             // logits per 16-byte load
    const T *z = logits + row * vocab;
    const long long per = (vocab + slices - 1) / slices;
    long long lo = per * slice, hi = lo + per;
    if (hi > vocab) hi = vocab;
    Lse3 a = {-INFINITY, 0.f, 0.f};
    if (lo < hi) {
        const T *p = z + lo;
        long long n = hi - lo;
        // peel to a 16-byte boundary
        long long head = ((16 - ((uintptr_t)p & 15)) & 15) / (long long)sizeof(T);
        if (head > n) head = n;
        if ((long long)lt < head) lse3_add1(a, widen<T>(p[lt]));
        p += head;
        n -= head;
        const long long n4 = n / kPer;
        const uint4 *p4 = (const uint4 *)p;
        // four loads in flight per thread; the vectors are added in ascending order
        for (long long i = lt; i < n4; i += 4 * kFeatThreads) {
            uint4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const long long k = i + u * kFeatThreads;
                if constexpr (Stream) {
                    const u32x4_nt t = __builtin_nontemporal_load((const u32x4_nt *)(p4 + (k < n4 ? k : i)));
                    v[u] = make_uint4(t[0], t[1], t[2], t[3]);
                } else {
                    v[u] = p4[k < n4 ? k : i];
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (i + u * kFeatThreads < n4) lse3_add_vec<T>(a, v[u]);
        }
        const long long tail = n - n4 * kPer;
        if ((long long)lt < tail) lse3_add1(a, widen<T>(p[n4 * kPer + lt]));
    }
    return a;
}

// tree merge of kFeatThreads triples sm[0..kFeatThreads) (thread lt owns sm[lt]); the result is sm[0].  Every
// thread of the workgroup calls it, also in workgroups made of several such groups (sm then is the group's part).
__device__ __forceinline__ void group_merge(Lse3 *sm, int lt)
{
    __syncthreads();
    for (int o = kFeatThreads / 2; o >= 64; o >>= 1) {
        if (lt < o) sm[lt] = lse3_merge(sm[lt], sm[lt + o]);
        __syncthreads();
    }
    // the last levels stay inside the group's first wavefront: the same pairs (lt, lt + o), passed by lane shuffles
    if (lt < 64) {
        Lse3 a = sm[lt];
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) {
            Lse3 b;
            b.m = __shfl_down(a.m, o, 64);
            b.s = __shfl_down(a.s, o, 64);
            b.t = __shfl_down(a.t, o, 64);
            a = lse3_merge(a, b);
        }
        if (lt == 0) sm[0] = a;
    }
    __syncthreads();
}

template <typename T, bool Stream>
__global__ __launch_bounds__(kFeatThreads) void k_lse_partial(const T *logits, long long vocab, int slices, float *ws)
{
    __shared__ Lse3 sm[kFeatThreads];
    const long long row = blockIdx.y;
    const int slice = blockIdx.x;
    sm[threadIdx.x] = thread_partial<T, Stream>(logits, vocab, slices, row, slice, threadIdx.x);
    group_merge(sm, threadIdx.x);
    if (threadIdx.x == 0) {
        float *w = ws + (row * slices + slice) * 4;
        w[0] = sm[0].m; w[1] = sm[0].s; w[2] = sm[0].t;
    }
}

__device__ __forceinline__ float entropy_of(const Lse3 &a) { return logf(a.s) - a.t / a.s; }
__device__ __forceinline__ float confidence_of(const Lse3 &a) { return 1.0f / a.s; }
__device__ __forceinline__ float rarity_from(long long c, long long seen)
{
    // one fp64 logarithm per token: the ratio is close to 1 for common tokens
    return (float)(-log((double)(c + 1) / (double)(seen + 1)));
}
__device__ __forceinline__ float rarity_of(long long id, long long vocab, const long long *counts, const long long *totals)
{
    const long long c = (id >= 0 && id < vocab) ? counts[id] : 0;        // an id outside the table counts as unseen
    return rarity_from(c, totals[0] + totals[1]);
}

// mean over the heads of the closed form of the population variance of a probability row: sum p^2 / l - 1 / l^2.
// Every thread of the workgroup calls it; the threads with `active` (kFeatThreads of them, numbered lt) do the
// work; the value is returned to every thread.
__device__ __forceinline__ float variance_from_sum_p2(const float *sum_p2_row, int Hq, int l, float *red, int lt, bool active)
{
    const float inv_l = l > 0 ? 1.0f / (float)l : 0.f;    // l <= 0: no attention row yet, V_t = 0
    if (active) {
        float s = 0.f;
        for (int h = lt; h < Hq; h += kFeatThreads) s += sum_p2_row[h] * inv_l - inv_l * inv_l;
        red[lt] = s;
    }
    __syncthreads();
    for (int o = kFeatThreads / 2; o >= 1; o >>= 1) {
        if (active && lt < o) red[lt] += red[lt + o];
        __syncthreads();
    }
    const float V = red[0] / (float)Hq;
    __syncthreads();
    return V;
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
    const float inv_l = 1.0f / (float)(l > 0 ? l : 1);
    float V = 0.f;
    if (l <= 0) {
        V = 0.f;                                     // no attention row yet (a sequence's first token): V_t = 0
    } else if (A.attn_probs) {
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
        V = variance_from_sum_p2(A.sum_p2 + t * A.Hq, A.Hq, l, red, threadIdx.x, true);
    }
    if (threadIdx.x != 0) return;
    Lse3 a = {-INFINITY, 0.f, 0.f};
    for (int s = 0; s < A.slices; ++s) {
        const float *w = A.ws + (t * A.slices + s) * 4;
        Lse3 b = {w[0], w[1], w[2]};
        a = lse3_merge(a, b);
    }
    float *f = A.feats + t * 4;
    f[0] = entropy_of(a);
    f[1] = rarity_of(A.token_ids[t], A.vocab, A.counts, A.totals);
    f[2] = V;
    f[3] = confidence_of(a);
}

// ---- fused per-step front end: features, controller and bucket bookkeeping in one launch --------------------
//
// One workgroup of four groups of kFeatThreads threads per row.  The groups take the row's slices in turn and
// reduce each exactly as k_lse_partial does, thread 0 merges the slice triples in slice order as
// k_features_finalize does, and the controller's row shape follows, so features and logits equal those of the
// separate kernels bit for bit.  A row never needs another row's result; the count update stays a kernel of its
// own behind this one, which keeps "every row reads the table before any count changes" a matter of stream order.
constexpr int kFrontGroups = 4;

struct FrontArgs {
    const void *logits;
    const int32_t *token_ids;
    const long long *counts;
    const long long *totals;
    const float *sum_p2;
    const int32_t *attn_len;
    const int32_t *seq_ids;
    float *feats;
    long long vocab;
    int slices, Hq, advance;
};

template <typename T>
__global__ __launch_bounds__(kFrontGroups * kFeatThreads) void k_front(FrontArgs F, MlpArgs M, CacheView cv, int staged)
{
    extern __shared__ float stage[];               // the controller's weights, fetched while the logits stream in
    __shared__ Lse3 sm[kFrontGroups * kFeatThreads];
    __shared__ Lse3 slice_res[kMaxSlices];
    __shared__ float act[2][kMaxWidth];
    const long long row = blockIdx.x;
    const int tid = threadIdx.x, g = tid / kFeatThreads, lt = tid % kFeatThreads;
    // thread 0 fetches what the row's serial tail needs (the token's count, the totals, the sequence's counters) now,
    // so that these dependent reads overlap the pass over the logits
    long long tok_count = 0, seen = 0;
    int seq = 0, pre[5] = {0, 0, 0, 0, 0};
    if (tid == 0) {
        const long long id = F.token_ids[row];
        tok_count = (id >= 0 && id < F.vocab) ? F.counts[id] : 0;
        seen = F.totals[0] + F.totals[1];
        if (F.advance) {
            seq = F.seq_ids ? F.seq_ids[row] : (int)row;
            if (seq >= 0 && seq < cv.max_seqs) {
#pragma unroll
                for (int c = 0; c < 5; ++c) pre[c] = cv.counts[(size_t)seq * 5 + c];
            }
        }
    }
    if (staged) mlp_stage_weights(M, stage, tid, kFrontGroups * kFeatThreads);
    // four rounds of slices at a time: their loads are issued together, their reductions follow one by one
    constexpr int kRounds = 4;
    for (int s0 = 0; s0 < F.slices; s0 += kFrontGroups * kRounds) {
        Lse3 part[kRounds];
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
            const int slice = s0 + r * kFrontGroups + g;
            part[r].m = -INFINITY; part[r].s = 0.f; part[r].t = 0.f;
            if (slice < F.slices) part[r] = thread_partial((const T *)F.logits, F.vocab, F.slices, row, slice, lt);
        }
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
            const int slice = s0 + r * kFrontGroups + g;
            if (s0 + r * kFrontGroups >= F.slices) break;           // uniform over the workgroup
            sm[tid] = part[r];
            group_merge(sm + g * kFeatThreads, lt);
            if (lt == 0 && slice < F.slices) slice_res[slice] = sm[tid];
        }
    }
    const float V = variance_from_sum_p2(F.sum_p2 + row * F.Hq, F.Hq, F.attn_len[row], (float *)sm, lt, g == 0);
    if (tid == 0) {
        Lse3 a = {-INFINITY, 0.f, 0.f};
        for (int s = 0; s < F.slices; ++s) a = lse3_merge(a, slice_res[s]);
        act[0][0] = entropy_of(a);
        act[0][1] = rarity_from(tok_count, seen);
        act[0][2] = V;
        act[0][3] = confidence_of(a);
        float *f = F.feats + row * 4;
        f[0] = act[0][0]; f[1] = act[0][1]; f[2] = act[0][2]; f[3] = act[0][3];
    }
    __syncthreads();
    const int cur = staged ? mlp_row_forward<true>(M, act, tid, stage) : mlp_row_forward<false>(M, act, tid, nullptr);
    if (tid == 0) {
        const int b = emit_decision(act[cur], 4, row, M.bits, M.logits);
        if (F.advance) advance_one_token(cv, seq, b, pre);
    }
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

template <typename T>
static int launch_lse_partial(const void *logits, int64_t n, int64_t vocab, int slices, float *ws, hipStream_t st)
{
    // beyond what the L2 caches hold together, the logits are streamed
    if ((long long)n * vocab * (long long)sizeof(T) >= (32LL << 20))
        hipLaunchKernelGGL((k_lse_partial<T, true>), dim3(slices, (unsigned)n), dim3(kFeatThreads), 0, st, (const T *)logits, (long long)vocab, slices, ws);
    else
        hipLaunchKernelGGL((k_lse_partial<T, false>), dim3(slices, (unsigned)n), dim3(kFeatThreads), 0, st, (const T *)logits, (long long)vocab, slices, ws);
    KVQ_HIP(hipGetLastError());
    return KVQ_OK;
}

template <typename T>
static int launch_front(const kvq::FrontArgs &F, const kvq::MlpArgs &M, const kvq::CacheView &cv, int64_t n, size_t lds, int staged, hipStream_t st)
{
    static size_t granted = 0;
    const int rc_lds = ensure_dynamic_lds((const void *)k_front<T>, lds, &granted);
    if (rc_lds != KVQ_OK) return rc_lds;
    hipLaunchKernelGGL(k_front<T>, dim3((unsigned)n), dim3(kFrontGroups * kFeatThreads), lds, st, F, M, cv, staged);
    KVQ_HIP(hipGetLastError());
    return KVQ_OK;
}

static int check_logits(const void *logits, int32_t dtype)
{
    if (dtype != KVQ_DTYPE_F32 && dtype != KVQ_DTYPE_F16 && dtype != KVQ_DTYPE_BF16) {
        set_error("logits_dtype %d is not one of KVQ_DTYPE_F32, KVQ_DTYPE_F16, KVQ_DTYPE_BF16", dtype);
        return KVQ_ERR_INVALID_ARG;
    }
    const uintptr_t align = dtype == KVQ_DTYPE_F32 ? 4 : 2;
    if (logits && ((uintptr_t)logits & (align - 1))) { set_error("logits pointer is not aligned to its element size"); return KVQ_ERR_INVALID_ARG; }
    return KVQ_OK;
}

extern "C" int kvq_features_typed(const void *logits, int32_t logits_dtype, int64_t n, int64_t vocab, const int32_t *token_ids,
                                  int64_t *counts, int64_t *totals, int32_t update_counts,
                                  const float *attn_probs, const float *sum_p2, const int32_t *attn_len,
                                  int32_t n_q_heads, int64_t ld, float *feats_out,
                                  void *workspace, size_t workspace_bytes, void *stream)
{
    if (n < 0 || vocab < 1) { set_error("n or vocab out of range"); return KVQ_ERR_INVALID_ARG; }
    const int rc_t = check_logits(logits, logits_dtype);
    if (rc_t != KVQ_OK) return rc_t;
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
    const int rc_l = logits_dtype == KVQ_DTYPE_F32   ? launch_lse_partial<float>(logits, n, vocab, slices, (float *)workspace, st)
                     : logits_dtype == KVQ_DTYPE_F16 ? launch_lse_partial<__half>(logits, n, vocab, slices, (float *)workspace, st)
                                                     : launch_lse_partial<Bf16>(logits, n, vocab, slices, (float *)workspace, st);
    if (rc_l != KVQ_OK) return rc_l;
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

extern "C" int kvq_features(const float *logits, int64_t n, int64_t vocab, const int32_t *token_ids,
                            int64_t *counts, int64_t *totals, int32_t update_counts,
                            const float *attn_probs, const float *sum_p2, const int32_t *attn_len,
                            int32_t n_q_heads, int64_t ld, float *feats_out,
                            void *workspace, size_t workspace_bytes, void *stream)
{
    return kvq_features_typed(logits, KVQ_DTYPE_F32, n, vocab, token_ids, counts, totals, update_counts, attn_probs, sum_p2,
                              attn_len, n_q_heads, ld, feats_out, workspace, workspace_bytes, stream);
}

extern "C" int kvq_features_controller_typed(const void *logits, int32_t logits_dtype, int64_t n, int64_t vocab,
                                             const int32_t *token_ids, int64_t *counts, int64_t *totals, int32_t update_counts,
                                             const float *sum_p2, const int32_t *attn_len, int32_t n_q_heads, const kvq_mlp *mlp,
                                             kvq_cache *cache, const int32_t *seq_ids, float *feats_out, uint8_t *bits_out,
                                             float *logits_out, void *stream)
{
    if (n < 0 || vocab < 1) { set_error("n or vocab out of range"); return KVQ_ERR_INVALID_ARG; }
    const int rc_t = check_logits(logits, logits_dtype);
    if (rc_t != KVQ_OK) return rc_t;
    MlpArgs M;
    const int rc0 = mlp_args_from(mlp, &M, nullptr);
    if (rc0 != KVQ_OK) return rc0;
    if (n == 0) return KVQ_OK;
    if (!logits || !token_ids || !counts || !totals || !sum_p2 || !attn_len || !feats_out || !bits_out) {
        set_error("NULL argument");
        return KVQ_ERR_INVALID_ARG;
    }
    if (n_q_heads < 1) { set_error("n_q_heads must be positive"); return KVQ_ERR_INVALID_ARG; }
    if (n > 65535) { set_error("n above 65535 rows per call is not supported"); return KVQ_ERR_UNSUPPORTED; }
    if (cache && n > cache->desc.max_seqs) { set_error("n %lld exceeds the cache's max_seqs", (long long)n); return KVQ_ERR_INVALID_ARG; }
    FrontArgs F;
    F.logits = logits;
    F.token_ids = token_ids;
    F.counts = (const long long *)counts;
    F.totals = (const long long *)totals;
    F.sum_p2 = sum_p2;
    F.attn_len = attn_len;
    F.seq_ids = seq_ids;
    F.feats = feats_out;
    F.vocab = vocab;
    F.slices = pick_slices(n, vocab);                             // the slicing of kvq_features: same rounding, same values
    F.Hq = n_q_heads;
    F.advance = cache ? 1 : 0;
    M.feats = feats_out;
    M.bits = bits_out;
    M.logits = logits_out;
    M.n = n;
    CacheView cv = {};
    if (cache) cv = cache->view;
    hipStream_t st = (hipStream_t)stream;
    const int stage_floats = mlp_stage_floats(M);
    const int staged = stage_floats <= kMlpStageMaxFloats;
    const size_t lds = staged ? (size_t)stage_floats * sizeof(float) : 0;
    const int rc_f = logits_dtype == KVQ_DTYPE_F32   ? launch_front<float>(F, M, cv, n, lds, staged, st)
                     : logits_dtype == KVQ_DTYPE_F16 ? launch_front<__half>(F, M, cv, n, lds, staged, st)
                                                     : launch_front<Bf16>(F, M, cv, n, lds, staged, st);
    if (rc_f != KVQ_OK) return rc_f;
    if (cache) {                                                   // host-side length bound: the launch is queued
        cache->len_bound += 1;
        if (cache->len_bound > cache->desc.max_context) cache->len_bound = cache->desc.max_context;
    }
    if (update_counts) {
        hipLaunchKernelGGL(k_counts_update, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, token_ids, (long long)n,
                           (long long)vocab, (unsigned long long *)counts, (unsigned long long *)totals);
        KVQ_HIP(hipGetLastError());
    }
    return KVQ_OK;
}

extern "C" int kvq_features_controller(const float *logits, int64_t n, int64_t vocab, const int32_t *token_ids,
                                       int64_t *counts, int64_t *totals, int32_t update_counts, const float *sum_p2,
                                       const int32_t *attn_len, int32_t n_q_heads, const kvq_mlp *mlp, kvq_cache *cache,
                                       const int32_t *seq_ids, float *feats_out, uint8_t *bits_out, float *logits_out,
                                       void *stream)
{
    return kvq_features_controller_typed(logits, KVQ_DTYPE_F32, n, vocab, token_ids, counts, totals, update_counts, sum_p2, attn_len,
                                         n_q_heads, mlp, cache, seq_ids, feats_out, bits_out, logits_out, stream);
}

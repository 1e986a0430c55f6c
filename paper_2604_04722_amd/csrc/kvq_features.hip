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
    // (a 64-bit division is a long emulated routine that would stand in front of the slice's first load)
    const long long per = vocab <= 0x7fffffffLL ? (long long)(((uint32_t)vocab + (uint32_t)slices - 1u) / (uint32_t)slices)
                                                : (vocab + slices - 1) / slices;
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

// ---- wavefront reductions by data-parallel-primitive moves (no LDS traffic) ----------------------------------------
template <int CTRL> __device__ __forceinline__ float dpp_f(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
template <int CTRL> __device__ __forceinline__ Lse3 dpp_lse3(const Lse3 &a)
{
    Lse3 b;
    b.m = dpp_f<CTRL>(a.m); b.s = dpp_f<CTRL>(a.s); b.t = dpp_f<CTRL>(a.t);
    return b;
}
__device__ __forceinline__ Lse3 lane_lse3(const Lse3 &a, int lane)
{
    Lse3 b;
    b.m = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, a.m), lane));
    b.s = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, a.s), lane));
    b.t = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, a.t), lane));
    return b;
}

// Merge of the 64 lanes' triples; the result is wave-uniform.  Pairs inside a quad, quads inside a half row, half rows
// inside a row of 16 lanes (each step joins two disjoint groups), then the four rows in a fixed order.
__device__ __forceinline__ Lse3 lse3_wave_merge(Lse3 a)
{
    a = lse3_merge(a, dpp_lse3<0xB1>(a));       // quad_perm [1,0,3,2]
    a = lse3_merge(a, dpp_lse3<0x4E>(a));       // quad_perm [2,3,0,1]
    a = lse3_merge(a, dpp_lse3<0x141>(a));      // row_half_mirror
    a = lse3_merge(a, dpp_lse3<0x140>(a));      // row_mirror
    return lse3_merge(lse3_merge(lane_lse3(a, 0), lane_lse3(a, 16)), lse3_merge(lane_lse3(a, 32), lane_lse3(a, 48)));
}

__device__ __forceinline__ float wave_sum_f(float v)
{
    v += dpp_f<0xB1>(v);
    v += dpp_f<0x4E>(v);
    v += dpp_f<0x141>(v);
    v += dpp_f<0x140>(v);
    const int i = __builtin_bit_cast(int, v);
    return (__builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 0)) + __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 16))) +
           (__builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 32)) + __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 48)));
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
    // the last levels stay inside the group's first wavefront
    if (lt < 64) {
        const Lse3 a = lse3_wave_merge(sm[lt]);
        if (lt == 0) sm[0] = a;
    }
    __syncthreads();
}

// gather != nullptr (the fused front end): slice 0 of each row also copies what the row's rarity feature needs -- the
// token's count and N + |V_obs| as they stand -- so that the kernel behind this one may count the tokens while it scores
// them: every read of the table then lies in this launch, every update in the next.
template <typename T, bool Stream>
__global__ __launch_bounds__(kFeatThreads) void k_lse_partial(const T *logits, long long vocab, int slices, float *ws,
                                                              const int32_t *token_ids, const long long *counts, const long long *totals,
                                                              long long *gather)
{
    __shared__ Lse3 sm[kFeatThreads];
    const long long row = blockIdx.y;
    const int slice = blockIdx.x;
    // The copy is a chain of dependent reads (token id -> its count): the id is asked for ahead of the logits and the
    // rest follows them, by a thread of the workgroup's last wavefront, which has the least to do in the merge -- in
    // front of the slice's loads the chain made slice 0, and with it the launch, two memory round trips longer.
    const bool copies = gather != nullptr && slice == 0 && threadIdx.x == kFeatThreads - 64;
    long long id = -1, seen = 0;
    if (copies) {
        id = token_ids[row];
        seen = totals[0] + totals[1];
    }
    sm[threadIdx.x] = thread_partial<T, Stream>(logits, vocab, slices, row, slice, threadIdx.x);
    if (copies) {
        gather[row * 2] = (id >= 0 && id < vocab) ? counts[id] : 0;       // an id outside the table counts as unseen
        gather[row * 2 + 1] = seen;
    }
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
// Called by one whole wavefront; the value is wave-uniform.
__device__ __forceinline__ float wave_variance_from_sum_p2(const float *sum_p2_row, int Hq, int l, int lane)
{
    const float inv_l = l > 0 ? 1.0f / (float)l : 0.f;    // l <= 0: no attention row yet, V_t = 0
    float s = 0.f;
    for (int h = lane; h < Hq; h += 64) s += sum_p2_row[h] * inv_l - inv_l * inv_l;
    return wave_sum_f(s) / (float)Hq;
}

// the row's slice triples, lane = slice (at most kMaxSlices = 64 of them), merged by the wavefront
__device__ __forceinline__ Lse3 wave_merge_slices(const float *ws, long long row, int slices, int lane)
{
    Lse3 a = {-INFINITY, 0.f, 0.f};
    if (lane < slices) {
        const float *w = ws + (row * slices + lane) * 4;
        a.m = w[0]; a.s = w[1]; a.t = w[2];
    }
    return lse3_wave_merge(a);
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
    }
    if (threadIdx.x >= 64) return;                   // the first wavefront finishes the row
    if (l > 0 && !A.attn_probs) V = wave_variance_from_sum_p2(A.sum_p2 + t * A.Hq, A.Hq, l, threadIdx.x);
    const Lse3 a = wave_merge_slices(A.ws, t, A.slices, threadIdx.x);
    if (threadIdx.x != 0) return;
    float *f = A.feats + t * 4;
    f[0] = entropy_of(a);
    f[1] = rarity_of(A.token_ids[t], A.vocab, A.counts, A.totals);
    f[2] = V;
    f[3] = confidence_of(a);
}

// ---- fused per-step front end: features, controller, bucket bookkeeping and count update in two launches ----------
//
// The pass over the logits is k_lse_partial's, spread over rows x slices workgroups (one compute unit per row took
// 9 us for 49 152 logits); slice 0 of each row also copies the row's table entries.  This kernel is the rest of the
// row, one workgroup each: the first wavefront merges the slice triples and forms the four features exactly as
// k_features_finalize does; the controller's row shape follows, then the new token's bucket bookkeeping and its count.  Features and logits equal those of the separate
// kernels bit for bit.  No row needs another row's result, and no row reads the table in this launch, so counting
// here keeps "every row reads the table before any count changes".
struct FrontArgs {
    const float *ws;
    const long long *gather;
    const int32_t *token_ids;
    unsigned long long *counts;
    unsigned long long *totals;
    const float *sum_p2;
    const int32_t *attn_len;
    const int32_t *seq_ids;
    float *feats;
    long long vocab, n;
    int slices, Hq, advance, update_counts;
};

__global__ __launch_bounds__(1024) void k_front_tail(FrontArgs F, MlpArgs M, CacheView cv)
{
    __shared__ float part[kRowPartMax];
    __shared__ float act[2][kMaxWidth];
    const long long row = blockIdx.x;
    const int tid = threadIdx.x;
    // Everything the row needs from memory is asked for here, in one batch: the controller's weights (every thread),
    // the gathered count and the sequence's counters and page entries (thread 0), the slice triples (first wavefront).
    const RowPrefetch pf = mlp_row_prefetch(M, tid);
    long long tok_count = 0, seen = 0;
    int seq = 0, pre[5] = {0, 0, 0, 0, 0}, pre_page[kClasses] = {0, 0, 0, 0};
    if (tid == 0) {
        tok_count = F.gather[row * 2];
        seen = F.gather[row * 2 + 1];
        if (F.advance) {
            seq = F.seq_ids ? F.seq_ids[row] : (int)row;
            if (seq >= 0 && seq < cv.max_seqs) {
#pragma unroll
                for (int c = 0; c < 5; ++c) pre[c] = cv.counts[(size_t)seq * 5 + c];
                prefetch_next_pages(cv, seq, pre, pre_page);
            }
        }
    }
    // the count update (c[id] += 1, N += n, |V_obs| += ids seen for the first time) is the second wavefront's first
    // lane's: it depends on nothing this kernel computes and runs beside the rest
    if (tid == 64 && F.update_counts) {
        if (row == 0) atomicAdd(&F.totals[0], (unsigned long long)F.n);
        const long long id = F.token_ids[row];
        if (id >= 0 && id < F.vocab) {
            const unsigned long long old = atomicAdd(&F.counts[id], 1ull);
            if (old == 0ull) atomicAdd(&F.totals[1], 1ull);
        }
    }
    Lse3 mine = {-INFINITY, 0.f, 0.f};
    int l = 0;
    if (tid < 64) {
        l = F.attn_len[row];
        if (tid < F.slices) {
            const float *w = F.ws + (row * F.slices + tid) * 4;
            mine.m = w[0]; mine.s = w[1]; mine.t = w[2];
        }
    }
    if (tid < 64) {
        const float V = wave_variance_from_sum_p2(F.sum_p2 + row * F.Hq, F.Hq, l, tid);      // (its loads travel with the triples')
        const Lse3 a = lse3_wave_merge(mine);
        if (tid == 0) {
            act[0][0] = entropy_of(a);
            act[0][1] = rarity_from(tok_count, seen);
            act[0][2] = V;
            act[0][3] = confidence_of(a);
            float *f = F.feats + row * 4;
            f[0] = act[0][0]; f[1] = act[0][1]; f[2] = act[0][2]; f[3] = act[0][3];
        }
    }
    __syncthreads();
    const int cur = mlp_row_forward(M, act, part, tid, (int)blockDim.x, pf);
    if (tid == 0) {
        const int b = emit_decision(act[cur], 4, row, M.bits, M.logits);
        if (F.advance) advance_one_token(cv, seq, b, pre, pre_page);
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
    const long long max_by_len = (vocab + 1023) / 1024;   // at least 1024 logits per slice: one 16-byte load per thread
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
    // slice triples of every row, then (fused front end) the row's gathered table entries
    return (size_t)n * kMaxSlices * 4 * sizeof(float) + (size_t)n * 2 * sizeof(long long) + 256;
}

template <typename T>
static int launch_lse_partial(const void *logits, int64_t n, int64_t vocab, int slices, float *ws, const int32_t *token_ids,
                              const int64_t *counts, const int64_t *totals, long long *gather, hipStream_t st)
{
    // beyond what the L2 caches hold together, the logits are streamed
    if ((long long)n * vocab * (long long)sizeof(T) >= (32LL << 20))
        hipLaunchKernelGGL((k_lse_partial<T, true>), dim3(slices, (unsigned)n), dim3(kFeatThreads), 0, st, (const T *)logits, (long long)vocab, slices, ws,
                           token_ids, (const long long *)counts, (const long long *)totals, gather);
    else
        hipLaunchKernelGGL((k_lse_partial<T, false>), dim3(slices, (unsigned)n), dim3(kFeatThreads), 0, st, (const T *)logits, (long long)vocab, slices, ws,
                           token_ids, (const long long *)counts, (const long long *)totals, gather);
    KVQ_HIP(hipGetLastError());
    return KVQ_OK;
}

static int launch_lse_partial_typed(int32_t dtype, const void *logits, int64_t n, int64_t vocab, int slices, float *ws,
                                    const int32_t *token_ids, const int64_t *counts, const int64_t *totals, long long *gather, hipStream_t st)
{
    return dtype == KVQ_DTYPE_F32   ? launch_lse_partial<float>(logits, n, vocab, slices, ws, token_ids, counts, totals, gather, st)
           : dtype == KVQ_DTYPE_F16 ? launch_lse_partial<__half>(logits, n, vocab, slices, ws, token_ids, counts, totals, gather, st)
                                    : launch_lse_partial<Bf16>(logits, n, vocab, slices, ws, token_ids, counts, totals, gather, st);
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
    const int rc_l = launch_lse_partial_typed(logits_dtype, logits, n, vocab, slices, (float *)workspace, nullptr, nullptr, nullptr, nullptr, st);
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
                                             float *logits_out, void *workspace, size_t workspace_bytes, void *stream)
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
    const size_t need = kvq_features_workspace(n, vocab) - 256;
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 15)) {
        set_error("workspace too small or not 16-byte aligned: %zu bytes given, %zu needed", workspace_bytes, need);
        return KVQ_ERR_INVALID_ARG;
    }
    hipStream_t st = (hipStream_t)stream;
    const int slices = pick_slices(n, vocab);                      // the slicing of kvq_features: same rounding, same values
    float *ws = (float *)workspace;
    long long *gather = (long long *)((char *)workspace + (size_t)n * kMaxSlices * 4 * sizeof(float));
    const int rc_l = launch_lse_partial_typed(logits_dtype, logits, n, vocab, slices, ws, token_ids, counts, totals, gather, st);
    if (rc_l != KVQ_OK) return rc_l;
    FrontArgs F;
    F.ws = ws;
    F.gather = gather;
    F.token_ids = token_ids;
    F.counts = (unsigned long long *)counts;
    F.totals = (unsigned long long *)totals;
    F.sum_p2 = sum_p2;
    F.attn_len = attn_len;
    F.seq_ids = seq_ids;
    F.feats = feats_out;
    F.vocab = vocab;
    F.n = n;
    F.slices = slices;
    F.Hq = n_q_heads;
    F.advance = cache ? 1 : 0;
    F.update_counts = update_counts ? 1 : 0;
    M.feats = feats_out;
    M.bits = bits_out;
    M.logits = logits_out;
    M.n = n;
    CacheView cv = {};
    if (cache) cv = cache->view;
    // a 128 x 128 layer is one work item per thread of a 1024-thread workgroup; with many rows workgroups of that size
    // would only queue up
    hipLaunchKernelGGL(k_front_tail, dim3((unsigned)n), dim3(n <= 256 ? 1024 : kRowThreads), 0, st, F, M, cv);
    KVQ_HIP(hipGetLastError());
    if (cache) {                                                   // host-side length bound: the launch is queued
        cache->len_bound += 1;
        if (cache->len_bound > cache->desc.max_context) cache->len_bound = cache->desc.max_context;
        cache->touched = true;
    }
    return KVQ_OK;
}

extern "C" int kvq_features_controller(const float *logits, int64_t n, int64_t vocab, const int32_t *token_ids,
                                       int64_t *counts, int64_t *totals, int32_t update_counts, const float *sum_p2,
                                       const int32_t *attn_len, int32_t n_q_heads, const kvq_mlp *mlp, kvq_cache *cache,
                                       const int32_t *seq_ids, float *feats_out, uint8_t *bits_out, float *logits_out,
                                       void *workspace, size_t workspace_bytes, void *stream)
{
    return kvq_features_controller_typed(logits, KVQ_DTYPE_F32, n, vocab, token_ids, counts, totals, update_counts, sum_p2, attn_len,
                                         n_q_heads, mlp, cache, seq_ids, feats_out, bits_out, logits_out, workspace, workspace_bytes, stream);
}

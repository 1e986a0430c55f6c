// Single-query decode attention over the precision-bucketed cache (paper Sec. 3.2:
// a = Softmax(q K^T / sqrt(d_k)) V, evaluated over k^, v^ of Sec. 3.7 at heterogeneous precision).
//
// Mapping.  A wavefront streams blocks of 64 tokens, lane = token.  Because a token's K (or V)
// vector is stored as NCH chunks of 16 bytes, chunk-major inside the block, every 16-byte-per-lane
// load instruction of the wave covers 1 KiB of consecutive memory.  The query is wave-uniform, so
// q . k^_j needs no cross-lane traffic at all: each lane dots its own token's codes with q pairs
// (v_dot2_f32_f16).  For V each lane scales its token's codes by its softmax weight into 64 fp32
// accumulators; the 64 lanes are summed once, when the wave has consumed all its blocks.
//
// Dequantization is folded out of the element loop.  A b-bit code c is turned into the fp16 number
// h = 1 + c*2^-S (or 1024 + c for 8 bit) by one shift and one and-or that drops the code into the
// mantissa of a constant; then x^ = min + scale*c = (min - OFF*scale) + (MUL*scale)*h, so that
//   q . k^_j      = (min - OFF*scale) * sum(q)  +  MUL*scale * (q . h_j)
//   sum_j p_j v^_j = sum_j p_j (min_j - OFF*scale_j)  +  sum_j (p_j MUL scale_j) h_j
// and the per-element work is extract + one dot2 (K) or extract + two mixed fp16->fp32 FMAs (V).
#include "kvq_internal.h"

namespace kvq {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kScoreScale = 0.125f * kLog2e;     // 1/sqrt(64), and exp(x) = exp2(x*log2 e)
constexpr int kPartialFloats = 68;                 // 64 channels, m, l, l2, pad
constexpr int kMaxSplits = 64;

template <int C> struct Cls;
template <> struct Cls<0> { static constexpr int BITS = 2, U = 4, NCH = 1, PAIRS = 8; static constexpr float OFF = 4.f, MUL = 4.f; };
template <> struct Cls<1> { static constexpr int BITS = 4, U = 2, NCH = 2, PAIRS = 4; static constexpr float OFF = 64.f, MUL = 64.f; };
template <> struct Cls<2> { static constexpr int BITS = 8, U = 1, NCH = 4, PAIRS = 2; static constexpr float OFF = 1024.f, MUL = 1.f; };
template <> struct Cls<3> { static constexpr int BITS = 16, U = 1, NCH = 8, PAIRS = 1; static constexpr float OFF = 0.f, MUL = 1.f; };

__device__ __forceinline__ half2_t as_h2(uint32_t u) { return __builtin_bit_cast(half2_t, u); }

// The pair (2m, 2m+1) of a word as two fp16 numbers h = f(code); p is a compile-time constant.
template <int C> __device__ __forceinline__ half2_t extract_pair(uint32_t w, int p)
{
    if constexpr (C == 0) {            // codes at bits 2p and 2p+16 -> mantissa bits [8,10): h = 1 + c/4
        const int sh = 8 - 2 * p;
        const uint32_t t = sh > 0 ? (w << sh) : sh < 0 ? (w >> (-sh)) : w;
        return as_h2((t & 0x03000300u) | 0x3C003C00u);
    } else if constexpr (C == 1) {     // codes at bits 4p and 4p+16 -> mantissa bits [4,8): h = 1 + c/64
        const int sh = 4 - 4 * p;
        const uint32_t t = sh > 0 ? (w << sh) : sh < 0 ? (w >> (-sh)) : w;
        return as_h2((t & 0x00F000F0u) | 0x3C003C00u);
    } else if constexpr (C == 2) {     // bytes p and p+2 under the exponent byte 0x64: h = 1024 + c
        return as_h2(__builtin_amdgcn_perm(0x64646464u, w, p == 0 ? 0x04020400u : 0x04030401u));
    } else {
        return as_h2(w);
    }
}

template <int CTRL> __device__ __forceinline__ float dpp_mov(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

// max / sum over the 64 lanes; the result is wave-uniform
__device__ __forceinline__ float wave_max(float v)
{
    v = fmaxf(v, dpp_mov<0xB1>(v));    // quad_perm [1,0,3,2]
    v = fmaxf(v, dpp_mov<0x4E>(v));    // quad_perm [2,3,0,1]
    v = fmaxf(v, dpp_mov<0x141>(v));   // row_half_mirror
    v = fmaxf(v, dpp_mov<0x140>(v));   // row_mirror: every lane of a row now holds the row's max
    const float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 0));
    const float b = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 16));
    const float c = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 32));
    const float d = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 48));
    return fmaxf(fmaxf(a, b), fmaxf(c, d));
}

__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_mov<0xB1>(v);
    v += dpp_mov<0x4E>(v);
    v += dpp_mov<0x141>(v);
    v += dpp_mov<0x140>(v);
    const float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 0));
    const float b = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 16));
    const float c = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 32));
    const float d = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 48));
    return (a + b) + (c + d);
}

struct WaveState {
    float m;          // running maximum of the scaled scores (log2 units), wave-uniform
    float l, l2;      // per lane: sum p, sum p^2 relative to m
    float zacc;       // per lane: sum p * (min - OFF*scale) of V
    float acc[kD];    // per lane: sum (p*MUL*scale) * h
};

struct AttnParams {
    CacheView cv;
    const uint32_t *q;          // [n_seq][Hq][32] fp16 pairs
    const int32_t *seq_ids;
    float *out, *lse, *p2, *ws;
    int32_t layer, n_seq, S;
};

template <int C> struct KRegs { uint2 meta[Cls<C>::U]; uint4 kc[Cls<C>::U][Cls<C>::NCH]; };
template <int C> struct VRegs { uint4 vc[Cls<C>::U][Cls<C>::NCH]; };

// byte offsets of the lanes' tokens inside a unit, with lanes past the end of the bucket redirected to
// token 0 of the unit (which always exists), so that every load is in bounds and reads finite data
template <int C> struct UnitAddr {
    const uint8_t *base;                       // unit base (first block of the unit)
    uint32_t tokoff[Cls<C>::U];                // block offset + token*16 for chunk loads
    uint32_t metaoff[Cls<C>::U];
    bool valid[Cls<C>::U];
};

template <int C>
__device__ __forceinline__ void unit_addr(UnitAddr<C> &ua, const uint8_t *base, int ntok, int lane)
{
    constexpr int BB = class_block_bytes(C);
    ua.base = base;
#pragma unroll
    for (int u = 0; u < Cls<C>::U; ++u) {
        const bool ok = u * kBlockTokens + lane < ntok;
        ua.valid[u] = ok;
        const uint32_t blk = ok ? (uint32_t)u : 0u;
        const uint32_t tok = ok ? (uint32_t)lane : 0u;
        ua.tokoff[u] = blk * BB + class_meta_bytes(C) + tok * 16u;
        ua.metaoff[u] = blk * BB + tok * 8u;
    }
}

template <int C> __device__ __forceinline__ void load_k(KRegs<C> &r, const UnitAddr<C> &ua)
{
#pragma unroll
    for (int u = 0; u < Cls<C>::U; ++u) {
        if constexpr (C != 3) r.meta[u] = *(const uint2 *)(ua.base + ua.metaoff[u]);
#pragma unroll
        for (int ch = 0; ch < Cls<C>::NCH; ++ch)
            r.kc[u][ch] = *(const uint4 *)(ua.base + ua.tokoff[u] + ch * (kBlockTokens * 16));
    }
}

template <int C> __device__ __forceinline__ void load_v(VRegs<C> &r, const UnitAddr<C> &ua)
{
    constexpr int VOFF = Cls<C>::NCH * kBlockTokens * 16;
#pragma unroll
    for (int u = 0; u < Cls<C>::U; ++u)
#pragma unroll
        for (int ch = 0; ch < Cls<C>::NCH; ++ch)
            r.vc[u][ch] = *(const uint4 *)(ua.base + ua.tokoff[u] + VOFF + ch * (kBlockTokens * 16));
}

__device__ __forceinline__ uint32_t word_of(const uint4 &v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }

__device__ __forceinline__ float half_lo(uint32_t u) { return (float)__builtin_bit_cast(half2_t, u).x; }
__device__ __forceinline__ float half_hi(uint32_t u) { return (float)__builtin_bit_cast(half2_t, u).y; }

// K stage of one unit: scores, running-max update, softmax weights.  Leaves in a[u] the factor that
// multiplies h of V (p*MUL*scale_v) for each of the unit's blocks.
template <int C>
__device__ __forceinline__ void compute_k(const KRegs<C> &r, const UnitAddr<C> &ua, const uint32_t (&q2)[32], float qs,
                                          WaveState &st, float (&a)[Cls<C>::U])
{
    constexpr int U = Cls<C>::U, NCH = Cls<C>::NCH, PAIRS = Cls<C>::PAIRS;
    float sc[U];
    float lmax = -INFINITY;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        float d0 = 0.f, d1 = 0.f;
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch)
#pragma unroll
            for (int wi = 0; wi < 4; ++wi) {
                const uint32_t w = word_of(r.kc[u][ch], wi);
#pragma unroll
                for (int p = 0; p < PAIRS; ++p) {
                    const int m = (ch * 4 + wi) * PAIRS + p;
                    const half2_t h = extract_pair<C>(w, p);
                    if (m & 1) d1 = __builtin_amdgcn_fdot2(h, as_h2(q2[m]), d1, false);
                    else       d0 = __builtin_amdgcn_fdot2(h, as_h2(q2[m]), d0, false);
                }
            }
        const float dot = d0 + d1;
        float s;
        if constexpr (C == 3) {
            s = dot * kScoreScale;
        } else {
            const float ks = half_lo(r.meta[u].x), kz = half_hi(r.meta[u].x);
            // q.k^ = (min - OFF*scale) * sum(q) + MUL*scale * (q.h); qs = sum(q)*kScoreScale
            s = (kz - Cls<C>::OFF * ks) * qs + (ks * (Cls<C>::MUL * kScoreScale)) * dot;
        }
        sc[u] = ua.valid[u] ? s : -INFINITY;
        lmax = fmaxf(lmax, sc[u]);
    }
    const float wm = wave_max(lmax);
    if (wm > st.m) {                               // wave-uniform branch
        const float f = __builtin_amdgcn_exp2f(st.m - wm);   // st.m = -inf on the first unit: f = 0
        st.l *= f;
        st.l2 *= f * f;
        st.zacc *= f;
#pragma unroll
        for (int c = 0; c < kD; ++c) st.acc[c] *= f;
        st.m = wm;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const float p = __builtin_amdgcn_exp2f(sc[u] - st.m);
        st.l += p;
        st.l2 = fmaf(p, p, st.l2);
        if constexpr (C == 3) {
            a[u] = p;
        } else {
            const float vs = half_lo(r.meta[u].y), vz = half_hi(r.meta[u].y);
            a[u] = p * (Cls<C>::MUL * vs);
            st.zacc = fmaf(p, vz - Cls<C>::OFF * vs, st.zacc);
        }
    }
}

template <int C>
__device__ __forceinline__ void compute_v(const VRegs<C> &r, const float (&a)[Cls<C>::U], WaveState &st)
{
    constexpr int U = Cls<C>::U, NCH = Cls<C>::NCH, PAIRS = Cls<C>::PAIRS;
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch)
#pragma unroll
            for (int wi = 0; wi < 4; ++wi) {
                const uint32_t w = word_of(r.vc[u][ch], wi);
#pragma unroll
                for (int p = 0; p < PAIRS; ++p) {
                    const int m = (ch * 4 + wi) * PAIRS + p;
                    const half2_t h = extract_pair<C>(w, p);
                    st.acc[2 * m] = fmaf(a[u], (float)h.x, st.acc[2 * m]);
                    st.acc[2 * m + 1] = fmaf(a[u], (float)h.y, st.acc[2 * m + 1]);
                }
            }
}

// All units [first, end) with stride `stride` of class C for one (sequence, kv-head, layer).
template <int C>
__device__ __forceinline__ void process_class(const CacheView &cv, int layer, int seq, int kvh, int cnt, int first, int end,
                                              int stride, int lane, const uint32_t (&q2)[32], float qs, WaveState &st)
{
    if (first >= end) return;
    constexpr int U = Cls<C>::U;
    constexpr int UT = U * kBlockTokens;               // tokens per unit
    const int32_t *pt = cv.page_table + ((size_t)seq * kClasses + C) * cv.max_pages_per_seq;
    const uint8_t *pool = cv.pool[C] + (size_t)layer * cv.layer_stride[C];
    const int upp = cv.blocks_per_page / U;            // units per page
    auto unit_base = [&](int ui) -> const uint8_t * {
        const int page = __builtin_amdgcn_readfirstlane(pt[ui / upp]);
        const int blk = (ui % upp) * U;
        return pool + (((size_t)page * cv.Hkv + kvh) * cv.blocks_per_page + blk) * (size_t)class_block_bytes(C);
    };
    KRegs<C> kr;
    VRegs<C> vr;
    UnitAddr<C> ua;
    int ui = first;
    unit_addr<C>(ua, unit_base(ui), min(cnt - ui * UT, UT), lane);
    load_k<C>(kr, ua);
    while (true) {
        load_v<C>(vr, ua);
        float a[U];
        compute_k<C>(kr, ua, q2, qs, st, a);
        const int un = ui + stride;
        const bool more = un < end;
        if (more) {
            unit_addr<C>(ua, unit_base(un), min(cnt - un * UT, UT), lane);
            load_k<C>(kr, ua);
        }
        compute_v<C>(vr, a, st);
        if (!more) break;
        ui = un;
    }
}

__device__ __forceinline__ int ceil_div_pos(long long a, int b) { return (int)((a + b - 1) / b); }

template <int NW>
__global__ __launch_bounds__(NW * 64) void k_decode_split(AttnParams P)
{
    const CacheView &cv = P.cv;
    const int G = cv.Hq / cv.Hkv;
    const int S = P.S;
    const int nunits = P.n_seq * cv.Hq * S;
    // Workgroups are dealt to the 8 XCDs round-robin by id.  Give each XCD a contiguous range of work
    // items instead, so that the G query heads that share one kv-head's bytes also share one L2.
    const int per_xcd = (nunits + 7) >> 3;
    const int unit = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((blockIdx.x >> 3) >= per_xcd || unit >= nunits) return;
    // unit = ((si*Hkv + kvh)*S + s)*G + g
    int r = unit;
    const int g = r % G; r /= G;
    const int s = r % S; r /= S;
    const int kvh = r % cv.Hkv;
    const int si = r / cv.Hkv;
    const int qh = kvh * G + g;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int seq = P.seq_ids ? P.seq_ids[si] : si;
    const bool seq_ok = seq >= 0 && seq < cv.max_seqs;
    if (!seq_ok) seq = 0;

    // the query as 32 fp16 pairs (wave-uniform) and sum(q)
    uint32_t q2[32];
    const uint32_t *qp = P.q + ((size_t)si * cv.Hq + qh) * 32;
    float qsum = 0.f;
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        q2[i] = qp[i];
        qsum += half_lo(q2[i]) + half_hi(q2[i]);
    }
    const float qs = qsum * kScoreScale;

    WaveState st;
    st.m = -INFINITY;
    st.l = st.l2 = st.zacc = 0.f;
#pragma unroll
    for (int c = 0; c < kD; ++c) st.acc[c] = 0.f;

    // This workgroup's share of the (sequence, kv-head)'s units: the units of the four classes form one
    // list, weighted by their bytes; split s takes the units whose start weight falls into its 1/S of the
    // total.  Inside the workgroup the list is dealt to the waves round-robin.
    int cnt[kClasses], nu[kClasses];
    constexpr int wgt[kClasses] = {20, 18, 17, 32};         // unit bytes / 512
    long long wtot = 0;
#pragma unroll
    for (int c = 0; c < kClasses; ++c) {
        cnt[c] = seq_ok ? cv.counts[(size_t)seq * 5 + c] : 0;
        nu[c] = (cnt[c] + class_unit_blocks(c) * kBlockTokens - 1) / (class_unit_blocks(c) * kBlockTokens);
        wtot += (long long)nu[c] * wgt[c];
    }
    const long long lo_w = wtot * s / S, hi_w = wtot * (s + 1) / S;
    long long wbase = 0;
    int dealt = 0;
    int first[kClasses], last[kClasses];
#pragma unroll
    for (int c = 0; c < kClasses; ++c) {
        const long long a = lo_w - wbase, b = hi_w - wbase;
        int klo = a <= 0 ? 0 : ceil_div_pos(a, wgt[c]);
        int khi = b <= 0 ? 0 : ceil_div_pos(b, wgt[c]);
        klo = min(klo, nu[c]);
        khi = min(khi, nu[c]);
        first[c] = klo + ((wave + NW - (dealt % NW)) % NW);
        last[c] = khi;
        dealt += khi - klo;
        wbase += (long long)nu[c] * wgt[c];
    }
    process_class<0>(cv, P.layer, seq, kvh, cnt[0], first[0], last[0], NW, lane, q2, qs, st);
    process_class<1>(cv, P.layer, seq, kvh, cnt[1], first[1], last[1], NW, lane, q2, qs, st);
    process_class<2>(cv, P.layer, seq, kvh, cnt[2], first[2], last[2], NW, lane, q2, qs, st);
    process_class<3>(cv, P.layer, seq, kvh, cnt[3], first[3], last[3], NW, lane, q2, qs, st);

    // ---- sum the 64 lanes: a transposing butterfly leaves channel c's total in lane c ----------------
#pragma unroll
    for (int half = 32; half >= 1; half >>= 1) {
        const bool upper = (lane & half) != 0;
#pragma unroll
        for (int i = 0; i < half; ++i) {
            const float keep = upper ? st.acc[i + half] : st.acc[i];
            const float send = upper ? st.acc[i] : st.acc[i + half];
            st.acc[i] = keep + __shfl_xor(send, half, 64);
        }
    }
    const float l = wave_sum(st.l), l2 = wave_sum(st.l2), z = wave_sum(st.zacc);
    const float mine = st.acc[0] + z;                      // channel `lane`, relative to exp2(m)

    __shared__ float sm[NW][kPartialFloats];
    sm[wave][lane] = mine;
    if (lane == 0) { sm[wave][64] = st.m; sm[wave][65] = l; sm[wave][66] = l2; }
    __syncthreads();
    if (wave != 0) return;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) M = fmaxf(M, sm[w][64]);
    float o = 0.f, L = 0.f, L2 = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const float mw = sm[w][64];
        const float f = mw == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mw - M);
        o = fmaf(f, sm[w][lane], o);
        L = fmaf(f, sm[w][65], L);
        L2 = fmaf(f * f, sm[w][66], L2);
    }
    if (S == 1) {
        const size_t oi = (size_t)si * cv.Hq + qh;
        const float inv = L > 0.f ? 1.0f / L : 0.f;
        P.out[oi * kD + lane] = o * inv;
        if (lane == 0) {
            if (P.lse) P.lse[oi] = L > 0.f ? (M + __builtin_amdgcn_logf(L)) * kLn2 : -INFINITY;
            if (P.p2) P.p2[oi] = L2 * inv * inv;
        }
    } else {
        float *w = P.ws + (size_t)unit * kPartialFloats;
        w[lane] = o;
        if (lane == 0) { w[64] = M; w[65] = L; w[66] = L2; }
    }
}

// Merge the S partial results of each (sequence, query head): one wavefront each, lane = channel.
__global__ __launch_bounds__(256) void k_decode_combine(const float *ws, int n_seq, int Hq, int Hkv, int S,
                                                        float *out, float *lse, float *p2)
{
    const int oi = (blockIdx.x * 256 + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (oi >= n_seq * Hq) return;
    const int G = Hq / Hkv;
    const int si = oi / Hq, qh = oi % Hq;
    const int kvh = qh / G, g = qh % G;
    const size_t u0 = ((size_t)(si * Hkv + kvh) * S) * G + g;
    float M = -INFINITY;
    for (int s = 0; s < S; ++s) M = fmaxf(M, ws[(u0 + (size_t)s * G) * kPartialFloats + 64]);
    float o = 0.f, L = 0.f, L2 = 0.f;
    for (int s = 0; s < S; ++s) {
        const float *w = ws + (u0 + (size_t)s * G) * kPartialFloats;
        const float mw = w[64];
        const float f = mw == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mw - M);
        o = fmaf(f, w[lane], o);
        L = fmaf(f, w[65], L);
        L2 = fmaf(f * f, w[66], L2);
    }
    const float inv = L > 0.f ? 1.0f / L : 0.f;
    out[(size_t)oi * kD + lane] = o * inv;
    if (lane == 0) {
        if (lse) lse[oi] = L > 0.f ? (M + __builtin_amdgcn_logf(L)) * kLn2 : -INFINITY;
        if (p2) p2[oi] = L2 * inv * inv;
    }
}

static int env_int(const char *name, int dflt)
{
    const char *e = getenv(name);
    if (!e || !*e) return dflt;
    return atoi(e);
}

}  // namespace kvq

using namespace kvq;

extern "C" size_t kvq_decode_attn_workspace(const kvq_cache *cache, int32_t n_seq)
{
    if (!cache || n_seq < 0) return 0;
    return (size_t)n_seq * cache->desc.n_q_heads * kMaxSplits * kPartialFloats * sizeof(float) + 256;
}

extern "C" int kvq_decode_attn(const kvq_cache *cache, int32_t layer, const void *q, const int32_t *seq_ids,
                               int32_t n_seq, float *out, float *lse_out, float *sum_p2_out,
                               void *workspace, size_t workspace_bytes, void *stream)
{
    if (!cache || !q || !out) { set_error("cache, q or out is NULL"); return KVQ_ERR_INVALID_ARG; }
    const kvq_cache_desc &d = cache->desc;
    if (layer < 0 || layer >= d.n_layers) { set_error("layer %d out of range", layer); return KVQ_ERR_INVALID_ARG; }
    if (n_seq < 0 || n_seq > d.max_seqs) { set_error("n_seq %d out of range (max_seqs %d)", n_seq, d.max_seqs); return KVQ_ERR_INVALID_ARG; }
    if (n_seq == 0) return KVQ_OK;
    const long long heads = (long long)n_seq * d.n_q_heads;
    // Split heuristic: enough workgroups to fill 256 CUs several times over, but at least ~8 units of
    // roughly 10-16 KiB per workgroup.  len_bound is an upper bound of the longest sequence.
    const long long est_units = (cache->len_bound + 63) / 64;
    long long S = (2048 + heads - 1) / heads;
    if (S > est_units / 8) S = est_units / 8;
    if (S < 1) S = 1;
    if (S > kMaxSplits) S = kMaxSplits;
    const int forced = env_int("KVQ_ATTN_SPLITS", 0);
    if (forced >= 1 && forced <= kMaxSplits) S = forced;
    if (heads * S > 0x3fffffffLL) { set_error("too many work items"); return KVQ_ERR_CAPACITY; }
    if (S > 1) {
        const size_t need = (size_t)heads * S * kPartialFloats * sizeof(float);
        if (!workspace || workspace_bytes < need) {
            set_error("workspace too small: %zu bytes given, %zu needed", workspace_bytes, need);
            return KVQ_ERR_INVALID_ARG;
        }
    }
    AttnParams P;
    P.cv = cache->view;
    P.q = (const uint32_t *)q;
    P.seq_ids = seq_ids;
    P.out = out;
    P.lse = lse_out;
    P.p2 = sum_p2_out;
    P.ws = (float *)workspace;
    P.layer = layer;
    P.n_seq = n_seq;
    P.S = (int)S;
    const int nunits = (int)(heads * S);
    const unsigned grid = (unsigned)(((nunits + 7) / 8) * 8);
    hipStream_t st = (hipStream_t)stream;
    const int nw = env_int("KVQ_ATTN_WAVES", 4);
    if (nw == 1) hipLaunchKernelGGL(k_decode_split<1>, dim3(grid), dim3(64), 0, st, P);
    else if (nw == 2) hipLaunchKernelGGL(k_decode_split<2>, dim3(grid), dim3(128), 0, st, P);
    else if (nw == 8) hipLaunchKernelGGL(k_decode_split<8>, dim3(grid), dim3(512), 0, st, P);
    else hipLaunchKernelGGL(k_decode_split<4>, dim3(grid), dim3(256), 0, st, P);
    KVQ_HIP(hipGetLastError());
    if (S > 1) {
        hipLaunchKernelGGL(k_decode_combine, dim3((unsigned)((heads + 3) / 4)), dim3(256), 0, st, (const float *)workspace,
                           n_seq, d.n_q_heads, d.n_kv_heads, (int)S, out, lse_out, sum_p2_out);
        KVQ_HIP(hipGetLastError());
    }
    return KVQ_OK;
}

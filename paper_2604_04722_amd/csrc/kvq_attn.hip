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
// Dequantization is folded out of the element loop.  A b-bit code c is turned into an fp16 number
// h = 1 + c/M by ONE and-or that drops the code bits into the mantissa of the constant 1.0, wherever
// in the mantissa they happen to sit (M = 2^(10 - bit position)); a shift is only needed for codes that
// lie outside the mantissa window, and one shifted word serves two or three code pairs ("targets" with
// different M).  For 8 bit a byte permute builds h = 1024 + c.  Then, with x^ = min + scale*c,
//   q . k^_j       = min_j * sum(q) + scale_j * ( sum_t M_t (q . h_j)_t  -  sum_t M_t sum(q)_t )
//   sum_j p_j v^_j = sum_j p_j min_j  -  M_t(c) * sum_j p_j scale_j  +  sum_j (p_j scale_j M_t(c)) h_jc
// so the per-element work is an and-or plus one packed dot (K) or two mixed fp16->fp32 FMAs (V), and
// the constant parts are carried as four extra accumulators per lane.
//
// Pipeline.  Every class streams through the same four 8-VGPR stage buffers (one stage = two
// 16-byte loads per lane = 2 KiB per wave): [K, V] of two consecutive units (2 and 4 bit), the four
// chunk pairs K01 K23 V01 V23 of an 8-bit block, or the eight chunk pairs of an FP16 block.  A buffer
// is reloaded as soon as it has been consumed, so three stages are always in flight behind the one
// being computed.
#include "kvq_internal.h"
#include "kvq_quant.h"

#include <mutex>

namespace kvq {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kScoreScale = 0.125f * kLog2e;     // 1/sqrt(64), and exp(x) = exp2(x*log2 e)
constexpr int kPartialFloats = 68;                 // 64 channels, m, l, l2, pad
constexpr int kMaxSplits = 64;

// U: blocks per unit; NCH: 16-byte chunks per vector; NT: extraction targets
template <int C> struct Cls;
template <> struct Cls<0> { static constexpr int U = 2, NCH = 1, NT = 3; };
template <> struct Cls<1> { static constexpr int U = 1, NCH = 2, NT = 2; };
template <> struct Cls<2> { static constexpr int U = 1, NCH = 4, NT = 1; };
template <> struct Cls<3> { static constexpr int U = 1, NCH = 8, NT = 1; };

// Relative cost of one unit of each class (2 bit: 128 tokens, 5 KiB; 4 bit: 64 tokens, 4.5 KiB; 8 bit: 8.5 KiB;
// FP16: 16 KiB), by which a (sequence, head)'s units are cut into ranges for its waves.  Bytes alone would give
// 10:9:17:32; the low-bit units also cost vector-ALU time for unpacking.  Two sets, both measured:
//   kUnitCost       every wave of the launch resident at once: the kernel's length is what the memory system gives all
//                   waves together, and these ratios (each class's time per unit when streamed alone) are the fastest;
//   kUnitCostRounds more workgroups than places (several rounds): a workgroup keeps its place until its slower wave is
//                   done, so the ratios that make a workgroup's waves END together win (time stamps on a ragged batch of
//                   64: 171 / 142 us per wave with the first set, 162 / 159 us with this one, the kernel 430 -> 416 us).
constexpr int kUnitCost[4] = {14, 11, 17, 32};
constexpr int kUnitCostRounds[4] = {26, 16, 17, 32};

// target multipliers M: h = 1 + c/M
#define KVQ_M0_0 4.f      /* 2-bit codes at mantissa bits [8,10) */
#define KVQ_M0_1 16.f     /*                              [6,8)  */
#define KVQ_M0_2 64.f     /*                              [4,6)  */
#define KVQ_M1_0 16.f     /* 4-bit codes at mantissa bits [6,10) */
#define KVQ_M1_1 256.f    /*                              [2,6)  */
#define KVQ_OFF2 1024.f   /* 8-bit: h = 1024 + c */

// target of pair p inside a word (see the extraction macros below)
__host__ __device__ constexpr int target0(int p) { return (p == 1 || p == 4 || p == 7) ? 0 : (p == 0 || p == 3 || p == 6) ? 1 : 2; }
__host__ __device__ constexpr int target1(int p) { return (p & 1) ? 0 : 1; }

__device__ __forceinline__ half2_t as_h2(uint32_t u) { return __builtin_bit_cast(half2_t, u); }

// (x & mask) | one.  VOP3 instructions of this target cannot carry 32-bit literals, so the masks are handed
// to the compiler as opaque SGPR values and the constant 1.0|1.0 as an opaque VGPR value (see Consts): the
// expression then selects to a single v_and_or_b32.
__device__ __forceinline__ uint32_t and_or(uint32_t x, uint32_t mask, uint32_t one) { return (x & mask) | one; }

struct Consts {
    uint32_t one;        // 0x3C003C00 in a VGPR
    uint32_t m2[3];      // 2-bit target masks (SGPRs)
    uint32_t m4[2];      // 4-bit target masks (SGPRs)
};

__device__ __forceinline__ Consts make_consts()
{
    Consts c;
    asm volatile("v_mov_b32 %0, 0x3c003c00" : "=v"(c.one));
    asm volatile("s_mov_b32 %0, 0x03000300" : "=s"(c.m2[0]));
    asm volatile("s_mov_b32 %0, 0x00c000c0" : "=s"(c.m2[1]));
    asm volatile("s_mov_b32 %0, 0x00300030" : "=s"(c.m2[2]));
    asm volatile("s_mov_b32 %0, 0x03c003c0" : "=s"(c.m4[0]));
    asm volatile("s_mov_b32 %0, 0x003c003c" : "=s"(c.m4[1]));
    return c;
}

template <int CTRL> __device__ __forceinline__ float dpp_mov(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

template <int CTRL> __device__ __forceinline__ int quad_mov_i(int v) { return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true); }
template <int CTRL> __device__ __forceinline__ float quad_mov_f(float v) { return dpp_mov<CTRL>(v); }

__device__ __forceinline__ float lane_bcast(float v, int lane)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

// max / sum over the 64 lanes; the result is wave-uniform
__device__ __forceinline__ float wave_max(float v)
{
    v = fmaxf(v, dpp_mov<0xB1>(v));    // quad_perm [1,0,3,2]
    v = fmaxf(v, dpp_mov<0x4E>(v));    // quad_perm [2,3,0,1]
    v = fmaxf(v, dpp_mov<0x141>(v));   // row_half_mirror
    v = fmaxf(v, dpp_mov<0x140>(v));   // row_mirror: every lane of a row now holds the row's max
    return fmaxf(fmaxf(lane_bcast(v, 0), lane_bcast(v, 16)), fmaxf(lane_bcast(v, 32), lane_bcast(v, 48)));
}

__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_mov<0xB1>(v);
    v += dpp_mov<0x4E>(v);
    v += dpp_mov<0x141>(v);
    v += dpp_mov<0x140>(v);
    return (lane_bcast(v, 0) + lane_bcast(v, 16)) + (lane_bcast(v, 32) + lane_bcast(v, 48));
}

struct WaveState {
    float m;          // running maximum of the scaled scores (log2 units), wave-uniform
    float l, l2;      // per lane: sum p, sum p^2 relative to m
    float z;          // per lane: sum p * min_v over the quantized classes
    float ps[3];      // per lane: sum p * scale_v per quantized class
    float acc[kD];    // per lane: sum (p * scale_v * M) * h   (FP16 class: sum p * v)
};

// wave-uniform constants derived from the query
struct QConst {
    float qs;         // sum(q) * kScoreScale
    float qm[3];      // class c: kScoreScale * sum_t M_t sum(q over target t)   (8 bit: 1024 * sum q)
};

struct AttnParams {
    CacheView cv;
    int32_t by_class;        // whole waves per class when a wave has at most this many units on average (0: never)
    const uint32_t *q;          // [n_seq][Hq][32] fp16 pairs
    const __half *k_new, *v_new; // fused append: the new token's K/V [n_seq][Hkv][64], or nullptr
    const int32_t *seq_ids;
    float *out, *lse, *p2, *ws;
    int32_t layer, n_seq, S;
    int32_t longest_first;      // ragged batches over more than one round of workgroups: see k_decode_split
    int32_t rounds;             // more workgroups than places: unit costs kUnitCostRounds
};

// Register budget: two waves per SIMD (256 VGPRs each).  The four-buffer ring, 64 accumulators and the per-class
// state need ~185 VGPRs; at three waves per SIMD (168) the compiler spills inside the loops, and every spill
// reload waits for ALL outstanding loads (they share one counter), which stalls the pipeline.
#ifndef KVQ_WAVES_PER_EU
#define KVQ_WAVES_PER_EU 2
#endif
#ifndef KVQ_NT_STAGE
#define KVQ_NT_STAGE 1
#endif
#ifndef KVQ_NT_META
#define KVQ_NT_META 0      /* measured: non-temporal 8-byte (scale, min) loads cost ~8% on the mixed workload */
#endif

// Cache bytes are read exactly once per launch: the loads are marked non-temporal so that they stream past
// L2 and the Infinity Cache instead of evicting each other there.
__device__ __forceinline__ uint4 ld_stream16(const uint8_t *p)
{
#if KVQ_NT_STAGE
    const u32x4 t = __builtin_nontemporal_load((const u32x4 *)p);
    return make_uint4(t.x, t.y, t.z, t.w);
#else
    return *(const uint4 *)p;
#endif
}

__device__ __forceinline__ uint2 ld_stream8(const uint8_t *p)
{
#if KVQ_NT_META
    const u32x2 t = __builtin_nontemporal_load((const u32x2 *)p);
    return make_uint2(t.x, t.y);
#else
    return *(const uint2 *)p;
#endif
}

struct Stage { uint4 v[2]; };        // one pipeline stage: two 16-byte loads per lane (2 KiB per wave)

__device__ __forceinline__ uint32_t word_of(const uint4 &v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }
__device__ __forceinline__ float half_lo(uint32_t u) { return (float)__builtin_bit_cast(half2_t, u).x; }
__device__ __forceinline__ float half_hi(uint32_t u) { return (float)__builtin_bit_cast(half2_t, u).y; }

// Issues the two loads of stage PART of a K (ISV = false) or V vector set.  Load i covers
//   2 bit: block i of the unit, its only chunk;   4 bit: chunk i;   8 bit / FP16: chunk 2*PART + i.
// Lanes past the end of the bucket are redirected to token 0 of the unit's first block (which always
// exists), so every load is in bounds and reads initialised, finite data.
template <int C, bool ISV, int PART>
__device__ __forceinline__ void issue_stage(Stage &s, const uint8_t *base, int ntok, int lane)
{
    constexpr int BB = class_block_bytes(C), META = class_meta_bytes(C);
    constexpr int VOFF = ISV ? Cls<C>::NCH * kBlockTokens * 16 : 0;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int u = C == 0 ? i : 0;
        const int ch = C == 0 ? 0 : 2 * PART + i;
        const bool ok = u * kBlockTokens + lane < ntok;
        const uint32_t off = (ok ? (uint32_t)(u * BB + lane * 16) : 0u) + (uint32_t)(META + VOFF + ch * (kBlockTokens * 16));
        s.v[i] = ld_stream16(base + off);
    }
}

template <int C>
__device__ __forceinline__ void issue_meta(uint2 (&m)[Cls<C>::U], const uint8_t *base, int ntok, int lane)
{
    constexpr int BB = class_block_bytes(C);
#pragma unroll
    for (int u = 0; u < Cls<C>::U; ++u) {
        const bool ok = u * kBlockTokens + lane < ntok;
        m[u] = ld_stream8(base + (ok ? (uint32_t)(u * BB + lane * 8) : 0u));
    }
}

// Running-max update and softmax weights for the U scores of one unit.  The wave-wide maximum is only
// reduced (and the accumulators rescaled) when some lane actually exceeds the running maximum.
template <int U>
__device__ __forceinline__ void softmax_step(float (&sc)[U], WaveState &st, float (&p)[U])
{
    float lmax = sc[0];
#pragma unroll
    for (int u = 1; u < U; ++u) lmax = fmaxf(lmax, sc[u]);
    if (__builtin_amdgcn_ballot_w64(lmax > st.m) != 0ull) {  // wave-uniform branch
        const float wm = wave_max(lmax);
        const float f = __builtin_amdgcn_exp2f(st.m - wm);   // st.m = -inf before the first unit: f = 0
        st.l *= f;
        st.l2 *= f * f;
        st.z *= f;
        st.ps[0] *= f; st.ps[1] *= f; st.ps[2] *= f;
#pragma unroll
        for (int c = 0; c < kD; ++c) st.acc[c] *= f;
        st.m = wm;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        p[u] = __builtin_amdgcn_exp2f(sc[u] - st.m);
        st.l += p[u];
        st.l2 = fmaf(p[u], p[u], st.l2);
    }
}

// ---- 2 bit: word = 16 codes; pair p sits at bits 2p (low half) and 2p+16 (high half) -----------------
// unshifted word: p=4 -> target 0, p=3 -> 1, p=2 -> 2;  word<<6: p=1 -> 0, p=0 -> 1;  word>>6: p=7 -> 0, p=6 -> 1, p=5 -> 2
#define KVQ_FOR_PAIRS_2BIT(W, BODY)                                   \
    {                                                                 \
        const uint32_t w_ = (W), l_ = w_ << 6, r_ = w_ >> 6;          \
        BODY(w_, 0, 4) BODY(w_, 1, 3) BODY(w_, 2, 2)                  \
        BODY(l_, 0, 1) BODY(l_, 1, 0)                                 \
        BODY(r_, 0, 7) BODY(r_, 1, 6) BODY(r_, 2, 5)                  \
    }
// ---- 4 bit: word = 8 codes; pair p at bits 4p and 4p+16 ---------------------------------------------
// word<<2: p=1 -> target 0, p=0 -> 1;  word>>6: p=3 -> 0, p=2 -> 1
#define KVQ_FOR_PAIRS_4BIT(W, BODY)                                   \
    {                                                                 \
        const uint32_t w_ = (W), l_ = w_ << 2, r_ = w_ >> 6;          \
        BODY(l_, 0, 1) BODY(l_, 1, 0) BODY(r_, 0, 3) BODY(r_, 1, 2)   \
    }

// With static per-channel keys (LO = true) the query carries the channel steps, and the fp16 pairs q2 alone would lose
// 2^-12 of every term: q2l holds the rounding remainders, scaled by 2^12 (kLoScale) so that they stay normal numbers;
// their dot products run in accumulators of their own and join with the inverse factor.
constexpr float kLoScale = 4096.0f, kLoInv = 1.0f / 4096.0f;

// sum_t M_t (q . h)_t of one 2-bit vector (one chunk)
template <bool LO = false>
__device__ __forceinline__ float dot_2bit(const uint4 &k, const uint32_t (&q2)[32], const uint32_t (&q2l)[32], const Consts &cs)
{
    float d[3] = {0.f, 0.f, 0.f}, e[3] = {0.f, 0.f, 0.f};
#pragma unroll
    for (int wi = 0; wi < 4; ++wi) {
#define KVQ_BODY(X, T, P)                                                                            \
    {                                                                                                \
        const half2_t h = as_h2(and_or(X, cs.m2[T], cs.one));                                        \
        d[T] = __builtin_amdgcn_fdot2(h, as_h2(q2[wi * 8 + (P)]), d[T], false);                      \
        if constexpr (LO) e[T] = __builtin_amdgcn_fdot2(h, as_h2(q2l[wi * 8 + (P)]), e[T], false);   \
    }
        KVQ_FOR_PAIRS_2BIT(word_of(k, wi), KVQ_BODY)
#undef KVQ_BODY
    }
    if constexpr (LO) {
#pragma unroll
        for (int t = 0; t < 3; ++t) d[t] = fmaf(e[t], kLoInv, d[t]);
    }
    return fmaf(KVQ_M0_2, d[2], fmaf(KVQ_M0_1, d[1], KVQ_M0_0 * d[0]));
}

// sum_t M_t (q . h)_t of one 4-bit vector (two chunks)
template <bool LO = false>
__device__ __forceinline__ float dot_4bit(const Stage &k, const uint32_t (&q2)[32], const uint32_t (&q2l)[32], const Consts &cs)
{
    float d[2] = {0.f, 0.f}, e[2] = {0.f, 0.f};
#pragma unroll
    for (int ch = 0; ch < 2; ++ch)
#pragma unroll
        for (int wi = 0; wi < 4; ++wi) {
#define KVQ_BODY(X, T, P)                                                                                    \
    {                                                                                                        \
        const half2_t h = as_h2(and_or(X, cs.m4[T], cs.one));                                                \
        d[T] = __builtin_amdgcn_fdot2(h, as_h2(q2[(ch * 4 + wi) * 4 + (P)]), d[T], false);                   \
        if constexpr (LO) e[T] = __builtin_amdgcn_fdot2(h, as_h2(q2l[(ch * 4 + wi) * 4 + (P)]), e[T], false); \
    }
            KVQ_FOR_PAIRS_4BIT(word_of(k.v[ch], wi), KVQ_BODY)
#undef KVQ_BODY
        }
    if constexpr (LO) { d[0] = fmaf(e[0], kLoInv, d[0]); d[1] = fmaf(e[1], kLoInv, d[1]); }
    return fmaf(KVQ_M1_1, d[1], KVQ_M1_0 * d[0]);
}

// (q . h) over chunks 2*PART, 2*PART+1 of an 8-bit vector: bytes 0 and 2, then bytes 1 and 3 of each word,
// each under the exponent byte 0x64 (h = 1024 + c)
template <int PART, bool LO = false>
__device__ __forceinline__ float dot_8bit(const Stage &k, const uint32_t (&q2)[32], const uint32_t (&q2l)[32], float d)
{
    float d0 = d, d1 = 0.f, e0 = 0.f, e1 = 0.f;
#pragma unroll
    for (int ch = 0; ch < 2; ++ch)
#pragma unroll
        for (int wi = 0; wi < 4; ++wi) {
            const uint32_t w = word_of(k.v[ch], wi);
            const int m = ((2 * PART + ch) * 4 + wi) * 2;
            const half2_t h0 = as_h2(__builtin_amdgcn_perm(0x64646464u, w, 0x04020400u));
            const half2_t h1 = as_h2(__builtin_amdgcn_perm(0x64646464u, w, 0x04030401u));
            d0 = __builtin_amdgcn_fdot2(h0, as_h2(q2[m]), d0, false);
            d1 = __builtin_amdgcn_fdot2(h1, as_h2(q2[m + 1]), d1, false);
            if constexpr (LO) {
                e0 = __builtin_amdgcn_fdot2(h0, as_h2(q2l[m]), e0, false);
                e1 = __builtin_amdgcn_fdot2(h1, as_h2(q2l[m + 1]), e1, false);
            }
        }
    if constexpr (LO) return fmaf(e0 + e1, kLoInv, d0 + d1);
    return d0 + d1;
}

// (q . k) over chunks 2*PART, 2*PART+1 of an FP16 vector (16 channels)
template <int PART> __device__ __forceinline__ float dot_fp16(const Stage &k, const uint32_t (&q2)[32], float d)
{
    float d0 = d, d1 = 0.f;
#pragma unroll
    for (int ch = 0; ch < 2; ++ch) {
        const int m = (2 * PART + ch) * 4;
        d0 = __builtin_amdgcn_fdot2(as_h2(k.v[ch].x), as_h2(q2[m]), d0, false);
        d1 = __builtin_amdgcn_fdot2(as_h2(k.v[ch].y), as_h2(q2[m + 1]), d1, false);
        d0 = __builtin_amdgcn_fdot2(as_h2(k.v[ch].z), as_h2(q2[m + 2]), d0, false);
        d1 = __builtin_amdgcn_fdot2(as_h2(k.v[ch].w), as_h2(q2[m + 3]), d1, false);
    }
    return d0 + d1;
}

__device__ __forceinline__ void acc_2bit(const uint4 &v, const float (&a)[3], const Consts &cs, WaveState &st)
{
#pragma unroll
    for (int wi = 0; wi < 4; ++wi) {
#define KVQ_BODY(X, T, P)                                                                               \
    {                                                                                                   \
        const half2_t h = as_h2(and_or(X, cs.m2[T], cs.one));                                      \
        st.acc[2 * (wi * 8 + (P))] = fmaf(a[T], (float)h.x, st.acc[2 * (wi * 8 + (P))]);                \
        st.acc[2 * (wi * 8 + (P)) + 1] = fmaf(a[T], (float)h.y, st.acc[2 * (wi * 8 + (P)) + 1]);        \
    }
        KVQ_FOR_PAIRS_2BIT(word_of(v, wi), KVQ_BODY)
#undef KVQ_BODY
    }
}

__device__ __forceinline__ void acc_4bit(const Stage &v, const float (&a)[2], const Consts &cs, WaveState &st)
{
#pragma unroll
    for (int ch = 0; ch < 2; ++ch)
#pragma unroll
        for (int wi = 0; wi < 4; ++wi) {
#define KVQ_BODY(X, T, P)                                                                                                 \
    {                                                                                                                     \
        const half2_t h = as_h2(and_or(X, cs.m4[T], cs.one));                                                        \
        st.acc[2 * ((ch * 4 + wi) * 4 + (P))] = fmaf(a[T], (float)h.x, st.acc[2 * ((ch * 4 + wi) * 4 + (P))]);            \
        st.acc[2 * ((ch * 4 + wi) * 4 + (P)) + 1] = fmaf(a[T], (float)h.y, st.acc[2 * ((ch * 4 + wi) * 4 + (P)) + 1]);    \
    }
            KVQ_FOR_PAIRS_4BIT(word_of(v.v[ch], wi), KVQ_BODY)
#undef KVQ_BODY
        }
}

template <int PART> __device__ __forceinline__ void acc_8bit(const Stage &v, float a, WaveState &st)
{
#pragma unroll
    for (int ch = 0; ch < 2; ++ch)
#pragma unroll
        for (int wi = 0; wi < 4; ++wi) {
            const uint32_t w = word_of(v.v[ch], wi);
            const int c = ((2 * PART + ch) * 4 + wi) * 4;
            const half2_t h0 = as_h2(__builtin_amdgcn_perm(0x64646464u, w, 0x04020400u));
            const half2_t h1 = as_h2(__builtin_amdgcn_perm(0x64646464u, w, 0x04030401u));
            st.acc[c] = fmaf(a, (float)h0.x, st.acc[c]);
            st.acc[c + 1] = fmaf(a, (float)h0.y, st.acc[c + 1]);
            st.acc[c + 2] = fmaf(a, (float)h1.x, st.acc[c + 2]);
            st.acc[c + 3] = fmaf(a, (float)h1.y, st.acc[c + 3]);
        }
}

template <int PART> __device__ __forceinline__ void acc_fp16(const Stage &v, float p, WaveState &st)
{
#pragma unroll
    for (int ch = 0; ch < 2; ++ch)
#pragma unroll
        for (int wi = 0; wi < 4; ++wi) {
            const half2_t h = as_h2(word_of(v.v[ch], wi));
            const int c = ((2 * PART + ch) * 4 + wi) * 2;
            st.acc[c] = fmaf(p, (float)h.x, st.acc[c]);
            st.acc[c + 1] = fmaf(p, (float)h.y, st.acc[c + 1]);
        }
}

// scores of a unit -> softmax weights -> V multipliers and constant-part accumulators (quantized classes)
// KCH: the keys use the static per-channel variant.  Then q already carries the channel steps and qc.qs the constant
// q . min, so every token has "scale 1, minimum 1" and the stored per-token key metadata is not looked at.
template <int C, bool KCH = false>
__device__ __forceinline__ void finish_k(const float (&dot)[Cls<C>::U], const uint2 (&meta)[Cls<C>::U], int ntok, int lane,
                                         const QConst &qc, WaveState &st, float (&a)[Cls<C>::U][Cls<C>::NT])
{
    constexpr int U = Cls<C>::U;
    float sc[U], p[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const float kscale = KCH ? 1.0f : half_lo(meta[u].x), kmin = KCH ? 1.0f : half_hi(meta[u].x);
        // q.k^ * kScoreScale = min*qs + scale*(kScoreScale * sum_t M_t d_t - qm)
        const float s = fmaf(kmin, qc.qs, kscale * fmaf(dot[u], kScoreScale, -qc.qm[C]));
        sc[u] = (u * kBlockTokens + lane < ntok) ? s : -INFINITY;
    }
    softmax_step<U>(sc, st, p);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const float vscale = half_lo(meta[u].y), vmin = half_hi(meta[u].y);
        const float pscale = p[u] * vscale;
        st.z = fmaf(p[u], vmin, st.z);
        st.ps[C] += pscale;
        if constexpr (C == 0) { a[u][0] = pscale * KVQ_M0_0; a[u][1] = pscale * KVQ_M0_1; a[u][2] = pscale * KVQ_M0_2; }
        else if constexpr (C == 1) { a[u][0] = pscale * KVQ_M1_0; a[u][1] = pscale * KVQ_M1_1; }
        else a[u][0] = pscale;
    }
}

struct ClassWalk {
    const int32_t *pt;          // page-table row of (seq, class)
    const uint8_t *pool;        // class pool at this layer
    int Hkv, kvh, bpp, bpp_log2, cnt;
    int pi0, page0;             // the page-table entry of the range's first unit (index, page id), fetched by the prologue
};

// The page table is read through the constant address space: with a wave-uniform index this is a scalar
// load, which does not queue behind (or force a wait on) the vector loads of the stage pipeline.
typedef const int32_t __attribute__((address_space(4))) *const_i32_ptr;

template <int C> __device__ __forceinline__ int units_per_page_log2(int bpp_log2) { return bpp_log2 - (Cls<C>::U == 2 ? 1 : 0); }

template <int C> __device__ __forceinline__ const uint8_t *unit_base_in(const ClassWalk &w, int ui, int page)
{
    constexpr int U = Cls<C>::U;
    const int sh = units_per_page_log2<C>(w.bpp_log2);   // page_tokens is a power of two
    const int blk = (ui & ((1 << sh) - 1)) * U;
    return w.pool + (((size_t)page * w.Hkv + w.kvh) * w.bpp + blk) * (size_t)class_block_bytes(C);
}

// (No "same page as last time?" shortcut here: a branch inside the pipelined loops makes the compiler's wait-count
// bookkeeping give up, and it then drains every outstanding stage load at the top of each iteration.)
template <int C> __device__ __forceinline__ const uint8_t *unit_base(const ClassWalk &w, int ui)
{
    const int sh = units_per_page_log2<C>(w.bpp_log2);
    return unit_base_in<C>(w, ui, ((const_i32_ptr)(uintptr_t)w.pt)[ui >> sh]);
}

// Outside the loops: a unit of the range's first page needs no look at the table.
template <int C> __device__ __forceinline__ const uint8_t *unit_base_start(const ClassWalk &w, int ui)
{
    const int sh = units_per_page_log2<C>(w.bpp_log2);
    if ((ui >> sh) == w.pi0) return unit_base_in<C>(w, ui, w.page0);
    return unit_base<C>(w, ui);
}

template <int C> __device__ __forceinline__ int unit_ntok(const ClassWalk &w, int ui)
{
    constexpr int UT = Cls<C>::U * kBlockTokens;
    return min(w.cnt - ui * UT, UT);
}

#define KVQ_FENCE() __builtin_amdgcn_sched_barrier(0)

// Prefetches past the end of a wave's range are not skipped: a conditional load would make the stage buffer a
// merge of "new load" and "old value", and the register copies that merge needs wait for every outstanding
// load.  Instead the loads are issued unconditionally with a token count of zero, which redirects all 64 lanes
// to the first 16 bytes of a unit that is known to exist: one cache line of traffic per load, no branch.

// Units k0, k0+step, ... < k1 of the 2-bit (two blocks per unit) or 4-bit (one block per unit) class: two
// stages per unit, K(n) -> b0/b2 and V(n) -> b1/b3 for even/odd n; each buffer is reloaded right after use.
template <int C, bool KCH = false>
__device__ __forceinline__ void run_low(const ClassWalk &w, int k0, int k1, int step, int lane, const uint32_t (&q2)[32],
                                        const uint32_t (&q2l)[32], const QConst &qc, const Consts &cs, WaveState &st)
{
    if (k0 >= k1) return;
    constexpr int U = Cls<C>::U, NT = Cls<C>::NT;
    Stage b0, b1, b2, b3;
    uint2 m0[U], m1[U];
    const uint8_t *safe = unit_base_start<C>(w, k0);
    {
        // (fenced like the loop body: the loop's wait counts assume that the buffers were asked for in the order in
        // which they are used, and the compiler takes the stricter of what the loop's two entries need; left to
        // itself it may ask for the first buffer last, and the loop then waits for ALL loads in every iteration)
        const int na = unit_ntok<C>(w, k0);
        KVQ_FENCE();
        issue_stage<C, false, 0>(b0, safe, na, lane);
        issue_meta<C>(m0, safe, na, lane);
        KVQ_FENCE();
        issue_stage<C, true, 0>(b1, safe, na, lane);
        KVQ_FENCE();
        const bool two = k0 + step < k1;
        const uint8_t *bb = two ? unit_base_start<C>(w, k0 + step) : safe;
        const int nb = two ? unit_ntok<C>(w, k0 + step) : 0;
        KVQ_FENCE();
        issue_stage<C, false, 0>(b2, bb, nb, lane);
        issue_meta<C>(m1, bb, nb, lane);
        KVQ_FENCE();
        issue_stage<C, true, 0>(b3, bb, nb, lane);
        KVQ_FENCE();
    }
    auto k_stage = [&](const Stage &b, const uint2 (&m)[U], int ntok, float (&a)[U][NT]) {
        float dot[U];
        if constexpr (C == 0) { dot[0] = dot_2bit<KCH>(b.v[0], q2, q2l, cs); dot[1] = dot_2bit<KCH>(b.v[1], q2, q2l, cs); }
        else dot[0] = dot_4bit<KCH>(b, q2, q2l, cs);
        finish_k<C, KCH>(dot, m, ntok, lane, qc, st, a);
    };
    auto v_stage = [&](const Stage &b, const float (&a)[U][NT]) {
        if constexpr (C == 0) { acc_2bit(b.v[0], a[0], cs, st); acc_2bit(b.v[1], a[1], cs, st); }
        else acc_4bit(b, a[0], cs, st);
    };
    for (int ui = k0; ui < k1; ui += 2 * step) {
        const bool more2 = ui + 2 * step < k1, more3 = ui + 3 * step < k1;
        const uint8_t *base2 = more2 ? unit_base<C>(w, ui + 2 * step) : safe;
        const uint8_t *base3 = more3 ? unit_base<C>(w, ui + 3 * step) : safe;
        const int n2 = more2 ? unit_ntok<C>(w, ui + 2 * step) : 0;
        const int n3 = more3 ? unit_ntok<C>(w, ui + 3 * step) : 0;
        const int n1 = ui + step < k1 ? unit_ntok<C>(w, ui + step) : 0;     // 0: every lane of the odd unit is masked
        float a[U][NT];
        KVQ_FENCE();
        k_stage(b0, m0, unit_ntok<C>(w, ui), a);
        KVQ_FENCE();
        issue_stage<C, false, 0>(b0, base2, n2, lane);
        issue_meta<C>(m0, base2, n2, lane);
        KVQ_FENCE();
        v_stage(b1, a);
        KVQ_FENCE();
        issue_stage<C, true, 0>(b1, base2, n2, lane);
        KVQ_FENCE();
        if (n1 > 0) {
            k_stage(b2, m1, n1, a);
            KVQ_FENCE();
            v_stage(b3, a);
        }
        KVQ_FENCE();
        issue_stage<C, false, 0>(b2, base3, n3, lane);
        issue_meta<C>(m1, base3, n3, lane);
        issue_stage<C, true, 0>(b3, base3, n3, lane);
        KVQ_FENCE();
    }
}

// Blocks of the 8-bit class: stages K01, K23, V01, V23 (chunk pairs) -> b0..b3.
template <bool KCH = false>
__device__ __forceinline__ void run_8bit(const ClassWalk &w, int k0, int k1, int step, int lane, const uint32_t (&q2)[32],
                                         const uint32_t (&q2l)[32], const QConst &qc, WaveState &st)
{
    if (k0 >= k1) return;
    Stage b0, b1, b2, b3;
    uint2 m0[1];
    const uint8_t *safe = unit_base_start<2>(w, k0);
    {
        const int na = unit_ntok<2>(w, k0);
        KVQ_FENCE();
        issue_stage<2, false, 0>(b0, safe, na, lane);
        KVQ_FENCE();
        issue_stage<2, false, 1>(b1, safe, na, lane);
        KVQ_FENCE();
        issue_meta<2>(m0, safe, na, lane);
        KVQ_FENCE();
        issue_stage<2, true, 0>(b2, safe, na, lane);
        KVQ_FENCE();
        issue_stage<2, true, 1>(b3, safe, na, lane);
        KVQ_FENCE();
    }
    for (int ui = k0; ui < k1; ui += step) {
        const bool more = ui + step < k1;
        const uint8_t *bn = more ? unit_base<2>(w, ui + step) : safe;
        const int nn = more ? unit_ntok<2>(w, ui + step) : 0;
        float dot[1], a[1][1];
        KVQ_FENCE();
        dot[0] = dot_8bit<0, KCH>(b0, q2, q2l, 0.f);
        KVQ_FENCE();
        issue_stage<2, false, 0>(b0, bn, nn, lane);
        KVQ_FENCE();
        dot[0] = dot_8bit<1, KCH>(b1, q2, q2l, dot[0]);
        KVQ_FENCE();
        issue_stage<2, false, 1>(b1, bn, nn, lane);
        KVQ_FENCE();
        finish_k<2, KCH>(dot, m0, unit_ntok<2>(w, ui), lane, qc, st, a);
        KVQ_FENCE();
        issue_meta<2>(m0, bn, nn, lane);
        KVQ_FENCE();
        acc_8bit<0>(b2, a[0][0], st);
        KVQ_FENCE();
        issue_stage<2, true, 0>(b2, bn, nn, lane);
        KVQ_FENCE();
        acc_8bit<1>(b3, a[0][0], st);
        KVQ_FENCE();
        issue_stage<2, true, 1>(b3, bn, nn, lane);
        KVQ_FENCE();
    }
}

// Blocks of the FP16 class: stages K0..K3 then V0..V3 (chunk pairs) cycle through b0..b3.
__device__ __forceinline__ void run_fp16(const ClassWalk &w, int k0, int k1, int step, int lane, const uint32_t (&q2)[32], WaveState &st)
{
    if (k0 >= k1) return;
    Stage b0, b1, b2, b3;
    const uint8_t *safe = unit_base_start<3>(w, k0);
    {
        const int na = unit_ntok<3>(w, k0);
        KVQ_FENCE();
        issue_stage<3, false, 0>(b0, safe, na, lane);
        KVQ_FENCE();
        issue_stage<3, false, 1>(b1, safe, na, lane);
        KVQ_FENCE();
        issue_stage<3, false, 2>(b2, safe, na, lane);
        KVQ_FENCE();
        issue_stage<3, false, 3>(b3, safe, na, lane);
        KVQ_FENCE();
    }
    const uint8_t *bc = safe;
    for (int ui = k0; ui < k1; ui += step) {
        const bool more = ui + step < k1;
        const int nc = unit_ntok<3>(w, ui);
        const uint8_t *bn = more ? unit_base<3>(w, ui + step) : safe;
        const int nn = more ? unit_ntok<3>(w, ui + step) : 0;
        KVQ_FENCE();
        float d = dot_fp16<0>(b0, q2, 0.f);
        KVQ_FENCE();
        issue_stage<3, true, 0>(b0, bc, nc, lane);
        KVQ_FENCE();
        d = dot_fp16<1>(b1, q2, d);
        KVQ_FENCE();
        issue_stage<3, true, 1>(b1, bc, nc, lane);
        KVQ_FENCE();
        d = dot_fp16<2>(b2, q2, d);
        KVQ_FENCE();
        issue_stage<3, true, 2>(b2, bc, nc, lane);
        KVQ_FENCE();
        d = dot_fp16<3>(b3, q2, d);
        KVQ_FENCE();
        issue_stage<3, true, 3>(b3, bc, nc, lane);
        KVQ_FENCE();
        float sc[1], p[1];
        sc[0] = lane < nc ? d * kScoreScale : -INFINITY;
        softmax_step<1>(sc, st, p);
        acc_fp16<0>(b0, p[0], st);
        KVQ_FENCE();
        issue_stage<3, false, 0>(b0, bn, nn, lane);
        KVQ_FENCE();
        acc_fp16<1>(b1, p[0], st);
        KVQ_FENCE();
        issue_stage<3, false, 1>(b1, bn, nn, lane);
        KVQ_FENCE();
        acc_fp16<2>(b2, p[0], st);
        KVQ_FENCE();
        issue_stage<3, false, 2>(b2, bn, nn, lane);
        KVQ_FENCE();
        acc_fp16<3>(b3, p[0], st);
        KVQ_FENCE();
        issue_stage<3, false, 3>(b3, bn, nn, lane);
        KVQ_FENCE();
        bc = bn;
    }
}

__device__ __forceinline__ int ceil_div_pos(uint32_t a, uint32_t b) { return (int)((a + b - 1u) / b); }

// Static per-channel keys, class C: q' = q (.) step_C as fp16 pairs q2 plus the fp16 remainders q2l (scaled by
// kLoScale; the product of two fp16 numbers is exact in fp32, so q2 + q2l / kLoScale carries it to ~2^-22), read back
// lane by lane into scalars; the constant q . min; and the class's mantissa-offset correction formed from the SAME
// rounded pairs that the packed dot products will use.  lane = channel while this runs.  Products beyond the fp16 range
// saturate.
template <int C>
__device__ __forceinline__ void kch_prepare(const AttnParams &P, int si, int qh, int kvh, int lane, uint32_t (&q2)[32],
                                            uint32_t (&q2l)[32], QConst &qc)
{
    const CacheView &cv = P.cv;
    const float qf = __half2float(((const __half *)P.q)[((size_t)si * cv.Hq + qh) * kD + lane]);
    const size_t ti = ((size_t)P.layer * cv.Hkv + kvh) * kD + lane;
    const float stp = __half2float(cv.kch_step[(size_t)C * cv.n_layers * cv.Hkv * kD + ti]);
    const float mn = __half2float(cv.kch_min[ti]);
    const float prod = fminf(fmaxf(qf * stp, -65504.0f), 65504.0f);
    const __half hi = __float2half_rn(prod);
    const __half lo = __float2half_rn((prod - __half2float(hi)) * kLoScale);
    const uint32_t mine = (uint32_t)__half_as_ushort(hi) | ((uint32_t)__half_as_ushort(lo) << 16);      // {hi, lo} of this channel
    const uint32_t other = (uint32_t)__shfl_xor((int)mine, 1, 64);
    const uint32_t even = (lane & 1) ? other : mine, odd = (lane & 1) ? mine : other;
    const uint32_t packed_hi = (even & 0xffffu) | (odd << 16), packed_lo = (even >> 16) | (odd & 0xffff0000u);
    float qsum = 0.f, t0[3] = {0.f, 0.f, 0.f}, t1[2] = {0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        q2[i] = (uint32_t)__builtin_amdgcn_readlane((int)packed_hi, 2 * i);
        {
            // the remainders live in vector registers (every lane the same value): the scalar file cannot hold 64 query
            // words next to the walk's pointers, and the vector file has the room
            const uint32_t t = (uint32_t)__builtin_amdgcn_readlane((int)packed_lo, 2 * i);
            asm volatile("v_mov_b32 %0, %1" : "=v"(q2l[i]) : "s"(t));
        }
        const float v = fmaf(half_lo(q2l[i]) + half_hi(q2l[i]), kLoInv, half_lo(q2[i]) + half_hi(q2[i]));
        qsum += v;
        t0[target0(i % 8)] += v;
        t1[target1(i % 4)] += v;
    }
    qc.qs = wave_sum(qf * mn) * kScoreScale;
    qc.qm[0] = (KVQ_M0_0 * t0[0] + KVQ_M0_1 * t0[1] + KVQ_M0_2 * t0[2]) * kScoreScale;
    qc.qm[1] = (KVQ_M1_0 * t1[0] + KVQ_M1_1 * t1[1]) * kScoreScale;
    qc.qm[2] = KVQ_OFF2 * qsum * kScoreScale;
}

template <int NW, bool KCH>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(KVQ_WAVES_PER_EU, KVQ_WAVES_PER_EU))) void k_decode_split(AttnParams P)
{
    const CacheView &cv = P.cv;
    // Every memory round trip before the first cache byte is asked for costs a launch of a few units per wave more than
    // the units themselves, so the prologue is three batches of loads, each behind ONE wait:
    //   1. the arguments (the compiler would fetch each where it is first used, and wait for each on its own);
    //   2. everything that hangs on the sequence and head alone: the class counts, the newest-token record, the query
    //      and the first six entries of the four page-table rows (one vector load, a word per lane: scalar loads that miss their
    //      cache are answered one line after the other, these travel side by side);
    //   3. only for a wave whose range starts beyond a class's first six pages: the entries it starts at.
    int S = P.S, n_seq = P.n_seq, Hq = cv.Hq, Hkv = cv.Hkv;
    const int longest_first = P.longest_first, layer = P.layer, by_class = P.by_class, rounds_arg = P.rounds;
    const int max_seqs = cv.max_seqs, mpps = cv.max_pages_per_seq, bpp = cv.blocks_per_page;
    const int32_t *const seq_ids = P.seq_ids;
    const uint32_t *const q_all = P.q;
    const __half *const k_new = P.k_new;
    const int32_t *const counts = cv.counts, *const last_rec = cv.last_rec, *const page_table = cv.page_table;
    const uint8_t *const pool0 = cv.pool[0];     // (the pools and layer strides share one 64-byte line of the argument block:
                                                 // asking for one of them now makes the later reads of the others short)
    // (the four that the work-item arithmetic starts from are outputs as well: nothing can then be scheduled ahead of
    // this point, behind a wait of its own for part of the loads)
    asm volatile("" : "+s"(S), "+s"(n_seq), "+s"(Hq), "+s"(Hkv)
                 : "s"(longest_first), "s"(layer), "s"(by_class), "s"(rounds_arg), "s"(max_seqs), "s"(mpps), "s"(bpp), "s"(seq_ids), "s"(q_all),
                   "s"(k_new), "s"(counts), "s"(last_rec), "s"(page_table), "s"(pool0));
    const uint32_t G = (uint32_t)Hq / (uint32_t)Hkv;
    const uint32_t nunits = (uint32_t)n_seq * (uint32_t)Hq * (uint32_t)S;
    // Workgroups are dealt to the 8 XCDs round-robin by id.  Give each XCD a contiguous range of work
    // items instead, so that the G query heads that share one kv-head's bytes also share one L2.
    const uint32_t per_xcd = (nunits + 7u) >> 3;
    const uint32_t unit = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
    if ((blockIdx.x >> 3) >= per_xcd || unit >= nunits) return;
    // unit = ((si*Hkv + kvh)*S + s)*G + g
    uint32_t r = unit;
    const int g = (int)(r % G); r /= G;
    int s = 0;
    if (S != 1) { s = (int)(r % (uint32_t)S); r /= (uint32_t)S; }
    const int kvh = (int)(r % (uint32_t)Hkv);
    int si = (int)(r / (uint32_t)Hkv);
    const int qh = kvh * (int)G + g;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (longest_first) {
        // A launch with more workgroups than fit at once is list scheduling in workgroup order: with the sequences in
        // arbitrary order the last round may start a long one (ragged batch: makespan up to 1.3x the mean).  So the
        // position si in the launch order takes the sequence of that RANK by length, longest first, dealt to the XCDs
        // eight at a time, every other eight the other way round (an XCD's k-th position has rank 8k + xcd for even k,
        // 8k + 7 - xcd for odd k: always in the same direction, XCD 0 would get the longest of every eight and 13 % more
        // tokens than XCD 7 on lengths spread evenly over a 1:4 range).  Every workgroup ranks the (at most 64) lengths
        // itself: lane = sequence, 64 lane reads.
        const int q8 = n_seq >> 3;
        const int lf_k = si % q8, lf_x = si / q8;
        const int want = lf_k * 8 + ((lf_k & 1) ? 7 - lf_x : lf_x);
        int my_len = -1;
        if (lane < n_seq) {
            const int sq = seq_ids ? seq_ids[lane] : lane;
            my_len = (sq >= 0 && sq < max_seqs) ? counts[(size_t)sq * 5 + 4] : 0;
        }
        int rank = 0;
        for (int j = 0; j < n_seq; ++j) {
            const int lj = __builtin_amdgcn_readlane(my_len, j);
            rank += (lj > my_len || (lj == my_len && j < lane)) ? 1 : 0;
        }
        const unsigned long long hit = __ballot(lane < n_seq && rank == want);
        si = (int)__builtin_ctzll(hit);
    }
    int seq = si;
    if (seq_ids) seq = ((const_i32_ptr)(uintptr_t)seq_ids)[si];
    const bool seq_ok = seq >= 0 && seq < max_seqs;
    if (!seq_ok) seq = 0;                                                    // row 0 exists: the loads below stay in bounds

    // ---- batch 2: ONE vector load instruction, a different address per lane, then lane reads into scalars ----
    //   lanes 0..31 the query's fp16 pairs, 32..35 the class counts, 36..39 the newest-token record,
    //   40 + 6 c + e entry e < 6 of class c's page-table row (indices past the row's end repeat its last entry)
    constexpr int kSpecLane = 40, kSpecPages = 6;
    const int32_t *const pt_seq = page_table + (size_t)seq * kClasses * mpps;
    const uint32_t *b2 = q_all + ((size_t)si * Hq + qh) * 32 + (lane < 32 ? lane : 0);
    if (lane >= 32 && lane < 36) b2 = (const uint32_t *)(counts + (size_t)seq * 5 + (lane - 32));
    if (lane >= 36 && lane < 40) b2 = (const uint32_t *)(last_rec + (size_t)seq * 4 + (lane - 36));
    if (lane >= kSpecLane) {
        const int sc = (lane - kSpecLane) / kSpecPages, se = (lane - kSpecLane) - sc * kSpecPages;
        b2 = (const uint32_t *)(pt_seq + (size_t)sc * mpps + min(se, mpps - 1));
    }
    const int b2v = (int)*b2;
    uint32_t q2[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) q2[i] = (uint32_t)__builtin_amdgcn_readlane(b2v, i);
    int cnt[kClasses] = {__builtin_amdgcn_readlane(b2v, 32), __builtin_amdgcn_readlane(b2v, 33), __builtin_amdgcn_readlane(b2v, 34),
                         __builtin_amdgcn_readlane(b2v, 35)};
    int4 rec = make_int4(__builtin_amdgcn_readlane(b2v, 36), __builtin_amdgcn_readlane(b2v, 37), __builtin_amdgcn_readlane(b2v, 38),
                         __builtin_amdgcn_readlane(b2v, 39));         // {last_T, bits, slot, page} of the newest token
    if (!seq_ok) cnt[0] = cnt[1] = cnt[2] = cnt[3] = 0;
    if (k_new == nullptr || !seq_ok) rec = make_int4(0, 0, 0, 0);

    // sum(q) and, per class, sum_t M_t sum(q over target t): lane = pair while the load's answer still lies across the
    // lanes (32 pairs at once and three reductions, instead of a chain of a hundred dependent scalar-operand additions
    // that every wave would walk through before its first load).  M is a power of two: 2^e with e from the pair's
    // position in its word (2 bit: pairs 1,4,7 -> 4, 0,3,6 -> 16, 2,5 -> 64; 4 bit: odd -> 16, even -> 256).
    QConst qc;
    {
        const float v = lane < 32 ? half_lo((uint32_t)b2v) + half_hi((uint32_t)b2v) : 0.f;
        const int e0 = (int)((0x24624624u >> (4 * (lane & 7))) & 15u);
        const int e1 = (lane & 1) ? 4 : 8;
        const float qsum = wave_sum(v);
        qc.qs = qsum * kScoreScale;
        qc.qm[0] = wave_sum(__builtin_ldexpf(v, e0)) * kScoreScale;
        qc.qm[1] = wave_sum(__builtin_ldexpf(v, e1)) * kScoreScale;
        qc.qm[2] = KVQ_OFF2 * qsum * kScoreScale;
    }
    const Consts cs = make_consts();

    WaveState st;
    st.m = -INFINITY;
    st.l = st.l2 = st.z = 0.f;
    st.ps[0] = st.ps[1] = st.ps[2] = 0.f;
#pragma unroll
    for (int c = 0; c < kD; ++c) st.acc[c] = 0.f;

    // This wave's share of the (sequence, kv-head)'s units: the units of the four classes form one list,
    // weighted by their cost; the S workgroups x NW waves cut the list into S*NW contiguous ranges of
    // equal weight (a unit belongs to the range that holds its start), so a wave meets one or two classes.
    int nu[kClasses];
    static_assert(kUnitCost[2] == kUnitCostRounds[2] && kUnitCost[3] == kUnitCostRounds[3], "the two sets differ in the low-bit classes only");
    const bool rounds = rounds_arg != 0;
    const int wgt[kClasses] = {rounds ? kUnitCostRounds[0] : kUnitCost[0], rounds ? kUnitCostRounds[1] : kUnitCost[1], kUnitCost[2], kUnitCost[3]};
    uint32_t wtot = 0;                                       // below 2^31: the host checks units x weight before the launch
    // Fused append: the newest token of the sequence (logged by the bookkeeping kernel, slot = last of its class)
    // is not read from the cache.  It is quantized in registers from k_new / v_new, joins the softmax as one extra
    // partial result, and the workgroup with s == 0, g == 0 stores it for later steps.
    bool has_new = false;
    int new_bits = 16, new_cls = 3, new_slot = 0, new_page = 0;
    {
        if (rec.x == 1) {                                     // (zeroed above when there is no new token to take)
            new_bits = rec.y;
            new_slot = rec.z;
            new_page = rec.w;
            new_cls = bits_to_class(new_bits);
            has_new = true;
        }
    }
    // The wave that will quantize the new token asks for its K, V and query element now and uses them after its walk:
    // their latency then costs that wave nothing.
    const bool does_new = has_new && s == 0 && wave == 0;
    __half new_kx = __ushort_as_half((unsigned short)0), new_vx = new_kx, new_qx = new_kx;
    if (does_new) {
        const size_t src = ((size_t)si * Hkv + kvh) * kD + lane;
        new_kx = k_new[src];
        new_vx = P.v_new[src];
        new_qx = ((const __half *)q_all)[((size_t)si * Hq + qh) * kD + lane];
    }
#pragma unroll
    for (int c = 0; c < kClasses; ++c) {
        if (has_new && c == new_cls) cnt[c] -= 1;
        nu[c] = (cnt[c] + class_unit_blocks(c) * kBlockTokens - 1) / (class_unit_blocks(c) * kBlockTokens);
        wtot += (uint32_t)nu[c] * (uint32_t)wgt[c];
    }
    const int J = S * NW, j = s * NW + wave;
    int first[kClasses] = {0, 0, 0, 0}, last[kClasses] = {0, 0, 0, 0};
    constexpr int step = 1;                                  // a wave's units are consecutive
    // Short ranges (one workgroup per head and up to a dozen units per wave: small batches, short contexts): a wave
    // that crosses from one class into the next pays that class's pipeline start, a full memory latency, a second
    // time, and its workgroup waits for it.  There the classes get whole waves instead, in proportion to their weight
    // (at least one for a class that has units; what rounding leaves over goes where the load per wave is largest),
    // and a wave's range lies inside its class.  Every wave of the (sequence, head) computes the same allocation from
    // the same numbers, so the quotients may be reciprocal approximations: the ranges tile a class whatever their
    // exact cut points are.
    const uint32_t nu_tot = (uint32_t)(nu[0] + nu[1] + nu[2] + nu[3]);
    const int nonempty = (nu[0] > 0) + (nu[1] > 0) + (nu[2] > 0) + (nu[3] > 0);
    bool ranged = false;
    if (S == 1 && nonempty > 1 && J >= 2 * nonempty && nu_tot <= (uint32_t)by_class * (uint32_t)J) {
        // lane = class (the lane's low two bits; every quad computes the same): four classes per instruction, and the
        // cross-class steps are moves inside a quad
        const int c4 = lane & 3;
        const int v_nu = c4 == 0 ? nu[0] : c4 == 1 ? nu[1] : c4 == 2 ? nu[2] : nu[3];
        const int v_wgt = c4 == 0 ? wgt[0] : c4 == 1 ? wgt[1] : c4 == 2 ? wgt[2] : wgt[3];
        const float v_wc = (float)(v_nu * v_wgt);                  // exact: below 2^24 here (at most a dozen units per wave)
        const float per_weight = (float)J * __builtin_amdgcn_rcpf((float)wtot);
        int v_n = v_nu > 0 ? max(1, (int)(v_wc * per_weight)) : 0;
        int used;
        {
            int t = v_n + quad_mov_i<0xB1>(v_n);                   // [1,0,3,2]
            t += quad_mov_i<0x4E>(t);                              // [2,3,0,1]
            used = __builtin_amdgcn_readfirstlane(t);
        }
        for (int it = 0; it < 2 * kClasses && used != J; ++it) {
            // too few waves handed out: the class with the largest load per wave gets one more; too many: the class
            // whose load per wave rises least gives one back (ties: the lowest class)
            const bool more = used < J;
            const int n = more ? v_n : v_n - 1;
            const bool ok = n > 0;
            const float load = v_wc * __builtin_amdgcn_rcpf((float)max(n, 1));
            const float key = ok ? (more ? load : -load) : -INFINITY;
            float best = fmaxf(key, quad_mov_f<0xB1>(key));
            best = fmaxf(best, quad_mov_f<0x4E>(best));
            const unsigned long long hit = __builtin_amdgcn_ballot_w64(ok && key == best) & 0xFull;
            if (hit == 0ull) break;
            const int pick = (int)__builtin_ctzll(hit);
            const int d = more ? 1 : -1;
            v_n += c4 == pick ? d : 0;
            used += d;
        }
        if (used == J) {
            // The waves take the classes in the order 2 bit, 4 bit, FP16, 8 bit: waves i and i + 4 of an eight-wave workgroup
            // share a SIMD, and this order pairs the class with the most unpacking arithmetic with the one that has none.
            const int n0 = quad_mov_i<0x00>(v_n), n1 = quad_mov_i<0x55>(v_n), n3 = quad_mov_i<0xFF>(v_n);     // class 0, 1, 3 to all
            const int before = (c4 > 0 ? n0 : 0) + (c4 > 1 ? n1 : 0) + (c4 == 2 ? n3 : 0);
            const int jc = j - before;
            const bool mine = jc >= 0 && jc < v_n;
            const float per_wave = (float)v_nu * __builtin_amdgcn_rcpf((float)max(v_n, 1));
            const int v_first = mine ? min((int)((float)jc * per_wave), v_nu) : 0;
            const int v_last = mine ? (jc + 1 == v_n ? v_nu : min((int)((float)(jc + 1) * per_wave), v_nu)) : 0;
#pragma unroll
            for (int c = 0; c < kClasses; ++c) {
                first[c] = __builtin_amdgcn_readlane(v_first, c);
                last[c] = __builtin_amdgcn_readlane(v_last, c);
            }
            ranged = true;
        }
    }
    if (!ranged) {
        // 64-bit division is a long emulated routine, and this runs before a wave's first load: 32 bits whenever
        // wtot * J fits (it does unless a context has millions of tokens)
        uint32_t lo_w, hi_w;
        if (S == 1) {                                        // the usual case: divisions by a constant
            if (((unsigned long long)wtot * (uint32_t)NW) >> 32 == 0) {
                lo_w = wtot * (uint32_t)wave / (uint32_t)NW;
                hi_w = wtot * (uint32_t)(wave + 1) / (uint32_t)NW;
            } else {
                lo_w = (uint32_t)((unsigned long long)wtot * (uint32_t)wave / (uint32_t)NW);
                hi_w = (uint32_t)((unsigned long long)wtot * (uint32_t)(wave + 1) / (uint32_t)NW);
            }
        } else if (((unsigned long long)wtot * (uint32_t)J) >> 32 == 0) {
            lo_w = wtot * (uint32_t)j / (uint32_t)J;
            hi_w = wtot * (uint32_t)(j + 1) / (uint32_t)J;
        } else {
            lo_w = (uint32_t)((unsigned long long)wtot * (uint32_t)j / (uint32_t)J);
            hi_w = (uint32_t)((unsigned long long)wtot * (uint32_t)(j + 1) / (uint32_t)J);
        }
        uint32_t wbase = 0;
#pragma unroll
        for (int c = 0; c < kClasses; ++c) {
            // (divisions by constants: both sets' quotients and a select, no division instruction sequence)
            const uint32_t dl = lo_w <= wbase ? 0u : lo_w - wbase, dh = hi_w <= wbase ? 0u : hi_w - wbase;
            const int ql = rounds ? ceil_div_pos(dl, (uint32_t)kUnitCostRounds[c]) : ceil_div_pos(dl, (uint32_t)kUnitCost[c]);
            const int qh_ = rounds ? ceil_div_pos(dh, (uint32_t)kUnitCostRounds[c]) : ceil_div_pos(dh, (uint32_t)kUnitCost[c]);
            const int klo = min(ql, nu[c]);
            const int khi = min(qh_, nu[c]);
            first[c] = klo;
            last[c] = khi;
            wbase += (uint32_t)nu[c] * (uint32_t)wgt[c];
        }
    }
    ClassWalk w;
    w.Hkv = Hkv; w.kvh = kvh; w.bpp = bpp; w.bpp_log2 = 31 - __builtin_clz(bpp);
    // ---- batch 3: the page-table entry that each class's range starts in, when batch 2 has not brought it ----
#define KVQ_PI0(C) (first[C] < last[C] ? first[C] >> units_per_page_log2<C>(w.bpp_log2) : 0)
    const int pi0_0 = KVQ_PI0(0), pi0_1 = KVQ_PI0(1), pi0_2 = KVQ_PI0(2), pi0_3 = KVQ_PI0(3);
    int pg0_0, pg0_1, pg0_2, pg0_3;
    if (max(max(pi0_0, pi0_1), max(pi0_2, pi0_3)) < kSpecPages) {
        pg0_0 = __builtin_amdgcn_readlane(b2v, kSpecLane + pi0_0);
        pg0_1 = __builtin_amdgcn_readlane(b2v, kSpecLane + kSpecPages + pi0_1);
        pg0_2 = __builtin_amdgcn_readlane(b2v, kSpecLane + 2 * kSpecPages + pi0_2);
        pg0_3 = __builtin_amdgcn_readlane(b2v, kSpecLane + 3 * kSpecPages + pi0_3);
    } else {
        // (a range's first unit exists, so its page index is below max_pages_per_seq; the four loads travel together)
        const int c4 = lane & 3;
        const int pi_l = c4 == 0 ? pi0_0 : c4 == 1 ? pi0_1 : c4 == 2 ? pi0_2 : pi0_3;
        const int b3v = pt_seq[(size_t)c4 * mpps + pi_l];
        pg0_0 = __builtin_amdgcn_readlane(b3v, 0); pg0_1 = __builtin_amdgcn_readlane(b3v, 1);
        pg0_2 = __builtin_amdgcn_readlane(b3v, 2); pg0_3 = __builtin_amdgcn_readlane(b3v, 3);
    }
#define KVQ_WALK(C)                                                                              \
    w.pt = page_table + ((size_t)seq * kClasses + (C)) * mpps;                                   \
    w.pool = cv.pool[C] + (size_t)layer * cv.layer_stride[C];                                    \
    w.cnt = cnt[C];                                                                              \
    w.pi0 = KVQ_PI0(C);                                                                          \
    w.page0 = pg0_##C;
    if constexpr (!KCH) {
        KVQ_WALK(0) run_low<0>(w, first[0], last[0], step, lane, q2, q2, qc, cs, st);
        KVQ_WALK(1) run_low<1>(w, first[1], last[1], step, lane, q2, q2, qc, cs, st);
        KVQ_WALK(2) run_8bit(w, first[2], last[2], step, lane, q2, q2, qc, st);
        KVQ_WALK(3) run_fp16(w, first[3], last[3], step, lane, q2, st);
    } else {
        // the FP16 class first, with q as it is; then each quantized class that this wave meets, with q scaled by the
        // class's channel steps (the scalars that held q are reused: the softmax does not care about the order)
        KVQ_WALK(3) run_fp16(w, first[3], last[3], step, lane, q2, st);
        uint32_t q2l[32];
        if (first[0] < last[0]) { kch_prepare<0>(P, si, qh, kvh, lane, q2, q2l, qc); KVQ_WALK(0) run_low<0, true>(w, first[0], last[0], step, lane, q2, q2l, qc, cs, st); }
        if (first[1] < last[1]) { kch_prepare<1>(P, si, qh, kvh, lane, q2, q2l, qc); KVQ_WALK(1) run_low<1, true>(w, first[1], last[1], step, lane, q2, q2l, qc, cs, st); }
        if (first[2] < last[2]) { kch_prepare<2>(P, si, qh, kvh, lane, q2, q2l, qc); KVQ_WALK(2) run_8bit<true>(w, first[2], last[2], step, lane, q2, q2l, qc, st); }
    }
#undef KVQ_WALK
#undef KVQ_PI0

    // ---- the fused new token: quantized in registers, stored for later steps, one more partial result -----------
    float new_score = -INFINITY, new_v = 0.f;
    if (does_new) {
        const int page = new_page;
        const int blk = (new_slot % cv.page_tokens) / kBlockTokens, tok = new_slot % kBlockTokens;
        uint8_t *base = cv.pool[new_cls] + block_offset(cv, new_cls, P.layer, page, kvh, blk);
        const size_t region = (size_t)class_chunks(new_cls) * kBlockTokens * 16;
        const int mb = class_meta_bytes(new_cls);
        __half *meta = (__half *)(base + tok * 8);
        const bool writer = g == 0;
        float khat;
        if (KCH && new_bits != 16) {
            const size_t ti = ((size_t)P.layer * cv.Hkv + kvh) * kD + lane;
            khat = quantize_store_kch(new_kx, new_bits, __half2float(cv.kch_min[ti]),
                                      __half2float(cv.kch_step[(size_t)new_cls * cv.n_layers * cv.Hkv * kD + ti]), lane, tok, base + mb, meta, writer);
        } else {
            khat = quantize_store(new_kx, new_bits, lane, tok, base + mb, meta, writer);
        }
        new_v = quantize_store(new_vx, new_bits, lane, tok, base + mb + region, meta + 2, writer);
        new_score = wave_sum(__half2float(new_qx) * khat) * kScoreScale;
    }

    // ---- sum the 64 lanes: a transposing butterfly leaves channel c's total in lane c ----------------
    // Level `half` pairs lane l with lane l ^ half: the lanes with that bit clear end up with the sum of acc[i], the
    // others with the sum of acc[i + half].  The two widest levels are the half- and row-swap instructions of this
    // chip (v_permlane32_swap exchanges lanes 32..63 of one register with lanes 0..31 of another, v_permlane16_swap the
    // odd 16-lane rows of one with the even rows of the other): one swap and one add per pair.  The narrow levels are
    // data-parallel-primitive moves inside a row of 16 lanes.  No LDS traffic at all.
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(st.acc[i]), __float_as_uint(st.acc[i + 32]), false, false);
        st.acc[i] = __uint_as_float(r.x) + __uint_as_float(r.y);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(st.acc[i]), __float_as_uint(st.acc[i + 16]), false, false);
        st.acc[i] = __uint_as_float(r.x) + __uint_as_float(r.y);
    }
#define KVQ_LEVEL(HALF, RECV)                                                  \
    {                                                                          \
        const bool upper = (lane & (HALF)) != 0;                               \
        _Pragma("unroll") for (int i = 0; i < (HALF); ++i) {                   \
            const float keep = upper ? st.acc[i + (HALF)] : st.acc[i];         \
            const float send = upper ? st.acc[i] : st.acc[i + (HALF)];         \
            st.acc[i] = keep + (RECV);                                         \
        }                                                                      \
    }
    KVQ_LEVEL(8, dpp_mov<0x128>(send))                     // row_ror:8 = lane ^ 8 inside a row
    KVQ_LEVEL(4, dpp_mov<0x141>(dpp_mov<0x1B>(send)))      // quad_perm [3,2,1,0] (lane ^ 3), then row_half_mirror (lane ^ 7)
    KVQ_LEVEL(2, dpp_mov<0x4E>(send))                      // quad_perm [2,3,0,1]
    KVQ_LEVEL(1, dpp_mov<0xB1>(send))                      // quad_perm [1,0,3,2]
#undef KVQ_LEVEL
    const float l = wave_sum(st.l), l2 = wave_sum(st.l2), z = wave_sum(st.z);
    const float ps0 = wave_sum(st.ps[0]), ps1 = wave_sum(st.ps[1]), ps2 = wave_sum(st.ps[2]);
    // channel `lane`: its pair index inside a word decides which target multiplier it was scaled with
    const int pr = lane >> 1;
    const int tg0 = target0(pr & 7), tg1 = target1(pr & 3);
    const float mul0 = tg0 == 0 ? KVQ_M0_0 : tg0 == 1 ? KVQ_M0_1 : KVQ_M0_2;
    const float mul1 = tg1 == 0 ? KVQ_M1_0 : KVQ_M1_1;
    const float mine = st.acc[0] + (z - mul0 * ps0 - mul1 * ps1 - KVQ_OFF2 * ps2);      // relative to exp2(m)

    __shared__ float sm[NW + 1][kPartialFloats];     // row NW: the fused new token (m = its score, l = l2 = 1, value = v^)
    sm[wave][lane] = mine;
    if (lane == 0) { sm[wave][64] = st.m; sm[wave][65] = l; sm[wave][66] = l2; }
    if (wave == 0) {
        sm[NW][lane] = new_v;
        if (lane == 0) { sm[NW][64] = new_score; sm[NW][65] = 1.f; sm[NW][66] = 1.f; }
    }
    __syncthreads();
    if (wave != 0) return;
    float M = -INFINITY;
#pragma unroll
    for (int i = 0; i <= NW; ++i) M = fmaxf(M, sm[i][64]);
    float o = 0.f, L = 0.f, L2 = 0.f;
#pragma unroll
    for (int i = 0; i <= NW; ++i) {
        const float mw = sm[i][64];
        const float f = mw == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mw - M);
        o = fmaf(f, sm[i][lane], o);
        L = fmaf(f, sm[i][65], L);
        L2 = fmaf(f * f, sm[i][66], L2);
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
        float *wsu = P.ws + (size_t)unit * kPartialFloats;           // a second kernel merges the S partial results
        wsu[lane] = o;
        if (lane == 0) { wsu[64] = M; wsu[65] = L; wsu[66] = L2; }
    }
}

// Merge the S partial results of each (sequence, query head): one wavefront each.  First lane s < S fetches the
// (maximum, sum, sum of squares) triple of split s, so that the S triples travel together instead of one after the
// other; then lane = channel, four splits' vectors in flight at a time.
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
    const float *w0 = ws + u0 * kPartialFloats;
    const size_t stride = (size_t)G * kPartialFloats;
    float mw = -INFINITY, lw = 0.f, l2w = 0.f;                   // S <= kMaxSplits = 64: one lane per split
    if (lane < S) {
        const float *w = w0 + lane * stride;
        mw = w[64]; lw = w[65]; l2w = w[66];
    }
    const float M = wave_max(mw);
    const float f = mw == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mw - M);
    const float L = wave_sum(f * lw), L2 = wave_sum(f * f * l2w);
    float o = 0.f;
    for (int s0 = 0; s0 < S; s0 += 4) {
        float v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = w0[(size_t)min(s0 + u, S - 1) * stride + lane];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (s0 + u < S) o = fmaf(lane_bcast(f, s0 + u), v[u], o);
    }
    const float inv = L > 0.f ? 1.0f / L : 0.f;
    out[(size_t)oi * kD + lane] = o * inv;
    if (lane == 0) {
        if (lse) lse[oi] = L > 0.f ? (M + __builtin_amdgcn_logf(L)) * kLn2 : -INFINITY;
        if (p2) p2[oi] = L2 * inv * inv;
    }
}

}  // namespace kvq

using namespace kvq;

extern "C" size_t kvq_decode_attn_workspace(const kvq_cache *cache, int32_t n_seq)
{
    if (!cache || n_seq < 0) return 0;
    return (size_t)n_seq * cache->desc.n_q_heads * kMaxSplits * kPartialFloats * sizeof(float) + 256;
}

struct AttnPlan { long long S; int nw; };

// Chooses the launch shape and checks the workspace against it; launches nothing, so an entry point can validate
// everything before it changes any state.  `extra_tokens` are tokens that will have been appended by launch time.
static int plan_attn(const kvq_cache *cache, int32_t n_seq, int extra_tokens, const void *workspace, size_t workspace_bytes,
                     AttnPlan *plan)
{
    const kvq_cache_desc &d = cache->desc;
    const long long heads = (long long)n_seq * d.n_q_heads;
    // the kernel sums units x weight (at most 255) of one sequence in 32 bits
    if ((d.max_context / kBlockTokens + 4) * 4 * 255 >= (1LL << 31)) {
        set_error("max_context %lld is beyond what the attention kernel's unit arithmetic covers", (long long)d.max_context);
        return KVQ_ERR_UNSUPPORTED;
    }
    // Work distribution: two waves fit a SIMD, 2048 on the chip, and a launch whose waves are all resident at once has
    // no second, under-filled round.  So a (sequence, query head) gets about 2048 / heads waves, but no more than one
    // per four units (10-16 KiB each), or the per-class pipelines never reach steady state.  Up to eight of them sit
    // in one workgroup, where their partial results merge through LDS; only beyond that is the sequence split over
    // workgroups, which costs a second kernel for the merge.  len_bound is an upper bound of the longest sequence.
    long long len_bound = cache->len_bound + extra_tokens;
    if (len_bound > d.max_context) len_bound = d.max_context;
    const long long est_units = (len_bound + 63) / 64;
    long long wph = 2048 / heads;
    if (wph > est_units / 4) wph = est_units / 4;
    if (wph < 2) wph = 2;
    const int nw_auto = wph >= 8 ? 8 : wph >= 4 ? 4 : wph >= 3 ? 3 : 2;
    long long S = wph >= 16 ? wph / 8 : 1;
    if (S > kMaxSplits) S = kMaxSplits;
    const Tuning &tn = tuning();
    if (tn.attn_splits >= 1 && tn.attn_splits <= kMaxSplits) S = tn.attn_splits;
    if (heads * S > 0x3fffffffLL) { set_error("too many work items"); return KVQ_ERR_CAPACITY; }
    if (S > 1) {
        const size_t need = (size_t)heads * S * kPartialFloats * sizeof(float);
        if (!workspace || workspace_bytes < need) {
            set_error("workspace too small: %zu bytes given, %zu needed", workspace_bytes, need);
            return KVQ_ERR_INVALID_ARG;
        }
    }
    int nw = tn.attn_waves;                                     // 1, 2, 3, 4 or 8; anything else: the rule above
    if (nw != 1 && nw != 2 && nw != 3 && nw != 4 && nw != 8) nw = nw_auto;
    plan->S = S;
    plan->nw = nw;
    return KVQ_OK;
}

static int launch_attn(const kvq_cache *cache, const AttnPlan &plan, int32_t layer, const void *q, const void *k_new,
                       const void *v_new, const int32_t *seq_ids, int32_t n_seq, float *out, float *lse_out,
                       float *sum_p2_out, void *workspace, void *stream)
{
    const kvq_cache_desc &d = cache->desc;
    const long long heads = (long long)n_seq * d.n_q_heads;
    const long long S = plan.S;
    const int nw = plan.nw;
    AttnParams P;
    P.cv = cache->view;
    P.q = (const uint32_t *)q;
    P.k_new = (const __half *)k_new;
    P.v_new = (const __half *)v_new;
    P.seq_ids = seq_ids;
    P.out = out;
    P.lse = lse_out;
    P.p2 = sum_p2_out;
    P.ws = (float *)workspace;
    P.layer = layer;
    P.n_seq = n_seq;
    P.S = (int)S;
    const Tuning &tn = tuning();
    P.by_class = tn.attn_by_class;
    const int nunits = (int)(heads * S);
    const unsigned grid = (unsigned)(((nunits + 7) / 8) * 8);
    hipStream_t st = (hipStream_t)stream;
    P.longest_first = tn.attn_longest_first >= 0 ? tn.attn_longest_first : (n_seq <= 64 && n_seq % 8 == 0 && heads * S * nw > 2048) ? 1 : 0;
    P.rounds = heads * S * nw > 2048 ? 1 : 0;
    if (n_seq > 64 || n_seq % 8 != 0) P.longest_first = 0;
    if (S > 1) P.longest_first = 0;                               // the merging kernel looks partial results up by output row
    if (!cache->view.k_channel) {
        if (nw == 1) hipLaunchKernelGGL((k_decode_split<1, false>), dim3(grid), dim3(64), 0, st, P);
        else if (nw == 2) hipLaunchKernelGGL((k_decode_split<2, false>), dim3(grid), dim3(128), 0, st, P);
        else if (nw == 3) hipLaunchKernelGGL((k_decode_split<3, false>), dim3(grid), dim3(192), 0, st, P);
        else if (nw == 8) hipLaunchKernelGGL((k_decode_split<8, false>), dim3(grid), dim3(512), 0, st, P);
        else hipLaunchKernelGGL((k_decode_split<4, false>), dim3(grid), dim3(256), 0, st, P);
    } else {
        if (nw == 1) hipLaunchKernelGGL((k_decode_split<1, true>), dim3(grid), dim3(64), 0, st, P);
        else if (nw == 2) hipLaunchKernelGGL((k_decode_split<2, true>), dim3(grid), dim3(128), 0, st, P);
        else if (nw == 3) hipLaunchKernelGGL((k_decode_split<3, true>), dim3(grid), dim3(192), 0, st, P);
        else if (nw == 8) hipLaunchKernelGGL((k_decode_split<8, true>), dim3(grid), dim3(512), 0, st, P);
        else hipLaunchKernelGGL((k_decode_split<4, true>), dim3(grid), dim3(256), 0, st, P);
    }
    KVQ_HIP(hipGetLastError());
    if (S > 1) {
        hipLaunchKernelGGL(k_decode_combine, dim3((unsigned)((heads + 3) / 4)), dim3(256), 0, st, (const float *)workspace,
                           n_seq, d.n_q_heads, d.n_kv_heads, (int)S, out, lse_out, sum_p2_out);
        KVQ_HIP(hipGetLastError());
    }
    return KVQ_OK;
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
    AttnPlan plan;
    const int rc = plan_attn(cache, n_seq, 0, workspace, workspace_bytes, &plan);
    if (rc != KVQ_OK) return rc;
    return launch_attn(cache, plan, layer, q, nullptr, nullptr, seq_ids, n_seq, out, lse_out, sum_p2_out, workspace, stream);
}

// ---- the same call for callers that cannot allocate ---------------------------------------------------------------
// The split launch's partial results go to a fixed array in the library's own device image instead of a caller
// workspace.  Every GPU the library runs on holds its own copy of the array, at its own address, until the process
// ends; the array's name is only a host-side handle, so the address is looked up once per device (with that device
// current) and that pointer is what the kernels get.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];          // per device, filled on the first call there
static std::mutex g_scratch_mutex;

static int static_scratch(void **out)
{
    int dev = -1;
    KVQ_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) { set_error("device index %d is beyond the %d this library keeps a scratch address for", dev, kMaxDevices); return KVQ_ERR_UNSUPPORTED; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        KVQ_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) { set_error("the scratch array has no device address"); return KVQ_ERR_DEVICE; }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return KVQ_OK;
}

extern "C" size_t kvq_decode_attn_static_capacity(void) { return kStaticScratchBytes; }

extern "C" int kvq_decode_attn_static(const kvq_cache *cache, int32_t layer, const void *q, const int32_t *seq_ids,
                                      int32_t n_seq, float *out, float *lse_out, float *sum_p2_out, void *stream)
{
    if (!cache || !q || !out) { set_error("cache, q or out is NULL"); return KVQ_ERR_INVALID_ARG; }
    const kvq_cache_desc &d = cache->desc;
    if (layer < 0 || layer >= d.n_layers) { set_error("layer %d out of range", layer); return KVQ_ERR_INVALID_ARG; }
    if (n_seq < 0 || n_seq > d.max_seqs) { set_error("n_seq %d out of range (max_seqs %d)", n_seq, d.max_seqs); return KVQ_ERR_INVALID_ARG; }
    if (n_seq == 0) return KVQ_OK;
    void *ws = nullptr;
    const int rc_s = static_scratch(&ws);
    if (rc_s != KVQ_OK) return rc_s;
    AttnPlan plan;
    const int rc = plan_attn(cache, n_seq, 0, ws, kStaticScratchBytes, &plan);
    if (rc != KVQ_OK) {
        if (rc == KVQ_ERR_INVALID_ARG) {           // the only argument plan_attn can object to here is the scratch size
            set_error("this launch needs more than the %zu bytes of the library's fixed scratch array "
                      "(%d sequences x %d query heads x its split count x %zu bytes): use kvq_decode_attn with a workspace",
                      kStaticScratchBytes, n_seq, d.n_q_heads, (size_t)kPartialFloats * sizeof(float));
            return KVQ_ERR_CAPACITY;
        }
        return rc;
    }
    return launch_attn(cache, plan, layer, q, nullptr, nullptr, seq_ids, n_seq, out, lse_out, sum_p2_out, ws, stream);
}

extern "C" int kvq_append_decode_attn(kvq_cache *cache, int32_t layer, const void *k, const void *v, const uint8_t *bits,
                                      const void *q, const int32_t *seq_ids, int32_t n_seq, float *out, float *lse_out,
                                      float *sum_p2_out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!cache || !k || !v || !q || !out) { set_error("cache, k, v, q or out is NULL"); return KVQ_ERR_INVALID_ARG; }
    const kvq_cache_desc &d = cache->desc;
    if (layer < 0 || layer >= d.n_layers) { set_error("layer %d out of range", layer); return KVQ_ERR_INVALID_ARG; }
    if (n_seq < 0 || n_seq > d.max_seqs) { set_error("n_seq %d out of range (max_seqs %d)", n_seq, d.max_seqs); return KVQ_ERR_INVALID_ARG; }
    if (n_seq == 0) return KVQ_OK;
    const bool bookkeeping = layer == 0 && bits;                   // bits == NULL: done by kvq_features_controller
    AttnPlan plan;                                                 // every check comes before the first state change
    const int rc0 = plan_attn(cache, n_seq, bookkeeping ? 1 : 0, workspace, workspace_bytes, &plan);
    if (rc0 != KVQ_OK) return rc0;
    if (bookkeeping) {
        const int rc = kvq_append_bookkeeping(cache, bits, seq_ids, n_seq, 1, stream);
        if (rc != KVQ_OK) return rc;
    }
    return launch_attn(cache, plan, layer, q, k, v, seq_ids, n_seq, out, lse_out, sum_p2_out, workspace, stream);
}

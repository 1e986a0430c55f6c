/*
 * kvq_oracle.c -- plain CPU oracle for the adaptive mixed-precision KV-cache hot path.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the smoke check and the
 * benchmark's "cpu_baseline" leg may load it.  It shares no code, header, table or helper with
 * the HIP library; the HIP library never calls it.
 *
 * It is written to be checked against the paper by eye: scalar loops, fp64 for every quantity
 * that has an exact definition (features, controller, attention), and emulated IEEE binary16 /
 * binary32 arithmetic for the one step that is an encoding and must agree bit for bit (the
 * quantizer).  No blocking, no fusion, no reordering.  OpenMP appears only as a "parallel for"
 * over independent (sequence, kv-head) units in the batch wrappers.
 *
 * Passages followed (paper sections / equations):
 *   - Sec. 3.2 "Preliminary": q, K<-Concat(K,k), V<-Concat(V,v), a = Softmax(q K^T / sqrt(d_k)) V.
 *   - Sec. 3.4 "Framework Overview": four stages; 16-bit class means FP16 storage.
 *   - Sec. 3.5 "Token-Level Saliency Features": entropy H_t, rarity R_t, attention variance V_t,
 *     confidence C_t, s_t = [H_t, R_t, V_t, C_t].
 *   - Sec. 3.6 "Lightweight Controller Network": ReLU MLP, logits o_t, argmax, IndexToBit;
 *     class index -> bit width {0,1,2,3} -> {2,4,8,16} (Algorithm 1, label mapping step).
 *   - Sec. 3.7 "Adaptive KV Quantization": k^ = Q_b(k), v^ = Q_b(v), appended to the cache.
 *
 * Readings of what the paper leaves open (the same list is kept in the design document):
 *   - Q_b is per (token, kv-head) vector of 64 elements, asymmetric min/max, with an fp16 scale and
 *     the fp16 minimum as zero-point; K and V are quantized independently with the same b.
 *   - logarithms are natural; C_t is the largest softmax probability; Var is the population
 *     variance (divide by the row length) of one attention-probability row per query head.
 *   - argmax ties go to the lowest class index.
 *   - grouped-query attention: query head h reads kv-head h / (Hq/Hkv).
 *
 * PINS: every function below is pinned by the CPU test-suite against closed forms, library
 * routines and brute force (see tests/test_oracle_*.py).  What cannot be pinned, because the
 * paper prints nothing to check it against, is the CHOICE of quantization scheme, of C_t and of
 * the variance axis: for those choices parity with the paper is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define KVQ_D 64           /* per-head feature dimension d (Sec. 3.2 notation) */
#define KVQ_REC 128        /* bytes reserved for one packed vector in the canonical dump */

/* ------------------------------------------------------------------------------------------ */
/* IEEE-754 binary16 <-> binary32, written out bit by bit (pinned exhaustively against numpy)  */
/* ------------------------------------------------------------------------------------------ */

float kvq_oracle_f16_to_f32(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) & 1u;
    uint32_t expo = (uint32_t)(h >> 10) & 0x1fu;
    uint32_t mant = (uint32_t)h & 0x3ffu;
    double v;
    if (expo == 0x1fu) {
        v = mant ? (double)NAN : (double)INFINITY;
    } else if (expo == 0) {
        v = ldexp((double)mant, -24);                 /* subnormal: mant * 2^-24 */
    } else {
        v = ldexp((double)(mant + 1024u), (int)expo - 25); /* (1 + mant/1024) * 2^(expo-15) */
    }
    return (float)(sign ? -v : v);                    /* every binary16 value is exact in binary32 */
}

uint16_t kvq_oracle_f32_to_f16(float f)
{
    /* round to nearest, ties to even; subnormals kept; overflow to infinity */
    uint32_t u;
    memcpy(&u, &f, 4);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    double a = fabs((double)f);
    if (isnan(f)) return (uint16_t)(sign | 0x7e00u);
    if (a >= 65520.0) return (uint16_t)(sign | 0x7c00u);      /* 65520 is the tie to 2^16 -> inf */
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                                        /* a = m * 2^e, m in [0.5,1) */
    int ulp_exp = (e - 1) - 10;                                /* exponent of one ulp for a normal result */
    if (ulp_exp < -24) ulp_exp = -24;                          /* subnormal spacing */
    double scaled = ldexp(a, -ulp_exp);                        /* exact: a power-of-two scaling */
    double r = nearbyint(scaled);                              /* default mode: ties to even */
    /* r is an integer number of ulps; rebuild the bit pattern */
    double val = ldexp(r, ulp_exp);
    if (val >= 65536.0) return (uint16_t)(sign | 0x7c00u);
    if (val < ldexp(1.0, -14)) {                               /* subnormal or zero */
        return (uint16_t)(sign | (uint16_t)ldexp(val, 24));
    }
    int e2;
    double m2 = frexp(val, &e2);                               /* val = m2 * 2^e2, m2 in [0.5,1) */
    uint32_t expo = (uint32_t)(e2 - 1 + 15);
    uint32_t mant = (uint32_t)(ldexp(m2, 11)) - 1024u;         /* (2*m2 - 1) * 1024 */
    return (uint16_t)(sign | (expo << 10) | mant);
}

/* array forms of the two conversions, so that the pins can sweep millions of values */
void kvq_oracle_f32_to_f16_array(const float *f, int64_t n, uint16_t *h)
{
    for (int64_t i = 0; i < n; ++i) h[i] = kvq_oracle_f32_to_f16(f[i]);
}

void kvq_oracle_f16_to_f32_array(const uint16_t *h, int64_t n, float *f)
{
    for (int64_t i = 0; i < n; ++i) f[i] = kvq_oracle_f16_to_f32(h[i]);
}

/* ------------------------------------------------------------------------------------------ */
/* Sec. 3.7: Q_b for one 64-element fp16 vector                                                */
/* ------------------------------------------------------------------------------------------ */

/*
 * codes: KVQ_REC bytes.  For b in {2,4,8}: element i occupies bits [i*b, i*b+b) of the byte stream
 * (little-endian bit order), remaining bytes zero.  For b = 16: the 64 binary16 patterns,
 * little-endian, and scale = zero = 0.
 * All arithmetic on the way to the codes is IEEE binary32, round-to-nearest-even, in this order:
 *   range = f32(max) - f32(min);  scale32 = range / levels;  scale_h = f16(scale32);  s = f32(scale_h)
 *   code_i = clamp(rint((f32(x_i) - f32(min)) / s), 0, levels)          (true division)
 * The zero-point is the fp16 minimum itself; a minimum that is a zero of either sign is stored as +0.
 */
void kvq_oracle_quantize_vec(const uint16_t *x, int bits, uint8_t *codes, uint16_t *scale_h, uint16_t *zero_h)
{
    memset(codes, 0, KVQ_REC);
    if (bits == 16) {
        for (int i = 0; i < KVQ_D; ++i) {
            codes[2 * i] = (uint8_t)(x[i] & 0xffu);
            codes[2 * i + 1] = (uint8_t)(x[i] >> 8);
        }
        *scale_h = 0;
        *zero_h = 0;
        return;
    }
    const int levels = (1 << bits) - 1;
    volatile float mn = kvq_oracle_f16_to_f32(x[0]);
    volatile float mx = mn;
    uint16_t mn_bits = x[0];
    for (int i = 1; i < KVQ_D; ++i) {
        float f = kvq_oracle_f16_to_f32(x[i]);
        if (f < mn) { mn = f; mn_bits = x[i]; }
        if (f > mx) { mx = f; }
    }
    if (mn == 0.0f) { mn = 0.0f; mn_bits = 0; }               /* canonical +0 */
    if (mx == 0.0f) { mx = 0.0f; }                            /* likewise: the range of a vector of zeros of either sign is +0 */
    volatile float range = mx - mn;
    volatile float scale32 = range / (float)levels;
    const uint16_t sh = kvq_oracle_f32_to_f16(scale32);
    volatile float s = kvq_oracle_f16_to_f32(sh);
    *scale_h = sh;
    *zero_h = mn_bits;
    if (s == 0.0f) return;                                     /* constant (or sub-resolution) vector: all codes 0 */
    for (int i = 0; i < KVQ_D; ++i) {
        volatile float d = kvq_oracle_f16_to_f32(x[i]) - mn;
        volatile float t = d / s;
        float r = rintf(t);                                    /* ties to even */
        if (r < 0.0f) r = 0.0f;
        if (r > (float)levels) r = (float)levels;
        uint32_t c = (uint32_t)r;
        int bit = i * bits;
        codes[bit >> 3] |= (uint8_t)(c << (bit & 7));          /* b divides 8: a code never straddles bytes */
    }
}

static inline uint32_t unpack_code(const uint8_t *codes, int bits, int i)
{
    int bit = i * bits;
    return ((uint32_t)codes[bit >> 3] >> (bit & 7)) & ((1u << bits) - 1u);
}

/* x^_i = zero + code_i * scale, evaluated in fp64 (exact: <=8-bit integer times an fp16 value plus an fp16 value) */
void kvq_oracle_dequantize_vec(const uint8_t *codes, uint16_t scale_h, uint16_t zero_h, int bits, double *out)
{
    if (bits == 16) {
        for (int i = 0; i < KVQ_D; ++i) {
            uint16_t h = (uint16_t)(codes[2 * i] | ((uint16_t)codes[2 * i + 1] << 8));
            out[i] = (double)kvq_oracle_f16_to_f32(h);
        }
        return;
    }
    const double s = (double)kvq_oracle_f16_to_f32(scale_h);
    const double z = (double)kvq_oracle_f16_to_f32(zero_h);
    for (int i = 0; i < KVQ_D; ++i) out[i] = z + (double)unpack_code(codes, bits, i) * s;
}

/*
 * Sec. 3.2 Concat + Sec. 3.7: quantize T new tokens of one sequence and one layer and write their
 * records at the tail of the canonical arrays.
 *   k, v     [T][Hkv][64] binary16 bit patterns
 *   bits     [T]          2/4/8/16, one decision per token shared by K, V and all heads
 *   codes    [T][Hkv][2][KVQ_REC]   (index 0 = K, 1 = V)
 *   meta     [T][Hkv][2][2]         (scale bits, zero bits)
 * Returns 0, or -1 on an invalid bit width.
 */
int kvq_oracle_append(const uint16_t *k, const uint16_t *v, const uint8_t *bits, int64_t T, int Hkv,
                      uint8_t *codes, uint16_t *meta)
{
    for (int64_t t = 0; t < T; ++t) {
        int b = bits[t];
        if (b != 2 && b != 4 && b != 8 && b != 16) return -1;
        for (int h = 0; h < Hkv; ++h) {
            int64_t vec = t * Hkv + h;
            kvq_oracle_quantize_vec(k + vec * KVQ_D, b, codes + (vec * 2 + 0) * KVQ_REC,
                                    meta + (vec * 2 + 0) * 2, meta + (vec * 2 + 0) * 2 + 1);
            kvq_oracle_quantize_vec(v + vec * KVQ_D, b, codes + (vec * 2 + 1) * KVQ_REC,
                                    meta + (vec * 2 + 1) * 2, meta + (vec * 2 + 1) * 2 + 1);
        }
    }
    return 0;
}

/* Batch form of the above for timing runs: the T tokens are independent, so they are split over threads. */
int kvq_oracle_append_parallel(const uint16_t *k, const uint16_t *v, const uint8_t *bits, int64_t T, int Hkv,
                               uint8_t *codes, uint16_t *meta)
{
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t t = 0; t < T; ++t)
        bad |= kvq_oracle_append(k + t * Hkv * KVQ_D, v + t * Hkv * KVQ_D, bits + t, 1, Hkv,
                                 codes + t * Hkv * 2 * KVQ_REC, meta + t * Hkv * 2 * 2) != 0;
    return bad ? -1 : 0;
}

/* ------------------------------------------------------------------------------------------ */
/* Sec. 3.2: a = Softmax(q K^^T / sqrt(d_k)) V^  for one sequence, all query heads             */
/* ------------------------------------------------------------------------------------------ */

/*
 *   q      [Hq][64] binary16 bit patterns
 *   bits   [len], codes [len][Hkv][2][KVQ_REC], meta [len][Hkv][2][2]  (canonical arrays)
 *   out    [Hq][64] fp64
 *   lse    [Hq] fp64 or NULL: log sum_j exp(s_j)
 *   probs  [Hq][ld] fp64 or NULL: the attention probabilities p_j (row h starts at probs + h*ld)
 * Every cached token j < len takes part, the newest one included, in its quantized form.
 */
void kvq_oracle_decode_attn(const uint16_t *q, const uint8_t *bits, const uint8_t *codes, const uint16_t *meta,
                            int64_t len, int Hq, int Hkv, double *out, double *lse, double *probs, int64_t ld)
{
    const int group = Hq / Hkv;
    const double inv_sqrt_d = 1.0 / sqrt((double)KVQ_D);
    double *score = (double *)malloc(sizeof(double) * (size_t)(len > 0 ? len : 1));
    for (int h = 0; h < Hq; ++h) {
        const int kvh = h / group;
        double qd[KVQ_D], kd[KVQ_D], vd[KVQ_D];
        for (int c = 0; c < KVQ_D; ++c) qd[c] = (double)kvq_oracle_f16_to_f32(q[h * KVQ_D + c]);
        double mx = -INFINITY;
        for (int64_t j = 0; j < len; ++j) {
            int64_t vec = j * Hkv + kvh;
            kvq_oracle_dequantize_vec(codes + (vec * 2 + 0) * KVQ_REC, meta[(vec * 2 + 0) * 2],
                                      meta[(vec * 2 + 0) * 2 + 1], bits[j], kd);
            double dot = 0.0;
            for (int c = 0; c < KVQ_D; ++c) dot += qd[c] * kd[c];
            score[j] = dot * inv_sqrt_d;
            if (score[j] > mx) mx = score[j];
        }
        double denom = 0.0;
        for (int64_t j = 0; j < len; ++j) denom += exp(score[j] - mx);
        double acc[KVQ_D];
        for (int c = 0; c < KVQ_D; ++c) acc[c] = 0.0;
        for (int64_t j = 0; j < len; ++j) {
            double p = exp(score[j] - mx) / denom;
            if (probs) probs[(int64_t)h * ld + j] = p;
            int64_t vec = j * Hkv + kvh;
            kvq_oracle_dequantize_vec(codes + (vec * 2 + 1) * KVQ_REC, meta[(vec * 2 + 1) * 2],
                                      meta[(vec * 2 + 1) * 2 + 1], bits[j], vd);
            for (int c = 0; c < KVQ_D; ++c) acc[c] += p * vd[c];
        }
        for (int c = 0; c < KVQ_D; ++c) out[h * KVQ_D + c] = acc[c];
        if (lse) lse[h] = (len > 0) ? mx + log(denom) : -INFINITY;
    }
    free(score);
}

/*
 * Batch wrapper: B sequences with fixed-stride canonical arrays (stride max_len tokens per
 * sequence), lengths lens[b].  Work is split over (sequence, kv-head) units only.
 *   q [B][Hq][64]; bits [B][max_len]; codes [B][max_len][Hkv][2][KVQ_REC]; meta [B][max_len][Hkv][2][2]
 *   out [B][Hq][64]; lse [B][Hq] or NULL; sum_p2 [B][Hq] or NULL (sum_j p_j^2 per query head)
 * Returns the number of threads the parallel region ran with.
 */
int kvq_oracle_decode_attn_batch(const uint16_t *q, const uint8_t *bits, const uint8_t *codes, const uint16_t *meta,
                                 const int32_t *lens, int B, int64_t max_len, int Hq, int Hkv,
                                 double *out, double *lse, double *sum_p2)
{
    const int group = Hq / Hkv;
    const double inv_sqrt_d = 1.0 / sqrt((double)KVQ_D);
    int threads_used = 1;
#pragma omp parallel
    {
#pragma omp single
        {
#ifdef _OPENMP
            threads_used = omp_get_num_threads();
#endif
        }
#pragma omp for collapse(2) schedule(dynamic, 1)
        for (int b = 0; b < B; ++b) {
            for (int kvh = 0; kvh < Hkv; ++kvh) {
                const int64_t len = lens[b];
                const uint8_t *sb = bits + (int64_t)b * max_len;
                const uint8_t *sc = codes + (int64_t)b * max_len * Hkv * 2 * KVQ_REC;
                const uint16_t *sm = meta + (int64_t)b * max_len * Hkv * 2 * 2;
                double *score = (double *)malloc(sizeof(double) * (size_t)(len > 0 ? len : 1));
                for (int g = 0; g < group; ++g) {
                    const int h = kvh * group + g;
                    const uint16_t *qh = q + ((int64_t)b * Hq + h) * KVQ_D;
                    double qd[KVQ_D], kd[KVQ_D], vd[KVQ_D], acc[KVQ_D];
                    for (int c = 0; c < KVQ_D; ++c) qd[c] = (double)kvq_oracle_f16_to_f32(qh[c]);
                    double mx = -INFINITY;
                    for (int64_t j = 0; j < len; ++j) {
                        int64_t vec = j * Hkv + kvh;
                        kvq_oracle_dequantize_vec(sc + (vec * 2 + 0) * KVQ_REC, sm[(vec * 2 + 0) * 2],
                                                  sm[(vec * 2 + 0) * 2 + 1], sb[j], kd);
                        double dot = 0.0;
                        for (int c = 0; c < KVQ_D; ++c) dot += qd[c] * kd[c];
                        score[j] = dot * inv_sqrt_d;
                        if (score[j] > mx) mx = score[j];
                    }
                    double denom = 0.0;
                    for (int64_t j = 0; j < len; ++j) denom += exp(score[j] - mx);
                    for (int c = 0; c < KVQ_D; ++c) acc[c] = 0.0;
                    double p2 = 0.0;
                    for (int64_t j = 0; j < len; ++j) {
                        double p = exp(score[j] - mx) / denom;
                        p2 += p * p;
                        int64_t vec = j * Hkv + kvh;
                        kvq_oracle_dequantize_vec(sc + (vec * 2 + 1) * KVQ_REC, sm[(vec * 2 + 1) * 2],
                                                  sm[(vec * 2 + 1) * 2 + 1], sb[j], vd);
                        for (int c = 0; c < KVQ_D; ++c) acc[c] += p * vd[c];
                    }
                    double *o = out + ((int64_t)b * Hq + h) * KVQ_D;
                    for (int c = 0; c < KVQ_D; ++c) o[c] = acc[c];
                    if (lse) lse[(int64_t)b * Hq + h] = (len > 0) ? mx + log(denom) : -INFINITY;
                    if (sum_p2) sum_p2[(int64_t)b * Hq + h] = p2;
                }
                free(score);
            }
        }
    }
    return threads_used;
}

/* ------------------------------------------------------------------------------------------ */
/* Sec. 3.5: s_t = [H_t, R_t, V_t, C_t]                                                         */
/* ------------------------------------------------------------------------------------------ */

/*
 *   logits      [n][vocab] fp32            z_t
 *   ids         [n]                        token id x_t
 *   counts      [vocab]                    c(.) as they stand BEFORE these n tokens are counted
 *   N, Vobs                                total observed tokens, distinct observed tokens (before)
 *   attn_probs  [n][Hq][ld] fp64           final-layer attention probabilities of the token's own row
 *   attn_len    [n]                        row length l (entries 0..l-1 of each row are used)
 *   feats       [n][4] fp32                H, R, V, C, each rounded once from fp64
 */
void kvq_oracle_features(const float *logits, int64_t n, int64_t vocab, const int32_t *ids,
                         const int64_t *counts, int64_t N, int64_t Vobs,
                         const double *attn_probs, const int32_t *attn_len, int Hq, int64_t ld, float *feats)
{
    for (int64_t t = 0; t < n; ++t) {
        const float *z = logits + t * vocab;
        /* p = Softmax(z); H = -sum p log p, with log p taken as the log-softmax so that p = 0 contributes 0 */
        double m = -INFINITY;
        for (int64_t v = 0; v < vocab; ++v) if ((double)z[v] > m) m = (double)z[v];
        double S = 0.0;
        for (int64_t v = 0; v < vocab; ++v) S += exp((double)z[v] - m);
        const double logS = log(S);
        double H = 0.0, pmax = 0.0;
        for (int64_t v = 0; v < vocab; ++v) {
            double p = exp((double)z[v] - m) / S;
            double logp = ((double)z[v] - m) - logS;
            H -= p * logp;
            if (p > pmax) pmax = p;
        }
        /* R = -log((c(x)+1) / (N + |V_obs| + 1)) */
        const double R = -log(((double)counts[ids[t]] + 1.0) / ((double)N + (double)Vobs + 1.0));
        /* V = (1/h) sum_i Var(A_i), population variance over the l entries of head i's row */
        const int64_t l = attn_len[t];
        double V = 0.0;
        for (int i = 0; i < Hq; ++i) {
            const double *row = attn_probs + (t * Hq + i) * ld;
            double mean = 0.0;
            for (int64_t j = 0; j < l; ++j) mean += row[j];
            mean /= (double)l;
            double var = 0.0;
            for (int64_t j = 0; j < l; ++j) var += (row[j] - mean) * (row[j] - mean);
            V += var / (double)l;
        }
        V /= (double)Hq;
        feats[t * 4 + 0] = (float)H;
        feats[t * 4 + 1] = (float)R;
        feats[t * 4 + 2] = (float)V;
        feats[t * 4 + 3] = (float)pmax;
    }
}

/*
 * Running-count update that follows a feature call (Sec. 3.5, "running count"): all n tokens are
 * scored against the table as passed in, then counted: c[id] += 1 each, N += n, and Vobs grows by
 * the number of distinct ids whose count was zero.  totals = {N, Vobs}.
 */
void kvq_oracle_counts_update(const int32_t *ids, int64_t n, int64_t *counts, int64_t *totals)
{
    for (int64_t t = 0; t < n; ++t) {
        if (counts[ids[t]] == 0) totals[1] += 1;
        counts[ids[t]] += 1;
    }
    totals[0] += n;
}

/* ------------------------------------------------------------------------------------------ */
/* Sec. 3.6: controller forward, argmax, IndexToBit                                             */
/* ------------------------------------------------------------------------------------------ */

/*
 *   feats   [n][dims[0]] fp32
 *   n_linear linear layers with sizes dims[0] -> dims[1] -> ... -> dims[n_linear]; ReLU after all but the last
 *   W[l]    row-major [dims[l+1]][dims[l]] fp32,  b[l] [dims[l+1]] fp32
 *   bits    [n]  2/4/8/16 = {2,4,8,16}[first index of the largest logit]
 *   logits  [n][dims[n_linear]] fp64 or NULL
 * All arithmetic in fp64 on the given fp32 numbers.
 */
void kvq_oracle_controller(const float *feats, int64_t n, int n_linear, const int32_t *dims,
                           const float *const *W, const float *const *bvec, uint8_t *bits, double *logits)
{
    static const uint8_t index_to_bit[4] = {2, 4, 8, 16};
    int maxw = 0;
    for (int l = 0; l <= n_linear; ++l) if (dims[l] > maxw) maxw = dims[l];
    double *cur = (double *)malloc(sizeof(double) * (size_t)maxw);
    double *nxt = (double *)malloc(sizeof(double) * (size_t)maxw);
    for (int64_t t = 0; t < n; ++t) {
        for (int i = 0; i < dims[0]; ++i) cur[i] = (double)feats[t * dims[0] + i];
        for (int l = 0; l < n_linear; ++l) {
            const int in = dims[l], outw = dims[l + 1];
            for (int o = 0; o < outw; ++o) {
                double a = (double)bvec[l][o];
                for (int i = 0; i < in; ++i) a += (double)W[l][(int64_t)o * in + i] * cur[i];
                if (l + 1 < n_linear && a < 0.0) a = 0.0;      /* ReLU on hidden layers only */
                nxt[o] = a;
            }
            double *tmp = cur; cur = nxt; nxt = tmp;
        }
        const int nout = dims[n_linear];
        int best = 0;
        for (int o = 1; o < nout; ++o) if (cur[o] > cur[best]) best = o;   /* strict: first maximum wins */
        bits[t] = index_to_bit[best];
        if (logits) for (int o = 0; o < nout; ++o) logits[t * nout + o] = cur[o];
    }
    free(cur);
    free(nxt);
}

/* ------------------------------------------------------------------------------------------ */
/* Sec. 3.3 (expected bit-width): E[b] = sum_x p(x) f(x), here the mean of the widths assigned */
/* to the n cached tokens; next to it the storage those widths imply under Q_b of Sec. 3.7 as   */
/* read in this file: per (token, kv-head), K and V each store 64*b/8 code bytes plus an fp16   */
/* scale and an fp16 minimum (b < 16), or 64 fp16 values (b = 16).                              */
/* ------------------------------------------------------------------------------------------ */
int kvq_oracle_accounting(const uint8_t *bits, int64_t n, int Hkv, int layers, double *expected_bits,
                          double *effective_bits, int64_t *payload_bytes)
{
    double sum_b = 0.0;
    int64_t bytes = 0;
    for (int64_t t = 0; t < n; ++t) {
        const int b = bits[t];
        if (b != 2 && b != 4 && b != 8 && b != 16) return -1;
        sum_b += (double)b;
        const int64_t one_vector = b == 16 ? (int64_t)KVQ_D * 2 : (int64_t)KVQ_D * b / 8 + 2 + 2;
        bytes += 2 * one_vector;                                  /* K and V */
    }
    bytes *= (int64_t)Hkv * layers;
    *expected_bits = n > 0 ? sum_b / (double)n : 0.0;
    /* bits actually stored per cached element, metadata included */
    *effective_bits = n > 0 ? (double)bytes * 8.0 / ((double)n * Hkv * layers * 2.0 * KVQ_D) : 0.0;
    *payload_bytes = bytes;
    return 0;
}

/* ------------------------------------------------------------------------------------------ */
/* Stand-in for the "rule-based dynamic KV policy" baseline of Sec. 4 (the paper only says it   */
/* uses hand-crafted heuristics; its rules are not given, so this rule is this build's own):    */
/* an importance score linear in the features, cut by three ascending thresholds.               */
/*   score = bias + sum_i w_i s_i (fp64 on the fp32 inputs), class = #{k : score > thr_k},      */
/*   bits = {2,4,8,16}[class].                                                                  */
/* ------------------------------------------------------------------------------------------ */
void kvq_oracle_rule_policy(const float *feats, int64_t n, const float *w, float bias, const float *thr, uint8_t *bits,
                            double *score)
{
    static const uint8_t index_to_bit[4] = {2, 4, 8, 16};
    for (int64_t t = 0; t < n; ++t) {
        double u = (double)bias;
        for (int i = 0; i < 4; ++i) u += (double)w[i] * (double)feats[t * 4 + i];
        int cls = 0;
        for (int k = 0; k < 3; ++k) if (u > (double)thr[k]) cls += 1;
        bits[t] = index_to_bit[cls];
        if (score) score[t] = u;
    }
}

/* ------------------------------------------------------------------------------------------ */
/* Variant Q_b for keys: static per-channel quantization.  The paper leaves Q_b open (Sec. 3.7) */
/* and cites per-channel key quantizers as related work (Sec. 2); this variant follows that     */
/* idea in its simplest form.  The caller supplies, per (kv-head, channel c), a minimum m_c and  */
/* a range r_c (fp16, from an offline calibration).  For a token stored at b bits:              */
/*   step_c = fp16(fp32(r_c) / levels),  code_c = clamp(rint((x_c - m_c) / fp32(step_c)), 0,     */
/*   levels) in IEEE binary32 (code 0 where the step is 0),  k^_c = m_c + code_c * step_c.       */
/* Values outside [m_c, m_c + r_c] clamp.  No per-token scale or minimum is stored for K (its    */
/* two meta entries stay 0); V and the 16-bit class are unchanged.                               */
/* ------------------------------------------------------------------------------------------ */
static uint16_t kch_step(uint16_t range_h, int levels)
{
    volatile float r = kvq_oracle_f16_to_f32(range_h);
    volatile float st = r / (float)levels;
    return kvq_oracle_f32_to_f16(st);
}

void kvq_oracle_kch_quantize_vec(const uint16_t *x, int bits, const uint16_t *kmin, const uint16_t *krange, uint8_t *codes)
{
    memset(codes, 0, KVQ_REC);
    if (bits == 16) {
        for (int i = 0; i < KVQ_D; ++i) {
            codes[2 * i] = (uint8_t)(x[i] & 0xffu);
            codes[2 * i + 1] = (uint8_t)(x[i] >> 8);
        }
        return;
    }
    const int levels = (1 << bits) - 1;
    for (int i = 0; i < KVQ_D; ++i) {
        volatile float s = kvq_oracle_f16_to_f32(kch_step(krange[i], levels));
        if (s == 0.0f) continue;
        volatile float d = kvq_oracle_f16_to_f32(x[i]) - kvq_oracle_f16_to_f32(kmin[i]);
        volatile float t = d / s;
        float r = rintf(t);
        if (r < 0.0f) r = 0.0f;
        if (r > (float)levels) r = (float)levels;
        uint32_t c = (uint32_t)r;
        int bit = i * bits;
        codes[bit >> 3] |= (uint8_t)(c << (bit & 7));
    }
}

void kvq_oracle_kch_dequantize_vec(const uint8_t *codes, int bits, const uint16_t *kmin, const uint16_t *krange, double *out)
{
    if (bits == 16) {
        kvq_oracle_dequantize_vec(codes, 0, 0, 16, out);
        return;
    }
    const int levels = (1 << bits) - 1;
    for (int i = 0; i < KVQ_D; ++i)
        out[i] = (double)kvq_oracle_f16_to_f32(kmin[i]) +
                 (double)unpack_code(codes, bits, i) * (double)kvq_oracle_f16_to_f32(kch_step(krange[i], levels));
}

/* kvq_oracle_append with the per-channel variant for K: kmin, krange are [Hkv][64] */
int kvq_oracle_append_kch(const uint16_t *k, const uint16_t *v, const uint8_t *bits, int64_t T, int Hkv,
                          const uint16_t *kmin, const uint16_t *krange, uint8_t *codes, uint16_t *meta)
{
    for (int64_t t = 0; t < T; ++t) {
        int b = bits[t];
        if (b != 2 && b != 4 && b != 8 && b != 16) return -1;
        for (int h = 0; h < Hkv; ++h) {
            int64_t vec = t * Hkv + h;
            kvq_oracle_kch_quantize_vec(k + vec * KVQ_D, b, kmin + h * KVQ_D, krange + h * KVQ_D, codes + (vec * 2 + 0) * KVQ_REC);
            meta[(vec * 2 + 0) * 2] = 0;
            meta[(vec * 2 + 0) * 2 + 1] = 0;
            kvq_oracle_quantize_vec(v + vec * KVQ_D, b, codes + (vec * 2 + 1) * KVQ_REC,
                                    meta + (vec * 2 + 1) * 2, meta + (vec * 2 + 1) * 2 + 1);
        }
    }
    return 0;
}

/* kvq_oracle_decode_attn (Sec. 3.2) over a cache whose keys use the per-channel variant */
void kvq_oracle_decode_attn_kch(const uint16_t *q, const uint8_t *bits, const uint8_t *codes, const uint16_t *meta,
                                const uint16_t *kmin, const uint16_t *krange, int64_t len, int Hq, int Hkv,
                                double *out, double *lse)
{
    const int group = Hq / Hkv;
    const double inv_sqrt_d = 1.0 / sqrt((double)KVQ_D);
    double *score = (double *)malloc(sizeof(double) * (size_t)(len > 0 ? len : 1));
    for (int h = 0; h < Hq; ++h) {
        const int kvh = h / group;
        double qd[KVQ_D], kd[KVQ_D], vd[KVQ_D];
        for (int c = 0; c < KVQ_D; ++c) qd[c] = (double)kvq_oracle_f16_to_f32(q[h * KVQ_D + c]);
        double mx = -INFINITY;
        for (int64_t j = 0; j < len; ++j) {
            int64_t vec = j * Hkv + kvh;
            kvq_oracle_kch_dequantize_vec(codes + (vec * 2 + 0) * KVQ_REC, bits[j], kmin + kvh * KVQ_D, krange + kvh * KVQ_D, kd);
            double dot = 0.0;
            for (int c = 0; c < KVQ_D; ++c) dot += qd[c] * kd[c];
            score[j] = dot * inv_sqrt_d;
            if (score[j] > mx) mx = score[j];
        }
        double denom = 0.0;
        for (int64_t j = 0; j < len; ++j) denom += exp(score[j] - mx);
        double acc[KVQ_D];
        for (int c = 0; c < KVQ_D; ++c) acc[c] = 0.0;
        for (int64_t j = 0; j < len; ++j) {
            double p = exp(score[j] - mx) / denom;
            int64_t vec = j * Hkv + kvh;
            kvq_oracle_dequantize_vec(codes + (vec * 2 + 1) * KVQ_REC, meta[(vec * 2 + 1) * 2],
                                      meta[(vec * 2 + 1) * 2 + 1], bits[j], vd);
            for (int c = 0; c < KVQ_D; ++c) acc[c] += p * vd[c];
        }
        for (int c = 0; c < KVQ_D; ++c) out[h * KVQ_D + c] = acc[c];
        if (lse) lse[h] = (len > 0) ? mx + log(denom) : -INFINITY;
    }
    free(score);
}

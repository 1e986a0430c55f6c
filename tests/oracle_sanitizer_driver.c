/* Runs every routine of the CPU oracle once on small pseudo-random inputs.  Built together with oracle/kvq_oracle.c
 * under -fsanitize=address,undefined by tests/test_oracle_sanitizers.py: any out-of-bounds access, use of
 * uninitialised padding through a wrong size, signed overflow or misaligned access in the oracle aborts the run. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

float kvq_oracle_f16_to_f32(uint16_t h);
uint16_t kvq_oracle_f32_to_f16(float f);
void kvq_oracle_quantize_vec(const uint16_t *x, int bits, uint8_t *codes, uint16_t *scale_h, uint16_t *zero_h);
void kvq_oracle_dequantize_vec(const uint8_t *codes, uint16_t scale_h, uint16_t zero_h, int bits, double *out);
int kvq_oracle_append(const uint16_t *k, const uint16_t *v, const uint8_t *bits, int64_t T, int Hkv, uint8_t *codes, uint16_t *meta);
int kvq_oracle_append_parallel(const uint16_t *k, const uint16_t *v, const uint8_t *bits, int64_t T, int Hkv, uint8_t *codes, uint16_t *meta);
void kvq_oracle_decode_attn(const uint16_t *q, const uint8_t *bits, const uint8_t *codes, const uint16_t *meta, int64_t len,
                            int Hq, int Hkv, double *out, double *lse, double *probs, int64_t ld);
int kvq_oracle_decode_attn_batch(const uint16_t *q, const uint8_t *bits, const uint8_t *codes, const uint16_t *meta,
                                 const int32_t *lens, int B, int64_t max_len, int Hq, int Hkv, double *out, double *lse, double *sum_p2);
void kvq_oracle_features(const float *logits, int64_t n, int64_t vocab, const int32_t *ids, const int64_t *counts, int64_t N,
                         int64_t Vobs, const double *attn_probs, const int32_t *attn_len, int Hq, int64_t ld, float *feats);
void kvq_oracle_counts_update(const int32_t *ids, int64_t n, int64_t *counts, int64_t *totals);
void kvq_oracle_controller(const float *feats, int64_t n, int n_linear, const int32_t *dims, const float *const *W,
                           const float *const *bvec, uint8_t *bits, double *logits);
int kvq_oracle_append_kch(const uint16_t *k, const uint16_t *v, const uint8_t *bits, int64_t T, int Hkv, const uint16_t *kmin,
                          const uint16_t *krange, uint8_t *codes, uint16_t *meta);
void kvq_oracle_decode_attn_kch(const uint16_t *q, const uint8_t *bits, const uint8_t *codes, const uint16_t *meta,
                                const uint16_t *kmin, const uint16_t *krange, int64_t len, int Hq, int Hkv, double *out, double *lse);
void kvq_oracle_rule_policy(const float *feats, int64_t n, const float *w, float bias, const float *thr, uint8_t *bits, double *score);
int kvq_oracle_accounting(const uint8_t *bits, int64_t n, int Hkv, int layers, double *expected_bits, double *effective_bits,
                          int64_t *payload_bytes);

static uint32_t state = 12345u;
static float frand(void)
{
    state = state * 1664525u + 1013904223u;
    return ((float)(state >> 8) / 8388608.0f) - 1.0f;            /* [-1, 1) */
}

int main(void)
{
    enum { T = 37, HKV = 3, HQ = 6, B = 2, VOCAB = 301, N = 5, LD = 40 };
    static const uint8_t widths[4] = {2, 4, 8, 16};
    /* exact-size heap buffers: an access one element past any of them is caught */
    uint16_t *k = malloc(sizeof(uint16_t) * B * T * HKV * 64), *v = malloc(sizeof(uint16_t) * B * T * HKV * 64);
    uint8_t *bits = malloc(B * T), *codes = malloc((size_t)B * T * HKV * 2 * 128);
    uint16_t *meta = malloc(sizeof(uint16_t) * B * T * HKV * 2 * 2), *q = malloc(sizeof(uint16_t) * B * HQ * 64);
    for (int i = 0; i < B * T * HKV * 64; ++i) { k[i] = kvq_oracle_f32_to_f16(3.0f * frand()); v[i] = kvq_oracle_f32_to_f16(frand()); }
    for (int i = 0; i < B * HQ * 64; ++i) q[i] = kvq_oracle_f32_to_f16(frand());
    for (int i = 0; i < B * T; ++i) bits[i] = widths[(state = state * 1664525u + 1013904223u) >> 30];
    for (int b = 0; b < B; ++b) {
        int rc = (b == 0 ? kvq_oracle_append : kvq_oracle_append_parallel)(k + (size_t)b * T * HKV * 64, v + (size_t)b * T * HKV * 64,
                     bits + b * T, T, HKV, codes + (size_t)b * T * HKV * 2 * 128, meta + (size_t)b * T * HKV * 2 * 2);
        if (rc != 0) return 2;
    }
    double deq[64];
    kvq_oracle_dequantize_vec(codes, meta[0], meta[1], bits[0], deq);
    double *out = malloc(sizeof(double) * B * HQ * 64), *lse = malloc(sizeof(double) * B * HQ), *p2 = malloc(sizeof(double) * B * HQ);
    double *probs = malloc(sizeof(double) * HQ * LD);
    kvq_oracle_decode_attn(q, bits, codes, meta, T, HQ, HKV, out, lse, probs, LD);
    const int32_t lens[B] = {T, T - 9};
    if (kvq_oracle_decode_attn_batch(q, bits, codes, meta, lens, B, T, HQ, HKV, out, lse, p2) <= 0) return 3;
    float *logits = malloc(sizeof(float) * N * VOCAB), feats[N * 4];
    int32_t ids[N], attn_len[N];
    int64_t *counts = calloc(VOCAB, sizeof(int64_t)), totals[2] = {0, 0};
    double *ap = malloc(sizeof(double) * N * HQ * LD);
    for (int i = 0; i < N * VOCAB; ++i) logits[i] = 2.0f * frand();
    for (int i = 0; i < N; ++i) { ids[i] = (i * 97) % VOCAB; attn_len[i] = LD - i; }
    ids[3] = ids[1];
    for (int i = 0; i < N * HQ * LD; ++i) ap[i] = 1.0 / LD;
    kvq_oracle_features(logits, N, VOCAB, ids, counts, 0, 0, ap, attn_len, HQ, LD, feats);
    kvq_oracle_counts_update(ids, N, counts, totals);
    if (totals[0] != N || totals[1] != N - 1) return 4;
    const int32_t dims[4] = {4, 7, 5, 4};
    float *W0 = malloc(sizeof(float) * 7 * 4), *W1 = malloc(sizeof(float) * 5 * 7), *W2 = malloc(sizeof(float) * 4 * 5);
    float b0[7], b1[5], b2[4];
    for (int i = 0; i < 28; ++i) W0[i] = frand();
    for (int i = 0; i < 35; ++i) W1[i] = frand();
    for (int i = 0; i < 20; ++i) W2[i] = frand();
    for (int i = 0; i < 7; ++i) b0[i] = frand();
    for (int i = 0; i < 5; ++i) b1[i] = frand();
    for (int i = 0; i < 4; ++i) b2[i] = frand();
    const float *Ws[3] = {W0, W1, W2}, *bs[3] = {b0, b1, b2};
    uint8_t dec[N];
    double lg[N * 4];
    kvq_oracle_controller(feats, N, 3, dims, Ws, bs, dec, lg);
    double eb, ef;
    int64_t nb;
    if (kvq_oracle_accounting(bits, B * T, HKV, 2, &eb, &ef, &nb) != 0) return 5;
    uint16_t *kmin = malloc(sizeof(uint16_t) * HKV * 64), *krange = malloc(sizeof(uint16_t) * HKV * 64);
    for (int i = 0; i < HKV * 64; ++i) { kmin[i] = kvq_oracle_f32_to_f16(-9.0f); krange[i] = kvq_oracle_f32_to_f16(18.0f); }
    if (kvq_oracle_append_kch(k, v, bits, T, HKV, kmin, krange, codes, meta) != 0) return 6;
    kvq_oracle_decode_attn_kch(q, bits, codes, meta, kmin, krange, T, HQ, HKV, out, lse);
    const float rw[4] = {0.1f, 0.07f, 50.0f, -1.0f}, rthr[3] = {0.1f, 0.4f, 0.9f};
    double rscore[N];
    kvq_oracle_rule_policy(feats, N, rw, 0.0f, rthr, dec, rscore);
    printf("ok %.3f %.3f %lld %d\n", eb, ef, (long long)nb, (int)dec[0]);
    free(kmin); free(krange);
    free(k); free(v); free(bits); free(codes); free(meta); free(q); free(out); free(lse); free(p2); free(probs);
    free(logits); free(counts); free(ap); free(W0); free(W1); free(W2);
    return 0;
}

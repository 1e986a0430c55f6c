/*
 * kvq.h -- C ABI of the MI355X (gfx950) library for adaptive mixed-precision KV-cache decoding.
 *
 * The four hot-path calls follow the four stages of the paper's pipeline (Sec. 3.4 "Framework
 * Overview"): token-level saliency features (Sec. 3.5), the controller that turns them into a
 * bit width per token (Sec. 3.6), quantize-and-append of the token's K/V at that width
 * (Sec. 3.7; Concat update of Sec. 3.2), and single-query decode attention over the resulting
 * heterogeneous-precision cache (Sec. 3.2, a = Softmax(q K^T / sqrt(d_k)) V).
 *
 * Conventions shared by every call
 *   - Return value: one of the KVQ_* status codes.  Nothing throws or aborts across this boundary;
 *     kvq_last_error() returns a thread-local description of the last failure on this thread.
 *   - Arguments are checked on the host before anything is launched: a call that returns an error
 *     has launched nothing and changed no state.
 *   - Pointers marked "device" are device memory owned by the caller and must stay valid until the
 *     work enqueued by the call has run.  Pointers marked "host" are read before the call returns.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the default stream).
 *     No call synchronizes unless its comment says so, and none of the four hot-path calls
 *     allocates or frees device memory.
 *   - Conditions that only the device can see (a page pool that runs dry, a sequence that would
 *     outgrow max_context, a bit width that is not 2/4/8/16) never fault: the offending tokens are
 *     dropped or stored as FP16, a sticky flag is raised in the cache, and kvq_cache_status()
 *     reports it.
 *   - Inputs must be finite.  NaN/Inf inputs give unspecified values, never a fault.
 *   - head_dim is 64.  fp16 means IEEE binary16; "bits" are always 2, 4, 8 or 16 (16 = FP16 storage).
 */
#ifndef KVQ_H
#define KVQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KVQ_HEAD_DIM 64
#define KVQ_EXPORT_REC 128   /* bytes per packed vector in the canonical export */

typedef enum {
    KVQ_OK = 0,
    KVQ_ERR_INVALID_ARG = 1,   /* null pointer, bad shape, bad layer index, ... */
    KVQ_ERR_CAPACITY = 2,      /* request cannot fit the cache as configured */
    KVQ_ERR_UNSUPPORTED = 3,   /* head_dim != 64, MLP wider than supported, ... */
    KVQ_ERR_DEVICE = 4,        /* a HIP call failed */
    KVQ_ERR_OOM = 5            /* arena too small / allocation failed */
} kvq_status;

/* sticky device-side flags reported by kvq_cache_status() */
#define KVQ_FLAG_POOL_EXHAUSTED 1u   /* a class page pool ran dry; tokens went to a sink page */
#define KVQ_FLAG_CONTEXT_FULL   2u   /* an append would exceed max_context; that sequence was skipped */
#define KVQ_FLAG_BAD_BITS       4u   /* a bit width other than 2/4/8/16 was seen; stored as FP16 */

typedef struct kvq_cache kvq_cache;   /* opaque */

typedef struct {
    int32_t n_layers;
    int32_t max_seqs;        /* sequence slots 0 .. max_seqs-1 */
    int32_t n_q_heads;       /* Hq, a multiple of n_kv_heads */
    int32_t n_kv_heads;      /* Hkv; query head h reads kv-head h / (Hq/Hkv) */
    int32_t head_dim;        /* must be 64 */
    int32_t page_tokens;     /* tokens per page, a power of two >= 256; 0 selects 256 */
    int64_t max_context;     /* largest number of tokens one sequence may hold, 1 .. 2^26 */
    int64_t pool_pages[4];   /* pages available to the 2/4/8/16-bit classes; 0 = enough for every
                                sequence to put max_context tokens into that class */
    void *arena;             /* device memory for the whole cache, 256-byte aligned, or NULL to let
                                kvq_cache_create allocate it with hipMalloc */
    size_t arena_bytes;      /* size of `arena` (ignored when arena is NULL) */
} kvq_cache_desc;

/* Controller MLP (Sec. 3.6): n_linear linear layers dims[0] -> dims[1] -> ... -> dims[n_linear],
 * ReLU after every layer but the last.  dims[0] = 4 (the feature vector), dims[n_linear] = 4 (one
 * logit per precision class), hidden widths at most 256.  W[l] is row-major [dims[l+1]][dims[l]],
 * b[l] is [dims[l+1]]; both fp32, device. */
typedef struct {
    int32_t n_linear;        /* 2 or 3 */
    int32_t dims[5];
    const float *W[4];
    const float *b[4];
} kvq_mlp;

const char *kvq_version(void);
const char *kvq_last_error(void);

/* ---------------------------------------------------------------------------------------------
 * Cache object: the heterogeneous-precision KV cache of Sec. 3.4 / 3.7.  Tokens of one sequence
 * are kept in four precision buckets (2/4/8-bit codes with an fp16 scale and fp16 minimum per
 * 64-vector, or raw fp16); attention is a sum over tokens, so bucket order does not change it.
 * The device layout is private; kvq_cache_export() gives a layout-independent dump.
 * ------------------------------------------------------------------------------------------- */

/* Bytes of device memory kvq_cache_create needs for `desc` (0 on an invalid descriptor). */
size_t kvq_cache_arena_bytes(const kvq_cache_desc *desc);

/* Creates a cache.  Synchronizes the device once (it clears the arena).  `*out` is owned by the
 * caller until kvq_cache_destroy.  With desc->arena == NULL the arena is hipMalloc'd and freed on
 * destroy; otherwise the caller keeps ownership of the arena. */
int kvq_cache_create(const kvq_cache_desc *desc, kvq_cache **out);
int kvq_cache_destroy(kvq_cache *cache);

/* Empties every sequence and returns all pages to the pools; clears the sticky flags. */
int kvq_cache_reset(kvq_cache *cache, void *stream);

/* Empties the listed sequences and returns their pages.  seq_ids: device int32[n_seq], distinct. */
int kvq_cache_free_seqs(kvq_cache *cache, const int32_t *seq_ids, int32_t n_seq, void *stream);

/* Launch-shape hint (never changes a result).  The library shapes an attention launch (waves per head, splits) for the
 * longest sequence the cache may hold.  It cannot see the lengths without a device round trip, so it keeps a host-side
 * high-water mark: every append raises it by the tokens appended, kvq_cache_reset clears it, kvq_cache_free_seqs does
 * not lower it (the host does not know which sequences remain).  A server that recycles sequences tells the library
 * the longest live length here; the mark continues to grow from that value. */
int kvq_cache_set_length_hint(kvq_cache *cache, int64_t longest_live_length);

/* Synchronizes `stream` and reports the sticky flags (KVQ_FLAG_*) and, if free_pages != NULL, the
 * number of free pages left in each class (host int64[4]). */
int kvq_cache_status(kvq_cache *cache, uint32_t *flags, int64_t *free_pages, void *stream);

/* Synchronizes `stream` and copies per-sequence token counts to the host:
 * counts is host int32[max_seqs][5] = tokens in the 2/4/8/16-bit classes and the total length. */
int kvq_cache_counts(kvq_cache *cache, int32_t *counts, void *stream);

/* Synchronizes `stream` and reports what the cache holds (Sec. 3.3: the expected bit-width E[b] = sum_x p(x) f(x),
 * here the mean width over all cached tokens), all sequences together:
 *   tokens[4]            cached tokens in the 2/4/8/16-bit classes
 *   expected_bits        E[b]; 0 for an empty cache
 *   effective_bits       bits stored per cached element with the fp16 (scale, minimum) pairs counted: 2.5/4.5/8.5/16 per class
 *   payload_bytes        sum over tokens of {40,72,136,256}[class] * n_kv_heads * n_layers
 *   pages_in_use[4], page_bytes_in_use   pages handed out per class and the arena bytes they occupy (all layers) */
typedef struct kvq_cache_usage {
    int64_t tokens[4];
    double expected_bits;
    double effective_bits;
    int64_t payload_bytes;
    int64_t pages_in_use[4];
    int64_t page_bytes_in_use;
} kvq_cache_usage;
int kvq_cache_usage_of(kvq_cache *cache, kvq_cache_usage *usage, void *stream);

/* Canonical dump of one (layer, sequence), in TOKEN order, for parity checks and save/restore.
 *   bits_out  device uint8 [max_tokens]                      the width b of each token
 *   codes_out device uint8 [max_tokens][Hkv][2][128]         index 0 = K, 1 = V.  b in {2,4,8}: element i
 *                                                            occupies bits [i*b, i*b+b) of the byte
 *                                                            stream (little-endian bit order), rest 0;
 *                                                            b = 16: the 64 fp16 patterns, little-endian
 *   meta_out  device uint16[max_tokens][Hkv][2][2]           fp16 bit patterns (scale, minimum); 0 for b = 16
 * Only the first len(seq) tokens are written; max_tokens bounds the buffers (tokens beyond it are
 * not written).  Read the length with kvq_cache_counts. */
int kvq_cache_export(const kvq_cache *cache, int32_t layer, int32_t seq, uint8_t *bits_out, uint8_t *codes_out,
                     uint16_t *meta_out, int64_t max_tokens, void *stream);

/* Variant Q_b for keys (the paper leaves Q_b open in Sec. 3.7 and cites per-channel key quantizers as related
 * work): static per-channel quantization.  kmin and krange are device fp16 [n_layers][n_kv_heads][64]: per channel a
 * minimum m_c and a range r_c from an offline calibration.  A key stored at b bits then uses
 *   step_c = fp16(fp32(r_c) / (2^b - 1)),  code_c = clamp(rint((x_c - m_c) / fp32(step_c)), 0, 2^b - 1)  (IEEE binary32,
 *   code 0 where the step is 0),  k^_c = m_c + code_c * step_c,
 * values outside [m_c, m_c + r_c] clamp, and no per-token scale or minimum is stored for K (the export shows 0 for
 * them).  Values, the 16-bit class, and every entry point's signature are unchanged; the attention kernel folds the
 * steps into q once per class instead of reading a scale and a minimum per token.  Choose the quantizer while the
 * cache is empty (after kvq_cache_create or kvq_cache_reset: a cache emptied by kvq_cache_free_seqs does not count,
 * call kvq_cache_reset first); kmin == krange == NULL returns to the per-token quantizer.  Appends with
 * many tokens per call take the wave-per-vector kernel in this mode. */
int kvq_cache_set_k_channel_quant(kvq_cache *cache, const void *kmin, const void *krange, void *stream);

/* Inverse of kvq_cache_export: appends n_tokens tokens to sequence `seq` from a canonical dump (the arrays
 * kvq_cache_export wrote, device memory), without re-quantizing anything, so that a cache can be saved, restored,
 * or moved to another cache or device.  As with kvq_append, the call with layer == 0 does the bucket bookkeeping
 * from `bits` (device uint8 [n_tokens]); calls with layer >= 1 place the same tokens' codes and must follow it
 * with the same seq and n_tokens (they ignore `bits`).  A restored sequence answers kvq_decode_attn bit for bit
 * like the original. */
int kvq_cache_import(kvq_cache *cache, int32_t layer, int32_t seq, const uint8_t *bits, const uint8_t *codes,
                     const uint16_t *meta, int64_t n_tokens, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Stage 1 -- token-level saliency features s_t = [H_t, R_t, V_t, C_t]  (Sec. 3.5)
 *   H_t = -sum_v p(v) ln p(v), p = Softmax(logits row)          (entropy equation)
 *   R_t = -ln((c(x_t)+1) / (N + |V_obs| + 1))                   (rarity equation)
 *   V_t = mean over query heads of the population variance of the token's final-layer attention
 *         probability row                                        (attention-variance equation)
 *   C_t = max_v p(v)                                            (the "confidence term"; the paper
 *         names it without a formula: this is the reading taken here)
 *
 *   logits     device fp32 [n][vocab], row-major
 *   token_ids  device int32 [n], each in [0, vocab)
 *   counts     device int64 [vocab]   running counts c(.)
 *   totals     device int64 [2]       {N, |V_obs|}
 *   update_counts  0: tables are read only.  1: after all n rows have been scored against the tables
 *              as passed in, every token is counted (c[id] += 1, N += n, |V_obs| += number of distinct
 *              ids whose count was 0); the result does not depend on thread order.
 *   Attention variance takes exactly one of two sources:
 *     attn_probs device fp32 [n][n_q_heads][ld]: the probability rows themselves, of which the first
 *                attn_len[t] entries are used, or
 *     sum_p2     device fp32 [n][n_q_heads]: sum_j p_j^2 of each row as emitted by kvq_decode_attn
 *                (then Var = sum_p2/l - 1/l^2, because the row sums to one).
 *   attn_len   device int32 [n]; a value <= 0 means "no attention row yet" (a sequence's first token): V = 0
 *   workspace  device, at least kvq_features_workspace(n, vocab) bytes, 256-byte aligned
 *   feats_out  device fp32 [n][4] = H, R, V, C
 * ------------------------------------------------------------------------------------------- */
size_t kvq_features_workspace(int64_t n, int64_t vocab);
int kvq_features(const float *logits, int64_t n, int64_t vocab, const int32_t *token_ids,
                 int64_t *counts, int64_t *totals, int32_t update_counts,
                 const float *attn_probs, const float *sum_p2, const int32_t *attn_len,
                 int32_t n_q_heads, int64_t ld, float *feats_out,
                 void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Stage 2 -- controller (Sec. 3.6): h1 = ReLU(W1 s + b1), h2 = ReLU(W2 h1 + b2), o = W3 h2 + b3,
 * class = argmax_k o_k (the softmax of the paper is monotone and is skipped; the first maximum wins
 * a tie), bits = {2,4,8,16}[class] (label mapping of Algorithm 1).
 *   feats       device fp32 [n][4]
 *   mlp         host struct; its W/b pointers are device memory
 *   bits_out    device uint8 [n]
 *   logits_out  device fp32 [n][4] or NULL
 * ------------------------------------------------------------------------------------------- */
int kvq_controller(const float *feats, int64_t n, const kvq_mlp *mlp, uint8_t *bits_out,
                   float *logits_out, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Comparison policy: a stand-in for the "rule-based dynamic KV policy" baseline of Sec. 4.  The paper only says that
 * baseline uses hand-crafted heuristics and never states them, so this rule is NOT the paper's: an importance score
 * linear in the features, cut by three ascending thresholds,
 *   score = bias + sum_i w[i] * s[i],   class = #{k : score > thr[k]},   bits = {2,4,8,16}[class]
 * (fp32, the products added in feature order).  Same role and output as kvq_controller.
 *   feats      device fp32 [n][4];  rule  host struct (thr ascending);  bits_out  device uint8 [n]
 *   score_out  device fp32 [n] or NULL
 * ------------------------------------------------------------------------------------------- */
typedef struct kvq_rule {
    float w[4];
    float bias;
    float thr[3];
} kvq_rule;
int kvq_rule_policy(const float *feats, int64_t n, const kvq_rule *rule, uint8_t *bits_out, float *score_out, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Stages 1 + 2 in one call, for the decode step (Sec. 3.4: saliency profiling, then the controller's decision,
 * then the token's place in the mixed-precision cache): the features of kvq_features in its sum_p2 form, the
 * decision of kvq_controller on them, the count update, and -- if `cache` is given -- the bucket bookkeeping that
 * kvq_append(layer 0, T = 1) would do with those decisions.  Results are bit-identical to the separate calls.
 * Two launches instead of five: the pass over the logits, spread over rows x slices workgroups (it also copies each
 * row's table entries, so that every read of the count table lies in the first launch and every update in the
 * second), then one workgroup per row for the rest.
 *   logits .. attn_len, n_q_heads   as in kvq_features (sum_p2 is required, there is no attn_probs form)
 *   mlp, bits_out, logits_out       as in kvq_controller
 *   cache      NULL, or the cache whose sequences receive one token each: row i belongs to sequence seq_ids[i]
 *              (i if seq_ids is NULL); the following kvq_append / kvq_append_decode_attn calls of this step then
 *              pass bits = NULL on layer 0, which means "bookkeeping already done"
 *   workspace  device, at least kvq_features_workspace(n, vocab) bytes, 16-byte aligned (slice results and the
 *              rows' table entries between the two launches)
 * ------------------------------------------------------------------------------------------- */
int kvq_features_controller(const float *logits, int64_t n, int64_t vocab, const int32_t *token_ids,
                            int64_t *counts, int64_t *totals, int32_t update_counts, const float *sum_p2,
                            const int32_t *attn_len, int32_t n_q_heads, const kvq_mlp *mlp, kvq_cache *cache,
                            const int32_t *seq_ids, float *feats_out, uint8_t *bits_out, float *logits_out,
                            void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * The same two calls for logits that the model emits in a 16-bit type (Sec. 3.5 defines the features on the
 * distribution p_t; a narrow logit is widened exactly, so the result is that of kvq_features / kvq_features_controller
 * on the widened row, and a row costs half the bytes).
 *   logits        device [n][vocab] of the type named by logits_dtype, aligned to its element size
 *   logits_dtype  KVQ_DTYPE_F32 (then identical to the untyped calls), KVQ_DTYPE_F16 or KVQ_DTYPE_BF16
 * Every other argument, the workspace and the error behaviour are those of the untyped call.
 * ------------------------------------------------------------------------------------------- */
enum { KVQ_DTYPE_F32 = 0, KVQ_DTYPE_F16 = 1, KVQ_DTYPE_BF16 = 2 };
int kvq_features_typed(const void *logits, int32_t logits_dtype, int64_t n, int64_t vocab, const int32_t *token_ids,
                       int64_t *counts, int64_t *totals, int32_t update_counts,
                       const float *attn_probs, const float *sum_p2, const int32_t *attn_len,
                       int32_t n_q_heads, int64_t ld, float *feats_out,
                       void *workspace, size_t workspace_bytes, void *stream);
int kvq_features_controller_typed(const void *logits, int32_t logits_dtype, int64_t n, int64_t vocab,
                                  const int32_t *token_ids, int64_t *counts, int64_t *totals, int32_t update_counts,
                                  const float *sum_p2, const int32_t *attn_len, int32_t n_q_heads, const kvq_mlp *mlp,
                                  kvq_cache *cache, const int32_t *seq_ids, float *feats_out, uint8_t *bits_out,
                                  float *logits_out, void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Stage 3 -- quantize and append (Sec. 3.7: k^ = Q_b(k), v^ = Q_b(v); Sec. 3.2: K <- Concat(K, k)).
 * Q_b for b in {2,4,8}, per (token, kv-head) vector x of 64 fp16 values, every step in IEEE binary32
 * round-to-nearest-even:  levels = 2^b - 1;  scale = fp16((max x - min x) / levels);  the stored
 * minimum is min x (a zero of either sign is stored as +0);  code_i = clamp(rint((x_i - min x) /
 * fp32(scale)), 0, levels), all codes 0 when scale == 0;  x^_i = min + code_i * scale.  b = 16 stores
 * x itself.  K and V are quantized independently with the same b; one b per token serves every
 * layer and kv-head.
 *
 *   layer   0 .. n_layers-1, or -1 for all layers in one call
 *   k, v    device fp16 [n_seq][T][Hkv][64]   (layer == -1: [n_layers][n_seq][T][Hkv][64])
 *   bits    device uint8 [n_seq][T]; read only by the call that does the bookkeeping (below)
 *   seq_ids device int32 [n_seq], distinct, or NULL for 0 .. n_seq-1
 * Bookkeeping rule: the bucket slots, page allocation and bit-width log of the T new tokens are
 * shared by all layers and are advanced by the call with layer == 0 (or layer == -1).  Calls with
 * layer >= 1 write the K/V of the tokens appended by the latest layer-0 call on those sequences and
 * must use the same n_seq, T and seq_ids; they ignore `bits`.  A layer-0 (or -1) call with bits == NULL
 * does no bookkeeping either: it follows a kvq_features_controller call that advanced the cache (T = 1).
 * ------------------------------------------------------------------------------------------- */
int kvq_append(kvq_cache *cache, int32_t layer, const void *k, const void *v, const uint8_t *bits,
               const int32_t *seq_ids, int32_t n_seq, int32_t T, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Stage 4 -- decode attention (Sec. 3.2): for every listed sequence and query head h,
 *   s_j = (q_h . k^_j) / sqrt(64),  p = Softmax(s) over all cached tokens j (the newest included, in
 *   its stored precision),  out_h = sum_j p_j v^_j,  with k^, v^ of kv-head h / (Hq/Hkv) dequantized
 *   in registers.  fp32 accumulation.
 *   q           device fp16 [n_seq][Hq][64]
 *   seq_ids     device int32 [n_seq] or NULL for 0 .. n_seq-1
 *   out         device fp32 [n_seq][Hq][64]; zeros for an empty sequence
 *   lse_out     device fp32 [n_seq][Hq] or NULL: ln sum_j exp(s_j)  (-inf for an empty sequence)
 *   sum_p2_out  device fp32 [n_seq][Hq] or NULL: sum_j p_j^2, the input of the attention-variance feature
 *   workspace   device, at least kvq_decode_attn_workspace(cache, n_seq) bytes, 256-byte aligned
 * ------------------------------------------------------------------------------------------- */
size_t kvq_decode_attn_workspace(const kvq_cache *cache, int32_t n_seq);
int kvq_decode_attn(const kvq_cache *cache, int32_t layer, const void *q, const int32_t *seq_ids,
                    int32_t n_seq, float *out, float *lse_out, float *sum_p2_out,
                    void *workspace, size_t workspace_bytes, void *stream);

/* The same call for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  It takes no workspace: the partial results of a
 * launch that splits sequences over workgroups go to a fixed array of kvq_decode_attn_static_capacity() bytes (8 MiB)
 * inside the library's device image, one copy per GPU, held until the process ends.  The call allocates and frees
 * nothing and only enqueues kernels.  Results equal kvq_decode_attn's.  A launch whose partial results would not fit
 * (n_seq x n_q_heads x splits x 272 bytes, with the split count the library picks for the cache's lengths) returns
 * KVQ_ERR_CAPACITY and launches nothing.  All calls on one GPU share that GPU's array: calls that overlap in time on
 * one GPU (different streams) race; calls on one stream are ordered and safe.  Nothing in the array has to be
 * cleared between calls (every partial result a launch reads, it has written itself). */
size_t kvq_decode_attn_static_capacity(void);
int kvq_decode_attn_static(const kvq_cache *cache, int32_t layer, const void *q, const int32_t *seq_ids,
                           int32_t n_seq, float *out, float *lse_out, float *sum_p2_out, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Stages 3 + 4 in one launch, for the decode step (one new token per sequence): the Concat update of
 * Sec. 3.2 followed by the attention of the same section, exactly as kvq_append(T = 1) followed by
 * kvq_decode_attn would compute them.  The new token is quantized in registers (Q_b of Sec. 3.7), takes
 * part in the softmax in its quantized form, and is stored into the cache for later steps; the older
 * tokens are streamed from the cache.  Saves one kernel launch per layer.
 *   k, v    device fp16 [n_seq][1][Hkv][64] (the new token)
 *   bits    device uint8 [n_seq]; read only when layer == 0, which also does the bookkeeping (see
 *           kvq_append); layers >= 1 must follow a layer-0 call with the same n_seq and seq_ids
 *   q, seq_ids, out, lse_out, sum_p2_out, workspace: as for kvq_decode_attn
 * ------------------------------------------------------------------------------------------- */
int kvq_append_decode_attn(kvq_cache *cache, int32_t layer, const void *k, const void *v, const uint8_t *bits,
                           const void *q, const int32_t *seq_ids, int32_t n_seq, float *out, float *lse_out,
                           float *sum_p2_out, void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Training step of the controller (Sec. 3.8 and the inner loop of Algorithm 1) on one mini-batch:
 *   o = f_theta(s), p = Softmax(o), y = {2,4,8,16} -> {0,1,2,3} of the label,
 *   L_ce = mean_i -log p_{i,y_i},  L_lat = mean_i sum_k p_ik c_k,  L_qual = 1 - mean_i sum_k p_ik q_k,
 *   L = alpha L_ce + beta L_lat + gamma L_qual,  theta <- Adam(theta, dL/dtheta).
 * The paper gives no values for c, q, alpha, beta, gamma or Adam's constants: all are arguments.  The derivative of
 * ReLU at 0 is 0.  Adam: m <- b1 m + (1-b1) g, v <- b2 v + (1-b2) g^2,
 * theta <- theta - lr (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps), no weight decay.  fp32 throughout.
 *   feats       device fp32 [n][4];  label_bits  device uint8 [n], values 2/4/8/16 (anything else counts as 16)
 *   mlp         host struct; its device weights and biases are UPDATED IN PLACE (hidden widths up to 128)
 *   adam_m/v    host structs of the same shape whose W/b pointers are the device first/second moment buffers,
 *               updated in place (zero them before step 1)
 *   step        t, counted from 1
 *   losses_out  device fp32 [4] = L, L_ce, L_lat, L_qual of the mini-batch before the update, or NULL
 *   grads_out   device fp32 [kvq_controller_param_count] in the order W1, b1, W2, b2, (W3, b3), or NULL
 *   workspace   device, at least kvq_controller_train_workspace(mlp, n) bytes, 16-byte aligned
 * Two launches, no allocation, no synchronization; the result does not depend on scheduling (no atomics).
 * ------------------------------------------------------------------------------------------- */
typedef struct kvq_train_hparams {
    float alpha, beta, gamma;       /* weights of the three loss terms */
    float c[4];                     /* latency cost per class */
    float q[4];                     /* quality score per class */
    float lr, beta1, beta2, eps;    /* Adam */
} kvq_train_hparams;
int64_t kvq_controller_param_count(const kvq_mlp *mlp);
size_t kvq_controller_train_workspace(const kvq_mlp *mlp, int64_t n);
int kvq_controller_train_step(const float *feats, const uint8_t *label_bits, int64_t n, const kvq_mlp *mlp,
                              const kvq_mlp *adam_m, const kvq_mlp *adam_v, const kvq_train_hparams *hp,
                              int64_t step, float *losses_out, float *grads_out, void *workspace,
                              size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Launch-shape overrides for tests and tuning runs (never needed in normal use; no part of the method).
 * The library keeps one process-wide table of small integers; the hot-path calls read that table and
 * never the environment.  The table starts from its defaults, overridden by the KVQ_* environment
 * variables as they stand when it is first needed; kvq_tuning_set changes an entry afterwards.
 *   name   host string: attn_splits (0 = automatic, 1..64), attn_waves (0, 1, 2, 3, 4, 8),
 *          attn_longest_first (-1 = automatic, 0, 1), attn_by_class, append_bulk_min_T,
 *          append_stream_min, append_block_min_T, controller_no_mfma, controller_waves,
 *          controller_wg_per_cu, train_no_mfma
 * KVQ_ERR_INVALID_ARG for an unknown name or a value outside the entry's range (nothing changes).
 * Not synchronised with calls running on other threads.
 * ------------------------------------------------------------------------------------------- */
int kvq_tuning_set(const char *name, int32_t value);
int kvq_tuning_get(const char *name, int32_t *value);

#ifdef __cplusplus
}
#endif
#endif /* KVQ_H */

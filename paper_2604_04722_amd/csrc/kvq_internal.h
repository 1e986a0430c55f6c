// Internal declarations shared by the HIP translation units of libkvq (not installed, not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>
#include <stddef.h>

#include "kvq.h"
#include "kvq_tuning.h"

namespace kvq {

// ----------------------------------------------------------------------------------------------
// Device layout of the precision-bucketed cache.
//
// A token's bit width (class 0..3 = 2/4/8/16 bit) is one decision shared by every layer and
// kv-head (paper Sec. 3.6: one b per token), so the bucket bookkeeping is per (sequence, class):
//   slot  = rank of the token among the sequence's tokens of its class,
//   page  = page_table[seq][class][slot / page_tokens]      (allocated from the class's pool)
//   block = 64 consecutive slots = one wavefront's worth of tokens (lane = token).
// One page id names memory for every layer and kv-head:
//   addr = pool[class] + layer*layer_stride[class] + ((page*Hkv + kvh)*blocks_per_page + blk)*block_bytes[class]
// Inside a block (NCH = 16-byte chunks per vector = 1/2/4/8):
//   [ meta: 64 tokens x 8 B  (half K scale, half K min, half V scale, half V min) ]   (absent for FP16)
//   [ K codes: NCH chunks x 64 tokens x 16 B ]   chunk-major: a wave's 16-B-per-lane load is 1 KiB contiguous
//   [ V codes: NCH chunks x 64 tokens x 16 B ]
// Inside a token's vector, 32-bit word w holds elements [w*per, (w+1)*per), per = 32/b.  The pair of
// elements (2m, 2m+1) sits at the same offset of the low and the high 16-bit half of its word:
// element w*per + r goes to bits  b*(r/2) + 16*(r%2).  One shift + one and-or then yields the pair as
// two fp16 values, ready for a packed dot with the matching pair of q (or a mixed-precision FMA).
// ----------------------------------------------------------------------------------------------

constexpr int kD = 64;                 // head_dim
constexpr int kBlockTokens = 64;       // one block = one wavefront of tokens
constexpr int kClasses = 4;

__host__ __device__ constexpr int class_bits(int c) { return c == 0 ? 2 : c == 1 ? 4 : c == 2 ? 8 : 16; }
__host__ __device__ constexpr int class_chunks(int c) { return c == 0 ? 1 : c == 1 ? 2 : c == 2 ? 4 : 8; }
__host__ __device__ constexpr int class_meta_bytes(int c) { return c == 3 ? 0 : kBlockTokens * 8; }
__host__ __device__ constexpr int class_block_bytes(int c)
{
    return class_meta_bytes(c) + 2 * class_chunks(c) * kBlockTokens * 16;
}
// blocks that one loop iteration of the attention kernel treats together (all inside one page)
__host__ __device__ constexpr int class_unit_blocks(int c) { return c == 0 ? 2 : 1; }

struct CacheView {
    uint8_t *pool[kClasses];
    size_t layer_stride[kClasses];
    int32_t *page_table;               // [max_seqs][4][max_pages_per_seq]
    int32_t *counts;                   // [max_seqs][5]: tokens per class, total length
    int32_t *last_T;                   // [max_seqs]: tokens accepted by the latest bookkeeping append
    int32_t *last_rec;                 // [max_seqs][4]: {last_T, bits, slot, page} of the newest token, one 16-byte read
                                       // for the single-token writers instead of four dependent ones
    uint8_t *bits_log;                 // [max_seqs][max_context]
    int32_t *slot_log;                 // [max_seqs][max_context]
    // slot -> position, written by the multi-token bookkeeping kernel (the prefill writer works a block of slots at a
    // time and asks which token sits in each).  Two classes share an array of max_context entries: one fills it from
    // the front, the other from the back; their counts never add up to more than the length.  See pos_log_index.
    int32_t *pos_log;                  // [max_seqs][2][max_context]
    int32_t *last_start;               // [max_seqs][4]: the class counts before the latest multi-token bookkeeping append
    // static per-channel key quantizer (a variant Q_b, off unless k_channel != 0): per (layer, kv-head, channel) the
    // minimum, and per quantized class the step fp16(range / levels)
    __half *kch_min;                   // [n_layers][Hkv][64]
    __half *kch_step;                  // [3][n_layers][Hkv][64]
    int32_t *free_stack[kClasses];     // [n_pages[c]] ids of free pages
    int32_t *free_top;                 // [4] number of free pages
    uint32_t *flags;                   // [1] sticky KVQ_FLAG_*
    int32_t n_pages[kClasses];         // usable pages; page id n_pages[c] is the sink page
    int32_t n_layers, max_seqs, Hq, Hkv;
    int32_t page_tokens, blocks_per_page, max_pages_per_seq;
    int32_t max_context;
    int32_t k_channel;                 // keys use the static per-channel variant
};

}  // namespace kvq

struct kvq_cache {
    kvq_cache_desc desc;
    kvq::CacheView view;
    void *arena;
    size_t arena_bytes;
    bool own_arena;
    int device;
    int64_t len_bound;                 // host-side upper bound of any sequence's length (split heuristic only): a high-water
                                       // mark that grows with every append and falls only by reset or the caller's hint
    bool touched;                      // something was appended or imported since create / reset
};

int kvq_append_bookkeeping(kvq_cache *cache, const uint8_t *bits, const int32_t *seq_ids, int n_seq, int T, void *stream);

namespace kvq {

void set_error(const char *fmt, ...);
int check_hip(hipError_t e, const char *what);

#define KVQ_HIP(call)                                              \
    do {                                                           \
        int _rc = ::kvq::check_hip((call), #call);                 \
        if (_rc != KVQ_OK) return _rc;                             \
    } while (0)

// Raises a kernel's dynamic-LDS limit when `bytes` needs it (above 48 KiB) and exceeds what this process has already
// set for that kernel (`*granted`, a static of the call site): the runtime call is not free on the host, and the
// per-step entry points would otherwise repeat it on every call.
inline int ensure_dynamic_lds(const void *kernel, size_t bytes, size_t *granted)
{
    if (bytes <= 48 * 1024 || bytes <= *granted) return KVQ_OK;
    const int rc = check_hip(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes),
                             "hipFuncSetAttribute(MaxDynamicSharedMemorySize)");
    if (rc == KVQ_OK) *granted = bytes;
    return rc;
}

// ---- small device helpers -------------------------------------------------------------------

__device__ __forceinline__ int bits_to_class(int b) { return b == 2 ? 0 : b == 4 ? 1 : b == 8 ? 2 : 3; }

__device__ __forceinline__ size_t block_offset(const CacheView &cv, int cls, int layer, int page, int kvh, int blk_in_page)
{
    return (size_t)layer * cv.layer_stride[cls] +
           (((size_t)page * cv.Hkv + kvh) * cv.blocks_per_page + blk_in_page) * (size_t)class_block_bytes(cls);
}

__device__ __forceinline__ size_t pos_log_index(const CacheView &cv, int seq, int cls, int slot)
{
    return ((size_t)seq * 2 + (cls >> 1)) * (size_t)cv.max_context + (size_t)((cls & 1) ? cv.max_context - 1 - slot : slot);
}

// Bucket bookkeeping of ONE new token of `seq` by a single thread: the same state changes as the bookkeeping
// kernel makes for T = 1 (slot = the class's count, a page popped from the class's free stack when the slot opens
// a page, bits and slot logged, counts advanced, flags raised on a full context, an empty pool or a bad width).
// `pre` holds the sequence's five counters and `pre_page` the page-table entry that each class's next slot falls
// into, both read earlier by the same thread (so that the reads overlap other work; the entry of a slot that opens a
// page is not looked at).
__device__ __forceinline__ void prefetch_next_pages(const CacheView &cv, int seq, const int (&pre)[5], int (&pre_page)[kClasses])
{
#pragma unroll
    for (int c = 0; c < kClasses; ++c) {
        const int idx = min(pre[c] / cv.page_tokens, cv.max_pages_per_seq - 1);
        pre_page[c] = cv.page_table[((size_t)seq * kClasses + c) * cv.max_pages_per_seq + idx];
    }
}

__device__ __forceinline__ void advance_one_token(const CacheView &cv, int seq, int b, const int (&pre)[5], const int (&pre_page)[kClasses])
{
    if (seq < 0 || seq >= cv.max_seqs) { atomicOr(cv.flags, KVQ_FLAG_CONTEXT_FULL); return; }
    int32_t *cnt = cv.counts + (size_t)seq * 5;
    const int len = pre[4];
    if ((int64_t)len + 1 > (int64_t)cv.max_context) {
        atomicOr(cv.flags, KVQ_FLAG_CONTEXT_FULL);
        cv.last_T[seq] = 0;
        cv.last_rec[(size_t)seq * 4] = 0;
        return;
    }
    if (b != 2 && b != 4 && b != 8 && b != 16) { atomicOr(cv.flags, KVQ_FLAG_BAD_BITS); b = 16; }
    const int c = bits_to_class(b);
    // (selected by arithmetic: a chain of conditionals over array elements becomes a select of their addresses, which
    // puts the arrays into scratch memory)
    const int m0 = -(int)(c == 0), m1 = -(int)(c == 1), m2 = -(int)(c == 2), m3 = -(int)(c == 3);
    const int slot = (pre[0] & m0) | (pre[1] & m1) | (pre[2] & m2) | (pre[3] & m3);
    int page_now = (pre_page[0] & m0) | (pre_page[1] & m1) | (pre_page[2] & m2) | (pre_page[3] & m3);
    if (slot % cv.page_tokens == 0) {
        const int idx = atomicSub(&cv.free_top[c], 1) - 1;
        if (idx < 0) {
            atomicAdd(&cv.free_top[c], 1);
            atomicOr(cv.flags, KVQ_FLAG_POOL_EXHAUSTED);
            page_now = cv.n_pages[c];                                  // sink page: in bounds, shared, garbage
        } else {
            page_now = cv.free_stack[c][idx];
        }
        cv.page_table[((size_t)seq * kClasses + c) * cv.max_pages_per_seq + slot / cv.page_tokens] = page_now;
    }
    const size_t pos = (size_t)seq * cv.max_context + len;
    cv.bits_log[pos] = (uint8_t)b;
    cv.slot_log[pos] = slot;
    cnt[c] = slot + 1;
    cnt[4] = len + 1;
    cv.last_T[seq] = 1;
    int32_t *rec = cv.last_rec + (size_t)seq * 4;
    rec[0] = 1; rec[1] = b; rec[2] = slot; rec[3] = page_now;
}

}  // namespace kvq

// Cache object, bucket bookkeeping, quantize-and-append (paper Sec. 3.7 + the Concat update of Sec. 3.2)
// and the canonical export.
#include "kvq_internal.h"

#include "kvq_quant.h"

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

namespace kvq {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int check_hip(hipError_t e, const char *what)
{
    if (e == hipSuccess) return KVQ_OK;
    set_error("HIP error %d (%s) in %s", (int)e, hipGetErrorString(e), what);
    return e == hipErrorOutOfMemory ? KVQ_ERR_OOM : KVQ_ERR_DEVICE;
}

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Everything the arena holds, in order.  Returns the total size; fills `v` when base != nullptr.
static size_t plan_arena(const kvq_cache_desc &d, CacheView *v, uint8_t *base)
{
    const int P = d.page_tokens ? d.page_tokens : 256;
    const int bpp = P / kBlockTokens;
    const int64_t mpps = (d.max_context + P - 1) / P;
    size_t off = 0;
    CacheView cv;
    memset(&cv, 0, sizeof(cv));
    cv.n_layers = d.n_layers;
    cv.max_seqs = d.max_seqs;
    cv.Hq = d.n_q_heads;
    cv.Hkv = d.n_kv_heads;
    cv.page_tokens = P;
    cv.blocks_per_page = bpp;
    cv.max_pages_per_seq = (int32_t)mpps;
    cv.max_context = (int32_t)d.max_context;
    for (int c = 0; c < kClasses; ++c) {
        int64_t np = d.pool_pages[c] > 0 ? d.pool_pages[c] : (int64_t)d.max_seqs * mpps;
        cv.n_pages[c] = (int32_t)np;
        const size_t page_bytes = (size_t)bpp * class_block_bytes(c);
        cv.layer_stride[c] = (size_t)(np + 1) * d.n_kv_heads * page_bytes;     // +1: the sink page
        cv.pool[c] = base + off;
        off = align256(off + cv.layer_stride[c] * d.n_layers);
    }
    cv.page_table = (int32_t *)(base + off);
    off = align256(off + sizeof(int32_t) * (size_t)d.max_seqs * kClasses * mpps);
    cv.counts = (int32_t *)(base + off);
    off = align256(off + sizeof(int32_t) * (size_t)d.max_seqs * 5);
    cv.last_T = (int32_t *)(base + off);
    off = align256(off + sizeof(int32_t) * (size_t)d.max_seqs);
    cv.last_rec = (int32_t *)(base + off);
    off = align256(off + sizeof(int32_t) * (size_t)d.max_seqs * 4);
    cv.bits_log = base + off;
    off = align256(off + (size_t)d.max_seqs * d.max_context);
    cv.slot_log = (int32_t *)(base + off);
    off = align256(off + sizeof(int32_t) * (size_t)d.max_seqs * d.max_context);
    cv.pos_log = (int32_t *)(base + off);
    off = align256(off + sizeof(int32_t) * (size_t)d.max_seqs * 2 * d.max_context);
    cv.last_start = (int32_t *)(base + off);
    off = align256(off + sizeof(int32_t) * (size_t)d.max_seqs * 4);
    for (int c = 0; c < kClasses; ++c) {
        cv.free_stack[c] = (int32_t *)(base + off);
        off = align256(off + sizeof(int32_t) * (size_t)cv.n_pages[c]);
    }
    cv.free_top = (int32_t *)(base + off);
    off = align256(off + sizeof(int32_t) * kClasses);
    cv.kch_min = (__half *)(base + off);
    off = align256(off + sizeof(__half) * (size_t)d.n_layers * d.n_kv_heads * kD);
    cv.kch_step = (__half *)(base + off);
    off = align256(off + sizeof(__half) * 3 * (size_t)d.n_layers * d.n_kv_heads * kD);
    cv.flags = (uint32_t *)(base + off);
    off = align256(off + sizeof(uint32_t));
    if (v) *v = cv;
    return off;
}

static bool valid_desc(const kvq_cache_desc *d)
{
    if (!d) { set_error("descriptor is NULL"); return false; }
    if (d->head_dim != kD) { set_error("head_dim must be 64 (got %d)", d->head_dim); return false; }
    if (d->n_layers < 1 || d->max_seqs < 1 || d->n_kv_heads < 1 || d->n_q_heads < 1) {
        set_error("n_layers, max_seqs, n_q_heads, n_kv_heads must be positive"); return false;
    }
    if (d->n_q_heads % d->n_kv_heads != 0) {
        set_error("n_q_heads (%d) must be a multiple of n_kv_heads (%d)", d->n_q_heads, d->n_kv_heads); return false;
    }
    const int P = d->page_tokens ? d->page_tokens : 256;
    if (P < 256 || (P & (P - 1)) != 0 || P > (1 << 20)) { set_error("page_tokens must be a power of two, at least 256"); return false; }
    // the upper limit keeps a sequence's units x class weight inside 32 bits in the attention kernel
    if (d->max_context < 1 || d->max_context > ((int64_t)1 << 26)) { set_error("max_context out of range (1 .. 2^26)"); return false; }
    const int64_t mpps = (d->max_context + P - 1) / P;
    for (int c = 0; c < kClasses; ++c) {
        if (d->pool_pages[c] < 0 || d->pool_pages[c] > 0x7ffffff0) { set_error("pool_pages[%d] out of range", c); return false; }
        if (d->pool_pages[c] == 0 && (int64_t)d->max_seqs * mpps > 0x7ffffff0) { set_error("default pool too large"); return false; }
    }
    return true;
}

// ---------------------------------------------------------------------------------------------
// kernels
// ---------------------------------------------------------------------------------------------

__global__ void k_reset(CacheView cv)
{
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int c = 0; c < kClasses; ++c) {
        const int n = cv.n_pages[c];
        // stack popped from the top: hand out low page ids first
        for (int64_t i = tid; i < n; i += stride) cv.free_stack[c][i] = (int32_t)(n - 1 - i);
    }
    for (int64_t i = tid; i < (int64_t)cv.max_seqs * 5; i += stride) cv.counts[i] = 0;
    for (int64_t i = tid; i < cv.max_seqs; i += stride) cv.last_T[i] = 0;
    for (int64_t i = tid; i < (int64_t)cv.max_seqs * 4; i += stride) cv.last_rec[i] = 0;
    if (tid < kClasses) cv.free_top[tid] = cv.n_pages[tid];
    if (tid == 0) *cv.flags = 0;
}

__global__ void k_free_seqs(CacheView cv, const int32_t *seq_ids, int n_seq)
{
    const int si = blockIdx.x;
    if (si >= n_seq) return;
    const int seq = seq_ids ? seq_ids[si] : si;
    if (seq < 0 || seq >= cv.max_seqs) return;
    int32_t *cnt = cv.counts + (size_t)seq * 5;
    for (int c = 0; c < kClasses; ++c) {
        const int np = (cnt[c] + cv.page_tokens - 1) / cv.page_tokens;
        const int32_t *pt = cv.page_table + ((size_t)seq * kClasses + c) * cv.max_pages_per_seq;
        for (int i = threadIdx.x; i < np; i += blockDim.x) {
            const int page = pt[i];
            if (page >= 0 && page < cv.n_pages[c]) {               // never the sink page
                const int idx = atomicAdd(&cv.free_top[c], 1);
                if (idx >= 0 && idx < cv.n_pages[c]) cv.free_stack[c][idx] = page;
            }
        }
    }
    __syncthreads();
    if (threadIdx.x < 5) cnt[threadIdx.x] = 0;
    if (threadIdx.x == 0) { cv.last_T[seq] = 0; cv.last_rec[(size_t)seq * 4] = 0; }
}

// Bucket bookkeeping for T new tokens of each listed sequence: one workgroup of 1 to 16 wavefronts per sequence walks
// the tokens 64 per wavefront at a time.  A ballot per class gives every token its rank among its wavefront's tokens of
// that class; the wavefronts' class counts go through LDS, and their exclusive prefix (a scan over at most 16 entries)
// turns the rank into the token's slot.  With one wavefront this is the decode-step shape; with 16 it allocates the
// slots of a long prompt 1024 tokens per pass.
constexpr int kAdvanceMaxWaves = 16;

__global__ __launch_bounds__(64 * kAdvanceMaxWaves) void k_advance(CacheView cv, const uint8_t *bits, const int32_t *seq_ids, int seq0, int n_seq, int T)
{
    __shared__ int wave_count[kAdvanceMaxWaves][kClasses];
    const int si = blockIdx.x;
    if (si >= n_seq) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n_waves = blockDim.x >> 6;
    const int seq = seq_ids ? seq_ids[si] : seq0 + si;
    if (seq < 0 || seq >= cv.max_seqs) {
        if (tid == 0) atomicOr(cv.flags, KVQ_FLAG_CONTEXT_FULL);
        return;
    }
    int32_t *cnt = cv.counts + (size_t)seq * 5;
    const int len = cnt[4];
    if ((int64_t)len + T > (int64_t)cv.max_context) {
        if (tid == 0) {
            atomicOr(cv.flags, KVQ_FLAG_CONTEXT_FULL);
            cv.last_T[seq] = 0;
            cv.last_rec[(size_t)seq * 4] = 0;
        }
        return;
    }
    int cc[kClasses] = {cnt[0], cnt[1], cnt[2], cnt[3]};
    if (tid < kClasses) cv.last_start[(size_t)seq * 4 + tid] = cnt[tid];
    bool bad = false;
    int newest_b = 0, newest_cls = 0, newest_slot = -1;            // set by the thread that handles the call's last token
    for (int t0 = 0; t0 < T; t0 += 64 * n_waves) {
        const int t = t0 + tid;
        const bool valid = t < T;
        int b = valid ? (int)bits[(size_t)si * T + t] : 0;
        if (valid && b != 2 && b != 4 && b != 8 && b != 16) { bad = true; b = 16; }
        const int cls = bits_to_class(b);
        int rank = 0;
#pragma unroll
        for (int c = 0; c < kClasses; ++c) {
            const unsigned long long mask = __ballot(valid && cls == c);
            if (cls == c) rank = __popcll(mask & ((1ull << lane) - 1ull));
            if (lane == 0) wave_count[wave][c] = __popcll(mask);
        }
        __syncthreads();
        int before = 0, total[kClasses] = {0, 0, 0, 0};
        for (int w = 0; w < n_waves; ++w) {
#pragma unroll
            for (int c = 0; c < kClasses; ++c) {
                const int n = wave_count[w][c];
                if (w < wave && c == cls) before += n;
                total[c] += n;
            }
        }
        if (valid) {
            const int slot = (cls == 0 ? cc[0] : cls == 1 ? cc[1] : cls == 2 ? cc[2] : cc[3]) + before + rank;
            if (slot % cv.page_tokens == 0) {
                int page;
                const int idx = atomicSub(&cv.free_top[cls], 1) - 1;
                if (idx < 0) {
                    atomicAdd(&cv.free_top[cls], 1);
                    atomicOr(cv.flags, KVQ_FLAG_POOL_EXHAUSTED);
                    page = cv.n_pages[cls];                            // sink page: in bounds, shared, garbage
                } else {
                    page = cv.free_stack[cls][idx];
                }
                cv.page_table[((size_t)seq * kClasses + cls) * cv.max_pages_per_seq + slot / cv.page_tokens] = page;
            }
            const size_t pos = (size_t)seq * cv.max_context + len + t;
            cv.bits_log[pos] = (uint8_t)b;
            cv.slot_log[pos] = slot;
            cv.pos_log[pos_log_index(cv, seq, cls, slot)] = len + t;
            if (t == T - 1) { newest_b = b; newest_cls = cls; newest_slot = slot; }
        }
#pragma unroll
        for (int c = 0; c < kClasses; ++c) cc[c] += total[c];
        __syncthreads();                                               // wave_count is rewritten by the next pass
    }
    if (__ballot(bad) != 0ull && lane == 0) atomicOr(cv.flags, KVQ_FLAG_BAD_BITS);
    if (tid == 0) {
        cnt[0] = cc[0]; cnt[1] = cc[1]; cnt[2] = cc[2]; cnt[3] = cc[3];
        cnt[4] = len + T;
        cv.last_T[seq] = T;
    }
    if (newest_slot >= 0) {
        // the page-table entry may have been written by another thread of this workgroup: the barriers of the loop
        // above order that write before this read
        const int page = cv.page_table[((size_t)seq * kClasses + newest_cls) * cv.max_pages_per_seq + newest_slot / cv.page_tokens];
        int32_t *rec = cv.last_rec + (size_t)seq * 4;
        rec[0] = T; rec[1] = newest_b; rec[2] = newest_slot; rec[3] = page;
    }
}

// One wavefront per (layer, sequence, token, kv-head): quantizes the K vector and the V vector and
// stores them at the slot the bookkeeping kernel assigned.  Tokens never share a byte, so any number
// of tokens can be written in parallel.
__global__ __launch_bounds__(256) void k_append_write(CacheView cv, int layer, const __half *k, const __half *v,
                                                      const int32_t *seq_ids, int n_seq, int T, long long total_vecs)
{
    // This kernel runs once per layer and decode step and lives on latency: its arguments come in one batch of scalar
    // loads behind one wait (the compiler would fetch each where it is first used and wait for each), and the wave's
    // place in the launch is taken apart in 32-bit scalar arithmetic whenever the launch is small enough for that (the
    // emulated 64-bit divisions were a third of the kernel's instructions).
    int Hkv = cv.Hkv;
    const int max_seqs = cv.max_seqs;
    const int32_t *const last_rec_p = cv.last_rec;
    const uint8_t *const pool0 = cv.pool[0];
    asm volatile("" : "+s"(Hkv) : "s"(layer), "s"(k), "s"(v), "s"(seq_ids), "s"(n_seq), "s"(T), "s"(total_vecs), "s"(max_seqs),
                 "s"(last_rec_p), "s"(pool0));
    const int lane = threadIdx.x & 63;
    int h, t, si, li;
    if (total_vecs <= 0x7fffffffLL) {
        const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)((blockIdx.x * 256u + threadIdx.x) >> 6));
        if (wave >= (uint32_t)total_vecs) return;
        uint32_t r = wave;
        h = (int)(r % (uint32_t)Hkv); r /= (uint32_t)Hkv;
        t = 0;
        if (T != 1) { t = (int)(r % (uint32_t)T); r /= (uint32_t)T; }
        si = (int)(r % (uint32_t)n_seq);
        li = (int)(r / (uint32_t)n_seq);
    } else {
        const long long wave = ((long long)blockIdx.x * 256 + threadIdx.x) >> 6;
        if (wave >= total_vecs) return;
        long long r = wave;
        h = (int)(r % Hkv); r /= Hkv;
        t = (int)(r % T); r /= T;
        si = (int)(r % n_seq);
        li = (int)(r / n_seq);
    }
    const int L = layer < 0 ? li : layer;
    const int seq = seq_ids ? seq_ids[si] : si;
    if (seq < 0 || seq >= max_seqs) return;
    // the vectors themselves do not depend on where they go: asked for first, they travel with the slot lookup
    const size_t src = ((((size_t)li * n_seq + si) * T + t) * Hkv + h) * kD + lane;
    const __half kx = k[src], vx = v[src];
    int b, slot, page;
    if (T == 1) {
        // the decode step: everything about the new token in one 16-byte read
        const int4 rec = *(const int4 *)(last_rec_p + (size_t)seq * 4);
        if (rec.x != 1) return;                                    // the bookkeeping call skipped this sequence
        b = rec.y; slot = rec.z; page = rec.w;
    } else {
        const int lastT = cv.last_T[seq];
        if (lastT != T || t >= lastT) return;
        const int len = cv.counts[(size_t)seq * 5 + 4];
        const size_t pos = (size_t)seq * cv.max_context + (len - lastT + t);
        b = cv.bits_log[pos];
        slot = cv.slot_log[pos];
        page = cv.page_table[((size_t)seq * kClasses + bits_to_class(b)) * cv.max_pages_per_seq + slot / cv.page_tokens];
    }
    const int cls = bits_to_class(b);
    const int blk = (slot % cv.page_tokens) / kBlockTokens;
    const int tok = slot % kBlockTokens;
    uint8_t *base = cv.pool[cls] + block_offset(cv, cls, L, page, h, blk);
    const int meta_bytes = class_meta_bytes(cls);
    const size_t region = (size_t)class_chunks(cls) * kBlockTokens * 16;
    __half *meta = (__half *)(base + tok * 8);
    if (cv.k_channel && b != 16) {
        const size_t ti = ((size_t)L * cv.Hkv + h) * kD + lane;
        const float mn = __half2float(cv.kch_min[ti]);
        const float st = __half2float(cv.kch_step[(size_t)cls * cv.n_layers * cv.Hkv * kD + ti]);
        quantize_store_kch(kx, b, mn, st, lane, tok, base + meta_bytes, meta);
    } else {
        quantize_store(kx, b, lane, tok, base + meta_bytes, meta);
    }
    quantize_store(vx, b, lane, tok, base + meta_bytes + region, meta + 2);
}

// per-class steps of the static per-channel key quantizer: step = fp16(range / levels), IEEE binary32 division
__global__ void k_set_kch(CacheView cv, const __half *kmin, const __half *krange, long long n)
{
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    cv.kch_min[i] = kmin[i];
    const float r = __half2float(krange[i]);
#pragma unroll
    for (int c = 0; c < 3; ++c) cv.kch_step[(size_t)c * n + i] = __float2half_rn(r / (float)((1 << class_bits(c)) - 1));
}

// ---- bulk (prefill) append: lane = token ------------------------------------------------------------------
//
// With many tokens per sequence in one call a lane takes a whole token: it holds the token's 64-element vector in 32
// registers (element pair (2m, 2m+1) per register, exactly the pairing of the cache's words), finds min and max
// without any cross-lane traffic, quantizes in place and writes its 16-byte chunks.  Two kernels share these pieces:
// k_append_bulk gives a wavefront 64 consecutive input tokens (lanes of one class hold consecutive slots, so their
// chunk stores are contiguous pieces of that class's block), k_append_blocks gives it 64 consecutive slots of one
// class (a whole block of the cache) and has it fetch the tokens that sit there.

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

// Q_b of the lane's vector, in place: p[m] becomes code(2m) | code(2m+1) << 16.  Returns scale bits | min bits << 16.
// Same arithmetic as quantize_store.  The quotient (x - min) / s is first formed with a reciprocal (error below
// 7e-5 for quotients up to 1.5 * 255); it decides the rounding unless it lies within 2^-12 of a tie, where the
// IEEE division is evaluated, so every code equals rint of the correctly rounded quotient.
// Packed fp16 min / max as the instructions themselves: the generic builtins first canonicalize every operand (a
// v_pk_max_f16 x, x each), which for a running minimum and maximum over 32 registers is as many instructions again.
__device__ __forceinline__ uint32_t pk_min_f16(uint32_t a, uint32_t b)
{
    uint32_t r;
    asm("v_pk_min_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ uint32_t pk_max_f16(uint32_t a, uint32_t b)
{
    uint32_t r;
    asm("v_pk_max_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// 1.0f that the optimizer cannot see through: fmaf((float)h, one, -m) is h - m rounded once, the same value as the
// binary32 subtraction of the converted half, but it is a single v_fma_mix_f32 that takes the half where it sits
// (either half of the pair register) instead of a conversion and a subtraction.
__device__ __forceinline__ float opaque_one()
{
    float one = 1.0f;
    asm volatile("" : "+s"(one));
    return one;
}

__device__ __forceinline__ uint32_t quantize_lane(uint32_t (&p)[32], float levels)
{
    uint32_t mnp = p[0], mxp = p[0];
#pragma unroll
    for (int m = 1; m < 32; ++m) {
        mnp = pk_min_f16(mnp, p[m]);
        mxp = pk_max_f16(mxp, p[m]);
    }
    const f16x2 mn2 = __builtin_bit_cast(f16x2, mnp), mx2 = __builtin_bit_cast(f16x2, mxp);
    float mn = fminf((float)mn2[0], (float)mn2[1]);
    float mx = fmaxf((float)mx2[0], (float)mx2[1]);
    if (mn == 0.0f) mn = 0.0f;
    if (mx == 0.0f) mx = 0.0f;
    const float range = mx - mn;
    const float scale32 = range / levels;                          // IEEE binary32 division
    const __half sh = __float2half_rn(scale32);
    const float s = __half2float(sh);
    const float inv = s != 0.0f ? __builtin_amdgcn_rcpf(s) : 0.0f;  // s == 0: every quotient reads 0, every code is 0
    // four elements at a time: one near-tie test (and one rarely taken branch) per group keeps the common path a
    // straight run of independent chains.  d >= 0 always (mn is the minimum), so no code is negative.
    constexpr float kNearTie = 0.5f - 0x1p-12f;
    const uint32_t ilevels = (uint32_t)levels;
    const float one = opaque_one(), nmn = -mn;
#pragma unroll
    for (int m = 0; m < 32; m += 2) {
        const f16x2 x0 = __builtin_bit_cast(f16x2, p[m]), x1 = __builtin_bit_cast(f16x2, p[m + 1]);
        const float d[4] = {fmaf((float)x0[0], one, nmn), fmaf((float)x0[1], one, nmn), fmaf((float)x1[0], one, nmn), fmaf((float)x1[1], one, nmn)};
        // rounding and conversion in one addition: q + 1.5 * 2^23 has an ulp of 1, so the sum is rint(q) (ties to even,
        // as v_rndne) and its low mantissa bits are the code itself (0 <= q < 2^16 here)
        constexpr float kMagic = 12582912.0f;
        float t[4];
        bool near = false;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            t[e] = fmaf(d[e], inv, kMagic);
            near |= fabsf(fmaf(d[e], inv, kMagic - t[e])) > kNearTie;
        }
        if (near) {
#pragma unroll
            for (int e = 0; e < 4; ++e) t[e] = rintf(d[e] / s) + kMagic;
        }
        // (low half of t[1]) << 16 | low half of t[0]
        p[m] = __builtin_amdgcn_perm(__float_as_uint(t[1]), __float_as_uint(t[0]), 0x05040100u);
        p[m + 1] = __builtin_amdgcn_perm(__float_as_uint(t[3]), __float_as_uint(t[2]), 0x05040100u);
    }
    // The clamp to `levels`: with a normal fp16 scale the largest quotient is at most levels / (1 - 2^-11), which
    // rounds to levels, so no code exceeds it.  Only a subnormal scale (a vector whose range is below levels * 2^-14)
    // can undershoot the exact quotient far enough; those rare lanes clamp their codes afterwards.
    if (s < 0x1p-14f) {
#pragma unroll
        for (int m = 0; m < 32; ++m) p[m] = min(p[m] & 0xffffu, ilevels) | (min(p[m] >> 16, ilevels) << 16);
    }
    return (uint32_t)__half_as_ushort(sh) | ((uint32_t)__half_as_ushort(__float2half_rn(mn)) << 16);
}

// Stores n16 16-byte chunks of the lane's registers p[0 .. 4 n16), chunk c at row c of the token's column.
// `streaming`: the wavefront holds a long run of this class, its piece of each chunk row is mostly whole cache
// lines, and the stores go past the cache (non-temporal); short pieces are stored normally so that the lines they
// share with the neighbouring tiles' pieces are put together in the cache before they reach memory.
template <int N16> __device__ __forceinline__ void store_chunks(const uint32_t (&p)[32], uint8_t *codes, int tok, bool streaming)
{
#pragma unroll
    for (int c = 0; c < N16; ++c) {
        u32x4 o;
        o[0] = p[4 * c]; o[1] = p[4 * c + 1]; o[2] = p[4 * c + 2]; o[3] = p[4 * c + 3];
        u32x4 *dst = (u32x4 *)(codes + (size_t)c * (kBlockTokens * 16) + tok * 16);
        // the streaming form is spelled out: two stores that differ only in the non-temporal hint are merged into
        // one plain store by the optimizer
        if (streaming) asm volatile("global_store_dwordx4 %0, %1, off nt" : : "v"(dst), "v"(o) : "memory");
        else *dst = o;
    }
}

constexpr int kStageRow = 2 * kD + 16;                             // LDS row: one 128-byte vector + 16 bytes of padding

// Coalesced read of a tile's 64 vectors (row stride `row_halves`): each load instruction takes 8 whole 128-byte
// rows, 8 lanes per row.  Rows past the ragged tail repeat the last valid row.
__device__ __forceinline__ void tile_load(u32x4 (&x)[8], const __half *tile_src, size_t row_halves, int nrow, int lane)
{
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int row = i * 8 + (lane >> 3);
        row = row < nrow ? row : nrow - 1;
        x[i] = __builtin_nontemporal_load((const u32x4 *)(tile_src + (size_t)row * row_halves) + (lane & 7));
    }
}

// Transposition through the wavefront's own LDS rows: afterwards lane t holds row t in p[0..31].  The padded row
// stride keeps both the 8-lanes-per-row writes and the lane-per-row reads free of bank conflicts.
__device__ __forceinline__ void tile_transpose(const u32x4 (&x)[8], uint32_t (&p)[32], uint8_t *stage, int lane)
{
#pragma unroll
    for (int i = 0; i < 8; ++i)
        *(u32x4 *)(stage + (i * 8 + (lane >> 3)) * kStageRow + (lane & 7) * 16) = x[i];
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const u32x4 y = *(const u32x4 *)(stage + lane * kStageRow + c * 16);
        p[4 * c + 0] = y[0]; p[4 * c + 1] = y[1]; p[4 * c + 2] = y[2]; p[4 * c + 3] = y[3];
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// The static per-channel variant of quantize_lane for a key vector: tab[c] = {step, 1 / step, minimum, -} of channel c
// for the lane's class (LDS; a lane read of a register would not do here: this runs under divergent control flow, and
// the lanes it would read from need not hold the value).  code = clamp(rint((x - min_c) / step_c), 0, levels) with the
// IEEE quotient deciding near a tie, code 0 where the step is 0.  Same arithmetic as quantize_store_kch.  p[m] becomes
// code(2m) | code(2m+1) << 16.
__device__ __forceinline__ void quantize_lane_kch(uint32_t (&p)[32], float levels, const float4 *tab)
{
    constexpr float kNearTie = 0.5f - 0x1p-12f;
#pragma unroll
    for (int m = 0; m < 32; ++m) {
        const f16x2 x = __builtin_bit_cast(f16x2, p[m]);
        float r[2];
        bool near = false;
        float d[2], st[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const float4 t = tab[2 * m + e];
            d[e] = (float)x[e] - t.z;
            st[e] = t.x;
            const float q = d[e] * t.y;
            r[e] = rintf(q);
            near |= fabsf(q - r[e]) > kNearTie;
        }
        if (near) {
#pragma unroll
            for (int e = 0; e < 2; ++e) r[e] = st[e] != 0.0f ? rintf(d[e] / st[e]) : 0.0f;
        }
#pragma unroll
        for (int e = 0; e < 2; ++e) r[e] = __builtin_amdgcn_fmed3f(r[e], 0.0f, levels);
        p[m] = (uint32_t)r[0] | ((uint32_t)r[1] << 16);
    }
}

// The per-channel key quantizer applied to rows as they were loaded (eight lanes per 128-byte row, so a lane holds the
// same eight channels 8 (lane % 8) .. + 7 of eight different rows): the lane needs the tables of its eight channels
// only, in registers, and the LDS transposition then moves 16-bit codes instead of fp16 values.  Same arithmetic as
// quantize_lane_kch; st / inv / mn: step, 1 / step (0 for a zero step) and minimum of the lane's channels.
__device__ __forceinline__ uint32_t quantize_pair_kch(uint32_t word, float levels, float st0, float st1, float inv0, float inv1, float mn0, float mn1)
{
    constexpr float kNearTie = 0.5f - 0x1p-12f;
    const f16x2 hv = __builtin_bit_cast(f16x2, word);
    const float d0 = (float)hv[0] - mn0, d1 = (float)hv[1] - mn1;
    const float q0 = d0 * inv0, q1 = d1 * inv1;
    float r0 = rintf(q0), r1 = rintf(q1);
    if (fabsf(q0 - r0) > kNearTie || fabsf(q1 - r1) > kNearTie) {
        r0 = st0 != 0.0f ? rintf(d0 / st0) : 0.0f;
        r1 = st1 != 0.0f ? rintf(d1 / st1) : 0.0f;
    }
    r0 = __builtin_amdgcn_fmed3f(r0, 0.0f, levels);
    r1 = __builtin_amdgcn_fmed3f(r1, 0.0f, levels);
    return (uint32_t)r0 | ((uint32_t)r1 << 16);
}

__device__ __forceinline__ void quantize_rows_kch(u32x4 (&x)[8], float levels, const float (&st)[8], const float (&inv)[8], const float (&mn)[8])
{
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        u32x4 v = x[i];
        v.x = quantize_pair_kch(v.x, levels, st[0], st[1], inv[0], inv[1], mn[0], mn[1]);
        v.y = quantize_pair_kch(v.y, levels, st[2], st[3], inv[2], inv[3], mn[2], mn[3]);
        v.z = quantize_pair_kch(v.z, levels, st[4], st[5], inv[4], inv[5], mn[4], mn[5]);
        v.w = quantize_pair_kch(v.w, levels, st[6], st[7], inv[6], inv[7], mn[6], mn[7]);
        x[i] = v;
    }
}

// Quantizes (classes 0..2) and stores the lane's vector.  The packing is one tree for all widths: a word of class b
// holds 16 / b pair registers, pair j at bit b * j, so joining neighbours with shifts b, 2b and 4b (per lane) turns
// the 32 pair registers into the 16 words of the 8-bit class after the first level, the 8 words of the 4-bit class
// after the second and the 4 words of the 2-bit class after the third -- 28 shift-or operations for whatever mix of
// classes the wavefront holds, where a packing routine per class would run one after the other.  The FP16 lanes
// store their registers as they are, before the tree overwrites them.
// kch_tab != nullptr: a key vector under the static per-channel variant (the token's own metadata entry is zero);
// the table is the one of this lane's class.
// quantized == true: p already holds the codes (a key vector of the per-channel variant quantized row-wise before the
// transposition); only the zero metadata entry, the packing and the stores are left.
__device__ __forceinline__ void quantize_pack_store(uint32_t (&p)[32], int cls, uint8_t *codes, uint32_t *meta, int tok, uint32_t streaming,
                                                    const float4 *kch_tab = nullptr, bool quantized = false)
{
    const int b = 2 << cls;
    if (cls == 3) store_chunks<8>(p, codes, tok, (streaming & 8u) != 0);
    else if (quantized) *meta = 0u;
    else if (kch_tab) { quantize_lane_kch(p, (float)((1 << b) - 1), kch_tab); *meta = 0u; }
    else *meta = quantize_lane(p, (float)((1 << b) - 1));
    const uint32_t s1 = (uint32_t)b & 31u, s2 = (uint32_t)(2 * b) & 31u, s3 = (uint32_t)(4 * b) & 31u;
#pragma unroll
    for (int i = 0; i < 16; ++i) p[i] = p[2 * i] | (p[2 * i + 1] << s1);
    if (cls == 2) store_chunks<4>(p, codes, tok, (streaming & 4u) != 0);
#pragma unroll
    for (int i = 0; i < 8; ++i) p[i] = p[2 * i] | (p[2 * i + 1] << s2);
    if (cls == 1) store_chunks<2>(p, codes, tok, (streaming & 2u) != 0);
#pragma unroll
    for (int i = 0; i < 4; ++i) p[i] = p[2 * i] | (p[2 * i + 1] << s3);
    if (cls == 0) store_chunks<1>(p, codes, tok, (streaming & 1u) != 0);
}

// One wavefront per (layer, sequence, tile of 64 input tokens, kv-head); k and v must be 16-byte aligned.
// KCH: the keys use the static per-channel variant; the wavefront then keeps its head's {step, 1 / step, minimum} per
// channel and quantized class in LDS.
template <bool KCH>
__global__ __launch_bounds__(256) void k_append_bulk(CacheView cv, int layer, const __half *k, const __half *v,
                                                     const int32_t *seq_ids, int n_seq, int T, int tiles, long long total_waves, int P_stream_min)
{
    __shared__ __attribute__((aligned(16))) uint8_t stage_all[4][kBlockTokens * kStageRow];
    __shared__ float4 kch_all[KCH ? 4 : 1][KCH ? 3 * kD : 1];
    const long long wave = ((long long)blockIdx.x * 256 + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    uint8_t *stage = stage_all[threadIdx.x >> 6];
    if (wave >= total_waves) return;
    long long r = wave;
    const int h = (int)(r % cv.Hkv); r /= cv.Hkv;
    const int tile = (int)(r % tiles); r /= tiles;
    const int si = (int)(r % n_seq);
    const int li = (int)(r / n_seq);
    const int L = layer < 0 ? li : layer;
    const int seq = seq_ids ? seq_ids[si] : si;
    if (seq < 0 || seq >= cv.max_seqs) return;
    const int lastT = cv.last_T[seq];
    if (lastT != T) return;                                        // the bookkeeping call skipped this sequence
    const int nrow = T - tile * kBlockTokens < kBlockTokens ? T - tile * kBlockTokens : kBlockTokens;
    const size_t row_halves = (size_t)cv.Hkv * kD;
    const size_t src = ((((size_t)li * n_seq + si) * T + (size_t)tile * kBlockTokens) * cv.Hkv + h) * kD;
    u32x4 x[8];
    uint32_t p[32];
    tile_load(x, k + src, row_halves, nrow, lane);

    // where this lane's token goes (lanes past the ragged tail compute nothing and store nothing)
    const bool valid = lane < nrow;
    int cls = 3, tok = 0;
    uint8_t *base = nullptr;
    if (valid) {
        const int len = cv.counts[(size_t)seq * 5 + 4];
        const size_t pos = (size_t)seq * cv.max_context + (len - lastT + tile * kBlockTokens + lane);
        const int b = cv.bits_log[pos];
        const int slot = cv.slot_log[pos];
        cls = bits_to_class(b);
        const int page = cv.page_table[((size_t)seq * kClasses + cls) * cv.max_pages_per_seq + slot / cv.page_tokens];
        const int blk = (slot % cv.page_tokens) / kBlockTokens;
        tok = slot % kBlockTokens;
        base = cv.pool[cls] + block_offset(cv, cls, L, page, h, blk);
    }
    const int meta_bytes = cls == 3 ? 0 : kBlockTokens * 8;
    const size_t region = (size_t)(1 << cls) * kBlockTokens * 16;
    uint32_t *meta = (uint32_t *)(base + tok * 8);

    tile_transpose(x, p, stage, lane);
    tile_load(x, v + src, row_halves, nrow, lane);                 // V is in flight while K is quantized
    // which classes have a long run in this tile (bit c: at least P_stream_min of the 64 tokens, i.e. pieces of 256 bytes
    // and more per chunk row with the default of 16)
    uint32_t streaming = 0;
#pragma unroll
    for (int c = 0; c < kClasses; ++c)
        if (__popcll(__ballot(valid && cls == c)) >= P_stream_min) streaming |= 1u << c;
    if constexpr (KCH) {
        float4 *tab = kch_all[threadIdx.x >> 6];
        const size_t ti = ((size_t)L * cv.Hkv + h) * kD + lane;
        const float minv = __half2float(cv.kch_min[ti]);
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            const float st = __half2float(cv.kch_step[(size_t)c * cv.n_layers * cv.Hkv * kD + ti]);
            tab[c * kD + lane] = make_float4(st, st != 0.0f ? __builtin_amdgcn_rcpf(st) : 0.0f, minv, 0.0f);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (valid) quantize_pack_store(p, cls, base + meta_bytes, meta, tok, streaming, tab + (cls < 3 ? cls : 0) * kD);
    } else {
        if (valid) quantize_pack_store(p, cls, base + meta_bytes, meta, tok, streaming);
    }
    tile_transpose(x, p, stage, lane);
    if (valid) quantize_pack_store(p, cls, base + meta_bytes + region, meta + 1, tok, streaming);
}

// The prefill writer proper: one wavefront per (layer, sequence, block of 64 slots of one class, kv-head), lane =
// slot.  Working from the output side means that a wavefront writes one whole block of the cache (every chunk row a
// contiguous kilobyte) and meets a single class, whatever the order of widths in the prompt; the token that sits in a
// slot comes from the slot -> position log, and its two 128-byte input rows are whole cache lines wherever it lies.
// Only the first and the last block of a class in a call are pieces.  A sequence's work items are the blocks its call
// touches, widest class first; `items` (at most tiles + 7) bounds their number and the surplus wavefronts leave at once.
constexpr int kGridY = 32768;
// wavefronts (kv-heads of one block of slots) per workgroup: its waves read adjacent 128-byte pieces of the same token
// rows.  Measured at the benchmark's shape (32 sequences x 2048 tokens): 4 waves 129-134 us, 8 waves 132-144 us, 2 waves
// 143-153 us.
constexpr int kBlkWaves = 4;
template <bool KCH>
__global__ __launch_bounds__(64 * kBlkWaves, (KCH ? 12 : 16) / kBlkWaves) void k_append_blocks(CacheView cv, int layer, const __half *k, const __half *v,
                                                       const int32_t *seq_ids, int n_seq, int n_pairs, int T, int items, int P_stream_min)
{
    __shared__ __attribute__((aligned(16))) uint8_t stage_all[kBlkWaves][kBlockTokens * kStageRow];
    // the wavefront's number inside the workgroup as a scalar: everything derived from it (work item, class, block
    // address) then lives in scalar registers and the class branches are uniform
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int iw = blockIdx.x * kBlkWaves + wv;                            // grid: x = (work item, kv-head), y and z = (layer, sequence)
    const int pair = blockIdx.z * kGridY + blockIdx.y;
    if (iw >= items * cv.Hkv || pair >= n_pairs) return;
    const int lane = threadIdx.x & 63;
    uint8_t *stage = stage_all[wv];
    const int h = iw % cv.Hkv, item = iw / cv.Hkv;
    const int si = pair % n_seq, li = pair / n_seq;
    const int L = layer < 0 ? li : layer;
    const int seq = seq_ids ? seq_ids[si] : si;
    if (seq < 0 || seq >= cv.max_seqs) return;
    if (cv.last_T[seq] != T) return;                                // the bookkeeping call skipped this sequence
    const int32_t *cnt = cv.counts + (size_t)seq * 5, *start = cv.last_start + (size_t)seq * 4;
    const int len0 = cnt[4] - T;
    // which block of which class this work item is
    int cls = -1, s0 = 0, lo = 0, hi = 0, left = item;
#pragma unroll
    for (int c = kClasses - 1; c >= 0; --c) {
        const int s = start[c], e = cnt[c];
        const int nb = e > s ? ((e - 1) >> 6) - (s >> 6) + 1 : 0;
        if (cls < 0 && left < nb) {
            cls = c;
            s0 = ((s >> 6) + left) << 6;
            lo = s > s0 ? s - s0 : 0;
            hi = e - s0 < kBlockTokens ? e - s0 : kBlockTokens;
        }
        left -= nb;
    }
    if (cls < 0) return;
    const bool valid = lane >= lo && lane < hi;
    int t = 0;
    if (valid) t = cv.pos_log[pos_log_index(cv, seq, cls, s0 + lane)] - len0;
    t = t < 0 ? 0 : t > T - 1 ? T - 1 : t;                          // in bounds whatever the log holds
    const int t_first = __shfl(t, lo);
    if (!valid) t = t_first;                                        // rows outside the piece repeat its first token
    const size_t row_halves = (size_t)cv.Hkv * kD;
    const size_t src = (((size_t)li * n_seq + si) * T * cv.Hkv + h) * kD;
    int row_t[8];                                                   // load i takes rows 8 i .. 8 i + 7, eight lanes per row
#pragma unroll
    for (int i = 0; i < 8; ++i) row_t[i] = __shfl(t, i * 8 + (lane >> 3));
    u32x4 x[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = __builtin_nontemporal_load((const u32x4 *)(k + src + (size_t)row_t[i] * row_halves) + (lane & 7));

    const int page = cv.page_table[((size_t)seq * kClasses + cls) * cv.max_pages_per_seq + s0 / cv.page_tokens];
    uint8_t *base = cv.pool[cls] + block_offset(cv, cls, L, page, h, (s0 % cv.page_tokens) / kBlockTokens);
    const bool streaming = hi - lo >= P_stream_min;
    const __half *vsrc = v + src + (lane & 7) * 8;
    // per-channel keys: the lane's eight channels' tables (the class is the wave's), asked for while the rows travel
    float kst[8], kinv[8], kmn[8];
    const bool kch_rows = KCH && cls < 3;
    if constexpr (KCH) {
        if (cls < 3) {
            const size_t ti = ((size_t)L * cv.Hkv + h) * kD + (lane & 7) * 8;
            const u32x4 mn4 = *(const u32x4 *)(cv.kch_min + ti);
            const u32x4 st4 = *(const u32x4 *)(cv.kch_step + (size_t)cls * cv.n_layers * cv.Hkv * kD + ti);
            const uint32_t mw[4] = {mn4.x, mn4.y, mn4.z, mn4.w}, sw[4] = {st4.x, st4.y, st4.z, st4.w};
#pragma unroll
            for (int wd = 0; wd < 4; ++wd) {
                const f16x2 a = __builtin_bit_cast(f16x2, mw[wd]), b2 = __builtin_bit_cast(f16x2, sw[wd]);
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    kmn[2 * wd + e] = (float)a[e];
                    kst[2 * wd + e] = (float)b2[e];
                    kinv[2 * wd + e] = kst[2 * wd + e] != 0.0f ? __builtin_amdgcn_rcpf(kst[2 * wd + e]) : 0.0f;
                }
            }
        }
    }
    // The class as the quantizer sees it sits in a vector register: the addresses above are scalar, but branches the
    // compiler knows to be uniform make it schedule the four widths' code so that the V rows in flight no longer fit
    // in four wavefronts' worth of registers.
    int cls_v = cls;
    asm volatile("" : "+v"(cls_v));
    const int meta_bytes = cls == 3 ? 0 : kBlockTokens * 8;
    const size_t region = (size_t)(1 << cls) * kBlockTokens * 16;
    uint32_t *meta = (uint32_t *)(base + lane * 8);
    const uint32_t stm = streaming ? 15u : 0u;
    uint32_t p[32];
    if constexpr (KCH) {
        if (kch_rows) quantize_rows_kch(x, (float)((1 << (2 << cls)) - 1), kst, kinv, kmn);
    }
    tile_transpose(x, p, stage, lane);
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = __builtin_nontemporal_load((const u32x4 *)(vsrc + (size_t)row_t[i] * row_halves));
    if (valid) quantize_pack_store(p, cls_v, base + meta_bytes, meta, lane, stm, nullptr, kch_rows);
    tile_transpose(x, p, stage, lane);
    if (valid) quantize_pack_store(p, cls_v, base + meta_bytes + region, meta + 1, lane, stm);
}

// Canonical dump of one (layer, sequence): one wavefront per (token, kv-head), lane = element.
__global__ __launch_bounds__(256) void k_export(CacheView cv, int layer, int seq, uint8_t *bits_out, uint8_t *codes_out,
                                                uint16_t *meta_out, long long max_tokens)
{
    const long long wave = ((long long)blockIdx.x * 256 + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    const int len = cv.counts[(size_t)seq * 5 + 4];
    const long long ntok = len < max_tokens ? len : max_tokens;
    if (wave >= ntok * cv.Hkv) return;
    const int h = (int)(wave % cv.Hkv);
    const long long t = wave / cv.Hkv;
    const size_t pos = (size_t)seq * cv.max_context + t;
    const int b = cv.bits_log[pos];
    const int slot = cv.slot_log[pos];
    const int cls = bits_to_class(b);
    const int page = cv.page_table[((size_t)seq * kClasses + cls) * cv.max_pages_per_seq + slot / cv.page_tokens];
    const int blk = (slot % cv.page_tokens) / kBlockTokens;
    const int tok = slot % kBlockTokens;
    const uint8_t *base = cv.pool[cls] + block_offset(cv, cls, layer, page, h, blk);
    const int meta_bytes = class_meta_bytes(cls);
    const size_t region = (size_t)class_chunks(cls) * kBlockTokens * 16;
    const int per = 32 / b;
    const int w = lane / per, r = lane % per;
    const uint32_t mask = b == 16 ? 0xffffu : ((1u << b) - 1u);
    for (int which = 0; which < 2; ++which) {
        const uint8_t *codes = base + meta_bytes + which * region;
        const uint32_t word = *(const uint32_t *)(codes + (size_t)(w >> 2) * (kBlockTokens * 16) + tok * 16 + (w & 3) * 4);
        const uint32_t code = (word >> (b * (r >> 1) + 16 * (r & 1))) & mask;
        const uint32_t canon = group_or(code << (b * r), per);      // element i at bits [i*b, i*b+b)
        uint32_t *rec = (uint32_t *)(codes_out + (((size_t)t * cv.Hkv + h) * 2 + which) * KVQ_EXPORT_REC);
        if (r == 0) rec[w] = canon;
        if (lane >= 2 * b && lane < 32) rec[lane] = 0u;             // words past the 8*b code bytes
        if (lane == 0) {
            uint16_t *m = meta_out + (((size_t)t * cv.Hkv + h) * 2 + which) * 2;
            if (cls == 3) { m[0] = 0; m[1] = 0; }
            else {
                const uint16_t *src = (const uint16_t *)(base + tok * 8 + which * 4);
                m[0] = src[0]; m[1] = src[1];
            }
        }
    }
    if (h == 0 && lane == 0) bits_out[t] = (uint8_t)b;
}

// Inverse of k_export for tokens that the bookkeeping kernel has just logged: one wavefront per (token, kv-head),
// lane = element.  The codes of the canonical record are moved into the cache's word layout, nothing is re-quantized.
__global__ __launch_bounds__(256) void k_import(CacheView cv, int layer, int seq, const uint8_t *codes_in, const uint16_t *meta_in,
                                                long long T)
{
    const long long wave = ((long long)blockIdx.x * 256 + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (wave >= T * cv.Hkv) return;
    const int lastT = cv.last_T[seq];
    if ((long long)lastT != T) return;                            // the bookkeeping call skipped this sequence
    const int h = (int)(wave % cv.Hkv);
    const long long t = wave / cv.Hkv;
    const int len = cv.counts[(size_t)seq * 5 + 4];
    const size_t pos = (size_t)seq * cv.max_context + (len - lastT + t);
    const int b = cv.bits_log[pos];
    const int slot = cv.slot_log[pos];
    const int cls = bits_to_class(b);
    const int page = cv.page_table[((size_t)seq * kClasses + cls) * cv.max_pages_per_seq + slot / cv.page_tokens];
    const int blk = (slot % cv.page_tokens) / kBlockTokens;
    const int tok = slot % kBlockTokens;
    uint8_t *base = cv.pool[cls] + block_offset(cv, cls, layer, page, h, blk);
    const int meta_bytes = class_meta_bytes(cls);
    const size_t region = (size_t)class_chunks(cls) * kBlockTokens * 16;
    const int per = 32 / b;
    const int w = lane / per, r = lane % per;
    const uint32_t mask = b == 16 ? 0xffffu : ((1u << b) - 1u);
    for (int which = 0; which < 2; ++which) {
        const uint32_t *rec = (const uint32_t *)(codes_in + (((size_t)t * cv.Hkv + h) * 2 + which) * KVQ_EXPORT_REC);
        const int bit = lane * b;                                 // element i at bits [i*b, i*b+b) of the record
        const uint32_t code = (rec[bit >> 5] >> (bit & 31)) & mask;
        const uint32_t word = group_or(code << (b * (r >> 1) + 16 * (r & 1)), per);
        uint8_t *codes = base + meta_bytes + which * region;
        if (r == 0) *(uint32_t *)(codes + (size_t)(w >> 2) * (kBlockTokens * 16) + tok * 16 + (w & 3) * 4) = word;
        if (lane == 0 && cls != 3) {
            const uint16_t *m = meta_in + (((size_t)t * cv.Hkv + h) * 2 + which) * 2;
            uint16_t *dst = (uint16_t *)(base + tok * 8 + which * 4);
            dst[0] = m[0]; dst[1] = m[1];
        }
    }
}

}  // namespace kvq

using namespace kvq;

// ---------------------------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------------------------

namespace kvq {

struct TuningKey { const char *name; const char *env; int Tuning::*field; int dflt, lo, hi; };

static const TuningKey kTuningKeys[] = {
    {"attn_splits", "KVQ_ATTN_SPLITS", &Tuning::attn_splits, 0, 0, 64},
    {"attn_waves", "KVQ_ATTN_WAVES", &Tuning::attn_waves, 0, 0, 8},
    {"attn_longest_first", "KVQ_ATTN_LONGEST_FIRST", &Tuning::attn_longest_first, -1, -1, 1},
    {"attn_by_class", "KVQ_ATTN_BY_CLASS", &Tuning::attn_by_class, 12, 0, 1 << 20},
    {"append_bulk_min_T", "KVQ_APPEND_BULK_MIN_T", &Tuning::append_bulk_min_T, 32, 1, 1 << 30},
    {"append_stream_min", "KVQ_APPEND_STREAM_MIN", &Tuning::append_stream_min, 16, 0, 65},
    {"append_block_min_T", "KVQ_APPEND_BLOCK_MIN_T", &Tuning::append_block_min_T, 512, 1, 1 << 30},
    {"controller_no_mfma", "KVQ_CONTROLLER_NO_MFMA", &Tuning::controller_no_mfma, 0, 0, 1},
    {"controller_waves", "KVQ_CONTROLLER_WAVES", &Tuning::controller_waves, 0, 0, 8},
    {"controller_wg_per_cu", "KVQ_CONTROLLER_WG_PER_CU", &Tuning::controller_wg_per_cu, 0, 0, 4},
    {"train_no_mfma", "KVQ_TRAIN_NO_MFMA", &Tuning::train_no_mfma, 0, 0, 1},
};

// The table's defaults, overridden by the KVQ_* environment variables as they stand when the table is first needed.
Tuning &tuning()
{
    static Tuning t = [] {
        Tuning v;
        for (const TuningKey &k : kTuningKeys) {
            int x = k.dflt;
            const char *e = getenv(k.env);
            if (e && *e) {
                const int y = atoi(e);
                if (y >= k.lo && y <= k.hi) x = y;
            }
            v.*(k.field) = x;
        }
        return v;
    }();
    return t;
}

}  // namespace kvq

extern "C" int kvq_tuning_set(const char *name, int32_t value)
{
    if (!name) { set_error("name is NULL"); return KVQ_ERR_INVALID_ARG; }
    for (const TuningKey &k : kTuningKeys)
        if (strcmp(name, k.name) == 0) {
            if (value < k.lo || value > k.hi) { set_error("%s = %d is outside %d .. %d", name, value, k.lo, k.hi); return KVQ_ERR_INVALID_ARG; }
            tuning().*(k.field) = value;
            return KVQ_OK;
        }
    set_error("unknown tuning entry '%s'", name);
    return KVQ_ERR_INVALID_ARG;
}

extern "C" int kvq_tuning_get(const char *name, int32_t *value)
{
    if (!name || !value) { set_error("name or value is NULL"); return KVQ_ERR_INVALID_ARG; }
    for (const TuningKey &k : kTuningKeys)
        if (strcmp(name, k.name) == 0) { *value = tuning().*(k.field); return KVQ_OK; }
    set_error("unknown tuning entry '%s'", name);
    return KVQ_ERR_INVALID_ARG;
}

extern "C" const char *kvq_version(void) { return "kvq 0.2 (gfx950)"; }
extern "C" const char *kvq_last_error(void) { return g_err; }

extern "C" size_t kvq_cache_arena_bytes(const kvq_cache_desc *desc)
{
    if (!valid_desc(desc)) return 0;
    return plan_arena(*desc, nullptr, nullptr);
}

extern "C" int kvq_cache_create(const kvq_cache_desc *desc, kvq_cache **out)
{
    if (!out) { set_error("out is NULL"); return KVQ_ERR_INVALID_ARG; }
    *out = nullptr;
    if (!valid_desc(desc)) return desc && desc->head_dim != kD ? KVQ_ERR_UNSUPPORTED : KVQ_ERR_INVALID_ARG;
    const size_t need = plan_arena(*desc, nullptr, nullptr);
    void *arena = desc->arena;
    bool own = false;
    if (arena) {
        if (((uintptr_t)arena & 255) != 0) { set_error("arena must be 256-byte aligned"); return KVQ_ERR_INVALID_ARG; }
        if (desc->arena_bytes < need) {
            set_error("arena too small: %zu bytes given, %zu needed", desc->arena_bytes, need);
            return KVQ_ERR_OOM;
        }
    } else {
        KVQ_HIP(hipMalloc(&arena, need));
        own = true;
    }
    kvq_cache *c = new (std::nothrow) kvq_cache;
    if (!c) { if (own) (void)hipFree(arena); set_error("host allocation failed"); return KVQ_ERR_OOM; }
    c->desc = *desc;
    c->arena = arena;
    c->arena_bytes = need;
    c->own_arena = own;
    c->len_bound = 0;
    c->touched = false;
    (void)hipGetDevice(&c->device);
    plan_arena(*desc, &c->view, (uint8_t *)arena);
    // Pages hold finite data from the start: lanes past the end of a bucket read in-bounds bytes and
    // weight them by zero, which is only safe if those bytes are never NaN/Inf patterns.
    hipError_t e = hipMemset(arena, 0, need);
    if (e == hipSuccess) {
        hipLaunchKernelGGL(k_reset, dim3(256), dim3(256), 0, 0, c->view);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        if (own) (void)hipFree(arena);
        delete c;
        return check_hip(e, "kvq_cache_create");
    }
    *out = c;
    return KVQ_OK;
}

extern "C" int kvq_cache_destroy(kvq_cache *cache)
{
    if (!cache) return KVQ_OK;
    int rc = KVQ_OK;
    if (cache->own_arena) rc = check_hip(hipFree(cache->arena), "hipFree(arena)");
    delete cache;
    return rc;
}

extern "C" int kvq_cache_reset(kvq_cache *cache, void *stream)
{
    if (!cache) { set_error("cache is NULL"); return KVQ_ERR_INVALID_ARG; }
    hipLaunchKernelGGL(k_reset, dim3(256), dim3(256), 0, (hipStream_t)stream, cache->view);
    KVQ_HIP(hipGetLastError());
    cache->len_bound = 0;
    cache->touched = false;
    return KVQ_OK;
}

extern "C" int kvq_cache_free_seqs(kvq_cache *cache, const int32_t *seq_ids, int32_t n_seq, void *stream)
{
    if (!cache) { set_error("cache is NULL"); return KVQ_ERR_INVALID_ARG; }
    if (n_seq < 0 || n_seq > cache->desc.max_seqs) { set_error("n_seq out of range"); return KVQ_ERR_INVALID_ARG; }
    if (n_seq == 0) return KVQ_OK;
    hipLaunchKernelGGL(k_free_seqs, dim3(n_seq), dim3(256), 0, (hipStream_t)stream, cache->view, seq_ids, n_seq);
    KVQ_HIP(hipGetLastError());
    return KVQ_OK;
}

extern "C" int kvq_cache_set_length_hint(kvq_cache *cache, int64_t longest_live_length)
{
    if (!cache) { set_error("cache is NULL"); return KVQ_ERR_INVALID_ARG; }
    if (longest_live_length < 0) { set_error("length hint is negative"); return KVQ_ERR_INVALID_ARG; }
    cache->len_bound = longest_live_length < cache->desc.max_context ? longest_live_length : cache->desc.max_context;
    return KVQ_OK;
}

extern "C" int kvq_cache_status(kvq_cache *cache, uint32_t *flags, int64_t *free_pages, void *stream)
{
    if (!cache || !flags) { set_error("cache or flags is NULL"); return KVQ_ERR_INVALID_ARG; }
    uint32_t f = 0;
    int32_t top[kClasses];
    KVQ_HIP(hipStreamSynchronize((hipStream_t)stream));
    KVQ_HIP(hipMemcpy(&f, cache->view.flags, sizeof(f), hipMemcpyDeviceToHost));
    KVQ_HIP(hipMemcpy(top, cache->view.free_top, sizeof(top), hipMemcpyDeviceToHost));
    *flags = f;
    if (free_pages) for (int c = 0; c < kClasses; ++c) free_pages[c] = top[c];
    return KVQ_OK;
}

extern "C" int kvq_cache_counts(kvq_cache *cache, int32_t *counts, void *stream)
{
    if (!cache || !counts) { set_error("cache or counts is NULL"); return KVQ_ERR_INVALID_ARG; }
    KVQ_HIP(hipStreamSynchronize((hipStream_t)stream));
    KVQ_HIP(hipMemcpy(counts, cache->view.counts, sizeof(int32_t) * (size_t)cache->desc.max_seqs * 5, hipMemcpyDeviceToHost));
    return KVQ_OK;
}

extern "C" int kvq_cache_usage_of(kvq_cache *cache, kvq_cache_usage *usage, void *stream)
{
    if (!cache || !usage) { set_error("cache or usage is NULL"); return KVQ_ERR_INVALID_ARG; }
    const kvq_cache_desc &d = cache->desc;
    int32_t *counts = new (std::nothrow) int32_t[(size_t)d.max_seqs * 5];
    if (!counts) { set_error("host allocation failed"); return KVQ_ERR_OOM; }
    int rc = kvq_cache_counts(cache, counts, stream);
    int32_t top[kClasses] = {0, 0, 0, 0};
    if (rc == KVQ_OK) rc = check_hip(hipMemcpy(top, cache->view.free_top, sizeof(top), hipMemcpyDeviceToHost), "hipMemcpy(free_top)");
    if (rc != KVQ_OK) { delete[] counts; return rc; }
    static const int bits_of[kClasses] = {2, 4, 8, 16};
    kvq_cache_usage u;
    memset(&u, 0, sizeof(u));
    int64_t total = 0;
    double sum_bits = 0.0;
    for (int c = 0; c < kClasses; ++c) {
        for (int s = 0; s < d.max_seqs; ++s) u.tokens[c] += counts[(size_t)s * 5 + c];
        total += u.tokens[c];
        sum_bits += (double)u.tokens[c] * bits_of[c];
        // per (token, kv-head): K and V codes, plus the two fp16 (scale, minimum) pairs of the quantized classes
        const int64_t per_token_head = class_block_bytes(c) / kBlockTokens;
        u.payload_bytes += u.tokens[c] * per_token_head * d.n_kv_heads * d.n_layers;
        const int free_now = top[c] < 0 ? 0 : top[c];
        u.pages_in_use[c] = (int64_t)cache->view.n_pages[c] - free_now;
        u.page_bytes_in_use += u.pages_in_use[c] * (int64_t)cache->view.blocks_per_page * class_block_bytes(c) * d.n_kv_heads * d.n_layers;
    }
    u.expected_bits = total > 0 ? sum_bits / (double)total : 0.0;
    u.effective_bits = total > 0 ? (double)u.payload_bytes * 8.0 / ((double)total * d.n_kv_heads * d.n_layers * 2.0 * kD) : 0.0;
    *usage = u;
    delete[] counts;
    return KVQ_OK;
}

extern "C" int kvq_cache_export(const kvq_cache *cache, int32_t layer, int32_t seq, uint8_t *bits_out, uint8_t *codes_out,
                                uint16_t *meta_out, int64_t max_tokens, void *stream)
{
    if (!cache || !bits_out || !codes_out || !meta_out) { set_error("NULL argument"); return KVQ_ERR_INVALID_ARG; }
    if (layer < 0 || layer >= cache->desc.n_layers) { set_error("layer %d out of range", layer); return KVQ_ERR_INVALID_ARG; }
    if (seq < 0 || seq >= cache->desc.max_seqs) { set_error("seq %d out of range", seq); return KVQ_ERR_INVALID_ARG; }
    if (max_tokens < 0) { set_error("max_tokens negative"); return KVQ_ERR_INVALID_ARG; }
    if (max_tokens == 0) return KVQ_OK;
    const int64_t cap = max_tokens < cache->desc.max_context ? max_tokens : cache->desc.max_context;
    const long long waves = (long long)cap * cache->desc.n_kv_heads;
    const unsigned grid = (unsigned)((waves + 3) / 4);
    hipLaunchKernelGGL(k_export, dim3(grid), dim3(256), 0, (hipStream_t)stream, cache->view, layer, seq, bits_out,
                       codes_out, meta_out, (long long)max_tokens);
    KVQ_HIP(hipGetLastError());
    return KVQ_OK;
}

extern "C" int kvq_cache_import(kvq_cache *cache, int32_t layer, int32_t seq, const uint8_t *bits, const uint8_t *codes,
                                const uint16_t *meta, int64_t n_tokens, void *stream)
{
    if (!cache || !codes || !meta) { set_error("cache, codes or meta is NULL"); return KVQ_ERR_INVALID_ARG; }
    const kvq_cache_desc &d = cache->desc;
    if (layer < 0 || layer >= d.n_layers) { set_error("layer %d out of range", layer); return KVQ_ERR_INVALID_ARG; }
    if (seq < 0 || seq >= d.max_seqs) { set_error("seq %d out of range", seq); return KVQ_ERR_INVALID_ARG; }
    if (n_tokens < 0) { set_error("n_tokens negative"); return KVQ_ERR_INVALID_ARG; }
    if (n_tokens > d.max_context) { set_error("n_tokens %lld exceeds max_context", (long long)n_tokens); return KVQ_ERR_CAPACITY; }
    if (layer == 0 && !bits) { set_error("bits is NULL on the bookkeeping call (layer 0)"); return KVQ_ERR_INVALID_ARG; }
    if (n_tokens == 0) return KVQ_OK;
    hipStream_t st = (hipStream_t)stream;
    if (layer == 0) {
        int waves = (int)((n_tokens + 63) / 64);
        if (waves > kAdvanceMaxWaves) waves = kAdvanceMaxWaves;
        hipLaunchKernelGGL(k_advance, dim3(1), dim3(64 * waves), 0, st, cache->view, bits, (const int32_t *)nullptr, seq, 1, (int)n_tokens);
        KVQ_HIP(hipGetLastError());
        cache->len_bound += n_tokens;
        if (cache->len_bound > d.max_context) cache->len_bound = d.max_context;
        cache->touched = true;
    }
    const long long waves = (long long)n_tokens * d.n_kv_heads;
    hipLaunchKernelGGL(k_import, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, st, cache->view, layer, seq, codes, meta,
                       (long long)n_tokens);
    KVQ_HIP(hipGetLastError());
    return KVQ_OK;
}

extern "C" int kvq_cache_set_k_channel_quant(kvq_cache *cache, const void *kmin, const void *krange, void *stream)
{
    if (!cache) { set_error("cache is NULL"); return KVQ_ERR_INVALID_ARG; }
    if ((kmin == nullptr) != (krange == nullptr)) { set_error("kmin and krange must both be given or both be NULL"); return KVQ_ERR_INVALID_ARG; }
    if (cache->touched) { set_error("the key quantizer can only be chosen while the cache is empty (create or reset it first)"); return KVQ_ERR_INVALID_ARG; }
    if (!kmin) { cache->view.k_channel = 0; return KVQ_OK; }
    const long long n = (long long)cache->desc.n_layers * cache->desc.n_kv_heads * kD;
    hipLaunchKernelGGL(k_set_kch, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, cache->view,
                       (const __half *)kmin, (const __half *)krange, n);
    KVQ_HIP(hipGetLastError());
    cache->view.k_channel = 1;
    return KVQ_OK;
}

// launches the bookkeeping kernel for T new tokens per listed sequence (internal; arguments already validated)
int kvq_append_bookkeeping(kvq_cache *cache, const uint8_t *bits, const int32_t *seq_ids, int n_seq, int T, void *stream)
{
    int waves = (T + 63) / 64;
    if (waves > kAdvanceMaxWaves) waves = kAdvanceMaxWaves;
    hipLaunchKernelGGL(k_advance, dim3(n_seq), dim3(64 * waves), 0, (hipStream_t)stream, cache->view, bits, seq_ids, 0, n_seq, T);
    KVQ_HIP(hipGetLastError());
    cache->len_bound += T;
    if (cache->len_bound > cache->desc.max_context) cache->len_bound = cache->desc.max_context;
    cache->touched = true;
    return KVQ_OK;
}

extern "C" int kvq_append(kvq_cache *cache, int32_t layer, const void *k, const void *v, const uint8_t *bits,
                          const int32_t *seq_ids, int32_t n_seq, int32_t T, void *stream)
{
    if (!cache || !k || !v) { set_error("cache, k or v is NULL"); return KVQ_ERR_INVALID_ARG; }
    const kvq_cache_desc &d = cache->desc;
    if (layer < -1 || layer >= d.n_layers) { set_error("layer %d out of range", layer); return KVQ_ERR_INVALID_ARG; }
    if (n_seq < 0 || n_seq > d.max_seqs) { set_error("n_seq %d out of range (max_seqs %d)", n_seq, d.max_seqs); return KVQ_ERR_INVALID_ARG; }
    if (T < 0) { set_error("T negative"); return KVQ_ERR_INVALID_ARG; }
    if ((int64_t)T > d.max_context) { set_error("T %d exceeds max_context", T); return KVQ_ERR_CAPACITY; }
    const bool bookkeeping = layer <= 0 && bits != nullptr;       // bits == NULL: done by kvq_features_controller
    if (n_seq == 0 || T == 0) return KVQ_OK;
    const long long nl = layer < 0 ? d.n_layers : 1;
    const long long total = nl * n_seq * (long long)T * d.n_kv_heads;
    if ((total + 3) / 4 > 0x7fffffffLL) { set_error("append too large for one launch"); return KVQ_ERR_CAPACITY; }
    hipStream_t st = (hipStream_t)stream;
    if (bookkeeping) {
        const int rc = kvq_append_bookkeeping(cache, bits, seq_ids, n_seq, T, stream);
        if (rc != KVQ_OK) return rc;
    }
    // many tokens per sequence: the lane-per-token kernel (needs 16-byte aligned vectors); else a wave per vector
    const Tuning &tn = tuning();
    if (T >= tn.append_bulk_min_T && (((uintptr_t)k | (uintptr_t)v) & 15) == 0) {
        const int tiles = (T + kBlockTokens - 1) / kBlockTokens;
        const long long waves = nl * n_seq * (long long)tiles * d.n_kv_heads;
        const int stream_min = tn.append_stream_min;
        // long prompts go block by block of the cache; below about 512 tokens per sequence the tile kernel's shorter
        // chain of dependent reads wins (measured at 32 sequences: 256 tokens 31 against 37 us, 512 tokens 53 against 48)
        const int block_min_T = tn.append_block_min_T;
        const int items = tiles + 7;                               // upper bound of the blocks one sequence's call touches
        const long long pairs = nl * n_seq, gx = ((long long)items * d.n_kv_heads + kBlkWaves - 1) / kBlkWaves;
        if (T >= block_min_T && gx * pairs <= (1LL << 24)) {       // (a launch beyond that size goes tile by tile)
            const dim3 grid((unsigned)gx, (unsigned)(pairs < kGridY ? pairs : kGridY), (unsigned)((pairs + kGridY - 1) / kGridY));
            if (cache->view.k_channel)
                hipLaunchKernelGGL(k_append_blocks<true>, grid, dim3(64 * kBlkWaves), 0, st, cache->view, layer,
                                   (const __half *)k, (const __half *)v, seq_ids, n_seq, (int)pairs, T, items, stream_min);
            else
                hipLaunchKernelGGL(k_append_blocks<false>, grid, dim3(64 * kBlkWaves), 0, st, cache->view, layer,
                                   (const __half *)k, (const __half *)v, seq_ids, n_seq, (int)pairs, T, items, stream_min);
        } else if (cache->view.k_channel)
            hipLaunchKernelGGL(k_append_bulk<true>, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, st, cache->view, layer,
                               (const __half *)k, (const __half *)v, seq_ids, n_seq, T, tiles, waves, stream_min);
        else
            hipLaunchKernelGGL(k_append_bulk<false>, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, st, cache->view, layer,
                               (const __half *)k, (const __half *)v, seq_ids, n_seq, T, tiles, waves, stream_min);
    } else {
        hipLaunchKernelGGL(k_append_write, dim3((unsigned)((total + 3) / 4)), dim3(256), 0, st, cache->view, layer,
                           (const __half *)k, (const __half *)v, seq_ids, n_seq, T, total);
    }
    KVQ_HIP(hipGetLastError());
    return KVQ_OK;
}

// Q_b of one 64-element fp16 vector held one element per lane (paper Sec. 3.7; the scheme is the reading stated in
// include/kvq.h), shared by the append kernel and by the fused append + attention kernel.
#pragma once

#include <hip/hip_fp16.h>

#include "kvq_internal.h"

namespace kvq {

// Cross-lane steps as data-parallel-primitive moves (no LDS permutes, which cost a round trip each): quad_perm
// [1,0,3,2] and [2,3,0,1] pair a lane with lane ^ 1 and lane ^ 2; once the quads are uniform, row_half_mirror brings in
// the other quad of an 8-lane group and row_mirror the other half of a 16-lane row.  All lanes must be active.
template <int CTRL> __device__ __forceinline__ uint32_t dpp_u32(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}
template <int CTRL> __device__ __forceinline__ float dpp_f32(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float row_of(float v, int lane)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

__device__ __forceinline__ float wave_min_all(float x)
{
    x = fminf(x, dpp_f32<0xB1>(x));
    x = fminf(x, dpp_f32<0x4E>(x));
    x = fminf(x, dpp_f32<0x141>(x));
    x = fminf(x, dpp_f32<0x140>(x));            // every lane of a row holds the row's minimum
    return fminf(fminf(row_of(x, 0), row_of(x, 16)), fminf(row_of(x, 32), row_of(x, 48)));
}
__device__ __forceinline__ float wave_max_all(float x)
{
    x = fmaxf(x, dpp_f32<0xB1>(x));
    x = fmaxf(x, dpp_f32<0x4E>(x));
    x = fmaxf(x, dpp_f32<0x141>(x));
    x = fmaxf(x, dpp_f32<0x140>(x));
    return fmaxf(fmaxf(row_of(x, 0), row_of(x, 16)), fmaxf(row_of(x, 32), row_of(x, 48)));
}

// OR of `word` over the aligned group of `per` lanes (per = 2, 4, 8 or 16; wave-uniform)
__device__ __forceinline__ uint32_t group_or(uint32_t word, int per)
{
    word |= dpp_u32<0xB1>(word);
    if (per >= 4) word |= dpp_u32<0x4E>(word);
    if (per >= 8) word |= dpp_u32<0x141>(word);
    if (per >= 16) word |= dpp_u32<0x140>(word);
    return word;
}

// Q_b of one 64-vector held one element per lane, written into its block.  Every lane passes the same
// uniform arguments.  `codes` points at the K or V code region of the block, `meta` at the token's
// (scale, min) pair for this tensor (nullptr for FP16).
//
// Returns the lane's dequantized element min + code*scale (exact product, one fp32 rounding on the sum), so that a
// caller can use the token in registers exactly as a later read of the cache would see it.  With store == false
// nothing is written.
__device__ __forceinline__ float quantize_store(__half xh, int b, int lane, int tok, uint8_t *codes, __half *meta, bool store = true)
{
    uint32_t word;
    int per;
    float deq;
    if (b == 16) {
        per = 2;
        word = (uint32_t)__half_as_ushort(xh) << (16 * (lane & 1));
        deq = __half2float(xh);
    } else {
        const float x = __half2float(xh);
        float mn = wave_min_all(x);
        float mx = wave_max_all(x);
        if (mn == 0.0f) mn = 0.0f;                                  // a zero minimum of either sign is stored as +0
        if (mx == 0.0f) mx = 0.0f;                                  // and a zero maximum counts as +0: zeros have range +0
        const float levels = (float)((1 << b) - 1);
        const float range = mx - mn;
        const float scale32 = range / levels;                      // IEEE binary32 division
        const __half sh = __float2half_rn(scale32);                // RNE, subnormals kept
        const float s = __half2float(sh);
        float code = 0.0f;
        if (s != 0.0f) {
            code = rintf((x - mn) / s);                            // IEEE division, ties to even
            code = fminf(fmaxf(code, 0.0f), levels);
        }
        per = 32 / b;
        const int r = lane % per;
        word = (uint32_t)code << (b * (r >> 1) + 16 * (r & 1));
        deq = fmaf(code, s, mn);
        if (store && lane == 0) {
            meta[0] = sh;
            meta[1] = __float2half_rn(mn);                         // exact: mn is an fp16 value
        }
    }
    word = group_or(word, per);
    if (store && lane % per == 0) {
        const int w = lane / per;
        *(uint32_t *)(codes + (size_t)(w >> 2) * (kBlockTokens * 16) + tok * 16 + (w & 3) * 4) = word;
    }
    return deq;
}

// Static per-channel variant for a key vector (lane = channel): the channel's minimum mn and step s are given (fp16
// values as floats), code = clamp(rint((x - mn) / s), 0, levels) in IEEE binary32, code 0 where s == 0; no per-token
// scale or minimum is stored.  Packing and return value as quantize_store.
__device__ __forceinline__ float quantize_store_kch(__half xh, int b, float mn, float s, int lane, int tok, uint8_t *codes, __half *meta,
                                                    bool store = true)
{
    // the token's own (scale, minimum) entry is unused by this variant: it is stored as zero, not left as it was
    if (store && lane == 0) *(uint32_t *)meta = 0u;
    const float levels = (float)((1 << b) - 1);
    float code = 0.0f;
    if (s != 0.0f) {
        code = rintf((__half2float(xh) - mn) / s);                  // IEEE division, ties to even
        code = fminf(fmaxf(code, 0.0f), levels);
    }
    const int per = 32 / b;
    const int r = lane % per;
    const uint32_t word = group_or((uint32_t)code << (b * (r >> 1) + 16 * (r & 1)), per);
    if (store && r == 0) {
        const int w = lane / per;
        *(uint32_t *)(codes + (size_t)(w >> 2) * (kBlockTokens * 16) + tok * 16 + (w & 3) * 4) = word;
    }
    return fmaf(code, s, mn);
}

}  // namespace kvq

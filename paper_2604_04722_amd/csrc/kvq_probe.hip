// Measurement helpers: a streaming read-reduce and a plain copy, used to find the HBM rate a trivial
// kernel attains on the same device and to calibrate hardware byte counters against a known size.
#include "kvq_internal.h"

namespace kvq {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// streaming load: marked non-temporal so that it does not allocate in L2 / Infinity Cache
__device__ __forceinline__ uint4 ld_stream(const uint4 *p)
{
    const u32x4 t = __builtin_nontemporal_load((const u32x4 *)p);
    return make_uint4(t.x, t.y, t.z, t.w);
}

__global__ __launch_bounds__(256) void k_probe_read(const uint4 *src, size_t n16, uint32_t *sink)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    uint32_t acc = 0;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const uint4 a = ld_stream(src + i), b = ld_stream(src + i + stride), c = ld_stream(src + i + 2 * stride), d = ld_stream(src + i + 3 * stride);
        acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    for (; i < n16; i += stride) {
        const uint4 a = ld_stream(src + i);
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    if (acc == 0x9e3779b9u) *sink = acc;          // practically never: keeps the loads alive
}

__global__ __launch_bounds__(256) void k_probe_copy(uint4 *dst, const uint4 *src, size_t n16)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i < n16; i += stride) dst[i] = ld_stream(src + i);
}

}  // namespace kvq

using namespace kvq;

extern "C" int kvq_probe_read(const void *src, size_t bytes, uint32_t *sink, void *stream)
{
    if (!src || !sink || (bytes & 15) || ((uintptr_t)src & 15)) { set_error("bad probe arguments"); return KVQ_ERR_INVALID_ARG; }
    if (bytes == 0) return KVQ_OK;
    const size_t n16 = bytes / 16;
    size_t blocks = (n16 + 256 * 8 - 1) / (256 * 8);
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(k_probe_read, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, (const uint4 *)src, n16, sink);
    KVQ_HIP(hipGetLastError());
    return KVQ_OK;
}

extern "C" int kvq_probe_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (!src || !dst || (bytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) {
        set_error("bad probe arguments");
        return KVQ_ERR_INVALID_ARG;
    }
    if (bytes == 0) return KVQ_OK;
    const size_t n16 = bytes / 16;
    size_t blocks = (n16 + 256 * 4 - 1) / (256 * 4);
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(k_probe_copy, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, (uint4 *)dst, (const uint4 *)src, n16);
    KVQ_HIP(hipGetLastError());
    return KVQ_OK;
}

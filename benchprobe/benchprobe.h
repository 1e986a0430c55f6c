/* libbenchprobe.so: three trivial kernels the benchmark times next to the library's own (not part of the method).
 *
 *   benchprobe_read  streaming read-reduce of `bytes` bytes: the read rate a kernel that does nothing else reaches
 *   benchprobe_copy  plain copy of `bytes` bytes: a transfer of known size to calibrate hardware byte counters against
 *   benchprobe_mix3  dst = a ^ b ^ c over `dst_bytes` bytes, the three sources back to back in src (3 x dst_bytes): the
 *                    rate of a kernel that reads three bytes for every byte it writes, as the prefill append does
 *
 * src, dst: device, 16-byte aligned; bytes: a multiple of 16; sink: device uint32[1] (practically never written);
 * stream: a hipStream_t as void*.  Each only enqueues one kernel.  Return 0 on success, 1 on bad arguments, 2 when the
 * launch failed.
 */
#ifndef BENCHPROBE_H
#define BENCHPROBE_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif
int benchprobe_read(const void *src, size_t bytes, uint32_t *sink, void *stream);
int benchprobe_copy(void *dst, const void *src, size_t bytes, void *stream);
int benchprobe_mix3(void *dst, const void *src, size_t dst_bytes, void *stream);
#ifdef __cplusplus
}
#endif
#endif

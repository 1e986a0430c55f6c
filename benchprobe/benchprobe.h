/* libbenchprobe.so: two trivial kernels the benchmark times next to the library's own (not part of the method).
 *
 *   benchprobe_read  streaming read-reduce of `bytes` bytes: the read rate a kernel that does nothing else reaches
 *   benchprobe_copy  plain copy of `bytes` bytes: a transfer of known size to calibrate hardware byte counters against
 *
 * src, dst: device, 16-byte aligned; bytes: a multiple of 16; sink: device uint32[1] (practically never written);
 * stream: a hipStream_t as void*.  Both only enqueue one kernel.  Return 0 on success, 1 on bad arguments, 2 when the
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
#ifdef __cplusplus
}
#endif
#endif

/*
 * medha_yardstick.h — two measurement yardsticks for the benchmark harness.
 *
 * Not part of the attention path and not in libmedha.so: they live in their own
 * shared library (libmedha_yardstick.so).  They put beside the data-sheet peaks
 * what the device at hand sustains, in the same run, when it does nothing but
 * bf16 matrix instructions and nothing but stream HBM into LDS: the clock under
 * load, and with it the attainable rate, differs from part to part.
 *
 * Both calls enqueue one kernel on `hip_stream` (a hipStream_t as void*), allocate
 * nothing and never synchronise.  Return 0, or -1 for null / misaligned /
 * non-positive arguments, -3 for a sink that is too small, -4 for a failed launch.
 */
#ifndef MEDHA_YARDSTICK_H_
#define MEDHA_YARDSTICK_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * `blocks` workgroups of 512 threads (two wavefronts per SIMD, as in the prefill
 * kernel); every wavefront chains `iters` rounds of 4 independent 32x32x16 bf16
 * matrix instructions on operands taken from `operands` (device, 16-byte aligned,
 * at least 5120 bytes of bf16 values of the caller's choice: switching power, and
 * with it the clock, depends on the data).  Work done:
 * blocks * 8 * iters * 4 * 32768 flop.  `sink` (device, at least blocks * 512
 * floats) receives checksums.
 */
int medha_yardstick_mfma_bf16(const void* operands, size_t operand_bytes, int32_t blocks,
                              int32_t iters, float* sink, size_t sink_floats, void* hip_stream);

/*
 * Streams `bytes` (a multiple of 65536) from `src` (device, 16-byte aligned) once,
 * HBM -> LDS with asynchronous 16-byte-per-lane loads, the way the key-split
 * attention kernel moves its K/V blocks but with no arithmetic at all: `blocks`
 * workgroups of 4 wavefronts, each wavefront with a private ring of two 16 KiB
 * stages, i.e. up to 128 KiB in flight per compute unit; consecutive 16 KiB
 * pieces go to consecutive wavefronts of the grid.  One dword per lane of every
 * piece is read back from LDS and folded into `sink` (device, at least
 * blocks * 256 uint32) so that every piece must have landed.
 */
int medha_yardstick_stream_lds(const void* src, size_t bytes, int32_t blocks, uint32_t* sink,
                               size_t sink_words, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MEDHA_YARDSTICK_H_ */

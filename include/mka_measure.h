/*
 * mka_measure.h - measurement helpers.  NOT part of the method and NOT part of libmka.so: three
 * micro-benchmarks, built into their own library (libmka_measure.so), that bench.py runs beside
 * the attention kernels so that every roofline line can be quoted against what this part
 * sustains in the same run as well as against the vendor peak.  Nothing in the product path
 * calls them.
 *
 * mka_measure_mfma_loop: `workgroups` x 8 waves each issue 4 * iters independent 32x32x16 bf16
 *   MFMAs (no memory traffic); `out` (device, workgroups * 512 floats) receives a checksum;
 *   *flops (host, nullable) the number of floating-point operations of the launch.
 * mka_measure_mfma_loop_data: the same loop (32 * iters MFMAs per wave) on operands that change
 *   from MFMA to MFMA: `frags` (device, 16-byte aligned, MKA_MEASURE_FRAG_BYTES bytes of bf16
 *   that the caller fills with the value distribution of its workload) supplies eight A and
 *   eight B fragments per lane.  The clock under matrix load is set by the board's power limit,
 *   and the power of an MFMA depends on its operand bits: this is the matrix pipe alone on
 *   realistic data.
 * mka_measure_stream_read: reads `bytes` (device, 16-byte aligned, at least 1 MiB) exactly once
 *   as six interleaved streams with 16-byte non-temporal loads, 24 loads per lane in flight -
 *   the access pattern of the decode kernel without its arithmetic; `out` (device, nullable) is
 *   only written in the practically impossible case that the xor of all words equals a magic
 *   constant.  A reference, not a bound: a kernel can sit a few per cent above it.
 * Both enqueue on `stream` (a hipStream_t) and return; the caller times them.  Return value: 0
 * on success, 2 for non-positive sizes or null buffers, 4 for a misaligned buffer, 7 if the
 * launch was refused (the numbering of mka_status in mka.h).
 */
#ifndef MKA_MEASURE_H_
#define MKA_MEASURE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

int32_t mka_measure_mfma_loop(float* out, int32_t workgroups, int32_t iters, double* flops,
                              void* stream);
#define MKA_MEASURE_FRAG_BYTES (16u * 512u * 16u)
int32_t mka_measure_mfma_loop_data(float* out, const void* frags, int32_t workgroups,
                                   int32_t iters, double* flops, void* stream);
int32_t mka_measure_stream_read(const void* src, size_t bytes, uint32_t* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MKA_MEASURE_H_ */

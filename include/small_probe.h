/*
 * small_probe.h -- C ABI of libsmall_probe: a measurement aid for the benchmark, NOT part of the layer library
 * (include/small.h, libsmall_hip). It measures the fp32 matrix rate the chip sustains, so that roofline fractions can
 * be quoted against a measured peak next to the published one, and what vector instructions cost beside it.
 */
#ifndef SMALL_PROBE_H
#define SMALL_PROBE_H

#ifdef __cplusplus
extern "C" {
#endif

/* Launches `workgroups` x 4 wavefronts on `stream` (a hipStream_t passed as void*; NULL: the default stream), each
 * running `iters` rounds of eight independent 16x16x4 fp32 matrix instructions on registers (2048 flop per
 * instruction and wavefront: workgroups * 4 * iters * 8 * 2048 flop in all). out: DEVICE pointer owned by the caller,
 * receives workgroups * 256 floats (checksums). Returns 0, 1 (out is NULL), 2 (workgroups outside 1 .. 2^20 or
 * iters < 1) or 5 (the launch failed); nothing is enqueued on an error. */
int small_probe_mfma(float *out, int workgroups, int iters, void *stream);

/* The same with vector-ALU work beside the matrix instructions: every wavefront runs `iters` rounds of `valu` (0, 32,
 * 64 or 96) independent fp32 multiply-adds on registers followed by sixteen 16x16x4 fp32 matrix instructions on four
 * accumulators. The time a round takes beyond valu = 0 is what vector instructions cost next to the matrix pipe.
 * out as above (a lane's checksum: its sixteen accumulator values plus valu * iters * a * b, with the operands a, b of
 * small_probe_mfma). Returns 0, 1 (out is NULL), 2 (workgroups or iters out of range, valu not one of the four) or 5. */
int small_probe_mfma_valu(float *out, int workgroups, int iters, int valu, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SMALL_PROBE_H */

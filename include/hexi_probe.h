/*
 * hexi_probe.h -- measurement aid of the benchmark, in its own library (libhexi_probe.so); not part of the
 * attention library's interface.
 */
#ifndef HEXI_PROBE_H
#define HEXI_PROBE_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

/*
 * A register-only loop of v_mfma_f32_32x32x16_bf16 on the whole chip (256 workgroups x 8 wavefronts x 4 x iters
 * MFMAs of 32768 flop), for the MFMA rate the part sustains on given operand bits (the shader clock is
 * power-limited and depends on them): the measured counterpart of the nominal matrix roof that the roofline of
 * the attention kernels (App. A.4, Eq. 11: the ring step's compute term) is quoted against.  operands: DEVICE,
 * 65536 bytes of bf16 values, 16-byte aligned; sink: DEVICE float[256 * 512], overwritten.  Enqueued on
 * hip_stream (a hipStream_t; NULL = the default stream); the caller times it.  Returns 0, or -1 (null pointer,
 * iters < 1), -3 (operands misaligned), -5 (launch refused).
 */
int hexi_mfma_probe(const void* operands, float* sink, int32_t iters, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* HEXI_PROBE_H */

/*
 * s4c_probe.h -- measurement probes of the benchmark (libs4c_probe.so).  No part of the
 * verification step and no part of libs4c: they give the benchmark the streaming-read rate and the
 * dense bf16 matrix-core rate that plain kernels reach on the GPU at hand, next to the published
 * peaks the rooflines are priced against.  The caller times them with events.
 *
 * Return value: 0 ok, -1 null pointer, -2 bad size or alignment, -5 launch failure.
 *   s4c_probe_stream_read  reads `bytes` (>= 16, buffer 16-byte aligned, device) once with 16-byte
 *                          loads from 4096 workgroups; sink: one device float (left alone).
 *   s4c_probe_mfma_bf16    256 workgroups x 8 wavefronts x iters x 32 matrix-core instructions
 *                          (shape 0: v_mfma_f32_32x32x16_bf16, shape 1: v_mfma_f32_16x16x32_bf16
 *                          with twice the instructions, same FLOP count) on register operands that
 *                          are one constant (random_operands = 0) or drawn from an approximate
 *                          standard normal (1) -- the rate depends on the data, because the clock
 *                          follows the multipliers' switching power.
 *                          sink: >= s4c_probe_mfma_sink_bytes() device bytes (overwritten);
 *                          *flops (host, nullable) receives the FLOP count of the launch.
 */
#ifndef S4C_PROBE_H
#define S4C_PROBE_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif
int s4c_probe_stream_read(const void* buffer, size_t bytes, float* sink, void* hip_stream);
size_t s4c_probe_mfma_sink_bytes(void);
int s4c_probe_mfma_bf16(int32_t random_operands, int32_t shape, int32_t iters, float* sink, double* flops,
                        void* hip_stream);
#ifdef __cplusplus
}
#endif
#endif

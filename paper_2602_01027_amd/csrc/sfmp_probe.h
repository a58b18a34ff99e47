/*
 * sfmp_probe.h - measurement aid of the benchmark, NOT part of the product library (libsfmp.so neither exports nor
 * needs it).  Built into its own shared object, libsfmp_probe.so.
 *
 * sfmp_probe_stream_read reads `bytes` (a multiple of 16, at least 16) from src_dev (device, 16-byte aligned) once
 * with plain streaming loads (256 workgroups of 16 wavefronts, the launch shape of the decode kernels; every wavefront
 * reads whole 1 KiB pieces, four independent 16-byte loads in flight per lane; no LDS, no barrier) and writes 2048 bytes of check words to out_dev (device, 4-byte aligned), so that a bench can time it and
 * print the streaming-read bandwidth this machine reaches beside the data-sheet figure.  Asynchronous on hip_stream
 * (a hipStream_t passed as void*).  Returns 0, -1 (NULL pointer), -2 (size / alignment) or -6 (launch failed).
 *
 * sfmp_probe_mfma_dot issues `count` independent v_mfma_f32_16x16x32_f16 instructions, one per workgroup: dot product
 * number t has A row 0 = a_dev[32 t .. 32 t + 31] and B column 0 = b_dev[32 t .. 32 t + 31] (fp16, device), every other
 * operand element and the accumulator zero, and out_dev[t] (fp32, device) receives result element (0, 0).  The tests
 * use it to pin what the error bound of the decode kernels assumes about this instruction (how products are aligned
 * before they are added when an operand is an fp16 denormal).  Same return values.
 */
#ifndef SFMP_PROBE_H
#define SFMP_PROBE_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif
int sfmp_probe_stream_read(const void* src_dev, int64_t bytes, void* out_dev, void* hip_stream);
int sfmp_probe_mfma_dot(const void* a_dev, const void* b_dev, int32_t count, void* out_dev, void* hip_stream);
#ifdef __cplusplus
}
#endif
#endif

/*
 * sfmp_probe.h - measurement aid of the benchmark, NOT part of the product library (libsfmp.so neither exports nor
 * needs it).  Built into its own shared object, libsfmp_probe.so.
 *
 * sfmp_probe_stream_read reads `bytes` (a multiple of 16, at least 16) from src_dev (device, 16-byte aligned) once
 * with plain streaming loads (256 workgroups of 16 wavefronts, the launch shape of the decode kernels; every wavefront
 * reads whole 1 KiB pieces, four independent 16-byte loads in flight per lane; no LDS, no barrier) and writes 2048 bytes of check words to out_dev (device, 4-byte aligned), so that a bench can time it and
 * print the streaming-read bandwidth this machine reaches beside the data-sheet figure.  Asynchronous on hip_stream
 * (a hipStream_t passed as void*).  Returns 0, -1 (NULL pointer), -2 (size / alignment) or -6 (launch failed).
 */
#ifndef SFMP_PROBE_H
#define SFMP_PROBE_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif
int sfmp_probe_stream_read(const void* src_dev, int64_t bytes, void* out_dev, void* hip_stream);
#ifdef __cplusplus
}
#endif
#endif

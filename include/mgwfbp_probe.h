/*
 * mgwfbp_probe.h - bandwidth probes of libmgwfbp.so.  NOT part of the method and not needed to
 * use the library: the benchmark calls them to calibrate the hardware counters (a plain copy of
 * known size) and to put the data path's rates next to what plain streaming kernels reach on the
 * same box.  They compute nothing the paper defines; each is a single kernel launch on the
 * caller's stream.  All pointers are device pointers, 16-byte aligned; n_elems a multiple of 4.
 * Status codes and mgwfbp_last_error() as in mgwfbp.h.
 *
 *   mgwfbp_probe_copy     dst[i] = src[i], one 16-byte access per lane and workgroup
 *                         (1 read + 1 write stream; the shape pack and unpack use)
 *   mgwfbp_probe_read     reads src[0 .. n_elems) and writes nothing (1 read stream); `sink`
 *                         is a device buffer of at least 16 bytes that is written only if the
 *                         data sums to an impossible value
 *   mgwfbp_probe_fill     dst[i] = value (1 write stream)
 *   mgwfbp_probe_streams  dst[i] = sum_g src[g*stride_elems + i] / n, a compiler-scheduled
 *                         loop (n read + 1 write streams; a baseline for the fused pass, not a
 *                         ceiling); n_streams in {1, 2, 4, 8, 16}, stride_elems >= n_elems
 */
#ifndef MGWFBP_PROBE_H
#define MGWFBP_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

int mgwfbp_probe_copy(const float *src, float *dst, uint64_t n_elems, void *hip_stream);
int mgwfbp_probe_read(const float *src, uint64_t n_elems, float *sink, void *hip_stream);
int mgwfbp_probe_fill(float *dst, float value, uint64_t n_elems, void *hip_stream);
int mgwfbp_probe_streams(const float *src, int32_t n_streams, uint64_t stride_elems,
                         uint64_t n_elems, float *dst, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MGWFBP_PROBE_H */

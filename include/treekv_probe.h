/*
 * treekv_probe.h - three small measurement kernels that price the TreeKV kernels' rooflines on the machine they
 * run on, next to the vendor's figures: a streaming read (what a decode launch's row traffic could reach), a
 * plain copy of known size (the reference the profiler's HBM byte counters are scaled by) and a matrix-pipe
 * issue-rate loop (what the prefill chunk's contractions could reach).  Not part of the method; bench.py calls
 * them for its `measured_peaks`.  Device pointers are caller-owned; calls only enqueue; `stream` is a
 * hipStream_t passed as void*; results are TREEKV_OK or a negative treekv_status (treekv.h).
 */
#ifndef TREEKV_PROBE_H
#define TREEKV_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Reads `bytes` (a multiple of 1 MiB, 16-byte aligned) once with 16-byte non-temporal lane loads -- the decode
 * kernel's load type -- from 512-thread workgroups that take `kib_per_workgroup` KiB each (a power of two, 32 .. 1024;
 * 1024 with 256 MiB is the decode kernel's launch shape) with `loads_in_flight` (2, 4 or 8) loads per thread
 * outstanding.  `sink` [1] float32 receives a value only if the data hashes to a fixed pattern (so the loads cannot
 * be dropped). */
int treekv_probe_read(const void* src, size_t bytes, int kib_per_workgroup, int loads_in_flight, float* sink, void* stream);

/* Copies `bytes` (a multiple of 1 MiB, both 16-byte aligned) with ordinary 16-byte loads and stores: exactly
 * `bytes` read and `bytes` written. */
int treekv_probe_copy(void* dst, const void* src, size_t bytes, void* stream);

/* Issues `iters` x 8 v_mfma_f32_16x16x32_bf16 per wave over 8 independent accumulators from `waves_per_simd`
 * (1 or 2) waves on every SIMD of `workgroups` 256-thread-per-wave-set workgroups; *flops (host, may be NULL)
 * receives the floating-point operations the launch performs (2 * 16 * 16 * 32 per instruction). */
int treekv_probe_mfma(float* sink, int workgroups, int waves_per_simd, int iters, double* flops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TREEKV_PROBE_H */

/*
 * ts_bench.h - measurement helpers exported by libts.so beside the layer's own calls (ts.h).
 *
 * None of these is part of the sparse-convolution path: a plain copy kernel and a register-only MFMA
 * loop (what the machine sustains, next to which the layer kernels are reported), and per-kernel
 * HIP-event timing of the library's own launches.  Benchmarks and profiling scripts use them; a
 * product that only runs layers never needs this header.
 */
#ifndef TS_BENCH_H
#define TS_BENCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Plain device-to-device streaming copy kernel (dst, src: device, 16-byte aligned; bytes a
 * multiple of 16; buffers must not overlap).  Not part of the layer: benchmarks use it as the
 * achievable-bandwidth reference and to calibrate hardware byte counters against a known size.
 */
int ts_copy_bytes(void *dst, const void *src, size_t bytes);
/*
 * Register-only loop of fp16 MFMA instructions on every matrix pipe (1024 workgroups x 4 waves x iters x
 * 8 instructions of 16x16x32): the achievable-MFMA reference of the benchmarks.  sink: device, at least
 * 1 MiB (never written unless the arithmetic misbehaves); *flops (host) receives the FLOPs one call executes.
 */
int ts_mfma_loop(int iters, void *sink, double *flops);

/*
 * Per-kernel timing for benchmarks.  While enabled, the library brackets each kernel launch
 * (or library sort) with a hipEvent pair on its stream; `only`, when not NULL/empty, restricts
 * this to the kernels whose name starts with it.  ts_profile_read synchronises the stream, writes one
 * line per kernel name, "name launches total_ms\n", into buf (host, cap bytes), and clears
 * the records.  Not thread-safe; off by default.
 */
int ts_profile_enable(int on, const char *only);
int ts_profile_read(char *buf, size_t cap);

#ifdef __cplusplus
}
#endif
#endif /* TS_BENCH_H */

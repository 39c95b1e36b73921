/*
 * hs_bench.h -- benchmark and profiling support of libhs: entry points that are not part of the
 * attention path's own calls (hs.h) but let a harness time its pieces.  Same conventions as hs.h.
 */
#ifndef HS_BENCH_H_
#define HS_BENCH_H_

#include "hs.h"

#ifdef __cplusplus
extern "C" {
#endif

/* hs_decode_attn in separable phases, for benchmarking and profiling: `phases` bit 0 launches
 * the split-KV kernel (reads Q and the cache, writes the partials into `workspace`), bit 1
 * launches the merge kernel (reads the partials, writes O and LSE).  phases == 3 is
 * hs_decode_attn; phases == 1 lets a caller time the kernel that streams the cache on its own
 * (back-to-back launches between two events).  Everything else as hs_decode_attn. */
HS_API int hs_decode_attn_phases(const hs_shape* shape, float scale, int32_t n_splits,
                          const void* Q, const hs_kv* kv, void* O, float* LSE,
                          void* workspace, void* stream, int phases);

/* Benchmark support: launches a register-resident loop of matrix instructions (kind 0: the dense
 * 16x16x32 bf16 form, 1: the 2:4 sparse 16x16x64 bf16 form that prefill and decode use) on every
 * compute unit, two waves per SIMD, no memory traffic, so that a caller can time it between two
 * events and set the attention kernels against the rate the matrix pipes reach on the chip at
 * hand, next to the published peak.  *flop [host] receives the dense-equivalent floating-point
 * operations of the launch (the sparse form counts the multiplications its dense equivalent
 * would do).  sink: 32 device bytes, 8-byte aligned; the first two int64 receive the shader
 * clocks and the constant-rate 100 MHz ticks one wave spent in the loop (their ratio is the clock
 * the chip sustained).  Asynchronous on `stream`. */
HS_API int hs_probe_mfma_rate(int kind, int32_t iters, void* sink, double* flop, void* stream);

/* Benchmark support: a load-only kernel with the access pattern of the split-KV decode kernel, so that a
 * caller can time what the memory system gives that pattern at a given size next to the 8 TB/s peak.
 * buf: device, n_tiles * 18432 bytes, 16-byte aligned, read as four pool regions (kept values of K: n_tiles
 * x 8192 B, positions of K: n_tiles x 1024 B, then the same for V); workgroups of 4 waves, wave w of workgroup
 * g reads tiles (n_tiles / n_workgroups) g + w + 4 i with two tiles in flight (non-temporal 16-byte loads);
 * n_tiles must be a multiple of 4 n_workgroups.  with_epilogue != 0 adds a combine through LDS and a 2 KiB
 * store per workgroup (what the decode kernel does with its partials).  sink: device, 64 + 2048 n_workgroups
 * bytes, 16-byte aligned.  Asynchronous on `stream`. */
HS_API int hs_probe_stream_read(const void* buf, int32_t n_tiles, int32_t n_workgroups, int with_epilogue,
                         void* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HS_BENCH_H_ */

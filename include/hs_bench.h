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

#ifdef __cplusplus
}
#endif
#endif /* HS_BENCH_H_ */

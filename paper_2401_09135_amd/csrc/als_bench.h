/*
 * als_bench.h -- measurement and tuning hooks of libals.so.  Internal: used by bench.py and by the
 * kernel tests that sweep tile variants; not part of the library's C ABI (include/als.h), no
 * stability promise.  The hooks are process-wide and not thread-safe.
 */
#ifndef ALS_BENCH_H
#define ALS_BENCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Benchmark hooks.  als_prof_enable(n), n >= 1, makes every n-th MFMA GEMM launch record a HIP
 * event before and after itself on its own stream (a timed launch costs about 20 us of host
 * time and orders the stream around it, so a throughput run samples); 0 switches it off;
 * als_prof_collect waits for the device and returns, per kernel instantiation (id), the number of launches, their summed duration in ms and their
 * summed algorithmic FLOPs (2 M N K), then forgets them.  Returns the number of entries
 * written (<= max_entries) or a negative error.  als_prof_kernel_name writes the kernel's
 * template name for an id. */
int als_prof_enable(int on);
int als_prof_collect(int max_entries, int32_t* ids, int64_t* launches, double* ms, double* flops);
int als_prof_kernel_name(int id, char* out, int out_len);
/* Benchmark hook: force the MFMA GEMM tile to 256x256, 256x128 or 128x128 with nbuf = 2
 * (LDS double buffer) or 1 (single buffer, more workgroups per CU); 0,0,0 = automatic choice
 * by shape.  Process-wide, not thread-safe. */
int als_k_set_gemm_tile(int bm, int bn, int nbuf);

#ifdef __cplusplus
}
#endif
#endif /* ALS_BENCH_H */

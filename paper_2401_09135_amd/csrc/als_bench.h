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
/* Host only (no GPU call): the work-item list of the grouped weight-gradient launch
 * (als_k_gemm_dw_grouped) for n products M[i] x N[i] over K, so that a CPU test can check that it
 * covers every 256 x 256 tile and every 64-wide K slice exactly once and stays inside its tables.
 * items_out: 6 ints per work item in launch order (product, tile row, tile column, partial-tile
 * slot or -1 for a tile written straight to the gradient, first K slice, number of K slices), at
 * most max_items of them; split_out: 5 ints per K-split tile (product, tile row, tile column, first
 * slot, number of slots), at most max_split; counts_out[6]: work items, split tiles, partial-tile
 * slots, the table capacities for items and split tiles, and the number of partial-tile slots the
 * workspace holds.  Errors (ALS_ERR_INVALID): null pointers, unsupported shapes. */
int als_k_gemm_dw_grouped_plan(int n, const int* M, const int* N, int K, int max_items, int32_t* items_out,
                               int max_split, int32_t* split_out, int32_t* counts_out);

#ifdef __cplusplus
}
#endif
#endif /* ALS_BENCH_H */

/*
 * tdk_bench.h -- measurement helpers exported by libtdk beside the product calls of tdk.h: per-kernel event
 * timing of the step calls, and plain copy / fill / page-pattern probes that show what HBM delivers for the
 * access patterns of the page kernels.  Nothing here computes any part of the method; a serving stack needs
 * none of it.
 */
#ifndef TDK_BENCH_H
#define TDK_BENCH_H

#include "tdk.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Kernel timing with HIP events on the caller's stream (off by default).  When on, every kernel
 * launch of the step calls is bracketed by two events; tdk_timing_read waits for them. */
#define TDK_KERNEL_REROTATE 0
#define TDK_KERNEL_FLAG     1
#define TDK_KERNEL_COMPACT  2
#define TDK_KERNEL_GATHER   3
#define TDK_KERNEL_DECODE   4
#define TDK_KERNEL_SCATTER  5
#define TDK_KERNEL_KEYDIFF  6
#define TDK_KERNEL_SELECT   7
#define TDK_KERNEL_MASTER   8
#define TDK_KERNEL_ATTEND_QROT   9
#define TDK_KERNEL_ATTEND_MASTER 10   /* also the launch that holds the master and the listed-pages pass together */
#define TDK_KERNEL_ATTEND_DIFF   11   /* (no launches of its own when that shared launch is used)                  */
#define TDK_KERNEL_ATTEND_MERGE  12
#define TDK_KERNEL_KINDS    13
tdk_status tdk_timing_enable(tdk_round* r, int32_t on);
tdk_status tdk_timing_read(tdk_round* r, int32_t kernel, double* total_ms, int64_t* launches);
tdk_status tdk_timing_reset(tdk_round* r);
const char* tdk_kernel_name(int32_t kernel);   /* device symbol name prefix, for profiler output */

/* Plain device copy / fill of `bytes` (multiple of 16) with 16-byte accesses: the measured HBM
 * ceiling the step kernels are compared with, and the known-size reference for traffic counters. */
tdk_status tdk_util_copy(void* dst, const void* src, size_t bytes, void* hip_stream);
tdk_status tdk_util_fill(void* dst, uint32_t word, size_t bytes, void* hip_stream);

/* Access-pattern probes: one workgroup per page fills (reads) page_bytes (multiple of 16) at
 * dst + page_ids[i] * page_bytes for i < n_pages; page_ids is DEV.  With a permuted id list this is
 * the page kernels' access pattern with no arithmetic.  The caller guarantees every id is in range.
 * sink16: 16 DEV bytes that are never written in practice (they keep the loads alive). */
tdk_status tdk_util_page_fill(void* dst, const int32_t* page_ids, int32_t n_pages, size_t page_bytes,
                              uint32_t word, void* hip_stream);
tdk_status tdk_util_page_read(const void* src, const int32_t* page_ids, int32_t n_pages, size_t page_bytes,
                              void* sink16, void* hip_stream);

/* The same probes in the access form of the page kernels: a workgroup takes `group` consecutive entries of
 * page_ids (as a work item takes a group of agents); its four wavefronts own interleaved rows of each page; a
 * lane touches the two halves of a head row in plane_k and two chunks 1 KB apart in plane_v (two planes of
 * [pages][page_tokens][num_kv_heads][128] bf16, like pool_k / pool_v); streaming stores (sc0 sc1 nt) /
 * non-temporal loads; every access of a wavefront's rows of one page is issued before any is waited for. */
tdk_status tdk_util_page_fill_product(void* plane_k, void* plane_v, const int32_t* page_ids, int32_t n_pages, int32_t group,
                                      int32_t num_kv_heads, int32_t page_tokens, uint32_t word, void* hip_stream);
tdk_status tdk_util_page_read_product(const void* plane_k, const void* plane_v, const int32_t* page_ids, int32_t n_pages,
                                      int32_t group, int32_t num_kv_heads, int32_t page_tokens, void* sink16, void* hip_stream);

/* Timeline of the page kernels (rerotate, compare, decode): with a stamp buffer set, every work item of their
 * launches gets the device's constant-rate clock (100 MHz; the low four bits replaced by the number of the
 * XCD it runs on) at its start to stamps[4 * id] and raises
 * stamps[4 * id + 1] to the clock at its end (uint64 each, id = number of the work item); rerotate also
 * records when the item's staging was complete (4 * id + 2) and when its first wavefront had issued the rows of
 * the first agent (4 * id + 3).  DEV buffer of
 * at least tdk_timeline_bytes(r) bytes, zeroed by the caller before each launch it wants to look at; NULL
 * switches the stamps off again.  Takes effect for launches enqueued after the call. */
size_t     tdk_timeline_bytes(const tdk_round* r);
tdk_status tdk_timeline_set(tdk_round* r, void* stamps, size_t bytes);

#ifdef __cplusplus
}
#endif
#endif

/*
 * prism_kv_tuning.h — measurement, tuning and test hooks of libprismkv.so.
 *
 * Nothing here is needed to serve: the calls of prism_kv.h run with the defaults these
 * knobs start at.  They exist so that benchmarks can time single kernels, sweeps can move
 * the work split of the decode kernel, and tests can force the rare paths.  All of them set
 * process-wide state that every later launch sees; restore the defaults (the values named
 * below) when done.  Return values follow prism_kv.h.
 */
#ifndef PRISM_KV_TUNING_H
#define PRISM_KV_TUNING_H
#include "prism_kv.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Per-kernel timing for measurements: with every = n > 0, every n-th decode_attention*
 * call brackets its attention kernel with HIP events on the library's stream (at most
 * 8192 calls are recorded); 0 switches it off.  pkv_timing_read waits for the stream,
 * returns the number of recorded calls and the summed kernel time in milliseconds, and
 * clears the record. */
int pkv_timing_enable(int every);
long pkv_timing_read(double *attention_ms);
/* Measured ceilings for comparison: reads a freshly allocated buffer of `bytes` bytes
 * (a power of two) `iters` times with a kernel that does no arithmetic and reports
 * the read bandwidth in GB/s.  granule_bytes = 0: plain streaming read; otherwise a
 * power of two >= 1024: whole granules of that size are read in a scrambled order,
 * the access pattern of paged KV tiles.  Allocates and frees its buffer; synchronises. */
int pkv_stream_read_probe(size_t bytes, size_t granule_bytes, int iters, double *gbps);
/* Measurement / test knobs of the attention work split: `items` = work items (waves)
 * per launch, `min_share` = smallest number of pages a wave may be given; 0 selects
 * the automatic value of either (items: what the chip holds at once; min_share: an
 * eighth of a mean row, within 4..16 pages). */
int pkv_set_split(int items, int min_share);
/* What a (sequence, kv head) segment is taken to cost besides its pages when the pages
 * are cut into shares, in pages (0..256; -1 = the default).  A wave whose share holds
 * many short sequences then gets fewer pages than one inside a long sequence. */
int pkv_set_segment_cost(int pages);
/* Which form of the decode kernel a launch uses: 0 = two waves per SIMD (2048 work items),
 * 1 = one wave per SIMD, one page pair in flight per wave, and only as many work items as keep
 * the memory system busy (512, 768 or 1024, by the page sizes and cache types of the launch),
 * -1 = the library decides by the launch: form 1 unless the launch is small (fewer than 10 240
 * page units) or its pages are so small that 1024 such waves could not saturate the memory
 * (e4m3 caches with 64-wide heads). */
int pkv_set_kernel_form(int form);
/* The form (0 or 1) of the most recent decode attention launch of this process. */
int pkv_last_kernel_form(void);
/* The work items (waves) of that launch, all its models together. */
int pkv_last_launch_items(void);
/* Cost model that shares the waves out among the models of a grouped launch: a page
 * costs per_mille/1000 + 0.1 per KiB of its K and V tile (-1 = the default: 800 in kernel
 * form 0, 1600 for bf16 pages in form 1). */
int pkv_set_page_cost(int per_mille);
/* The eight XCDs of the chip do not get the same memory bandwidth, and work-groups are
 * dealt to them in turn; so each block of eight consecutive attention work items is
 * cut in proportion to eight weights rather than evenly.  The library finds the weights
 * by itself: the first launches of a process that fill the chip (256 work items or more)
 * also record how long each XCD's waves streamed, the sums travel to the host behind the
 * launch, and a later launch that finds them there moves the weights toward equal times
 * (24 updates, the first 8 coarse; nothing ever waits, and launches under stream capture
 * are left alone).  After those, every eighth such launch is still measured and moves the
 * weights by a tenth of the way, so that they follow the load (what the XCDs differ by
 * depends on it).  pkv_tune_xcd(n) restarts all that with n quick updates (0 = stop: the
 * weights stay as they are).  pkv_set_xcd_weights sets them by hand and stops the tuning
 * (w: 8 positive floats, host memory, copied; NULL = all equal; they are scaled to mean 1
 * and clamped to [0.75, 1.25]); pkv_get_xcd_weights copies the current ones to w[8].  Weights change where
 * the split-K boundaries fall, hence the rounding of the results (by about 1e-6
 * relative), not what is computed.  PKV_E_ARG on a bad argument. */
int pkv_set_xcd_weights(const float *w);
int pkv_get_xcd_weights(float *w);
int pkv_tune_xcd(int updates);
/* Host-side check of the multiply-shift division the kernels use to split a block
 * id into (frame, slot): returns n / d computed that way. */
uint32_t pkv_debug_fastdiv(uint32_t n, uint32_t d);
/* Test hook for the out-of-memory path of elastic pools: after `after` more successful frame
 * mappings the next one is refused as if the driver had no memory left, once (-1 = never). */
int pkv_debug_fail_frame_map(int after);

#ifdef __cplusplus
}
#endif
#endif

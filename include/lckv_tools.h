/*
 * lckv_tools.h - measurement and tuning hooks of liblckv (see lckv.h for the method's calls).  None of these is
 * part of the decode path: they time its kernels, probe the device, or override a choice the library makes on
 * its own.  Same conventions as lckv.h.
 */
#ifndef LCKV_TOOLS_H
#define LCKV_TOOLS_H

#include "lckv.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Force the number of keys per split (a multiple of 16; 0 = choose from B, Hkv and max_len_hint).  The split
 * of a sequence's keys never depends on other sequences' lengths.  Host only; meant for tests and tuning. */
int lckv_set_split_tokens(lckv_cache *cache, int32_t tokens);

/* Force the width of the bf16 decode-attention workgroups: 4, 8 or 16 waves (16 only at D = 64; a larger request
 * is cut to what D allows), 0 = the planner's choice.  By default a plan of two splits becomes one workgroup of 8
 * waves and, at D = 64, a plan of three or four splits one of 16 waves: its waves are merged through LDS and no
 * split partials go through memory.  With a forced width the number of splits stays what it would be at width 4
 * (or what lckv_set_split_tokens asks for).  fp32 caches ignore it.  Host only. */
int lckv_set_workgroup_waves(lckv_cache *cache, int32_t waves);

/* How the attention kernels read K/V: AUTO uses the nontemporal hint when one layer's pass over its slot is
 * larger than the 256 MB last-level cache (nothing of it would survive until the next layer's pass), plain loads
 * otherwise (a small shared slot is re-read by every condensed layer and may stay cached).  Host only. */
#define LCKV_LOAD_AUTO 0
#define LCKV_LOAD_TEMPORAL 1
#define LCKV_LOAD_NONTEMPORAL 2
int lckv_set_load_policy(lckv_cache *cache, int32_t policy);

/* Tuning knob of the bf16 prompt-encoding kernel: 16-position query blocks per wave, 2 or 4 (0 = default).
 * Host only. */
int lckv_set_prefill_tile(lckv_cache *cache, int32_t query_blocks_per_wave);

/* Bound on a wait at the device-wide barrier of lckv_step_one_launch, in milliseconds (default 2000; 0 makes
 * the first workgroup to arrive give up at once - the tests use that to walk the error path: every workgroup
 * leaves the kernel, LCKV_DEV_ERR_BARRIER is raised).  Host only. */
int lckv_set_barrier_wait_ms(lckv_cache *cache, double ms);

/* Kernel timing for benchmarks: while enabled, every attention kernel launch is bracketed by HIP events on
 * its stream (do not enable during graph capture).  lckv_profile_read SYNCHRONISES, returns the number of
 * timed launches and their summed duration since the last read, and resets both. */
int lckv_profile_enable(lckv_cache *cache, int32_t enable);
int lckv_profile_read(lckv_cache *cache, int32_t *n_launches, double *total_ms);
/* The individual durations (milliseconds, launch order) of the launches timed since the last lckv_profile_read:
 * up to `capacity` of them are written to host array `ms`, *n_launches gets their number.  SYNCHRONISES; does not
 * reset (call it before lckv_profile_read). */
int lckv_profile_launch_ms(lckv_cache *cache, float *ms, int32_t capacity, int32_t *n_launches);

/* Measurement aid: read `bytes` (a multiple of 2 MiB is read, the rest ignored) of device memory with the
 * attention kernel's load pattern (with or without the nontemporal hint) and discard them; timing it gives the
 * read bandwidth reachable on the device at hand, to set beside the published peak.  Only enqueues. */
int lckv_hbm_read_probe(lckv_cache *cache, const void *dev_buf, size_t bytes, int32_t nontemporal, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* LCKV_TOOLS_H */

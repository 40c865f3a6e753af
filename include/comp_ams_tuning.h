/*
 * comp_ams_tuning.h - measurement and tuning aids of the library declared in comp_ams.h.
 *
 * Nothing here is needed to use the library, and nothing here changes a result: the setters choose between
 * launch shapes and cache policies that compute the same bits (the defaults are chosen from the sizes), the
 * rest reads timings and selection records or copies memory for calibration.  The benchmark and the tests that
 * check "results never depend on it" are the callers.  Conventions as in comp_ams.h.
 */
#ifndef COMP_AMS_TUNING_H
#define COMP_AMS_TUNING_H

#include "comp_ams.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Cache policy, a tuning aid (no effect on results).  rows: how a step loads the stored rows (error
 * memory / Markov sequences); state: how it loads and stores theta, m, v, vhat.  1 = as a stream
 * (non-temporal: the data is not kept in the caches), 0 = ordinary accesses, -1 = chosen from the
 * sizes (the default: the rows stream when they exceed 224 MB in total, i.e. when they could not
 * stay in the 256 MB memory-side cache until the next step anyway; the state is left cached only
 * if it fits likewise - with CD-Adam the server's two vectors count with it - and, under error
 * feedback, only if the rows stream).  May be called between steps.
 */
int comp_ams_set_streaming(comp_ams_t *h, int32_t rows, int32_t state);

/*
 * Order in which the workgroups of the streaming pass take the 4096-coordinate tiles of a row, a tuning
 * aid (no effect on results).  The chip hands workgroups to its eight XCDs in turn; with chunk > 0
 * every XCD works through `chunk` consecutive tiles of each group of 8 * chunk tiles, with chunk = 0
 * consecutive tiles go to consecutive XCDs, -1 = chosen from the sizes (the default: 16 when the
 * stored rows exceed 1 GiB in total and the method keeps them - error feedback, CD-Adam - except for
 * CD-Adam's Top-k / Rand-k steps on 16-bit gradients; else 0; Top-k / Rand-k under error feedback: 0 while
 * the rows stay in the caches, else 8, or 16 for rows of 64 Mi coordinates or more; the update without
 * compression, which takes its tiles the same way: 16 with at least 16 workers whose gradients exceed 1 GiB
 * in total).  chunk <= 65536.  May be called between steps.
 */
int comp_ams_set_tile_order(comp_ams_t *h, int32_t chunk);

/*
 * Bytes of LDS a workgroup of the streaming pass reserves, a tuning aid (no effect on results): the
 * amount decides how many workgroups share a compute unit (160 KB each), to which the pass responds by a
 * few per cent.  -1 = chosen from the sizes, the method and the gradient type (the default), else
 * 0 .. 61440.  BLOCKSIGN: the pass always gets at least what its block table needs (24 KB when a tile
 * holds several blocks' pieces).  TOPK / RANDK: the amount is added to the 24 KB of candidate staging
 * lists the pass always holds (default under error feedback with 32-bit gradients: 9 KB, or 7000 bytes
 * for rows under 64 Mi coordinates that do not stay in the caches; else none);
 * no effect on vectors of at most 16 tiles.  May be called between steps.
 */
int comp_ams_set_pass_lds(comp_ams_t *h, int32_t bytes);

/*
 * Per-kernel timing for measurement (Section-independent; a benchmark aid).  While enabled, every
 * kernel that comp_ams_step launches carries two HIP events on the step's stream that are stamped
 * with the kernel's own begin and end (hipExtLaunchKernel), so a slot's time is kernel time
 * without the gaps between launches; event creation makes such steps slower and allocate, so
 * keep it off otherwise.
 * Enabling or disabling waits for pending work and discards earlier recordings.
 */
int comp_ams_profile(comp_ams_t *h, int enable);

/*
 * Reads one timing slot (slots are numbered from 0; one per kernel of the library): *name
 * receives a static string, *total_ms the summed event time of all recorded launches,
 * *launches their count; any output pointer may be NULL.  Waits for pending work.  Returns 1 (not
 * an error) when slot is past the last one.
 */
int comp_ams_profile_read(comp_ams_t *h, int32_t slot, const char **name, double *total_ms, int64_t *launches);

/*
 * TOPK handles: how the last step found worker i's threshold, as 8 host words - the fine-bin
 * guess prepared for the next step, the slack (fine bins) behind it, whether the last step's guess
 * was too high (candidates listed twice), the number of magnitude bits left open by the histogram
 * stage, the magnitude prefix, the rank inside it, whether a whole bin was kept, and the fine bin
 * (top 17 magnitude bits) of the threshold.  For diagnosis and tuning; not needed to use the library.
 */
int comp_ams_get_selection_info(comp_ams_t *h, int32_t worker, uint32_t *out_host);

/*
 * Measurement aid, no handle needed: a plain 16-bytes-per-lane copy of `count` floats
 * (a positive multiple of 4, both pointers 16-byte aligned, device memory) dst <- src, enqueued on
 * hip_stream.  Benchmarks use it to calibrate HBM traffic counters and as the copy ceiling.
 */
int comp_ams_probe_copy(float *dst_dev, const float *src_dev, int64_t count, void *hip_stream);

/*
 * Measurement aid, no handle needed: the access pattern of the library's streaming passes with nothing else -
 * x[i][j] = x[i][j] + g[i][j] in place for `rows` rows of d floats each (row-major, d a positive multiple of 4,
 * both pointers 16-byte aligned, device memory), enqueued on hip_stream.  It moves exactly 12 bytes per element;
 * what it reaches is the practical ceiling on this chip for a kernel that reads two arrays and writes one of them
 * back, which benchmarks report next to the passes' own rate.
 */
int comp_ams_probe_update(float *x_dev, const float *g_dev, int64_t rows, int64_t d, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* COMP_AMS_TUNING_H */

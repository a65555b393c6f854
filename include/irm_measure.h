/*
 * irm_measure.h -- measurement aids of libirm (AMD MI355X, gfx950).
 *
 * Not part of the serving contract in irm.h: launch-shape knobs for sweeps, event timing
 * of the row kernels inside a timed loop, and a plain copy of known traffic that scales
 * hardware counters.  A serving engine needs none of these; results never depend on them.
 */
#ifndef IRM_MEASURE_H
#define IRM_MEASURE_H

#include "irm.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Tuning knobs for measurements (launch shapes only; results never change).
 * knob 0: grid.x of the re-attach row kernel = tile slots per layer (0 = one per
 *         possible tile)
 * knob 1: c_KV rows per wave and tile (1, 2, 4, 8 or 16; fp8 rows: not 1)
 * knob 2: bit 0 = non-temporal loads, bit 1 = non-temporal stores
 * knob 3: which tiles an XCD serves in the row kernel: 2 = one contiguous eighth of the launch's whole
 *         (layer, tile) list, 1 = an eighth of every layer's tiles, 0 = tile x to workgroup x
 *         (round-robin), 3 = the library's choice (default: 2 from 32 layers on over bf16 rows, else 1);
 *         the k_r-only kernel and the miss path's copy follow the same values over their own lists
 * knob 4: waves per workgroup (1, 2, 4, 8 or 16; fp8 rows: 4 or more); a tile is
 *         waves x rows-per-wave rows, at least 4
 * knob 5: 1 = irm_cdc_chunk always selects cuts with the serial walk (else only for
 *         requests with more than 4096 candidate positions)
 * knob 6: rows per lane of the k_r-only kernel (2, 4 or 8; its tile is 32 times that)
 * knob 7: layers a workgroup of the k_r-only kernel keeps its tile for (0 = chosen by batch size)
 * knob 8: polls one in-kernel wait of irm_attend_ref may take before the wave gives up and raises
 *         IRM_FLAG_WAIT_TIMEOUT (default 2^18; 0 makes every wait that is not met at once give up:
 *         for tests of that path, the results of such a call are not to be used) */
irm_status irm_ctx_tune(irm_ctx *ctx, uint32_t knob, uint32_t value);

/* Kernel timing for measurements.  irm_ctx_profile_begin creates max_samples
 * pairs of HIP events; while enabled, every `every`-th irm_reattach,
 * irm_reattach_kr, irm_reattach_ref or irm_attend_ref (the first one included)
 * records one pair around its row kernel(s) on the caller's stream (calls past
 * max_samples are not sampled).  irm_ctx_profile_end waits for the stream, returns the summed
 * elapsed milliseconds and the number of samples, destroys the events and
 * disables sampling.  Not for use under graph capture. */
irm_status irm_ctx_profile_begin(irm_ctx *ctx, uint32_t max_samples, uint32_t every);
irm_status irm_ctx_profile_end(irm_ctx *ctx, void *stream, float *total_ms, uint32_t *n_samples);

/* Measurement aid: a plain copy of `bytes` (multiple of 16) from d_src to d_dst
 * with 16-byte accesses, `grid` workgroups of 256 lanes (0 = default).  Its HBM
 * traffic is known exactly (bytes read + bytes written), which calibrates
 * hardware counters and gives the copy bandwidth the machine can reach. */
irm_status irm_calibrate_copy(void *d_dst, const void *d_src, uint64_t bytes, uint32_t grid, void *stream);

/* Measurement aid: a shaped stream over `bytes` of d_src and/or d_dst.  `grid` workgroups of
 * `lanes` lanes (a multiple of 64, at most 1024) each own a contiguous range and walk it in
 * steps of lanes x vectors_per_lane 16-byte vectors (1, 2, 4, 9, 18 or 36 per lane): all loads
 * of a step are issued before its stores.  IRM_YARDSTICK_COPY reads d_src and writes d_dst
 * (traffic 2 x bytes), IRM_YARDSTICK_READ only reads d_src (the data must not be the one
 * pattern that would make it store; any random fill is fine), IRM_YARDSTICK_WRITE only
 * writes d_dst.  bytes must be a multiple of grid x lanes x vectors_per_lane x 16.  With
 * IRM_YARDSTICK_XCD_RANGES or-ed into the mode (grid a multiple of 8) workgroup x takes range
 * (x % 8) * grid / 8 + x / 8, so that every XCD streams one contiguous eighth, the mapping of
 * the row kernels; without it workgroup x takes range x.  With one step per workgroup (grid =
 * bytes / (lanes x vectors_per_lane x 16)) the stream is dispatched in address order with no
 * loop, the launch shape of the row kernels.  What these reach bounds what a kernel that moves
 * rows can reach. */
#define IRM_YARDSTICK_COPY 0u
#define IRM_YARDSTICK_READ 1u
#define IRM_YARDSTICK_WRITE 2u
#define IRM_YARDSTICK_XCD_RANGES 4u
irm_status irm_yardstick(void *d_dst, const void *d_src, uint64_t bytes, uint32_t mode, uint32_t grid,
                         uint32_t lanes, uint32_t vectors_per_lane, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* IRM_MEASURE_H */

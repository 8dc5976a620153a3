/*
 * adacomp_debug.h -- diagnostics, tuning knobs and kernel timing of libadacomp.
 *
 * NOT part of the stable contract of adacomp.h: these calls exist for the library's own tests and
 * benchmark, may change or disappear, and act on process-wide state.  The flags are read by the
 * compute calls without any ordering against calls in flight on other threads: set them while no
 * compute call runs.  The timing calls are serialised among themselves and with the compute calls
 * by a lock, but they record events on whatever stream the timed call uses, so one timed run at a
 * time gives meaningful numbers.
 */
#ifndef ADACOMP_DEBUG_H
#define ADACOMP_DEBUG_H

#include "adacomp.h"

#ifdef __cplusplus
extern "C" {
#endif

/* The g_max vector (one float per bin, layers in table order, bins in order) is not needed once
 * the layer scale is known, so compress does not store it unless adacomp_debug_keep_gmax(1) has
 * been called.  adacomp_workspace_gmax says where it is then left inside the workspace: byte
 * offset and number of floats for the first learner of a call, and (if not NULL) the distance in
 * bytes to the next learner's vector in a batched call.  For tests of the first loop of
 * Algorithm 2. */
int adacomp_debug_keep_gmax(int enable);
int adacomp_workspace_gmax(const adacomp_layer_t *layers, uint32_t n_layers, size_t *byte_offset,
                           size_t *n_bins_total, size_t *learner_stride);

/* Plain float4 device copy of n floats (dst, src 16-byte aligned): the reference kernel against
 * which HBM byte counters and the achievable copy bandwidth are calibrated. */
int adacomp_copy_f32(float *dst, const float *src, size_t n, void *hip_stream);

/* The two streaming ceilings the hot kernels are measured against, with the access pattern of the
 * streaming pass of compress and nothing else (tiles of 4096 elements, 16 per thread, streaming
 * 16-byte loads and stores, the same tile order): x <- x + y in place, 12 bytes per element as
 * pack() moves (read dW, read residue, write residue); and x <- value, 4 bytes per element as the
 * dense sum of unpack() writes.  x, y 16-byte aligned and distinct, n a multiple of 4. */
int adacomp_triad_f32(float *x, const float *y, size_t n, void *hip_stream);
int adacomp_fill_f32(float *x, float value, size_t n, void *hip_stream);
/* The same triad with at most workgroups_per_cu (3 .. 8; adacomp_triad_f32 is 8) workgroups resident on
 * a compute unit: HBM serves this access pattern better with fewer bytes in flight, so the ceiling a
 * kernel is held against is the best of these, not the full-residency one. */
int adacomp_triad_resident_f32(float *x, const float *y, size_t n, uint32_t workgroups_per_cu, void *hip_stream);

/* Host-only exhaustive check of the multiply-shift constants the kernels use to turn an element
 * index into a bin index (every L_T in 1..16384 against every index below 16384). 0 if all agree. */
int adacomp_selftest_binindex(void);

/* Tuning knob of adacomp_unpack_accumulate / adacomp_unpack_update, read by adacomp_workspace_init.
 * A workgroup of the unpack kernel serves a run of up to 8 neighbouring output tiles (4096 elements
 * each) that share their per-bin bookkeeping; the run length is halved until at least n_groups
 * workgroups remain, so that small tables still fill the GPU.  Results do not depend on it.
 * 0 restores the default (2048).  Process-wide; not synchronised with calls on other threads.
 * Returns ADACOMP_OK. */
int adacomp_tuning_unpack_min_groups(uint32_t n_groups);

/* Tuning knob of the compress calls, read at every call.  Tables of up to 512 compress tiles and
 * 16 layers skip the separate scan launch (layer scales, word offsets): the placement kernel works
 * them out itself.  enable = 0 makes such tables take the three-launch path of the large ones;
 * non-zero restores the default.  Results do not depend on it while the float64 sum of every layer's
 * g_max vector is exact (see "Arithmetic" in adacomp.h); beyond that a layer scale may differ in its
 * last bit between the two paths.  Process-wide; not synchronised with
 * calls on other threads.  Returns ADACOMP_OK. */
int adacomp_tuning_fold_scan(int enable);

/* Tuning knob of the eager compress calls, read at every call.  Large tables with short bins
 * (some L_T <= 64) correct the residue tile by tile, whole 64-byte lines at a time, in the placement
 * kernel; enable = 0 makes them take the word-by-word placement of the other tables; non-zero
 * restores the default.  Results do not depend on it.  Returns ADACOMP_OK. */
int adacomp_tuning_place_tiled(int enable);

/* Per-kernel timing of the streaming kernel (k_fused) of adacomp_compress / adacomp_compress_batch
 * with HIP events on the caller's stream.  enable = k > 0 starts recording every k-th launch (and
 * clears earlier records; an event pair costs a few microseconds between back-to-back launches, so
 * a timed run samples); 0 stops.  adacomp_timing_read synchronises the recorded events and returns their
 * summed duration, the number of launches and the number of learners those launches covered. */
int adacomp_timing_enable(int enable);
int adacomp_timing_read(double *total_ms, uint64_t *n_launches, uint64_t *n_learners);

#ifdef __cplusplus
}
#endif
#endif

/*
 * mt_debug.h - measurement and testing aids of the multi-tenant worker runtime.  Not part of
 * the serving interface (include/mt.h); exported by the same library.
 */
#ifndef MT_DEBUG_H
#define MT_DEBUG_H

#include "mt.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Per-kernel timing of mt_run, for measurement.  While enabled, mt_run brackets every
 * kernel it enqueues with HIP events on the run's stream (this costs a few microseconds
 * per kernel, so throughput is measured with it off).  mt_get_profile synchronises the
 * stream of the last profiled mt_run and fills *out with elapsed milliseconds; entries
 * of launches that did not happen are 0. */
typedef struct {
    float batcher_ms, gather_ms, head_ms;
    float fc_ms[MT_MAX_LAYERS];     /* grouped FC launch of each layer index          */
    float fc_big_ms[MT_MAX_LAYERS]; /* grouped big-tile FC launch of each layer index */
    float conv_ms[MT_MAX_LAYERS];   /* grouped convolution launch of each layer index */
    float gap_ms[MT_MAX_LAYERS];    /* pooling launch of each layer index             */
    float ops_ms[MT_MAX_LAYERS];    /* max-pool / residual-add launch of each layer index */
    float total_ms;                 /* first kernel start to last kernel end          */
} mt_profile;
mt_status mt_set_profiling(mt_ctx* ctx, int enable);
mt_status mt_get_profile(mt_ctx* ctx, mt_profile* out);

/* Testing aid: fill the context's internal activation and logits buffers with NaN bit
 * patterns (synchronous).  A correct run overwrites or zero-fills everything it later
 * reads, so results must not change.  Errors: MT_ESTATE (host-only), MT_EDEVICE. */
mt_status mt_debug_poison(mt_ctx* ctx);

/* Measurement aid: one plain copy kernel (16 bytes per lane, grid-stride) of `bytes` bytes
 * (a multiple of 16) from `src` to `dst`, both device memory owned by the caller, on `stream`
 * of the current device.  It reads and writes exactly `bytes` bytes once each, which is what
 * hardware byte counters are calibrated against.  Errors: MT_EINVAL (null pointer, size not
 * a multiple of 16), MT_EDEVICE (launch failure). */
mt_status mt_debug_copy(void* dst, const void* src, uint64_t bytes, void* stream);

/* Measurement aid: how the library would split a fully-connected layer of one tenant that
 * has `rows` requests in a run and `out_features` outputs, in a run that uses its
 * compute-bound kernel (large batches; the decision per run and per layer index is the
 * library's): the number of rows that kernel serves, the remaining rows being served by the
 * weight-streaming kernel; 0 if the layer does not qualify at all.  Pure function of its
 * arguments; needs no context and no device.  Lets a benchmark attribute flops to the
 * kernel that performed them. */
uint32_t mt_debug_big_tile_rows(uint32_t rows, uint32_t out_features);

/* Measurement aid: which of the two compute-bound FC kernels serves a layer index whose shortest
 * fan-in among the registered models is `in_features`: 1 if one workgroup per compute unit walks
 * the 256x256 tiles (mt::fc_big_walk_kernel), 0 if every tile gets a workgroup of its own
 * (mt::fc_big_kernel; also what MT_BIG_WALK=0 in the environment of mt_create selects).  Pure
 * function of its argument; needs no context and no device.  Lets a benchmark name the kernel
 * whose launches it timed. */
uint32_t mt_debug_big_tile_walk(uint32_t in_features);

/* Measurement and test aid: how a convolution layer is cut into tiles (paper section 3.1: the layer set is closed,
 * so the library can choose a tiling per layer shape when a model is registered).  A k x k convolution of an
 * in_h x in_w image with in_channels channels (padded to a multiple of 8) and pad (k - 1) / 2, elements of
 * elem_size bytes (2 or 4).  Returns 1 and writes the tiling if the layer's tiles are whole output rows whose input
 * rows are held in LDS: *rows_per_tile output rows of one image per tile, or, if *images_per_tile > 1, that many
 * whole images of *rows_per_tile rows each; *tiles_per_image tiles cover an image; *frame_bytes is the LDS the
 * input rows of a tile take.  Returns 0 (and writes zeros) if the layer's tiles are runs of 128 output pixels
 * gathered tap by tap.  Pure function of its arguments; needs no context and no device; NULL outputs are skipped. */
int mt_debug_conv_row_tiling(uint32_t in_h, uint32_t in_w, uint32_t in_channels, uint32_t ksize, uint32_t stride, uint32_t elem_size,
                             uint32_t* rows_per_tile, uint32_t* images_per_tile, uint32_t* tiles_per_image, uint64_t* frame_bytes);

/* Measurement aid: what a loop of nothing but bf16 matrix instructions sustains on the current
 * device.  Runs, on `stream`, a kernel in which every wavefront issues v_mfma_f32_32x32x16_bf16
 * on pseudo-random operands (eight independent accumulators, two wavefronts per SIMD, no memory
 * traffic) for about ten milliseconds, waits for it, and writes the rate in TFLOP/s to *tflops.
 * The chip lowers its clock under matrix load, so this figure, not the published peak, is what a
 * compute-bound kernel can approach.  Allocates (and frees) a small device buffer.
 * Errors: MT_EINVAL (null), MT_EDEVICE. */
mt_status mt_debug_mfma_rate(void* stream, double* tflops);

#ifdef __cplusplus
}
#endif
#endif /* MT_DEBUG_H */

/*
 * libegeria: timing instrumentation for benchmarks.  Not part of the method and
 * not needed by any caller of include/egeria.h; exported for bench.py, which
 * times one kernel class inside a larger timed region.
 */
#ifndef EGERIA_PROFILE_H
#define EGERIA_PROFILE_H

#include "egeria.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Time every launch
 * of one kernel class with a pair of HIP events recorded on the launch's own
 * stream, so that a caller can time that kernel inside a larger timed region.
 * egeria_profile_begin arms recording for up to max_launches launches (events
 * are host-side objects the library creates once and reuses).
 * egeria_profile_end waits for the recorded events, writes the durations in
 * milliseconds to the HOST array ms_out (at most `capacity` of them), stores
 * the number recorded in *n_out (HOST) and disarms.  Process wide, not
 * thread-safe; do not use while a stream is being captured. */
typedef enum {
    EGERIA_KERNEL_NONE = 0,
    EGERIA_KERNEL_ABSMAX = 1,       /* absolute-maximum reduction            */
    EGERIA_KERNEL_QUANTIZE = 2,     /* fp32/bf16 -> int8 map                 */
    EGERIA_KERNEL_GEMM = 3,         /* int8 GEMM / implicit-GEMM convolution */
    EGERIA_KERNEL_GRAM = 4,         /* split-K Gram partials of the metric   */
    EGERIA_KERNEL_ATTENTION = 5,
    EGERIA_KERNEL_LAYERNORM = 6,
    EGERIA_KERNEL_CACHE_COPY = 7    /* row copies of the activation cache    */
} egeria_kernel_class;

egeria_status egeria_profile_begin(int32_t kernel_class, int32_t max_launches);
/* Between begin and end: paused != 0 stops recording (launches go out without events, which cost
 * host time), paused == 0 resumes it.  Lets a caller sample some steps of a timed loop only. */
egeria_status egeria_profile_pause(int32_t paused);
egeria_status egeria_profile_end(float *ms_out, int32_t capacity, int32_t *n_out);

/* The attention of a Transformer layer on its own, for measuring the fast kernel's error against the fp64
 * one (bench.py --attention-error).  qkv: fp32 [B, S, 3 * hidden] (q | k | v per token), ctx: fp32
 * [B, S, hidden] out.  mode 0: the fp64 kernel of observed runs.  mode 1: the fp32 matrix-core kernel of
 * unobserved runs; records then receives B * heads * ceil(S / 64) pairs {uint32 bit pattern of the largest
 * |ctx| of a workgroup's 64 queries x head dims, fp32 error bound E of those values} (DEVICE, 16-byte
 * aligned; ignored in mode 0).  Limits as for the Transformer kinds of egeria_ref_forward. */
egeria_status egeria_profile_attention(const float *qkv, int32_t B, int32_t S, int32_t hidden, int32_t heads,
                                       int32_t mode, float *ctx, void *records, void *stream);

/* Unobserved runs of the Transformer kinds evaluate attention with the certified fp32 kernels when the two
 * products take at least this many flops (4 * batch * heads * seq^2 * head size; default 5e9), with the fp64
 * kernel below it: the results are the same, the certified path has four launches of fixed cost.  Sets the
 * threshold (a negative value leaves it unchanged) and returns the previous one; process-wide, for tests that
 * exercise the certified kernels on small shapes. */
double egeria_profile_attention_threshold(double min_flops);

/* What the device delivers to kernels shaped like this library's: one small complete kernel per kind, run
 * twice (the second run is timed with events on `stream`).  ms_out: duration of that run; work_out: what it
 * did - operations (matrix instructions: 2 per multiply-add) or bytes (LDS, L2 -> LDS, copy: read + written).
 * iters: length of the inner loop (ignored by the copy); scratch: DEVICE, at least 256 MiB. */
typedef enum {
    EGERIA_MICRO_MFMA_I8 = 0,        /* v_mfma_i32_32x32x32_i8, two workgroups of four waves per compute unit */
    EGERIA_MICRO_MFMA_BF16 = 1,      /* v_mfma_f32_32x32x16_bf16 */
    EGERIA_MICRO_MFMA_F32_32 = 2,    /* v_mfma_f32_32x32x2_f32 */
    EGERIA_MICRO_MFMA_F32_16 = 3,    /* v_mfma_f32_16x16x4_f32 */
    EGERIA_MICRO_MFMA_F64 = 4,       /* v_mfma_f64_16x16x4_f64 */
    EGERIA_MICRO_LDS_READ = 5,       /* ds_read_b128 without bank conflicts */
    EGERIA_MICRO_LDS_WRITE = 6,      /* ds_write_b128 without bank conflicts */
    EGERIA_MICRO_L2_TO_LDS_LINE = 7, /* buffer loads with the LDS modifier, whole 128-byte lines of L2-resident rows */
    EGERIA_MICRO_L2_TO_LDS_HALF = 8, /* ... half lines (64 bytes per row and request) */
    EGERIA_MICRO_HBM_COPY = 9,       /* 128 MiB copied with 16-byte accesses */
    EGERIA_MICRO_BF16_CHAIN = 10,    /* mfma_f32_32x32x16_bf16, one dependent chain per wave, one wave per SIMD */
    EGERIA_MICRO_BF16_CHAIN_VALU = 11, /* ... with eight independent fp32 vector instructions after each */
    EGERIA_MICRO_BF16_CHAIN_VALU2 = 12 /* ... and two waves per SIMD */
} egeria_micro_kind;
egeria_status egeria_microbench(int32_t kind, int32_t iters, void *scratch, size_t scratch_bytes, float *ms_out,
                                double *work_out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* EGERIA_PROFILE_H */

/*
 * lrd_measure.h -- measurement aids of the library for low-rank-decomposed layers (see lrd.h).
 *
 * NOT part of the layer ABI.  Nothing here computes any step of the paper's method; these calls
 * exist so that a benchmark can (a) time the product kernels of a layer pass with events on the
 * launch stream, (b) compare the two evaluation orders of a pair (Section 2, Fig. 1: two
 * consecutive layers, with the rank-r intermediate in memory or kept on chip), and (c) measure,
 * in the same run, what the machine delivers to a loop of matrix instructions with no memory in
 * it and to a plain streaming kernel, as denominators next to the published peaks.
 *
 * Unlike the calls of lrd.h, lrd_set_fusion and the event log keep PROCESS-WIDE mutable state
 * and are not safe against concurrent use from several threads.
 */
#ifndef LRD_MEASURE_H
#define LRD_MEASURE_H

#include <stddef.h>
#include <stdint.h>

#include "lrd.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * How a bf16 pair with r <= 256 is evaluated.  LRD_FUSION_AUTO (default) lets the library choose
 * per shape; LRD_FUSION_ALWAYS keeps the rank-r intermediate in LDS between the two products
 * whenever the fused kernel supports the shape; LRD_FUSION_NEVER runs two separate products
 * through an intermediate in memory (H_save or the workspace).  Results agree up to fp32
 * summation order.  Process-wide; returns the previous mode, or -1 (and changes nothing) for an
 * unknown mode.
 */
enum { LRD_FUSION_AUTO = 0, LRD_FUSION_ALWAYS = 1, LRD_FUSION_NEVER = 2 };
int32_t lrd_set_fusion(int32_t mode);

/*
 * Event log of the matrix products of the layer passes.  Between lrd_profile_log_start and
 * lrd_profile_log_stop every product the library launches (H = X.V^T, dU = dY^T.H, a convolution
 * core, ...) is bracketed by hipEventRecord on its launch stream with the next pair of caller-owned
 * events, events[2i] before and events[2i + 1] after product i (hipEvent_t passed as void*), and
 * described by record i; products beyond n_pairs are not logged.  A product whose reduction is
 * split (splits > 1) is bracketed together with the kernel that sums its slices.  The caller
 * synchronises and reads the elapsed times itself.  Logging costs two event records per product,
 * so it belongs in a separate, eager pass, not in a captured graph.
 */
enum {
    LRD_ROLE_NONE = 0,        /* any other product (convolution layers, dense layers, recomputed intermediates) */
    LRD_ROLE_FWD_DOWN = 1,    /* H  = X.V^T   */
    LRD_ROLE_FWD_UP = 2,      /* Y  = H.U^T   */
    LRD_ROLE_DGRAD_UP = 3,    /* dH = dY.U    */
    LRD_ROLE_DGRAD_DOWN = 4,  /* dX = dH.V    */
    LRD_ROLE_WGRAD_U = 5,     /* dU = dY^T.H  */
    LRD_ROLE_WGRAD_V = 6      /* dV = dH^T.X  */
};
typedef struct {
    int32_t role;             /* LRD_ROLE_* */
    int32_t gather;           /* 0 plain product, 1 / 2 / 3 convolution forward / data gradient / weight gradient */
    int32_t epilogue;         /* 0 none, 1 activation stored beside the result, 2 result times activation gradient */
    int32_t splits;           /* slices of the reduction (1: one kernel) */
    int64_t M, N, K;          /* result M x N, reduction length K */
    int64_t batch;            /* products of this shape the launch ran (1 unless batched) */
    char kernel[64];          /* the kernel that ran the product (template and tile), NUL-terminated */
} lrd_profile_record;
lrd_status lrd_profile_log_start(void** events, int32_t n_pairs);
/* Stops logging and copies up to `capacity` records to `out` (host, nullable); returns the number of
 * products logged since lrd_profile_log_start. */
int32_t lrd_profile_log_stop(lrd_profile_record* out, int32_t capacity);

/*
 * Launches `workgroups` workgroups of four wavefronts that each issue `iters` rounds of four
 * independent bf16 matrix instructions (32x32x16, fp32 accumulation) on registers only; the caller
 * times the launch with events on `hip_stream`.  *flops_host (host, nullable) receives the
 * floating-point operations of the launch.  sink: device, at least workgroups * 256 floats,
 * written so that the loop cannot be removed.  Stateless.
 */
lrd_status lrd_measure_mfma_loop(float* sink, int32_t workgroups, int32_t iters, double* flops_host, void* hip_stream);

/*
 * Launches `workgroups` workgroups of four wavefronts that each read `iters` rounds of eight 16-byte
 * words per lane from LDS (ds_read_b128, eight in flight), in the pattern of an operand fragment; the caller times the
 * launch.  *bytes_host (host, nullable) receives the LDS bytes read by the launch (divide by the time
 * and by the compute units the workgroups cover for bytes per second per unit).  sink: device, at least
 * workgroups * 256 words.  Stateless.
 */
lrd_status lrd_measure_lds_read(uint32_t* sink, int32_t workgroups, int32_t iters, double* bytes_host, void* hip_stream);

/*
 * One pass of a plain streaming kernel over `bytes` bytes (a multiple of 16; 16 bytes per lane
 * per access): LRD_STREAM_READ sums src into a few words of dst (dst: at least 16 KiB),
 * LRD_STREAM_WRITE fills dst, LRD_STREAM_COPY copies src to dst.  src / dst are device pointers,
 * 16-byte aligned.  Stateless.
 */
enum { LRD_STREAM_READ = 0, LRD_STREAM_WRITE = 1, LRD_STREAM_COPY = 2 };
lrd_status lrd_measure_stream(const void* src, void* dst, size_t bytes, int32_t mode, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* LRD_MEASURE_H */

/*
 * alise_ops.h -- C ABI of the two fused elementwise / row operators of the transformer layer
 * for MI355X (gfx950): residual add + LayerNorm, and bias + ReLU; plus the streaming-read probe
 * that the measurements use as their bandwidth ceiling.
 *
 * ALISE (arXiv 2410.23537) Sec. 3.3 "Implementation" lists fused kernels for LayerNorm,
 * Attention and ReLU and batches LayerNorm and ReLU over the irregularly shaped token batches
 * of iteration-level scheduling; Sec. 2 "Transformer Architecture" places LayerNorm and the
 * residual connection around the attention and FFN modules.  The attention kernels are in
 * alise_kv.h; these are the other two.  Both work on a flat [rows, width] matrix of fp16:
 * a row is one token of the running batch, however the batch was put together.
 *
 * The general rules of alise_kv.h hold (device pointers, caller-owned buffers, work is
 * enqueued on `hip_stream` and not waited for, host-checkable arguments are checked before
 * any HIP call, same status codes).  Every matrix pointer must be 16-byte aligned and the
 * width a multiple of 8 (rows are read and written in 16-byte units).
 */
#ifndef ALISE_OPS_H
#define ALISE_OPS_H

#include "alise_kv.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Residual add + LayerNorm over the rows of a [rows, hidden] matrix
 * [Sec. 3.3 "Implementation": fused LayerNorm; Sec. 2: LayerNorm and residual connection].
 *
 *     h = fp16(x + residual)            the exact sum, rounded once to nearest even; h = x when
 *                                       residual is NULL
 *     y = fp16(gamma * (h - mean) / sqrt(var + eps) + beta)
 *
 * mean and var (the biased variance, divided by hidden) run over the fp16 values of h of
 * one row and are computed in fp32, the mean first and the squared deviations from it
 * second.  h is bit-exact; y is the fp32 result rounded once, so it can differ from the
 * correctly rounded exact value by one unit in the last place of fp16.
 *
 * x, residual: device, fp16 [rows, hidden], read.   gamma, beta: device, fp16 [hidden], read.
 * h_out: device, fp16 [rows, hidden], written; may be NULL when the sum is not needed, and may
 *        alias x or residual (each element is read before it is written, by the same thread).
 * y_out: device, fp16 [rows, hidden], written; may alias x or residual likewise, not h_out.
 * rows >= 0 (0: nothing is done and no pointer is looked at); 8 <= hidden <= 16384, a multiple
 * of 8, else ALISE_UNSUPPORTED.  eps >= 0 and finite, else ALISE_INVALID_ARGUMENT.
 */
int alise_add_layernorm(const void *x, const void *residual, const void *gamma, const void *beta,
                        float eps, void *h_out, void *y_out, int64_t rows, int32_t hidden,
                        void *hip_stream);

/*
 * Bias + ReLU over a [rows, cols] matrix [Sec. 3.3 "Implementation": fused ReLU; the
 * activation between the two linear layers of the FFN of Sec. 2].
 *
 *     y = fp16(max(x + bias, 0))        the exact sum, rounded once to nearest even; a result
 *                                       of -0 is stored as +0.  Bit-exact.
 *
 * x: device, fp16 [rows, cols], read.   bias: device, fp16 [cols], read; NULL = no bias.
 * y_out: device, fp16 [rows, cols], written; may be x itself (in place).
 * rows >= 0 (0: nothing is done and no pointer is looked at); cols >= 8, a multiple of 8, and
 * rows * cols below 2^35 elements, else ALISE_UNSUPPORTED.
 */
int alise_bias_relu(const void *x, const void *bias, void *y_out, int64_t rows, int32_t cols,
                    void *hip_stream);

/*
 * Streaming-read probe: a measurement utility, not an operation of the paper.  The decode step is
 * "memory-bound" (Sec. 4.2) and its figure of merit here is the fraction of the HBM bandwidth it
 * sustains; this call measures what a kernel that does nothing but read sustains on the same
 * device, the ceiling beside the published peak.
 *
 * Reads `bytes` bytes at src once (16-byte non-temporal loads from a persistent grid) and stores
 * the exclusive-or of all 32-bit words read into *xor_out (0 for bytes == 0).
 *
 * src: device, 16-byte aligned, read.   bytes: a multiple of 16, else ALISE_UNSUPPORTED.
 * xor_out: device, one uint32, written (cleared first, then combined with atomics: do not read it
 * before the stream has passed the call).
 */
int alise_hbm_read_probe(const void *src, size_t bytes, void *xor_out, void *hip_stream);

/*
 * Issue probe: a measurement utility, not an operation of the paper.  The chunked-prefill and the
 * grouped-query kernels mix matrix instructions with the vector instructions that dequantize and
 * form the softmax weights; what bounds them depends on whether the two kinds run side by side on
 * a SIMD.  Every wave of a launch that gives each SIMD two waves runs `iters` rounds of
 *   mode 1: 16 independent v_mfma_f32_16x16x32_f16,
 *   mode 2: 64 independent v_fma_f32 (about the same time as mode 1 when run alone),
 *   mode 3: both.
 * The caller times the three launches (bench.py: `issue_overlap`).  Nothing of interest is
 * written; `sink` (device, one float, 4-byte aligned) only keeps the instruction chains alive.
 * iters in [0, 2^24]; another mode returns ALISE_UNSUPPORTED.
 */
int alise_issue_overlap_probe(int32_t mode, int32_t iters, void *sink, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* ALISE_OPS_H */

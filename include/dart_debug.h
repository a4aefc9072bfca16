/*
 * dart_debug.h -- diagnostic entry points of libdart.so.  NOT part of the product interface
 * (include/dart.h): they exist for this repository's own tests and benchmark, may change
 * without notice and must not be called from serving code.
 */
#ifndef DART_DEBUG_H
#define DART_DEBUG_H

#include "dart.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Diagnostic (tests only): copy a named fp32 workspace of the last forward call to host
 * memory after synchronising the device.  Names: "xn" (normed layer input; rows are 2 d wide on a front-end context), "resid", "qkv",
 * "att_out" (attention output), "y" (after attention residual), "yn", "hmid" (SwiGLU
 * product), "u" (after MLP residual).  Buffers hold 16 rows and are those of the single-sequence
 * calls: the batched calls hand most of these rows on as packed operand tiles and do not store
 * them.  Returns the number of floats copied (at most max_count) or -1 on error. */
int64_t dart_debug_read(dart_ctx *ctx, const char *name, float *host_out, int64_t max_count);

/* Diagnostic (benchmark only): enqueue only the LM-head projection (the final step of
 * dart_draft_forward, Sec. 3.2) on the final-normed rows the last forward call left in the
 * workspace; logits_out device [rows][vocab] fp32.  multi_row = 0: the kernel of the
 * single-sequence call (rows <= 16); 1: the kernels of the batched call (bf16 contexts,
 * rows <= 16 * max_K): operand conversion pass + contraction; 2: the contraction alone, on the
 * operand tiles a preceding call with multi_row = 1 and the same rows left behind.  Used to
 * time those kernels in isolation. */
dart_status dart_debug_lm_head(dart_ctx *ctx, int rows, int multi_row, float *logits_out,
                               void *stream);

/* Diagnostic (benchmark only): enqueue only the LM-head kernel of dart_draft_forward_topk (the
 * projection that also selects each workgroup's k best candidates, Sec. 3.2 + Alg. 1) on the
 * final-normed rows the last forward call left in the workspace; rows <= 8.  The per-workgroup
 * candidate lists stay in the context's workspace and the row merge is not run.  logits_out:
 * device [rows][vocab] fp32, or NULL to skip the store as dart_draft_forward_topk does without
 * a logits buffer.  DART_ERR_STATE on contexts whose LM head does not select (fp32 storage,
 * front end, d beyond one k-chunk). */
dart_status dart_debug_lm_head_select(dart_ctx *ctx, int rows, int k, float *logits_out, void *stream);

/* Diagnostic (benchmark only): the name and launch shape of the kernel that
 * dart_debug_lm_head(ctx, rows, multi_row != 0, ...) -- or, with multi_row = 3,
 * dart_debug_lm_head_select(ctx, rows, ...) -- launches for the LM head, as text
 * ("gemv_bf16_kernel<20,20,0,true,true> grid=184x512"), written to buf (at most len bytes
 * including the terminator).  Counter summaries under profiles/ are keyed by this string.
 * Returns the length written, or -1 on error. */
int dart_debug_lm_head_key(dart_ctx *ctx, int rows, int multi_row, char *buf, int len);

/* Diagnostic (benchmark only): a plain streaming read of `bytes` bytes of device memory at
 * `buf` (16-byte aligned) by `workgroups` workgroups of 512 threads, 16 bytes per lane per
 * load, with the non-temporal hint the weight streams use (non_temporal != 0) or as ordinary
 * cached loads; nothing is written (`sink`, device, 4 bytes, may be NULL).  The read rate of
 * this kernel is the practical ceiling the weight-streaming kernels are compared with. */
dart_status dart_debug_stream_read(const void *buf, int64_t bytes, int workgroups, int non_temporal,
                                   void *sink, void *stream);

#ifdef DART_TUNING
/* Tuning builds only (library compiled with -DDART_TUNING; the product build does not export
 * this symbol and its launch tunables are constants): override a launch tunable of the kernels by name
 * ("gemv_wgs", "gemv_xcd", "gemv_depth", "gemv_nt", "gemv_nt_min_mb", "gemv_split", "gemm_wgs", "attn_seg").  Process-wide,
 * not thread-safe.  Returns 0, or -1 for an unknown name. */
int dart_debug_set(const char *name, int value);
#endif

#ifdef __cplusplus
}
#endif
#endif /* DART_DEBUG_H */

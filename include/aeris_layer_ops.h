/*
 * aeris_layer_ops.h -- C ABI of the element-wise operations around the window attention in an
 * AERIS transformer layer (MI355X / gfx950), in the same library as aeris_winattn.h.
 *
 * The AERIS paper ("AERIS Model Architecture") builds every layer from a pre-RMSNorm (in place
 * of LayerNorm), an attention or SwiGLU branch, and adaptive-layer-norm values alpha, beta,
 * gamma that a layer-specific linear map derives from the diffusion-time embedding.  It prints
 * no formulas; the ones below are those of the works it cites for each part.  The input
 * projections of the two branches (QKV, SwiGLU up-projection) are offered with the RMSNorm and
 * the modulation folded in (last section of this file), the output projections as a plain
 * bf16 product; the backward products of the projections are plain GEMMs left to the caller.
 *
 * Rows are tokens.  Activations are bf16, row-major [n_rows, channels], rows contiguous
 * (stride = channels).  The sample of row i is i / rows_per_sample: the tokens of one sample
 * share one diffusion time and therefore one (alpha, beta, gamma).  Parameters and conditioning
 * vectors are fp32: w [channels]; alpha, beta, gamma [n_samples, channels] with
 * n_samples = n_rows / rows_per_sample.  All arithmetic is fp32; bf16 results are rounded to
 * nearest even.  Sums over tokens are taken in a fixed order (no atomics): results are bitwise
 * reproducible from call to call.
 *
 * Limits: channels % 8 == 0 and 8 <= channels <= AERIS_MAX_CHANNELS; hidden % 8 == 0;
 * n_rows % rows_per_sample == 0 and at most 2^20 samples (AERIS_ERR_INVALID_SHAPE /
 * AERIS_ERR_NOT_DIVISIBLE otherwise).  Pointers are DEVICE pointers, 16-byte aligned, owned by the
 * caller; inputs are read-only and outputs fully overwritten.  The library allocates nothing and
 * never synchronises: calls only enqueue kernels on `hip_stream` (a hipStream_t passed as
 * void*; NULL is the default stream).  Errors are the AERIS_ERR_* codes of aeris_winattn.h;
 * arguments are checked before anything is launched.
 */
#ifndef AERIS_LAYER_OPS_H
#define AERIS_LAYER_OPS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AERIS_MAX_CHANNELS 4096

/*
 * Pre-RMSNorm with adaptive modulation (Model Architecture: pre RMSNorm; alpha, beta, gamma of
 * the adaptive layer norm).  For every row:
 *     r = (mean_c x_c^2 + eps)^(-1/2),  h_c = x_c r w_c (1 + gamma_{b,c}) + beta_{b,c}.
 * Outputs h [n_rows, channels] bf16 and r [n_rows] fp32 (kept for the backward pass; r may be
 * NULL if it is not wanted).
 */
int aeris_rmsnorm_adaln_fwd(const void* x, const float* w, const float* gamma, const float* beta,
                            float eps, int64_t n_rows, int64_t rows_per_sample, int32_t channels,
                            void* h, float* r, void* hip_stream);

/*
 * Backward of the above, given dh [n_rows, channels] bf16 and the r of the forward call:
 *     n = x r,  dn = dh w (1 + gamma),  dx = r (dn - n mean_c(dn n))           bf16
 *     dbeta_{b,c}  = sum_{rows of b} dh_c
 *     dgamma_{b,c} = w_c sum_{rows of b} dh_c n_c
 *     dw_c         = sum_b (1 + gamma_{b,c}) sum_{rows of b} dh_c n_c          fp32
 * dw, dgamma, dbeta may each be NULL (not wanted).  `workspace` holds the per-workgroup partial
 * column sums; its size comes from the function below.
 */
size_t aeris_rmsnorm_adaln_bwd_workspace_bytes(int64_t n_rows, int64_t rows_per_sample,
                                               int32_t channels);
int aeris_rmsnorm_adaln_bwd(const void* x, const float* w, const float* gamma, const float* r,
                            const void* dh, int64_t n_rows, int64_t rows_per_sample,
                            int32_t channels, void* dx, float* dw, float* dgamma, float* dbeta,
                            void* workspace, size_t workspace_bytes, void* hip_stream);
/*
 * The same with the residual connection around the normalised branch closed in the same pass
 * (a layer computes x + branch(RMSNorm(x)), so x receives the branch's gradient plus the
 * gradient dres [n_rows, channels] bf16 that arrives along the residual path):
 *     dx = dres + r (dn - n mean_c(dn n))
 * summed in fp32 and rounded to bf16 once.  dres may be NULL (then this is the call above); it
 * must not overlap dx.
 */
int aeris_rmsnorm_adaln_bwd_residual(const void* x, const float* w, const float* gamma,
                                     const float* r, const void* dh, const void* dres,
                                     int64_t n_rows, int64_t rows_per_sample, int32_t channels,
                                     void* dx, float* dw, float* dgamma, float* dbeta,
                                     void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Gated residual connection (Model Architecture: alpha of the adaptive layer norm gates the
 * branch before it joins the residual stream):  out = x + alpha_b * y, all bf16.
 * `out` may alias x or y.
 */
int aeris_gate_residual_fwd(const void* x, const void* y, const float* alpha, int64_t n_rows,
                            int64_t rows_per_sample, int32_t channels, void* out,
                            void* hip_stream);

/*
 * Backward of the gated residual, given dout (the gradient with respect to x is dout itself):
 *     dy = alpha_b * dout   (bf16),   dalpha_{b,c} = sum_{rows of b} dout_c y_c   (fp32).
 * dy may alias dout.  dalpha may be NULL.
 */
size_t aeris_gate_residual_bwd_workspace_bytes(int64_t n_rows, int64_t rows_per_sample,
                                               int32_t channels);
int aeris_gate_residual_bwd(const void* y, const float* alpha, const void* dout, int64_t n_rows,
                            int64_t rows_per_sample, int32_t channels, void* dy, float* dalpha,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * SwiGLU gate (Model Architecture: SwiGLU in the fully connected layers) on the packed up
 * projection uv [n_rows, 2*hidden] = [u | v]:  g = silu(u) * v,  silu(u) = u / (1 + exp(-u)).
 * g is [n_rows, hidden] bf16.
 */
int aeris_swiglu_fwd(const void* uv, int64_t n_rows, int32_t hidden, void* g, void* hip_stream);

/*
 * Backward of the gate, given dg [n_rows, hidden]:  with s = 1 / (1 + exp(-u)),
 *     du = dg v s (1 + u (1 - s)),   dv = dg u s;   duv [n_rows, 2*hidden] = [du | dv] bf16.
 * duv may alias uv.
 */
int aeris_swiglu_bwd(const void* uv, const void* dg, int64_t n_rows, int32_t hidden, void* duv,
                     void* hip_stream);

/*
 * Input projections with the pre-RMSNorm and the modulation folded in (Model Architecture:
 * RMSNorm and the adaptive-layer-norm values precede the projection of queries, keys and values
 * and the SwiGLU feed-forward part).  With h as in aeris_rmsnorm_adaln_fwd and a weight
 * `weight` [out_features, channels] bf16 (one row per output feature, rows contiguous):
 *     y [n_rows, out_features] = h weight^T          (bf16)
 * h is never written.  The call computes r by a row pass over x, folds w (1 + gamma_b) into a
 * per-sample copy of the weight (rounded to bf16: the products multiply in bf16) and beta_b
 * into a per-sample bias beta_b weight^T (fp32), and runs one bf16 GEMM on the raw rows x whose
 * epilogue applies r and the bias:  y_i = r_i x_i Wf_b^T + bias_b.
 * For QKV, weight = [Wq ; Wk ; Wv] gives y = [B, H, W, 3, heads, head_dim], the packed layout
 * the attention entry points take through their stride fields.
 * Limits: channels % 64 == 0, 64 <= channels <= AERIS_MAX_PROJECTION_CHANNELS,
 * out_features % 8 == 0, out_features * channels < 2^31.  workspace: >=
 * aeris_norm_linear_workspace_bytes(...) bytes (folded weights, biases, r), 16-byte aligned,
 * contents undefined before and after.
 */
#define AERIS_MAX_PROJECTION_CHANNELS 8192
size_t aeris_norm_linear_workspace_bytes(int64_t n_rows, int64_t rows_per_sample,
                                         int32_t channels, int32_t out_features);
int aeris_norm_linear_fwd(const void* x, const float* w, const float* gamma, const float* beta,
                          float eps, const void* weight, int64_t n_rows, int64_t rows_per_sample,
                          int32_t channels, int32_t out_features, void* y, void* workspace,
                          size_t workspace_bytes, void* hip_stream);

/*
 * The SwiGLU up-projection the same way, with the gate as a second epilogue: weight
 * [2*hidden, channels] = [u rows ; v rows],  uv = h weight^T,  g = silu(u) v  [n_rows, hidden]
 * bf16, formed from the fp32 accumulators.  uv [n_rows, 2*hidden] bf16 is also written if the
 * pointer is not NULL (aeris_swiglu_bwd needs it).  workspace as above with
 * out_features = 2*hidden.
 */
int aeris_norm_linear_swiglu_fwd(const void* x, const float* w, const float* gamma,
                                 const float* beta, float eps, const void* weight, int64_t n_rows,
                                 int64_t rows_per_sample, int32_t channels, int32_t hidden,
                                 void* g, void* uv, void* workspace, size_t workspace_bytes,
                                 void* hip_stream);

/* Output projection of a branch: y [n_rows, out_features] = x weight^T, bf16 in and out, fp32
 * accumulation, same kernel without the folded parts.  Limits as above. */
int aeris_linear_fwd(const void* x, const void* weight, int64_t n_rows, int32_t channels,
                     int32_t out_features, void* y, void* hip_stream);

/*
 * Gradients of a projection y = x weight^T (the backward pass of each projection of a layer):
 *     dx      [n_rows, channels]       = dy weight        (bf16, fp32 accumulation)
 *     dweight [out_features, channels] = dy^T x           (fp32)
 * x [n_rows, channels], weight [out_features, channels], dy [n_rows, out_features]: bf16, rows
 * contiguous, read only.  Either output may be NULL (then its operand x or weight may be too).
 * dweight is overwritten, not accumulated into; it is the sum of per-row-range partial results
 * added in a fixed order, so it does not depend on the schedule.
 * Limits: channels % 64 == 0, out_features % 64 == 0, out_features * channels < 2^31; any
 * n_rows >= 1.  workspace: >= aeris_linear_bwd_workspace_bytes(...) bytes
 * (the transposed weight and the partial results), 16-byte aligned, contents undefined before
 * and after.  Errors as elsewhere: AERIS_ERR_ codes, checked before any launch.
 */
size_t aeris_linear_bwd_workspace_bytes(int64_t n_rows, int32_t channels, int32_t out_features);
int aeris_linear_bwd(const void* x, const void* weight, const void* dy, int64_t n_rows,
                     int32_t channels, int32_t out_features, void* dx, float* dweight,
                     void* workspace, size_t workspace_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* AERIS_LAYER_OPS_H */

/*
 * fdg_kernels.h -- C ABI of the individual gfx950 kernels behind the FDG module worker (fdg.h).
 *
 * These are the layer operations a module's forward (Section III-A of arXiv 1906.09108) and its
 * chain-rule backward (Eq. 8, Eq. 9, Eq. 10) are made of, exposed one by one so that each can be
 * checked against its definition and timed against its roofline.  The paper names the layers only by
 * architecture (ResNet / WRN, Table III, optimiser in Section V-A); the arithmetic of each entry point
 * is stated in its comment.
 *
 * All pointers are DEVICE pointers.  Activations are NHWC; "bf16" buffers hold raw bfloat16 (uint16_t
 * storage), "f32" buffers hold float.  Channel counts of bf16 activations must be multiples of 8.
 *
 * SUMS ARRAYS.  Per-channel sums that are taken over many workgroups (the batch-norm statistics, the two sums of a
 * batch-norm backward) live in an opaque "sums array" of fdgk_sums_bytes(c) bytes for c channels (16-byte aligned;
 * two sums per channel).  Every workgroup adds its partial sum, reduced in a fixed order inside the workgroup, into a
 * fixed-point total (two 64-bit words) with integer atomics; integer addition is associative, so the totals -- and with
 * them every result of these entry points -- are the same bits on every run, whatever order the workgroups arrive in
 * (a partial sum of 2^39 or more, in a network that is blowing up, goes to a floating-point word instead).
 * A sums array must be ZERO (all bytes) before its producer runs.  fdgk_sums_read synchronises hip_stream and returns
 * the totals as host doubles: host_out[0..c) = first sum, host_out[c..2c) = second sum.
 * Nothing is allocated; the caller owns every buffer.  `hip_stream` is a hipStream_t (NULL = null
 * stream); calls only enqueue.  Return value: 0 on success, otherwise the hipError_t of the failed
 * check or launch (1 = invalid value for a shape the kernels do not take).
 */
#ifndef FDG_KERNELS_H_
#define FDG_KERNELS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Convolution geometry shared by the three passes: ksize 3 (padding 1) or 1 (padding 0), stride 1 or 2,
 * input [n, h, w, cip] with cip = ci rounded up to 8 (padding channels zero), output
 * [n, ho, wo, co], ho = (h-1)/stride + 1.  co must be a multiple of 8.                            */

/* y = conv(x, w) (+ addend):  y[n,ho,wo,o] = sum_{r,q,i} x[n, ho*s+r-p, wo*s+q-p, i] * w[o,r,q,i].
 *   x_b16 [n,h,w,cip]; w_b16 [co][ksize*ksize][cip]; addend_f32 optional [n,ho,wo,co];
 *   y_f32 / y_b16 optional outputs (at least one);  stats_sums optional sums array of co channels, zero it first:
 *   first sum += sum of bf16(y[..,o]), second sum += sum of bf16(y[..,o])^2 over all pixels -- the
 *   batch-norm statistics of the tensor just written, taken in the epilogue instead of a second pass. */
size_t fdgk_sums_bytes(int c);
int fdgk_sums_read(const void* sums, int c, double* host_out, void* hip_stream);
int fdgk_conv_fwd(const void* x_b16, const void* w_b16, const float* addend_f32, float* y_f32, void* y_b16,
                  void* stats_sums, int n, int h, int w, int ci, int co, int ksize, int stride, void* hip_stream);

/* y = conv3x3(act, w), unit stride, with act = relu(batchnorm(x_raw) [+ res]) worked out on the convolution's input patch
 * on chip (Section III: a module's forward is the plain forward; this fuses two of its steps, it changes no value):
 *   act_b16 [n,h,w,ci] receives relu(gamma * (x_raw - mean) / sqrt(var + eps) + beta [+ res_f32]) in bf16, the convolution
 *   reads exactly those values; act_f32 (optional) receives the same in fp32; res_f32 (optional, [n,h,w,ci]) is a block's
 *   shortcut.  mean and the biased var come from x_sums, the complete sums array of x_raw (fdgk_bn_stats or a producing
 *   convolution's stats_sums); run_mean / run_var (optional, both or neither) take one running-statistics step with
 *   `momentum` (unbiased variance).  y_b16 [n,h,w,co]; stats_sums as fdgk_conv_fwd.
 * Narrow layers only (ci = co in {16, 32, 64}, at most 1024 pixel tiles): fdgk_conv_fwd_bn_applies says (1 / 0); elsewhere
 * the call returns 1 (hipErrorInvalidValue) and enqueues nothing.                                                       */
int fdgk_conv_fwd_bn_applies(int n, int h, int w, int ci, int co, int with_residual);
int fdgk_conv_fwd_bn(const void* x_raw_b16, const void* x_sums, const float* gamma, const float* beta, float eps,
                     const float* res_f32, void* act_b16, float* act_f32, float* run_mean, float* run_var, float momentum,
                     const void* w_b16, void* y_b16, void* stats_sums, int n, int h, int w, int ci, int co, void* hip_stream);

/* Data gradient, the adjoint of fdgk_conv_fwd in x:
 *   dx[n,hi,wi,i] = sum_{o,r,q : hi = ho*s+r-p, wi = wo*s+q-p} dy[n,ho,wo,o] * w[o,r,q,i]  (+ addend)
 *   dy_b16 [n,ho,wo,co]; wt_b16 = the same weights stored [cip][ksize*ksize][co];
 *   addend_f32 optional [n,h,w,cip]; if addmask_b16 ([n,h,w,cip]) is given the addend counts only
 *   where addmask > 0 (a ReLU gate);  dx_f32 / dx_b16 optional outputs [n,h,w,cip].               */
int fdgk_conv_dgrad(const void* dy_b16, const void* wt_b16, const float* addend_f32, const void* addmask_b16,
                    float* dx_f32, void* dx_b16, int n, int h, int w, int ci, int co, int ksize, int stride,
                    void* hip_stream);

/* The data gradient of a 3x3 unit-stride convolution whose incoming gradient dy is the apply half of a batch-norm
 * backward (Eq. 8 / Eq. 9 through BN o conv), done on the convolution's input patch on chip:
 *   dy = gamma * invstd * (g - sum g / M - xhat * sum(g xhat) / M),   dx = data gradient of dy (+ addend as fdgk_conv_dgrad),
 * with g [n,h,w,co] the gated gradient at the batch norm's output (bf16, or fp32 with g_is_f32), x_b16 [n,h,w,co] the batch
 * norm's input, x_sums its forward sums and gsums = (sum g, sum g*x) as fdgk_conv_dgrad_gated / _feeding_next leave them.
 * dy_b16 [n,h,w,co] receives dy (what the weight gradient of the same convolution reads); dgamma = sum g xhat, dbeta = sum g.
 * Narrow layers only (ci = co in {16, 32, 64}, at most 1024 pixel tiles): fdgk_conv_dgrad_bn_applies says (1 / 0); elsewhere
 * the call returns 1 (hipErrorInvalidValue) and enqueues nothing.                                                        */
int fdgk_conv_dgrad_bn_applies(int n, int h, int w, int ci, int co, int g_is_f32);
int fdgk_conv_dgrad_bn(const void* g, int g_is_f32, const void* x_b16, const void* x_sums, const void* gsums, const float* gamma,
                       float eps, void* dy_b16, float* dgamma, float* dbeta, const void* wt_b16, const float* addend_f32,
                       const void* addmask_b16, float* dx_f32, void* dx_b16, int n, int h, int w, int ci, int co,
                       void* hip_stream);

/* The data gradient ending in the ReLU and the batch norm it back-propagates into next (Eq. 8 / Eq. 9 applied to
 * conv o ReLU o BN): with gate_b16 = the ReLU's output and bnx_b16 = the batch norm's input, both [n,h,w,cip],
 *   dx = gate > 0 ? (data gradient + addend) : 0,
 *   first sum of channel i += sum over pixels of bf16(dx[..,i]),  second sum += sum of bf16(dx[..,i]) * bnx[..,i]
 * (gsums: a sums array of cip channels, zero it first): the two reductions of the batch-norm backward, taken in the output stage of the
 * convolution instead of a pass of their own.  The wide kernels and the narrow kernel do this: fdgk_conv_dgrad_gates
 * says (1 / 0) whether a shape is covered, fdgk_conv_dgrad_gated returns hipErrorInvalidValue (1) where it is not.  */
int fdgk_conv_dgrad_gates(int n, int h, int w, int ci, int co, int ksize, int stride);
/* The same for the last data gradient of a block, whose fp32 result plus the shortcut gradient (addend, counted where
 * addmask > 0) is the gradient at the output of the layer BELOW: gate_b16 = that layer's output, bnx_b16 = the input
 * of that layer's last batch norm, and the two sums are taken from the fp32 values (dx_f32 is required; it is what
 * that batch norm's backward reads).  Where a kernel's output stage sums the fp32 values: narrow layers (16 / 32 / 64
 * channels in and out, 3x3, stride 1) and 1x1 unit-stride layers that the two-workgroup form of the wide gather kernel
 * runs (input channels a multiple of 64, at most 1024 output channels of the convolution, 300 tiles or more); 1 elsewhere. */
int fdgk_conv_dgrad_feeding_next(const void* dy_b16, const void* wt_b16, const float* addend_f32, const void* addmask_b16,
                                 const void* gate_b16, const void* bnx_b16, void* gsums, float* dx_f32, void* dx_b16,
                                 int n, int h, int w, int ci, int co, int ksize, int stride, void* hip_stream);
int fdgk_conv_dgrad_gated(const void* dy_b16, const void* wt_b16, const float* addend_f32, const void* gate_b16,
                          const void* bnx_b16, void* gsums, float* dx_f32, void* dx_b16, int n, int h, int w, int ci,
                          int co, int ksize, int stride, void* hip_stream);
/* fdgk_conv_dgrad_gated of a 3x3 stride-2 convolution with the data gradient of the 1x1 stride-2 projection that reads
 * the same input added before the gate, in one launch (a block whose shortcut projects: Eq. 8 summed over the two
 * consumers of the block's first activation):
 *   dx = gate > 0 ? dgrad3x3(dy, wt) + dgrad1x1(dy2, wt2) : 0,   sums as fdgk_conv_dgrad_gated;
 * with gate_b16, bnx_b16 and gsums all NULL: dx = dgrad3x3(dy, wt) + dgrad1x1(dy2, wt2), nothing gated, no sums.
 * dy_b16, dy2_b16 [n,ho,wo,co]; wt_b16 [cip][9][co]; wt2_b16 [cip][1][co]; gate, bnx, dx [n,h,w,cip].
 * fdgk_conv_dgrad_pair_applies says (1 / 0) whether the shape is covered (wide layers, h, w >= 2, co % 64 == 0);
 * elsewhere the call returns 1 (hipErrorInvalidValue) and enqueues nothing.                                       */
int fdgk_conv_dgrad_pair_applies(int n, int h, int w, int ci, int co);
int fdgk_conv_dgrad_gated_pair(const void* dy_b16, const void* wt_b16, const void* dy2_b16, const void* wt2_b16,
                               const void* gate_b16, const void* bnx_b16, void* gsums, float* dx_f32, void* dx_b16, int n,
                               int h, int w, int ci, int co, void* hip_stream);

/* Weight gradient, the adjoint in w, into dw_f32 [co][ksize*ksize][ci]:
 *   dw[o,r,q,i] (+)= sum_{n,ho,wo} dy[n,ho,wo,o] * x[n, ho*s+r-p, wo*s+q-p, i].
 * overwrite == 0: the sum is ADDED to dw (zero it first for the plain gradient); overwrite != 0: dw is
 * written, whatever it held before.  The pixel dimension may be split over workgroups.  With scratch_f32
 * (DEVICE memory, scratch_bytes long, 16-byte aligned, contents irrelevant, may be NULL) the splits store
 * partial arrays there and a second kernel adds them; without it they add with fp32 atomics.
 * fdgk_conv_wgrad_scratch_bytes returns the size that is useful for a shape (0 if the shape never uses
 * scratch).                                                                                            */
size_t fdgk_conv_wgrad_scratch_bytes(int n, int h, int w, int ci, int co, int ksize, int stride);
int fdgk_conv_wgrad(const void* x_b16, const void* dy_b16, float* dw_f32, float* scratch_f32, size_t scratch_bytes,
                    int overwrite,
                    int n, int h, int w, int ci, int co, int ksize, int stride, void* hip_stream);

/* Training-mode batch normalisation over the m rows of x_b16 [m, c].
 * stats:  sums (a sums array of c channels, zero it first): first sum += sum x, second sum += sum x^2.
 * apply:  y = relu?( gamma*(x-mean)/sqrt(var+eps) + beta  [+ res_f32] ), mean/var (biased) from sums; the variance
 *         sum x^2 / m - mean^2 is taken in double on the exact totals.                                  */
int fdgk_bn_stats(const void* x_b16, void* sums, int m, int c, void* hip_stream);
int fdgk_bn_apply(const void* x_b16, const void* sums, const float* gamma, const float* beta,
                  const float* res_f32, float* y_f32, void* y_b16, int m, int c, float eps, int relu,
                  void* hip_stream);

/* Backward of y = relu(bn(x) [+ ...]) given dy (fp32 if dy_is_f32 else bf16) and the ReLU output
 * mask_b16 (gradient passes where mask > 0):  g = dy*[mask>0];  dbeta = sum g;  dgamma = sum g*xhat;
 *   dx = gamma/sqrt(var+eps) * (g - dbeta/m - xhat*dgamma/m)  (+ addend_f32).
 * scratch_sums (a sums array of c channels) must be zero on entry.  dx_f32 / dx_b16 optional.       */
int fdgk_bn_bwd(const void* dy, int dy_is_f32, const void* mask_b16, const void* x_b16, const void* sums,
                const float* gamma, void* scratch_sums, const float* addend_f32, float* dx_f32, void* dx_b16,
                float* dgamma, float* dbeta, int m, int c, float eps, void* hip_stream);

/* fdgk_bn_bwd for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the same computation and the same kernels, but the scratch sums array lives in an
 * array that is part of the library's code object (one copy per GPU, 96 KiB, held until the process ends) instead of a
 * caller-provided scratch_sums.  The call allocates and frees nothing.  Limit: c <= fdgk_bn_bwd_static_max_c() (2048);
 * a larger c (or c % 8 != 0, m <= 0, a required pointer NULL) returns 1 (hipErrorInvalidValue) and enqueues nothing.
 * The array is cleared by a fill kernel on hip_stream at the start of every call and keeps the last call's sums
 * afterwards.  Every call on one GPU shares that GPU's array: calls that may overlap on one GPU (different streams,
 * different host threads) race; order them.  The device that owns hip_stream must be the current device.        */
int fdgk_bn_bwd_static_max_c(void);
int fdgk_bn_bwd_static(const void* dy, int dy_is_f32, const void* mask_b16, const void* x_b16, const void* sums,
                       const float* gamma, const float* addend_f32, float* dx_f32, void* dx_b16, float* dgamma, float* dbeta,
                       int m, int c, float eps, void* hip_stream);

/* The second half of fdgk_bn_bwd for a gradient g_b16 [m, c] that is already gated and whose sums
 * gsums (a sums array: sum g, sum g*x) were left by fdgk_conv_dgrad_gated: dbeta = sum g, dgamma = (sum g*x - mean * sum g) / sqrt(var+eps),
 * dx as in fdgk_bn_bwd.                                                                                */
int fdgk_bn_bwd_gated(const void* g_b16, const void* x_b16, const void* sums, const float* gamma,
                      const void* gsums, const float* addend_f32, float* dx_f32, void* dx_b16, float* dgamma,
                      float* dbeta, int m, int c, float eps, void* hip_stream);

/* Momentum SGD with coupled weight decay (Eq. 11 with the optimiser of Section V-A), count % 4 == 0:
 *   g' = g + wd*theta;  v = mu*v + g';  theta = theta - lr*v.                                       */
int fdgk_sgd(float* theta, float* v, const float* g, size_t count, float lr, float mu, float wd, void* hip_stream);

/* ---- classifier head of a top module (Algorithm I: the top module turns z into the loss and starts the backward) ----
 * All device pointers, fp32 dense unless marked _b16.
 * fdgk_avgpool:    pooled[n, c] = mean over hw of o_b16[n, hw, c]              (c % 8 == 0, n <= 65535)
 * fdgk_fc_fwd:     logits[n, j] = sum_c pooled[n, c] w[j, c] + b[j]
 * fdgk_softmax_ce: y[0] = mean_n (logsumexp(logits[n, :]) - logits[n, label_n]), y[1 + n*j_count + j] = logits[n, j],
 *                  dlogits[n, j] = (softmax(logits[n, :])[j] - [j == label_n]) / n_count; a label outside 0 .. j_count-1 is clamped
 * fdgk_fc_bwd:     dw[j, c] = sum_n dlogits[n, j] pooled[n, c];  db[j] = sum_n dlogits[n, j];  dpooled[n, c] = sum_j dlogits[n, j] w[j, c]
 * fdgk_pool_bwd:   g[n, hw, c] = dpooled[n, c] / hw_count into g_f32 and / or g_b16 (either may be NULL)                       */
int fdgk_avgpool(const void* o_b16, float* pooled, int n, int hw, int c, void* hip_stream);
int fdgk_fc_fwd(const float* pooled, const float* w, const float* b, float* logits, int n, int c, int j, void* hip_stream);
int fdgk_softmax_ce(const float* logits, const int32_t* labels, float* y, float* dlogits, int n, int j, void* hip_stream);
int fdgk_fc_bwd(const float* pooled, const float* w, const float* dlogits, float* dw, float* db, float* dpooled, int n, int c,
                int j, void* hip_stream);
int fdgk_pool_bwd(const float* dpooled, float* g_f32, void* g_b16, int n, int hw, int c, void* hip_stream);

/* ---- layout changes at the module boundary (the C ABI of the module speaks fp32 NCHW, the kernels NHWC) ----
 * fdgk_nchw_to_nhwc: dst[n, hw, cc] = scale * src[n, cc, hw] for cc < c and 0 for c <= cc < cp (cp = the channel pitch, >= c), into
 *                    dst_f32 and / or dst_b16 (rounded to nearest even); scale is the shrinking factor beta of Eq. 15 when the
 *                    tensor is the gradient handed down by the module above, else 1.
 * fdgk_nhwc_to_nchw: dst[n, cc, hw] = src[n, hw, cc] for cc < c, src with channel pitch cp.                                      */
int fdgk_nchw_to_nhwc(const float* src, float* dst_f32, void* dst_b16, int n, int c, int hw, int cp, float scale, void* hip_stream);
int fdgk_nhwc_to_nchw(const float* src, float* dst, int n, int c, int hw, int cp, void* hip_stream);

/* ---- layers of the Tiny-ImageNet networks of Table V (ResNet-18's ImageNet stem, MobileNet-v2's depthwise convolution) ----
 * All tensors NHWC bf16 unless marked, c % 8 == 0.
 * fdgk_im2col7:       col[m, kh, kw, cc] = x8[n, 2 oh - 3 + kh, 2 ow - 3 + kw, cc] for kh < 7, kw < 7 inside the image, else 0
 *                     (m = (n, oh, ow) over the output grid ((h-1)/2+1) x ((w-1)/2+1); kw runs to 8, cc over the 8 stored input
 *                     channels): the 448 operand elements of output pixel m of a 7x7 convolution with stride 2 and padding 3,
 *                     which is then fdgk_conv_fwd / fdgk_conv_wgrad with ksize 1 and ci = 448 on col.
 * fdgk_maxpool3s2:    y[n, ho, wo, c] = max over the 3x3 window at stride 2, padding 1 (windows clipped to the image), into
 *                     y_f32 and / or y_b16.
 * fdgk_maxpool3s2_bwd: dx_f32[n, h, w, c] = sum of dy_f32 over the windows whose first maximum in scan order (rows, then
 *                     columns) is (h, w); x_b16 is the pool's input.
 * fdgk_dwconv3_*:     depthwise 3x3 convolution, padding 1, stride 1 or 2; wt_b16 = [9][c] (tap-major), dw_f32 = [c][9];
 *                     the weight gradient takes scratch of fdgk_dwconv3_wgrad_scratch_bytes and adds its parts in a fixed
 *                     order (same bits every run).                                                                         */
int fdgk_im2col7(const void* x8_b16, void* col_b16, int n, int h, int w, void* hip_stream);
int fdgk_maxpool3s2(const void* x_b16, float* y_f32, void* y_b16, int n, int h, int w, int c, void* hip_stream);
int fdgk_maxpool3s2_bwd(const void* x_b16, const float* dy_f32, float* dx_f32, int n, int h, int w, int c, void* hip_stream);
int fdgk_dwconv3_fwd(const void* x_b16, const void* wt_b16, void* y_b16, int n, int h, int w, int c, int stride, void* hip_stream);
int fdgk_dwconv3_dgrad(const void* dy_b16, const void* wt_b16, void* dx_b16, int n, int h, int w, int c, int stride, void* hip_stream);
size_t fdgk_dwconv3_wgrad_scratch_bytes(int n, int h, int w, int c, int stride);
int fdgk_dwconv3_wgrad(const void* x_b16, const void* dy_b16, float* dw_f32, float* scratch_f32, size_t scratch_bytes, int n, int h,
                       int w, int c, int stride, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* FDG_KERNELS_H_ */

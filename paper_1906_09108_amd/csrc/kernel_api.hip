// C entry points for the individual kernels (declared in include/fdg_kernels.h): argument checks and
// marshalling only.
#include "../../include/fdg_kernels.h"
#include "fdg_internal.h"

using namespace fdg;

namespace {
bool conv_shape(ConvShape& c, int n, int h, int w, int ci, int co, int ksize, int stride) {
  if (n <= 0 || h <= 0 || w <= 0 || ci <= 0 || co <= 0 || co % 8 != 0) return false;
  if ((ksize != 3 && ksize != 1) || (stride != 1 && stride != 2)) return false;
  c = ConvShape{n, h, w, ci, (ci + 7) / 8 * 8, co, ksize * ksize, stride};
  return true;
}
inline hipStream_t st(void* s) { return static_cast<hipStream_t>(s); }
}  // namespace

extern "C" {

int fdgk_conv_fwd(const void* x_b16, const void* w_b16, const float* addend_f32, float* y_f32, void* y_b16,
                  float* stats_f32, int n, int h, int w, int ci, int co, int ksize, int stride, void* hip_stream) {
  ConvShape c;
  if (!x_b16 || !w_b16 || (!y_f32 && !y_b16) || !conv_shape(c, n, h, w, ci, co, ksize, stride)) return (int)hipErrorInvalidValue;
  return (int)conv_forward(c, static_cast<const bf16_t*>(x_b16), static_cast<const bf16_t*>(w_b16), addend_f32, y_f32,
                           static_cast<bf16_t*>(y_b16), stats_f32, st(hip_stream));
}

int fdgk_conv_dgrad(const void* dy_b16, const void* wt_b16, const float* addend_f32, const void* addmask_b16,
                    float* dx_f32, void* dx_b16, int n, int h, int w, int ci, int co, int ksize, int stride,
                    void* hip_stream) {
  ConvShape c;
  if (!dy_b16 || !wt_b16 || (!dx_f32 && !dx_b16) || !conv_shape(c, n, h, w, ci, co, ksize, stride)) return (int)hipErrorInvalidValue;
  return (int)conv_dgrad(c, static_cast<const bf16_t*>(dy_b16), static_cast<const bf16_t*>(wt_b16), addend_f32,
                         static_cast<const bf16_t*>(addmask_b16), dx_f32, static_cast<bf16_t*>(dx_b16), st(hip_stream));
}

int fdgk_conv_dgrad_gated(const void* dy_b16, const void* wt_b16, const float* addend_f32, const void* gate_b16,
                          const void* bnx_b16, float* gsums_f32, float* dx_f32, void* dx_b16, int n, int h, int w, int ci,
                          int co, int ksize, int stride, void* hip_stream) {
  ConvShape c;
  if (!dy_b16 || !wt_b16 || !gate_b16 || !bnx_b16 || !gsums_f32 || (!dx_f32 && !dx_b16) ||
      !conv_shape(c, n, h, w, ci, co, ksize, stride))
    return (int)hipErrorInvalidValue;
  return (int)conv_dgrad_gated(c, static_cast<const bf16_t*>(dy_b16), static_cast<const bf16_t*>(wt_b16), addend_f32,
                               static_cast<const bf16_t*>(gate_b16), static_cast<const bf16_t*>(bnx_b16), gsums_f32, dx_f32,
                               static_cast<bf16_t*>(dx_b16), st(hip_stream));
}

int fdgk_conv_dgrad_feeding_next(const void* dy_b16, const void* wt_b16, const float* addend_f32, const void* addmask_b16,
                                 const void* gate_b16, const void* bnx_b16, float* gsums_f32, float* dx_f32, void* dx_b16,
                                 int n, int h, int w, int ci, int co, int ksize, int stride, void* hip_stream) {
  ConvShape c;
  if (!dy_b16 || !wt_b16 || !gate_b16 || !bnx_b16 || !gsums_f32 || !dx_f32 || !conv_shape(c, n, h, w, ci, co, ksize, stride))
    return (int)hipErrorInvalidValue;
  return (int)conv_dgrad_feeding_next(c, static_cast<const bf16_t*>(dy_b16), static_cast<const bf16_t*>(wt_b16), addend_f32,
                                      static_cast<const bf16_t*>(addmask_b16), static_cast<const bf16_t*>(gate_b16),
                                      static_cast<const bf16_t*>(bnx_b16), gsums_f32, dx_f32, static_cast<bf16_t*>(dx_b16),
                                      st(hip_stream));
}

int fdgk_conv_dgrad_gates(int n, int h, int w, int ci, int co, int ksize, int stride) {
  ConvShape c;
  return conv_shape(c, n, h, w, ci, co, ksize, stride) && conv_dgrad_gates(c) ? 1 : 0;
}

size_t fdgk_conv_wgrad_scratch_bytes(int n, int h, int w, int ci, int co, int ksize, int stride) {
  ConvShape c;
  if (!conv_shape(c, n, h, w, ci, co, ksize, stride)) return 0;
  return conv_wgrad_scratch_bytes(c);
}

int fdgk_conv_wgrad(const void* x_b16, const void* dy_b16, float* dw_f32, float* scratch_f32, size_t scratch_bytes,
                    int overwrite,
                    int n, int h, int w, int ci, int co, int ksize, int stride, void* hip_stream) {
  ConvShape c;
  if (!x_b16 || !dy_b16 || !dw_f32 || !conv_shape(c, n, h, w, ci, co, ksize, stride)) return (int)hipErrorInvalidValue;
  return (int)conv_wgrad(c, static_cast<const bf16_t*>(x_b16), static_cast<const bf16_t*>(dy_b16), dw_f32, scratch_f32,
                         scratch_bytes, overwrite != 0, st(hip_stream));
}

int fdgk_bn_stats(const void* x_b16, float* sums_f32, int m, int c, void* hip_stream) {
  if (!x_b16 || !sums_f32) return (int)hipErrorInvalidValue;
  return (int)launch_bn_stats(static_cast<const bf16_t*>(x_b16), sums_f32, m, c, st(hip_stream));
}

int fdgk_bn_apply(const void* x_b16, const float* sums_f32, const float* gamma, const float* beta,
                  const float* res_f32, float* y_f32, void* y_b16, int m, int c, float eps, int relu,
                  void* hip_stream) {
  if (!x_b16 || !sums_f32 || !gamma || !beta || (!y_f32 && !y_b16)) return (int)hipErrorInvalidValue;
  BnApplyArgs a{};
  a.x = static_cast<const bf16_t*>(x_b16); a.sums = sums_f32; a.gamma = gamma; a.beta = beta; a.res_f32 = res_f32;
  a.out_f32 = y_f32; a.out_b16 = static_cast<bf16_t*>(y_b16);
  a.M = m; a.C = c; a.eps = eps; a.momentum = 0.f; a.relu = relu;
  return (int)launch_bn_apply(a, st(hip_stream));
}

int fdgk_bn_bwd(const void* dy, int dy_is_f32, const void* mask_b16, const void* x_b16, const float* sums_f32,
                const float* gamma, float* scratch_f32, const float* addend_f32, float* dx_f32, void* dx_b16,
                float* dgamma, float* dbeta, int m, int c, float eps, void* hip_stream) {
  if (!dy || !mask_b16 || !x_b16 || !sums_f32 || !gamma || !scratch_f32 || !dgamma || !dbeta) return (int)hipErrorInvalidValue;
  BnBwdArgs a{};
  a.dy = dy; a.dy_is_f32 = dy_is_f32; a.mask = static_cast<const bf16_t*>(mask_b16);
  a.x = static_cast<const bf16_t*>(x_b16); a.sums = sums_f32; a.gamma = gamma; a.bsums = scratch_f32;
  a.addend = addend_f32; a.out_f32 = dx_f32; a.out_b16 = static_cast<bf16_t*>(dx_b16);
  a.dgamma = dgamma; a.dbeta = dbeta; a.M = m; a.C = c; a.eps = eps;
  hipError_t e = launch_bn_bwd_reduce(a, st(hip_stream));
  if (e != hipSuccess) return (int)e;
  return (int)launch_bn_bwd_apply(a, st(hip_stream));
}

int fdgk_bn_bwd_gated(const void* g_b16, const void* x_b16, const float* sums_f32, const float* gamma,
                      const float* gsums_f32, const float* addend_f32, float* dx_f32, void* dx_b16, float* dgamma,
                      float* dbeta, int m, int c, float eps, void* hip_stream) {
  if (!g_b16 || !x_b16 || !sums_f32 || !gamma || !gsums_f32 || !dgamma || !dbeta) return (int)hipErrorInvalidValue;
  BnBwdArgs a{};
  a.dy = g_b16; a.dy_is_f32 = 0; a.mask = nullptr; a.x = static_cast<const bf16_t*>(x_b16); a.sums = sums_f32;
  a.gamma = gamma; a.bsums = const_cast<float*>(gsums_f32);
  a.addend = addend_f32; a.out_f32 = dx_f32; a.out_b16 = static_cast<bf16_t*>(dx_b16);
  a.dgamma = dgamma; a.dbeta = dbeta; a.M = m; a.C = c; a.eps = eps;
  a.dy_gated = 1; a.raw_sums = 1;
  return (int)launch_bn_bwd_apply(a, st(hip_stream));
}

int fdgk_sgd(float* theta, float* v, const float* g, size_t count, float lr, float mu, float wd, void* hip_stream) {
  if (!theta || !v || !g) return (int)hipErrorInvalidValue;
  return (int)launch_sgd(theta, v, g, count, lr, mu, wd, st(hip_stream));
}

}  // extern "C"

// C entry points for the individual kernels (declared in include/fdg_kernels.h): argument checks and
// marshalling only.
#include "../../include/fdg_kernels.h"
#include "fdg_internal.h"

#include <cstring>
#include <mutex>
#include <vector>

using namespace fdg;

namespace {
bool conv_shape(ConvShape& c, int n, int h, int w, int ci, int co, int ksize, int stride) {
  if (n <= 0 || h <= 0 || w <= 0 || ci <= 0 || co <= 0 || co % 8 != 0) return false;
  if ((ksize != 3 && ksize != 1) || (stride != 1 && stride != 2)) return false;
  c = ConvShape{n, h, w, ci, (ci + 7) / 8 * 8, co, ksize * ksize, stride};
  return true;
}
inline hipStream_t st(void* s) { return static_cast<hipStream_t>(s); }

// ---- the scratch of the entry point that allocates nothing (fdgk_bn_bwd_static) ----
// One array per GPU, held until the process ends: the two per-channel sums (exact, two 64-bit words each) of a batch-norm
// backward for up to kStaticMaxC channels: 96 KiB.  In host code the array's name is only a stand-in; its device address is looked up once per
// device (with that device current) and that pointer is what kernels, fills and copies are given.
constexpr int kStaticMaxC = 2048;
constexpr int kStaticMaxDevices = 64;
static __device__ __align__(256) stat_t scratch[2 * kStaticMaxC * kStatWords];
std::mutex g_scratch_lock;
stat_t* g_scratch_ptr[kStaticMaxDevices] = {};

// the current device's copy of `scratch`, or nullptr with *err set
stat_t* static_scratch(hipError_t* err) {
  int dev = -1;
  *err = hipGetDevice(&dev);
  if (*err != hipSuccess) return nullptr;
  if (dev < 0 || dev >= kStaticMaxDevices) { *err = hipErrorInvalidDevice; return nullptr; }
  std::lock_guard<std::mutex> hold(g_scratch_lock);
  if (!g_scratch_ptr[dev]) {
    stat_t* p = nullptr;
    *err = hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch));
    if (*err != hipSuccess || !p) {
      if (*err == hipSuccess) *err = hipErrorInvalidSymbol;
      (void)hipGetLastError();
      return nullptr;
    }
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}
}  // namespace

extern "C" {

int fdgk_conv_fwd(const void* x_b16, const void* w_b16, const float* addend_f32, float* y_f32, void* y_b16,
                  void* stats_sums, int n, int h, int w, int ci, int co, int ksize, int stride, void* hip_stream) {
  ConvShape c;
  if (!x_b16 || !w_b16 || (!y_f32 && !y_b16) || !conv_shape(c, n, h, w, ci, co, ksize, stride)) return (int)hipErrorInvalidValue;
  return (int)conv_forward(c, static_cast<const bf16_t*>(x_b16), static_cast<const bf16_t*>(w_b16), addend_f32, y_f32,
                           static_cast<bf16_t*>(y_b16), static_cast<stat_t*>(stats_sums), st(hip_stream));
}

int fdgk_conv_fwd_bn_applies(int n, int h, int w, int ci, int co, int with_residual) {
  ConvShape c;
  return conv_shape(c, n, h, w, ci, co, 3, 1) && conv_forward_bn_applies(c, with_residual != 0) ? 1 : 0;
}

int fdgk_conv_fwd_bn(const void* x_raw_b16, const void* x_sums, const float* gamma, const float* beta, float eps,
                     const float* res_f32, void* act_b16, float* act_f32, float* run_mean, float* run_var, float momentum,
                     const void* w_b16, void* y_b16, void* stats_sums, int n, int h, int w, int ci, int co, void* hip_stream) {
  ConvShape c;
  if (!x_raw_b16 || !x_sums || !gamma || !beta || !act_b16 || !w_b16 || !y_b16 || !conv_shape(c, n, h, w, ci, co, 3, 1))
    return (int)hipErrorInvalidValue;
  ConvInputBn bn{};
  bn.res_f32 = res_f32; bn.act_out_f32 = act_f32;
  bn.x_raw = static_cast<const bf16_t*>(x_raw_b16); bn.sums = static_cast<const stat_t*>(x_sums); bn.gamma = gamma; bn.beta = beta;
  bn.act_out = static_cast<bf16_t*>(act_b16); bn.run_mean = run_mean; bn.run_var = run_var; bn.eps = eps; bn.momentum = momentum;
  return (int)conv_forward_bn(c, bn, static_cast<const bf16_t*>(w_b16), nullptr, nullptr, static_cast<bf16_t*>(y_b16),
                              static_cast<stat_t*>(stats_sums), st(hip_stream));
}

int fdgk_conv_dgrad_bn_applies(int n, int h, int w, int ci, int co, int g_is_f32) {
  ConvShape c;
  return conv_shape(c, n, h, w, ci, co, 3, 1) && conv_dgrad_bn_applies(c, g_is_f32 != 0) ? 1 : 0;
}

int fdgk_conv_dgrad_bn(const void* g, int g_is_f32, const void* x_b16, const void* x_sums, const void* gsums, const float* gamma,
                       float eps, void* dy_b16, float* dgamma, float* dbeta, const void* wt_b16, const float* addend_f32,
                       const void* addmask_b16, float* dx_f32, void* dx_b16, int n, int h, int w, int ci, int co,
                       void* hip_stream) {
  ConvShape c;
  if (!g || !x_b16 || !x_sums || !gsums || !gamma || !dy_b16 || !dgamma || !dbeta || !wt_b16 || (!dx_f32 && !dx_b16) ||
      !conv_shape(c, n, h, w, ci, co, 3, 1))
    return (int)hipErrorInvalidValue;
  ConvInputBnBwd bn{};
  bn.g = g; bn.g_is_f32 = g_is_f32 ? 1 : 0; bn.x = static_cast<const bf16_t*>(x_b16); bn.sums = static_cast<const stat_t*>(x_sums);
  bn.bsums = static_cast<const stat_t*>(gsums); bn.gamma = gamma; bn.dgamma = dgamma; bn.dbeta = dbeta;
  bn.dy_out = static_cast<bf16_t*>(dy_b16); bn.eps = eps;
  return (int)conv_dgrad_after_bn(c, bn, static_cast<const bf16_t*>(wt_b16), addend_f32, static_cast<const bf16_t*>(addmask_b16),
                                  nullptr, nullptr, nullptr, false, dx_f32, static_cast<bf16_t*>(dx_b16), st(hip_stream));
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
                          const void* bnx_b16, void* gsums, float* dx_f32, void* dx_b16, int n, int h, int w, int ci,
                          int co, int ksize, int stride, void* hip_stream) {
  ConvShape c;
  if (!dy_b16 || !wt_b16 || !gate_b16 || !bnx_b16 || !gsums || (!dx_f32 && !dx_b16) ||
      !conv_shape(c, n, h, w, ci, co, ksize, stride))
    return (int)hipErrorInvalidValue;
  return (int)conv_dgrad_gated(c, static_cast<const bf16_t*>(dy_b16), static_cast<const bf16_t*>(wt_b16), addend_f32,
                               static_cast<const bf16_t*>(gate_b16), static_cast<const bf16_t*>(bnx_b16), static_cast<stat_t*>(gsums), dx_f32,
                               static_cast<bf16_t*>(dx_b16), st(hip_stream));
}

int fdgk_conv_dgrad_pair_applies(int n, int h, int w, int ci, int co) {
  ConvShape c, cp;
  return conv_shape(c, n, h, w, ci, co, 3, 2) && conv_shape(cp, n, h, w, ci, co, 1, 2) && conv_dgrad_pair_applies(c, cp) ? 1 : 0;
}

int fdgk_conv_dgrad_gated_pair(const void* dy_b16, const void* wt_b16, const void* dy2_b16, const void* wt2_b16,
                               const void* gate_b16, const void* bnx_b16, void* gsums, float* dx_f32, void* dx_b16, int n,
                               int h, int w, int ci, int co, void* hip_stream) {
  ConvShape c, cp;
  if (!dy_b16 || !wt_b16 || !dy2_b16 || !wt2_b16 || (!dx_f32 && !dx_b16) ||
      !conv_shape(c, n, h, w, ci, co, 3, 2) || !conv_shape(cp, n, h, w, ci, co, 1, 2))
    return (int)hipErrorInvalidValue;
  return (int)conv_dgrad_gated_pair(c, static_cast<const bf16_t*>(dy_b16), static_cast<const bf16_t*>(wt_b16), cp,
                                    static_cast<const bf16_t*>(dy2_b16), static_cast<const bf16_t*>(wt2_b16),
                                    static_cast<const bf16_t*>(gate_b16), static_cast<const bf16_t*>(bnx_b16),
                                    static_cast<stat_t*>(gsums), dx_f32, static_cast<bf16_t*>(dx_b16), st(hip_stream));
}

int fdgk_conv_dgrad_feeding_next(const void* dy_b16, const void* wt_b16, const float* addend_f32, const void* addmask_b16,
                                 const void* gate_b16, const void* bnx_b16, void* gsums, float* dx_f32, void* dx_b16,
                                 int n, int h, int w, int ci, int co, int ksize, int stride, void* hip_stream) {
  ConvShape c;
  if (!dy_b16 || !wt_b16 || !gate_b16 || !bnx_b16 || !gsums || !dx_f32 || !conv_shape(c, n, h, w, ci, co, ksize, stride))
    return (int)hipErrorInvalidValue;
  return (int)conv_dgrad_feeding_next(c, static_cast<const bf16_t*>(dy_b16), static_cast<const bf16_t*>(wt_b16), addend_f32,
                                      static_cast<const bf16_t*>(addmask_b16), static_cast<const bf16_t*>(gate_b16),
                                      static_cast<const bf16_t*>(bnx_b16), static_cast<stat_t*>(gsums), dx_f32, static_cast<bf16_t*>(dx_b16),
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

size_t fdgk_sums_bytes(int c) { return c > 0 ? stat_elems((size_t)c) * sizeof(stat_t) : 0; }

int fdgk_sums_read(const void* sums, int c, double* host_out, void* hip_stream) {
  if (!sums || !host_out || c <= 0) return (int)hipErrorInvalidValue;
  hipError_t e = hipStreamSynchronize(st(hip_stream));
  if (e != hipSuccess) return (int)e;
  std::vector<stat_t> raw(stat_elems((size_t)c));
  e = hipMemcpy(raw.data(), sums, raw.size() * sizeof(stat_t), hipMemcpyDeviceToHost);
  if (e != hipSuccess) return (int)e;
  for (int i = 0; i < 2 * c; ++i) {   // words: hi [2][c], lo [2][c], big [2][c] (a double)
    double big;
    memcpy(&big, &raw[4 * (size_t)c + i], sizeof(big));
    host_out[i] = big + ((double)raw[i] * 0x1p-11 + (double)raw[2 * (size_t)c + i] * 0x1p-62);
  }
  return 0;
}

int fdgk_bn_stats(const void* x_b16, void* sums, int m, int c, void* hip_stream) {
  if (!x_b16 || !sums) return (int)hipErrorInvalidValue;
  return (int)launch_bn_stats(static_cast<const bf16_t*>(x_b16), static_cast<stat_t*>(sums), m, c, st(hip_stream));
}

int fdgk_bn_apply(const void* x_b16, const void* sums, const float* gamma, const float* beta,
                  const float* res_f32, float* y_f32, void* y_b16, int m, int c, float eps, int relu,
                  void* hip_stream) {
  if (!x_b16 || !sums || !gamma || !beta || (!y_f32 && !y_b16)) return (int)hipErrorInvalidValue;
  BnApplyArgs a{};
  a.x = static_cast<const bf16_t*>(x_b16); a.sums = static_cast<const stat_t*>(sums); a.gamma = gamma; a.beta = beta; a.res_f32 = res_f32;
  a.out_f32 = y_f32; a.out_b16 = static_cast<bf16_t*>(y_b16);
  a.M = m; a.C = c; a.eps = eps; a.momentum = 0.f; a.relu = relu;
  return (int)launch_bn_apply(a, st(hip_stream));
}

int fdgk_bn_bwd(const void* dy, int dy_is_f32, const void* mask_b16, const void* x_b16, const void* sums,
                const float* gamma, void* scratch_sums, const float* addend_f32, float* dx_f32, void* dx_b16,
                float* dgamma, float* dbeta, int m, int c, float eps, void* hip_stream) {
  if (!dy || !mask_b16 || !x_b16 || !sums || !gamma || !scratch_sums || !dgamma || !dbeta) return (int)hipErrorInvalidValue;
  BnBwdArgs a{};
  a.dy = dy; a.dy_is_f32 = dy_is_f32; a.mask = static_cast<const bf16_t*>(mask_b16);
  a.x = static_cast<const bf16_t*>(x_b16); a.sums = static_cast<const stat_t*>(sums); a.gamma = gamma;
  a.bsums = static_cast<stat_t*>(scratch_sums);
  a.addend = addend_f32; a.out_f32 = dx_f32; a.out_b16 = static_cast<bf16_t*>(dx_b16);
  a.dgamma = dgamma; a.dbeta = dbeta; a.M = m; a.C = c; a.eps = eps;
  hipError_t e = launch_bn_bwd_reduce(a, st(hip_stream));
  if (e != hipSuccess) return (int)e;
  return (int)launch_bn_bwd_apply(a, st(hip_stream));
}

int fdgk_bn_bwd_static_max_c(void) { return kStaticMaxC; }

int fdgk_bn_bwd_static(const void* dy, int dy_is_f32, const void* mask_b16, const void* x_b16, const void* sums,
                       const float* gamma, const float* addend_f32, float* dx_f32, void* dx_b16, float* dgamma, float* dbeta,
                       int m, int c, float eps, void* hip_stream) {
  if (!dy || !mask_b16 || !x_b16 || !sums || !gamma || !dgamma || !dbeta) return (int)hipErrorInvalidValue;
  if (c <= 0 || c > kStaticMaxC || c % 8 != 0 || m <= 0) return (int)hipErrorInvalidValue;   // beyond the array: refused
  hipError_t e = hipSuccess;
  stat_t* sums2 = static_scratch(&e);
  if (!sums2) return (int)e;
  // the array keeps the last call's sums: the part this call adds into starts at zero (a fill kernel, so that a
  // caller may record the call into a graph)
  e = launch_fill_zero(sums2, stat_elems((size_t)c) * sizeof(stat_t), st(hip_stream));
  if (e != hipSuccess) return (int)e;
  return fdgk_bn_bwd(dy, dy_is_f32, mask_b16, x_b16, sums, gamma, sums2, addend_f32, dx_f32, dx_b16, dgamma, dbeta, m, c,
                     eps, hip_stream);
}

int fdgk_bn_bwd_gated(const void* g_b16, const void* x_b16, const void* sums, const float* gamma,
                      const void* gsums, const float* addend_f32, float* dx_f32, void* dx_b16, float* dgamma,
                      float* dbeta, int m, int c, float eps, void* hip_stream) {
  if (!g_b16 || !x_b16 || !sums || !gamma || !gsums || !dgamma || !dbeta) return (int)hipErrorInvalidValue;
  BnBwdArgs a{};
  a.dy = g_b16; a.dy_is_f32 = 0; a.mask = nullptr; a.x = static_cast<const bf16_t*>(x_b16);
  a.sums = static_cast<const stat_t*>(sums);
  a.gamma = gamma; a.bsums = const_cast<stat_t*>(static_cast<const stat_t*>(gsums));
  a.addend = addend_f32; a.out_f32 = dx_f32; a.out_b16 = static_cast<bf16_t*>(dx_b16);
  a.dgamma = dgamma; a.dbeta = dbeta; a.M = m; a.C = c; a.eps = eps;
  a.dy_gated = 1; a.raw_sums = 1;
  return (int)launch_bn_bwd_apply(a, st(hip_stream));
}

int fdgk_sgd(float* theta, float* v, const float* g, size_t count, float lr, float mu, float wd, void* hip_stream) {
  if (!theta || !v || !g) return (int)hipErrorInvalidValue;
  return (int)launch_sgd(theta, v, g, count, lr, mu, wd, st(hip_stream));
}

int fdgk_avgpool(const void* o_b16, float* pooled, int n, int hw, int c, void* hip_stream) {
  if (!o_b16 || !pooled || n <= 0 || hw <= 0 || c <= 0) return (int)hipErrorInvalidValue;
  return (int)launch_avgpool(static_cast<const bf16_t*>(o_b16), pooled, n, hw, c, st(hip_stream));
}

int fdgk_fc_fwd(const float* pooled, const float* w, const float* b, float* logits, int n, int c, int j, void* hip_stream) {
  if (!pooled || !w || !b || !logits || n <= 0 || c <= 0 || j <= 0) return (int)hipErrorInvalidValue;
  return (int)launch_fc_fwd(pooled, w, b, logits, n, c, j, st(hip_stream));
}

int fdgk_softmax_ce(const float* logits, const int32_t* labels, float* y, float* dlogits, int n, int j, void* hip_stream) {
  if (!logits || !labels || !y || !dlogits || n <= 0 || j <= 0) return (int)hipErrorInvalidValue;
  return (int)launch_softmax_ce(logits, labels, y, dlogits, n, j, st(hip_stream));
}

int fdgk_fc_bwd(const float* pooled, const float* w, const float* dlogits, float* dw, float* db, float* dpooled, int n, int c,
                int j, void* hip_stream) {
  if (!pooled || !w || !dlogits || !dw || !db || !dpooled || n <= 0 || c <= 0 || j <= 0) return (int)hipErrorInvalidValue;
  return (int)launch_fc_bwd(pooled, w, dlogits, dw, db, dpooled, n, c, j, st(hip_stream));
}

int fdgk_pool_bwd(const float* dpooled, float* g_f32, void* g_b16, int n, int hw, int c, void* hip_stream) {
  if (!dpooled || (!g_f32 && !g_b16) || n <= 0 || hw <= 0 || c <= 0) return (int)hipErrorInvalidValue;
  return (int)launch_pool_bwd(dpooled, g_f32, static_cast<bf16_t*>(g_b16), n, hw, c, st(hip_stream));
}

int fdgk_nchw_to_nhwc(const float* src, float* dst_f32, void* dst_b16, int n, int c, int hw, int cp, float scale, void* hip_stream) {
  if (!src || (!dst_f32 && !dst_b16) || n <= 0 || n > 65535 || c <= 0 || hw <= 0 || cp < c) return (int)hipErrorInvalidValue;
  return (int)launch_nchw_to_nhwc(src, dst_f32, static_cast<bf16_t*>(dst_b16), n, c, hw, cp, scale, st(hip_stream));
}

int fdgk_nhwc_to_nchw(const float* src, float* dst, int n, int c, int hw, int cp, void* hip_stream) {
  if (!src || !dst || n <= 0 || n > 65535 || c <= 0 || hw <= 0 || cp < c) return (int)hipErrorInvalidValue;
  return (int)launch_nhwc_to_nchw(src, dst, n, c, hw, cp, st(hip_stream));
}

int fdgk_im2col7(const void* x8_b16, void* col_b16, int n, int h, int w, void* hip_stream) {
  if (!x8_b16 || !col_b16) return (int)hipErrorInvalidValue;
  return (int)launch_im2col7(static_cast<const bf16_t*>(x8_b16), static_cast<bf16_t*>(col_b16), n, h, w, st(hip_stream));
}

int fdgk_maxpool3s2(const void* x_b16, float* y_f32, void* y_b16, int n, int h, int w, int c, void* hip_stream) {
  if (!x_b16) return (int)hipErrorInvalidValue;
  return (int)launch_maxpool3s2(static_cast<const bf16_t*>(x_b16), y_f32, static_cast<bf16_t*>(y_b16), n, h, w, c, st(hip_stream));
}

int fdgk_maxpool3s2_bwd(const void* x_b16, const float* dy_f32, float* dx_f32, int n, int h, int w, int c, void* hip_stream) {
  if (!x_b16 || !dy_f32 || !dx_f32) return (int)hipErrorInvalidValue;
  return (int)launch_maxpool3s2_bwd(static_cast<const bf16_t*>(x_b16), dy_f32, dx_f32, n, h, w, c, st(hip_stream));
}

int fdgk_dwconv3_fwd(const void* x_b16, const void* wt_b16, void* y_b16, int n, int h, int w, int c, int stride, void* hip_stream) {
  if (!x_b16 || !wt_b16 || !y_b16) return (int)hipErrorInvalidValue;
  return (int)launch_dwconv3_fwd(static_cast<const bf16_t*>(x_b16), static_cast<const bf16_t*>(wt_b16), static_cast<bf16_t*>(y_b16), n, h,
                                 w, c, stride, st(hip_stream));
}

int fdgk_dwconv3_dgrad(const void* dy_b16, const void* wt_b16, void* dx_b16, int n, int h, int w, int c, int stride, void* hip_stream) {
  if (!dy_b16 || !wt_b16 || !dx_b16) return (int)hipErrorInvalidValue;
  return (int)launch_dwconv3_dgrad(static_cast<const bf16_t*>(dy_b16), static_cast<const bf16_t*>(wt_b16), static_cast<bf16_t*>(dx_b16), n,
                                   h, w, c, stride, st(hip_stream));
}

size_t fdgk_dwconv3_wgrad_scratch_bytes(int n, int h, int w, int c, int stride) { return dwconv3_wgrad_scratch_bytes(n, h, w, c, stride); }

int fdgk_dwconv3_wgrad(const void* x_b16, const void* dy_b16, float* dw_f32, float* scratch_f32, size_t scratch_bytes, int n, int h,
                       int w, int c, int stride, void* hip_stream) {
  if (!x_b16 || !dy_b16 || !dw_f32) return (int)hipErrorInvalidValue;
  return (int)launch_dwconv3_wgrad(static_cast<const bf16_t*>(x_b16), static_cast<const bf16_t*>(dy_b16), dw_f32, scratch_f32,
                                   scratch_bytes, n, h, w, c, stride, st(hip_stream));
}

}  // extern "C"

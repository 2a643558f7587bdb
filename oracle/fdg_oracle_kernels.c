/*
 * CPU ORACLE -- TEST INFRASTRUCTURE ONLY.  Nothing on the product path may link or call this file.
 *
 * Layer arithmetic of one FDG module (arXiv 1906.09108), written as the plain definitions with nested
 * loops: the paper names its layers only by architecture (ResNet / WRN, Table III) and states the
 * module-level rule -- back-propagation by the chain rule inside a module (Eq. 8, Eq. 9, Eq. 10) --
 * so every routine here is the textbook forward map of a layer or its exact adjoint.
 *
 * Tensors are dense NCHW.  The element type `real` is chosen at compile time (-DFDG_REAL=float or
 * double; two shared objects are built from this one file).  Long sums (batch statistics, weight
 * gradients, losses) accumulate in double in both builds.  OpenMP only spreads independent outer
 * iterations over cores; it never changes what is computed per element.
 *
 * No blocking, fusion or reordering beyond loop order: each function can be checked against its
 * one-line definition in the comment above it.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#ifndef FDG_REAL
#define FDG_REAL float
#endif
typedef FDG_REAL real;

#define IDX4(n, c, h, w, C, H, W) ((((size_t)(n) * (C) + (c)) * (H) + (h)) * (W) + (w))

static int out_size(int in, int k, int s, int p) { return (in + 2 * p - k) / s + 1; }

/* Output positions o in [*lo, *hi) are exactly those whose input position o*s+off lies in [0, in). */
static void inside_range(int in, int outn, int s, int off, int* lo, int* hi) {
  int a = 0, b = outn;
  while (a < outn && a * s + off < 0) ++a;
  while (b > a && (b - 1) * s + off >= in) --b;
  *lo = a;
  *hi = b;
}

/* y[n,co,ho,wo] = sum_{ci,r,q} x[n,ci,ho*s+r-p,wo*s+q-p] * w[co,ci,r,q]   (zero outside the image) */
void fdgref_conv2d_fwd(const real* x, const real* w, real* y, int N, int Ci, int H, int W, int Co, int k,
                       int s, int p) {
  const int Ho = out_size(H, k, s, p), Wo = out_size(W, k, s, p);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int co = 0; co < Co; ++co) {
      real* yp = y + IDX4(n, co, 0, 0, Co, Ho, Wo);
      for (int i = 0; i < Ho * Wo; ++i) yp[i] = 0;
      for (int ci = 0; ci < Ci; ++ci)
        for (int r = 0; r < k; ++r)
          for (int q = 0; q < k; ++q) {
            const real wv = w[(((size_t)co * Ci + ci) * k + r) * k + q];
            for (int ho = 0; ho < Ho; ++ho) {
              const int h = ho * s + r - p;
              if (h < 0 || h >= H) continue;
              const real* xr = x + IDX4(n, ci, h, 0, Ci, H, W);
              int lo, hi;
              inside_range(W, Wo, s, q - p, &lo, &hi);
              for (int wo = lo; wo < hi; ++wo) yp[ho * Wo + wo] += wv * xr[wo * s + q - p];
            }
          }
    }
}

/* Adjoint of the forward map in x:  dx[n,ci,h,w] = sum_{co,r,q : h=ho*s+r-p, w=wo*s+q-p} dy[n,co,ho,wo] * w[co,ci,r,q] */
void fdgref_conv2d_bwd_data(const real* dy, const real* w, real* dx, int N, int Ci, int H, int W, int Co,
                            int k, int s, int p) {
  const int Ho = out_size(H, k, s, p), Wo = out_size(W, k, s, p);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int ci = 0; ci < Ci; ++ci) {
      real* dxp = dx + IDX4(n, ci, 0, 0, Ci, H, W);
      for (int i = 0; i < H * W; ++i) dxp[i] = 0;
      for (int co = 0; co < Co; ++co)
        for (int r = 0; r < k; ++r)
          for (int q = 0; q < k; ++q) {
            const real wv = w[(((size_t)co * Ci + ci) * k + r) * k + q];
            const real* dyp = dy + IDX4(n, co, 0, 0, Co, Ho, Wo);
            for (int ho = 0; ho < Ho; ++ho) {
              const int h = ho * s + r - p;
              if (h < 0 || h >= H) continue;
              int lo, hi;
              inside_range(W, Wo, s, q - p, &lo, &hi);
              for (int wo = lo; wo < hi; ++wo) dxp[h * W + wo * s + q - p] += wv * dyp[ho * Wo + wo];
            }
          }
    }
}

/* Adjoint in w:  dw[co,ci,r,q] = sum_{n,ho,wo} dy[n,co,ho,wo] * x[n,ci,ho*s+r-p,wo*s+q-p] */
void fdgref_conv2d_bwd_weight(const real* x, const real* dy, real* dw, int N, int Ci, int H, int W, int Co,
                              int k, int s, int p) {
  const int Ho = out_size(H, k, s, p), Wo = out_size(W, k, s, p);
#pragma omp parallel for collapse(2) schedule(static)
  for (int co = 0; co < Co; ++co)
    for (int ci = 0; ci < Ci; ++ci)
      for (int r = 0; r < k; ++r)
        for (int q = 0; q < k; ++q) {
          double acc = 0.0;
          for (int n = 0; n < N; ++n) {
            const real* dyp = dy + IDX4(n, co, 0, 0, Co, Ho, Wo);
            for (int ho = 0; ho < Ho; ++ho) {
              const int h = ho * s + r - p;
              if (h < 0 || h >= H) continue;
              const real* xr = x + IDX4(n, ci, h, 0, Ci, H, W);
              int lo, hi;
              inside_range(W, Wo, s, q - p, &lo, &hi);
              for (int wo = lo; wo < hi; ++wo) acc += (double)dyp[ho * Wo + wo] * (double)xr[wo * s + q - p];
            }
          }
          dw[(((size_t)co * Ci + ci) * k + r) * k + q] = (real)acc;
        }
}

/* Training-mode batch normalisation over (N,H,W) per channel:
 *   mean_c = average of x;  var_c = average of (x-mean_c)^2 (biased, two passes);
 *   invstd_c = 1/sqrt(var_c+eps);  xhat = (x-mean_c)*invstd_c;  y = gamma_c*xhat + beta_c.
 * Also returns mean, biased var and invstd per channel. */
void fdgref_bn_fwd(const real* x, const real* gamma, const real* beta, real* y, real* mean, real* var,
                   real* invstd, int N, int C, int H, int W, double eps) {
  const int HW = H * W;
  const double M = (double)N * HW;
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c) {
    double s = 0.0;
    for (int n = 0; n < N; ++n) {
      const real* xp = x + IDX4(n, c, 0, 0, C, H, W);
      for (int i = 0; i < HW; ++i) s += (double)xp[i];
    }
    const double mu = s / M;
    double v = 0.0;
    for (int n = 0; n < N; ++n) {
      const real* xp = x + IDX4(n, c, 0, 0, C, H, W);
      for (int i = 0; i < HW; ++i) {
        const double d = (double)xp[i] - mu;
        v += d * d;
      }
    }
    v /= M;
    const double is = 1.0 / sqrt(v + eps);
    mean[c] = (real)mu;
    var[c] = (real)v;
    invstd[c] = (real)is;
    for (int n = 0; n < N; ++n) {
      const real* xp = x + IDX4(n, c, 0, 0, C, H, W);
      real* yp = y + IDX4(n, c, 0, 0, C, H, W);
      for (int i = 0; i < HW; ++i) yp[i] = (real)((double)gamma[c] * (((double)xp[i] - mu) * is) + (double)beta[c]);
    }
  }
}

/* Exact adjoint of fdgref_bn_fwd (mean and variance depend on x):
 *   dbeta_c = sum dy;  dgamma_c = sum dy*xhat;
 *   dx = gamma_c*invstd_c*(dy - dbeta_c/M - xhat*dgamma_c/M),  M = N*H*W. */
void fdgref_bn_bwd(const real* x, const real* dy, const real* gamma, const real* mean, const real* invstd,
                   real* dx, real* dgamma, real* dbeta, int N, int C, int H, int W) {
  const int HW = H * W;
  const double M = (double)N * HW;
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c) {
    const double mu = mean[c], is = invstd[c];
    double sb = 0.0, sg = 0.0;
    for (int n = 0; n < N; ++n) {
      const real* xp = x + IDX4(n, c, 0, 0, C, H, W);
      const real* gp = dy + IDX4(n, c, 0, 0, C, H, W);
      for (int i = 0; i < HW; ++i) {
        sb += (double)gp[i];
        sg += (double)gp[i] * (((double)xp[i] - mu) * is);
      }
    }
    dbeta[c] = (real)sb;
    dgamma[c] = (real)sg;
    const double a = (double)gamma[c] * is;
    for (int n = 0; n < N; ++n) {
      const real* xp = x + IDX4(n, c, 0, 0, C, H, W);
      const real* gp = dy + IDX4(n, c, 0, 0, C, H, W);
      real* dp = dx + IDX4(n, c, 0, 0, C, H, W);
      for (int i = 0; i < HW; ++i) {
        const double xh = ((double)xp[i] - mu) * is;
        dp[i] = (real)(a * ((double)gp[i] - sb / M - xh * sg / M));
      }
    }
  }
}

/* y = max(x, 0) */
void fdgref_relu_fwd(const real* x, real* y, size_t count) {
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < count; ++i) y[i] = x[i] > 0 ? x[i] : 0;
}

/* dx = dy where x > 0, else 0 (derivative taken as 0 at x == 0) */
void fdgref_relu_bwd(const real* x, const real* dy, real* dx, size_t count) {
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < count; ++i) dx[i] = x[i] > 0 ? dy[i] : 0;
}

/* ---- layers of the Tiny-ImageNet networks of Table V (ResNet-18's ImageNet stem, MobileNet-v2's blocks) ---- */

/* y = min(max(x, 0), 6) */
void fdgref_relu6_fwd(const real* x, real* y, size_t count) {
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < count; ++i) y[i] = x[i] > 0 ? (x[i] < 6 ? x[i] : 6) : 0;
}

/* dx = dy where 0 < x < 6, else 0 (derivative taken as 0 at both corners).  x may be the layer's input or its
 * clamped output: the two are equal exactly where the test holds. */
void fdgref_relu6_bwd(const real* x, const real* dy, real* dx, size_t count) {
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < count; ++i) dx[i] = (x[i] > 0 && x[i] < 6) ? dy[i] : 0;
}

/* Max-pool k x k, stride s, padding p (padding never wins: windows are clipped to the image):
 *   y[n,c,ho,wo] = max over the window of x.  Among equal maxima the FIRST in scan order (rows, then columns) is the
 *   one the gradient goes to. */
void fdgref_maxpool_fwd(const real* x, real* y, int N, int C, int H, int W, int k, int s, int p) {
  const int Ho = out_size(H, k, s, p), Wo = out_size(W, k, s, p);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int c = 0; c < C; ++c) {
      const real* xp = x + IDX4(n, c, 0, 0, C, H, W);
      real* yp = y + IDX4(n, c, 0, 0, C, Ho, Wo);
      for (int ho = 0; ho < Ho; ++ho)
        for (int wo = 0; wo < Wo; ++wo) {
          int have = 0;
          real best = 0;
          for (int r = 0; r < k; ++r)
            for (int q = 0; q < k; ++q) {
              const int h = ho * s + r - p, w = wo * s + q - p;
              if (h < 0 || h >= H || w < 0 || w >= W) continue;
              if (!have || xp[h * W + w] > best) { best = xp[h * W + w]; have = 1; }
            }
          yp[ho * Wo + wo] = best;
        }
    }
}

/* dx[n,c,h,w] = sum of dy over the windows whose (first) maximum sits at (h,w) */
void fdgref_maxpool_bwd(const real* x, const real* dy, real* dx, int N, int C, int H, int W, int k, int s, int p) {
  const int Ho = out_size(H, k, s, p), Wo = out_size(W, k, s, p);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int c = 0; c < C; ++c) {
      const real* xp = x + IDX4(n, c, 0, 0, C, H, W);
      const real* dyp = dy + IDX4(n, c, 0, 0, C, Ho, Wo);
      real* dxp = dx + IDX4(n, c, 0, 0, C, H, W);
      for (int i = 0; i < H * W; ++i) dxp[i] = 0;
      for (int ho = 0; ho < Ho; ++ho)
        for (int wo = 0; wo < Wo; ++wo) {
          int at = -1;
          real best = 0;
          for (int r = 0; r < k; ++r)
            for (int q = 0; q < k; ++q) {
              const int h = ho * s + r - p, w = wo * s + q - p;
              if (h < 0 || h >= H || w < 0 || w >= W) continue;
              if (at < 0 || xp[h * W + w] > best) { best = xp[h * W + w]; at = h * W + w; }
            }
          if (at >= 0) dxp[at] += dyp[ho * Wo + wo];
        }
    }
}

/* Depthwise convolution (one k x k filter per channel, w[c,r,q]):
 *   y[n,c,ho,wo] = sum_{r,q} x[n,c,ho*s+r-p,wo*s+q-p] * w[c,r,q] */
void fdgref_dwconv2d_fwd(const real* x, const real* w, real* y, int N, int C, int H, int W, int k, int s, int p) {
  const int Ho = out_size(H, k, s, p), Wo = out_size(W, k, s, p);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int c = 0; c < C; ++c) {
      const real* xp = x + IDX4(n, c, 0, 0, C, H, W);
      real* yp = y + IDX4(n, c, 0, 0, C, Ho, Wo);
      for (int ho = 0; ho < Ho; ++ho)
        for (int wo = 0; wo < Wo; ++wo) {
          double acc = 0.0;
          for (int r = 0; r < k; ++r)
            for (int q = 0; q < k; ++q) {
              const int h = ho * s + r - p, ww = wo * s + q - p;
              if (h < 0 || h >= H || ww < 0 || ww >= W) continue;
              acc += (double)xp[h * W + ww] * (double)w[((size_t)c * k + r) * k + q];
            }
          yp[ho * Wo + wo] = (real)acc;
        }
    }
}

/* dx[n,c,h,w] = sum_{r,q : h=ho*s+r-p, w=wo*s+q-p} dy[n,c,ho,wo] * w[c,r,q] */
void fdgref_dwconv2d_bwd_data(const real* dy, const real* w, real* dx, int N, int C, int H, int W, int k, int s, int p) {
  const int Ho = out_size(H, k, s, p), Wo = out_size(W, k, s, p);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int c = 0; c < C; ++c) {
      const real* dyp = dy + IDX4(n, c, 0, 0, C, Ho, Wo);
      real* dxp = dx + IDX4(n, c, 0, 0, C, H, W);
      for (int i = 0; i < H * W; ++i) dxp[i] = 0;
      for (int ho = 0; ho < Ho; ++ho)
        for (int wo = 0; wo < Wo; ++wo)
          for (int r = 0; r < k; ++r)
            for (int q = 0; q < k; ++q) {
              const int h = ho * s + r - p, ww = wo * s + q - p;
              if (h < 0 || h >= H || ww < 0 || ww >= W) continue;
              dxp[h * W + ww] += dyp[ho * Wo + wo] * w[((size_t)c * k + r) * k + q];
            }
    }
}

/* dw[c,r,q] = sum_{n,ho,wo} dy[n,c,ho,wo] * x[n,c,ho*s+r-p,wo*s+q-p] */
void fdgref_dwconv2d_bwd_weight(const real* x, const real* dy, real* dw, int N, int C, int H, int W, int k, int s, int p) {
  const int Ho = out_size(H, k, s, p), Wo = out_size(W, k, s, p);
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c)
    for (int r = 0; r < k; ++r)
      for (int q = 0; q < k; ++q) {
        double acc = 0.0;
        for (int n = 0; n < N; ++n) {
          const real* xp = x + IDX4(n, c, 0, 0, C, H, W);
          const real* dyp = dy + IDX4(n, c, 0, 0, C, Ho, Wo);
          for (int ho = 0; ho < Ho; ++ho)
            for (int wo = 0; wo < Wo; ++wo) {
              const int h = ho * s + r - p, ww = wo * s + q - p;
              if (h < 0 || h >= H || ww < 0 || ww >= W) continue;
              acc += (double)dyp[ho * Wo + wo] * (double)xp[h * W + ww];
            }
        }
        dw[((size_t)c * k + r) * k + q] = (real)acc;
      }
}

/* p[n,c] = average over (h,w) of x[n,c,h,w] */
void fdgref_avgpool_fwd(const real* x, real* p, int N, int C, int H, int W) {
  const int HW = H * W;
#pragma omp parallel for schedule(static)
  for (int nc = 0; nc < N * C; ++nc) {
    double s = 0.0;
    for (int i = 0; i < HW; ++i) s += (double)x[(size_t)nc * HW + i];
    p[nc] = (real)(s / HW);
  }
}

/* dx[n,c,h,w] = dp[n,c] / (H*W) */
void fdgref_avgpool_bwd(const real* dp, real* dx, int N, int C, int H, int W) {
  const int HW = H * W;
#pragma omp parallel for schedule(static)
  for (int nc = 0; nc < N * C; ++nc)
    for (int i = 0; i < HW; ++i) dx[(size_t)nc * HW + i] = (real)((double)dp[nc] / HW);
}

/* logits[n,j] = b[j] + sum_c p[n,c]*Wt[j,c] */
void fdgref_fc_fwd(const real* p, const real* Wt, const real* b, real* logits, int N, int C, int J) {
  for (int n = 0; n < N; ++n)
    for (int j = 0; j < J; ++j) {
      double s = (double)b[j];
      for (int c = 0; c < C; ++c) s += (double)p[(size_t)n * C + c] * (double)Wt[(size_t)j * C + c];
      logits[(size_t)n * J + j] = (real)s;
    }
}

/* dWt[j,c] = sum_n dl[n,j]*p[n,c];  db[j] = sum_n dl[n,j];  dp[n,c] = sum_j dl[n,j]*Wt[j,c] */
void fdgref_fc_bwd(const real* p, const real* Wt, const real* dl, real* dWt, real* db, real* dp, int N, int C,
                   int J) {
  for (int j = 0; j < J; ++j) {
    double sb = 0.0;
    for (int n = 0; n < N; ++n) sb += (double)dl[(size_t)n * J + j];
    db[j] = (real)sb;
    for (int c = 0; c < C; ++c) {
      double s = 0.0;
      for (int n = 0; n < N; ++n) s += (double)dl[(size_t)n * J + j] * (double)p[(size_t)n * C + c];
      dWt[(size_t)j * C + c] = (real)s;
    }
  }
  for (int n = 0; n < N; ++n)
    for (int c = 0; c < C; ++c) {
      double s = 0.0;
      for (int j = 0; j < J; ++j) s += (double)dl[(size_t)n * J + j] * (double)Wt[(size_t)j * C + c];
      dp[(size_t)n * C + c] = (real)s;
    }
}

/* Softmax cross-entropy, mean over the batch, with the log-sum-exp shifted by the row maximum:
 *   loss = (1/N) sum_n [ log sum_j exp(l[n,j]) - l[n,label_n] ];
 *   dl[n,j] = (softmax(l[n,:])[j] - [j == label_n]) / N.      Returns the loss. */
double fdgref_softmax_ce(const real* logits, const int32_t* labels, real* dl, int N, int J) {
  double loss = 0.0;
  for (int n = 0; n < N; ++n) {
    const real* l = logits + (size_t)n * J;
    double mx = (double)l[0];
    for (int j = 1; j < J; ++j)
      if ((double)l[j] > mx) mx = (double)l[j];
    double z = 0.0;
    for (int j = 0; j < J; ++j) z += exp((double)l[j] - mx);
    const double lse = mx + log(z);
    loss += lse - (double)l[labels[n]];
    for (int j = 0; j < J; ++j) {
      const double sm = exp((double)l[j] - lse);
      dl[(size_t)n * J + j] = (real)((sm - (j == labels[n] ? 1.0 : 0.0)) / N);
    }
  }
  return loss / N;
}

/* Momentum SGD with coupled L2 weight decay on the CURRENT parameters (Eq. 11 with the optimiser of
 * Section V-A):  g' = g + wd*theta;  v = mu*v + g';  theta = theta - lr*v. */
void fdgref_sgd_momentum(real* theta, real* v, const real* g, size_t count, double lr, double mu, double wd) {
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < count; ++i) {
    const real gp = (real)((double)g[i] + wd * (double)theta[i]);
    v[i] = (real)(mu * (double)v[i] + (double)gp);
    theta[i] = (real)((double)theta[i] - lr * (double)v[i]);
  }
}

/* Round every element to the nearest bfloat16 (8 significand bits, ties to even) and store it back in
 * `real`.  This is the storage precision of the MFMA operands and saved activations of the bf16 path;
 * the oracle applies it only in its "bf16 storage" mode, at the points where that path stores bf16. */
void fdgref_round_bf16(real* x, size_t count) {
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < count; ++i) {
    float f = (float)x[i];
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7f800000u) != 0x7f800000u) {          /* finite: add half an ulp of bf16, ties to even */
      u += 0x7fffu + ((u >> 16) & 1u);
      u &= 0xffff0000u;
    }
    memcpy(&f, &u, sizeof f);
    x[i] = (real)f;
  }
}

int fdgref_sizeof_real(void) { return (int)sizeof(real); }

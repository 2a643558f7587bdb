// Kernels of the layers that only the Tiny-ImageNet networks of Table V need: the ImageNet stem of ResNet-18 (7x7
// convolution of stride 2 as row gathers + a 1x1 contraction, 3x3 max-pool of stride 2) and the depthwise 3x3 convolution of
// MobileNet-v2's inverted residual block.  All of them move each tensor once and do a handful of operations per element:
// HBM-bound.  Tensors are NHWC; a thread owns 8 consecutive channels of one pixel (one 16-byte bf16 access).
#include "fdg_internal.h"

namespace fdg {
namespace {

__device__ __forceinline__ float lo16(uint32_t u) { return __builtin_bit_cast(float, u << 16); }
__device__ __forceinline__ float hi16(uint32_t u) { return __builtin_bit_cast(float, u & 0xffff0000u); }
__device__ __forceinline__ void unpack(const uint4& u, float (&f)[8]) {
  f[0] = lo16(u.x); f[1] = hi16(u.x); f[2] = lo16(u.y); f[3] = hi16(u.y);
  f[4] = lo16(u.z); f[5] = hi16(u.z); f[6] = lo16(u.w); f[7] = hi16(u.w);
}
__device__ __forceinline__ uint32_t pack2(float a, float b) {
  const bf16_t l = (bf16_t)a, h = (bf16_t)b;
  return (uint32_t)__builtin_bit_cast(uint16_t, l) | ((uint32_t)__builtin_bit_cast(uint16_t, h) << 16);
}
__device__ __forceinline__ uint4 pack(const float (&f)[8]) {
  return make_uint4(pack2(f[0], f[1]), pack2(f[2], f[3]), pack2(f[4], f[5]), pack2(f[6], f[7]));
}
__device__ __forceinline__ void store_f32(float* p, const float (&f)[8]) {
  *reinterpret_cast<float4*>(p) = make_float4(f[0], f[1], f[2], f[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(f[4], f[5], f[6], f[7]);
}
__device__ __forceinline__ void load_f32(const float* p, float (&f)[8]) {
  const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
}
int grid_for(size_t threads) {
  const size_t b = (threads + 255) / 256;
  return (int)(b < 1 ? 1 : b);
}

// ---- 7x7 convolution of stride 2, padding 3, over an input of 8 stored channels --------------------------------
// col[m, kh, kw, c] = x[n, 2 oh - 3 + kh, 2 ow - 3 + kw, c] (m = (n, oh, ow); kh < 7; kw < 8, the column kw = 7 is zero, as is
// everything outside the image).  Row m of col is the 448-element operand of output pixel m: the convolution is
// col [M, 448] times w [Co, 448] and its weight gradient dy^T col, which the 1x1 kernels compute.
__global__ __launch_bounds__(256) void im2col7_kernel(const uint4* __restrict__ x, uint4* __restrict__ col, int N, int H, int W,
                                                      int Ho, int Wo) {
  const size_t total = (size_t)N * Ho * Wo * 56;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int kw = (int)(i % 8), kh = (int)((i / 8) % 7);
  const size_t m = i / 56;
  const int ow = (int)(m % Wo), oh = (int)((m / Wo) % Ho), n = (int)(m / ((size_t)Wo * Ho));
  const int h = 2 * oh - 3 + kh, w = 2 * ow - 3 + kw;
  uint4 v = make_uint4(0u, 0u, 0u, 0u);
  if (kw < 7 && h >= 0 && h < H && w >= 0 && w < W) v = x[((size_t)n * H + h) * W + w];
  col[i] = v;
}

// ---- 3x3 max-pool of stride 2, padding 1 --------------------------------------------------------------------------
__global__ __launch_bounds__(256) void maxpool3s2_kernel(const bf16_t* __restrict__ x, float* __restrict__ y_f32,
                                                         bf16_t* __restrict__ y_b16, int N, int H, int W, int C, int Ho, int Wo) {
  const int CG = C / 8;
  const size_t total = (size_t)N * Ho * Wo * CG;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int cg = (int)(i % CG);
  const size_t m = i / CG;
  const int wo = (int)(m % Wo), ho = (int)((m / Wo) % Ho), n = (int)(m / ((size_t)Wo * Ho));
  float best[8];
  bool have = false;
#pragma unroll
  for (int r = 0; r < 3; ++r)
#pragma unroll
    for (int q = 0; q < 3; ++q) {
      const int h = 2 * ho - 1 + r, w = 2 * wo - 1 + q;
      if (h < 0 || h >= H || w < 0 || w >= W) continue;
      float f[8];
      unpack(*reinterpret_cast<const uint4*>(x + (((size_t)n * H + h) * W + w) * C + cg * 8), f);
#pragma unroll
      for (int k = 0; k < 8; ++k) best[k] = (!have || f[k] > best[k]) ? f[k] : best[k];
      have = true;
    }
  const size_t o = m * C + cg * 8;
  if (y_f32) store_f32(y_f32 + o, best);
  if (y_b16) *reinterpret_cast<uint4*>(y_b16 + o) = pack(best);   // exact: a maximum of bf16 values
}

// dx[n, h, w, c] = sum of dy over the windows whose FIRST maximum (rows, then columns) is the cell (h, w).  One thread per
// input cell and 8 channels; it looks at the (at most four) windows that contain the cell.
__global__ __launch_bounds__(256) void maxpool3s2_bwd_kernel(const bf16_t* __restrict__ x, const float* __restrict__ dy,
                                                             float* __restrict__ dx, int N, int H, int W, int C, int Ho, int Wo) {
  const int CG = C / 8;
  const size_t total = (size_t)N * H * W * CG;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int cg = (int)(i % CG);
  const size_t pix = i / CG;
  const int w0 = (int)(pix % W), h0 = (int)((pix / W) % H), n = (int)(pix / ((size_t)W * H));
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  // windows ho with 2 ho - 1 <= h0 <= 2 ho + 1
  const int ho_lo = h0 / 2, ho_hi = (h0 + 1) / 2, wo_lo = w0 / 2, wo_hi = (w0 + 1) / 2;
  for (int ho = ho_lo; ho <= ho_hi; ++ho) {
    if (ho >= Ho) continue;
    for (int wo = wo_lo; wo <= wo_hi; ++wo) {
      if (wo >= Wo) continue;
      float best[8];
      bool mine[8] = {false, false, false, false, false, false, false, false};
      bool have = false;
#pragma unroll
      for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int q = 0; q < 3; ++q) {
          const int h = 2 * ho - 1 + r, w = 2 * wo - 1 + q;
          if (h < 0 || h >= H || w < 0 || w >= W) continue;
          float f[8];
          unpack(*reinterpret_cast<const uint4*>(x + (((size_t)n * H + h) * W + w) * C + cg * 8), f);
          const bool me = h == h0 && w == w0;
#pragma unroll
          for (int k = 0; k < 8; ++k)
            if (!have || f[k] > best[k]) { best[k] = f[k]; mine[k] = me; }
          have = true;
        }
      float g[8];
      load_f32(dy + (((size_t)n * Ho + ho) * Wo + wo) * C + cg * 8, g);
#pragma unroll
      for (int k = 0; k < 8; ++k)
        if (mine[k]) acc[k] += g[k];
    }
  }
  store_f32(dx + pix * C + cg * 8, acc);
}

// ---- depthwise 3x3 convolution, padding 1, stride 1 or 2; wt = [9][C] bf16 (tap-major) ------------------------------
__global__ __launch_bounds__(256) void dwconv3_fwd_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ wt,
                                                          bf16_t* __restrict__ y, int N, int H, int W, int C, int Ho, int Wo, int stride) {
  const int CG = C / 8;
  const size_t total = (size_t)N * Ho * Wo * CG;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int cg = (int)(i % CG);
  const size_t m = i / CG;
  const int wo = (int)(m % Wo), ho = (int)((m / Wo) % Ho), n = (int)(m / ((size_t)Wo * Ho));
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int r = 0; r < 3; ++r)
#pragma unroll
    for (int q = 0; q < 3; ++q) {
      const int h = ho * stride - 1 + r, w = wo * stride - 1 + q;
      if (h < 0 || h >= H || w < 0 || w >= W) continue;
      float f[8], k[8];
      unpack(*reinterpret_cast<const uint4*>(x + (((size_t)n * H + h) * W + w) * C + cg * 8), f);
      unpack(*reinterpret_cast<const uint4*>(wt + (size_t)(r * 3 + q) * C + cg * 8), k);
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] += f[j] * k[j];
    }
  *reinterpret_cast<uint4*>(y + m * C + cg * 8) = pack(acc);
}

// dx[n, h, w, c] = sum over taps (r, q) and output cells with ho * stride - 1 + r = h, wo * stride - 1 + q = w of dy * w[r][q][c]
__global__ __launch_bounds__(256) void dwconv3_dgrad_kernel(const bf16_t* __restrict__ dy, const bf16_t* __restrict__ wt,
                                                            bf16_t* __restrict__ dx, float* __restrict__ dx_f32, int N, int H, int W, int C,
                                                            int Ho, int Wo, int stride) {
  const int CG = C / 8;
  const size_t total = (size_t)N * H * W * CG;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int cg = (int)(i % CG);
  const size_t pix = i / CG;
  const int w0 = (int)(pix % W), h0 = (int)((pix / W) % H), n = (int)(pix / ((size_t)W * H));
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int r = 0; r < 3; ++r)
#pragma unroll
    for (int q = 0; q < 3; ++q) {
      const int hs = h0 + 1 - r, ws = w0 + 1 - q;
      if (hs < 0 || ws < 0 || hs % stride != 0 || ws % stride != 0) continue;
      const int ho = hs / stride, wo = ws / stride;
      if (ho >= Ho || wo >= Wo) continue;
      float g[8], k[8];
      unpack(*reinterpret_cast<const uint4*>(dy + (((size_t)n * Ho + ho) * Wo + wo) * C + cg * 8), g);
      unpack(*reinterpret_cast<const uint4*>(wt + (size_t)(r * 3 + q) * C + cg * 8), k);
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] += g[j] * k[j];
    }
  if (dx) *reinterpret_cast<uint4*>(dx + pix * C + cg * 8) = pack(acc);
  if (dx_f32) {
    float* o = dx_f32 + pix * C + cg * 8;
    *reinterpret_cast<float4*>(o) = make_float4(acc[0], acc[1], acc[2], acc[3]);
    *reinterpret_cast<float4*>(o + 4) = make_float4(acc[4], acc[5], acc[6], acc[7]);
  }
}

// Weight gradient, first pass: workgroup (channel block bx of 8 groups of 8 channels, pixel chunk by) adds dy * x over its
// output pixels for all nine taps; the 32 pixel lanes of a channel group are summed through LDS in a fixed order and the
// result goes to part[by][tap][c].  Second pass: dw[c][tap] = sum over chunks, in order.
__global__ __launch_bounds__(256) void dwconv3_wgrad_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dy,
                                                            float* __restrict__ part, int N, int H, int W, int C, int Ho, int Wo,
                                                            int stride, int pixels_per_chunk) {
  __shared__ float red[32][65];
  const int CG = C / 8;
  const int cgl = threadIdx.x & 7, pl = threadIdx.x >> 3;
  const int cg = blockIdx.x * 8 + cgl;
  const size_t M = (size_t)N * Ho * Wo;
  const size_t m_lo = (size_t)blockIdx.y * pixels_per_chunk;
  const size_t m_hi = m_lo + pixels_per_chunk < M ? m_lo + pixels_per_chunk : M;
  float acc[9][8];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[t][j] = 0.f;
  if (cg < CG) {
    for (size_t m = m_lo + pl; m < m_hi; m += 32) {
      const int wo = (int)(m % Wo), ho = (int)((m / Wo) % Ho), n = (int)(m / ((size_t)Wo * Ho));
      float g[8];
      unpack(*reinterpret_cast<const uint4*>(dy + m * C + cg * 8), g);
#pragma unroll
      for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int q = 0; q < 3; ++q) {
          const int h = ho * stride - 1 + r, w = wo * stride - 1 + q;
          if (h < 0 || h >= H || w < 0 || w >= W) continue;
          float f[8];
          unpack(*reinterpret_cast<const uint4*>(x + (((size_t)n * H + h) * W + w) * C + cg * 8), f);
#pragma unroll
          for (int j = 0; j < 8; ++j) acc[r * 3 + q][j] += g[j] * f[j];
        }
    }
  }
#pragma unroll
  for (int t = 0; t < 9; ++t) {
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 8; ++j) red[pl][cgl * 8 + j] = acc[t][j];
    __syncthreads();
    if (threadIdx.x < 64) {
      const int c = blockIdx.x * 64 + threadIdx.x;
      if (c < C) {
        float s = 0.f;
#pragma unroll 8
        for (int k = 0; k < 32; ++k) s += red[k][threadIdx.x];
        part[((size_t)blockIdx.y * 9 + t) * C + c] = s;
      }
    }
  }
}
__global__ __launch_bounds__(256) void dwconv3_wgrad_reduce_kernel(const float* __restrict__ part, float* __restrict__ dw, int C,
                                                                   int chunks) {
  const int i = blockIdx.x * 256 + threadIdx.x;   // (tap, c)
  if (i >= 9 * C) return;
  const int t = i / C, c = i % C;
  float s = 0.f;
  for (int k = 0; k < chunks; ++k) s += part[((size_t)k * 9 + t) * C + c];
  dw[(size_t)c * 9 + t] = s;
}

int dw_chunks(int N, int Ho, int Wo, int C) {
  const size_t M = (size_t)N * Ho * Wo;
  const int cblocks = (C / 8 + 7) / 8;
  size_t chunks = (1024 + cblocks - 1) / cblocks;
  const size_t most = (M + 255) / 256;            // at least 256 pixels per chunk
  if (chunks > most) chunks = most;
  return (int)(chunks < 1 ? 1 : chunks);
}

}  // namespace

hipError_t launch_im2col7(const bf16_t* x8, bf16_t* col, int N, int H, int W, hipStream_t s) {
  if (N <= 0 || H <= 0 || W <= 0) return hipErrorInvalidValue;
  const int Ho = (H - 1) / 2 + 1, Wo = (W - 1) / 2 + 1;
  const size_t total = (size_t)N * Ho * Wo * 56;
  if (total >= ((size_t)1 << 31) * 256) return hipErrorInvalidValue;
  hipLaunchKernelGGL(im2col7_kernel, dim3(grid_for(total)), dim3(256), 0, s, reinterpret_cast<const uint4*>(x8),
                     reinterpret_cast<uint4*>(col), N, H, W, Ho, Wo);
  return hipGetLastError();
}

hipError_t launch_maxpool3s2(const bf16_t* x, float* y_f32, bf16_t* y_b16, int N, int H, int W, int C, hipStream_t s) {
  if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || C % 8 != 0 || (!y_f32 && !y_b16)) return hipErrorInvalidValue;
  const int Ho = (H - 1) / 2 + 1, Wo = (W - 1) / 2 + 1;
  hipLaunchKernelGGL(maxpool3s2_kernel, dim3(grid_for((size_t)N * Ho * Wo * (C / 8))), dim3(256), 0, s, x, y_f32, y_b16, N, H, W, C, Ho, Wo);
  return hipGetLastError();
}

hipError_t launch_maxpool3s2_bwd(const bf16_t* x, const float* dy, float* dx, int N, int H, int W, int C, hipStream_t s) {
  if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || C % 8 != 0) return hipErrorInvalidValue;
  const int Ho = (H - 1) / 2 + 1, Wo = (W - 1) / 2 + 1;
  hipLaunchKernelGGL(maxpool3s2_bwd_kernel, dim3(grid_for((size_t)N * H * W * (C / 8))), dim3(256), 0, s, x, dy, dx, N, H, W, C, Ho, Wo);
  return hipGetLastError();
}

hipError_t launch_dwconv3_fwd(const bf16_t* x, const bf16_t* wt, bf16_t* y, int N, int H, int W, int C, int stride, hipStream_t s) {
  if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || C % 8 != 0 || (stride != 1 && stride != 2)) return hipErrorInvalidValue;
  const int Ho = (H - 1) / stride + 1, Wo = (W - 1) / stride + 1;
  hipLaunchKernelGGL(dwconv3_fwd_kernel, dim3(grid_for((size_t)N * Ho * Wo * (C / 8))), dim3(256), 0, s, x, wt, y, N, H, W, C, Ho, Wo, stride);
  return hipGetLastError();
}

hipError_t launch_dwconv3_dgrad(const bf16_t* dy, const bf16_t* wt, bf16_t* dx, int N, int H, int W, int C, int stride, hipStream_t s,
                                float* dx_f32) {
  if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || C % 8 != 0 || (stride != 1 && stride != 2) || (!dx && !dx_f32)) return hipErrorInvalidValue;
  const int Ho = (H - 1) / stride + 1, Wo = (W - 1) / stride + 1;
  hipLaunchKernelGGL(dwconv3_dgrad_kernel, dim3(grid_for((size_t)N * H * W * (C / 8))), dim3(256), 0, s, dy, wt, dx, dx_f32, N, H, W, C, Ho, Wo,
                     stride);
  return hipGetLastError();
}

size_t dwconv3_wgrad_scratch_bytes(int N, int H, int W, int C, int stride) {
  if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || C % 8 != 0 || (stride != 1 && stride != 2)) return 0;
  const int Ho = (H - 1) / stride + 1, Wo = (W - 1) / stride + 1;
  return (size_t)dw_chunks(N, Ho, Wo, C) * 9 * C * sizeof(float);
}

hipError_t launch_dwconv3_wgrad(const bf16_t* x, const bf16_t* dy, float* dw, float* scratch, size_t scratch_bytes, int N, int H, int W,
                                int C, int stride, hipStream_t s) {
  const size_t need = dwconv3_wgrad_scratch_bytes(N, H, W, C, stride);
  if (!need || !scratch || scratch_bytes < need) return hipErrorInvalidValue;
  const int Ho = (H - 1) / stride + 1, Wo = (W - 1) / stride + 1;
  const int chunks = dw_chunks(N, Ho, Wo, C);
  const size_t M = (size_t)N * Ho * Wo;
  const int per = (int)((M + chunks - 1) / chunks);
  hipLaunchKernelGGL(dwconv3_wgrad_kernel, dim3((C / 8 + 7) / 8, chunks), dim3(256), 0, s, x, dy, scratch, N, H, W, C, Ho, Wo, stride, per);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(dwconv3_wgrad_reduce_kernel, dim3((9 * C + 255) / 256), dim3(256), 0, s, scratch, dw, C, chunks);
  return hipGetLastError();
}

}  // namespace fdg

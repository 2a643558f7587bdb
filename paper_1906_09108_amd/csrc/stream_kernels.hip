// Bandwidth-bound kernels of the FDG module step: batch normalisation (forward statistics / apply,
// backward reduce / apply), layout changes at the module boundary, the classification head, the
// momentum-SGD update of Eq. 11 and the bf16 weight snapshot.  All tensors are NHWC [M, C]; a thread
// always owns 8 consecutive channels of one pixel (one 16-byte bf16 access), so a wavefront reads
// whole contiguous rows.
#include "fdg_internal.h"

namespace fdg {

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __builtin_bit_cast(float, u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __builtin_bit_cast(float, u & 0xffff0000u); }
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  bf16_t l = (bf16_t)lo, h = (bf16_t)hi;
  return (uint32_t)__builtin_bit_cast(uint16_t, l) | ((uint32_t)__builtin_bit_cast(uint16_t, h) << 16);
}
__device__ __forceinline__ void unpack8(const uint4& u, float (&f)[8]) {
  f[0] = bf16_lo(u.x); f[1] = bf16_hi(u.x); f[2] = bf16_lo(u.y); f[3] = bf16_hi(u.y);
  f[4] = bf16_lo(u.z); f[5] = bf16_hi(u.z); f[6] = bf16_lo(u.w); f[7] = bf16_hi(u.w);
}
__device__ __forceinline__ uint4 pack8(const float (&f)[8]) {
  return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
}
__device__ __forceinline__ void load8_f32(const float* p, float (&f)[8]) {
  const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
}
// the same, adding the copies of a replicated sums array (rep = floats between copies, 0: one copy)
__device__ __forceinline__ void load8_rep(const float* p, int rep, float (&v)[8]) {
  load8_f32(p, v);
  if (rep > 0) {
#pragma unroll
    for (int r = 1; r < kStatReplicas; ++r) {
      float t[8];
      load8_f32(p + (size_t)r * rep, t);
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] += t[i];
    }
  }
}
__device__ __forceinline__ float load_rep(const float* p, int rep) {
  float v = p[0];
  if (rep > 0)
    for (int r = 1; r < kStatReplicas; ++r) v += p[(size_t)r * rep];
  return v;
}
__device__ __forceinline__ void store8_f32(float* p, const float (&f)[8]) {
  *reinterpret_cast<float4*>(p) = make_float4(f[0], f[1], f[2], f[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(f[4], f[5], f[6], f[7]);
}

constexpr int kThreads = 256;

// Per-channel reductions over the rows of an [M, C] tensor.  A block owns up to 64 channels (CGB groups
// of 8 channels, CGB in {1,2,4,8}) and a range of rows; thread t handles channel group t % CGB of row lane
// t / CGB, so a wavefront reads whole 128-byte row segments.  Partials of the row lanes are added
// through LDS and each block ends with one atomic add per channel and value.
struct ReduceShape {
  int CGB, RL, rows_per_block;
  dim3 grid;
};
static ReduceShape reduce_shape(int M, int C) {
  ReduceShape r;
  const int CG = C / 8;
  r.CGB = CG >= 8 ? 8 : (CG >= 4 ? 4 : (CG >= 2 ? 2 : 1));
  r.RL = kThreads / r.CGB;
  const int cblocks = (CG + r.CGB - 1) / r.CGB;
  int rblocks = (1024 + cblocks - 1) / cblocks;                 // about four blocks per compute unit
  const int max_rblocks = (M + r.RL * 4 - 1) / (r.RL * 4);      // at least four rows per thread
  if (rblocks > max_rblocks) rblocks = max_rblocks;
  if (rblocks < 1) rblocks = 1;
  int rpb = (M + rblocks - 1) / rblocks;
  rpb = (rpb + r.RL - 1) / r.RL * r.RL;
  r.rows_per_block = rpb;
  r.grid = dim3(cblocks, (M + rpb - 1) / rpb, 1);
  return r;
}

template <int NV>
__device__ __forceinline__ void block_reduce_to_global(float (&v)[NV][8], float* const (&dst)[NV], int cgl, int rl, int CGB,
                                                       int RL, int c_base, int C, float* smem /* [NV][RL][CGB*8] */) {
  const int W = CGB * 8;
#pragma unroll
  for (int q = 0; q < NV; ++q)
#pragma unroll
    for (int i = 0; i < 8; ++i) smem[(q * RL + rl) * W + cgl * 8 + i] = v[q][i];
  __syncthreads();
  for (int t = threadIdx.x; t < NV * W; t += blockDim.x) {
    const int q = t / W, col = t % W;
    if (c_base + col >= C) continue;
    float s = 0.f;
    for (int rr = 0; rr < RL; ++rr) s += smem[(q * RL + rr) * W + col];
    atomicAdd(dst[q] + c_base + col, s);
  }
}

// ---- BN forward statistics: sums[c] += sum x, sums[C + c] += sum x^2 --------------------------------
__global__ __launch_bounds__(kThreads) void bn_stats_kernel(const bf16_t* __restrict__ x, float* __restrict__ sums, int M,
                                                            int C, int CGB, int rows_per_block) {
  extern __shared__ float smem[];
  const int RL = kThreads / CGB;
  const int cgl = threadIdx.x % CGB, rl = threadIdx.x / CGB;
  const int cg = blockIdx.x * CGB + cgl;
  const bool cvalid = cg * 8 < C;
  float v[2][8];
#pragma unroll
  for (int i = 0; i < 8; ++i) v[0][i] = v[1][i] = 0.f;
  const int row_lo = blockIdx.y * rows_per_block, row_hi = min(M, row_lo + rows_per_block);
  if (cvalid) {
#pragma unroll 4
    for (int row = row_lo + rl; row < row_hi; row += RL) {
      float f[8];
      unpack8(*reinterpret_cast<const uint4*>(x + (size_t)row * C + cg * 8), f);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        v[0][i] += f[i];
        v[1][i] += f[i] * f[i];
      }
    }
  }
  float* const dst[2] = {sums, sums + C};
  block_reduce_to_global<2>(v, dst, cgl, rl, CGB, RL, blockIdx.x * CGB * 8, C, smem);
}

hipError_t launch_bn_stats(const bf16_t* x, float* sums, int M, int C, hipStream_t s) {
  if (C % 8 != 0 || C > 2048 || M <= 0) return hipErrorInvalidValue;
  const ReduceShape r = reduce_shape(M, C);
  hipLaunchKernelGGL(bn_stats_kernel, r.grid, dim3(kThreads), 2 * kThreads * 8 * sizeof(float), s, x, sums, M, C, r.CGB,
                     r.rows_per_block);
  return hipGetLastError();
}

// ---- BN apply: y = relu?( gamma*xhat + beta [+ res] [+ gamma2*xhat2 + beta2] ) ------------------------
__device__ __forceinline__ void bn_running(const float* sums, int rep, float* run_mean, float* run_var, int C, int M, float mom) {
  const float invM = 1.f / (float)M;
  const float unbias = M > 1 ? (float)M / (float)(M - 1) : 1.f;
  for (int c = threadIdx.x; c < C; c += blockDim.x) {
    const float mean = load_rep(sums + c, rep) * invM;
    const float var = fmaxf(load_rep(sums + C + c, rep) * invM - mean * mean, 0.f);
    run_mean[c] = (1.f - mom) * run_mean[c] + mom * mean;
    run_var[c] = (1.f - mom) * run_var[c] + mom * var * unbias;
  }
}

// Elementwise kernels over [M, C] with per-channel constants: a thread keeps ONE group of 8 channels for all
// of its rows, so the constants are computed once per thread and stay in registers (no LDS, no per-element
// lookups), and a wavefront reads whole 128- or 256-byte row segments.
struct ApplyShape {
  int CGB, RL, rows_per_block;
  dim3 grid;
};
static ApplyShape apply_shape(int M, int C) {
  ApplyShape r;
  const int CG = C / 8;
  r.CGB = CG >= 16 ? 16 : (CG >= 8 ? 8 : (CG >= 4 ? 4 : (CG >= 2 ? 2 : 1)));
  r.RL = kThreads / r.CGB;
  const int cblocks = (CG + r.CGB - 1) / r.CGB;
  int rblocks = (2048 + cblocks - 1) / cblocks;
  const int max_rblocks = (M + r.RL * 4 - 1) / (r.RL * 4);      // at least four rows per thread
  if (rblocks > max_rblocks) rblocks = max_rblocks;
  if (rblocks < 1) rblocks = 1;
  int rpb = (M + rblocks - 1) / rblocks;
  rpb = (rpb + r.RL - 1) / r.RL * r.RL;
  r.rows_per_block = rpb;
  r.grid = dim3(cblocks, (M + rpb - 1) / rpb, 1);
  return r;
}

// The copies of NA replicated per-channel arrays added once per block instead of once per thread: thread
// (cgl = tid % CGB, rl = tid / CGB) with rl < kStatReplicas loads copy rl of its channel group (8 floats per array),
// the copies are added across the lanes of wave 0 (needs kStatReplicas * CGB <= 64, CGB a power of two) and parked
// in LDS, where every thread of the block picks up the sums of its channel group.  All threads of the block call.
template <int NA>
__device__ __forceinline__ void fold_replicas(const float* const (&src)[NA], const int (&rep)[NA], int c0, bool cvalid, int CGB,
                                              float (&out)[NA][8]) {
  __shared__ float4 parked[8][NA][2];
  const int cgl = threadIdx.x % CGB, rl = threadIdx.x / CGB;
  if (rl < kStatReplicas) {
    float v[NA][8];
#pragma unroll
    for (int a = 0; a < NA; ++a) {
      if (cvalid && (rl == 0 || rep[a] > 0)) load8_f32(src[a] + c0 + (size_t)rl * rep[a], v[a]);
      else {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[a][i] = 0.f;
      }
    }
    for (int off = CGB; off < kStatReplicas * CGB; off <<= 1) {
#pragma unroll
      for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int i = 0; i < 8; ++i) v[a][i] += __shfl_xor(v[a][i], off);
    }
    if (rl == 0) {
#pragma unroll
      for (int a = 0; a < NA; ++a) {
        parked[cgl][a][0] = make_float4(v[a][0], v[a][1], v[a][2], v[a][3]);
        parked[cgl][a][1] = make_float4(v[a][4], v[a][5], v[a][6], v[a][7]);
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int a = 0; a < NA; ++a) {
    const float4 lo = parked[cgl][a][0], hi = parked[cgl][a][1];
    out[a][0] = lo.x; out[a][1] = lo.y; out[a][2] = lo.z; out[a][3] = lo.w;
    out[a][4] = hi.x; out[a][5] = hi.y; out[a][6] = hi.z; out[a][7] = hi.w;
  }
}

// scale / shift of 8 channels from the accumulated sums
__device__ __forceinline__ void bn_coeffs8(const float* sums, int rep, const float* gamma, const float* beta, int C, int c0, float invM,
                                           float eps, float (&sc)[8], float (&sh)[8]) {
  float s1[8], s2[8], g[8], b[8];
  load8_rep(sums + c0, rep, s1);
  load8_rep(sums + C + c0, rep, s2);
  load8_f32(gamma + c0, g);
  load8_f32(beta + c0, b);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float mean = s1[i] * invM;
    const float var = fmaxf(s2[i] * invM - mean * mean, 0.f);
    const float gi = g[i] * rsqrtf(var + eps);
    sc[i] = gi;
    sh[i] = b[i] - mean * gi;
  }
}

__device__ __forceinline__ void bn_coeffs8_from(const float (&s1)[8], const float (&s2)[8], const float* gamma, const float* beta,
                                                int c0, float invM, float eps, float (&sc)[8], float (&sh)[8]) {
  float g[8], b[8];
  load8_f32(gamma + c0, g);
  load8_f32(beta + c0, b);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float mean = s1[i] * invM;
    const float var = fmaxf(s2[i] * invM - mean * mean, 0.f);
    const float gi = g[i] * rsqrtf(var + eps);
    sc[i] = gi;
    sh[i] = b[i] - mean * gi;
  }
}

// FOLD: the sums are replicated and added once per block through LDS; a kernel of its own so that the plain form
// allocates no LDS (it then fits beside workgroups of the convolutions that fill a compute unit's LDS).
template <bool FOLD>
__global__ __launch_bounds__(kThreads) void bn_apply_kernel(BnApplyArgs a, int CGB, int rows_per_block) {
  const int C = a.C;
  if (blockIdx.x == 0 && blockIdx.y == 0) {
    if (a.run_mean) bn_running(a.sums, a.rep_stride, a.run_mean, a.run_var, C, a.M, a.momentum);
    if (a.x2 && a.run_mean2) bn_running(a.sums2, a.rep_stride, a.run_mean2, a.run_var2, C, a.M, a.momentum);
  }
  const int RL = kThreads / CGB;
  const int cg = blockIdx.x * CGB + threadIdx.x % CGB, rl = threadIdx.x / CGB;
  const int c0 = cg * 8;
  const float invM = 1.f / (float)a.M;
  float sc[8], sh[8], sc2[8], sh2[8];
  if constexpr (FOLD) {
    const float* const src[4] = {a.sums, a.sums + C, a.x2 ? a.sums2 : a.sums, a.x2 ? a.sums2 + C : a.sums + C};
    const int rep[4] = {a.rep_stride, a.rep_stride, a.rep_stride, a.rep_stride};
    float f[4][8];
    fold_replicas<4>(src, rep, c0, c0 < C, CGB, f);
    if (c0 >= C) return;
    bn_coeffs8_from(f[0], f[1], a.gamma, a.beta, c0, invM, a.eps, sc, sh);
    if (a.x2) bn_coeffs8_from(f[2], f[3], a.gamma2, a.beta2, c0, invM, a.eps, sc2, sh2);
  } else {
    if (c0 >= C) return;
    bn_coeffs8(a.sums, a.rep_stride, a.gamma, a.beta, C, c0, invM, a.eps, sc, sh);
    if (a.x2) bn_coeffs8(a.sums2, a.rep_stride, a.gamma2, a.beta2, C, c0, invM, a.eps, sc2, sh2);
  }
  const int row_lo = blockIdx.y * rows_per_block, row_hi = min(a.M, row_lo + rows_per_block);
#pragma unroll 4
  for (int row = row_lo + rl; row < row_hi; row += RL) {
    const size_t o = (size_t)row * C + c0;
    float f[8];
    unpack8(*reinterpret_cast<const uint4*>(a.x + o), f);
#pragma unroll
    for (int i = 0; i < 8; ++i) f[i] = f[i] * sc[i] + sh[i];
    if (a.res_f32) {
      float rr[8];
      load8_f32(a.res_f32 + o, rr);
#pragma unroll
      for (int i = 0; i < 8; ++i) f[i] += rr[i];
    }
    if (a.x2) {
      float g[8];
      unpack8(*reinterpret_cast<const uint4*>(a.x2 + o), g);
#pragma unroll
      for (int i = 0; i < 8; ++i) f[i] += g[i] * sc2[i] + sh2[i];
    }
    if (a.relu) {
#pragma unroll
      for (int i = 0; i < 8; ++i) f[i] = fmaxf(f[i], 0.f);
    }
    if (a.out_f32) store8_f32(a.out_f32 + o, f);
    if (a.out_b16) *reinterpret_cast<uint4*>(a.out_b16 + o) = pack8(f);
  }
}

static int stream_grid(size_t units) {
  size_t b = (units + kThreads - 1) / kThreads;
  if (b > 2048) b = 2048;
  if (b < 1) b = 1;
  return (int)b;
}

hipError_t launch_bn_apply(const BnApplyArgs& a, hipStream_t s) {
  if (a.C % 8 != 0 || a.C > 2048 || a.M <= 0) return hipErrorInvalidValue;
  const auto al16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
  if (!al16(a.sums) || !al16(a.gamma) || !al16(a.beta) || (a.x2 && (!al16(a.sums2) || !al16(a.gamma2) || !al16(a.beta2))))
    return hipErrorInvalidValue;   // per-channel vectors are read 16 bytes at a time
  const ApplyShape r = apply_shape(a.M, a.C);
  if (a.rep_stride > 0 && r.CGB * kStatReplicas <= 64)
    hipLaunchKernelGGL(bn_apply_kernel<true>, r.grid, dim3(kThreads), 0, s, a, r.CGB, r.rows_per_block);
  else
    hipLaunchKernelGGL(bn_apply_kernel<false>, r.grid, dim3(kThreads), 0, s, a, r.CGB, r.rows_per_block);
  return hipGetLastError();
}

// ---- BN backward ---------------------------------------------------------------------------------
template <bool DY_F32>
__device__ __forceinline__ void load_masked_dy(const void* dy, const bf16_t* mask, size_t o, float (&g)[8]) {
  if (DY_F32)
    load8_f32(reinterpret_cast<const float*>(dy) + o, g);
  else
    unpack8(*reinterpret_cast<const uint4*>(reinterpret_cast<const bf16_t*>(dy) + o), g);
  if (!mask) return;   // dy was gated where it was produced
  float mk[8];
  unpack8(*reinterpret_cast<const uint4*>(mask + o), mk);
#pragma unroll
  for (int i = 0; i < 8; ++i)
    if (!(mk[i] > 0.f)) g[i] = 0.f;
}

template <bool DY_F32>
__global__ __launch_bounds__(kThreads) void bn_bwd_reduce_kernel(BnBwdArgs a, int CGB, int rows_per_block) {
  extern __shared__ float smem[];  // 2 * 256 * 8 floats
  const int C = a.C;
  const int RL = kThreads / CGB;
  const int cgl = threadIdx.x % CGB, rl = threadIdx.x / CGB;
  const int cg = blockIdx.x * CGB + cgl;
  const bool cvalid = cg * 8 < C;
  float mu[8], iv[8];
  float v[2][8];
#pragma unroll
  for (int i = 0; i < 8; ++i) v[0][i] = v[1][i] = 0.f;
  if (cvalid) {
    const float invM = 1.f / (float)a.M;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int c = cg * 8 + i;
      const float m = load_rep(a.sums + c, a.rep_stride) * invM;
      const float var = fmaxf(load_rep(a.sums + C + c, a.rep_stride) * invM - m * m, 0.f);
      mu[i] = m;
      iv[i] = rsqrtf(var + a.eps);
    }
    const int row_lo = blockIdx.y * rows_per_block, row_hi = min(a.M, row_lo + rows_per_block);
#pragma unroll 2
    for (int row = row_lo + rl; row < row_hi; row += RL) {
      const size_t o = (size_t)row * C + cg * 8;
      float g[8], xv[8];
      load_masked_dy<DY_F32>(a.dy, a.mask, o, g);
      unpack8(*reinterpret_cast<const uint4*>(a.x + o), xv);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        v[0][i] += g[i];
        v[1][i] += g[i] * ((xv[i] - mu[i]) * iv[i]);
      }
    }
  }
  float* const dst[2] = {a.bsums, a.bsums + C};
  block_reduce_to_global<2>(v, dst, cgl, rl, CGB, RL, blockIdx.x * CGB * 8, C, smem);
}

hipError_t launch_bn_bwd_reduce(const BnBwdArgs& a, hipStream_t s) {
  if (a.C % 8 != 0 || a.C > 2048 || a.M <= 0 || !a.mask) return hipErrorInvalidValue;
  const ReduceShape r = reduce_shape(a.M, a.C);
  const size_t sm = 2 * (size_t)kThreads * 8 * sizeof(float);
  if (a.dy_is_f32)
    hipLaunchKernelGGL(bn_bwd_reduce_kernel<true>, r.grid, dim3(kThreads), sm, s, a, r.CGB, r.rows_per_block);
  else
    hipLaunchKernelGGL(bn_bwd_reduce_kernel<false>, r.grid, dim3(kThreads), sm, s, a, r.CGB, r.rows_per_block);
  return hipGetLastError();
}

// dx = gamma*invstd*(g - S1/M - xhat*S2/M) [+ addend];  dgamma = S2, dbeta = S1
template <bool DY_F32, bool FOLD>
__global__ __launch_bounds__(kThreads) void bn_bwd_apply_kernel(BnBwdArgs a, int CGB, int rows_per_block) {
  const int C = a.C;
  const int RL = kThreads / CGB;
  const int cg = blockIdx.x * CGB + threadIdx.x % CGB, rl = threadIdx.x / CGB;
  const int c0 = cg * 8;
  const float invM = 1.f / (float)a.M;
  // per channel: xhat = x*is - mean*is;  dx = gi*g - gi*k1 - gi*k2*xhat = gi*g + (pa*x + pb)
  float gi[8], pa[8], pb[8];
  {
    float s1[8], s2[8], gm[8], b1[8], b2[8];
    if constexpr (FOLD) {   // replicated sums: added once per block through LDS (see bn_apply_kernel)
      const float* const src[4] = {a.sums, a.sums + C, a.bsums, a.bsums + C};
      const int rep[4] = {a.rep_stride, a.rep_stride, a.brep_stride, a.brep_stride};
      float f[4][8];
      fold_replicas<4>(src, rep, c0, c0 < C, CGB, f);
      if (c0 >= C) return;
#pragma unroll
      for (int i = 0; i < 8; ++i) { s1[i] = f[0][i]; s2[i] = f[1][i]; b1[i] = f[2][i]; b2[i] = f[3][i]; }
    } else {
      if (c0 >= C) return;
      load8_rep(a.sums + c0, a.rep_stride, s1);
      load8_rep(a.sums + C + c0, a.rep_stride, s2);
      load8_rep(a.bsums + c0, a.brep_stride, b1);
      load8_rep(a.bsums + C + c0, a.brep_stride, b2);
    }
    load8_f32(a.gamma + c0, gm);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float mean = s1[i] * invM;
      const float var = fmaxf(s2[i] * invM - mean * mean, 0.f);
      const float is = rsqrtf(var + a.eps);
      if (a.raw_sums) b2[i] = is * (b2[i] - mean * b1[i]);   // sum g*xhat from sum g*x and sum g
      gi[i] = gm[i] * is;
      const float k1 = b1[i] * invM, k2 = b2[i] * invM;
      pa[i] = -gi[i] * k2 * is;
      pb[i] = -gi[i] * k1 + gi[i] * k2 * is * mean;
    }
    if (blockIdx.y == 0 && rl == 0) {
      store8_f32(a.dbeta + c0, b1);
      store8_f32(a.dgamma + c0, b2);
    }
  }
  if (!a.out_f32 && !a.out_b16) return;
  const int row_lo = blockIdx.y * rows_per_block, row_hi = min(a.M, row_lo + rows_per_block);
#pragma unroll 4
  for (int row = row_lo + rl; row < row_hi; row += RL) {
    const size_t o = (size_t)row * C + c0;
    float g[8], xv[8];
    load_masked_dy<DY_F32>(a.dy, a.mask, o, g);
    unpack8(*reinterpret_cast<const uint4*>(a.x + o), xv);
#pragma unroll
    for (int i = 0; i < 8; ++i) g[i] = gi[i] * g[i] + (pa[i] * xv[i] + pb[i]);
    if (a.addend) {
      float ad[8];
      load8_f32(a.addend + o, ad);
#pragma unroll
      for (int i = 0; i < 8; ++i) g[i] += ad[i];
    }
    if (a.out_f32) store8_f32(a.out_f32 + o, g);
    if (a.out_b16) *reinterpret_cast<uint4*>(a.out_b16 + o) = pack8(g);
  }
}

hipError_t launch_bn_bwd_apply(const BnBwdArgs& a_in, hipStream_t s) {
  BnBwdArgs a = a_in;
  if (a.dy_gated) a.mask = nullptr;
  if (a.C % 8 != 0 || a.C > 2048 || a.M <= 0 || (!a.mask && !a.dy_gated)) return hipErrorInvalidValue;
  const auto al16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
  if (!al16(a.sums) || !al16(a.gamma) || !al16(a.bsums) || !al16(a.dgamma) || !al16(a.dbeta)) return hipErrorInvalidValue;
  ApplyShape r = apply_shape(a.M, a.C);
  if (!a.out_f32 && !a.out_b16) r.grid.y = 1;   // only dgamma / dbeta
  const bool fold = (a.rep_stride > 0 || a.brep_stride > 0) && r.CGB * kStatReplicas <= 64;
  if (a.dy_is_f32) {
    if (fold) hipLaunchKernelGGL((bn_bwd_apply_kernel<true, true>), r.grid, dim3(kThreads), 0, s, a, r.CGB, r.rows_per_block);
    else hipLaunchKernelGGL((bn_bwd_apply_kernel<true, false>), r.grid, dim3(kThreads), 0, s, a, r.CGB, r.rows_per_block);
  } else {
    if (fold) hipLaunchKernelGGL((bn_bwd_apply_kernel<false, true>), r.grid, dim3(kThreads), 0, s, a, r.CGB, r.rows_per_block);
    else hipLaunchKernelGGL((bn_bwd_apply_kernel<false, false>), r.grid, dim3(kThreads), 0, s, a, r.CGB, r.rows_per_block);
  }
  return hipGetLastError();
}

// ---- layout changes at the module boundary -----------------------------------------------------
// src fp32 [N, C, HW] -> dst [N, HW, Cp] (channels >= C are zero), scaled.  32x32 tiles through LDS.
__global__ __launch_bounds__(kThreads) void nchw_to_nhwc_kernel(const float* __restrict__ src, float* __restrict__ dst_f32,
                                                                bf16_t* __restrict__ dst_b16, int C, int HW, int Cp,
                                                                float scale) {
  __shared__ float tile[32][33];
  const int n = blockIdx.z, hw0 = blockIdx.x * 32, c0 = blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
  for (int i = ty; i < 32; i += 8) {
    const int c = c0 + i, hw = hw0 + tx;
    tile[i][tx] = (c < C && hw < HW) ? src[((size_t)n * C + c) * HW + hw] * scale : 0.f;
  }
  __syncthreads();
  for (int i = ty; i < 32; i += 8) {
    const int hw = hw0 + i, c = c0 + tx;
    if (hw < HW && c < Cp) {
      const float v = tile[tx][i];
      const size_t o = ((size_t)n * HW + hw) * Cp + c;
      if (dst_f32) dst_f32[o] = v;
      if (dst_b16) dst_b16[o] = (bf16_t)v;
    }
  }
}

hipError_t launch_nchw_to_nhwc(const float* src, float* dst_f32, bf16_t* dst_b16, int N, int C, int HW, int Cp,
                               float scale, hipStream_t s) {
  dim3 grid((HW + 31) / 32, (Cp + 31) / 32, N);
  hipLaunchKernelGGL(nchw_to_nhwc_kernel, grid, dim3(kThreads), 0, s, src, dst_f32, dst_b16, C, HW, Cp, scale);
  return hipGetLastError();
}

// src fp32 [N, HW, Cp] -> dst [N, C, HW]
__global__ __launch_bounds__(kThreads) void nhwc_to_nchw_kernel(const float* __restrict__ src, float* __restrict__ dst, int C,
                                                                int HW, int Cp) {
  __shared__ float tile[32][33];
  const int n = blockIdx.z, hw0 = blockIdx.x * 32, c0 = blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  for (int i = ty; i < 32; i += 8) {
    const int hw = hw0 + i, c = c0 + tx;
    tile[i][tx] = (hw < HW && c < C) ? src[((size_t)n * HW + hw) * Cp + c] : 0.f;
  }
  __syncthreads();
  for (int i = ty; i < 32; i += 8) {
    const int c = c0 + i, hw = hw0 + tx;
    if (c < C && hw < HW) dst[((size_t)n * C + c) * HW + hw] = tile[tx][i];
  }
}

hipError_t launch_nhwc_to_nchw(const float* src, float* dst, int N, int C, int HW, int Cp, hipStream_t s) {
  dim3 grid((HW + 31) / 32, (C + 31) / 32, N);
  hipLaunchKernelGGL(nhwc_to_nchw_kernel, grid, dim3(kThreads), 0, s, src, dst, C, HW, Cp);
  return hipGetLastError();
}

// ---- head -------------------------------------------------------------------------------------------
// pooled[n, c] = mean over the HW pixels of o[n, :, c].  One block per image and 256 channels: 32 groups of 8
// channels (one 16-byte load per pixel) x 8 pixel phases, so that every thread has only HW/8 independent loads
// and the eight partial sums of a channel are added, in a fixed order, through LDS.
__global__ __launch_bounds__(256) void avgpool_kernel(const bf16_t* __restrict__ o, float* __restrict__ pooled, int N, int HW, int C) {
  __shared__ float part[8][256 + 8];
  const int n = blockIdx.y, c0 = blockIdx.x * 256;
  const int cg = threadIdx.x & 31, ph = threadIdx.x >> 5;
  const int c = c0 + cg * 8;
  float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (c < C) {   // C % 8 == 0
    const bf16_t* src = o + (size_t)n * HW * C + c;
#pragma unroll 8
    for (int p = ph; p < HW; p += 8) {
      float f[8];
      unpack8(*reinterpret_cast<const uint4*>(src + (size_t)p * C), f);
#pragma unroll
      for (int i = 0; i < 8; ++i) s[i] += f[i];
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) part[ph][cg * 8 + i] = s[i];
  __syncthreads();
  const int cc = c0 + threadIdx.x;
  if (cc < C) {
    float t = 0.f;
#pragma unroll
    for (int q = 0; q < 8; ++q) t += part[q][threadIdx.x];
    pooled[(size_t)n * C + cc] = t / (float)HW;
  }
}
hipError_t launch_avgpool(const bf16_t* o, float* pooled, int N, int HW, int C, hipStream_t s) {
  if (C % 8 != 0 || N <= 0 || N > 65535) return hipErrorInvalidValue;
  hipLaunchKernelGGL(avgpool_kernel, dim3((C + 255) / 256, N), dim3(256), 0, s, o, pooled, N, HW, C);
  return hipGetLastError();
}

__global__ void fc_fwd_kernel(const float* __restrict__ pooled, const float* __restrict__ W, const float* __restrict__ b,
                              float* __restrict__ logits, int N, int C, int J) {
  // one wavefront per (n, j)
  const int gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, lane = threadIdx.x & 63;
  if (gw >= N * J) return;
  const int n = gw / J, j = gw % J;
  float s = 0.f;
  for (int c = lane; c < C; c += 64) s += pooled[(size_t)n * C + c] * W[(size_t)j * C + c];
  for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off, 64);
  if (lane == 0) logits[gw] = s + b[j];
}
hipError_t launch_fc_fwd(const float* pooled, const float* W, const float* b, float* logits, int N, int C, int J,
                         hipStream_t s) {
  hipLaunchKernelGGL(fc_fwd_kernel, dim3((N * J * 64 + 255) / 256), dim3(256), 0, s, pooled, W, b, logits, N, C, J);
  return hipGetLastError();
}

// single block: per-row log-sum-exp, loss, dlogits
__global__ __launch_bounds__(kThreads) void softmax_ce_kernel(const float* __restrict__ logits, const int32_t* __restrict__ labels,
                                                              float* __restrict__ y, float* __restrict__ dl, int N, int J) {
  __shared__ float red[kThreads];
  float part = 0.f;
  for (int n = threadIdx.x; n < N; n += kThreads) {
    const float* l = logits + (size_t)n * J;
    float mx = l[0];
    for (int j = 1; j < J; ++j) mx = fmaxf(mx, l[j]);
    float z = 0.f;
    for (int j = 0; j < J; ++j) z += expf(l[j] - mx);
    const float lse = mx + logf(z);
    const int lab = min(max(labels[n], 0), J - 1);
    part += lse - l[lab];
    for (int j = 0; j < J; ++j) {
      const float sm = expf(l[j] - lse);
      dl[(size_t)n * J + j] = (sm - (j == lab ? 1.f : 0.f)) / (float)N;
      y[1 + (size_t)n * J + j] = l[j];
    }
  }
  red[threadIdx.x] = part;
  __syncthreads();
  for (int off = kThreads / 2; off > 0; off >>= 1) {
    if (threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) y[0] = red[0] / (float)N;
}
hipError_t launch_softmax_ce(const float* logits, const int32_t* labels, float* y, float* dl, int N, int J,
                             hipStream_t s) {
  hipLaunchKernelGGL(softmax_ce_kernel, dim3(1), dim3(kThreads), 0, s, logits, labels, y, dl, N, J);
  return hipGetLastError();
}

// dW[j,c] = sum_n dl[n,j] p[n,c];  db[j] = sum_n dl[n,j];  dp[n,c] = sum_j dl[n,j] W[j,c]
// Blocks [0, dp_blocks): one thread per dp element (J terms).  The other blocks: one per class j and 64
// channels; the batch is dealt to 4 thread groups so that a thread has N/4 independent loads, and the four
// partial sums are added in a fixed order through LDS.  db[j] comes from the blocks of channel chunk 0.
__global__ __launch_bounds__(256) void fc_bwd_kernel(const float* __restrict__ pooled, const float* __restrict__ W,
                                                     const float* __restrict__ dl, float* __restrict__ dW, float* __restrict__ db,
                                                     float* __restrict__ dp, int N, int C, int J, int dp_blocks) {
  __shared__ float part[4][64];
  __shared__ float bpart[4];
  if ((int)blockIdx.x < dp_blocks) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx < N * C) {
      const int n = idx / C, c = idx % C;
      float s = 0.f;
      for (int j = 0; j < J; ++j) s += dl[(size_t)n * J + j] * W[(size_t)j * C + c];
      dp[idx] = s;
    }
    return;
  }
  const int b = blockIdx.x - dp_blocks, chunks = (C + 63) / 64;
  const int j = b / chunks, c = (b % chunks) * 64 + (threadIdx.x & 63), q = threadIdx.x >> 6;
  float s = 0.f, sb = 0.f;
  const bool cok = c < C;
#pragma unroll 8
  for (int n = q; n < N; n += 4) {
    const float d = dl[(size_t)n * J + j];
    sb += d;
    if (cok) s += d * pooled[(size_t)n * C + c];
  }
  part[q][threadIdx.x & 63] = s;
  if ((threadIdx.x & 63) == 0) bpart[q] = sb;
  __syncthreads();
  if (q == 0) {
    if (cok) dW[(size_t)j * C + c] = (part[0][threadIdx.x] + part[1][threadIdx.x]) + (part[2][threadIdx.x] + part[3][threadIdx.x]);
    if (threadIdx.x == 0 && b % chunks == 0) db[j] = (bpart[0] + bpart[1]) + (bpart[2] + bpart[3]);
  }
}
hipError_t launch_fc_bwd(const float* pooled, const float* W, const float* dl, float* dW, float* db, float* dp,
                         int N, int C, int J, hipStream_t s) {
  const int dp_blocks = (N * C + 255) / 256, w_blocks = J * ((C + 63) / 64);
  hipLaunchKernelGGL(fc_bwd_kernel, dim3(dp_blocks + w_blocks), dim3(256), 0, s, pooled, W, dl, dW, db, dp, N, C, J, dp_blocks);
  return hipGetLastError();
}

__global__ void pool_bwd_kernel(const float* __restrict__ dp, float* __restrict__ g_f32, bf16_t* __restrict__ g_b16, int N,
                                int HW, int C) {
  const size_t total = (size_t)N * HW * C;
  const float inv = 1.f / (float)HW;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int c = (int)(i % C);
    const int n = (int)(i / ((size_t)HW * C));
    const float v = dp[(size_t)n * C + c] * inv;
    if (g_f32) g_f32[i] = v;
    if (g_b16) g_b16[i] = (bf16_t)v;
  }
}
hipError_t launch_pool_bwd(const float* dp, float* g_f32, bf16_t* g_b16, int N, int HW, int C, hipStream_t s) {
  hipLaunchKernelGGL(pool_bwd_kernel, dim3(stream_grid((size_t)N * HW * C)), dim3(256), 0, s, dp, g_f32, g_b16, N, HW, C);
  return hipGetLastError();
}

// ---- momentum SGD (Eq. 11 with the optimiser of Section V-A) ------------------------------------------
__global__ __launch_bounds__(kThreads) void sgd_kernel(float4* __restrict__ theta, float4* __restrict__ v,
                                                       const float4* __restrict__ g, size_t n4, float lr, float mu, float wd) {
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += (size_t)gridDim.x * kThreads) {
    float4 t = theta[i], m = v[i];
    const float4 gg = g[i];
    m.x = mu * m.x + (gg.x + wd * t.x);
    m.y = mu * m.y + (gg.y + wd * t.y);
    m.z = mu * m.z + (gg.z + wd * t.z);
    m.w = mu * m.w + (gg.w + wd * t.w);
    t.x -= lr * m.x;
    t.y -= lr * m.y;
    t.z -= lr * m.z;
    t.w -= lr * m.w;
    v[i] = m;
    theta[i] = t;
  }
}
hipError_t launch_sgd(float* theta, float* v, const float* g, size_t count, float lr, float mu, float wd, hipStream_t s) {
  if (count % 4 != 0) return hipErrorInvalidValue;
  if (count == 0) return hipSuccess;
  const size_t n4 = count / 4;
  size_t blocks = (n4 + kThreads - 1) / kThreads;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(sgd_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, s, reinterpret_cast<float4*>(theta),
                     reinterpret_cast<float4*>(v), reinterpret_cast<const float4*>(g), n4, lr, mu, wd);
  return hipGetLastError();
}

// ---- bf16 weight snapshot ------------------------------------------------------------------------
// One block converts one 64 (co) x 64 (ci) tile of one filter tap of one convolution: it reads the fp32
// master [Co][T][Ci] along ci, writes the forward layout [Co][T][Cip] along ci and, after a transpose
// through LDS, the data-gradient layout [Cip][T][Co] along co, so every access is coalesced.
__global__ __launch_bounds__(kThreads) void emit_weights_kernel(const float* __restrict__ params, bf16_t* __restrict__ warena,
                                                                const WeightEmitEntry* __restrict__ table, int nconv) {
  __shared__ float tile[64][65];
  int lo = 0, hi = nconv - 1;   // the conv this block belongs to (block_start is ascending)
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (table[mid].block_start <= blockIdx.x) lo = mid; else hi = mid - 1;
  }
  const WeightEmitEntry e = table[lo];
  const int cit = (e.Cip + 63) / 64, cot = (e.Co + 63) / 64;
  int local = blockIdx.x - e.block_start;
  const int ci0 = (local % cit) * 64;
  local /= cit;
  const int co0 = (local % cot) * 64, t = local / cot;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int r = ty; r < 64; r += 4) {
    const int co = co0 + r, ci = ci0 + tx;
    float v = 0.f;
    if (co < e.Co && ci < e.Ci) v = params[e.src_off + ((size_t)co * e.T + t) * e.Ci + ci];
    tile[r][tx] = v;
    if (co < e.Co && ci < e.Cip) warena[e.w_off + ((size_t)co * e.T + t) * e.Cip + ci] = (bf16_t)v;
  }
  __syncthreads();
  for (int r = ty; r < 64; r += 4) {
    const int ci = ci0 + r, co = co0 + tx;
    if (ci < e.Cip && co < e.Co) warena[e.wt_off + ((size_t)ci * e.T + t) * e.Co + co] = (bf16_t)tile[tx][r];
  }
}
hipError_t launch_emit_weights(const float* params, bf16_t* warena, const WeightEmitEntry* table_dev, int nconv,
                               int total_blocks, hipStream_t s) {
  if (nconv <= 0) return hipSuccess;
  hipLaunchKernelGGL(emit_weights_kernel, dim3(total_blocks), dim3(kThreads), 0, s, params, warena, table_dev, nconv);
  return hipGetLastError();
}

// ---- fills ------------------------------------------------------------------------------------------
__global__ void fill_zero_kernel(uint4* p, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
    p[i] = make_uint4(0, 0, 0, 0);
}
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
  if (bytes % 16 != 0) return hipErrorInvalidValue;
  if (bytes == 0) return hipSuccess;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(stream_grid(bytes / 16)), dim3(256), 0, s, reinterpret_cast<uint4*>(p), bytes / 16);
  return hipGetLastError();
}
__global__ void fill_f32_kernel(float* p, size_t n, float v) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}
hipError_t launch_fill_f32(float* p, size_t count, float v, hipStream_t s) {
  if (count == 0) return hipSuccess;
  hipLaunchKernelGGL(fill_f32_kernel, dim3(stream_grid(count)), dim3(256), 0, s, p, count, v);
  return hipGetLastError();
}

}  // namespace fdg

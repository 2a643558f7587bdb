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
// ---- per-channel constants, worked out once per wave ------------------------------------------------
// A thread of the elementwise kernels owns a group of 8 channels, and the 64 / CGB lanes of a wave that own the same
// group would each repeat the 64-bit arithmetic that turns the group's exact totals into the constants of the row
// loop.  Instead the lanes share it: lane (cgl = lane % CGB, sub = lane / CGB) takes channel sub % 8 of the group (two
// channels, sub and sub + 4, when only four lanes share a group) and, where the sums exist in copies, the copies
// sub / 8, sub / 8 + parts, ...; the integer words of the copies are added across those lanes, the lane works out the
// constants of its channel(s), and they travel to the lanes that need them by lane shuffles.  No LDS.  Every lane of a
// wave must take part (shuffles), also the lanes whose channel group does not exist.
struct LaneShare {
  int CGB, cgl, sub, nch, part, parts;
  __device__ __forceinline__ explicit LaneShare(int cgb) : CGB(cgb) {
    const int lane = threadIdx.x & 63, S = 64 / cgb;   // CGB divides 64
    cgl = lane % cgb; sub = lane / cgb;
    nch = S >= 8 ? 1 : 2;
    part = S >= 8 ? sub / 8 : 0;
    parts = S >= 8 ? S / 8 : 1;
  }
  // k-th channel of the group this lane works on (k < nch)
  __device__ __forceinline__ int channel(int k) const { return nch == 1 ? sub % 8 : sub + 4 * k; }
  // the value lane-computed for channel i of the group, given this lane's values r[k]
  __device__ __forceinline__ float gather(const float (&r)[2], int i) const {
    return nch == 1 ? __shfl(r[0], cgl + CGB * i) : __shfl(i < 4 ? r[0] : r[1], cgl + CGB * (i & 3));
  }
};
// The words of one of the two sums (which = 0 / 1) of channel c in the COPIES copies this lane takes (copy part,
// part + parts, ...; COPIES * parts = kStatReplicas, or COPIES = 1 and rep = 0 where the array is a single copy, which
// every lane then reads).  Loads only -- nothing is added and nothing depends on `valid` (a lane without a channel is given
// an existing one and its result is dropped) -- so that a kernel issues the loads of ALL the sums it needs back to back
// and waits for memory once.
template <int COPIES>
struct RawTotal { long long hi[COPIES], lo[COPIES], big[COPIES]; };
template <int COPIES>
__device__ __forceinline__ void chan_load(RawTotal<COPIES>& t, const LaneShare& ls, const stat_t* stats, int C, int which, int c, int rep) {
  const stat_t* p = stats + (size_t)which * C + c;
#pragma unroll
  for (int j = 0; j < COPIES; ++j) {
    const stat_t* q = p + (size_t)(ls.part + j * ls.parts) * rep;
    t.hi[j] = q[0];
    t.lo[j] = q[2 * (size_t)C];
    t.big[j] = q[4 * (size_t)C];
  }
}
// The total: this lane's copies (added as integers, hence independent of the order the workgroups arrived in) as a
// double, then -- where there are copies -- the other lanes' in a fixed order.
template <int COPIES>
__device__ __forceinline__ double chan_total(const RawTotal<COPIES>& t, const LaneShare& ls, int rep) {
  long long hi = 0, lo = 0;
  double big = 0.0;
#pragma unroll
  for (int j = 0; j < COPIES; ++j) {
    hi += t.hi[j];
    lo += t.lo[j];
    big += __builtin_bit_cast(double, t.big[j]);
  }
  double v = stat_value(hi, lo, __builtin_bit_cast(long long, big));
  if (rep > 0)
    for (int off = 8 * ls.CGB; off < 64; off <<= 1) v += __shfl_xor(v, off);   // lanes 8 * CGB apart hold the other copies
  return v;
}
// copies a lane takes for an array with (rep > 0) or without copies: the template argument of the functions above
static int host_copies_per_lane(int CGB, int rep) {
  const int S = 64 / CGB, parts = S >= 8 ? S / 8 : 1;   // as in LaneShare
  return rep > 0 ? kStatReplicas / parts : 1;
}
// Batch mean and 1 / sqrt(variance + eps) from the totals sum x and sum x^2 over M rows.  The subtraction that gives the
// variance is done in double on the exact totals, so a mean that is large against the spread costs no digits here.
__device__ __forceinline__ void bn_moments(double s1, double s2, double invM, float eps, float& mean, float& is) {
  const double m = s1 * invM;
  const double var = fmax(s2 * invM - m * m, 0.0);
  mean = (float)m;
  is = rsqrtf((float)var + eps);
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
__device__ __forceinline__ void block_reduce_to_global(float (&v)[NV][8], stat_t* stats, int cgl, int rl, int CGB,
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
    stat_add(stats, C, q, c_base + col, s);
  }
}

// ---- BN forward statistics: sums[c] += sum x, sums[C + c] += sum x^2 --------------------------------
__global__ __launch_bounds__(kThreads) void bn_stats_kernel(const bf16_t* __restrict__ x, stat_t* __restrict__ sums, int M,
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
  block_reduce_to_global<2>(v, sums, cgl, rl, CGB, RL, blockIdx.x * CGB * 8, C, smem);
}

hipError_t launch_bn_stats(const bf16_t* x, stat_t* sums, int M, int C, hipStream_t s) {
  if (C % 8 != 0 || C > 2048 || M <= 0) return hipErrorInvalidValue;
  const ReduceShape r = reduce_shape(M, C);
  hipLaunchKernelGGL(bn_stats_kernel, r.grid, dim3(kThreads), 2 * kThreads * 8 * sizeof(float), s, x, sums, M, C, r.CGB,
                     r.rows_per_block);
  return hipGetLastError();
}

// ---- BN apply: y = relu?( gamma*xhat + beta [+ res] [+ gamma2*xhat2 + beta2] ) ------------------------
__device__ __forceinline__ void bn_running(const stat_t* sums, int rep, float* run_mean, float* run_var, int C, int M, float mom) {
  const double invM = 1.0 / (double)M;
  const float unbias = M > 1 ? (float)M / (float)(M - 1) : 1.f;
  for (int c = threadIdx.x; c < C; c += blockDim.x) {
    const double mean = stat_load(sums, C, 0, c, rep) * invM;
    const float var = (float)fmax(stat_load(sums, C, 1, c, rep) * invM - mean * mean, 0.0);
    run_mean[c] = (1.f - mom) * run_mean[c] + mom * (float)mean;
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
  // at most 8 groups (64 channels) per block: eight lanes of a wave then share a group and each works out the constants
  // of ONE channel (LaneShare); with 16 groups a lane has two channels and the kernels of the 640-channel layers lose
  // 2 - 3 us per launch
  r.CGB = CG >= 8 ? 8 : (CG >= 4 ? 4 : (CG >= 2 ? 2 : 1));
  r.RL = kThreads / r.CGB;
  const int cblocks = (CG + r.CGB - 1) / r.CGB;
  int rblocks = (1024 + cblocks - 1) / cblocks;                 // four workgroups per compute unit: one round of waves
  const int max_rblocks = (M + r.RL * 4 - 1) / (r.RL * 4);      // at least four rows per thread
  if (rblocks > max_rblocks) rblocks = max_rblocks;
  if (rblocks < 1) rblocks = 1;
  int rpb = (M + rblocks - 1) / rblocks;
  rpb = (rpb + r.RL - 1) / r.RL * r.RL;
  r.rows_per_block = rpb;
  r.grid = dim3(cblocks, (M + rpb - 1) / rpb, 1);
  return r;
}

// scale and shift of the 8 channels from c0 on (and of the second operand's, if there is one), see LaneShare
template <int COPIES>
__device__ __forceinline__ void bn_apply_setup(const BnApplyArgs& a, const LaneShare& ls, int c0, float (&sc)[8], float (&sh)[8],
                                               float (&sc2)[8], float (&sh2)[8]) {
  const int C = a.C;
  const double invM = 1.0 / (double)a.M;
  const bool two = a.x2 != nullptr;
  const stat_t* sums2 = two ? a.sums2 : a.sums;
  const float *gamma2 = two ? a.gamma2 : a.gamma, *beta2 = two ? a.beta2 : a.beta;
  RawTotal<COPIES> raw[2][2][2];   // [channel of this lane][x | x2][sum | sum of squares]
  float gm[2][2], bt[2][2];
  float r_sc[2] = {0.f, 0.f}, r_sh[2] = {0.f, 0.f}, r_sc2[2] = {0.f, 0.f}, r_sh2[2] = {0.f, 0.f};
  auto load = [&](int k) {   // called with constants: the arrays stay in registers
    const int c = c0 + ls.channel(k);
    chan_load(raw[k][0][0], ls, a.sums, C, 0, c, a.rep_stride);
    chan_load(raw[k][0][1], ls, a.sums, C, 1, c, a.rep_stride);
    gm[k][0] = a.gamma[c];
    bt[k][0] = a.beta[c];
    if (two) {
      chan_load(raw[k][1][0], ls, sums2, C, 0, c, a.rep_stride);
      chan_load(raw[k][1][1], ls, sums2, C, 1, c, a.rep_stride);
      gm[k][1] = gamma2[c];
      bt[k][1] = beta2[c];
    }
  };
  auto compute = [&](int k) {
    float mean, is;
    bn_moments(chan_total(raw[k][0][0], ls, a.rep_stride), chan_total(raw[k][0][1], ls, a.rep_stride), invM, a.eps, mean, is);
    r_sc[k] = gm[k][0] * is;
    r_sh[k] = bt[k][0] - mean * r_sc[k];
    if (two) {
      bn_moments(chan_total(raw[k][1][0], ls, a.rep_stride), chan_total(raw[k][1][1], ls, a.rep_stride), invM, a.eps, mean, is);
      r_sc2[k] = gm[k][1] * is;
      r_sh2[k] = bt[k][1] - mean * r_sc2[k];
    }
  };
  // every load first (one wait for memory), then the arithmetic -- unless a lane has two channels in eight copies each,
  // which would not fit the registers
  load(0);
  if (COPIES < 8 && ls.nch == 2) load(1);
  compute(0);
  if (ls.nch == 2) {
    if (COPIES >= 8) load(1);
    compute(1);
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    sc[i] = ls.gather(r_sc, i);
    sh[i] = ls.gather(r_sh, i);
  }
  if (two) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      sc2[i] = ls.gather(r_sc2, i);
      sh2[i] = ls.gather(r_sh2, i);
    }
  }
}

template <int COPIES>   // copies of the sums a lane takes (copies_per_lane): a kernel each, so that each has the registers it needs
__global__ __launch_bounds__(kThreads) void bn_apply_kernel(BnApplyArgs a, int CGB, int rows_per_block) {
  const int C = a.C;
  if (blockIdx.x == 0 && blockIdx.y == 0) {
    if (a.run_mean) bn_running(a.sums, a.rep_stride, a.run_mean, a.run_var, C, a.M, a.momentum);
    if (a.x2 && a.run_mean2) bn_running(a.sums2, a.rep_stride, a.run_mean2, a.run_var2, C, a.M, a.momentum);
  }
  const int RL = kThreads / CGB;
  const int cg = blockIdx.x * CGB + threadIdx.x % CGB, rl = threadIdx.x / CGB;
  const int c0 = cg * 8;
  // The first rows of this thread are requested BEFORE the per-channel constants are worked out, so that the two trips
  // to memory overlap (a launch of this kernel lasts about as long as two trips take).
  constexpr int NPRE = 4;
  const int row_lo = blockIdx.y * rows_per_block, row_hi = min(a.M, row_lo + rows_per_block);
  uint4 px[NPRE];
#pragma unroll
  for (int j = 0; j < NPRE; ++j) {
    const int row = row_lo + rl + j * RL;
    px[j] = (c0 < C && row < row_hi) ? *reinterpret_cast<const uint4*>(a.x + (size_t)row * C + c0) : make_uint4(0u, 0u, 0u, 0u);
  }
  float sc[8], sh[8], sc2[8], sh2[8];
  {
    const LaneShare ls(CGB);
    const bool valid = c0 < C;
    bn_apply_setup<COPIES>(a, ls, valid ? c0 : 0, sc, sh, sc2, sh2);
    if (!valid) return;
  }
  auto one_row = [&](int row, const uint4& xu) {
    const size_t o = (size_t)row * C + c0;
    float f[8];
    unpack8(xu, f);
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
      if (a.relu == 2) {
#pragma unroll
        for (int i = 0; i < 8; ++i) f[i] = fminf(f[i], 6.f);
      }
    }
    if (a.out_f32) store8_f32(a.out_f32 + o, f);
    if (a.out_b16) *reinterpret_cast<uint4*>(a.out_b16 + o) = pack8(f);
  };
#pragma unroll
  for (int j = 0; j < NPRE; ++j) {
    const int row = row_lo + rl + j * RL;
    if (row < row_hi) one_row(row, px[j]);
  }
#pragma unroll 4
  for (int row = row_lo + rl + NPRE * RL; row < row_hi; row += RL) one_row(row, *reinterpret_cast<const uint4*>(a.x + (size_t)row * C + c0));
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
  switch (host_copies_per_lane(r.CGB, a.rep_stride)) {
    case 1: hipLaunchKernelGGL(bn_apply_kernel<1>, r.grid, dim3(kThreads), 0, s, a, r.CGB, r.rows_per_block); break;
    case 2: hipLaunchKernelGGL(bn_apply_kernel<2>, r.grid, dim3(kThreads), 0, s, a, r.CGB, r.rows_per_block); break;
    case 4: hipLaunchKernelGGL(bn_apply_kernel<4>, r.grid, dim3(kThreads), 0, s, a, r.CGB, r.rows_per_block); break;
    default: hipLaunchKernelGGL(bn_apply_kernel<8>, r.grid, dim3(kThreads), 0, s, a, r.CGB, r.rows_per_block); break;
  }
  return hipGetLastError();
}

// ---- BN backward ---------------------------------------------------------------------------------
template <bool DY_F32>
__device__ __forceinline__ void load_masked_dy(const void* dy, const bf16_t* mask, float hi, size_t o, float (&g)[8]) {
  if (DY_F32)
    load8_f32(reinterpret_cast<const float*>(dy) + o, g);
  else
    unpack8(*reinterpret_cast<const uint4*>(reinterpret_cast<const bf16_t*>(dy) + o), g);
  if (!mask) return;   // dy was gated where it was produced
  float mk[8];
  unpack8(*reinterpret_cast<const uint4*>(mask + o), mk);
#pragma unroll
  for (int i = 0; i < 8; ++i)
    if (!(mk[i] > 0.f) || mk[i] >= hi) g[i] = 0.f;
}
// the upper end of the gate: +inf unless the activation was clamped (ReLU6)
__device__ __forceinline__ float gate_top(float gate_hi) { return gate_hi > 0.f ? gate_hi : __builtin_inff(); }

// batch mean and 1 / sqrt(variance + eps) of the 8 channels from c0 on, see LaneShare
template <int COPIES>
__device__ __forceinline__ void bn_moments_setup(const stat_t* sums, int rep, int C, int M, float eps, const LaneShare& ls, int c0,
                                                 float (&mu)[8], float (&iv)[8]) {
  const double invM = 1.0 / (double)M;
  RawTotal<COPIES> raw[2][2];
  float r_mu[2] = {0.f, 0.f}, r_iv[2] = {0.f, 0.f};
  auto load = [&](int k) {   // called with constants: the arrays stay in registers
    const int c = c0 + ls.channel(k);
    chan_load(raw[k][0], ls, sums, C, 0, c, rep);
    chan_load(raw[k][1], ls, sums, C, 1, c, rep);
  };
  auto compute = [&](int k) { bn_moments(chan_total(raw[k][0], ls, rep), chan_total(raw[k][1], ls, rep), invM, eps, r_mu[k], r_iv[k]); };
  load(0);
  if (ls.nch == 2) load(1);
  compute(0);
  if (ls.nch == 2) compute(1);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    mu[i] = ls.gather(r_mu, i);
    iv[i] = ls.gather(r_iv, i);
  }
}

template <bool DY_F32, int COPIES>
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
  {
    const LaneShare ls(CGB);
    const int c0 = cvalid ? cg * 8 : 0;
    bn_moments_setup<COPIES>(a.sums, a.rep_stride, C, a.M, a.eps, ls, c0, mu, iv);
  }
  if (cvalid) {
    const int row_lo = blockIdx.y * rows_per_block, row_hi = min(a.M, row_lo + rows_per_block);
#pragma unroll 2
    for (int row = row_lo + rl; row < row_hi; row += RL) {
      const size_t o = (size_t)row * C + cg * 8;
      float g[8], xv[8];
      load_masked_dy<DY_F32>(a.dy, a.mask, gate_top(a.gate_hi), o, g);
      unpack8(*reinterpret_cast<const uint4*>(a.x + o), xv);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        v[0][i] += g[i];
        v[1][i] += g[i] * ((xv[i] - mu[i]) * iv[i]);
      }
    }
  }
  block_reduce_to_global<2>(v, a.bsums, cgl, rl, CGB, RL, blockIdx.x * CGB * 8, C, smem);
}

hipError_t launch_bn_bwd_reduce(const BnBwdArgs& a, hipStream_t s) {
  if (a.C % 8 != 0 || a.C > 2048 || a.M <= 0 || (!a.mask && !a.dy_gated)) return hipErrorInvalidValue;
  const ReduceShape r = reduce_shape(a.M, a.C);
  const size_t sm = 2 * (size_t)kThreads * 8 * sizeof(float);
#define FDG_LAUNCH_REDUCE(F32, CP) \
  hipLaunchKernelGGL((bn_bwd_reduce_kernel<F32, CP>), r.grid, dim3(kThreads), sm, s, a, r.CGB, r.rows_per_block)
  switch (host_copies_per_lane(r.CGB, a.rep_stride)) {
    case 1: if (a.dy_is_f32) FDG_LAUNCH_REDUCE(true, 1); else FDG_LAUNCH_REDUCE(false, 1); break;
    case 2: if (a.dy_is_f32) FDG_LAUNCH_REDUCE(true, 2); else FDG_LAUNCH_REDUCE(false, 2); break;
    case 4: if (a.dy_is_f32) FDG_LAUNCH_REDUCE(true, 4); else FDG_LAUNCH_REDUCE(false, 4); break;
    default: if (a.dy_is_f32) FDG_LAUNCH_REDUCE(true, 8); else FDG_LAUNCH_REDUCE(false, 8); break;
  }
#undef FDG_LAUNCH_REDUCE
  return hipGetLastError();
}

// Constants of the batch-norm backward for the 8 channels from c0 on, see LaneShare.  Per channel: xhat = x*is - mean*is;
// dx = gi*g - gi*k1 - gi*k2*xhat = gi*g + (pa*x + pb).  The lanes with `writes` store dbeta and dgamma of their channel(s).
// The forward and the backward sums have copies (a.rep_stride == a.brep_stride > 0) or neither has.
template <int COPIES>
__device__ __forceinline__ void bn_bwd_setup(const BnBwdArgs& a, const LaneShare& ls, int c0, bool writes, float (&gi)[8],
                                             float (&pa)[8], float (&pb)[8]) {
  const int C = a.C, rep = a.rep_stride;
  const double invMd = 1.0 / (double)a.M;
  const float invM = (float)invMd;
  RawTotal<COPIES> raw[2][2][2];   // [channel of this lane][forward sums | backward sums][first | second sum]
  float gm[2];
  float r_gi[2] = {0.f, 0.f}, r_pa[2] = {0.f, 0.f}, r_pb[2] = {0.f, 0.f};
  auto load = [&](int k) {   // called with constants: the arrays stay in registers
    const int c = c0 + ls.channel(k);
    chan_load(raw[k][0][0], ls, a.sums, C, 0, c, rep);
    chan_load(raw[k][0][1], ls, a.sums, C, 1, c, rep);
    chan_load(raw[k][1][0], ls, a.bsums, C, 0, c, rep);
    chan_load(raw[k][1][1], ls, a.bsums, C, 1, c, rep);
    gm[k] = a.gamma[c];
  };
  auto compute = [&](int k) {
    const int c = c0 + ls.channel(k);
    const double s1 = chan_total(raw[k][0][0], ls, rep), s2 = chan_total(raw[k][0][1], ls, rep);
    const double t1 = chan_total(raw[k][1][0], ls, rep), t2 = chan_total(raw[k][1][1], ls, rep);
    float mean, is;
    bn_moments(s1, s2, invMd, a.eps, mean, is);
    const float b1 = (float)t1;
    // sum g*xhat from sum g*x and sum g: the difference is taken in double on the exact totals
    const float b2 = a.raw_sums ? is * (float)(t2 - (s1 * invMd) * t1) : (float)t2;
    const float g = gm[k] * is;
    const float k1 = b1 * invM, k2 = b2 * invM;
    r_gi[k] = g;
    r_pa[k] = -g * k2 * is;
    r_pb[k] = -g * k1 + g * k2 * is * mean;
    if (writes) {
      a.dbeta[c] = b1;
      a.dgamma[c] = b2;
    }
  };
  // every load first (one wait for memory), then the arithmetic -- unless a lane has two channels in eight copies each,
  // which would not fit the registers
  load(0);
  if (COPIES < 8 && ls.nch == 2) load(1);
  compute(0);
  if (ls.nch == 2) {
    if (COPIES >= 8) load(1);
    compute(1);
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    gi[i] = ls.gather(r_gi, i);
    pa[i] = ls.gather(r_pa, i);
    pb[i] = ls.gather(r_pb, i);
  }
}

// dx = gamma*invstd*(g - S1/M - xhat*S2/M) [+ addend];  dgamma = S2, dbeta = S1
template <bool DY_F32, int COPIES>
__global__ __launch_bounds__(kThreads) void bn_bwd_apply_kernel(BnBwdArgs a, int CGB, int rows_per_block) {
  const int C = a.C;
  const int RL = kThreads / CGB;
  const int cg = blockIdx.x * CGB + threadIdx.x % CGB, rl = threadIdx.x / CGB;
  const int c0 = cg * 8;
  // as in bn_apply_kernel: the first rows are requested before the per-channel constants are worked out
  constexpr int NPRE = 4;
  const bool rows_wanted = a.out_f32 || a.out_b16;
  const int row_lo = blockIdx.y * rows_per_block, row_hi = rows_wanted ? min(a.M, row_lo + rows_per_block) : 0;
  uint4 pdy[NPRE][DY_F32 ? 2 : 1], px[NPRE], pmk[NPRE];
#pragma unroll
  for (int j = 0; j < NPRE; ++j) {
    const int row = row_lo + rl + j * RL;
    const bool on = c0 < C && row < row_hi;
    const size_t o = on ? (size_t)row * C + c0 : 0;
    if (DY_F32) {
      pdy[j][0] = on ? *reinterpret_cast<const uint4*>(reinterpret_cast<const float*>(a.dy) + o) : make_uint4(0u, 0u, 0u, 0u);
      pdy[j][DY_F32 ? 1 : 0] = on ? *reinterpret_cast<const uint4*>(reinterpret_cast<const float*>(a.dy) + o + 4) : make_uint4(0u, 0u, 0u, 0u);
    } else {
      pdy[j][0] = on ? *reinterpret_cast<const uint4*>(reinterpret_cast<const bf16_t*>(a.dy) + o) : make_uint4(0u, 0u, 0u, 0u);
    }
    px[j] = on ? *reinterpret_cast<const uint4*>(a.x + o) : make_uint4(0u, 0u, 0u, 0u);
    pmk[j] = (on && a.mask) ? *reinterpret_cast<const uint4*>(a.mask + o) : make_uint4(0u, 0u, 0u, 0u);
  }
  float gi[8], pa[8], pb[8];
  {
    const LaneShare ls(CGB);
    const bool valid = c0 < C;
    const bool writes = valid && blockIdx.y == 0 && threadIdx.x < 64 && ls.part == 0;   // one lane per channel of the block
    bn_bwd_setup<COPIES>(a, ls, valid ? c0 : 0, writes, gi, pa, pb);
    if (!valid) return;
  }
  if (!rows_wanted) return;
  auto finish_row = [&](int row, float (&g)[8], const uint4& xu) {
    const size_t o = (size_t)row * C + c0;
    float xv[8];
    unpack8(xu, xv);
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
  };
#pragma unroll
  for (int j = 0; j < NPRE; ++j) {
    const int row = row_lo + rl + j * RL;
    if (row >= row_hi) continue;
    float g[8];
    if (DY_F32) {
      const uint4 lo = pdy[j][0], hi = pdy[j][DY_F32 ? 1 : 0];
      g[0] = __builtin_bit_cast(float, lo.x); g[1] = __builtin_bit_cast(float, lo.y); g[2] = __builtin_bit_cast(float, lo.z);
      g[3] = __builtin_bit_cast(float, lo.w); g[4] = __builtin_bit_cast(float, hi.x); g[5] = __builtin_bit_cast(float, hi.y);
      g[6] = __builtin_bit_cast(float, hi.z); g[7] = __builtin_bit_cast(float, hi.w);
    } else {
      unpack8(pdy[j][0], g);
    }
    if (a.mask) {
      float mk[8];
      unpack8(pmk[j], mk);
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (!(mk[i] > 0.f) || mk[i] >= gate_top(a.gate_hi)) g[i] = 0.f;
    }
    finish_row(row, g, px[j]);
  }
#pragma unroll 4
  for (int row = row_lo + rl + NPRE * RL; row < row_hi; row += RL) {
    const size_t o = (size_t)row * C + c0;
    float g[8];
    load_masked_dy<DY_F32>(a.dy, a.mask, gate_top(a.gate_hi), o, g);
    finish_row(row, g, *reinterpret_cast<const uint4*>(a.x + o));
  }
}

hipError_t launch_bn_bwd_apply(const BnBwdArgs& a_in, hipStream_t s) {
  BnBwdArgs a = a_in;
  if (a.dy_gated) a.mask = nullptr;
  if (a.C % 8 != 0 || a.C > 2048 || a.M <= 0 || (!a.mask && !a.dy_gated)) return hipErrorInvalidValue;
  const auto al16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
  if (!al16(a.sums) || !al16(a.gamma) || !al16(a.bsums) || !al16(a.dgamma) || !al16(a.dbeta)) return hipErrorInvalidValue;
  if (a.rep_stride != a.brep_stride) return hipErrorInvalidValue;   // copies of both sums arrays, or of neither
  ApplyShape r = apply_shape(a.M, a.C);
  if (!a.out_f32 && !a.out_b16) r.grid.y = 1;   // only dgamma / dbeta
#define FDG_LAUNCH_APPLY(F32, CP) \
  hipLaunchKernelGGL((bn_bwd_apply_kernel<F32, CP>), r.grid, dim3(kThreads), 0, s, a, r.CGB, r.rows_per_block)
  switch (host_copies_per_lane(r.CGB, a.rep_stride)) {
    case 1: if (a.dy_is_f32) FDG_LAUNCH_APPLY(true, 1); else FDG_LAUNCH_APPLY(false, 1); break;
    case 2: if (a.dy_is_f32) FDG_LAUNCH_APPLY(true, 2); else FDG_LAUNCH_APPLY(false, 2); break;
    case 4: if (a.dy_is_f32) FDG_LAUNCH_APPLY(true, 4); else FDG_LAUNCH_APPLY(false, 4); break;
    default: if (a.dy_is_f32) FDG_LAUNCH_APPLY(true, 8); else FDG_LAUNCH_APPLY(false, 8); break;
  }
#undef FDG_LAUNCH_APPLY
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

// ---- update and snapshot in one pass ---------------------------------------------------------------
// Eq. 11 on every parameter AND the bf16 copies of the updated convolution weights that the next forward will use (both
// layouts), so that theta is read once: 12 bytes read and 8 + 2 * 2 written per convolution weight.  Blocks
// [0, conv_blocks) take one 64 (co) x 64 (ci) tile of one tap of one convolution, as emit_weights_kernel does: the
// update runs along ci (16 lanes x float4 = one 256-byte run per output channel), the new value goes to the
// forward layout [co][tap][cip] from registers and to the data-gradient layout [cip][tap][co] after a transpose
// through LDS.  The other blocks update the small parameters (batch-norm scale / shift, the classifier) and copy
// them, fp32, into the snapshot.  Convolutions whose input channels are not a multiple of 4 (the 3-channel stem)
// take one element per lane instead of four.
__global__ __launch_bounds__(kThreads) void sgd_emit_kernel(float* __restrict__ params, float* __restrict__ mom,
                                                            const float* __restrict__ grads, bf16_t* __restrict__ warena,
                                                            float* __restrict__ small_snap, const WeightEmitEntry* __restrict__ table,
                                                            int nconv, int conv_blocks, size_t small_off, size_t small_count,
                                                            float lr, float mu, float wd) {
  __shared__ float tile[64][65];
  if ((int)blockIdx.x >= conv_blocks) {   // small parameters: flat, four at a time
    const size_t i4 = (size_t)(blockIdx.x - conv_blocks) * kThreads + threadIdx.x;
    if (i4 * 4 >= small_count) return;
    const size_t i = small_off + i4 * 4;
    float4 t = *reinterpret_cast<const float4*>(params + i), m = *reinterpret_cast<const float4*>(mom + i);
    const float4 g = *reinterpret_cast<const float4*>(grads + i);
    m.x = mu * m.x + (g.x + wd * t.x); m.y = mu * m.y + (g.y + wd * t.y);
    m.z = mu * m.z + (g.z + wd * t.z); m.w = mu * m.w + (g.w + wd * t.w);
    t.x -= lr * m.x; t.y -= lr * m.y; t.z -= lr * m.z; t.w -= lr * m.w;
    *reinterpret_cast<float4*>(mom + i) = m;
    *reinterpret_cast<float4*>(params + i) = t;
    *reinterpret_cast<float4*>(small_snap + i4 * 4) = t;
    return;
  }
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
  if (e.Ci % 4 == 0) {
    const int ci = ci0 + 4 * (threadIdx.x & 15);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int col = (threadIdx.x >> 4) + 16 * r, co = co0 + col;
      float4 th = make_float4(0.f, 0.f, 0.f, 0.f);
      if (co < e.Co && ci < e.Ci) {
        const size_t o = e.src_off + ((size_t)co * e.T + t) * e.Ci + ci;
        th = *reinterpret_cast<const float4*>(params + o);
        float4 m = *reinterpret_cast<const float4*>(mom + o);
        const float4 g = *reinterpret_cast<const float4*>(grads + o);
        m.x = mu * m.x + (g.x + wd * th.x); m.y = mu * m.y + (g.y + wd * th.y);
        m.z = mu * m.z + (g.z + wd * th.z); m.w = mu * m.w + (g.w + wd * th.w);
        th.x -= lr * m.x; th.y -= lr * m.y; th.z -= lr * m.z; th.w -= lr * m.w;
        *reinterpret_cast<float4*>(mom + o) = m;
        *reinterpret_cast<float4*>(params + o) = th;
      }
      const int cl = 4 * (threadIdx.x & 15);
      tile[col][cl] = th.x; tile[col][cl + 1] = th.y; tile[col][cl + 2] = th.z; tile[col][cl + 3] = th.w;
      if (co < e.Co && ci < e.Cip)   // the padding channels of the copy are written too (zeros)
        *reinterpret_cast<uint2*>(warena + e.w_off + ((size_t)co * e.T + t) * e.Cip + ci) =
            make_uint2(pack_bf16x2(th.x, th.y), pack_bf16x2(th.z, th.w));
    }
  } else {
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int r = ty; r < 64; r += 4) {
      const int co = co0 + r, ci = ci0 + tx;
      float th = 0.f;
      if (co < e.Co && ci < e.Ci) {
        const size_t o = e.src_off + ((size_t)co * e.T + t) * e.Ci + ci;
        th = params[o];
        const float m = mu * mom[o] + (grads[o] + wd * th);
        th -= lr * m;
        mom[o] = m;
        params[o] = th;
      }
      tile[r][tx] = th;
      if (co < e.Co && ci < e.Cip) warena[e.w_off + ((size_t)co * e.T + t) * e.Cip + ci] = (bf16_t)th;
    }
  }
  __syncthreads();
  // data-gradient layout: 8 consecutive output channels of one input channel per lane (16 bytes)
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    const int cil = (threadIdx.x >> 3) + 32 * r, ci = ci0 + cil, col = 8 * (threadIdx.x & 7), co = co0 + col;
    if (ci < e.Cip && co < e.Co) {   // Co is a multiple of 8: a group of 8 exists or does not
      float f[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) f[j] = tile[col + j][cil];
      *reinterpret_cast<uint4*>(warena + e.wt_off + ((size_t)ci * e.T + t) * e.Co + co) = pack8(f);
    }
  }
}
hipError_t launch_sgd_emit(float* params, float* mom, const float* grads, bf16_t* warena, float* small_snap,
                           const WeightEmitEntry* table_dev, int nconv, int conv_blocks, size_t small_off, size_t small_count,
                           float lr, float mu, float wd, hipStream_t s) {
  if (small_off % 4 != 0 || small_count % 4 != 0 || conv_blocks < 0) return hipErrorInvalidValue;
  const size_t small_blocks = (small_count / 4 + kThreads - 1) / kThreads;
  const size_t blocks = (size_t)conv_blocks + small_blocks;
  if (blocks == 0) return hipSuccess;
  hipLaunchKernelGGL(sgd_emit_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, s, params, mom, grads, warena, small_snap, table_dev,
                     nconv, conv_blocks, small_off, small_count, lr, mu, wd);
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

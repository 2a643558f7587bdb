// Implicit-GEMM convolutions on gfx950 matrix cores (v_mfma_f32_16x16x32_bf16, fp32 accumulate).
//
// Two kernels serve every convolution of an FDG module step (Section III-A of arXiv 1906.09108: the
// forward of the newest batch, and the chain-rule backward of Eq. 10 on the stale batch):
//   conv_gather_kernel : out[pixel, c] = sum_{tap,k} in[pixel+tap, k] * w[c, tap, k]
//                        forward convolution and data gradient (flipped taps, transposed weights,
//                        stride-2 data gradient as four parity classes).
//   conv_wgrad_kernel  : dw[co, tap, ci] += sum_pixel dy[pixel, co] * x[pixel+tap, ci]
//                        the contraction runs over pixels, so both operands are transposed in
//                        registers on their way to LDS; split over pixels with fp32 atomics.
//
// MFMA operand layout used throughout (16x16x32, 64 lanes): lane l supplies row (l & 15) of A and
// column (l & 15) of B, each with the 8 consecutive k values 8*(l >> 4) .. +7; lane l receives
// D[4*(l >> 4) + v][l & 15] in accumulator component v.
#include <algorithm>
#include "conv_common.h"
#include <stdio.h>
#include <stdlib.h>

namespace fdg {

static thread_local const char* g_last_kernel = "";
void note_kernel(const char* name) { g_last_kernel = name; }
const char* last_kernel() { return g_last_kernel; }

// ------------------------------------------------------------------------------------------------
// gather-form convolution
// ------------------------------------------------------------------------------------------------
// Several output geometries in one launch (GatherConvArgs::nclass > 1: the parity classes of a stride-2 data gradient):
// blockIdx.z is the class, which replaces the output grid, its offsets and the tap list.
template <int BM, int BN, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(256) void conv_gather_kernel(GatherConvArgs a_in) {
  static_assert(WAVES_M * WAVES_N == 4, "four waves");
  GatherConvArgs a = a_in;
  const int cls = a_in.nclass > 1 ? (int)blockIdx.z : 0;
  if (a_in.nclass > 1) {
    a.OH = a_in.cOH[cls]; a.OW = a_in.cOW[cls]; a.ooh = a_in.cooh[cls]; a.oow = a_in.coow[cls]; a.ntaps = a_in.cntaps[cls];
  }
  constexpr int PITCH = 40;  // 32 k values + 8 pad: 80-byte rows keep 16-lane b128 reads conflict free
  constexpr int TM = BM / WAVES_M, TN = BN / WAVES_N;
  constexpr int FM = TM / 16, FN = TN / 16;
  constexpr int UX = (BM * 4 + 255) / 256;  // 16-byte units per thread of the pixel tile
  constexpr int UW = (BN * 4 + 255) / 256;  // ... of the weight tile
  __shared__ __attribute__((aligned(16))) bf16_t sX[2][BM * PITCH];
  __shared__ __attribute__((aligned(16))) bf16_t sW[2][BN * PITCH];
  __shared__ int sTap[16];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave % WAVES_M, wave_n = wave / WAVES_M;
  const int Mtot = a.N * a.OH * a.OW;
  const int m0 = blockIdx.x * BM, c0 = blockIdx.y * BN;
  if (m0 >= Mtot) return;   // a class with fewer tiles than the largest one (the whole workgroup leaves)
  if (tid < 16) sTap[tid] = tid < a.ntaps ? (a_in.nclass > 1 ? a_in.ctap[cls][tid & 3] : a_in.tap[tid < 9 ? tid : 0]) : 0;

  // per-thread rows of the two tiles: row = tid/4 + 64*j, fixed k-unit kq = tid%4
  const int kq = tid & 3;
  int pbase[UX], ih0[UX], iw0[UX];
#pragma unroll
  for (int j = 0; j < UX; ++j) {
    const int row = (tid >> 2) + 64 * j, m = m0 + row;
    if (row < BM && m < Mtot) {
      const int ow = m % a.OW, t2 = m / a.OW, oh = t2 % a.OH, n = t2 / a.OH;
      pbase[j] = n * a.Hi * a.Wi;
      ih0[j] = oh * a.in_stride;
      iw0[j] = ow * a.in_stride;
    } else {
      pbase[j] = 0;
      ih0[j] = -(1 << 20);
      iw0[j] = 0;
    }
  }
  const bf16_t* wrow[UW];
  bool wok[UW];
#pragma unroll
  for (int j = 0; j < UW; ++j) {
    const int row = (tid >> 2) + 64 * j, c = c0 + row;
    wok[j] = row < BN && c < a.w_rows;
    wrow[j] = a.w + (size_t)(wok[j] ? c : 0) * a.Kw;
  }
  const int cpt = a.Ci >> 3;  // 16-byte units per tap
  int tap = kq / cpt, c8 = kq % cpt;
  const int nchunks = (a.ntaps * cpt + 3) >> 2;

  f32x4 acc[FN][FM];
#pragma unroll
  for (int i = 0; i < FN; ++i)
#pragma unroll
    for (int j = 0; j < FM; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  uint4 rx[UX], rw[UW];
  const uint4 zero4 = make_uint4(0, 0, 0, 0);
  __syncthreads();  // sTap visible

  auto load_global = [&]() {
    const bool tv = tap < a.ntaps;
    const int tp = tv ? sTap[tap] : pack_tap(0, 0, 0);
    const int dh = (tp & 0xff) - 8, dw = ((tp >> 8) & 0xff) - 8, kofs = tp >> 16;
#pragma unroll
    for (int j = 0; j < UX; ++j) {
      const int ih = ih0[j] + dh, iw = iw0[j] + dw;
      const bool ok = tv && (unsigned)ih < (unsigned)a.Hi && (unsigned)iw < (unsigned)a.Wi;
      rx[j] = ok ? *reinterpret_cast<const uint4*>(a.in + ((size_t)(pbase[j] + ih * a.Wi + iw) * a.Ci + c8 * 8))
                 : zero4;
    }
#pragma unroll
    for (int j = 0; j < UW; ++j)
      rw[j] = (tv && wok[j]) ? *reinterpret_cast<const uint4*>(wrow[j] + (size_t)kofs * a.Ci + c8 * 8) : zero4;
    // advance this thread's k-unit by one chunk (4 units)
    c8 += 4;
    while (c8 >= cpt) {
      c8 -= cpt;
      ++tap;
    }
  };
  auto store_lds = [&](int buf) {
#pragma unroll
    for (int j = 0; j < UX; ++j) {
      const int row = (tid >> 2) + 64 * j;
      if (row < BM) *reinterpret_cast<uint4*>(&sX[buf][row * PITCH + kq * 8]) = rx[j];
    }
#pragma unroll
    for (int j = 0; j < UW; ++j) {
      const int row = (tid >> 2) + 64 * j;
      if (row < BN) *reinterpret_cast<uint4*>(&sW[buf][row * PITCH + kq * 8]) = rw[j];
    }
  };

  load_global();
  store_lds(0);
  __syncthreads();
  for (int kc = 0; kc < nchunks; ++kc) {
    const int buf = kc & 1;
    const bool more = kc + 1 < nchunks;
    if (more) load_global();
    bf16x8 fa[FN], fb[FM];
#pragma unroll
    for (int f = 0; f < FN; ++f)
      fa[f] = *reinterpret_cast<const bf16x8*>(&sW[buf][(wave_n * TN + f * 16 + (lane & 15)) * PITCH + (lane >> 4) * 8]);
#pragma unroll
    for (int f = 0; f < FM; ++f)
      fb[f] = *reinterpret_cast<const bf16x8*>(&sX[buf][(wave_m * TM + f * 16 + (lane & 15)) * PITCH + (lane >> 4) * 8]);
#pragma unroll
    for (int i = 0; i < FN; ++i)
#pragma unroll
      for (int j = 0; j < FM; ++j) acc[i][j] = mfma16(fa[i], fb[j], acc[i][j]);
    if (more) store_lds(buf ^ 1);
    __syncthreads();
  }

  store_tile<FM, FN, BN>(a, acc, m0 + wave_m * TM, c0, wave_n * TN, lane);
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
static hipError_t run_gather(const GatherConvArgs& a, hipStream_t s) {
  int Mtot = a.N * a.OH * a.OW;
  if (a.nclass > 1) {
    if (a.nclass > 4) return hipErrorInvalidValue;
    Mtot = 0;
    for (int i = 0; i < a.nclass; ++i) {
      if (a.cntaps[i] < 0 || a.cntaps[i] > 4) return hipErrorInvalidValue;
      Mtot = std::max(Mtot, a.N * a.cOH[i] * a.cOW[i]);
    }
    if (Mtot <= 0) return hipErrorInvalidValue;
  }
  dim3 grid((Mtot + BM - 1) / BM, (a.Co + BN - 1) / BN, a.nclass > 1 ? a.nclass : 1);
  static char name[64];
  if (!name[0]) snprintf(name, sizeof(name), "conv_gather_kernel<%d, %d, %d, %d>", BM, BN, WAVES_M, WAVES_N);
  note_kernel(name);
  hipLaunchKernelGGL((conv_gather_kernel<BM, BN, WAVES_M, WAVES_N>), grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_conv_gather(const GatherConvArgs& a, hipStream_t s) {
  if (a.Ci % 8 != 0 || a.Co % 4 != 0 || a.ntaps < 0 || a.ntaps > 9 || (a.nclass <= 1 && a.N * a.OH * a.OW <= 0) || a.Kw % 8 != 0)
    return hipErrorInvalidValue;
  if (conv_gather_wide_applies(a)) return launch_conv_gather_wide(a, s);
  if (conv_narrow_applies(a)) return launch_conv_narrow(a, s);
  if (a.gate || a.bnx) return hipErrorInvalidValue;   // the generic kernel is not asked for them (conv_dgrad_gates)
  if (a.Co <= 16) return run_gather<256, 16, 4, 1>(a, s);
  if (a.Co <= 32) return run_gather<256, 32, 4, 1>(a, s);
  if (a.Co <= 64) return run_gather<128, 64, 2, 2>(a, s);
  return run_gather<128, 128, 2, 2>(a, s);
}

// ------------------------------------------------------------------------------------------------
// weight gradient
// ------------------------------------------------------------------------------------------------
// 8 pixels x 8 channels (one uint4 per pixel) -> per channel the 8 pixels as one uint4
__device__ __forceinline__ void transpose8x8(const uint4 (&r)[8], uint4 (&o)[8]) {
#define FDG_TR_PAIR(F, P)                                                        \
  {                                                                              \
    uint32_t lo[4], hi[4];                                                       \
    _Pragma("unroll") for (int q = 0; q < 4; ++q) {                              \
      const uint32_t p0 = r[2 * q].F, p1 = r[2 * q + 1].F;                       \
      lo[q] = (p0 & 0xffffu) | (p1 << 16);                                       \
      hi[q] = (p0 >> 16) | (p1 & 0xffff0000u);                                   \
    }                                                                            \
    o[2 * P] = make_uint4(lo[0], lo[1], lo[2], lo[3]);                           \
    o[2 * P + 1] = make_uint4(hi[0], hi[1], hi[2], hi[3]);                       \
  }
  FDG_TR_PAIR(x, 0)
  FDG_TR_PAIR(y, 1)
  FDG_TR_PAIR(z, 2)
  FDG_TR_PAIR(w, 3)
#undef FDG_TR_PAIR
}

struct WgradLaunch {
  int chunks_per_split;
  int ci_tiles;
  float* partial;        // when set: pixel split z, contraction part wk store their block at partial + (z * WK + wk) * split_stride
  size_t split_stride;   // (plain stores: a second kernel adds the parts in a fixed order); else fp32 atomics into dw
};

template <int BM, int BN, int WM, int WN, int WK>
__global__ __launch_bounds__(256) void conv_wgrad_kernel(WgradArgs a, WgradLaunch L) {
  static_assert(WM * WN * WK == 4, "four waves");
  constexpr int KSTEPS = WK == 1 ? 2 : 1;
  constexpr int BK = 32 * WK * KSTEPS;
  constexpr int PITCH = BK + 8;
  constexpr int TM = BM / WM, TN = BN / WN;
  constexpr int FA = TM / 16, FB = TN / 16;
  constexpr int CGA = BM / 8, CGB = BN / 8, PG = BK / 8;
  constexpr int NUA = CGA * PG, NUB = CGB * PG;
  static_assert(NUA + NUB <= 256, "one 8x8 unit per thread");
  __shared__ __attribute__((aligned(16))) bf16_t sA[2][BM * PITCH];
  __shared__ __attribute__((aligned(16))) bf16_t sB[2][BN * PITCH];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WM, wn = (wave / WM) % WN, wk = wave / (WM * WN);
  const int Mtot = a.N * a.OH * a.OW;
  const int co0 = blockIdx.x * BM;
  const int tapi = blockIdx.y / L.ci_tiles, ci0 = (blockIdx.y % L.ci_tiles) * BN;
  const int tp = a.tap[tapi];
  const int dh = (tp & 0xff) - 8, dw = ((tp >> 8) & 0xff) - 8;
  const int total_chunks = (Mtot + BK - 1) / BK;
  const int chunk_lo = blockIdx.z * L.chunks_per_split;
  const int chunk_hi = min(total_chunks, chunk_lo + L.chunks_per_split);
  const bool row8 = (a.OW % 8) == 0;  // the 8 pixels of a unit share one image row

  const bool isA = tid < NUA, isB = !isA && tid < NUA + NUB;
  const int u = isA ? tid : tid - NUA;
  const int cg = isA ? u % CGA : u % CGB, pg = isA ? u / CGA : u / CGB;
  const int chan = (isA ? co0 : ci0) + cg * 8;
  const bool chan_ok = isA ? chan < a.Co : (isB && chan < a.Cx);

  f32x4 acc[FA][FB];
#pragma unroll
  for (int i = 0; i < FA; ++i)
#pragma unroll
    for (int j = 0; j < FB; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  uint4 r[8];
  const uint4 zero4 = make_uint4(0, 0, 0, 0);
  auto load_global = [&](int chunk) {
    const int mb = chunk * BK + pg * 8;
    if (isA) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int m = mb + i;
        r[i] = (chan_ok && m < Mtot) ? *reinterpret_cast<const uint4*>(a.dy + (size_t)m * a.Co + chan) : zero4;
      }
    } else if (row8) {
      const int ow0 = mb % a.OW, t2 = mb / a.OW, oh = t2 % a.OH, n = t2 / a.OH;
      const int ih = oh * a.stride + dh;
      const bool rowok = chan_ok && mb < Mtot && (unsigned)ih < (unsigned)a.Hi;
      const size_t rbase = ((size_t)n * a.Hi + ih) * a.Wi;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int iw = (ow0 + i) * a.stride + dw;
        r[i] = (rowok && (unsigned)iw < (unsigned)a.Wi)
                   ? *reinterpret_cast<const uint4*>(a.x + (rbase + iw) * a.Cx + chan)
                   : zero4;
      }
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int m = mb + i;
        const int ow = m % a.OW, t2 = m / a.OW, oh = t2 % a.OH, n = t2 / a.OH;
        const int ih = oh * a.stride + dh, iw = ow * a.stride + dw;
        const bool ok = chan_ok && m < Mtot && (unsigned)ih < (unsigned)a.Hi && (unsigned)iw < (unsigned)a.Wi;
        r[i] = ok ? *reinterpret_cast<const uint4*>(a.x + (((size_t)n * a.Hi + ih) * a.Wi + iw) * a.Cx + chan) : zero4;
      }
    }
  };
  auto store_lds = [&](int buf) {
    if (!(isA || isB)) return;
    uint4 o[8];
    transpose8x8(r, o);
    bf16_t* base = (isA ? sA[buf] : sB[buf]) + (cg * 8) * PITCH + pg * 8;
#pragma unroll
    for (int c = 0; c < 8; ++c) *reinterpret_cast<uint4*>(base + c * PITCH) = o[c];
  };

  if (chunk_lo < chunk_hi) {
    load_global(chunk_lo);
    store_lds(0);
  }
  __syncthreads();
  for (int ch = chunk_lo; ch < chunk_hi; ++ch) {
    const int buf = (ch - chunk_lo) & 1;
    const bool more = ch + 1 < chunk_hi;
    if (more) load_global(ch + 1);
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      const int kslot = (WK == 1 ? ks : wk) * 32 + (lane >> 4) * 8;
      bf16x8 fa[FA], fb[FB];
#pragma unroll
      for (int f = 0; f < FA; ++f)
        fa[f] = *reinterpret_cast<const bf16x8*>(&sA[buf][(wm * TM + f * 16 + (lane & 15)) * PITCH + kslot]);
#pragma unroll
      for (int f = 0; f < FB; ++f)
        fb[f] = *reinterpret_cast<const bf16x8*>(&sB[buf][(wn * TN + f * 16 + (lane & 15)) * PITCH + kslot]);
#pragma unroll
      for (int i = 0; i < FA; ++i)
#pragma unroll
        for (int j = 0; j < FB; ++j) acc[i][j] = mfma16(fa[i], fb[j], acc[i][j]);
    }
    if (more) store_lds(buf ^ 1);
    __syncthreads();
  }

  // D[co][ci]: lane holds co = 4*(lane>>4)+v, ci = lane&15
  if (chunk_lo >= chunk_hi) return;
  float* part = L.partial ? L.partial + (size_t)(blockIdx.z * WK + wk) * L.split_stride : nullptr;
#pragma unroll
  for (int i = 0; i < FA; ++i)
#pragma unroll
    for (int j = 0; j < FB; ++j) {
      const int ci = ci0 + wn * TN + j * 16 + (lane & 15);
      if (ci >= a.Ci) continue;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int co = co0 + wm * TM + i * 16 + 4 * (lane >> 4) + v;
        if (co >= a.Co) continue;
        const size_t o = ((size_t)co * a.ntaps + tapi) * a.Ci + ci;
        if (part) part[o] = acc[i][j][v];
        else atomicAdd(a.dw + o, acc[i][j][v]);
      }
    }
}

// pixel splits of the kernel above for a shape, and the parts (splits x contraction parts) its partial sums take
template <int BM, int BN, int WK>
static void wgrad_plan(const WgradArgs& a, int& splits, int& chunks_per_split, int& parts) {
  constexpr int BK = 32 * WK * (WK == 1 ? 2 : 1);
  const int Mtot = a.N * a.OH * a.OW;
  const int co_tiles = (a.Co + BM - 1) / BM, ci_tiles = (a.Ci + BN - 1) / BN;
  const int total_chunks = (Mtot + BK - 1) / BK;
  const int base = co_tiles * ci_tiles * a.ntaps;
  splits = (1024 + base - 1) / base;
  if (splits > total_chunks) splits = total_chunks;
  if (splits < 1) splits = 1;
  chunks_per_split = (total_chunks + splits - 1) / splits;
  splits = (total_chunks + chunks_per_split - 1) / chunks_per_split;   // every split has at least one chunk
  parts = splits * WK;
}
hipError_t launch_wgrad_reduce(float* dw, const float* partial, size_t elems, int parts, int overwrite, hipStream_t s);

template <int BM, int BN, int WM, int WN, int WK>
static hipError_t run_wgrad(const WgradArgs& a, hipStream_t s) {
  const int co_tiles = (a.Co + BM - 1) / BM, ci_tiles = (a.Ci + BN - 1) / BN;
  int splits, parts;
  WgradLaunch L;
  wgrad_plan<BM, BN, WK>(a, splits, L.chunks_per_split, parts);
  L.ci_tiles = ci_tiles;
  const size_t elems = (size_t)a.Co * a.ntaps * a.Ci;
  // with scratch memory every part stores its block and a second kernel adds the parts in a fixed order (the result is
  // the same on every run); without it the parts add into dw with fp32 atomics
  const bool stored = a.scratch && elems % 4 == 0 && a.scratch_bytes >= (size_t)parts * elems * sizeof(float);
  L.partial = stored ? a.scratch : nullptr;
  L.split_stride = elems;
  if (!stored && a.overwrite) {   // atomics only add
    hipError_t e = launch_fill_f32(a.dw, elems, 0.f, s);
    if (e != hipSuccess) return e;
  }
  dim3 grid(co_tiles, ci_tiles * a.ntaps, splits);
  static char name[64];
  if (!name[0]) snprintf(name, sizeof(name), "conv_wgrad_kernel<%d, %d, %d, %d, %d>", BM, BN, WM, WN, WK);
  note_kernel(name);
  hipLaunchKernelGGL((conv_wgrad_kernel<BM, BN, WM, WN, WK>), grid, dim3(256), 0, s, a, L);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !stored) return e;
  return launch_wgrad_reduce(a.dw, a.scratch, elems, parts, a.overwrite, s);
}

// bytes of scratch with which the kernel above stores its parts instead of adding them with atomics
static size_t generic_wgrad_scratch_bytes(const WgradArgs& a) {
  int splits, cps, parts;
  if (a.Co <= 64 && a.Cx <= 64) wgrad_plan<32, 32, 4>(a, splits, cps, parts);
  else if (a.Cx <= 32) wgrad_plan<128, 32, 1>(a, splits, cps, parts);
  else wgrad_plan<128, 128, 1>(a, splits, cps, parts);
  const size_t elems = (size_t)a.Co * a.ntaps * a.Ci;
  return elems % 4 == 0 ? (size_t)parts * elems * sizeof(float) : 0;
}

hipError_t launch_conv_wgrad(const WgradArgs& a, hipStream_t s) {
  if (a.Co % 8 != 0 || a.Cx % 8 != 0 || a.Ci > a.Cx || a.ntaps < 1 || a.ntaps > 9 || a.N * a.OH * a.OW <= 0)
    return hipErrorInvalidValue;
  if (conv_wgrad128_applies(a)) return launch_conv_wgrad128(a, s);
  if (conv_wgrad_tall_applies(a)) return launch_conv_wgrad_tall(a, s);
  if (conv_wgrad_wide_applies(a)) return launch_conv_wgrad_wide(a, s);
  if (conv_wgrad_narrow_applies(a) && a.scratch && a.scratch_bytes >= conv_wgrad_narrow_scratch_bytes(a))
    return launch_conv_wgrad_narrow(a, s);
  if (a.Co <= 64 && a.Cx <= 64) return run_wgrad<32, 32, 1, 1, 4>(a, s);
  if (a.Cx <= 32) return run_wgrad<128, 32, 4, 1, 1>(a, s);   // many output channels from few inputs (WRN's 16 -> 160)
  return run_wgrad<128, 128, 2, 2, 1>(a, s);
}

// ------------------------------------------------------------------------------------------------
// geometry of the three passes of one convolution
// ------------------------------------------------------------------------------------------------
static GatherConvArgs forward_args(const ConvShape& c, const bf16_t* x, const bf16_t* w, const float* addend, float* out_f32,
                                   bf16_t* out_b16, stat_t* stats, int stats_rep_stride) {
  GatherConvArgs a{};
  a.stats_rep_stride = stats_rep_stride;
  a.in = x; a.w = w; a.addend = addend; a.addmask = nullptr; a.out_f32 = out_f32; a.out_b16 = out_b16; a.stats = stats;
  a.N = c.N; a.Hi = c.Hi; a.Wi = c.Wi; a.Ci = c.Cip;
  a.OH = c.Ho(); a.OW = c.Wo(); a.in_stride = c.stride;
  a.OHf = c.Ho(); a.OWf = c.Wo(); a.out_stride = 1; a.ooh = 0; a.oow = 0;
  a.Co = c.Co; a.w_rows = c.Co; a.Kw = c.T * c.Cip;
  a.ntaps = c.T;
  if (c.T == 9) {
    for (int r = 0; r < 3; ++r)
      for (int q = 0; q < 3; ++q) a.tap[r * 3 + q] = pack_tap(r - 1, q - 1, r * 3 + q);
  } else {
    a.tap[0] = pack_tap(0, 0, 0);
  }
  return a;
}

hipError_t conv_forward(const ConvShape& c, const bf16_t* x, const bf16_t* w, const float* addend, float* out_f32,
                        bf16_t* out_b16, stat_t* stats, hipStream_t s, int stats_rep_stride) {
  return launch_conv_gather(forward_args(c, x, w, addend, out_f32, out_b16, stats, stats_rep_stride), s);
}

bool conv_forward_bn_applies(const ConvShape& c, bool with_residual) {
  if (c.Ci != c.Cip) return false;
  return conv_narrow_transforms(forward_args(c, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0), with_residual ? 3 : 0);
}

hipError_t conv_forward_bn(const ConvShape& c, const ConvInputBn& bn, const bf16_t* w, const float* addend, float* out_f32,
                           bf16_t* out_b16, stat_t* stats, hipStream_t s, int stats_rep_stride) {
  if (!bn.x_raw || !bn.sums || !bn.gamma || !bn.beta || !bn.act_out || !conv_forward_bn_applies(c, bn.res_f32 != nullptr))
    return hipErrorInvalidValue;
  GatherConvArgs a = forward_args(c, nullptr, w, addend, out_f32, out_b16, stats, stats_rep_stride);
  a.tr_mode = 1; a.tr_p = bn.x_raw; a.tr_q = bn.res_f32; a.tr_out = bn.act_out; a.tr_out_f32 = bn.act_out_f32; a.tr_sums = bn.sums; a.tr_gamma = bn.gamma; a.tr_beta = bn.beta;
  a.tr_run_mean = bn.run_mean; a.tr_run_var = bn.run_mean ? bn.run_var : nullptr;
  a.tr_eps = bn.eps; a.tr_momentum = bn.momentum; a.tr_rep_stride = bn.rep_stride;
  return launch_conv_narrow(a, s);
}

static hipError_t conv_dgrad_impl(const ConvShape& c, const bf16_t* dy, const bf16_t* wt, const float* addend,
                                  const bf16_t* addmask, const bf16_t* gate, const bf16_t* bnx, stat_t* gsums, float* out_f32,
                                  bf16_t* out_b16, hipStream_t s, bool stats_f32 = false, int rep_stride = 0,
                                  const bf16_t* dy2 = nullptr, const bf16_t* wt2 = nullptr, const ConvInputBnBwd* bn = nullptr);

hipError_t conv_dgrad(const ConvShape& c, const bf16_t* dy, const bf16_t* wt, const float* addend,
                      const bf16_t* addmask, float* out_f32, bf16_t* out_b16, hipStream_t s) {
  return conv_dgrad_impl(c, dy, wt, addend, addmask, nullptr, nullptr, nullptr, out_f32, out_b16, s);
}

// the narrow kernel, or the two-workgroup form of the wide gather kernel (1x1 layers), runs the whole data gradient of
// this layer: their output stages take the sums of the fp32 values
bool conv_dgrad_feeds_next(const ConvShape& c) {
  if (c.stride != 1 || (c.T != 9 && c.T != 1)) return false;
  GatherConvArgs a{};
  a.N = c.N; a.Hi = c.Ho(); a.Wi = c.Wo(); a.Ci = c.Co; a.Co = c.Cip; a.w_rows = c.Cip; a.Kw = c.T * c.Co;
  a.OH = c.Hi; a.OW = c.Wi; a.OHf = c.Hi; a.OWf = c.Wi; a.in_stride = 1; a.out_stride = 1; a.ntaps = c.T;
  if (c.T == 9) {
    for (int r = 0; r < 3; ++r)
      for (int q = 0; q < 3; ++q) a.tap[r * 3 + q] = pack_tap(1 - r, 1 - q, r * 3 + q);
    return conv_narrow_applies(a);
  }
  a.tap[0] = pack_tap(0, 0, 0);
  return conv_gather_pair_applies(a);
}

hipError_t conv_dgrad_feeding_next(const ConvShape& c, const bf16_t* dy, const bf16_t* wt, const float* addend,
                                   const bf16_t* addmask, const bf16_t* gate, const bf16_t* bnx, stat_t* gsums, float* out_f32,
                                   bf16_t* out_b16, hipStream_t s, int gsums_rep_stride) {
  if (!gate || !bnx || !gsums || !out_f32 || !conv_dgrad_feeds_next(c)) return hipErrorInvalidValue;
  return conv_dgrad_impl(c, dy, wt, addend, addmask, gate, bnx, gsums, out_f32, out_b16, s, /*stats_f32=*/true, gsums_rep_stride);
}

// The gate and the sums are taken where the wide kernels or the narrow kernel run the whole data gradient.
bool conv_dgrad_gates(const ConvShape& c) {
  GatherConvArgs a{};
  a.Hi = c.Ho(); a.Wi = c.Wo(); a.Ci = c.Co; a.Co = c.Cip; a.Kw = c.T * c.Co; a.ntaps = 1;
  if (conv_gather_wide_applies(a) && (c.stride == 1 || (c.Hi >= 2 && c.Wi >= 2))) return true;
  return conv_dgrad_feeds_next(c);
}

hipError_t conv_dgrad_gated(const ConvShape& c, const bf16_t* dy, const bf16_t* wt, const float* addend, const bf16_t* gate,
                            const bf16_t* bnx, stat_t* gsums, float* out_f32, bf16_t* out_b16, hipStream_t s,
                            int gsums_rep_stride) {
  if (!gate || !bnx || !gsums || !conv_dgrad_gates(c)) return hipErrorInvalidValue;
  return conv_dgrad_impl(c, dy, wt, addend, nullptr, gate, bnx, gsums, out_f32, out_b16, s, false, gsums_rep_stride);
}

bool conv_dgrad_bn_applies(const ConvShape& c, bool g_is_f32) {
  if (c.stride != 1 || c.T != 9 || c.Ci != c.Cip) return false;
  GatherConvArgs a{};
  a.N = c.N; a.Hi = c.Ho(); a.Wi = c.Wo(); a.Ci = c.Co; a.Co = c.Cip; a.w_rows = c.Cip; a.Kw = c.T * c.Co;
  a.OH = c.Hi; a.OW = c.Wi; a.OHf = c.Hi; a.OWf = c.Wi; a.in_stride = 1; a.out_stride = 1; a.ntaps = 9;
  for (int r = 0; r < 3; ++r)
    for (int q = 0; q < 3; ++q) a.tap[r * 3 + q] = pack_tap(1 - r, 1 - q, r * 3 + q);
  return conv_narrow_transforms(a, g_is_f32 ? 2 : 1);
}

hipError_t conv_dgrad_after_bn(const ConvShape& c, const ConvInputBnBwd& bn, const bf16_t* wt, const float* addend,
                               const bf16_t* addmask, const bf16_t* gate, const bf16_t* bnx, stat_t* gsums, bool sums_of_f32,
                               float* out_f32, bf16_t* out_b16, hipStream_t s, int gsums_rep_stride) {
  if (!conv_dgrad_bn_applies(c, bn.g_is_f32 != 0) || (!out_f32 && !out_b16)) return hipErrorInvalidValue;
  const bool sums = gate || bnx || gsums;
  if (sums && (!gate || !bnx || !gsums)) return hipErrorInvalidValue;
  if (sums_of_f32 && (!sums || !out_f32)) return hipErrorInvalidValue;
  return conv_dgrad_impl(c, nullptr, wt, addend, addmask, gate, bnx, gsums, out_f32, out_b16, s, sums_of_f32, gsums_rep_stride, nullptr,
                         nullptr, &bn);
}

// the stride-2 wide path below takes both data gradients: 3x3 and 1x1 with the same stride-2 geometry and channel counts
bool conv_dgrad_pair_applies(const ConvShape& c, const ConvShape& cp) {
  if (c.stride != 2 || cp.stride != 2 || c.T != 9 || cp.T != 1 || c.N != cp.N || c.Hi != cp.Hi || c.Wi != cp.Wi ||
      c.Ci != cp.Ci || c.Cip != cp.Cip || c.Co != cp.Co || c.Hi < 2 || c.Wi < 2 || c.Co % 64 != 0)
    return false;
  GatherConvArgs probe{};
  probe.Hi = c.Ho(); probe.Wi = c.Wo(); probe.Ci = c.Co; probe.Co = c.Cip; probe.w_rows = c.Cip; probe.Kw = c.T * c.Co; probe.ntaps = 1;
  return conv_gather_wide_applies(probe);
}

hipError_t conv_dgrad_gated_pair(const ConvShape& c, const bf16_t* dy, const bf16_t* wt, const ConvShape& cp, const bf16_t* dy2,
                                 const bf16_t* wt2, const bf16_t* gate, const bf16_t* bnx, stat_t* gsums, float* out_f32,
                                 bf16_t* out_b16, hipStream_t s, int gsums_rep_stride) {
  const bool gated = gate || bnx || gsums;
  if (!dy2 || !wt2 || (gated && (!gate || !bnx || !gsums)) || !conv_dgrad_pair_applies(c, cp)) return hipErrorInvalidValue;
  return conv_dgrad_impl(c, dy, wt, nullptr, nullptr, gate, bnx, gsums, out_f32, out_b16, s, false, gsums_rep_stride, dy2, wt2);
}

static hipError_t conv_dgrad_impl(const ConvShape& c, const bf16_t* dy, const bf16_t* wt, const float* addend,
                                  const bf16_t* addmask, const bf16_t* gate, const bf16_t* bnx, stat_t* gsums, float* out_f32,
                                  bf16_t* out_b16, hipStream_t s, bool stats_f32, int rep_stride, const bf16_t* dy2,
                                  const bf16_t* wt2, const ConvInputBnBwd* bn) {
  GatherConvArgs a{};
  a.stats_rep_stride = rep_stride;
  a.in = dy; a.w = wt; a.addend = addend; a.addmask = addmask; a.out_f32 = out_f32; a.out_b16 = out_b16;
  a.gate = gate; a.bnx = bnx; a.stats = gsums; a.stats_f32 = stats_f32 ? 1 : 0;
  a.N = c.N; a.Hi = c.Ho(); a.Wi = c.Wo(); a.Ci = c.Co;
  a.in_stride = 1;
  a.OHf = c.Hi; a.OWf = c.Wi;
  a.Co = c.Cip; a.w_rows = c.Cip; a.Kw = c.T * c.Co;
  if (c.stride == 1) {
    if (dy2) return hipErrorInvalidValue;
    // input pixel (hi, wi) receives dy[hi + 1 - r, wi + 1 - q] * w[., r, q, .]
    a.OH = c.Hi; a.OW = c.Wi; a.out_stride = 1; a.ooh = 0; a.oow = 0;
    a.ntaps = c.T;
    if (c.T == 9) {
      for (int r = 0; r < 3; ++r)
        for (int q = 0; q < 3; ++q) a.tap[r * 3 + q] = pack_tap(1 - r, 1 - q, r * 3 + q);
    } else {
      a.tap[0] = pack_tap(0, 0, 0);
    }
    if (bn) {   // the batch-norm backward that produces dy, on the patch (narrow kernel)
      if (!bn->g || !bn->x || !bn->sums || !bn->bsums || !bn->gamma || !bn->dgamma || !bn->dbeta || !bn->dy_out ||
          !conv_narrow_transforms(a, bn->g_is_f32 ? 2 : 1))
        return hipErrorInvalidValue;
      a.in = nullptr;
      a.tr_mode = 2; a.tr_p = bn->g; a.tr_p_f32 = bn->g_is_f32 ? 1 : 0; a.tr_q = bn->x; a.tr_out = bn->dy_out;
      a.tr_sums = bn->sums; a.tr_bsums = bn->bsums; a.tr_gamma = bn->gamma; a.tr_dgamma = bn->dgamma; a.tr_dbeta = bn->dbeta;
      a.tr_eps = bn->eps; a.tr_rep_stride = bn->rep_stride;
      return launch_conv_narrow(a, s);
    }
    return launch_conv_gather(a, s);
  }
  if (bn) return hipErrorInvalidValue;
  // stride 2: input pixels of one parity class (ph, pw) share one set of taps:
  // hi = 2*oh + ph receives tap r only if hi + 1 - r is even, from output row (hi + 1 - r) / 2.
  {
    // wide layers: all four classes in one launch, heaviest first (4, 2, 2, 1 taps of a 3x3 filter)
    GatherConvArgs probe = a;
    probe.OH = (c.Hi + 1) / 2; probe.OW = (c.Wi + 1) / 2; probe.ntaps = 1; probe.tap[0] = pack_tap(0, 0, 0);
    if (conv_gather_wide_applies(probe) && c.Hi >= 2 && c.Wi >= 2) {
      static const int order[4][2] = {{1, 1}, {0, 1}, {1, 0}, {0, 0}};
      a.nclass = 4;
      a.out_stride = 2;
      for (int i = 0; i < 4; ++i) {
        const int ph = order[i][0], pw = order[i][1];
        a.cOH[i] = (c.Hi - ph + 1) / 2; a.cOW[i] = (c.Wi - pw + 1) / 2;
        a.cooh[i] = ph; a.coow[i] = pw;
        int nt = 0;
        if (c.T == 9) {
          for (int r = 0; r < 3; ++r) {
            if (((ph + 1 - r) & 1) != 0) continue;
            for (int q = 0; q < 3; ++q) {
              if (((pw + 1 - q) & 1) != 0) continue;
              a.ctap[i][nt++] = pack_tap((ph + 1 - r) / 2, (pw + 1 - q) / 2, r * 3 + q);
            }
          }
        } else if (ph == 0 && pw == 0) {
          a.ctap[i][nt++] = pack_tap(0, 0, 0);
        }
        a.cntaps[i] = nt;
        if (ph == 0 && pw == 0 && dy2) {   // the projection's only tap reaches the even pixels
          a.in2 = dy2; a.w2 = wt2; a.Kw2 = c.Co; a.cls2 = i;
        }
      }
      a.OH = a.cOH[0]; a.OW = a.cOW[0]; a.ooh = 1; a.oow = 1; a.ntaps = 0;
      return launch_conv_gather_wide(a, s);
    }
  }
  if (dy2) return hipErrorInvalidValue;   // only the launch above adds a second data gradient
  // the other layers: the classes that have pixels, in one launch of the generic kernel (a class per blockIdx.z)
  a.nclass = 0;
  a.out_stride = 2;
  for (int ph = 0; ph < 2; ++ph)
    for (int pw = 0; pw < 2; ++pw) {
      const int oh = (c.Hi - ph + 1) / 2, ow = (c.Wi - pw + 1) / 2;
      if (oh <= 0 || ow <= 0) continue;
      const int i = a.nclass++;
      a.cOH[i] = oh; a.cOW[i] = ow; a.cooh[i] = ph; a.coow[i] = pw;
      int nt = 0;
      if (c.T == 9) {
        for (int r = 0; r < 3; ++r) {
          if (((ph + 1 - r) & 1) != 0) continue;
          for (int q = 0; q < 3; ++q) {
            if (((pw + 1 - q) & 1) != 0) continue;
            a.ctap[i][nt++] = pack_tap((ph + 1 - r) / 2, (pw + 1 - q) / 2, r * 3 + q);
          }
        }
      } else if (ph == 0 && pw == 0) {
        a.ctap[i][nt++] = pack_tap(0, 0, 0);
      }
      a.cntaps[i] = nt;
    }
  if (a.nclass == 0) return hipSuccess;
  a.OH = a.cOH[0]; a.OW = a.cOW[0]; a.ooh = a.cooh[0]; a.oow = a.coow[0]; a.ntaps = a.cntaps[0];
  for (int t = 0; t < a.ntaps; ++t) a.tap[t] = a.ctap[0][t];
  if (a.nclass == 1) a.nclass = 0;   // a single class is the plain form
  return launch_conv_gather(a, s);
}

// A 1x1 convolution with unit stride does not see the image: its pixels are one long list, and the weight-gradient
// kernels that take whole rows of 1, 2, .. 32 or 64 pixels per 64-pixel step (conv_wgrad128_applies and the others)
// get it as images of two rows of 32, whatever the real width (14 x 14 in ResNet-101's third stage).
static ConvShape wgrad_view(const ConvShape& c) {
  const long long pixels = (long long)c.N * c.Hi * c.Wi;
  if (c.T != 1 || c.stride != 1 || pixels % 64 != 0 || pixels / 64 > 0x7fffffff || (c.Wi >= 1 && 64 % c.Wi == 0)) return c;
  ConvShape v = c;
  v.N = (int)(pixels / 64); v.Hi = 2; v.Wi = 32;
  return v;
}

size_t conv_wgrad_scratch_bytes(const ConvShape& c_in) {
  const ConvShape c = wgrad_view(c_in);
  WgradArgs a{};
  a.Co = c.Co; a.Ci = c.Ci; a.Cx = c.Cip; a.OW = c.Wo(); a.ntaps = c.T;
  a.N = c.N; a.OH = c.Ho(); a.Hi = c.Hi; a.Wi = c.Wi; a.stride = c.stride;
  for (int r = 0; r < 3; ++r)
    for (int q = 0; q < 3; ++q) a.tap[r * 3 + q] = pack_tap(r - 1, q - 1, 0);
  a.Cx = c.Cip;
  if (conv_wgrad_narrow_applies(a)) return conv_wgrad_narrow_scratch_bytes(a);
  if (!(conv_wgrad_wide_applies(a) || conv_wgrad128_applies(a) || conv_wgrad_tall_applies(a))) return generic_wgrad_scratch_bytes(a);
  // room for the partial sums of the pixel splits: 8 of them, or as many as it takes the 160 x 160 kernel to fill
  // the chip when a layer has few blocks (160 -> 160: 9 blocks per filter)
  size_t splits = 8;
  if (!conv_wgrad128_applies(a) && !conv_wgrad_tall_applies(a)) {
    const size_t tiles = (size_t)(c.Co / 160) * (c.Ci / 160) * c.T;
    splits = std::min<size_t>(32, std::max<size_t>(8, (256 + tiles - 1) / tiles));
  }
  return splits * c.Co * c.T * c.Ci * 4;
}

static WgradArgs wgrad_args(const ConvShape& c_in, const bf16_t* x, const bf16_t* dy, float* dw, float* scratch,
                            size_t scratch_bytes, bool overwrite) {
  const ConvShape c = wgrad_view(c_in);
  WgradArgs a{};
  a.dy = dy; a.x = x; a.dw = dw; a.scratch = scratch; a.scratch_bytes = scratch_bytes;
  a.overwrite = overwrite ? 1 : 0;
  a.N = c.N; a.OH = c.Ho(); a.OW = c.Wo(); a.Co = c.Co;
  a.Hi = c.Hi; a.Wi = c.Wi; a.Cx = c.Cip; a.Ci = c.Ci;
  a.stride = c.stride; a.ntaps = c.T;
  if (c.T == 9) {
    for (int r = 0; r < 3; ++r)
      for (int q = 0; q < 3; ++q) a.tap[r * 3 + q] = pack_tap(r - 1, q - 1, 0);
  } else {
    a.tap[0] = pack_tap(0, 0, 0);
  }
  return a;
}

// the dispatch of launch_conv_wgrad reaches the narrow kernel for this layer (given enough scratch)
static bool wgrad_runs_narrow(const WgradArgs& a) {
  return !conv_wgrad128_applies(a) && !conv_wgrad_tall_applies(a) && !conv_wgrad_wide_applies(a) && conv_wgrad_narrow_applies(a);
}
bool conv_wgrad_defers(const ConvShape& c) { return wgrad_runs_narrow(wgrad_args(c, nullptr, nullptr, nullptr, nullptr, 0, true)); }

hipError_t conv_wgrad_settle(WgradDebt& debt, hipStream_t s) {
  if (debt.slices <= 0) return hipSuccess;
  const hipError_t e = launch_wgrad_slices_reduce(debt.dw, debt.partial, debt.n4, debt.slices, debt.stride4, debt.overwrite, s);
  debt = WgradDebt{};
  return e;
}

hipError_t conv_wgrad(const ConvShape& c_in, const bf16_t* x, const bf16_t* dy, float* dw, float* scratch,
                      size_t scratch_bytes, bool overwrite, hipStream_t s, WgradDebt* debt) {
  WgradArgs a = wgrad_args(c_in, x, dy, dw, scratch, scratch_bytes, overwrite);
  if (!debt) return launch_conv_wgrad(a, s);
  const bool narrow = wgrad_runs_narrow(a) && a.scratch && a.scratch_bytes >= conv_wgrad_narrow_scratch_bytes(a) &&
                      a.N * a.OH * a.OW > 0 && a.scratch != debt->partial;
  if (!narrow) {
    if (hipError_t e = conv_wgrad_settle(*debt, s); e != hipSuccess) return e;
    return launch_conv_wgrad(a, s);
  }
  a.prev_dw = debt->dw; a.prev_partial = debt->partial; a.prev_n4 = debt->n4; a.prev_slices = debt->slices;
  a.prev_overwrite = debt->overwrite; a.prev_stride4 = debt->stride4;
  a.defer_reduce = 1;
  const hipError_t e = launch_conv_wgrad_narrow(a, s);
  if (e != hipSuccess) return e;   // (an invalid launch enqueued nothing: the debt handed in is still owed)
  const size_t n = (size_t)a.Co * 9 * a.Ci;
  debt->dw = dw; debt->partial = scratch; debt->n4 = (int)(n / 4); debt->slices = conv_wgrad_narrow_slices(a);
  debt->overwrite = a.overwrite; debt->stride4 = n / 4;
  return hipSuccess;
}

}  // namespace fdg

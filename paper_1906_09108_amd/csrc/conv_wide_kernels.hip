// Gather-form convolution for wide layers (input channels a multiple of 64): the WRN-28-10 shapes,
// where the convolution is a dense contraction far above the MFMA ridge.
//
// Differences from the generic kernel in conv_kernels.hip:
//   * operands go from global memory straight into LDS (global_load_lds_dwordx4, 16 bytes per lane, lane l
//     of a wave lands at base + 16*l), several k-chunks ahead, with no register staging;
//   * a k-chunk is 64 channels of ONE filter tap (Ci % 64 == 0), so tap offsets and zero padding are
//     decided per row, not per element; rows outside the image read a 16-byte zero word instead;
//   * LDS rows are 128 bytes with the 16-byte unit index XORed by (row >> 1) & 7, which makes both the
//     DMA writes (8 consecutive rows per wave instruction) and the 16-lane MFMA operand reads conflict free;
//   * the tile is 128 pixels x 160 channels: 160 divides the WRN widths 320 and 640, giving 256 or 512
//     workgroups for the 8x8 and 16x16 stages, i.e. whole rounds of the 256 compute units;
//   * workgroups are numbered so that the eight XCDs (workgroup id mod 8) each own a contiguous range of
//     pixel tiles with all of their channel tiles, keeping operand reuse inside one L2.
#include "conv_common.h"

namespace fdg {

__device__ __attribute__((aligned(16))) uint32_t g_zero_word[4] = {0u, 0u, 0u, 0u};

__device__ __forceinline__ void dma16(const void* gsrc, void* lds_wave_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                   (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
}

// s_waitcnt vmcnt(n) only (expcnt and lgkmcnt left at "no wait")
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 0xf) | ((N >> 4) << 14) | (0x7 << 4) | (0xf << 8));
}

template <int BM, int BN, int WM, int WN, int STAGES>
__global__ __launch_bounds__(256) void conv_gather_dma_kernel(GatherConvArgs a, int m_tiles, int n_tiles) {
  static_assert(WM * WN == 4, "four waves");
  static_assert(BM % 32 == 0 && BN % 32 == 0, "row groups of 8 per wave instruction");
  constexpr int ROWB = 128;                 // bytes per LDS row = 64 bf16 of one tap
  constexpr int R = BM + BN;
  constexpr int JX = BM / 32, JW = BN / 32; // DMA instructions per thread per chunk: pixel rows, weight rows
  constexpr int NJ = JX + JW;
  constexpr int TM = BM / WM, TN = BN / WN;
  constexpr int FM = TM / 16, FN = TN / 16;
  static_assert(TM % 16 == 0 && TN % 16 == 0, "whole MFMA blocks per wave");
  static_assert((STAGES - 2) * NJ < 64, "vmcnt range");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // STAGES * R * ROWB

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: it selects DMA destinations
  const int wave_m = wave % WM, wave_n = wave / WM;
  const int Mtot = a.N * a.OH * a.OW;

  // workgroup -> tile, XCD aware: hardware deals workgroup ids round robin over 8 XCDs
  int t = blockIdx.x;
  const int total = m_tiles * n_tiles;
  if ((total & 7) == 0) t = (blockIdx.x & 7) * (total >> 3) + (blockIdx.x >> 3);
  const int m0 = (t / n_tiles) * BM, c0 = (t % n_tiles) * BN;

  // ---- per-thread DMA sources: row = 8*(4*j + wave) + lane/8, LDS unit lane%8 holds k-unit u ----
  const char* src[NJ];   // address of this thread's 16 bytes at tap (0,0), chunk offset 0
  int hw[JX];            // (ih0 << 16) | iw0 of pixel rows; rows past the end get an always-outside marker
  bool wok[JW];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int row = 8 * (4 * j + wave) + (lane >> 3);
    const int u = (lane & 7) ^ ((row >> 1) & 7);
    if (j < JX) {
      const int m = m0 + row;
      if (m < Mtot) {
        const int ow = m % a.OW, t2 = m / a.OW, oh = t2 % a.OH, n = t2 / a.OH;
        const int ih0 = oh * a.in_stride, iw0 = ow * a.in_stride;
        hw[j] = (ih0 << 16) | iw0;
        src[j] = reinterpret_cast<const char*>(a.in) + (((size_t)n * a.Hi + ih0) * a.Wi + iw0) * (size_t)a.Ci * 2 + u * 16;
      } else {
        hw[j] = 0x7fff0000;
        src[j] = reinterpret_cast<const char*>(a.in);
      }
    } else {
      const int c = c0 + row - BM;
      wok[j - JX] = c < a.w_rows;
      src[j] = reinterpret_cast<const char*>(a.w) + (size_t)(wok[j - JX] ? c : 0) * a.Kw * 2 + u * 16;
    }
  }
  const char* zero = reinterpret_cast<const char*>(g_zero_word);
  const int cpc = a.Ci >> 6;              // chunks per tap
  const int nchunks = a.ntaps * cpc;

  auto issue = [&](int kc) {
    unsigned char* stage = smem + (size_t)(kc % STAGES) * (R * ROWB);
    const int tapi = kc / cpc, cb = (kc - tapi * cpc) * 128;   // byte offset of the 64-channel block
    const int tp = a.tap[tapi];
    const int dh = (tp & 0xff) - 8, dw = ((tp >> 8) & 0xff) - 8, kofs = tp >> 16;
    const long xoff = ((long)dh * a.Wi + dw) * a.Ci * 2 + cb;
    const long woff = (long)kofs * a.Ci * 2 + cb;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const char* g;
      if (j < JX) {
        const int ih = (hw[j] >> 16) + dh, iw = (hw[j] & 0xffff) + dw;
        g = ((unsigned)ih < (unsigned)a.Hi && (unsigned)iw < (unsigned)a.Wi) ? src[j] + xoff : zero;
      } else {
        g = wok[j - JX] ? src[j] + woff : zero;
      }
      dma16(g, stage + (size_t)(8 * (4 * j + wave)) * ROWB);
    }
  };

  f32x4 acc[FN][FM];
#pragma unroll
  for (int i = 0; i < FN; ++i)
#pragma unroll
    for (int j = 0; j < FM; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // LDS byte offsets of this lane's operand rows (unit swizzle applied per k-step below)
  int xrow[FM], wrow[FN];
#pragma unroll
  for (int f = 0; f < FM; ++f) xrow[f] = wave_m * TM + f * 16 + (lane & 15);
#pragma unroll
  for (int f = 0; f < FN; ++f) wrow[f] = BM + wave_n * TN + f * 16 + (lane & 15);

#pragma unroll
  for (int p = 0; p < STAGES - 1; ++p)
    if (p < nchunks) issue(p);

  for (int kc = 0; kc < nchunks; ++kc) {
    // chunk kc has landed once at most the (STAGES-2) younger chunks are still in flight
    if (kc + STAGES - 2 < nchunks) wait_vmcnt<(STAGES - 2) * NJ>(); else wait_vmcnt<0>();
    // Everybody's part of chunk kc is in LDS and everybody is done reading chunk kc-1.  A bare s_barrier:
    // __syncthreads() would add a fence that waits for ALL outstanding DMA, younger chunks included.
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (kc + STAGES - 1 < nchunks) issue(kc + STAGES - 1);   // overwrites the buffer of chunk kc-1
    const unsigned char* stage = smem + (size_t)(kc % STAGES) * (R * ROWB);
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const int u = ks * 4 + (lane >> 4);
      bf16x8 fa[FN], fb[FM];
#pragma unroll
      for (int f = 0; f < FN; ++f)
        fa[f] = *reinterpret_cast<const bf16x8*>(stage + wrow[f] * ROWB + ((u ^ ((wrow[f] >> 1) & 7)) << 4));
#pragma unroll
      for (int f = 0; f < FM; ++f)
        fb[f] = *reinterpret_cast<const bf16x8*>(stage + xrow[f] * ROWB + ((u ^ ((xrow[f] >> 1) & 7)) << 4));
#pragma unroll
      for (int i = 0; i < FN; ++i)
#pragma unroll
        for (int j = 0; j < FM; ++j) acc[i][j] = mfma16(fa[i], fb[j], acc[i][j]);
    }
  }
  store_tile<FM, FN>(a, acc, m0 + wave_m * TM, c0 + wave_n * TN, lane);
}

bool conv_gather_wide_applies(const GatherConvArgs& a) {
  return a.Ci % 64 == 0 && a.Co >= 128 && a.ntaps >= 1 && a.Kw % 8 == 0 && a.Hi < 32768 && a.Wi < 32768;
}

template <int BM, int BN, int WM, int WN, int STAGES>
static hipError_t run_wide(const GatherConvArgs& a, hipStream_t s) {
  constexpr size_t lds = (size_t)STAGES * (BM + BN) * 128;
  static bool configured = false;   // one attribute call per instantiation (idempotent, so a race is harmless)
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_gather_dma_kernel<BM, BN, WM, WN, STAGES>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int Mtot = a.N * a.OH * a.OW;
  const int m_tiles = (Mtot + BM - 1) / BM, n_tiles = (a.Co + BN - 1) / BN;
  hipLaunchKernelGGL((conv_gather_dma_kernel<BM, BN, WM, WN, STAGES>), dim3(m_tiles * n_tiles), dim3(256), lds, s, a,
                     m_tiles, n_tiles);
  return hipGetLastError();
}

hipError_t launch_conv_gather_wide(const GatherConvArgs& a, hipStream_t s) {
  if (!conv_gather_wide_applies(a) || a.N * a.OH * a.OW <= 0) return hipErrorInvalidValue;
  if (a.Co % 160 == 0) return run_wide<128, 160, 2, 2, 4>(a, s);
  return run_wide<128, 128, 2, 2, 4>(a, s);
}

}  // namespace fdg

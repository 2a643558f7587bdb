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
#include <stdio.h>
#include <stdlib.h>
#include <type_traits>
#include <utility>

namespace fdg {

__device__ __attribute__((aligned(16))) uint32_t g_zero_word[4] = {0u, 0u, 0u, 0u};

__device__ __forceinline__ void dma16(const void* gsrc, void* lds_wave_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                   (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
}

// Workgroups are dealt to the 8 XCDs round robin (XCD = block index mod 8).  This is the inverse numbering: the
// blocks that run on one XCD get consecutive logical indices (any grid size), so that neighbours in the logical
// order share an L2.
__device__ __forceinline__ int xcd_consecutive(int block, int total) {
  const int base = total >> 3, rem = total & 7, x = block & 7, q = block >> 3;
  return x * base + (x < rem ? x : rem) + q;
}

// s_waitcnt vmcnt(n) only (expcnt and lgkmcnt left at "no wait")
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 0xf) | ((N >> 4) << 14) | (0x7 << 4) | (0xf << 8));
}

template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// Four waves: wave_m = wave & 1 owns 64 of the tile's 128 pixels and ALL of its BN channels as 2 x (BN/32)
// accumulator blocks of 32x32; wk = wave >> 1 takes one 32-channel half of every 64-channel k-chunk.  So a
// wave reads 2 + BN/32 operand fragments for every 2 * BN/32 MFMAs (the best ratio four waves can get on a
// 128 x 160 tile) and the two k-halves are added once, through LDS, after the main loop.
// KTAIL: the input channels are not a multiple of 64 (WRN's 160): the last 64-channel chunk of every tap is
// partly beyond the tensor, and those 16-byte units are loaded from the zero word, for pixels and weights alike.
constexpr size_t gather_dma_lds_bytes(int BN, int STAGES) {
  size_t need = (size_t)STAGES * (128 + BN) * 128;
  if (need < (size_t)4 * (BN / 32) * 16 * 256) need = (size_t)4 * (BN / 32) * 16 * 256;
  if (need < (size_t)4 * out_stage_bytes(BN) + stats_stage_bytes(BN)) need = (size_t)4 * out_stage_bytes(BN) + stats_stage_bytes(BN);
  return need;
}

template <int BN, int STAGES, bool KTAIL, bool F32S = false>
__device__ __forceinline__ void gather_dma_body(const GatherConvArgs& a, int m_tiles, int n_tiles) {
  constexpr int BM = 128;
  static_assert(BN % 32 == 0, "whole 32x32 blocks");
  constexpr int ROWB = 128;                 // bytes per LDS row = 64 bf16 of one tap
  constexpr int R = BM + BN;
  constexpr int JX = BM / 32, JW = BN / 32; // DMA instructions per thread per chunk: pixel rows, weight rows
  constexpr int NJ = JX + JW;
  constexpr int FM = 2, FN = BN / 32;
  static_assert((STAGES - 2) * NJ < 64, "vmcnt range");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // gather_dma_lds_bytes(BN, STAGES): stages, or the output stage if larger

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: it selects DMA destinations
  const int wave_m = wave & 1, wk = wave >> 1;

  // workgroup -> tile, XCD aware: hardware deals workgroup ids round robin over 8 XCDs
  GatherConvArgs b = a;      // the geometry this workgroup works on
  int t = blockIdx.x, cls = 0;
  if (a.nclass > 1) {
    // classes are ordered by decreasing work, so the plain order lets the dispatcher balance them
    while (cls + 1 < a.nclass && t >= a.cls_start[cls + 1]) ++cls;
    t -= a.cls_start[cls];
    b.OH = a.cOH[cls]; b.OW = a.cOW[cls]; b.ooh = a.cooh[cls]; b.oow = a.coow[cls]; b.ntaps = a.cntaps[cls];
  } else {
    const int total = m_tiles * n_tiles;
    if ((total & 7) == 0) t = (blockIdx.x & 7) * (total >> 3) + (blockIdx.x >> 3);
  }
  const int Mtot = b.N * b.OH * b.OW;
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
        const int ow = m % b.OW, t2 = m / b.OW, oh = t2 % b.OH, n = t2 / b.OH;
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
  const int cpc = (a.Ci + 63) >> 6;       // chunks per tap
  const int nchunks = b.ntaps * cpc;
  // the k-unit this lane loads is the same for all its rows: (row >> 1) & 7 = (4 * (wave & 1) + (lane >> 4)) & 7
  const int ku = (lane & 7) ^ ((4 * (wave & 1) + (lane >> 4)) & 7);

  auto issue = [&](int kc) {
    unsigned char* stage = smem + (size_t)(kc % STAGES) * (R * ROWB);
    const int tapi = kc / cpc, cb = (kc - tapi * cpc) * 128;   // byte offset of the 64-channel block
    const bool kv = !KTAIL || (cb >> 1) + ku * 8 < a.Ci;       // this lane's 8 channels exist
    const int tp = a.nclass > 1 ? a.ctap[cls][tapi] : a.tap[tapi];
    const int dh = (tp & 0xff) - 8, dw = ((tp >> 8) & 0xff) - 8, kofs = tp >> 16;
    const long xoff = ((long)dh * a.Wi + dw) * a.Ci * 2 + cb;
    const long woff = (long)kofs * a.Ci * 2 + cb;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const char* g;
      if (j < JX) {
        const int ih = (hw[j] >> 16) + dh, iw = (hw[j] & 0xffff) + dw;
        g = ((unsigned)ih < (unsigned)a.Hi && (unsigned)iw < (unsigned)a.Wi && kv) ? src[j] + xoff : zero;
      } else {
        g = (wok[j - JX] && kv) ? src[j] + woff : zero;
      }
      dma16(g, stage + (size_t)(8 * (4 * j + wave)) * ROWB);
    }
  };

  f32x16 acc[FN][FM];
#pragma unroll
  for (int i = 0; i < FN; ++i)
#pragma unroll
    for (int j = 0; j < FM; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // LDS rows of this lane's operand fragments (unit swizzle applied per k-step below)
  int xrow[FM], wrow[FN];
#pragma unroll
  for (int f = 0; f < FM; ++f) xrow[f] = wave_m * 64 + f * 32 + (lane & 31);
#pragma unroll
  for (int f = 0; f < FN; ++f) wrow[f] = BM + f * 32 + (lane & 31);

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
    for (int ss = 0; ss < 2; ++ss) {        // the two 16-channel steps of this wave's half chunk
      const int u = 4 * wk + 2 * ss + (lane >> 5);
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
        for (int j = 0; j < FM; ++j) acc[i][j] = mfma32(fa[i], fb[j], acc[i][j]);
    }
  }
  wait_vmcnt<0>();
  combine_and_store32<FN, BN, F32S>(b, acc, m0, c0, wave_m, wk, lane, smem);
}

// Within 256 registers, so that two workgroups (two waves per SIMD) fit a compute unit: the two-stage form.
// F32S: sums of the fp32 values in the output stage (GatherConvArgs::stats_f32), for a data gradient that feeds the layer below.
template <int BN, int STAGES, bool KTAIL, bool F32S>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void conv_gather_dma_pair_kernel(
    GatherConvArgs a, int m_tiles, int n_tiles) {
  gather_dma_body<BN, STAGES, KTAIL, F32S>(a, m_tiles, n_tiles);
}

// ------------------------------------------------------------------------------------------------
// Gather form with the hand-pinned pipeline of the patch kernel below (its description of the half steps, the
// fragment sets and the explicit waits applies word for word): what the patch form cannot take -- stride 2, 1x1,
// the parity classes of a stride-2 data gradient, images wider than 32 pixels.
// ------------------------------------------------------------------------------------------------
// A step is one 64-channel block of one tap (taps outer, channel blocks inner).  Its stage holds 128 pixel rows and
// BN weight rows; WS stages, the group of loads for step i + WS - 1 goes out during step i, one load every SPACING
// slots after the barrier of that step.  A pixel row that the tap moves outside the image (or that does not exist)
// is loaded from a 16-byte zero word: whether it does is one bit per tap and load, worked out once per lane.
// The per-tap offsets sit in the lanes of two registers (lane t: tap t) and are fetched with a lane read, so the
// loop reads no kernel argument by a run-time index.  Steps may number anything from 0 (a class of a 1x1 stride-2
// data gradient that no tap reaches: its result is the addend, or zero) upwards.
template <int BN, int WS, bool KTAIL>
__global__ __launch_bounds__(256) void conv_gather_pipe_kernel(GatherConvArgs a, int m_tiles, int n_tiles) {
  constexpr int BM = 128, ROWB = 128;
  static_assert(BN % 32 == 0, "whole 32x32 blocks");
  constexpr int JX = BM / 32, JW = BN / 32, NJ = JX + JW;
  constexpr int FM = 2, FN = BN / 32;
  constexpr int SBYTES = (BM + BN) * ROWB;
  static_assert(WS >= 3 && (WS - 2) * NJ < 64, "vmcnt range");
  static_assert((size_t)WS * SBYTES >= (size_t)4 * FN * 16 * 256 && (size_t)WS * SBYTES >= (size_t)4 * out_stage_bytes(BN) + stats_stage_bytes(BN), "room for the output stage");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // WS * SBYTES

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave_m = wave & 1, wk = wave >> 1;

  GatherConvArgs b = a;      // the geometry this workgroup works on
  int t = blockIdx.x, cls = 0;
  if (a.nclass > 1) {
    // classes are ordered by decreasing work, so the plain order lets the dispatcher balance them
    while (cls + 1 < a.nclass && t >= a.cls_start[cls + 1]) ++cls;
    t -= a.cls_start[cls];
    b.OH = a.cOH[cls]; b.OW = a.cOW[cls]; b.ooh = a.cooh[cls]; b.oow = a.coow[cls]; b.ntaps = a.cntaps[cls];
  } else {
    const int total = m_tiles * n_tiles;
    if ((total & 7) == 0) t = (blockIdx.x & 7) * (total >> 3) + (blockIdx.x >> 3);
  }
  const int Mtot = b.N * b.OH * b.OW;
  const int m0 = (t / n_tiles) * BM, c0 = (t % n_tiles) * BN;
  const int ntaps = b.ntaps;
  const int cpc = (a.Ci + 63) >> 6;       // channel blocks per tap
  // a second source (see GatherConvArgs::in2) is one more tap, number ntaps, with pointers of its own
  const bool has2 = a.in2 != nullptr && cls == a.cls2;
  const int nsteps = (ntaps + (has2 ? 1 : 0)) * cpc;
  const long long delta2 = has2 ? reinterpret_cast<const char*>(a.in2) - reinterpret_cast<const char*>(a.in) : 0;

  // lane t < ntaps: byte offsets of tap t in the input (pixel shift) and in a weight row
  int tapw = pack_tap(0, 0, 0);
  if (lane < ntaps) tapw = a.nclass > 1 ? a.ctap[cls][lane & 3] : a.tap[lane < 9 ? lane : 0];
  const int xd_v = (((tapw & 0xff) - 8) * a.Wi + (((tapw >> 8) & 0xff) - 8)) * a.Ci * 2;
  const int wd_v = (tapw >> 16) * a.Ci * 2;

  // ---- per-thread DMA sources: row = 8*(4*j + wave) + lane/8, LDS unit lane%8 holds k-unit u ----
  const char* xsrc[JX];   // address of this thread's 16 bytes at tap (0,0), channel block 0
  unsigned vmask[JX];     // bit t: the row's pixel exists under tap t
  unsigned woff[JW];      // weight rows: 32-bit offsets from a.w (rows past the last channel read the last one: never stored)
  unsigned woff2[JW];     // the same into a.w2
  int tdh[9], tdw[9];     // the taps' pixel shifts as scalars
#pragma unroll
  for (int i = 0; i < 9; ++i) {
    const int tw = __builtin_amdgcn_readlane(tapw, i);
    tdh[i] = (tw & 0xff) - 8; tdw[i] = ((tw >> 8) & 0xff) - 8;
  }
#pragma unroll
  for (int j = 0; j < JX; ++j) {
    const int row = 8 * (4 * j + wave) + (lane >> 3);
    const int u = (lane & 7) ^ ((row >> 1) & 7);
    const int m = m0 + row;
    const bool exists = m < Mtot;
    const int mm = exists ? m : 0;
    const int ow = mm % b.OW, t2 = mm / b.OW, oh = t2 % b.OH, n = t2 / b.OH;
    const int ih0 = oh * a.in_stride, iw0 = ow * a.in_stride;
    xsrc[j] = reinterpret_cast<const char*>(a.in) + (((size_t)n * a.Hi + ih0) * a.Wi + iw0) * (size_t)a.Ci * 2 + u * 16;
    unsigned vm = 0;
#pragma unroll
    for (int i = 0; i < 9; ++i)
      if (i < ntaps && (unsigned)(ih0 + tdh[i]) < (unsigned)a.Hi && (unsigned)(iw0 + tdw[i]) < (unsigned)a.Wi) vm |= 1u << i;
    if (has2 && ih0 < a.Hi && iw0 < a.Wi) vm |= 1u << ntaps;
    vmask[j] = exists ? vm : 0u;
  }
#pragma unroll
  for (int j = 0; j < JW; ++j) {
    const int row = 8 * (4 * j + wave) + (lane >> 3);
    const int u = (lane & 7) ^ ((row >> 1) & 7);
    int c = c0 + row;
    c = c >= a.w_rows ? a.w_rows - 1 : c;
    woff[j] = (unsigned)c * (unsigned)(a.Kw * 2) + u * 16;
    woff2[j] = (unsigned)c * (unsigned)(a.Kw2 * 2) + u * 16;
    asm volatile("" : "+v"(woff[j]), "+v"(woff2[j]));   // two registers each, chosen between by a select (not a table in memory)
  }
  // the k-unit this lane loads is the same for all its rows: (row >> 1) & 7 = (4 * (wave & 1) + (lane >> 4)) & 7
  const int ku = (lane & 7) ^ ((4 * (wave & 1) + (lane >> 4)) & 7);
  const bool tail_ok = !KTAIL || (cpc - 1) * 64 + ku * 8 < a.Ci;   // this lane's 8 channels exist in the last block
  const uint64_t zaddr = (uint64_t)g_zero_word;
  uint32_t zero_lo = (uint32_t)zaddr, zero_hi = (uint32_t)(zaddr >> 32);
  asm volatile("" : "+v"(zero_lo), "+v"(zero_hi));

  // load J of the group of step (tap gt, channel block gc) into stage islot
  int gt = 0, gc = 0;      // the step whose group goes out next
  auto issue_one = [&](auto j_tag, int islot, long long xoff, const char* wbase, bool src2, unsigned tapbit, bool lastblk) {
    constexpr int J = decltype(j_tag)::value;
    unsigned char* dst = smem + islot * SBYTES + (8 * (4 * J + wave)) * ROWB;
    if constexpr (J < JX) {
      bool ok = (vmask[J] & tapbit) != 0;
      if (KTAIL) ok = ok && (!lastblk || tail_ok);
      const uint64_t pa = (uint64_t)(xsrc[J] + xoff);
      const uint32_t lo = ok ? (uint32_t)pa : zero_lo, hi = ok ? (uint32_t)(pa >> 32) : zero_hi;
      dma16((const char*)(((uint64_t)hi << 32) | lo), dst);
    } else {
      const unsigned w1 = woff[J - JX], w2 = woff2[J - JX];
      const unsigned wo = src2 ? w2 : w1;
      if (KTAIL) {
        const bool ok = !lastblk || tail_ok;
        const uint64_t pa = (uint64_t)(wbase + (size_t)wo);
        const uint32_t lo = ok ? (uint32_t)pa : zero_lo, hi = ok ? (uint32_t)(pa >> 32) : zero_hi;
        dma16((const char*)(((uint64_t)hi << 32) | lo), dst);
      } else {
        dma16(wbase + (size_t)wo, dst);
      }
    }
  };
  auto advance = [&]() {
    ++gc;
    if (gc == cpc) { gc = 0; ++gt; }
  };
  // where the group of step (gt, gc) reads: pixel byte offset from xsrc, weight base pointer
  auto group_of = [&](long long& xoff, const char*& wbase, bool& src2, unsigned& tapbit, bool& lastblk) {
    src2 = gt == ntaps;   // only reached with has2
    xoff = (src2 ? delta2 : (long long)__builtin_amdgcn_readlane(xd_v, gt)) + gc * 128;
    wbase = src2 ? reinterpret_cast<const char*>(a.w2) + gc * 128
                 : reinterpret_cast<const char*>(a.w) + (__builtin_amdgcn_readlane(wd_v, gt) + gc * 128);
    tapbit = 1u << gt;
    lastblk = gc == cpc - 1;
  };

  // the first groups go out before the rest of the set-up
#pragma unroll
  for (int p = 0; p < WS - 1; ++p)
    if (p < nsteps) {
      long long xoff; const char* wbase; bool src2, lastblk; unsigned tapbit;
      group_of(xoff, wbase, src2, tapbit, lastblk);
      static_for<NJ>([&](auto j) { issue_one(j, p, xoff, wbase, src2, tapbit, lastblk); });
      advance();
    }

  f32x16 acc[FN][FM];
#pragma unroll
  for (int i = 0; i < FN; ++i)
#pragma unroll
    for (int j = 0; j < FM; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // LDS addresses of this lane's operand fragments in stage 0 for the two 16-channel steps of its half block;
  // blocks are 32 rows = 4096 bytes apart (an immediate offset)
  const unsigned lds0 = (unsigned)(uintptr_t)((__attribute__((address_space(3))) unsigned char*)smem);
  unsigned xl[2], wl[2];
#pragma unroll
  for (int ss = 0; ss < 2; ++ss) {
    const unsigned swz = (((4 * wk + 2 * ss + (lane >> 5)) ^ (((lane & 31) >> 1) & 7)) << 4);
    xl[ss] = lds0 + (wave_m * 64 + (lane & 31)) * ROWB + swz;
    wl[ss] = lds0 + (BM + (lane & 31)) * ROWB + swz;
  }

  constexpr int NM = FN * FM, NFRAG = FN + FM;
  static_assert(NFRAG + 2 <= NM, "slots of a half step");
  constexpr int SPACING = (2 * NM - 2) / NJ >= 2 ? 2 : 1;
  static_assert(2 + (NJ - 1) * SPACING < 2 * NM, "the group fits the step");
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  u32x4 fa[2][FN], fb[2][FM];
  // fragment idx of a half step in the order the MFMAs need them: B0, A0, B1, A1, A2, ...
  auto read_one = [&](auto set_tag, auto idx_tag, unsigned wcur, unsigned xcur) {
    constexpr int S = decltype(set_tag)::value, IDX = decltype(idx_tag)::value;
    if constexpr (IDX == 0 || IDX == 2) {
      constexpr int f = IDX / 2;
      u32x4& dst = fb[S][f];
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(xcur), "i"(f * 32 * ROWB));
    } else {
      constexpr int f = IDX == 1 ? 0 : IDX - 2;
      u32x4& dst = fa[S][f];
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(wcur), "i"(f * 32 * ROWB));
    }
  };
  auto before_mma = [&](auto set_tag, auto k_tag, auto n_tag) {
    constexpr int S = decltype(set_tag)::value, K = decltype(k_tag)::value, N = decltype(n_tag)::value;
    static_assert(N >= 0 && N <= 15, "lgkmcnt range");
    if constexpr (K == 0) {
      u32x4 &r0 = fb[S][0], &r1 = fa[S][0];
      asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(r0), "+v"(r1) : "n"(N));
    } else if constexpr (K == 1) {
      u32x4& r0 = fb[S][1];
      asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(r0) : "n"(N));
    } else if constexpr (K % 2 == 0) {
      u32x4& r0 = fa[S][K / 2];
      asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(r0) : "n"(N));
    }
  };
  auto left_after = [](int K) constexpr { return (FN + 2) - (K == 0 ? 2 : (K == 1 ? 3 : 3 + K / 2)); };
  auto mma_one = [&](auto set_tag, auto k_tag) {
    constexpr int S = decltype(set_tag)::value, K = decltype(k_tag)::value;
    acc[K / FM][K % FM] = mfma32(__builtin_bit_cast(bf16x8, fa[S][K / FM]), __builtin_bit_cast(bf16x8, fb[S][K % FM]),
                                 acc[K / FM][K % FM]);
  };
  using set0 = std::integral_constant<int, 0>;
  using set1 = std::integral_constant<int, 1>;

  int slot = 0;   // stage of the current step
  // MORE: a next step exists (its first fragments are read in the second half; the barrier that makes it visible is
  // taken after slot 1).  ISSUE: the group of step i + WS - 1 goes out.  PEND: loads that may still be in flight at
  // the barrier with the next step's group landed.
  auto step_body = [&](auto more_tag, auto issue_tag, auto pend_tag) {
    constexpr bool MORE = decltype(more_tag)::value, ISSUE = decltype(issue_tag)::value;
    constexpr int PEND = decltype(pend_tag)::value;
    const int nslot = slot == WS - 1 ? 0 : slot + 1;
    const int islot = slot == 0 ? WS - 1 : slot - 1;
    const unsigned wcur1 = wl[1] + slot * SBYTES, xcur1 = xl[1] + slot * SBYTES;
    const unsigned wnext0 = wl[0] + nslot * SBYTES, xnext0 = xl[0] + nslot * SBYTES;
    long long xoff = 0;
    const char* wbase = nullptr;
    unsigned tapbit = 0;
    bool src2 = false, lastblk = false;
    if constexpr (ISSUE) group_of(xoff, wbase, src2, tapbit, lastblk);
    auto issue_at = [&](auto s_tag) {
      constexpr int SL = decltype(s_tag)::value;
      if constexpr (ISSUE && SL >= 2 && (SL - 2) % SPACING == 0 && (SL - 2) / SPACING < NJ)
        issue_one(std::integral_constant<int, (SL - 2) / SPACING>{}, islot, xoff, wbase, src2, tapbit, lastblk);
    };
    // first half step: MFMAs of set 0, reads of this step's second half into set 1
    static_for<NM>([&](auto k) {
      constexpr int K = decltype(k)::value;
      if constexpr (K <= 1 || K % 2 == 0)
        before_mma(set0{}, k, std::integral_constant<int, left_after(K) + (K < NFRAG ? K : NFRAG)>{});
      mma_one(set0{}, k);
      if constexpr (K < NFRAG) read_one(set1{}, k, wcur1, xcur1);
      if constexpr (MORE && K == 1) {
        wait_vmcnt<PEND>();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
      }
      issue_at(std::integral_constant<int, K>{});
      __builtin_amdgcn_sched_barrier(0);
    });
    // second half step: MFMAs of set 1, the next step's first reads into set 0
    static_for<NM>([&](auto k) {
      constexpr int K = decltype(k)::value;
      if constexpr (K <= 1 || K % 2 == 0)
        before_mma(set1{}, k, std::integral_constant<int, left_after(K) + ((MORE && K > 2) ? (K - 2 < NFRAG ? K - 2 : NFRAG) : 0)>{});
      mma_one(set1{}, k);
      if constexpr (MORE && K >= 2 && K - 2 < NFRAG) read_one(set0{}, std::integral_constant<int, K - 2>{}, wnext0, xnext0);
      issue_at(std::integral_constant<int, NM + K>{});
      __builtin_amdgcn_sched_barrier(0);
    });
    slot = nslot;
    if constexpr (ISSUE) advance();
  };

  if (nsteps > 0) {
    if (nsteps >= WS - 1) wait_vmcnt<(WS - 2) * NJ>(); else wait_vmcnt<0>();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    static_for<NFRAG>([&](auto idx) { read_one(set0{}, idx, wl[0], xl[0]); });
    int i = 0;
    for (; i + WS - 1 < nsteps; ++i)
      step_body(std::true_type{}, std::true_type{}, std::integral_constant<int, (WS - 3) * NJ>{});
    // the last WS - 1 steps (or all of them): nothing left to load, everything in flight is waited for
    for (; i + 1 < nsteps; ++i) step_body(std::true_type{}, std::false_type{}, std::integral_constant<int, 0>{});
    step_body(std::false_type{}, std::false_type{}, std::integral_constant<int, 0>{});
  }
  wait_vmcnt<0>();
  combine_and_store32<FN, BN>(b, acc, m0, c0, wave_m, wk, lane, smem);
}

// ------------------------------------------------------------------------------------------------
// 3x3, stride 1, padding 1 (forward and stride-1 data gradient of the wide layers): patch form.
// ------------------------------------------------------------------------------------------------
// The nine taps of such a convolution read the same input pixels, shifted.  A tile of 128 consecutive output
// pixels m0 .. m0+127 (linear in n, oh, ow; input and output grids coincide) only ever touches the input
// pixels m0 - W - 1 .. m0 + 128 + W, so for each 64-channel block that range ("patch", PR rows) is landed in
// LDS ONCE and the taps address it with a per-lane row shift; only the weights stream per tap.  Against the
// generic wide kernel this moves 1.6x fewer bytes from L2 to LDS and, with the patch double buffered per
// channel block and the weights WS stages deep, looks nine taps (patch) and WS-1 taps (weights) ahead, which
// covers an L2 miss.  A tap that falls outside the image reads a zero region of LDS instead.
//
// Order of the direct-to-LDS loads in every wave: patch(0), w(0..WS-2), then per step i = 9c + t one group:
// w(i+WS-1) and, for t < XG, a share of patch(c+1).  Barrier i+1 (step i+1 visible) is taken after slot 1 of
// step i; loads complete in order, so "w(i+1) has landed" is vmcnt <= the sizes of the WS-3 groups issued after
// the one that carried it.
// KTAIL: the input channels are not a multiple of 64 (WRN's 160).  The last channel block is then partly beyond the
// tensor: its 16-byte units past the last channel are loaded from the zero word, for the patch and the weights alike,
// which costs every load of such a layer a per-lane address select (the other layers keep the uniform-base form).
template <int BN, int PR, int WS, bool KTAIL>
__global__ __launch_bounds__(256) void conv_patch_kernel(GatherConvArgs a, int m_tiles, int n_tiles) {
  constexpr int BM = 128, ROWB = 128;
  static_assert(BN % 32 == 0 && PR % 32 == 0, "whole DMA instructions and 32x32 blocks");
  constexpr int JX = PR / 32, JW = BN / 32;
  constexpr int FM = 2, FN = BN / 32;
  constexpr int XBYTES = PR * ROWB + 256, WBYTES = BN * ROWB;   // a patch buffer ends with two rows of zeros
  constexpr int LDS_BYTES = 2 * XBYTES + WS * WBYTES;
  static_assert((WS - 2) * JW + JX < 64, "vmcnt range");
  static_assert(WS >= 3 && WS <= 9, "pipeline depth");
  static_assert((size_t)LDS_BYTES >= (size_t)4 * FN * 16 * 256 && (size_t)LDS_BYTES >= (size_t)4 * out_stage_bytes(BN) + stats_stage_bytes(BN), "room for the output stage");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // LDS_BYTES

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave_m = wave & 1, wk = wave >> 1;
  const int Mtot = a.N * a.OH * a.OW;
  const int W = a.Wi, H = a.Hi;

  int t = blockIdx.x;
  const int total = m_tiles * n_tiles;
  if ((total & 7) == 0) t = (blockIdx.x & 7) * (total >> 3) + (blockIdx.x >> 3);
  const int m0 = (t / n_tiles) * BM, c0 = (t % n_tiles) * BN;

  if (tid < 32)   // the zero rows of both patch buffers; visible after the first barrier
    reinterpret_cast<uint4*>(smem + (tid >> 4) * XBYTES + PR * ROWB)[tid & 15] = make_uint4(0u, 0u, 0u, 0u);

  // ---- per-thread DMA sources as 32-bit offsets from a wave-uniform base (the address then needs no vector
  //      arithmetic).  Rows that do not exist (patch rows before the first or after the last pixel, weight
  //      rows past the last channel of a ragged tile) read some row that does: nothing valid refers to them. ----
  unsigned xoff[JX], woff[JW];
#pragma unroll
  for (int j = 0; j < JX; ++j) {
    const int p = 8 * (4 * j + wave) + (lane >> 3);
    const int u = (lane & 7) ^ ((p >> 1) & 7);
    int q = m0 - W - 1 + p;
    q = q < 0 ? 0 : (q >= Mtot ? Mtot - 1 : q);
    xoff[j] = (unsigned)q * (unsigned)(a.Ci * 2) + u * 16;
  }
#pragma unroll
  for (int j = 0; j < JW; ++j) {
    const int row = 8 * (4 * j + wave) + (lane >> 3);
    const int u = (lane & 7) ^ ((row >> 1) & 7);
    int c = c0 + row;
    c = c >= a.w_rows ? a.w_rows - 1 : c;
    woff[j] = (unsigned)c * (unsigned)(a.Kw * 2) + u * 16;
  }
  int tko[9];
#pragma unroll
  for (int i = 0; i < 9; ++i) tko[i] = (a.tap[i] >> 16) * a.Ci * 2;   // byte offset of the tap's k block in a weight row
  const int cpc = (a.Ci + 63) >> 6;   // channel blocks
  // KTAIL: bit j (patch loads) / bit 16 + j (weight loads): this lane's unit exists in the last channel block
  unsigned tail_ok = 0;
  uint32_t zero_lo = 0, zero_hi = 0;
  if (KTAIL) {
#pragma unroll
    for (int j = 0; j < JX; ++j) {
      const int p = 8 * (4 * j + wave) + (lane >> 3);
      const int u = (lane & 7) ^ ((p >> 1) & 7);
      if ((cpc - 1) * 64 + u * 8 < a.Ci) tail_ok |= 1u << j;
    }
#pragma unroll
    for (int j = 0; j < JW; ++j) {
      const int row = 8 * (4 * j + wave) + (lane >> 3);
      const int u = (lane & 7) ^ ((row >> 1) & 7);
      if ((cpc - 1) * 64 + u * 8 < a.Ci) tail_ok |= 1u << (16 + j);
    }
    const uint64_t z = (uint64_t)g_zero_word;
    zero_lo = (uint32_t)z; zero_hi = (uint32_t)(z >> 32);
    asm volatile("" : "+v"(zero_lo), "+v"(zero_hi));
  }
  static_assert(JX <= 16 && JW <= 16, "bits of tail_ok");

  auto issue_x_one = [&](int j, int c) {
    const char* base = reinterpret_cast<const char*>(a.in) + (size_t)c * 128;
    unsigned char* dst = smem + (c & 1) * XBYTES + (8 * (4 * j + wave)) * ROWB;
    if (KTAIL) {
      const bool ok = c != cpc - 1 || ((tail_ok >> j) & 1u);
      const uint64_t pa = (uint64_t)(base + (size_t)xoff[j]);
      const uint32_t lo = ok ? (uint32_t)pa : zero_lo, hi = ok ? (uint32_t)(pa >> 32) : zero_hi;
      dma16((const char*)(((uint64_t)hi << 32) | lo), dst);
    } else {
      dma16(base + (size_t)xoff[j], dst);
    }
  };
  // cblock: the channel block the weights belong to
  auto issue_w_one = [&](int j, int slot, int kbyte, int cblock) {
    const char* base = reinterpret_cast<const char*>(a.w) + (size_t)kbyte;
    unsigned char* dst = smem + 2 * XBYTES + slot * WBYTES + (8 * (4 * j + wave)) * ROWB;
    if (KTAIL) {
      const bool ok = cblock != cpc - 1 || ((tail_ok >> (16 + j)) & 1u);
      const uint64_t pa = (uint64_t)(base + (size_t)woff[j]);
      const uint32_t lo = ok ? (uint32_t)pa : zero_lo, hi = ok ? (uint32_t)(pa >> 32) : zero_hi;
      dma16((const char*)(((uint64_t)hi << 32) | lo), dst);
    } else {
      dma16(base + (size_t)woff[j], dst);
    }
  };
  // the first loads go out before the rest of the set-up, which then runs while they are in flight
#pragma unroll
  for (int j = 0; j < JX; ++j) issue_x_one(j, 0);
#pragma unroll
  for (int p = 0; p < WS - 1; ++p)   // 9 taps >= WS - 1 steps always exist
#pragma unroll
    for (int j = 0; j < JW; ++j) issue_w_one(j, p, tko[p], 0);

  f32x16 acc[FN][FM];
#pragma unroll
  for (int i = 0; i < FN; ++i)
#pragma unroll
    for (int j = 0; j < FM; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // ---- LDS addresses of this lane's operand fragments, computed once ----
  // pixels (operand B): for every tap, pixel block and 16-channel step the address inside patch buffer 0 -- the
  // shifted patch row, or a zero row at the same bank position when the tap falls outside the image; the
  // whole table moves by +-XBYTES when the channel block changes buffers.
  // weights (operand A): one address per 16-channel step; blocks are 4096 bytes apart (an immediate offset).
  const unsigned lds0 = (unsigned)(uintptr_t)((__attribute__((address_space(3))) unsigned char*)smem);
  unsigned xaddr[9][FM][2], wlane[2];
#pragma unroll
  for (int f = 0; f < FM; ++f) {
    const int r = wave_m * 64 + f * 32 + (lane & 31);
    const int m = m0 + r;
    const bool inside = m < Mtot;
    const int ow = m % a.OW, oh = (m / a.OW) % a.OH;
#pragma unroll
    for (int i = 0; i < 9; ++i) {
      const int dh = (a.tap[i] & 0xff) - 8, dw = ((a.tap[i] >> 8) & 0xff) - 8;
      const int p = r + W + 1 + dh * W + dw;
      const bool ok = inside && (unsigned)(oh + dh) < (unsigned)H && (unsigned)(ow + dw) < (unsigned)W;
      const int rowoff = ok ? p * ROWB : (PR + (p & 1)) * ROWB;
#pragma unroll
      for (int ss = 0; ss < 2; ++ss)
        xaddr[i][f][ss] = lds0 + rowoff + (((4 * wk + 2 * ss + (lane >> 5)) ^ ((p >> 1) & 7)) << 4);
    }
  }
#pragma unroll
  for (int ss = 0; ss < 2; ++ss)
    wlane[ss] = lds0 + 2 * XBYTES + (lane & 31) * ROWB + (((4 * wk + 2 * ss + (lane >> 5)) ^ (((lane & 31) >> 1) & 7)) << 4);

  // Operand fragments, two sets: while the MFMAs of one 16-channel half step run from one set, the reads of
  // the next half step fill the other, so LDS latency stays behind the matrix pipe even with one wave per
  // SIMD.  The compiler's scheduler would undo this to save registers, so each half step is written as
  // NM (MFMA, piece of other work) pairs pinned with scheduling barriers.
  constexpr int NM = FN * FM, NFRAG = FN + FM;
  static_assert(NFRAG + 2 <= NM && 2 + JW < NM, "slots of a half step");
  // The reads are inline assembly with explicit waits: left to the compiler every half step would begin with a
  // wait for ALL outstanding LDS reads, the ones issued a moment ago included, which exposes the LDS latency
  // twice per step.  LDS reads return in order, so "the first m fragments of this set have landed" is
  // lgkmcnt <= (fragments of the set still to come) + (fragments of the other set issued meanwhile).
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  u32x4 fa[2][FN], fb[2][FM];
  // fragment idx of a half step in the order the MFMAs need them: B0, A0, B1, A1, A2, ...
  // wcur: this lane's weight address for the step's stage and 16-channel step; xshift: 0, or the distance to
  // the other patch buffer when the fragment belongs to the next channel block.
  auto read_one = [&](auto set_tag, auto idx_tag, unsigned wcur, auto tap_tag, auto ss_tag, int xshift) {
    constexpr int S = decltype(set_tag)::value, IDX = decltype(idx_tag)::value, T = decltype(tap_tag)::value;
    constexpr int SS = decltype(ss_tag)::value;
    if constexpr (IDX == 0 || IDX == 2) {
      constexpr int f = IDX / 2;
      u32x4& dst = fb[S][f];
      const unsigned addr = xaddr[T][f][SS] + xshift;
      asm volatile("ds_read_b128 %0, %1" : "=v"(dst) : "v"(addr));
    } else {
      constexpr int f = IDX == 1 ? 0 : IDX - 2;
      u32x4& dst = fa[S][f];
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(wcur), "i"(f * 32 * ROWB));
    }
  };
  // Before MFMA K (K = 2 i + j uses A_i and B_j): the fragments it is the first to use have landed when at
  // most N reads are outstanding; the wait is tied to their registers so that the MFMA cannot move above it.
  auto before_mma = [&](auto set_tag, auto k_tag, auto n_tag) {
    constexpr int S = decltype(set_tag)::value, K = decltype(k_tag)::value, N = decltype(n_tag)::value;
    static_assert(N >= 0 && N <= 15, "lgkmcnt range");
    if constexpr (K == 0) {
      u32x4 &r0 = fb[S][0], &r1 = fa[S][0];
      asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(r0), "+v"(r1) : "n"(N));
    } else if constexpr (K == 1) {
      u32x4& r0 = fb[S][1];
      asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(r0) : "n"(N));
    } else if constexpr (K % 2 == 0) {
      u32x4& r0 = fa[S][K / 2];
      asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(r0) : "n"(N));
    }
  };
  // fragments of a set not yet needed when MFMA K starts
  auto left_after = [](int K) constexpr { return (FN + 2) - (K == 0 ? 2 : (K == 1 ? 3 : 3 + K / 2)); };
  auto mma_one = [&](auto set_tag, auto k_tag) {
    constexpr int S = decltype(set_tag)::value, K = decltype(k_tag)::value;
    acc[K / FM][K % FM] = mfma32(__builtin_bit_cast(bf16x8, fa[S][K / FM]), __builtin_bit_cast(bf16x8, fb[S][K % FM]),
                                 acc[K / FM][K % FM]);
  };
  using set0 = std::integral_constant<int, 0>;
  using set1 = std::integral_constant<int, 1>;

  // Barrier e makes step e visible and is taken inside step e - 1.  Before it every wave has finished
  // reading step e - 2, whose weight stage therefore receives step e + WS - 2 right after it.
  wait_vmcnt<(WS - 2) * JW>();
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  using tap0 = std::integral_constant<int, 0>;
  using ss0 = std::integral_constant<int, 0>;
  using ss1 = std::integral_constant<int, 1>;
  static_for<NFRAG>([&](auto idx) { read_one(set0{}, idx, wlane[0], tap0{}, ss0{}, 0); });

  // Loads are issued thinly: a step's group of loads -- the weights of step i + WS - 1 and, in the first XG steps
  // of a channel block, a share of the next block's patch -- goes out one load every other slot over the whole
  // step.  Issued in a burst, the loads fill the address queue, the wave stalls on the next one and the MFMAs
  // behind it starve, although the step has time for all of them.
  constexpr int XG = 11 - WS;                       // groups that may carry patch loads (landed by the block's end)
  constexpr int PER = (JX + XG - 1) / XG;           // patch loads per such group
  static_assert(3 + 2 * (JW + PER - 1) < 2 * NM, "one load every other slot fits the step");
  // loads in the group of tap t (t < 0: a tap of the previous block, or the prologue)
  auto gsize = [](int t, bool last) constexpr {
    if (t < 0) return JW;
    const int w = last ? (t + WS - 1 <= 8 ? JW : 0) : JW;
    const int left = JX - t * PER;
    const int x = (!last && t < XG && left > 0) ? (left < PER ? left : PER) : 0;
    return w + x;
  };
  int slot = 0;   // weight stage of the current step
  auto chunk_body = [&](int c, auto last_tag) {
    constexpr bool LAST = decltype(last_tag)::value;
    const int to_other = (c & 1) ? -XBYTES : XBYTES;   // from this block's patch buffer to the other one
    if (c > 0) {
#pragma unroll
      for (int i = 0; i < 9; ++i)
#pragma unroll
        for (int f = 0; f < FM; ++f)
#pragma unroll
          for (int ss = 0; ss < 2; ++ss) xaddr[i][f][ss] -= to_other;   // the table follows the block into its buffer
    }
    static_for<9>([&](auto t_tag) {
      constexpr int T = decltype(t_tag)::value;
      const int nslot = slot == WS - 1 ? 0 : slot + 1;
      const int islot = slot == 0 ? WS - 1 : slot - 1;
      const unsigned wcur1 = wlane[1] + slot * WBYTES, wnext0 = wlane[0] + nslot * WBYTES;
      constexpr bool MORE = !(LAST && T == 8);            // a next step exists
      constexpr int TT = T + WS - 1;                      // tap of the step whose weights are issued now
      constexpr bool ISSUE_W = TT < 9 || !LAST;
      constexpr int NW = ISSUE_W ? JW : 0;
      constexpr int NX = gsize(T, LAST) - NW;             // patch loads of this group: pieces T*PER ...
      const int kbyte = TT < 9 ? tko[TT < 9 ? TT : 0] + c * 128 : tko[TT < 9 ? 0 : TT - 9] + (c + 1) * 128;
      const int wblock = TT < 9 ? c : c + 1;
      // load idx of the group goes out after the MFMA of global slot 3 + 2 idx (slots 0 .. 2 NM - 1 over both halves)
      auto issue_at = [&](auto s_tag) {
        constexpr int SL = decltype(s_tag)::value;
        if constexpr (SL >= 3 && (SL - 3) % 2 == 0) {
          constexpr int IDX = (SL - 3) / 2;
          if constexpr (IDX < NW) issue_w_one(IDX, islot, kbyte, wblock);
          else if constexpr (IDX - NW < NX) issue_x_one(T * PER + IDX - NW, c + 1);
        }
      };
      // first half step: MFMAs of set 0, reads of this step's second half into set 1.  After slot 1: barrier
      // T+1 (next step visible; everybody done reading the previous step, whose stage the group overwrites).
      static_for<NM>([&](auto k) {
        constexpr int K = decltype(k)::value;
        // set 1 is filled one fragment per slot from slot 0 on
        if constexpr (K <= 1 || K % 2 == 0)
          before_mma(set0{}, k, std::integral_constant<int, left_after(K) + (K < NFRAG ? K : NFRAG)>{});
        mma_one(set0{}, k);
        if constexpr (K < NFRAG) read_one(set1{}, k, wcur1, t_tag, ss1{}, 0);
        if constexpr (MORE && K == 1) {
          constexpr int PENDING = (WS >= 4 ? gsize(T - 1, LAST) : 0) + (WS >= 5 ? gsize(T - 2, LAST) : 0) +
                                  (WS >= 6 ? gsize(T - 3, LAST) : 0) + (WS >= 7 ? gsize(T - 4, LAST) : 0);
          static_assert(WS <= 7, "terms above");
          wait_vmcnt<PENDING>();
          asm volatile("" ::: "memory");
          __builtin_amdgcn_s_barrier();
          asm volatile("" ::: "memory");
        }
        if constexpr (MORE) issue_at(std::integral_constant<int, K>{});
        __builtin_amdgcn_sched_barrier(0);
      });
      // second half step: MFMAs of set 1, the next step's first reads into set 0
      static_for<NM>([&](auto k) {
        constexpr int K = decltype(k)::value;
        // set 0 of the next step is filled one fragment per slot from slot 2 on (when there is a next step)
        if constexpr (K <= 1 || K % 2 == 0)
          before_mma(set1{}, k, std::integral_constant<int, left_after(K) + ((MORE && K > 2) ? (K - 2 < NFRAG ? K - 2 : NFRAG) : 0)>{});
        mma_one(set1{}, k);
        if constexpr (MORE) {
          if constexpr (K >= 2 && K - 2 < NFRAG) {
            if constexpr (T < 8) read_one(set0{}, std::integral_constant<int, K - 2>{}, wnext0, std::integral_constant<int, (T + 1) % 9>{}, ss0{}, 0);
            else read_one(set0{}, std::integral_constant<int, K - 2>{}, wnext0, tap0{}, ss0{}, to_other);
          }
          issue_at(std::integral_constant<int, NM + K>{});
        }
        __builtin_amdgcn_sched_barrier(0);
      });
      slot = nslot;
    });
  };
  for (int c = 0; c < cpc - 1; ++c) chunk_body(c, std::false_type{});
  chunk_body(cpc - 1, std::true_type{});

  wait_vmcnt<0>();
  combine_and_store32<FN, BN>(a, acc, m0, c0, wave_m, wk, lane, smem);
}

// The patch form on tiles of 256 pixels with EIGHT waves, two per SIMD, for layers whose 128-pixel tiles would need
// two rounds of workgroups (the 320-channel layers at 16x16: 512 tiles): one round of twice as large workgroups halves
// what every workgroup pays before and after its main loop, and a weight stage is shared by four pixel waves
// instead of two.  Wave (wave_m = wave & 3, wk = wave >> 2) owns 64 pixels x BN channels (2 x BN/32 accumulator
// blocks) and one 32-channel half of every 64-channel block, as in the four-wave kernel.  To fit 256 registers there
// is a single set of fragments: the MFMAs of a half step run pixel block by pixel block (K = FN j + i), so P0 is free
// after MFMA FN-1, W_i after MFMA FN+i, P1 after the last one, and each is read again for the next half step right
// there; the partner wave on the SIMD covers the rest of the latency.  The second half step of a tap differs from the
// first by bit 5 of every fragment address.  Weight stages are BN rows: with 64 rows per load instruction of the
// workgroup BN = 160 needs 2.5 of them, so the third load of waves 4 .. 7 goes to a dump area (every wave then counts
// the same number of loads).
template <int BN, int PR, int WS, bool KTAIL>
__global__ __launch_bounds__(512) void conv_patch256_kernel(GatherConvArgs a, int m_tiles, int n_tiles) {
  constexpr int BM = 256, ROWB = 128, NWAVES = 8;
  static_assert(BN % 32 == 0 && PR % 64 == 0, "whole DMA instructions and 32x32 blocks");
  constexpr int JX = PR / 64, JW = (BN + 63) / 64;
  constexpr int FM = 2, FN = BN / 32;
  constexpr int XBYTES = PR * ROWB + 256, WBYTES = BN * ROWB;   // a patch buffer ends with two rows of zeros
  constexpr int DUMP = 2 * XBYTES + WS * WBYTES;                // 1 KB per wave_m that nobody reads, or one for all
  constexpr int DUMP_EACH = DUMP + 4096 <= 160 * 1024 ? 1024 : 0;
  constexpr int LDS_BYTES = DUMP + (DUMP_EACH ? 4096 : 1024);
  static_assert(LDS_BYTES <= 160 * 1024, "LDS of one compute unit");
  static_assert((WS - 2) * JW + JX < 64, "vmcnt range");
  static_assert(WS >= 3 && WS <= 7, "pipeline depth");
  static_assert((size_t)LDS_BYTES >= (size_t)4 * FN * 4096 && (size_t)LDS_BYTES >= (size_t)8 * out_stage16_bytes(BN) &&
                (size_t)LDS_BYTES >= (size_t)2 * stats_stage_bytes(BN), "room for the output stage");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // LDS_BYTES

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave_m = wave & 3, wk = wave >> 2;
  const int Mtot = a.N * a.OH * a.OW;
  const int W = a.Wi, H = a.Hi;

  int t = blockIdx.x;
  const int total = m_tiles * n_tiles;
  if ((total & 7) == 0) t = (blockIdx.x & 7) * (total >> 3) + (blockIdx.x >> 3);
  const int m0 = (t / n_tiles) * BM, c0 = (t % n_tiles) * BN;

  if (tid < 32)   // the zero rows of both patch buffers; visible after the first barrier
    reinterpret_cast<uint4*>(smem + (tid >> 4) * XBYTES + PR * ROWB)[tid & 15] = make_uint4(0u, 0u, 0u, 0u);

  // ---- per-thread DMA sources as 32-bit offsets from a wave-uniform base; rows that do not exist read some row
  //      that does (nothing valid refers to them) ----
  unsigned xoff[JX], woff[JW];
#pragma unroll
  for (int j = 0; j < JX; ++j) {
    const int p = 8 * (NWAVES * j + wave) + (lane >> 3);
    const int u = (lane & 7) ^ ((p >> 1) & 7);
    int q = m0 - W - 1 + p;
    q = q < 0 ? 0 : (q >= Mtot ? Mtot - 1 : q);
    xoff[j] = (unsigned)q * (unsigned)(a.Ci * 2) + u * 16;
  }
#pragma unroll
  for (int j = 0; j < JW; ++j) {
    const int row = 8 * (NWAVES * j + wave) + (lane >> 3);
    const int u = (lane & 7) ^ ((row >> 1) & 7);
    int c = c0 + row;
    c = c >= a.w_rows ? a.w_rows - 1 : c;
    woff[j] = (unsigned)c * (unsigned)(a.Kw * 2) + u * 16;
  }
  int tko[9];
#pragma unroll
  for (int i = 0; i < 9; ++i) tko[i] = (a.tap[i] >> 16) * a.Ci * 2;   // byte offset of the tap's k block in a weight row
  const int cpc = (a.Ci + 63) >> 6;   // channel blocks
  // KTAIL (as in conv_patch_kernel): bit j (patch loads) / bit 16 + j (weight loads): this lane's unit exists in the
  // last channel block; the others come from the zero word
  unsigned tail_ok = 0;
  uint32_t zero_lo = 0, zero_hi = 0;
  if (KTAIL) {
#pragma unroll
    for (int j = 0; j < JX; ++j) {
      const int p = 8 * (NWAVES * j + wave) + (lane >> 3);
      const int u = (lane & 7) ^ ((p >> 1) & 7);
      if ((cpc - 1) * 64 + u * 8 < a.Ci) tail_ok |= 1u << j;
    }
#pragma unroll
    for (int j = 0; j < JW; ++j) {
      const int row = 8 * (NWAVES * j + wave) + (lane >> 3);
      const int u = (lane & 7) ^ ((row >> 1) & 7);
      if ((cpc - 1) * 64 + u * 8 < a.Ci) tail_ok |= 1u << (16 + j);
    }
    const uint64_t z = (uint64_t)g_zero_word;
    zero_lo = (uint32_t)z; zero_hi = (uint32_t)(z >> 32);
    asm volatile("" : "+v"(zero_lo), "+v"(zero_hi));
  }
  static_assert(JX <= 16 && JW <= 16, "bits of tail_ok");

  auto issue_x_one = [&](int j, int c) {
    const char* base = reinterpret_cast<const char*>(a.in) + (size_t)c * 128;
    unsigned char* dst = smem + (c & 1) * XBYTES + (8 * (NWAVES * j + wave)) * ROWB;
    if (KTAIL) {
      const bool ok = c != cpc - 1 || ((tail_ok >> j) & 1u);
      const uint64_t pa = (uint64_t)(base + (size_t)xoff[j]);
      const uint32_t lo = ok ? (uint32_t)pa : zero_lo, hi = ok ? (uint32_t)(pa >> 32) : zero_hi;
      dma16((const char*)(((uint64_t)hi << 32) | lo), dst);
    } else {
      dma16(base + (size_t)xoff[j], dst);
    }
  };
  // cblock: the channel block the weights belong to
  auto issue_w_one = [&](int j, int slot, int kbyte, int cblock) {
    const char* base = reinterpret_cast<const char*>(a.w) + (size_t)kbyte;
    const int row0 = 8 * (NWAVES * j + wave);   // rows past the stage: the load still happens, into the dump area
    unsigned char* dst = row0 < BN ? smem + 2 * XBYTES + slot * WBYTES + row0 * ROWB : smem + DUMP + (wave & 3) * DUMP_EACH;
    if (KTAIL) {
      const bool ok = cblock != cpc - 1 || ((tail_ok >> (16 + j)) & 1u);
      const uint64_t pa = (uint64_t)(base + (size_t)woff[j]);
      const uint32_t lo = ok ? (uint32_t)pa : zero_lo, hi = ok ? (uint32_t)(pa >> 32) : zero_hi;
      dma16((const char*)(((uint64_t)hi << 32) | lo), dst);
    } else {
      dma16(base + (size_t)woff[j], dst);
    }
  };
#pragma unroll
  for (int j = 0; j < JX; ++j) issue_x_one(j, 0);
#pragma unroll
  for (int p = 0; p < WS - 1; ++p)   // 9 taps >= WS - 1 steps always exist
#pragma unroll
    for (int j = 0; j < JW; ++j) issue_w_one(j, p, tko[p], 0);

  f32x16 acc[FN][FM];
#pragma unroll
  for (int i = 0; i < FN; ++i)
#pragma unroll
    for (int j = 0; j < FM; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // ---- LDS addresses of this lane's fragments for the first 16-channel step of its half (the second one: ^ 32):
  //      per tap and pixel block the shifted patch row in buffer 0 (or a zero row at the same bank position when the
  //      tap falls outside the image); one address for the weights ----
  const unsigned lds0 = (unsigned)(uintptr_t)((__attribute__((address_space(3))) unsigned char*)smem);
  unsigned xaddr[9][FM], wlane;
#pragma unroll
  for (int f = 0; f < FM; ++f) {
    const int r = wave_m * 64 + f * 32 + (lane & 31);
    const int m = m0 + r;
    const bool inside = m < Mtot;
    const int ow = m % a.OW, oh = (m / a.OW) % a.OH;
#pragma unroll
    for (int i = 0; i < 9; ++i) {
      const int dh = (a.tap[i] & 0xff) - 8, dw = ((a.tap[i] >> 8) & 0xff) - 8;
      const int p = r + W + 1 + dh * W + dw;
      const bool ok = inside && (unsigned)(oh + dh) < (unsigned)H && (unsigned)(ow + dw) < (unsigned)W;
      const int rowoff = ok ? p * ROWB : (PR + (p & 1)) * ROWB;
      xaddr[i][f] = lds0 + rowoff + (((4 * wk + (lane >> 5)) ^ ((p >> 1) & 7)) << 4);
    }
  }
  wlane = lds0 + 2 * XBYTES + (lane & 31) * ROWB + (((4 * wk + (lane >> 5)) ^ (((lane & 31) >> 1) & 7)) << 4);
  if (lds0 & 127u) return;   // "^ 32" below flips the unit only if the LDS base is a multiple of 128 (it is 0: no static LDS)

  // fragments in read order: position 0 = P0, 1 .. FN = W0 .. W(FN-1), FN+1 = P1
  constexpr int NM = FN * FM, NFRAG = FN + FM;
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  u32x4 fw[FN], fp[FM];
  // wcur: this lane's weight address in the step's stage; SS: which 16-channel step of the half
  auto read_pos = [&](auto pos_tag, unsigned wcur, auto tap_tag, auto ss_tag, int xshift) {
    constexpr int POS = decltype(pos_tag)::value, T = decltype(tap_tag)::value, SS = decltype(ss_tag)::value;
    if constexpr (POS == 0 || POS == FN + 1) {
      constexpr int f = POS == 0 ? 0 : 1;
      u32x4& dst = fp[f];
      const unsigned addr = (xaddr[T][f] + xshift) ^ (SS * 32);
      asm volatile("ds_read_b128 %0, %1" : "=v"(dst) : "v"(addr));
    } else {
      constexpr int f = POS - 1;
      u32x4& dst = fw[f];
      const unsigned addr = wcur ^ (SS * 32);
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "i"(f * 32 * ROWB));
    }
  };
  auto wait_p = [&](auto f_tag, auto n_tag) {
    constexpr int F = decltype(f_tag)::value, N = decltype(n_tag)::value;
    static_assert(N >= 0 && N <= 15, "lgkmcnt range");
    u32x4& r = fp[F];
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(r) : "n"(N));
  };
  auto wait_w = [&](auto f_tag, auto n_tag) {
    constexpr int F = decltype(f_tag)::value, N = decltype(n_tag)::value;
    static_assert(N >= 0 && N <= 15, "lgkmcnt range");
    u32x4& r = fw[F];
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(r) : "n"(N));
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;

  wait_vmcnt<(WS - 2) * JW>();
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  static_for<NFRAG>([&](auto pos) { read_pos(pos, wlane, I0{}, I0{}, 0); });

  // loads of a step's group (the weights of step i + WS - 1 and, in the first XG steps of a channel block, a share of
  // the next block's patch) go out in the first half step after the MFMAs of slots 2, 3, 5, 7: after the barrier
  constexpr int XG = 11 - WS;
  constexpr int PER = (JX + XG - 1) / XG;
  static_assert(JW + PER <= 2 + (NM - 4) / 2, "load slots of a half step");
  auto gsize = [](int t, bool last) constexpr {
    if (t < 0) return JW;
    const int w = last ? (t + WS - 1 <= 8 ? JW : 0) : JW;
    const int left = JX - t * PER;
    const int x = (!last && t < XG && left > 0) ? (left < PER ? left : PER) : 0;
    return w + x;
  };
  int slot = 0;   // weight stage of the current step
  auto chunk_body = [&](int c, auto last_tag) {
    constexpr bool LAST = decltype(last_tag)::value;
    const int to_other = (c & 1) ? -XBYTES : XBYTES;   // from this block's patch buffer to the other one
    if (c > 0) {
#pragma unroll
      for (int i = 0; i < 9; ++i)
#pragma unroll
        for (int f = 0; f < FM; ++f) xaddr[i][f] -= to_other;   // the table follows the block into its buffer
    }
    static_for<9>([&](auto t_tag) {
      constexpr int T = decltype(t_tag)::value;
      const int nslot = slot == WS - 1 ? 0 : slot + 1;
      const int islot = slot == 0 ? WS - 1 : slot - 1;
      const unsigned wcur = wlane + slot * WBYTES, wnext = wlane + nslot * WBYTES;
      constexpr bool MORE = !(LAST && T == 8);            // a next step exists
      constexpr int TT = T + WS - 1;                      // tap of the step whose weights are issued now
      constexpr bool ISSUE_W = TT < 9 || !LAST;
      constexpr int NWL = ISSUE_W ? JW : 0;
      constexpr int NX = gsize(T, LAST) - NWL;            // patch loads of this group: pieces T*PER ...
      const int kbyte = TT < 9 ? tko[TT < 9 ? TT : 0] + c * 128 : tko[TT < 9 ? 0 : TT - 9] + (c + 1) * 128;
      using next_tap = std::integral_constant<int, (T + 1) % 9>;
      const int next_shift = T < 8 ? 0 : to_other;
      static_for<2>([&](auto ss_tag) {
        constexpr int SS = decltype(ss_tag)::value;
        constexpr bool FOLLOWS = SS == 0 || MORE;          // a half step follows this one
        static_for<NM>([&](auto k) {
          constexpr int K = decltype(k)::value;
          // this half step's reads went out as P0 W0 .. W(FN-1) P1; the next one's start after MFMA FN-1
          if constexpr (K == 0) {
            wait_p(I0{}, std::integral_constant<int, FN + 1>{});
            wait_w(I0{}, std::integral_constant<int, FN>{});
          } else if constexpr (K < FN) {
            wait_w(std::integral_constant<int, K>{}, std::integral_constant<int, FN - K>{});
          } else if constexpr (K == FN) {
            wait_p(I1{}, std::integral_constant<int, FOLLOWS ? 1 : 0>{});
          }
          acc[K % FN][K / FN] = mfma32(__builtin_bit_cast(bf16x8, fw[K % FN]), __builtin_bit_cast(bf16x8, fp[K / FN]),
                                       acc[K % FN][K / FN]);
          if constexpr (FOLLOWS) {
            // the following half step: the second 16 channels of this tap, or the first of the next tap
            auto rd = [&](auto pos_tag) {
              if constexpr (SS == 0) read_pos(pos_tag, wcur, t_tag, I1{}, 0);
              else read_pos(pos_tag, wnext, next_tap{}, I0{}, next_shift);
            };
            if constexpr (K == FN - 1) rd(I0{});
            if constexpr (K >= FN) rd(std::integral_constant<int, K - FN + 1>{});
            if constexpr (K == NM - 1) rd(std::integral_constant<int, FN + 1>{});
          }
          if constexpr (SS == 0 && MORE && K == 1) {
            constexpr int PENDING = (WS >= 4 ? gsize(T - 1, LAST) : 0) + (WS >= 5 ? gsize(T - 2, LAST) : 0) +
                                    (WS >= 6 ? gsize(T - 3, LAST) : 0) + (WS >= 7 ? gsize(T - 4, LAST) : 0);
            wait_vmcnt<PENDING>();
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
          }
          if constexpr (SS == 0 && MORE && (K == 2 || K == 3 || (K >= 5 && K % 2 == 1))) {
            constexpr int IDX = K <= 3 ? K - 2 : 2 + (K - 5) / 2;
            if constexpr (IDX < NWL) issue_w_one(IDX, islot, kbyte, TT < 9 ? c : c + 1);
            else if constexpr (IDX - NWL < NX) issue_x_one(T * PER + IDX - NWL, c + 1);
          }
          __builtin_amdgcn_sched_barrier(0);
        });
      });
      slot = nslot;
    });
  };
  for (int c = 0; c < cpc - 1; ++c) chunk_body(c, std::false_type{});
  chunk_body(cpc - 1, std::true_type{});

  wait_vmcnt<0>();
  combine8_and_store32<FN, BN>(a, acc, m0, c0, wave_m, wk, lane, smem);
}

// the patch form needs: nine taps within +-1, unit strides, coinciding input and output grids
static bool conv_patch_applies(const GatherConvArgs& a) {
  if (a.Ci % 64 != 0 && (a.Ci % 8 != 0 || a.Ci < 128)) return false;   // whole channel blocks, or >= 2 with a partly filled last one
  if (a.ntaps != 9 || a.in_stride != 1 || a.out_stride != 1 || a.ooh != 0 || a.oow != 0) return false;
  if (a.OH != a.Hi || a.OW != a.Wi || a.OHf != a.OH || a.OWf != a.OW || a.Wi > 32 || a.Wi < 1) return false;
  if (a.w_rows != a.Co) return false;                                     // no rows of zeros inside the weight matrix
  if ((long long)a.N * a.Hi * a.Wi * a.Ci * 2 >= (1ll << 32) || (long long)a.w_rows * a.Kw * 2 >= (1ll << 32)) return false;   // 32-bit load offsets
  for (int i = 0; i < 9; ++i) {
    const int dh = (a.tap[i] & 0xff) - 8, dw = ((a.tap[i] >> 8) & 0xff) - 8;
    if (dh < -1 || dh > 1 || dw < -1 || dw > 1) return false;
  }
  return true;
}

template <int BN, int PR, bool KTAIL>
static hipError_t run_patch_k(const GatherConvArgs& a, hipStream_t s) {
  constexpr int WS = 5;
  constexpr size_t lds = (size_t)2 * (PR * 128 + 256) + (size_t)WS * BN * 128;
  static_assert(lds + 2 * BN * 4 <= 160 * 1024, "LDS of one compute unit");
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_patch_kernel<BN, PR, WS, KTAIL>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int Mtot = a.N * a.OH * a.OW;
  const int m_tiles = (Mtot + 127) / 128, n_tiles = (a.Co + BN - 1) / BN;
  static char name[64];
  if (!name[0]) snprintf(name, sizeof(name), KTAIL ? "conv_patch_kernel<%d, %d, %d, true>" : "conv_patch_kernel<%d, %d, %d>", BN, PR, WS);
  note_kernel(name);
  hipLaunchKernelGGL((conv_patch_kernel<BN, PR, WS, KTAIL>), dim3(m_tiles * n_tiles), dim3(256), lds, s, a, m_tiles, n_tiles);
  return hipGetLastError();
}

template <int BN, int PR>
static hipError_t run_patch(const GatherConvArgs& a, hipStream_t s) {
  return a.Ci % 64 == 0 ? run_patch_k<BN, PR, false>(a, s) : run_patch_k<BN, PR, true>(a, s);
}

template <int BN, int PR, int WS, bool KTAIL>
static hipError_t run_patch256(const GatherConvArgs& a, hipStream_t s) {
  constexpr size_t body = (size_t)2 * (PR * 128 + 256) + (size_t)WS * BN * 128;
  constexpr size_t lds = body + (body + 4096 <= 160 * 1024 ? 4096 : 1024);   // the kernel's LDS_BYTES
  static_assert(lds <= 160 * 1024, "LDS of one compute unit");
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_patch256_kernel<BN, PR, WS, KTAIL>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int Mtot = a.N * a.OH * a.OW;
  const int m_tiles = (Mtot + 255) / 256, n_tiles = (a.Co + BN - 1) / BN;
  static char name[64];
  if (!name[0]) snprintf(name, sizeof(name), KTAIL ? "conv_patch256_kernel<%d, %d, %d, true>" : "conv_patch256_kernel<%d, %d, %d>", BN, PR, WS);
  note_kernel(name);
  hipLaunchKernelGGL((conv_patch256_kernel<BN, PR, WS, KTAIL>), dim3(m_tiles * n_tiles), dim3(512), lds, s, a, m_tiles, n_tiles);
  return hipGetLastError();
}

template <int BN>
static hipError_t run_patch_rows(const GatherConvArgs& a, hipStream_t s) {
  // 256-pixel tiles where 128-pixel tiles need more than one round of workgroups and the larger ones still fill the chip
  {
    const int Mtot = a.N * a.OH * a.OW, n_tiles = (a.Co + BN - 1) / BN;
    const int t128 = (Mtot + 127) / 128 * n_tiles, t256 = (Mtot + 255) / 256 * n_tiles;
    if (t128 > 256 && t256 >= 224) {
      if (a.Ci % 64 != 0) return run_patch256<BN, 384, 3, true>(a, s);
      return 256 + 2 * a.Wi + 2 <= 320 ? run_patch256<BN, 320, 3, false>(a, s) : run_patch256<BN, 384, 3, false>(a, s);
    }
  }
  const int rows = 128 + 2 * a.Wi + 2;   // patch rows in use
  if (rows <= 160) return run_patch<BN, 160>(a, s);
  if (rows <= 192) return run_patch<BN, 192>(a, s);
  return run_patch<BN, 224>(a, s);
}

bool conv_gather_wide_applies(const GatherConvArgs& a) {
  // input channels: whole 64-channel chunks, or at least two chunks with a partly filled last one (160 = 2.5 chunks)
  const bool k_ok = a.Ci % 64 == 0 || (a.Ci % 8 == 0 && a.Ci >= 128);
  if ((long long)a.w_rows * a.Kw * 2 >= (1ll << 32)) return false;   // 32-bit offsets into the weight matrix
  return k_ok && a.Co >= 128 && a.ntaps >= 1 && a.ntaps <= 9 && a.Kw % 8 == 0 && a.Hi < 32768 && a.Wi < 32768;
}

template <int BN, int STAGES, bool KTAIL>
static hipError_t run_wide_k(const GatherConvArgs& a, hipStream_t s) {
  constexpr size_t lds = (size_t)STAGES * (128 + BN) * 128;
  static_assert(lds <= 160 * 1024 && lds >= gather_dma_lds_bytes(BN, 1), "LDS of one compute unit; room for the output stage");
  static bool configured = false;   // one attribute call per instantiation (idempotent, so a race is harmless)
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_gather_pipe_kernel<BN, STAGES, KTAIL>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int n_tiles = (a.Co + BN - 1) / BN;
  static char name[64];
  if (!name[0]) snprintf(name, sizeof(name), "conv_gather_pipe_kernel<%d, %d, %s>", BN, STAGES, KTAIL ? "true" : "false");
  note_kernel(name);
  if (a.nclass > 1) {
    GatherConvArgs m = a;
    int tiles = 0;
    for (int i = 0; i < a.nclass; ++i) {
      m.cls_start[i] = tiles;
      tiles += (a.N * a.cOH[i] * a.cOW[i] + 127) / 128 * n_tiles;
    }
    m.cls_start[a.nclass] = tiles;
    if (tiles <= 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL((conv_gather_pipe_kernel<BN, STAGES, KTAIL>), dim3(tiles), dim3(256), lds, s, m, 0, n_tiles);
    return hipGetLastError();
  }
  const int Mtot = a.N * a.OH * a.OW;
  const int m_tiles = (Mtot + 127) / 128;
  hipLaunchKernelGGL((conv_gather_pipe_kernel<BN, STAGES, KTAIL>), dim3(m_tiles * n_tiles), dim3(256), lds, s, a, m_tiles, n_tiles);
  return hipGetLastError();
}

template <bool F32S>
static hipError_t run_wide_pair_f(const GatherConvArgs& a, hipStream_t s) {
  constexpr int BN = 128, STAGES = 2;
  constexpr size_t lds = gather_dma_lds_bytes(BN, STAGES);
  static_assert(2 * lds <= 160 * 1024, "two workgroups in the LDS of one compute unit");
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_gather_dma_pair_kernel<BN, STAGES, false, F32S>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  note_kernel(F32S ? "conv_gather_dma_pair_kernel<128, 2, feeding>" : "conv_gather_dma_pair_kernel<128, 2>");
  const int m_tiles = (a.N * a.OH * a.OW + 127) / 128, n_tiles = (a.Co + BN - 1) / BN;
  hipLaunchKernelGGL((conv_gather_dma_pair_kernel<BN, STAGES, false, F32S>), dim3(m_tiles * n_tiles), dim3(256), lds, s, a, m_tiles, n_tiles);
  return hipGetLastError();
}
static hipError_t run_wide_pair(const GatherConvArgs& a, hipStream_t s) {
  return (a.stats && a.stats_f32) ? run_wide_pair_f<true>(a, s) : run_wide_pair_f<false>(a, s);
}

// The two-workgroup form runs this layer (and with it the output stage that can take the sums of the fp32 values).
bool conv_gather_pair_applies(const GatherConvArgs& a) {
  if (a.nclass > 1 || a.Co % 160 == 0 || a.Ci % 64 != 0 || !conv_gather_wide_applies(a) || conv_patch_applies(a)) return false;
  const int steps = a.ntaps * ((a.Ci + 63) / 64);
  const long tiles = (long)((a.N * a.OH * a.OW + 127) / 128) * ((a.Co + 127) / 128);
  return steps <= 16 && tiles >= 300;   // a short contraction over more tiles than compute units
}

template <int BN, int STAGES>
static hipError_t run_wide(const GatherConvArgs& a, hipStream_t s) {
  return a.Ci % 64 == 0 ? run_wide_k<BN, STAGES, false>(a, s) : run_wide_k<BN, STAGES, true>(a, s);
}

hipError_t launch_conv_gather_wide(const GatherConvArgs& a, hipStream_t s) {
  if (a.w_rows != a.Co) return hipErrorInvalidValue;   // weight rows past the last one are clamped, not zero
  if (a.nclass > 1) {   // the caller has checked conv_gather_wide_applies on the common fields
    if (a.nclass > 4 || a.Ci % 8 != 0 || a.Ci < 64 || a.Co < 128) return hipErrorInvalidValue;
    return a.Co % 160 == 0 ? run_wide<160, 4>(a, s) : run_wide<128, 4>(a, s);
  }
  if (!conv_gather_wide_applies(a) || a.N * a.OH * a.OW <= 0) return hipErrorInvalidValue;
  if (a.stats && a.stats_f32 && !conv_gather_pair_applies(a)) return hipErrorInvalidValue;   // only that form takes the sums of the fp32 values
  if (conv_patch_applies(a)) return a.Co % 160 == 0 ? run_patch_rows<160>(a, s) : run_patch_rows<128>(a, s);
  // A short contraction (a 1x1 convolution: at most 16 steps per tile) over more tiles than compute units: two stages
  // instead of four are 75 KB of LDS, so two workgroups share a compute unit, one's output stage runs beside the
  // other's loads and main loop, and 257 .. 512 tiles take one round instead of two.
  if (conv_gather_pair_applies(a)) return run_wide_pair(a, s);
  if (a.Co % 160 == 0) return run_wide<160, 4>(a, s);
  return run_wide<128, 4>(a, s);
}

// ------------------------------------------------------------------------------------------------
// Weight gradient for wide layers: dw[co, tap, ci] += sum_pixel dy[pixel, co] * x[pixel + tap, ci]
// ------------------------------------------------------------------------------------------------
// Both operands are [pixel][channel] in memory while the MFMA wants, per lane, 8 consecutive pixels of one
// channel.  The tiles are landed in LDS as they are (direct global-to-LDS loads, 64 pixels x 160 channels
// of dy and of the shifted x per chunk) and read with ds_read_b64_tr_b16, which transposes on the way
// out: in a group of 16 lanes, lanes 4j..4j+3 address 16 consecutive bf16 of pixel j, and lane i
// receives element i of pixels 0..3.  Two such reads give a lane its 8 pixels (k values); which 8 is
// free as long as both operands agree: lane group g takes pixels 4g..4g+3 and 16+4g..16+4g+3 of a
// 32-pixel step.  Rows are 320 bytes, so 4 consecutive pixels fall into 4 different 64-byte windows of
// the banks; the 32-byte slot index is XORed with bit 2 of the pixel so that 8 consecutive pixels are
// conflict free.  One workgroup owns a 160 x 160 block of one tap and a range of pixel chunks; partial
// sums are added with fp32 atomics.
typedef short v4s16 __attribute__((ext_vector_type(4)));

// Both halves of a fragment as inline assembly, not through the builtin: the compiler treats the builtin as a
// possible LDS store and makes every one of them wait for ALL outstanding direct-to-LDS loads.  The caller
// waits (lds_wait_frags) before it uses the values.
__device__ __forceinline__ void lds_read_tr8(unsigned lds_addr, v4s16& lo, v4s16& hi) {
  asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(lo) : "v"(lds_addr));
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:5120" : "=v"(hi) : "v"(lds_addr));   // 16 rows of 320 bytes further
}
__device__ __forceinline__ bf16x8 join_tr8(v4s16 lo, v4s16 hi) {
  typedef short v8s16 __attribute__((ext_vector_type(8)));
  const v8s16 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, both);
}

struct WgradWideLaunch {
  int co_tiles, ci_tiles, splits, chunks_per_split;
  float* partial;        // when set: split s stores its block at partial + s * split_stride (no atomics)
  size_t split_stride;   // elements of one [Co][T][Ci] array
};

template <int STAGES>
__global__ __launch_bounds__(256) void conv_wgrad_dma_kernel(WgradArgs a, WgradWideLaunch L) {
  constexpr int BC = 160;                  // channels per operand tile
  constexpr int BKP = 64;                  // pixels per chunk
  constexpr int ROWB = BC * 2;             // 320 bytes per pixel row
  constexpr int UPR = BC / 8;              // 16-byte units per row (20)
  constexpr int PART = BKP * ROWB;         // bytes of one operand tile (20480)
  constexpr int JP = BKP * UPR / 256;      // DMA instructions per thread per operand (5)
  constexpr int NJ = 2 * JP;
  constexpr int F = 5;                     // 80 channels per wave side = 5 MFMA blocks
  static_assert((STAGES - 2) * NJ < 64, "vmcnt range");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // STAGES * 2 * PART

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave & 1, wn = wave >> 1;
  const int Mtot = a.N * a.OH * a.OW;

  // workgroup -> (split, tap, co tile, ci tile); XCD aware as in the forward kernel
  int t = blockIdx.x;
  const int total = gridDim.x;
  if ((total & 7) == 0) t = (blockIdx.x & 7) * (total >> 3) + (blockIdx.x >> 3);
  const int ci_t = t % L.ci_tiles; t /= L.ci_tiles;
  const int co_t = t % L.co_tiles; t /= L.co_tiles;
  const int tapi = t % a.ntaps;
  const int split = t / a.ntaps;
  const int co0 = co_t * BC, ci0 = ci_t * BC;
  const int tp = a.tap[tapi];
  const int dh = (tp & 0xff) - 8, dw = ((tp >> 8) & 0xff) - 8;
  const int total_chunks = (Mtot + BKP - 1) / BKP;
  const int chunk_lo = split * L.chunks_per_split;
  const int chunk_hi = min(total_chunks, chunk_lo + L.chunks_per_split);
  const int nchunks = chunk_hi - chunk_lo;
  if (nchunks <= 0) return;

  // ---- per-thread DMA sources ----
  int arow[JP];              // pixel row within the chunk, dy tile
  const char* asrc[JP];      // dy address of pixel row 0 of chunk 0 for this lane's unit
  int bm[JP], bn_[JP], boh[JP], biw[JP];   // x tile: running pixel index, image, output row, input column (or -1)
  int bcol[JP];              // byte offset of this lane's channel unit within a pixel
#pragma unroll
  for (int j = 0; j < JP; ++j) {
    const int P = 64 * (4 * j + wave) + lane;
    const int r = P / UPR, up = P % UPR;
    const int u = 2 * ((up >> 1) ^ ((r >> 2) & 1)) + (up & 1);
    arow[j] = r;
    asrc[j] = reinterpret_cast<const char*>(a.dy) + ((size_t)r * a.Co + co0 + u * 8) * 2;
    const int m = chunk_lo * BKP + r;
    bm[j] = m;
    const int mm = m < Mtot ? m : 0;
    const int ow = mm % a.OW, t2 = mm / a.OW;
    boh[j] = t2 % a.OH;
    bn_[j] = t2 / a.OH;
    const int iw = ow * a.stride + dw;
    biw[j] = ((unsigned)iw < (unsigned)a.Wi) ? iw : -1;
    bcol[j] = (ci0 + u * 8) * 2;
  }
  const char* zero = reinterpret_cast<const char*>(g_zero_word);
  const int d_oh = BKP / a.OW;   // the launcher guarantees OW divides 64

  auto issue = [&](int c) {   // c = chunk index relative to chunk_lo
    unsigned char* stage = smem + (size_t)(c % STAGES) * (2 * PART);
    const size_t abase = (size_t)(chunk_lo + c) * BKP * a.Co * 2;
#pragma unroll
    for (int j = 0; j < JP; ++j) {
      const bool ok = (chunk_lo + c) * BKP + arow[j] < Mtot;
      dma16(ok ? asrc[j] + abase : zero, stage + (size_t)(64 * (4 * j + wave)) * 16);
    }
#pragma unroll
    for (int j = 0; j < JP; ++j) {
      const int ih = boh[j] * a.stride + dh;
      const bool ok = bm[j] < Mtot && biw[j] >= 0 && (unsigned)ih < (unsigned)a.Hi;
      const char* g = reinterpret_cast<const char*>(a.x) +
                      (((size_t)bn_[j] * a.Hi + ih) * a.Wi + biw[j]) * (size_t)a.Cx * 2 + bcol[j];
      dma16(ok ? g : zero, stage + PART + (size_t)(64 * (4 * j + wave)) * 16);
      // advance this row to the next chunk
      bm[j] += BKP;
      boh[j] += d_oh;
      while (boh[j] >= a.OH) {
        boh[j] -= a.OH;
        bn_[j] += 1;
      }
    }
  };

  f32x4 acc[F][F];
#pragma unroll
  for (int i = 0; i < F; ++i)
#pragma unroll
    for (int j = 0; j < F; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // this lane's read address inside a tile for MFMA block f and k-step ks:
  //   pixel r = 32*ks + 4*(lane>>4) + ((lane&15)>>2), channels cbase + 16*f + 4*(lane&3)
  const int g = lane >> 4, i16 = lane & 15;
  const int r_in_step = 4 * g + (i16 >> 2);
  const unsigned lds0 = (unsigned)(uintptr_t)((__attribute__((address_space(3))) unsigned char*)smem);

#pragma unroll
  for (int p = 0; p < STAGES - 1; ++p)
    if (p < nchunks) issue(p);

  for (int c = 0; c < nchunks; ++c) {
    if (c + STAGES - 2 < nchunks) wait_vmcnt<(STAGES - 2) * NJ>(); else wait_vmcnt<0>();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (c + STAGES - 1 < nchunks) issue(c + STAGES - 1);
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const int r = 32 * ks + r_in_step;
      const int swz = (r >> 2) & 1;   // the same for r and r + 16
      v4s16 alo[F], ahi[F], blo[F], bhi[F];
#pragma unroll
      for (int f = 0; f < F; ++f) {
        const int slot_a = ((wm * 80 + f * 16) >> 4) ^ swz, slot_b = ((wn * 80 + f * 16) >> 4) ^ swz;
        const unsigned base = lds0 + (unsigned)(c % STAGES) * (2 * PART) + r * ROWB + (i16 & 3) * 8;
        lds_read_tr8(base + slot_a * 32, alo[f], ahi[f]);
        lds_read_tr8(base + PART + slot_b * 32, blo[f], bhi[f]);
      }
      // all of them have landed; tied to the registers so that no MFMA moves above the wait
      static_assert(F == 5, "operand list");
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(alo[0]), "+v"(ahi[0]), "+v"(alo[1]), "+v"(ahi[1]), "+v"(alo[2]), "+v"(ahi[2]), "+v"(alo[3]), "+v"(ahi[3]),
                     "+v"(alo[4]), "+v"(ahi[4]), "+v"(blo[0]), "+v"(bhi[0]), "+v"(blo[1]), "+v"(bhi[1]), "+v"(blo[2]), "+v"(bhi[2]),
                     "+v"(blo[3]), "+v"(bhi[3]), "+v"(blo[4]), "+v"(bhi[4]));
      bf16x8 fa[F], fb[F];
#pragma unroll
      for (int f = 0; f < F; ++f) {
        fa[f] = join_tr8(alo[f], ahi[f]);
        fb[f] = join_tr8(blo[f], bhi[f]);
      }
#pragma unroll
      for (int i = 0; i < F; ++i)
#pragma unroll
        for (int j = 0; j < F; ++j) acc[i][j] = mfma16(fa[i], fb[j], acc[i][j]);
    }
  }

  // D[co][ci]: lane holds co = 4*(lane>>4)+v, ci = lane&15 of each 16x16 block
#pragma unroll
  for (int i = 0; i < F; ++i)
#pragma unroll
    for (int j = 0; j < F; ++j) {
      const int ci = ci0 + wn * 80 + j * 16 + (lane & 15);
      if (ci >= a.Ci) continue;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int co = co0 + wm * 80 + i * 16 + 4 * (lane >> 4) + v;
        if (co >= a.Co) continue;
        const size_t o = ((size_t)co * a.ntaps + tapi) * a.Ci + ci;
        if (L.partial) L.partial[(size_t)split * L.split_stride + o] = acc[i][j][v];
        else atomicAdd(a.dw + o, acc[i][j][v]);
      }
    }
}

// dw (+)= sum over splits of the partial arrays
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(float4* __restrict__ dw, const float4* __restrict__ partial,
                                                           size_t n4, int splits, size_t stride4, int overwrite) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) {
    float4 s = overwrite ? make_float4(0.f, 0.f, 0.f, 0.f) : dw[i];
    for (int k = 0; k < splits; ++k) {
      const float4 p = partial[(size_t)k * stride4 + i];
      s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
    }
    dw[i] = s;
  }
}

// The same for many parts of a small array: 16 lanes share a float4 of dw, lane q adds the parts q, q + 16, ... and the
// sixteen partial sums are added through LDS in lane order (a fixed order).
__global__ __launch_bounds__(256) void wgrad_reduce_lanes_kernel(float4* __restrict__ dw, const float4* __restrict__ partial,
                                                                 size_t n4, int parts, size_t stride4, int overwrite) {
  __shared__ float4 sh[16][16];
  const int e = threadIdx.x & 15, q = threadIdx.x >> 4;
  const size_t i = (size_t)blockIdx.x * 16 + e;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (i < n4) {
#pragma unroll 4
    for (int k = q; k < parts; k += 16) {
      const float4 p = partial[(size_t)k * stride4 + i];
      s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
    }
  }
  sh[q][e] = s;
  __syncthreads();
  if (q == 0 && i < n4) {
    float4 t = overwrite ? make_float4(0.f, 0.f, 0.f, 0.f) : dw[i];
#pragma unroll
    for (int j = 0; j < 16; ++j) { t.x += sh[j][e].x; t.y += sh[j][e].y; t.z += sh[j][e].z; t.w += sh[j][e].w; }
    dw[i] = t;
  }
}

hipError_t launch_wgrad_reduce(float* dw, const float* partial, size_t elems, int parts, int overwrite, hipStream_t s) {
  if (elems % 4 != 0 || parts < 1) return hipErrorInvalidValue;
  const size_t n4 = elems / 4;
  if (parts >= 32) {
    hipLaunchKernelGGL(wgrad_reduce_lanes_kernel, dim3((unsigned)((n4 + 15) / 16)), dim3(256), 0, s, reinterpret_cast<float4*>(dw),
                       reinterpret_cast<const float4*>(partial), n4, parts, n4, overwrite);
    return hipGetLastError();
  }
  size_t blocks = (n4 + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, s, reinterpret_cast<float4*>(dw),
                     reinterpret_cast<const float4*>(partial), n4, parts, n4, overwrite);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Weight gradient, 128 x 128 blocks on 32x32x16 MFMAs
// ------------------------------------------------------------------------------------------------
// A block is 128 output channels x 128 input channels of one tap.  (Letting every wave own the whole block and a part of
// the pixels would read each staged byte exactly once, but 256 accumulator registers leave the compiler no room and it
// spills: the waves split the block, see the kernel.)  Tiles are [pixel][128 channels] (256-byte rows) read with the
// transposing LDS load; the 32-byte slot of a row is XORed with 2 * (pixel & 3) so that the 4 pixels x 2 channel blocks
// a half wave reads in one pass cover all banks.  The x source of a row advances by a constant per chunk (the launcher
// requires Hi == stride * OH and OW | 64, or the flat form), and whether the row falls into the padding repeats with a
// short period over the chunks, so row validity is a per-lane bit mask indexed by chunk phase.  Operand reads run one
// half step ahead of the MFMAs, pinned with scheduling barriers as in the patch kernel.
struct Wgrad128Launch {
  int co_tiles, ci_tiles, splits, chunks_per_split;
  float* partial;        // when set: split s stores its block at partial + s * split_stride
  size_t split_stride;
  int period;            // row validity repeats every `period` chunks
  int d_oh;              // output rows per chunk (64 / OW), reduced mod OH
  int step_w;            // flat form (any width, unit stride): a chunk moves a pixel by 64 = d_oh rows and step_w columns
  long long a_step, b_step;   // bytes from one chunk to the next in dy and in x
};

// EIGHT waves, two per SIMD.  Four waves would issue the direct-to-LDS loads, the LDS reads
// and the MFMAs of a step one after the other and end up at the sum of the three times; LDS reads of four waves also
// top out near 80 bytes per clock against 150 with eight.  Here wave (wm, wn, wk) owns 64 output channels x 64 input
// channels (2 x 2 accumulator blocks: 64 registers, so two waves fit a SIMD easily) and two of the four 16-pixel
// steps of every 64-pixel chunk; while one wave of a SIMD waits for its reads or for the load queue, the other
// one's MFMAs run.  Fragments are double buffered (a step's reads are issued during the step before it, two per
// MFMA slot), next-chunk / still-loading are compile-time tags, load addresses are 32-bit offsets from two
// uniform pointers that advance with the chunk.
// FLAT: unit stride and any image width.  The input pixel of output pixel P under tap (dh, dw) is P + dh W + dw
// wherever it exists, so chunks need not start a row: the x pointer advances 64 pixels per chunk, and only the
// validity of a lane's pixel (does the tap stay inside the image?) depends on where the chunk starts; it repeats
// every OH OW / gcd(64, OH OW) chunks (49 for 7, 14, 28 and 56 pixels square), one bit of a 64-bit mask each.
template <int STAGES, bool FLAT>
__global__ __launch_bounds__(512) void conv_wgrad128w8_kernel(WgradArgs a, Wgrad128Launch L) {
  constexpr int BC = 128, BKP = 64, ROWB = BC * 2, PART = BKP * ROWB, STAGE = 2 * PART, NT = 512, NW = NT / 64;
  constexpr int JP = BKP * (BC / 8) / NT, NJ = 2 * JP;   // loads per thread, chunk and operand: 2
  constexpr int NM = 4;                                  // MFMAs per wave and 16-pixel step
  static_assert(STAGES >= 3 && (STAGES - 2) * NJ < 64, "pipeline depth / vmcnt range");
  static_assert(STAGES * STAGE >= NW * 2 * 4096, "room for the exchange of the partial blocks");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // STAGES * STAGE

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave & 1, wn = (wave >> 1) & 1, wk = wave >> 2;

  // Every block streams its channels of both operands over all its pixels, and what an XCD's blocks have in
  // common is fetched once into its L2.  So the blocks of an XCD are consecutive in the order (split, output
  // tile, input tile, tap): one pixel split (or two), few channel tiles, all their taps.  Dealt round robin,
  // every XCD would fetch both operands in full: 8 x 21 MB per launch.
  int t = xcd_consecutive(blockIdx.x, gridDim.x);
  const int tapi = t % a.ntaps; t /= a.ntaps;
  const int ci_t = t % L.ci_tiles; t /= L.ci_tiles;
  const int co_t = t % L.co_tiles;
  const int split = t / L.co_tiles;
  const int co0 = co_t * BC, ci0 = ci_t * BC;
  const int tp = a.tap[tapi];
  const int dh = (tp & 0xff) - 8, dw = ((tp >> 8) & 0xff) - 8;
  const int total_chunks = (a.N * a.OH * a.OW) / BKP;
  const int chunk_lo = split * L.chunks_per_split;
  const int n = min(total_chunks, chunk_lo + L.chunks_per_split) - chunk_lo;
  if (n <= 0) return;

  // ---- per-thread DMA sources: 32-bit byte offsets from two uniform pointers that advance with the chunk.  The x
  //      pointer starts one input row and one pixel before the chunk's first pixel, so that the offsets of taps
  //      that reach backwards stay non-negative (rows outside the image are never loaded) ----
  const int m0 = chunk_lo * BKP;
  const int oh0 = (m0 / a.OW) % a.OH, n0 = m0 / (a.OW * a.OH);    // not FLAT: BKP % OW == 0, m0 starts an output row
  const long long xrow0 = (long long)n0 * a.Hi + oh0 * a.stride;
  const int margin = (a.Wi + 1) * a.Cx * 2;
  const char* a_next = reinterpret_cast<const char*>(a.dy) + (size_t)m0 * a.Co * 2;
  const char* b_next = reinterpret_cast<const char*>(a.x) + (FLAT ? (long long)m0 : xrow0 * a.Wi) * a.Cx * 2 - margin;
  typedef typename std::conditional<FLAT, unsigned long long, unsigned>::type mask_t;
  unsigned aoff32[JP], boff32[JP];
  mask_t bmask[JP];
#pragma unroll
  for (int j = 0; j < JP; ++j) {
    const int P = 64 * (NW * j + wave) + lane;
    const int r = P >> 4, up = P & 15;
    const int u = 2 * ((up >> 1) ^ (2 * (r & 3))) + (up & 1);           // 256-byte rows: slot ^ 2 * (pixel & 3)
    aoff32[j] = (unsigned)((r * a.Co + co0 + u * 8) * 2);
    mask_t mask = 0;
    if constexpr (FLAT) {
      boff32[j] = (unsigned)(margin + ((r + dh * a.Wi + dw) * a.Cx + ci0 + u * 8) * 2);
      int ow = (m0 + r) % a.OW, oh = ((m0 + r) / a.OW) % a.OH;
      for (int q = 0; q < L.period; ++q) {
        if ((unsigned)(ow + dw) < (unsigned)a.Wi && (unsigned)(oh + dh) < (unsigned)a.Hi) mask |= (mask_t)1 << q;
        ow += L.step_w;
        const int carry = ow >= a.OW ? 1 : 0;
        ow -= carry * a.OW;
        oh += L.d_oh + carry;          // d_oh < OH: below 2 OH
        if (oh >= a.OH) oh -= a.OH;
      }
    } else {
      const int ow = r % a.OW, orow = r / a.OW;
      const int iw = ow * a.stride + dw;
      const bool colok = (unsigned)iw < (unsigned)a.Wi;
      boff32[j] = (unsigned)(margin + (((orow * a.stride + dh) * a.Wi + iw) * a.Cx + ci0 + u * 8) * 2);
      int ohq = (oh0 + orow) % a.OH;
      for (int q = 0; q < L.period; ++q) {
        if (colok && (unsigned)(ohq * a.stride + dh) < (unsigned)a.Hi) mask |= (mask_t)1 << q;
        ohq += L.d_oh;
        if (ohq >= a.OH) ohq -= a.OH;
      }
    }
    bmask[j] = mask;
  }
  const uint64_t zero_addr = (uint64_t)g_zero_word;
  uint32_t zero_lo = (uint32_t)zero_addr, zero_hi = (uint32_t)(zero_addr >> 32);
  asm volatile("" : "+s"(zero_lo), "+s"(zero_hi));   // kept in two registers (rebuilt from the program counter otherwise)

  const unsigned lds0 = (unsigned)(uintptr_t)((__attribute__((address_space(3))) unsigned char*)smem);
  mask_t phase_bit = 1;                    // 1 << ((chunk being issued) mod period)
  const mask_t last_phase_bit = (mask_t)1 << (L.period - 1);
  unsigned issue_stage = 0;                // LDS byte offset of the stage being filled
  auto issue_one = [&](int d) {
    unsigned char* stage = smem + issue_stage;
    if (d < JP) {
      dma16(a_next + aoff32[d], stage + (64 * (NW * d + wave)) * 16);
    } else {
      const int j = d - JP;
      const bool ok = (bmask[j] & phase_bit) != 0;
      const uint64_t pa = (uint64_t)(b_next + boff32[j]);
      const uint32_t lo = ok ? (uint32_t)pa : zero_lo, hi = ok ? (uint32_t)(pa >> 32) : zero_hi;
      dma16((const char*)(((uint64_t)hi << 32) | lo), stage + PART + (64 * (NW * j + wave)) * 16);
    }
  };
  auto issue_done = [&]() {
    phase_bit = phase_bit == last_phase_bit ? (mask_t)1 : phase_bit << 1;
    issue_stage = issue_stage == (STAGES - 1) * STAGE ? 0u : issue_stage + STAGE;
    a_next += L.a_step;
    b_next += L.b_step;
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // ---- operand reads: lane group g = lane >> 4 takes channels 16*(g&1).. of a 32-channel block and pixels
  //      8*(g>>1) .. +7 of a 16-pixel step (two transposing reads of 4 pixels each); this wave's steps are
  //      2 wk and 2 wk + 1 of the chunk ----
  unsigned foff[4];   // 0, 1: dy blocks 2 wm, 2 wm + 1;  2, 3: x blocks 2 wn, 2 wn + 1
  {
    const int g = lane >> 4, i16 = lane & 15;
    const int prow = 32 * wk + 8 * (g >> 1) + (i16 >> 2);
    const int x = 2 * ((i16 >> 2) & 3);
#pragma unroll
    for (int f = 0; f < 2; ++f) {
      foff[f] = lds0 + prow * ROWB + (i16 & 3) * 8 + (((2 * (2 * wm + f) + (g & 1)) ^ x) * 32);
      foff[2 + f] = lds0 + PART + prow * ROWB + (i16 & 3) * 8 + (((2 * (2 * wn + f) + (g & 1)) ^ x) * 32);
    }
  }
  // fragment index by position in read order = the order the MFMAs (K = 2 i + j) first need them: A0 B0 B1 A1
  v4s16 flo[2][4], fhi[2][4];   // [set][fragment]: fragment 0, 1 = dy; 2, 3 = x
  auto read_pos = [&](auto set_tag, auto pos_tag, unsigned stage_off, auto ks_tag) {
    constexpr int S = decltype(set_tag)::value, POS = decltype(pos_tag)::value, KS = decltype(ks_tag)::value;
    constexpr int F = POS == 0 ? 0 : (POS == 1 ? 2 : (POS == 2 ? 3 : 1));
    const unsigned addr = foff[F] + stage_off;
    v4s16 &lo = flo[S][F], &hi = fhi[S][F];
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(addr), "i"((KS * 16) * ROWB));
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(addr), "i"((KS * 16 + 4) * ROWB));
  };
  auto wait_frag = [&](auto set_tag, auto f_tag, auto n_tag) {   // fragment F has landed when at most N reads are outstanding
    constexpr int S = decltype(set_tag)::value, F = decltype(f_tag)::value, N = decltype(n_tag)::value;
    static_assert(N >= 0 && N <= 15, "lgkmcnt range");
    v4s16 &lo = flo[S][F], &hi = fhi[S][F];
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(lo), "+v"(hi) : "n"(N));
  };
  auto frag = [&](auto set_tag, int f) {
    constexpr int S = decltype(set_tag)::value;
    typedef short v8s16 __attribute__((ext_vector_type(8)));
    const v8s16 both = __builtin_shufflevector(flo[S][f], fhi[S][f], 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>;
  using I3 = std::integral_constant<int, 3>;

  // prologue: chunks 0 .. STAGES-2 in flight, chunk 0 visible, the fragments of its first step read
#pragma unroll
  for (int p = 0; p < STAGES - 1; ++p)
    if (p < n) {
#pragma unroll
      for (int d = 0; d < NJ; ++d) issue_one(d);
      issue_done();
    }
  static_for<STAGES - 1>([&](auto q_tag) {
    constexpr int Q = decltype(q_tag)::value;   // chunks issued after chunk 0
    if ((n < STAGES - 1 ? n : STAGES - 1) - 1 == Q) wait_vmcnt<Q * NJ>();
  });
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  static_for<4>([&](auto pos) { read_pos(I0{}, pos, 0u, I0{}); });

  // One 16-pixel step = 4 (MFMA, piece) slots on fragment set KS.  Pieces: after MFMA k the two reads of fragment
  // position k of the following step into the other set (`more`: there is a following step); after slot 1 of a
  // chunk's first step the barrier that makes the next chunk visible (`bar`); one load of chunk c+STAGES-1 in
  // slots 2, 3 of the first step and 0, 1 of the second (`issue`).
  unsigned rd_stage = 0;   // LDS byte offset of the stage of chunk c
  auto step = [&](auto ks_tag, auto more_tag, auto bar_tag, auto issue_tag, unsigned next_stage) {
    constexpr int KS = decltype(ks_tag)::value;
    constexpr bool more = decltype(more_tag)::value, bar = decltype(bar_tag)::value, issue = decltype(issue_tag)::value;
    using set = std::integral_constant<int, KS>;
    using other = std::integral_constant<int, 1 - KS>;
    const unsigned rd = KS == 0 ? rd_stage : next_stage;   // where the following step's operands are
    static_for<NM>([&](auto k) {
      constexpr int K = decltype(k)::value;
      // this step's reads went out in the order A0 B0 B1 A1, two each; K newer pairs follow them by now
      if constexpr (K == 0) {
        wait_frag(set{}, I0{}, std::integral_constant<int, 6>{});
        wait_frag(set{}, I2{}, std::integral_constant<int, 4>{});
      } else if constexpr (K == 1) {
        wait_frag(set{}, I3{}, std::integral_constant<int, more ? 4 : 2>{});
      } else if constexpr (K == 2) {
        wait_frag(set{}, I1{}, std::integral_constant<int, more ? 4 : 0>{});
      }
      acc[K >> 1][K & 1] = mfma32(frag(set{}, K >> 1), frag(set{}, 2 + (K & 1)), acc[K >> 1][K & 1]);
      if constexpr (more) read_pos(other{}, k, rd, other{});
      if constexpr (bar && K == 1) {
        if constexpr (issue) wait_vmcnt<(STAGES - 3) * NJ>(); else wait_vmcnt<0>();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
      }
      if constexpr (issue) {
        if constexpr (KS == 0 && K >= 2) issue_one(K - 2);
        if constexpr (KS == 1 && K < 2) issue_one(K + 2);
      }
      __builtin_amdgcn_sched_barrier(0);
    });
  };
  auto chunk = [&](auto next_tag, auto issue_tag) {
    const unsigned next_stage = rd_stage == (STAGES - 1) * STAGE ? 0u : rd_stage + STAGE;
    step(I0{}, std::true_type{}, next_tag, issue_tag, next_stage);
    step(I1{}, next_tag, std::false_type{}, issue_tag, next_stage);
    if constexpr (decltype(issue_tag)::value) issue_done();
    rd_stage = next_stage;
  };
  {
    using yes = std::true_type;
    using no = std::false_type;
    int c = 0;
    for (; c + STAGES - 1 < n; ++c) chunk(yes{}, yes{});
    for (; c + 1 < n; ++c) chunk(yes{}, no{});
    if (c < n) chunk(no{}, no{});
  }

  // ---- add the two pixel halves: wave (wm, wn, wk) keeps block row wk of its two and receives its partner's ----
  wait_vmcnt<0>();
  __syncthreads();
  f32x4* mine = reinterpret_cast<f32x4*>(smem) + (size_t)wave * 512;
  const f32x4* theirs = reinterpret_cast<const f32x4*>(smem) + (size_t)(wave ^ 4) * 512;
  f32x16 keep[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const f32x16 give = wk == 0 ? acc[1][j] : acc[0][j];
    keep[j] = wk == 0 ? acc[0][j] : acc[1][j];
#pragma unroll
    for (int g = 0; g < 4; ++g)
      mine[(j * 4 + g) * 64 + lane] = f32x4{give[4 * g], give[4 * g + 1], give[4 * g + 2], give[4 * g + 3]};
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const f32x4 p = theirs[(j * 4 + g) * 64 + lane];
      keep[j][4 * g] += p[0]; keep[j][4 * g + 1] += p[1]; keep[j][4 * g + 2] += p[2]; keep[j][4 * g + 3] += p[3];
    }
  // D block: lane holds column ci = 32 j + (lane & 31), rows co = 8 (v >> 2) + 4 (lane >> 5) + (v & 3) of the block row
  float* dst = L.partial ? L.partial + (size_t)split * L.split_stride : a.dw;
  const int mode = (L.partial || (L.splits == 1 && a.overwrite)) ? 0 : (L.splits > 1 ? 1 : 2);
  const int ntaps = a.ntaps, Ci = a.Ci;
  const int co_base = co0 + 64 * wm + 32 * wk + 4 * (lane >> 5);
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int ci = ci0 + 64 * wn + 32 * j + (lane & 31);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int co = co_base + 8 * (v >> 2) + (v & 3);
      float* o = dst + ((size_t)co * ntaps + tapi) * Ci + ci;
      const float val = keep[j][v];
      if (mode == 0) *o = val;
      else if (mode == 1) atomicAdd(o, val);
      else *o += val;
    }
  }
}

// Chunks per repetition of the flat form's validity pattern (0: the flat form does not apply): unit stride, any width.
static int wgrad128_flat_period(const WgradArgs& a) {
  if (a.stride != 1 || a.Hi != a.OH || a.Wi != a.OW || a.OW < 1 || a.OH < 1) return 0;
  const long long img = (long long)a.OH * a.OW;
  long long g = img, h = 64;
  while (h) { const long long r = g % h; g = h; h = r; }
  const long long period = img / g;
  return period <= 64 ? (int)period : 0;
}

bool conv_wgrad128_applies(const WgradArgs& a) {
  if (a.Co % 128 != 0 || a.Ci % 128 != 0 || a.Cx != a.Ci || a.ntaps < 1) return false;
  if (a.OW < 1 || (a.N * a.OH * a.OW) % 64 != 0) return false;
  if (64 % a.OW != 0 || a.OH > 32) return wgrad128_flat_period(a) > 0;
  return a.Hi == a.stride * a.OH;
}

hipError_t launch_conv_wgrad128(const WgradArgs& a, hipStream_t s) {
  if (!conv_wgrad128_applies(a) || a.N * a.OH * a.OW <= 0) return hipErrorInvalidValue;
  constexpr int STAGES = 5;   // 5 x 32 KB: all of the LDS
  constexpr size_t lds = (size_t)STAGES * 2 * 64 * 256;
  static bool configured = false;
  if (!configured) {
    configured = true;   // (the two forms of the kernel are configured where they are launched)
  }
  const int total_chunks = a.N * a.OH * a.OW / 64;
  Wgrad128Launch L;
  L.co_tiles = a.Co / 128;
  L.ci_tiles = a.Ci / 128;
  const int tiles = L.co_tiles * L.ci_tiles * a.ntaps;
  const size_t elems = (size_t)a.Co * a.ntaps * a.Ci;
  // pixel splits only when the blocks alone leave most compute units idle, and only through scratch
  const int max_by_scratch = a.scratch ? (int)(a.scratch_bytes / (elems * 4)) : 0;
  int S = 1;
  if (tiles <= 128 && max_by_scratch >= 2) {
    S = 256 / tiles;
    if (S > max_by_scratch) S = max_by_scratch;
    if (S > total_chunks / 8) S = total_chunks / 8;
    if (S < 1) S = 1;
  }
  L.chunks_per_split = (total_chunks + S - 1) / S;
  L.splits = (total_chunks + L.chunks_per_split - 1) / L.chunks_per_split;
  L.partial = L.splits > 1 ? a.scratch : nullptr;
  L.split_stride = elems;
  const int d_oh_full = 64 / a.OW;
  L.d_oh = d_oh_full % a.OH;
  int g = L.d_oh == 0 ? a.OH : L.d_oh, h = a.OH;   // gcd(d_oh, OH)
  while (h) { const int r = g % h; g = h; h = r; }
  L.period = a.OH / g;
  L.a_step = (long long)64 * a.Co * 2;
  L.b_step = (long long)d_oh_full * a.stride * a.Wi * a.Cx * 2;
  L.step_w = 0;
  const bool flat = 64 % a.OW != 0 || a.OH > 32;   // conv_wgrad128_applies has checked that the flat form applies then
  if (flat) {
    L.period = wgrad128_flat_period(a);
    if (L.period <= 0) return hipErrorInvalidValue;
    L.d_oh = d_oh_full % a.OH;
    L.step_w = 64 % a.OW;
    L.b_step = (long long)64 * a.Cx * 2;
    static bool configured_flat = false;
    if (!configured_flat) {
      hipError_t e8 = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_wgrad128w8_kernel<STAGES, true>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e8 != hipSuccess) return e8;
      configured_flat = true;
    }
    note_kernel("conv_wgrad128w8_kernel<5, flat>");
    hipLaunchKernelGGL((conv_wgrad128w8_kernel<STAGES, true>), dim3(tiles * L.splits), dim3(512), lds, s, a, L);
  } else {
    static bool configured8 = false;
    if (!configured8) {
      hipError_t e8 = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_wgrad128w8_kernel<STAGES, false>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e8 != hipSuccess) return e8;
      configured8 = true;
    }
    note_kernel("conv_wgrad128w8_kernel<5>");
    hipLaunchKernelGGL((conv_wgrad128w8_kernel<STAGES, false>), dim3(tiles * L.splits), dim3(512), lds, s, a, L);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !L.partial) return e;
  const size_t n4 = elems / 4;
  size_t blocks = (n4 + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, s, reinterpret_cast<float4*>(a.dw),
                     reinterpret_cast<const float4*>(a.scratch), n4, L.splits, elems / 4, a.overwrite);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Weight gradient, 320 x 64 blocks (the 320-channel layers: 320 = 5 * 64 has no 128-wide tiling)
// ------------------------------------------------------------------------------------------------
// The same scheme as the 128 x 128 kernel with another shape: the block is 320 output channels x 64 input
// channels of one tap, wave_m = wave & 1 owns 160 output channels (5 fragments of dy) and all 64 input channels
// (2 fragments of x): 10 accumulator blocks, 7 fragment reads per 10 MFMAs.  A 64-pixel chunk of such a block
// would be 48 KB, too few stages for the LDS, so a chunk is 32 pixels (24 KB per stage) and each wave (wk =
// wave >> 1) takes ONE 16-pixel step of it; the fragments of chunk c+1 are read during the MFMAs of chunk c.
// Rows are 640 bytes (dy) and 128 bytes (x): the row pitch is 4 mod 8 slots of 32 bytes, so pixels p and p+2
// start in the same banks and the slot is XORed with 2 * ((pixel >> 1) & 1).
template <int STAGES>
__global__ __launch_bounds__(256) void conv_wgrad_tall_kernel(WgradArgs a, Wgrad128Launch L) {
  constexpr int TA = 320, TB = 64, BKP = 32;
  constexpr int ROWA = TA * 2, ROWBB = TB * 2, PARTA = BKP * ROWA, PARTB = BKP * ROWBB, STAGE = PARTA + PARTB;
  constexpr int UA = TA / 8, UB = TB / 8;                  // 16-byte units per row
  constexpr int JA = BKP * UA / 256, JB = BKP * UB / 256, NJ = JA + JB;
  constexpr int FA = 5, FB = 2, NF = FA + FB, NM = FA * FB;
  static_assert(BKP * UA % 256 == 0 && BKP * UB % 256 == 0, "whole load instructions");
  static_assert(STAGES >= 4 && (STAGES - 2) * NJ < 64, "pipeline depth / vmcnt range");
  static_assert(STAGES * STAGE >= 4 * FA * 16 * 256, "room for the exchange of the partial blocks");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // STAGES * STAGE

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave_m = wave & 1, wk = wave >> 1;

  // blocks of one XCD: consecutive in the order (split, output tile, input tile, tap), see the 128 x 128 kernel
  int t = xcd_consecutive(blockIdx.x, gridDim.x);
  const int tapi = t % a.ntaps; t /= a.ntaps;
  const int ci_t = t % L.ci_tiles; t /= L.ci_tiles;
  const int co_t = t % L.co_tiles;
  const int split = t / L.co_tiles;
  const int co0 = co_t * TA, ci0 = ci_t * TB;
  const int tp = a.tap[tapi];
  const int dh = (tp & 0xff) - 8, dw = ((tp >> 8) & 0xff) - 8;
  const int total_chunks = (a.N * a.OH * a.OW) / BKP;
  const int chunk_lo = split * L.chunks_per_split;
  const int n = min(total_chunks, chunk_lo + L.chunks_per_split) - chunk_lo;
  if (n <= 0) return;

  // ---- per-thread DMA sources: instruction j of this wave covers the 64 units 64*(4j+wave) .. of a tile ----
  const char* aptr[JA];
  const char* bptr[JB];
  unsigned bmask[JB];
#pragma unroll
  for (int j = 0; j < JA; ++j) {
    const int P = 64 * (4 * j + wave) + lane;
    const int r = P / UA, up = P % UA;
    const int u = 2 * ((up >> 1) ^ (2 * ((r >> 1) & 1))) + (up & 1);
    aptr[j] = reinterpret_cast<const char*>(a.dy) + ((size_t)(chunk_lo * BKP + r) * a.Co + co0 + u * 8) * 2;
  }
#pragma unroll
  for (int j = 0; j < JB; ++j) {
    const int P = 64 * (4 * j + wave) + lane;
    const int r = P / UB, up = P % UB;
    const int u = 2 * ((up >> 1) ^ (2 * ((r >> 1) & 1))) + (up & 1);
    const int m = chunk_lo * BKP + r;
    const int ow = m % a.OW, t2 = m / a.OW, oh = t2 % a.OH, nimg = t2 / a.OH;
    const int iw = ow * a.stride + dw;
    const bool colok = (unsigned)iw < (unsigned)a.Wi;
    bptr[j] = reinterpret_cast<const char*>(a.x) +
              ((((long long)nimg * a.Hi + oh * a.stride + dh) * a.Wi + iw) * a.Cx + ci0 + u * 8) * 2;
    unsigned mask = 0;
    int ohq = oh;
    for (int q = 0; q < L.period; ++q) {
      if (colok && (unsigned)(ohq * a.stride + dh) < (unsigned)a.Hi) mask |= 1u << q;
      ohq += L.d_oh;
      if (ohq >= a.OH) ohq -= a.OH;
    }
    bmask[j] = mask;
  }
  const char* zero = reinterpret_cast<const char*>(g_zero_word);

  int issue_phase = 0;   // (chunk being issued) mod period
  auto issue_one = [&](int d, int c) {   // piece d of chunk c (relative to chunk_lo)
    unsigned char* stage = smem + (size_t)(c % STAGES) * STAGE;
    if (d < JA) {
      dma16(aptr[d] + (long long)c * L.a_step, stage + (64 * (4 * d + wave)) * 16);
    } else {
      const int j = d - JA;
      const bool ok = (bmask[j] >> issue_phase) & 1u;
      const uint64_t pa = (uint64_t)(bptr[j] + (long long)c * L.b_step), pz = (uint64_t)zero;
      const uint32_t lo = ok ? (uint32_t)pa : (uint32_t)pz, hi = ok ? (uint32_t)(pa >> 32) : (uint32_t)(pz >> 32);
      dma16((const char*)(((uint64_t)hi << 32) | lo), stage + PARTA + (64 * (4 * j + wave)) * 16);
    }
  };
  auto issue_done = [&]() { issue_phase = issue_phase + 1 == L.period ? 0 : issue_phase + 1; };

  f32x16 acc[FA][FB];
#pragma unroll
  for (int i = 0; i < FA; ++i)
#pragma unroll
    for (int j = 0; j < FB; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // ---- operand reads (see the 128 x 128 kernel): lane group g = lane >> 4 takes channels 16*(g&1).. of a
  //      32-channel block and pixels 8*(g>>1) .. +7 of this wave's 16 ----
  int aoff[FA], boff[FB];
  {
    const int g = lane >> 4, i16 = lane & 15;
    const int prow = 16 * wk + 8 * (g >> 1) + (i16 >> 2);
    const int x = 2 * (((i16 >> 2) >> 1) & 1);
#pragma unroll
    for (int f = 0; f < FA; ++f)
      aoff[f] = prow * ROWA + (i16 & 3) * 8 + (((2 * (FA * wave_m + f) + (g & 1)) ^ x) * 32);
#pragma unroll
    for (int f = 0; f < FB; ++f) boff[f] = PARTA + prow * ROWBB + (i16 & 3) * 8 + (((2 * f + (g & 1)) ^ x) * 32);
  }
  const unsigned lds0 = (unsigned)(uintptr_t)((__attribute__((address_space(3))) unsigned char*)smem);
  // fragment position in issue order = the order the MFMAs (K = FB i + j) need them: A0, B0, B1, A1, ..., A4
  v4s16 flo[2][NF], fhi[2][NF];   // index: F < FA: dy fragment F; else x fragment F - FA
  auto read_one = [&](auto set_tag, auto idx_tag, int c) {
    constexpr int S = decltype(set_tag)::value, IDX = decltype(idx_tag)::value;
    constexpr int POS = IDX >> 1, H = IDX & 1;
    constexpr int F = POS == 0 ? 0 : (POS <= FB ? FA + POS - 1 : POS - FB);
    int off;
    if constexpr (F < FA) off = aoff[F]; else off = boff[F - FA];
    const unsigned addr = lds0 + (unsigned)(c % STAGES) * STAGE + off;
    v4s16& v = H == 0 ? flo[S][F] : fhi[S][F];
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "i"(H * 4 * (F < FA ? ROWA : ROWBB)));
  };
  // Before MFMA K the fragments it is the first to use have landed when at most N reads are outstanding.
  auto before_mma = [&](auto set_tag, auto k_tag, auto n_tag) {
    constexpr int S = decltype(set_tag)::value, K = decltype(k_tag)::value, N = decltype(n_tag)::value;
    static_assert(N >= 0 && N <= 15, "lgkmcnt range");
    if constexpr (K == 0) {
      v4s16 &l0 = flo[S][0], &h0 = fhi[S][0], &l1 = flo[S][FA], &h1 = fhi[S][FA];
      asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(l0), "+v"(h0), "+v"(l1), "+v"(h1) : "n"(N));
    } else if constexpr (K < FB) {
      v4s16 &l0 = flo[S][FA + K], &h0 = fhi[S][FA + K];
      asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(l0), "+v"(h0) : "n"(N));
    } else if constexpr (K % FB == 0) {
      v4s16 &l0 = flo[S][K / FB], &h0 = fhi[S][K / FB];
      asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(l0), "+v"(h0) : "n"(N));
    }
  };
  auto needed = [](int K) constexpr { return K < FB ? K + 2 : FB + 1 + K / FB; };   // fragments used up to MFMA K
  auto frag = [&](auto set_tag, int f) {
    constexpr int S = decltype(set_tag)::value;
    typedef short v8s16 __attribute__((ext_vector_type(8)));
    const v8s16 both = __builtin_shufflevector(flo[S][f], fhi[S][f], 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
  };
  auto mma_one = [&](auto set_tag, auto k_tag) {
    constexpr int K = decltype(k_tag)::value;
    acc[K / FB][K % FB] = mfma32(frag(set_tag, K / FB), frag(set_tag, FA + K % FB), acc[K / FB][K % FB]);
  };

  auto settle = [&](auto set_tag) {   // every fragment of the set has landed
    constexpr int S = decltype(set_tag)::value;
    static_for<NF>([&](auto f_tag) {
      constexpr int F = decltype(f_tag)::value;
      v4s16 &l0 = flo[S][F], &h0 = fhi[S][F];
      asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(l0), "+v"(h0));
    });
  };

  // prologue: chunks 0 .. STAGES-2 in flight, chunk 0 visible, its fragments in set 0
#pragma unroll
  for (int p = 0; p < STAGES - 1; ++p)
    if (p < n) {
#pragma unroll
      for (int d = 0; d < NJ; ++d) issue_one(d, p);
      issue_done();
    }
  // chunk 0 has landed when at most the chunks issued after it are outstanding: min(n, STAGES-1) - 1 of them
  static_for<STAGES - 1>([&](auto q_tag) {
    constexpr int Q = decltype(q_tag)::value;   // chunks after chunk 0
    if ((n < STAGES - 1 ? n : STAGES - 1) - 1 == Q) wait_vmcnt<Q * NJ>();
  });
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  using set0 = std::integral_constant<int, 0>;
  using set1 = std::integral_constant<int, 1>;
  static_for<2 * NF>([&](auto idx) { read_one(set0{}, idx, 0); });

  // One chunk = NM (MFMA, piece) slots on one fragment set.  After slot 1: barrier c+1 (chunk c+1 visible,
  // everybody done reading chunk c-1).  Slots 2 .. NF+1: the reads of chunk c+1 into the other set, two per
  // slot.  Slots 2 ..: the NJ loads of chunk c+STAGES-1 into the stage of chunk c-1, one per slot.
  // Whether a next chunk exists and whether there is still something to load are compile-time tags (a taken
  // branch costs the single wave of a SIMD more than an MFMA lasts), and the fragment set alternates at compile
  // time too (the loops below take chunks in pairs): a run-time choice of the set makes the compiler shuffle
  // all accumulators between the two variants.
  static_assert(NF + 2 <= NM && NJ + 2 <= NM, "slots of a chunk");
  auto step = [&](auto set_tag, int c, auto next_tag, auto issue_tag) {
    constexpr int S = decltype(set_tag)::value;
    using other = std::integral_constant<int, 1 - S>;
    constexpr bool next = decltype(next_tag)::value, issue = decltype(issue_tag)::value;
    static_for<NM>([&](auto k) {
      constexpr int K = decltype(k)::value;
      if constexpr (K < FB || K % FB == 0) {
        // reads of the other set issued meanwhile: two per slot from slot 2 on (with no next chunk everything
        // is waited for at slot 2 instead)
        constexpr int NEWER = K > 2 ? 2 * ((K - 2) < NF ? (K - 2) : NF) : 0;
        before_mma(set_tag, k, std::integral_constant<int, 2 * (NF - needed(K)) + NEWER>{});
      }
      mma_one(set_tag, k);
      if constexpr (next) {
        if constexpr (K == 1) {
          // chunk c+1 has landed when only the chunks issued after it are outstanding; once nothing is issued
          // any more, simply wait for everything
          if constexpr (issue) wait_vmcnt<(STAGES - 3) * NJ>(); else wait_vmcnt<0>();
          asm volatile("" ::: "memory");
          __builtin_amdgcn_s_barrier();
          asm volatile("" ::: "memory");
        }
        if constexpr (K >= 2 && K - 2 < NF) {
          read_one(other{}, std::integral_constant<int, 2 * (K - 2)>{}, c + 1);
          read_one(other{}, std::integral_constant<int, 2 * (K - 2) + 1>{}, c + 1);
        }
      } else {
        if constexpr (K == 2) settle(set_tag);
      }
      if constexpr (K >= 2 && K - 2 < NJ) {
        if constexpr (issue) issue_one(K - 2, c + STAGES - 1);
      }
      __builtin_amdgcn_sched_barrier(0);
    });
    if constexpr (issue) issue_done();
  };
  {
    using yes = std::true_type;
    using no = std::false_type;
    int c = 0;
    for (; c + STAGES < n; c += 2) {        // both chunks of the pair still load
      step(set0{}, c, yes{}, yes{});
      step(set1{}, c + 1, yes{}, yes{});
    }
    if (c + STAGES - 1 < n) {               // one more chunk to load: a mixed pair (n >= STAGES >= 4: c + 1 < n - 1)
      step(set0{}, c, yes{}, yes{});
      step(set1{}, c + 1, yes{}, no{});
      c += 2;
    }
    for (; c + 2 < n; c += 2) {
      step(set0{}, c, yes{}, no{});
      step(set1{}, c + 1, yes{}, no{});
    }
    if (c + 2 == n) {
      step(set0{}, c, yes{}, no{});
      step(set1{}, c + 1, no{}, no{});
    } else if (c < n) {
      step(set0{}, c, no{}, no{});
    }
  }

  // ---- add the two pixel halves: wave (wave_m, wk) keeps input-channel block wk of its two and receives its
  //      partner's sums for it ----
  wait_vmcnt<0>();
  __syncthreads();
  f32x4* mine = reinterpret_cast<f32x4*>(smem) + (size_t)wave * (FA * 4 * 64);
  const f32x4* theirs = reinterpret_cast<const f32x4*>(smem) + (size_t)(wave ^ 2) * (FA * 4 * 64);
  f32x16 keep[FA];
#pragma unroll
  for (int i = 0; i < FA; ++i) {
    const f32x16 give = wk == 0 ? acc[i][1] : acc[i][0];
    keep[i] = wk == 0 ? acc[i][0] : acc[i][1];
#pragma unroll
    for (int g = 0; g < 4; ++g)
      mine[(i * 4 + g) * 64 + lane] = f32x4{give[4 * g], give[4 * g + 1], give[4 * g + 2], give[4 * g + 3]};
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < FA; ++i)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const f32x4 p = theirs[(i * 4 + g) * 64 + lane];
      keep[i][4 * g] += p[0]; keep[i][4 * g + 1] += p[1]; keep[i][4 * g + 2] += p[2]; keep[i][4 * g + 3] += p[3];
    }
  // D block i: lane holds column ci = 32 wk + (lane & 31), rows co = 32 i + 8 (v >> 2) + 4 (lane >> 5) + (v & 3)
  float* dst = L.partial ? L.partial + (size_t)split * L.split_stride : a.dw;
  const int mode = (L.partial || (L.splits == 1 && a.overwrite)) ? 0 : (L.splits > 1 ? 1 : 2);
  const int ntaps = a.ntaps, Ci = a.Ci;
  const int ci = ci0 + 32 * wk + (lane & 31);
  const int co_base = co0 + 160 * wave_m + 4 * (lane >> 5);
#pragma unroll
  for (int i = 0; i < FA; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int co = co_base + 32 * i + 8 * (v >> 2) + (v & 3);
      float* o = dst + ((size_t)co * ntaps + tapi) * Ci + ci;
      const float val = keep[i][v];
      if (mode == 0) *o = val;
      else if (mode == 1) atomicAdd(o, val);
      else *o += val;
    }
}

bool conv_wgrad_tall_applies(const WgradArgs& a) {
  if (a.Co % 320 != 0 || a.Ci % 64 != 0 || a.Cx != a.Ci || a.ntaps < 1) return false;
  if (a.OW < 1 || 32 % a.OW != 0 || (a.N * a.OH * a.OW) % 32 != 0 || a.OH > 32) return false;
  return a.Hi == a.stride * a.OH;
}

hipError_t launch_conv_wgrad_tall(const WgradArgs& a, hipStream_t s) {
  if (!conv_wgrad_tall_applies(a) || a.N * a.OH * a.OW <= 0) return hipErrorInvalidValue;
  constexpr int STAGES = 4;   // 4 x 24 KB (deeper rings measured slower)
  constexpr size_t lds = (size_t)STAGES * 32 * (640 + 128);
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_wgrad_tall_kernel<STAGES>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int total_chunks = a.N * a.OH * a.OW / 32;
  Wgrad128Launch L;
  L.co_tiles = a.Co / 320;
  L.ci_tiles = a.Ci / 64;
  const int tiles = L.co_tiles * L.ci_tiles * a.ntaps;
  const size_t elems = (size_t)a.Co * a.ntaps * a.Ci;
  const int max_by_scratch = a.scratch ? (int)(a.scratch_bytes / (elems * 4)) : 0;
  int S = 1;
  if (tiles <= 128 && max_by_scratch >= 2) {
    S = 256 / tiles;
    if (S > max_by_scratch) S = max_by_scratch;
    if (S > total_chunks / 16) S = total_chunks / 16;
    if (S < 1) S = 1;
  }
  L.chunks_per_split = (total_chunks + S - 1) / S;
  L.splits = (total_chunks + L.chunks_per_split - 1) / L.chunks_per_split;
  L.partial = L.splits > 1 ? a.scratch : nullptr;
  L.split_stride = elems;
  const int d_oh_full = 32 / a.OW;
  L.d_oh = d_oh_full % a.OH;
  int g = L.d_oh == 0 ? a.OH : L.d_oh, h = a.OH;   // gcd(d_oh, OH)
  while (h) { const int r = g % h; g = h; h = r; }
  L.period = a.OH / g;
  L.a_step = (long long)32 * a.Co * 2;
  L.b_step = (long long)d_oh_full * a.stride * a.Wi * a.Cx * 2;
  note_kernel("conv_wgrad_tall_kernel<4>");
  hipLaunchKernelGGL((conv_wgrad_tall_kernel<STAGES>), dim3(tiles * L.splits), dim3(256), lds, s, a, L);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !L.partial) return e;
  const size_t n4 = elems / 4;
  size_t blocks = (n4 + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, s, reinterpret_cast<float4*>(a.dw),
                     reinterpret_cast<const float4*>(a.scratch), n4, L.splits, elems / 4, a.overwrite);
  return hipGetLastError();
}

bool conv_wgrad_wide_applies(const WgradArgs& a) {
  return a.Co % 160 == 0 && a.Ci % 160 == 0 && a.Cx == a.Ci && a.OW >= 1 && 64 % a.OW == 0 && a.ntaps >= 1;
}

hipError_t launch_conv_wgrad_wide(const WgradArgs& a, hipStream_t s) {
  if (!conv_wgrad_wide_applies(a) || a.N * a.OH * a.OW <= 0) return hipErrorInvalidValue;
  constexpr int STAGES = 3;
  constexpr size_t lds = (size_t)STAGES * 2 * 64 * 320;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_wgrad_dma_kernel<STAGES>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int Mtot = a.N * a.OH * a.OW;
  WgradWideLaunch L;
  L.co_tiles = a.Co / 160;
  L.ci_tiles = a.Ci / 160;
  const int tiles = L.co_tiles * L.ci_tiles * a.ntaps;
  const int total_chunks = (Mtot + 63) / 64;
  const size_t elems = (size_t)a.Co * a.ntaps * a.Ci;
  // Number of pixel splits.  With scratch memory each split stores its partial block and a second kernel
  // adds them (cost: the partials are written and read once); without it the splits add with atomics, which
  // cost more the more splits there are.  Model: rounds of 256 workgroups x chunks per split x ~1 us, plus the
  // partial traffic at ~3 TB/s.
  const int max_by_scratch = a.scratch ? (int)(a.scratch_bytes / (elems * 4)) : 0;
  int best = 1;
  if (max_by_scratch >= 2) {
    double best_cost = 1e30;
    for (int S = 1; S <= 32 && S <= max_by_scratch && S <= total_chunks; ++S) {
      const int rounds = (tiles * S + 255) / 256, cps = (total_chunks + S - 1) / S;
      const double cost = (double)rounds * cps * 1.0 + (S > 1 ? (2.0 * S + 2.0) * elems * 4 / 3.0e6 : 0.0);
      if (cost < best_cost) { best_cost = cost; best = S; }
    }
  } else {
    best = 512 / tiles;   // atomics: about two rounds of workgroups
    if (best > total_chunks / 4) best = total_chunks / 4;
    if (best < 1) best = 1;
  }
  L.chunks_per_split = (total_chunks + best - 1) / best;
  L.splits = (total_chunks + L.chunks_per_split - 1) / L.chunks_per_split;
  const bool use_partial = max_by_scratch >= 2 && L.splits > 1;
  L.partial = use_partial ? a.scratch : nullptr;
  L.split_stride = elems;
  if (a.overwrite && !use_partial) {   // the atomics path only adds
    hipError_t e = launch_fill_f32(a.dw, elems, 0.f, s);
    if (e != hipSuccess) return e;
  }
  note_kernel("conv_wgrad_dma_kernel<3>");
  hipLaunchKernelGGL((conv_wgrad_dma_kernel<STAGES>), dim3(tiles * L.splits), dim3(256), lds, s, a, L);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !use_partial) return e;
  const size_t n4 = elems / 4;   // Ci % 160 == 0, so a multiple of 4
  size_t blocks = (n4 + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, s, reinterpret_cast<float4*>(a.dw),
                     reinterpret_cast<const float4*>(a.scratch), n4, L.splits, elems / 4, a.overwrite);
  return hipGetLastError();
}

}  // namespace fdg

// Convolutions of the narrow layers (16, 32 or 64 channels in and out, or the stem's 3 -- stored as 8 -- into 16 / 32 /
// 64; 3x3, unit stride): the ResNet-56 / -110 / -1202 stages and the first stage of ResNet-18.  Such a layer moves a few megabytes and does a few hundred
// megaflops per launch, so what a launch costs is the length of the dependent chain inside one workgroup, not the
// arithmetic: the generic kernel walks the contraction in 32-wide chunks, each chunk a round trip global memory ->
// registers -> LDS -> barrier, and a filter tap at a time re-reads the pixels nine times.  Here a workgroup
//   * lands the whole patch of its pixel tile (the tile's pixels with one image row and one pixel on either side,
//     contiguous in NHWC memory) in LDS with ONE burst of direct-to-LDS loads,
//   * holds the whole filter in registers as MFMA operand fragments (9 * Ci * Co bf16: 20, 72 or 144 registers per
//     lane), loaded straight from global memory while the patch is in flight,
//   * and then runs all MFMAs of its tile from LDS with no further barrier: a filter tap is a shift of the row
//     index inside the patch, a tap outside the image reads a row of zeros.
// Same arguments and output stage (store_tile: addend, gated addend, ReLU gate, fp32 / bf16 output, batch-norm sums
// of the forward or of the backward that follows) as the generic gather kernel, so forward and data gradient (flipped taps, transposed filter) both run through it.
#include "conv_common.h"
#include <stdio.h>
#include <stdlib.h>

namespace fdg {

namespace {

__device__ __attribute__((aligned(16))) uint32_t g_narrow_zero[4] = {0u, 0u, 0u, 0u};

__device__ __forceinline__ void narrow_dma16(const void* gsrc, void* lds_wave_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                   (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
}

// Workgroups are dealt to the 8 XCDs round robin (XCD = block index mod 8).  The inverse numbering: the blocks that
// run on one XCD get consecutive logical indices, so that neighbouring tiles -- which share their halo rows -- are
// fetched through the same L2.
__device__ __forceinline__ int narrow_xcd_consecutive(int block, int total) {
  const int base = total >> 3, rem = total & 7, x = block & 7, q = block >> 3;
  return x * base + (x < rem ? x : rem) + q;
}

// n / d for n < 2^30 and d <= 1024 with one 64-bit multiply: magic = ceil(2^40 / d) (exact: the error term
// n * (magic * d - 2^40) stays below 2^40)
__device__ __forceinline__ int narrow_div(int n, unsigned long long magic) {
  return (int)(((unsigned long long)(unsigned)n * magic) >> 40);
}
struct NarrowLaunch {
  int units;                        // 16-byte units of patch in LDS (a multiple of 256)
  unsigned long long magic_w, magic_h;
  int same_masks;                   // a workgroup's tiles are whole images apart: the tap masks of its first tile hold for all
};

// Output stage: what store_tile does for a same-grid unit-stride output (so the flat pixel index is the output
// index and no coordinates are needed), with every optional operand of all J pixel blocks requested before the
// first is used -- one memory round trip instead of one per operand and block.  The per-channel sums stay in the
// caller's registers (s1, s2) until narrow_flush_sums.
template <int J, int NB, int WN, int CO>
__device__ __forceinline__ void narrow_store(const GatherConvArgs& a, const f32x4 (&acc)[NB][J], int m_base, int wave, int lane,
                                             int Mtot, float (&s1)[NB][4], float (&s2)[NB][4]) {
  constexpr int WM = 4 / WN;
  const int wn = wave / WM;
  const int c0 = wn * NB * 16 + 4 * (lane >> 4);   // this lane's first channel of block 0
  size_t o[J];
  bool okp[J];
#pragma unroll
  for (int j = 0; j < J; ++j) {
    const int m = m_base + j * 16 + (lane & 15);
    okp[j] = m < Mtot;
    o[j] = (size_t)(okp[j] ? m : 0) * CO + c0;
  }
  float4 ad[J][NB];
  uint2 mk[J][NB], gt[J][NB], bx[J][NB];
  const bool want_bx = a.bnx && a.stats;
  if (a.addend) {
#pragma unroll
    for (int j = 0; j < J; ++j)
#pragma unroll
      for (int i = 0; i < NB; ++i) ad[j][i] = *reinterpret_cast<const float4*>(a.addend + o[j] + i * 16);
  }
  if (a.addend && a.addmask) {
#pragma unroll
    for (int j = 0; j < J; ++j)
#pragma unroll
      for (int i = 0; i < NB; ++i) mk[j][i] = *reinterpret_cast<const uint2*>(a.addmask + o[j] + i * 16);
  }
  if (a.gate) {
#pragma unroll
    for (int j = 0; j < J; ++j)
#pragma unroll
      for (int i = 0; i < NB; ++i) gt[j][i] = *reinterpret_cast<const uint2*>(a.gate + o[j] + i * 16);
  }
  if (want_bx) {
#pragma unroll
    for (int j = 0; j < J; ++j)
#pragma unroll
      for (int i = 0; i < NB; ++i) bx[j][i] = *reinterpret_cast<const uint2*>(a.bnx + o[j] + i * 16);
  }
#pragma unroll
  for (int j = 0; j < J; ++j)
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      f32x4 v = acc[i][j];
      if (a.addend) {
        float4 d = ad[j][i];
        if (a.addmask) {
          if (!(bf16_lo(mk[j][i].x) > 0.f)) d.x = 0.f;
          if (!(bf16_hi(mk[j][i].x) > 0.f)) d.y = 0.f;
          if (!(bf16_lo(mk[j][i].y) > 0.f)) d.z = 0.f;
          if (!(bf16_hi(mk[j][i].y) > 0.f)) d.w = 0.f;
        }
        v[0] += d.x; v[1] += d.y; v[2] += d.z; v[3] += d.w;
      }
      if (a.gate) {
        if (!(bf16_lo(gt[j][i].x) > 0.f)) v[0] = 0.f;
        if (!(bf16_hi(gt[j][i].x) > 0.f)) v[1] = 0.f;
        if (!(bf16_lo(gt[j][i].y) > 0.f)) v[2] = 0.f;
        if (!(bf16_hi(gt[j][i].y) > 0.f)) v[3] = 0.f;
      }
      const uint2 packed = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
      if (okp[j]) {
        if (a.out_f32) *reinterpret_cast<float4*>(a.out_f32 + o[j] + i * 16) = make_float4(v[0], v[1], v[2], v[3]);
        if (a.out_b16) *reinterpret_cast<uint2*>(a.out_b16 + o[j] + i * 16) = packed;
        if (a.stats) {
          const bool f = a.stats_f32 != 0;
          const float r0 = f ? v[0] : bf16_lo(packed.x), r1 = f ? v[1] : bf16_hi(packed.x);
          const float r2 = f ? v[2] : bf16_lo(packed.y), r3 = f ? v[3] : bf16_hi(packed.y);
          s1[i][0] += r0; s1[i][1] += r1; s1[i][2] += r2; s1[i][3] += r3;
          if (want_bx) {
            s2[i][0] += r0 * bf16_lo(bx[j][i].x); s2[i][1] += r1 * bf16_hi(bx[j][i].x);
            s2[i][2] += r2 * bf16_lo(bx[j][i].y); s2[i][3] += r3 * bf16_hi(bx[j][i].y);
          } else {
            s2[i][0] += r0 * r0; s2[i][1] += r1 * r1; s2[i][2] += r2 * r2; s2[i][3] += r3 * r3;
          }
        }
      }
    }
}

// The per-channel sums a workgroup gathered over its tiles: over the 16 lanes that hold the same 4 channels, then one
// slot per wave in LDS, then over the waves (a fixed order), then one exact add per channel and value into this workgroup's copy.
template <int NB, int WN, int CO>
__device__ __forceinline__ void narrow_flush_sums(const GatherConvArgs& a, const float (&s1)[NB][4], const float (&s2)[NB][4],
                                                  int wave, int lane) {
  constexpr int WM = 4 / WN;
  if (a.stats) {
    __shared__ float red[4][2][NB * 16];
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        float x1 = s1[i][v], x2 = s2[i][v];
#pragma unroll
        for (int off = 8; off > 0; off >>= 1) {
          x1 += __shfl_xor(x1, off, 16);
          x2 += __shfl_xor(x2, off, 16);
        }
        if ((lane & 15) == 0) {
          red[wave][0][i * 16 + 4 * (lane >> 4) + v] = x1;
          red[wave][1][i * 16 + 4 * (lane >> 4) + v] = x2;
        }
      }
    __syncthreads();
    for (int t = threadIdx.x; t < 2 * CO; t += 256) {
      const int which = t / CO, c = t % CO;
      const int owner = c / (NB * 16), cl = c % (NB * 16);   // the WM waves with wn == owner hold channel c
      float sum = 0.f;
#pragma unroll
      for (int w = 0; w < WM; ++w) sum += red[owner * WM + w][which][cl];
      stat_add(a.stats + (size_t)(blockIdx.x % kStatReplicas) * a.stats_rep_stride, CO, which, c, sum);
    }
  }
}

// CI input channels; a wave owns J blocks of 16 pixels and NB blocks of 16 output channels; WN waves side by side
// over the output channels (Co = 16 * NB * WN), 4 / WN over the pixels.  LDS: two patch buffers, each `units` 16-byte
// units of patch (a multiple of 256: whole load rounds of the workgroup) followed by 128 bytes of zeros.
template <int CI, int NB, int WN, int J>
__global__ __launch_bounds__(256) void conv_narrow_kernel(GatherConvArgs a, NarrowLaunch L) {
  constexpr int WM = 4 / WN, TP = 16 * J * WM, CO = 16 * NB * WN;
  constexpr int U = CI / 8, ROWB = CI * 2;          // 16-byte units and bytes of one pixel
  constexpr int S = (9 * CI + 31) / 32;             // 32-wide steps of the contraction (taps x channels)
  constexpr int SWZ_SHIFT = U == 2 ? 2 : (U == 4 ? 1 : 0);   // (U == 1, the 8-channel stem input: nothing to swizzle)   // unit index ^= (row >> SWZ_SHIFT) & (U - 1): b128 reads of 8 consecutive rows hit 8 bank groups
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave % WM, wn = wave / WM;
  const int W = a.Wi, H = a.Hi;
  const int Mtot = a.N * H * W;
  const int units = L.units;                         // patch row r holds pixel m0 - W - 1 + r
  const int ntiles = (Mtot + TP - 1) / TP;

  const unsigned bufs = (unsigned)units * 16u + 128u;   // bytes of one patch buffer: the patch, then 128 bytes of zeros
  if (tid < 16) reinterpret_cast<uint4*>(smem + (size_t)(tid >> 3) * bufs + (size_t)units * 16)[tid & 7] = make_uint4(0u, 0u, 0u, 0u);

  // ---- the filter: fragment (s, nb) = rows 16 nb .. +15 of this wave's channels, k = 32 s + 8 (lane >> 4) .. +7.
  //      Loaded once; a workgroup then takes tiles blockIdx.x, blockIdx.x + gridDim.x, ... (with 64 channels and
  //      many pixels the filter, 144 registers per lane, would otherwise be most of what the kernel reads) ----
  bf16x8 wf[S][NB];
  {
    const int g = lane >> 4;
#pragma unroll
    for (int s = 0; s < S; ++s)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const int co = (wn * NB + nb) * 16 + (lane & 15);
        const int k = 32 * s + 8 * g;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (k < 9 * CI && co < a.w_rows) v = *reinterpret_cast<const uint4*>(a.w + (size_t)co * a.Kw + k);
        wf[s][nb] = __builtin_bit_cast(bf16x8, v);
      }
  }
  float s1[NB][4], s2[NB][4];   // per-channel sums of this lane's outputs over all tiles (only with a.stats)
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int v = 0; v < 4; ++v) s1[i][v] = s2[i][v] = 0.f;

  constexpr int SA = CI == 64 ? 9 : S;
  const unsigned zero_addr = (unsigned)units * 16u;
  unsigned xaddr[J][SA];
  const int first_tile = narrow_xcd_consecutive(blockIdx.x, gridDim.x);
  // the patch of a tile: one burst of loads, lane i of a round lands at unit position base + i of buffer `buf`
  auto issue_patch = [&](int tile, int buf) {
    const int m0 = tile * TP;
    for (int base = wave * 64; base < units; base += 256) {
      const int pos = base + lane;
      const int r = pos / U, us = pos % U;           // stored position -> row and swizzled unit
      const int u = us ^ ((r >> SWZ_SHIFT) & (U - 1));
      int q = m0 - W - 1 + r;                        // rows that do not exist read some row that does: nothing valid refers to them
      q = q < 0 ? 0 : (q >= Mtot ? Mtot - 1 : q);
      narrow_dma16(a.in + (size_t)q * CI + u * 8, smem + (size_t)buf * bufs + (size_t)base * 16);
    }
  };
  // Two patch buffers: while the MFMAs of a tile run, the patch of the workgroup's next tile is already on its way.
  if (first_tile < ntiles) issue_patch(first_tile, 0);
  int cur = 0;
  for (int tile = first_tile; tile < ntiles; tile += gridDim.x) {
    const int m0 = tile * TP;

    // ---- LDS address of this lane's pixel fragment for every pixel block and step.  With 64 channels the two
    //      steps of a tap differ by unit bit 2 = address bit 6 (the zero area is 128 bytes for that), so one
    //      address serves both ----
    if (tile == first_tile || !L.same_masks) {
      const int g = lane >> 4;
#pragma unroll
      for (int j = 0; j < J; ++j) {
        const int pl = (wm * J + j) * 16 + (lane & 15);
        const int m = m0 + pl;
        const bool inside = m < Mtot;
        const int row = narrow_div(m, L.magic_w), ow = m - row * W;   // image row over the whole batch, column
        const int oh = row - narrow_div(row, L.magic_h) * H;
#pragma unroll
        for (int s = 0; s < SA; ++s) {
          // which tap and which unit of the pixel this lane's 8 k values are
          const int slot = CI == 8 ? 4 * s + g : (CI == 16 ? 2 * s + (g >> 1) : s);
          const int u = CI == 8 ? 0 : (CI == 16 ? (g & 1) : g);
          unsigned addr = zero_addr;
          if (slot < 9) {
            const int tp = a.tap[slot];
            const int dh = (tp & 0xff) - 8, dw = ((tp >> 8) & 0xff) - 8;
            const bool ok = inside && (unsigned)(oh + dh) < (unsigned)H && (unsigned)(ow + dw) < (unsigned)W;
            const int r = pl + W + 1 + dh * W + dw;
            if (ok) addr = (unsigned)(r * ROWB + ((u ^ ((r >> SWZ_SHIFT) & (U - 1))) << 4));
          }
          xaddr[j][s] = addr;
        }
      }
    }

    f32x4 acc[NB][J];
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
      for (int j = 0; j < J; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    __builtin_amdgcn_s_waitcnt(0);   // every load of this wave has landed (this tile's patch in LDS, the filter in registers)
    __syncthreads();                 // ... of every wave; and every wave is done reading the other buffer
    if (tile + (int)gridDim.x < ntiles) issue_patch(tile + gridDim.x, cur ^ 1);

    const unsigned char* patch = smem + (size_t)cur * bufs;
#pragma unroll
    for (int j = 0; j < J; ++j)
#pragma unroll
      for (int s = 0; s < S; ++s) {
        const unsigned addr = CI == 64 ? (xaddr[j][s >> 1] ^ ((s & 1) << 6)) : xaddr[j][s];
        const bf16x8 b = *reinterpret_cast<const bf16x8*>(patch + addr);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[nb][j] = mfma16(wf[s][nb], b, acc[nb][j]);
      }

    narrow_store<J, NB, WN, CO>(a, acc, m0 + wm * J * 16, wave, lane, Mtot, s1, s2);
    cur ^= 1;
  }
  narrow_flush_sums<NB, WN, CO>(a, s1, s2, wave, lane);
}

template <int CI, int NB, int WN, int J>
hipError_t run_narrow(const GatherConvArgs& a, hipStream_t s) {
  constexpr int WM = 4 / WN, TP = 16 * J * WM, U = CI / 8;
  const int Mtot = a.N * a.OH * a.OW;
  const int rows = TP + 2 * a.Wi + 2;
  const int units = (rows * U + 255) / 256 * 256;
  const size_t lds = 2 * ((size_t)units * 16 + 128);   // two patch buffers, each followed by its zero area
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_narrow_kernel<CI, NB, WN, J>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
    if (e != hipSuccess) return e;
    configured = true;
  }
  static char name[64];
  if (!name[0]) snprintf(name, sizeof(name), "conv_narrow_kernel<%d, %d, %d, %d>", CI, NB, WN, J);
  note_kernel(name);
  NarrowLaunch L;
  L.units = units;
  L.magic_w = ((1ull << 40) + a.Wi - 1) / a.Wi;
  L.magic_h = ((1ull << 40) + a.Hi - 1) / a.Hi;
  const int ntiles = (Mtot + TP - 1) / TP, grid = ntiles < 512 ? ntiles : 512;
  L.same_masks = ((long long)grid * TP) % ((long long)a.Hi * a.Wi) == 0 ? 1 : 0;
  hipLaunchKernelGGL((conv_narrow_kernel<CI, NB, WN, J>), dim3(grid), dim3(256), lds, s, a, L);
  return hipGetLastError();
}

// pixel blocks per wave: the largest of 4, 2, 1 that still leaves two workgroups per compute unit
template <int CI, int NB, int WN>
hipError_t run_narrow_j(const GatherConvArgs& a, hipStream_t s) {
  constexpr int WM = 4 / WN;
  const int Mtot = a.N * a.OH * a.OW;
  if (Mtot >= 512 * 64 * WM) return run_narrow<CI, NB, WN, 4>(a, s);
  if (Mtot >= 512 * 32 * WM) return run_narrow<CI, NB, WN, 2>(a, s);
  return run_narrow<CI, NB, WN, 1>(a, s);
}

// ------------------------------------------------------------------------------------------------
// The same with an input transform (GatherConvArgs::tr_mode): the batch-norm pass that would precede the
// convolution -- forward batch norm + ReLU, or the apply half of a batch-norm backward -- runs on the patch in LDS.
// ------------------------------------------------------------------------------------------------
// A narrow layer's launch is a chain of dependent round trips, and so is the batch-norm pass before it: fused, the
// pass costs one more trip through LDS instead of a launch.  The workgroup lands the RAW patches (p, and q in mode 2)
// beside the convolution's patch buffer, works out the per-channel coefficients from the exact sums while those
// loads are in flight (thread c < CI: channel c; a table in LDS), then every thread turns its units of the patch:
// y = act(A p + B q + C), rounded to bf16, written where the convolution reads it (same rows, same unit swizzle) and,
// for the pixels of the workgroup's own tile, to tr_out in global memory -- the tensor the backward (or the weight
// gradient) reads later.  Halo rows are transformed by every workgroup that needs them; the zero area stays zero, so
// padding is zero AFTER the transform, as it must be.  One tile per workgroup; the rest (filter in registers, MFMAs,
// output stage) is conv_narrow_kernel's.
// VAR: 0 forward batch norm + ReLU of p (bf16);  1 / 2 batch-norm backward of p (bf16 / fp32) with q;  3 forward batch
// norm of p (bf16) + fp32 residual r (tr_q) + ReLU.  The forward forms also write y in fp32 where tr_out_f32 is given.
template <int CI, int NB, int WN, int J, int VAR>
__global__ __launch_bounds__(256) void conv_narrow_tr_kernel(GatherConvArgs a, NarrowLaunch L) {
  constexpr bool PF32 = VAR == 2, WQ = VAR == 1 || VAR == 2, WR = VAR == 3;
  constexpr int WM = 4 / WN, TP = 16 * J * WM, CO = 16 * NB * WN;
  constexpr int U = CI / 8, ROWB = CI * 2;
  constexpr int S = (9 * CI + 31) / 32;
  constexpr int SWZ_SHIFT = U == 2 ? 2 : (U == 4 ? 1 : 0);
  constexpr int UP = PF32 ? 2 * U : U;                 // 16-byte units of one pixel of p
  static_assert(CI == 16 || CI == 32 || CI == 64, "real input channels");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave % WM, wn = wave / WM;
  const int W = a.Wi, H = a.Hi;
  const int Mtot = a.N * H * W;
  const int units = L.units;
  const int tile = narrow_xcd_consecutive(blockIdx.x, gridDim.x);
  const int m0 = tile * TP;

  unsigned char* patch = smem;                                   // units * 16, then 128 bytes of zeros
  float* coef = reinterpret_cast<float*>(smem + (size_t)units * 16 + 128);   // A[CI], B[CI], C[CI]
  unsigned char* rawp = reinterpret_cast<unsigned char*>(coef + 3 * CI);
  unsigned char* rawq = rawp + (size_t)units * (PF32 ? 32 : 16);
  if (tid < 8) reinterpret_cast<uint4*>(patch + (size_t)units * 16)[tid] = make_uint4(0u, 0u, 0u, 0u);

  // ---- the words of the sums, requested first and used last (below, after everything else has been issued and the
  //      fragment addresses worked out), so that this trip to memory runs beside the others.  Eight lanes per channel,
  //      one per copy of the sums; slot sl of a thread is (channel, copy) number tid + 256 sl ----
  constexpr int NS = (8 * CI + 255) / 256, NSUM = WQ ? 4 : 2;
  long long w_hi[NS][NSUM], w_lo[NS][NSUM];
  double w_big[NS][NSUM];
  float w_gamma[NS], w_beta[NS];
#pragma unroll
  for (int sl = 0; sl < NS; ++sl) {
    const int t = tid + 256 * sl, c = t >> 3, rp = t & 7, rep = a.tr_rep_stride;
    const bool has = t < 8 * CI && (rep > 0 || rp == 0);       // a single copy: only the first lane of the eight reads
    const bool first = t < 8 * CI && rp == 0;
    w_gamma[sl] = first ? a.tr_gamma[c] : 0.f;
    w_beta[sl] = (first && !WQ) ? a.tr_beta[c] : 0.f;
#pragma unroll
    for (int k = 0; k < NSUM; ++k) {
      const stat_t* q = (k < 2 ? a.tr_sums : a.tr_bsums) + (size_t)(k & 1) * CI + (has ? c : 0) + (size_t)(has && rep > 0 ? rp : 0) * rep;
      w_hi[sl][k] = has ? q[0] : 0;
      w_lo[sl][k] = has ? q[2 * (size_t)CI] : 0;
      w_big[sl][k] = has ? __builtin_bit_cast(double, q[4 * (size_t)CI]) : 0.0;
    }
  }

  // ---- the raw patches: row r holds pixel m0 - W - 1 + r (rows that do not exist read some row that does) ----
  {
    const int units_p = units * (PF32 ? 2 : 1);
    for (int base = wave * 64; base < units_p; base += 256) {
      const int pos = base + lane;
      const int r = pos / UP, up = pos % UP;
      int q = m0 - W - 1 + r;
      q = q < 0 ? 0 : (q >= Mtot ? Mtot - 1 : q);
      narrow_dma16(reinterpret_cast<const char*>(a.tr_p) + (size_t)q * (CI * (PF32 ? 4 : 2)) + up * 16, rawp + (size_t)base * 16);
    }
    if (WQ) {
      for (int base = wave * 64; base < units; base += 256) {
        const int pos = base + lane;
        const int r = pos / U, uq = pos % U;
        int q = m0 - W - 1 + r;
        q = q < 0 ? 0 : (q >= Mtot ? Mtot - 1 : q);
        narrow_dma16(reinterpret_cast<const char*>(a.tr_q) + (size_t)q * ROWB + uq * 16, rawq + (size_t)base * 16);
      }
    }
    if (WR) {   // the residual: fp32, two units per 8 channels
      for (int base = wave * 64; base < 2 * units; base += 256) {
        const int pos = base + lane;
        const int r = pos / (2 * U), ur = pos % (2 * U);
        int q = m0 - W - 1 + r;
        q = q < 0 ? 0 : (q >= Mtot ? Mtot - 1 : q);
        narrow_dma16(reinterpret_cast<const char*>(a.tr_q) + (size_t)q * (CI * 4) + ur * 16, rawq + (size_t)base * 16);
      }
    }
  }

  // ---- the filter (as conv_narrow_kernel) ----
  bf16x8 wf[S][NB];
  {
    const int g = lane >> 4;
#pragma unroll
    for (int s = 0; s < S; ++s)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const int co = (wn * NB + nb) * 16 + (lane & 15);
        const int k = 32 * s + 8 * g;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (k < 9 * CI && co < a.w_rows) v = *reinterpret_cast<const uint4*>(a.w + (size_t)co * a.Kw + k);
        wf[s][nb] = __builtin_bit_cast(bf16x8, v);
      }
  }

  // ---- LDS address of this lane's pixel fragment for every pixel block and step (as conv_narrow_kernel) ----
  constexpr int SA = CI == 64 ? 9 : S;
  const unsigned zero_addr = (unsigned)units * 16u;
  unsigned xaddr[J][SA];
  {
    const int g = lane >> 4;
#pragma unroll
    for (int j = 0; j < J; ++j) {
      const int pl = (wm * J + j) * 16 + (lane & 15);
      const int m = m0 + pl;
      const bool inside = m < Mtot;
      const int row = narrow_div(m, L.magic_w), ow = m - row * W;
      const int oh = row - narrow_div(row, L.magic_h) * H;
#pragma unroll
      for (int s = 0; s < SA; ++s) {
        const int slot = CI == 16 ? 2 * s + (g >> 1) : s;
        const int u = CI == 16 ? (g & 1) : g;
        unsigned addr = zero_addr;
        if (slot < 9) {
          const int tp = a.tap[slot];
          const int dh = (tp & 0xff) - 8, dw = ((tp >> 8) & 0xff) - 8;
          const bool ok = inside && (unsigned)(oh + dh) < (unsigned)H && (unsigned)(ow + dw) < (unsigned)W;
          const int r = pl + W + 1 + dh * W + dw;
          if (ok) addr = (unsigned)(r * ROWB + ((u ^ ((r >> SWZ_SHIFT) & (U - 1))) << 4));
        }
        xaddr[j][s] = addr;
      }
    }
  }

  // ---- per-channel coefficients from the exact sums (the same expressions as the batch-norm kernels): the integer
  //      words are added across the eight lanes of a channel, lane 0 of the eight works out the channel's constants ----
#pragma unroll
  for (int sl = 0; sl < NS; ++sl) {
    if (256 * sl + (tid & ~63) >= 8 * CI) break;               // whole waves take part in the shuffles (8 CI is a multiple of 64)
    const int t = tid + 256 * sl, c = t >> 3, rp = t & 7;
    double tot[NSUM];
#pragma unroll
    for (int k = 0; k < NSUM; ++k) {
      long long hi = w_hi[sl][k], lo = w_lo[sl][k];
      double big = w_big[sl][k];
#pragma unroll
      for (int off = 1; off < 8; off <<= 1) {
        hi += __shfl_xor(hi, off);
        lo += __shfl_xor(lo, off);
        big += __shfl_xor(big, off);
      }
      tot[k] = stat_value(hi, lo, __builtin_bit_cast(long long, big));
    }
    if (rp != 0) continue;
    const double s1 = tot[0], s2 = tot[1];
    const double invMd = 1.0 / (double)Mtot;
    const double md = s1 * invMd;
    const double var = fmax(s2 * invMd - md * md, 0.0);
    const float mean = (float)md, is = rsqrtf((float)var + a.tr_eps);
    const float g = w_gamma[sl] * is;
    float A = g, B = 0.f, C;
    if (!WQ) {
      C = w_beta[sl] - mean * g;
      if (blockIdx.x == 0 && a.tr_run_mean) {
        const float unbias = Mtot > 1 ? (float)Mtot / (float)(Mtot - 1) : 1.f, mom = a.tr_momentum;
        a.tr_run_mean[c] = (1.f - mom) * a.tr_run_mean[c] + mom * mean;
        a.tr_run_var[c] = (1.f - mom) * a.tr_run_var[c] + mom * (float)var * unbias;
      }
    } else {
      const double t1 = tot[WQ ? 2 : 0], t2 = tot[WQ ? 3 : 1];
      const float invM = (float)invMd;
      const float b1 = (float)t1;
      const float b2 = is * (float)(t2 - md * t1);     // sum g*xhat from sum g*x and sum g, the difference in double
      const float k1 = b1 * invM, k2 = b2 * invM;
      B = -g * k2 * is;
      C = -g * k1 + g * k2 * is * mean;
      if (blockIdx.x == 0) {
        a.tr_dbeta[c] = b1;
        a.tr_dgamma[c] = b2;
      }
    }
    coef[c] = A; coef[CI + c] = B; coef[2 * CI + c] = C;
  }

  __builtin_amdgcn_s_waitcnt(0);   // this wave's loads have landed (raw patches in LDS, filter in registers)
  __syncthreads();                 // ... and every wave's; the coefficient table is written

  // ---- the transform: conv-patch unit `pos` = row pos / U, stored unit pos % U holding channel unit u ----
  for (int pos = tid; pos < units; pos += 256) {
    const int r = pos / U, us = pos % U;
    const int u = us ^ ((r >> SWZ_SHIFT) & (U - 1));
    float pv[8], y[8];
    if (PF32) {
      const float4 lo = *reinterpret_cast<const float4*>(rawp + ((size_t)r * UP + 2 * u) * 16);
      const float4 hi = *reinterpret_cast<const float4*>(rawp + ((size_t)r * UP + 2 * u + 1) * 16);
      pv[0] = lo.x; pv[1] = lo.y; pv[2] = lo.z; pv[3] = lo.w; pv[4] = hi.x; pv[5] = hi.y; pv[6] = hi.z; pv[7] = hi.w;
    } else {
      const uint4 v = *reinterpret_cast<const uint4*>(rawp + ((size_t)r * UP + u) * 16);
      pv[0] = bf16_lo(v.x); pv[1] = bf16_hi(v.x); pv[2] = bf16_lo(v.y); pv[3] = bf16_hi(v.y);
      pv[4] = bf16_lo(v.z); pv[5] = bf16_hi(v.z); pv[6] = bf16_lo(v.w); pv[7] = bf16_hi(v.w);
    }
    const float4 A0 = *reinterpret_cast<const float4*>(coef + 8 * u), A1 = *reinterpret_cast<const float4*>(coef + 8 * u + 4);
    const float4 C0 = *reinterpret_cast<const float4*>(coef + 2 * CI + 8 * u), C1 = *reinterpret_cast<const float4*>(coef + 2 * CI + 8 * u + 4);
    const float Av[8] = {A0.x, A0.y, A0.z, A0.w, A1.x, A1.y, A1.z, A1.w};
    const float Cv[8] = {C0.x, C0.y, C0.z, C0.w, C1.x, C1.y, C1.z, C1.w};
    if (WQ) {
      const uint4 v = *reinterpret_cast<const uint4*>(rawq + ((size_t)r * U + u) * 16);
      const float qv[8] = {bf16_lo(v.x), bf16_hi(v.x), bf16_lo(v.y), bf16_hi(v.y), bf16_lo(v.z), bf16_hi(v.z), bf16_lo(v.w), bf16_hi(v.w)};
      const float4 B0 = *reinterpret_cast<const float4*>(coef + CI + 8 * u), B1 = *reinterpret_cast<const float4*>(coef + CI + 8 * u + 4);
      const float Bv[8] = {B0.x, B0.y, B0.z, B0.w, B1.x, B1.y, B1.z, B1.w};
#pragma unroll
      for (int i = 0; i < 8; ++i) y[i] = Av[i] * pv[i] + (Bv[i] * qv[i] + Cv[i]);
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) y[i] = pv[i] * Av[i] + Cv[i];
      if (WR) {
        const float4 r0 = *reinterpret_cast<const float4*>(rawq + ((size_t)r * 2 * U + 2 * u) * 16);
        const float4 r1 = *reinterpret_cast<const float4*>(rawq + ((size_t)r * 2 * U + 2 * u + 1) * 16);
        y[0] += r0.x; y[1] += r0.y; y[2] += r0.z; y[3] += r0.w; y[4] += r1.x; y[5] += r1.y; y[6] += r1.z; y[7] += r1.w;
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) y[i] = fmaxf(y[i], 0.f);
    }
    const uint4 packed = make_uint4(pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3]), pack_bf16x2(y[4], y[5]), pack_bf16x2(y[6], y[7]));
    *reinterpret_cast<uint4*>(patch + (size_t)pos * 16) = packed;
    const int pl = r - (W + 1);
    if (pl >= 0 && pl < TP && m0 + pl < Mtot) {
      *reinterpret_cast<uint4*>(a.tr_out + (size_t)(m0 + pl) * CI + 8 * u) = packed;
      if (!WQ && a.tr_out_f32) {
        float* o = a.tr_out_f32 + (size_t)(m0 + pl) * CI + 8 * u;
        *reinterpret_cast<float4*>(o) = make_float4(y[0], y[1], y[2], y[3]);
        *reinterpret_cast<float4*>(o + 4) = make_float4(y[4], y[5], y[6], y[7]);
      }
    }
  }
  __syncthreads();

  f32x4 acc[NB][J];
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int j = 0; j < J; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int j = 0; j < J; ++j)
#pragma unroll
    for (int s = 0; s < S; ++s) {
      const unsigned addr = CI == 64 ? (xaddr[j][s >> 1] ^ ((s & 1) << 6)) : xaddr[j][s];
      const bf16x8 b = *reinterpret_cast<const bf16x8*>(patch + addr);
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) acc[nb][j] = mfma16(wf[s][nb], b, acc[nb][j]);
    }

  float s1[NB][4], s2[NB][4];
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int v = 0; v < 4; ++v) s1[i][v] = s2[i][v] = 0.f;
  narrow_store<J, NB, WN, CO>(a, acc, m0 + wm * J * 16, wave, lane, Mtot, s1, s2);
  narrow_flush_sums<NB, WN, CO>(a, s1, s2, wave, lane);
}

// LDS of the kernel above for `units` units of patch
static size_t narrow_tr_lds(int units, int CI, int var) {
  return (size_t)units * 16 + 128 + (size_t)12 * CI + (size_t)units * (var == 2 ? 32 : 16) +
         ((var == 1 || var == 2) ? (size_t)units * 16 : (var == 3 ? (size_t)units * 32 : 0));
}
constexpr int kNarrowTrMaxTiles = 1024;   // beyond that a workgroup per tile re-reads the filter too often: the looped kernel runs
constexpr size_t kNarrowTrMaxLds = 150 * 1024;

template <int CI, int NB, int WN, int J, int VAR>
hipError_t run_narrow_tr(const GatherConvArgs& a, hipStream_t s) {
  constexpr int WM = 4 / WN, TP = 16 * J * WM, U = CI / 8;
  const int Mtot = a.N * a.OH * a.OW;
  const int rows = TP + 2 * a.Wi + 2;
  const int units = (rows * U + 255) / 256 * 256;
  const size_t lds = narrow_tr_lds(units, CI, VAR);
  const int ntiles = (Mtot + TP - 1) / TP;
  if (lds > kNarrowTrMaxLds || ntiles > kNarrowTrMaxTiles) return hipErrorInvalidValue;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_narrow_tr_kernel<CI, NB, WN, J, VAR>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kNarrowTrMaxLds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  static char name[80];
  if (!name[0]) snprintf(name, sizeof(name), "conv_narrow_tr_kernel<%d, %d, %d, %d, %s>", CI, NB, WN, J, VAR == 0 ? "bn fwd" : (VAR == 1 ? "bn bwd" : (VAR == 2 ? "bn bwd f32" : "bn fwd + res")));
  note_kernel(name);
  NarrowLaunch L;
  L.units = units;
  L.magic_w = ((1ull << 40) + a.Wi - 1) / a.Wi;
  L.magic_h = ((1ull << 40) + a.Hi - 1) / a.Hi;
  L.same_masks = 0;
  hipLaunchKernelGGL((conv_narrow_tr_kernel<CI, NB, WN, J, VAR>), dim3(ntiles), dim3(256), lds, s, a, L);
  return hipGetLastError();
}

// pixel blocks per wave as run_narrow_j
template <int WM>
static int narrow_j_for(int Mtot) { return Mtot >= 512 * 64 * WM ? 4 : (Mtot >= 512 * 32 * WM ? 2 : 1); }

template <int CI, int NB, int WN, int VAR>
hipError_t run_narrow_tr_j(const GatherConvArgs& a, hipStream_t s) {
  switch (narrow_j_for<4 / WN>(a.N * a.OH * a.OW)) {
    case 4: return run_narrow_tr<CI, NB, WN, 4, VAR>(a, s);
    case 2: return run_narrow_tr<CI, NB, WN, 2, VAR>(a, s);
    default: return run_narrow_tr<CI, NB, WN, 1, VAR>(a, s);
  }
}
template <int VAR>
hipError_t run_narrow_tr_c(const GatherConvArgs& a, hipStream_t s) {
  if (a.Ci == 16) return run_narrow_tr_j<16, 1, 1, VAR>(a, s);
  if (a.Ci == 32) return run_narrow_tr_j<32, 2, 1, VAR>(a, s);
  return run_narrow_tr_j<64, 2, 2, VAR>(a, s);
}


// ------------------------------------------------------------------------------------------------
// Weight gradient of the same layers: dw[co, tap, ci] = sum over pixels of dy[pixel, co] * x[pixel + tap, ci]
// ------------------------------------------------------------------------------------------------
// The contraction runs over pixels and the result is tiny (C x 9 x C), so the generic kernel's split (one filter tap
// and one range of pixels per workgroup, fp32 atomics into dw after a fill kernel) reads x nine times and ends in
// hundreds of atomics per address.  Here a workgroup owns a range of image rows for ALL nine taps:
//   * x and dy of those rows land in LDS once, in a PADDED layout: every image row has a zero pixel on either side
//     and every image a zero row above and below (lanes whose destination is padding load the zero word).  A tap is
//     then a constant shift of the position index with no masking: what a shifted read picks up beyond the image
//     is a stored zero, and positions that are padding in dy contribute nothing;
//   * the operands are read with the transposing LDS load (8 pixels of one channel per lane) and every wave keeps
//     the whole [16 co][9 taps][C ci] block of its output-channel block in registers;
//   * waves that share an output-channel block split the pixel steps and add their blocks through LDS; the
//     workgroup's sum goes to its own slice of a scratch array, and a second kernel adds the slices.
struct NarrowWgradLaunch {
  int R;            // padded rows per tile
  int tiles;        // tiles in all; workgroup b takes tiles b, b + gridDim.x, ...
  int PW, HP;       // padded row length W + 2 and padded image height H + 2
  int rows_total;   // N * HP
  int KP;           // positions a workgroup contracts over: R * PW rounded up to 32
  int xunits, dyunits;   // 16-byte units of the two LDS regions (multiples of 256)
  int fold_off;          // LDS byte offset of 4 KB for adding up an earlier launch's slices
  float* partial;
  size_t stride;    // floats per slice
};

typedef short n_v4s16 __attribute__((ext_vector_type(4)));
// One operand fragment = two transposing reads (pixels 4g .. 4g+3 and 16 more rows further).  The reads are inline
// assembly without a wait, so that a whole batch is in flight before the first use: narrow_frags_landed() waits
// once, narrow_join() ties the registers to that wait (volatile statements keep their order).
struct NarrowFrag { n_v4s16 lo, hi; };
__device__ __forceinline__ void narrow_read_tr8(NarrowFrag& f, unsigned addr, unsigned second) {
  asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(f.lo) : "v"(addr));
  asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(f.hi) : "v"(addr + second));
}
__device__ __forceinline__ void narrow_frags_landed() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
__device__ __forceinline__ bf16x8 narrow_join(NarrowFrag& f) {
  asm volatile("" : "+v"(f.lo), "+v"(f.hi));
  typedef short v8s16 __attribute__((ext_vector_type(8)));
  const v8s16 both = __builtin_shufflevector(f.lo, f.hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, both);
}

// STEM: x has 8 channels in memory (3 real ones, the stem of a network); in LDS a position of x is 16 channels wide with
// the upper 8 zero, so that the same transposing reads apply, and only the real input channels are stored.
template <int C, bool STEM>
__global__ __launch_bounds__(256) void conv_wgrad_narrow_kernel(WgradArgs a, NarrowWgradLaunch L) {
  constexpr int U = C / 8, ROWB = C * 2, NCB = C / 16, WK = 4 / NCB;
  constexpr int UX = STEM ? 2 : U, ROWBX = UX * 16, NCBI = STEM ? 1 : NCB;   // x side: units, bytes, 16-channel blocks
  constexpr bool SWZ_DY = C == 64, SWZ_X = !STEM && C == 64;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wcb = wave % NCB, wk = wave / NCB;
  const int W = a.Wi, H = a.Hi, PW = L.PW, HP = L.HP;
  const char* zero = reinterpret_cast<const char*>(g_narrow_zero);

  // position idx of a region -> source pixel.  x region: idx 0 is one position before padded row pr0 - 1;
  // dy region: idx 0 is the first position of padded row pr0.  With 64 channels the 32-byte slot of a position is
  // XORed with bit 1 of idx (the four pixels of a transposing read then fall into four bank groups).
  int pr0 = 0;                                       // first padded row (over all images) of the current tile
  // ulog: log2 of the units per position in LDS; src_units: units per pixel that exist in memory (the others are
  // zeros); pitch: channels per pixel in memory
  auto fill = [&](const bf16_t* src, int units, int lead, int first_row, int nrows, int lds_unit0, int ulog, int src_units,
                  int pitch, bool swz) {
    for (int base = wave * 64; base < units; base += 256) {
      const int pos = base + lane;
      const int idx = pos >> ulog, us = pos & ((1 << ulog) - 1);
      const int u = swz ? (us ^ ((idx & 2) << 1)) : us;
      const int xp = idx - lead;
      const int lr = xp >= 0 ? xp / PW : -1;
      const int c = xp - lr * PW;
      const int gr = first_row + lr;
      const int n = gr >= 0 ? gr / HP : 0;
      const int hr = gr - n * HP;
      const bool ok = u < src_units && lr >= 0 && lr < nrows && gr >= 0 && gr < L.rows_total && hr >= 1 && hr <= H && c >= 1 && c <= W;
      const char* g = reinterpret_cast<const char*>(src + (((size_t)n * H + (hr - 1)) * W + (c - 1)) * pitch + u * 8);
      narrow_dma16(ok ? g : zero, smem + (size_t)(lds_unit0 + base) * 16);
    }
  };
  constexpr int ULOG = U == 2 ? 1 : (U == 4 ? 2 : 3), UXLOG = UX == 2 ? 1 : (UX == 4 ? 2 : 3);
  f32x4 acc[9][NCBI];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int j = 0; j < NCBI; ++j) acc[t][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  int shift[9];   // x idx of a tap relative to the dy position
#pragma unroll
  for (int t = 0; t < 9; ++t) {
    const int dh = (a.tap[t] & 0xff) - 8, dw = ((a.tap[t] >> 8) & 0xff) - 8;
    shift[t] = 1 + (1 + dh) * PW + dw;
  }

  const int g = lane >> 4, i16 = lane & 15;
  const unsigned dy0 = (unsigned)L.xunits * 16u;
  constexpr int TB = NCBI == 1 ? 9 : 3;              // taps whose fragments are read in one batch
  const int first_tile = narrow_xcd_consecutive(blockIdx.x, gridDim.x);
  // The slices an earlier launch left (WgradArgs::prev_*): a block of 16 float4 of that result per workgroup and round, 16
  // thread groups take every 16th slice each and the 16 partial sums are added in order (wgrad_slices_reduce_kernel's
  // order: the same bits).  The first round's loads go out behind this launch's own first loads and share their wait.
  // (its 4 KB of LDS follow the operand regions: the transposing reads below take LDS addresses counted from the start of
  // the dynamic area, which must therefore stay at address 0 -- no static LDS in this kernel)
  float4* fold_red = reinterpret_cast<float4*>(smem + L.fold_off);
  const int fold_blocks = a.prev_slices > 0 ? (a.prev_n4 + 15) / 16 : 0;
  const int fgrp = tid >> 4;
  auto fold_load = [&](int blk) {
    const int i = blk * 16 + (tid & 15);
    float4 v[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int k = fgrp + 16 * j;
      v[j] = (i < a.prev_n4 && k < a.prev_slices) ? reinterpret_cast<const float4*>(a.prev_partial)[(size_t)k * a.prev_stride4 + i]
                                                  : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    float4 sacc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int j = 0; j < 16; ++j) { sacc.x += v[j].x; sacc.y += v[j].y; sacc.z += v[j].z; sacc.w += v[j].w; }
    return sacc;
  };
  auto fold_store = [&](int blk) {   // after a barrier that follows fold_red[tid] = fold_load(blk)
    const int i = blk * 16 + (tid & 15);
    if (fgrp == 0 && i < a.prev_n4) {
      float4* dst = reinterpret_cast<float4*>(a.prev_dw) + i;
      float4 t = a.prev_overwrite ? make_float4(0.f, 0.f, 0.f, 0.f) : *dst;
      for (int k = 0; k < 16; ++k) {
        const float4 p = fold_red[k * 16 + (tid & 15)];
        t.x += p.x; t.y += p.y; t.z += p.z; t.w += p.w;
      }
      *dst = t;
    }
  };
  for (int tile = first_tile; tile < L.tiles; tile += gridDim.x) {
    if (tile != first_tile) __syncthreads();           // every wave is done reading the previous tile
    pr0 = tile * L.R;
    fill(a.x, L.xunits, 1, pr0 - 1, L.R + 2, 0, UXLOG, STEM ? 1 : UX, STEM ? 8 : C, SWZ_X);
    fill(a.dy, L.dyunits, 0, pr0, L.R, L.xunits, ULOG, U, C, SWZ_DY);
    const bool folds = tile == first_tile && (int)blockIdx.x < fold_blocks;
    if (folds) fold_red[tid] = fold_load(blockIdx.x);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (folds) {
      fold_store(blockIdx.x);
      for (int blk = blockIdx.x + gridDim.x; blk < fold_blocks; blk += gridDim.x) {   // more blocks than workgroups (64 channels)
        const float4 sacc = fold_load(blk);
        __syncthreads();
        fold_red[tid] = sacc;
        __syncthreads();
        fold_store(blk);
      }
    }
    for (int st = wk; st < L.KP / 32; st += WK) {
      const int pp = st * 32 + 4 * g + (i16 >> 2);     // this lane's first pixel position of the step
      const int aslot = SWZ_DY ? (wcb ^ (pp & 2)) : wcb;
      NarrowFrag ra;
      narrow_read_tr8(ra, dy0 + (unsigned)(pp * ROWB + aslot * 32 + (i16 & 3) * 8), 16 * ROWB);
      bf16x8 fa;
#pragma unroll
      for (int t0 = 0; t0 < 9; t0 += TB) {
        NarrowFrag rb[TB][NCBI];
#pragma unroll
        for (int t = 0; t < TB; ++t) {
          const int idx = pp + shift[t0 + t];
#pragma unroll
          for (int j = 0; j < NCBI; ++j) {
            const int bslot = SWZ_X ? (j ^ (idx & 2)) : j;
            narrow_read_tr8(rb[t][j], (unsigned)(idx * ROWBX + bslot * 32 + (i16 & 3) * 8), 16 * ROWBX);
          }
        }
        narrow_frags_landed();
        if (t0 == 0) fa = narrow_join(ra);
#pragma unroll
        for (int t = 0; t < TB; ++t)
#pragma unroll
          for (int j = 0; j < NCBI; ++j) acc[t0 + t][j] = mfma16(fa, narrow_join(rb[t][j]), acc[t0 + t][j]);
      }
    }
  }

  // ---- add the blocks of the waves that share an output-channel block, then store the workgroup's slice ----
  if (WK > 1) {
    __syncthreads();   // every wave is done with the tiles
    float4* red = reinterpret_cast<float4*>(smem);
    if (wk > 0) {
#pragma unroll
      for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int j = 0; j < NCBI; ++j)
          red[(((wk - 1) * NCB + wcb) * 9 * NCBI + t * NCBI + j) * 64 + lane] = make_float4(acc[t][j][0], acc[t][j][1], acc[t][j][2], acc[t][j][3]);
    }
    __syncthreads();
    if (wk == 0) {
      for (int o = 1; o < WK; ++o)
#pragma unroll
        for (int t = 0; t < 9; ++t)
#pragma unroll
          for (int j = 0; j < NCBI; ++j) {
            const float4 v = red[(((o - 1) * NCB + wcb) * 9 * NCBI + t * NCBI + j) * 64 + lane];
            acc[t][j][0] += v.x; acc[t][j][1] += v.y; acc[t][j][2] += v.z; acc[t][j][3] += v.w;
          }
    }
  }
  if (wk == 0) {
    float* out = L.partial + (size_t)blockIdx.x * L.stride;
#pragma unroll
    for (int t = 0; t < 9; ++t) {
#pragma unroll
      for (int j = 0; j < NCBI; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int co = wcb * 16 + 4 * g + v, ci = j * 16 + i16;
          if (ci < a.Ci) out[((size_t)co * 9 + t) * a.Ci + ci] = acc[t][j][v];
        }
    }
  }
}

// dw (+)= sum of the slices: a block owns 16 float4 of the result, 16 thread groups take every 16th slice each
__global__ __launch_bounds__(256) void wgrad_slices_reduce_kernel(float4* __restrict__ dw, const float4* __restrict__ partial,
                                                                  int n4, int slices, size_t stride4, int overwrite) {
  __shared__ float4 red[256];
  const int i = blockIdx.x * 16 + (threadIdx.x & 15), grp = threadIdx.x >> 4;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (i < n4) {
#pragma unroll 4
    for (int k = grp; k < slices; k += 16) {
      const float4 p = partial[(size_t)k * stride4 + i];
      s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
    }
  }
  red[threadIdx.x] = s;
  __syncthreads();
  if (grp == 0 && i < n4) {
    float4 t = overwrite ? make_float4(0.f, 0.f, 0.f, 0.f) : dw[i];
    for (int k = 0; k < 16; ++k) {
      const float4 p = red[k * 16 + (threadIdx.x & 15)];
      t.x += p.x; t.y += p.y; t.z += p.z; t.w += p.w;
    }
    dw[i] = t;
  }
}

struct NarrowWgradPlan { NarrowWgradLaunch L; int blocks; size_t lds; };

// tile height: about one tile per compute unit, within 96 KB of LDS; at most 256 workgroups (and slices)
static bool wgrad_narrow_is_stem(const WgradArgs& a) { return a.Cx == 8 && a.Ci <= 8 && a.Co != a.Cx; }

bool plan_wgrad_narrow(const WgradArgs& a, NarrowWgradPlan& P) {
  const int C = a.Co, U = C / 8, ROWB = C * 2;
  const int UX = wgrad_narrow_is_stem(a) ? 2 : U, NCBI = wgrad_narrow_is_stem(a) ? 1 : C / 16;
  const int PW = a.Wi + 2, HP = a.Hi + 2;
  const long long rows_total = (long long)a.N * HP;
  if (rows_total * PW >= (1ll << 30)) return false;
  int R = (int)((rows_total + 255) / 256);
  if (R < 1) R = 1;
  for (;; --R) {
    const int KP = (R * PW + 31) / 32 * 32;
    const int xpos = KP + 2 * PW + 2, xunits = (xpos * UX + 255) / 256 * 256, dyunits = (KP * U + 255) / 256 * 256;
    const size_t tiles = (size_t)(xunits + dyunits) * 16;
    const size_t red = C == 64 ? 0 : (size_t)3 * 9 * NCBI * 1024;   // blocks of the waves that are added
    if (tiles <= 96 * 1024 || R == 1) {
      if (tiles > 96 * 1024) return false;
      P.L.R = R; P.L.PW = PW; P.L.HP = HP; P.L.rows_total = (int)rows_total; P.L.KP = KP;
      P.L.xunits = xunits; P.L.dyunits = dyunits;
      P.L.tiles = (int)((rows_total + R - 1) / R);
      P.blocks = P.L.tiles < 256 ? P.L.tiles : 256;
      P.lds = tiles > red ? tiles : red;
      P.L.fold_off = (int)((P.lds + 15) / 16 * 16);
      P.lds = (size_t)P.L.fold_off + 4096;
      (void)ROWB;
      return true;
    }
  }
}

}  // namespace

bool conv_narrow_applies(const GatherConvArgs& a) {
  const bool stem = a.Ci == 8 && (a.Co == 16 || a.Co == 32 || a.Co == 64);   // 3 input channels stored as 8
  const bool widens = a.Ci == 16 && a.Co == 160;   // the first block of a wide network (WRN-28-10: 16 -> 160)
  if (!stem && a.Ci != 16 && a.Ci != 32 && a.Ci != 64) return false;
  if ((!stem && !widens && a.Co != a.Ci) || a.w_rows != a.Co || a.Kw != 9 * a.Ci) return false;
  if (a.ntaps != 9 || a.in_stride != 1 || a.out_stride != 1 || a.ooh != 0 || a.oow != 0 || a.nclass > 1) return false;
  if (a.OH != a.Hi || a.OW != a.Wi || a.OHf != a.OH || a.OWf != a.OW || a.Wi < 1 || a.Wi > 1024 || a.Hi > 1024) return false;
  if ((long long)a.N * a.Hi * a.Wi >= (1ll << 30)) return false;
  for (int i = 0; i < 9; ++i) {
    const int dh = (a.tap[i] & 0xff) - 8, dw = ((a.tap[i] >> 8) & 0xff) - 8;
    if (dh < -1 || dh > 1 || dw < -1 || dw > 1 || (a.tap[i] >> 16) != i) return false;
  }
  // two patch buffers of the largest tile in LDS, within the 96 KB the kernels are configured for
  const int tp_max = a.Ci == 64 ? 128 : 256;
  if (2 * ((((size_t)(tp_max + 2 * a.Wi + 2) * (a.Ci / 8) + 255) / 256 * 256) * 16 + 128) > 96 * 1024) return false;
  return true;
}

// var as the kernel's VAR
bool conv_narrow_transforms(const GatherConvArgs& a, int var) {
  if (!conv_narrow_applies(a) || (a.Ci != 16 && a.Ci != 32 && a.Ci != 64) || a.Co != a.Ci) return false;
  const int Mtot = a.N * a.OH * a.OW;
  const int WM = a.Ci == 64 ? 2 : 4;
  const int J = Mtot >= 512 * 64 * WM ? 4 : (Mtot >= 512 * 32 * WM ? 2 : 1);
  const int TP = 16 * J * WM;
  const int units = ((TP + 2 * a.Wi + 2) * (a.Ci / 8) + 255) / 256 * 256;
  return Mtot > 0 && (Mtot + TP - 1) / TP <= kNarrowTrMaxTiles && var >= 0 && var <= 3 && narrow_tr_lds(units, a.Ci, var) <= kNarrowTrMaxLds;
}

hipError_t launch_conv_narrow(const GatherConvArgs& a, hipStream_t s) {
  if (!conv_narrow_applies(a) || a.N * a.OH * a.OW <= 0) return hipErrorInvalidValue;
  if (a.tr_mode != 0) {
    const bool wq = a.tr_mode == 2;
    const int var = wq ? (a.tr_p_f32 ? 2 : 1) : (a.tr_q ? 3 : 0);   // forward form: tr_q, if given, is the fp32 residual
    if ((a.tr_mode != 1 && a.tr_mode != 2) || !a.tr_p || !a.tr_out || !a.tr_sums || !a.tr_gamma || (wq && (!a.tr_q || !a.tr_bsums || !a.tr_dgamma || !a.tr_dbeta)) ||
        (!wq && (!a.tr_beta || a.tr_p_f32)) || !conv_narrow_transforms(a, var))
      return hipErrorInvalidValue;
    switch (var) {
      case 0: return run_narrow_tr_c<0>(a, s);
      case 1: return run_narrow_tr_c<1>(a, s);
      case 2: return run_narrow_tr_c<2>(a, s);
      default: return run_narrow_tr_c<3>(a, s);
    }
  }
  if (a.Ci == 8) return a.Co == 16 ? run_narrow_j<8, 1, 1>(a, s) : (a.Co == 32 ? run_narrow_j<8, 2, 1>(a, s) : run_narrow_j<8, 4, 1>(a, s));
  if (a.Ci == 16 && a.Co == 160)   // at most two pixel blocks per wave: five channel blocks each already fill the registers
    return a.N * a.OH * a.OW >= 512 * 32 * 2 ? run_narrow<16, 5, 2, 2>(a, s) : run_narrow<16, 5, 2, 1>(a, s);
  if (a.Ci == 16) return run_narrow_j<16, 1, 1>(a, s);
  if (a.Ci == 32) return run_narrow_j<32, 2, 1>(a, s);
  return run_narrow_j<64, 2, 2>(a, s);
}

bool conv_wgrad_narrow_applies(const WgradArgs& a) {
  if (a.Co != 16 && a.Co != 32 && a.Co != 64) return false;
  const bool same = a.Ci == a.Co && a.Cx == a.Co;                  // C -> C
  if (!same && !wgrad_narrow_is_stem(a)) return false;              // or the stem: 3 (stored as 8) -> C
  if (a.Ci < 1 || a.ntaps != 9 || a.stride != 1 || a.OH != a.Hi || a.OW != a.Wi) return false;
  for (int i = 0; i < 9; ++i) {
    const int dh = (a.tap[i] & 0xff) - 8, dw = ((a.tap[i] >> 8) & 0xff) - 8;
    if (dh < -1 || dh > 1 || dw < -1 || dw > 1) return false;
  }
  NarrowWgradPlan P;
  return plan_wgrad_narrow(a, P);
}

size_t conv_wgrad_narrow_scratch_bytes(const WgradArgs& a) {
  NarrowWgradPlan P;
  if (!conv_wgrad_narrow_applies(a) || !plan_wgrad_narrow(a, P)) return 0;
  return (size_t)P.blocks * a.Co * 9 * a.Ci * 4;
}

template <int C, bool STEM>
static hipError_t run_wgrad_narrow(const WgradArgs& a, const NarrowWgradPlan& P, hipStream_t s) {
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_wgrad_narrow_kernel<C, STEM>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 100 * 1024 + 16);
    if (e != hipSuccess) return e;
    configured = true;
  }
  static char name[64];
  if (!name[0]) snprintf(name, sizeof(name), STEM ? "conv_wgrad_narrow_kernel<%d, stem>" : "conv_wgrad_narrow_kernel<%d>", C);
  note_kernel(name);
  hipLaunchKernelGGL((conv_wgrad_narrow_kernel<C, STEM>), dim3(P.blocks), dim3(256), P.lds, s, a, P.L);
  return hipGetLastError();
}

hipError_t launch_conv_wgrad_narrow(const WgradArgs& a, hipStream_t s) {
  NarrowWgradPlan P;
  if (!conv_wgrad_narrow_applies(a) || !plan_wgrad_narrow(a, P)) return hipErrorInvalidValue;
  const size_t n = (size_t)a.Co * 9 * a.Ci;
  if (!a.scratch || a.scratch_bytes < (size_t)P.blocks * n * 4) return hipErrorInvalidValue;
  P.L.partial = a.scratch;
  P.L.stride = n;
  if (a.prev_slices > 0 && (!a.prev_dw || !a.prev_partial || a.prev_n4 <= 0 || a.prev_slices > 256 || a.prev_partial == a.scratch))
    return hipErrorInvalidValue;
  hipError_t e;
  if (wgrad_narrow_is_stem(a))
    e = a.Co == 16 ? run_wgrad_narrow<16, true>(a, P, s) : (a.Co == 32 ? run_wgrad_narrow<32, true>(a, P, s) : run_wgrad_narrow<64, true>(a, P, s));
  else
    e = a.Co == 16 ? run_wgrad_narrow<16, false>(a, P, s) : (a.Co == 32 ? run_wgrad_narrow<32, false>(a, P, s) : run_wgrad_narrow<64, false>(a, P, s));
  if (e != hipSuccess || a.defer_reduce) return e;
  return launch_wgrad_slices_reduce(a.dw, a.scratch, (int)(n / 4), P.blocks, n / 4, a.overwrite, s);
}

hipError_t launch_wgrad_slices_reduce(float* dw, const float* partial, int n4, int slices, size_t stride4, int overwrite, hipStream_t s) {
  if (!dw || !partial || n4 <= 0 || slices <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(wgrad_slices_reduce_kernel, dim3((n4 + 15) / 16), dim3(256), 0, s, reinterpret_cast<float4*>(dw),
                     reinterpret_cast<const float4*>(partial), n4, slices, stride4, overwrite);
  return hipGetLastError();
}

int conv_wgrad_narrow_slices(const WgradArgs& a) {
  NarrowWgradPlan P;
  return (conv_wgrad_narrow_applies(a) && plan_wgrad_narrow(a, P)) ? P.blocks : 0;
}

}  // namespace fdg

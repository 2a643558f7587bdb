// Pieces shared by the convolution kernels: MFMA wrapper, bf16 packing, and the output stage.
#pragma once
#include "fdg_internal.h"

namespace fdg {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

typedef float f32x16 __attribute__((ext_vector_type(16)));
// v_mfma_f32_32x32x16_bf16: lane l supplies row (l & 31) of A and column (l & 31) of B with the 8 consecutive
// k values 8*(l >> 5) .. +7; it receives D[8*(v >> 2) + 4*(l >> 5) + (v & 3)][l & 31] in component v.
// One wave per SIMD keeps the matrix pipe ~97 % busy with this shape (the 16x16x32 shape needs two).
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  bf16_t l = (bf16_t)lo, h = (bf16_t)hi;
  return (uint32_t)__builtin_bit_cast(uint16_t, l) | ((uint32_t)__builtin_bit_cast(uint16_t, h) << 16);
}
__device__ __forceinline__ float bf16_lo(uint32_t u) { return __builtin_bit_cast(float, u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __builtin_bit_cast(float, u & 0xffff0000u); }

// Output stage of a gather-form convolution.  acc[i][j] is the 16x16 result block of channel group i
// and pixel group j of this wave: lane l holds channels 4*(l>>4) .. +3 of pixel (l & 15).  Adds the
// optional fp32 addend (gated by addmask > 0 when given), applies the optional gate, writes fp32 and/or bf16 and
// adds the per-channel sums (of the bf16 output and its square, or with bnx of the output and output * bnx).
// BN = channels of the workgroup tile starting at c_tile; this wave's channels start at c_tile + c_wave.
// Must be called by all threads of the workgroup (the statistics are combined through LDS).
template <int FM, int FN, int BN>
__device__ __forceinline__ void store_tile(const GatherConvArgs& a, const f32x4 (&acc)[FN][FM], int m_base, int c_tile,
                                           int c_wave, int lane) {
  const int Mtot = a.N * a.OH * a.OW;
  const int c_base = c_tile + c_wave;
  float s1[FN][4], s2[FN][4];   // batch-norm statistics of this lane's pixels (only with a.stats)
#pragma unroll
  for (int i = 0; i < FN; ++i)
#pragma unroll
    for (int v = 0; v < 4; ++v) s1[i][v] = s2[i][v] = 0.f;
#pragma unroll
  for (int j = 0; j < FM; ++j) {
    const int m = m_base + j * 16 + (lane & 15);
    if (m >= Mtot) continue;
    const int ow = m % a.OW, t2 = m / a.OW, oh = t2 % a.OH, n = t2 / a.OH;
    const size_t opix = ((size_t)n * a.OHf + oh * a.out_stride + a.ooh) * a.OWf + ow * a.out_stride + a.oow;
#pragma unroll
    for (int i = 0; i < FN; ++i) {
      const int c = c_base + i * 16 + 4 * (lane >> 4);
      if (c >= a.Co) continue;
      const size_t o = opix * a.Co + c;
      f32x4 v = acc[i][j];
      if (a.addend) {
        float4 ad = *reinterpret_cast<const float4*>(a.addend + o);
        if (a.addmask) {
          const uint2 mk = *reinterpret_cast<const uint2*>(a.addmask + o);
          if (!(bf16_lo(mk.x) > 0.f)) ad.x = 0.f;
          if (!(bf16_hi(mk.x) > 0.f)) ad.y = 0.f;
          if (!(bf16_lo(mk.y) > 0.f)) ad.z = 0.f;
          if (!(bf16_hi(mk.y) > 0.f)) ad.w = 0.f;
        }
        v[0] += ad.x;
        v[1] += ad.y;
        v[2] += ad.z;
        v[3] += ad.w;
      }
      if (a.gate) {   // data gradient that ends in a ReLU: kept where the ReLU's output was positive
        const uint2 gt = *reinterpret_cast<const uint2*>(a.gate + o);
        if (!(bf16_lo(gt.x) > 0.f)) v[0] = 0.f;
        if (!(bf16_hi(gt.x) > 0.f)) v[1] = 0.f;
        if (!(bf16_lo(gt.y) > 0.f)) v[2] = 0.f;
        if (!(bf16_hi(gt.y) > 0.f)) v[3] = 0.f;
      }
      if (a.out_f32) *reinterpret_cast<float4*>(a.out_f32 + o) = make_float4(v[0], v[1], v[2], v[3]);
      const uint2 packed = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
      if (a.out_b16) *reinterpret_cast<uint2*>(a.out_b16 + o) = packed;
      if (a.stats) {
        const bool f = a.stats_f32 != 0;
        const float r0 = f ? v[0] : bf16_lo(packed.x), r1 = f ? v[1] : bf16_hi(packed.x);
        const float r2 = f ? v[2] : bf16_lo(packed.y), r3 = f ? v[3] : bf16_hi(packed.y);
        s1[i][0] += r0; s1[i][1] += r1; s1[i][2] += r2; s1[i][3] += r3;
        if (a.bnx) {   // the two sums of the batch-norm backward that follows: sum g and sum g * x
          const uint2 bx = *reinterpret_cast<const uint2*>(a.bnx + o);
          s2[i][0] += r0 * bf16_lo(bx.x); s2[i][1] += r1 * bf16_hi(bx.x);
          s2[i][2] += r2 * bf16_lo(bx.y); s2[i][3] += r3 * bf16_hi(bx.y);
        } else {
          s2[i][0] += r0 * r0; s2[i][1] += r1 * r1; s2[i][2] += r2 * r2; s2[i][3] += r3 * r3;
        }
      }
    }
  }
  if (a.stats) {
    // Reduce over pixels: first across the 16 lanes that hold the same 4 channels, then across the waves of the
    // workgroup through LDS in wave order (a fixed order: the workgroup's partial sum is reproducible), so that the
    // workgroup ends with one exact add per channel and value (stat_add).
    constexpr int NW = 4;                       // waves of the workgroup (256 threads)
    __shared__ float red[NW][2 * BN];
    __syncthreads();   // the main loop's LDS traffic is over for every wave
    for (int t = threadIdx.x; t < NW * 2 * BN; t += blockDim.x) (&red[0][0])[t] = 0.f;
    __syncthreads();
    const int wave = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i < FN; ++i)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        float x1 = s1[i][v], x2 = s2[i][v];
#pragma unroll
        for (int off = 8; off > 0; off >>= 1) {
          x1 += __shfl_xor(x1, off, 16);
          x2 += __shfl_xor(x2, off, 16);
        }
        if ((lane & 15) == 0) {
          const int cl = c_wave + i * 16 + 4 * (lane >> 4) + v;
          red[wave][cl] = x1;
          red[wave][BN + cl] = x2;
        }
      }
    __syncthreads();
    for (int t = threadIdx.x; t < 2 * BN; t += blockDim.x) {
      const int c = c_tile + (t % BN);
      if (c < a.Co)
        stat_add(a.stats + (size_t)(blockIdx.x % kStatReplicas) * a.stats_rep_stride, a.Co, t / BN, c,
                 (red[0][t] + red[1][t]) + (red[2][t] + red[3][t]));
    }
  }
}

// Output stage for 32x32 accumulator blocks, one wave = 32 pixels x BN channels.
// acc[i] covers channels c_tile + 32 i .. +31: lane l holds pixel m_base + (l & 31) and, in components
// 4g..4g+3, channels 8g + 4*(l >> 5) .. +3 of the block.  A lane per pixel would write 8- or 16-byte pieces
// 2*Co bytes apart, so the block is first turned through LDS (rows of BN floats, padded by 16 bytes so that
// the 16-byte column writes of 16 consecutive pixels fall into different banks) and then leaves row by row:
// consecutive lanes carry consecutive 4-channel units of a pixel, which makes the addend and mask reads and
// the fp32 / bf16 stores contiguous runs of BN channels.  `lds` is this wave's private region of
// OUT_STAGE_BYTES(BN) bytes; the main loop's LDS traffic of the whole workgroup must be over.
// Must be called by all threads of the workgroup (the statistics are combined through LDS).
constexpr int out_stage_pitch(int BN) { return BN * 4 + 16; }
constexpr int out_stage_bytes(int BN) { return 32 * out_stage_pitch(BN) + 128; }
// where the lanes park their partial statistics: 4 waves x PERIOD x 64 lanes x 8 floats (PERIOD = 5 for 160 channels)
constexpr int stats_stage_bytes(int BN) { return 4 * ((BN / 4) % 16 == 0 ? 1 : (BN / 4) / 8) * 64 * 32; }

// Kernels with eight waves (256 registers, 8 regions in the LDS) turn the block ROWS = 16 pixels at a time, issue the
// loads of GROUP = 5 iterations together (about 14 registers per iteration) and park the statistics of PARKW = 8
// waves where the regions were (stats_lds may then overlap them: a barrier separates the two uses).
// F32S: the per-channel sums are of the fp32 values (a data gradient whose fp32 result the batch norm below reads),
// not of their bf16 roundings.
template <int FN, int BN, int GROUP = 10, int ROWS = 32, int PARKW = 4, bool F32S = false>
__device__ __forceinline__ void store_rows32(const GatherConvArgs& a, const f32x16 (&acc)[FN], int m_base, int c_tile,
                                             int lane, unsigned char* lds, unsigned char* stats_lds) {
  static_assert(FN * 32 == BN, "one wave carries all channels of the tile");
  static_assert(ROWS == 32 || ROWS == 16, "whole or half blocks");
  constexpr int PITCH = out_stage_pitch(BN);
  constexpr int UNITS = BN / 4;                       // 16-byte fp32 units per pixel
  constexpr int ITERS = ROWS * UNITS / 64;
  constexpr int PERIOD = UNITS % 64 == 0 ? 1 : (UNITS % 32 == 0 ? 1 : (UNITS % 16 == 0 ? UNITS / 16 : (UNITS % 8 == 0 ? UNITS / 8 : UNITS)));
  static_assert((64 * PERIOD) % UNITS == 0 && ITERS % PERIOD == 0 && (ROWS * UNITS) % 64 == 0, "unit assignment repeats every PERIOD iterations");
  static_assert(stats_stage_bytes(BN) == 4 * PERIOD * 64 * 32, "size of the statistics stage");
  const int Mtot = a.N * a.OH * a.OW;
  // The arguments live in constant memory, and a compiler short of scalar registers re-reads them at every
  // use: one scalar load and a full wait per pointer test, twenty times over.  Read what the row loop needs
  // once, into values the compiler cannot trace back to memory.
  typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
  typedef const f32x4 __attribute__((address_space(1))) * gcf4;
  typedef f32x4 __attribute__((address_space(1))) * gf4;
  typedef const u32x2 __attribute__((address_space(1))) * gcu2;
  typedef u32x2 __attribute__((address_space(1))) * gu2;
  uint64_t p_addend = (uint64_t)a.addend, p_mask = (uint64_t)a.addmask, p_f32 = (uint64_t)a.out_f32, p_b16 = (uint64_t)a.out_b16;
  uint64_t p_gate = (uint64_t)a.gate, p_bnx = (uint64_t)a.bnx;
  int Co = a.Co;
  int want_stats = a.stats != nullptr;
  asm volatile("" : "+v"(p_addend), "+v"(p_mask), "+v"(p_f32), "+v"(p_b16), "+v"(Co), "+v"(want_stats), "+v"(p_gate), "+v"(p_bnx));
  float s1[PERIOD][4], s2[PERIOD][4];
#pragma unroll
  for (int k = 0; k < PERIOD; ++k)
#pragma unroll
    for (int e = 0; e < 4; ++e) s1[k][e] = s2[k][e] = 0.f;
#pragma unroll
  for (int part = 0; part < 32 / ROWS; ++part) {
  {
    const int p = lane & 31, half = lane >> 5;
    if (ROWS == 32 || p / ROWS == part) {
#pragma unroll
      for (int i = 0; i < FN; ++i)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *reinterpret_cast<f32x4*>(lds + (p % ROWS) * PITCH + (i * 32 + 8 * g + 4 * half) * 4) =
              f32x4{acc[i][4 * g], acc[i][4 * g + 1], acc[i][4 * g + 2], acc[i][4 * g + 3]};
    }
    if (lane < ROWS) {
      const int m = m_base + part * ROWS + lane;
      int pix = -1;
      if (m < Mtot) {
        const int ow = m % a.OW, t2 = m / a.OW, oh = t2 % a.OH, n = t2 / a.OH;
        pix = (n * a.OHf + oh * a.out_stride + a.ooh) * a.OWf + ow * a.out_stride + a.oow;
      }
      *reinterpret_cast<int*>(lds + ROWS * PITCH + 4 * lane) = pix;
    }
  }
  asm volatile("" ::: "memory");   // same wave, LDS operations stay in order: no barrier needed
  // Rows leave in groups of G iterations: first every load of the group (LDS tile, addend, mask) from addresses
  // that are safe whether or not the element exists, then the arithmetic and the stores.  Written as one
  // conditional body per iteration the loads would each sit behind a branch and pay their latency one by one.
  constexpr int G = ITERS % GROUP == 0 ? GROUP : 8;
  static_assert(ITERS % G == 0 && G % PERIOD == 0, "whole groups");
#pragma unroll
  for (int it0 = 0; it0 < ITERS; it0 += G) {
    bool ok[G];
    size_t o[G];
    f32x4 v[G];
    f32x4 ad[G];
    u32x2 mk[G], gt[G], bx[G];
#pragma unroll
    for (int k = 0; k < G; ++k) {
      const int q = (it0 + k) * 64 + lane;
      const int p = q / UNITS, un = q % UNITS;
      const int pix = *reinterpret_cast<const int*>(lds + ROWS * PITCH + 4 * p);
      const int c = c_tile + un * 4;
      ok[k] = pix >= 0 && c < Co;
      o[k] = ok[k] ? (size_t)pix * Co + c : 0;
      v[k] = *reinterpret_cast<const f32x4*>(lds + p * PITCH + un * 16);
    }
    if (p_gate) {
#pragma unroll
      for (int k = 0; k < G; ++k) gt[k] = *(gcu2)(p_gate + 2 * o[k]);
    }
    if (p_bnx) {
#pragma unroll
      for (int k = 0; k < G; ++k) bx[k] = *(gcu2)(p_bnx + 2 * o[k]);
    }
    if (p_addend) {
#pragma unroll
      for (int k = 0; k < G; ++k) ad[k] = *(gcf4)(p_addend + 4 * o[k]);
      if (p_mask) {
#pragma unroll
        for (int k = 0; k < G; ++k) mk[k] = *(gcu2)(p_mask + 2 * o[k]);
#pragma unroll
        for (int k = 0; k < G; ++k) {
          if (!(bf16_lo(mk[k][0]) > 0.f)) ad[k][0] = 0.f;
          if (!(bf16_hi(mk[k][0]) > 0.f)) ad[k][1] = 0.f;
          if (!(bf16_lo(mk[k][1]) > 0.f)) ad[k][2] = 0.f;
          if (!(bf16_hi(mk[k][1]) > 0.f)) ad[k][3] = 0.f;
        }
      }
#pragma unroll
      for (int k = 0; k < G; ++k) {
        v[k] += ad[k];
      }
    }
    if (p_gate) {
#pragma unroll
      for (int k = 0; k < G; ++k) {
        if (!(bf16_lo(gt[k][0]) > 0.f)) v[k][0] = 0.f;
        if (!(bf16_hi(gt[k][0]) > 0.f)) v[k][1] = 0.f;
        if (!(bf16_lo(gt[k][1]) > 0.f)) v[k][2] = 0.f;
        if (!(bf16_hi(gt[k][1]) > 0.f)) v[k][3] = 0.f;
      }
    }
#pragma unroll
    for (int k = 0; k < G; ++k) {
      const u32x2 packed = {pack_bf16x2(v[k][0], v[k][1]), pack_bf16x2(v[k][2], v[k][3])};
      if (ok[k]) {
        if (p_f32) *(gf4)(p_f32 + 4 * o[k]) = v[k];
        if (p_b16) *(gu2)(p_b16 + 2 * o[k]) = packed;
        if (want_stats) {
          const float r0 = F32S ? v[k][0] : bf16_lo(packed[0]), r1 = F32S ? v[k][1] : bf16_hi(packed[0]);
          const float r2 = F32S ? v[k][2] : bf16_lo(packed[1]), r3 = F32S ? v[k][3] : bf16_hi(packed[1]);
          const int kk = (it0 + k) % PERIOD;
          s1[kk][0] += r0; s1[kk][1] += r1; s1[kk][2] += r2; s1[kk][3] += r3;
          if (p_bnx) {
            s2[kk][0] += r0 * bf16_lo(bx[k][0]); s2[kk][1] += r1 * bf16_hi(bx[k][0]);
            s2[kk][2] += r2 * bf16_lo(bx[k][1]); s2[kk][3] += r3 * bf16_hi(bx[k][1]);
          } else {
            s2[kk][0] += r0 * r0; s2[kk][1] += r1 * r1; s2[kk][2] += r2 * r2; s2[kk][3] += r3 * r3;
          }
        }
      }
    }
  }
  asm volatile("" ::: "memory");   // the next part overwrites the rows only after this part's reads (same wave, in order)
  }   // part
  if (a.stats) {
    if (PARKW != 4) __syncthreads();   // the statistics are parked where the rows were
    // Per-channel sums of the workgroup: every lane parks its partial sums in LDS, then one thread per channel
    // and value adds the lanes that carried that channel (LDS float atomics would do the same in one step but
    // run at a few lane operations per clock: 15-25 us per launch).
    float* park = reinterpret_cast<float*>(stats_lds);
    const int wave = threadIdx.x >> 6;
#pragma unroll
    for (int k = 0; k < PERIOD; ++k) {
      f32x4* dst = reinterpret_cast<f32x4*>(park + (size_t)((wave * PERIOD + k) * 64 + lane) * 8);
      dst[0] = f32x4{s1[k][0], s1[k][1], s1[k][2], s1[k][3]};
      dst[1] = f32x4{s2[k][0], s2[k][1], s2[k][2], s2[k][3]};
    }
    __syncthreads();
    for (int t = threadIdx.x; t < 2 * BN; t += blockDim.x) {
      const int cl = t % BN, which = t / BN;
      const int c = c_tile + cl;
      if (c >= a.Co) continue;
      const int un = cl >> 2, e = cl & 3;
      float sum = 0.f;
#pragma unroll
      for (int k = 0; k < PERIOD; ++k) {
        const int l0 = ((un - k * 64) % UNITS + UNITS) % UNITS;   // lanes with (k*64 + lane) % UNITS == un
        for (int l = l0; l < 64; l += UNITS)
#pragma unroll
          for (int w = 0; w < PARKW; ++w) sum += park[(size_t)((w * PERIOD + k) * 64 + l) * 8 + which * 4 + e];
      }
      stat_add(a.stats + (size_t)(blockIdx.x % kStatReplicas) * a.stats_rep_stride, a.Co, which, c, sum);
    }
  }
}

// End of a wide kernel whose four waves are (wave_m, wk): wave_m owns 64 pixels as two 32-pixel blocks j, wk
// one half of the contraction.  The two halves are added through LDS so that every wave ends with one
// 32-pixel block (wave wk keeps block j = wk and receives its partner's), then all four run the output stage.
// smem must hold max(4 * FN * 16 * 256, 4 * out_stage_bytes(BN) + stats_stage_bytes(BN)) bytes and be idle (no loads
// in flight).
template <int FN, int BN, bool F32S = false>
__device__ __forceinline__ void combine_and_store32(const GatherConvArgs& a, f32x16 (&acc)[FN][2], int m_tile, int c_tile,
                                                    int wave_m, int wk, int lane, unsigned char* smem) {
  __syncthreads();
  f32x4* mine = reinterpret_cast<f32x4*>(smem) + (size_t)(wave_m * 2 + wk) * (FN * 4 * 64);
  const f32x4* theirs = reinterpret_cast<const f32x4*>(smem) + (size_t)(wave_m * 2 + (wk ^ 1)) * (FN * 4 * 64);
  f32x16 keep[FN];
#pragma unroll
  for (int i = 0; i < FN; ++i) {
    const f32x16 give = wk == 0 ? acc[i][1] : acc[i][0];
    keep[i] = wk == 0 ? acc[i][0] : acc[i][1];
#pragma unroll
    for (int g = 0; g < 4; ++g)
      mine[(i * 4 + g) * 64 + lane] = f32x4{give[4 * g], give[4 * g + 1], give[4 * g + 2], give[4 * g + 3]};
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < FN; ++i)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const f32x4 p = theirs[(i * 4 + g) * 64 + lane];
      keep[i][4 * g] += p[0]; keep[i][4 * g + 1] += p[1]; keep[i][4 * g + 2] += p[2]; keep[i][4 * g + 3] += p[3];
    }
  __syncthreads();
  const int wave = wave_m * 2 + wk;
  store_rows32<FN, BN, 10, 32, 4, F32S>(a, keep, m_tile + wave_m * 64 + wk * 32, c_tile, lane, smem + (size_t)wave * out_stage_bytes(BN),
                       smem + (size_t)4 * out_stage_bytes(BN));
}

// End of the 256-pixel kernel: eight waves (wave_m, wk), wave_m = wave & 3 owns 64 pixels as two 32-pixel blocks j, wk =
// wave >> 2 one half of the contraction.  The halves are added in two rounds (80 KB each: in round j the waves with
// wk != j park block j and the waves with wk == j add it), then every wave holds the 32-pixel block j = wk of its 64
// pixels and all eight run the output stage, 16 pixels at a time (8 regions of 10.6 KB).
constexpr int out_stage16_bytes(int BN) { return 16 * out_stage_pitch(BN) + 128; }
template <int FN, int BN>
__device__ __forceinline__ void combine8_and_store32(const GatherConvArgs& a, f32x16 (&acc)[FN][2], int m_tile, int c_tile,
                                                     int wave_m, int wk, int lane, unsigned char* smem) {
  f32x16 keep[FN];
#pragma unroll
  for (int i = 0; i < FN; ++i) keep[i] = wk == 0 ? acc[i][0] : acc[i][1];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    __syncthreads();
    f32x4* area = reinterpret_cast<f32x4*>(smem) + (size_t)(wave_m * FN) * 256;
    if (wk != j) {
#pragma unroll
      for (int i = 0; i < FN; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q)
          area[(i * 4 + q) * 64 + lane] = f32x4{acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
    }
    __syncthreads();
    if (wk == j) {
#pragma unroll
      for (int i = 0; i < FN; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const f32x4 p = area[(i * 4 + q) * 64 + lane];
          keep[i][4 * q] += p[0]; keep[i][4 * q + 1] += p[1]; keep[i][4 * q + 2] += p[2]; keep[i][4 * q + 3] += p[3];
        }
    }
  }
  __syncthreads();
  const int wave = wave_m + 4 * wk;
  store_rows32<FN, BN, 5, 16, 8>(a, keep, m_tile + wave_m * 64 + wk * 32, c_tile, lane,
                                 smem + (size_t)wave * out_stage16_bytes(BN), smem);
}

// The wide-channel kernel (conv_wide_kernels.hip): input channels a multiple of 64.
bool conv_gather_wide_applies(const GatherConvArgs& a);
bool conv_gather_pair_applies(const GatherConvArgs& a);   // the two-workgroup form of the wide gather kernel runs it
hipError_t launch_conv_gather_wide(const GatherConvArgs& a, hipStream_t s);
// The wide-channel weight gradient: output and input channels multiples of 160, output width dividing 64.
bool conv_wgrad_wide_applies(const WgradArgs& a);
hipError_t launch_conv_wgrad_wide(const WgradArgs& a, hipStream_t s);
// The same for channel counts that are multiples of 128: 128 x 128 blocks, contraction split over the waves.
bool conv_wgrad128_applies(const WgradArgs& a);
hipError_t launch_conv_wgrad128(const WgradArgs& a, hipStream_t s);
// Output channels a multiple of 320, input channels a multiple of 64: 320 x 64 blocks.
bool conv_wgrad_tall_applies(const WgradArgs& a);
hipError_t launch_conv_wgrad_tall(const WgradArgs& a, hipStream_t s);

}  // namespace fdg

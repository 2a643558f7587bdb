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
// optional fp32 addend (gated by addmask > 0 when given) and writes fp32 and/or bf16.
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
      if (a.out_f32) *reinterpret_cast<float4*>(a.out_f32 + o) = make_float4(v[0], v[1], v[2], v[3]);
      const uint2 packed = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
      if (a.out_b16) *reinterpret_cast<uint2*>(a.out_b16 + o) = packed;
      if (a.stats) {
        const float r0 = bf16_lo(packed.x), r1 = bf16_hi(packed.x), r2 = bf16_lo(packed.y), r3 = bf16_hi(packed.y);
        s1[i][0] += r0; s1[i][1] += r1; s1[i][2] += r2; s1[i][3] += r3;
        s2[i][0] += r0 * r0; s2[i][1] += r1 * r1; s2[i][2] += r2 * r2; s2[i][3] += r3 * r3;
      }
    }
  }
  if (a.stats) {
    // Reduce over pixels: first across the 16 lanes that hold the same 4 channels, then across the waves
    // of the workgroup in LDS, so that the workgroup ends with one global atomic per channel and value.
    __shared__ float red[2 * BN];
    __syncthreads();   // the main loop's LDS traffic is over for every wave
    for (int t = threadIdx.x; t < 2 * BN; t += blockDim.x) red[t] = 0.f;
    __syncthreads();
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
          atomicAdd(&red[cl], x1);
          atomicAdd(&red[BN + cl], x2);
        }
      }
    __syncthreads();
    for (int t = threadIdx.x; t < 2 * BN; t += blockDim.x) {
      const int c = c_tile + (t % BN);
      if (c < a.Co) atomicAdd(a.stats + (t / BN) * a.Co + c, red[t]);
    }
  }
}

// The same output stage for 32x32 accumulator blocks: acc[i][j] covers channels c_base + 32 i .. and pixels
// m_base + 32 j ..; lane l holds pixel (l & 31) and, in components 4g..4g+3, channels 8g + 4*(l >> 5) .. +3.
template <int FM, int FN, int BN>
__device__ __forceinline__ void store_tile32(const GatherConvArgs& a, const f32x16 (&acc)[FN][FM], int m_base, int c_tile,
                                             int c_wave, int lane, bool active) {
  const int Mtot = a.N * a.OH * a.OW;
  const int c_base = c_tile + c_wave;
  float s1[FN][16], s2[FN][16];
#pragma unroll
  for (int i = 0; i < FN; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) s1[i][v] = s2[i][v] = 0.f;
#pragma unroll
  for (int j = 0; j < FM; ++j) {
    const int m = m_base + j * 32 + (lane & 31);
    if (m >= Mtot || !active) continue;
    const int ow = m % a.OW, t2 = m / a.OW, oh = t2 % a.OH, n = t2 / a.OH;
    const size_t opix = ((size_t)n * a.OHf + oh * a.out_stride + a.ooh) * a.OWf + ow * a.out_stride + a.oow;
#pragma unroll
    for (int i = 0; i < FN; ++i)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int c = c_base + i * 32 + 8 * g + 4 * (lane >> 5);
        if (c >= a.Co) continue;
        const size_t o = opix * a.Co + c;
        float v0 = acc[i][j][4 * g], v1 = acc[i][j][4 * g + 1], v2 = acc[i][j][4 * g + 2], v3 = acc[i][j][4 * g + 3];
        if (a.addend) {
          float4 ad = *reinterpret_cast<const float4*>(a.addend + o);
          if (a.addmask) {
            const uint2 mk = *reinterpret_cast<const uint2*>(a.addmask + o);
            if (!(bf16_lo(mk.x) > 0.f)) ad.x = 0.f;
            if (!(bf16_hi(mk.x) > 0.f)) ad.y = 0.f;
            if (!(bf16_lo(mk.y) > 0.f)) ad.z = 0.f;
            if (!(bf16_hi(mk.y) > 0.f)) ad.w = 0.f;
          }
          v0 += ad.x; v1 += ad.y; v2 += ad.z; v3 += ad.w;
        }
        if (a.out_f32) *reinterpret_cast<float4*>(a.out_f32 + o) = make_float4(v0, v1, v2, v3);
        const uint2 packed = make_uint2(pack_bf16x2(v0, v1), pack_bf16x2(v2, v3));
        if (a.out_b16) *reinterpret_cast<uint2*>(a.out_b16 + o) = packed;
        if (a.stats) {
          const float r0 = bf16_lo(packed.x), r1 = bf16_hi(packed.x), r2 = bf16_lo(packed.y), r3 = bf16_hi(packed.y);
          s1[i][4 * g] += r0; s1[i][4 * g + 1] += r1; s1[i][4 * g + 2] += r2; s1[i][4 * g + 3] += r3;
          s2[i][4 * g] += r0 * r0; s2[i][4 * g + 1] += r1 * r1; s2[i][4 * g + 2] += r2 * r2; s2[i][4 * g + 3] += r3 * r3;
        }
      }
  }
  if (a.stats) {
    __shared__ float red[2 * BN];
    __syncthreads();
    for (int t = threadIdx.x; t < 2 * BN; t += blockDim.x) red[t] = 0.f;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < FN; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float x1 = s1[i][v], x2 = s2[i][v];
#pragma unroll
        for (int off = 16; off > 0; off >>= 1) {   // the 32 lanes with equal (lane >> 5) hold the same channels
          x1 += __shfl_xor(x1, off, 32);
          x2 += __shfl_xor(x2, off, 32);
        }
        if ((lane & 31) == 0 && active) {
          const int cl = c_wave + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
          atomicAdd(&red[cl], x1);
          atomicAdd(&red[BN + cl], x2);
        }
      }
    __syncthreads();
    for (int t = threadIdx.x; t < 2 * BN; t += blockDim.x) {
      const int c = c_tile + (t % BN);
      if (c < a.Co) atomicAdd(a.stats + (t / BN) * a.Co + c, red[t]);
    }
  }
}

// The wide-channel kernel (conv_wide_kernels.hip): input channels a multiple of 64.
bool conv_gather_wide_applies(const GatherConvArgs& a);
hipError_t launch_conv_gather_wide(const GatherConvArgs& a, hipStream_t s);
// The wide-channel weight gradient: output and input channels multiples of 160, output width dividing 64.
bool conv_wgrad_wide_applies(const WgradArgs& a);
hipError_t launch_conv_wgrad_wide(const WgradArgs& a, hipStream_t s);

}  // namespace fdg

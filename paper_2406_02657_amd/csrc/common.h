// Device-side helpers shared by the gfx950 kernels: storage types, conversions,
// wavefront (64-lane) reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bt {

constexpr int kWave = 64;

// Storage element of bf16 mode: raw bits, converted by hand (round to nearest even).
struct bf16_t { uint16_t v; };

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

template <class T> __device__ __forceinline__ float to_float(T x);
template <> __device__ __forceinline__ float to_float<float>(float x) { return x; }
template <> __device__ __forceinline__ float to_float<bf16_t>(bf16_t x) { return bf16_bits_to_float(x.v); }

template <class T> __device__ __forceinline__ T from_float(float x);
template <> __device__ __forceinline__ float from_float<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16_t from_float<bf16_t>(float x) { bf16_t r; r.v = float_to_bf16_bits(x); return r; }

// 16-byte chunk of storage elements <-> floats.  EPC = elements per chunk.
template <class T> struct Chunk;
template <> struct Chunk<float> {
  static constexpr int EPC = 4;
  __device__ __forceinline__ static void unpack(const uint4& c, float* f) {
    f[0] = __uint_as_float(c.x); f[1] = __uint_as_float(c.y);
    f[2] = __uint_as_float(c.z); f[3] = __uint_as_float(c.w);
  }
  __device__ __forceinline__ static uint4 pack(const float* f) {
    return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
  }
};
template <> struct Chunk<bf16_t> {
  static constexpr int EPC = 8;
  __device__ __forceinline__ static void unpack(const uint4& c, float* f) {
    f[0] = __uint_as_float(c.x << 16); f[1] = __uint_as_float(c.x & 0xFFFF0000u);
    f[2] = __uint_as_float(c.y << 16); f[3] = __uint_as_float(c.y & 0xFFFF0000u);
    f[4] = __uint_as_float(c.z << 16); f[5] = __uint_as_float(c.z & 0xFFFF0000u);
    f[6] = __uint_as_float(c.w << 16); f[7] = __uint_as_float(c.w & 0xFFFF0000u);
  }
  __device__ __forceinline__ static uint4 pack(const float* f) {
    uint4 c;
    c.x = (uint32_t)float_to_bf16_bits(f[0]) | ((uint32_t)float_to_bf16_bits(f[1]) << 16);
    c.y = (uint32_t)float_to_bf16_bits(f[2]) | ((uint32_t)float_to_bf16_bits(f[3]) << 16);
    c.z = (uint32_t)float_to_bf16_bits(f[4]) | ((uint32_t)float_to_bf16_bits(f[5]) << 16);
    c.w = (uint32_t)float_to_bf16_bits(f[6]) | ((uint32_t)float_to_bf16_bits(f[7]) << 16);
    return c;
  }
};

// Store an activation that will be a GEMM operand.  With lo_off != 0 (bf16 mode) the
// value is kept as two bf16 numbers, hi at p[i] and the rounding remainder lo at
// p[i + lo_off], so that hi + lo carries about 16 mantissa bits into the MFMAs.
template <class T>
__device__ __forceinline__ void store_act(T* p, size_t i, size_t lo_off, float v) {
  const T hi = from_float<T>(v);
  p[i] = hi;
  if (lo_off) p[i + lo_off] = from_float<T>(v - to_float<T>(hi));
}

// Four consecutive activations at once (i a multiple of 4): one 8- or 16-byte store per plane.
template <class T>
__device__ __forceinline__ void store_act4(T* p, size_t i, size_t lo_off, float a, float b, float c, float d);
template <>
__device__ __forceinline__ void store_act4<float>(float* p, size_t i, size_t, float a, float b, float c, float d) {
  *reinterpret_cast<float4*>(p + i) = make_float4(a, b, c, d);
}
template <>
__device__ __forceinline__ void store_act4<bf16_t>(bf16_t* p, size_t i, size_t lo_off, float a, float b, float c, float d) {
  const uint32_t ha = float_to_bf16_bits(a), hb = float_to_bf16_bits(b), hc = float_to_bf16_bits(c), hd = float_to_bf16_bits(d);
  *reinterpret_cast<uint2*>(p + i) = make_uint2(ha | (hb << 16), hc | (hd << 16));
  if (lo_off) {
    const uint32_t la = float_to_bf16_bits(a - bf16_bits_to_float(ha)), lb = float_to_bf16_bits(b - bf16_bits_to_float(hb));
    const uint32_t lc = float_to_bf16_bits(c - bf16_bits_to_float(hc)), ld = float_to_bf16_bits(d - bf16_bits_to_float(hd));
    *reinterpret_cast<uint2*>(p + i + lo_off) = make_uint2(la | (lb << 16), lc | (ld << 16));
  }
}

// All-reduce over the 16 lanes of a DPP row (lanes 16 g .. 16 g + 15) by rotations inside the row
// (control 0x120 + n = rotate right by n): register to register, where a shuffle goes through the
// LDS crossbar.  After the four steps every lane of the row holds the result.
template <int CTRL>
__device__ __forceinline__ float dpp_row_ror(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, dpp_row_ror<0x128>(v)); v = fmaxf(v, dpp_row_ror<0x124>(v));
  v = fmaxf(v, dpp_row_ror<0x122>(v)); v = fmaxf(v, dpp_row_ror<0x121>(v));
  return v;
}
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_row_ror<0x128>(v); v += dpp_row_ror<0x124>(v);
  v += dpp_row_ror<0x122>(v); v += dpp_row_ror<0x121>(v);
  return v;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}

}  // namespace bt

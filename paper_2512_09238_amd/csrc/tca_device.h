// Device-side helpers for the gfx950 kernels: storage-type loads, wave64
// reductions.  Wavefront size is 64 throughout.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tca {

constexpr int kWave = 64;

struct bf16_t { uint16_t bits; };   // storage only; arithmetic is done after widening

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// Round-to-nearest-even float -> bf16 bits (inputs are finite here; NaN stays NaN).
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Elements carried by one 16-byte vector load of storage type T.
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  __device__ static __forceinline__ void load(const float* p, float (&out)[4]) {
    float4 v = *reinterpret_cast<const float4*>(p);
    out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
  }
};
template <> struct Vec16<bf16_t> {
  static constexpr int N = 8;
  __device__ static __forceinline__ void load(const bf16_t* p, float (&out)[8]) {
    uint4 v = *reinterpret_cast<const uint4*>(p);
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      out[2 * i] = __uint_as_float(w[i] << 16);
      out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};

template <typename T> __device__ __forceinline__ float load_f32(const T* p);
template <> __device__ __forceinline__ float load_f32<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float load_f32<bf16_t>(const bf16_t* p) { return bf16_to_f32(p->bits); }

template <typename T> __device__ __forceinline__ void store_f32(T* p, float v);
template <> __device__ __forceinline__ void store_f32<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_f32<bf16_t>(bf16_t* p, float v) { p->bits = f32_to_bf16(v); }

// A lane's contiguous slice of N elements of a row, widened to float.  N*sizeof(T)
// is 8, 16 or 32 bytes and the address is aligned to it.
template <typename T, int N> __device__ __forceinline__ void load_slice(const T* p, float (&out)[N]);
template <> __device__ __forceinline__ void load_slice<float, 4>(const float* p, float (&out)[4]) {
  Vec16<float>::load(p, out);
}
template <> __device__ __forceinline__ void load_slice<float, 8>(const float* p, float (&out)[8]) {
  float a[4], b[4];
  Vec16<float>::load(p, a);
  Vec16<float>::load(p + 4, b);
#pragma unroll
  for (int i = 0; i < 4; ++i) { out[i] = a[i]; out[4 + i] = b[i]; }
}
template <> __device__ __forceinline__ void load_slice<bf16_t, 8>(const bf16_t* p, float (&out)[8]) {
  Vec16<bf16_t>::load(p, out);
}
template <> __device__ __forceinline__ void load_slice<bf16_t, 4>(const bf16_t* p, float (&out)[4]) {
  uint2 v = *reinterpret_cast<const uint2*>(p);
  out[0] = __uint_as_float(v.x << 16); out[1] = __uint_as_float(v.x & 0xffff0000u);
  out[2] = __uint_as_float(v.y << 16); out[3] = __uint_as_float(v.y & 0xffff0000u);
}

// Butterfly reductions over the low `width` lanes groups of a wave (width a power of two <= 64).
template <typename V> __device__ __forceinline__ V group_sum(V v, int width) {
  for (int o = width >> 1; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
template <typename V> __device__ __forceinline__ V group_max(V v, int width) {
  for (int o = width >> 1; o > 0; o >>= 1) {
    V u = __shfl_xor(v, o, kWave);
    v = u > v ? u : v;
  }
  return v;
}

}  // namespace tca

// Device-side helpers for the gfx950 kernels: storage-type loads, wave64
// reductions.  Wavefront size is 64 throughout.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tca {

constexpr int kWave = 64;

struct bf16_t { uint16_t bits; };   // storage only; arithmetic is done after widening

struct fp8_t { uint8_t bits; };     // OCP FP8 E4M3 code of the decode cache; read back as code * row scale

// Four E4M3 codes of one dword widened to float (two at a time on the conversion unit).
__device__ __forceinline__ void fp8x4_to_f32(uint32_t w, float& a, float& b, float& c, float& d) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false), hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true);
  a = lo.x; b = lo.y; c = hi.x; d = hi.y;
}
// Four floats (already divided by the row scale, magnitude <= 448 up to rounding) to four codes,
// round to nearest even; the clamp keeps a quotient that rounding pushed past 448 finite.
__device__ __forceinline__ uint32_t f32x4_to_fp8(float a, float b, float c, float d) {
  const float lim = 448.f;
  a = fminf(fmaxf(a, -lim), lim); b = fminf(fmaxf(b, -lim), lim);
  c = fminf(fmaxf(c, -lim), lim); d = fminf(fmaxf(d, -lim), lim);
  int p = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false);
  p = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, p, true);
  return (uint32_t)p;
}

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

// Raw 16-byte load and its later widening: lets many loads stay in flight at
// 4 registers each.
typedef unsigned int raw16_t __attribute__((ext_vector_type(4)));
template <typename T> __device__ __forceinline__ raw16_t load_raw16(const T* p) {
  return *reinterpret_cast<const raw16_t*>(p);
}
template <typename T> __device__ __forceinline__ void widen_raw16(raw16_t v, float (&out)[Vec16<T>::N]);
template <> __device__ __forceinline__ void widen_raw16<float>(raw16_t v, float (&out)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) out[i] = __uint_as_float(v[i]);
}
template <> __device__ __forceinline__ void widen_raw16<bf16_t>(raw16_t v, float (&out)[8]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    out[2 * i] = __uint_as_float(v[i] << 16);
    out[2 * i + 1] = __uint_as_float(v[i] & 0xffff0000u);
  }
}

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

// The same slice kept as loaded (N*sizeof(T) bytes) and widened when it is used, so that
// loads issued ahead of their use cost few registers.
template <typename T, int N>
struct RawSlice {
  static constexpr int W = N * (int)sizeof(T) / 4;       // dwords: 1, 2, 4 or 8
  uint32_t w[W];
  __device__ __forceinline__ void load(const T* p) {
    if constexpr (W == 1) {
      w[0] = *reinterpret_cast<const uint32_t*>(p);
    } else if constexpr (W == 2) {
      const uint2 v = *reinterpret_cast<const uint2*>(p);
      w[0] = v.x; w[1] = v.y;
    } else {
#pragma unroll
      for (int i = 0; i < W / 4; ++i) {
        const uint4 v = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(p) + 16 * i);
        w[4 * i] = v.x; w[4 * i + 1] = v.y; w[4 * i + 2] = v.z; w[4 * i + 3] = v.w;
      }
    }
  }
  __device__ __forceinline__ void widen(float (&out)[N]) const {
    if constexpr (sizeof(T) == 4) {
#pragma unroll
      for (int i = 0; i < N; ++i) out[i] = __uint_as_float(w[i]);
    } else if constexpr (sizeof(T) == 1) {
#pragma unroll
      for (int i = 0; i < W; ++i) fp8x4_to_f32(w[i], out[4 * i], out[4 * i + 1], out[4 * i + 2], out[4 * i + 3]);
    } else {
#pragma unroll
      for (int i = 0; i < W; ++i) {
        out[2 * i] = __uint_as_float(w[i] << 16);
        out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
      }
    }
  }
};

// Lane exchanges on the vector ALU (DPP), which are several times cheaper than
// the LDS-crossbar shuffles.  Patterns (all within a row of 16 lanes):
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <-> 7-i inside each group of 8
constexpr int kDppMirror = 0x140;     // lane i <-> 15-i inside the row
template <int CTRL> __device__ __forceinline__ float dpp_f32(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
template <int CTRL> __device__ __forceinline__ double dpp_f64(double v) {
  const long long b = __double_as_longlong(v);
  const int lo = __builtin_amdgcn_update_dpp(0, (int)(b & 0xffffffffll), CTRL, 0xF, 0xF, false);
  const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), CTRL, 0xF, 0xF, false);
  return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
// sum over the 16 lanes of a row, result in every lane
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_f32<kDppXor1>(v);
  v += dpp_f32<kDppXor2>(v);
  v += dpp_f32<kDppHalfMirror>(v);
  v += dpp_f32<kDppMirror>(v);
  return v;
}
__device__ __forceinline__ double row16_sum(double v) {
  v += dpp_f64<kDppXor1>(v);
  v += dpp_f64<kDppXor2>(v);
  v += dpp_f64<kDppHalfMirror>(v);
  v += dpp_f64<kDppMirror>(v);
  return v;
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

// Sum of G per-lane partials (G <= 16) over the LPR lanes that share a row (LPR = 8, 16 or 32
// consecutive lanes).  Exchange steps pair lane i with its mirror image inside
// groups of 32 (LDS shuffle), 16, 8 (DPP mirrors), then xor 2 and xor 1 (DPP quad
// permutes).  While a lane still carries more than one head, a step halves the
// heads it carries: the lower lane of a pair keeps the lower half.  The total of
// head g ends up in every lane whose position bits spell g.
template <int G, int LPR>
struct GroupReduce {
  static constexpr int GP = G <= 1 ? 1 : (G <= 2 ? 2 : (G <= 4 ? 4 : (G <= 8 ? 8 : 16)));   // padded to a power of two
  template <int W> __device__ static __forceinline__ double exchange(double v) {
    if constexpr (W == 32) return __shfl_xor(v, 31, kWave) ;   // i <-> 31-i inside 32 lanes
    else if constexpr (W == 16) return dpp_f64<kDppMirror>(v);
    else if constexpr (W == 8) return dpp_f64<kDppHalfMirror>(v);
    else if constexpr (W == 4) return dpp_f64<kDppXor2>(v);
    else return dpp_f64<kDppXor1>(v);
  }
  // is this lane the upper one of its pair at width W?
  template <int W> __device__ static __forceinline__ bool upper(int sub) {
    if constexpr (W >= 8) return (sub & (W - 1)) >= W / 2;
    else return (sub & (W / 2)) != 0;
  }
  template <int W, int N> __device__ static __forceinline__ void step(double (&acc)[GP], int sub) {
    if constexpr (W >= 2) {
      if constexpr (N > 1) {
        const bool hi = upper<W>(sub);
#pragma unroll
        for (int i = 0; i < N / 2; ++i) {
          const double send = hi ? acc[i] : acc[i + N / 2];
          const double keep = hi ? acc[i + N / 2] : acc[i];
          acc[i] = keep + exchange<W>(send);
        }
        step<W / 2, N / 2>(acc, sub);
      } else {
        acc[0] += exchange<W>(acc[0]);
        step<W / 2, 1>(acc, sub);
      }
    }
  }
  __device__ static __forceinline__ double run(double (&acc)[GP], int sub) {
    step<LPR, GP>(acc, sub);
    return acc[0];
  }
  template <int W, int N> __device__ static __forceinline__ int head_bits(int sub, int g) {
    if constexpr (W >= 2 && N > 1) return head_bits<W / 2, N / 2>(sub, (g << 1) | (upper<W>(sub) ? 1 : 0));
    else return g;
  }
  // head whose total this lane holds after run()
  __device__ static __forceinline__ int head_of(int sub) { return head_bits<LPR, GP>(sub, 0); }
};


}  // namespace tca

// 16-byte row fragments: one lane moves 4 fp32 or 8 fp16 table elements per load.
#pragma once

#include "common.h"

namespace hctr {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <typename T>
struct RowVec;

// load = load_raw + widen.  Kernels that keep several row loads in flight call load_raw for all of
// them first and widen afterwards: a conversion (or any use) right behind a load that sits under a
// branch makes the compiler wait for that load before it issues the next one.
template <>
struct RowVec<float> {
  static constexpr int VEC = 4;
  typedef f32x4 Raw;
  __device__ static __forceinline__ Raw load_raw(const float* p) { return *reinterpret_cast<const f32x4*>(p); }
  __device__ static __forceinline__ void widen(const Raw& x, float (&v)[4]) {
    v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
  }
  __device__ static __forceinline__ void load(const float* p, float (&v)[4]) { widen(load_raw(p), v); }
};

__device__ __forceinline__ float half_bits_to_float(uint32_t h16) {
  return __half2float(__ushort_as_half((unsigned short)h16));
}

template <>
struct RowVec<__half> {
  static constexpr int VEC = 8;
  typedef u32x4 Raw;
  __device__ static __forceinline__ Raw load_raw(const __half* p) { return *reinterpret_cast<const u32x4*>(p); }
  __device__ static __forceinline__ void widen(const Raw& x, float (&v)[8]) {
    const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = half_bits_to_float(w[i] & 0xFFFFu);
      v[2 * i + 1] = half_bits_to_float(w[i] >> 16);
    }
  }
  __device__ static __forceinline__ void load(const __half* p, float (&v)[8]) { widen(load_raw(p), v); }
};

// Streaming store of N consecutive floats (N = 4 or 8): the pooled output is written once and not
// read again by this library, so it should not displace table rows from L2.
template <int N>
__device__ __forceinline__ void store_stream(float* p, const float (&v)[N]) {
#pragma unroll
  for (int i = 0; i < N; i += 4) {
    f32x4 x = {v[i], v[i + 1], v[i + 2], v[i + 3]};
    __builtin_nontemporal_store(x, reinterpret_cast<f32x4*>(p + i));
  }
}

// The same into an fp16 output: N floats rounded to nearest even, 2 * N bytes.
template <int N>
__device__ __forceinline__ void store_stream(__half* p, const float (&v)[N]) {
  uint32_t w[N / 2];
#pragma unroll
  for (int i = 0; i < N / 2; ++i)
    w[i] = (uint32_t)__half_as_ushort(__float2half_rn(v[2 * i])) |
           ((uint32_t)__half_as_ushort(__float2half_rn(v[2 * i + 1])) << 16);
  if constexpr (N == 4) {
    u32x2 x = {w[0], w[1]};
    __builtin_nontemporal_store(x, reinterpret_cast<u32x2*>(p));
  } else {
#pragma unroll
    for (int i = 0; i < N / 2; i += 4) {
      u32x4 x = {w[i], w[i + 1], w[i + 2], w[i + 3]};
      __builtin_nontemporal_store(x, reinterpret_cast<u32x4*>(p + 2 * i));
    }
  }
}

template <int N>
__device__ __forceinline__ void store_plain(float* p, const float (&v)[N]) {
#pragma unroll
  for (int i = 0; i < N; i += 4) *reinterpret_cast<f32x4*>(p + i) = f32x4{v[i], v[i + 1], v[i + 2], v[i + 3]};
}

__device__ __forceinline__ f32x4 load4(const float* p) { return *reinterpret_cast<const f32x4*>(p); }
__device__ __forceinline__ void store4(float* p, f32x4 x) { *reinterpret_cast<f32x4*>(p) = x; }

// 4 table elements widened to fp32 / narrowed from fp32 (round to nearest even).
__device__ __forceinline__ f32x4 load_row4(const float* t) { return load4(t); }
__device__ __forceinline__ void store_row4(float* t, f32x4 x) { store4(t, x); }
__device__ __forceinline__ f32x4 load_row4(const __half* t) {
  u32x2 raw = *reinterpret_cast<const u32x2*>(t);
  return f32x4{half_bits_to_float(raw.x & 0xFFFFu), half_bits_to_float(raw.x >> 16),
               half_bits_to_float(raw.y & 0xFFFFu), half_bits_to_float(raw.y >> 16)};
}
__device__ __forceinline__ void store_row4(__half* t, f32x4 x) {
  u32x2 o;
  o.x = (uint32_t)__half_as_ushort(__float2half_rn(x.x)) | ((uint32_t)__half_as_ushort(__float2half_rn(x.y)) << 16);
  o.y = (uint32_t)__half_as_ushort(__float2half_rn(x.z)) | ((uint32_t)__half_as_ushort(__float2half_rn(x.w)) << 16);
  *reinterpret_cast<u32x2*>(t) = o;
}

// Streaming (non-temporal) read of 4 gradient elements, widened to fp32, for rows that are read
// exactly once: the load does not displace what is reused (headline backward 0.329 -> 0.293 ms).
__device__ __forceinline__ f32x4 load_stream4(const float* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
}
__device__ __forceinline__ f32x4 load_stream4(const __half* p) {
  const u32x2 raw = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p));
  return f32x4{half_bits_to_float(raw.x & 0xFFFFu), half_bits_to_float(raw.x >> 16),
               half_bits_to_float(raw.y & 0xFFFFu), half_bits_to_float(raw.y >> 16)};
}

// Four elements as a load brings them, before they are widened to fp32 (fp32: four words; fp16: the
// first two words hold four halves).  The backward kernels request all pieces of a step raw and
// widen them afterwards, for the reason given at RowVec.  The pointer argument of widen4 only
// selects the element type.
struct Raw4 { u32x4 bits; };
__device__ __forceinline__ Raw4 load_raw4(const float* p) { return Raw4{*reinterpret_cast<const u32x4*>(p)}; }
__device__ __forceinline__ Raw4 load_raw4(const __half* p) {
  const u32x2 x = *reinterpret_cast<const u32x2*>(p);
  return Raw4{u32x4{x.x, x.y, 0u, 0u}};
}
__device__ __forceinline__ Raw4 load_stream_raw4(const float* p) {
  return Raw4{__builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p))};
}
__device__ __forceinline__ Raw4 load_stream_raw4(const __half* p) {
  const u32x2 x = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p));
  return Raw4{u32x4{x.x, x.y, 0u, 0u}};
}
__device__ __forceinline__ f32x4 widen4(const Raw4& r, const float*) {
  return f32x4{__uint_as_float(r.bits.x), __uint_as_float(r.bits.y), __uint_as_float(r.bits.z),
               __uint_as_float(r.bits.w)};
}
__device__ __forceinline__ f32x4 widen4(const Raw4& r, const __half*) {
  return f32x4{half_bits_to_float(r.bits.x & 0xFFFFu), half_bits_to_float(r.bits.x >> 16),
               half_bits_to_float(r.bits.y & 0xFFFFu), half_bits_to_float(r.bits.y >> 16)};
}

// Read-modify-write of 4 table elements: t <- t - lr * g (fp16 storage: widen, update in fp32,
// round to nearest even).
__device__ __forceinline__ void sgd_update4(float* t, f32x4 g, float lr) {
  f32x4 x = load4(t);
  x.x -= lr * g.x; x.y -= lr * g.y; x.z -= lr * g.z; x.w -= lr * g.w;
  store4(t, x);
}
__device__ __forceinline__ void sgd_update4(__half* t, f32x4 g, float lr) {
  u32x2 raw = *reinterpret_cast<const u32x2*>(t);
  float a = half_bits_to_float(raw.x & 0xFFFFu) - lr * g.x;
  float b = half_bits_to_float(raw.x >> 16) - lr * g.y;
  float c = half_bits_to_float(raw.y & 0xFFFFu) - lr * g.z;
  float d = half_bits_to_float(raw.y >> 16) - lr * g.w;
  u32x2 o;
  o.x = (uint32_t)__half_as_ushort(__float2half_rn(a)) | ((uint32_t)__half_as_ushort(__float2half_rn(b)) << 16);
  o.y = (uint32_t)__half_as_ushort(__float2half_rn(c)) | ((uint32_t)__half_as_ushort(__float2half_rn(d)) << 16);
  *reinterpret_cast<u32x2*>(t) = o;
}

}  // namespace hctr

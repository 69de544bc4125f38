// Device-side helpers shared by the cosine-attention kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cotten {

// bfloat16 storage type: the upper 16 bits of an IEEE float.
struct bf16 {
  uint16_t bits;
};

// IEEE half storage type.
struct f16 {
  uint16_t bits;
};

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(f16 x) {
  return static_cast<float>(__builtin_bit_cast(_Float16, x.bits));
}
__device__ __forceinline__ float to_float(bf16 x) {
  return __uint_as_float(static_cast<uint32_t>(x.bits) << 16);
}

template <typename T>
__device__ __forceinline__ T from_float(float x);
template <>
__device__ __forceinline__ float from_float<float>(float x) {
  return x;
}
// Round to nearest even; NaN stays NaN (quiet bit forced).
template <>
__device__ __forceinline__ bf16 from_float<bf16>(float x) {
  uint32_t u = __float_as_uint(x);
  bf16 r;
  if ((u & 0x7fffffffu) > 0x7f800000u) {
    r.bits = static_cast<uint16_t>((u >> 16) | 0x0040u);
  } else {
    u += 0x7fffu + ((u >> 16) & 1u);
    r.bits = static_cast<uint16_t>(u >> 16);
  }
  return r;
}

// Round to nearest even (hardware conversion); values beyond the half range become Inf.
template <>
__device__ __forceinline__ f16 from_float<f16>(float x) {
  f16 r;
  r.bits = __builtin_bit_cast(uint16_t, static_cast<_Float16>(x));
  return r;
}

// CH consecutive elements of type T moved as one aligned vector (16 bytes per
// instruction where CH * sizeof(T) allows it).
template <typename T, int CH>
struct alignas((CH * sizeof(T)) >= 16 ? 16 : (CH * sizeof(T))) Chunk {
  T v[CH];
};

template <typename T, int CH>
__device__ __forceinline__ void load_chunk(const T* __restrict__ p, float (&out)[CH]) {
  const Chunk<T, CH> c = *reinterpret_cast<const Chunk<T, CH>*>(p);
#pragma unroll
  for (int i = 0; i < CH; ++i) out[i] = to_float(c.v[i]);
}

template <typename T, int CH>
__device__ __forceinline__ void store_chunk(T* __restrict__ p, const float (&in)[CH]) {
  Chunk<T, CH> c;
#pragma unroll
  for (int i = 0; i < CH; ++i) c.v[i] = from_float<T>(in[i]);
  *reinterpret_cast<Chunk<T, CH>*>(p) = c;
}

// Sum over the 8 consecutive lanes that share one row.
__device__ __forceinline__ float sum8(float x) {
  x += __shfl_xor(x, 1);
  x += __shfl_xor(x, 2);
  x += __shfl_xor(x, 4);
  return x;
}

// 1 / sqrt(ss + eps) with IEEE square root and division (no fast-math).
__device__ __forceinline__ float inv_norm(float ss, float eps) {
  return 1.0f / sqrtf(ss + eps);
}

}  // namespace cotten

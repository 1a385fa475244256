// Device helpers shared by the matrix-product kernels: activations, operand loads with bounds
// and alignment handling, and the rounding of float32 operands to bf16.
#pragma once

#include "common.h"

namespace pfg {
namespace dev {

enum AMode : int { A_F32 = 0, A_BF16 = 1, A_F32_TO_BF16 = 2 };

__device__ __forceinline__ float act_value(int act, float z) {
  switch (act) {
    case ACT_RELU: return z > 0.f ? z : 0.f;
    case ACT_TANH: return tanhf(z);
    case ACT_GELU: return 0.5f * z * (1.f + erff(z * 0.70710678118654752440f));
    default: return z;
  }
}

__device__ __forceinline__ float act_deriv(int act, float z) {
  switch (act) {
    case ACT_RELU: return z > 0.f ? 1.f : 0.f;
    case ACT_TANH: { float t = tanhf(z); return 1.f - t * t; }
    case ACT_GELU: {
      float Phi = 0.5f * (1.f + erff(z * 0.70710678118654752440f));
      float pdf = 0.39894228040143267794f * __expf(-0.5f * z * z);
      return Phi + z * pdf;
    }
    default: return 1.f;
  }
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 v = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, v);
}

// Up to 16 bytes of one operand row, k in [k0, k0 + n): float32 source.
__device__ __forceinline__ f32x4 load4_f32(const float *row, int k0, int K, bool vec_ok) {
  f32x4 v = {0.f, 0.f, 0.f, 0.f};
  if (row == nullptr) return v;
  if (vec_ok && k0 + 4 <= K) {
    v = *reinterpret_cast<const f32x4 *>(row + k0);
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (k0 + e < K) v[e] = row[k0 + e];
  }
  return v;
}

__device__ __forceinline__ u32x4 load8_bf16(const __bf16 *row, int k0, int K, bool vec_ok) {
  u32x4 v = {0u, 0u, 0u, 0u};
  if (row == nullptr) return v;
  if (vec_ok && k0 + 8 <= K) {
    v = *reinterpret_cast<const u32x4 *>(row + k0);
  } else {
    const uint16_t *r16 = reinterpret_cast<const uint16_t *>(row);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      uint32_t bits = (k0 + e < K) ? (uint32_t)r16[k0 + e] : 0u;
      v[e >> 1] |= bits << ((e & 1) * 16);
    }
  }
  return v;
}

// Raw registers of one 16-byte LDS chunk of the A operand, before scaling / rounding.
template <int AMODE> struct RawA;
template <> struct RawA<A_F32> { f32x4 v, s; };
template <> struct RawA<A_BF16> { u32x4 v; };
template <> struct RawA<A_F32_TO_BF16> { f32x4 v0, v1, s0, s1; };

template <int AMODE>
__device__ __forceinline__ RawA<AMODE> fetch_a(const void *row, const float *srow, int k0, int K,
                                               bool vec_ok, bool svec_ok) {
  RawA<AMODE> r;
  if constexpr (AMODE == A_F32) {
    r.v = load4_f32(static_cast<const float *>(row), k0, K, vec_ok);
    if (srow) r.s = load4_f32(srow, k0, K, svec_ok);
  } else if constexpr (AMODE == A_BF16) {
    r.v = load8_bf16(static_cast<const __bf16 *>(row), k0, K, vec_ok);
  } else {
    r.v0 = load4_f32(static_cast<const float *>(row), k0, K, vec_ok);
    r.v1 = load4_f32(static_cast<const float *>(row), k0 + 4, K, vec_ok);
    if (srow) {
      r.s0 = load4_f32(srow, k0, K, svec_ok);
      r.s1 = load4_f32(srow, k0 + 4, K, svec_ok);
    }
  }
  return r;
}

template <int AMODE>
__device__ __forceinline__ u32x4 finish_a(const RawA<AMODE> &r, bool scaled) {
  if constexpr (AMODE == A_F32) {
    f32x4 v = scaled ? r.v * r.s : r.v;
    return __builtin_bit_cast(u32x4, v);
  } else if constexpr (AMODE == A_BF16) {
    return r.v;
  } else {
    f32x4 a = scaled ? r.v0 * r.s0 : r.v0;
    f32x4 b = scaled ? r.v1 * r.s1 : r.v1;
    u32x4 o = {pack_bf16(a[0], a[1]), pack_bf16(a[2], a[3]), pack_bf16(b[0], b[1]),
               pack_bf16(b[2], b[3])};
    return o;
  }
}

}  // namespace dev
}  // namespace pfg

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

// phi''(z); 0 for the piecewise-linear activations (also at the kink of ReLU)
__device__ __forceinline__ float act_deriv2(int act, float z) {
  switch (act) {
    case ACT_TANH: { float t = tanhf(z); return -2.f * t * (1.f - t * t); }
    case ACT_GELU: return 0.39894228040143267794f * __expf(-0.5f * z * z) * (2.f - z * z);
    default: return 0.f;
  }
}

// Reverse LSTM cell update of step t for row m (example m / S), unit k, given dh = the cotangent of
// that step's hidden state:
//   dc   += dh * o * (1 - tanh(c_t)^2)
//   dz_o  = dh * tanh(c_t) * o (1 - o)
//   dz_i  = dc * g * i (1 - i),  dz_g = dc * i * (1 - g^2),  dz_f = dc * c_{t-1} * f (1 - f)
//   dc_{t-1} = dc * f
// The same update on values already in registers.
// seed: added to the cotangent of the hidden state before the update (an iteration of a while loop
// enters the reverse loop at its own last trip with the cotangent of its final state)
struct LstmCellIn { float i, g, f, o, c, cprev, dc, seed; };
// dz_row2 (may be nullptr): a second row that receives the same four values
__device__ __forceinline__ void lstm_reverse_cell_store(const LstmCellIn &v, float dh, float *dz_row,
                                                        float *dcp, int H, int k, float *dz_row2 = nullptr) {
  const float tc = tanhf(v.c);
  const float dct = v.dc + dh * v.o * (1.f - tc * tc);
  const float zi = dct * v.g * v.i * (1.f - v.i), zg = dct * v.i * (1.f - v.g * v.g);
  const float zf = dct * v.cprev * v.f * (1.f - v.f), zo = dh * tc * v.o * (1.f - v.o);
  dz_row[k] = zi;
  dz_row[H + k] = zg;
  dz_row[2 * H + k] = zf;
  dz_row[3 * H + k] = zo;
  if (dz_row2) {
    dz_row2[k] = zi;
    dz_row2[H + k] = zg;
    dz_row2[2 * H + k] = zf;
    dz_row2[3 * H + k] = zo;
  }
  *dcp = dct * v.f;
}

__device__ __forceinline__ void lstm_reverse_cell(const float *gates, const float *cs, float *dc,
                                                  float *dz, int64_t dz_ld, int H, int T, int t,
                                                  int S, int m, int k, float dh) {
  const int64_t b = m / S;
  const float *grow = gates + (b * T + t) * 4 * (int64_t)H;
  const float i = grow[k], g = grow[H + k], f = grow[2 * H + k], o = grow[3 * H + k];
  const float tc = tanhf(cs[(b * T + t) * (int64_t)H + k]);
  const float cprev = t > 0 ? cs[(b * T + t - 1) * (int64_t)H + k] : 0.f;
  float *dcp = dc + (int64_t)m * H + k;
  const float dct = *dcp + dh * o * (1.f - tc * tc);
  float *out = dz + (int64_t)m * dz_ld;
  out[k] = dct * g * i * (1.f - i);
  out[H + k] = dct * i * (1.f - g * g);
  out[2 * H + k] = dct * cprev * f * (1.f - f);
  out[3 * H + k] = dh * tc * o * (1.f - o);
  *dcp = dct * f;
}

// The same update for four consecutive hidden units k .. k + 3 on 16-byte operands (all row starts
// and k must be 16-byte aligned: H, dz_ld multiples of 4).
__device__ __forceinline__ void lstm_reverse_cell4(const float *gates, const float *cs, float *dc,
                                                   float *dz, int64_t dz_ld, int H, int T, int t,
                                                   int S, int m, int k, f32x4 dh) {
  const int64_t b = m / S;
  const float *grow = gates + (b * T + t) * 4 * (int64_t)H + k;
  const f32x4 i = *reinterpret_cast<const f32x4 *>(grow);
  const f32x4 g = *reinterpret_cast<const f32x4 *>(grow + H);
  const f32x4 f = *reinterpret_cast<const f32x4 *>(grow + 2 * H);
  const f32x4 o = *reinterpret_cast<const f32x4 *>(grow + 3 * H);
  const f32x4 c = *reinterpret_cast<const f32x4 *>(cs + (b * T + t) * (int64_t)H + k);
  f32x4 cprev = {0.f, 0.f, 0.f, 0.f};
  if (t > 0) cprev = *reinterpret_cast<const f32x4 *>(cs + (b * T + t - 1) * (int64_t)H + k);
  f32x4 *dcp = reinterpret_cast<f32x4 *>(dc + (int64_t)m * H + k);
  f32x4 tc;
#pragma unroll
  for (int q = 0; q < 4; ++q) tc[q] = tanhf(c[q]);
  const f32x4 dct = *dcp + dh * o * (1.f - tc * tc);
  float *out = dz + (int64_t)m * dz_ld + k;
  *reinterpret_cast<f32x4 *>(out) = dct * g * i * (1.f - i);
  *reinterpret_cast<f32x4 *>(out + H) = dct * i * (1.f - g * g);
  *reinterpret_cast<f32x4 *>(out + 2 * H) = dct * cprev * f * (1.f - f);
  *reinterpret_cast<f32x4 *>(out + 3 * H) = dh * tc * o * (1.f - o);
  *dcp = dct * f;
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 v = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, v);
}

// Operand loads come in two flavours, chosen per launch on the host.
//
// FAST: every operand is 16-byte aligned with 16-byte-multiple strides and the contraction length
// is a multiple of the chunk, so a chunk is either wholly inside or wholly outside the row.  The
// load is then one unconditional 16-byte load from a clamped address (chunks past the end are
// zeroed when the registers are consumed): no branch, nothing that would make the compiler wait
// for earlier loads, so many loads stay in flight.  Row pointers are never null (out-of-range rows are clamped to the last row; what they
// produce is never stored).
//
// General: any alignment and length; element-wise loads with bounds checks where needed.

// The FAST loads return whatever sits at the clamped address; the caller zeroes a chunk whose
// k0 is past the end LATER, when it consumes the registers (a select placed here would make
// the compiler wait for the load at once and serialise all loads of a stage).
__device__ __forceinline__ f32x4 load4_f32_fast(const float *row, int k0, int K) {
  return *reinterpret_cast<const f32x4 *>(row + min(k0, K - 4));
}

__device__ __forceinline__ u32x4 load8_bf16_fast(const __bf16 *row, int k0, int K) {
  return *reinterpret_cast<const u32x4 *>(row + min(k0, K - 8));
}

// Up to 16 bytes of one operand row, k in [k0, k0 + 4): float32 source (nullptr row = zeros).
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

template <bool FAST>
__device__ __forceinline__ f32x4 ld4(const float *row, int k0, int K, bool vec_ok) {
  if constexpr (FAST) return load4_f32_fast(row, k0, K);
  else return load4_f32(row, k0, K, vec_ok);
}

template <bool FAST>
__device__ __forceinline__ u32x4 ld8(const __bf16 *row, int k0, int K, bool vec_ok) {
  if constexpr (FAST) return load8_bf16_fast(row, k0, K);
  else return load8_bf16(row, k0, K, vec_ok);
}

// Raw registers of one 16-byte LDS chunk of the A operand, before scaling / rounding.
template <int AMODE> struct RawA;
template <> struct RawA<A_F32> { f32x4 v, s; };
template <> struct RawA<A_BF16> { u32x4 v; };
template <> struct RawA<A_F32_TO_BF16> { f32x4 v0, v1, s0, s1; };

// scaled is uniform over the workgroup (a scale operand exists); a null srow (general loads, row
// out of range) reads as zeros.
template <int AMODE, bool FAST>
__device__ __forceinline__ RawA<AMODE> fetch_a(const void *row, const float *srow, bool scaled,
                                               int k0, int K, bool vec_ok, bool svec_ok) {
  RawA<AMODE> r;
  if constexpr (AMODE == A_F32) {
    r.v = ld4<FAST>(static_cast<const float *>(row), k0, K, vec_ok);
    if (scaled) r.s = ld4<FAST>(srow, k0, K, svec_ok);
  } else if constexpr (AMODE == A_BF16) {
    r.v = ld8<FAST>(static_cast<const __bf16 *>(row), k0, K, vec_ok);
  } else {
    r.v0 = ld4<FAST>(static_cast<const float *>(row), k0, K, vec_ok);
    r.v1 = ld4<FAST>(static_cast<const float *>(row), k0 + 4, K, vec_ok);
    if (scaled) {
      r.s0 = ld4<FAST>(srow, k0, K, svec_ok);
      r.s1 = ld4<FAST>(srow, k0 + 4, K, svec_ok);
    }
  }
  return r;
}

// Host side: may this product take the FAST loads?  check_w = false leaves W out of it (for a
// kernel that reads W element by element).
inline bool fast_loads_ok(const GemmArgs &g, bool check_w = true) {
  const int a_elem = (g.bf16 && !g.a_is_f32) ? 2 : 4;
  const int w_elem = g.bf16 ? 2 : 4;
  const int kchunk = g.bf16 ? 8 : 4;          // k elements per 16-byte LDS chunk
  auto aligned = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
  if (!aligned(g.A) || (g.lda * a_elem) % 16 || (g.a_batch_stride * a_elem) % 16) return false;
  if (g.a_scale && (!aligned(g.a_scale) || (g.ld_scale * 4) % 16)) return false;
  if (g.nbatch > 1 && ((g.batch_A * a_elem) % 16 || (g.batch_W * w_elem) % 16 ||
                       (g.batch_scale * 4) % 16))
    return false;
  if (g.K % kchunk || g.K < kchunk) return false;
  if (!check_w) return true;
  if (!aligned(g.W) || (g.ldw * w_elem) % 16) return false;
  if (g.w_kn && (g.N % (16 / w_elem) || g.N < 16 / w_elem)) return false;
  return true;
}

// zero: the chunk lies past the end of the contraction (FAST loads only; the general loads
// zero-fill by themselves).
template <int AMODE>
__device__ __forceinline__ u32x4 finish_a(const RawA<AMODE> &r, bool scaled, bool zero = false) {
  if (zero) return u32x4{0u, 0u, 0u, 0u};
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

// Cotangent step through the last layer for the 32 rows of a head tile, on the vector ALUs (the
// contraction is only N <= 32 = 4 N4 long):
//     g_prev[m, i] = phi'(z[m, i]) * sum_j delta[m, j] * W[i, j]
// The columns i of one tile are shared out over the `groups` workgroups that computed the same
// tile (group index `cg`); inside a workgroup a thread owns one column and one band of rows
// (consecutive threads store consecutive i of a row).  It keeps W[i, :] in registers; delta rows
// come from LDS (zero beyond N); the mask value of the next row is requested while the current
// one is computed.
// AHEAD: mask values requested ahead of the row being computed (1: the next row's, for callers
// that want the loop short; 4: four rows' at a time, for walks that are pure memory latency).
template <int N4, int NT, int AHEAD = 1>
__device__ __forceinline__ void head_cotangent(const GemmArgs &g, const float (*hd)[32], int m0,
                                               int tile_rows, int tid, int cg, int groups) {
  const int K = g.K, N = g.N;
  const int cols = (K + groups - 1) / groups;            // columns of this workgroup
  const int c_begin = cg * cols, c_end = min(c_begin + cols, K);
  const int bands = cols >= NT ? 1 : NT / cols;          // row bands worked on side by side
  const int band = cols >= NT ? 0 : tid / cols;
  const int c_first = c_begin + (cols >= NT ? tid : tid - band * cols);
  if (band >= bands) return;
  const int rows_per_band = (tile_rows + bands - 1) / bands;
  const int r_begin = band * rows_per_band, r_end = min(r_begin + rows_per_band, tile_rows);
  if (r_begin >= r_end) return;
#pragma unroll 1
  for (int i = c_first; i < c_end; i += NT) {
    float w[4 * N4];
#pragma unroll
    for (int j = 0; j < 4 * N4; ++j) {
      const int64_t at = (int64_t)i * g.ldw + min(j, N - 1);      // clamped: delta is 0 there
      w[j] = g.bf16 ? (float)static_cast<const __bf16 *>(g.W)[at] : static_cast<const float *>(g.W)[at];
    }
    const float *mcol = g.head_mask + (int64_t)m0 * K + i;
    float *gcol = g.head_gprev + (int64_t)m0 * K + i;
    if constexpr (AHEAD > 1) {
#pragma unroll 1
      for (int r0 = r_begin; r0 < r_end; r0 += AHEAD) {
        float mv[AHEAD];
#pragma unroll
        for (int u = 0; u < AHEAD; ++u) mv[u] = mcol[(int64_t)min(r0 + u, r_end - 1) * K];
#pragma unroll
        for (int u = 0; u < AHEAD; ++u) {
          const int r = r0 + u;
          if (r < r_end) {
            float acc = 0.f;
#pragma unroll
            for (int j4 = 0; j4 < N4; ++j4) {
              const f32x4 dv = *reinterpret_cast<const f32x4 *>(&hd[r][4 * j4]);
              acc += dv[0] * w[4 * j4] + dv[1] * w[4 * j4 + 1] + dv[2] * w[4 * j4 + 2] + dv[3] * w[4 * j4 + 3];
            }
            gcol[(int64_t)r * K] = acc * mv[u];
          }
        }
      }
      continue;
    }
    float nxt = mcol[(int64_t)r_begin * K];
#pragma unroll 1
    for (int r = r_begin; r < r_end; ++r) {
      const float cur = nxt;
      nxt = mcol[(int64_t)min(r + 1, r_end - 1) * K];
      float acc = 0.f;
#pragma unroll
      for (int j4 = 0; j4 < N4; ++j4) {
        const f32x4 dv = *reinterpret_cast<const f32x4 *>(&hd[r][4 * j4]);
        acc += dv[0] * w[4 * j4] + dv[1] * w[4 * j4 + 1] + dv[2] * w[4 * j4 + 2] + dv[3] * w[4 * j4 + 3];
      }
      gcol[(int64_t)r * K] = acc * cur;
    }
  }
}

}  // namespace dev
}  // namespace pfg

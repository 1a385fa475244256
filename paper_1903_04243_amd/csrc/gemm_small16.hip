// Matrix product for problems so small that even 32 x 32 tiles leave most compute units idle
// (a 128 x 512 output is 64 such tiles on 256 units, and float32 MFMA throughput on 64 units is
// then a visible part of a few-microsecond kernel).  Same scheme as the 32 x 32 small-problem
// kernel -- a workgroup owns one tile of C, its waves split the contraction index, operands go
// from global memory straight to MFMA registers, partial tiles are summed in a fixed order through
// LDS -- with 16 x 16 tiles on v_mfma_f32_16x16x4_f32, i.e. four times as many workgroups.
// float32 operands only; epilogues EPI_NONE, EPI_BIAS, EPI_FORWARD, EPI_MASK and (LSTM
// instantiation) EPI_LSTM_BWD; no A scaling, no batching.  Rows chosen on the device (GemmArgs::sub)
// are supported.
//
// Operand layout of the 16 x 16 x 4 MFMA: lane l supplies A[l % 16][l / 16] and B[l / 16][l % 16] and
// receives D[4 (l / 16) + r][l % 16] in accumulator register r.  A lane loads 16 bytes = four
// consecutive k of its row (column) per slice of 16 k and feeds element j to MFMA j of the slice;
// both operands use the same assignment of k to (lane quarter, j), which is all a contraction needs.
#include "common.h"
#include "gemm_device.h"

namespace pfg {

namespace {

using namespace dev;

constexpr int kRing = 4;      // slices in flight per wave

// SUB: the instantiation for rows chosen on the device (GemmArgs::sub), kept apart so that the
// others carry none of its loads and branches.
// BATCH: the instantiation for batched products (the second grid index selects the entry; operands
// at fixed strides, EPI_NONE), apart for the same reason.
template <bool WKN, int NW, bool LSTM, bool SUB, bool BATCH = false>
__global__ __launch_bounds__(64 * NW) void gemm_small16_kernel(const GemmArgs g) {
  __shared__ float red[NW][16][17];
  const float *gA = static_cast<const float *>(g.A), *gW = static_cast<const float *>(g.W);
  float *gC = g.C;
  if constexpr (BATCH) {
    const int64_t z = blockIdx.y;
    gA += z * g.batch_A;
    gW += z * g.batch_W;
    gC += z * g.batch_C;
  }

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, kq = lane >> 4;
  const int N = g.N, K = g.K;
  const int tiles_m = (g.M + 15) / 16;
  // rows chosen on the device: the column tiles of a row tile are numbered next to each other, so that
  // the live workgroups (the first row tiles) come first in the launch
  const int tiles_n = SUB ? (int)gridDim.x / tiles_m : 1;
  const int m0 = (SUB ? (int)blockIdx.x / tiles_n : (int)blockIdx.x % tiles_m) * 16;
  const int n0 = (SUB ? (int)blockIdx.x % tiles_n : (int)blockIdx.x / tiles_m) * 16;
  const int epi = g.epilogue;
  // rows chosen on the device: the live row count comes from memory, tiles past it have nothing to do
  const int M = SUB ? g.sub[0] : g.M;
  if (SUB && m0 >= M) return;
  const int sub_off = SUB ? g.sub[1] : 0;

  // operand rows of this lane (clamped: what out-of-range rows and columns produce is not stored)
  int mc = min(m0 + r16, M - 1);
  if (SUB && g.sub_gather) mc = g.sub_rows[sub_off + mc];
  const int nc = min(n0 + r16, N - 1);
  const float *a_row = gA + (int64_t)(mc / g.S) * g.a_batch_stride +
                       (int64_t)(mc % g.S) * g.lda;
  const float *W = gW;
  const float *w_row = WKN ? W + nc : W + (int64_t)nc * g.ldw;      // column nc of [K, N] / row nc of [N, K]
  const bool a_vec = ((reinterpret_cast<uintptr_t>(gA) & 15) == 0) && (g.lda % 4 == 0) &&
                     (g.a_batch_stride % 4 == 0) && (K % 4 == 0);
  const bool w_vec = !WKN && ((reinterpret_cast<uintptr_t>(gW) & 15) == 0) && (g.ldw % 4 == 0) &&
                     (K % 4 == 0);

  // Epilogue assignment: thread t < 256 finishes element (t / 16, t % 16); what it needs from global
  // memory for that is requested here, ahead of the contraction.
  const int erow = tid >> 4, ecol = tid & 15;
  const int em = m0 + erow, en = n0 + ecol;
  const bool elive = tid < 256 && em < M && en < N;
  float aux = (epi == EPI_MASK) ? 1.f : 0.f;
  if (elive) {
    if ((epi == EPI_BIAS || epi == EPI_FORWARD) && g.bias) aux = static_cast<const float *>(g.bias)[en];
    if (epi == EPI_MASK) aux = g.emask[(int64_t)(em / g.S) * g.ld_emask + en];
  }
  LstmCellIn cell{};
  if constexpr (LSTM) {
    if (elive && epi == EPI_LSTM_BWD && en >= g.n_split) {
      const int H = g.lstm_H, T = g.lstm_T, t = g.lstm_step, k = en - g.n_split;
      const int64_t b = em / g.S;
      const float *grow = g.lstm_gates + (b * T + t) * 4 * (int64_t)H;
      const float *crow = g.lstm_cs + (b * T + t) * (int64_t)H;
      cell.i = grow[k]; cell.g = grow[H + k]; cell.f = grow[2 * H + k]; cell.o = grow[3 * H + k];
      cell.c = crow[k];
      cell.cprev = t > 0 ? crow[k - H] : 0.f;
      cell.dc = g.lstm_dc[(int64_t)em * H + k];
    }
  }

  // One slice = 16 consecutive k; this lane's four are k0 + 4 kq .. + 3.
  auto load = [&](int slice, f32x4 &a, f32x4 &w) {
    const int k0 = slice * 16 + 4 * kq;
    if (a_vec) {
      a = *reinterpret_cast<const f32x4 *>(a_row + min(k0, K - 4));         // zeroed at use if past K
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) a[e] = a_row[min(k0 + e, K - 1)];
    }
    if constexpr (WKN) {
#pragma unroll
      for (int e = 0; e < 4; ++e) w[e] = w_row[(int64_t)min(k0 + e, K - 1) * g.ldw];
    } else {
      if (w_vec) {
        w = *reinterpret_cast<const f32x4 *>(w_row + min(k0, K - 4));
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = w_row[min(k0 + e, K - 1)];
      }
    }
  };

  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  auto compute = [&](int slice, f32x4 a, f32x4 w) {
    const int k0 = slice * 16 + 4 * kq;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      // clamped loads repeat the last values past the end of the contraction: drop them here
      const float a_e = (k0 + e < K) ? a[e] : 0.f;
      const float w_e = w[e];
      acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a_e, w_e, acc, 0, 0, 0);
    }
  };

  // wave w handles slices w, w + NW, ...; kRing - 1 of them are in flight ahead of the MFMAs
  const int nslices = (K + 15) / 16;
  f32x4 ra[kRing], rw[kRing];
#pragma unroll
  for (int u = 0; u < kRing - 1; ++u)
    if (wave + u * NW < nslices) load(wave + u * NW, ra[u], rw[u]);
  for (int base = wave; base < nslices; base += kRing * NW) {
#pragma unroll
    for (int u = 0; u < kRing; ++u) {
      const int cur = base + u * NW;
      if (cur < nslices) {
        const int nxt = cur + (kRing - 1) * NW;
        if (nxt < nslices) load(nxt, ra[(u + kRing - 1) % kRing], rw[(u + kRing - 1) % kRing]);
        compute(cur, ra[u], rw[u]);
      }
    }
  }

  // fixed-order reduction of the NW partial tiles
#pragma unroll
  for (int r = 0; r < 4; ++r) red[wave][4 * kq + r][r16] = acc[r];
  __syncthreads();
  if (!elive) return;
  float v = 0.f;
#pragma unroll
  for (int w = 0; w < NW; ++w) v += red[w][erow][ecol];

  const int64_t off = (int64_t)((SUB && g.sub_scatter) ? g.sub_rows[sub_off + em] : em) * g.ldc + en;
  if constexpr (LSTM) {
    if (epi == EPI_LSTM_BWD) {
      if (en < g.n_split) {
        gC[off] = v;
      } else {
        const int k = en - g.n_split;
        lstm_reverse_cell_store(cell, v, g.lstm_dz + (int64_t)em * g.lstm_dz_ld,
                                g.lstm_dc + (int64_t)em * g.lstm_H + k, g.lstm_H, k);
      }
      return;
    }
  }
  if (epi == EPI_FORWARD) {
    const float z = v + aux;
    if (g.C2) g.C2[off] = act_deriv(g.act, z);
    if (g.C == nullptr) return;
    v = act_value(g.act, z);
  } else if (epi == EPI_BIAS) {
    v += aux;
  } else if (epi == EPI_MASK) {
    v *= aux;
  }
  if (g.streaming)
    __builtin_nontemporal_store(v, gC + off);
  else
    gC[off] = v;
}

template <bool WKN, bool LSTM, bool SUB = false>
hipError_t launch16(const GemmArgs &g, hipStream_t stream) {
  const int64_t tiles = (int64_t)((g.M + 15) / 16) * ((g.N + 15) / 16);
  if constexpr (!LSTM && !SUB) {
    if (g.nbatch > 1) {
      const dim3 grid((unsigned)tiles, (unsigned)g.nbatch);
      if ((g.K + 15) / 16 >= 16)
        PFG_KERNEL((gemm_small16_kernel<WKN, 8, false, false, true>), grid, dim3(512), 0, stream, g);
      else
        PFG_KERNEL((gemm_small16_kernel<WKN, 4, false, false, true>), grid, dim3(256), 0, stream, g);
      return hipGetLastError();
    }
  }
  if (g.nbatch > 1) return hipErrorInvalidValue;
  // eight waves once each gets at least two slices of 16 k, else four
  if ((g.K + 15) / 16 >= 16)
    PFG_KERNEL((gemm_small16_kernel<WKN, 8, LSTM, SUB>), dim3((unsigned)tiles), dim3(512), 0, stream, g);
  else
    PFG_KERNEL((gemm_small16_kernel<WKN, 4, LSTM, SUB>), dim3((unsigned)tiles), dim3(256), 0, stream, g);
  return hipGetLastError();
}

}  // namespace

// Batched products with tiny outputs (at most 16 tiles of 16 x 16 per entry) and a contraction long
// enough to share out over the waves: one launch, an entry per second grid index.  (The per-example
// filter gradient of a first conv block, [k k c_in, h w] x [h w, c_out], is of this kind.)
bool small16_batched_applies(const GemmArgs &g) {
  if (g.nbatch <= 1 || g.nbatch > 65535 || g.bf16 || g.a_scale || !g.a_is_f32 || g.sub || g.sym_n > 0 || g.a_km)
    return false;
  if (g.epilogue != EPI_NONE) return false;
  const int64_t tiles16 = (int64_t)((g.M + 15) / 16) * ((g.N + 15) / 16);
  return tiles16 <= 16 && g.K >= 64;
}

bool small16_applies(const GemmArgs &g) {
  if (g.nbatch > 1) return small16_batched_applies(g);
  if (g.bf16 || g.a_scale || !g.a_is_f32) return false;
  if (g.sub && g.epilogue == EPI_LSTM_BWD) return false;
  if (g.epilogue != EPI_NONE && g.epilogue != EPI_BIAS && g.epilogue != EPI_FORWARD &&
      g.epilogue != EPI_MASK && g.epilogue != EPI_LSTM_BWD)
    return false;
  // worth it while 32 x 32 tiles would occupy at most half of the 256 compute units
  const int64_t tiles32 = (int64_t)((g.M + 31) / 32) * ((g.N + 31) / 32);
  return tiles32 <= 128;
}

hipError_t launch_gemm_small16(const GemmArgs &g, hipStream_t stream) {
  if (g.M <= 0 || g.N <= 0 || g.K <= 0) return hipSuccess;
  if (g.epilogue == EPI_LSTM_BWD)
    return g.w_kn ? launch16<true, true>(g, stream) : launch16<false, true>(g, stream);
  if (g.sub) return g.w_kn ? launch16<true, false, true>(g, stream) : launch16<false, false, true>(g, stream);
  return g.w_kn ? launch16<true, false>(g, stream) : launch16<false, false>(g, stream);
}

}  // namespace pfg

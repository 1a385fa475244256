// Matrix product for SMALL problems (few rows or a short contraction), where the LDS-tiled
// kernel would leave most of the chip idle and the run time is one dependent latency chain.
//
// A workgroup owns one 32 x 32 tile of C and splits the contraction index over its NW waves
// (wave w takes k-slices w, w + NW, ...).  Operands go straight from global memory (L2-resident
// at these sizes) into MFMA registers, several slices in flight per wave; the NW partial tiles
// are then summed in a fixed order through LDS, so the result does not depend on timing.  The
// fused epilogues are those of the tiled kernel, plus EPI_HEAD: when the whole row of logits
// fits one tile (d_L <= 32), softmax cross-entropy's gradient and loss are produced in the same
// launch as the last forward layer.
#include "common.h"
#include "gemm_device.h"

namespace pfg {

namespace {

using namespace dev;

// LSTM: the instantiation that carries the two LSTM epilogues (float32 only).  They live in a
// separate instantiation so that the kernels of the dense-network path stay as small as they were:
// with a handful of waves per launch, every extra instruction on the way shows in the run time.
// SUB: the instantiation for rows chosen on the device (GemmArgs::sub), apart for the same reason.
template <int AMODE, bool WKN, int NW, bool FAST, bool LSTM = false, bool SUB = false>
__global__ __launch_bounds__(64 * NW) void gemm_skinny_kernel(const GemmArgs g) {
  constexpr bool BF16 = (AMODE != A_F32);
  constexpr int ELEM = BF16 ? 2 : 4;
  constexpr int EPC = 16 / ELEM;       // k elements one lane feeds to the MFMA(s) of a slice
  constexpr int KSLICE = 2 * EPC;      // k elements per slice (two lane halves)
  constexpr int R = 4;                 // slices in flight per wave (8 was measured slower)
  constexpr int NT = 64 * NW;

  __shared__ __align__(16) float red[NW][32][36];   // row stride 144 B: 16-byte aligned rows
  __shared__ __align__(16) float hd[32][32];   // EPI_HEAD: delta rows of the tile, zero-padded
  __shared__ int lab[32];                      // EPI_HEAD: labels of the tile's rows

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int half = lane >> 5;
  const int l32 = lane & 31;
  const int N = g.N, K = g.K;
  const int tiles_m = (g.M + 31) / 32;
  // rows chosen on the device: only the first row tiles are live, so the column tiles of a row tile
  // are numbered next to each other -- the live workgroups then come first in the launch and the ones
  // with nothing to do are dealt with while those run (unless the caller asks for the other numbering)
  const int tiles_n_all = SUB ? (int)gridDim.x / tiles_m : 1;
  const bool live_first = SUB && !g.sub_rows_fastest;
  const int m0 = (live_first ? (int)blockIdx.x / tiles_n_all : (int)blockIdx.x % tiles_m) * 32;
  // rows chosen on the device: the live row count comes from memory, tiles past it have nothing to do.
  // When the list is known to start at entry 0 and to have g.M readable entries (sub_offset_zero), the
  // list entries this lane needs are requested together with the count instead of behind it; an
  // entry past the count is then replaced by iteration 0, whose rows exist and whose results are dropped.
  const bool spec = SUB && g.sub_offset_zero;
  int spec_a = 0, spec_e = 0;
  if (spec) {
    spec_a = g.sub_rows[min(m0 + l32, g.M - 1)];
    spec_e = g.sub_rows[min(m0 + (tid >> 3), g.M - 1)];
  }
  const int M = SUB ? g.sub[0] : g.M;
  if (SUB && m0 >= M) return;
  const int sub_off = (SUB && !spec) ? g.sub[1] : 0;
  // EPI_HEAD has a single column tile (N <= 32); the second grid index then counts the workgroups
  // that share out the fused cotangent step of one row tile (each recomputes the tile's logits)
  const bool is_head = (g.epilogue == EPI_HEAD);
  const int second = live_first ? (int)blockIdx.x % tiles_n_all : (int)blockIdx.x / tiles_m;
  const int n0 = is_head ? 0 : second * 32;
  // EPI_LSTM_FWD: the tile's 32 columns are the four gate columns of the 8 hidden units
  // 8 * second .. 8 * second + 7 (column gate * H + unit of W_h), not 32 consecutive columns
  const bool lstm_fwd = LSTM && WKN && (g.epilogue == EPI_LSTM_FWD);

  const bool a_vec_ok = ((reinterpret_cast<uintptr_t>(g.A) & 15) == 0) &&
                        ((g.lda * (AMODE == A_BF16 ? 2 : 4)) % 16 == 0) &&
                        ((g.a_batch_stride * (AMODE == A_BF16 ? 2 : 4)) % 16 == 0);
  const bool s_vec_ok = g.a_scale && ((reinterpret_cast<uintptr_t>(g.a_scale) & 15) == 0) &&
                        ((g.ld_scale * 4) % 16 == 0);
  const bool w_vec_ok = ((reinterpret_cast<uintptr_t>(g.W) & 15) == 0) && ((g.ldw * ELEM) % 16 == 0);
  const bool scaled = (g.a_scale != nullptr);
  const int epi = g.epilogue;
  const bool head_step = (epi == EPI_HEAD) && (g.head_gprev != nullptr);
  const int tile_rows = min(32, g.M - m0);
  // operands of the head that do not depend on this kernel's product are fetched early, off the
  // critical path (the barriers of the reduction order these LDS writes before their reads)
  if (epi == EPI_HEAD && tid < 32) lab[tid] = (tid < tile_rows) ? g.labels[m0 + tid] : -1;

  // this lane's A row and W column
  const void *a_row = nullptr;
  const float *a_srow = nullptr;
  {
    const int m = m0 + l32;
    if (FAST || m < M) {
      int mc = FAST ? min(m, M - 1) : m;           // FAST: rows past the end re-read the last row
      if (SUB && g.sub_gather) mc = spec ? (m < M ? spec_a : 0) : g.sub_rows[sub_off + mc];
      const int64_t b = mc / g.S, s = mc % g.S;
      const int64_t off = b * g.a_batch_stride + s * g.lda;
      if constexpr (AMODE == A_BF16)
        a_row = static_cast<const __bf16 *>(g.A) + off;
      else
        a_row = static_cast<const float *>(g.A) + off;
      if (scaled) a_srow = g.a_scale + b * g.ld_scale;
    }
  }
  const int n = lstm_fwd ? (l32 >> 3) * g.lstm_H + 8 * second + (l32 & 7) : n0 + l32;
  const bool n_in = lstm_fwd ? (8 * second + (l32 & 7) < g.lstm_H) : (n < N);
  const void *w_row = nullptr;           // !WKN: row n of W [N, K]
  if constexpr (!WKN) {
    if (FAST || n_in) {
      const int nc = FAST ? min(n, N - 1) : n;
      if constexpr (BF16)
        w_row = static_cast<const __bf16 *>(g.W) + (int64_t)nc * g.ldw;
      else
        w_row = static_cast<const float *>(g.W) + (int64_t)nc * g.ldw;
    }
  }

  RawA<AMODE> ra[R];
  u32x4 rw[R];

  auto load = [&](int slice, RawA<AMODE> &a, u32x4 &w) {
    const int k0 = slice * KSLICE + half * EPC;
    a = fetch_a<AMODE, FAST>(a_row, a_srow, scaled, k0, K, a_vec_ok, s_vec_ok);
    if constexpr (!WKN) {
      if constexpr (BF16)
        w = ld8<FAST>(static_cast<const __bf16 *>(w_row), k0, K, w_vec_ok);
      else
        w = __builtin_bit_cast(u32x4, ld4<FAST>(static_cast<const float *>(w_row), k0, K, w_vec_ok));
    } else if constexpr (FAST) {
      // W is [K, N]: EPC strided loads down column n (coalesced across the 32 lanes of a half);
      // indices clamped, no branches (out-of-range values are zeroed in compute())
      const int nc = min(n, N - 1);
      u32x4 v = {0u, 0u, 0u, 0u};
      if constexpr (BF16) {
        const uint16_t *col = static_cast<const uint16_t *>(g.W) + nc;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const uint32_t bits = (uint32_t)col[(int64_t)min(k0 + e, K - 1) * g.ldw];
          v[e >> 1] |= bits << ((e & 1) * 16);
        }
      } else {
        const float *col = static_cast<const float *>(g.W) + nc;
        f32x4 f;
#pragma unroll
        for (int e = 0; e < 4; ++e) f[e] = col[(int64_t)min(k0 + e, K - 1) * g.ldw];
        v = __builtin_bit_cast(u32x4, f);
      }
      w = v;
    } else {
      // W is [K, N]: EPC strided loads down column n (coalesced across the 32 lanes of a half)
      u32x4 v = {0u, 0u, 0u, 0u};
      if (n_in) {
        if constexpr (BF16) {
          const uint16_t *col = static_cast<const uint16_t *>(g.W) + n;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const uint32_t bits = (k0 + e < K) ? (uint32_t)col[(int64_t)(k0 + e) * g.ldw] : 0u;
            v[e >> 1] |= bits << ((e & 1) * 16);
          }
        } else {
          const float *col = static_cast<const float *>(g.W) + n;
          f32x4 f = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (k0 + e < K) f[e] = col[(int64_t)(k0 + e) * g.ldw];
          v = __builtin_bit_cast(u32x4, f);
        }
      }
      w = v;
    }
  };

  // Epilogue assignment: each thread finishes Q consecutive columns of one row.  What it needs
  // from global memory for that (bias or mask values) does not depend on the product, so it is
  // requested here, before the contraction, and has arrived by the time it is used.
  constexpr int Q = 1024 / NT;                    // 4 (NW = 4) or 2 (NW = 8)
  static_assert(Q == 2 || Q == 4, "the epilogue expects 256 or 512 threads");
  const int row = tid / (32 / Q), col = (tid % (32 / Q)) * Q;
  const int m = m0 + row, nn = n0 + col;
  const bool row_in = m < M;
  const bool all_in = row_in && (nn + Q <= N);
  const int64_t off = (int64_t)((SUB && g.sub_scatter && row_in) ? g.sub_rows[sub_off + m] : m) * g.ldc + nn;
  const bool want_bias = (epi == EPI_BIAS || epi == EPI_FORWARD || epi == EPI_HEAD) && g.bias;
  // Q-wide register vectors (not arrays: an array indexed inside a rolled loop would be moved out
  // of registers)
  typedef float fq __attribute__((ext_vector_type(Q)));
  fq aux;                                        // bias (added) or mask (multiplied)
#pragma unroll
  for (int q = 0; q < Q; ++q) aux[q] = (epi == EPI_MASK) ? 1.f : 0.f;
  if (row_in) {
    if (want_bias) {
#pragma unroll
      for (int q = 0; q < Q; ++q)
        if (nn + q < N)
          aux[q] = g.bf16 ? (float)static_cast<const __bf16 *>(g.bias)[nn + q]
                          : static_cast<const float *>(g.bias)[nn + q];
    } else if (epi == EPI_MASK) {
      const float *mp = g.emask + (int64_t)(m / g.S) * g.ld_emask + nn;
      if (all_in && ((reinterpret_cast<uintptr_t>(mp) & (4 * Q - 1)) == 0)) {
        const fq mv = *reinterpret_cast<const fq *>(mp);
#pragma unroll
        for (int q = 0; q < Q; ++q) aux[q] = mv[q];
      } else {
#pragma unroll
        for (int q = 0; q < Q; ++q)
          if (nn + q < N) aux[q] = mp[q];
      }
    }
  }

  // EPI_LSTM_FWD: thread (row, unit) = (tid / 8, tid % 8) of the first 256 threads finishes one
  // cell; what it adds to the product is requested here, ahead of the contraction
  f32x4 lstm_z = {0.f, 0.f, 0.f, 0.f};
  float lstm_cprev = 0.f, lstm_hw = 0.f;       // lstm_hw: this cell's entry of the halting vector
  const int lstm_m = m0 + (tid >> 3), lstm_k = 8 * second + (tid & 7);
  const bool lstm_live = lstm_fwd && tid < 256 && lstm_m < M && lstm_k < g.lstm_H;
  // rows chosen on the device (the active list of a while loop): row lstm_m of the product is
  // iteration lstm_p, whose token row and state are read and written in place
  int64_t lstm_p = lstm_m;
  if constexpr (LSTM && WKN) {
    if (lstm_live) {
      if (SUB) lstm_p = spec ? spec_e : g.sub_rows[sub_off + lstm_m];
      const int H = g.lstm_H, T = g.lstm_T, t = g.lstm_step;
      const int64_t zr = g.lstm_zx_rows ? (int64_t)g.lstm_zx_rows[lstm_p] + t : lstm_p * T + t;
      const float *zrow = g.lstm_zx + zr * 4 * H + lstm_k;
      lstm_z = f32x4{zrow[0], zrow[H], zrow[2 * H], zrow[3 * H]};
      if (g.lstm_has_prev)
        lstm_cprev = g.lstm_cs_w[lstm_p * g.lstm_state_ld + (t - 1) * g.lstm_state_ts + lstm_k];
      if (SUB && g.lstm_score_part) lstm_hw = g.lstm_halt_w[lstm_k];
    }
  }

  // EPI_LSTM_BWD: the gate values, cell states and running dc of this thread's Q elements are
  // requested ahead of the contraction too
  LstmCellIn lb0{}, lb1{}, lb2{}, lb3{};
  // the row that owns dc and dz (SUB: the iteration behind row m of the list) and, with SUB, the
  // token row of its trip lstm_step, where the gate values and cell states were kept
  int64_t bwd_p = m, bwd_tok = 0;
  if constexpr (LSTM && !WKN) {
    if (epi == EPI_LSTM_BWD && row_in) {
      const int H = g.lstm_H, T = g.lstm_T, t = g.lstm_step;
      int64_t hist = (int64_t)(m / g.S) * T + t;          // row of the gate and cell-state history
      if constexpr (SUB) {
        bwd_p = g.sub_rows[sub_off + m];
        bwd_tok = hist = (int64_t)g.lstm_zx_rows[bwd_p] + t;
      }
      const float *grow = g.lstm_gates + hist * 4 * (int64_t)H;
      const float *crow = g.lstm_cs + hist * (int64_t)H;
      const float *dcrow = g.lstm_dc + bwd_p * H;
      const float *seedrow = nullptr;
      if constexpr (SUB) {
        if (g.lstm_seed && g.lstm_steps[bwd_p] == t + 1) seedrow = g.lstm_seed + bwd_p * H;
      }
      auto fetch = [&](int q, LstmCellIn &v) {
        const int k = nn + q - g.n_split;
        if (k < 0 || nn + q >= N) return;
        v.i = grow[k]; v.g = grow[H + k]; v.f = grow[2 * H + k]; v.o = grow[3 * H + k];
        v.c = crow[k];
        v.cprev = t > 0 ? crow[k - H] : 0.f;
        v.dc = dcrow[k];
        if (SUB && seedrow) v.seed = seedrow[k];
      };
      fetch(0, lb0);
      fetch(1, lb1);
      if constexpr (Q == 4) {
        fetch(2, lb2);
        fetch(3, lb3);
      }
    }
  }

  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;

  // slice: the k-slice the registers were loaded for (FAST loads are zeroed here, not when issued)
  auto compute = [&](int slice, const RawA<AMODE> &a, u32x4 w) {
    const bool past = FAST && (slice * KSLICE + half * EPC >= K);
    const u32x4 av = finish_a<AMODE>(a, scaled, past);
    if (FAST && (past || (WKN && !n_in))) w = u32x4{0u, 0u, 0u, 0u};
    if constexpr (BF16) {
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av),
                                                    __builtin_bit_cast(bf16x8, w), acc, 0, 0, 0);
    } else {
      const f32x4 af = __builtin_bit_cast(f32x4, av), wf = __builtin_bit_cast(f32x4, w);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float a_e = af[e], w_e = wf[e];
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a_e, w_e, acc, 0, 0, 0);
      }
    }
  };

  // wave w handles slices w, w + NW, ...; R - 1 of them are in flight ahead of the MFMAs
  const int nslices = (K + KSLICE - 1) / KSLICE;
#pragma unroll
  for (int u = 0; u < R - 1; ++u)
    if (wave + u * NW < nslices) load(wave + u * NW, ra[u], rw[u]);
  for (int base = wave; base < nslices; base += R * NW) {
#pragma unroll
    for (int u = 0; u < R; ++u) {
      const int cur = base + u * NW;
      if (cur < nslices) {
        const int nxt = cur + (R - 1) * NW;
        if (nxt < nslices) load(nxt, ra[(u + R - 1) % R], rw[(u + R - 1) % R]);
        compute(cur, ra[u], rw[u]);
      }
    }
  }

  // ---- fixed-order reduction of the NW partial tiles ----
#pragma unroll
  for (int r = 0; r < 16; ++r) red[wave][8 * (r >> 2) + 4 * half + (r & 3)][l32] = acc[r];
  __syncthreads();

  // Each thread finishes Q consecutive columns of one row: it sums the NW partial tiles, fetches
  // the bias / mask values it needs in one go (a vector load when alignment allows) and writes
  // its Q results, again as one vector when possible.  One pass, no loop: with so few waves the
  // latency of every dependent global access counts.
  if constexpr (LSTM && WKN) {
    if (lstm_fwd) {
      float score_piece = 0.f;       // this cell's share of the halting score of its row
      if (lstm_live) {
        const int H = g.lstm_H, T = g.lstm_T, t = g.lstm_step;
        const int r = tid >> 3, u = tid & 7;
        f32x4 z = lstm_z;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
          z[0] += red[w][r][u];
          z[1] += red[w][r][8 + u];
          z[2] += red[w][r][16 + u];
          z[3] += red[w][r][24 + u];
        }
        const float gi = 1.f / (1.f + __expf(-z[0])), gg = tanhf(z[1]);
        const float gf = 1.f / (1.f + __expf(-z[2])), go = 1.f / (1.f + __expf(-z[3]));
        const float c = gf * lstm_cprev + gi * gg;
        if (g.lstm_gates_w) {
          float *grow = g.lstm_gates_w + (lstm_p * T + t) * 4 * H + lstm_k;
          grow[0] = gi; grow[H] = gg; grow[2 * H] = gf; grow[3 * H] = go;
        }
        const int64_t at = lstm_p * g.lstm_state_ld + t * g.lstm_state_ts + lstm_k;
        const float hnew = go * tanhf(c);
        g.lstm_cs_w[at] = c;
        g.lstm_hs_w[at] = hnew;
        if (g.lstm_zx_rows && (g.lstm_tok_gates || g.lstm_tok_c || g.lstm_tok_h)) {
          const int64_t zr = (int64_t)g.lstm_zx_rows[lstm_p] + t;      // the token row of (iteration, step)
          if (g.lstm_tok_gates) {
            float *grow = g.lstm_tok_gates + zr * 4 * H + lstm_k;
            grow[0] = gi; grow[H] = gg; grow[2 * H] = gf; grow[3 * H] = go;
          }
          if (g.lstm_tok_c) g.lstm_tok_c[zr * H + lstm_k] = c;
          if (g.lstm_tok_h) g.lstm_tok_h[zr * H + lstm_k] = hnew;
        }
        score_piece = hnew * lstm_hw;
      }
      if constexpr (SUB) {
        // the eight cells of a row that this workgroup finished sit in eight neighbouring lanes: their
        // shares are added in a fixed pattern and the first lane stores the piece
        if (g.lstm_score_part && tid < 256) {
#pragma unroll
          for (int off = 4; off > 0; off >>= 1) score_piece += __shfl_xor(score_piece, off, 8);
          if ((tid & 7) == 0 && lstm_m < M) g.lstm_score_part[lstm_p * g.lstm_score_ld + second] = score_piece;
        }
      }
      return;
    }
  }
  {
    fq v;
#pragma unroll
    for (int q = 0; q < Q; ++q) v[q] = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w)
#pragma unroll
      for (int q = 0; q < Q; ++q) v[q] += red[w][row][col + q];
    if (epi == EPI_HEAD) {
      // keep the biased logits in LDS for the softmax pass below
#pragma unroll
      for (int q = 0; q < Q; ++q) {
        v[q] += aux[q];
        red[0][row][col + q] = v[q];   // safe: these slots are read and written by this thread only
        if (row_in && nn + q < N && g.C && second == 0) g.C[off + q] = v[q];
      }
    } else if (row_in) {
      fq out2;
      if (epi == EPI_FORWARD) {
#pragma unroll 1
        for (int q = 0; q < Q; ++q) {              // rolled: the activation code is long
          const float z = v[q] + aux[q];
          out2[q] = act_deriv(g.act, z);
          v[q] = act_value(g.act, z);
        }
      } else if (epi == EPI_BIAS) {
#pragma unroll
        for (int q = 0; q < Q; ++q) v[q] += aux[q];
      } else if (epi == EPI_MASK) {
#pragma unroll
        for (int q = 0; q < Q; ++q) v[q] *= aux[q];
      }
      if (LSTM && epi == EPI_LSTM_BWD && nn + Q > g.n_split) {
        // this thread's columns reach into the hidden-state cotangent: element by element, with
        // constant indices into v[] (an index known only at run time would move the array out of
        // registers)
        auto finish = [&](int q, float val, const LstmCellIn &in) {
          if (nn + q >= N) return;
          if (nn + q < g.n_split) {
            g.C[off + q] = val;
          } else {
            const int k = nn + q - g.n_split;
            float *row2 = (SUB && g.lstm_tok_dz) ? g.lstm_tok_dz + bwd_tok * 4 * g.lstm_H : nullptr;
            lstm_reverse_cell_store(in, SUB ? val + in.seed : val, g.lstm_dz + bwd_p * g.lstm_dz_ld,
                                    g.lstm_dc + bwd_p * g.lstm_H + k, g.lstm_H, k, row2);
          }
        };
        finish(0, v[0], lb0);
        finish(1, v[1], lb1);
        if constexpr (Q == 4) {
          finish(2, v[2], lb2);
          finish(3, v[3], lb3);
        }
        return;     // nothing follows the epilogue for this kind of product
      }
      const bool vec_c = all_in && g.C && ((reinterpret_cast<uintptr_t>(g.C + off) & (4 * Q - 1)) == 0);
      const bool vec_c2 = all_in && (epi == EPI_FORWARD) &&
                          ((reinterpret_cast<uintptr_t>(g.C2 + off) & (4 * Q - 1)) == 0);
      if (epi == EPI_FORWARD && g.C2) {
        if (vec_c2) {
          fq o2;
#pragma unroll
          for (int q = 0; q < Q; ++q) o2[q] = out2[q];
          *reinterpret_cast<fq *>(g.C2 + off) = o2;
        } else {
#pragma unroll
          for (int q = 0; q < Q; ++q)
            if (nn + q < N) g.C2[off + q] = out2[q];
        }
      }
      if (g.C) {
        if (vec_c) {
          fq o1;
#pragma unroll
          for (int q = 0; q < Q; ++q) o1[q] = v[q];
          if (g.streaming)
            __builtin_nontemporal_store(o1, reinterpret_cast<fq *>(g.C + off));
          else
            *reinterpret_cast<fq *>(g.C + off) = o1;
        } else {
#pragma unroll
          for (int q = 0; q < Q; ++q)
            if (nn + q < N) g.C[off + q] = v[q];
        }
      }
    }
  }

  if (epi == EPI_HEAD) {
    // Softmax cross-entropy on the rows of the tile: delta = softmax(y) - onehot(label),
    // loss = -log softmax(y)[label].  N <= 32: each half of a wave takes one row per pass, and
    // the reductions stay inside the half.  These few waves run the code once, so what they pay
    // for is instruction fetch: the loops below are kept rolled and short on purpose.
    __syncthreads();
#pragma unroll 1
    for (int row0 = 2 * wave; row0 < 32; row0 += 2 * NW) {
      const int row = row0 + half;
      const int m = m0 + row;
      const bool valid = row < tile_rows;
      const bool live = valid && (l32 < N);
      const float y = live ? red[0][row][l32] : -INFINITY;
      float mx = y;
#pragma unroll
      for (int off = 16; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
      const float ex = live ? __expf(y - mx) : 0.f;
      const int label = lab[row];
      float den = ex, others = (l32 == label) ? 0.f : ex;
#pragma unroll
      for (int off = 16; off > 0; off >>= 1) {
        den += __shfl_xor(den, off, 64);
        others += __shfl_xor(others, off, 64);
      }
      const float inv = valid ? 1.f / den : 0.f;
      // p[label] - 1 = -(sum of the other classes) / den, free of cancellation
      const float delta = (l32 == label) ? -others * inv : ex * inv;
      if (live && second == 0) g.C2[(int64_t)m * g.ldc + l32] = delta;
      hd[row][l32] = live ? delta : 0.f;       // kept, zero-padded, for the cotangent step below
      const bool label_ok = (label >= 0) && (label < N);
      const float yl = __shfl(y, half * 32 + (label_ok ? label : 0), 64);
      if (g.loss && valid && l32 == 0 && second == 0) g.loss[m] = __logf(den) - ((label_ok ? yl : mx) - mx);
    }
    if (head_step) {
      __syncthreads();
      switch ((N + 3) >> 2) {
        case 1: head_cotangent<1, NT>(g, hd, m0, tile_rows, tid, second, (int)gridDim.x / tiles_m); break;
        case 2: head_cotangent<2, NT>(g, hd, m0, tile_rows, tid, second, (int)gridDim.x / tiles_m); break;
        case 3: head_cotangent<3, NT>(g, hd, m0, tile_rows, tid, second, (int)gridDim.x / tiles_m); break;
        case 4: head_cotangent<4, NT>(g, hd, m0, tile_rows, tid, second, (int)gridDim.x / tiles_m); break;
        case 5: head_cotangent<5, NT>(g, hd, m0, tile_rows, tid, second, (int)gridDim.x / tiles_m); break;
        case 6: head_cotangent<6, NT>(g, hd, m0, tile_rows, tid, second, (int)gridDim.x / tiles_m); break;
        case 7: head_cotangent<7, NT>(g, hd, m0, tile_rows, tid, second, (int)gridDim.x / tiles_m); break;
        default: head_cotangent<8, NT>(g, hd, m0, tile_rows, tid, second, (int)gridDim.x / tiles_m); break;
      }
    }
  }
}

template <int AMODE, bool WKN, int NW>
hipError_t launch_nw(const GemmArgs &g, hipStream_t stream) {
  int64_t tiles = (int64_t)((g.M + 31) / 32) * ((g.N + 31) / 32);
  if (g.epilogue == EPI_LSTM_FWD) tiles = (int64_t)((g.M + 31) / 32) * ((g.lstm_H + 7) / 8);
  if (g.epilogue == EPI_HEAD && g.head_gprev) {
    // share the fused cotangent step of each row tile out over several workgroups of at least 64
    // columns each: up to 8, or more while the launch stays within one workgroup per compute unit
    // (a workgroup walks its rows one after the other, so fewer columns mean more row bands)
    const int row_tiles = (g.M + 31) / 32;
    const int cap = 256 / row_tiles > 8 ? 256 / row_tiles : 8;
    int groups = g.K / 64;
    groups = groups < 1 ? 1 : (groups > cap ? cap : groups);
    tiles *= groups;
  }
  // the element-wise column loads of the [K, N] layout put no condition on W
  const bool lstm = (g.epilogue == EPI_LSTM_FWD || g.epilogue == EPI_LSTM_BWD);
  if constexpr (AMODE == A_F32 && WKN) {
    if (g.epilogue == EPI_LSTM_FWD && g.sub) {
      // the fused LSTM step on the rows of a device-side list
      if (fast_loads_ok(g, false))
        PFG_KERNEL((gemm_skinny_kernel<AMODE, WKN, NW, true, true, true>), dim3((unsigned)tiles),
                   dim3(64 * NW), 0, stream, g);
      else
        PFG_KERNEL((gemm_skinny_kernel<AMODE, WKN, NW, false, true, true>), dim3((unsigned)tiles),
                   dim3(64 * NW), 0, stream, g);
      return hipGetLastError();
    }
  }
  if constexpr (AMODE == A_F32 && !WKN) {
    if (g.epilogue == EPI_LSTM_BWD && g.sub) {
      // a reverse trip of a while loop on the rows of the list the forward loop kept for it
      if (!g.sub_gather || g.sub_scatter || !g.lstm_zx_rows) return hipErrorInvalidValue;
      if (fast_loads_ok(g, true))
        PFG_KERNEL((gemm_skinny_kernel<AMODE, WKN, NW, true, true, true>), dim3((unsigned)tiles),
                   dim3(64 * NW), 0, stream, g);
      else
        PFG_KERNEL((gemm_skinny_kernel<AMODE, WKN, NW, false, true, true>), dim3((unsigned)tiles),
                   dim3(64 * NW), 0, stream, g);
      return hipGetLastError();
    }
  }
  if (lstm && g.sub) return hipErrorInvalidValue;
  if constexpr (AMODE == A_F32) {
    if (lstm) {
      if (fast_loads_ok(g, !WKN))
        PFG_KERNEL((gemm_skinny_kernel<AMODE, WKN, NW, true, true>), dim3((unsigned)tiles),
                   dim3(64 * NW), 0, stream, g);
      else
        PFG_KERNEL((gemm_skinny_kernel<AMODE, WKN, NW, false, true>), dim3((unsigned)tiles),
                   dim3(64 * NW), 0, stream, g);
      return hipGetLastError();
    }
  }
  if (lstm) return hipErrorInvalidValue;     // the LSTM epilogues exist in float32 only
  if constexpr (AMODE == A_F32) {
    if (g.sub) {
      if (fast_loads_ok(g, !WKN))
        PFG_KERNEL((gemm_skinny_kernel<AMODE, WKN, NW, true, false, true>), dim3((unsigned)tiles),
                   dim3(64 * NW), 0, stream, g);
      else
        PFG_KERNEL((gemm_skinny_kernel<AMODE, WKN, NW, false, false, true>), dim3((unsigned)tiles),
                   dim3(64 * NW), 0, stream, g);
      return hipGetLastError();
    }
  }
  if (g.sub) return hipErrorInvalidValue;    // rows chosen on the device: float32 only
  if (fast_loads_ok(g, !WKN))
    PFG_KERNEL((gemm_skinny_kernel<AMODE, WKN, NW, true>), dim3((unsigned)tiles),
                       dim3(64 * NW), 0, stream, g);
  else
    PFG_KERNEL((gemm_skinny_kernel<AMODE, WKN, NW, false>), dim3((unsigned)tiles),
                       dim3(64 * NW), 0, stream, g);
  return hipGetLastError();
}

template <int AMODE, bool WKN>
hipError_t launch_mode(const GemmArgs &g, hipStream_t stream) {
  // eight waves once each gets about four k-slices, else four (the epilogue wants at least 256
  // threads on the 1024 outputs of a tile; with a short contraction some waves only help there)
  const int kslice = (AMODE == A_F32) ? 8 : 16;
  const int slices = (g.K + kslice - 1) / kslice;
  // (the fused LSTM step on the rows of a device-side list does better on four: measured on 1024
  // sequences of 1 to 100 tokens 14.7 against 16.3 us per trip; the reverse trip, with its four times
  // longer contraction, and the step on all rows are better off with eight)
  if (slices >= 32 && !(g.epilogue == EPI_LSTM_FWD && g.sub)) return launch_nw<AMODE, WKN, 8>(g, stream);
  return launch_nw<AMODE, WKN, 4>(g, stream);
}

}  // namespace

hipError_t launch_gemm_skinny(const GemmArgs &g, hipStream_t stream) {
  if (g.M <= 0 || g.N <= 0 || g.K <= 0) return hipSuccess;
  if (g.epilogue == EPI_HEAD && g.N > 32) return hipErrorInvalidValue;
  if (g.epilogue == EPI_LSTM_FWD && (g.bf16 || !g.w_kn || g.N != 4 * g.lstm_H || g.nbatch > 1))
    return hipErrorInvalidValue;
  if (small16_applies(g)) return launch_gemm_small16(g, stream);
  if (g.nbatch > 1) {
    // small batched products: one launch per product (this kernel has no batch index)
    const int a_elem = (g.bf16 && !g.a_is_f32) ? 2 : 4, w_elem = g.bf16 ? 2 : 4;
    for (int z = 0; z < g.nbatch; ++z) {
      GemmArgs one = g;
      one.nbatch = 0;
      one.A = static_cast<const char *>(g.A) + (int64_t)z * g.batch_A * a_elem;
      one.W = static_cast<const char *>(g.W) + (int64_t)z * g.batch_W * w_elem;
      if (g.a_scale) one.a_scale = g.a_scale + (int64_t)z * g.batch_scale;
      one.C = g.C + (int64_t)z * g.batch_C;
      hipError_t e = launch_gemm_skinny(one, stream);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }
  if (!g.bf16)
    return g.w_kn ? launch_mode<A_F32, true>(g, stream) : launch_mode<A_F32, false>(g, stream);
  if (g.a_is_f32)
    return g.w_kn ? launch_mode<A_F32_TO_BF16, true>(g, stream)
                  : launch_mode<A_F32_TO_BF16, false>(g, stream);
  return g.w_kn ? launch_mode<A_BF16, true>(g, stream) : launch_mode<A_BF16, false>(g, stream);
}

}  // namespace pfg

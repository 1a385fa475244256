// MFMA-tiled matrix product for the stacked forward pass and the cotangent propagation.
//
// Section 3.4 of the paper turns matmul(X[i], Y) with a loop-invariant Y into ONE matmul over
// the rows of all iterations folded together ([n * x, y] x [y, z]).  Here the folded row index is
// m = b * S + s (example b, seed row s); the weights are the invariant operand and are never
// tiled.  The activation-derivative mask, which is invariant over s, is broadcast in registers
// (Section 3.4's broadcasting rule) either onto the A operand while it is staged or onto the
// accumulators before they are stored.
//
// Tiling (gfx950, wave64): a workgroup is 4 waves in a 2 x 2 arrangement; each wave owns
// TM x TN MFMA tiles of 32 x 32, so the workgroup tile is (64 TM) x (64 TN).  Both operands are
// staged in LDS as [row][k] with 16 bytes of padding per row, so that one ds_read_b128 per lane
// fetches 16 bytes of k for one row: four k-steps of v_mfma_f32_32x32x2_f32, or one
// v_mfma_f32_32x32x16_bf16.  The k index is permuted identically for both operands, which a
// contraction does not notice.  Global loads for stage t+1 are issued before the MFMA loop of
// stage t and written to the other LDS buffer after it (one barrier per stage).
#include "common.h"
#include "gemm_device.h"

namespace pfg {

namespace {

using namespace dev;


// WGM x WGN: arrangement of the workgroup's waves over the tile (2 x 2, or 4 x 2 for the largest).
// SUB: the instantiation for rows chosen on the device (GemmArgs::sub; float32),
// kept apart so that the others carry none of its loads and branches (inside the unrolled epilogue
// they cost a store-bound product a quarter of its speed).
// AKM: the instantiation that reads A stored as [K, M] (float32, FAST loads only).
// LSTMF: the instantiation with the LSTM cell update in its epilogue (EPI_LSTM_FWD; float32, W in
// [K, N] layout, FAST loads, 64 x 64 tiles): a tile's 64 columns are the four gate columns of 16
// hidden units (gate * H + unit of W_h), not 64 consecutive columns.
// GATHER: the instantiations whose A operand is the patch matrix of an image batch, gathered from
// the images while staging (GemmArgs::conv_k; with AKM the contraction runs over the positions).
template <int AMODE, bool WKN, int TM, int TN, int BKB, bool FAST, int WGM = 2, int WGN = 2, bool SUB = false,
          bool AKM = false, bool LSTMF = false, bool GATHER = false>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_kernel(const GemmArgs g) {
  static_assert(!GATHER || (AMODE == A_F32 && WKN && FAST && !SUB && !LSTMF && TM == 1 && TN == 1),
                "gathered patches: float32, [K, N] weights, FAST loads, 64 x 64 tiles");
  static_assert(!AKM || (AMODE == A_F32 && FAST && !SUB), "transposed A: float32, FAST loads, no row subsets");
  static_assert(!LSTMF || (AMODE == A_F32 && WKN && FAST && !SUB && !AKM && TM == 1 && TN == 1 && WGM == 2 && WGN == 2),
                "fused LSTM step: float32, [K, N] weights, FAST loads, 64 x 64 tiles");
  constexpr int kThreads = 64 * WGM * WGN;
  constexpr bool BF16 = (AMODE != A_F32);
  constexpr int ELEM = BF16 ? 2 : 4;
  // batched product: the second grid index selects the product; its operands sit at fixed strides
  const void *gA = g.A, *gW = g.W;
  const float *gScale = g.a_scale;
  float *gC = g.C;
  if (g.nbatch > 1) {
    const int64_t z = blockIdx.y;
    gA = static_cast<const char *>(g.A) + z * g.batch_A * (AMODE == A_BF16 ? 2 : 4);
    gW = static_cast<const char *>(g.W) + z * g.batch_W * ELEM;
    if (g.a_scale) gScale = g.a_scale + z * g.batch_scale;
    gC = g.C + z * g.batch_C;
  }
  constexpr int EPC = 16 / ELEM;            // elements per 16-byte chunk
  constexpr int BK = BKB / ELEM;            // k elements per stage
  constexpr int CPR = BKB / 16;             // chunks per LDS row
  constexpr int STRIDE = BKB + 16;          // LDS row stride in bytes
  constexpr int BM = 32 * TM * WGM, BN = 32 * TN * WGN;
  constexpr int A_CHUNKS = BM * CPR / kThreads;
  constexpr int W_CHUNKS = BN * CPR / kThreads;
  // bf16 weights in [K, N] layout (forward) stay in that layout in LDS, rows of BN values, and
  // are transposed on the way to the MFMA registers by ds_read_b64_tr_b16
  constexpr bool WTR = WKN && BF16;
  constexpr int W_STRIDE = WTR ? BN * 2 + 16 : STRIDE;
  constexpr int W_ROWS = WTR ? BK : BN;
  constexpr int STAGE = BM * STRIDE + W_ROWS * W_STRIDE;
  static_assert(BM * CPR % kThreads == 0 && BN * CPR % kThreads == 0, "tile / thread mismatch");

  extern __shared__ __align__(16) unsigned char smem[];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int half = lane >> 5;
  const int l32 = lane & 31;
  const int wm = (wave / WGN) * (32 * TM);
  const int wn = (wave % WGN) * (32 * TN);

  // Consecutive workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2.  Give
  // every XCD a contiguous run of tiles that walks the N tiles of one M tile before moving on, so
  // that a band of A rows is fetched into one L2 once and reused there for all its N tiles.
  const int tiles_m = (g.M + BM - 1) / BM;
  const int tiles_n = LSTMF ? (g.lstm_H + 15) / 16 : (g.N + BN - 1) / BN;
  int tile_m, tile_n;
  bool mirror = false;       // symmetric blocks: this tile also stands for its mirror image
  if (AMODE == A_F32 && BM == BN && g.sym_n > 0) {
    // tiles on and above the diagonal of each sym_n x sym_n block: row ti of a block has the
    // tiles tn = ti .. T - 1
    const int T = g.sym_n / BM, tri = T * (T + 1) / 2;
    const int total = (g.M / g.sym_n) * tri;
    int t = blockIdx.x;
    if (total % 8 == 0) t = (t % 8) * (total / 8) + t / 8;
    int p = t % tri, ti = 0;
    while (p >= T - ti) { p -= T - ti; ++ti; }
    tile_m = (t / tri) * T + ti;
    tile_n = ti + p;
    mirror = p > 0;
  } else if (SUB) {
    // Rows chosen on the device: only the first tiles along M are live, how many is not known to
    // the host.  Row tiles are dealt to the XCDs in turn (tile_m = 8 i + xcd), so that the live ones
    // spread over all eight whatever their number; an XCD still walks the N tiles of a row tile
    // one after the other.  The grid is rounded up to whole rounds of eight row tiles.
    const int xcd = blockIdx.x % 8, idx = blockIdx.x / 8;
    tile_m = (idx / tiles_n) * 8 + xcd;
    tile_n = idx % tiles_n;
    if (tile_m >= tiles_m) return;
  } else {
    const int total = tiles_m * tiles_n;
    int t = blockIdx.x;
    if (total % 8 == 0) t = (t % 8) * (total / 8) + t / 8;
    tile_m = t / tiles_n;
    tile_n = t % tiles_n;
  }
  const int m0 = tile_m * BM;
  const int n0 = tile_n * BN;
  // rows chosen on the device: the live row count comes from memory, tiles past it have nothing to do
  const int M = SUB ? g.sub[0] : g.M, N = g.N, K = g.K;
  if (SUB && m0 >= M) return;
  const int sub_off = SUB ? g.sub[1] : 0;

  const bool a_vec_ok = ((reinterpret_cast<uintptr_t>(gA) & 15) == 0) &&
                        ((g.lda * (AMODE == A_BF16 ? 2 : 4)) % 16 == 0) &&
                        ((g.a_batch_stride * (AMODE == A_BF16 ? 2 : 4)) % 16 == 0);
  const bool s_vec_ok = gScale && ((reinterpret_cast<uintptr_t>(gScale) & 15) == 0) &&
                        ((g.ld_scale * 4) % 16 == 0);
  const bool w_vec_ok = ((reinterpret_cast<uintptr_t>(gW) & 15) == 0) &&
                        ((g.ldw * ELEM) % 16 == 0);
  const bool scaled = (gScale != nullptr);

  // ---- per-thread staging assignments ----
  const void *a_row[A_CHUNKS];
  const float *a_srow[A_CHUNKS];
  int a_lds[A_CHUNKS];
  int a_k[A_CHUNKS];
  int a_m[A_CHUNKS];             // AKM: first row m of the chunk (global)
  int a_yx[A_CHUNKS];            // GATHER: (y << 16) | x of the chunk's position, or (ky << 16) | kx of its tap (AKM)
  bool a_live[A_CHUNKS];         // GATHER: does the chunk fetched last lie inside the image and the operand
  // small quotients by float reciprocals (operands below 2^24; off by one at most, then corrected)
  const float inv_c = GATHER ? 1.f / (float)g.conv_c : 0.f, inv_kw = GATHER ? 1.f / (float)g.conv_k : 0.f,
              inv_w = GATHER ? 1.f / (float)g.conv_w : 0.f;
  auto qdiv = [](int n, int d, float inv) {
    int q = (int)((float)n * inv);
    const int r = n - q * d;
    if (r < 0) --q;
    if (r >= d) ++q;
    return q;
  };
#pragma unroll
  for (int c = 0; c < A_CHUNKS; ++c) {
    const int id = tid + kThreads * c;
    if constexpr (GATHER && AKM) {
      // the chunk's four rows m are four channels of one filter tap: fixed for the whole product
      const int kl = id % BK, mg = id / BK;
      a_k[c] = kl;
      a_m[c] = m0 + mg * EPC;
      a_lds[c] = (mg * EPC) * STRIDE + kl * ELEM;
      const int tap = qdiv(a_m[c], g.conv_c, inv_c), ci = a_m[c] - tap * g.conv_c;
      const int ky = qdiv(tap, g.conv_k, inv_kw), kx = tap - ky * g.conv_k;
      a_yx[c] = (ky << 16) | kx;
      a_row[c] = static_cast<const float *>(gA) + ci;
      a_srow[c] = nullptr;
      continue;
    }
    if constexpr (GATHER && !AKM) {
      // the chunk's row m is one position of one image: fixed for the whole product
      const int row = id / CPR, kc = id % CPR;
      const int m = min(m0 + row, M - 1);
      a_lds[c] = row * STRIDE + kc * 16;
      a_k[c] = kc * EPC;
      a_m[c] = m0 + row;
      const int hw = g.conv_h * g.conv_w;
      const int b = m / hw, pos = m - b * hw;
      const int y = qdiv(pos, g.conv_w, inv_w), x = pos - y * g.conv_w;
      a_yx[c] = (y << 16) | x;
      a_row[c] = static_cast<const float *>(gA) + ((int64_t)b * hw + pos) * g.conv_c;
      a_srow[c] = nullptr;
      continue;
    }
    a_yx[c] = 0;
    a_live[c] = false;
    if constexpr (AKM) {
      // A is [K, M]: a chunk is 16 bytes along m at one k and is scattered into the [m][k] LDS
      // layout element by element (as for float32 weights in [K, N] layout)
      const int kl = id % BK, mg = id / BK;
      a_k[c] = kl;
      a_m[c] = m0 + mg * EPC;
      a_lds[c] = (mg * EPC) * STRIDE + kl * ELEM;
      a_row[c] = nullptr;
      a_srow[c] = nullptr;
      continue;
    }
    a_m[c] = 0;
    const int row = id / CPR, kc = id % CPR;
    const int m = m0 + row;
    a_lds[c] = row * STRIDE + kc * 16;
    a_k[c] = kc * EPC;
    a_row[c] = nullptr;
    a_srow[c] = nullptr;
    if (FAST || m < M) {
      int mc = FAST ? min(m, M - 1) : m;           // FAST: rows past the end re-read the last row
      if (SUB && g.sub_gather) mc = g.sub_rows[sub_off + mc];
      const int64_t b = mc / g.S, s = mc % g.S;
      const int64_t off = b * g.a_batch_stride + s * g.lda;
      if constexpr (AMODE == A_BF16)
        a_row[c] = static_cast<const __bf16 *>(gA) + off;
      else
        a_row[c] = static_cast<const float *>(gA) + off;
      if (scaled) a_srow[c] = gScale + b * g.ld_scale;
    }
  }

  // W chunks.  WKN == false: rows are n, 16 bytes along k (same shape as A).
  // WKN == true: W is [K, N]; a chunk is 16 bytes along n at one k and is scattered into the
  // [n][k] LDS layout element by element.
  const void *w_row[W_CHUNKS];   // !WKN: row pointer of n (or nullptr)
  int w_lds[W_CHUNKS];
  int w_k[W_CHUNKS];             // k offset of the chunk inside a stage
  int w_n[W_CHUNKS];             // WKN: first n of the chunk (global)
#pragma unroll
  for (int c = 0; c < W_CHUNKS; ++c) {
    const int id = tid + kThreads * c;
    if constexpr (!WKN) {
      const int row = id / CPR, kc = id % CPR;
      const int n = n0 + row;
      w_lds[c] = row * STRIDE + kc * 16;
      w_k[c] = kc * EPC;
      w_n[c] = n;
      w_row[c] = nullptr;
      if (FAST || n < N) {
        const int nc = FAST ? min(n, N - 1) : n;
        if constexpr (BF16)
          w_row[c] = static_cast<const __bf16 *>(gW) + (int64_t)nc * g.ldw;
        else
          w_row[c] = static_cast<const float *>(gW) + (int64_t)nc * g.ldw;
      }
    } else if constexpr (WTR) {
      constexpr int NGR = BN / 8;                  // 16-byte pieces per tile row
      const int kl = id / NGR, ng = id % NGR;      // consecutive lanes: consecutive pieces of a row
      w_k[c] = kl;
      w_n[c] = n0 + ng * 8;
      w_lds[c] = kl * W_STRIDE + ng * 16;
      w_row[c] = nullptr;
    } else {
      const int kl = id % BK, ng = id / BK;
      w_k[c] = kl;
      w_n[c] = n0 + ng * EPC;
      if constexpr (LSTMF) {
        // tile column 4 ng: gate (4 ng) / 16 of unit 16 tile_n + (4 ng) % 16; a chunk of four units
        // past the state size (H is a multiple of 4 here) is marked as out of range
        const int unit = 16 * tile_n + ((ng * EPC) & 15);
        w_n[c] = unit < g.lstm_H ? ((ng * EPC) >> 4) * g.lstm_H + unit : N;
      }
      w_lds[c] = (ng * EPC) * STRIDE + kl * ELEM;
      w_row[c] = nullptr;
    }
  }

  RawA<AMODE> ra[A_CHUNKS];
  u32x4 rw[W_CHUNKS];

  // One 16-byte chunk of the A operand (and of its scale) / of the W operand for stage kt.
  // sc: does the A operand carry a scale (passed as a literal where the caller has branched on
  // it once, so that no per-chunk select remains)
  auto fetch_a_chunk = [&](int c, int kt, bool sc) {
    if constexpr (GATHER) {
      const int p = (g.conv_k - 1) / 2;
      int y, x, ky, kx, ci;
      bool live;
      if constexpr (AKM) {
        const int k = kt * BK + a_k[c];            // the position
        y = qdiv(k, g.conv_w, inv_w); x = k - y * g.conv_w;
        ky = a_yx[c] >> 16; kx = a_yx[c] & 0xffff; ci = 0;
        live = k < K && a_m[c] < M;
      } else {
        const int k = kt * BK + a_k[c];            // (tap, channel)
        const int tap = qdiv(k, g.conv_c, inv_c);
        ci = k - tap * g.conv_c;
        ky = qdiv(tap, g.conv_k, inv_kw); kx = tap - ky * g.conv_k;
        y = a_yx[c] >> 16; x = a_yx[c] & 0xffff;
        live = k < K && a_m[c] < M;
      }
      const int yy = y + ky - p, xx = x + kx - p;
      live = live && yy >= 0 && yy < g.conv_h && xx >= 0 && xx < g.conv_w;
      // the load itself is unconditional, from a pixel inside the image (no branch in the loop);
      // what it brings for a patch entry outside the image is dropped when the chunk is stored
      const int yc = min(max(yy, 0), g.conv_h - 1), xc = min(max(xx, 0), g.conv_w - 1);
      const float *base = AKM ? static_cast<const float *>(a_row[c])
                              : static_cast<const float *>(a_row[c]) - ((int64_t)y * g.conv_w + x) * g.conv_c;
      ra[c].v = *reinterpret_cast<const f32x4 *>(base + ((int64_t)yc * g.conv_w + xc) * g.conv_c + ci);
      a_live[c] = live;
      return;
    }
    if constexpr (AKM) {
      // 16 bytes along m of row k; both indices clamped (zeroed in stash if out of range)
      const int k = kt * BK + a_k[c];
      ra[c].v = load4_f32_fast(static_cast<const float *>(gA) + (int64_t)min(k, K - 1) * g.lda, a_m[c], M);
    } else {
      ra[c] = fetch_a<AMODE, FAST>(a_row[c], a_srow[c], sc, kt * BK + a_k[c], K, a_vec_ok, s_vec_ok);
    }
  };
  auto fetch_w_chunk = [&](int c, int kt) {
    const int kbase = kt * BK;
    if constexpr (!WKN) {
      if constexpr (BF16)
        rw[c] = ld8<FAST>(static_cast<const __bf16 *>(w_row[c]), kbase + w_k[c], K, w_vec_ok);
      else
        rw[c] = __builtin_bit_cast(
            u32x4, ld4<FAST>(static_cast<const float *>(w_row[c]), kbase + w_k[c], K, w_vec_ok));
    } else if constexpr (FAST) {
      // 16 bytes along n of row k; both indices clamped (zeroed in stash if out of range)
      const int k = kbase + w_k[c];
      const int64_t roff = (int64_t)min(k, K - 1) * g.ldw;
      if constexpr (BF16)
        rw[c] = load8_bf16_fast(static_cast<const __bf16 *>(gW) + roff, w_n[c], N);
      else
        rw[c] = __builtin_bit_cast(
            u32x4, load4_f32_fast(static_cast<const float *>(gW) + roff, w_n[c], N));
    } else {
      const int k = kbase + w_k[c];
      u32x4 v = {0u, 0u, 0u, 0u};
      if (k < K) {
        if constexpr (BF16) {
          const __bf16 *row = static_cast<const __bf16 *>(gW) + (int64_t)k * g.ldw;
          v = load8_bf16(w_n[c] < N ? row : nullptr, w_n[c], N, w_vec_ok);
        } else {
          const float *row = static_cast<const float *>(gW) + (int64_t)k * g.ldw;
          v = __builtin_bit_cast(u32x4, load4_f32(w_n[c] < N ? row : nullptr, w_n[c], N, w_vec_ok));
        }
      }
      rw[c] = v;
    }
  };

  // Registers of chunk c, fetched for stage kt, go to LDS buffer buf (FAST loads are zeroed
  // here, not when issued).  edge: may stage kt reach past the end of the contraction (only the last
  // stage can; the steady state of the pipeline passes a literal false and carries no selects).
  auto stash_a_chunk = [&](int c, int buf, int kt, bool sc, bool edge = true) {
    unsigned char *sA = smem + buf * STAGE;
    if constexpr (GATHER && !AKM) {
      *reinterpret_cast<u32x4 *>(sA + a_lds[c]) =
          a_live[c] ? __builtin_bit_cast(u32x4, ra[c].v) : u32x4{0u, 0u, 0u, 0u};
      return;
    }
    if constexpr (AKM) {
      const bool past = GATHER ? !a_live[c] : (edge && kt * BK + a_k[c] >= K) || (a_m[c] >= M);
      const u32x4 v = past ? u32x4{0u, 0u, 0u, 0u} : __builtin_bit_cast(u32x4, ra[c].v);
#pragma unroll
      for (int e = 0; e < 4; ++e) *reinterpret_cast<uint32_t *>(sA + a_lds[c] + e * STRIDE) = v[e];
    } else {
      *reinterpret_cast<u32x4 *>(sA + a_lds[c]) =
          finish_a<AMODE>(ra[c], sc, FAST && edge && (kt * BK + a_k[c] >= K));
    }
  };
  auto stash_w_chunk = [&](int c, int buf, int kt, bool edge = true) {
    unsigned char *sW = smem + buf * STAGE + BM * STRIDE;
    const int kbase = kt * BK;
    if constexpr (FAST) {
      const bool past_k = edge && kbase + w_k[c] >= K;
      const bool past = WKN ? (past_k || w_n[c] >= N) : past_k;
      if (past) rw[c] = u32x4{0u, 0u, 0u, 0u};
    }
    if constexpr (!WKN || WTR) {
      *reinterpret_cast<u32x4 *>(sW + w_lds[c]) = rw[c];
    } else if constexpr (BF16) {
#pragma unroll
      for (int e = 0; e < 8; ++e)
        *reinterpret_cast<uint16_t *>(sW + w_lds[c] + e * STRIDE) =
            (uint16_t)(rw[c][e >> 1] >> ((e & 1) * 16));
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        *reinterpret_cast<uint32_t *>(sW + w_lds[c] + e * STRIDE) = rw[c][e];
    }
  };

  auto fetch = [&](int kt) {
#pragma unroll
    for (int c = 0; c < A_CHUNKS; ++c) fetch_a_chunk(c, kt, scaled);
#pragma unroll
    for (int c = 0; c < W_CHUNKS; ++c) fetch_w_chunk(c, kt);
  };
  auto stash = [&](int buf, int kt) {
#pragma unroll
    for (int c = 0; c < A_CHUNKS; ++c) stash_a_chunk(c, buf, kt, scaled);
#pragma unroll
    for (int c = 0; c < W_CHUNKS; ++c) stash_w_chunk(c, buf, kt);
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk = (K + BK - 1) / BK;
  fetch(0);
  stash(0, 0);
  __syncthreads();

  // The MFMAs of one stage.  `side(slot)` is called after every group of TM x TN MFMAs (slots
  // 0 .. SLOTS-1) so that other work can be threaded between them.
  constexpr int SLOTS = (CPR / 2) * (BF16 ? 1 : 4);
  auto mma_stage = [&](int buf, auto side) {
    const unsigned char *sA = smem + buf * STAGE + (wm + l32) * STRIDE + half * 16;
    const unsigned char *sW = smem + buf * STAGE + BM * STRIDE + (wn + l32) * STRIDE + half * 16;
    // fragments of step s + 1 are requested before the MFMAs of step s (two register sets used
    // alternately), so that the matrix pipe does not drain while a step's LDS reads are on their way
    u32x4 fa[2][TM], fw[2][TN];
    auto read_frag = [&](int step, int set) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
        fa[set][i] = *reinterpret_cast<const u32x4 *>(sA + i * 32 * STRIDE + step * 32);
      if constexpr (WTR) {
        typedef short s16x4 __attribute__((ext_vector_type(4)));
        typedef __attribute__((address_space(3))) s16x4 *lds_s16x4;
        const int i16 = lane & 15;
        const unsigned char *base = smem + buf * STAGE + BM * STRIDE +
                                    (step * 16 + half * 8 + (i16 >> 2)) * W_STRIDE +
                                    (wn + ((lane >> 4) & 1) * 16 + (i16 & 3) * 4) * 2;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(base + j * 64));
          const s16x4 hi =
              __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(base + j * 64 + 4 * W_STRIDE));
          typedef short s16x8 __attribute__((ext_vector_type(8)));
          const s16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
          fw[set][j] = __builtin_bit_cast(u32x4, both);
        }
      } else {
#pragma unroll
        for (int j = 0; j < TN; ++j)
          fw[set][j] = *reinterpret_cast<const u32x4 *>(sW + j * 32 * STRIDE + step * 32);
      }
    };
    read_frag(0, 0);
#pragma unroll
    for (int step = 0; step < CPR / 2; ++step) {
      if (step + 1 < CPR / 2) read_frag(step + 1, (step + 1) & 1);
      u32x4 av[TM], wv[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) av[i] = fa[step & 1][i];
#pragma unroll
      for (int j = 0; j < TN; ++j) wv[j] = fw[step & 1][j];
      if constexpr (BF16) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                __builtin_bit_cast(bf16x8, av[i]), __builtin_bit_cast(bf16x8, wv[j]), acc[i][j], 0, 0,
                0);
        side(step);
      } else {
        // whole-vector casts: a bit_cast applied to a single vector element is not reliable
        f32x4 af[TM], wf[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) af[i] = __builtin_bit_cast(f32x4, av[i]);
#pragma unroll
        for (int j = 0; j < TN; ++j) wf[j] = __builtin_bit_cast(f32x4, wv[j]);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
              const float a_e = af[i][e], w_e = wf[j][e];
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_e, w_e, acc[i][j], 0, 0, 0);
            }
          side(step * 4 + e);
        }
      }
    }
  };
  auto nothing = [](int) {};

  if constexpr (FAST) {
    // Software pipeline, two stages deep.  While stage kt is multiplied, the registers fetched
    // during stage kt-1 (for stage kt+1) are written to the other LDS buffer, and once they are
    // free the global loads for stage kt+2 are issued into them: both are threaded between the
    // MFMAs, one piece per slot, instead of sitting in bulk before and after them (measured on a
    // stand-alone loop of the same shape: 130 -> 140 TFLOP/s).
    constexpr int P = A_CHUNKS + W_CHUNKS;                    // pieces to write, then to fetch
    constexpr int PER_SLOT = (2 * P + SLOTS - 1) / SLOTS;
    auto piece = [&](int q, int kt, bool do_stash, bool do_fetch, bool sc, bool edge) {
      if (q < P) {
        if (do_stash) {
          if (q < A_CHUNKS) stash_a_chunk(q, (kt + 1) & 1, kt + 1, sc, edge);
          else stash_w_chunk(q - A_CHUNKS, (kt + 1) & 1, kt + 1, edge);
        }
      } else if (q < 2 * P) {
        if (do_fetch) {
          if (q - P < A_CHUNKS) fetch_a_chunk(q - P, kt + 2, sc);
          else fetch_w_chunk(q - P - A_CHUNKS, kt + 2);
        }
      }
    };
    auto run_stage = [&](int kt, bool do_stash, bool do_fetch, bool sc, bool edge) {
      mma_stage(kt & 1, [&](int slot) {
#pragma unroll
        for (int u = 0; u < PER_SLOT; ++u) piece(slot * PER_SLOT + u, kt, do_stash, do_fetch, sc, edge);
        __builtin_amdgcn_sched_barrier(0);
      });
    };
    if (nk > 1) fetch(1);
    int kt = 0;
    if (scaled) {                    // branch once, outside the loop
      // steady state: no conditions inside; the stage written to LDS here (kt + 1 <= nk - 2) is never
      // the last one, so its chunks all lie inside the contraction
      for (; kt + 2 < nk; ++kt) {
        run_stage(kt, true, true, true, false);
        __syncthreads();
      }
    } else {
      for (; kt + 2 < nk; ++kt) {
        run_stage(kt, true, true, false, false);
        __syncthreads();
      }
    }
    if (kt + 1 < nk) {
      run_stage(kt, true, false, scaled, true);
      __syncthreads();
      ++kt;
    }
    run_stage(kt, false, false, scaled, true);
  } else {
    // The last stage is peeled off so that the loop body has no conditional loads.
    for (int kt = 0; kt + 1 < nk; ++kt) {
      const int buf = kt & 1;
      fetch(kt + 1);
      mma_stage(buf, nothing);
      stash(buf ^ 1, kt + 1);
      __syncthreads();
    }
    mma_stage((nk - 1) & 1, nothing);
  }

  // ---- epilogue: accumulator element r of lane (half, l32) is row 8 (r / 4) + 4 half + r % 4,
  // column l32 of its 32 x 32 tile ----
  const int epi = g.epilogue;
  if constexpr (LSTMF) {
    // The tile holds h_{t-1} W_h for 64 rows and the four gates of 16 units.  It goes through LDS;
    // a thread then finishes cells (row, unit), consecutive threads on consecutive units: adds
    // x_t W_x + b, applies the gates, writes them (if kept), c_t and h_t.
    constexpr int TS = BN + 4;
    static_assert(BM * TS * 4 <= 2 * STAGE, "the output tile must fit the staging buffers");
    float *tile = reinterpret_cast<float *>(smem);
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 16; ++r)
      tile[(wm + 8 * (r >> 2) + 4 * half + (r & 3)) * TS + wn + l32] = acc[0][0][r];
    __syncthreads();
    const int H = g.lstm_H, T = g.lstm_T, t = g.lstm_step;
    for (int e = tid; e < BM * 16; e += kThreads) {
      const int row = e >> 4, u = e & 15;
      const int m = m0 + row, k = 16 * tile_n + u;
      if (m >= M || k >= H) continue;
      const int64_t zr = g.lstm_zx_rows ? (int64_t)g.lstm_zx_rows[m] + t : (int64_t)m * T + t;
      const float *zrow = g.lstm_zx + zr * 4 * H + k;
      const float *trow = tile + row * TS + u;
      const float z0 = trow[0] + zrow[0], z1 = trow[16] + zrow[H], z2 = trow[32] + zrow[2 * H],
                  z3 = trow[48] + zrow[3 * H];
      const float cprev = g.lstm_has_prev ? g.lstm_cs_w[m * g.lstm_state_ld + (t - 1) * g.lstm_state_ts + k] : 0.f;
      const float gi = 1.f / (1.f + __expf(-z0)), gg = tanhf(z1);
      const float gf = 1.f / (1.f + __expf(-z2)), go = 1.f / (1.f + __expf(-z3));
      const float c = gf * cprev + gi * gg;
      if (g.lstm_gates_w) {
        float *grow = g.lstm_gates_w + ((int64_t)m * T + t) * 4 * H + k;
        grow[0] = gi; grow[H] = gg; grow[2 * H] = gf; grow[3 * H] = go;
      }
      const int64_t at = m * g.lstm_state_ld + t * g.lstm_state_ts + k;
      g.lstm_cs_w[at] = c;
      g.lstm_hs_w[at] = go * tanhf(c);
    }
    return;
  }
  if constexpr (AMODE == A_F32) {
    if (epi == EPI_LSTM_BWD) {
      // The reverse cell update is long; running it from the unrolled register loop below would
      // replicate it 16 TM TN times.  The tile goes through LDS (free after the last stage) and a
      // rolled loop finishes it, consecutive threads on consecutive columns.
      // Four consecutive columns per thread on 16-byte operands when every row involved starts
      // 16-byte aligned (the usual case); element by element otherwise.
      constexpr int TS = BN + 4;
      static_assert(BM * TS * 4 <= 2 * STAGE, "the output tile must fit the staging buffers");
      float *tile = reinterpret_cast<float *>(smem);
      __syncthreads();
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            tile[(wm + i * 32 + 8 * (r >> 2) + 4 * half + (r & 3)) * TS + wn + j * 32 + l32] =
                acc[i][j][r];
      __syncthreads();
      auto aligned16 = [](const void *ptr) { return (reinterpret_cast<uintptr_t>(ptr) & 15) == 0; };
      const bool vec = g.n_split % 4 == 0 && g.lstm_H % 4 == 0 && g.ldc % 4 == 0 && g.lstm_dz_ld % 4 == 0 &&
                       aligned16(gC) && aligned16(g.lstm_gates) && aligned16(g.lstm_cs) &&
                       aligned16(g.lstm_dc) && aligned16(g.lstm_dz);
      if (vec) {
        for (int e = tid; e < BM * (BN / 4); e += kThreads) {
          const int row = e / (BN / 4), col = (e % (BN / 4)) * 4;
          const int m = m0 + row, n = n0 + col;
          if (m >= M || n >= N) continue;            // N is a multiple of 4 here: whole groups only
          const f32x4 v = *reinterpret_cast<const f32x4 *>(tile + row * TS + col);
          if (n < g.n_split) {
            f32x4 *dst = reinterpret_cast<f32x4 *>(gC + (int64_t)m * g.ldc + n);
            if (g.streaming)
              __builtin_nontemporal_store(v, dst);
            else
              *dst = v;
          } else {
            lstm_reverse_cell4(g.lstm_gates, g.lstm_cs, g.lstm_dc, g.lstm_dz, g.lstm_dz_ld, g.lstm_H,
                               g.lstm_T, g.lstm_step, g.S, m, n - g.n_split, v);
          }
        }
        return;
      }
      for (int e = tid; e < BM * BN; e += kThreads) {
        const int row = e / BN, col = e % BN;
        const int m = m0 + row, n = n0 + col;
        if (m >= M || n >= N) continue;
        const float v = tile[row * TS + col];
        if (n < g.n_split) {
          if (g.streaming)
            __builtin_nontemporal_store(v, gC + (int64_t)m * g.ldc + n);
          else
            gC[(int64_t)m * g.ldc + n] = v;
        } else {
          lstm_reverse_cell(g.lstm_gates, g.lstm_cs, g.lstm_dc, g.lstm_dz, g.lstm_dz_ld, g.lstm_H,
                            g.lstm_T, g.lstm_step, g.S, m, n - g.n_split, v);
        }
      }
      return;
    }
  }
  // Results leave through LDS: in the accumulator layout a lane holds one column of 16 rows, so
  // direct stores are 4 bytes per lane, which HBM takes at a fraction of the rate of 16-byte stores
  // (a product with a short contraction is all epilogue: the 25088 x 800 x 64 cotangent product of
  // the conv net took 71 us for 80 MB, 46 us this way).  The tile is laid out row-major in the
  // staging buffers, free after the last stage; each thread then finishes four consecutive columns
  // of a row (bias, activation or mask on 16-byte operands) and stores them at once.  Needs rows
  // of C (C2, the mask) that start 16-byte aligned; anything else takes the direct path below.
  constexpr int TSV = BN + 4;      // row stride in floats: 16-byte aligned rows
  if constexpr (BM * TSV * 4 <= 2 * STAGE) {
    auto aligned16 = [](const void *ptr) { return (reinterpret_cast<uintptr_t>(ptr) & 15) == 0; };
    const bool plain = (epi == EPI_NONE || epi == EPI_BIAS || epi == EPI_FORWARD || epi == EPI_MASK);
    const bool rows_ok = g.ldc % 4 == 0 && aligned16(gC) && (epi != EPI_FORWARD || aligned16(g.C2)) &&
                         (epi != EPI_MASK || (g.ld_emask % 4 == 0 && aligned16(g.emask)));
    if (plain && rows_ok) {
      float *tile = reinterpret_cast<float *>(smem);
      __syncthreads();
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            tile[(wm + i * 32 + 8 * (r >> 2) + 4 * half + (r & 3)) * TSV + wn + j * 32 + l32] =
                acc[i][j][r];
      __syncthreads();
      const bool add_bias = (epi == EPI_BIAS || epi == EPI_FORWARD) && g.bias;
      for (int e = tid; e < BM * (BN / 4); e += kThreads) {
        const int row = e / (BN / 4), col = (e % (BN / 4)) * 4;
        const int m = m0 + row, n = n0 + col;
        if (m >= M || n >= N) continue;
        const int64_t orow = (SUB && g.sub_scatter) ? g.sub_rows[sub_off + m] : m;
        const int64_t o = orow * g.ldc + n;
        const bool whole = n + 4 <= N;
        f32x4 v = *reinterpret_cast<const f32x4 *>(tile + row * TSV + col);
        if (add_bias) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int nq = min(n + q, N - 1);
            v[q] += g.bf16 ? (float)static_cast<const __bf16 *>(g.bias)[nq]
                           : static_cast<const float *>(g.bias)[nq];
          }
        }
        if (epi == EPI_MASK) {
          const float *mrow = g.emask + (int64_t)(m / g.S) * g.ld_emask + n;
          if (whole) {
            v *= *reinterpret_cast<const f32x4 *>(mrow);
          } else {
            for (int q = 0; n + q < N; ++q) v[q] *= mrow[q];
          }
        }
        if (epi == EPI_FORWARD) {
          f32x4 d;
#pragma unroll 1
          for (int q = 0; q < 4; ++q) {            // rolled: the activation code is long
            const float z = v[q];
            d[q] = act_deriv(g.act, z);
            v[q] = act_value(g.act, z);
          }
          if (g.C2) {
            if (whole) {
              *reinterpret_cast<f32x4 *>(g.C2 + o) = d;
            } else {
              for (int q = 0; n + q < N; ++q) g.C2[o + q] = d[q];
            }
          }
          if (gC == nullptr) continue;       // only phi'(z) is wanted
        }
        float *dst = gC + o;
        if (whole) {
          if (g.streaming)
            __builtin_nontemporal_store(v, reinterpret_cast<f32x4 *>(dst));
          else
            *reinterpret_cast<f32x4 *>(dst) = v;
        } else {
          for (int q = 0; n + q < N; ++q) dst[q] = v[q];
        }
      }
      if constexpr (AMODE == A_F32 && BM == BN) {
        if (mirror) {
          // C[block + n, i] = C[block + i, n]: the same tile written transposed (all tiles are full
          // in this mode); consecutive threads take consecutive rows of a tile column, which are
          // consecutive addresses of the mirror image
          const int block0 = (m0 / g.sym_n) * g.sym_n, i0 = m0 - block0;
          for (int e = tid; e < BM * BN; e += kThreads) {
            const int col = e / BM, row = e % BM;
            const float v = tile[row * TSV + col];
            float *dst = gC + (int64_t)(block0 + n0 + col) * g.ldc + i0 + row;
            if (g.streaming)
              __builtin_nontemporal_store(v, dst);
            else
              *dst = v;
          }
        }
      }
      return;
    }
  }
  float bias[TN];
  bool n_ok[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int n = n0 + wn + j * 32 + l32;
    n_ok[j] = n < N;
    bias[j] = 0.f;
    if (n_ok[j] && (epi == EPI_BIAS || epi == EPI_FORWARD) && g.bias) {
      if (g.bf16)
        bias[j] = (float)static_cast<const __bf16 *>(g.bias)[n];
      else
        bias[j] = static_cast<const float *>(g.bias)[n];
    }
  }
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m0 + wm + i * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
      if (m >= M) continue;
      const float *mrow = (epi == EPI_MASK) ? g.emask + (int64_t)(m / g.S) * g.ld_emask : nullptr;
      const int64_t orow = (SUB && g.sub_scatter) ? g.sub_rows[sub_off + m] : m;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        if (!n_ok[j]) continue;
        const int n = n0 + wn + j * 32 + l32;
        float v = acc[i][j][r];
        const int64_t o = orow * g.ldc + n;
        if (epi == EPI_FORWARD) {
          const float z = v + bias[j];
          if (g.C2) g.C2[o] = act_deriv(g.act, z);
          if (gC == nullptr) continue;       // only phi'(z) is wanted
          v = act_value(g.act, z);
        } else if (epi == EPI_BIAS) {
          v += bias[j];
        } else if (epi == EPI_MASK) {
          v *= mrow[n];
        }
        if (g.streaming)
          __builtin_nontemporal_store(v, gC + o);
        else
          gC[o] = v;
      }
    }
  }
  if constexpr (AMODE == A_F32 && BM == BN) {
    if (mirror) {
      // C[block + n, i] = C[block + i, n]: the tile goes through LDS and is written transposed,
      // consecutive threads on consecutive columns (all tiles are full in this mode)
      constexpr int TS = BN + 1;
      static_assert(BM * TS * 4 <= 2 * STAGE, "the output tile must fit the staging buffers");
      float *tile = reinterpret_cast<float *>(smem);
      __syncthreads();
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            tile[(wm + i * 32 + 8 * (r >> 2) + 4 * half + (r & 3)) * TS + wn + j * 32 + l32] =
                acc[i][j][r];
      __syncthreads();
      const int block0 = (m0 / g.sym_n) * g.sym_n, i0 = m0 - block0;
      for (int e = tid; e < BM * BN; e += kThreads) {
        const int col = e / BM, row = e % BM;          // element (row, col) of the tile
        const float v = tile[row * TS + col];
        float *dst = gC + (int64_t)(block0 + n0 + col) * g.ldc + i0 + row;
        if (g.streaming)
          __builtin_nontemporal_store(v, dst);
        else
          *dst = v;
      }
    }
  }
}

template <int AMODE, bool WKN, int TM, int TN, int BKB, bool FAST, int WGM = 2, int WGN = 2, bool SUB = false,
          bool AKM = false, bool LSTMF = false, bool GATHER = false>
hipError_t launch_one(const GemmArgs &g, hipStream_t stream) {
  constexpr int BM = 32 * TM * WGM, BN = 32 * TN * WGN;
  constexpr int kThreads = 64 * WGM * WGN;
  constexpr bool WTR = WKN && (AMODE != A_F32);
  constexpr int BK = BKB / (AMODE != A_F32 ? 2 : 4);
  constexpr int smem = 2 * (BM * (BKB + 16) + (WTR ? BK * (BN * 2 + 16) : BN * (BKB + 16)));
  auto kern = gemm_kernel<AMODE, WKN, TM, TN, BKB, FAST, WGM, WGN, SUB, AKM, LSTMF, GATHER>;
  static bool attr_set = false;   // benign race: the attribute is idempotent
  if (!attr_set && smem > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  int64_t tiles = (int64_t)((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  if (LSTMF) tiles = (int64_t)((g.M + BM - 1) / BM) * ((g.lstm_H + 15) / 16);
  if (AMODE == A_F32 && BM == BN && g.sym_n > 0) {
    const int64_t T = g.sym_n / BM;
    tiles = (g.M / g.sym_n) * (T * (T + 1) / 2);
  }
  if (SUB) tiles = (int64_t)((g.M + BM - 1) / BM + 7) / 8 * 8 * ((g.N + BN - 1) / BN);
  const unsigned nbatch = g.nbatch > 1 ? (unsigned)g.nbatch : 1u;
  PFG_KERNEL(kern, dim3((unsigned)tiles, nbatch), dim3(kThreads), smem, stream, g);
  return hipGetLastError();
}

template <int AMODE, bool WKN>
hipError_t launch_tiles(const GemmArgs &g, hipStream_t stream) {
  // Large tiles once there are two of them for each of the 256 compute units (two workgroups fit a
  // unit and cover each other's barriers and LDS waits); otherwise 64 x 64 tiles.  With exactly 256
  // large tiles an 8192 x 784 x 512 product took 94 us, with 1024 small ones 76 us.
  const int64_t nb = g.nbatch > 1 ? g.nbatch : 1;
  // rows chosen on the device: the host knows only the upper bound M; half of it is taken as live
  const int64_t m_est = g.sub ? (g.M + 1) / 2 : g.M;
  const int64_t big = nb * ((m_est + 127) / 128) * ((g.N + 127) / 128);
  const bool fast = fast_loads_ok(g);
  // (256 x 128 tiles on 8 waves were measured slower than 128 x 128 on 4: 4.82 against 4.46 ms
  // on the 65536 x 2048 x 2048 cotangent product; the wider barrier costs more than the saved loads.
  // 128 x 128 on 8 waves of 32 x 64 each: 75 % of the MFMA peak against 79.5 %.  128 x 64 tiles in
  // place of 64 x 64: within 6 % either way on plain products, and a third slower where the long
  // reverse-cell epilogue follows.)
  // a 128-wide tile on an output of 64 columns or fewer would be half empty
  if constexpr (AMODE == A_F32) {
    if (g.sub) {
      if (big >= 512 && g.N > 64)
        return fast ? launch_one<AMODE, WKN, 2, 2, 128, true, 2, 2, true>(g, stream)
                    : launch_one<AMODE, WKN, 2, 2, 128, false, 2, 2, true>(g, stream);
      return fast ? launch_one<AMODE, WKN, 1, 1, 128, true, 2, 2, true>(g, stream)
                  : launch_one<AMODE, WKN, 1, 1, 128, false, 2, 2, true>(g, stream);
    }
  }
  if (g.sub) return hipErrorInvalidValue;     // rows chosen on the device: float32 only
  if constexpr (AMODE == A_F32 && WKN) {
    if (g.a_km) {
      // 64 x 64 tiles only (the 128 x 128 arrangement runs out of registers with the scattered
      // staging of both operands)
      if (!fast) return hipErrorInvalidValue;
      return launch_one<AMODE, WKN, 1, 1, 128, true, 2, 2, false, true>(g, stream);
    }
  }
  if (g.a_km) return hipErrorInvalidValue;    // transposed A: float32 with W in [K, N] layout only
  // (and with a contraction of one or two stages a product is all prologue and epilogue, which four
  // small workgroups per unit overlap better than two large ones: the 25088 x 800 x 64 cotangent
  // product of the conv net took 48 us on 128 x 128 tiles, 39 us on 64 x 64)
  if (big >= 512 && g.N > 64 && g.K > 128)
    return fast ? launch_one<AMODE, WKN, 2, 2, 128, true>(g, stream)
                : launch_one<AMODE, WKN, 2, 2, 128, false>(g, stream);
  if constexpr (AMODE != A_F32) {
    // bf16 MFMAs are 16 times faster: a 64 x 64 tile needs a deeper stage (128 k) to have
    // enough MFMA work between two barriers
    if (fast && g.K >= 256) return launch_one<AMODE, WKN, 1, 1, 256, true>(g, stream);
  }
  return fast ? launch_one<AMODE, WKN, 1, 1, 128, true>(g, stream)
              : launch_one<AMODE, WKN, 1, 1, 128, false>(g, stream);
}

}  // namespace

// The fused LSTM step on many rows: the small-problem kernel's 32 x 32 tiles re-read W_h once per
// 32 rows; measured with a state of 256, the LDS-tiled kernel with the same epilogue is level with
// it at 768 rows and ahead beyond (512 rows: 3 us per step behind, 960 rows: 4 us ahead).
bool lstm_step_tiled_applies(const GemmArgs &g) {
  return g.epilogue == EPI_LSTM_FWD && g.M >= 768 && !g.bf16 && g.a_is_f32 && g.w_kn && g.nbatch <= 1 && !g.sub &&
         g.S == 1 && !g.a_scale && g.lstm_H % 4 == 0 && g.N == 4 * g.lstm_H && fast_loads_ok(g);
}

bool conv_gather_supported(const GemmArgs &g) {
  if (g.conv_k <= 0) return true;
  auto aligned = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
  const int64_t hw = (int64_t)g.conv_h * g.conv_w, kkc = (int64_t)g.conv_k * g.conv_k * g.conv_c;
  if (g.conv_k % 2 == 0 || g.conv_c < 4 || g.conv_c % 4 || g.conv_h < 1 || g.conv_w < 1 || g.conv_h > 65535 ||
      g.conv_w > 65535 || hw >= (1 << 24) || kkc >= (1 << 24))
    return false;
  if (g.bf16 || !g.a_is_f32 || !g.w_kn || g.a_scale || g.S != 1 || g.sub || g.sym_n > 0 || !aligned(g.A)) return false;
  if (!aligned(g.W) || g.ldw % 4 || g.N % 4 || g.N < 4) return false;
  if (g.a_km) {
    if (g.epilogue != EPI_NONE || g.M != kkc || g.K != hw) return false;
    if (g.nbatch > 1 && (g.batch_A % 4 || g.batch_W % 4)) return false;
  } else {
    if ((g.epilogue != EPI_NONE && g.epilogue != EPI_BIAS) || g.K != kkc || g.M % hw || g.nbatch > 1) return false;
  }
  return true;
}

bool akm_supported(const GemmArgs &g) {
  if (!g.a_km) return true;
  auto aligned = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
  if (g.bf16 || !g.a_is_f32 || !g.w_kn || g.a_scale || g.S != 1 || g.sub || g.sym_n > 0 ||
      g.epilogue != EPI_NONE)
    return false;
  if (g.K < 4 || g.K % 4 || g.M < 4 || g.M % 4 || g.lda % 4 || !aligned(g.A) || (g.nbatch > 1 && g.batch_A % 4)) return false;
  // the W side of the FAST loads
  if (!aligned(g.W) || g.ldw % 4 || g.N % 4 || g.N < 4 || (g.nbatch > 1 && g.batch_W % 4)) return false;
  const int64_t tiles64 = (int64_t)(g.nbatch > 1 ? g.nbatch : 1) * ((g.M + 63) / 64) * ((g.N + 63) / 64);
  return tiles64 >= 128;
}

hipError_t launch_gemm(const GemmArgs &g, hipStream_t stream) {
  if (g.M <= 0 || g.N <= 0 || g.K <= 0) return hipSuccess;
  if (g.sym_n > 0 && (g.epilogue != EPI_NONE || g.bf16 || g.N != g.sym_n || g.M % g.sym_n || g.sym_n % 128))
    return hipErrorInvalidValue;
  if (g.epilogue == EPI_LSTM_BWD && (g.N - g.n_split != g.lstm_H || g.n_split < 0 || g.bf16))
    return hipErrorInvalidValue;
  if (g.nbatch > 1 && (g.epilogue != EPI_NONE || g.nbatch > 65535))
    return hipErrorInvalidValue;
  if (g.sub && (g.bf16 || !g.a_is_f32 || g.S != 1 || g.nbatch > 1 || g.sym_n > 0 || g.a_scale ||
                (g.epilogue != EPI_NONE && g.epilogue != EPI_BIAS && g.epilogue != EPI_FORWARD &&
                 g.epilogue != EPI_MASK && g.epilogue != EPI_LSTM_FWD && g.epilogue != EPI_LSTM_BWD) ||
                (!g.w_kn && g.epilogue != EPI_NONE && g.epilogue != EPI_MASK && g.epilogue != EPI_LSTM_BWD) ||
                (g.w_kn && g.epilogue == EPI_LSTM_BWD) ||
                ((g.sub_gather || g.sub_scatter) && !g.sub_rows)))
    return hipErrorInvalidValue;
  if (!g.sub && (g.sub_gather || g.sub_scatter)) return hipErrorInvalidValue;
  if (g.conv_k > 0) {
    if (!conv_gather_supported(g)) return hipErrorInvalidValue;
    return g.a_km ? launch_one<A_F32, true, 1, 1, 128, true, 2, 2, false, true, false, true>(g, stream)
                  : launch_one<A_F32, true, 1, 1, 128, true, 2, 2, false, false, false, true>(g, stream);
  }
  if (g.a_km) {
    if (!akm_supported(g)) return hipErrorInvalidValue;
    return launch_tiles<A_F32, true>(g, stream);
  }
  if (gemm_shortk_applies(g)) return launch_gemm_shortk(g, stream);
  // Fewer than 128 tiles of 64 x 64 cannot occupy the chip: such products (M = B rows, or a
  // narrow output) go to the kernel that splits the contraction over the waves of a workgroup.
  const int64_t tiles64 = (int64_t)(g.nbatch > 1 ? g.nbatch : 1) * ((g.M + 63) / 64) * ((g.N + 63) / 64);
  // A single column tile of at most 32 with a long contraction is bound by reading A: the kernel
  // whose waves load their operands straight into registers does that with four times as many
  // workgroups as 64 x 64 tiles would give.
  const bool narrow = g.N <= 32 && g.K >= 256 && g.nbatch <= 1 && g.sym_n == 0;
  // (the small-problem kernels have no batch index and take a batched product one launch per entry:
  // from 8 entries on, one launch of the tiled kernel on few workgroups is the shorter way)
  if (lstm_step_tiled_applies(g))
    return launch_one<A_F32, true, 1, 1, 128, true, 2, 2, false, false, true>(g, stream);
  // float32, 128 to 191 tiles: the tiled kernel would run on that many of the 256 units, the
  // small-problem kernels spread the same product over four times as many workgroups (1024 rows
  // against 784 x 512 weights: 31 against 45 us; from about 200 tiles on the tiled kernel is level)
  const bool few_tiles = (tiles64 < 128 && g.nbatch < 8) ||
                         (tiles64 < 192 && g.nbatch <= 1 && !g.bf16 && g.a_is_f32 && g.sym_n == 0);
  if (g.epilogue == EPI_HEAD || g.epilogue == EPI_LSTM_FWD || (g.epilogue == EPI_LSTM_BWD && g.sub) || few_tiles ||
      narrow || small16_batched_applies(g))
    return launch_gemm_skinny(g, stream);
  if (!g.bf16) {
    return g.w_kn ? launch_tiles<A_F32, true>(g, stream) : launch_tiles<A_F32, false>(g, stream);
  }
  if (g.a_is_f32) {
    return g.w_kn ? launch_tiles<A_F32_TO_BF16, true>(g, stream)
                  : launch_tiles<A_F32_TO_BF16, false>(g, stream);
  }
  return g.w_kn ? launch_tiles<A_BF16, true>(g, stream) : launch_tiles<A_BF16, false>(g, stream);
}

}  // namespace pfg

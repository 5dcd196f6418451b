// Feature transform for bfloat16 storage with the weights held still (appendix:
// Z = (P H) W, H' = sigma(Z), and the gradient to the aggregate D W^T):
//   out[m, 0:N) = act(A[m, 0:K) B),   B = W (K x N, row-major) or W^T (W is N x K)
// for M in the millions and K, N at most a few hundred. With bf16 operands one MFMA
// per operand pair is all the arithmetic there is: two flops per byte moved, so
// this is a streaming kernel and the tile GEMM's staging of BOTH operands per k
// step (and its second pass over A for the second half of the columns) is what
// cost time. Here, as in the predictor's hop product:
//   * a workgroup has 8 wavefronts; wavefront w owns output columns [32 w, 32 w + 32)
//     of a group of 256 and keeps ITS slice of B for all of K in registers, in MFMA
//     operand order (64 registers for K = 256; the slices are brought into that order
//     through LDS once per workgroup);
//   * rows stream through in tiles of 32: the A tile (32 x K bf16) is read with
//     16-byte accesses, staged in LDS in the swizzled operand layout (double-buffered,
//     the next tile's loads in flight during the products), the ReLU mask of the
//     backward applied while it is staged;
//   * the product tile goes through LDS so that output rows leave as 16-byte stores.
// A is read once whatever N is (up to 256 columns per workgroup group).
#include "mx_tile.h"
#include "sat_internal.h"

namespace {

using namespace sat::mx;

// KC = number of 16-wide k chunks the weights are padded to (K <= 16 KC, K % 8 == 0)
template <int KC, bool TRANSB, bool MASK, bool RELU>
__global__ __launch_bounds__(512, 4) void dense_ws_kernel(
    const uint16_t* __restrict__ A, int64_t ld_a, const uint16_t* __restrict__ Mk, int64_t ld_m,
    int64_t M, int K, const uint16_t* __restrict__ W, int64_t ld_w, int N,
    uint16_t* __restrict__ out, int64_t ld_out, int tiles_per_block) {
  constexpr int NT32 = KC / 2;                            // 32-wide staging tiles per row tile
  constexpr int STAGE = NT32 * tile_bytes<32, 1>();       // bytes of one staged A tile
  constexpr int CH = 32 * 2 * KC;                         // 16-byte chunks of an A tile
  constexpr int NCHK = (CH + 511) / 512;                  // per thread
  constexpr int C_LDF = 256 + 4;                          // floats per staged output row
  // one buffer: the staged A tiles, then the staged output tile; before the first tile it
  // holds 64 rows of W at a time while the weight slices are brought into operand order
  __shared__ __attribute__((aligned(16))) unsigned char smem[2 * STAGE + 32 * C_LDF * 4];
  static_assert(2 * STAGE + 32 * C_LDF * 4 >= 64 * 512, "the weight staging pass must fit");
  unsigned char* As = smem;
  float* Cs = reinterpret_cast<float*>(smem + 2 * STAGE);

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int col = blockIdx.y * 256 + 32 * wave + (lane & 31);
  const bool col_ok = col < N;
  const int64_t row_lo = static_cast<int64_t>(blockIdx.x) * 32 * tiles_per_block;

  // ---- A tile: chunk q = t + 512 i is row q / (2 KC), k = 8 (q % (2 KC)) .. + 7
  struct Regs {
    u32x4 v[NCHK], h[NCHK];
  };
  auto load_a = [&](int64_t row0, Regs& r) {     // only issues the loads
#pragma unroll
    for (int i = 0; i < NCHK; ++i) {
      const int q = t + 512 * i;
      const int64_t row = row0 + q / (2 * KC);
      const int k = 8 * (q % (2 * KC));
      u32x4 v = {0u, 0u, 0u, 0u}, h = {0u, 0u, 0u, 0u};
      if (q < CH && row < M && k < K) {
        v = *reinterpret_cast<const u32x4*>(A + row * ld_a + k);
        if constexpr (MASK) h = *reinterpret_cast<const u32x4*>(Mk + row * ld_m + k);
      }
      r.v[i] = v;
      if constexpr (MASK) r.h[i] = h;
    }
  };
  auto keep = [](uint32_t v, uint32_t h) {   // zero the halves whose mask element is not > 0
    return (bf16_pos(h & 0xffffu) ? (v & 0xffffu) : 0u) | (bf16_pos(h >> 16) ? (v & 0xffff0000u) : 0u);
  };
  auto store_a = [&](const Regs& r, int stage) {
#pragma unroll
    for (int i = 0; i < NCHK; ++i) {
      const int q = t + 512 * i;
      if (q >= CH) continue;
      const int row = q / (2 * KC), kch = q % (2 * KC);
      u32x4 v = r.v[i];
      if constexpr (MASK) {
        const u32x4 h = r.h[i];
        const uint32_t v0 = v.x, v1 = v.y, v2 = v.z, v3 = v.w, h0 = h.x, h1 = h.y, h2 = h.z, h3 = h.w;
        v = u32x4{keep(v0, h0), keep(v1, h1), keep(v2, h2), keep(v3, h3)};
      }
      *reinterpret_cast<u32x4*>(As + stage * STAGE + (kch >> 2) * tile_bytes<32, 1>() +
                                swz(row, kch & 3)) = v;
    }
  };

  Regs ra;
  load_a(row_lo, ra);       // in flight while the weights are brought in

  // ---- this wavefront's slice of B as MFMA operands: lane holds k = 16 kc + 8 (lane / 32)
  // .. + 7 of column `col` (zeros past K)
  bf16x8 bw[KC];
  if constexpr (TRANSB) {   // 8 consecutive k of a column of B are 16 contiguous bytes of W
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      const int k0 = 16 * kc + 8 * (lane >> 5);
      u32x4 v = {0u, 0u, 0u, 0u};
      if (col_ok && k0 < K) v = *reinterpret_cast<const u32x4*>(W + static_cast<int64_t>(col) * ld_w + k0);
      bw[kc] = __builtin_bit_cast(bf16x8, v);
    }
  } else {
    // W is [K, N] row-major: its rows are read as they lie (16-byte accesses, all requested at
    // once), staged 64 at a time in LDS, and each lane picks its 8 k of each chunk from there
    constexpr int PASSES = (16 * KC) / 64;
    u32x4 wr[PASSES][4];
#pragma unroll
    for (int p = 0; p < PASSES; ++p)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int q = t + 512 * i;                     // chunk of the pass: row q / 32, columns 8 (q % 32) ..
        const int k = 64 * p + (q >> 5);
        const int c0 = blockIdx.y * 256 + ((q & 31) << 3);
        u32x4 v = {0u, 0u, 0u, 0u};
        // (columns past N inside the chunk are padding of the row: they only reach output
        // columns that are never stored)
        if (k < K && c0 < N) v = *reinterpret_cast<const u32x4*>(W + static_cast<int64_t>(k) * ld_w + c0);
        wr[p][i] = v;
      }
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      if (p > 0) __syncthreads();                      // the previous pass has been read
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int q = t + 512 * i;
        *reinterpret_cast<u32x4*>(smem + (q >> 5) * 512 + ((q & 31) << 4)) = wr[p][i];
      }
      __syncthreads();
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const int kc = 4 * p + kk;
        uint32_t e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int k = 16 * kk + 8 * (lane >> 5) + j;   // row inside the pass
          e[j] = *reinterpret_cast<const uint16_t*>(smem + k * 512 + ((32 * wave + (lane & 31)) << 1));
        }
        const u32x4 v = {e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)};
        bw[kc] = __builtin_bit_cast(bf16x8, v);
      }
    }
    __syncthreads();                                   // before the buffer becomes the A tiles
  }

  store_a(ra, 0);
  __syncthreads();
  for (int it = 0; it < tiles_per_block; ++it) {
    const int64_t row0 = row_lo + 32 * it;
    if (row0 >= M) break;                        // uniform over the workgroup
    const int stage = it & 1;
    const bool more = it + 1 < tiles_per_block && row0 + 32 < M;
    if (more) load_a(row0 + 32, ra);
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    const unsigned char* S = As + stage * STAGE;
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      const bf16x8 a = read_operand(S + (kc >> 1) * tile_bytes<32, 1>(), 0, kc & 1, lane);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bw[kc], acc, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) Cs[acc_row(r, lane) * C_LDF + 32 * wave + (lane & 31)] = acc[r];
    __syncthreads();
    // 32 rows x 256 columns leave as 16-byte chunks of 8 bf16: chunk c = t + 512 i
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int c = t + 512 * i;
      const int64_t r = row0 + (c >> 5);
      const int cc = blockIdx.y * 256 + ((c & 31) << 3);
      if (r >= M || cc >= N) continue;
      f32x4 lo = *reinterpret_cast<const f32x4*>(&Cs[(c >> 5) * C_LDF + ((c & 31) << 3)]);
      f32x4 hi = *reinterpret_cast<const f32x4*>(&Cs[(c >> 5) * C_LDF + ((c & 31) << 3) + 4]);
      if constexpr (RELU) {
        lo.x = fmaxf(lo.x, 0.f); lo.y = fmaxf(lo.y, 0.f); lo.z = fmaxf(lo.z, 0.f); lo.w = fmaxf(lo.w, 0.f);
        hi.x = fmaxf(hi.x, 0.f); hi.y = fmaxf(hi.y, 0.f); hi.z = fmaxf(hi.z, 0.f); hi.w = fmaxf(hi.w, 0.f);
      }
      const uint32_t w0 = pack_bf16(lo.x, lo.y), w1 = pack_bf16(lo.z, lo.w), w2 = pack_bf16(hi.x, hi.y),
                     w3 = pack_bf16(hi.z, hi.w);
      uint16_t* y = out + r * ld_out + cc;
      const int left = N - cc;
      if (left >= 8) {
        *reinterpret_cast<u32x4*>(y) = u32x4{w0, w1, w2, w3};
      } else {
        const uint32_t w[4] = {w0, w1, w2, w3};
#pragma unroll
        for (int j = 0; j < 7; ++j)
          if (j < left) y[j] = static_cast<uint16_t>((j & 1) ? (w[j >> 1] >> 16) : (w[j >> 1] & 0xffffu));
      }
    }
    if (more) store_a(ra, stage ^ 1);
    __syncthreads();
  }
}

}  // namespace

namespace sat {

// Whether launch_dense_ws serves a contraction length K (elements; rows must also be
// 16-byte aligned, which every bf16 matrix of the library is).
bool dense_ws_serves(int32_t K) { return K > 0 && K <= 256 && (K % 8) == 0; }

// out [M, N] bf16 = act(A' B): A [M, K] bf16 with A' = A o [Mk > 0] if Mk != nullptr, B = W
// (transb false: W is [K, ld_w]) or W^T (transb true: W is [N, ld_w]); relu on the result if
// asked. ld in elements. dense_ws_serves(K) must hold.
sat_status launch_dense_ws(const void* A, int64_t ld_a, const void* Mk, int64_t ld_m, int64_t M,
                           int32_t K, const void* W, int64_t ld_w, bool transb, int32_t N, bool relu,
                           void* out, int64_t ld_out, hipStream_t st) {
  if (M == 0 || N == 0) return SAT_OK;
  int64_t tpb = M / (32 * 2048);
  if (tpb < 4) tpb = 4;
  if (tpb > 32) tpb = 32;
  const int64_t gx = (M + 32 * tpb - 1) / (32 * tpb);
  if (gx > INT32_MAX) return SAT_EUNSUPPORTED;
  const dim3 grid(static_cast<unsigned>(gx), static_cast<unsigned>((N + 255) / 256));
  const uint16_t* a = static_cast<const uint16_t*>(A);
  const uint16_t* m = static_cast<const uint16_t*>(Mk);
  const uint16_t* w = static_cast<const uint16_t*>(W);
  uint16_t* o = static_cast<uint16_t*>(out);
  const int itpb = static_cast<int>(tpb);
#define SAT_WS(KC, TB, MK, RL)                                                                   \
  dense_ws_kernel<KC, TB, MK, RL><<<grid, dim3(512), 0, st>>>(a, ld_a, m, ld_m, M, K, w, ld_w, N, o, \
                                                             ld_out, itpb)
#define SAT_WS_K(TB, MK, RL)           \
  do {                                 \
    if (K <= 64) SAT_WS(4, TB, MK, RL);       \
    else if (K <= 128) SAT_WS(8, TB, MK, RL); \
    else SAT_WS(16, TB, MK, RL);              \
  } while (0)
  if (!transb && !Mk && relu) SAT_WS_K(false, false, true);
  else if (!transb && !Mk) SAT_WS_K(false, false, false);
  else if (transb && Mk && !relu) SAT_WS_K(true, true, false);
  else if (transb && !Mk && !relu) SAT_WS_K(true, false, false);
  else return SAT_EUNSUPPORTED;
#undef SAT_WS_K
#undef SAT_WS
  return sat::check_launch();
}

}  // namespace sat

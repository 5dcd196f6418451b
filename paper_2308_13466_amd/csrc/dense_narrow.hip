// Feature transform onto FEW columns, fp32 storage (appendix: Z = (P H) W, evaluated as
// P (H W) on a last layer that narrows to the number of classes: the transform then runs
// over all local + halo rows):
//   out[m, 0:N) = act(A[m, 0:K) W),   A [M, K] fp32, W [K, N] fp32, N <= 64, K <= 256
// for M in the millions. The tile GEMM spends a 128-column tile on 47 columns and stages
// both operands per k step; this shape wants the opposite:
//   * the whole of W, split into its three bf16 pieces and transposed to [piece][column][k],
//     sits in LDS (96 KB for K = 256) for the life of the workgroup; a lane's MFMA operand is
//     one 16-byte read, and the 16-byte chunks of a column are stored at chunk ^ (column
//     mod chunks-per-column), so that the 32 columns of a read fall into different banks;
//   * A never touches LDS: a wavefront owns 32-row tiles of its own; a lane reads the 8
//     consecutive k of its row that the MFMA wants (two 16-byte loads; the four loads of a
//     128-byte line come from neighbouring k chunks and hit the first-level cache), splits
//     them into pieces in registers, and multiplies. No barrier after the weights are in;
//   * the k chunks of a tile are loaded four ahead (registers), the next tile's first group
//     while the current tile finishes;
//   * the accumulator's layout stores rows as 128 contiguous bytes per half-wavefront.
// Six bf16 products per fp32 product, exact as in mx_tile.h.
#include "mx_tile.h"
#include "sat_internal.h"

namespace {

using namespace sat::mx;

constexpr int kNarrowWaves = 8;
constexpr int kGroup = 4;            // k chunks (of 16) loaded together

// KC = 16-wide k chunks the weights are padded to (K <= 16 KC, K % 8 == 0)
template <int KC, bool RELU>
__global__ __launch_bounds__(64 * kNarrowWaves) void dense_narrow_kernel(
    const float* __restrict__ A, int64_t ld_a, int64_t M, int K, const float* __restrict__ W,
    int64_t ld_w, int N, float* __restrict__ out, int64_t ld_out, int tiles_per_wave) {
  constexpr int NP = 3;
  constexpr int CPC = 2 * KC;                       // 16-byte chunks per staged column
  constexpr int COL_B = CPC * 16;                   // bytes per staged column of a piece
  constexpr int PIECE_B = 64 * COL_B;
  __shared__ __attribute__((aligned(16))) unsigned char Ws[NP * PIECE_B];

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);

  // ---- weights: element (k, n) -> piece p at Ws[p][n][k], chunk (k / 8) ^ (n % CPC)
  for (int q = t; q < 16 * KC * 16; q += 64 * kNarrowWaves) {   // one float4 (4 columns) each
    const int k = q >> 4, n0 = (q & 15) << 2;
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (k < K && n0 < N) v = *reinterpret_cast<const f32x4*>(W + static_cast<int64_t>(k) * ld_w + n0);
    const float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + j;
      uint32_t pc[NP];
      split2<NP>(n < N ? e[j] : 0.f, 0.f, pc);      // (columns past N: padding of W's rows)
      unsigned char* dst = Ws + n * COL_B + ((((k >> 3) ^ (n % CPC))) << 4) + ((k & 7) << 1);
#pragma unroll
      for (int p = 0; p < NP; ++p)
        *reinterpret_cast<uint16_t*>(dst + p * PIECE_B) = static_cast<uint16_t>(pc[p] & 0xffffu);
    }
  }
  __syncthreads();

  const int r = lane & 31, half = lane >> 5;
  const int64_t tile0 = (static_cast<int64_t>(blockIdx.x) * kNarrowWaves + wave) * tiles_per_wave;

  struct AG {
    f32x4 v[kGroup][2];
  };
  // the 8 k of this lane's row for the k chunks [g * kGroup, +kGroup) of the tile at row0;
  // rows past M re-read the last row (their results are not stored), k past K reads zeros
  auto load_group = [&](int64_t row0, int g, AG& a) {
    const int64_t row = row0 + r < M ? row0 + r : M - 1;
    const float* src = A + row * ld_a + 8 * half;
#pragma unroll
    for (int i = 0; i < kGroup; ++i) {
      const int k8 = 16 * (g * kGroup + i) + 8 * half;
      f32x4 lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
      if (k8 < K) {                                   // K % 8 == 0: whole groups of 8
        lo = *reinterpret_cast<const f32x4*>(src + 16 * (g * kGroup + i));
        hi = *reinterpret_cast<const f32x4*>(src + 16 * (g * kGroup + i) + 4);
      }
      a.v[i][0] = lo;
      a.v[i][1] = hi;
    }
  };

  constexpr int NG = KC / kGroup;
  static_assert(KC % kGroup == 0, "k chunks come in groups");
  AG cur = {}, nxt = {};
  if (tile0 * 32 < M) load_group(tile0 * 32, 0, cur);
  for (int it = 0; it < tiles_per_wave; ++it) {
    const int64_t row0 = (tile0 + it) * 32;
    if (row0 >= M) break;
    f32x16 acc[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[j][q] = 0.f;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      // the following group: of this tile, or the first of the next
      if (g + 1 < NG) load_group(row0, g + 1, nxt);
      else if (it + 1 < tiles_per_wave && row0 + 32 < M) load_group(row0 + 32, 0, nxt);
#pragma unroll
      for (int i = 0; i < kGroup; ++i) {
        const int kc = g * kGroup + i;
        uint32_t p0[NP], p1[NP], p2[NP], p3[NP];
        split2<NP>(cur.v[i][0].x, cur.v[i][0].y, p0);
        split2<NP>(cur.v[i][0].z, cur.v[i][0].w, p1);
        split2<NP>(cur.v[i][1].x, cur.v[i][1].y, p2);
        split2<NP>(cur.v[i][1].z, cur.v[i][1].w, p3);
        bf16x8 a[NP];
#pragma unroll
        for (int p = 0; p < NP; ++p) a[p] = __builtin_bit_cast(bf16x8, u32x4{p0[p], p1[p], p2[p], p3[p]});
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          if (32 * j >= N) continue;                  // uniform: the second column tile may be empty
          const int n = 32 * j + r;
          const unsigned char* col = Ws + n * COL_B + (((2 * kc + half) ^ (n % CPC)) << 4);
          bf16x8 b[NP];
#pragma unroll
          for (int p = 0; p < NP; ++p) b[p] = *reinterpret_cast<const bf16x8*>(col + p * PIECE_B);
#pragma unroll
          for (int q = 0; q < n_products<NP>(); ++q)
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[product_a<NP>(q)], b[product_b<NP>(q)],
                                                             acc[j], 0, 0, 0);
        }
      }
      cur = nxt;
    }
    // rows leave in the accumulator's layout: register q of a lane is row acc_row(q, lane),
    // column 32 j + lane % 32, i.e. 128 contiguous bytes per half-wavefront and register
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int c = 32 * j + r;
      if (c >= N) continue;
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int64_t row = row0 + acc_row(q, lane);
        if (row < M) {
          const float x = acc[j][q];
          out[row * ld_out + c] = RELU ? fmaxf(x, 0.f) : x;
        }
      }
    }
  }
}

}  // namespace

namespace sat {

// Whether launch_dense_narrow serves the shape (fp32 only).
bool dense_narrow_serves(int32_t K, int32_t N) { return K > 0 && K <= 256 && (K % 8) == 0 && N > 0 && N <= 64; }

// out [M, N] fp32 = act(A [M, K] W [K, N]); ld in elements; rows 16-byte aligned.
sat_status launch_dense_narrow(const void* A, int64_t ld_a, int64_t M, int32_t K, const void* W,
                               int64_t ld_w, int32_t N, bool relu, void* out, int64_t ld_out,
                               hipStream_t st) {
  if (M == 0 || N == 0) return SAT_OK;
  // tiles per wavefront: enough to spread the staging of W (its cost is that of about four
  // row tiles), few enough that the last workgroups do not leave the chip idle
  int64_t tpw = M / (32 * kNarrowWaves * 1024);
  if (tpw < 2) tpw = 2;
  if (tpw > 16) tpw = 16;
  const int64_t gx = (M + 32 * kNarrowWaves * tpw - 1) / (32 * kNarrowWaves * tpw);
  if (gx > INT32_MAX) return SAT_EUNSUPPORTED;
  const dim3 grid(static_cast<unsigned>(gx)), block(64 * kNarrowWaves);
  const float* a = static_cast<const float*>(A);
  const float* w = static_cast<const float*>(W);
  float* o = static_cast<float*>(out);
  const int itpw = static_cast<int>(tpw);
#define SAT_NARROW(KC)                                                                          \
  do {                                                                                          \
    if (relu) dense_narrow_kernel<KC, true><<<grid, block, 0, st>>>(a, ld_a, M, K, w, ld_w, N, o, ld_out, itpw); \
    else dense_narrow_kernel<KC, false><<<grid, block, 0, st>>>(a, ld_a, M, K, w, ld_w, N, o, ld_out, itpw);     \
  } while (0)
  if (K <= 64) SAT_NARROW(4);
  else if (K <= 128) SAT_NARROW(8);
  else SAT_NARROW(16);
#undef SAT_NARROW
  return sat::check_launch();
}

}  // namespace sat

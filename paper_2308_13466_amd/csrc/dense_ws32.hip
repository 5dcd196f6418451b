// Feature transform for fp32 storage with the weights held still (appendix:
// Z = (P H) W, H' = sigma(Z), and the gradient to the aggregate (D o [H' > 0]) W^T):
//   out[m, 0:N) = act(A'[m, 0:K) B),   B = W (K x N, row-major) or W^T (W is N x K),
//   A' = A, or A with the elements whose mask value is not > 0 set to zero,
// for M in the hundreds of thousands and more, K <= 256. Per row of A the exact fp32
// product costs six bf16 MFMAs per 16 k and 32 columns (mx_tile.h) and 2 (K + N) * 4 bytes
// of memory traffic: at 256 -> 256 both bounds are within 20 % of each other (0.096 ms of
// products, 0.079 ms of HBM time for 306k rows), so neither may wait for the other, and the
// tile GEMM's staging of both operands per k step leaves the matrix pipe idle two thirds of
// the time. Here:
//   * a workgroup has 8 wavefronts; wavefront w owns output columns [32 w, 32 w + 32) of a
//     group of 256 and keeps ITS slice of B for all of K in registers, split into the three
//     bf16 pieces and in MFMA operand order (192 registers for K = 256: two wavefronts per
//     SIMD, one workgroup per compute unit);
//   * rows stream through in tiles of 32. A wavefront reads eight 128-byte segments per
//     load instruction (8 rows x 32 k), splits them and writes the pieces to LDS in the
//     swizzled operand layout (a wavefront's write covers 512 contiguous bytes per piece: no
//     bank conflicts). Two LDS buffers, ONE barrier per tile;
//   * the registers that receive a tile's loads are emptied into LDS during the first
//     products of the tile BEFORE (where that buffer is free), and the loads of the tile
//     after are issued at once: every load has a whole tile's products to arrive, which is
//     what HBM's latency under load asks for (32 KB in flight per compute unit);
//   * products leave straight from the accumulators: a store instruction writes two rows of
//     32 columns, 128 contiguous bytes each.
#include "mx_tile.h"
#include "sat_internal.h"

namespace {

using namespace sat::mx;

// base + off bytes, base a pointer every lane holds alike (scalar registers), off a 32-bit
// lane offset: such an access needs one vector register for its address.
__device__ __forceinline__ const float* at_bytes(const float* base, uint32_t off) {
  return reinterpret_cast<const float*>(reinterpret_cast<const unsigned char*>(base) + off);
}
__device__ __forceinline__ float* at_bytes(float* base, uint32_t off) {
  return reinterpret_cast<float*>(reinterpret_cast<unsigned char*>(base) + off);
}

// KC = number of 16-wide k chunks the operands are padded to (K <= 16 KC, K % 4 == 0);
// KFULL: K == 16 KC (no k needs clamping or zeroing); NFULL: N % 256 == 0 (every lane has a
// column: the stores then sit in the tile loop's one basic block, and the waits for the next
// tile's loads, issued before them, need not wait for the stores as well)
template <int KC, bool KFULL, bool NFULL, bool TRANSB, bool MASK, bool RELU>
__global__ __launch_bounds__(512, 2) void dense_ws32_kernel(
    const float* __restrict__ A, int64_t ld_a, const float* __restrict__ Mk, int64_t ld_m,
    int64_t M, int K, const float* __restrict__ W, int64_t ld_w, int N, float* __restrict__ out,
    int64_t ld_out, int tiles_per_block) {
  constexpr int NP = 3;
  constexpr int NT32 = KC / 2;                            // 32-wide staging tiles per row tile
  constexpr int STAGE = NT32 * tile_bytes<32, NP>();      // bytes of one staged A tile
  constexpr int NLD = (NT32 * 4) / 8;                     // 8-row x 32-k blocks per wavefront
  static_assert(NT32 * 4 % 8 == 0 && NLD >= 1, "blocks divide among the 8 wavefronts");
  // With a mask and K = 256 the registers do not hold a whole tile of loads (and masks) beside
  // the weights: the blocks then travel in two halves, each with half a tile's products to arrive.
  constexpr int NPH = KC == 16 ? 2 : 1;
  constexpr int LP = NLD / NPH;                           // blocks in flight per wavefront
  __shared__ __attribute__((aligned(16))) unsigned char As[2 * STAGE];

  const int t = threadIdx.x;
  const int lane0 = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int64_t row_lo = static_cast<int64_t>(blockIdx.x) * 32 * tiles_per_block;

  // ---- this wavefront's slice of B as MFMA operands: lane holds k = 16 kc + 8 (lane / 32)
  // .. + 7 of column `col`, split into three pieces (zeros past K and past N; the loads
  // themselves go to a valid element whatever k and the column)
  bf16x8 bw[KC][NP];
  {
  const int col = blockIdx.y * 256 + 32 * wave + (lane0 & 31);
  const bool col_ok = col < N;
  const int colc = col_ok ? col : N - 1;
#pragma unroll
  for (int kc = 0; kc < KC; ++kc) {
    const int k0 = 16 * kc + 8 * (lane0 >> 5);
    float e[8];
    // (an element that must read as zero is loaded all the same and its bits are cleared: a
    // select would let the compiler put each load under its own branch, with its own wait)
    auto bits_if = [](float x, bool ok) {
      return __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, x) & (ok ? 0xffffffffu : 0u));
    };
    if constexpr (TRANSB) {      // 8 consecutive k of a column of B are contiguous in W
      const int ka = k0 < K ? k0 : K - 4, kb = k0 + 4 < K ? k0 + 4 : K - 4;
      const f32x4 a = *reinterpret_cast<const f32x4*>(W + static_cast<int64_t>(colc) * ld_w + ka);
      const f32x4 b = *reinterpret_cast<const f32x4*>(W + static_cast<int64_t>(colc) * ld_w + kb);
      const bool oa = col_ok && k0 < K, ob = col_ok && k0 + 4 < K;
      e[0] = bits_if(a.x, oa); e[1] = bits_if(a.y, oa); e[2] = bits_if(a.z, oa); e[3] = bits_if(a.w, oa);
      e[4] = bits_if(b.x, ob); e[5] = bits_if(b.y, ob); e[6] = bits_if(b.z, ob); e[7] = bits_if(b.w, ob);
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int k = k0 + j < K ? k0 + j : K - 1;
        e[j] = bits_if(W[static_cast<int64_t>(k) * ld_w + colc], col_ok && k0 + j < K);
      }
    }
    uint32_t q[4][NP];
#pragma unroll
    for (int h = 0; h < 4; ++h) split2<NP>(e[2 * h], e[2 * h + 1], q[h]);
#pragma unroll
    for (int p = 0; p < NP; ++p)
      bw[kc][p] = __builtin_bit_cast(bf16x8, u32x4{q[0][p], q[1][p], q[2][p], q[3][p]});
  }
  }

  // Everything below that depends on the lane is derived from here on: computed before the
  // weights came in, those values would have to survive the moment when all of the weights and
  // their loads are live, and the ones that did not fit would be reloaded from scratch memory
  // in every tile (a scratch reload waits for every global load in flight).
  int lane = lane0;
  asm volatile("" : "+v"(lane));
  const int col = blockIdx.y * 256 + 32 * wave + (lane & 31);
  const bool col_ok = col < N;

  // ---- A tile: block c = wave + 8 i is staging tile c % NT32 (k = 32 (c % NT32) ..), rows
  // 8 (c / NT32) .. + 7; lane: row lane / 8 of the block, 4 k at 4 (lane % 8). Addresses are a
  // per-wavefront base (scalar registers) plus ONE 32-bit lane offset, which keeps them out of
  // the vector registers the weights need. M is a multiple of 32 (the launcher sees to it), so
  // a tile is either whole or past the end; a request past the end reads the matrix's last tile
  // instead (staged, never multiplied). k past K reads the last four k of the row and is zeroed
  // when it is staged.
  struct Regs {
    f32x4 v[LP], h[LP];
  };
  const int l_row = lane >> 3, l_k = (lane & 7) << 2;
  const uint32_t off_a = (static_cast<uint32_t>(l_row) * static_cast<uint32_t>(ld_a) + static_cast<uint32_t>(l_k)) << 2;
  const uint32_t off_m = (static_cast<uint32_t>(l_row) * static_cast<uint32_t>(ld_m) + static_cast<uint32_t>(l_k)) << 2;
  auto load_one = [&](int64_t row0, int blk, int i, Regs& r) {   // block blk into register set i
    const int c = wave + 8 * blk;
    const int64_t rb = (row0 < M ? row0 : M - 32) + 8 * (c / NT32);     // uniform
    if constexpr (KFULL) {
      r.v[i] = *reinterpret_cast<const f32x4*>(at_bytes(A + rb * ld_a + 32 * (c % NT32), off_a));
      if constexpr (MASK) r.h[i] = *reinterpret_cast<const f32x4*>(at_bytes(Mk + rb * ld_m + 32 * (c % NT32), off_m));
    } else {
      int k = 32 * (c % NT32) + l_k;
      k = k < K ? k : K - 4;                                            // K % 4 == 0: whole groups of 4
      const uint32_t oa = (static_cast<uint32_t>(l_row) * static_cast<uint32_t>(ld_a) + static_cast<uint32_t>(k)) << 2;
      r.v[i] = *reinterpret_cast<const f32x4*>(at_bytes(A + rb * ld_a, oa));
      if constexpr (MASK) {
        const uint32_t om = (static_cast<uint32_t>(l_row) * static_cast<uint32_t>(ld_m) + static_cast<uint32_t>(k)) << 2;
        r.h[i] = *reinterpret_cast<const f32x4*>(at_bytes(Mk + rb * ld_m, om));
      }
    }
  };
  auto store_one = [&](const Regs& r, int i, int blk, int stage) {
    const int c = wave + 8 * blk;
    f32x4 f = r.v[i];
    if constexpr (MASK) {
      const f32x4 h = r.h[i];
      f.x = h.x > 0.f ? f.x : 0.f;
      f.y = h.y > 0.f ? f.y : 0.f;
      f.z = h.z > 0.f ? f.z : 0.f;
      f.w = h.w > 0.f ? f.w : 0.f;
    }
    if constexpr (!KFULL)
      if (32 * (c % NT32) + l_k >= K) f = f32x4{0.f, 0.f, 0.f, 0.f};
    uint32_t lo[NP], hi[NP];
    split2<NP>(f.x, f.y, lo);
    split2<NP>(f.z, f.w, hi);
    unsigned char* s = As + stage * STAGE + (c % NT32) * tile_bytes<32, NP>() +
                       swz(8 * (c / NT32) + l_row, l_k >> 3) + (((l_k >> 2) & 1) << 3);
#pragma unroll
    for (int p = 0; p < NP; ++p) *reinterpret_cast<u32x2*>(s + p * piece_bytes<32>()) = u32x2{lo[p], hi[p]};
  };

  Regs ra;
#pragma unroll
  for (int i = 0; i < LP; ++i) load_one(row_lo, i, i, ra);
  // Slot j (0 <= j < NLD) of tile `it`: block j of tile it + 1 leaves its registers for the
  // buffer that tile will be read from, and the registers take the next request: the block LP
  // further on, which lies in tile it + 1 or it + 2 (past the end of the matrix that is valid
  // memory again: staged, never multiplied).
  auto slot = [&](int it, int j) {
    const int64_t row1 = row_lo + 32 * static_cast<int64_t>(it + 1);
    store_one(ra, j % LP, j, (it + 1) & 1);
    if (j + LP < NLD) load_one(row1, j + LP, j % LP, ra);
    else load_one(row1 + 32, j + LP - NLD, j % LP, ra);
    // (the request stays HERE: left to itself the scheduler sinks it to the end of the tile to
    // shorten the registers' live range, and the load then has no time to arrive)
    __builtin_amdgcn_sched_barrier(0);
  };

  // tile 0 into buffer 0, the first blocks of tile 1 requested
#pragma unroll
  for (int j = 0; j < NLD; ++j) slot(-1, j);
  __syncthreads();

  for (int it = 0; it < tiles_per_block; ++it) {
    const int64_t row0 = row_lo + 32 * it;
    if (row0 >= M) break;                        // uniform over the workgroup
    const int stage = it & 1;
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    const unsigned char* S = As + stage * STAGE;
    auto frag = [&](int kc, int p) {
      return read_operand(S + (kc >> 1) * tile_bytes<32, NP>() + p * piece_bytes<32>(), 0, kc & 1, lane);
    };
    // The six products of a k chunk in the order a3 b1, a2 b2, a2 b1, a1 b3, a1 b2, a1 b1 (small
    // terms first); a piece of A is read for the NEXT chunk as soon as its last product of this
    // chunk has been issued, so that no second set of fragment registers is needed and every
    // LDS read still has three to five products (of this wavefront alone) to arrive. The
    // scheduling barriers keep that order: left alone, the compiler reads all three pieces just
    // before their first use and the matrix pipe waits for LDS sixteen times per tile.
    bf16x8 a0 = frag(0, 0), a1 = frag(0, 1), a2 = frag(0, 2);
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, bw[kc][0], acc, 0, 0, 0);
      if (kc + 1 < KC) a2 = frag(kc + 1, 2);
      __builtin_amdgcn_sched_barrier(0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, bw[kc][1], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, bw[kc][0], acc, 0, 0, 0);
      if (kc + 1 < KC) a1 = frag(kc + 1, 1);
      __builtin_amdgcn_sched_barrier(0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, bw[kc][2], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, bw[kc][1], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, bw[kc][0], acc, 0, 0, 0);
      if (kc + 1 < KC) a0 = frag(kc + 1, 0);
      __builtin_amdgcn_sched_barrier(0);
      // between the products: a slot's block of the NEXT tile goes to the other buffer, whose
      // last readers passed the barrier that ended the previous tile. (Slots at the start of
      // their part of the tile: in its middle they were measured 8 % slower.)
      if (kc % (KC / NPH) < LP) slot(it, (kc / (KC / NPH)) * LP + kc % (KC / NPH));
    }
    // register r of a lane is row 8 (r / 4) + 4 (lane / 32) + r % 4, column lane % 32: a scalar
    // row base plus one 32-bit lane offset
    if (NFULL || col_ok) {
      const uint32_t off_y = (static_cast<uint32_t>(4 * (lane >> 5)) * static_cast<uint32_t>(ld_out) +
                              static_cast<uint32_t>(col)) << 2;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float x = acc[r];
        float* yr = out + (row0 + 8 * (r >> 2) + (r & 3)) * ld_out;
        *at_bytes(yr, off_y) = RELU ? fmaxf(x, 0.f) : x;
      }
    }
    __syncthreads();
  }
}

}  // namespace

namespace sat {

// Whether launch_dense_ws32 serves the shape: contraction length K, M rows.
bool dense_ws32_serves(int32_t K, int64_t M) { return K >= 4 && K <= 256 && (K % 4) == 0 && M >= 65536; }

// out [M, N] fp32 = act(A' B): A [M, K] fp32 with A' = A o [Mk > 0] if Mk != nullptr, B = W
// (transb false: W is [K, ld_w]) or W^T (transb true: W is [N, ld_w]); relu on the result if
// asked. ld in elements, rows 16-byte aligned. dense_ws32_serves(K, M) must hold and M must be
// a multiple of 32 (the caller gives the last M % 32 rows to another kernel).
sat_status launch_dense_ws32(const void* A, int64_t ld_a, const void* Mk, int64_t ld_m, int64_t M,
                             int32_t K, const void* W, int64_t ld_w, bool transb, int32_t N,
                             bool relu, void* out, int64_t ld_out, hipStream_t st) {
  if (M == 0 || N == 0) return SAT_OK;
  if (M % 32 != 0) return SAT_EINVAL;
  // one workgroup per compute unit and column group, each with an equal share of the tiles
  // (bringing the weights into registers costs about as much as one tile)
  const int64_t tiles = (M + 31) / 32;
  int64_t tpb = (tiles + 255) / 256;
  if (tpb > (1 << 20)) return SAT_EUNSUPPORTED;
  const int64_t gx = (tiles + tpb - 1) / tpb;
  const dim3 grid(static_cast<unsigned>(gx), static_cast<unsigned>((N + 255) / 256));
  const float* a = static_cast<const float*>(A);
  const float* m = static_cast<const float*>(Mk);
  const float* w = static_cast<const float*>(W);
  float* o = static_cast<float*>(out);
  const int itpb = static_cast<int>(tpb);
#define SAT_WS(KC, TB, MK, RL)                                                                       \
  do {                                                                                              \
    if (K == 16 * KC && N % 256 == 0)                                                               \
      dense_ws32_kernel<KC, true, true, TB, MK, RL><<<grid, dim3(512), 0, st>>>(                    \
          a, ld_a, m, ld_m, M, K, w, ld_w, N, o, ld_out, itpb);                                     \
    else if (K == 16 * KC)                                                                          \
      dense_ws32_kernel<KC, true, false, TB, MK, RL><<<grid, dim3(512), 0, st>>>(                   \
          a, ld_a, m, ld_m, M, K, w, ld_w, N, o, ld_out, itpb);                                     \
    else if (N % 256 == 0)                                                                          \
      dense_ws32_kernel<KC, false, true, TB, MK, RL><<<grid, dim3(512), 0, st>>>(                   \
          a, ld_a, m, ld_m, M, K, w, ld_w, N, o, ld_out, itpb);                                     \
    else                                                                                            \
      dense_ws32_kernel<KC, false, false, TB, MK, RL><<<grid, dim3(512), 0, st>>>(                  \
          a, ld_a, m, ld_m, M, K, w, ld_w, N, o, ld_out, itpb);                                     \
  } while (0)
#define SAT_WS_K(TB, MK, RL)                  \
  do {                                        \
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

// dW = A^T B reduced over the rows (nodes): A [n, d_a], B [n, d_b] row-major,
// C [d_a, d_b] fp32. The weight-gradient product of the feature transform
// (appendix: G_W = (P H)^T D with D = G o sigma'(Z)) and, with other operands,
// of the predictor's training.
//
// The contraction index is the ROW index of both operands, so neither operand is
// laid out the way the MFMA wants it (8 consecutive k per lane). Design:
//   * a workgroup (2 x 2 wavefronts) owns a (64 MT) x (64 NT) output tile - up to the
//     whole 256 x 256 matrix, 256 accumulator registers per lane - and a contiguous
//     range of nodes; the accumulators stay in registers for the whole range, so an
//     operand element is read from memory once per output tile and the LDS traffic
//     per product is low (MT + NT operand fragments for MT * NT products);
//   * per step it takes KS nodes: their rows are read with 16-byte accesses as they
//     lie in memory (fully coalesced), split into bf16 pieces (fp32 data: three
//     pieces, exact; bf16 data: as it is) and written to LDS in the SAME node-major
//     order, 8-byte stores, no conflicts;
//   * the MFMA fragments are then read TRANSPOSED out of LDS. A lane needs 8
//     consecutive nodes of one column, i.e. 8 reads. To make those reads wide, the
//     T tiles of a wavefront interleave their columns (MFMA row r of tile i is column
//     T r + i of the wavefront's range): one 2T-byte read per node then serves all T
//     tiles, 8 reads per operand piece instead of 8 T (rows padded so that the two
//     half-wavefronts hit different banks). The output tile is stored with the same
//     column permutation undone;
//   * global loads of the next step are in flight (registers) while the current step
//     multiplies; LDS is double-buffered, one barrier per step;
//   * the relu mask (B used only where mask > 0) is applied in registers.
// Each workgroup writes its partial tile; the caller sums the partial tiles in a
// fixed order (no float atomics).
#ifndef SAT_DW_KERNEL_H_
#define SAT_DW_KERNEL_H_

#include <type_traits>

#include "mx_tile.h"

namespace sat {
namespace dw {

using namespace sat::mx;

template <int ES>
struct Cfg {
  static constexpr int NP = ES == 4 ? 3 : 1;   // bf16 pieces per element
  static constexpr int KS = ES == 4 ? 16 : 32; // nodes per step
  static constexpr int EPV = 16 / ES;          // elements per 16-byte access
};

template <int ES, int T>   // T = MT or NT: LDS bytes of one operand stage
constexpr int stage_bytes() {
  return Cfg<ES>::NP * Cfg<ES>::KS * (64 * T * 2 + 8);
}
template <int ES, int MT, int NT>
constexpr int smem_bytes() {
  return 2 * (stage_bytes<ES, MT>() + stage_bytes<ES, NT>());
}

// positive test on a bf16 bit pattern
__device__ __forceinline__ bool pos16(uint32_t h) { return (h & 0x8000u) == 0 && (h & 0x7fffu) != 0; }

template <int ES, int MT, int NT, bool MASK>
__global__ __launch_bounds__(256) void dw_kernel(const void* __restrict__ A, int64_t ld_a, int d_a,
                                                 const void* __restrict__ B, int64_t ld_b, int d_b,
                                                 const void* __restrict__ M, int64_t ld_m, int64_t n,
                                                 int64_t n_per_block, float* __restrict__ part,
                                                 int64_t ld_part, int64_t part_stride) {
  typedef Cfg<ES> C;
  constexpr int NP = C::NP, KS = C::KS, EPV = C::EPV;
  constexpr int BMX = 64 * MT, BNX = 64 * NT;
  constexpr int ROWA = BMX * 2 + 8, ROWB = BNX * 2 + 8;   // bytes per node row of a piece
  constexpr int VA = KS * (BMX / EPV) / 256;              // 16-byte accesses per thread per step
  constexpr int VB = KS * (BNX / EPV) / 256;
  static_assert(VA >= 1 && VB >= 1, "tile too small for 256 threads");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* const sA = smem;                                   // [2][NP][KS][ROWA]
  unsigned char* const sB = smem + 2 * stage_bytes<ES, MT>();       // [2][NP][KS][ROWB]

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int m_base = blockIdx.x * BMX, n_base = blockIdx.y * BNX;
  const int64_t k_lo = static_cast<int64_t>(blockIdx.z) * n_per_block;
  const int64_t k_hi = k_lo + n_per_block < n ? k_lo + n_per_block : n;

  // this thread's accesses: row r = (t + 256 i) / VPR, vector column cv = (t + 256 i) % VPR
  constexpr int VPRA = BMX / EPV, VPRB = BNX / EPV;
  u32x4 ra[VA], rb[VB], rmk[MASK ? VB : 1];

  // Issue the global loads of the KS nodes from k0 on. Nothing here looks at the loaded
  // values (the mask and the padding columns are dealt with in store()), so the loads
  // stay in flight while the previous step multiplies.
  auto load = [&](int64_t k0) {
#pragma unroll
    for (int i = 0; i < VA; ++i) {
      const int q = t + 256 * i;
      const int64_t k = k0 + q / VPRA;
      const int c = m_base + (q % VPRA) * EPV;
      u32x4 v = {0u, 0u, 0u, 0u};
      if (k < k_hi && c < d_a)
        v = *reinterpret_cast<const u32x4*>(static_cast<const unsigned char*>(A) + (k * ld_a + c) * ES);
      ra[i] = v;
    }
#pragma unroll
    for (int i = 0; i < VB; ++i) {
      const int q = t + 256 * i;
      const int64_t k = k0 + q / VPRB;
      const int c = n_base + (q % VPRB) * EPV;
      u32x4 v = {0u, 0u, 0u, 0u}, hm = {0u, 0u, 0u, 0u};
      if (k < k_hi && c < d_b) {
        v = *reinterpret_cast<const u32x4*>(static_cast<const unsigned char*>(B) + (k * ld_b + c) * ES);
        if constexpr (MASK)
          hm = *reinterpret_cast<const u32x4*>(static_cast<const unsigned char*>(M) + (k * ld_m + c) * ES);
      }
      rb[i] = v;
      if constexpr (MASK) rmk[i] = hm;
    }
  };

  // elements at or beyond column limit d lie in the row's padding: zero them
  auto clip = [&](u32x4 v, int c, int d) {
    if (c + EPV > d) {
      uint32_t w[4] = {v.x, v.y, v.z, v.w};
      if constexpr (ES == 4) {
#pragma unroll
        for (int e = 1; e < 4; ++e)
          if (c + e >= d) w[e] = 0u;
      } else {
        const int left = d - c;   // valid 2-byte elements (<= 0: none)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (2 * e >= left) w[e] = 0u;
          else if (2 * e + 1 >= left) w[e] &= 0xffffu;
        }
      }
      v = u32x4{w[0], w[1], w[2], w[3]};
    }
    return v;
  };
  auto apply_mask = [&](u32x4 v, u32x4 hm) {
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
    const uint32_t h[4] = {hm.x, hm.y, hm.z, hm.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if constexpr (ES == 4) {
        if (!(__builtin_bit_cast(float, h[e]) > 0.f)) w[e] = 0u;
      } else {
        if (!pos16(h[e] & 0xffffu)) w[e] &= 0xffff0000u;
        if (!pos16(h[e] >> 16)) w[e] &= 0x0000ffffu;
      }
    }
    return u32x4{w[0], w[1], w[2], w[3]};
  };

  // registers -> LDS stage `st`, node-major, split into pieces
  auto store_one = [&](const u32x4 v, unsigned char* base, int row_bytes, int r, int c_local) {
    unsigned char* p0 = base + r * row_bytes + c_local * 2;
    if constexpr (ES == 4) {
      const f32x4 f = __builtin_bit_cast(f32x4, v);
      uint32_t lo[NP], hi[NP];
      split2<NP>(f.x, f.y, lo);
      split2<NP>(f.z, f.w, hi);
#pragma unroll
      for (int p = 0; p < NP; ++p)
        *reinterpret_cast<u32x2*>(p0 + p * KS * row_bytes) = u32x2{lo[p], hi[p]};
    } else {
      *reinterpret_cast<u32x2*>(p0) = u32x2{v.x, v.y};
      *reinterpret_cast<u32x2*>(p0 + 8) = u32x2{v.z, v.w};
    }
  };
  auto store = [&](int st) {
    unsigned char* a = sA + st * stage_bytes<ES, MT>();
    unsigned char* b = sB + st * stage_bytes<ES, NT>();
#pragma unroll
    for (int i = 0; i < VA; ++i) {
      const int q = t + 256 * i;
      const int cl = (q % VPRA) * EPV;
      store_one(clip(ra[i], m_base + cl, d_a), a, ROWA, q / VPRA, cl);
    }
#pragma unroll
    for (int i = 0; i < VB; ++i) {
      const int q = t + 256 * i;
      const int cl = (q % VPRB) * EPV;
      u32x4 v = rb[i];
      if constexpr (MASK) v = apply_mask(v, rmk[i]);
      store_one(clip(v, n_base + cl, d_b), b, ROWB, q / VPRB, cl);
    }
  };

  // MFMA fragments of all T tiles of a wavefront for one piece and one kc. Tile i's row
  // (lane % 32) is column  col0 + T (lane % 32) + i  of the staged slab; nodes
  // 16 kc + 8 (lane / 32) .. + 7. One 2T-byte read per node covers the T tiles.
  auto frags = [&](auto t_tag, const unsigned char* piece, int row_bytes, int col0, int kc,
                   auto& out, int pidx) {
    constexpr int T = decltype(t_tag)::value;
    const unsigned char* p = piece + (16 * kc + 8 * (lane >> 5)) * row_bytes + (col0 + T * (lane & 31)) * 2;
    uint32_t raw[8][(T + 1) / 2];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      if constexpr (T == 4) {
        const u32x2 v = *reinterpret_cast<const u32x2*>(p + e * row_bytes);
        raw[e][0] = v.x;
        raw[e][1] = v.y;
      } else if constexpr (T == 2) {
        raw[e][0] = *reinterpret_cast<const uint32_t*>(p + e * row_bytes);
      } else {   // one tile per wavefront (an operand of at most 64 columns): 2 bytes per node
        raw[e][0] = *reinterpret_cast<const uint16_t*>(p + e * row_bytes);
      }
    }
#pragma unroll
    for (int i = 0; i < T; ++i) {
      uint32_t w[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t a0 = raw[2 * e][i >> 1], a1 = raw[2 * e + 1][i >> 1];
        w[e] = (i & 1) ? ((a0 >> 16) | (a1 & 0xffff0000u)) : ((a0 & 0xffffu) | (a1 << 16));
      }
      out[i][pidx] = __builtin_bit_cast(bf16x8, u32x4{w[0], w[1], w[2], w[3]});
    }
  };

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int64_t steps = k_hi > k_lo ? (k_hi - k_lo + KS - 1) / KS : 0;
  if (steps > 0) {
    load(k_lo);
    store(0);
  }
  __syncthreads();
  for (int64_t s = 0; s < steps; ++s) {
    const int st = static_cast<int>(s & 1);
    if (s + 1 < steps) load(k_lo + (s + 1) * KS);
    const unsigned char* a = sA + st * stage_bytes<ES, MT>();
    const unsigned char* b = sB + st * stage_bytes<ES, NT>();
#pragma unroll
    for (int kc = 0; kc < KS / 16; ++kc) {
      bf16x8 fa[MT][NP], fb[NT][NP];
#pragma unroll
      for (int p = 0; p < NP; ++p) {
        frags(std::integral_constant<int, MT>{}, a + p * KS * ROWA, ROWA, 32 * MT * wm, kc, fa, p);
        frags(std::integral_constant<int, NT>{}, b + p * KS * ROWB, ROWB, 32 * NT * wn, kc, fb, p);
      }
#pragma unroll
      for (int q = 0; q < n_products<NP>(); ++q)
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
          for (int j = 0; j < NT; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i][product_a<NP>(q)],
                                                                fb[j][product_b<NP>(q)], acc[i][j],
                                                                0, 0, 0);
    }
    if (s + 1 < steps) store(st ^ 1);
    __syncthreads();
  }

  // partial tile of this workgroup
  float* out = part + static_cast<int64_t>(blockIdx.z) * part_stride;
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int col = n_base + 32 * NT * wn + NT * (lane & 31) + j;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m_base + 32 * MT * wm + MT * acc_row(r, lane) + i;
        if (row < d_a && col < d_b) out[static_cast<int64_t>(row) * ld_part + col] = acc[i][j][r];
      }
    }
}

}  // namespace dw
}  // namespace sat
#endif  // SAT_DW_KERNEL_H_

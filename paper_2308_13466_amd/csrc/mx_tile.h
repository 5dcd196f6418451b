// Tile GEMM on the bf16 MFMA pipe of gfx950 (v_mfma_f32_32x32x16_bf16), used
// for bf16 data directly and for fp32 data through an exact three-way split.
//
// Why: the fp32 MFMA pipe peaks at 157 TFLOP/s, the bf16 pipe at 2.5 PFLOP/s
// (16x). An fp32 value x is split into three bf16 pieces x = x1 + x2 + x3
// (x1 = bf16(x), x2 = bf16(x - x1), x3 = bf16(x - x1 - x2); each subtraction is
// exact in fp32 and the three 8-bit significands cover fp32's 24 bits). A
// product a*b is then the sum of nine piece products, each EXACT in the
// MFMA's fp32 accumulator (8 x 8 bit significands). The six products with
// i + j <= 4 are kept; the dropped ones are below 2^-24 |a b|, i.e. below one
// fp32 rounding of the product itself. Six bf16 MFMAs cost 6/16 of one fp32
// MFMA's time for the same k-extent, and one instruction covers 16 k instead
// of 2, so the accumulator is also rounded less often than on the fp32 pipe.
//
// Layout: a workgroup of 256 threads (4 wavefronts, 2 x 2) owns a 128 x 128
// tile, K in steps of 32. Operand tiles are staged in LDS per piece as
// [mn][k] bf16 with k contiguous, 64 bytes per row and no padding; the four
// 16-byte chunks of a row are stored at chunk ^ f(row), f = (bit1 ^ bit3) | bit2 << 1
// of the row number. A lane's MFMA operand (8 consecutive k of one row) is one
// 16-byte LDS read; LDS has 64 banks of 4 bytes and serves such a read 16 lanes
// at a time, so 16 consecutive rows of one chunk must land on 16 different
// 16-byte bank groups: the row's bit 0 picks the half of the 128-byte line, f
// the chunk, and bits 1..3 all enter f, which makes them distinct (measured:
// no bank conflicts in these reads; with f = (row >> 1) & 3 rows r and r + 8
// collided and a third of the LDS cycles were conflicts). Tile writes (whole
// rows) are conflict free under either. fp32 operands are split while
// they are written to LDS; global loads for step i+1 are issued before the
// MFMAs of step i.
#ifndef SAT_MX_TILE_H_
#define SAT_MX_TILE_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sat {
namespace mx {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int BM = 128, BN = 128, BK = 32;
constexpr int ROW_B = BK * 2;  // bytes per staged row: 32 bf16, chunks swizzled (see swz)

// byte offset inside a staged piece of 16-byte chunk `chunk` (0..3) of row `row`
__device__ __forceinline__ int swz(int row, int chunk) {
  const int f = (((row >> 1) ^ (row >> 3)) & 1) | (((row >> 2) & 1) << 1);
  return row * ROW_B + ((chunk ^ f) << 4);
}

template <int MN>
constexpr int piece_bytes() { return MN * ROW_B; }
template <int MN, int NP>
constexpr int tile_bytes() { return NP * MN * ROW_B; }

enum class Layout { KContig, MNContig };

// Operand of fp32 or bf16 elements (the kernel's template parameter says which):
// element (mn, k) at p[mn * ld + k] (KContig) or p[k * ld + mn] (MNContig), ld in
// elements; mask (optional, same element type) has the same indexing with its
// own ld, and an element whose mask value is not > 0 reads as 0.
struct Operand {
  const void* p;
  int64_t ld;
  const void* mask;
  int64_t ld_mask;
};

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {  // RNE, a in the low half
  const f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ float low_as_f32(uint32_t p) { return __builtin_bit_cast(float, p << 16); }
__device__ __forceinline__ float high_as_f32(uint32_t p) {
  return __builtin_bit_cast(float, p & 0xffff0000u);
}

// out[p] = packed p-th pieces of (x0, x1)
template <int NP>
__device__ __forceinline__ void split2(float x0, float x1, uint32_t (&out)[NP]) {
  out[0] = pack_bf16(x0, x1);
  if constexpr (NP > 1) {
    x0 -= low_as_f32(out[0]);
    x1 -= high_as_f32(out[0]);
    out[1] = pack_bf16(x0, x1);
  }
  if constexpr (NP > 2) {
    x0 -= low_as_f32(out[1]);
    x1 -= high_as_f32(out[1]);
    out[2] = pack_bf16(x0, x1);
  }
}

// One thread's share (MN / 8 floats) of an MN x 32 fp32 operand tile.
//  KContig : v[i] = 4 consecutive k of row (t / 8 + 32 i), k = 4 (t % 8)
//  MNContig: v[2g], v[2g+1] = 8 consecutive k of column mn = t % MN,
//            k = 8 (t / MN + (256 / MN) g)            (needs MN >= 64)
// load_tile only ISSUES the loads: nothing looks at the loaded values until
// store_tile, so they stay in flight across the products of the previous step.
// The relu mask (h, raw values of the mask matrix) and the zeroing of elements
// past the end of K (kleft = valid elements from this thread's first k) are
// therefore applied in store_tile.
template <int MN>
struct TileRegs {
  f32x4 v[MN / 32];
  f32x4 h[MN / 32];
  int kleft;
};

// part: -1 = the whole share, 0 / 1 = its first / second half (the two halves together are the whole)
template <int MN, Layout L, bool MASK>
__device__ __forceinline__ void load_tile(const Operand& op, int64_t mn0, int64_t mn_lim,
                                          int64_t k0, int64_t k_lim, TileRegs<MN>& r, int t,
                                          int part = -1) {
  if constexpr (L == Layout::KContig) {
    const int64_t k = k0 + ((t & 7) << 2);
    const int64_t left = k_lim - k;
    r.kleft = left > 4 ? 4 : static_cast<int>(left);
#pragma unroll
    for (int i = 0; i < MN / 32; ++i) {
      if (part >= 0 && (2 * i) / (MN / 32) != part) continue;
      f32x4 v = {0.f, 0.f, 0.f, 0.f}, h = {0.f, 0.f, 0.f, 0.f};
      const int64_t mn = mn0 + (t >> 3) + 32 * i;
      if (mn < mn_lim && k < k_lim) {
        v = *reinterpret_cast<const f32x4*>(static_cast<const float*>(op.p) + mn * op.ld + k);
        if constexpr (MASK)
          h = *reinterpret_cast<const f32x4*>(static_cast<const float*>(op.mask) + mn * op.ld_mask + k);
      }
      r.v[i] = v;
      if constexpr (MASK) r.h[i] = h;
    }
  } else {
    static_assert(!MASK, "masked operands are row-major in k");
    static_assert(MN >= 64 && MN <= 256, "MNContig tiles are 64..256 wide");
    constexpr int KG = 256 / MN;  // k-groups of 8 covered by the thread index
    const int64_t mn = mn0 + (t % MN);
    const bool mn_ok = mn < mn_lim;
    r.kleft = 4;
#pragma unroll
    for (int g = 0; g < MN / 64; ++g) {
      if (part >= 0 && (2 * g) / (MN / 64) != part) continue;
      const int64_t k8 = k0 + 8 * ((t / MN) + KG * g);
      float e[8];
      if (mn_ok && k8 + 8 <= k_lim) {   // the usual case: one test for the eight loads
        const float* src = static_cast<const float*>(op.p) + k8 * op.ld + mn;
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = src[j * op.ld];
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          float x = 0.f;
          if (mn_ok && k8 + j < k_lim) x = static_cast<const float*>(op.p)[(k8 + j) * op.ld + mn];
          e[j] = x;
        }
      }
      r.v[2 * g] = f32x4{e[0], e[1], e[2], e[3]};
      r.v[2 * g + 1] = f32x4{e[4], e[5], e[6], e[7]};
    }
  }
}

// Apply mask and K tail, split the registers into NP bf16 pieces and write them to
// the staged tile at S (piece p at S + p * piece_bytes<MN>()).
template <int MN, Layout L, int NP, bool MASK>
__device__ __forceinline__ void store_tile(const TileRegs<MN>& r, unsigned char* S, int t) {
  if constexpr (L == Layout::KContig) {
#pragma unroll
    for (int i = 0; i < MN / 32; ++i) {
      f32x4 v = r.v[i];
      if constexpr (MASK) {
        v.x = r.h[i].x > 0.f ? v.x : 0.f;
        v.y = r.h[i].y > 0.f ? v.y : 0.f;
        v.z = r.h[i].z > 0.f ? v.z : 0.f;
        v.w = r.h[i].w > 0.f ? v.w : 0.f;
      }
      if (r.kleft < 4) {
        if (r.kleft < 2) v.y = 0.f;
        if (r.kleft < 3) v.z = 0.f;
        v.w = 0.f;
      }
      uint32_t lo[NP], hi[NP];
      split2<NP>(v.x, v.y, lo);
      split2<NP>(v.z, v.w, hi);
      unsigned char* s = S + swz((t >> 3) + 32 * i, (t & 7) >> 1) + ((t & 1) << 3);
#pragma unroll
      for (int p = 0; p < NP; ++p)
        *reinterpret_cast<u32x2*>(s + p * piece_bytes<MN>()) = u32x2{lo[p], hi[p]};
    }
  } else {
    constexpr int KG = 256 / MN;
#pragma unroll
    for (int g = 0; g < MN / 64; ++g) {
      uint32_t q0[NP], q1[NP], q2[NP], q3[NP];
      split2<NP>(r.v[2 * g].x, r.v[2 * g].y, q0);
      split2<NP>(r.v[2 * g].z, r.v[2 * g].w, q1);
      split2<NP>(r.v[2 * g + 1].x, r.v[2 * g + 1].y, q2);
      split2<NP>(r.v[2 * g + 1].z, r.v[2 * g + 1].w, q3);
      unsigned char* s = S + swz(t % MN, (t / MN) + KG * g);
#pragma unroll
      for (int p = 0; p < NP; ++p)
        *reinterpret_cast<u32x4*>(s + p * piece_bytes<MN>()) = u32x4{q0[p], q1[p], q2[p], q3[p]};
    }
  }
}

// ---- bf16 operands (one piece, no split): the tile is MN x 32 bf16 = MN / 64
// 16-byte chunks per thread.
//  KContig : chunk c = t + 256 i is row c / 4, k = 8 (c % 4): a plain 16-byte copy
//  MNContig: v[g] = 8 consecutive k of column mn = t % MN, k = 8 (t / MN + (256 / MN) g),
//            gathered with 2-byte loads (coalesced across the wavefront)
template <int MN>
struct TileRegsB {
  u32x4 v[MN / 64];
  u32x4 h[MN / 64];   // raw mask chunks (MASK only)
  int kleft;          // valid elements (<= 8) from this thread's first k
};

// bf16 value > 0: sign clear and not zero
__device__ __forceinline__ bool bf16_pos(uint32_t h) { return (h & 0x8000u) == 0 && (h & 0x7fffu) != 0; }

template <int MN, Layout L, bool MASK>
__device__ __forceinline__ void load_tile_b(const Operand& op, int64_t mn0, int64_t mn_lim,
                                            int64_t k0, int64_t k_lim, TileRegsB<MN>& r, int t,
                                            int part = -1) {
  const uint16_t* P = static_cast<const uint16_t*>(op.p);
  const uint16_t* Mk = static_cast<const uint16_t*>(op.mask);
  if constexpr (L == Layout::KContig) {
    const int64_t k = k0 + ((t & 3) << 3);   // (t + 256 i) & 3 == t & 3
    const int64_t left = k_lim - k;
    r.kleft = left > 8 ? 8 : static_cast<int>(left);
#pragma unroll
    for (int i = 0; i < MN / 64; ++i) {
      if (part >= 0 && (2 * i) / (MN / 64) != part) continue;
      const int c = t + 256 * i;
      const int64_t mn = mn0 + (c >> 2);
      u32x4 v = {0u, 0u, 0u, 0u}, h = {0u, 0u, 0u, 0u};
      if (mn < mn_lim && k < k_lim) {
        v = *reinterpret_cast<const u32x4*>(P + mn * op.ld + k);
        if constexpr (MASK) h = *reinterpret_cast<const u32x4*>(Mk + mn * op.ld_mask + k);
      }
      r.v[i] = v;
      if constexpr (MASK) r.h[i] = h;
    }
  } else {
    static_assert(!MASK, "masked operands are row-major in k");
    static_assert(MN >= 64 && MN <= 256, "MNContig tiles are 64..256 wide");
    constexpr int KG = 256 / MN;
    const int64_t mn = mn0 + (t % MN);
    const bool mn_ok = mn < mn_lim;
    r.kleft = 8;
#pragma unroll
    for (int g = 0; g < MN / 64; ++g) {
      if (part >= 0 && (2 * g) / (MN / 64) != part) continue;
      const int64_t k8 = k0 + 8 * ((t / MN) + KG * g);
      uint32_t e[8];
      if (mn_ok && k8 + 8 <= k_lim) {   // the usual case: one test for the eight loads
        const uint16_t* src = P + k8 * op.ld + mn;
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = src[j * op.ld];
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          uint32_t x = 0u;
          if (mn_ok && k8 + j < k_lim) x = P[(k8 + j) * op.ld + mn];
          e[j] = x;
        }
      }
      r.v[g] = u32x4{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)};
    }
  }
}

template <int MN, Layout L, bool MASK>
__device__ __forceinline__ void store_tile_b(const TileRegsB<MN>& r, unsigned char* S, int t) {
  if constexpr (L == Layout::KContig) {
#pragma unroll
    for (int i = 0; i < MN / 64; ++i) {
      const int c = t + 256 * i;
      uint32_t w[4] = {r.v[i].x, r.v[i].y, r.v[i].z, r.v[i].w};
      if constexpr (MASK) {
        const uint32_t h[4] = {r.h[i].x, r.h[i].y, r.h[i].z, r.h[i].w};
#pragma unroll
        for (int q = 0; q < 4; ++q)
          w[q] &= (bf16_pos(h[q] & 0xffffu) ? 0xffffu : 0u) | (bf16_pos(h[q] >> 16) ? 0xffff0000u : 0u);
      }
      if (r.kleft < 8) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if (2 * q >= r.kleft) w[q] = 0u;
          else if (2 * q + 1 >= r.kleft) w[q] &= 0xffffu;
        }
      }
      *reinterpret_cast<u32x4*>(S + swz(c >> 2, c & 3)) = u32x4{w[0], w[1], w[2], w[3]};
    }
  } else {
    constexpr int KG = 256 / MN;
#pragma unroll
    for (int g = 0; g < MN / 64; ++g)
      *reinterpret_cast<u32x4*>(S + swz(t % MN, (t / MN) + KG * g)) = r.v[g];
  }
}

// Element-size dispatch: ES = 4 -> fp32 operands split into three pieces,
// ES = 2 -> bf16 operands used as they are.
template <int ES> struct Pieces { static constexpr int N = ES == 4 ? 3 : 1; };
template <int ES, int MN> struct RegsOf;
template <int MN> struct RegsOf<4, MN> { typedef TileRegs<MN> type; };
template <int MN> struct RegsOf<2, MN> { typedef TileRegsB<MN> type; };

template <int ES, int MN, Layout L, bool MASK>
__device__ __forceinline__ void load_any(const Operand& op, int64_t mn0, int64_t mn_lim, int64_t k0,
                                         int64_t k_lim, typename RegsOf<ES, MN>::type& r, int t,
                                         int part = -1) {
  if constexpr (ES == 4) load_tile<MN, L, MASK>(op, mn0, mn_lim, k0, k_lim, r, t, part);
  else load_tile_b<MN, L, MASK>(op, mn0, mn_lim, k0, k_lim, r, t, part);
}
template <int ES, int MN, Layout L, bool MASK>
__device__ __forceinline__ void store_any(const typename RegsOf<ES, MN>::type& r, unsigned char* S,
                                          int t) {
  if constexpr (ES == 4) store_tile<MN, L, 3, MASK>(r, S, t);
  else store_tile_b<MN, L, MASK>(r, S, t);
}

// 16-byte MFMA operand of `lane`: row (row0 + lane % 32), k = 16 kc + 8 (lane / 32) .. + 7
__device__ __forceinline__ bf16x8 read_operand(const unsigned char* piece, int row0, int kc,
                                               int lane) {
  return *reinterpret_cast<const bf16x8*>(piece + swz(row0 + (lane & 31), 2 * kc + (lane >> 5)));
}

// Which piece products are accumulated, small terms first: for NP = 3 the six
// with i + j <= 4 (0-based piece indices below), for NP = 1 the single product.
template <int NP>
constexpr int n_products() { return NP == 3 ? 6 : 1; }
template <int NP>
constexpr int product_a(int q) {
  return NP == 3 ? (q == 0 ? 0 : q == 1 ? 2 : q == 2 ? 1 : q == 3 ? 0 : q == 4 ? 1 : 0) : 0;
}
template <int NP>
constexpr int product_b(int q) {
  return NP == 3 ? (q == 0 ? 2 : q == 1 ? 0 : q == 2 ? 1 : q == 3 ? 1 : q == 4 ? 0 : 0) : 0;
}

// acc[i][j] += A(64 wm + 32 i .., :) * B(64 wn + 32 j .., :)^T over one BK step.
// mid(b), b = 0..3: called between blocks of products; the kernel issues the next step's global
// loads there, a quarter at a time (issued in one burst they hold the wavefront at the memory
// pipe while the matrix pipe idles).
template <int NP, class Mid>
__device__ __forceinline__ void mma_step(const unsigned char* As, const unsigned char* Bs, int wm,
                                         int wn, int lane, f32x16 (&acc)[2][2], Mid&& mid) {
#pragma unroll
  for (int kc = 0; kc < BK / 16; ++kc) {
    bf16x8 a[2][NP], b[2][NP];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int p = 0; p < NP; ++p) {
        a[i][p] = read_operand(As + p * piece_bytes<BM>(), 64 * wm + 32 * i, kc, lane);
        b[i][p] = read_operand(Bs + p * piece_bytes<BN>(), 64 * wn + 32 * i, kc, lane);
      }
#pragma unroll
    for (int q = 0; q < n_products<NP>(); ++q) {
      if (q == 0 || (n_products<NP>() > 1 && q == n_products<NP>() / 2)) {
        __builtin_amdgcn_sched_barrier(0);
        if (n_products<NP>() > 1) mid(2 * kc + (q == 0 ? 0 : 1));
        else { mid(2 * kc); mid(2 * kc + 1); }   // one product per block: two quarters at once
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              a[i][product_a<NP>(q)], b[j][product_b<NP>(q)], acc[i][j], 0, 0, 0);
    }
  }
}

// Position of accumulator register r of a 32 x 32 block held by `lane`:
// column = lane % 32, row = 8 (r / 4) + 4 (lane / 32) + r % 4.
__device__ __forceinline__ int acc_row(int r, int lane) {
  return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
}

// kStore: C = acc; kStoreRelu: C = max(acc, 0); kStorePartial: slice blockIdx.z of a
// split-K workspace; kStoreAddRows: C[m, :] = acc + add[row(m), :] with
// row(m) = add_ids ? add_ids[m] : add_base + m (rows outside [0, add_rows) are skipped).
enum Epilogue { kStore = 0, kStoreRelu = 1, kStorePartial = 2, kStoreAddRows = 3 };

struct EpiArgs {
  int64_t split_stride;
  const void* add;   // residual rows, same element type as C
  int64_t ld_add;
  const int32_t* add_ids;
  int64_t add_base;
  int64_t add_rows;
};

constexpr int C_LD = 128 + 4;  // floats per row of the staged output half-tile
template <int NP>
constexpr int smem_bytes() {
  return (2 * tile_bytes<128, NP>() > 64 * C_LD * 4) ? 2 * tile_bytes<128, NP>() : 64 * C_LD * 4;
}

// C[M, N] = A * B. ESI = bytes per input element: 4 -> fp32 operands, three-way
// split, fp32-equivalent accuracy; 2 -> bf16 operands, one product. ESO = bytes per
// output element (fp32, or bf16 rounded to nearest-even); sums are fp32 either way.
// A: element (m, k); B: element (n, k) in the Operand sense above.
template <int ESI, Layout LA, bool MASK_A, Layout LB, bool MASK_B, int EPI, int ESO = 4>
__global__ __launch_bounds__(256, 2) void gemm_kernel(Operand A, Operand B, int64_t M, int64_t N,
                                                      int64_t K, int64_t k_per_split, void* C,
                                                      int64_t ldc, EpiArgs ep) {
  constexpr int NP = Pieces<ESI>::N;
  __shared__ __attribute__((aligned(16))) unsigned char smem[smem_bytes<NP>()];
  unsigned char* As = smem;
  unsigned char* Bs = smem + tile_bytes<BM, NP>();
  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int64_t m0 = static_cast<int64_t>(blockIdx.x) * BM;
  const int64_t n0 = static_cast<int64_t>(blockIdx.y) * BN;
  const int64_t k_begin = static_cast<int64_t>(blockIdx.z) * k_per_split;
  const int64_t k_end = (k_begin + k_per_split < K) ? k_begin + k_per_split : K;

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  typename RegsOf<ESI, BM>::type ra;
  typename RegsOf<ESI, BN>::type rb;
  if (k_begin < k_end) {
    load_any<ESI, BM, LA, MASK_A>(A, m0, M, k_begin, k_end, ra, t);
    load_any<ESI, BN, LB, MASK_B>(B, n0, N, k_begin, k_end, rb, t);
  }
  for (int64_t k0 = k_begin; k0 < k_end; k0 += BK) {
    __syncthreads();
    store_any<ESI, BM, LA, MASK_A>(ra, As, t);
    store_any<ESI, BN, LB, MASK_B>(rb, Bs, t);
    __syncthreads();
    const bool more = k0 + BK < k_end;
    auto mid = [&](int blk) __attribute__((always_inline)) {   // blk = 0..3: A halves, then B halves
      if (!more) return;
      if (blk < 2) load_any<ESI, BM, LA, MASK_A>(A, m0, M, k0 + BK, k_end, ra, t, blk);
      else load_any<ESI, BN, LB, MASK_B>(B, n0, N, k0 + BK, k_end, rb, t, blk - 2);
    };
    mma_step<NP>(As, Bs, wm, wn, lane, acc, mid);
  }

  // ---- epilogue: the tile goes through LDS (the operand staging is free now)
  // so that global accesses are 4 consecutive columns per lane and whole row
  // segments per wavefront; two passes of 64 rows each.
  float* Cs = reinterpret_cast<float*>(smem);
  unsigned char* Cb = static_cast<unsigned char*>(C);
  if constexpr (EPI == kStorePartial)
    Cb += static_cast<int64_t>(blockIdx.z) * ep.split_stride * ESO;
  const int c = lane & 31;
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    __syncthreads();
    if (wm == p) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            Cs[(i * 32 + acc_row(r, lane)) * C_LD + wn * 64 + j * 32 + c] = acc[i][j][r];
    }
    __syncthreads();
    const int64_t n = n0 + ((t & 31) << 2);
    int64_t src[8];
    if constexpr (EPI == kStoreAddRows) {
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int64_t m = m0 + p * 64 + (t >> 5) + 8 * q;
        int64_t sr = -1;
        if (m < M) {
          sr = ep.add_ids ? static_cast<int64_t>(ep.add_ids[m]) : ep.add_base + m;
          if (sr < 0 || sr >= ep.add_rows) sr = -1;  // bad id: leave the row alone
        }
        src[q] = sr;
      }
    }
    f32x4 v[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      v[q] = *reinterpret_cast<const f32x4*>(&Cs[((t >> 5) + 8 * q) * C_LD + ((t & 31) << 2)]);
      if constexpr (EPI == kStoreRelu) {
        v[q].x = v[q].x > 0.f ? v[q].x : 0.f;
        v[q].y = v[q].y > 0.f ? v[q].y : 0.f;
        v[q].z = v[q].z > 0.f ? v[q].z : 0.f;
        v[q].w = v[q].w > 0.f ? v[q].w : 0.f;
      }
      if constexpr (EPI == kStoreAddRows) {
        if (src[q] >= 0 && n < N) {
          if constexpr (ESO == 4) {
            v[q] += *reinterpret_cast<const f32x4*>(static_cast<const float*>(ep.add) +
                                                    src[q] * ep.ld_add + n);
          } else {
            const u32x2 w = *reinterpret_cast<const u32x2*>(static_cast<const uint16_t*>(ep.add) +
                                                            src[q] * ep.ld_add + n);
            v[q].x += low_as_f32(w.x);
            v[q].y += high_as_f32(w.x);
            v[q].z += low_as_f32(w.y);
            v[q].w += high_as_f32(w.y);
          }
        }
      }
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int64_t m = m0 + p * 64 + (t >> 5) + 8 * q;
      if (m >= M || n >= N) continue;
      if constexpr (EPI == kStoreAddRows) {
        if (src[q] < 0) continue;
      }
      const int64_t left = N - n;
      if constexpr (ESO == 4) {
        float* y = reinterpret_cast<float*>(Cb) + m * ldc + n;
        if (left >= 4) {
          *reinterpret_cast<f32x4*>(y) = v[q];
        } else {
          y[0] = v[q].x;
          if (left > 1) y[1] = v[q].y;
          if (left > 2) y[2] = v[q].z;
        }
      } else {
        uint16_t* y = reinterpret_cast<uint16_t*>(Cb) + m * ldc + n;
        const u32x2 w = {pack_bf16(v[q].x, v[q].y), pack_bf16(v[q].z, v[q].w)};
        if (left >= 4) {
          *reinterpret_cast<u32x2*>(y) = w;
        } else {
          y[0] = static_cast<uint16_t>(w.x & 0xffffu);
          if (left > 1) y[1] = static_cast<uint16_t>(w.x >> 16);
          if (left > 2) y[2] = static_cast<uint16_t>(w.y & 0xffffu);
        }
      }
    }
  }
}

}  // namespace mx
}  // namespace sat

#endif  // SAT_MX_TILE_H_

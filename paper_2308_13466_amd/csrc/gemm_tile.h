// fp32 MFMA tile GEMM building blocks for gfx950 (64-wide wavefronts).
//
// A workgroup of 256 threads (4 wavefronts, 2 x 2) owns a 128 x 128 tile of
// C = A * B and walks K in steps of 32. Each wavefront owns a 64 x 64 sub-tile
// as 2 x 2 blocks of v_mfma_f32_32x32x2_f32 (16 accumulator registers each).
// Operand tiles are staged in LDS k-major (S[k][mn]), which is the order the
// MFMA operands want: lanes 0-31 read 32 consecutive mn at k, lanes 32-63 at
// k+1. Global loads for step i+1 are issued into registers before the MFMAs of
// step i, so HBM/L2 latency hides behind the matrix pipe.
//
// An operand is described by where its contiguous axis lies:
//   KContig : element (mn, k) at p[mn * ld + k]  (transposing store into LDS)
//   MNContig: element (mn, k) at p[k * ld + mn]  (direct 16-byte store into LDS)
// and may carry a same-shaped mask matrix: elements whose mask value is not
// > 0 are read as 0 (that is how relu'(Z) is applied without materialising dZ).
// Every base pointer must be 16-byte aligned and every ld a multiple of 4.
#ifndef SAT_GEMM_TILE_H_
#define SAT_GEMM_TILE_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sat {
namespace gemm {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 32;
constexpr int LDS_LD = 128 + 4;              // floats per k-row of a staged 128-wide tile
constexpr int TILE_FLOATS = BK * LDS_LD;     // one 128 x 32 operand tile in LDS

enum class Layout { KContig, MNContig };

struct Operand {
  const float* p;
  int64_t ld;
  const float* mask;  // nullptr or same indexing as p with its own ld
  int64_t ld_mask;
};

// Registers holding one thread's share of an MN x 32 operand tile
// (MN a multiple of 32, at most 512): MN / 32 16-byte vectors.
template <int MN>
struct TileRegs {
  f32x4 v[MN / 32];
};

template <int MN>
constexpr int lds_ld() { return MN + 4; }  // floats per k-row of a staged tile

template <int MN, Layout L, bool MASK>
__device__ __forceinline__ void load_tile(const Operand& op, int64_t mn0, int64_t mn_lim,
                                          int64_t k0, int64_t k_lim, TileRegs<MN>& r, int t) {
  constexpr int kThreadsPerK = MN / 4;            // MNContig: threads covering one k-row
  constexpr int kRowsPerPass = 256 / kThreadsPerK == 0 ? 1 : 256 / kThreadsPerK;
#pragma unroll
  for (int i = 0; i < MN / 32; ++i) {
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if constexpr (L == Layout::KContig) {
      const int64_t mn = mn0 + (t >> 3) + 32 * i;
      const int64_t k = k0 + ((t & 7) << 2);
      if (mn < mn_lim && k < k_lim) {
        v = *reinterpret_cast<const f32x4*>(op.p + mn * op.ld + k);
        if constexpr (MASK) {
          const f32x4 h = *reinterpret_cast<const f32x4*>(op.mask + mn * op.ld_mask + k);
          v.x = h.x > 0.f ? v.x : 0.f;
          v.y = h.y > 0.f ? v.y : 0.f;
          v.z = h.z > 0.f ? v.z : 0.f;
          v.w = h.w > 0.f ? v.w : 0.f;
        }
        if (k + 3 >= k_lim) {
          if (k + 1 >= k_lim) v.y = 0.f;
          if (k + 2 >= k_lim) v.z = 0.f;
          v.w = 0.f;
        }
      }
    } else {
      static_assert(MN <= 1024, "tile too wide");
      const int64_t k = k0 + t / kThreadsPerK + kRowsPerPass * i;
      const int64_t mn = mn0 + ((t % kThreadsPerK) << 2);
      if (k < k_lim && mn < mn_lim) {
        v = *reinterpret_cast<const f32x4*>(op.p + k * op.ld + mn);
        if constexpr (MASK) {
          const f32x4 h = *reinterpret_cast<const f32x4*>(op.mask + k * op.ld_mask + mn);
          v.x = h.x > 0.f ? v.x : 0.f;
          v.y = h.y > 0.f ? v.y : 0.f;
          v.z = h.z > 0.f ? v.z : 0.f;
          v.w = h.w > 0.f ? v.w : 0.f;
        }
        if (mn + 3 >= mn_lim) {
          if (mn + 1 >= mn_lim) v.y = 0.f;
          if (mn + 2 >= mn_lim) v.z = 0.f;
          v.w = 0.f;
        }
      }
    }
    r.v[i] = v;
  }
}

template <int MN, Layout L>
__device__ __forceinline__ void store_tile(const TileRegs<MN>& r, float* S, int t) {
  constexpr int LD = lds_ld<MN>();
  constexpr int kThreadsPerK = MN / 4;
  constexpr int kRowsPerPass = 256 / kThreadsPerK == 0 ? 1 : 256 / kThreadsPerK;
#pragma unroll
  for (int i = 0; i < MN / 32; ++i) {
    if constexpr (L == Layout::KContig) {
      float* s = S + ((t & 7) << 2) * LD + (t >> 3) + 32 * i;
      s[0] = r.v[i].x;
      s[LD] = r.v[i].y;
      s[2 * LD] = r.v[i].z;
      s[3 * LD] = r.v[i].w;
    } else {
      *reinterpret_cast<f32x4*>(S + (t / kThreadsPerK + kRowsPerPass * i) * LD +
                                ((t % kThreadsPerK) << 2)) = r.v[i];
    }
  }
}

// acc[bm][bn] += As[:, 64*wm + 32*bm ..] ^T * Bs[:, 64*wn + 32*bn ..] over one BK step.
__device__ __forceinline__ void mma_step(const float* As, const float* Bs, int wm, int wn,
                                         int lane, f32x16 (&acc)[2][2]) {
  const int kr = lane >> 5;
  const int c = lane & 31;
#pragma unroll
  for (int kk = 0; kk < BK; kk += 2) {
    const float* a = As + (kk + kr) * LDS_LD + wm * 64 + c;
    const float* b = Bs + (kk + kr) * LDS_LD + wn * 64 + c;
    const float a0 = a[0], a1 = a[32], b0 = b[0], b1 = b[32];
    acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
    acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
    acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
    acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
  }
}

// Position of accumulator register r of a 32 x 32 MFMA block held by `lane`:
// column = lane % 32, row = 8 * (r / 4) + 4 * (lane / 32) + r % 4.
__device__ __forceinline__ int acc_row(int r, int lane) {
  return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
}

// kStore: C = acc; kStoreRelu: C = max(acc, 0); kStorePartial: slice blockIdx.z of a
// split-K workspace; kStoreAddRows: C[m, :] = acc + add[row(m), :] with
// row(m) = add_ids ? add_ids[m] : add_base + m (rows outside [0, add_rows) are skipped).
enum Epilogue { kStore = 0, kStoreRelu = 1, kStorePartial = 2, kStoreAddRows = 3 };

struct EpiArgs {
  int64_t split_stride;
  const float* add;
  int64_t ld_add;
  const int32_t* add_ids;
  int64_t add_base;
  int64_t add_rows;
};


template <Layout LA, bool MASK_A, Layout LB, bool MASK_B, int EPI>
__global__ __launch_bounds__(256, 2) void gemm_f32_kernel(Operand A, Operand B, int64_t M,
                                                          int64_t N, int64_t K,
                                                          int64_t k_per_split, float* C,
                                                          int64_t ldc, EpiArgs ep) {
  __shared__ __attribute__((aligned(16))) float smem[2 * TILE_FLOATS];
  float* As = smem;
  float* Bs = smem + TILE_FLOATS;
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

  TileRegs<BM> ra;
  TileRegs<BN> rb;
  if (k_begin < k_end) {
    load_tile<BM, LA, MASK_A>(A, m0, M, k_begin, k_end, ra, t);
    load_tile<BN, LB, MASK_B>(B, n0, N, k_begin, k_end, rb, t);
  }
  for (int64_t k0 = k_begin; k0 < k_end; k0 += BK) {
    __syncthreads();
    store_tile<BM, LA>(ra, As, t);
    store_tile<BN, LB>(rb, Bs, t);
    __syncthreads();
    if (k0 + BK < k_end) {
      load_tile<BM, LA, MASK_A>(A, m0, M, k0 + BK, k_end, ra, t);
      load_tile<BN, LB, MASK_B>(B, n0, N, k0 + BK, k_end, rb, t);
    }
    mma_step(As, Bs, wm, wn, lane, acc);
  }

  // ---- epilogue: the tile goes through LDS (the operand buffers are free now)
  // so that global accesses are 16 bytes per lane and 512 bytes per row
  // segment; two passes of 64 rows each fit the 33 KiB of operand staging.
  float* Cb = C;
  if constexpr (EPI == kStorePartial) Cb += static_cast<int64_t>(blockIdx.z) * ep.split_stride;
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
            smem[(i * 32 + acc_row(r, lane)) * LDS_LD + wn * 64 + j * 32 + c] = acc[i][j][r];
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
      v[q] = *reinterpret_cast<const f32x4*>(&smem[((t >> 5) + 8 * q) * LDS_LD + ((t & 31) << 2)]);
      if constexpr (EPI == kStoreRelu) {
        v[q].x = v[q].x > 0.f ? v[q].x : 0.f;
        v[q].y = v[q].y > 0.f ? v[q].y : 0.f;
        v[q].z = v[q].z > 0.f ? v[q].z : 0.f;
        v[q].w = v[q].w > 0.f ? v[q].w : 0.f;
      }
      if constexpr (EPI == kStoreAddRows) {
        if (src[q] >= 0 && n < N)
          v[q] += *reinterpret_cast<const f32x4*>(ep.add + src[q] * ep.ld_add + n);
      }
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int64_t m = m0 + p * 64 + (t >> 5) + 8 * q;
      if (m >= M || n >= N) continue;
      if constexpr (EPI == kStoreAddRows) {
        if (src[q] < 0) continue;
      }
      float* y = Cb + m * ldc + n;
      const int64_t left = N - n;
      if (left >= 4) {
        *reinterpret_cast<f32x4*>(y) = v[q];
      } else {
        y[0] = v[q].x;
        if (left > 1) y[1] = v[q].y;
        if (left > 2) y[2] = v[q].z;
      }
    }
  }
}


}  // namespace gemm
}  // namespace sat

#endif  // SAT_GEMM_TILE_H_

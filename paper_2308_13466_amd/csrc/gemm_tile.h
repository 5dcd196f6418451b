// fp32 MFMA (v_mfma_f32_32x32x2_f32) tile building blocks for gfx950, used by
// the predictor's LSTM kernel. Operand tiles are staged in LDS k-major
// (S[k][mn]), which is the order the fp32 MFMA operands want: lanes 0-31 read
// 32 consecutive mn at k, lanes 32-63 at k+1. Global loads for step i+1 are
// issued into registers before the MFMAs of step i.
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

}  // namespace gemm
}  // namespace sat

#endif  // SAT_GEMM_TILE_H_

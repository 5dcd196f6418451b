// Embedding predictor g_omega, inference (Eq. 7; Sec. "Embedding Predictor": an
// RNN-GNN made of an LSTM over the last tau epochs' cached embeddings and a GCN
// over the partition-plus-halo graph). Output: predicted halo embeddings,
// written in place into the halo rows of Hbar.
//
// Two kernels.
//  lstm_kernel: a workgroup owns 32*WM nodes and all 4*d_s gate columns. Per
//   time step the gate pre-activations [x_s | h_{s-1}] [Wx | Wh]^T are one fp32
//   MFMA GEMM whose accumulators never leave registers: a wavefront holds the
//   i, f, g, o blocks of the same (node, hidden-unit) positions, so the cell
//   update is register-local; c stays in registers across steps and h goes to
//   LDS k-major, which is exactly the A-operand layout of the next step's
//   recurrent product. Only S = h_tau [n_bar, d_s] is written to memory. The
//   window rows can be read straight out of the history table through ids.
//  hop_kernel: a workgroup owns 64 halo nodes: gathers and weights the S rows
//   of each node's local neighbours (transposed halo block) plus its own,
//   keeps the [64, d_s] aggregate in LDS, multiplies by Wg on the MFMA pipe and
//   adds the newest cached embedding in the epilogue.
#include <math.h>

#include "gemm_tile.h"
#include "sat_internal.h"

namespace sat {
// rows.hip: dst[k, 0:d) = src[(ids ? ids[k] : k + id_base), 0:d)
sat_status row_gather(const void* src, int64_t ld_src, void* dst, int64_t ld_dst,
                      const int32_t* ids, int64_t id_base, int64_t n, int64_t n_src_rows,
                      int32_t d, hipStream_t stream);
}  // namespace sat

namespace {

using namespace sat::gemm;
using sat::kWave;

constexpr int kMaxTau = 8;
struct SlotPtrs {
  const float* p[kMaxTau];
};

__device__ __forceinline__ float sigmoidf_(float x) { return 1.0f / (1.0f + expf(-x)); }

template <int DS>
__global__ __launch_bounds__(256) void lstm_kernel(SlotPtrs slots, int tau, int64_t n_rows_slot,
                                                   int64_t ld_slot,
                                                   const int32_t* __restrict__ ids,
                                                   int64_t n_nodes, int d,
                                                   const float* __restrict__ Wx,
                                                   const float* __restrict__ Wh,
                                                   const float* __restrict__ bias,
                                                   float* __restrict__ S) {
  constexpr int WN = DS / 32;   // wavefronts along hidden units
  constexpr int WM = 4 / WN;    // wavefronts along nodes
  constexpr int BMR = 32 * WM;  // nodes per workgroup
  constexpr int NB = 4 * DS;    // gate columns
  constexpr int LDA = lds_ld<BMR>(), LDB = lds_ld<NB>(), LDH = BMR + 4;
  __shared__ __attribute__((aligned(16))) float As[BK * LDA];
  __shared__ __attribute__((aligned(16))) float Bs[BK * LDB];
  __shared__ __attribute__((aligned(16))) float Hs[DS * LDH];

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int kr = lane >> 5, c = lane & 31;
  const int64_t node0 = static_cast<int64_t>(blockIdx.x) * BMR;

  // table row of each node this thread loads x for (-1: nothing to load)
  int64_t arow[BMR / 32];
#pragma unroll
  for (int i = 0; i < BMR / 32; ++i) {
    const int64_t node = node0 + (t >> 3) + 32 * i;
    int64_t r = -1;
    if (node < n_nodes) {
      r = ids ? static_cast<int64_t>(ids[node]) : node;
      if (r < 0 || r >= n_rows_slot) r = -1;
    }
    arow[i] = r;
  }
  const int unit = 32 * wn + c;
  const float b_i = bias[unit], b_f = bias[DS + unit], b_g = bias[2 * DS + unit],
              b_o = bias[3 * DS + unit];

  float cstate[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) cstate[r] = 0.f;
  float hval[16];

  const Operand opx{Wx, static_cast<int64_t>(d), nullptr, 0};
  const Operand oph{Wh, static_cast<int64_t>(DS), nullptr, 0};

  for (int s = 0; s < tau; ++s) {
    f32x16 acc[4];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[g][r] = 0.f;

    // ---- input part: x_s Wx^T, K = d
    const float* xs = slots.p[s];
    auto load_x = [&](int k0, TileRegs<BMR>& ra) {
#pragma unroll
      for (int i = 0; i < BMR / 32; ++i) {
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        const int k = k0 + ((t & 7) << 2);
        if (arow[i] >= 0 && k < d) {
          v = *reinterpret_cast<const f32x4*>(xs + arow[i] * ld_slot + k);
          if (k + 3 >= d) {
            if (k + 1 >= d) v.y = 0.f;
            if (k + 2 >= d) v.z = 0.f;
            v.w = 0.f;
          }
        }
        ra.v[i] = v;
      }
    };
    TileRegs<BMR> ra;
    TileRegs<NB> rb;
    load_x(0, ra);
    load_tile<NB, Layout::KContig, false>(opx, 0, NB, 0, d, rb, t);
    for (int k0 = 0; k0 < d; k0 += BK) {
      __syncthreads();
      store_tile<BMR, Layout::KContig>(ra, As, t);
      store_tile<NB, Layout::KContig>(rb, Bs, t);
      __syncthreads();
      if (k0 + BK < d) {
        load_x(k0 + BK, ra);
        load_tile<NB, Layout::KContig, false>(opx, 0, NB, k0 + BK, d, rb, t);
      }
#pragma unroll
      for (int kk = 0; kk < BK; kk += 2) {
        const float a = As[(kk + kr) * LDA + 32 * wm + c];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const float bv = Bs[(kk + kr) * LDB + g * DS + 32 * wn + c];
          acc[g] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, bv, acc[g], 0, 0, 0);
        }
      }
    }
    // ---- recurrent part: h_{s-1} Wh^T, K = DS (h_0 = 0: nothing to add at s = 0)
    if (s > 0) {
      load_tile<NB, Layout::KContig, false>(oph, 0, NB, 0, DS, rb, t);
      for (int k0 = 0; k0 < DS; k0 += BK) {
        __syncthreads();
        store_tile<NB, Layout::KContig>(rb, Bs, t);
        __syncthreads();
        if (k0 + BK < DS) load_tile<NB, Layout::KContig, false>(oph, 0, NB, k0 + BK, DS, rb, t);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
          const float a = Hs[(k0 + kk + kr) * LDH + 32 * wm + c];
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const float bv = Bs[(kk + kr) * LDB + g * DS + 32 * wn + c];
            acc[g] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, bv, acc[g], 0, 0, 0);
          }
        }
      }
    }
    // ---- cell update, register-local
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float gi = sigmoidf_(acc[0][r] + b_i);
      const float gf = sigmoidf_(acc[1][r] + b_f);
      const float gg = tanhf(acc[2][r] + b_g);
      const float go = sigmoidf_(acc[3][r] + b_o);
      cstate[r] = gf * cstate[r] + gi * gg;
      hval[r] = go * tanhf(cstate[r]);
    }
    if (s + 1 < tau) {
      __syncthreads();  // every wavefront has finished reading Hs for this step
#pragma unroll
      for (int r = 0; r < 16; ++r) Hs[unit * LDH + 32 * wm + acc_row(r, lane)] = hval[r];
      // the next step's first __syncthreads orders these writes before any read
    }
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int64_t node = node0 + 32 * wm + acc_row(r, lane);
    if (node < n_nodes) S[node * DS + unit] = hval[r];
  }
}

template <int DS>
__global__ __launch_bounds__(256) void hop_kernel(const int64_t* __restrict__ h_colptr,
                                                  const int32_t* __restrict__ h_row,
                                                  const float* __restrict__ h_val,
                                                  const float* __restrict__ h_self,
                                                  int64_t n_local, int64_t n_halo,
                                                  const float* __restrict__ S,
                                                  const float* __restrict__ Wg, int d,
                                                  const float* __restrict__ newest,
                                                  int64_t n_rows_slot, int64_t ld_slot,
                                                  const int32_t* __restrict__ ids,
                                                  float* __restrict__ Hbar, int64_t ld) {
  constexpr int BMH = 64;             // halo nodes per workgroup
  constexpr int G = DS / 4;           // lanes covering one S row with 16-byte loads
  constexpr int NG = kWave / G;       // neighbours taken at once by a wavefront
  constexpr int LDG = BMH + 4;
  __shared__ __attribute__((aligned(16))) float Ag[DS * LDG];      // aggregate, k-major
  __shared__ __attribute__((aligned(16))) float Bs[BK * LDS_LD];   // Wg tile [32 x 128]

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int64_t u0 = static_cast<int64_t>(blockIdx.x) * BMH;

  // ---- phase 1: Ag[:, m] = h_self[u] S[n_local+u] + sum_k h_val[k] S[h_row[k]]
  {
    const int gl = lane % G, grp = lane / G;
    for (int rr = 0; rr < BMH / 4; ++rr) {
      const int m = wave * (BMH / 4) + rr;
      const int64_t u = u0 + m;
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
      if (u < n_halo) {
        if (grp == 0) {
          const f32x4 x = *reinterpret_cast<const f32x4*>(S + (n_local + u) * DS + gl * 4);
          acc = h_self[u] * x;
        }
        const int64_t s = h_colptr[u], e = h_colptr[u + 1];
        for (int64_t base = s; base < e; base += kWave) {
          const int cnt = static_cast<int>(e - base < kWave ? e - base : kWave);
          int32_t rj = 0;
          float vj = 0.f;
          if (lane < cnt) {
            rj = h_row[base + lane];
            vj = h_val[base + lane];
          }
          const bool ok = static_cast<uint32_t>(rj) < static_cast<uint64_t>(n_local);
          for (int j = 0; j < cnt; j += NG) {
            const int32_t r2 = __shfl(rj, j + grp);
            const float v2 = __shfl(vj, j + grp);
            const bool ok2 = __shfl(static_cast<int>(ok), j + grp) != 0 && (j + grp < cnt);
            if (ok2) {
              const f32x4 x = *reinterpret_cast<const f32x4*>(S + static_cast<int64_t>(r2) * DS + gl * 4);
              acc += v2 * x;
            }
          }
        }
      }
#pragma unroll
      for (int off = G; off < kWave; off <<= 1) {
        acc.x += __shfl_xor(acc.x, off);
        acc.y += __shfl_xor(acc.y, off);
        acc.z += __shfl_xor(acc.z, off);
        acc.w += __shfl_xor(acc.w, off);
      }
      if (grp == 0) {
        Ag[(gl * 4 + 0) * LDG + m] = acc.x;
        Ag[(gl * 4 + 1) * LDG + m] = acc.y;
        Ag[(gl * 4 + 2) * LDG + m] = acc.z;
        Ag[(gl * 4 + 3) * LDG + m] = acc.w;
      }
    }
  }

  // ---- phase 2: Hbar[n_local + u, :] = newest[u, :] + Ag^T Wg, 128 columns at a time
  const int wm = wave >> 1, wn = wave & 1;
  const int kr = lane >> 5, c = lane & 31;
  const Operand opg{Wg, static_cast<int64_t>(d), nullptr, 0};
  // table row of the newest embedding for the rows this lane stores
  for (int n0 = 0; n0 < d; n0 += 128) {
    f32x16 acc[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    TileRegs<128> rb;
    load_tile<128, Layout::MNContig, false>(opg, n0, d, 0, DS, rb, t);
    for (int k0 = 0; k0 < DS; k0 += BK) {
      __syncthreads();  // also orders phase 1's Ag writes before the first read
      store_tile<128, Layout::MNContig>(rb, Bs, t);
      __syncthreads();
      if (k0 + BK < DS) load_tile<128, Layout::MNContig, false>(opg, n0, d, k0 + BK, DS, rb, t);
#pragma unroll
      for (int kk = 0; kk < BK; kk += 2) {
        const float a = Ag[(k0 + kk + kr) * LDG + 32 * wm + c];
        const float b0 = Bs[(kk + kr) * LDS_LD + 64 * wn + c];
        const float b1 = Bs[(kk + kr) * LDS_LD + 64 * wn + 32 + c];
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b0, acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b1, acc[1], 0, 0, 0);
      }
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int64_t u = u0 + 32 * wm + acc_row(r, lane);
      if (u >= n_halo) continue;
      int64_t src = ids ? static_cast<int64_t>(ids[n_local + u]) : n_local + u;
      if (src < 0 || src >= n_rows_slot) continue;  // bad id: leave the row alone
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int col = n0 + 64 * wn + 32 * j + c;
        if (col < d) Hbar[(n_local + u) * ld + col] = newest[src * ld_slot + col] + acc[j][r];
      }
    }
  }
}

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

}  // namespace

extern "C" int64_t sat_predict_workspace_bytes(int64_t n_local, int64_t n_halo, int32_t d,
                                               int32_t d_s, int32_t tau) {
  (void)d;
  (void)tau;
  if (n_local < 0 || n_halo < 0 || d_s <= 0) return 0;
  return round_up((n_local + n_halo) * static_cast<int64_t>(d_s) * 4, 256);
}

extern "C" sat_status sat_predict(const sat_part_view* pv, const sat_predictor* w,
                                  const void* const* slots, int64_t n_rows_slot,
                                  int64_t ld_slot, const int32_t* ids, void* Hbar, int64_t ld,
                                  int32_t dtype, void* workspace, int64_t workspace_bytes,
                                  void* stream) {
  if (!pv || !w || !slots) return SAT_EINVAL;
  if (pv->n_local < 0 || pv->n_halo < 0 || pv->nnz_halo < 0 || n_rows_slot < 0) return SAT_EINVAL;
  if (w->d < 0 || w->tau < 1) return SAT_EINVAL;
  if (dtype != SAT_F32) return dtype == SAT_BF16 ? SAT_EUNSUPPORTED : SAT_EINVAL;
  if (w->tau > kMaxTau) return SAT_EUNSUPPORTED;
  const int64_t n_bar = pv->n_local + pv->n_halo;
  if (n_bar > INT32_MAX) return SAT_EUNSUPPORTED;
  const int d = w->d;
  if (pv->n_halo == 0 || d == 0) return SAT_OK;
  if (!Hbar || ld < d || ld_slot < d) return SAT_EINVAL;
  for (int s = 0; s < w->tau; ++s)
    if (!slots[s]) return SAT_EINVAL;
  if (!sat::aligned16(Hbar) || (ld % 4) != 0 || (ld_slot % 4) != 0) return SAT_EALIGN;
  for (int s = 0; s < w->tau; ++s)
    if (!sat::aligned16(slots[s])) return SAT_EALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const float* newest = static_cast<const float*>(slots[w->tau - 1]);
  float* halo_out = static_cast<float*>(Hbar) + pv->n_local * ld;

  if (w->bypass) {
    return sat::row_gather(newest, ld_slot, halo_out, ld, ids ? ids + pv->n_local : nullptr,
                           pv->n_local, pv->n_halo, n_rows_slot, d, st);
  }

  if (!w->Wx || !w->Wh || !w->b || !w->Wg) return SAT_EINVAL;
  if (w->d_s != 32 && w->d_s != 64 && w->d_s != 128) return SAT_EUNSUPPORTED;
  if ((d % 4) != 0) return SAT_EUNSUPPORTED;  // Wx, Wg rows are d floats, read 16 bytes at a time
  if (!sat::aligned16(w->Wx) || !sat::aligned16(w->Wh) || !sat::aligned16(w->Wg)) return SAT_EALIGN;
  if (!pv->h_colptr || !pv->h_self || (pv->nnz_halo > 0 && (!pv->h_row || !pv->h_val)))
    return SAT_EINVAL;
  const int64_t need = sat_predict_workspace_bytes(pv->n_local, pv->n_halo, d, w->d_s, w->tau);
  if (!workspace || workspace_bytes < need) return SAT_EWORKSPACE;
  if (!sat::aligned256(workspace)) return SAT_EALIGN;
  float* S = static_cast<float*>(workspace);

  SlotPtrs sp;
  for (int s = 0; s < kMaxTau; ++s)
    sp.p[s] = s < w->tau ? static_cast<const float*>(slots[s]) : nullptr;

#define SAT_LSTM(DS)                                                                          \
  do {                                                                                        \
    constexpr int rows = 32 * (4 / ((DS) / 32));                                              \
    const int64_t blocks = (n_bar + rows - 1) / rows;                                         \
    lstm_kernel<DS><<<dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st>>>(               \
        sp, w->tau, n_rows_slot, ld_slot, ids, n_bar, d, w->Wx, w->Wh, w->b, S);              \
  } while (0)
#define SAT_HOP(DS)                                                                           \
  do {                                                                                        \
    const int64_t blocks = (pv->n_halo + 63) / 64;                                            \
    hop_kernel<DS><<<dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st>>>(                \
        pv->h_colptr, pv->h_row, pv->h_val, pv->h_self, pv->n_local, pv->n_halo, S, w->Wg, d, \
        newest, n_rows_slot, ld_slot, ids, static_cast<float*>(Hbar), ld);                    \
  } while (0)
  switch (w->d_s) {
    case 32: SAT_LSTM(32); break;
    case 64: SAT_LSTM(64); break;
    default: SAT_LSTM(128); break;
  }
  sat_status rc = sat::check_launch();
  if (rc != SAT_OK) return rc;
  switch (w->d_s) {
    case 32: SAT_HOP(32); break;
    case 64: SAT_HOP(64); break;
    default: SAT_HOP(128); break;
  }
#undef SAT_LSTM
#undef SAT_HOP
  return sat::check_launch();
}

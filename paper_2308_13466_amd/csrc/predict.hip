// Embedding predictor g_omega, inference (Eq. 7; Sec. "Embedding Predictor": an
// RNN-GNN made of an LSTM over the last tau epochs' cached embeddings and a GCN
// over the partition-plus-halo graph). Output: predicted halo embeddings,
// written in place into the halo rows of Hbar.
//
// Steps of a call (each its own kernel, all on the caller's stream):
//  1. LSTM. d_s = 32, 64: lstm_mx.hip, gate pre-activations on the bf16 MFMA pipe
//     (fp32 operands split exactly into three bf16 pieces, six products per
//     element pair; bf16 history rows are used as they are, three products). A
//     workgroup owns 128 nodes and all 4*d_s gate columns; c stays in registers
//     across the tau steps and h goes through LDS in the A-operand layout of the
//     next step's recurrent product. d_s = 128 (fp32 rows only): lstm_kernel
//     below, the same scheme on the fp32 MFMA instruction. Only S = h_tau
//     [n_bar, d_s] (fp32) is written to memory; the window rows are read straight
//     out of the history tables through ids.
//  2. hop aggregation: the kernel of spmm.hip walks the transposed halo block
//     with the diagonal term (A_hat[u,u] S_u) folded in and leaves the
//     [n_halo, d_s] aggregate in the workspace. Halo nodes have very few local
//     neighbours each, so this gather is a latency problem: it needs many
//     independent rows in flight, which that kernel's group-per-row form gives.
//  3. hop product: the tile GEMM of mx_tile.h multiplies the aggregate by Wg and,
//     in its epilogue, adds the newest cached embedding (fetched through the id
//     list) and stores the halo rows of Hbar in the call's element type.
// With bypass set the call is one row gather of the newest slot.
#include <math.h>

#include "gemm_tile.h"
#include "mx_tile.h"
#include "sat_internal.h"

namespace sat {
// rows.hip: dst[k, 0:d) = src[(ids ? ids[k] : k + id_base), 0:d)
sat_status row_gather(const void* src, int64_t ld_src, void* dst, int64_t ld_dst,
                      const int32_t* ids, int64_t id_base, int64_t n, int64_t n_src_rows,
                      int32_t d, int es, hipStream_t stream);
// spmm.hip: Y = M X (+ diag(self_val) X[self_off + i])
sat_status launch_spmm(const int64_t* rowptr, const int64_t* row_end, const int32_t* col,
                       const float* val, const void* X, int64_t ld_x, int64_t n_x_rows, void* Y,
                       int64_t ld_y, int64_t n_rows, int32_t d, int es, const float* self_val,
                       int64_t self_off, int64_t total_entries, hipStream_t stream);
// lstm_mx.hip: the LSTM on the bf16 MFMA pipe (d_s = 32, 64)
int64_t lstm_mx_workspace_bytes(int32_t d, int32_t d_s);
sat_status launch_lstm_mx(const void* const* slot_ptrs, int es_x, int tau, int64_t n_rows_slot,
                          int64_t ld_slot, const int32_t* ids, int64_t n_nodes, int32_t d,
                          int32_t d_s, const float* Wx, const float* Wh, const float* b, float* S,
                          void* ws, hipStream_t st, float* save = nullptr, float* const* proj = nullptr,
                          int n_proj_valid = 0);
// hop_product.hip: out[m] = add[row(m)] + Agg[m] Wg, fp32, weights-stationary streaming kernel
sat_status launch_hop_product(const float* Agg, int64_t M, int32_t ds, const float* Wg, int32_t d,
                              const void* add, int64_t ld_add, const int32_t* add_ids,
                              int64_t add_base, int64_t add_rows, void* out, int64_t ld_out, int eso,
                              hipStream_t st);
}  // namespace sat

namespace {

using namespace sat::gemm;
using sat::kWave;

constexpr int kMaxTau = 8;
struct SlotPtrs {
  const float* p[kMaxTau];
};

// Gate non-linearities on the hardware exp2 / reciprocal units (about 1 ulp
// each): sigmoid(x) = 1 / (1 + 2^(-x log2 e)), tanh(x) = 2 sigmoid(2x) - 1. The
// absolute error is ~2e-7, two orders below the 1e-5 the results are held to,
// and they cost a handful of instructions instead of a libm call each; the
// cell update runs 5 of them per hidden unit per step between MFMA phases.
__device__ __forceinline__ float sigmoidf_(float x) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x));
}
__device__ __forceinline__ float tanhf_(float x) {
  return 2.0f * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-2.8853900817779268f * x)) - 1.0f;
}

// out[c * R + r] = in[r * C + c]: the LSTM weights are re-laid k-major once per
// call so that the gate-weight tiles load with coalesced 16-byte accesses and go
// to LDS without a transposing store.
__global__ __launch_bounds__(256) void transpose_kernel(const float* __restrict__ in, int R, int C,
                                                        float* __restrict__ out) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= R * C) return;
  const int c = idx / R, r = idx - c * R;
  out[idx] = in[r * C + c];
}

// WxT [d, 4*DS] and WhT [DS, 4*DS] are the transposed (k-major) weights.
template <int DS>
__global__ __launch_bounds__(256, DS <= 64 ? 2 : 1) void lstm_kernel(SlotPtrs slots, int tau,
                                                      int64_t n_rows_slot, int64_t ld_slot,
                                                      const int32_t* __restrict__ ids,
                                                      int64_t n_nodes, int d,
                                                      const float* __restrict__ WxT,
                                                      const float* __restrict__ WhT,
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

  const Operand opx{WxT, static_cast<int64_t>(NB), nullptr, 0};
  const Operand oph{WhT, static_cast<int64_t>(NB), nullptr, 0};

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
    load_tile<NB, Layout::MNContig, false>(opx, 0, NB, 0, d, rb, t);
    for (int k0 = 0; k0 < d; k0 += BK) {
      __syncthreads();
      store_tile<BMR, Layout::KContig>(ra, As, t);
      store_tile<NB, Layout::MNContig>(rb, Bs, t);
      __syncthreads();
      if (k0 + BK < d) {
        load_x(k0 + BK, ra);
        load_tile<NB, Layout::MNContig, false>(opx, 0, NB, k0 + BK, d, rb, t);
      }
      if (s == 0) {   // c_0 = 0: the forget gate's block is not needed in the first step
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
          const float a = As[(kk + kr) * LDA + 32 * wm + c];
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            if (g == 1) continue;
            const float bv = Bs[(kk + kr) * LDB + g * DS + 32 * wn + c];
            acc[g] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, bv, acc[g], 0, 0, 0);
          }
        }
      } else {
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
    }
    // ---- recurrent part: h_{s-1} Wh^T, K = DS (h_0 = 0: nothing to add at s = 0)
    if (s > 0) {
      load_tile<NB, Layout::MNContig, false>(oph, 0, NB, 0, DS, rb, t);
      for (int k0 = 0; k0 < DS; k0 += BK) {
        __syncthreads();
        store_tile<NB, Layout::MNContig>(rb, Bs, t);
        __syncthreads();
        if (k0 + BK < DS) load_tile<NB, Layout::MNContig, false>(oph, 0, NB, k0 + BK, DS, rb, t);
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
      const float gg = tanhf_(acc[2][r] + b_g);
      const float go = sigmoidf_(acc[3][r] + b_o);
      if (s == 0) {
        cstate[r] = gi * gg;   // c_0 = 0: the forget gate has nothing to scale
      } else {
        const float gf = sigmoidf_(acc[1][r] + b_f);
        cstate[r] = gf * cstate[r] + gi * gg;
      }
      hval[r] = go * tanhf_(cstate[r]);
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

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

}  // namespace

extern "C" int64_t sat_predict_workspace_bytes(int64_t n_local, int64_t n_halo, int32_t d,
                                               int32_t d_s, int32_t tau) {
  (void)d;
  (void)tau;
  if (n_local < 0 || n_halo < 0 || d_s <= 0) return 0;
  // S [n_bar, d_s], the hop aggregate [n_halo, d_s], then the re-laid weights:
  // bf16 pieces for d_s <= 64, k-major fp32 copies of Wx, Wh for d_s = 128
  const int64_t w_fp32 = round_up(static_cast<int64_t>(d) * 4 * d_s * 4, 256) +
                         round_up(static_cast<int64_t>(d_s) * 4 * d_s * 4, 256);
  const int64_t w_mx = sat::lstm_mx_workspace_bytes(d, d_s);
  return round_up((n_local + n_halo) * static_cast<int64_t>(d_s) * 4, 256) +
         round_up(n_halo * static_cast<int64_t>(d_s) * 4, 256) + (w_mx > 0 ? w_mx : w_fp32);
}

namespace {

// LSTM states of n_nodes rows (the first half of sat_predict): S [n_nodes, d_s]. wts: room for
// the re-laid weights (bf16 pieces for d_s <= 64, k-major fp32 copies of Wx, Wh for d_s = 128).
sat_status run_states(const sat_predictor* w, const void* const* slots, int64_t n_rows_slot,
                      int64_t ld_slot, const int32_t* ids, int64_t n_bar, int es, float* S, float* WxT,
                      float* const* proj, int32_t n_proj_valid, hipStream_t st) {
  const int d = w->d;
  sat_status rc;
  if (proj) {
    if (w->d_s > 64) return SAT_EUNSUPPORTED;      // only the split-bf16 LSTM keeps projections
    if (n_proj_valid < 0 || n_proj_valid >= w->tau) return SAT_EINVAL;   // the newest slot is always new
    for (int s = 0; s < w->tau; ++s)
      if ((s < n_proj_valid && !proj[s]) || (reinterpret_cast<uintptr_t>(proj[s]) & 3u)) return SAT_EINVAL;
  }
  if (w->d_s <= 64) {
    rc = sat::launch_lstm_mx(slots, es, w->tau, n_rows_slot, ld_slot, ids, n_bar, d, w->d_s, w->Wx,
                             w->Wh, w->b, S, WxT, st, nullptr, proj, n_proj_valid);
  } else {
    float* WhT = WxT + round_up(static_cast<int64_t>(d) * 4 * w->d_s * 4, 256) / 4;
    const int nb = 4 * w->d_s;
    transpose_kernel<<<dim3((nb * d + 255) / 256), dim3(256), 0, st>>>(w->Wx, nb, d, WxT);
    transpose_kernel<<<dim3((nb * w->d_s + 255) / 256), dim3(256), 0, st>>>(w->Wh, nb, w->d_s, WhT);
    if ((rc = sat::check_launch()) != SAT_OK) return rc;
    SlotPtrs sp;
    for (int s = 0; s < kMaxTau; ++s)
      sp.p[s] = s < w->tau ? static_cast<const float*>(slots[s]) : nullptr;
    constexpr int rows = 32;  // nodes per workgroup of lstm_kernel<128>
    const int64_t blocks = (n_bar + rows - 1) / rows;
    lstm_kernel<128><<<dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st>>>(
        sp, w->tau, n_rows_slot, ld_slot, ids, n_bar, d, WxT, WhT, w->b, S);
    rc = sat::check_launch();
  }
  return rc;
}

// The hop (second half of sat_predict): halo_out[u, :] = add[row(u), :] + Agg[u, :] Wg with
// Agg[u] = A_hat[u,u] S[n_local + u] + sum_k h_val[k] S[h_row[k]], row(u) = add_ids ? add_ids[u] : add_base + u.
sat_status run_hop(const sat_part_view* pv, const sat_predictor* w, const float* S, float* Agg,
                   const void* newest, int64_t n_rows_slot, int64_t ld_slot, const int32_t* add_ids,
                   int64_t add_base, void* halo_out, int64_t ld, int es, hipStream_t st) {
  const int d = w->d;
  sat_status rc;
  // hop, part 1: Agg[u] = A_hat[u,u] S[n_local + u] + sum_k h_val[k] S[h_row[k]]
  rc = sat::launch_spmm(pv->h_colptr, nullptr, pv->h_row, pv->h_val, S, w->d_s,
                        pv->n_local, Agg, w->d_s, pv->n_halo, w->d_s, 4, pv->h_self, pv->n_local,
                        pv->nnz_halo, st);
  if (rc != SAT_OK) return rc;
  // hop, part 2: Hbar[n_local + u, :] = newest[row(u), :] + Agg[u, :] Wg
  {
    const int64_t gx = (pv->n_halo + sat::mx::BM - 1) / sat::mx::BM;
    const dim3 grid(static_cast<unsigned>(gx),
                    static_cast<unsigned>((d + sat::mx::BN - 1) / sat::mx::BN), 1);
    const sat::mx::Operand a{Agg, static_cast<int64_t>(w->d_s), nullptr, 0};
    const sat::mx::Operand b{w->Wg, static_cast<int64_t>(d), nullptr, 0};
    const sat::mx::EpiArgs ep{0, newest, ld_slot, add_ids, add_base,
                              n_rows_slot};
    if (w->d_s <= 64)
      return sat::launch_hop_product(Agg, pv->n_halo, w->d_s, w->Wg, d, newest, ld_slot,
                                     add_ids, add_base, n_rows_slot,
                                     halo_out, ld, es, st);
    if (es == 4)
      sat::mx::gemm_kernel<4, sat::mx::Layout::KContig, false, sat::mx::Layout::MNContig, false,
                           sat::mx::kStoreAddRows, 4>
          <<<grid, dim3(256), 0, st>>>(a, b, pv->n_halo, d, w->d_s, w->d_s, halo_out, ld, ep);
    else   // fp32 aggregate and weights, bf16 residual rows and output
      sat::mx::gemm_kernel<4, sat::mx::Layout::KContig, false, sat::mx::Layout::MNContig, false,
                           sat::mx::kStoreAddRows, 2>
          <<<grid, dim3(256), 0, st>>>(a, b, pv->n_halo, d, w->d_s, w->d_s, halo_out, ld, ep);
  }
  return sat::check_launch();
}

// sat_predict; with proj != nullptr the input projections of the window's slots are read from /
// written to the caller's cache (sat_predict_cached).
sat_status predict_impl(const sat_part_view* pv, const sat_predictor* w, const void* const* slots,
                        int64_t n_rows_slot, int64_t ld_slot, const int32_t* ids, void* Hbar,
                        int64_t ld, int32_t dtype, float* const* proj, int32_t n_proj_valid,
                        void* workspace, int64_t workspace_bytes, void* stream) {
  if (!pv || !w || !slots) return SAT_EINVAL;
  if (pv->n_local < 0 || pv->n_halo < 0 || pv->nnz_halo < 0 || n_rows_slot < 0) return SAT_EINVAL;
  if (w->d < 0 || w->tau < 1) return SAT_EINVAL;
  if (dtype != SAT_F32 && dtype != SAT_BF16) return SAT_EINVAL;
  const int es = dtype == SAT_BF16 ? 2 : 4;
  if (w->tau > kMaxTau) return SAT_EUNSUPPORTED;
  const int64_t n_bar = pv->n_local + pv->n_halo;
  if (n_bar > INT32_MAX) return SAT_EUNSUPPORTED;
  const int d = w->d;
  if (pv->n_halo == 0 || d == 0) return SAT_OK;
  if (!Hbar || ld < d || ld_slot < d) return SAT_EINVAL;
  for (int s = 0; s < w->tau; ++s)
    if (!slots[s]) return SAT_EINVAL;
  if (!sat::aligned16(Hbar) || ((ld * es) % 16) != 0 || ((ld_slot * es) % 16) != 0)
    return SAT_EALIGN;
  for (int s = 0; s < w->tau; ++s)
    if (!sat::aligned16(slots[s])) return SAT_EALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const void* newest = slots[w->tau - 1];
  void* halo_out = static_cast<unsigned char*>(Hbar) + pv->n_local * ld * es;

  if (w->bypass) {
    return sat::row_gather(newest, ld_slot, halo_out, ld, ids ? ids + pv->n_local : nullptr,
                           pv->n_local, pv->n_halo, n_rows_slot, d, es, st);
  }

  if (!w->Wx || !w->Wh || !w->b || !w->Wg) return SAT_EINVAL;
  if (w->d_s != 32 && w->d_s != 64 && w->d_s != 128) return SAT_EUNSUPPORTED;
  if ((d % 4) != 0) return SAT_EUNSUPPORTED;  // Wg rows are d floats, read 16 bytes at a time
  if (es == 2 && ((d % 8) != 0 || w->d_s > 64)) return SAT_EUNSUPPORTED;  // bf16 rows: 16-byte chunks
  if (!sat::aligned16(w->Wx) || !sat::aligned16(w->Wh) || !sat::aligned16(w->Wg)) return SAT_EALIGN;
  if (!pv->h_colptr || !pv->h_self || (pv->nnz_halo > 0 && (!pv->h_row || !pv->h_val)))
    return SAT_EINVAL;
  const int64_t need = sat_predict_workspace_bytes(pv->n_local, pv->n_halo, d, w->d_s, w->tau);
  if (!workspace || workspace_bytes < need) return SAT_EWORKSPACE;
  if (!sat::aligned256(workspace)) return SAT_EALIGN;
  float* S = static_cast<float*>(workspace);
  float* Agg = S + round_up(n_bar * static_cast<int64_t>(w->d_s) * 4, 256) / 4;
  float* WxT = Agg + round_up(pv->n_halo * static_cast<int64_t>(w->d_s) * 4, 256) / 4;
  sat_status rc = run_states(w, slots, n_rows_slot, ld_slot, ids, n_bar, es, S, WxT, proj, n_proj_valid, st);
  if (rc != SAT_OK) return rc;
  return run_hop(pv, w, S, Agg, newest, n_rows_slot, ld_slot, ids ? ids + pv->n_local : nullptr, pv->n_local,
                 halo_out, ld, es, st);
}

}  // namespace

extern "C" sat_status sat_predict(const sat_part_view* pv, const sat_predictor* w,
                                  const void* const* slots, int64_t n_rows_slot,
                                  int64_t ld_slot, const int32_t* ids, void* Hbar, int64_t ld,
                                  int32_t dtype, void* workspace, int64_t workspace_bytes,
                                  void* stream) {
  return predict_impl(pv, w, slots, n_rows_slot, ld_slot, ids, Hbar, ld, dtype, nullptr, 0, workspace,
                      workspace_bytes, stream);
}

extern "C" sat_status sat_predict_cached(const sat_part_view* pv, const sat_predictor* w,
                                         const void* const* slots, int64_t n_rows_slot,
                                         int64_t ld_slot, const int32_t* ids, void* Hbar,
                                         int64_t ld, int32_t dtype, float* const* proj,
                                         int32_t n_proj_valid, void* workspace,
                                         int64_t workspace_bytes, void* stream) {
  if (!proj) return SAT_EINVAL;
  return predict_impl(pv, w, slots, n_rows_slot, ld_slot, ids, Hbar, ld, dtype, proj, n_proj_valid,
                      workspace, workspace_bytes, stream);
}

// ---- the two halves of sat_predict as calls of their own
extern "C" int64_t sat_predict_states_workspace_bytes(int32_t d, int32_t d_s) {
  if (d <= 0 || d_s <= 0) return 0;
  const int64_t w_fp32 = round_up(static_cast<int64_t>(d) * 4 * d_s * 4, 256) +
                         round_up(static_cast<int64_t>(d_s) * 4 * d_s * 4, 256);
  const int64_t w_mx = sat::lstm_mx_workspace_bytes(d, d_s);
  return w_mx > 0 ? w_mx : w_fp32;
}

extern "C" sat_status sat_predict_states(const sat_predictor* w, const void* const* slots,
                                         int64_t n_rows_slot, int64_t ld_slot, const int32_t* ids,
                                         int64_t n_nodes, int32_t dtype, float* S, void* workspace,
                                         int64_t workspace_bytes, void* stream) {
  if (!w || !slots || n_nodes < 0 || n_rows_slot < 0) return SAT_EINVAL;
  if (w->d < 0 || w->tau < 1 || w->bypass) return SAT_EINVAL;
  if (dtype != SAT_F32 && dtype != SAT_BF16) return SAT_EINVAL;
  const int es = dtype == SAT_BF16 ? 2 : 4;
  if (w->tau > kMaxTau || n_nodes > INT32_MAX) return SAT_EUNSUPPORTED;
  const int d = w->d;
  if (n_nodes == 0 || d == 0) return SAT_OK;
  if (!S || ld_slot < d) return SAT_EINVAL;
  for (int s = 0; s < w->tau; ++s)
    if (!slots[s]) return SAT_EINVAL;
  if (!w->Wx || !w->Wh || !w->b) return SAT_EINVAL;
  if (w->d_s != 32 && w->d_s != 64 && w->d_s != 128) return SAT_EUNSUPPORTED;
  if ((d % 4) != 0) return SAT_EUNSUPPORTED;
  if (es == 2 && ((d % 8) != 0 || w->d_s > 64)) return SAT_EUNSUPPORTED;
  if (((ld_slot * es) % 16) != 0 || !sat::aligned16(w->Wx) || !sat::aligned16(w->Wh) ||
      (reinterpret_cast<uintptr_t>(S) & 15u))
    return SAT_EALIGN;
  for (int s = 0; s < w->tau; ++s)
    if (!sat::aligned16(slots[s])) return SAT_EALIGN;
  const int64_t need = sat_predict_states_workspace_bytes(d, w->d_s);
  if (!workspace || workspace_bytes < need) return SAT_EWORKSPACE;
  if (!sat::aligned256(workspace)) return SAT_EALIGN;
  return run_states(w, slots, n_rows_slot, ld_slot, ids, n_nodes, es, S, static_cast<float*>(workspace),
                    nullptr, 0, static_cast<hipStream_t>(stream));
}

extern "C" int64_t sat_predict_hop_workspace_bytes(int64_t n_halo, int32_t d_s) {
  if (n_halo < 0 || d_s <= 0) return 0;
  return round_up(n_halo * static_cast<int64_t>(d_s) * 4, 256);
}

extern "C" sat_status sat_predict_hop(const sat_part_view* pv, const sat_predictor* w, const float* S,
                                      const void* newest, int64_t n_rows_newest, int64_t ld_newest,
                                      const int32_t* halo_ids, void* Hbar, int64_t ld, int32_t dtype,
                                      void* workspace, int64_t workspace_bytes, void* stream) {
  if (!pv || !w) return SAT_EINVAL;
  if (pv->n_local < 0 || pv->n_halo < 0 || pv->nnz_halo < 0 || n_rows_newest < 0) return SAT_EINVAL;
  if (w->d < 0 || w->bypass) return SAT_EINVAL;
  if (dtype != SAT_F32 && dtype != SAT_BF16) return SAT_EINVAL;
  const int es = dtype == SAT_BF16 ? 2 : 4;
  const int d = w->d;
  if (pv->n_halo == 0 || d == 0) return SAT_OK;
  if (!S || !newest || !Hbar || ld < d || ld_newest < d || !w->Wg) return SAT_EINVAL;
  if (w->d_s != 32 && w->d_s != 64 && w->d_s != 128) return SAT_EUNSUPPORTED;
  if ((d % 4) != 0) return SAT_EUNSUPPORTED;
  if (es == 2 && ((d % 8) != 0 || w->d_s > 64)) return SAT_EUNSUPPORTED;
  if (!sat::aligned16(Hbar) || !sat::aligned16(newest) || ((ld * es) % 16) != 0 ||
      ((ld_newest * es) % 16) != 0 || !sat::aligned16(w->Wg) || (reinterpret_cast<uintptr_t>(S) & 15u))
    return SAT_EALIGN;
  if (!pv->h_colptr || !pv->h_self || (pv->nnz_halo > 0 && (!pv->h_row || !pv->h_val))) return SAT_EINVAL;
  unsigned char* halo_out = static_cast<unsigned char*>(Hbar) + pv->n_local * ld * es;
  // the residual rows may BE the output rows (row u onto row u); any other overlap is refused,
  // and so is that one where the tile GEMM writes the output (d_s = 128)
  const unsigned char* nb = static_cast<const unsigned char*>(newest);
  const unsigned char* ne = nb + n_rows_newest * ld_newest * es;
  const unsigned char* oe = halo_out + pv->n_halo * ld * es;
  const bool overlap = nb < oe && halo_out < ne;
  const bool in_place = nb == halo_out && ld_newest == ld && halo_ids == nullptr;
  if (overlap && (!in_place || w->d_s > 64)) return SAT_EINVAL;
  const int64_t need = sat_predict_hop_workspace_bytes(pv->n_halo, w->d_s);
  if (!workspace || workspace_bytes < need) return SAT_EWORKSPACE;
  if (!sat::aligned256(workspace)) return SAT_EALIGN;
  return run_hop(pv, w, S, static_cast<float*>(workspace), newest, n_rows_newest, ld_newest, halo_ids, 0,
                 halo_out, ld, es, static_cast<hipStream_t>(stream));
}

// Feature transform H' = sigma((P H) W) and its backward (appendix: forward
// Z = P H W, H' = sigma(Z); backward D = G o sigma'(Z), G_W = (P H)^T D, and
// D W^T handed to the transpose aggregation).
//
// All three products run through one tile kernel on the bf16 MFMA pipe with an
// exact three-way split of the fp32 operands (fp32-equivalent accuracy at 6/16
// of the fp32 pipe's cost, see mx_tile.h):
//   forward : C = AGG * W            A KContig (AGG rows), B MNContig (W rows)
//   dAGG    : C = dZ * W^T           A KContig with relu mask, B KContig (W read transposed)
//   dW      : C = AGG^T * dZ         A MNContig (AGG rows are k), B MNContig with relu
//             mask; K = n is split over blockIdx.z and the partial tiles are
//             summed by a second kernel in a fixed order (no float atomics, so
//             results are identical from run to run).
// dZ = dH o [Hout > 0] is never written to memory: the mask is applied while the
// operand tile is loaded.
#include <atomic>

#include "dw_kernel.h"
#include "mx_tile.h"
#include "sat_internal.h"

namespace sat {
bool dense_ws_serves(int32_t K);
sat_status launch_dense_ws(const void* A, int64_t ld_a, const void* Mk, int64_t ld_m, int64_t M,
                           int32_t K, const void* W, int64_t ld_w, bool transb, int32_t N, bool relu,
                           void* out, int64_t ld_out, hipStream_t st);
bool dense_narrow_serves(int32_t K, int32_t N);
bool dense_ws32_serves(int32_t K, int64_t M);
sat_status launch_dense_ws32(const void* A, int64_t ld_a, const void* Mk, int64_t ld_m, int64_t M,
                             int32_t K, const void* W, int64_t ld_w, bool transb, int32_t N,
                             bool relu, void* out, int64_t ld_out, hipStream_t st);
sat_status launch_dense_narrow(const void* A, int64_t ld_a, int64_t M, int32_t K, const void* W,
                               int64_t ld_w, int32_t N, bool relu, void* out, int64_t ld_out,
                               hipStream_t st);
}  // namespace sat

namespace {

using namespace sat::mx;

// out[i] = sum over slices s of part[s * stride + i], in a fixed order.
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* __restrict__ part,
                                                              int64_t stride, int splits,
                                                              int64_t rows, int cols,
                                                              int64_t ld_part,
                                                              float* __restrict__ out,
                                                              int64_t ld_out) {
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= rows * cols) return;
  const int64_t r = idx / cols;
  const int c = static_cast<int>(idx - r * cols);
  const float* p = part + r * ld_part + c;
  // eight independent running sums (slices k, k+8, ...) so eight loads are in flight,
  // combined in a fixed tree: the result does not depend on timing
  float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  int k = 0;
  for (; k + 8 <= splits; k += 8) {
#pragma unroll
    for (int u = 0; u < 8; ++u) s[u] += p[(k + u) * stride];
  }
  for (int u = 0; k < splits; ++k, ++u) s[u] += p[k * stride];
  out[r * ld_out + c] = ((s[0] + s[1]) + (s[2] + s[3])) + ((s[4] + s[5]) + (s[6] + s[7]));
}

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

struct SplitPlan {
  int splits;
  int64_t k_per_split;
  int64_t ld_part;       // floats per row of a partial tile
  int64_t split_stride;  // floats per partial matrix
};

// How the reduction over the n rows of dW = AGG^T dZ is cut into node ranges: about one
// workgroup per compute unit in total (a workgroup holds its whole output tile in
// registers and fills a compute unit), every range a multiple of 32 nodes and at
// least 256 nodes long.
SplitPlan plan_dw(int64_t n, int32_t d_in, int32_t d_out) {
  SplitPlan p;
  const int bmx = d_in <= 128 ? 128 : 256, bnx = d_out <= 64 ? 64 : (d_out <= 128 ? 128 : 256);
  const int64_t tiles = ((d_in + bmx - 1) / bmx) * static_cast<int64_t>((d_out + bnx - 1) / bnx);
  int64_t want = (256 + tiles - 1) / tiles;
  int64_t max_by_k = (n + 255) / 256;
  if (max_by_k < 1) max_by_k = 1;
  int64_t s = want < max_by_k ? want : max_by_k;
  if (s < 1) s = 1;
  p.k_per_split = round_up((n + s - 1) / s, 32);
  if (p.k_per_split < 32) p.k_per_split = 32;
  p.splits = static_cast<int>((n + p.k_per_split - 1) / p.k_per_split);
  if (p.splits < 1) p.splits = 1;
  p.ld_part = round_up(d_out, 4);
  p.split_stride = static_cast<int64_t>(d_in) * p.ld_part;
  return p;
}

template <int ES, int MT, int NT, bool MASK>
sat_status launch_dw_one(const dim3 grid, const void* A, int64_t ld_a, int d_a, const void* B,
                         int64_t ld_b, int d_b, const void* M, int64_t ld_m, int64_t n,
                         const SplitPlan& p, float* part, hipStream_t s) {
  constexpr int smem = sat::dw::smem_bytes<ES, MT, NT>();
  // Dynamic LDS above 64 KB needs an opt-in per kernel AND per device. One bit per device,
  // set after the call succeeded; two threads that both find it clear both make the call,
  // which is harmless. A failed opt-in is reported here, not as a launch error later.
  static std::atomic<uint64_t> opted_in{0};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess && (dev < 0 || dev >= 64)) return SAT_EUNSUPPORTED;
  if (e == hipSuccess && !((opted_in.load(std::memory_order_acquire) >> dev) & 1ull)) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&sat::dw::dw_kernel<ES, MT, NT, MASK>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e == hipSuccess) opted_in.fetch_or(1ull << dev, std::memory_order_release);
  }
  if (e != hipSuccess) {
    sat::set_last_hip_error(e);
    return SAT_EHIP;
  }
  sat::dw::dw_kernel<ES, MT, NT, MASK><<<grid, dim3(256), smem, s>>>(
      A, ld_a, d_a, B, ld_b, d_b, M, ld_m, n, p.k_per_split, part, p.ld_part, p.split_stride);
  return sat::check_launch();
}

// part[z] = (rows of range z of A)^T (same rows of B, masked), z < p.splits
template <int ES>
sat_status launch_dw(const void* A, int64_t ld_a, int d_a, const void* B, int64_t ld_b, int d_b,
                     const void* M, int64_t ld_m, int64_t n, const SplitPlan& p, float* part,
                     hipStream_t s) {
  const bool big_m = d_a > 128, big_n = d_b > 128, small_n = d_b <= 64;
  const int bmx = big_m ? 256 : 128, bnx = big_n ? 256 : (small_n ? 64 : 128);
  const dim3 grid(static_cast<unsigned>((d_a + bmx - 1) / bmx), static_cast<unsigned>((d_b + bnx - 1) / bnx),
                  static_cast<unsigned>(p.splits));
#define SAT_DW(MT, NT)                                                                                 \
  (M ? launch_dw_one<ES, MT, NT, true>(grid, A, ld_a, d_a, B, ld_b, d_b, M, ld_m, n, p, part, s)        \
     : launch_dw_one<ES, MT, NT, false>(grid, A, ld_a, d_a, B, ld_b, d_b, M, ld_m, n, p, part, s))
  if (big_m && big_n) return SAT_DW(4, 4);
  if (big_m) return small_n ? SAT_DW(4, 1) : SAT_DW(4, 2);
  if (big_n) return SAT_DW(2, 4);
  return small_n ? SAT_DW(2, 1) : SAT_DW(2, 2);
#undef SAT_DW
}

sat_status check_mat(const void* p, int64_t rows, int64_t cols, int64_t ld, int es = 4) {
  if (rows > 0 && cols > 0) {
    if (!p || ld < cols) return SAT_EINVAL;
    if (!sat::aligned16(p) || ((ld * es) % 16) != 0) return SAT_EALIGN;
  }
  return SAT_OK;
}

// ES = bytes per element of AGG, W, H (4: fp32, 2: bf16)
template <int ES>
sat_status run_fwd(const void* AGG, int64_t ld_a, int64_t n, int32_t d_in, int32_t d_out,
                   const void* W, int64_t ld_w, int32_t act, void* H, int64_t ld_h, hipStream_t s) {
  if constexpr (ES == 2) {   // bf16: one product per operand pair, a streaming kernel serves it
    // (up to 128 output columns the tile GEMM reads A once as well and starts faster)
    if (sat::dense_ws_serves(d_in) && d_out > 128)
      return sat::launch_dense_ws(AGG, ld_a, nullptr, 0, n, d_in, W, ld_w, false, d_out,
                                  act == SAT_ACT_RELU, H, ld_h, s);
  }
  if constexpr (ES == 4) {   // fp32 onto few columns and many rows: the weights stay in LDS
    if (sat::dense_narrow_serves(d_in, d_out) && n >= 8192)
      return sat::launch_dense_narrow(AGG, ld_a, n, d_in, W, ld_w, d_out, act == SAT_ACT_RELU, H, ld_h, s);
    // fp32 onto more than 128 columns: the weights stay in registers for whole 32-row tiles,
    // the last n % 32 rows go through the tile GEMM below
    if (sat::dense_ws32_serves(d_in, n) && d_out > 128) {
      const int64_t n_ws = n & ~static_cast<int64_t>(31);
      const sat_status st = sat::launch_dense_ws32(AGG, ld_a, nullptr, 0, n_ws, d_in, W, ld_w, false, d_out,
                                                   act == SAT_ACT_RELU, H, ld_h, s);
      if (st != SAT_OK || n_ws == n) return st;
      AGG = static_cast<const float*>(AGG) + n_ws * ld_a;
      H = static_cast<float*>(H) + n_ws * ld_h;
      n -= n_ws;
    }
  }
  const int64_t gx = (n + BM - 1) / BM;
  if (gx > INT32_MAX) return SAT_EUNSUPPORTED;
  const dim3 grid(static_cast<unsigned>(gx), static_cast<unsigned>((d_out + BN - 1) / BN), 1);
  const Operand a{AGG, ld_a, nullptr, 0};
  const Operand b{W, ld_w, nullptr, 0};
  const int64_t K = d_in;
  if (act == SAT_ACT_RELU)
    gemm_kernel<ES, Layout::KContig, false, Layout::MNContig, false, kStoreRelu, ES>
        <<<grid, dim3(256), 0, s>>>(a, b, n, d_out, K, K > 0 ? K : 1, H, ld_h, EpiArgs{});
  else
    gemm_kernel<ES, Layout::KContig, false, Layout::MNContig, false, kStore, ES>
        <<<grid, dim3(256), 0, s>>>(a, b, n, d_out, K, K > 0 ? K : 1, H, ld_h, EpiArgs{});
  return sat::check_launch();
}

template <int ES>
sat_status run_bwd(const void* dH, int64_t ld_dh, const void* mask, int64_t ld_ho, const void* AGG,
                   int64_t ld_a, const void* W, int64_t ld_w, int64_t n, int32_t d_in,
                   int32_t d_out, float* dW, int64_t ld_dw, void* dAGG, int64_t ld_da,
                   float* part, hipStream_t s) {
  sat_status st;
  const bool relu = mask != nullptr;
  // dW = AGG^T dZ : reduced over the n rows, node ranges over blockIdx.z; fp32 out
  if (dW) {
    const SplitPlan p = plan_dw(n, d_in, d_out);
    if ((st = launch_dw<ES>(AGG, ld_a, d_in, dH, ld_dh, d_out, mask, ld_ho, n, p, part, s)) != SAT_OK)
      return st;
    const int64_t total = static_cast<int64_t>(d_in) * d_out;
    reduce_partials_kernel<<<dim3(static_cast<unsigned>((total + 255) / 256)), dim3(256), 0, s>>>(
        part, p.split_stride, p.splits, d_in, d_out, p.ld_part, dW, ld_dw);
    if ((st = sat::check_launch()) != SAT_OK) return st;
  }
  // dAGG = dZ W^T : M = n, N = d_in, K = d_out
  if constexpr (ES == 2) {
    if (dAGG && sat::dense_ws_serves(d_out) && d_in > 128)
      return sat::launch_dense_ws(dH, ld_dh, mask, ld_ho, n, d_out, W, ld_w, true, d_in, false, dAGG,
                                  ld_da, s);
  }
  if constexpr (ES == 4) {
    if (dAGG && sat::dense_ws32_serves(d_out, n) && d_in > 128) {
      const int64_t n_ws = n & ~static_cast<int64_t>(31);
      st = sat::launch_dense_ws32(dH, ld_dh, mask, ld_ho, n_ws, d_out, W, ld_w, true, d_in, false, dAGG,
                                  ld_da, s);
      if (st != SAT_OK || n_ws == n) return st;
      dH = static_cast<const float*>(dH) + n_ws * ld_dh;
      if (mask) mask = static_cast<const float*>(mask) + n_ws * ld_ho;
      dAGG = static_cast<float*>(dAGG) + n_ws * ld_da;
      n -= n_ws;
    }
  }
  if (dAGG) {
    const int64_t gx = (n + BM - 1) / BM;
    if (gx > INT32_MAX) return SAT_EUNSUPPORTED;
    const dim3 grid(static_cast<unsigned>(gx), static_cast<unsigned>((d_in + BN - 1) / BN), 1);
    const Operand a{dH, ld_dh, mask, ld_ho};
    const Operand b{W, ld_w, nullptr, 0};
    const int64_t K = d_out;
    if (relu)
      gemm_kernel<ES, Layout::KContig, true, Layout::KContig, false, kStore, ES>
          <<<grid, dim3(256), 0, s>>>(a, b, n, d_in, K, K, dAGG, ld_da, EpiArgs{});
    else
      gemm_kernel<ES, Layout::KContig, false, Layout::KContig, false, kStore, ES>
          <<<grid, dim3(256), 0, s>>>(a, b, n, d_in, K, K, dAGG, ld_da, EpiArgs{});
    if ((st = sat::check_launch()) != SAT_OK) return st;
  }
  return SAT_OK;
}

}  // namespace

extern "C" sat_status sat_dense_fwd(const void* AGG, int64_t ld_a, int64_t n, int32_t d_in,
                                    int32_t d_out, const void* W, int64_t ld_w, int32_t act,
                                    int32_t dtype, void* H, int64_t ld_h, void* stream) {
  if (n < 0 || d_in < 0 || d_out < 0) return SAT_EINVAL;
  if (act != SAT_ACT_IDENTITY && act != SAT_ACT_RELU) return SAT_EINVAL;
  if (dtype != SAT_F32 && dtype != SAT_BF16) return SAT_EINVAL;
  const int es = dtype == SAT_BF16 ? 2 : 4;
  sat_status st;
  if ((st = check_mat(AGG, n, d_in, ld_a, es)) != SAT_OK) return st;
  if ((st = check_mat(W, d_in, d_out, ld_w, es)) != SAT_OK) return st;
  if ((st = check_mat(H, n, d_out, ld_h, es)) != SAT_OK) return st;
  if (n == 0 || d_out == 0) return SAT_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  return es == 2 ? run_fwd<2>(AGG, ld_a, n, d_in, d_out, W, ld_w, act, H, ld_h, s)
                 : run_fwd<4>(AGG, ld_a, n, d_in, d_out, W, ld_w, act, H, ld_h, s);
}

extern "C" int64_t sat_dense_bwd_workspace_bytes(int64_t n, int32_t d_in, int32_t d_out) {
  if (n <= 0 || d_in <= 0 || d_out <= 0) return 0;
  const SplitPlan p = plan_dw(n, d_in, d_out);
  return static_cast<int64_t>(p.splits) * p.split_stride * static_cast<int64_t>(sizeof(float));
}

extern "C" sat_status sat_dense_bwd(const void* dH, int64_t ld_dh, const void* Hout,
                                    int64_t ld_ho, const void* AGG, int64_t ld_a, const void* W,
                                    int64_t ld_w, int64_t n, int32_t d_in, int32_t d_out,
                                    int32_t act, int32_t dtype, float* dW, int64_t ld_dw,
                                    void* dAGG, int64_t ld_da, void* workspace,
                                    int64_t workspace_bytes, void* stream) {
  if (n < 0 || d_in < 0 || d_out < 0) return SAT_EINVAL;
  if (act != SAT_ACT_IDENTITY && act != SAT_ACT_RELU) return SAT_EINVAL;
  if (dtype != SAT_F32 && dtype != SAT_BF16) return SAT_EINVAL;
  const int es = dtype == SAT_BF16 ? 2 : 4;
  sat_status st;
  if ((st = check_mat(dH, n, d_out, ld_dh, es)) != SAT_OK) return st;
  if (act == SAT_ACT_RELU && (st = check_mat(Hout, n, d_out, ld_ho, es)) != SAT_OK) return st;
  if (dW && (st = check_mat(AGG, n, d_in, ld_a, es)) != SAT_OK) return st;
  if ((st = check_mat(W, d_in, d_out, ld_w, es)) != SAT_OK) return st;
  if (dW && (st = check_mat(dW, d_in, d_out, ld_dw, 4)) != SAT_OK) return st;
  if (dAGG && (st = check_mat(dAGG, n, d_in, ld_da, es)) != SAT_OK) return st;
  if (d_in == 0 || d_out == 0) return SAT_OK;
  const int64_t need = dW ? sat_dense_bwd_workspace_bytes(n, d_in, d_out) : 0;
  if (need > 0 && (!workspace || workspace_bytes < need)) return SAT_EWORKSPACE;
  if (need > 0 && !sat::aligned256(workspace)) return SAT_EALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (n == 0) {
    if (!dW) return SAT_OK;
    // empty reduction: dW = 0 (the reduce kernel with zero slices writes zeros)
    const int64_t total = static_cast<int64_t>(d_in) * d_out;
    reduce_partials_kernel<<<dim3(static_cast<unsigned>((total + 255) / 256)), dim3(256), 0, s>>>(
        dW, 0, 0, d_in, d_out, ld_dw, dW, ld_dw);
    return sat::check_launch();
  }
  const void* mask = act == SAT_ACT_RELU ? Hout : nullptr;
  float* part = static_cast<float*>(workspace);
  return es == 2 ? run_bwd<2>(dH, ld_dh, mask, ld_ho, AGG, ld_a, W, ld_w, n, d_in, d_out, dW, ld_dw,
                              dAGG, ld_da, part, s)
                 : run_bwd<4>(dH, ld_dh, mask, ld_ho, AGG, ld_a, W, ld_w, n, d_in, d_out, dW, ld_dw,
                              dAGG, ld_da, part, s);
}

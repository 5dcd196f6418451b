// Training of the embedding predictor on one partition (Eq. 11, and Eq. 12
// through the per-node weights): loss and gradients of one hidden layer's
// predictor, and the plain gradient step of Alg. 1's "embedding predictor
// update".
//
// The partition supervises the predictor where it knows the truth, on its local
// nodes: pred[v] = newest[v] + (row v of [P_in | P_out] times S) Wg against the
// fresh embedding the forward pass of this step produced for v;
// loss = sum_v weight[v] |pred[v] - target[v]|^2 / (d sum_v weight[v]).
//
// The call is a sequence of kernels the library already has, plus four small
// element-wise ones defined here:
//   forward   LSTM over all nodes of the partition and its halo with every step's
//             gates, cell and hidden state kept (lstm_mx.hip; for d_s = 128, which that
//             kernel does not take, each step as two products of the feature transform
//             and an element-wise step defined here), aggregation of S
//             over the local rows (spmm.hip), product with Wg plus the newest
//             rows (tile GEMM, mx_tile.h), weighted squared error (here);
//   backward  dWg and the gradient of the aggregate (the feature transform's
//             backward, dense.hip), its transpose aggregation to all nodes
//             including the halo rows (spmm.hip), then per time step, newest
//             first: gate gradients (here), dWx and dWh as products reduced over
//             the nodes (dense.hip), db as column sums (here), and the gradient
//             of the previous hidden state (the feature transform, dense.hip).
// Every reduction over nodes runs in a fixed order: results are run-to-run
// identical. With bfloat16 storage (history tables and targets) everything computed here
// stays fp32: the window's rows are widened on the way in.
#include <math.h>

#include "mx_tile.h"
#include "sat_internal.h"

namespace sat {
sat_status row_gather(const void* src, int64_t ld_src, void* dst, int64_t ld_dst,
                      const int32_t* ids, int64_t id_base, int64_t n, int64_t n_src_rows,
                      int32_t d, int es, hipStream_t stream);
sat_status launch_spmm(const int64_t* rowptr, const int64_t* row_end, const int32_t* col,
                       const float* val, const void* X, int64_t ld_x, int64_t n_x_rows, void* Y,
                       int64_t ld_y, int64_t n_rows, int32_t d, int es, const float* self_val,
                       int64_t self_off, int64_t total_entries, hipStream_t stream);
int64_t lstm_mx_workspace_bytes(int32_t d, int32_t d_s);
sat_status launch_lstm_mx(const void* const* slot_ptrs, int es_x, int tau, int64_t n_rows_slot,
                          int64_t ld_slot, const int32_t* ids, int64_t n_nodes, int32_t d,
                          int32_t d_s, const float* Wx, const float* Wh, const float* b, float* S,
                          void* ws, hipStream_t st, float* save, float* const* proj = nullptr,
                          int n_proj_valid = 0);
sat_status launch_hop_product(const float* Agg, int64_t M, int32_t ds, const float* Wg, int32_t d,
                              const void* add, int64_t ld_add, const int32_t* add_ids,
                              int64_t add_base, int64_t add_rows, void* out, int64_t ld_out, int eso,
                              hipStream_t st);
}  // namespace sat

namespace {

constexpr int kMaxTau = 8;
constexpr int kRedBlocks = 512;   // first-stage blocks of the fixed-order reductions

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// block-wide sum in a fixed order (tree over the thread index); result in thread 0
__device__ __forceinline__ float block_sum_256(float v, float* sh) {
  sh[threadIdx.x] = v;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if (threadIdx.x < off) sh[threadIdx.x] += sh[threadIdx.x + off];
    __syncthreads();
  }
  return sh[0];
}

__global__ __launch_bounds__(256) void fill_kernel(float* p, int64_t n, float v) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i < n) p[i] = v;
}

// y[r, 0:cols) += a * x[r, 0:cols)
__global__ __launch_bounds__(256) void axpy_rows_kernel(float* y, int64_t ld_y, const float* x,
                                                        int64_t ld_x, int rows, int cols, float a) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i >= static_cast<int64_t>(rows) * cols) return;
  const int r = static_cast<int>(i / cols), c = static_cast<int>(i - static_cast<int64_t>(r) * cols);
  y[r * ld_y + c] += a * x[r * ld_x + c];
}

// part[b] = sum of w over block b's contiguous share (weights of the mini-batch)
__global__ __launch_bounds__(256) void weight_sum_kernel(const float* __restrict__ w, int64_t n,
                                                         float* __restrict__ part) {
  __shared__ float sh[256];
  const int64_t per = (n + gridDim.x - 1) / gridDim.x;
  const int64_t lo = blockIdx.x * per, hi = lo + per < n ? lo + per : n;
  float acc = 0.f;
  for (int64_t i = lo + threadIdx.x; i < hi; i += 256) acc += w[i];
  const float s = block_sum_256(acc, sh);
  if (threadIdx.x == 0) part[blockIdx.x] = s;
}

// out[0] = sum of part[0..n) in index order, times scale (or divided by *denominator)
__global__ __launch_bounds__(256) void finish_sum_kernel(const float* __restrict__ part, int n,
                                                         float scale, const float* denominator,
                                                         float* __restrict__ out) {
  __shared__ float sh[256];
  float acc = 0.f;
  for (int i = threadIdx.x; i < n; i += 256) acc += part[i];
  const float s = block_sum_256(acc, sh);
  if (threadIdx.x == 0) out[0] = denominator ? s * scale / denominator[0] : s * scale;
}

// element i of a matrix stored as fp32 (ES = 4) or bfloat16 (ES = 2)
template <int ES>
__device__ __forceinline__ float elem(const void* p, int64_t i) {
  if constexpr (ES == 4) {
    return static_cast<const float*>(p)[i];
  } else {
    return __builtin_bit_cast(float, static_cast<uint32_t>(static_cast<const uint16_t*>(p)[i]) << 16);
  }
}

// P [n, ld_p] holds pred on entry and d loss / d pred on exit:
//   diff = pred - target;  P = 2 w diff / (d wsum);  part[b] = sum w diff^2 over the block's rows
// wsum_dev: device scalar sum of the weights (weights given) or nullptr (wsum = n).
// T (and N) hold elements of ES bytes. If N != nullptr the residual term has not been added
// to P yet: pred = P + N[row(r)], row(r) = ids ? ids[r] : r (rows outside [0, n_rows_n) add 0).
template <int ES>
__global__ __launch_bounds__(256) void sq_error_kernel(float* __restrict__ P, int64_t ld_p,
                                                       const void* __restrict__ T, int64_t ld_t,
                                                       const void* __restrict__ N, int64_t ld_n,
                                                       const int32_t* __restrict__ ids,
                                                       int64_t n_rows_n,
                                                       const float* __restrict__ w,
                                                       const float* __restrict__ wsum_dev, int64_t n,
                                                       int d, float* __restrict__ part) {
  __shared__ float sh[256];
  const float wsum = wsum_dev ? wsum_dev[0] : static_cast<float>(n);
  const float k = wsum > 0.f ? 2.0f / (static_cast<float>(d) * wsum) : 0.f;
  const int64_t per = (n + gridDim.x - 1) / gridDim.x;
  const int64_t lo = blockIdx.x * per, hi = lo + per < n ? lo + per : n;
  float acc = 0.f;
  for (int64_t r = lo; r < hi; ++r) {
    const float wr = w ? w[r] : 1.0f;
    int64_t nr = -1;
    if (N) {
      nr = ids ? static_cast<int64_t>(ids[r]) : r;
      if (nr < 0 || nr >= n_rows_n) nr = -1;
    }
    for (int c = threadIdx.x; c < d; c += 256) {
      float pred = P[r * ld_p + c];
      if (nr >= 0) pred += elem<ES>(N, nr * ld_n + c);
      const float diff = pred - elem<ES>(T, r * ld_t + c);
      acc += wr * diff * diff;
      P[r * ld_p + c] = k * wr * diff;
    }
  }
  const float s = block_sum_256(acc, sh);
  if (threadIdx.x == 0) part[blockIdx.x] = s;
}

// dst [n, ld_dst] fp32 = rows (ids ? ids[r] : r) of a bfloat16 table, widened (rows outside the
// table: zeros)
__global__ __launch_bounds__(256) void widen_rows_kernel(const uint16_t* __restrict__ src, int64_t ld_src,
                                                         const int32_t* __restrict__ ids,
                                                         int64_t n_src_rows, float* __restrict__ dst,
                                                         int64_t ld_dst, int64_t n, int d) {
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  const int pairs = d / 2;                       // d % 8 == 0 here
  if (idx >= n * pairs) return;
  const int64_t r = idx / pairs;
  const int c = 2 * static_cast<int>(idx - r * pairs);
  int64_t sr = ids ? static_cast<int64_t>(ids[r]) : r;
  uint32_t wv = 0;
  if (sr >= 0 && sr < n_src_rows) wv = *reinterpret_cast<const uint32_t*>(src + sr * ld_src + c);
  float2 o;
  o.x = __builtin_bit_cast(float, wv << 16);
  o.y = __builtin_bit_cast(float, wv & 0xffff0000u);
  *reinterpret_cast<float2*>(dst + r * ld_dst + c) = o;
}

// One time step of the LSTM's back-propagation, element-wise over (node, hidden unit).
// rec: this step's saved record [n, 6 ds] = activated i, f, g, o, then c_s, h_s;
// c_prev: the previous step's record (nullptr at the first step: c_0 = 0).
// dh [n, ds]: gradient of h_s. dc [n, ds]: gradient of c_s arriving from the later step,
// replaced by the gradient of c_{s-1}. da [n, 4 ds]: gradient of the gate pre-activations.
__global__ __launch_bounds__(256) void lstm_bwd_gates_kernel(const float* __restrict__ rec,
                                                             const float* __restrict__ rec_prev,
                                                             const float* __restrict__ dh,
                                                             float* __restrict__ dc,
                                                             float* __restrict__ da, int64_t n,
                                                             int ds) {
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= n * ds) return;
  const int64_t node = idx / ds;
  const int u = static_cast<int>(idx - node * ds);
  const float* r = rec + node * (6 * ds) + u;
  const float gi = r[0], gf = r[ds], gg = r[2 * ds], go = r[3 * ds], c = r[4 * ds];
  const float cp = rec_prev ? rec_prev[node * (6 * ds) + 4 * ds + u] : 0.f;
  const float tc = tanhf(c);
  const float g_h = dh[idx];
  const float g_o = g_h * tc;
  const float g_c = dc[idx] + g_h * go * (1.0f - tc * tc);
  float* a = da + node * (4 * ds) + u;
  a[0] = g_c * gg * gi * (1.0f - gi);
  a[ds] = g_c * cp * gf * (1.0f - gf);
  a[2 * ds] = g_c * gi * (1.0f - gg * gg);
  a[3 * ds] = g_o * go * (1.0f - go);
  dc[idx] = g_c * gf;
}

// out [C, R] = in [R, C] transposed
__global__ __launch_bounds__(256) void transpose_kernel(const float* __restrict__ in, int R, int C,
                                                        float* __restrict__ out) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= R * C) return;
  const int r = i / C, c = i - r * C;
  out[static_cast<int64_t>(c) * R + r] = in[i];
}

// One time step of the LSTM with its record kept, element-wise over (node, hidden unit):
// pre-activations a = px + ph + b (px = x_s Wx^T, ph = h_{s-1} Wh^T, both [n, 4 ds]; ph
// nullptr at the first step, where h_0 = c_0 = 0), gates i, f, o = sigmoid, g = tanh,
// c_s = f c_{s-1} + i g, h_s = o tanh(c_s); rec [n, 6 ds] = i, f, g, o, c_s, h_s.
__global__ __launch_bounds__(256) void lstm_step_save_kernel(const float* __restrict__ px,
                                                             const float* __restrict__ ph,
                                                             const float* __restrict__ bias,
                                                             const float* __restrict__ rec_prev,
                                                             float* __restrict__ rec, int64_t n,
                                                             int ds) {
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= n * ds) return;
  const int64_t node = idx / ds;
  const int u = static_cast<int>(idx - node * ds);
  const int64_t a0 = node * (4 * ds) + u;
  float a[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    a[g] = px[a0 + g * ds];
    if (ph) a[g] += ph[a0 + g * ds];
    a[g] += bias[g * ds + u];
  }
  const float gi = 1.0f / (1.0f + expf(-a[0]));
  const float gf = 1.0f / (1.0f + expf(-a[1]));
  const float gg = tanhf(a[2]);
  const float go = 1.0f / (1.0f + expf(-a[3]));
  const float cp = rec_prev ? rec_prev[node * (6 * ds) + 4 * ds + u] : 0.f;
  const float c = gf * cp + gi * gg;
  float* r = rec + node * (6 * ds) + u;
  r[0] = gi;
  r[ds] = gf;
  r[2 * ds] = gg;
  r[3 * ds] = go;
  r[4 * ds] = c;
  r[5 * ds] = go * tanhf(c);
}

// part[b][c] = sum over block b's rows of A[r, c]   (A [n, cols]; blockIdx.y: block of 256 columns)
__global__ __launch_bounds__(256) void col_sum_kernel(const float* __restrict__ A, int64_t n,
                                                      int cols, float* __restrict__ part) {
  const int64_t per = (n + gridDim.x - 1) / gridDim.x;
  const int64_t lo = blockIdx.x * per, hi = lo + per < n ? lo + per : n;
  const int c = blockIdx.y * 256 + threadIdx.x;
  if (c >= cols) return;
  // eight rows at a time, each into its own partial sum: eight loads in flight per thread
  float a[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) a[u] = 0.f;
  int64_t r = lo;
  for (; r + 8 <= hi; r += 8) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = A[(r + u) * cols + c];
#pragma unroll
    for (int u = 0; u < 8; ++u) a[u] += v[u];
  }
  for (; r < hi; ++r) a[0] += A[r * cols + c];
  part[static_cast<int64_t>(blockIdx.x) * cols + c] =
      ((a[0] + a[1]) + (a[2] + a[3])) + ((a[4] + a[5]) + (a[6] + a[7]));
}
// out[c] += sum over b of part[b][c], b ascending
__global__ __launch_bounds__(256) void col_sum_finish_kernel(const float* __restrict__ part,
                                                             int blocks, int cols,
                                                             float* __restrict__ out) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= cols) return;
  float acc = 0.f;
  for (int b = 0; b < blocks; ++b) acc += part[static_cast<int64_t>(b) * cols + c];
  out[c] += acc;
}

__global__ __launch_bounds__(256) void sgd_kernel(float* __restrict__ p, const float* __restrict__ g,
                                                  int64_t n, float lr) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i < n) p[i] -= lr * g[i];
}

struct Plan {   // byte offsets into the workspace, all multiples of 256
  int64_t S, save, wsplit, aggS, pred, part, wsum, daggS, dh0, dh1, dc, da, xwin, tmpW, dws, wT, ph, total;
};

Plan plan(int64_t n_l, int64_t n_h, int32_t d, int32_t ds, int32_t tau) {
  const int64_t n_bar = n_l + n_h;
  Plan L{};
  int64_t off = 0;
  auto take = [&](int64_t bytes) {
    const int64_t at = off;
    off += round_up(bytes > 0 ? bytes : 1, 256);
    return at;
  };
  L.S = take(n_bar * ds * 4);
  L.save = take(static_cast<int64_t>(tau) * n_bar * 6 * ds * 4);
  L.wsplit = take(sat::lstm_mx_workspace_bytes(d, ds));
  L.aggS = take(n_l * ds * 4);
  L.pred = take(n_l * static_cast<int64_t>(d) * 4);
  L.part = take(static_cast<int64_t>(kRedBlocks) * 4 * ds * 4);
  L.wsum = take(256);
  L.daggS = take(n_l * ds * 4);
  L.dh0 = take(n_bar * ds * 4);
  L.dh1 = take(n_bar * ds * 4);
  L.dc = take(n_bar * ds * 4);
  L.da = take(n_bar * 4 * ds * 4);
  L.xwin = take(n_bar * static_cast<int64_t>(d) * 4);
  L.tmpW = take(static_cast<int64_t>(4 * ds) * (d > ds ? d : ds) * 4);
  int64_t dws = sat_dense_bwd_workspace_bytes(n_bar, 4 * ds, d);
  const int64_t w2 = sat_dense_bwd_workspace_bytes(n_bar, 4 * ds, ds);
  const int64_t w3 = sat_dense_bwd_workspace_bytes(n_l, ds, d);
  if (w2 > dws) dws = w2;
  if (w3 > dws) dws = w3;
  L.dws = take(dws);
  // d_s = 128: transposed copies of Wx and Wh, and the recurrent part of a step's pre-activations
  L.wT = take(ds > 64 ? static_cast<int64_t>(4 * ds) * (d + ds) * 4 : 0);
  L.ph = take(ds > 64 ? n_bar * 4 * ds * 4 : 0);
  L.total = off;
  return L;
}

inline dim3 blocks_for(int64_t n) { return dim3(static_cast<unsigned>((n + 255) / 256)); }

}  // namespace

extern "C" int64_t sat_predictor_train_workspace_bytes(int64_t n_local, int64_t n_halo, int32_t d,
                                                       int32_t d_s, int32_t tau) {
  if (n_local < 0 || n_halo < 0 || d <= 0 || d_s <= 0 || tau < 1) return 0;
  return plan(n_local, n_halo, d, d_s, tau).total;
}

extern "C" sat_status sat_predictor_grad(const sat_part_view* pv, const sat_predictor* w,
                                         const void* const* slots, int64_t n_rows_slot,
                                         int64_t ld_slot, const int32_t* ids, const void* target,
                                         int64_t ld_target, const float* weight, int32_t dtype,
                                         float* dWx, float* dWh, float* db, float* dWg,
                                         float* loss, void* workspace, int64_t workspace_bytes,
                                         void* stream) {
  if (!pv || !w || !slots) return SAT_EINVAL;
  if (pv->n_local < 0 || pv->n_halo < 0 || pv->nnz < 0 || pv->nnz_halo < 0 || n_rows_slot < 0)
    return SAT_EINVAL;
  if (dtype != SAT_F32 && dtype != SAT_BF16) return SAT_EINVAL;
  if (w->d <= 0 || w->tau < 1 || w->bypass) return SAT_EINVAL;
  if (w->tau > kMaxTau) return SAT_EUNSUPPORTED;
  if (w->d_s != 32 && w->d_s != 64 && w->d_s != 128) return SAT_EUNSUPPORTED;
  const int d = w->d, ds = w->d_s, tau = w->tau;
  const int es = dtype == SAT_BF16 ? 2 : 4;
  if (ds > 64 && es == 2) return SAT_EUNSUPPORTED;   // (as in sat_predict)
  if ((d % (16 / es)) != 0) return SAT_EUNSUPPORTED;
  const int64_t n_l = pv->n_local, n_h = pv->n_halo, n_bar = n_l + n_h;
  if (n_bar > INT32_MAX) return SAT_EUNSUPPORTED;
  if (!w->Wx || !w->Wh || !w->b || !w->Wg || !dWx || !dWh || !db || !dWg || !loss) return SAT_EINVAL;
  if (n_l == 0) return SAT_EINVAL;   // nothing to supervise
  if (!target || ld_target < d || ld_slot < d) return SAT_EINVAL;
  for (int s = 0; s < tau; ++s)
    if (!slots[s]) return SAT_EINVAL;
  if (!pv->rowptr || !pv->split || !pv->col || !pv->val) return SAT_EINVAL;
  if (n_h > 0 && (!pv->h_colptr || (pv->nnz_halo > 0 && (!pv->h_row || !pv->h_val)))) return SAT_EINVAL;
  if (!sat::aligned16(target) || (ld_target % (16 / es)) != 0 || (ld_slot % (16 / es)) != 0)
    return SAT_EALIGN;
  for (int s = 0; s < tau; ++s)
    if (!sat::aligned16(slots[s])) return SAT_EALIGN;
  if (!sat::aligned16(w->Wx) || !sat::aligned16(w->Wh) || !sat::aligned16(w->Wg) ||
      !sat::aligned16(dWx) || !sat::aligned16(dWh) || !sat::aligned16(dWg))
    return SAT_EALIGN;
  const Plan L = plan(n_l, n_h, d, ds, tau);
  if (!workspace || workspace_bytes < L.total) return SAT_EWORKSPACE;
  if (!sat::aligned256(workspace)) return SAT_EALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  unsigned char* base = static_cast<unsigned char*>(workspace);
  auto f = [&](int64_t off) { return reinterpret_cast<float*>(base + off); };
  float *S = f(L.S), *save = f(L.save), *aggS = f(L.aggS), *pred = f(L.pred), *part = f(L.part),
        *wsum = f(L.wsum), *daggS = f(L.daggS), *dc = f(L.dc), *da = f(L.da), *xwin = f(L.xwin),
        *tmpW = f(L.tmpW);
  float* dh[2] = {f(L.dh0), f(L.dh1)};
  void* dws = base + L.dws;
  const int64_t dws_bytes = L.wT - L.dws;
  const int64_t rec = 6 * static_cast<int64_t>(ds);
  sat_status rc;

  if (!ids && n_rows_slot < n_bar) return SAT_EINVAL;
  // ---- forward
  const float* Sp = S;        // the last hidden states, ld_S floats per node
  int64_t ld_S = ds;
  if (ds <= 64) {
    rc = sat::launch_lstm_mx(slots, es, tau, n_rows_slot, ld_slot, ids, n_bar, d, ds, w->Wx, w->Wh, w->b,
                             S, base + L.wsplit, st, save);
    if (rc != SAT_OK) return rc;
  } else {
    float* WxT = f(L.wT);
    float* WhT = WxT + static_cast<int64_t>(4 * ds) * d;
    float* ph = f(L.ph);
    transpose_kernel<<<blocks_for(static_cast<int64_t>(4 * ds) * d), dim3(256), 0, st>>>(w->Wx, 4 * ds, d, WxT);
    transpose_kernel<<<blocks_for(static_cast<int64_t>(4 * ds) * ds), dim3(256), 0, st>>>(w->Wh, 4 * ds, ds, WhT);
    if ((rc = sat::check_launch()) != SAT_OK) return rc;
    for (int s = 0; s < tau; ++s) {
      const void* xs = slots[s];
      int64_t ld_x = ld_slot;
      if (ids) {
        rc = sat::row_gather(slots[s], ld_slot, xwin, d, ids, 0, n_bar, n_rows_slot, d, 4, st);
        if (rc != SAT_OK) return rc;
        xs = xwin;
        ld_x = d;
      }
      float* rec_s = save + static_cast<int64_t>(s) * n_bar * rec;
      const float* rec_p = s > 0 ? save + static_cast<int64_t>(s - 1) * n_bar * rec : nullptr;
      rc = sat_dense_fwd(xs, ld_x, n_bar, d, 4 * ds, WxT, 4 * ds, SAT_ACT_IDENTITY, SAT_F32, da, 4 * ds,
                         stream);
      if (rc != SAT_OK) return rc;
      if (s > 0) {
        rc = sat_dense_fwd(rec_p + 5 * ds, rec, n_bar, ds, 4 * ds, WhT, 4 * ds, SAT_ACT_IDENTITY, SAT_F32,
                           ph, 4 * ds, stream);
        if (rc != SAT_OK) return rc;
      }
      lstm_step_save_kernel<<<blocks_for(n_bar * ds), dim3(256), 0, st>>>(da, s > 0 ? ph : nullptr, w->b,
                                                                          rec_p, rec_s, n_bar, ds);
      if ((rc = sat::check_launch()) != SAT_OK) return rc;
    }
    Sp = save + static_cast<int64_t>(tau - 1) * n_bar * rec + 5 * ds;
    ld_S = rec;
  }
  rc = sat::launch_spmm(pv->rowptr, nullptr, pv->col, pv->val, Sp, ld_S, n_bar, aggS, ds, n_l, ds, 4,
                        nullptr, 0, pv->nnz, st);
  if (rc != SAT_OK) return rc;
  const bool fused_add = es == 4 && ds <= 64;
  if (fused_add) {   // pred = newest rows + aggS Wg in one kernel
    rc = sat::launch_hop_product(aggS, n_l, ds, w->Wg, d, slots[tau - 1], ld_slot, ids, 0, n_rows_slot,
                                 pred, d, 4, st);
  } else {         // bf16 tables, d_s = 128: the product alone (fp32), the newest rows are added with the error
    rc = sat_dense_fwd(aggS, ds, n_l, ds, d, w->Wg, d, SAT_ACT_IDENTITY, SAT_F32, pred, d, stream);
  }
  if (rc != SAT_OK) return rc;
  const float* wsum_dev = nullptr;
  if (weight) {
    weight_sum_kernel<<<dim3(kRedBlocks), dim3(256), 0, st>>>(weight, n_l, part);
    finish_sum_kernel<<<dim3(1), dim3(256), 0, st>>>(part, kRedBlocks, 1.0f, nullptr, wsum);
    wsum_dev = wsum;
  }
  if (fused_add)
    sq_error_kernel<4><<<dim3(kRedBlocks), dim3(256), 0, st>>>(pred, d, target, ld_target, nullptr, 0, nullptr,
                                                               0, weight, wsum_dev, n_l, d, part);
  else if (es == 4)
    sq_error_kernel<4><<<dim3(kRedBlocks), dim3(256), 0, st>>>(pred, d, target, ld_target, slots[tau - 1],
                                                               ld_slot, ids, n_rows_slot, weight, wsum_dev,
                                                               n_l, d, part);
  else
    sq_error_kernel<2><<<dim3(kRedBlocks), dim3(256), 0, st>>>(pred, d, target, ld_target, slots[tau - 1],
                                                               ld_slot, ids, n_rows_slot, weight, wsum_dev,
                                                               n_l, d, part);
  if (weight)
    finish_sum_kernel<<<dim3(1), dim3(256), 0, st>>>(part, kRedBlocks, 1.0f / d, wsum, loss);
  else
    finish_sum_kernel<<<dim3(1), dim3(256), 0, st>>>(part, kRedBlocks,
                                                     1.0f / (static_cast<float>(d) * n_l), nullptr, loss);
  if ((rc = sat::check_launch()) != SAT_OK) return rc;

  // ---- backward through the hop: dWg = aggS^T dpred, daggS = dpred Wg^T, dS = [P_in | P_out]^T daggS
  rc = sat_dense_bwd(pred, d, nullptr, 0, aggS, ds, w->Wg, d, n_l, ds, d, SAT_ACT_IDENTITY, SAT_F32,
                     dWg, d, daggS, ds, dws, dws_bytes, stream);
  if (rc != SAT_OK) return rc;
  rc = sat_spmm_bwd(pv, daggS, ds, ds, SAT_F32, dh[0], ds, n_h > 0 ? dh[0] + n_l * ds : nullptr, ds,
                    nullptr, 0, stream);
  if (rc != SAT_OK) return rc;

  // ---- backward through the LSTM, newest step first
  fill_kernel<<<blocks_for(n_bar * ds), dim3(256), 0, st>>>(dc, n_bar * ds, 0.f);
  fill_kernel<<<blocks_for(static_cast<int64_t>(4 * ds) * d), dim3(256), 0, st>>>(dWx, static_cast<int64_t>(4 * ds) * d, 0.f);
  fill_kernel<<<blocks_for(static_cast<int64_t>(4 * ds) * ds), dim3(256), 0, st>>>(dWh, static_cast<int64_t>(4 * ds) * ds, 0.f);
  fill_kernel<<<blocks_for(4 * ds), dim3(256), 0, st>>>(db, 4 * ds, 0.f);
  if ((rc = sat::check_launch()) != SAT_OK) return rc;
  int cur = 0;
  for (int s = tau - 1; s >= 0; --s) {
    const float* rec_s = save + static_cast<int64_t>(s) * n_bar * rec;
    const float* rec_p = s > 0 ? save + static_cast<int64_t>(s - 1) * n_bar * rec : nullptr;
    lstm_bwd_gates_kernel<<<blocks_for(n_bar * ds), dim3(256), 0, st>>>(rec_s, rec_p, dh[cur], dc, da,
                                                                        n_bar, ds);
    if ((rc = sat::check_launch()) != SAT_OK) return rc;
    // dWx += da^T x_s  (x_s: the slot's rows of the partition's nodes, local then halo)
    const void* xs = slots[s];
    int64_t ld_x = ld_slot;
    if (es == 2) {   // the products below are fp32: widen the window's rows on the way
      widen_rows_kernel<<<blocks_for(n_bar * (d / 2)), dim3(256), 0, st>>>(
          static_cast<const uint16_t*>(slots[s]), ld_slot, ids, n_rows_slot, xwin, d, n_bar, d);
      if ((rc = sat::check_launch()) != SAT_OK) return rc;
      xs = xwin;
      ld_x = d;
    } else if (ids) {
      rc = sat::row_gather(slots[s], ld_slot, xwin, d, ids, 0, n_bar, n_rows_slot, d, 4, st);
      if (rc != SAT_OK) return rc;
      xs = xwin;
      ld_x = d;
    }
    rc = sat_dense_bwd(xs, ld_x, nullptr, 0, da, 4 * ds, w->Wx, d, n_bar, 4 * ds, d, SAT_ACT_IDENTITY,
                       SAT_F32, tmpW, d, nullptr, 0, dws, dws_bytes, stream);
    if (rc != SAT_OK) return rc;
    axpy_rows_kernel<<<blocks_for(static_cast<int64_t>(4 * ds) * d), dim3(256), 0, st>>>(
        dWx, d, tmpW, d, 4 * ds, d, 1.0f);
    col_sum_kernel<<<dim3(kRedBlocks, (4 * ds + 255) / 256), dim3(256), 0, st>>>(da, n_bar, 4 * ds, part);
    col_sum_finish_kernel<<<dim3((4 * ds + 255) / 256), dim3(256), 0, st>>>(part, kRedBlocks, 4 * ds, db);
    if ((rc = sat::check_launch()) != SAT_OK) return rc;
    if (s > 0) {
      // dWh += da^T h_{s-1};  dh_{s-1} = da Wh
      rc = sat_dense_bwd(rec_p + 5 * ds, rec, nullptr, 0, da, 4 * ds, w->Wh, ds, n_bar, 4 * ds, ds,
                         SAT_ACT_IDENTITY, SAT_F32, tmpW, ds, nullptr, 0, dws, dws_bytes, stream);
      if (rc != SAT_OK) return rc;
      axpy_rows_kernel<<<blocks_for(static_cast<int64_t>(4 * ds) * ds), dim3(256), 0, st>>>(
          dWh, ds, tmpW, ds, 4 * ds, ds, 1.0f);
      rc = sat_dense_fwd(da, 4 * ds, n_bar, 4 * ds, ds, w->Wh, ds, SAT_ACT_IDENTITY, SAT_F32,
                         dh[cur ^ 1], ds, stream);
      if (rc != SAT_OK) return rc;
      cur ^= 1;
    }
  }
  return sat::check_launch();
}

extern "C" sat_status sat_sgd_update(float* param, const float* grad, int64_t n, float lr,
                                     void* stream) {
  if (n < 0) return SAT_EINVAL;
  if (n == 0) return SAT_OK;
  if (!param || !grad) return SAT_EINVAL;
  if (blocks_for(n).x == 0 || (n + 255) / 256 > INT32_MAX) return SAT_EUNSUPPORTED;
  sgd_kernel<<<blocks_for(n), dim3(256), 0, static_cast<hipStream_t>(stream)>>>(param, grad, n, lr);
  return sat::check_launch();
}

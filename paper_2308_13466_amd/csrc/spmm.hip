// Normalised-adjacency aggregation AGG = [P_in | P_out] * Hbar (appendix, SAT
// forward) and its transpose products (appendix, SAT backward).
//
// The work is a gather of nnz feature rows: 2 flops per 4 gathered bytes, so
// the memory system is the only bound and the design goal is bytes in flight.
// Mapping for 64-wide wavefronts:
//   * a workgroup of 8 wavefronts owns 8 consecutive CSR rows, one row per
//     wavefront (row-split);
//   * the row's column ids and values are read 64 at a time with one coalesced
//     access and handed out with cross-lane reads;
//   * a group of G lanes covers a feature row with 16-byte loads (G = 64 for
//     256 floats: one 1 KiB row per wavefront access); for narrower rows the
//     64/G groups take different neighbours at once and are summed with
//     lane-xor shuffles at the end;
//   * U neighbours per group are fetched back to back before any of them is
//     used, so a wavefront keeps U * NCH KiB of gathers in flight;
//   * up to NCH 16-byte accumulators per lane: rows up to 1024 floats wide are
//     aggregated in a single walk of the index list;
//   * degree skew: a row longer than kLongRow entries is not walked by its
//     owner alone; after the short rows are done, all 8 wavefronts of the
//     workgroup split it into 8 contiguous pieces and their partial sums are
//     added through LDS in a fixed order (deterministic, no atomics).
// The same kernel serves P_in^T (the local-column prefix of each row, P_in
// being symmetric), P_out^T (through the transposed halo block) and the
// predictor's hop (transposed halo block plus a diagonal term).
#include "sat_internal.h"

namespace {

using sat::kWave;
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kRowsPerBlock = 8;   // wavefronts per workgroup
constexpr int kLongRow = 512;      // entries; longer rows are walked cooperatively

struct SpmmArgs {
  const int64_t* row_begin;
  const int64_t* row_end;
  const int32_t* col;
  const float* val;
  const float* X;
  int64_t ld_x;
  int64_t n_x_rows;
  float* Y;
  int64_t ld_y;
  int64_t n_rows;
  int32_t d;
  const float* self_val;  // nullable: Y[i] += self_val[i] * X[self_off + i]
  int64_t self_off;
};

// acc += sum over entries [s, e) of val * X[col]; all lanes of the wavefront take part.
template <int G, int NCH, int U>
__device__ __forceinline__ void walk_entries(const SpmmArgs& a, int64_t s, int64_t e, int col_base,
                                             int lane, f32x4 (&acc)[NCH]) {
  constexpr int NG = kWave / G;
  const int gl = lane % G;
  const int grp = lane / G;
  const float* Xc = a.X + col_base;
  for (int64_t base = s; base < e; base += kWave) {
    const int cnt = static_cast<int>(e - base < kWave ? e - base : kWave);
    int32_t c = 0;
    float v = 0.f;
    if (lane < cnt) {
      c = a.col[base + lane];
      v = a.val[base + lane];
    }
    if (static_cast<uint32_t>(c) >= static_cast<uint64_t>(a.n_x_rows)) {  // bad id: no contribution
      c = 0;
      v = 0.f;
    }
    for (int j0 = 0; j0 < cnt; j0 += NG * U) {
      int32_t cj[U];
      float vj[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        // entries past the end re-read the last valid row with weight 0
        const int idx = j0 + u * NG + grp;
        const int idc = idx < cnt ? idx : cnt - 1;
        if constexpr (G == kWave) {
          cj[u] = __builtin_amdgcn_readlane(c, idc);
          vj[u] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), idc));
        } else {
          cj[u] = __shfl(c, idc);
          vj[u] = __shfl(v, idc);
        }
        if (idx >= cnt) vj[u] = 0.f;
      }
      f32x4 x[U][NCH];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float* xr = Xc + static_cast<int64_t>(cj[u]) * a.ld_x;
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
          const int c0 = (ch * G + gl) * 4;
          x[u][ch] = (col_base + c0 < a.d) ? *reinterpret_cast<const f32x4*>(xr + c0)
                                           : f32x4{0.f, 0.f, 0.f, 0.f};
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) acc[ch] += vj[u] * x[u][ch];
    }
  }
}

template <int G, int NCH>
__device__ __forceinline__ void reduce_groups(f32x4 (&acc)[NCH]) {
  if constexpr (G < kWave) {
#pragma unroll
    for (int off = G; off < kWave; off <<= 1) {
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) {
        acc[ch].x += __shfl_xor(acc[ch].x, off);
        acc[ch].y += __shfl_xor(acc[ch].y, off);
        acc[ch].z += __shfl_xor(acc[ch].z, off);
        acc[ch].w += __shfl_xor(acc[ch].w, off);
      }
    }
  }
}

__device__ __forceinline__ void store_masked(float* y, int left, const f32x4& v) {
  if (left >= 4) {
    *reinterpret_cast<f32x4*>(y) = v;
  } else if (left > 0) {
    y[0] = v.x;
    if (left > 1) y[1] = v.y;
    if (left > 2) y[2] = v.z;
  }
}

template <int G, int NCH, int U>
__global__ __launch_bounds__(kRowsPerBlock * kWave) void spmm_kernel(SpmmArgs a) {
  constexpr int kPartFloats = G * 4 * NCH;  // floats of one wavefront's partial row
  __shared__ int64_t long_s[kRowsPerBlock], long_e[kRowsPerBlock];
  __shared__ __attribute__((aligned(16))) float part[kRowsPerBlock][kPartFloats];

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t row0 = static_cast<int64_t>(blockIdx.x) * kRowsPerBlock;
  const int64_t row = row0 + wave;
  const int gl = lane % G;
  const int grp = lane / G;
  const int col_base = blockIdx.y * kPartFloats;

  int64_t s = 0, e = 0;
  if (row < a.n_rows) {
    s = a.row_begin[row];
    e = a.row_end[row];
  }
  const bool is_long = (e - s) > kLongRow;
  if (lane == 0) {
    long_s[wave] = is_long ? s : 0;
    long_e[wave] = is_long ? e : 0;
  }

  // ---- short rows: one wavefront each
  if (row < a.n_rows && !is_long) {
    f32x4 acc[NCH];
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) acc[ch] = f32x4{0.f, 0.f, 0.f, 0.f};
    walk_entries<G, NCH, U>(a, s, e, col_base, lane, acc);
    if (a.self_val != nullptr && grp == 0) {
      const float sv = a.self_val[row];
      const float* xr = a.X + (a.self_off + row) * a.ld_x + col_base;
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) {
        const int c0 = (ch * G + gl) * 4;
        if (col_base + c0 < a.d) acc[ch] += sv * *reinterpret_cast<const f32x4*>(xr + c0);
      }
    }
    reduce_groups<G, NCH>(acc);
    if (grp == 0) {
      float* yr = a.Y + row * a.ld_y + col_base;
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) {
        const int c0 = (ch * G + gl) * 4;
        store_masked(yr + c0, a.d - (col_base + c0), acc[ch]);
      }
    }
  }
  __syncthreads();

  // ---- long rows of this workgroup: all wavefronts share each one
  for (int w = 0; w < kRowsPerBlock; ++w) {
    const int64_t ls = long_s[w], le = long_e[w];
    if (le <= ls) continue;  // uniform over the workgroup
    const int64_t piece = ((le - ls + kRowsPerBlock - 1) / kRowsPerBlock + kWave - 1) / kWave * kWave;
    int64_t ps = ls + wave * piece;
    int64_t pe = ps + piece < le ? ps + piece : le;
    if (ps > le) ps = le;
    f32x4 acc[NCH];
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) acc[ch] = f32x4{0.f, 0.f, 0.f, 0.f};
    walk_entries<G, NCH, U>(a, ps, pe, col_base, lane, acc);
    const int64_t lrow = row0 + w;
    if (a.self_val != nullptr && wave == 0 && grp == 0) {
      const float sv = a.self_val[lrow];
      const float* xr = a.X + (a.self_off + lrow) * a.ld_x + col_base;
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) {
        const int c0 = (ch * G + gl) * 4;
        if (col_base + c0 < a.d) acc[ch] += sv * *reinterpret_cast<const f32x4*>(xr + c0);
      }
    }
    reduce_groups<G, NCH>(acc);
    if (grp == 0) {
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch)
        *reinterpret_cast<f32x4*>(&part[wave][(ch * G + gl) * 4]) = acc[ch];
    }
    __syncthreads();
    // fixed-order sum of the 8 partial rows, 16 bytes per thread
    for (int q = threadIdx.x; q < kPartFloats / 4; q += kRowsPerBlock * kWave) {
      f32x4 sum = *reinterpret_cast<const f32x4*>(&part[0][q * 4]);
#pragma unroll
      for (int k = 1; k < kRowsPerBlock; ++k) sum += *reinterpret_cast<const f32x4*>(&part[k][q * 4]);
      store_masked(a.Y + lrow * a.ld_y + col_base + q * 4, a.d - (col_base + q * 4), sum);
    }
    __syncthreads();
  }
}


// Short rows, narrow features (G <= 32, one 16-byte accumulator per lane): a
// group of G lanes owns a whole row, so a wavefront works on 64/G rows at once.
// When rows hold only a handful of entries (the transposed halo block averages
// under three) the walk is a chain of dependent loads per row, and the number of
// rows in flight is what sets the speed. A row longer than max_len is walked
// afterwards by all 64 lanes of the wavefront its group belongs to (64/G
// neighbours at a time), so the occasional longer row does not stall one group.
template <int G, int U>
__global__ __launch_bounds__(256) void spmm_group_kernel(SpmmArgs a, int64_t max_len) {
  constexpr int NG = kWave / G;
  const int lane = threadIdx.x & (kWave - 1);
  const int gl = lane % G;
  const int grp = lane / G;
  const int64_t row = (static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6)) * NG + grp;
  int64_t s = 0, e = 0;
  if (row < a.n_rows) {
    s = a.row_begin[row];
    e = a.row_end[row];
  }
  const int64_t s0 = s, e0 = e;
  const bool mine = row < a.n_rows && (e - s) <= max_len;
  if (!mine) e = s;
  const int c0 = gl * 4;
  const bool col_ok = c0 < a.d;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  if (mine && a.self_val != nullptr && col_ok)
    acc = a.self_val[row] * *reinterpret_cast<const f32x4*>(a.X + (a.self_off + row) * a.ld_x + c0);
  for (int64_t base = s; base < e; base += G) {
    const int cnt = static_cast<int>(e - base < G ? e - base : G);
    int32_t c = 0;
    float v = 0.f;
    if (gl < cnt) {
      c = a.col[base + gl];
      v = a.val[base + gl];
    }
    if (static_cast<uint32_t>(c) >= static_cast<uint64_t>(a.n_x_rows)) {
      c = 0;
      v = 0.f;
    }
    for (int j0 = 0; j0 < cnt; j0 += U) {
      int32_t cj[U];
      float vj[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int idx = j0 + u;
        const int idc = idx < cnt ? idx : cnt - 1;
        cj[u] = __shfl(c, grp * G + idc);
        vj[u] = __shfl(v, grp * G + idc);
        if (idx >= cnt) vj[u] = 0.f;
      }
      f32x4 x[U];
#pragma unroll
      for (int u = 0; u < U; ++u)
        x[u] = col_ok ? *reinterpret_cast<const f32x4*>(a.X + static_cast<int64_t>(cj[u]) * a.ld_x + c0)
                      : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int u = 0; u < U; ++u) acc += vj[u] * x[u];
    }
  }
  if (mine && col_ok) store_masked(a.Y + row * a.ld_y + c0, a.d - c0, acc);

  // rows too long for one group: one bit per group, handled one after another
  uint64_t todo = __ballot(row < a.n_rows && !mine && gl == 0);
  while (todo) {
    const int src = __builtin_ctzll(todo);
    todo &= todo - 1;
    const int64_t rs = __shfl(s0, src), re = __shfl(e0, src), r = __shfl(row, src);
    f32x4 wacc[1] = {f32x4{0.f, 0.f, 0.f, 0.f}};
    walk_entries<G, 1, U>(a, rs, re, 0, lane, wacc);
    if (a.self_val != nullptr && grp == 0 && col_ok)
      wacc[0] += a.self_val[r] * *reinterpret_cast<const f32x4*>(a.X + (a.self_off + r) * a.ld_x + c0);
    reduce_groups<G, 1>(wacc);
    if (grp == 0 && col_ok) store_masked(a.Y + r * a.ld_y + c0, a.d - c0, wacc[0]);
  }
}

}  // namespace

namespace sat {

// Y[n_rows, d] = M * X (+ diag(self_val) * X[self_off + i]) where row i of M is
// (col, val)[row_begin[i] .. row_end[i]). Pointers are device pointers; X and Y
// 16-byte aligned with ld % 4 == 0 (checked by the callers).
sat_status launch_spmm(const int64_t* row_begin, const int64_t* row_end, const int32_t* col,
                       const float* val, const float* X, int64_t ld_x, int64_t n_x_rows, float* Y,
                       int64_t ld_y, int64_t n_rows, int32_t d, const float* self_val,
                       int64_t self_off, int64_t total_entries, hipStream_t stream) {
  if (n_rows == 0 || d == 0) return SAT_OK;
  const int64_t bx = (n_rows + kRowsPerBlock - 1) / kRowsPerBlock;
  if (bx > INT32_MAX) return SAT_EUNSUPPORTED;
  const int nvec = (d + 3) / 4;
  const dim3 block(kRowsPerBlock * kWave);
  const SpmmArgs a{row_begin, row_end, col, val, X, ld_x, n_x_rows, Y, ld_y, n_rows, d, self_val,
                   self_off};
  // Few entries per row and narrow features: a group of lanes per row.
  constexpr int64_t kGroupMaxLen = 64;
  if (nvec <= 32 && total_entries < 16 * n_rows) {
    int g = 1;
    while (g < nvec) g <<= 1;
    const int64_t rows_per_block = 4 * (kWave / g);
    const int64_t gb = (n_rows + rows_per_block - 1) / rows_per_block;
    if (gb > INT32_MAX) return SAT_EUNSUPPORTED;
    const dim3 ggrid(static_cast<unsigned>(gb));
    switch (g) {
      case 1: spmm_group_kernel<1, 4><<<ggrid, dim3(256), 0, stream>>>(a, kGroupMaxLen); break;
      case 2: spmm_group_kernel<2, 4><<<ggrid, dim3(256), 0, stream>>>(a, kGroupMaxLen); break;
      case 4: spmm_group_kernel<4, 4><<<ggrid, dim3(256), 0, stream>>>(a, kGroupMaxLen); break;
      case 8: spmm_group_kernel<8, 4><<<ggrid, dim3(256), 0, stream>>>(a, kGroupMaxLen); break;
      case 16: spmm_group_kernel<16, 4><<<ggrid, dim3(256), 0, stream>>>(a, kGroupMaxLen); break;
      default: spmm_group_kernel<32, 4><<<ggrid, dim3(256), 0, stream>>>(a, kGroupMaxLen); break;
    }
    return sat::check_launch();
  }
#define SAT_SPMM_LAUNCH(G, NCH, U)                                                            \
  do {                                                                                        \
    const int per_pass = (G) * 4 * (NCH);                                                     \
    const dim3 grid(static_cast<unsigned>(bx), static_cast<unsigned>((d + per_pass - 1) / per_pass)); \
    spmm_kernel<G, NCH, U><<<grid, block, 0, stream>>>(a);                                    \
  } while (0)
  if (nvec <= 1) SAT_SPMM_LAUNCH(1, 1, 4);
  else if (nvec <= 2) SAT_SPMM_LAUNCH(2, 1, 4);
  else if (nvec <= 4) SAT_SPMM_LAUNCH(4, 1, 4);
  else if (nvec <= 8) SAT_SPMM_LAUNCH(8, 1, 4);
  else if (nvec <= 16) SAT_SPMM_LAUNCH(16, 1, 4);
  else if (nvec <= 32) SAT_SPMM_LAUNCH(32, 1, 4);
  else if (nvec <= 64) SAT_SPMM_LAUNCH(64, 1, 8);
  else if (nvec <= 128) SAT_SPMM_LAUNCH(64, 2, 4);
  else if (nvec <= 192) SAT_SPMM_LAUNCH(64, 3, 2);
  else SAT_SPMM_LAUNCH(64, 4, 2);
#undef SAT_SPMM_LAUNCH
  return sat::check_launch();
}

}  // namespace sat

namespace {

using sat::launch_spmm;

sat_status validate_view(const sat_part_view* pv) {
  if (!pv) return SAT_EINVAL;
  if (pv->n_local < 0 || pv->n_halo < 0 || pv->nnz < 0 || pv->nnz_halo < 0) return SAT_EINVAL;
  if (pv->n_local + pv->n_halo > INT32_MAX) return SAT_EUNSUPPORTED;
  if (!pv->rowptr) return SAT_EINVAL;
  if (pv->n_local > 0 && (!pv->split || (pv->nnz > 0 && (!pv->col || !pv->val)))) return SAT_EINVAL;
  return SAT_OK;
}

sat_status validate_dense(const void* p, int64_t rows, int64_t ld, int32_t d) {
  if (rows > 0 && d > 0) {
    if (!p || ld < d) return SAT_EINVAL;
    if (!sat::aligned16(p) || (ld % 4) != 0) return SAT_EALIGN;
  }
  return SAT_OK;
}

}  // namespace

extern "C" int64_t sat_spmm_workspace_bytes(const sat_part_view* pv, int32_t d) {
  (void)pv;
  (void)d;
  return 0;
}

extern "C" sat_status sat_spmm_fwd(const sat_part_view* pv, const void* Hbar, int64_t ld_in,
                                   int32_t d, int32_t dtype, void* AGG, int64_t ld_out,
                                   void* workspace, int64_t workspace_bytes, void* stream) {
  (void)workspace;
  (void)workspace_bytes;
  sat_status st = validate_view(pv);
  if (st != SAT_OK) return st;
  if (d < 0) return SAT_EINVAL;
  if (dtype != SAT_F32) return dtype == SAT_BF16 ? SAT_EUNSUPPORTED : SAT_EINVAL;
  if ((st = validate_dense(Hbar, pv->n_local + pv->n_halo, ld_in, d)) != SAT_OK) return st;
  if ((st = validate_dense(AGG, pv->n_local, ld_out, d)) != SAT_OK) return st;
  return launch_spmm(pv->rowptr, pv->rowptr + 1, pv->col, pv->val, static_cast<const float*>(Hbar),
                     ld_in, pv->n_local + pv->n_halo, static_cast<float*>(AGG), ld_out,
                     pv->n_local, d, nullptr, 0, pv->nnz, static_cast<hipStream_t>(stream));
}

extern "C" sat_status sat_spmm_bwd(const sat_part_view* pv, const void* dAGG, int64_t ld_in,
                                   int32_t d, int32_t dtype, void* dH_local, int64_t ld_out,
                                   void* dH_halo, int64_t ld_halo, void* workspace,
                                   int64_t workspace_bytes, void* stream) {
  (void)workspace;
  (void)workspace_bytes;
  sat_status st = validate_view(pv);
  if (st != SAT_OK) return st;
  if (d < 0) return SAT_EINVAL;
  if (dtype != SAT_F32) return dtype == SAT_BF16 ? SAT_EUNSUPPORTED : SAT_EINVAL;
  if ((st = validate_dense(dAGG, pv->n_local, ld_in, d)) != SAT_OK) return st;
  if ((st = validate_dense(dH_local, pv->n_local, ld_out, d)) != SAT_OK) return st;
  if (dH_halo) {
    if ((st = validate_dense(dH_halo, pv->n_halo, ld_halo, d)) != SAT_OK) return st;
    if (pv->n_halo > 0 && (!pv->h_colptr || (pv->nnz_halo > 0 && (!pv->h_row || !pv->h_val))))
      return SAT_EINVAL;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  // P_in^T = P_in: row i's local columns are [rowptr[i], split[i])
  st = launch_spmm(pv->rowptr, pv->split, pv->col, pv->val, static_cast<const float*>(dAGG), ld_in,
                   pv->n_local, static_cast<float*>(dH_local), ld_out, pv->n_local, d, nullptr, 0, pv->nnz - pv->nnz_halo, s);
  if (st != SAT_OK || !dH_halo) return st;
  return launch_spmm(pv->h_colptr, pv->h_colptr + 1, pv->h_row, pv->h_val,
                     static_cast<const float*>(dAGG), ld_in, pv->n_local,
                     static_cast<float*>(dH_halo), ld_halo, pv->n_halo, d, nullptr, 0, pv->nnz_halo, s);
}

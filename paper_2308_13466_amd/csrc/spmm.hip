// Normalised-adjacency aggregation AGG = [P_in | P_out] * Hbar (appendix, SAT
// forward) and its transpose products (appendix, SAT backward).
//
// The work is a gather of nnz feature rows: 2 flops per 4 gathered bytes, so
// the memory system is the only bound. Mapping for 64-wide wavefronts:
//   * one wavefront per CSR row (row-split); the row's column ids and values
//     are read 64 at a time with one coalesced access and handed out with
//     cross-lane reads;
//   * a group of G lanes covers a feature row with 16-byte loads (G = 64 for
//     d >= 256 floats: exactly one 1 KiB row per wavefront access); for narrower
//     rows the 64/G groups take different neighbours at once and are summed
//     with lane-xor shuffles at the end;
//   * up to NCH 16-byte accumulators per lane, so rows up to 1024 floats wide
//     are aggregated in a single walk of the index list.
// The same kernel serves P_in^T (the local-column prefix of each row, P_in
// being symmetric) and P_out^T (through the transposed halo block).
#include "sat_internal.h"

namespace {

using sat::kWave;
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int G, int NCH>
__global__ __launch_bounds__(256) void spmm_row_wave_kernel(
    const int64_t* __restrict__ row_begin, const int64_t* __restrict__ row_end,
    const int32_t* __restrict__ col, const float* __restrict__ val, const float* __restrict__ X,
    int64_t ld_x, int64_t n_x_rows, float* __restrict__ Y, int64_t ld_y, int64_t n_rows,
    int32_t d) {
  constexpr int NG = kWave / G;  // neighbours processed at once by a wavefront
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + wave;
  if (row >= n_rows) return;
  const int gl = lane % G;
  const int grp = lane / G;
  const int col_base = blockIdx.y * (G * 4 * NCH);
  const int64_t s = row_begin[row];
  const int64_t e = row_end[row];

  f32x4 acc[NCH];
#pragma unroll
  for (int ch = 0; ch < NCH; ++ch) acc[ch] = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int64_t base = s; base < e; base += kWave) {
    const int cnt = static_cast<int>(e - base < kWave ? e - base : kWave);
    int32_t c = 0;
    float v = 0.f;
    if (lane < cnt) {
      c = col[base + lane];
      v = val[base + lane];
    }
    const bool ok = static_cast<uint32_t>(c) < static_cast<uint64_t>(n_x_rows);
    for (int j = 0; j < cnt; j += NG) {
      int32_t cj;
      float vj;
      bool okj;
      if constexpr (G == kWave) {
        cj = __builtin_amdgcn_readlane(c, j);
        vj = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), j));
        okj = __builtin_amdgcn_readlane(static_cast<int>(ok), j) != 0;
      } else {
        cj = __shfl(c, j + grp);
        vj = __shfl(v, j + grp);
        okj = __shfl(static_cast<int>(ok), j + grp) != 0 && (j + grp < cnt);
      }
      if (okj) {
        const float* xr = X + static_cast<int64_t>(cj) * ld_x + col_base;
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
          const int c0 = (ch * G + gl) * 4;
          if (col_base + c0 < d) {
            const f32x4 x = *reinterpret_cast<const f32x4*>(xr + c0);
            acc[ch] += vj * x;
          }
        }
      }
    }
  }

  if constexpr (NG > 1) {
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
  if (grp == 0) {
    float* yr = Y + row * ld_y + col_base;
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      const int c0 = (ch * G + gl) * 4;
      const int left = d - (col_base + c0);
      if (left >= 4) {
        *reinterpret_cast<f32x4*>(yr + c0) = acc[ch];
      } else if (left > 0) {
        yr[c0] = acc[ch].x;
        if (left > 1) yr[c0 + 1] = acc[ch].y;
        if (left > 2) yr[c0 + 2] = acc[ch].z;
      }
    }
  }
}

// Y[n_rows, d] = M * X where row i of M is (col, val)[row_begin[i] .. row_end[i]).
sat_status launch_spmm(const int64_t* row_begin, const int64_t* row_end, const int32_t* col,
                       const float* val, const float* X, int64_t ld_x, int64_t n_x_rows, float* Y,
                       int64_t ld_y, int64_t n_rows, int32_t d, hipStream_t stream) {
  if (n_rows == 0 || d == 0) return SAT_OK;
  const int64_t bx = (n_rows + 3) / 4;
  if (bx > INT32_MAX) return SAT_EUNSUPPORTED;
  const int nvec = (d + 3) / 4;
  const dim3 block(256);
#define SAT_SPMM_LAUNCH(G, NCH)                                                               \
  do {                                                                                        \
    const int per_pass = (G) * 4 * (NCH);                                                     \
    const dim3 grid(static_cast<unsigned>(bx), static_cast<unsigned>((d + per_pass - 1) / per_pass)); \
    spmm_row_wave_kernel<G, NCH><<<grid, block, 0, stream>>>(row_begin, row_end, col, val, X, \
                                                             ld_x, n_x_rows, Y, ld_y, n_rows, d); \
  } while (0)
  if (nvec <= 1) SAT_SPMM_LAUNCH(1, 1);
  else if (nvec <= 2) SAT_SPMM_LAUNCH(2, 1);
  else if (nvec <= 4) SAT_SPMM_LAUNCH(4, 1);
  else if (nvec <= 8) SAT_SPMM_LAUNCH(8, 1);
  else if (nvec <= 16) SAT_SPMM_LAUNCH(16, 1);
  else if (nvec <= 32) SAT_SPMM_LAUNCH(32, 1);
  else if (nvec <= 64) SAT_SPMM_LAUNCH(64, 1);
  else if (nvec <= 128) SAT_SPMM_LAUNCH(64, 2);
  else if (nvec <= 192) SAT_SPMM_LAUNCH(64, 3);
  else SAT_SPMM_LAUNCH(64, 4);
#undef SAT_SPMM_LAUNCH
  return sat::check_launch();
}

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
                     pv->n_local, d, static_cast<hipStream_t>(stream));
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
                   pv->n_local, static_cast<float*>(dH_local), ld_out, pv->n_local, d, s);
  if (st != SAT_OK || !dH_halo) return st;
  return launch_spmm(pv->h_colptr, pv->h_colptr + 1, pv->h_row, pv->h_val,
                     static_cast<const float*>(dAGG), ld_in, pv->n_local,
                     static_cast<float*>(dH_halo), ld_halo, pv->n_halo, d, s);
}

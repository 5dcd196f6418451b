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
//     lane-xor shuffles at the end (bf16 rows: a 16-byte load is 8 elements, so
//     256 bf16 take 32 lanes and two neighbours go at once);
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
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kRowsPerBlock = 8;   // wavefronts per workgroup
constexpr int kLongRow = 512;      // entries; longer rows are walked cooperatively

// A 16-byte chunk of a feature row held as fp32: 4 fp32 elements, or 8 bf16
// elements kept de-interleaved (q[0] = elements 0,2,4,6, q[1] = elements 1,3,5,7:
// widening a packed pair is then one shift and one mask on the whole vector).
// ES = bytes per element. Sums are always carried in fp32; bf16 results are
// rounded to nearest-even once, when the output row is stored.
template <int ES>
struct Chunk {
  static constexpr int N = 16 / ES;   // elements
  static constexpr int NV = N / 4;    // fp32 vectors
  f32x4 q[NV];
  __device__ __forceinline__ void zero() {
#pragma unroll
    for (int k = 0; k < NV; ++k) q[k] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  __device__ __forceinline__ void load(const unsigned char* p) {
    if constexpr (ES == 4) {
      q[0] = *reinterpret_cast<const f32x4*>(p);
    } else {
      const u32x4 w = *reinterpret_cast<const u32x4*>(p);
      q[0] = __builtin_bit_cast(f32x4, w << 16);
      q[1] = __builtin_bit_cast(f32x4, w & 0xffff0000u);
    }
  }
  __device__ __forceinline__ void fma(float s, const Chunk& x) {
#pragma unroll
    for (int k = 0; k < NV; ++k) q[k] += s * x.q[k];
  }
  __device__ __forceinline__ void add(const Chunk& x) {
#pragma unroll
    for (int k = 0; k < NV; ++k) q[k] += x.q[k];
  }
  __device__ __forceinline__ void xor_add(int off) {
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      q[k].x += __shfl_xor(q[k].x, off);
      q[k].y += __shfl_xor(q[k].y, off);
      q[k].z += __shfl_xor(q[k].z, off);
      q[k].w += __shfl_xor(q[k].w, off);
    }
  }
  // raw fp32 image (N floats) for the LDS partial-sum buffer
  __device__ __forceinline__ void to_lds(float* p) const {
#pragma unroll
    for (int k = 0; k < NV; ++k) *reinterpret_cast<f32x4*>(p + 4 * k) = q[k];
  }
  __device__ __forceinline__ void from_lds(const float* p) {
#pragma unroll
    for (int k = 0; k < NV; ++k) q[k] = *reinterpret_cast<const f32x4*>(p + 4 * k);
  }
  // store the first min(left, N) elements at p (p is 16-byte aligned)
  __device__ __forceinline__ void store(unsigned char* p, int left) const {
    if constexpr (ES == 4) {
      if (left >= 4) {
        *reinterpret_cast<f32x4*>(p) = q[0];
      } else {
        float* y = reinterpret_cast<float*>(p);
        y[0] = q[0].x;
        if (left > 1) y[1] = q[0].y;
        if (left > 2) y[2] = q[0].z;
      }
    } else {
      u32x4 w;
      w.x = pack2(q[0].x, q[1].x);
      w.y = pack2(q[0].y, q[1].y);
      w.z = pack2(q[0].z, q[1].z);
      w.w = pack2(q[0].w, q[1].w);
      if (left >= 8) {
        *reinterpret_cast<u32x4*>(p) = w;
      } else {
        uint16_t* y = reinterpret_cast<uint16_t*>(p);
        const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
        for (int i = 0; i < left; ++i)
          y[i] = static_cast<uint16_t>((i & 1) ? (ww[i >> 1] >> 16) : (ww[i >> 1] & 0xffffu));
      }
    }
  }
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {  // RNE, lo in the low half
    const f32x2 pr = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));
  }
};

struct SpmmArgs {
  const int64_t* row_begin;
  const int64_t* row_end;
  const int32_t* col;
  const float* val;
  const unsigned char* X;  // [n_x_rows, ld_x] elements of ES bytes
  int64_t ld_x;            // bytes
  int64_t n_x_rows;
  unsigned char* Y;        // [n_rows, ld_y]
  int64_t ld_y;            // bytes
  int64_t n_rows;
  int32_t d;               // elements per row
  const float* self_val;   // nullable: Y[i] += self_val[i] * X[self_off + i]
  int64_t self_off;
};

// acc += sum over entries [s, e) of val * X[col]; all lanes of the wavefront take part.
// Lane (grp, gl) handles chunk (ch * G + gl) of the feature row, counted from
// element col_base.
template <int ES, int G, int NCH, int U>
__device__ __forceinline__ void walk_entries(const SpmmArgs& a, int64_t s, int64_t e, int col_base,
                                             int lane, Chunk<ES> (&acc)[NCH]) {
  constexpr int NG = kWave / G;
  constexpr int EPL = Chunk<ES>::N;
  const int gl = lane % G;
  const int grp = lane / G;
  const unsigned char* Xc = a.X + static_cast<int64_t>(col_base) * ES;
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
      Chunk<ES> x[U][NCH];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const unsigned char* xr = Xc + static_cast<int64_t>(cj[u]) * a.ld_x;
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
          const int c0 = (ch * G + gl) * EPL;
          if (col_base + c0 < a.d)
            x[u][ch].load(xr + c0 * ES);
          else
            x[u][ch].zero();
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) acc[ch].fma(vj[u], x[u][ch]);
    }
  }
}

template <int ES, int G, int NCH>
__device__ __forceinline__ void reduce_groups(Chunk<ES> (&acc)[NCH]) {
  if constexpr (G < kWave) {
#pragma unroll
    for (int off = G; off < kWave; off <<= 1) {
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) acc[ch].xor_add(off);
    }
  }
}

// acc += self_val[row] * X[self_off + row] (lanes of group 0 only)
template <int ES, int G, int NCH>
__device__ __forceinline__ void add_self(const SpmmArgs& a, int64_t row, int col_base, int gl,
                                         Chunk<ES> (&acc)[NCH]) {
  constexpr int EPL = Chunk<ES>::N;
  const float sv = a.self_val[row];
  const unsigned char* xr = a.X + (a.self_off + row) * a.ld_x + static_cast<int64_t>(col_base) * ES;
#pragma unroll
  for (int ch = 0; ch < NCH; ++ch) {
    const int c0 = (ch * G + gl) * EPL;
    if (col_base + c0 < a.d) {
      Chunk<ES> x;
      x.load(xr + c0 * ES);
      acc[ch].fma(sv, x);
    }
  }
}

template <int ES, int G, int NCH, int U>
__global__ __launch_bounds__(kRowsPerBlock * kWave) void spmm_kernel(SpmmArgs a) {
  constexpr int EPL = Chunk<ES>::N;
  constexpr int kPartElems = G * EPL * NCH;  // elements of one wavefront's partial row
  __shared__ int64_t long_s[kRowsPerBlock], long_e[kRowsPerBlock];
  __shared__ __attribute__((aligned(16))) float part[kRowsPerBlock][kPartElems];

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t row0 = static_cast<int64_t>(blockIdx.x) * kRowsPerBlock;
  const int64_t row = row0 + wave;
  const int gl = lane % G;
  const int grp = lane / G;
  const int col_base = blockIdx.y * kPartElems;

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
    Chunk<ES> acc[NCH];
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) acc[ch].zero();
    walk_entries<ES, G, NCH, U>(a, s, e, col_base, lane, acc);
    if (a.self_val != nullptr && grp == 0) add_self<ES, G, NCH>(a, row, col_base, gl, acc);
    reduce_groups<ES, G, NCH>(acc);
    if (grp == 0) {
      unsigned char* yr = a.Y + row * a.ld_y + static_cast<int64_t>(col_base) * ES;
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) {
        const int c0 = (ch * G + gl) * EPL;
        const int left = a.d - (col_base + c0);
        if (left > 0) acc[ch].store(yr + c0 * ES, left);
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
    Chunk<ES> acc[NCH];
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) acc[ch].zero();
    walk_entries<ES, G, NCH, U>(a, ps, pe, col_base, lane, acc);
    const int64_t lrow = row0 + w;
    if (a.self_val != nullptr && wave == 0 && grp == 0) add_self<ES, G, NCH>(a, lrow, col_base, gl, acc);
    reduce_groups<ES, G, NCH>(acc);
    if (grp == 0) {
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) acc[ch].to_lds(&part[wave][(ch * G + gl) * EPL]);
    }
    __syncthreads();
    // fixed-order sum of the 8 partial rows, one 16-byte output chunk per thread
    for (int q = threadIdx.x; q < kPartElems / EPL; q += kRowsPerBlock * kWave) {
      Chunk<ES> sum, other;
      sum.from_lds(&part[0][q * EPL]);
#pragma unroll
      for (int k = 1; k < kRowsPerBlock; ++k) {
        other.from_lds(&part[k][q * EPL]);
        sum.add(other);
      }
      const int left = a.d - (col_base + q * EPL);
      if (left > 0)
        sum.store(a.Y + lrow * a.ld_y + static_cast<int64_t>(col_base + q * EPL) * ES, left);
    }
    __syncthreads();
  }
}

// Short rows, narrow features (G <= 32, one 16-byte accumulator chunk per lane):
// a group of G lanes owns a whole row, so a wavefront works on 64/G rows at once.
// When rows hold only a handful of entries (the transposed halo block averages
// under three) the walk is a chain of dependent loads per row, and the number of
// rows in flight is what sets the speed. A row longer than max_len is walked
// afterwards by all 64 lanes of the wavefront its group belongs to (64/G
// neighbours at a time), so the occasional longer row does not stall one group.
template <int ES, int G, int U>
__global__ __launch_bounds__(256) void spmm_group_kernel(SpmmArgs a, int64_t max_len) {
  constexpr int NG = kWave / G;
  constexpr int EPL = Chunk<ES>::N;
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
  const int c0 = gl * EPL;
  const bool col_ok = c0 < a.d;
  Chunk<ES> acc;
  acc.zero();
  if (mine && a.self_val != nullptr && col_ok) {
    Chunk<ES> x;
    x.load(a.X + (a.self_off + row) * a.ld_x + c0 * ES);
    acc.fma(a.self_val[row], x);
  }
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
      Chunk<ES> x[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (col_ok)
          x[u].load(a.X + static_cast<int64_t>(cj[u]) * a.ld_x + c0 * ES);
        else
          x[u].zero();
      }
#pragma unroll
      for (int u = 0; u < U; ++u) acc.fma(vj[u], x[u]);
    }
  }
  if (mine && col_ok) acc.store(a.Y + row * a.ld_y + c0 * ES, a.d - c0);

  // rows too long for one group: one bit per group, handled one after another
  uint64_t todo = __ballot(row < a.n_rows && !mine && gl == 0);
  while (todo) {
    const int src = __builtin_ctzll(todo);
    todo &= todo - 1;
    const int64_t rs = __shfl(s0, src), re = __shfl(e0, src), r = __shfl(row, src);
    Chunk<ES> wacc[1];
    wacc[0].zero();
    walk_entries<ES, G, 1, U>(a, rs, re, 0, lane, wacc);
    if (a.self_val != nullptr && grp == 0) add_self<ES, G, 1>(a, r, 0, gl, wacc);
    reduce_groups<ES, G, 1>(wacc);
    if (grp == 0 && col_ok) wacc[0].store(a.Y + r * a.ld_y + c0 * ES, a.d - c0);
  }
}

}  // namespace

namespace sat {

// Y[n_rows, d] = M * X (+ diag(self_val) * X[self_off + i]) where row i of M is
// (col, val)[row_begin[i] .. row_end[i]). X and Y hold elements of es bytes
// (4: fp32, 2: bf16; sums in fp32 either way), ld in elements. Pointers are
// device pointers; X and Y 16-byte aligned with ld * es % 16 == 0 (checked by
// the callers).
template <int ES>
static sat_status launch_spmm_es(const SpmmArgs& a, int64_t total_entries, hipStream_t stream) {
  const int64_t n_rows = a.n_rows;
  const int32_t d = a.d;
  const int64_t bx = (n_rows + kRowsPerBlock - 1) / kRowsPerBlock;
  if (bx > INT32_MAX) return SAT_EUNSUPPORTED;
  constexpr int EPL = 16 / ES;
  const int nvec = (d + EPL - 1) / EPL;   // 16-byte chunks per row
  const dim3 block(kRowsPerBlock * kWave);
  // Few entries per row and narrow rows: a group of lanes per row.
  constexpr int64_t kGroupMaxLen = 64;
  if (nvec <= 32 && total_entries < 16 * n_rows) {
    int g = 1;
    while (g < nvec) g <<= 1;
    const int64_t rows_per_block = 4 * (kWave / g);
    const int64_t gb = (n_rows + rows_per_block - 1) / rows_per_block;
    if (gb > INT32_MAX) return SAT_EUNSUPPORTED;
    const dim3 ggrid(static_cast<unsigned>(gb));
    switch (g) {
      case 1: spmm_group_kernel<ES, 1, 4><<<ggrid, dim3(256), 0, stream>>>(a, kGroupMaxLen); break;
      case 2: spmm_group_kernel<ES, 2, 4><<<ggrid, dim3(256), 0, stream>>>(a, kGroupMaxLen); break;
      case 4: spmm_group_kernel<ES, 4, 4><<<ggrid, dim3(256), 0, stream>>>(a, kGroupMaxLen); break;
      case 8: spmm_group_kernel<ES, 8, 4><<<ggrid, dim3(256), 0, stream>>>(a, kGroupMaxLen); break;
      case 16: spmm_group_kernel<ES, 16, 4><<<ggrid, dim3(256), 0, stream>>>(a, kGroupMaxLen); break;
      default: spmm_group_kernel<ES, 32, 4><<<ggrid, dim3(256), 0, stream>>>(a, kGroupMaxLen); break;
    }
    return sat::check_launch();
  }
#define SAT_SPMM_LAUNCH(G, NCH, U)                                                            \
  do {                                                                                        \
    const int per_pass = (G) * EPL * (NCH);                                                   \
    const dim3 grid(static_cast<unsigned>(bx), static_cast<unsigned>((d + per_pass - 1) / per_pass)); \
    spmm_kernel<ES, G, NCH, U><<<grid, block, 0, stream>>>(a);                                \
  } while (0)
  if (nvec <= 1) SAT_SPMM_LAUNCH(1, 1, 4);
  else if (nvec <= 2) SAT_SPMM_LAUNCH(2, 1, 4);
  else if (nvec <= 4) SAT_SPMM_LAUNCH(4, 1, 4);
  else if (nvec <= 8) SAT_SPMM_LAUNCH(8, 1, 4);
  else if (nvec <= 16) SAT_SPMM_LAUNCH(16, 1, 4);
  else if (nvec <= 32) SAT_SPMM_LAUNCH(32, 1, 4);
  else if (nvec <= 64) SAT_SPMM_LAUNCH(64, 1, ES == 4 ? 8 : 4);
  else if (nvec <= 128) SAT_SPMM_LAUNCH(64, 2, ES == 4 ? 4 : 2);
  else if (nvec <= 192) SAT_SPMM_LAUNCH(64, 3, 2);
  else SAT_SPMM_LAUNCH(64, 4, ES == 4 ? 2 : 1);
#undef SAT_SPMM_LAUNCH
  return sat::check_launch();
}

sat_status launch_spmm(const int64_t* row_begin, const int64_t* row_end, const int32_t* col,
                       const float* val, const void* X, int64_t ld_x, int64_t n_x_rows, void* Y,
                       int64_t ld_y, int64_t n_rows, int32_t d, int es, const float* self_val,
                       int64_t self_off, int64_t total_entries, hipStream_t stream) {
  if (n_rows == 0 || d == 0) return SAT_OK;
  const SpmmArgs a{row_begin, row_end, col, val, static_cast<const unsigned char*>(X), ld_x * es,
                   n_x_rows, static_cast<unsigned char*>(Y), ld_y * es, n_rows, d, self_val,
                   self_off};
  return es == 2 ? launch_spmm_es<2>(a, total_entries, stream)
                 : launch_spmm_es<4>(a, total_entries, stream);
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

sat_status validate_dense(const void* p, int64_t rows, int64_t ld, int32_t d, int es) {
  if (rows > 0 && d > 0) {
    if (!p || ld < d) return SAT_EINVAL;
    if (!sat::aligned16(p) || ((ld * es) % 16) != 0) return SAT_EALIGN;
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
  if (dtype != SAT_F32 && dtype != SAT_BF16) return SAT_EINVAL;
  const int es = dtype == SAT_BF16 ? 2 : 4;
  if ((st = validate_dense(Hbar, pv->n_local + pv->n_halo, ld_in, d, es)) != SAT_OK) return st;
  if ((st = validate_dense(AGG, pv->n_local, ld_out, d, es)) != SAT_OK) return st;
  return launch_spmm(pv->rowptr, pv->rowptr + 1, pv->col, pv->val, Hbar, ld_in,
                     pv->n_local + pv->n_halo, AGG, ld_out, pv->n_local, d, es, nullptr, 0, pv->nnz,
                     static_cast<hipStream_t>(stream));
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
  if (dtype != SAT_F32 && dtype != SAT_BF16) return SAT_EINVAL;
  const int es = dtype == SAT_BF16 ? 2 : 4;
  if ((st = validate_dense(dAGG, pv->n_local, ld_in, d, es)) != SAT_OK) return st;
  if ((st = validate_dense(dH_local, pv->n_local, ld_out, d, es)) != SAT_OK) return st;
  if (dH_halo) {
    if ((st = validate_dense(dH_halo, pv->n_halo, ld_halo, d, es)) != SAT_OK) return st;
    if (pv->n_halo > 0 && (!pv->h_colptr || (pv->nnz_halo > 0 && (!pv->h_row || !pv->h_val))))
      return SAT_EINVAL;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  // P_in^T = P_in: row i's local columns are [rowptr[i], split[i])
  st = launch_spmm(pv->rowptr, pv->split, pv->col, pv->val, dAGG, ld_in, pv->n_local, dH_local,
                   ld_out, pv->n_local, d, es, nullptr, 0, pv->nnz - pv->nnz_halo, s);
  if (st != SAT_OK || !dH_halo) return st;
  return launch_spmm(pv->h_colptr, pv->h_colptr + 1, pv->h_row, pv->h_val, dAGG, ld_in,
                     pv->n_local, dH_halo, ld_halo, pv->n_halo, d, es, nullptr, 0, pv->nnz_halo, s);
}

// Pull and push of history-table rows (Alg. 1: "Pull H_out" / "Push computed
// embeddings"): row-granular gather and scatter, bit-exact copies.
//
// sat_history_gather_add is the pull of the stale-gradient term of the appendix's
// SAT backward (P_out^T D~^(t-1) W^T, kept in a gradient table by the partitions
// that computed it): out[k, :] += table[ids[k], :], added in fp32.
//
// HBM-bound and reuse-free, so the only goals are full-width memory
// transactions and enough bytes in flight. A group of G lanes (G a power of two
// up to 64, chosen so one pass of 16-byte accesses covers a row where possible)
// owns one row; the 64/G groups of a wavefront own consecutive rows, so a
// wavefront's id reads are one coalesced access and its row copies are
// contiguous on the dense side.
#include "sat_internal.h"

namespace {

using sat::kWave;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// GATHER: dense[k, :] = table[ids[k], :]   (SCATTER: table[ids[k], :] = dense[k, :])
// Rows are handled as bytes (row_bytes, leading dimensions in bytes), so the same
// kernels serve 4-byte and 2-byte elements; the tail after the last whole
// 16-byte chunk is copied in 2-byte units.
template <int G, bool SCATTER>
__global__ __launch_bounds__(256) void row_copy_vec_kernel(
    const unsigned char* __restrict__ src, int64_t ld_src, unsigned char* __restrict__ dst,
    int64_t ld_dst, const int32_t* __restrict__ ids, int64_t id_base, int64_t n,
    int64_t n_table_rows, int32_t row_bytes) {
  constexpr int kRowsPerBlock = 256 / G;
  const int lane_in_group = threadIdx.x % G;
  const int64_t k = static_cast<int64_t>(blockIdx.x) * kRowsPerBlock + threadIdx.x / G;
  if (k >= n) return;
  const int64_t r = ids ? static_cast<int64_t>(ids[k]) : k + id_base;
  if (r < 0 || r >= n_table_rows) return;  // bad id: skip the row
  const unsigned char* s = src + (SCATTER ? k : r) * ld_src;
  unsigned char* t = dst + (SCATTER ? r : k) * ld_dst;
  const int nvec = row_bytes >> 4;
  for (int v = lane_in_group; v < nvec; v += G) {
    const u32x4 x = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(s) + v);
    __builtin_nontemporal_store(x, reinterpret_cast<u32x4*>(t) + v);
  }
  const uint16_t* s2 = reinterpret_cast<const uint16_t*>(s);
  uint16_t* t2 = reinterpret_cast<uint16_t*>(t);
  for (int c = (nvec << 3) + lane_in_group; c < (row_bytes >> 1); c += G) t2[c] = s2[c];
}

// Fallback for rows that are not 16-byte aligned: 2-byte units.
template <bool SCATTER>
__global__ __launch_bounds__(256) void row_copy_elem_kernel(
    const unsigned char* __restrict__ src, int64_t ld_src, unsigned char* __restrict__ dst,
    int64_t ld_dst, const int32_t* __restrict__ ids, int64_t id_base, int64_t n,
    int64_t n_table_rows, int32_t row_bytes) {
  const int lane = threadIdx.x % kWave;
  const int64_t k = static_cast<int64_t>(blockIdx.x) * (256 / kWave) + threadIdx.x / kWave;
  if (k >= n) return;
  const int64_t r = ids ? static_cast<int64_t>(ids[k]) : k + id_base;
  if (r < 0 || r >= n_table_rows) return;
  const uint16_t* s = reinterpret_cast<const uint16_t*>(src + (SCATTER ? k : r) * ld_src);
  uint16_t* t = reinterpret_cast<uint16_t*>(dst + (SCATTER ? r : k) * ld_dst);
  for (int c = lane; c < (row_bytes >> 1); c += kWave) t[c] = s[c];
}

// sum of two elements of ES bytes (fp32, or bf16 added in fp32 and rounded to nearest-even)
__device__ __forceinline__ uint32_t add_word_bf16(uint32_t a, uint32_t b) {
  const f32x2 s = {__builtin_bit_cast(float, a << 16) + __builtin_bit_cast(float, b << 16),
                   __builtin_bit_cast(float, a & 0xffff0000u) + __builtin_bit_cast(float, b & 0xffff0000u)};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(s, bf16x2));
}

// dst[k, :] += table[ids[k], :]; rows 16-byte aligned, d elements of ES bytes.
template <int G, int ES>
__global__ __launch_bounds__(256) void row_gather_add_kernel(
    const unsigned char* __restrict__ table, int64_t ld_table, unsigned char* __restrict__ dst,
    int64_t ld_dst, const int32_t* __restrict__ ids, int64_t n, int64_t n_table_rows, int32_t d) {
  constexpr int kRowsPerBlock = 256 / G;
  constexpr int EPV = 16 / ES;
  const int lane_in_group = threadIdx.x % G;
  const int64_t k = static_cast<int64_t>(blockIdx.x) * kRowsPerBlock + threadIdx.x / G;
  if (k >= n) return;
  const int64_t r = static_cast<int64_t>(ids[k]);
  if (r < 0 || r >= n_table_rows) return;  // bad id: nothing is added to the row
  const unsigned char* s = table + r * ld_table;
  unsigned char* t = dst + k * ld_dst;
  const int nvec = d / EPV;
  for (int v = lane_in_group; v < nvec; v += G) {
    const u32x4 x = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(s) + v);
    const u32x4 y = reinterpret_cast<const u32x4*>(t)[v];
    u32x4 z;
    if constexpr (ES == 4) {
      z = __builtin_bit_cast(u32x4, __builtin_bit_cast(f32x4, x) + __builtin_bit_cast(f32x4, y));
    } else {
      z.x = add_word_bf16(x.x, y.x);
      z.y = add_word_bf16(x.y, y.y);
      z.z = add_word_bf16(x.z, y.z);
      z.w = add_word_bf16(x.w, y.w);
    }
    reinterpret_cast<u32x4*>(t)[v] = z;
  }
  for (int c = nvec * EPV + lane_in_group; c < d; c += G) {   // ragged tail, one element at a time
    if constexpr (ES == 4) {
      reinterpret_cast<float*>(t)[c] += reinterpret_cast<const float*>(s)[c];
    } else {
      const uint32_t a = reinterpret_cast<const uint16_t*>(s)[c], b = reinterpret_cast<uint16_t*>(t)[c];
      reinterpret_cast<uint16_t*>(t)[c] = static_cast<uint16_t>(add_word_bf16(a, b) & 0xffffu);
    }
  }
}

// ld_src / ld_dst in ELEMENTS of es bytes (es = 2 or 4), d elements per row.
template <bool SCATTER>
sat_status launch_row_copy(const void* src, int64_t ld_src, void* dst, int64_t ld_dst,
                           const int32_t* ids, int64_t id_base, int64_t n, int64_t n_table_rows,
                           int32_t d, int es, hipStream_t stream) {
  if (n == 0 || d == 0) return SAT_OK;
  const unsigned char* s = static_cast<const unsigned char*>(src);
  unsigned char* t = static_cast<unsigned char*>(dst);
  const int64_t lds = ld_src * es, ldd = ld_dst * es;
  const int32_t row_bytes = d * es;
  const bool vec = sat::aligned16(src) && sat::aligned16(dst) && (lds % 16 == 0) && (ldd % 16 == 0);
  if (!vec) {
    const int64_t blocks = (n + 3) / 4;
    if (blocks > INT32_MAX) return SAT_EUNSUPPORTED;
    row_copy_elem_kernel<SCATTER><<<dim3(static_cast<unsigned>(blocks)), dim3(256), 0, stream>>>(
        s, lds, t, ldd, ids, id_base, n, n_table_rows, row_bytes);
    return sat::check_launch();
  }
  const int nvec = (row_bytes + 15) / 16;
  int g = 1;
  while (g < 64 && g < nvec) g <<= 1;
  const int64_t rows_per_block = 256 / g;
  const int64_t blocks = (n + rows_per_block - 1) / rows_per_block;
  if (blocks > INT32_MAX) return SAT_EUNSUPPORTED;
  const dim3 grid(static_cast<unsigned>(blocks)), block(256);
#define SAT_ROWCOPY_CASE(G)                                                                    \
  case G:                                                                                      \
    row_copy_vec_kernel<G, SCATTER><<<grid, block, 0, stream>>>(s, lds, t, ldd, ids, id_base, n, \
                                                                n_table_rows, row_bytes);      \
    break;
  switch (g) {
    SAT_ROWCOPY_CASE(1)
    SAT_ROWCOPY_CASE(2)
    SAT_ROWCOPY_CASE(4)
    SAT_ROWCOPY_CASE(8)
    SAT_ROWCOPY_CASE(16)
    SAT_ROWCOPY_CASE(32)
    SAT_ROWCOPY_CASE(64)
  }
#undef SAT_ROWCOPY_CASE
  return sat::check_launch();
}

sat_status validate(const void* table, int64_t n_rows, int64_t ld_table, const int32_t* ids,
                    int64_t n, int32_t d, const void* dense, int64_t ld_dense, int32_t dtype) {
  if (n < 0 || d < 0 || n_rows < 0) return SAT_EINVAL;
  if (dtype != SAT_F32 && dtype != SAT_BF16) return SAT_EINVAL;
  if (n == 0 || d == 0) return SAT_OK;
  if (!table || !ids || !dense) return SAT_EINVAL;
  if (ld_table < d || ld_dense < d) return SAT_EINVAL;
  return SAT_OK;
}

}  // namespace

namespace sat {
// dst[k, 0:d) = src[(ids ? ids[k] : k + id_base), 0:d), elements of es bytes; used by the
// predictor's bypass mode.
sat_status row_gather(const void* src, int64_t ld_src, void* dst, int64_t ld_dst,
                      const int32_t* ids, int64_t id_base, int64_t n, int64_t n_src_rows,
                      int32_t d, int es, hipStream_t stream) {
  return launch_row_copy<false>(src, ld_src, dst, ld_dst, ids, id_base, n, n_src_rows, d, es,
                                stream);
}
}  // namespace sat

extern "C" sat_status sat_history_gather(const void* table, int64_t n_rows, int64_t ld_table,
                                         const int32_t* ids, int64_t n, int32_t d, void* out,
                                         int64_t ld_out, int32_t dtype, void* stream) {
  sat_status st = validate(table, n_rows, ld_table, ids, n, d, out, ld_out, dtype);
  if (st != SAT_OK) return st;
  return launch_row_copy<false>(table, ld_table, out, ld_out, ids, 0, n, n_rows, d,
                                dtype == SAT_BF16 ? 2 : 4, static_cast<hipStream_t>(stream));
}

extern "C" sat_status sat_history_push(void* table, int64_t n_rows, int64_t ld_table,
                                       const int32_t* ids, int64_t n, int32_t d, const void* H,
                                       int64_t ld_h, int32_t dtype, void* stream) {
  sat_status st = validate(table, n_rows, ld_table, ids, n, d, H, ld_h, dtype);
  if (st != SAT_OK) return st;
  return launch_row_copy<true>(H, ld_h, table, ld_table, ids, 0, n, n_rows, d,
                               dtype == SAT_BF16 ? 2 : 4, static_cast<hipStream_t>(stream));
}

extern "C" sat_status sat_history_gather_add(const void* table, int64_t n_rows, int64_t ld_table,
                                             const int32_t* ids, int64_t n, int32_t d, void* out,
                                             int64_t ld_out, int32_t dtype, void* stream) {
  sat_status st = validate(table, n_rows, ld_table, ids, n, d, out, ld_out, dtype);
  if (st != SAT_OK) return st;
  if (n == 0 || d == 0) return SAT_OK;
  const int es = dtype == SAT_BF16 ? 2 : 4;
  if (!sat::aligned16(table) || !sat::aligned16(out) || (ld_table * es) % 16 != 0 ||
      (ld_out * es) % 16 != 0)
    return SAT_EALIGN;
  const int nvec = (d * es + 15) / 16;
  int g = 1;
  while (g < 64 && g < nvec) g <<= 1;
  const int64_t rows_per_block = 256 / g;
  const int64_t blocks = (n + rows_per_block - 1) / rows_per_block;
  if (blocks > INT32_MAX) return SAT_EUNSUPPORTED;
  const dim3 grid(static_cast<unsigned>(blocks)), block(256);
  const unsigned char* s = static_cast<const unsigned char*>(table);
  unsigned char* t = static_cast<unsigned char*>(out);
  hipStream_t hs = static_cast<hipStream_t>(stream);
#define SAT_GADD_CASE(G)                                                                       \
  case G:                                                                                      \
    if (es == 4)                                                                               \
      row_gather_add_kernel<G, 4><<<grid, block, 0, hs>>>(s, ld_table * es, t, ld_out * es, ids, n, \
                                                          n_rows, d);                          \
    else                                                                                       \
      row_gather_add_kernel<G, 2><<<grid, block, 0, hs>>>(s, ld_table * es, t, ld_out * es, ids, n, \
                                                          n_rows, d);                          \
    break;
  switch (g) {
    SAT_GADD_CASE(1)
    SAT_GADD_CASE(2)
    SAT_GADD_CASE(4)
    SAT_GADD_CASE(8)
    SAT_GADD_CASE(16)
    SAT_GADD_CASE(32)
    SAT_GADD_CASE(64)
  }
#undef SAT_GADD_CASE
  return sat::check_launch();
}

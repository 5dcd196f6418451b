// Compression of stored embeddings (Sec. "Data Compression for Historical
// Embedding Storage"): every value is rounded to a number of decimal places and
// written as a variable-length run of printable characters following the
// published Encoded Polyline Algorithm Format (zigzag the signed integer, 5-bit
// groups from the low end, bit 0x20 marks "more follows", plus 63). Values are
// coded one by one (no deltas); a row of the table is the concatenation of its
// values' codes and an offset array says where each row starts.
//
// All of it is byte and integer work on top of three fp32 operations per value
// (multiply by 10^p, add 1/2, floor - each correctly rounded, never fused), so the
// codes are reproducible bit for bit. Kernels:
//   plan    one wavefront per row sums the code lengths of its values; an in-place
//           exclusive scan (2048 elements per workgroup, recursive over the workgroup
//           totals) turns the sizes into offsets, row_off[n] = total bytes;
//   encode  one wavefront per row; 64 values at a time: code length per lane,
//           wavefront prefix sum for the byte position, byte stores;
//   decode  one wavefront per requested row (gathered through an id list): the row's
//           bytes are staged in LDS; a ballot of the "last group" bits gives every
//           byte its value index; the lane holding a value's first byte assembles it
//           and stores q / 10^p (one correctly rounded division).
// HBM-bound: the dense side moves d * s bytes per row, the coded side 1 - 3 bytes
// per value.
#include "sat_internal.h"

namespace {

using sat::kWave;
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int kScanBlock = 2048;   // elements per workgroup of the scan (256 threads x 8)
constexpr int kMaxGroups = 7;      // 5-bit groups of a 32-bit zigzag value

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

template <int ES>
__device__ __forceinline__ float load_elem(const void* row, int c) {
  if constexpr (ES == 4) {
    return static_cast<const float*>(row)[c];
  } else {
    const uint32_t h = static_cast<const uint16_t*>(row)[c];
    return __builtin_bit_cast(float, h << 16);
  }
}

// zigzag code of floor(v * scale + 1/2); |q| is held at 2^30 (exact in fp32; the largest
// magnitude whose shifted code fits 32 bits for either sign: 2^31 and 2^31 - 1); +-inf and
// products that overflow land there; NaN codes as 0
__device__ __forceinline__ uint32_t zigzag_of(float v, float scale) {
  float x = floorf(__fadd_rn(__fmul_rn(v, scale), 0.5f));
  if (!(x == x)) x = 0.f;
  x = fminf(fmaxf(x, -1073741824.0f), 1073741824.0f);
  const int32_t q = static_cast<int32_t>(x);
  return (static_cast<uint32_t>(q) << 1) ^ static_cast<uint32_t>(q >> 31);
}
__device__ __forceinline__ int groups_of(uint32_t u) {
  const int bits = 32 - __builtin_clz(u | 1u);
  return (bits + 4) / 5;
}

__device__ __forceinline__ int wave_sum(int x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
  return x;
}
// inclusive prefix sum over the 64 lanes
__device__ __forceinline__ int wave_scan(int x, int lane) {
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const int y = __shfl_up(x, off);
    if (lane >= off) x += y;
  }
  return x;
}

// sizes[k] = bytes of row k's code (k < n); sizes[n] = 0
template <int ES>
__global__ __launch_bounds__(256) void code_size_kernel(const void* __restrict__ H, int64_t ld_bytes,
                                                        int64_t n, int d, float scale,
                                                        int64_t* __restrict__ sizes) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t k = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (k > n) return;
  if (k == n) {
    if (lane == 0) sizes[n] = 0;
    return;
  }
  const void* row = static_cast<const unsigned char*>(H) + k * ld_bytes;
  int acc = 0;
  for (int c = lane; c < d; c += kWave) acc += groups_of(zigzag_of(load_elem<ES>(row, c), scale));
  acc = wave_sum(acc);
  if (lane == 0) sizes[k] = acc;
}

// In-place exclusive scan of blocks of kScanBlock elements; totals[b] = sum of block b.
__global__ __launch_bounds__(256) void scan_blocks_kernel(int64_t* __restrict__ a, int64_t n,
                                                          int64_t* __restrict__ totals) {
  __shared__ int64_t sh[256];
  const int64_t base = static_cast<int64_t>(blockIdx.x) * kScanBlock + threadIdx.x * 8;
  int64_t v[8];
  int64_t sum = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    v[i] = base + i < n ? a[base + i] : 0;
    sum += v[i];
  }
  sh[threadIdx.x] = sum;
  __syncthreads();
  for (int off = 1; off < 256; off <<= 1) {   // inclusive scan of the thread sums
    const int64_t y = threadIdx.x >= off ? sh[threadIdx.x - off] : 0;
    __syncthreads();
    sh[threadIdx.x] += y;
    __syncthreads();
  }
  int64_t run = sh[threadIdx.x] - sum;        // exclusive prefix of this thread
  if (threadIdx.x == 255) totals[blockIdx.x] = sh[255];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    if (base + i < n) a[base + i] = run;
    run += v[i];
  }
}
__global__ __launch_bounds__(256) void add_block_offsets_kernel(int64_t* __restrict__ a, int64_t n,
                                                                const int64_t* __restrict__ offs) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i < n) a[i] += offs[i / kScanBlock];
}

// exclusive scan of a[0..n) in place; ws holds the totals of every level
sat_status scan_in_place(int64_t* a, int64_t n, int64_t* ws, hipStream_t st) {
  const int64_t nb = (n + kScanBlock - 1) / kScanBlock;
  if (nb > INT32_MAX) return SAT_EUNSUPPORTED;
  scan_blocks_kernel<<<dim3(static_cast<unsigned>(nb)), dim3(256), 0, st>>>(a, n, ws);
  sat_status rc = sat::check_launch();
  if (rc != SAT_OK || nb == 1) return rc;
  if ((rc = scan_in_place(ws, nb, ws + round_up(nb, 32), st)) != SAT_OK) return rc;
  add_block_offsets_kernel<<<dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0, st>>>(a, n, ws);
  return sat::check_launch();
}
int64_t scan_ws_elems(int64_t n) {
  int64_t total = 0;
  while (n > 1) {
    n = (n + kScanBlock - 1) / kScanBlock;
    total += round_up(n, 32);
    if (n == 1) break;
  }
  return total + 32;
}

template <int ES>
__global__ __launch_bounds__(256) void encode_kernel(const void* __restrict__ H, int64_t ld_bytes,
                                                     int64_t n, int d, float scale,
                                                     const int64_t* __restrict__ row_off,
                                                     uint8_t* __restrict__ codes, int64_t capacity) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t k = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (k >= n) return;
  const int64_t b0 = row_off[k], b1 = row_off[k + 1];
  if (b0 < 0 || b1 < b0 || b1 > capacity) return;   // never write outside the caller's buffer
  const void* row = static_cast<const unsigned char*>(H) + k * ld_bytes;
  int64_t pos = b0;
  for (int c0 = 0; c0 < d; c0 += kWave) {
    const int c = c0 + lane;
    uint32_t u = 0;
    int len = 0;
    if (c < d) {
      u = zigzag_of(load_elem<ES>(row, c), scale);
      len = groups_of(u);
    }
    const int incl = wave_scan(len, lane);
    int64_t p = pos + (incl - len);
    if (p + len <= b1) {   // (holds when row_off came from the plan of the same data)
      for (int j = 0; j < len; ++j) {
        const uint32_t g = (u >> (5 * j)) & 0x1Fu;
        codes[p + j] = static_cast<uint8_t>((j + 1 < len ? (g | 0x20u) : g) + 63u);
      }
    }
    pos += __shfl(incl, kWave - 1);
  }
}

// The same codes, assembled in LDS and written out in 16-byte pieces. One wavefront per row;
// a lane takes the 16 / ES values of one 16-byte load at a time, so a wavefront covers
// 64 * 16 / ES values per pass: code lengths per lane, one wavefront prefix sum for the lane's
// byte position, the bytes go to the row's image in LDS. The image sits at the same offset
// modulo 16 as the row's place in the code array (phase = row_off % 16), so that its whole
// 16-byte pieces go out as aligned 16-byte stores and only the two ends byte by byte. Needs
// the code array 16-byte aligned and rows of at most row_cap - 16 bytes of code.
template <int ES>
__global__ __launch_bounds__(256) void encode_lds_kernel(const void* __restrict__ H, int64_t ld_bytes,
                                                         int64_t n, int d, float scale,
                                                         const int64_t* __restrict__ row_off,
                                                         uint8_t* __restrict__ codes, int64_t capacity,
                                                         int row_cap) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  constexpr int VPL = 16 / ES;   // values per lane and pass
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x >> 6;
  const int64_t k = static_cast<int64_t>(blockIdx.x) * 4 + wave;
  if (k >= n) return;
  const int64_t b0 = row_off[k], b1 = row_off[k + 1];
  if (b0 < 0 || b1 < b0 || b1 > capacity) return;   // never write outside the caller's buffer
  const int phase = static_cast<int>(b0 & 15);
  if (b1 - b0 > row_cap - 16) return;               // (cannot happen: a value takes at most 7 bytes)
  const int nb = static_cast<int>(b1 - b0);
  unsigned char* mine = lds + wave * row_cap;
  const unsigned char* row = static_cast<const unsigned char*>(H) + k * ld_bytes;
  const bool row_vec = (reinterpret_cast<uintptr_t>(row) & 15u) == 0;
  int pos = phase;
  for (int c0 = 0; c0 < d; c0 += kWave * VPL) {
    const int c = c0 + lane * VPL;
    uint32_t u[VPL];
    int len[VPL];
    int total = 0;
    if (row_vec && c + VPL <= d) {
      typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
      const u32x4 w = *reinterpret_cast<const u32x4*>(row + static_cast<int64_t>(c) * ES);
      const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
      for (int j = 0; j < VPL; ++j) {
        float v;
        if constexpr (ES == 4) v = __builtin_bit_cast(float, ww[j]);
        else v = __builtin_bit_cast(float, (j & 1) ? (ww[j >> 1] & 0xffff0000u) : (ww[j >> 1] << 16));
        u[j] = zigzag_of(v, scale);
        len[j] = groups_of(u[j]);
        total += len[j];
      }
    } else {
#pragma unroll
      for (int j = 0; j < VPL; ++j) {
        u[j] = 0;
        len[j] = 0;
        if (c + j < d) {
          u[j] = zigzag_of(load_elem<ES>(row, c + j), scale);
          len[j] = groups_of(u[j]);
        }
        total += len[j];
      }
    }
    const int incl = wave_scan(total, lane);
    int p = pos + (incl - total);
    if (p + total <= phase + nb) {   // (holds when row_off came from the plan of the same data)
#pragma unroll
      for (int j = 0; j < VPL; ++j) {
        for (int g = 0; g < len[j]; ++g) {
          const uint32_t grp = (u[j] >> (5 * g)) & 0x1Fu;
          mine[p + g] = static_cast<uint8_t>((g + 1 < len[j] ? (grp | 0x20u) : grp) + 63u);
        }
        p += len[j];
      }
    }
    pos += __shfl(incl, kWave - 1);
  }
  // (a wavefront reads back only what it wrote itself: no barrier needed)
  // ---- flush: 16-byte pieces of [phase, phase + nb) relative to the aligned address below
  uint8_t* gbase = codes + (b0 - phase);             // 16-byte aligned (codes is)
  const int end = phase + nb;
  const int pieces = (end + 15) >> 4;
  for (int pc = lane; pc < pieces; pc += kWave) {
    const int lo = pc << 4, hi = lo + 16;
    if (lo >= phase && hi <= end) {
      typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
      *reinterpret_cast<u32x4*>(gbase + lo) = *reinterpret_cast<const u32x4*>(mine + lo);
    } else {
      const int a = lo > phase ? lo : phase, b = hi < end ? hi : end;
      for (int i = a; i < b; ++i) gbase[i] = mine[i];
    }
  }
}

// The values of one row whose nb bytes a wavefront has staged in LDS (`mine`): a lane per
// byte, 64 at a time; a ballot of the "last group" bits numbers the values, the lane that
// holds a value's first byte assembles it and writes element idx of the output row.
template <int ES>
__device__ __forceinline__ void decode_staged_row(const unsigned char* mine, int nb, int d, float scale,
                                                  unsigned char* orow, int lane) {
  int done = 0;                 // values completed before this chunk
  bool prev_last = true;        // the byte before this chunk ended a value (or the row starts)
  for (int base = 0; base < nb; base += kWave) {
    const int i = base + lane;
    const uint32_t b = i < nb ? static_cast<uint32_t>(mine[i]) - 63u : 0u;
    const bool last = i < nb && (b & 0x20u) == 0;
    const uint64_t m = __ballot(last);
    const uint64_t below = lane == 0 ? 0ull : (m & ((1ull << lane) - 1ull));
    const bool starts = i < nb && (lane == 0 ? prev_last : ((m >> (lane - 1)) & 1ull) != 0);
    if (starts) {
      const int idx = done + __builtin_popcountll(below);
      if (idx < d) {
        uint32_t u = 0;
        for (int j = 0; j < kMaxGroups && i + j < nb; ++j) {
          const uint32_t g = static_cast<uint32_t>(mine[i + j]) - 63u;
          u |= (g & 0x1Fu) << (5 * j);
          if ((g & 0x20u) == 0) break;
        }
        const int32_t q = static_cast<int32_t>(u >> 1) ^ -static_cast<int32_t>(u & 1u);
        const float v = __fdiv_rn(static_cast<float>(q), scale);
        if constexpr (ES == 4) {
          reinterpret_cast<float*>(orow)[idx] = v;
        } else {
          const f32x2 pr = {v, 0.f};
          const uint32_t w = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));
          reinterpret_cast<uint16_t*>(orow)[idx] = static_cast<uint16_t>(w & 0xffffu);
        }
      }
    }
    done += __builtin_popcountll(m);
    prev_last = ((m >> (kWave - 1)) & 1ull) != 0;
  }
}

// out[k, 0:d) = decoded row (ids ? ids[k] : k). A wavefront takes kDecRows consecutive k; its
// LDS slice holds one row (row_cap bytes) at a time. A row is a chain of dependent accesses
// (id, offsets, bytes, values): lanes 0..kDecRows-1 fetch ids and offsets of all the
// wavefront's rows at once, and when every row has at most kDecFast bytes (the usual case)
// the bytes of all of them are requested before the first is decoded.
constexpr int kDecRows = 4, kDecFast = 512;
template <int ES>
__global__ __launch_bounds__(256) void decode_kernel(const uint8_t* __restrict__ codes,
                                                     const int64_t* __restrict__ row_off,
                                                     int64_t n_rows, const int32_t* __restrict__ ids,
                                                     int64_t n, int d, float scale, int row_cap,
                                                     void* __restrict__ out, int64_t ld_bytes) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x >> 6;
  const int64_t k0 = (static_cast<int64_t>(blockIdx.x) * 4 + wave) * kDecRows;
  if (k0 >= n) return;
  int64_t b0_l = 0;
  int nb_l = -1;                                    // -1: nothing to do for this row
  if (lane < kDecRows && k0 + lane < n) {
    const int64_t r = ids ? static_cast<int64_t>(ids[k0 + lane]) : k0 + lane;
    if (r >= 0 && r < n_rows) {                     // bad id: the row is left alone
      b0_l = row_off[r];
      const int64_t nb64 = row_off[r + 1] - b0_l;
      if (nb64 >= 0) nb_l = nb64 > row_cap ? row_cap : static_cast<int>(nb64);   // never over 7 d bytes
    }
  }
  int64_t b0[kDecRows];
  int nb[kDecRows];
  bool fast = true;
#pragma unroll
  for (int j = 0; j < kDecRows; ++j) {
    const uint32_t lo = __builtin_amdgcn_readlane(static_cast<uint32_t>(b0_l), j);
    const uint32_t hi = __builtin_amdgcn_readlane(static_cast<uint32_t>(static_cast<uint64_t>(b0_l) >> 32), j);
    b0[j] = static_cast<int64_t>((static_cast<uint64_t>(hi) << 32) | lo);
    nb[j] = __builtin_amdgcn_readlane(nb_l, j);
    fast = fast && nb[j] <= kDecFast;
  }
  // (a wavefront reads back only what it wrote itself: no barrier needed, the LDS
  // accesses of one wavefront are ordered)
  unsigned char* mine = lds + wave * row_cap;
  unsigned char* orow = static_cast<unsigned char*>(out) + k0 * ld_bytes;
  if (fast) {
    constexpr int NC = kDecFast / kWave;
    uint8_t reg[kDecRows][NC];
#pragma unroll
    for (int j = 0; j < kDecRows; ++j)
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int i = c * kWave + lane;
        reg[j][c] = i < nb[j] ? codes[b0[j] + i] : static_cast<uint8_t>(0);
      }
#pragma unroll
    for (int j = 0; j < kDecRows; ++j) {
      if (nb[j] < 0) continue;
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int i = c * kWave + lane;
        if (i < nb[j]) mine[i] = reg[j][c];
      }
      decode_staged_row<ES>(mine, nb[j], d, scale, orow + j * ld_bytes, lane);
    }
  } else {
#pragma unroll 1
    for (int j = 0; j < kDecRows; ++j) {
      if (nb[j] < 0) continue;
      for (int i = lane; i < nb[j]; i += kWave) mine[i] = codes[b0[j] + i];
      decode_staged_row<ES>(mine, nb[j], d, scale, orow + j * ld_bytes, lane);
    }
  }
}

float scale_of(int precision) {
  float s = 1.0f;
  for (int i = 0; i < precision; ++i) s *= 10.0f;   // exact in fp32 up to 10^10
  return s;
}

sat_status check_dense(const void* p, int64_t ld, int64_t n, int32_t d, int32_t precision,
                       int32_t dtype) {
  if (n < 0 || d < 0) return SAT_EINVAL;
  if (dtype != SAT_F32 && dtype != SAT_BF16) return SAT_EINVAL;
  if (precision < 0 || precision > 9) return SAT_EINVAL;
  if (n > 0 && d > 0 && (!p || ld < d)) return SAT_EINVAL;
  return SAT_OK;
}

}  // namespace

extern "C" int64_t sat_history_compress_workspace_bytes(int64_t n) {
  if (n < 0) return 0;
  return scan_ws_elems(n + 1) * static_cast<int64_t>(sizeof(int64_t));
}

extern "C" sat_status sat_history_compress_plan(const void* H, int64_t ld_h, int64_t n, int32_t d,
                                                int32_t precision, int32_t dtype, int64_t* row_off,
                                                void* workspace, int64_t workspace_bytes,
                                                void* stream) {
  sat_status rc = check_dense(H, ld_h, n, d, precision, dtype);
  if (rc != SAT_OK) return rc;
  if (!row_off) return SAT_EINVAL;
  if (!workspace || workspace_bytes < sat_history_compress_workspace_bytes(n)) return SAT_EWORKSPACE;
  if ((reinterpret_cast<uintptr_t>(workspace) & 7u) != 0) return SAT_EALIGN;
  const int64_t blocks = (n + 1 + 3) / 4;
  if (blocks > INT32_MAX) return SAT_EUNSUPPORTED;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int es = dtype == SAT_BF16 ? 2 : 4;
  const float scale = scale_of(precision);
  if (es == 4)
    code_size_kernel<4><<<dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st>>>(H, ld_h * es, n, d,
                                                                                 scale, row_off);
  else
    code_size_kernel<2><<<dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st>>>(H, ld_h * es, n, d,
                                                                                 scale, row_off);
  if ((rc = sat::check_launch()) != SAT_OK) return rc;
  return scan_in_place(row_off, n + 1, static_cast<int64_t*>(workspace), st);
}

extern "C" sat_status sat_history_compress_encode(const void* H, int64_t ld_h, int64_t n, int32_t d,
                                                  int32_t precision, int32_t dtype,
                                                  const int64_t* row_off, uint8_t* codes,
                                                  int64_t capacity, void* stream) {
  sat_status rc = check_dense(H, ld_h, n, d, precision, dtype);
  if (rc != SAT_OK) return rc;
  if (capacity < 0) return SAT_EINVAL;
  if (n == 0 || d == 0) return SAT_OK;
  if (!row_off || (!codes && capacity > 0)) return SAT_EINVAL;
  const int64_t blocks = (n + 3) / 4;
  if (blocks > INT32_MAX) return SAT_EUNSUPPORTED;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int es = dtype == SAT_BF16 ? 2 : 4;
  const float scale = scale_of(precision);
  // rows of up to 2338 values with a 16-byte aligned code array: assembled in LDS, written in
  // 16-byte pieces; otherwise byte stores straight to memory
  const int row_cap = static_cast<int>(round_up(static_cast<int64_t>(kMaxGroups) * d, 16)) + 32;
  const int smem = 4 * row_cap;
  if (smem <= 64 * 1024 && (reinterpret_cast<uintptr_t>(codes) & 15u) == 0) {
    if (es == 4)
      encode_lds_kernel<4><<<dim3(static_cast<unsigned>(blocks)), dim3(256), smem, st>>>(
          H, ld_h * es, n, d, scale, row_off, codes, capacity, row_cap);
    else
      encode_lds_kernel<2><<<dim3(static_cast<unsigned>(blocks)), dim3(256), smem, st>>>(
          H, ld_h * es, n, d, scale, row_off, codes, capacity, row_cap);
    return sat::check_launch();
  }
  if (es == 4)
    encode_kernel<4><<<dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st>>>(H, ld_h * es, n, d, scale,
                                                                              row_off, codes, capacity);
  else
    encode_kernel<2><<<dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st>>>(H, ld_h * es, n, d, scale,
                                                                              row_off, codes, capacity);
  return sat::check_launch();
}

extern "C" sat_status sat_history_decompress(const uint8_t* codes, const int64_t* row_off,
                                             int64_t n_rows, const int32_t* ids, int64_t n, int32_t d,
                                             int32_t precision, int32_t dtype, void* out,
                                             int64_t ld_out, void* stream) {
  sat_status rc = check_dense(out, ld_out, n, d, precision, dtype);
  if (rc != SAT_OK) return rc;
  if (n_rows < 0) return SAT_EINVAL;
  if (n == 0 || d == 0) return SAT_OK;
  if (!codes || !row_off) return SAT_EINVAL;
  const int row_cap = static_cast<int>(round_up(static_cast<int64_t>(kMaxGroups) * d, 16));
  const int smem = 4 * row_cap;
  if (smem > 64 * 1024) return SAT_EUNSUPPORTED;   // rows wider than 2340 values
  const int64_t blocks = (n + 4 * kDecRows - 1) / (4 * kDecRows);
  if (blocks > INT32_MAX) return SAT_EUNSUPPORTED;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int es = dtype == SAT_BF16 ? 2 : 4;
  const float scale = scale_of(precision);
  if (es == 4)
    decode_kernel<4><<<dim3(static_cast<unsigned>(blocks)), dim3(256), smem, st>>>(
        codes, row_off, n_rows, ids, n, d, scale, row_cap, out, ld_out * es);
  else
    decode_kernel<2><<<dim3(static_cast<unsigned>(blocks)), dim3(256), smem, st>>>(
        codes, row_off, n_rows, ids, n, d, scale, row_cap, out, ld_out * es);
  return sat::check_launch();
}

// Second half of the predictor's hop (Eq. 7; Sec. "Embedding Predictor"):
//   out[m, :] = add[row(m), :] + Agg[m, 0:DS) * Wg        Agg [M, DS], Wg [DS, d], fp32
// i.e. the aggregated LSTM states times the hop's weight matrix plus the newest
// cached embedding (the residual), written to the predicted rows.
//
// M is in the millions, DS is 32 or 64: two flops per 16 bytes moved, so this is a
// streaming kernel and the products only have to stay out of the way. Layout of the
// work, weights-stationary:
//   * a workgroup has 8 wavefronts; wavefront w owns output columns [32 w, 32 w + 32)
//     of a group of 256 and keeps ITS slice of Wg in registers for the whole
//     workgroup, already split into the three bf16 pieces of the exact fp32 product
//     (mx_tile.h) and already in MFMA operand order: 48 registers for DS = 64;
//   * rows are streamed in tiles of 32: the tile of Agg (8 KiB) is read with one
//     16-byte access per thread, split and staged in LDS (double-buffered, one
//     barrier per tile); each wavefront multiplies it with its weight slice;
//   * the product tile goes through LDS so that the residual rows (random rows of the
//     history table, fetched through the id list) and the output rows move as 16-byte
//     accesses, whole rows per 64 lanes; the residual rows are requested BEFORE the
//     products of the tile and added after them, and the next tile of Agg is in flight
//     meanwhile. Two workgroups fit a compute unit (registers capped at 128), which is
//     what keeps enough bytes in flight.
#include "mx_tile.h"
#include "sat_internal.h"

namespace {

using namespace sat::mx;

constexpr int kTilesPerBlock = 8;   // 32-row tiles per workgroup (256 rows)

// ESO = bytes per element of the residual rows and of the output (4: fp32, 2: bf16, the
// sum rounded to nearest-even once); Agg and Wg are fp32 either way. `add` and `out` may be the
// same matrix with row(m) = m (a thread reads the 16 bytes it later writes, and no others of
// that row), so neither is declared free of aliases.
template <int DS, int ESO>
__global__ __launch_bounds__(512, 4) void hop_product_kernel(
    const float* __restrict__ Agg, int64_t M, const float* __restrict__ Wg, int d,
    const void* add, int64_t ld_add, const int32_t* __restrict__ add_ids,
    int64_t add_base, int64_t add_rows, void* out, int64_t ld_out) {
  constexpr int NP = 3;
  constexpr int KC = DS / 16;                       // 16-wide k chunks
  constexpr int NCH = DS / 32;                      // 32-wide staging chunks
  constexpr int STAGE = NCH * tile_bytes<32, NP>(); // bytes of one staged Agg tile
  constexpr int C_LDF = 256 + 4;                    // floats per staged output row
  __shared__ __attribute__((aligned(16))) unsigned char As[2 * STAGE];
  __shared__ __attribute__((aligned(16))) float Cs[32 * C_LDF];

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int col = blockIdx.y * 256 + 32 * wave + (lane & 31);
  const bool col_ok = col < d;
  const int64_t row_lo = static_cast<int64_t>(blockIdx.x) * (32 * kTilesPerBlock);

  // ---- this wavefront's slice of Wg as MFMA B fragments: lane holds k = 16 kc + 8 (lane / 32)
  // .. + 7 of column `col`, split into three pieces
  bf16x8 bw[KC][NP];
#pragma unroll
  for (int kc = 0; kc < KC; ++kc) {
    float e[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int k = 16 * kc + 8 * (lane >> 5) + j;
      e[j] = col_ok ? Wg[static_cast<int64_t>(k) * d + col] : 0.f;
    }
    uint32_t q[4][NP];
#pragma unroll
    for (int h = 0; h < 4; ++h) split2<NP>(e[2 * h], e[2 * h + 1], q[h]);
#pragma unroll
    for (int p = 0; p < NP; ++p)
      bw[kc][p] = __builtin_bit_cast(bf16x8, u32x4{q[0][p], q[1][p], q[2][p], q[3][p]});
  }

  // ---- Agg tile: 32 rows x DS floats = 8 DS 16-byte accesses, one per thread (t < 8 DS)
  const int a_row = t / (DS / 4), a_k = (t % (DS / 4)) * 4;
  const bool a_thread = t < 8 * DS;
  auto load_a = [&](int64_t row0) {
    u32x4 v = {0u, 0u, 0u, 0u};
    const int64_t r = row0 + a_row;
    if (a_thread && r < M) v = *reinterpret_cast<const u32x4*>(Agg + r * DS + a_k);
    return v;
  };
  auto store_a = [&](const u32x4 v, int stage) {
    if (!a_thread) return;
    const f32x4 f = __builtin_bit_cast(f32x4, v);
    uint32_t lo[NP], hi[NP];
    split2<NP>(f.x, f.y, lo);
    split2<NP>(f.z, f.w, hi);
    const int kk = a_k & 31;
    unsigned char* s = As + stage * STAGE + (a_k >> 5) * tile_bytes<32, NP>() + swz(a_row, kk >> 3) +
                       (((kk >> 2) & 1) << 3);
#pragma unroll
    for (int p = 0; p < NP; ++p) *reinterpret_cast<u32x2*>(s + p * piece_bytes<32>()) = u32x2{lo[p], hi[p]};
  };

  // Chunk c = t + 512 i of a tile lies in row c / 64 = wave + 8 i: the same for the whole wavefront.
  // Lanes 0..3 fetch the ids of the wavefront's four rows, one tile ahead (so the id list's
  // latency is never waited for), and the rows' table rows are read out of those lanes.
  auto load_ids = [&](int64_t row0) __attribute__((always_inline)) {
    const int64_t r = row0 + wave + 8 * (lane & 3);
    int32_t v = -1;
    if (add_ids != nullptr && r < M) v = add_ids[r];
    return v;
  };
  int32_t id_next = load_ids(row_lo);
  u32x4 ra = load_a(row_lo);
  store_a(ra, 0);
  __syncthreads();
  for (int it = 0; it < kTilesPerBlock; ++it) {
    const int64_t row0 = row_lo + 32 * it;
    if (row0 >= M) break;                        // uniform over the workgroup
    const int stage = it & 1;
    const bool more = it + 1 < kTilesPerBlock && row0 + 32 < M;
    const int32_t id_cur = id_next;
    if (more) {
      id_next = load_ids(row0 + 32);
      ra = load_a(row0 + 32);
    }
    // residual rows of this tile: requested now, used after the products. Thread t owns the
    // 16-byte chunks c = t + 512 i of the 32 x 256 tile: row c / 64, columns 4 (c % 64) .. + 3.
    f32x4 res[4];
    bool ok[4];
    int64_t srcs[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t r = row0 + wave + 8 * i;
      int64_t sr = -1;
      if (r < M)
        sr = add_ids ? static_cast<int64_t>(__builtin_amdgcn_readlane(id_cur, i)) : add_base + r;
      srcs[i] = sr;
    }
    const int cc = blockIdx.y * 256 + (lane << 2);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t src = srcs[i] < add_rows ? srcs[i] : -1;    // bad id (negative or too large): the row is left alone
      ok[i] = src >= 0 && cc < d;
      res[i] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (ok[i]) {
        if constexpr (ESO == 4) {
          res[i] = *reinterpret_cast<const f32x4*>(static_cast<const float*>(add) + src * ld_add + cc);
        } else {   // four bf16: kept raw in the first two lanes of res until they are added
          const u32x2 w = *reinterpret_cast<const u32x2*>(static_cast<const uint16_t*>(add) +
                                                          src * ld_add + cc);
          // (scalars first: a bit cast applied directly to a vector element reads element 0)
          const uint32_t wx = w.x, wy = w.y;
          res[i].x = __builtin_bit_cast(float, wx);
          res[i].y = __builtin_bit_cast(float, wy);
        }
      }
    }
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    const unsigned char* S = As + stage * STAGE;
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      bf16x8 a[NP];
#pragma unroll
      for (int p = 0; p < NP; ++p)
        a[p] = read_operand(S + (kc >> 1) * tile_bytes<32, NP>() + p * piece_bytes<32>(), 0, kc & 1, lane);
#pragma unroll
      for (int q = 0; q < n_products<NP>(); ++q)
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[product_a<NP>(q)], bw[kc][product_b<NP>(q)], acc,
                                                      0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) Cs[acc_row(r, lane) * C_LDF + 32 * wave + (lane & 31)] = acc[r];
    __syncthreads();
    // sums first (one wait for the residual rows), then the stores back to back
    f32x4 sum[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = t + 512 * i;
      f32x4 v = *reinterpret_cast<const f32x4*>(&Cs[(c >> 6) * C_LDF + ((c & 63) << 2)]);
      if constexpr (ESO == 4) {
        v += res[i];
      } else {
        const float rx = res[i].x, ry = res[i].y;
        const uint32_t w0 = __builtin_bit_cast(uint32_t, rx), w1 = __builtin_bit_cast(uint32_t, ry);
        v.x += low_as_f32(w0);
        v.y += high_as_f32(w0);
        v.z += low_as_f32(w1);
        v.w += high_as_f32(w1);
      }
      sum[i] = v;
    }
    // (keeps the four sums, and with them the one wait for the residual rows, in front of the
    // stores: sunk into the guarded blocks below, each sum would wait for the previous row's
    // stores to complete as well)
    asm volatile("" : "+v"(sum[0]), "+v"(sum[1]), "+v"(sum[2]), "+v"(sum[3]));
    const int left = d - cc;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (!ok[i]) continue;
      const int64_t r = row0 + wave + 8 * i;
      const f32x4 v = sum[i];
      if constexpr (ESO == 4) {
        float* y = static_cast<float*>(out) + r * ld_out + cc;
        if (left >= 4) {
          *reinterpret_cast<f32x4*>(y) = v;
        } else {
          y[0] = v.x;
          if (left > 1) y[1] = v.y;
          if (left > 2) y[2] = v.z;
        }
      } else {
        const u32x2 w = {pack_bf16(v.x, v.y), pack_bf16(v.z, v.w)};
        uint16_t* y = static_cast<uint16_t*>(out) + r * ld_out + cc;
        if (left >= 4) {
          *reinterpret_cast<u32x2*>(y) = w;
        } else {
          y[0] = static_cast<uint16_t>(w.x & 0xffffu);
          if (left > 1) y[1] = static_cast<uint16_t>(w.x >> 16);
          if (left > 2) y[2] = static_cast<uint16_t>(w.y & 0xffffu);
        }
      }
    }
    if (more) store_a(ra, stage ^ 1);
    __syncthreads();
  }
}

}  // namespace

namespace sat {

// out[m, 0:d) = add[(add_ids ? add_ids[m] : add_base + m), 0:d) + Agg[m, 0:ds) Wg, m < M; rows
// whose table row falls outside [0, add_rows) are not written. Agg and Wg fp32; add and out
// elements of eso bytes (4 fp32, 2 bf16), ld in elements; ds = 32 or 64.
sat_status launch_hop_product(const float* Agg, int64_t M, int32_t ds, const float* Wg, int32_t d,
                              const void* add, int64_t ld_add, const int32_t* add_ids,
                              int64_t add_base, int64_t add_rows, void* out, int64_t ld_out, int eso,
                              hipStream_t st) {
  if (M == 0 || d == 0) return SAT_OK;
  const int64_t gx = (M + 32 * kTilesPerBlock - 1) / (32 * kTilesPerBlock);
  if (gx > INT32_MAX) return SAT_EUNSUPPORTED;
  if ((ds != 32 && ds != 64) || (eso != 2 && eso != 4)) return SAT_EUNSUPPORTED;
  const dim3 grid(static_cast<unsigned>(gx), static_cast<unsigned>((d + 255) / 256));
#define SAT_HOP(DS, ESO)                                                                          \
  hop_product_kernel<DS, ESO><<<grid, dim3(512), 0, st>>>(Agg, M, Wg, d, add, ld_add, add_ids,      \
                                                          add_base, add_rows, out, ld_out)
  if (ds == 64 && eso == 4) SAT_HOP(64, 4);
  else if (ds == 64) SAT_HOP(64, 2);
  else if (eso == 4) SAT_HOP(32, 4);
  else SAT_HOP(32, 2);
#undef SAT_HOP
  return sat::check_launch();
}

}  // namespace sat

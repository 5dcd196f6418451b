// Normalised-adjacency aggregation AGG = [P_in | P_out] * Hbar (appendix, SAT
// forward) and its transpose products (appendix, SAT backward).
//
// The work is a gather of nnz feature rows: 2 flops per 4 gathered bytes, so
// the memory system is the only bound and the design goal is bytes in flight,
// whatever the degree distribution looks like.
//
// spmm_stream_kernel (entry-balanced row split):
//   * a workgroup of 8 wavefronts owns R consecutive CSR rows; their entries
//     are one contiguous span of the index arrays, which is cut into 8 equal
//     pieces, one per wavefront, regardless of where rows begin and end. A hub
//     row is thereby spread over the wavefronts of its workgroup, and a
//     wavefront never idles because its row happened to be short;
//   * all 64 lanes cover one feature row (4, 8 or 16 bytes per lane and up to
//     4 such chunks, so 256 B .. 4 KiB rows are one entry per access);
//   * the entry list is consumed as a stream through a ring of U gathers in
//     flight: as soon as the oldest gather has been added to the running row
//     sum its registers are refilled with the entry U positions ahead, across
//     row boundaries. Column ids and values are read 64 at a time, one chunk
//     ahead, and handed out with cross-lane reads into scalar registers;
//   * a row ends when the stream position passes its end offset (a scalar
//     compare per entry): the running sum is stored and cleared. Rows without
//     entries are stored as zeros on the way;
//   * a row cut by a piece boundary leaves partial sums in LDS; after a
//     barrier they are added in wavefront order (deterministic, no atomics);
//   * entries whose column id is outside the operand (the halo columns, when
//     the transpose product P_in^T walks only local columns) are squeezed out
//     of each 64-entry chunk before the ring sees them.
// spmm_slot_kernel: the same split for rows of at most 256 bytes, several entries per
//   gather instruction (a group of lanes per row), because there the wavefront's per-entry
//   bookkeeping, not memory, is what one entry per instruction waits for.
// spmm_group_kernel: rows of a handful of entries and narrow features (the
//   transposed halo block of the predictor's hop): a group of G lanes per row,
//   64/G rows per wavefront, because there the number of independent rows in
//   flight is what sets the speed.
// The same code serves P_in^T (P_in being symmetric), P_out^T (through the
// transposed halo block) and the predictor's hop (transposed halo block plus a
// diagonal term).
#include "sat_internal.h"

namespace {

using sat::kWave;
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int kWaves = 8;            // wavefronts per workgroup
constexpr int kMaxRowsPerBlock = 128;
constexpr int32_t kEnd = 0x7fffffff;
constexpr int kFold = 32;            // entries summed into one first-level partial sum

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {  // two RNE bf16, lo in the low half
  const f32x2 pr = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));
}

// NW consecutive 32-bit words of a feature row, held as fp32. ES = bytes per
// element: 4 (fp32: NW elements) or 2 (bf16: 2*NW elements, kept de-interleaved:
// lo = even elements, hi = odd elements, so widening is one shift and one mask
// on the whole vector). Sums are carried in fp32; bf16 results are rounded to
// nearest-even once, when the output row is stored.
template <int ES, int NW>
struct Piece {
  typedef float F __attribute__((ext_vector_type(NW)));
  typedef uint32_t W __attribute__((ext_vector_type(NW)));
  static constexpr int N = NW * 4 / ES;   // elements
  static constexpr int NQ = 4 / ES == 2 ? 2 : 1;
  F q[NQ];
  __device__ __forceinline__ void zero() {
#pragma unroll
    for (int k = 0; k < NQ; ++k) q[k] = F(0.f);
  }
  static __device__ __forceinline__ W load_raw(const unsigned char* p) {
    return *reinterpret_cast<const W*>(p);
  }
  __device__ __forceinline__ void load(const unsigned char* p) { widen(load_raw(p)); }
  __device__ __forceinline__ void widen(const W w) {
    if constexpr (ES == 4) {
      q[0] = __builtin_bit_cast(F, w);
    } else {
      q[0] = __builtin_bit_cast(F, w << 16);
      q[1] = __builtin_bit_cast(F, w & 0xffff0000u);
    }
  }
  __device__ __forceinline__ void fma(float s, const Piece& x) {
#pragma unroll
    for (int k = 0; k < NQ; ++k) q[k] += s * x.q[k];
  }
  __device__ __forceinline__ void keep_if(bool keep) {   // per lane: zero unless keep
#pragma unroll
    for (int k = 0; k < NQ; ++k)
#pragma unroll
      for (int i = 0; i < NW; ++i) q[k][i] = keep ? q[k][i] : 0.f;
  }
  __device__ __forceinline__ void add(const Piece& x) {
#pragma unroll
    for (int k = 0; k < NQ; ++k) q[k] += x.q[k];
  }
  __device__ __forceinline__ void xor_add(int off) {
#pragma unroll
    for (int k = 0; k < NQ; ++k)
#pragma unroll
      for (int i = 0; i < NW; ++i) q[k][i] += __shfl_xor(q[k][i], off);
  }
  // raw fp32 image (N floats) for LDS partial sums
  __device__ __forceinline__ void to_lds(float* p) const {
#pragma unroll
    for (int k = 0; k < NQ; ++k) *reinterpret_cast<F*>(p + NW * k) = q[k];
  }
  __device__ __forceinline__ void from_lds(const float* p) {
#pragma unroll
    for (int k = 0; k < NQ; ++k) q[k] = *reinterpret_cast<const F*>(p + NW * k);
  }
  // store the first min(left, N) elements at p (p aligned to 4 * NW bytes)
  __device__ __forceinline__ void store(unsigned char* p, int left) const {
    W w;
    if constexpr (ES == 4) {
      w = __builtin_bit_cast(W, q[0]);
    } else {
#pragma unroll
      for (int i = 0; i < NW; ++i) w[i] = pack2(q[0][i], q[1][i]);
    }
    if (left >= N) {
      *reinterpret_cast<W*>(p) = w;
    } else if constexpr (ES == 4) {
      uint32_t* y = reinterpret_cast<uint32_t*>(p);
#pragma unroll
      for (int i = 0; i < NW; ++i)
        if (i < left) y[i] = w[i];
    } else {
      uint16_t* y = reinterpret_cast<uint16_t*>(p);
#pragma unroll
      for (int i = 0; i < NW; ++i) {
        if (2 * i < left) y[2 * i] = static_cast<uint16_t>(w[i] & 0xffffu);
        if (2 * i + 1 < left) y[2 * i + 1] = static_cast<uint16_t>(w[i] >> 16);
      }
    }
  }
};

template <int ES>
using Chunk = Piece<ES, 4>;   // 16 bytes of a row

struct SpmmArgs {
  const int64_t* row_begin;  // row i is entries [row_begin[i], row_end[i]) ...
  const int64_t* row_end;
  const int64_t* rowptr;     // ... a prefix of [rowptr[i], rowptr[i+1]); entries of that range
                             // at or after row_end[i] have col >= n_x_rows
  const int32_t* col;
  const float* val;
  const unsigned char* X;  // [n_x_rows, ld_x] elements of ES bytes
  int64_t ld_x;            // bytes
  int64_t n_x_rows;
  unsigned char* Y;        // [n_rows, ld_y]
  int64_t ld_y;            // bytes
  int64_t n_rows;
  int32_t d;               // elements per row
  int32_t rows_per_block;  // stream kernel: R rows per workgroup for the first n_big_blocks
  int32_t n_big_blocks;    // workgroups, R / 4 rows for the rest (see launch_spmm_es)
  const float* self_val;   // nullable: Y[i] += self_val[i] * X[self_off + i]
  int64_t self_off;
};

__device__ __forceinline__ int rl(int v, int lane) { return __builtin_amdgcn_readlane(v, lane); }
__device__ __forceinline__ float rlf(float v, int lane) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

template <int ES, int NW, int NCH, int U>
__global__ __launch_bounds__(kWaves * kWave) void spmm_stream_kernel(SpmmArgs a) {
  typedef Piece<ES, NW> P;
  constexpr int EPL = P::N;                       // elements per lane per chunk
  constexpr int kPassElems = kWave * EPL * NCH;   // elements of a row covered by one pass
  __shared__ int64_t rp[kMaxRowsPerBlock + 1];
  __shared__ int32_t head_row[kWaves], head_closed[kWaves], tail_row[kWaves];
  __shared__ __attribute__((aligned(16))) float part[kWaves][2][kPassElems];

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int big = a.rows_per_block, nbig = a.n_big_blocks;
  const int bid = blockIdx.x;
  const int R = bid < nbig ? big : big / 4;
  const int64_t row0 = bid < nbig ? static_cast<int64_t>(bid) * big
                                  : static_cast<int64_t>(nbig) * big + static_cast<int64_t>(bid - nbig) * R;
  const int nr = static_cast<int>(a.n_rows - row0 < R ? a.n_rows - row0 : R);
  const int col_base = blockIdx.y * kPassElems;

  for (int t = threadIdx.x; t <= nr; t += kWaves * kWave) rp[t] = a.rowptr[row0 + t];
  if (threadIdx.x < kWaves) {
    head_row[threadIdx.x] = -1;
    head_closed[threadIdx.x] = 0;
    tail_row[threadIdx.x] = -1;
  }
  __syncthreads();

  // this lane's slice of a row: element offsets and validity per chunk
  int el0[NCH];
#pragma unroll
  for (int ch = 0; ch < NCH; ++ch) el0[ch] = col_base + (ch * kWave + lane) * EPL;

  auto store_row = [&](int r, P (&acc)[NCH]) {   // final value of local row r of this workgroup
    const int64_t row = row0 + r;
    if (a.self_val != nullptr) {
      const float sv = a.self_val[row];
      const unsigned char* xr = a.X + (a.self_off + row) * a.ld_x;
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch)
        if (el0[ch] < a.d) {
          P x;
          x.load(xr + static_cast<int64_t>(el0[ch]) * ES);
          acc[ch].fma(sv, x);
        }
    }
    unsigned char* yr = a.Y + row * a.ld_y;
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      const int left = a.d - el0[ch];
      if (left > 0) acc[ch].store(yr + static_cast<int64_t>(el0[ch]) * ES, left);
    }
  };

  const int64_t e0 = rp[0];
  const int32_t total = static_cast<int32_t>(rp[nr] - e0);   // < 2^31: checked by the host
  const int32_t per = ((total + kWaves - 1) / kWaves + kWave - 1) / kWave * kWave;
  const int32_t ps = wave * per;                                  // offsets relative to e0
  const int32_t pe = ps + per < total ? ps + per : total;

  if (wave == 0 || ps < total) {
    // first row of this piece: rows that end at or before ps belong to earlier pieces
    int cur = 0;
    if (wave != 0)
      for (int k0 = 0; k0 < nr; k0 += kWave) {
        const int k = k0 + lane;
        cur += __builtin_popcountll(__ballot(k < nr && static_cast<int32_t>(rp[k + 1] - e0) <= ps));
      }
    cur = __builtin_amdgcn_readfirstlane(cur);
    const int first = cur;
    const bool head_partial =
        __builtin_amdgcn_readfirstlane(static_cast<int32_t>(rp[cur < nr ? cur : nr] - e0)) < ps;
    int32_t cur_end =
        cur < nr ? __builtin_amdgcn_readfirstlane(static_cast<int32_t>(rp[cur + 1] - e0)) : kEnd;

    // Two-level sum: `acc` takes the products of up to kFold entries, then is folded into
    // `tot`. A plain running sum over a hub row's thousand-odd entries of one piece lets
    // the rounding errors of like-signed terms pile up linearly.
    P acc[NCH], tot[NCH];
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      acc[ch].zero();
      tot[ch].zero();
    }
    int rounds = 0;

    auto flush = [&]() {   // row `cur` ends inside this piece
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) acc[ch].add(tot[ch]);
      if (cur == first && head_partial) {
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) acc[ch].to_lds(&part[wave][0][(ch * kWave + lane) * EPL]);
        if (lane == 0) {
          head_row[wave] = cur;
          head_closed[wave] = 1;
        }
      } else {
        store_row(cur, acc);
      }
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) {
        acc[ch].zero();
        tot[ch].zero();
      }
      ++cur;
      cur_end = cur < nr ? __builtin_amdgcn_readfirstlane(static_cast<int32_t>(rp[cur + 1] - e0)) : kEnd;
    };

    // ---- index chunks: `c, v, p` hold the current 64 (squeezed) entries, `rc, rv` the raw next ones
    int32_t c = 0, p = 0, rc = 0;
    float v = 0.f, rv = 0.f;
    int cnt = 0, idx = 0;             // entries in the current chunk / next one to hand out
    int32_t raw_base = ps;            // offset of the raw chunk
    bool has_raw = ps < pe;
    auto load_raw = [&]() {
      const int32_t o = raw_base + lane;
      rc = -1;
      rv = 0.f;
      if (o < pe) {
        rc = a.col[e0 + o];
        rv = a.val[e0 + o];
      }
    };
    if (has_raw) load_raw();
    auto shift = [&]() {              // raw chunk -> current chunk (squeezed), fetch the following raw chunk
      const bool ok = static_cast<uint32_t>(rc) < static_cast<uint64_t>(a.n_x_rows);
      const uint64_t mask = __ballot(ok);
      cnt = __builtin_popcountll(mask);
      const int32_t o = raw_base + lane;
      const int n_raw = pe - raw_base < kWave ? pe - raw_base : kWave;
      if (cnt == n_raw) {             // nothing to squeeze out (valid entries are lanes 0..n_raw-1)
        c = rc;
        v = rv;
        p = o;
      } else {
        const int below = __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                                    __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0));
        const int dest = (ok ? below : cnt + (lane - below)) << 2;
        c = __builtin_amdgcn_ds_permute(dest, rc);
        v = __builtin_bit_cast(float, __builtin_amdgcn_ds_permute(dest, __builtin_bit_cast(int, rv)));
        p = __builtin_amdgcn_ds_permute(dest, o);
      }
      idx = 0;
      raw_base += kWave;
      has_raw = raw_base < pe;
      if (has_raw) load_raw();
    };

    // ---- ring of U gathers
    typename P::W x[U][NCH];          // raw words; widened to fp32 when they are added
    float sv[U];
    int32_t sp[U];
    auto fetch = [&](int u) {
      while (idx >= cnt) {
        if (!has_raw) {
          sp[u] = kEnd;
          return;
        }
        shift();
      }
      const int32_t cj = rl(c, idx);
      sv[u] = rlf(v, idx);
      sp[u] = rl(p, idx);
      ++idx;
      const unsigned char* xr = a.X + static_cast<int64_t>(cj) * a.ld_x;
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) {
        if (el0[ch] < a.d)
          x[u][ch] = P::load_raw(xr + static_cast<int64_t>(el0[ch]) * ES);
        else
          x[u][ch] = typename P::W(0u);
      }
    };
#pragma unroll
    for (int u = 0; u < U; ++u) fetch(u);
    bool more = true;
    while (more) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (sp[u] == kEnd) {
          more = false;
          break;
        }
        while (sp[u] >= cur_end) flush();
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
          P xw;
          xw.widen(x[u][ch]);
          acc[ch].fma(sv[u], xw);
        }
        fetch(u);
      }
      if (++rounds == kFold / U) {
        rounds = 0;
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
          tot[ch].add(acc[ch]);
          acc[ch].zero();
        }
      }
    }
    // rows that end inside this piece after its last entry (trailing skipped entries, empty rows)
    while (cur < nr && cur_end <= pe) flush();
    // a row that continues into the next piece
    if (cur < nr && __builtin_amdgcn_readfirstlane(static_cast<int32_t>(rp[cur] - e0)) < pe) {
      const int slot = (cur == first && head_partial) ? 0 : 1;
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) acc[ch].add(tot[ch]);
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) acc[ch].to_lds(&part[wave][slot][(ch * kWave + lane) * EPL]);
      if (lane == 0) {
        if (slot == 0)
          head_row[wave] = cur;   // the whole piece lies inside one row; head_closed stays 0
        else
          tail_row[wave] = cur;
      }
    }
  }
  __syncthreads();

  // ---- rows cut by piece boundaries: the wavefront in whose piece the row ended adds the
  // partial sums in piece order: the tail of the piece it began in, then the heads after it
  if (head_row[wave] >= 0 && head_closed[wave]) {
    int ws = -1;
    for (int k = 0; k < wave; ++k)
      if (tail_row[k] >= 0) ws = k;
    if (ws >= 0) {
      P sum[NCH], other;
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) sum[ch].from_lds(&part[ws][1][(ch * kWave + lane) * EPL]);
      for (int k = ws + 1; k <= wave; ++k) {
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
          other.from_lds(&part[k][0][(ch * kWave + lane) * EPL]);
          sum[ch].add(other);
        }
      }
      store_row(head_row[wave], sum);
    }
  }
}

// Rows of at most 512 bytes: the same entry-balanced split of a workgroup's span into eight
// pieces, but the stream is consumed a SLOT at a time: a group of G lanes (16 bytes per
// lane) covers one feature row, so one gather instruction fetches the rows of 64 / G
// consecutive entries, each group with its own entry's column id, weight and stream position
// (cross-lane reads of the 64-entry index chunk). With one entry per instruction the
// wavefront's per-entry bookkeeping - three cross-lane reads into scalar registers, the
// scalar address, the row-end compare - is what short rows wait for (the counters show few
// requests in flight and no translation misses); here it is paid once per slot. A lane
// accumulates its group's entries; when a row ends the groups' partial sums are added across
// the wavefront and group 0 stores the row. A row that ends inside a slot is handled by
// weight masks: entries at or past the row's end are held back until the row has been
// stored. Everything else (pieces, rows cut by piece boundaries, the squeeze of out-of-range
// columns, two-level sums) is as in spmm_stream_kernel.
template <int ES, int G, int U>
__global__ __launch_bounds__(kWaves * kWave) void spmm_slot_kernel(SpmmArgs a) {
  typedef Chunk<ES> P;
  constexpr int EPL = P::N;                 // elements per lane
  constexpr int EPI = kWave / G;            // entries per gather instruction
  constexpr int kRowElems = G * EPL;        // elements of a row one pass covers
  __shared__ int64_t rp[kMaxRowsPerBlock + 1];
  __shared__ int32_t head_row[kWaves], head_closed[kWaves], tail_row[kWaves];
  __shared__ __attribute__((aligned(16))) float part[kWaves][2][kRowElems];

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int gl = lane % G, grp = lane / G;
  const int big = a.rows_per_block, nbig = a.n_big_blocks;
  const int bid = blockIdx.x;
  const int R = bid < nbig ? big : big / 4;
  const int64_t row0 = bid < nbig ? static_cast<int64_t>(bid) * big
                                  : static_cast<int64_t>(nbig) * big + static_cast<int64_t>(bid - nbig) * R;
  const int nr = static_cast<int>(a.n_rows - row0 < R ? a.n_rows - row0 : R);

  for (int t = threadIdx.x; t <= nr; t += kWaves * kWave) rp[t] = a.rowptr[row0 + t];
  if (threadIdx.x < kWaves) {
    head_row[threadIdx.x] = -1;
    head_closed[threadIdx.x] = 0;
    tail_row[threadIdx.x] = -1;
  }
  __syncthreads();

  const int el0 = gl * EPL;                 // this lane's elements of a row
  const bool el_ok = el0 < a.d;

  auto store_row = [&](int r, P& sum) {     // final value of local row r; group 0 holds it
    if (grp != 0 || !el_ok) return;
    const int64_t row = row0 + r;
    if (a.self_val != nullptr) {
      P x;
      x.load(a.X + (a.self_off + row) * a.ld_x + static_cast<int64_t>(el0) * ES);
      sum.fma(a.self_val[row], x);
    }
    sum.store(a.Y + row * a.ld_y + static_cast<int64_t>(el0) * ES, a.d - el0);
  };
  auto across_groups = [&](P& x) {          // every lane ends up with the sum over the groups
#pragma unroll
    for (int off = G; off < kWave; off <<= 1) x.xor_add(off);
  };

  const int64_t e0 = rp[0];
  const int32_t total = static_cast<int32_t>(rp[nr] - e0);   // < 2^31: checked by the host
  const int32_t per = ((total + kWaves - 1) / kWaves + kWave - 1) / kWave * kWave;
  const int32_t ps = wave * per;                                  // offsets relative to e0
  const int32_t pe = ps + per < total ? ps + per : total;

  if (wave == 0 || ps < total) {
    int cur = 0;
    if (wave != 0)
      for (int k0 = 0; k0 < nr; k0 += kWave) {
        const int k = k0 + lane;
        cur += __builtin_popcountll(__ballot(k < nr && static_cast<int32_t>(rp[k + 1] - e0) <= ps));
      }
    cur = __builtin_amdgcn_readfirstlane(cur);
    const int first = cur;
    const bool head_partial =
        __builtin_amdgcn_readfirstlane(static_cast<int32_t>(rp[cur < nr ? cur : nr] - e0)) < ps;
    int32_t cur_end =
        cur < nr ? __builtin_amdgcn_readfirstlane(static_cast<int32_t>(rp[cur + 1] - e0)) : kEnd;

    P acc, tot;
    acc.zero();
    tot.zero();
    int rounds = 0;

    auto flush = [&]() {   // row `cur` ends inside this piece
      acc.add(tot);
      across_groups(acc);
      if (cur == first && head_partial) {
        if (grp == 0) acc.to_lds(&part[wave][0][el0]);
        if (lane == 0) {
          head_row[wave] = cur;
          head_closed[wave] = 1;
        }
      } else {
        store_row(cur, acc);
      }
      acc.zero();
      tot.zero();
      ++cur;
      cur_end = cur < nr ? __builtin_amdgcn_readfirstlane(static_cast<int32_t>(rp[cur + 1] - e0)) : kEnd;
    };

    // ---- index chunks, exactly as in spmm_stream_kernel
    int32_t c = 0, p = 0, rc = 0;
    float v = 0.f, rv = 0.f;
    int cnt = 0, idx = 0;
    int32_t raw_base = ps;
    bool has_raw = ps < pe;
    auto load_raw = [&]() {
      const int32_t o = raw_base + lane;
      rc = -1;
      rv = 0.f;
      if (o < pe) {
        rc = a.col[e0 + o];
        rv = a.val[e0 + o];
      }
    };
    if (has_raw) load_raw();
    auto shift = [&]() {
      const bool ok = static_cast<uint32_t>(rc) < static_cast<uint64_t>(a.n_x_rows);
      const uint64_t mask = __ballot(ok);
      cnt = __builtin_popcountll(mask);
      const int32_t o = raw_base + lane;
      const int n_raw = pe - raw_base < kWave ? pe - raw_base : kWave;
      if (cnt == n_raw) {
        c = rc;
        v = rv;
        p = o;
      } else {
        const int below = __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                                    __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0));
        const int dest = (ok ? below : cnt + (lane - below)) << 2;
        c = __builtin_amdgcn_ds_permute(dest, rc);
        v = __builtin_bit_cast(float, __builtin_amdgcn_ds_permute(dest, __builtin_bit_cast(int, rv)));
        p = __builtin_amdgcn_ds_permute(dest, o);
      }
      idx = 0;
      raw_base += kWave;
      has_raw = raw_base < pe;
      if (has_raw) load_raw();
    };

    // ---- ring of U slots: per lane the raw words of its group's row, the entry's weight and
    // stream position; per slot (scalar) the position of its last entry
    typename P::W x[U];
    float wv[U];
    int32_t wp[U];
    int32_t slast[U];
    auto fetch = [&](int u) {
      while (idx >= cnt) {
        if (!has_raw) {
          slast[u] = kEnd;
          return;
        }
        shift();
      }
      // entry of this lane's group; groups past the chunk's last entry re-read that entry's
      // row with weight 0
      const int e = idx + grp;
      const int ec = e < cnt ? e : cnt - 1;
      const int32_t cj = __builtin_amdgcn_ds_bpermute(ec << 2, c);
      const float vj = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(ec << 2, __builtin_bit_cast(int, v)));
      wp[u] = __builtin_amdgcn_ds_bpermute(ec << 2, p);
      wv[u] = e < cnt ? vj : 0.f;
      const int last = idx + EPI < cnt ? idx + EPI : cnt;
      slast[u] = rl(p, last - 1);
      idx += EPI;
      if (el_ok)
        x[u] = P::load_raw(a.X + static_cast<int64_t>(cj) * a.ld_x + static_cast<int64_t>(el0) * ES);
      else
        x[u] = typename P::W(0u);
    };
#pragma unroll
    for (int u = 0; u < U; ++u) fetch(u);
    bool more = true;
    while (more) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (slast[u] == kEnd) {
          more = false;
          break;
        }
        P xw;
        xw.widen(x[u]);
        if (slast[u] < cur_end) {
          // the whole slot lies inside row `cur` (rows that ended before it were stored when the
          // slot that held their last entry was consumed, or are stored right below)
          acc.fma(wv[u], xw);
        } else {
          // a row ends inside the slot, or ended exactly before it: entries are applied row by
          // row, selected by their stream position. The rows of the other entries are masked
          // out, not multiplied by zero: a non-finite value must not leak into a row that does
          // not reference it.
          int32_t lo = -kEnd;
          while (true) {
            P xm = xw;
            xm.keep_if(wp[u] >= lo && wp[u] < cur_end);
            acc.fma(wv[u], xm);
            if (slast[u] < cur_end) break;
            lo = cur_end;
            flush();
          }
        }
        fetch(u);
      }
      if (++rounds == kFold / U) {
        rounds = 0;
        tot.add(acc);
        acc.zero();
      }
    }
    // rows that end inside this piece after its last entry (trailing skipped entries, empty rows)
    while (cur < nr && cur_end <= pe) flush();
    // a row that continues into the next piece
    if (cur < nr && __builtin_amdgcn_readfirstlane(static_cast<int32_t>(rp[cur] - e0)) < pe) {
      const int slot = (cur == first && head_partial) ? 0 : 1;
      acc.add(tot);
      across_groups(acc);
      if (grp == 0) acc.to_lds(&part[wave][slot][el0]);
      if (lane == 0) {
        if (slot == 0)
          head_row[wave] = cur;   // the whole piece lies inside one row; head_closed stays 0
        else
          tail_row[wave] = cur;
      }
    }
  }
  __syncthreads();

  // ---- rows cut by piece boundaries, added in piece order by the wavefront the row ended in
  if (head_row[wave] >= 0 && head_closed[wave]) {
    int ws = -1;
    for (int k = 0; k < wave; ++k)
      if (tail_row[k] >= 0) ws = k;
    if (ws >= 0 && grp == 0) {
      P sum, other;
      sum.from_lds(&part[ws][1][el0]);
      for (int k = ws + 1; k <= wave; ++k) {
        other.from_lds(&part[k][0][el0]);
        sum.add(other);
      }
      store_row(head_row[wave], sum);
    }
  }
}

// acc += sum over entries [s, e) of val * X[col]; all lanes of the wavefront take part
// (64/G entries at a time). Lane (grp, gl) handles 16-byte chunk gl of the feature row.
template <int ES, int G, int U>
__device__ __forceinline__ void walk_entries(const SpmmArgs& a, int64_t s, int64_t e, int lane,
                                             Chunk<ES>& acc) {
  constexpr int NG = kWave / G;
  constexpr int EPL = Chunk<ES>::N;
  const int gl = lane % G;
  const int grp = lane / G;
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
        cj[u] = __shfl(c, idc);
        vj[u] = __shfl(v, idc);
        if (idx >= cnt) vj[u] = 0.f;
      }
      Chunk<ES> x[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (gl * EPL < a.d)
          x[u].load(a.X + static_cast<int64_t>(cj[u]) * a.ld_x + gl * EPL * ES);
        else
          x[u].zero();
      }
#pragma unroll
      for (int u = 0; u < U; ++u) acc.fma(vj[u], x[u]);
    }
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
  // A row is a chain of dependent loads (its bounds, its entries' ids, the rows they name), and
  // the chain's length is the kernel's time. So the first chunk of ids is requested before the
  // loop, together with the diagonal term, and the diagonal term is added after the row's
  // entries: added first, its load would be waited for before the ids are even requested.
  auto load_ids = [&](int64_t base, int32_t& c, float& v) {
    c = 0;
    v = 0.f;
    if (base + gl < e) {
      c = a.col[base + gl];
      v = a.val[base + gl];
    }
  };
  int32_t c_next;
  float v_next;
  load_ids(s, c_next, v_next);
  const bool with_self = mine && a.self_val != nullptr && col_ok;
  Chunk<ES> xself;
  xself.zero();
  float vself = 0.f;
  if (with_self) {
    xself.load(a.X + (a.self_off + row) * a.ld_x + c0 * ES);
    vself = a.self_val[row];
  }
  for (int64_t base = s; base < e; base += G) {
    const int cnt = static_cast<int>(e - base < G ? e - base : G);
    int32_t c = c_next;
    float v = v_next;
    if (base + G < e) load_ids(base + G, c_next, v_next);
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
  if (with_self) acc.fma(vself, xself);
  if (mine && col_ok) acc.store(a.Y + row * a.ld_y + c0 * ES, a.d - c0);

  // rows too long for one group: one bit per group, handled one after another
  uint64_t todo = __ballot(row < a.n_rows && !mine && gl == 0);
  while (todo) {
    const int src = __builtin_ctzll(todo);
    todo &= todo - 1;
    const int64_t rs = __shfl(s0, src), re = __shfl(e0, src), r = __shfl(row, src);
    Chunk<ES> wacc;
    wacc.zero();
    walk_entries<ES, G, U>(a, rs, re, lane, wacc);
    if (a.self_val != nullptr && grp == 0 && col_ok) {
      Chunk<ES> x;
      x.load(a.X + (a.self_off + r) * a.ld_x + c0 * ES);
      wacc.fma(a.self_val[r], x);
    }
#pragma unroll
    for (int off = G; off < kWave; off <<= 1) wacc.xor_add(off);
    if (grp == 0 && col_ok) wacc.store(a.Y + r * a.ld_y + c0 * ES, a.d - c0);
  }
}

}  // namespace

namespace sat {

// Y[n_rows, d] = M * X (+ diag(self_val) * X[self_off + i]) where row i of M is
// (col, val)[rowptr[i] .. row_end[i]) with row_end = rowptr + 1 if row_end is
// NULL. A caller that passes row_end guarantees that the entries it cuts off,
// [row_end[i], rowptr[i+1]), all have col >= n_x_rows (they are skipped by
// their column id, not by position). X and Y hold elements of es bytes (4:
// fp32, 2: bf16; sums in fp32 either way), ld in elements. Pointers are device
// pointers; X and Y 16-byte aligned with ld * es % 16 == 0 (checked by the
// callers). total_entries = rowptr[n_rows] - rowptr[0], known to the caller.
template <int ES>
static sat_status launch_spmm_es(SpmmArgs a, int64_t total_entries, hipStream_t stream) {
  const int64_t n_rows = a.n_rows;
  const int32_t d = a.d;
  constexpr int EPL = 16 / ES;
  const int nvec = (d + EPL - 1) / EPL;   // 16-byte chunks per row
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
  // Stream kernel. Offsets inside a workgroup's span are 32-bit and 8 * (an eighth of the
  // span, rounded up) must not overflow.
  if (total_entries >= (int64_t{1} << 30)) return SAT_EUNSUPPORTED;
  // rows per workgroup: about 384 entries per wavefront
  int64_t R = 8;
  const int64_t want = kWaves * 384 * n_rows / (total_entries > 0 ? total_entries : 1);
  while (R < kMaxRowsPerBlock && R < want) R <<= 1;
  a.rows_per_block = static_cast<int32_t>(R);
  // Workgroups are dispatched in index order and live for a few hundred microseconds, so
  // the last ones would run on a half-empty chip: the last eighth of the rows goes to
  // workgroups a quarter the size.
  const int64_t n_big = n_rows / R * 7 / 8;
  const int64_t rest = n_rows - n_big * R;
  const int64_t bx = n_big + (rest + R / 4 - 1) / (R / 4);
  a.n_big_blocks = static_cast<int32_t>(n_big);
  if (bx > INT32_MAX) return SAT_EUNSUPPORTED;
  const dim3 block(kWaves * kWave);
  const int row_bytes = d * ES;
#define SAT_SPMM_LAUNCH(NW, NCH, U)                                                           \
  do {                                                                                        \
    const int per_pass = kWave * (NW) * 4 * (NCH);                                            \
    const dim3 grid(static_cast<unsigned>(bx),                                                \
                    static_cast<unsigned>((row_bytes + per_pass - 1) / per_pass));            \
    spmm_stream_kernel<ES, NW, NCH, U><<<grid, block, 0, stream>>>(a);                        \
  } while (0)
  // Rows up to 256 bytes: four or eight entries per gather instruction (22 G rows/s against
  // 14 with one entry per instruction on 256-byte rows). From 257 bytes on a row fills two
  // or more cache lines per entry and the one-entry kernel already runs at the memory
  // system's rate (with two entries per instruction it was measured slower on 400-byte rows,
  // 1.72 against 1.21 ms, and the same on 512-byte rows).
  if (row_bytes <= 256) {
    const dim3 grid(static_cast<unsigned>(bx));
    if (row_bytes <= 128) spmm_slot_kernel<ES, 8, 8><<<grid, block, 0, stream>>>(a);
    else spmm_slot_kernel<ES, 16, 8><<<grid, block, 0, stream>>>(a);
    return sat::check_launch();
  }
  if (row_bytes <= 512) SAT_SPMM_LAUNCH(2, 1, 16);
  else if (row_bytes <= 1024) SAT_SPMM_LAUNCH(4, 1, 16);
  else if (row_bytes <= 2048 || ES == 2) SAT_SPMM_LAUNCH(4, 2, 8);
  else if constexpr (ES == 4) {   // fp32 partial sums of wider bf16 rows would not fit LDS: more passes
    if (row_bytes <= 3072) SAT_SPMM_LAUNCH(4, 3, 4);
    else SAT_SPMM_LAUNCH(4, 4, 4);
  }
#undef SAT_SPMM_LAUNCH
  return sat::check_launch();
}

sat_status launch_spmm(const int64_t* rowptr, const int64_t* row_end, const int32_t* col,
                       const float* val, const void* X, int64_t ld_x, int64_t n_x_rows, void* Y,
                       int64_t ld_y, int64_t n_rows, int32_t d, int es, const float* self_val,
                       int64_t self_off, int64_t total_entries, hipStream_t stream) {
  if (n_rows == 0 || d == 0) return SAT_OK;
  const SpmmArgs a{rowptr, row_end ? row_end : rowptr + 1, rowptr, col, val,
                   static_cast<const unsigned char*>(X), ld_x * es, n_x_rows,
                   static_cast<unsigned char*>(Y), ld_y * es, n_rows, d, 0, 0, self_val, self_off};
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
  return launch_spmm(pv->rowptr, nullptr, pv->col, pv->val, Hbar, ld_in,
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
  // P_in^T = P_in: row i's local columns are [rowptr[i], split[i]); the entries after
  // split[i] are halo columns, whose relabelled ids are >= n_local
  st = launch_spmm(pv->rowptr, pv->split, pv->col, pv->val, dAGG, ld_in, pv->n_local, dH_local,
                   ld_out, pv->n_local, d, es, nullptr, 0, pv->nnz, s);
  if (st != SAT_OK || !dH_halo) return st;
  return launch_spmm(pv->h_colptr, nullptr, pv->h_row, pv->h_val, dAGG, ld_in,
                     pv->n_local, dH_halo, ld_halo, pv->n_halo, d, es, nullptr, 0, pv->nnz_halo, s);
}

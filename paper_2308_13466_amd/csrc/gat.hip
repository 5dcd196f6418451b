// Graph attention backbone of the partition step (Eq. 1 / Eq. 2 with attention
// as the aggregation function; the layer itself follows Velickovic et al.,
// "Graph Attention Networks", Eq. 1-4): attention scores, edge softmax and
// weighted aggregation over the partition view's rows, and the full backward.
//
// Nothing per edge is ever stored: the forward keeps, per local row and head,
// the maximum of the scores and the reciprocal of the sum of exponentials, and
// every later pass recomputes alpha_ij = exp(LeakyReLU(el_i + er_j) - max_i) / sum_i
// from the two per-node score vectors. All three edge passes are gathers of
// nnz feature rows, so the memory system is the bound, as for the normalised
// adjacency product.
//
// Mapping (all edge kernels): a workgroup of 8 wavefronts owns 64 consecutive
// rows, wavefront w taking rows w, w + 8, ... . A row's entries are taken
// 64 at a time in two phases:
//   * entry phase, one entry per lane: column id, the per-head scores of that
//     column (a 4K-byte read), exponentials, per-head weights written to the
//     wavefront's slice of LDS. In the forward this phase also carries the
//     running maximum of the online softmax and rescales the sums;
//   * feature phase: G lanes cover a feature row (16 bytes each where the width allows:
//     4 fp32 or 8 bf16 elements, so that one gather instruction requests 1 KiB either
//     way; 4 bf16 elements otherwise), the 64/G groups take different entries, 8 gathers
//     per group are issued back to back before any is used; each lane reads the weight
//     of its own head from LDS.
// Per-head dot products (the gradient with respect to alpha) are kept as per-lane
// partial sums and reduced across lanes once per row, not per entry.
// Rows longer than kLongRow entries are left for a second phase in which all 8
// wavefronts split the row into contiguous pieces and combine their partial
// results through LDS in wavefront order (deterministic; no atomics anywhere).
#include <math.h>

#include "sat_internal.h"

namespace {

using sat::kWave;
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int kWaves = 8;
constexpr int kRowsPerBlock = 64;
constexpr int kLongRow = 1024;
constexpr int kU = 8;         // gathers in flight per lane group
// (with 16-byte shares of bf16 rows: 6, the most that keeps the entry loop free of spills; with
// 8 heads, whose per-head values take the registers of two more gathers: 6 and 4)
template <int K, int V>
constexpr int kUof = (V == 2 ? 6 : kU) - (K == 8 ? 2 : 0);
constexpr int kMaxD = 256;     // 64 lanes x 4 elements

// Four consecutive elements of a row: the bits as loaded (nothing may touch them before
// all gathers of a round have been issued, or each load is waited for on its own) ...
template <int ES>
struct Raw4 {
  typedef f32x4 T;
};
template <>
struct Raw4<2> {
  typedef u32x2 T;
};
template <int ES>
__device__ __forceinline__ typename Raw4<ES>::T load_raw4(const unsigned char* p) {
  return *reinterpret_cast<const typename Raw4<ES>::T*>(p);
}
// ... and as fp32
template <int ES>
__device__ __forceinline__ f32x4 widen4(typename Raw4<ES>::T w) {
  if constexpr (ES == 4) {
    return w;
  } else {
    const uint32_t w0 = w.x, w1 = w.y;
    f32x4 r;
    r.x = __builtin_bit_cast(float, w0 << 16);
    r.y = __builtin_bit_cast(float, w0 & 0xffff0000u);
    r.z = __builtin_bit_cast(float, w1 << 16);
    r.w = __builtin_bit_cast(float, w1 & 0xffff0000u);
    return r;
  }
}
template <int ES>
__device__ __forceinline__ f32x4 load4(const unsigned char* p) {
  return widen4<ES>(load_raw4<ES>(p));
}

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {   // two RNE bf16
  const f32x2 pr = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));
}

// the first min(left, 4) elements of v to p
template <int ES>
__device__ __forceinline__ void store4(unsigned char* p, f32x4 v, int left) {
  if constexpr (ES == 4) {
    if (left >= 4) {
      *reinterpret_cast<f32x4*>(p) = v;
    } else {
      float* y = reinterpret_cast<float*>(p);
      if (left > 0) y[0] = v.x;
      if (left > 1) y[1] = v.y;
      if (left > 2) y[2] = v.z;
    }
  } else {
    const uint32_t w0 = pack2(v.x, v.y), w1 = pack2(v.z, v.w);
    if (left >= 4) {
      u32x2 w;
      w.x = w0;
      w.y = w1;
      *reinterpret_cast<u32x2*>(p) = w;
    } else {
      uint16_t* y = reinterpret_cast<uint16_t*>(p);
      if (left > 0) y[0] = static_cast<uint16_t>(w0 & 0xffffu);
      if (left > 1) y[1] = static_cast<uint16_t>(w0 >> 16);
      if (left > 2) y[2] = static_cast<uint16_t>(w1 & 0xffffu);
    }
  }
}

__device__ __forceinline__ f32x4 clip4(f32x4 v, int left) {   // zero the elements at or after `left`
  if (left < 4) v.w = 0.f;
  if (left < 3) v.z = 0.f;
  if (left < 2) v.y = 0.f;
  if (left < 1) v.x = 0.f;
  return v;
}

__device__ __forceinline__ float dot4(f32x4 a, f32x4 b) {
  return a.x * b.x + a.y * b.y + a.z * b.z + a.w * b.w;
}

// A lane's share of a gathered row: V chunks of four consecutive elements (V = 2: eight
// bf16 elements, one 16-byte load), as loaded and as fp32.
template <int ES, int V>
struct RawV {
  typedef typename Raw4<ES>::T T;
};
template <>
struct RawV<2, 2> {
  typedef u32x4 T;
};
template <int ES, int V>
__device__ __forceinline__ typename RawV<ES, V>::T load_raw(const unsigned char* p) {
  static_assert(V == 1 || (V == 2 && ES == 2), "lane shares are at most 16 bytes");
  return *reinterpret_cast<const typename RawV<ES, V>::T*>(p);
}
template <int ES, int V>
__device__ __forceinline__ void widen(typename RawV<ES, V>::T w, f32x4 (&out)[V]) {
  if constexpr (V == 1) {
    out[0] = widen4<ES>(w);
  } else {
    u32x2 lo, hi;
    lo.x = w.x;
    lo.y = w.y;
    hi.x = w.z;
    hi.y = w.w;
    out[0] = widen4<2>(lo);
    out[1] = widen4<2>(hi);
  }
}
template <int ES, int V>
__device__ __forceinline__ void load_share(const unsigned char* p, int left, f32x4 (&out)[V]) {
  widen<ES, V>(load_raw<ES, V>(p), out);
#pragma unroll
  for (int v = 0; v < V; ++v) out[v] = clip4(out[v], left - 4 * v);
}
template <int ES, int V>
__device__ __forceinline__ void store_share(unsigned char* p, const f32x4 (&o)[V], int left) {
#pragma unroll
  for (int v = 0; v < V; ++v)
    if (left > 4 * v) store4<ES>(p + static_cast<int64_t>(4 * v) * ES, o[v], left - 4 * v);
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  return v;
}
// a value all lanes hold alike, moved to a scalar register
__device__ __forceinline__ float uniform_f32(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int32_t, v)));
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

// v[h] for a per-lane head index h, as K and-or steps on the bit patterns (a chain of
// selects is turned into an indexed read of a private array by the compiler)
template <int K>
__device__ __forceinline__ float pick(const float (&v)[K], int h) {
  uint32_t r = 0;
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const uint32_t mask = static_cast<uint32_t>(-static_cast<int32_t>(h == k));
    r |= __builtin_bit_cast(uint32_t, v[k]) & mask;
  }
  return __builtin_bit_cast(float, r);
}

// K consecutive floats at p (p aligned to 4 * K bytes)
template <int K>
__device__ __forceinline__ void load_heads(const float* p, float (&v)[K]) {
  if constexpr (K == 1) {
    v[0] = p[0];
  } else if constexpr (K == 2) {
    const f32x2 t = *reinterpret_cast<const f32x2*>(p);
    v[0] = t.x;
    v[1] = t.y;
  } else {
#pragma unroll
    for (int q = 0; q < K / 4; ++q) {
      const f32x4 t = *reinterpret_cast<const f32x4*>(p + 4 * q);
      v[4 * q] = t.x;
      v[4 * q + 1] = t.y;
      v[4 * q + 2] = t.z;
      v[4 * q + 3] = t.w;
    }
  }
}

// How the lanes of a wavefront cover rows of d = K * F elements: G = 2^lg_g lanes per
// row (4 * 2^lg_v elements each), LH = 2^lg_lh consecutive lanes per head.
struct Lanes {
  int32_t d, lg_g, lg_lh, lg_v;
};

struct WalkArgs {
  const int64_t* row_begin;   // row r holds entries [row_begin[r], row_end[r]) of col
  const int64_t* row_end;
  const int32_t* col;         // rows of X
  int64_t n_rows;
  int64_t n_x_rows;           // entries with col outside [0, n_x_rows) contribute nothing
  const unsigned char* X;     // gathered operand, ld_x bytes per row
  int64_t ld_x;
  Lanes ln;
  float slope;
};

struct LaneIds {
  int lane, gl, grp, ng, h, el0, left;
  bool col_ok, leader;
};

__device__ __forceinline__ LaneIds lane_ids(const Lanes& ln, int heads) {
  LaneIds L;
  L.lane = threadIdx.x & (kWave - 1);
  L.gl = L.lane & ((1 << ln.lg_g) - 1);
  L.grp = L.lane >> ln.lg_g;
  L.ng = kWave >> ln.lg_g;
  L.h = L.gl >> ln.lg_lh;
  L.el0 = L.gl << (2 + ln.lg_v);
  L.left = ln.d - L.el0;
  L.col_ok = L.left > 0;
  // the lane that ends up holding (and writes) its head's reduced scalars
  L.leader = L.grp == 0 && (L.gl & ((1 << ln.lg_lh) - 1)) == 0 && L.h < heads;
  return L;
}

// sum over the lanes that hold the same head: the LH lanes of the head in every group
__device__ __forceinline__ float head_sum(float v, const Lanes& ln) {
  for (int b = 0; b < ln.lg_lh; ++b) v += __shfl_xor(v, 1 << b);
  for (int b = ln.lg_g; b < 6; ++b) v += __shfl_xor(v, 1 << b);
  return v;
}
__device__ __forceinline__ f32x4 group_sum(f32x4 v, const Lanes& ln) {   // over the 64/G groups
  for (int b = ln.lg_g; b < 6; ++b) {
    v.x += __shfl_xor(v.x, 1 << b);
    v.y += __shfl_xor(v.y, 1 << b);
    v.z += __shfl_xor(v.z, 1 << b);
    v.w += __shfl_xor(v.w, 1 << b);
  }
  return v;
}
template <int V>
__device__ __forceinline__ void group_sum(const f32x4 (&v)[V], const Lanes& ln, f32x4 (&out)[V]) {
#pragma unroll
  for (int i = 0; i < V; ++i) out[i] = group_sum(v[i], ln);
}

__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// Walk entries [s, e) of a.col. `pre(c, ok)`: called first with one entry per lane (ok false
// for lanes past the end and for ids out of range; c is then 0); it only REQUESTS the
// per-node scores the entry needs. `entry(c, ok, w)`: called for the same lane and entry once
// the first round of gathers has been issued; it writes the entry's NW per-head weights to
// w[0 .. NW). `feature(x, w, valid)`: called for each lane's share x (V chunks of four
// elements) of a gathered row, w the weights of that entry in LDS. `fold()`: called after the last entry of
// each batch of 64: the callers sum a batch on its own and add it to the row's running sum
// there, which keeps the chains of additions short on rows of thousands of entries.
template <int ES, int V, int NW, int U, class Pre, class Entry, class Feature, class Fold>
__device__ __forceinline__ void walk(const WalkArgs& a, const LaneIds& L, int64_t s, int64_t e,
                                     int32_t* s_col, float* s_w, Pre&& pre, Entry&& entry,
                                     Feature&& feature, Fold&& fold) {
  // rows whose width is not a whole number of chunks, or fewer chunks than lanes in a group:
  // the lanes' shares are clipped to the row (lanes past it get zeros)
  const bool clip = a.ln.d != ((4 * V) << a.ln.lg_g);
  for (int64_t base = s; base < e; base += kWave) {
    const int cnt = static_cast<int>(e - base < kWave ? e - base : kWave);
    int32_t c = -1;
    if (L.lane < cnt) c = a.col[base + L.lane];
    const bool ok = static_cast<uint64_t>(static_cast<uint32_t>(c)) < static_cast<uint64_t>(a.n_x_rows);
    if (!ok) c = 0;
    wave_lds_fence();               // the previous batch's reads of LDS are done
    s_col[L.lane] = c;
    wave_lds_fence();
    typename RawV<ES, V>::T x[U];
    // entry handled in slot u of the round that starts at j0 (past the end: the last
    // entry again, with weight 0); recomputed where it is needed rather than kept
    auto slot = [&](int j0, int u, bool& valid) __attribute__((always_inline)) {
      const int idx = j0 + u * L.ng + L.grp;
      valid = idx < cnt;
      return valid ? idx : cnt - 1;
    };
    auto issue = [&](int j0) __attribute__((always_inline)) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        bool valid;
        const int32_t cj = s_col[slot(j0, u, valid)];
        // lanes past the row's width re-read its first chunk; their sums are never stored
        x[u] = load_raw<ES, V>(a.X + static_cast<int64_t>(cj) * a.ld_x +
                               static_cast<int64_t>(L.col_ok ? L.el0 : 0) * ES);
      }
    };
    auto consume = [&](int j0) __attribute__((always_inline)) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        bool valid;
        const int idc = slot(j0, u, valid);
        f32x4 xw[V];
        widen<ES, V>(x[u], xw);
        if (clip) {
#pragma unroll
          for (int v = 0; v < V; ++v) xw[v] = clip4(xw[v], L.left - 4 * v);
        }
        feature(xw, s_w + idc * NW, valid);
        // (the conversions of all U shares moved ahead of the first use would not fit the registers)
        if constexpr (V == 2) __builtin_amdgcn_sched_barrier(0);
      }
    };
    // The first round of gathers needs the ids only: it is in flight while the entry phase
    // computes the weights. The scores are requested BEFORE the gathers: a wavefront's loads
    // complete in the order they were issued, so requested after them the scores would only
    // be there once every gathered row of the round is.
    pre(c, ok);
    __builtin_amdgcn_sched_barrier(0);
    issue(0);
    __builtin_amdgcn_sched_barrier(0);
    entry(c, ok, s_w + L.lane * NW);
    wave_lds_fence();
    consume(0);
    for (int j0 = L.ng * U; j0 < cnt; j0 += L.ng * U) {
      issue(j0);
      consume(j0);
    }
    fold();
  }
}

// A value every lane of the wavefront holds alike, moved to scalar registers so that the
// loops and branches it controls are scalar ones.
__device__ __forceinline__ int64_t uniform64(int64_t v) {
  const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v));
  const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(static_cast<uint64_t>(v) >> 32));
  return static_cast<int64_t>((static_cast<uint64_t>(hi) << 32) | lo);
}

// Rows of a workgroup: wavefront w takes rows w, w + 8, ...; rows longer than kLongRow are
// flagged in LDS beforehand and left for the cooperative phase. Row ownership is static
// on purpose: every loop bound and branch around the cross-lane operations is then a
// scalar that all lanes share by construction. (Drawing rows from a counter with one
// lane and broadcasting the result let the compiler thread that lane's branch into the
// neighbouring one-lane store of the previous iteration and split the wavefront for good.)
struct RowSpans {
  int64_t begin[kRowsPerBlock], end[kRowsPerBlock];
  int is_long[kRowsPerBlock];
};
__device__ __forceinline__ void flag_long_rows(const WalkArgs& a, int64_t row0, int nr, RowSpans* sp) {
  for (int t = threadIdx.x; t < nr; t += kWaves * kWave) {
    const int64_t b = a.row_begin[row0 + t], e = a.row_end[row0 + t];
    sp->begin[t] = b;
    sp->end[t] = e;
    sp->is_long[t] = e - b > kLongRow ? 1 : 0;
  }
  __syncthreads();
}

__device__ __forceinline__ void piece_of(int64_t s, int64_t e, int wave, int64_t& ps, int64_t& pe) {
  const int64_t len = e - s;
  const int64_t per = ((len + kWaves - 1) / kWaves + kWave - 1) / kWave * kWave;
  ps = s + wave * per;
  if (ps > e) ps = e;
  pe = ps + per < e ? ps + per : e;
}

// ---------------------------------------------------------------- attention scores
// el[r, k] = <a_dst[k], Z[r, k]> (r < n_dst), er[r, k] = <a_src[k], Z[r, k]> (r < n)
constexpr int kScoreRows = 8;   // row slots per wavefront (each slot: 64/G rows)
template <int ES>
__global__ __launch_bounds__(256) void gat_scores_kernel(const unsigned char* Z, int64_t ld_z, int64_t n,
                                                        int64_t n_dst, int heads, Lanes ln,
                                                        const float* a_dst, const float* a_src,
                                                        float* el, float* er) {
  const LaneIds L = lane_ids(ln, heads);
  const int64_t row0 = (static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6)) * kScoreRows * L.ng + L.grp;
  f32x4 ad(0.f), as(0.f);
  if (L.left > 0) { ad.x = a_dst[L.el0]; as.x = a_src[L.el0]; }
  if (L.left > 1) { ad.y = a_dst[L.el0 + 1]; as.y = a_src[L.el0 + 1]; }
  if (L.left > 2) { ad.z = a_dst[L.el0 + 2]; as.z = a_src[L.el0 + 2]; }
  if (L.left > 3) { ad.w = a_dst[L.el0 + 3]; as.w = a_src[L.el0 + 3]; }
  typename Raw4<ES>::T raw[kScoreRows];
#pragma unroll
  for (int q = 0; q < kScoreRows; ++q) {
    int64_t row = row0 + q * L.ng;
    if (row >= n) row = n - 1;            // n > 0: checked by the host
    raw[q] = load_raw4<ES>(Z + row * ld_z + static_cast<int64_t>(L.col_ok ? L.el0 : 0) * ES);
  }
#pragma unroll
  for (int q = 0; q < kScoreRows; ++q) {
    const int64_t row = row0 + q * L.ng;
    const f32x4 z = clip4(widen4<ES>(raw[q]), L.left);
    float pd = dot4(z, ad), ps = dot4(z, as);
    for (int b = 0; b < ln.lg_lh; ++b) {
      pd += __shfl_xor(pd, 1 << b);
      ps += __shfl_xor(ps, 1 << b);
    }
    if (row < n && (L.gl & ((1 << ln.lg_lh) - 1)) == 0 && L.h < heads) {
      er[row * heads + L.h] = ps;
      if (row < n_dst) el[row * heads + L.h] = pd;
    }
  }
}

// ---------------------------------------------------------------- forward
// H[i] = act(sum_j alpha_ij Z_j), stats[i, k] = (max_j e_ij, 1 / sum_j exp(e_ij - max))
template <int ES, int K, int V>
__global__ __launch_bounds__(kWaves * kWave, 4) void gat_fwd_kernel(WalkArgs a, const float* __restrict__ el,
                                                                const float* __restrict__ er, int relu,
                                                                unsigned char* Y, int64_t ld_y,
                                                                float* stats) {
  __shared__ RowSpans sp;
  __shared__ int32_t s_col[kWaves][kWave];
  __shared__ float s_w[kWaves][kWave * K];
  constexpr int HDR = (2 * K + 3) / 4 * 4;
  __shared__ __attribute__((aligned(16))) float s_part[kWaves][HDR + kMaxD];
  const LaneIds L = lane_ids(a.ln, K);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t row0 = static_cast<int64_t>(blockIdx.x) * kRowsPerBlock;
  const int nr = static_cast<int>(a.n_rows - row0 < kRowsPerBlock ? a.n_rows - row0 : kRowsPerBlock);
  flag_long_rows(a, row0, nr, &sp);

  float m[K], l[K], eli[K];
  f32x4 acc[V];
  auto reset = [&](int64_t row) __attribute__((always_inline)) {
#pragma unroll
    for (int k = 0; k < K; ++k) {
      m[k] = -INFINITY;
      l[k] = 0.f;
    }
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = f32x4(0.f);
    load_heads<K>(el + row * K, eli);
  };
  float erv[K];
  auto pre = [&](int32_t c, bool) __attribute__((always_inline)) {
    load_heads<K>(er + static_cast<int64_t>(c) * K, erv);
  };
  auto entry = [&](int32_t, bool ok, float* w) __attribute__((always_inline)) {
    float e[K];
    float scale[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const float s = eli[k] + erv[k];
      e[k] = ok ? (s > 0.f ? s : a.slope * s) : -INFINITY;
      // (the running maximum is the same in every lane: kept in scalar registers)
      const float bm = wave_max(e[k]);
      const float mn = uniform_f32(fmaxf(m[k], bm));
      // first entries of the row: m = -inf, nothing accumulated yet to rescale
      scale[k] = m[k] == -INFINITY ? 0.f : expf(m[k] - mn);
      const float p = e[k] == -INFINITY ? 0.f : expf(e[k] - mn);
      l[k] = l[k] * scale[k] + p;
      m[k] = mn;
      w[k] = p;
    }
    const float sc = pick<K>(scale, L.h);
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] *= sc;
  };
  // the current batch of 64 entries (all under the current maximum). With 16-byte shares of
  // bf16 rows the registers for it are not there, and the rounding of a long fp32 chain is far
  // below that of the stored result: those sum into acc directly.
  constexpr int VB = V == 1 ? 1 : 0;
  f32x4 bacc[VB + 1];
  bacc[0] = f32x4(0.f);
  auto feature = [&](const f32x4 (&x)[V], const float* w, bool valid) __attribute__((always_inline)) {
    const float p = valid ? w[L.h] : 0.f;
    if constexpr (VB) {
      bacc[0] += p * x[0];
    } else {
#pragma unroll
      for (int v = 0; v < V; ++v) acc[v] += p * x[v];
    }
  };
  auto fold = [&]() __attribute__((always_inline)) {
    if constexpr (VB) {
      acc[0] += bacc[0];
      bacc[0] = f32x4(0.f);
    }
  };
  auto store = [&](int64_t row, const f32x4 (&sum)[V], const float (&mm)[K], const float (&ll)[K]) {
    float inv[K];
#pragma unroll
    for (int k = 0; k < K; ++k) inv[k] = ll[k] > 0.f ? 1.f / ll[k] : 0.f;
    f32x4 o[V];
#pragma unroll
    for (int v = 0; v < V; ++v) {
      o[v] = sum[v] * pick<K>(inv, L.h);
      if (relu) {
        o[v].x = fmaxf(o[v].x, 0.f);
        o[v].y = fmaxf(o[v].y, 0.f);
        o[v].z = fmaxf(o[v].z, 0.f);
        o[v].w = fmaxf(o[v].w, 0.f);
      }
    }
    if (L.grp == 0 && L.col_ok)
      store_share<ES, V>(Y + row * ld_y + static_cast<int64_t>(L.el0) * ES, o, L.left);
    if (L.lane < K) {
      const float mv = pick<K>(mm, L.lane), iv = pick<K>(inv, L.lane);
      f32x2 t;
      t.x = mv == -INFINITY ? 0.f : mv;   // a row without entries
      t.y = iv;
      *reinterpret_cast<f32x2*>(stats + (row * K + L.lane) * 2) = t;
    }
  };

  // ---- short rows
  for (int r = wave; r < nr; r += kWaves) {
    if (__builtin_amdgcn_readfirstlane(sp.is_long[r])) continue;
    const int64_t row = row0 + r;
    const int64_t s = uniform64(sp.begin[r]), e = uniform64(sp.end[r]);
    reset(row);
    walk<ES, V, K, kUof<K, V>>(a, L, s, e, s_col[wave], s_w[wave], pre, entry, feature, fold);
    float ll[K];
#pragma unroll
    for (int k = 0; k < K; ++k) ll[k] = wave_sum(l[k]);
    f32x4 tot[V];
    group_sum<V>(acc, a.ln, tot);
    store(row, tot, m, ll);
  }
  __syncthreads();
  // ---- long rows: a contiguous piece per wavefront, combined in wavefront order
  for (int r = 0; r < nr; ++r) {
    if (!__builtin_amdgcn_readfirstlane(sp.is_long[r])) continue;   // the same for every wavefront
    const int64_t row = row0 + r;
    const int64_t s = uniform64(sp.begin[r]), e = uniform64(sp.end[r]);
    int64_t ps, pe;
    piece_of(s, e, wave, ps, pe);
    reset(row);
    walk<ES, V, K, kUof<K, V>>(a, L, ps, pe, s_col[wave], s_w[wave], pre, entry, feature, fold);
    f32x4 part[V];
    group_sum<V>(acc, a.ln, part);
    float lk[K];
#pragma unroll
    for (int k = 0; k < K; ++k) lk[k] = wave_sum(l[k]);
    if (L.lane < K) {     // every lane holds all K values; lane k stores those of head k
      s_part[wave][L.lane] = pick<K>(m, L.lane);
      s_part[wave][K + L.lane] = pick<K>(lk, L.lane);
    }
    if (L.grp == 0) {
#pragma unroll
      for (int v = 0; v < V; ++v) *reinterpret_cast<f32x4*>(&s_part[wave][HDR + L.el0 + 4 * v]) = part[v];
    }
    __syncthreads();
    if (wave == 0) {
      float mm[K], ll[K], f[K];
#pragma unroll
      for (int k = 0; k < K; ++k) {
        mm[k] = -INFINITY;
        for (int w = 0; w < kWaves; ++w) mm[k] = fmaxf(mm[k], s_part[w][k]);
        ll[k] = 0.f;
      }
      f32x4 sum[V];
#pragma unroll
      for (int v = 0; v < V; ++v) sum[v] = f32x4(0.f);
      for (int w = 0; w < kWaves; ++w) {
#pragma unroll
        for (int k = 0; k < K; ++k) {
          const float mw = s_part[w][k];
          f[k] = mw == -INFINITY ? 0.f : expf(mw - mm[k]);
          ll[k] += s_part[w][K + k] * f[k];
        }
#pragma unroll
        for (int v = 0; v < V; ++v) {
          const f32x4 pw = *reinterpret_cast<const f32x4*>(&s_part[w][HDR + L.el0 + 4 * v]);
          sum[v] += pick<K>(f, L.h) * pw;
        }
      }
      store(row, sum, mm, ll);
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------- backward, destination side
// For every local row i (entries j, gathered Z_j), with g_i = dOUT_i:
//   D_i   = sum_j alpha_ij <g_i, Z_j>            (per head)
//   d_el_i = sum_j alpha_ij LeakyReLU'(s_ij) (<g_i, Z_j> - D_i)
// and rowstat[i, k] = (el, max, 1/sum, D) for the source-side pass.
template <int ES, int K, int V>
__global__ __launch_bounds__(kWaves * kWave, 4) void gat_bwd_dst_kernel(
    WalkArgs a, const float* __restrict__ el, const float* __restrict__ er, const float* __restrict__ stats,
    const unsigned char* dOUT, int64_t ld_g, float* d_el, f32x4* rowstat) {
  __shared__ RowSpans sp;
  __shared__ int32_t s_col[kWaves][kWave];
  __shared__ float s_w[kWaves][kWave * 2 * K];
  __shared__ float s_part[kWaves][3 * K];
  const LaneIds L = lane_ids(a.ln, K);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t row0 = static_cast<int64_t>(blockIdx.x) * kRowsPerBlock;
  const int nr = static_cast<int>(a.n_rows - row0 < kRowsPerBlock ? a.n_rows - row0 : kRowsPerBlock);
  flag_long_rows(a, row0, nr, &sp);

  float eli[K], mi[K], inv[K], w1s[K];
  f32x4 g[V];
  float accD, acc1;
  auto reset = [&](int64_t row) __attribute__((always_inline)) {
    load_heads<K>(el + row * K, eli);
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const f32x2 t = *reinterpret_cast<const f32x2*>(stats + (row * K + k) * 2);
      mi[k] = t.x;
      inv[k] = t.y;
      w1s[k] = 0.f;
    }
#pragma unroll
    for (int v = 0; v < V; ++v) g[v] = f32x4(0.f);
    if (L.col_ok) load_share<ES, V>(dOUT + row * ld_g + static_cast<int64_t>(L.el0) * ES, L.left, g);
    accD = 0.f;
    acc1 = 0.f;
  };
  float erv[K];
  auto pre = [&](int32_t c, bool) __attribute__((always_inline)) {
    load_heads<K>(er + static_cast<int64_t>(c) * K, erv);
  };
  auto entry = [&](int32_t, bool ok, float* w) __attribute__((always_inline)) {
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const float s = eli[k] + erv[k];
      const float e = s > 0.f ? s : a.slope * s;
      const float al = ok ? expf(e - mi[k]) * inv[k] : 0.f;
      const float w1 = al * (s > 0.f ? 1.f : a.slope);
      w1s[k] += w1;
      w[k] = al;
      w[K + k] = w1;
    }
  };
  float bD = 0.f, b1 = 0.f;
  auto feature = [&](const f32x4 (&x)[V], const float* w, bool valid) __attribute__((always_inline)) {
    float dt = dot4(g[0], x[0]);
#pragma unroll
    for (int v = 1; v < V; ++v) dt += dot4(g[v], x[v]);
    const float al = valid ? w[L.h] : 0.f;
    const float w1 = valid ? w[K + L.h] : 0.f;
    bD += al * dt;
    b1 += w1 * dt;
  };
  auto fold = [&]() __attribute__((always_inline)) {
    accD += bD;
    acc1 += b1;
    bD = 0.f;
    b1 = 0.f;
  };
  auto store = [&](int64_t row, float D, float t1, const float (&ws)[K]) {   // head leaders hold D, t1
    if (L.leader) {
      const float wsum = pick<K>(ws, L.h);
      d_el[row * K + L.h] = t1 - D * wsum;
      f32x4 rs;
      rs.x = pick<K>(eli, L.h);
      rs.y = pick<K>(mi, L.h);
      rs.z = pick<K>(inv, L.h);
      rs.w = D;
      rowstat[row * K + L.h] = rs;
    }
  };

  for (int r = wave; r < nr; r += kWaves) {
    if (__builtin_amdgcn_readfirstlane(sp.is_long[r])) continue;
    const int64_t row = row0 + r;
    const int64_t s = uniform64(sp.begin[r]), e = uniform64(sp.end[r]);
    reset(row);
    walk<ES, V, 2 * K, kUof<K, V>>(a, L, s, e, s_col[wave], s_w[wave], pre, entry, feature, fold);
    float ws[K];
#pragma unroll
    for (int k = 0; k < K; ++k) ws[k] = wave_sum(w1s[k]);
    store(row, head_sum(accD, a.ln), head_sum(acc1, a.ln), ws);
  }
  __syncthreads();
  for (int r = 0; r < nr; ++r) {
    if (!__builtin_amdgcn_readfirstlane(sp.is_long[r])) continue;   // the same for every wavefront
    const int64_t row = row0 + r;
    const int64_t s = uniform64(sp.begin[r]), e = uniform64(sp.end[r]);
    int64_t ps, pe;
    piece_of(s, e, wave, ps, pe);
    reset(row);
    walk<ES, V, 2 * K, kUof<K, V>>(a, L, ps, pe, s_col[wave], s_w[wave], pre, entry, feature, fold);
    const float D = head_sum(accD, a.ln), t1 = head_sum(acc1, a.ln);
    float wk[K];
#pragma unroll
    for (int k = 0; k < K; ++k) wk[k] = wave_sum(w1s[k]);
    if (L.lane < K) s_part[wave][2 * K + L.lane] = pick<K>(wk, L.lane);
    if (L.leader) {
      s_part[wave][L.h] = D;
      s_part[wave][K + L.h] = t1;
    }
    __syncthreads();
    if (wave == 0) {
      float Dh = 0.f, th = 0.f, ws[K];
#pragma unroll
      for (int k = 0; k < K; ++k) ws[k] = 0.f;
      for (int w = 0; w < kWaves; ++w) {
        if (L.leader) {
          Dh += s_part[w][L.h];
          th += s_part[w][K + L.h];
        }
#pragma unroll
        for (int k = 0; k < K; ++k) ws[k] += s_part[w][2 * K + k];
      }
      store(row, Dh, th, ws);
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------- backward, source side
// For every row j of the transposed structure (entries: the local rows i that have j as
// a neighbour; gathered g_i = dOUT_i and rowstat_i), j = row_off + r:
//   d_er_j = sum_i alpha_ij LeakyReLU'(s_ij) (<g_i, Z_j> - D_i)
//   dZ_j   = sum_i alpha_ij g_i + d_er_j a_src + d_el_j a_dst   (the last term for local j)
template <int ES, int K, int V, int U>
__global__ __launch_bounds__(kWaves * kWave, (U <= 2 && K < 8) ? 6 : 4) void gat_bwd_src_kernel(
    WalkArgs a, int64_t row_off, int64_t n_local, const float* __restrict__ er, const f32x4* __restrict__ rowstat,
    const unsigned char* Z, int64_t ld_z, const float* __restrict__ d_el, const float* a_dst, const float* a_src,
    unsigned char* dZ, int64_t ld_dz, float* d_er) {
  __shared__ RowSpans sp;
  __shared__ int32_t s_col[kWaves][kWave];
  __shared__ float s_w[kWaves][kWave * 2 * K];
  constexpr int HDR = (2 * K + 3) / 4 * 4;
  __shared__ __attribute__((aligned(16))) float s_part[kWaves][HDR + kMaxD];
  // the two attention vectors, zero past their end: every row's last step adds a multiple of
  // them, and read from memory there they would be a dependent load (and a wait for every
  // gather in flight) per row
  __shared__ __attribute__((aligned(16))) float s_avec[2][kMaxD];
  for (int i = threadIdx.x; i < kMaxD; i += kWaves * kWave) {
    s_avec[0][i] = i < a.ln.d ? a_src[i] : 0.f;
    s_avec[1][i] = i < a.ln.d ? a_dst[i] : 0.f;
  }
  const LaneIds L = lane_ids(a.ln, K);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t row0 = static_cast<int64_t>(blockIdx.x) * kRowsPerBlock;
  const int nr = static_cast<int>(a.n_rows - row0 < kRowsPerBlock ? a.n_rows - row0 : kRowsPerBlock);
  flag_long_rows(a, row0, nr, &sp);   // (its barrier publishes s_avec as well)

  float erj[K], wds[K];
  f32x4 z[V], acc[V];
  float accd;
  auto reset = [&](int64_t jj) __attribute__((always_inline)) {
    load_heads<K>(er + jj * K, erj);
#pragma unroll
    for (int k = 0; k < K; ++k) wds[k] = 0.f;
#pragma unroll
    for (int v = 0; v < V; ++v) {
      z[v] = f32x4(0.f);
      acc[v] = f32x4(0.f);
    }
    if (L.col_ok) load_share<ES, V>(Z + jj * ld_z + static_cast<int64_t>(L.el0) * ES, L.left, z);
    accd = 0.f;
  };
  // (the instance with two gathers in flight has no registers to hold the row statistics across
  // the gathers' issue: it requests them in the entry phase)
  constexpr bool kEarly = U > 2 && K < 8;   // (8 heads: 32 registers per entry)
  f32x4 rsv[K];
  auto pre = [&](int32_t c, bool) __attribute__((always_inline)) {
    if constexpr (kEarly) {
#pragma unroll
      for (int k = 0; k < K; ++k) rsv[k] = rowstat[static_cast<int64_t>(c) * K + k];
    }
  };
  auto entry = [&](int32_t c, bool ok, float* w) __attribute__((always_inline)) {
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const f32x4 rs = kEarly ? rsv[k] : rowstat[static_cast<int64_t>(c) * K + k];
      const float rel = rs.x, rm = rs.y, rinv = rs.z, rD = rs.w;
      const float s = rel + erj[k];
      const float e = s > 0.f ? s : a.slope * s;
      const float al = ok ? expf(e - rm) * rinv : 0.f;
      const float w1 = al * (s > 0.f ? 1.f : a.slope);
      wds[k] += w1 * rD;
      w[k] = al;
      w[K + k] = w1;
    }
  };
  // (batch sums as in the forward kernel: kept apart only where a lane's share is one chunk)
  constexpr int VB = V == 1 ? 1 : 0;
  f32x4 bacc[VB + 1];
  bacc[0] = f32x4(0.f);
  float baccd = 0.f;
  auto feature = [&](const f32x4 (&x)[V], const float* w, bool valid) __attribute__((always_inline)) {
    const float al = valid ? w[L.h] : 0.f;
    const float w1 = valid ? w[K + L.h] : 0.f;
    float dt = dot4(z[0], x[0]);
    if constexpr (VB) {
      bacc[0] += al * x[0];
    } else {
#pragma unroll
      for (int v = 0; v < V; ++v) {
        acc[v] += al * x[v];
        if (v > 0) dt += dot4(z[v], x[v]);
      }
    }
    baccd += w1 * dt;
  };
  auto fold = [&]() __attribute__((always_inline)) {
    if constexpr (VB) {
      acc[0] += bacc[0];
      bacc[0] = f32x4(0.f);
    }
    accd += baccd;
    baccd = 0.f;
  };
  // sum: this lane's share of sum_i alpha_ij g_i; t1: sum_i w1 <g_i, Z_j> of the lane's head
  auto store = [&](int64_t jj, const f32x4 (&sum)[V], float t1, const float (&wd)[K]) {
    const float der = t1 - pick<K>(wd, L.h);
    if (L.grp == 0 && L.col_ok) {
      f32x4 o[V];
#pragma unroll
      for (int v = 0; v < V; ++v) {
        const f32x4 as = *reinterpret_cast<const f32x4*>(&s_avec[0][L.el0 + 4 * v]);
        o[v] = sum[v] + der * as;
      }
      if (jj < n_local) {
        const float de = d_el[jj * K + L.h];
#pragma unroll
        for (int v = 0; v < V; ++v) {
          const f32x4 ad = *reinterpret_cast<const f32x4*>(&s_avec[1][L.el0 + 4 * v]);
          o[v] += de * ad;
        }
      }
      store_share<ES, V>(dZ + jj * ld_dz + static_cast<int64_t>(L.el0) * ES, o, L.left);
    }
    if (L.leader) d_er[jj * K + L.h] = der;
  };

  for (int r = wave; r < nr; r += kWaves) {
    if (__builtin_amdgcn_readfirstlane(sp.is_long[r])) continue;
    const int64_t row = row0 + r;
    const int64_t s = uniform64(sp.begin[r]), e = uniform64(sp.end[r]);
    reset(row_off + row);
    walk<ES, V, 2 * K, U>(a, L, s, e, s_col[wave], s_w[wave], pre, entry, feature, fold);
    float wd[K];
#pragma unroll
    for (int k = 0; k < K; ++k) wd[k] = wave_sum(wds[k]);
    f32x4 tot[V];
    group_sum<V>(acc, a.ln, tot);
    store(row_off + row, tot, head_sum(accd, a.ln), wd);
  }
  __syncthreads();
  for (int r = 0; r < nr; ++r) {
    if (!__builtin_amdgcn_readfirstlane(sp.is_long[r])) continue;   // the same for every wavefront
    const int64_t row = row0 + r;
    const int64_t s = uniform64(sp.begin[r]), e = uniform64(sp.end[r]);
    int64_t ps, pe;
    piece_of(s, e, wave, ps, pe);
    reset(row_off + row);
    walk<ES, V, 2 * K, U>(a, L, ps, pe, s_col[wave], s_w[wave], pre, entry, feature, fold);
    f32x4 part[V];
    group_sum<V>(acc, a.ln, part);
    const float t1 = head_sum(accd, a.ln);
    float wk[K];
#pragma unroll
    for (int k = 0; k < K; ++k) wk[k] = wave_sum(wds[k]);
    if (L.lane < K) s_part[wave][K + L.lane] = pick<K>(wk, L.lane);
    if (L.leader) s_part[wave][L.h] = t1;
    if (L.grp == 0) {
#pragma unroll
      for (int v = 0; v < V; ++v) *reinterpret_cast<f32x4*>(&s_part[wave][HDR + L.el0 + 4 * v]) = part[v];
    }
    __syncthreads();
    if (wave == 0) {
      f32x4 sum[V];
#pragma unroll
      for (int v = 0; v < V; ++v) sum[v] = f32x4(0.f);
      float th = 0.f, wd[K];
#pragma unroll
      for (int k = 0; k < K; ++k) wd[k] = 0.f;
      const int hh = L.h < K ? L.h : 0;
      for (int w = 0; w < kWaves; ++w) {
#pragma unroll
        for (int v = 0; v < V; ++v) sum[v] += *reinterpret_cast<const f32x4*>(&s_part[w][HDR + L.el0 + 4 * v]);
        th += s_part[w][hh];
#pragma unroll
        for (int k = 0; k < K; ++k) wd[k] += s_part[w][K + k];
      }
      store(row_off + row, sum, th, wd);
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------- small kernels
// dOUT = dH o [H > 0]
template <int ES>
__global__ __launch_bounds__(256) void gat_mask_kernel(const unsigned char* dH, int64_t ld_dh,
                                                      const unsigned char* H, int64_t ld_h, int64_t n,
                                                      int32_t d, unsigned char* out, int64_t ld_o) {
  const int nv = (d + 3) / 4;
  const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (t >= n * nv) return;
  const int64_t r = t / nv;
  const int c0 = static_cast<int>(t - r * nv) * 4;
  const f32x4 g = load4<ES>(dH + r * ld_dh + static_cast<int64_t>(c0) * ES);
  const f32x4 h = load4<ES>(H + r * ld_h + static_cast<int64_t>(c0) * ES);
  f32x4 o;
  o.x = h.x > 0.f ? g.x : 0.f;
  o.y = h.y > 0.f ? g.y : 0.f;
  o.z = h.z > 0.f ? g.z : 0.f;
  o.w = h.w > 0.f ? g.w : 0.f;
  store4<ES>(out + r * ld_o + static_cast<int64_t>(c0) * ES, o, d - c0);
}

// Gradient of the attention vectors: da_dst[f] = sum_{i < n_dst} d_el[i, head(f)] Z[i, f],
// da_src[f] = sum_{j < n} d_er[j, head(f)] Z[j, f]. Each workgroup sums a contiguous range
// of rows into part[block][2][d]; attn_finish_kernel adds the workgroups in index order.
template <int ES>
__global__ __launch_bounds__(256) void gat_attn_grad_kernel(const unsigned char* Z, int64_t ld_z,
                                                           int64_t n, int64_t n_dst, int heads,
                                                           Lanes ln, const float* d_el,
                                                           const float* d_er, int64_t rows_per_block,
                                                           float* part) {
  __shared__ float red[4][2][kMaxD];
  const LaneIds L = lane_ids(ln, heads);
  const int wave = threadIdx.x >> 6;
  const int64_t r0 = static_cast<int64_t>(blockIdx.x) * rows_per_block;
  const int64_t r1 = r0 + rows_per_block < n ? r0 + rows_per_block : n;
  const int hh = L.h < heads ? L.h : 0;
  f32x4 sd(0.f), ss(0.f);
  for (int64_t r = r0 + wave * L.ng + L.grp; r < r1; r += 4 * L.ng) {
    if (!L.col_ok) continue;
    const f32x4 z = clip4(load4<ES>(Z + r * ld_z + static_cast<int64_t>(L.el0) * ES), L.left);
    ss += d_er[r * heads + hh] * z;
    if (r < n_dst) sd += d_el[r * heads + hh] * z;
  }
  sd = group_sum(sd, ln);
  ss = group_sum(ss, ln);
  if (L.grp == 0) {
    *reinterpret_cast<f32x4*>(&red[wave][0][L.el0]) = sd;
    *reinterpret_cast<f32x4*>(&red[wave][1][L.el0]) = ss;
  }
  __syncthreads();
  const int d = ln.d;
  for (int t = threadIdx.x; t < 2 * d; t += 256) {
    const int which = t / d, f = t - which * d;
    float s = 0.f;
    for (int w = 0; w < 4; ++w) s += red[w][which][f];
    part[(static_cast<int64_t>(blockIdx.x) * 2 + which) * d + f] = s;
  }
}

// 32 outputs per workgroup; 8 slices of the workgroups' partial sums are added side by
// side, then the slices in order
__global__ __launch_bounds__(256) void gat_attn_finish_kernel(const float* part, int64_t n_blocks, int32_t d,
                                                             float* da_dst, float* da_src) {
  __shared__ float red[8][32];
  const int c = threadIdx.x & 31, sl = threadIdx.x >> 5;
  const int t = blockIdx.x * 32 + c;           // output index in [0, 2 d)
  float s = 0.f;
  if (t < 2 * d) {
    const int which = t / d, f = t - which * d;
    for (int64_t b = sl; b < n_blocks; b += 8) s += part[(b * 2 + which) * d + f];
  }
  red[sl][c] = s;
  __syncthreads();
  if (sl == 0 && t < 2 * d) {
    float tot = 0.f;
    for (int k = 0; k < 8; ++k) tot += red[k][c];
    const int which = t / d, f = t - which * d;
    (which == 0 ? da_dst : da_src)[f] = tot;
  }
}

// ---------------------------------------------------------------- host side
constexpr int kAttnBlocks = 1024;

bool lanes_for(int32_t heads, int32_t d_head, Lanes* ln) {
  if (heads != 1 && heads != 2 && heads != 4 && heads != 8) return false;
  if (d_head <= 0) return false;
  const int64_t d = static_cast<int64_t>(heads) * d_head;
  if (d > kMaxD) return false;
  int lg_g = 0, lg_lh = 0;
  if (heads == 1) {
    while ((4 << lg_g) < d) ++lg_g;
    lg_lh = lg_g;
  } else {
    if (d_head % 4 != 0) return false;
    const int lh = d_head / 4;
    if ((lh & (lh - 1)) != 0) return false;
    while ((1 << lg_lh) < lh) ++lg_lh;
    lg_g = lg_lh;
    for (int k = heads; k > 1; k >>= 1) ++lg_g;
  }
  ln->d = static_cast<int32_t>(d);
  ln->lg_g = lg_g;
  ln->lg_lh = lg_lh;
  ln->lg_v = 0;
  return true;
}

// The layout the edge kernels use: 16-byte lane shares (8 elements) for bf16 rows of 256
// bytes and more whose width and head width are 8 times a power of two, else `ln` itself.
Lanes edge_lanes(const Lanes& ln, int es) {
  Lanes w = ln;
  if (es == 2 && ln.d >= 128 && ln.d == (4 << ln.lg_g) && ln.lg_lh >= 1) {
    w.lg_g = ln.lg_g - 1;
    w.lg_lh = ln.lg_lh - 1;
    w.lg_v = 1;
  }
  return w;
}

sat_status check_dense(const void* p, int64_t rows, int64_t ld, int64_t d, int es) {
  if (rows > 0 && d > 0) {
    if (!p || ld < d) return SAT_EINVAL;
    if (!sat::aligned16(p) || ((ld * es) % 16) != 0) return SAT_EALIGN;
  }
  return SAT_OK;
}

sat_status check_view(const sat_part_view* pv, bool need_transpose) {
  if (!pv) return SAT_EINVAL;
  if (pv->n_local < 0 || pv->n_halo < 0 || pv->nnz < 0 || pv->nnz_halo < 0) return SAT_EINVAL;
  if (pv->n_local + pv->n_halo > INT32_MAX) return SAT_EUNSUPPORTED;
  if (!pv->rowptr) return SAT_EINVAL;
  if (pv->n_local > 0 && (!pv->split || (pv->nnz > 0 && !pv->col))) return SAT_EINVAL;
  if (need_transpose && pv->n_halo > 0 && (!pv->h_colptr || (pv->nnz_halo > 0 && !pv->h_row)))
    return SAT_EINVAL;
  return SAT_OK;
}

struct BwdPlan {
  int64_t off_dout, off_rowstat, off_del, off_der, off_part, total;
};

BwdPlan bwd_plan(int64_t n_local, int64_t n_halo, int32_t heads, int32_t d_head, int es) {
  auto up = [](int64_t v) { return (v + 255) / 256 * 256; };
  const int64_t d = static_cast<int64_t>(heads) * d_head;
  const int64_t ld = (d * es + 15) / 16 * 16;     // bytes per row of the masked gradient
  BwdPlan p;
  int64_t o = 0;
  p.off_dout = o;
  o += up(n_local * ld);
  p.off_rowstat = o;
  o += up(n_local * heads * 16);
  p.off_del = o;
  o += up(n_local * heads * 4);
  p.off_der = o;
  o += up((n_local + n_halo) * heads * 4);
  p.off_part = o;
  o += up(static_cast<int64_t>(kAttnBlocks) * 2 * d * 4);
  p.total = o;
  return p;
}

template <int ES, int K, int V>
sat_status run_fwd(const sat_part_view* pv, const void* Z, int64_t ld_z, Lanes ln, const float* el,
                   const float* er, float slope, int32_t act, void* H, int64_t ld_h, float* stats,
                   hipStream_t s) {
  const WalkArgs a{pv->rowptr, pv->rowptr + 1, pv->col, pv->n_local, pv->n_local + pv->n_halo,
                   static_cast<const unsigned char*>(Z), ld_z * ES, ln, slope};
  const int64_t gb = (pv->n_local + kRowsPerBlock - 1) / kRowsPerBlock;
  if (gb > INT32_MAX) return SAT_EUNSUPPORTED;
  gat_fwd_kernel<ES, K, V><<<dim3(static_cast<unsigned>(gb)), dim3(kWaves * kWave), 0, s>>>(
      a, el, er, act == SAT_ACT_RELU ? 1 : 0, static_cast<unsigned char*>(H), ld_h * ES, stats);
  return sat::check_launch();
}

// ln: the layout of the row-streaming kernels, lw: that of the edge kernels (V chunks per lane)
template <int ES, int K, int V>
sat_status run_bwd(const sat_part_view* pv, const void* Z, int64_t ld_z, Lanes ln, Lanes lw, const float* el,
                   const float* er, const float* stats, float slope, int32_t act, const void* dH,
                   int64_t ld_dh, const void* H, int64_t ld_h, const float* a_dst, const float* a_src,
                   void* dZ, int64_t ld_dz, float* da_dst, float* da_src, unsigned char* ws,
                   hipStream_t s) {
  const int64_t n_l = pv->n_local, n_h = pv->n_halo, n_bar = n_l + n_h;
  const int32_t d = ln.d;
  const BwdPlan p = bwd_plan(n_l, n_h, K, d / K, ES);
  f32x4* rowstat = reinterpret_cast<f32x4*>(ws + p.off_rowstat);
  float* d_el = reinterpret_cast<float*>(ws + p.off_del);
  float* d_er = reinterpret_cast<float*>(ws + p.off_der);
  float* part = reinterpret_cast<float*>(ws + p.off_part);
  const unsigned char* dOUT = static_cast<const unsigned char*>(dH);
  int64_t ld_g = ld_dh * ES;
  sat_status st;
  if (act == SAT_ACT_RELU) {
    unsigned char* m = ws + p.off_dout;
    const int64_t ldm = (static_cast<int64_t>(d) * ES + 15) / 16 * 16;
    const int64_t total = n_l * ((d + 3) / 4);
    const int64_t gb = (total + 255) / 256;
    if (gb > INT32_MAX) return SAT_EUNSUPPORTED;
    gat_mask_kernel<ES><<<dim3(static_cast<unsigned>(gb)), dim3(256), 0, s>>>(
        dOUT, ld_g, static_cast<const unsigned char*>(H), ld_h * ES, n_l, d, m, ldm);
    if ((st = sat::check_launch()) != SAT_OK) return st;
    dOUT = m;
    ld_g = ldm;
  }
  const dim3 block(kWaves * kWave);
  {   // destination side: rows i, gathers Z_j
    const WalkArgs a{pv->rowptr, pv->rowptr + 1, pv->col, n_l, n_bar,
                     static_cast<const unsigned char*>(Z), ld_z * ES, lw, slope};
    const int64_t gb = (n_l + kRowsPerBlock - 1) / kRowsPerBlock;
    if (gb > INT32_MAX) return SAT_EUNSUPPORTED;
    gat_bwd_dst_kernel<ES, K, V><<<dim3(static_cast<unsigned>(gb)), block, 0, s>>>(a, el, er, stats, dOUT,
                                                                             ld_g, d_el, rowstat);
    if ((st = sat::check_launch()) != SAT_OK) return st;
  }
  {   // source side, local rows j: the transposed entries of row j's local columns are those
      // columns themselves (the local block's pattern is symmetric)
    const WalkArgs a{pv->rowptr, pv->split, pv->col, n_l, n_l, dOUT, ld_g, lw, slope};
    const int64_t gb = (n_l + kRowsPerBlock - 1) / kRowsPerBlock;
    gat_bwd_src_kernel<ES, K, V, kUof<K, V>><<<dim3(static_cast<unsigned>(gb)), block, 0, s>>>(
        a, 0, n_l, er, rowstat, static_cast<const unsigned char*>(Z), ld_z * ES, d_el, a_dst, a_src,
        static_cast<unsigned char*>(dZ), ld_dz * ES, d_er);
    if ((st = sat::check_launch()) != SAT_OK) return st;
  }
  if (n_h > 0) {   // source side, halo rows: the transposed halo block
    const WalkArgs a{pv->h_colptr, pv->h_colptr + 1, pv->h_row, n_h, n_l, dOUT, ld_g, lw, slope};
    const int64_t gb = (n_h + kRowsPerBlock - 1) / kRowsPerBlock;
    if (gb > INT32_MAX) return SAT_EUNSUPPORTED;
    // rows of a few entries each: what counts is the number of rows in flight, so this
    // instance keeps 2 gathers in flight per group and fits twice as many wavefronts
    gat_bwd_src_kernel<ES, K, V, 2><<<dim3(static_cast<unsigned>(gb)), block, 0, s>>>(
        a, n_l, n_l, er, rowstat, static_cast<const unsigned char*>(Z), ld_z * ES, d_el, a_dst, a_src,
        static_cast<unsigned char*>(dZ), ld_dz * ES, d_er);
    if ((st = sat::check_launch()) != SAT_OK) return st;
  }
  {   // attention vectors
    const int64_t rpb = (n_bar + kAttnBlocks - 1) / kAttnBlocks;
    const int64_t nb = (n_bar + rpb - 1) / rpb;
    gat_attn_grad_kernel<ES><<<dim3(static_cast<unsigned>(nb)), dim3(256), 0, s>>>(
        static_cast<const unsigned char*>(Z), ld_z * ES, n_bar, n_l, K, ln, d_el, d_er, rpb, part);
    if ((st = sat::check_launch()) != SAT_OK) return st;
    gat_attn_finish_kernel<<<dim3(static_cast<unsigned>((2 * d + 31) / 32)), dim3(256), 0, s>>>(
        part, nb, d, da_dst, da_src);
    if ((st = sat::check_launch()) != SAT_OK) return st;
  }
  return SAT_OK;
}

}  // namespace

extern "C" sat_status sat_gat_scores(const void* Z, int64_t ld_z, int64_t n, int64_t n_dst,
                                     int32_t heads, int32_t d_head, const float* a_dst,
                                     const float* a_src, int32_t dtype, float* el, float* er,
                                     void* stream) {
  if (n < 0 || n_dst < 0 || n_dst > n) return SAT_EINVAL;
  if (dtype != SAT_F32 && dtype != SAT_BF16) return SAT_EINVAL;
  if (heads <= 0 || d_head <= 0) return SAT_EINVAL;
  Lanes ln;
  if (!lanes_for(heads, d_head, &ln)) return SAT_EUNSUPPORTED;
  const int es = dtype == SAT_BF16 ? 2 : 4;
  sat_status st;
  if ((st = check_dense(Z, n, ld_z, ln.d, es)) != SAT_OK) return st;
  if (n == 0) return SAT_OK;
  if (!a_dst || !a_src || !er || (n_dst > 0 && !el)) return SAT_EINVAL;
  const int64_t rows_per_block = 4 * kScoreRows * (kWave >> ln.lg_g);
  const int64_t gb = (n + rows_per_block - 1) / rows_per_block;
  if (gb > INT32_MAX) return SAT_EUNSUPPORTED;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (es == 2)
    gat_scores_kernel<2><<<dim3(static_cast<unsigned>(gb)), dim3(256), 0, s>>>(
        static_cast<const unsigned char*>(Z), ld_z * 2, n, n_dst, heads, ln, a_dst, a_src, el, er);
  else
    gat_scores_kernel<4><<<dim3(static_cast<unsigned>(gb)), dim3(256), 0, s>>>(
        static_cast<const unsigned char*>(Z), ld_z * 4, n, n_dst, heads, ln, a_dst, a_src, el, er);
  return sat::check_launch();
}

#define SAT_GAT_DISPATCH(FN, ...)                                   \
  do {                                                              \
    if (es == 2 && lw.lg_v == 1) {                                  \
      switch (heads) {                                              \
        case 1: return FN<2, 1, 2>(__VA_ARGS__);                    \
        case 2: return FN<2, 2, 2>(__VA_ARGS__);                    \
        case 4: return FN<2, 4, 2>(__VA_ARGS__);                    \
        default: return FN<2, 8, 2>(__VA_ARGS__);                   \
      }                                                             \
    }                                                               \
    if (es == 2) {                                                  \
      switch (heads) {                                              \
        case 1: return FN<2, 1, 1>(__VA_ARGS__);                    \
        case 2: return FN<2, 2, 1>(__VA_ARGS__);                    \
        case 4: return FN<2, 4, 1>(__VA_ARGS__);                    \
        default: return FN<2, 8, 1>(__VA_ARGS__);                   \
      }                                                             \
    }                                                               \
    switch (heads) {                                                \
      case 1: return FN<4, 1, 1>(__VA_ARGS__);                      \
      case 2: return FN<4, 2, 1>(__VA_ARGS__);                      \
      case 4: return FN<4, 4, 1>(__VA_ARGS__);                      \
      default: return FN<4, 8, 1>(__VA_ARGS__);                     \
    }                                                               \
  } while (0)

extern "C" sat_status sat_gat_aggregate_fwd(const sat_part_view* pv, const void* Z, int64_t ld_z,
                                            int32_t heads, int32_t d_head, int32_t dtype,
                                            const float* el, const float* er, float slope,
                                            int32_t act, void* H, int64_t ld_h, float* stats,
                                            void* stream) {
  sat_status st = check_view(pv, false);
  if (st != SAT_OK) return st;
  if (dtype != SAT_F32 && dtype != SAT_BF16) return SAT_EINVAL;
  if (act != SAT_ACT_IDENTITY && act != SAT_ACT_RELU) return SAT_EINVAL;
  if (heads <= 0 || d_head <= 0) return SAT_EINVAL;
  Lanes ln;
  if (!lanes_for(heads, d_head, &ln)) return SAT_EUNSUPPORTED;
  const int es = dtype == SAT_BF16 ? 2 : 4;
  if ((st = check_dense(Z, pv->n_local + pv->n_halo, ld_z, ln.d, es)) != SAT_OK) return st;
  if ((st = check_dense(H, pv->n_local, ld_h, ln.d, es)) != SAT_OK) return st;
  if (pv->n_local == 0) return SAT_OK;
  if (!el || !er || !stats) return SAT_EINVAL;
  if (!sat::aligned16(el) || !sat::aligned16(er) || !sat::aligned16(stats)) return SAT_EALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const Lanes lw = edge_lanes(ln, es);
  SAT_GAT_DISPATCH(run_fwd, pv, Z, ld_z, lw, el, er, slope, act, H, ld_h, stats, s);
}

extern "C" int64_t sat_gat_aggregate_bwd_workspace_bytes(int64_t n_local, int64_t n_halo,
                                                         int32_t heads, int32_t d_head,
                                                         int32_t dtype) {
  if (n_local < 0 || n_halo < 0 || heads <= 0 || d_head <= 0) return 0;
  return bwd_plan(n_local, n_halo, heads, d_head, dtype == SAT_BF16 ? 2 : 4).total;
}

extern "C" sat_status sat_gat_aggregate_bwd(const sat_part_view* pv, const void* Z, int64_t ld_z,
                                            int32_t heads, int32_t d_head, int32_t dtype,
                                            const float* el, const float* er, const float* stats,
                                            float slope, int32_t act, const void* dH, int64_t ld_dh,
                                            const void* H, int64_t ld_h, const float* a_dst,
                                            const float* a_src, void* dZ, int64_t ld_dz,
                                            float* da_dst, float* da_src, void* workspace,
                                            int64_t workspace_bytes, void* stream) {
  sat_status st = check_view(pv, true);
  if (st != SAT_OK) return st;
  if (dtype != SAT_F32 && dtype != SAT_BF16) return SAT_EINVAL;
  if (act != SAT_ACT_IDENTITY && act != SAT_ACT_RELU) return SAT_EINVAL;
  if (heads <= 0 || d_head <= 0) return SAT_EINVAL;
  Lanes ln;
  if (!lanes_for(heads, d_head, &ln)) return SAT_EUNSUPPORTED;
  const int es = dtype == SAT_BF16 ? 2 : 4;
  const int64_t n_l = pv->n_local, n_bar = pv->n_local + pv->n_halo;
  if ((st = check_dense(Z, n_bar, ld_z, ln.d, es)) != SAT_OK) return st;
  if ((st = check_dense(dH, n_l, ld_dh, ln.d, es)) != SAT_OK) return st;
  if (act == SAT_ACT_RELU && (st = check_dense(H, n_l, ld_h, ln.d, es)) != SAT_OK) return st;
  if ((st = check_dense(dZ, n_bar, ld_dz, ln.d, es)) != SAT_OK) return st;
  if (!a_dst || !a_src || !da_dst || !da_src) return SAT_EINVAL;
  if (n_bar > 0 && (!er || (n_l > 0 && (!el || !stats)))) return SAT_EINVAL;
  const int64_t need = bwd_plan(n_l, pv->n_halo, heads, d_head, es).total;
  if (!workspace || workspace_bytes < need) return SAT_EWORKSPACE;
  if (!sat::aligned256(workspace)) return SAT_EALIGN;
  if (!sat::aligned16(el) || !sat::aligned16(er) || !sat::aligned16(stats)) return SAT_EALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  if (n_l == 0) {   // no rows, hence no halo rows either: only the attention gradients, zero
    gat_attn_finish_kernel<<<dim3(static_cast<unsigned>((2 * ln.d + 31) / 32)), dim3(256), 0, s>>>(
        reinterpret_cast<const float*>(ws), 0, ln.d, da_dst, da_src);
    return sat::check_launch();
  }
  const Lanes lw = edge_lanes(ln, es);
  SAT_GAT_DISPATCH(run_bwd, pv, Z, ld_z, ln, lw, el, er, stats, slope, act, dH, ld_dh, H, ld_h, a_dst,
                   a_src, dZ, ld_dz, da_dst, da_src, ws, s);
}

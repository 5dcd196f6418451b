// LSTM of the embedding predictor (Sec. "Embedding Predictor") on the bf16 MFMA
// pipe with the exact three-way fp32 split of mx_tile.h, for hidden sizes 32
// and 64.
//
// A workgroup owns 128 nodes and all 4*d_s gate columns. Per time step the gate
// pre-activations [x_s | h_{s-1}] [Wx | Wh]^T are accumulated in registers
// (a wavefront holds the i, f, g, o blocks of the same (node, hidden unit)
// positions, so the cell update is register-local), c stays in registers, and
// h goes to LDS already split into bf16 pieces in the [node][unit] layout the
// next step's recurrent product reads as its A operand. Only S = h_tau is
// written to memory.
//
// The weights are split once per call by a small kernel into bf16 pieces
// [piece][gate column][k] (k padded to a multiple of 32 with zeros), so every
// workgroup streams them from L2 with plain 16-byte copies; x_s tiles are read
// from the history table through the id list and split while they are written
// to LDS. 128 nodes per workgroup (rather than 64) halves the weight traffic
// per node, which is what bounds this kernel once the products run 2.7x faster
// than on the fp32 pipe.
#include <math.h>

#include "mx_tile.h"
#include "sat_internal.h"

namespace {

using namespace sat::mx;

constexpr int kMaxTau = 8;
constexpr int kR = 128;  // nodes per workgroup (64 in the instance that runs from kept projections only)

struct SlotPtrs {
  const void* p[kMaxTau];
};

// Cached input projections (optional): proj[s] [n_nodes, 4 DS] fp32 holds x_s Wx^T of window
// slot s, node-major, gate blocks i, f, g, o. The first n_valid slots are READ instead of
// being multiplied out again (their x rows and the Wx tiles are then not loaded at all); a
// later slot (other than the window's first) whose pointer is not null is WRITTEN once its
// input part has been accumulated, before the recurrent part is added. Consecutive windows share all but one slot, and the
// accumulator of the input part is the same sum in the same order whichever step of the
// window the slot is, so reading it back gives bit-identical gates.
struct ProjPtrs {
  float* p[kMaxTau];
  int n_valid;
};

__device__ __forceinline__ float sigmoidf_(float x) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x));
}
__device__ __forceinline__ float tanhf_(float x) {
  return 2.0f * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-2.8853900817779268f * x)) - 1.0f;
}

// W [rows, k_in] fp32 (dense) -> P [3][rows][k_pad] bf16 pieces, zero for k >= k_in.
__global__ __launch_bounds__(256) void split_weights_kernel(const float* __restrict__ W, int rows,
                                                            int k_in, int k_pad,
                                                            uint16_t* __restrict__ P) {
  const int idx = blockIdx.x * 256 + threadIdx.x;  // one pair of k per thread
  const int pairs = k_pad / 2;
  if (idx >= rows * pairs) return;
  const int r = idx / pairs, k = 2 * (idx - r * pairs);
  const float x0 = k < k_in ? W[r * k_in + k] : 0.f;
  const float x1 = k + 1 < k_in ? W[r * k_in + k + 1] : 0.f;
  uint32_t pc[3];
  split2<3>(x0, x1, pc);
#pragma unroll
  for (int p = 0; p < 3; ++p)
    *reinterpret_cast<uint32_t*>(P + (static_cast<int64_t>(p) * rows + r) * k_pad + k) = pc[p];
}

// ESX = bytes per element of the cached embeddings x (4: fp32, split three ways;
// 2: bf16, used as it is, so the input products need one x piece only).
// WAVES = wavefronts per workgroup (4 or 8). LDS holds one workgroup per compute
// unit whatever WAVES is, so with 8 every SIMD has two wavefronts and one of them
// can read operands from LDS while the other's products run.
// R = nodes per workgroup. XPART false: every step's input part comes from the kept
// projections (proj.n_valid == tau): no x tile and no Wx tile is touched, the x staging
// buffer is not allocated.
template <int DS, int ESX, int WAVES, bool CACHE, int R = kR, bool XPART = true>
__global__ __launch_bounds__(64 * WAVES) void lstm_mx_kernel(SlotPtrs slots, int tau, int64_t n_rows_slot,
                                                      int64_t ld_slot,
                                                      const int32_t* __restrict__ ids,
                                                      int64_t n_nodes, int d, int k_pad,
                                                      const uint16_t* __restrict__ WxP,
                                                      const uint16_t* __restrict__ WhP,
                                                      const float* __restrict__ bias,
                                                      float* __restrict__ S,
                                                      float* __restrict__ save, ProjPtrs proj) {
  constexpr int NP = 3;             // pieces of an fp32 operand (x rows, h)
  // pieces of the weights: all three against fp32 rows (the exact product); two against bf16
  // rows, whose own precision (8 bits) the third piece (bits 17..24 of a weight) cannot matter to
  constexpr int NPB = ESX == 4 ? 3 : 2;
  constexpr int NT = 64 * WAVES;    // threads
  constexpr int WN = DS / 32;       // wavefronts along hidden units
  constexpr int WM = WAVES / WN;    // wavefronts along nodes
  constexpr int RB = R / (32 * WM); // 32-row blocks per wavefront
  static_assert(RB >= 1 && RB * 32 * WM == R, "wavefront grid must tile the node block");
  constexpr int NB = 4 * DS;        // gate columns
  constexpr int H_ROW_B = DS * 2 + 16;        // bytes per node row of a staged h piece
  constexpr int H_PIECE_B = R * H_ROW_B;
  constexpr int B_CHUNKS = NPB * NB * 4 / NT; // 16-byte weight chunks per thread per K step
  static_assert(XPART || CACHE, "without an input part every step is a cached one");
  __shared__ __attribute__((aligned(16))) unsigned char As[XPART ? 2 * tile_bytes<R, NP>() : 16];
  __shared__ __attribute__((aligned(16))) unsigned char Bs[tile_bytes<NB, NPB>()];
  __shared__ __attribute__((aligned(16))) unsigned char Hs[NP * H_PIECE_B];

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int c = lane & 31;
  const int64_t node0 = static_cast<int64_t>(blockIdx.x) * R;

  // An x tile is R rows of 32 elements = 16-byte chunks q = t + NT i of row q / CPR,
  // CPR chunks per row (fp32: 8, bf16: 4). Table row of each chunk's node (-1: nothing
  // to load):
  constexpr int CPR = ESX == 4 ? 8 : 4;
  constexpr int XROWS = R * CPR / NT;
  int64_t arow[XROWS];
#pragma unroll
  for (int i = 0; i < XROWS; ++i) {
    const int64_t node = node0 + (t + NT * i) / CPR;
    int64_t r = -1;
    if (XPART && node < n_nodes) {
      r = ids ? static_cast<int64_t>(ids[node]) : node;
      if (r < 0 || r >= n_rows_slot) r = -1;
    }
    arow[i] = r;
  }
  const int unit = 32 * wn + c;
  const float b_i = bias[unit], b_f = bias[DS + unit], b_g = bias[2 * DS + unit],
              b_o = bias[3 * DS + unit];

  float cstate[RB][16];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int r = 0; r < 16; ++r) cstate[rb][r] = 0.f;
  float hval[RB][16];

  // weight chunk c (16 bytes): piece = c / (NB * 4), column n = (c / 4) % NB, k chunk = c % 4
  auto load_w = [&](const uint16_t* P, int kp, int k0, u32x4 (&rw)[B_CHUNKS]) {
#pragma unroll
    for (int i = 0; i < B_CHUNKS; ++i) {
      const int ch = t + NT * i;
      const int piece = ch / (NB * 4), n = (ch >> 2) % NB, kc = ch & 3;
      rw[i] = *reinterpret_cast<const u32x4*>(P + (static_cast<int64_t>(piece) * NB + n) * kp + k0 +
                                              8 * kc);
    }
  };
  // the chunks i with i % 6 == part only (the six parts together are load_w)
  auto load_w_part = [&](const uint16_t* P, int kp, int k0, u32x4 (&rw)[B_CHUNKS], auto part_tag) {
    constexpr int PART = decltype(part_tag)::value;
#pragma unroll
    for (int i = PART; i < B_CHUNKS; i += 6) {
      const int ch = t + NT * i;
      const int piece = ch / (NB * 4), n = (ch >> 2) % NB, kc = ch & 3;
      rw[i] = *reinterpret_cast<const u32x4*>(P + (static_cast<int64_t>(piece) * NB + n) * kp + k0 +
                                              8 * kc);
    }
  };
  auto store_w = [&](const u32x4 (&rw)[B_CHUNKS]) {
#pragma unroll
    for (int i = 0; i < B_CHUNKS; ++i) {
      const int ch = t + NT * i;
      const int piece = ch / (NB * 4), n = (ch >> 2) % NB, kc = ch & 3;
      *reinterpret_cast<u32x4*>(Bs + piece * piece_bytes<NB>() + swz(n, kc)) = rw[i];
    }
  };

  const int nk = k_pad / BK;
  struct XRegs {
    u32x4 v[XROWS];
  };
  auto load_x = [&](int j, XRegs& ra) {   // x tile j of the stream (zeros past the end)
    const int sj = j / nk;
    const bool live = sj < tau;
    if constexpr (ESX == 4) {
      const int k = (j - sj * nk) * BK + ((t & 7) << 2);
      const float* xs = static_cast<const float*>(slots.p[live ? sj : 0]);
#pragma unroll
      for (int i = 0; i < XROWS; ++i) {
        u32x4 v = {0u, 0u, 0u, 0u};
        // only ISSUE the load here: anything that looks at v (the zeroing of elements past
        // d is in store_x) would make the wavefront wait for HBM before its products
        if (live && arow[i] >= 0 && k < d)
          v = *reinterpret_cast<const u32x4*>(xs + arow[i] * ld_slot + k);
        ra.v[i] = v;
      }
    } else {
      const int k = (j - sj * nk) * BK + ((t & 3) << 3);
      const uint16_t* xs = static_cast<const uint16_t*>(slots.p[live ? sj : 0]);
#pragma unroll
      for (int i = 0; i < XROWS; ++i) {
        u32x4 v = {0u, 0u, 0u, 0u};
        if (live && arow[i] >= 0 && k < d) {   // d % 8 == 0 here: whole chunks only
          v = *reinterpret_cast<const u32x4*>(xs + arow[i] * ld_slot + k);
        }
        ra.v[i] = v;
      }
    }
  };
  auto store_x = [&](const XRegs& ra, unsigned char* dst, int j) {   // j: the tile's stream index
    const int kx = (j % nk) * BK + ((t & 7) << 2);   // fp32: first of this thread's 4 elements
#pragma unroll
    for (int i = 0; i < XROWS; ++i) {
      const int q = t + NT * i;
      if constexpr (ESX == 4) {   // 4 floats -> 4 bf16 of each of the three pieces
        uint32_t lo[NP], hi[NP];
        // (cast the whole vector: a bit cast applied to one vector element reads element 0)
        f32x4 f = __builtin_bit_cast(f32x4, ra.v[i]);
        if (kx + 3 >= d) {   // elements past d lie in the row's padding
          if (kx + 1 >= d) f.y = 0.f;
          if (kx + 2 >= d) f.z = 0.f;
          f.w = 0.f;
        }
        split2<NP>(f.x, f.y, lo);
        split2<NP>(f.z, f.w, hi);
        unsigned char* sdst = dst + swz(q >> 3, (q & 7) >> 1) + ((q & 1) << 3);
#pragma unroll
        for (int p = 0; p < NP; ++p)
          *reinterpret_cast<u32x2*>(sdst + p * piece_bytes<R>()) = u32x2{lo[p], hi[p]};
      } else {
        *reinterpret_cast<u32x4*>(dst + swz(q >> 2, q & 3)) = ra.v[i];
      }
    }
  };
  // steps [0, s_first) take their input part from the cache: the stream of x tiles starts at
  // step s_first
  const int s_first = !XPART ? tau : CACHE ? (proj.n_valid < tau ? proj.n_valid : tau) : 0;
  const int j0 = s_first * nk;
  u32x4 rw[B_CHUNKS];
  XRegs ra0;
  if (XPART && s_first < tau) {
    if constexpr (!CACHE) load_w(WxP, k_pad, 0, rw);
    load_x(j0, ra0);
    store_x(ra0, As + (j0 & 1) * tile_bytes<R, NP>(), j0);   // first tile -> its half of the double buffer
    load_x(j0 + 1, ra0);
  }

  // Gate pre-activations of the input part of step s from the kept projections, in the
  // accumulator's layout: for a fixed register the 32 lanes of a half-wavefront read 128
  // contiguous bytes of one node's row. One base address per group of four registers (rows
  // 8 q + 4 (lane / 32) + 0..3): the sixteen loads of a group differ by constants that fit
  // the instruction's offset field. Only issues the loads.
  const bool whole = CACHE && node0 + R <= n_nodes;      // uniform: every node of the block exists
  auto load_gates = [&](int s, f32x16 (&acc)[RB][4]) __attribute__((always_inline)) {
      const float* P = proj.p[s];
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int64_t nodeq = node0 + 32 * (wm * RB + rb) + 8 * q + 4 * (lane >> 5);
          if (whole) {
            const float* base = P + nodeq * NB + unit;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
              for (int g = 0; g < 4; ++g) {
                if (g == 1 && s == 0) continue;     // c_0 = 0: the forget gate is not looked at
                acc[rb][g][4 * q + i] = base[i * NB + g * DS];
              }
          } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const bool ok = nodeq + i < n_nodes;
              const float* row = P + (ok ? nodeq + i : 0) * NB + unit;
#pragma unroll
              for (int g = 0; g < 4; ++g) {
                if (g == 1 && s == 0) continue;
                acc[rb][g][4 * q + i] = ok ? row[g * DS] : 0.f;
              }
            }
          }
        }
  };
  // One time step. cached_tag: whether the step's input part comes from the kept projections
  // (a compile-time switch: the two kinds of step are separate loops below, so neither
  // carries the other's registers).
  auto step = [&](int s, auto cached_tag) __attribute__((always_inline)) {
    constexpr bool cached = CACHE && decltype(cached_tag)::value;
    f32x16 acc[RB][4];
    if constexpr (cached) {
      // (requesting step s + 1's gates a step ahead, into a second set of accumulators, was
      // tried for the instance that runs from kept projections only: 36 registers spill)
      load_gates(s, acc);
    } else {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[rb][g][r] = 0.f;
    }

    // one K step of products, B from the staged weight tile (always three pieces).
    // A operand: the staged x tile `Ax` (swizzled 64-byte rows), or if Ax == nullptr
    // the h pieces in Hs (padded rows), k chunk offset a_kc0. NPA = number of A
    // pieces: 3 for fp32 data (six products), 1 for bf16 x (three products:
    // the value itself against each weight piece, smallest first).
    auto products = [&](auto npa_tag, const unsigned char* Ax, int a_kc0, auto&& mid) {
      constexpr int NPA = decltype(npa_tag)::value;
      constexpr int NQ = NPA == 3 ? (NPB == 3 ? 6 : 5) : NPB;
#pragma unroll
      for (int kc = 0; kc < BK / 16; ++kc) {
        bf16x8 a[RB][NPA];
#pragma unroll
        for (int p = 0; p < NPA; ++p)
#pragma unroll
          for (int rb = 0; rb < RB; ++rb)
            a[rb][p] = Ax ? read_operand(Ax + p * piece_bytes<R>(), 32 * (wm * RB + rb), kc, lane)
                          : *reinterpret_cast<const bf16x8*>(
                                Hs + p * H_PIECE_B + (32 * (wm * RB + rb) + c) * H_ROW_B +
                                32 * (a_kc0 + kc) + 16 * (lane >> 5));
        // two gates at a time: their weight fragments are all that is held besides a
#pragma unroll
        for (int gp = 0; gp < 2; ++gp) {
          // the step's global loads go out a few at a time between the blocks of products: issued
          // in one burst they hold the wavefront at the memory pipe while the matrix pipe idles
          bf16x8 b[2][NPB];
#pragma unroll
          for (int p = 0; p < NPB; ++p)
#pragma unroll
            for (int g = 0; g < 2; ++g)
              b[g][p] = read_operand(Bs + p * piece_bytes<NB>(), (2 * gp + g) * DS + 32 * wn, kc, lane);
#pragma unroll
          for (int q = 0; q < NQ; ++q) {
            // the step's global loads go out one or two at a time between the products: issued in
            // one burst they hold the wavefront at the memory pipe while the matrix pipe idles
            if (q == 0 || q == NQ / 2) {
              __builtin_amdgcn_sched_barrier(0);
              mid(4 * kc + 2 * gp + (q == 0 ? 0 : 1));
              __builtin_amdgcn_sched_barrier(0);
            }
            // (a piece, b piece), smallest terms first; with two weight pieces against three
            // pieces of h: (2,0) (1,1) (1,0) (0,1) (0,0)
            const int pa = NPA == 3 ? (NPB == 3 ? product_a<3>(q) : (q == 0 ? 2 : (q < 3 ? 1 : 0))) : 0;
            const int pb = NPA == 3 ? (NPB == 3 ? product_b<3>(q) : (q == 1 || q == 3 ? 1 : 0)) : NPB - 1 - q;
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
              for (int g = 0; g < 2; ++g) {
                // c_0 = 0: the forget gate is not needed at the first step. (A run-time test on
                // purpose: as a compile-time switch it removes the branches between the
                // products, and the scheduler then hoists operand reads until it spills.)
                if (s == 0 && 2 * gp + g == 1) continue;
                acc[rb][2 * gp + g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    a[rb][pa], b[g][pb], acc[rb][2 * gp + g], 0, 0, 0);
              }
          }
        }
      }
    };

    // ---- input part: x_s Wx^T, K = d (padded to k_pad with zero weights). The x
    // tiles of all time steps form one stream j = s * nk + i. Their rows come
    // from HBM through the id list (the slowest loads of the kernel), so they get
    // two product phases to arrive: while tile j is multiplied out of one half of
    // the LDS double buffer, tile j+1 already sits in the other half and tile j+2
    // is in flight in registers. Weight tiles (L2) form one stream too (per time step
    // the nk tiles of Wx, then from the second step on the tiles of Wh) and are always
    // one tile ahead in registers, across the phase boundary as well (not across the cell
    // update: the registers are needed there).
    if constexpr (CACHE) {
      if (!cached) load_w(WxP, k_pad, 0, rw);
      if (cached && s > 0) load_w(WhP, DS, 0, rw);   // (the input part, when it runs, leaves this tile in flight)
    } else {
      if (s > 0) load_w(WxP, k_pad, 0, rw);
    }
    for (int i = 0; i < (cached ? 0 : nk); ++i) {
      const int j = s * nk + i;
      __syncthreads();
      store_w(rw);
      store_x(ra0, As + ((j + 1) & 1) * tile_bytes<R, NP>(), j + 1);
      __syncthreads();
      // next weight tile: the input part's next one, or the recurrent part's first
      const bool w_in = i + 1 < nk;
      const bool w_any = w_in || s > 0;
      const uint16_t* wP = w_in ? WxP : WhP;
      const int w_kp = w_in ? k_pad : DS;
      const int w_k0 = w_in ? (i + 1) * BK : 0;
      auto mid = [&](int blk) __attribute__((always_inline)) {   // blk = 0..7
        if (blk == 0) load_x(j + 2, ra0);
        else if (!w_any || blk == 1) return;
        else if (blk == 2) load_w_part(wP, w_kp, w_k0, rw, std::integral_constant<int, 0>{});
        else if (blk == 3) load_w_part(wP, w_kp, w_k0, rw, std::integral_constant<int, 1>{});
        else if (blk == 4) load_w_part(wP, w_kp, w_k0, rw, std::integral_constant<int, 2>{});
        else if (blk == 5) load_w_part(wP, w_kp, w_k0, rw, std::integral_constant<int, 3>{});
        else if (blk == 6) load_w_part(wP, w_kp, w_k0, rw, std::integral_constant<int, 4>{});
        else load_w_part(wP, w_kp, w_k0, rw, std::integral_constant<int, 5>{});
      };
      products(std::integral_constant<int, ESX == 4 ? 3 : 1>{}, As + (j & 1) * tile_bytes<R, NP>(), 0, mid);
    }
    // keep the input part for the windows to come (not at s = 0: the forget gate's columns are
    // skipped there, and a window's oldest slot is never read again anyway)
    if (CACHE && !cached && s > 0 && proj.p[s] != nullptr) {
      float* P = proj.p[s];
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int64_t nodeq = node0 + 32 * (wm * RB + rb) + 8 * q + 4 * (lane >> 5);
          float* base = P + nodeq * NB + unit;
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (whole || nodeq + i < n_nodes) {
#pragma unroll
              for (int g = 0; g < 4; ++g) {
                // with a window of two a kept matrix is only ever read at the first step, where
                // the forget gate is not looked at: its block is not written at all
                if (g == 1 && tau == 2) continue;
                base[i * NB + g * DS] = acc[rb][g][4 * q + i];
              }
            }
        }
    }
    // ---- recurrent part: h_{s-1} Wh^T, K = DS (h_0 = 0: nothing to add at s = 0)
    if (s > 0) {
      for (int k0 = 0; k0 < DS; k0 += BK) {
        __syncthreads();
        store_w(rw);
        __syncthreads();
        const bool w_more = k0 + BK < DS;
        auto mid = [&](int blk) __attribute__((always_inline)) {
          if (blk < 2 || !w_more) return;
          if (blk == 2) load_w_part(WhP, DS, k0 + BK, rw, std::integral_constant<int, 0>{});
          else if (blk == 3) load_w_part(WhP, DS, k0 + BK, rw, std::integral_constant<int, 1>{});
          else if (blk == 4) load_w_part(WhP, DS, k0 + BK, rw, std::integral_constant<int, 2>{});
          else if (blk == 5) load_w_part(WhP, DS, k0 + BK, rw, std::integral_constant<int, 3>{});
          else if (blk == 6) load_w_part(WhP, DS, k0 + BK, rw, std::integral_constant<int, 4>{});
          else load_w_part(WhP, DS, k0 + BK, rw, std::integral_constant<int, 5>{});
        };
        products(std::integral_constant<int, 3>{}, nullptr, k0 / 16, mid);
      }
    }
    // ---- cell update, register-local
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float gi = sigmoidf_(acc[rb][0][r] + b_i);
        const float gg = tanhf_(acc[rb][2][r] + b_g);
        const float go = sigmoidf_(acc[rb][3][r] + b_o);
        float gf = 0.f;   // c_0 = 0: the forget gate does not matter at the first step
        if (s == 0) {
          cstate[rb][r] = gi * gg;
        } else {
          gf = sigmoidf_(acc[rb][1][r] + b_f);
          cstate[rb][r] = __builtin_fmaf(gf, cstate[rb][r], gi * gg);   // (one rounding of gi gg, then one of the sum: spelt out so that every kernel that updates a cell does the same)
        }
        hval[rb][r] = go * tanhf_(cstate[rb][r]);
        if (save != nullptr) {   // training: keep the step's gates, cell and hidden state
          const int64_t node = node0 + 32 * (wm * RB + rb) + acc_row(r, lane);
          if (node < n_nodes) {
            float* rec = save + (static_cast<int64_t>(s) * n_nodes + node) * (6 * DS) + unit;
            rec[0] = gi;
            rec[DS] = gf;
            rec[2 * DS] = gg;
            rec[3 * DS] = go;
            rec[4 * DS] = cstate[rb][r];
            rec[5 * DS] = hval[rb][r];
          }
        }
      }
    if (s + 1 < tau) {
      __syncthreads();  // every wavefront has finished reading Hs for this step
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          uint32_t pc[NP];
          split2<NP>(hval[rb][r], 0.f, pc);
          const int row = 32 * (wm * RB + rb) + acc_row(r, lane);
#pragma unroll
          for (int p = 0; p < NP; ++p)
            *reinterpret_cast<uint16_t*>(Hs + p * H_PIECE_B + row * H_ROW_B + 2 * unit) =
                static_cast<uint16_t>(pc[p] & 0xffffu);
        }
      // the next step's first __syncthreads orders these writes before any read
    }
  };
  if constexpr (CACHE)
    for (int s = 0; s < s_first; ++s) step(s, std::true_type{});
  if constexpr (XPART)
    for (int s = s_first; s < tau; ++s) step(s, std::false_type{});
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int64_t node = node0 + 32 * (wm * RB + rb) + acc_row(r, lane);
      if (node < n_nodes) S[node * DS + unit] = hval[rb][r];
    }
}

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

}  // namespace

namespace sat {

// lstm_proj.hip: P = x Wx^T for one slot, bit-compatible with the input part accumulated here
bool lstm_proj_serves(int32_t d, int32_t d_s, int es_x, int64_t n_nodes);
sat_status launch_lstm_proj(const void* X, int64_t n_rows_slot, int64_t ld_slot, const int32_t* ids,
                            int64_t n_nodes, const void* WxP, float* P, hipStream_t st);

// lstm_recur.hip: the time steps alone, from kept projections of every slot (d_s = 64)
sat_status launch_lstm_recur(float* const* proj, int tau, int64_t n_nodes, const void* WhP, const float* bias,
                             float* S, hipStream_t st);

// lstm_fused16.hip: the whole LSTM over bf16 rows of 256 elements with all weights in registers
bool lstm_fused16_serves(int32_t d, int32_t d_s, int es_x, int64_t n_nodes);
sat_status launch_lstm_fused16(const void* const* slot_ptrs, int tau, int64_t n_rows_slot, int64_t ld_slot,
                               const int32_t* ids, int64_t n_nodes, const void* WxP, const void* WhP,
                               const float* bias, float* S, hipStream_t st);

// Bytes of workspace the split-weight copies need (0 if this path does not serve d_s).
int64_t lstm_mx_workspace_bytes(int32_t d, int32_t d_s) {
  if (d_s != 32 && d_s != 64) return 0;
  const int64_t k_pad = round_up(d, 32);
  return round_up(3 * 4 * d_s * k_pad * 2, 256) + round_up(3 * 4 * d_s * static_cast<int64_t>(d_s) * 2, 256);
}

// S [n_nodes, d_s] = last hidden state of the LSTM over the tau slots (elements of
// es_x bytes: 4 fp32, 2 bf16; weights and S are fp32). ws points at
// lstm_mx_workspace_bytes() bytes, 256-byte aligned. Only d_s = 32 and 64.
// proj (nullable): HOST array of tau device pointers (each nullable), see ProjPtrs; the first
// n_proj_valid of them are read, the others written.
// save (nullable): [tau][n_nodes][6 d_s] fp32, per step and node the activated gates
// i, f, g, o, the cell state c and the hidden state h (what back-propagation needs).
sat_status launch_lstm_mx(const void* const* slot_ptrs, int es_x, int tau, int64_t n_rows_slot,
                          int64_t ld_slot, const int32_t* ids, int64_t n_nodes, int32_t d,
                          int32_t d_s, const float* Wx, const float* Wh, const float* b, float* S,
                          void* ws, hipStream_t st, float* save, float* const* proj, int n_proj_valid) {
  const int k_pad = static_cast<int>(round_up(d, 32));
  const int nb = 4 * d_s;
  uint16_t* WxP = static_cast<uint16_t*>(ws);
  uint16_t* WhP = WxP + round_up(3 * static_cast<int64_t>(nb) * k_pad * 2, 256) / 2;
  split_weights_kernel<<<dim3((nb * (k_pad / 2) + 255) / 256), dim3(256), 0, st>>>(Wx, nb, d, k_pad,
                                                                                  WxP);
  split_weights_kernel<<<dim3((nb * (d_s / 2) + 255) / 256), dim3(256), 0, st>>>(Wh, nb, d_s, d_s,
                                                                                WhP);
  sat_status rc = sat::check_launch();
  if (rc != SAT_OK) return rc;
  SlotPtrs sp;
  for (int s = 0; s < kMaxTau; ++s) sp.p[s] = s < tau ? slot_ptrs[s] : nullptr;
  ProjPtrs pp;
  for (int s = 0; s < kMaxTau; ++s) pp.p[s] = (proj && s < tau) ? proj[s] : nullptr;
  pp.n_valid = proj ? n_proj_valid : 0;
  // Steady state of a sliding window: every slot but the newest has its projection. The newest
  // one's is then made by the weights-in-registers product kernel (same sums, bit for bit),
  // and the time steps run from the kept matrices alone: no x tile, no Wx tile in this kernel.
  if (proj && save == nullptr && n_proj_valid == tau - 1 && tau >= 2 && proj[tau - 1] != nullptr &&
      lstm_proj_serves(d, d_s, es_x, n_nodes)) {
    rc = launch_lstm_proj(slot_ptrs[tau - 1], n_rows_slot, ld_slot, ids, n_nodes, WxP, proj[tau - 1], st);
    if (rc != SAT_OK) return rc;
    pp.n_valid = tau;
  }
  if (pp.n_valid == tau && proj && d_s == 64 && (reinterpret_cast<uintptr_t>(b) & 15u) == 0) {
    // the time steps alone: weights in registers, products transposed, gates requested a step
    // ahead (lstm_recur.hip). (This kernel's own instance for the case, XPART = false, took
    // 0.96 ms on the bench workload; with 64 nodes and four wavefronts per workgroup, two
    // workgroups per compute unit, 1.38 ms: the weight tiles are then staged twice as often.)
    bool aligned = true;
    for (int s = 0; s < tau; ++s) aligned = aligned && (reinterpret_cast<uintptr_t>(proj[s]) & 15u) == 0;
    if (aligned) return launch_lstm_recur(proj, tau, n_nodes, WhP, b, S, st);
  }
  if (pp.n_valid == tau && proj && d_s == 64 && es_x == 4) {   // the same from this file's kernel
    const int64_t blocks = (n_nodes + kR - 1) / kR;
    if (blocks > INT32_MAX) return SAT_EUNSUPPORTED;
    lstm_mx_kernel<64, 4, 8, true, kR, false><<<dim3(static_cast<unsigned>(blocks)), dim3(512), 0, st>>>(
        sp, tau, n_rows_slot, ld_slot, ids, n_nodes, d, k_pad, WxP, WhP, b, S, save, pp);
    return sat::check_launch();
  }
  // bf16 rows of 256 elements, nothing kept and nothing to keep: weights in registers, the
  // rows through an LDS tile (same sums, bit for bit)
  if (!proj && save == nullptr && lstm_fused16_serves(d, d_s, es_x, n_nodes) && n_rows_slot > 0 &&
      (reinterpret_cast<uintptr_t>(b) & 15u) == 0 && (ld_slot % 8) == 0) {
    bool aligned = true;
    for (int s = 0; s < tau; ++s) aligned = aligned && (reinterpret_cast<uintptr_t>(slot_ptrs[s]) & 15u) == 0;
    if (aligned) return launch_lstm_fused16(slot_ptrs, tau, n_rows_slot, ld_slot, ids, n_nodes, WxP, WhP, b, S, st);
  }
  const int64_t blocks = (n_nodes + kR - 1) / kR;
  if (blocks > INT32_MAX) return SAT_EUNSUPPORTED;
  const dim3 grid(static_cast<unsigned>(blocks));
#define SAT_LSTM_MX(DS, ESX, WAVES)                                                            \
  do {                                                                                         \
    if (proj)                                                                                  \
      lstm_mx_kernel<DS, ESX, WAVES, true><<<grid, dim3(64 * WAVES), 0, st>>>(                 \
          sp, tau, n_rows_slot, ld_slot, ids, n_nodes, d, k_pad, WxP, WhP, b, S, save, pp);    \
    else                                                                                       \
      lstm_mx_kernel<DS, ESX, WAVES, false><<<grid, dim3(64 * WAVES), 0, st>>>(                \
          sp, tau, n_rows_slot, ld_slot, ids, n_nodes, d, k_pad, WxP, WhP, b, S, save, pp);    \
  } while (0)
  if (d_s == 32 && es_x == 4) SAT_LSTM_MX(32, 4, 4);
  else if (d_s == 32) SAT_LSTM_MX(32, 2, 4);
  else if (es_x == 4) SAT_LSTM_MX(64, 4, 8);
  else SAT_LSTM_MX(64, 2, 8);
#undef SAT_LSTM_MX
  return sat::check_launch();
}

}  // namespace sat

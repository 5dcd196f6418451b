// LSTM of the embedding predictor (Sec. "Embedding Predictor") over bf16 rows of 256
// elements, d_s = 64, every slot multiplied out, with ALL weights in registers.
//
// The products are formed TRANSPOSED, gates^T = Wx x^T + Wh h^T: wavefront w of a workgroup
// owns hidden units 8 w .. 8 w + 7, its 32 MFMA rows being row 8 g + u = gate g of unit
// 8 w + u; those rows of Wx (two bf16 pieces per weight against bf16 rows, as in lstm_mx.hip:
// 128 registers) and of Wh (32 registers) stay in registers for the life of the workgroup,
// the nodes are the columns. A lane's accumulator registers are then all four gates of four
// units of ONE node: the cell update is register-local, c never leaves registers, h leaves
// as 8-byte LDS writes per piece and S as 16-byte stores. No weight tile is ever staged or
// streamed; what moves is the window's rows, once: wavefront w reads the 512-byte rows of
// nodes 4 w .. 4 w + 3 of the next (tile, slot) a step ahead (two rows per load instruction,
// whole lines), and writes them to a padded row-major tile in LDS at the end of the step;
// every wavefront reads its MFMA column operands from that tile (16-byte reads, rows padded
// by 16 bytes so that 16 lanes cover all banks). A workgroup walks many tiles of 32 nodes
// with ONE barrier per time step: the row tile and h both alternate between two buffers.
// The input part of a step does not depend on the step before it: it is multiplied out
// one step early, in the same stretch of code as that step's cell update, so that products
// and transcendentals can be in flight together (measured: 10 % of the kernel's time; pinning
// one product between every few vector instructions with scheduling fences gave no more).
//
// Bit-compatibility with lstm_mx_kernel<64, 2, ...>: an accumulator element takes the same
// products in the same order (x part: k chunks ascending, the low weight piece before the
// high one; h part: k chunks ascending, (h piece, W piece) = (2,0) (1,1) (1,0) (0,1) (0,0);
// which operand is the MFMA's row operand does not change an element's sum), then the same
// bias addition and the same activation code. (At the first step the forget gate's rows are
// multiplied out here and not looked at.)
#include "mx_tile.h"
#include "sat_internal.h"

namespace {

using namespace sat::mx;

constexpr int kD = 256, kDS = 64, kNB = 4 * kDS, kR = 32, kMaxTau = 8;
constexpr int kXRowB = kD * 2 + 16;            // bytes per node row of the staged x tile (padded)
constexpr int kHRowB = kDS * 2 + 16;           // bytes per node row of a staged h piece (padded)
constexpr int kHPieceB = kR * kHRowB;
constexpr int kKX = kD / 16, kKH = kDS / 16;   // 16-wide k chunks of the two parts

struct Slots16 {
  const unsigned char* p[kMaxTau];
};

__device__ __forceinline__ float sigmoidf_(float x) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x));
}
__device__ __forceinline__ float tanhf_(float x) {
  return 2.0f * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-2.8853900817779268f * x)) - 1.0f;
}

// IDS: rows of the slots through the id list (else row of node k is k).
template <bool IDS>
__global__ __launch_bounds__(512, 2) void lstm_fused16_kernel(Slots16 slots, int tau, int64_t n_rows_slot,
                                                             int64_t row_bytes,
                                                             const int32_t* __restrict__ ids,
                                                             int64_t n_nodes,
                                                             const uint16_t* __restrict__ WxP,
                                                             const uint16_t* __restrict__ WhP,
                                                             const float* __restrict__ bias,
                                                             float* __restrict__ S) {
  constexpr int NP = 3;        // pieces of h
  constexpr int NPW = 2;       // pieces of a weight
  __shared__ __attribute__((aligned(16))) unsigned char Xs[2][kR * kXRowB];
  __shared__ __attribute__((aligned(16))) unsigned char Hs[2][NP * kHPieceB];
  __shared__ __attribute__((aligned(16))) float Bs[kNB];
  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int half = lane >> 5, c = lane & 31;

  // weights: row m = lane % 32 of this wavefront is gate m / 8 of unit 8 wave + m % 8, i.e.
  // gate column n = (m / 8) * 64 + 8 wave + m % 8 of the split-weight arrays [3][256][k]
  bf16x8 awx[kKX][NPW], awh[kKH][NPW];
  {
    const int n = (c >> 3) * kDS + 8 * wave + (c & 7);
#pragma unroll
    for (int kc = 0; kc < kKX; ++kc)
#pragma unroll
      for (int p = 0; p < NPW; ++p)
        awx[kc][p] = *reinterpret_cast<const bf16x8*>(WxP + (static_cast<int64_t>(p) * kNB + n) * kD + 16 * kc +
                                                      8 * half);
#pragma unroll
    for (int kc = 0; kc < kKH; ++kc)
#pragma unroll
      for (int p = 0; p < NPW; ++p)
        awh[kc][p] = *reinterpret_cast<const bf16x8*>(WhP + (static_cast<int64_t>(p) * kNB + n) * kDS + 16 * kc +
                                                      8 * half);
  }
  // this lane's units: 8 wave + 4 half + 0..3 (of node c of the tile); their biases wait in LDS
  const int unit0 = 8 * wave + 4 * half;
  if (t < kNB) Bs[t] = bias[t];

  // This lane's two rows of a tile's x rows: nodes node0 + 4 wave + 2 i + half, bytes 16 c .. 16 c + 15.
  // A node whose table row is outside the table contributes zeros (its loads go to row 0 and
  // are masked when they are staged); nodes past the end take the last node's row (never stored).
  const int64_t n_tiles = (n_nodes + kR - 1) / kR;
  const int64_t G = gridDim.x;
  auto node_of = [&](int64_t tile, int i) __attribute__((always_inline)) {
    const int64_t node = tile * kR + 4 * wave + 2 * i + half;
    return node < n_nodes ? node : n_nodes - 1;
  };
  auto load_ids = [&](int64_t tile, int32_t (&out)[2]) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 2; ++i) out[i] = IDS ? ids[node_of(tile, i)] : 0;
  };
  int64_t xrow[2];
  uint32_t xmask[2];
  auto rows_of = [&](int64_t tile, const int32_t (&idv)[2], int64_t (&row)[2], uint32_t (&mask)[2])
      __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int64_t r = IDS ? static_cast<int64_t>(idv[i]) : node_of(tile, i);
      const bool ok = static_cast<uint64_t>(r) < static_cast<uint64_t>(n_rows_slot);
      row[i] = ok ? r : 0;
      mask[i] = ok ? 0xffffffffu : 0u;
    }
  };
  u32x4 xr[2];
  auto load_x = [&](int s) __attribute__((always_inline)) {     // only issues the loads
    const unsigned char* base = slots.p[s];
#pragma unroll
    for (int i = 0; i < 2; ++i) xr[i] = *reinterpret_cast<const u32x4*>(base + xrow[i] * row_bytes + 16 * c);
  };
  auto stage_x = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      u32x4 v = xr[i];
      v.x &= xmask[i];
      v.y &= xmask[i];
      v.z &= xmask[i];
      v.w &= xmask[i];
      *reinterpret_cast<u32x4*>(Xs[buf] + (4 * wave + 2 * i + half) * kXRowB + 16 * c) = v;
    }
  };
  // k chunks [k0, k1) of the input part of the tile staged in X: the low weight piece, then the
  // high one, per chunk
  auto x_part = [&](const unsigned char* X, int k0, int k1, f32x16& a) __attribute__((always_inline)) {
#pragma unroll
    for (int kc = k0; kc < k1; ++kc) {
      const bf16x8 x = *reinterpret_cast<const bf16x8*>(X + c * kXRowB + 32 * kc + 16 * half);
      a = __builtin_amdgcn_mfma_f32_32x32x16_bf16(awx[kc][1], x, a, 0, 0, 0);
      a = __builtin_amdgcn_mfma_f32_32x32x16_bf16(awx[kc][0], x, a, 0, 0, 0);
    }
  };

  // The steps of this workgroup form one sequence (tile, s): s = 0 .. tau - 1 of tiles
  // blockIdx.x, blockIdx.x + G, ... . (lt, ls): the step whose rows were requested last.
  // Step k's rows are requested two steps before it runs, staged one step before, and its
  // input part is multiplied out during step k - 1, between the transcendentals of that
  // step's cell update (it does not depend on h_{k-1}); step k itself then starts from those
  // sums, adds the recurrent part and updates the cell.
  int32_t id_next[2];             // ids of tile lt + G
  int64_t lt = blockIdx.x;
  int ls = 0;
  {
    int32_t id0[2];
    load_ids(lt, id0);
    rows_of(lt, id0, xrow, xmask);
    load_x(0);
    load_ids(lt + G, id_next);
    stage_x(0);
  }
  auto request_next = [&]() __attribute__((always_inline)) {
    // selects on scalar conditions and loads that are issued either way (past the last tile
    // they re-read rows that exist): a branch here would meet in copies of registers whose
    // loads are in flight, i.e. in a wait
    const bool same_tile = ls + 1 < tau;
    int64_t nrow[2];
    uint32_t nmask[2];
    rows_of(lt + G, id_next, nrow, nmask);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      xrow[i] = same_tile ? xrow[i] : nrow[i];
      xmask[i] = same_tile ? xmask[i] : nmask[i];
    }
    lt = same_tile ? lt : lt + G;
    ls = same_tile ? ls + 1 : 0;
    load_x(ls);
    load_ids(lt + G, id_next);   // (re-read while the tile stays the same)
  };
  request_next();                 // rows of the second step
  __syncthreads();                // the first step's tile and the biases are in LDS
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  x_part(Xs[0], 0, kKX, acc);
  f32x4 cstate = {0.f, 0.f, 0.f, 0.f};
  int par = 0;                    // Xs[par]: the tile of the current step (already multiplied out)
  for (int64_t tile = blockIdx.x; tile < n_tiles; tile += G) {
    const int64_t node0 = tile * kR;
    for (int s = 0; s < tau; ++s) {
      stage_x(par ^ 1);           // the next step's rows have had a whole step to arrive
      request_next();             // the rows of the step after it
      __syncthreads();            // the next step's tile and h_{s-1} of every unit are in LDS
      const unsigned char* Xn = Xs[par ^ 1];
      const unsigned char* Hr = Hs[(s + 1) & 1];
      unsigned char* Hw = Hs[s & 1];
      // ---- recurrent part (h_0 = 0: nothing to add at s = 0)
      if (s > 0) {
#pragma unroll
        for (int kc = 0; kc < kKH; ++kc) {
          bf16x8 h[NP];
#pragma unroll
          for (int p = 0; p < NP; ++p)
            h[p] = *reinterpret_cast<const bf16x8*>(Hr + p * kHPieceB + c * kHRowB + 32 * kc + 16 * half);
          // (h piece, W piece): (2,0) (1,1) (1,0) (0,1) (0,0)
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(awh[kc][0], h[2], acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(awh[kc][1], h[1], acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(awh[kc][0], h[1], acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(awh[kc][1], h[0], acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(awh[kc][0], h[0], acc, 0, 0, 0);
        }
      }
      // ---- cell update, register-local (gates i, f, g, o of units unit0 + j sit in acc[4 g + j]),
      // a unit at a time between the quarters of the next step's input part
      f32x16 accn;
#pragma unroll
      for (int r = 0; r < 16; ++r) accn[r] = 0.f;
      const f32x4 bi4 = *reinterpret_cast<const f32x4*>(&Bs[unit0]);
      const f32x4 bf4 = *reinterpret_cast<const f32x4*>(&Bs[kDS + unit0]);
      const f32x4 bg4 = *reinterpret_cast<const f32x4*>(&Bs[2 * kDS + unit0]);
      const f32x4 bo4 = *reinterpret_cast<const f32x4*>(&Bs[3 * kDS + unit0]);
      const float bi[4] = {bi4.x, bi4.y, bi4.z, bi4.w};
      const float bf[4] = {bf4.x, bf4.y, bf4.z, bf4.w};
      const float bg[4] = {bg4.x, bg4.y, bg4.z, bg4.w};
      const float bo[4] = {bo4.x, bo4.y, bo4.z, bo4.w};
      float cs[4] = {cstate.x, cstate.y, cstate.z, cstate.w};
      float hv[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        x_part(Xn, (kKX / 4) * j, (kKX / 4) * (j + 1), accn);
        const float gi = sigmoidf_(acc[j] + bi[j]);
        const float gg = tanhf_(acc[8 + j] + bg[j]);
        const float go = sigmoidf_(acc[12 + j] + bo[j]);
        if (s == 0) {
          cs[j] = gi * gg;
        } else {
          const float gf = sigmoidf_(acc[4 + j] + bf[j]);
          cs[j] = __builtin_fmaf(gf, cs[j], gi * gg);
        }
        hv[j] = go * tanhf_(cs[j]);
      }
      cstate = f32x4{cs[0], cs[1], cs[2], cs[3]};
      if (s + 1 < tau) {        // h for the next step's product: three bf16 pieces, node-major
        uint32_t lo[NP], hi[NP];
        split2<NP>(hv[0], hv[1], lo);
        split2<NP>(hv[2], hv[3], hi);
#pragma unroll
        for (int p = 0; p < NP; ++p)
          *reinterpret_cast<u32x2*>(Hw + p * kHPieceB + c * kHRowB + 2 * unit0) = u32x2{lo[p], hi[p]};
      } else {
        const int64_t node = node0 + c;
        if (node < n_nodes) *reinterpret_cast<f32x4*>(S + node * kDS + unit0) = f32x4{hv[0], hv[1], hv[2], hv[3]};
      }
      acc = accn;
      par ^= 1;
    }
  }
}

}  // namespace

namespace sat {

// Whether launch_lstm_fused16 serves the shape: bf16 rows of 256 elements, d_s = 64.
bool lstm_fused16_serves(int32_t d, int32_t d_s, int es_x, int64_t n_nodes) {
  return d == kD && d_s == kDS && es_x == 2 && n_nodes >= 32768;
}

// S [n_nodes, 64] = last hidden state of the LSTM over the tau slots (device, bf16 rows of 256
// elements, ld_slot elements apart, 16-byte aligned; row of node k: ids ? ids[k] : k, rows
// outside [0, n_rows_slot) count as zeros). WxP / WhP: the split-weight arrays lstm_mx.hip
// makes of Wx ([3][256][256] bf16) and Wh ([3][256][64]); bias [256] fp32, 16-byte aligned.
sat_status launch_lstm_fused16(const void* const* slot_ptrs, int tau, int64_t n_rows_slot, int64_t ld_slot,
                               const int32_t* ids, int64_t n_nodes, const void* WxP, const void* WhP,
                               const float* bias, float* S, hipStream_t st) {
  if (n_nodes == 0) return SAT_OK;
  if (tau < 1 || tau > kMaxTau || n_rows_slot <= 0) return SAT_EUNSUPPORTED;
  Slots16 sp;
  for (int s = 0; s < kMaxTau; ++s) sp.p[s] = s < tau ? static_cast<const unsigned char*>(slot_ptrs[s]) : nullptr;
  // one workgroup per compute unit (its registers fill two wavefronts per SIMD), each walking
  // its share of the 32-node tiles
  const int64_t tiles = (n_nodes + kR - 1) / kR;
  const int64_t blocks = tiles < 256 ? tiles : 256;
  const dim3 grid(static_cast<unsigned>(blocks)), block(512);
  const uint16_t* wx = static_cast<const uint16_t*>(WxP);
  const uint16_t* wh = static_cast<const uint16_t*>(WhP);
  if (ids)
    lstm_fused16_kernel<true><<<grid, block, 0, st>>>(sp, tau, n_rows_slot, ld_slot * 2, ids, n_nodes, wx, wh, bias, S);
  else
    lstm_fused16_kernel<false><<<grid, block, 0, st>>>(sp, tau, n_rows_slot, ld_slot * 2, ids, n_nodes, wx, wh, bias,
                                                       S);
  return sat::check_launch();
}

}  // namespace sat

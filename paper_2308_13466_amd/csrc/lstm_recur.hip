// The time steps of the predictor's LSTM (Sec. "Embedding Predictor") when EVERY slot's input
// projection x_s Wx^T is at hand (kept from earlier windows, the newest made by
// lstm_proj.hip): per node only 4 d_s numbers per step are read, the recurrent product
// h_{s-1} Wh^T (K = d_s = 64) and the cell update remain. d_s = 64.
//
// The products are formed TRANSPOSED, gates^T = Wh h^T: the weights are the MFMA's row
// operand and stay in registers for the life of the workgroup (wavefront w owns hidden units
// 8 w .. 8 w + 7, its 32 rows being row 8 g + u = gate g of unit 8 w + u: 48 registers), the
// nodes are the columns. In the accumulator of such a product a lane holds, for ONE node,
// rows 8 (r / 4) + 4 (lane / 32) + r % 4, i.e. all four gates of four units: the cell update is
// register-local, h leaves as 8-byte LDS writes per piece and S as 16-byte stores. No weight
// tile is staged. The kept gates come in through LDS: read from memory in a lane's own
// layout they would be 16-byte slivers of 64 different cache lines per load instruction (a
// wavefront owns 8 of a row's 64 units per gate), which keeps the address and first-level
// cache units busy 90 % of the time; instead wavefront w reads the whole rows of nodes
// 8 w .. 8 w + 7 (one 1 KiB row per instruction, eight lines fully used), a step ahead into
// registers, and writes them to a row-major tile in LDS at the end of the step; every
// wavefront then starts its accumulators from its slivers of that tile (16-byte LDS reads,
// rows padded by 16 bytes so that 16 lanes cover all banks). A workgroup walks many tiles of
// 64 nodes; the rows of the next (tile, step) are in flight while the products and the
// transcendentals of the current one run.
//
// Bit-compatibility with lstm_mx_kernel: the accumulator starts from the kept projection and
// takes the same products in the same order (k chunks ascending; (h1 W3) (h3 W1) (h2 W2)
// (h1 W2) (h2 W1) (h1 W1) inside a chunk; which operand is the row operand does not change an
// element's sum), then the same bias addition and the same activation code.
#include "mx_tile.h"
#include "sat_internal.h"

namespace {

using namespace sat::mx;

constexpr int kDS = 64, kNB = 4 * kDS, kR = 64, kBlocks = kR / 32, kMaxTau = 8;
constexpr int kHRowB = kDS * 2 + 16;           // bytes per node row of a staged h piece (padded)
constexpr int kHPieceB = kR * kHRowB;
constexpr int kGRowB = kNB * 4 + 16;           // bytes per node row of the staged gates (padded)
constexpr int kRowsPerWave = kR / 8;           // rows of the gate tile a wavefront brings in

struct RecurProj {
  const float* p[kMaxTau];
};

__device__ __forceinline__ float sigmoidf_(float x) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x));
}
__device__ __forceinline__ float tanhf_(float x) {
  return 2.0f * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-2.8853900817779268f * x)) - 1.0f;
}

__global__ __launch_bounds__(512, 2) void lstm_recur_kernel(RecurProj proj, int tau, int64_t n_nodes,
                                                           const uint16_t* __restrict__ WhP,
                                                           const float* __restrict__ bias,
                                                           float* __restrict__ S) {
  constexpr int NP = 3;
  // h_s goes to Hs[s % 2]: the products of step s (reading h_{s-1}) and its cell update
  // (writing h_s) then need no barrier between them and can be interleaved
  __shared__ __attribute__((aligned(16))) unsigned char Hs[2][NP * kHPieceB];
  __shared__ __attribute__((aligned(16))) unsigned char Gs[kR * kGRowB];
  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int half = lane >> 5, c = lane & 31;

  // weights: row m = lane % 32 of this wavefront is gate m / 8 of unit 8 wave + m % 8, i.e.
  // gate column n = (m / 8) * 64 + 8 wave + m % 8 of the split-weight array [3][256][64]
  bf16x8 aw[kDS / 16][NP];
  {
    const int n = (c >> 3) * kDS + 8 * wave + (c & 7);
#pragma unroll
    for (int kc = 0; kc < kDS / 16; ++kc)
#pragma unroll
      for (int p = 0; p < NP; ++p)
        aw[kc][p] = *reinterpret_cast<const bf16x8*>(WhP + (static_cast<int64_t>(p) * kNB + n) * kDS + 16 * kc +
                                                     8 * half);
  }
  // this lane's units: 8 wave + 4 half + 0..3 (of one node per 32-node block)
  const int unit0 = 8 * wave + 4 * half;
  f32x4 b_gate[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) b_gate[g] = *reinterpret_cast<const f32x4*>(bias + g * kDS + unit0);

  // Rows of the kept gate pre-activations of step s, nodes node0 + 8 wave + 0..7: lane L takes
  // bytes 16 L .. 16 L + 15 of a row. At the first step the forget gate's block (lanes 16..31)
  // is never looked at: those lanes read the input gate's block again (same lines). Only
  // issues the loads.
  f32x4 rows[kRowsPerWave];
  auto load_rows = [&](int64_t node0, int s) __attribute__((always_inline)) {
    const float* P = proj.p[s];
    const int col = (s == 0 && (lane >> 4) == 1) ? 4 * (lane - 16) : 4 * lane;
#pragma unroll
    for (int i = 0; i < kRowsPerWave; ++i) {
      int64_t node = node0 + kRowsPerWave * wave + i;
      node = node < n_nodes ? node : n_nodes - 1;       // (rows past the end: not stored)
      rows[i] = *reinterpret_cast<const f32x4*>(P + node * kNB + col);
    }
  };
  auto stage_rows = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < kRowsPerWave; ++i)
      *reinterpret_cast<f32x4*>(Gs + (kRowsPerWave * wave + i) * kGRowB + 16 * lane) = rows[i];
  };

  // A workgroup walks tiles blockIdx.x, blockIdx.x + gridDim.x, ...
  const int64_t n_tiles = (n_nodes + kR - 1) / kR;
  f32x4 cstate[kBlocks], hval[kBlocks];
  f32x16 acc[kBlocks];
  if (static_cast<int64_t>(blockIdx.x) < n_tiles) {
    load_rows(static_cast<int64_t>(blockIdx.x) * kR, 0);
    stage_rows();
  }
  for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
    const int64_t node0 = tile * kR;
    for (int s = 0; s < tau; ++s) {
      // the rows of the next (tile, step), a whole step ahead. One call with scalar operands, also
      // after the last tile's last step (where it re-reads the table's last row: clamped inside):
      // two calls behind a branch meet in copies of the loaded registers, i.e. in a wait.
      const bool same_tile = s + 1 < tau;
      load_rows(same_tile ? node0 : (tile + gridDim.x) * kR, same_tile ? s + 1 : 0);
      __syncthreads();          // the gate tile of this step and h_{s-1} of every unit are in LDS
      const unsigned char* Hr = Hs[(s + 1) & 1];
      unsigned char* Hw = Hs[s & 1];
      // this lane's slivers: acc[b][4 g + j] = gates[32 b + c][64 g + unit0 + j]
#pragma unroll
      for (int b = 0; b < kBlocks; ++b) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          if (g == 1 && s == 0) continue;                 // c_0 = 0: the forget gate is not looked at
          const f32x4 v = *reinterpret_cast<const f32x4*>(Gs + (32 * b + c) * kGRowB + 4 * (g * kDS + unit0));
          acc[b][4 * g + 0] = v.x;
          acc[b][4 * g + 1] = v.y;
          acc[b][4 * g + 2] = v.z;
          acc[b][4 * g + 3] = v.w;
        }
      }
      __syncthreads();          // every wavefront has taken its slivers: the tile may be overwritten
      if (s > 0) {
        // (block by block: the cell update of a block's nodes can then issue between the products
        // of the next block, which do not depend on it)
#pragma unroll
        for (int b = 0; b < kBlocks; ++b) {
#pragma unroll
          for (int kc = 0; kc < kDS / 16; ++kc) {
            bf16x8 h[NP];
#pragma unroll
            for (int p = 0; p < NP; ++p)
              h[p] = *reinterpret_cast<const bf16x8*>(Hr + p * kHPieceB + (32 * b + c) * kHRowB + 32 * kc +
                                                      16 * half);
            // (h piece, W piece): (0,2) (2,0) (1,1) (0,1) (1,0) (0,0)
#pragma unroll
            for (int q = 0; q < n_products<NP>(); ++q)
              acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aw[kc][product_b<NP>(q)], h[product_a<NP>(q)],
                                                               acc[b], 0, 0, 0);
          }
        }
      }
      // cell update, register-local: gates i, f, g, o of units unit0 + j sit in acc[b][4 g + j]
#pragma unroll
      for (int b = 0; b < kBlocks; ++b) {
        float cs[4] = {cstate[b].x, cstate[b].y, cstate[b].z, cstate[b].w};
        if (s == 0) cs[0] = cs[1] = cs[2] = cs[3] = 0.f;
        float hv[4];
        const float bi[4] = {b_gate[0].x, b_gate[0].y, b_gate[0].z, b_gate[0].w};
        const float bf[4] = {b_gate[1].x, b_gate[1].y, b_gate[1].z, b_gate[1].w};
        const float bg[4] = {b_gate[2].x, b_gate[2].y, b_gate[2].z, b_gate[2].w};
        const float bo[4] = {b_gate[3].x, b_gate[3].y, b_gate[3].z, b_gate[3].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float gi = sigmoidf_(acc[b][j] + bi[j]);
          const float gg = tanhf_(acc[b][8 + j] + bg[j]);
          const float go = sigmoidf_(acc[b][12 + j] + bo[j]);
          if (s == 0) {
            cs[j] = gi * gg;
          } else {
            const float gf = sigmoidf_(acc[b][4 + j] + bf[j]);
            cs[j] = __builtin_fmaf(gf, cs[j], gi * gg);
          }
          hv[j] = go * tanhf_(cs[j]);
        }
        cstate[b] = f32x4{cs[0], cs[1], cs[2], cs[3]};
        hval[b] = f32x4{hv[0], hv[1], hv[2], hv[3]};
        if (s + 1 < tau) {        // h for the next step's product: three bf16 pieces, node-major
          uint32_t lo[NP], hi[NP];
          split2<NP>(hv[0], hv[1], lo);
          split2<NP>(hv[2], hv[3], hi);
#pragma unroll
          for (int p = 0; p < NP; ++p)
            *reinterpret_cast<u32x2*>(Hw + p * kHPieceB + (32 * b + c) * kHRowB + 2 * unit0) = u32x2{lo[p], hi[p]};
        } else {
          const int64_t node = node0 + 32 * b + c;
          if (node < n_nodes) *reinterpret_cast<f32x4*>(S + node * kDS + unit0) = hval[b];
        }
      }
      // the next (tile, step)'s rows have had the whole step to arrive
      stage_rows();
    }
  }
}

}  // namespace

namespace sat {

// S [n_nodes, 64] = last hidden state of the LSTM whose per-step input parts are the kept
// projections proj[0 .. tau) (device, [n_nodes, 256] fp32 each, 16-byte aligned; the forget
// gate's block of proj[0] is never read). WhP: the split-weight array lstm_mx.hip makes of Wh
// ([3][256][64] bf16); bias [256] fp32, 16-byte aligned.
sat_status launch_lstm_recur(float* const* proj, int tau, int64_t n_nodes, const void* WhP, const float* bias,
                             float* S, hipStream_t st) {
  if (n_nodes == 0) return SAT_OK;
  if (tau < 1 || tau > kMaxTau) return SAT_EUNSUPPORTED;
  RecurProj pp;
  for (int s = 0; s < kMaxTau; ++s) pp.p[s] = s < tau ? proj[s] : nullptr;
  // one workgroup per compute unit (its registers fill two wavefronts per SIMD), each walking
  // its share of the 64-node tiles
  const int64_t tiles = (n_nodes + kR - 1) / kR;
  const int64_t blocks = tiles < 256 ? tiles : 256;
  lstm_recur_kernel<<<dim3(static_cast<unsigned>(blocks)), dim3(512), 0, st>>>(
      pp, tau, n_nodes, static_cast<const uint16_t*>(WhP), bias, S);
  return sat::check_launch();
}

}  // namespace sat

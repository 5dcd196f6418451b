// Input projection of the predictor's LSTM for ONE ring slot (Sec. "Embedding Predictor",
// the W_x x_s term of the gates), as a kernel of its own:
//   P[m, 0:256) = x[row(m), 0:256) Wx^T,   row(m) = ids ? ids[m] : m,   m < n_nodes
// for d = 256 and d_s = 64 (256 gate columns), fp32 rows. Consecutive windows share all but
// their newest slot, and a slot's projection does not depend on its place in the window, so
// in the steady state this product is the only part of the LSTM that touches the embeddings;
// the time steps themselves then run from the kept projections alone.
//
// Bit-compatibility with lstm_mx_kernel is the point of the arithmetic below: for every
// (node, gate column) the same bf16 pieces (mx_tile.h's split of x, the split-weight array
// of lstm_mx.hip) enter the same instruction in the same order - k chunks of 16 ascending,
// inside a chunk the products (a1 b3) (a3 b1) (a2 b2) (a1 b2) (a2 b1) (a1 b1) - starting from
// a zero accumulator, so the sums are the same fp32 numbers.
//
// Layout of the work (the weights held still, as in dense_ws32.hip): a workgroup has 8
// wavefronts, wavefront w owns gate columns [32 w, 32 w + 32) and keeps its slice of the
// split weights for all of K in registers (192). Rows stream through in tiles of 32: a load
// instruction fetches ONE row (64 lanes x 16 bytes = the row's 1 KiB; its table row is a
// scalar, read through lanes 0..3 one tile ahead), the row is split and written to LDS
// (the eight 32-k staging tiles of a row tile lie 64 bytes off a multiple of 256 apart, so
// the eight 64-byte pieces of one such write fall on all banks twice, which is what 512
// bytes cost anyway). Two LDS buffers, one barrier per tile; the rows of the next tile are
// staged, and those after them requested, between the products of this one.
#include "mx_tile.h"
#include "sat_internal.h"

namespace {

using namespace sat::mx;

constexpr int kK = 256, kN = 256, kKC = kK / 16, kNT32 = kK / 32;
constexpr int kTileStride = tile_bytes<32, 3>() + 64;      // bytes between staging tiles
constexpr int kStage = kNT32 * kTileStride;

// TAIL false: every tile of the launch is whole (rows [row_begin, n_nodes), a multiple of 32):
// the stores then sit in the tile loop's one basic block, and the waits for the next tile's
// rows, requested before them, need not wait for the stores as well. TAIL true: the launch is
// the one last, partial tile. IDS: rows come through the id list (a compile-time switch: a test
// of the pointer inside the tile loop would split it into several basic blocks, and with them
// the bookkeeping that lets a wait for a row's load leave the later stores in flight).
template <bool TAIL, bool IDS>
__global__ __launch_bounds__(512, 2) void lstm_proj_kernel(
    const float* __restrict__ X, int64_t n_rows_slot, int64_t ld_slot, const int32_t* __restrict__ ids,
    int64_t row_begin, int64_t n_nodes, const uint16_t* __restrict__ WxP, float* __restrict__ P,
    int tiles_per_block) {
  constexpr int NP = 3;
  __shared__ __attribute__((aligned(16))) unsigned char As[2 * kStage];

  const int t = threadIdx.x;
  const int lane0 = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int64_t row_lo = row_begin + static_cast<int64_t>(blockIdx.x) * 32 * tiles_per_block;

  // ---- this wavefront's slice of the split weights, already in MFMA operand order in
  // memory: piece p of column n is the 512 contiguous bytes at (p * 256 + n) * 256 elements
  bf16x8 bw[kKC][NP];
  {
    const int col = 32 * wave + (lane0 & 31);
#pragma unroll
    for (int kc = 0; kc < kKC; ++kc)
#pragma unroll
      for (int p = 0; p < NP; ++p)
        bw[kc][p] = *reinterpret_cast<const bf16x8*>(WxP + (static_cast<int64_t>(p) * kN + col) * kK + 16 * kc +
                                                     8 * (lane0 >> 5));
  }
  // (what follows derives its lane constants after the weights are in: see dense_ws32.hip)
  int lane = lane0;
  asm volatile("" : "+v"(lane));
  const int col = 32 * wave + (lane & 31);

  // Table rows of the wavefront's four rows (w, w + 8, w + 16, w + 24) of the tile at row0:
  // the index is the same for every lane, so these are scalar loads into scalar registers
  // (the vector registers are all taken). Nothing looks at the values here, so the four loads
  // go out together; a row past the end takes the last node's id (it is staged and, if the
  // tile is multiplied at all, its products are not stored).
  struct Ids {
    int32_t r[4];
  };
  auto load_ids = [&](int64_t row0) __attribute__((always_inline)) {
    Ids v;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t m = row0 + wave + 8 * i;
      const int64_t mc = m < n_nodes ? m : n_nodes - 1;
      v.r[i] = IDS ? ids[mc] : static_cast<int32_t>(mc);
    }
    return v;
  };
  // an id outside the table reads as a row of zeros
  auto in_table = [&](int32_t r) { return r >= 0 && r < n_rows_slot; };
  // the whole row per instruction, lane = 4 k
  const uint32_t off_x = static_cast<uint32_t>(lane) << 4;
  auto load_row = [&](const Ids& idv, int i) {
    const int32_t r = idv.r[i];
    const float* base = X + static_cast<int64_t>(in_table(r) ? r : 0) * ld_slot;
    return *reinterpret_cast<const f32x4*>(reinterpret_cast<const unsigned char*>(base) + off_x);
  };
  // lane part of the staged address: staging tile lane / 8, chunk (lane % 8) / 2, half lane % 2
  const uint32_t off_s = static_cast<uint32_t>((lane >> 3) * kTileStride + (((lane & 7) >> 1) << 4) +
                                               ((lane & 1) << 3));
  auto store_row = [&](f32x4 f, const Ids& idv, int i, int stage) {
    if (!in_table(idv.r[i])) f = f32x4{0.f, 0.f, 0.f, 0.f};    // uniform
    uint32_t lo[NP], hi[NP];
    split2<NP>(f.x, f.y, lo);
    split2<NP>(f.z, f.w, hi);
    const int row = wave + 8 * i;                              // uniform
    const int fsw = (((row >> 1) ^ (row >> 3)) & 1) | (((row >> 2) & 1) << 1);   // swz()'s chunk flip
    unsigned char* s = As + stage * kStage + row * ROW_B + (off_s ^ static_cast<uint32_t>(fsw << 4));
#pragma unroll
    for (int p = 0; p < NP; ++p) *reinterpret_cast<u32x2*>(s + p * piece_bytes<32>()) = u32x2{lo[p], hi[p]};
  };

  // ids: of the tile being staged (id_a) and of the one after (id_b)
  Ids id_a = load_ids(row_lo);
  Ids id_b = load_ids(row_lo + 32);
  f32x4 ra[2];
  ra[0] = load_row(id_a, 0);
  ra[1] = load_row(id_a, 1);
  // Slot j (0..3) of tile `it`: row j of tile it + 1 leaves its registers for the buffer that
  // tile is read from, and the registers take the row two further on (tile it + 1 or it + 2).
  // id_a: ids of tile it + 1, id_b: of tile it + 2.
  auto slot = [&](int it, int j) {
    store_row(ra[j & 1], id_a, j, (it + 1) & 1);
    ra[j & 1] = j < 2 ? load_row(id_a, j + 2) : load_row(id_b, j - 2);
    __builtin_amdgcn_sched_barrier(0);     // the request stays here (see dense_ws32.hip)
  };
#pragma unroll
  for (int j = 0; j < 4; ++j) slot(-1, j);
  id_a = id_b;
  id_b = load_ids(row_lo + 64);
  __syncthreads();

  auto tile = [&](int it) __attribute__((always_inline)) {
    const int64_t row0 = row_lo + 32 * it;
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    const unsigned char* S = As + (it & 1) * kStage;
    auto frag = [&](int kc, int p) {
      return read_operand(S + (kc >> 1) * kTileStride + p * piece_bytes<32>(), 0, kc & 1, lane);
    };
    bf16x8 a0 = frag(0, 0), a1 = frag(0, 1), a2 = frag(0, 2);
#pragma unroll
    for (int kc = 0; kc < kKC; ++kc) {
      // product order of mx_tile.h; a piece is read for the next chunk once its last product of
      // this one has been issued (the first piece, needed first again, one product early into
      // registers of its own)
      bf16x8 a0n = a0;
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, bw[kc][2], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, bw[kc][0], acc, 0, 0, 0);
      if (kc + 1 < kKC) a2 = frag(kc + 1, 2);
      __builtin_amdgcn_sched_barrier(0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, bw[kc][1], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, bw[kc][1], acc, 0, 0, 0);
      if (kc + 1 < kKC) a0n = frag(kc + 1, 0);
      __builtin_amdgcn_sched_barrier(0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, bw[kc][0], acc, 0, 0, 0);
      if (kc + 1 < kKC) a1 = frag(kc + 1, 1);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, bw[kc][0], acc, 0, 0, 0);
      a0 = a0n;
      __builtin_amdgcn_sched_barrier(0);
      // (slots in the middle of each half of the tile, not at its start: should a wait for a
      // row's load ever include the previous tile's stores, they have completed by then)
      if ((kc & 7) == 4 || (kc & 7) == 5) slot(it, 2 * (kc >> 3) + (kc & 7) - 4);
      if (kc == 14) {
        // the ids move up once the last slot has used them, and the next ones are requested
        id_a = id_b;
        id_b = load_ids(row0 + 96);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // register r of a lane is row 8 (r / 4) + 4 (lane / 32) + r % 4, column lane % 32
    {
      const uint32_t off_y = (static_cast<uint32_t>(4 * (lane >> 5)) * kN + static_cast<uint32_t>(col)) << 2;
      const int64_t left = n_nodes - row0 - 4 * (lane >> 5);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int dr = 8 * (r >> 2) + (r & 3);
        float* yr = P + (row0 + dr) * kN;
        if (!TAIL || dr < left) *reinterpret_cast<float*>(reinterpret_cast<unsigned char*>(yr) + off_y) = acc[r];
      }
    }
    __syncthreads();
  };
  // One basic block per tile and the test at the bottom: with a test at the top that jumps to
  // the latch, the bookkeeping of what is in flight is merged over that path too and the counted
  // waits (a row's load may leave the 16 later stores in flight) shrink to a wait for nearly
  // everything. (Every workgroup of a launch has a first tile: the grid is sized from the
  // tile count; n_nodes - row_lo is a multiple of 32 here or the launch is the one tail tile.)
  const int64_t left_tiles = (n_nodes - row_lo + 31) / 32;
  const int my_tiles = left_tiles < tiles_per_block ? static_cast<int>(left_tiles) : tiles_per_block;
  // The first tile stands outside the loop for the same reason: the loop is then entered with
  // the same loads and stores in flight as it is re-entered with.
  tile(0);
  if (my_tiles > 1) {
    int it = 1;
    do {
      tile(it);
      ++it;
    } while (it < my_tiles);
  }
}

}  // namespace

namespace sat {

// Whether launch_lstm_proj serves the shape.
bool lstm_proj_serves(int32_t d, int32_t d_s, int es_x, int64_t n_nodes) {
  return d == kK && 4 * d_s == kN && es_x == 4 && n_nodes >= 32768;
}

// P [n_nodes, 256] fp32 = x rows (through ids, fp32, ld_slot elements apart) times Wx^T, with
// WxP the split-weight array lstm_mx.hip makes of Wx ([3][256][256] bf16). lstm_proj_serves()
// must hold; rows 16-byte aligned.
sat_status launch_lstm_proj(const void* X, int64_t n_rows_slot, int64_t ld_slot, const int32_t* ids,
                            int64_t n_nodes, const void* WxP, float* P, hipStream_t st) {
  if (n_nodes == 0) return SAT_OK;
  const float* x = static_cast<const float*>(X);
  const uint16_t* w = static_cast<const uint16_t*>(WxP);
  const int64_t n_full = n_nodes & ~static_cast<int64_t>(31);
  if (n_full > 0) {
    // one workgroup per compute unit, each with an equal share of the whole tiles
    const int64_t tiles = n_full / 32;
    const int64_t tpb = (tiles + 255) / 256;
    if (tpb > (1 << 20)) return SAT_EUNSUPPORTED;
    const int64_t gx = (tiles + tpb - 1) / tpb;
    const dim3 grid(static_cast<unsigned>(gx));
    if (ids)
      lstm_proj_kernel<false, true><<<grid, dim3(512), 0, st>>>(x, n_rows_slot, ld_slot, ids, 0, n_full, w, P,
                                                              static_cast<int>(tpb));
    else
      lstm_proj_kernel<false, false><<<grid, dim3(512), 0, st>>>(x, n_rows_slot, ld_slot, ids, 0, n_full, w, P,
                                                               static_cast<int>(tpb));
  }
  if (n_full < n_nodes) {
    if (ids)
      lstm_proj_kernel<true, true><<<dim3(1), dim3(512), 0, st>>>(x, n_rows_slot, ld_slot, ids, n_full, n_nodes,
                                                                 w, P, 1);
    else
      lstm_proj_kernel<true, false><<<dim3(1), dim3(512), 0, st>>>(x, n_rows_slot, ld_slot, ids, n_full, n_nodes,
                                                                  w, P, 1);
  }
  return sat::check_launch();
}

}  // namespace sat

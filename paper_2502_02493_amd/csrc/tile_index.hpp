// Index arithmetic of the weight stream, shared by the gfx950 kernels (device) and by the host-side walk
// that checks it (easyspec_weight_walk): which k-tiles a wave takes, where a row tile and a lane's piece of
// a fragment lie in a packed matrix, which unit a workgroup's slot takes.  Plain integer functions, no
// device intrinsics; the kernels call exactly these, so what the walk checks is what the kernels compute.
#pragma once
#include <stddef.h>

#if defined(__HIPCC__) || defined(__CUDACC__)
#define ES_HD __host__ __device__ __forceinline__
#else
#define ES_HD inline
#endif

namespace es {

constexpr int kBatchTiles = 8;  // weight fragments (1 KB each at 16 rows) a wave keeps in flight

// k-tiles per batch when a wave streams RT row tiles side by side
ES_HD constexpr int batch_len(int RT) { return kBatchTiles / RT; }
// The waves of a workgroup split K interleaved: wave w takes k-tiles w, w + NW, w + 2 NW, ...; load u of the
// batch that starts at k-tile kt is k-tile kt + u * NW.
ES_HD constexpr int batch_tile(int kt, int u, int NW) { return kt + u * NW; }
// a batch is full when its last load is still inside the matrix; the first k-tile of the next batch
ES_HD constexpr bool batch_is_full(int kt, int U, int NW, int nkt) { return batch_tile(kt, U - 1, NW) < nkt; }
ES_HD constexpr int next_batch(int kt, int U, int NW) { return kt + U * NW; }

// u32x4 (16-byte pieces) of one row tile of a packed matrix: nkt fragments of [4 k-groups][R rows]
ES_HD constexpr size_t row_tile_pieces(int nkt, int R) { return (size_t)nkt * (4 * R); }
// pieces per fragment: the stride between the fragments of consecutive k-tiles
ES_HD constexpr int fragment_pieces(int R) { return 4 * R; }
// A lane's piece inside a fragment of R <= 16 rows: k-group (lane / 16) times R plus its row; the lanes of
// the rows a low tile does not have re-read its last row (their results are dropped).
ES_HD constexpr int lane_piece(int lane, int R) {
  const int row = lane & 15;
  return (lane >> 4) * R + (row < R ? row : R - 1);
}
// Slot p of a workgroup whose first unit (row tile, tile of rotation pairs) is u0: a missing last unit
// re-reads the last existing one (its results are dropped).
ES_HD constexpr int clamped_unit(int u0, int p, int units) { return u0 + p < units ? u0 + p : units - 1; }
ES_HD constexpr int ceil_div(int a, int b) { return (a + b - 1) / b; }

// ------------------------------------------------------------------------------------------
// Layout of an activation operand x[col][k] (col < 16, k < K) of a weight contraction, per part
// (hi, lo), in elements; EPL = elements per 16-byte fragment, KT = EPL * 4 = elements per k-tile.
// It depends on the number of columns of the forward pass, which producer and consumer both know:
//   up to kPlainCols columns: plain rows, x[col][k] at col * K + k.  A wave's B fragments of one
//     k-tile are then one 64-byte run per column: the fewest cache lines for one or two columns.
//   more columns: tiles of KT consecutive k, inside a tile [k-group (4)][column (pitch)][EPL
//     elements] — the order in which the lanes of a wave take their 16-byte fragments (lane =
//     k-group * 16 + column) — so that the fragment loads of one k-tile and part are contiguous
//     runs instead of one cache line per column (measured: 6-column calibration 7 % faster, 8-wide
//     tree level 12 %; with one column the tiles would touch four times the lines of plain rows).
//     The pitch follows the column count (xpitch): what these loads cost is the number of 128-byte
//     lines a wave asks the L2 for, and a 4-column pass with a pitch of 16 touches four half-used
//     lines per k-tile and part where a pitch of 4 touches two.
// ------------------------------------------------------------------------------------------
constexpr int kPlainCols = 2;
constexpr int kOperandCols = 16;  // columns an operand slot has room for (= kMaxCols)

// 16-byte fragments per k-group of a tile: the column count rounded up to an even number (tiles
// are then whole 128-byte lines), except that 7, 8, 15 and 16 columns keep 16, where packing
// saves no line and costs the spread over 256-byte blocks
ES_HD constexpr int xpitch(int ncols) {
  const int even = (ncols + 1) & ~1;
  return (even & 7) == 0 ? kOperandCols : even;
}
ES_HD constexpr size_t xoff_elems(int EPL, int ncols, int K, int col, int k) {
  const int KT = 4 * EPL;
  if (ncols <= kPlainCols) return (size_t)col * K + k;
  const int pitch = xpitch(ncols);
  return (size_t)(k / KT) * (pitch * KT) + (size_t)((k % KT) / EPL) * (pitch * EPL) + col * EPL + (k % EPL);
}
// 16-byte fragments between the fragments of consecutive k-tiles
ES_HD constexpr int xtile_fragments(int ncols) { return ncols <= kPlainCols ? 4 : 4 * xpitch(ncols); }

// Element offset, inside an operand slot, of B fragment q (< NB) of `lane` for k-tile 0, or -1 if the lane
// loads nothing (its MFMA column is no live token column).  A slot holds PARTS parts (hi, lo) of kOperandCols * K
// elements.  NB = 1: the lane's MFMA column c reads the hi term of column c, or (two parts, "folded") column
// ncols + c the lo term of column c.  NB = 2: fragment 0 is the hi term, fragment 1 the lo term of column c.
ES_HD constexpr long x_fragment_elems(int EPL, int PARTS, int NB, int ncols, int K, int lane, int q) {
  const int col = lane & 15, kg = lane >> 4;
  const long part = (long)kOperandCols * K;
  if (NB == 1) {
    const bool is_lo = PARTS == 2 && col >= ncols;
    const int src = is_lo ? col - ncols : col;
    if (src >= ncols) return -1;
    return (is_lo ? part : 0) + (long)xoff_elems(EPL, ncols, K, src, kg * EPL);
  }
  if (col >= ncols) return -1;
  return (q ? part : 0) + (long)xoff_elems(EPL, ncols, K, col, kg * EPL);
}


// ------------------------------------------------------------------------------------------
// Vector attention with scores from the matrix cores (bf16 caches, 16 lanes per K row): how a batch of
// K rows passes through a wave's own LDS into MFMA A fragments, and where a slot's score comes out.
// A batch is `loads` loads of 4 slots (lane = sub * 16 + piece: slot 4 j + sub of the batch, 16-byte piece
// `piece` of its row); the stage holds up to 32 rows of 16 pieces.
// ------------------------------------------------------------------------------------------
constexpr int kStageRowPieces = 16;
// where load j of `lane` is stored: row = the slot's number in the batch, the pieces of a row XORed by its number
ES_HD constexpr int stage_store_piece(int lane, int j) {
  const int row = 4 * j + (lane >> 4);
  return row * kStageRowPieces + ((lane & 15) ^ (row & 15));
}
// Tile t of 16 slots: A row r = lane % 16 carries slot (r % 4) * 4 + r / 4 of the tile, k-group lane / 16 of
// k-tile kt its piece 4 kt + lane / 16: the stage index that lane reads for (t, kt)
ES_HD constexpr int stage_tile_slot(int lane) { return ((lane & 15) & 3) * 4 + ((lane & 15) >> 2); }
ES_HD constexpr int stage_fetch_piece(int lane, int t, int kt) {
  const int slot = stage_tile_slot(lane);
  return (t * 16 + slot) * kStageRowPieces + ((4 * kt + (lane >> 4)) ^ slot);
}
// The MFMA result of tile t holds, in element i of lane (lane / 16, any column), the score of A row 4 (lane / 16) + i,
// which by stage_tile_slot is slot 4 i + lane / 16 of the tile: the slot of the batch whose V row load 4 t + i brings to the lane.
ES_HD constexpr int score_slot_in_batch(int lane, int t, int i) { return t * 16 + 4 * i + (lane >> 4); }

}  // namespace es

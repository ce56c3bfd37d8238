// Tiling arithmetic shared, from one source, by the host (queries, validation) and the HIP kernel.
// A plan reaches the GPU as a table of flat boxes (at most two-dimensional pieces of a move); the tiles
// are never materialised: tile number b is located by a search in the boxes' tile prefix sums and its
// extent follows from the box's tiling parameters.
#pragma once

#include <cstdint>

#include "tpx.h"

#if defined(__HIPCC__)
#define TPX_HD __host__ __device__ inline
#else
#define TPX_HD inline
#endif

namespace tpx {

// Unit (i, j), 0 <= i < nrows, 0 <= j < run_units, of 1 << unit_log2 bytes goes from
// src_off + i*src_pitch + j*src_step to dst_off + i*dst_pitch + j*dst_step.  The box is cut into
// ceil(nrows / rows_per_tile) x chunks_per_row tiles of rows_per_tile rows by chunk_units units.
struct FlatBox {
  uint64_t src_off, dst_off;
  uint64_t src_pitch, dst_pitch;
  uint64_t src_step, dst_step;
  uint32_t run_units;
  uint32_t nrows;
  uint32_t rows_per_tile;
  uint32_t chunk_units;
  uint32_t chunks_per_row;
  uint32_t first_tile;  // number of tiles of all earlier boxes
  uint16_t src_rank, dst_rank;
  uint8_t kind;         // TPX_TILE_*
  uint8_t unit_log2;
  uint8_t n_dst;            // the tile is written to buffers dst_rank + k * dst_rank_stride, k < n_dst
  uint8_t dst_rank_stride;
  uint32_t seg_first;       // MERGE boxes: first entry in the segment table, segments per row,
  uint32_t n_seg;           // units per segment (0: the segments' widths differ, each has its own)
  uint32_t seg_units;
  uint32_t rows_first;      // tile order inside the box: 0 = along a row of tiles first, 1 = down a column of tiles first
};
static_assert(sizeof(FlatBox) == 96, "FlatBox layout");

constexpr uint32_t kCoarseShift = 6;  // one coarse entry per 64 tiles
constexpr uint32_t kMaxSegLds = 64;    // segments of a merge box whose table the kernel can stage in LDS

// Transposing tiles that the kernel moves in one shot (whole tile in flight, staged once through LDS) are
// kBlockBytes large.  For an element of eb bytes the planner cuts a transposing move into blocks of
// block_i(eb, nI) elements along the axis that is contiguous on the destination (nI its extent) by
// kBlockBytes / (block_i * eb) elements along the axis that is contiguous on the source: 1 KiB destination
// segments where the move is that long, never fewer than 64 elements.  0 = no one-shot shape for this element
// size (the general path is used).
constexpr uint32_t kBlockBytes = 65536;
TPX_HD uint32_t block_i(uint32_t eb, uint64_t nI) {
  if (eb != 2 && eb != 4 && eb != 8) return 0;
  uint32_t want = 1024 / eb;
  while (want > nI && want > 64) want >>= 1;
  return want;
}

TPX_HD uint32_t tiles_of(const FlatBox& b) {
  return ((b.nrows + b.rows_per_tile - 1) / b.rows_per_tile) * b.chunks_per_row;
}

// Index of the box that contains tile `tile`: the last box whose first_tile is <= tile.
// coarse[k] is that index for tile k << kCoarseShift, so the search is confined to a short range.
TPX_HD uint32_t find_box(const uint32_t* first_tile, const uint32_t* coarse, uint32_t n_boxes, uint32_t tile) {
  uint32_t lo = coarse[tile >> kCoarseShift];
  uint32_t hi = coarse[(tile >> kCoarseShift) + 1];  // box of a later tile: an upper bound
  if (hi >= n_boxes) hi = n_boxes - 1;
  while (lo < hi) {
    const uint32_t mid = (lo + hi + 1) >> 1;
    if (first_tile[mid] <= tile) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// The `local`-th tile of box b.
TPX_HD tpx_tile tile_of(const FlatBox& b, uint32_t local) {
  tpx_tile t{};
  uint32_t rb, c;
  if (b.rows_first) {  // consecutive tiles advance along the rows (the destination-contiguous axis of a transposing box)
    const uint32_t nrb = (b.nrows + b.rows_per_tile - 1) / b.rows_per_tile;
    c = local / nrb;
    rb = local - c * nrb;
  } else {
    rb = local / b.chunks_per_row;
    c = local - rb * b.chunks_per_row;
  }
  const uint32_t row0 = rb * b.rows_per_tile;
  const uint32_t col0 = c * b.chunk_units;
  t.nrows = b.nrows - row0 < b.rows_per_tile ? b.nrows - row0 : b.rows_per_tile;
  t.run_units = b.run_units - col0 < b.chunk_units ? b.run_units - col0 : b.chunk_units;
  t.src_off = b.src_off + uint64_t(row0) * b.src_pitch + uint64_t(col0) * b.src_step;
  t.dst_off = b.dst_off + uint64_t(row0) * b.dst_pitch + uint64_t(col0) * b.dst_step;
  t.src_pitch = b.src_pitch;
  t.dst_pitch = b.dst_pitch;
  t.src_step = b.src_step;
  t.dst_step = b.dst_step;
  t.src_rank = b.src_rank;
  t.dst_rank = b.dst_rank;
  t.kind = b.kind;
  t.unit_log2 = b.unit_log2;
  t.n_dst = b.n_dst;
  t.dst_rank_stride = b.dst_rank_stride;
  t.seg_first = b.seg_first;
  t.n_seg = b.n_seg;
  t.seg_units = b.seg_units;
  if (b.kind == TPX_TILE_MERGE) t.src_off = row0;  // sources are per segment; the tile only needs its first row
  return t;
}

}  // namespace tpx

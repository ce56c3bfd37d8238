// Dataset-state re-partitioning (paper sections 2.2 and 5.2).  The paper requires that after a change of
// the data-parallel degree every sample is still consumed exactly once per epoch, in the same order, with
// the global batch unchanged, and that each data partition has its own index.  Reading used here: with
// global order G, global batch B and D replicas (b = B/D), replica j's index array is the concatenation
// over steps k of G[k*B + j*b, k*B + (j+1)*b), clipped to the epoch length.
//
// Viewing G as a matrix of B columns, partition j is the column block [j*b, (j+1)*b) stored row by row,
// so going from D to D' replicas is a re-slicing of the column axis - the same split / move / merge as
// for a row-parallel weight - plus one ragged last row.
#include <algorithm>

#include "tpx_internal.hpp"

namespace tpx {

namespace {
// entries of partition j in the ragged last step of `tail` samples
uint64_t tail_part(uint64_t tail, uint64_t b, uint64_t j) {
  const uint64_t lo = j * b;
  return tail > lo ? std::min(b, tail - lo) : 0;
}
}  // namespace

tpx_status plan_dataset_moves(tpx_plan_s& plan, uint64_t n, uint32_t B, uint32_t eb, uint32_t D, uint32_t Dn,
                              const uint64_t* src_cursors, std::vector<uint64_t>& dst_cursors) {
  if (!B || !D || !Dn) return fail(TPX_ERR_INVALID_ARG, "dataset: batch and replica counts must be >= 1");
  if (D > TPX_MAX_RANKS || Dn > TPX_MAX_RANKS) return fail(TPX_ERR_INVALID_ARG, "dataset: more than TPX_MAX_RANKS replicas");
  if (eb != 8 && eb != 16) return fail(TPX_ERR_INVALID_ARG, "dataset: index entries must be 8 or 16 bytes");
  if (B % D || B % Dn) return fail(TPX_ERR_INDIVISIBLE, "dataset: global batch not divisible by the replica count");
  if (!src_cursors) return fail(TPX_ERR_INVALID_ARG, "dataset: src_cursors is NULL");
  const uint64_t b = B / D, bn = B / Dn;
  const uint64_t full = n / B, tail = n % B;

  // partition sizes on both sides
  for (int side = 0; side < 2; ++side) {
    Side& s = plan.side[side];
    s = Side{};
    const uint32_t deg = side ? Dn : D;
    const uint64_t w = side ? bn : b;
    s.alive.assign(deg, 1);
    s.ranks.resize(deg);
    s.bytes.resize(deg);
    for (uint32_t j = 0; j < deg; ++j) s.bytes[j] = (full * w + tail_part(tail, w, j)) * eb;
  }

  // cursors: the job has done `steps` whole steps iff every replica has consumed min(its entries, steps * b).
  // The furthest any replica has got, in local batches, is the only candidate; the ragged end counts as a step.
  uint64_t steps = 0;
  for (uint32_t j = 0; j < D; ++j) steps = std::max(steps, (src_cursors[j] + b - 1) / b);
  for (uint32_t j = 0; j < D; ++j) {
    const uint64_t size_j = full * b + tail_part(tail, b, j);
    if (src_cursors[j] > size_j) return fail(TPX_ERR_CURSOR, "dataset: cursor of partition " + std::to_string(j) + " is past its end");
    if (src_cursors[j] != std::min(size_j, steps * b))
      return fail(TPX_ERR_CURSOR, "dataset: cursor of partition " + std::to_string(j) + " is not where " + std::to_string(steps) + " whole steps leave it");
  }
  dst_cursors.resize(Dn);
  for (uint32_t j = 0; j < Dn; ++j) dst_cursors[j] = std::min(full * bn + tail_part(tail, bn, j), steps * bn);

  // split + move + merge on the column axis
  plan.boxes.clear();
  uint64_t pieces = 0;
  std::vector<tpx_box> tails;
  for (uint32_t jn = 0; jn < Dn; ++jn) {
    uint64_t pos = jn * bn;
    const uint64_t end = (jn + 1) * bn;
    tails.clear();  // the pieces of the whole steps stay neighbours in the list (they merge into whole new rows); the ragged step follows
    while (pos < end) {
      const uint64_t j = pos / b;
      const uint64_t cut = std::min(end, (j + 1) * b);
      ++pieces;
      if (full) {  // the whole steps: `full` rows of (cut - pos) entries
        tpx_box bx{};
        bx.kind = TPX_BOX_COPY;
        bx.src_rank = uint32_t(j);
        bx.dst_rank = jn;
        bx.n_dst = 1;
        bx.elem_bytes = eb;
        bx.src_off = (pos - j * b) * eb;
        bx.dst_off = (pos - jn * bn) * eb;
        bx.run_bytes = (cut - pos) * eb;
        if (full > 1 && !(cut - pos == b && cut - pos == bn)) {
          bx.ndim = 1;
          bx.extent[0] = full;
          bx.src_stride[0] = b * eb;
          bx.dst_stride[0] = bn * eb;
        } else {
          bx.run_bytes *= full;  // one row, or identical partitions: a single run
        }
        plan.boxes.push_back(bx);
      }
      if (tail > pos) {  // the ragged last step
        tpx_box bx{};
        bx.kind = TPX_BOX_COPY;
        bx.src_rank = uint32_t(j);
        bx.dst_rank = jn;
        bx.n_dst = 1;
        bx.elem_bytes = eb;
        bx.src_off = (full * b + (pos - j * b)) * eb;
        bx.dst_off = (full * bn + (pos - jn * bn)) * eb;
        bx.run_bytes = (std::min(cut, tail) - pos) * eb;
        tails.push_back(bx);
      }
      pos = cut;
    }
    plan.boxes.insert(plan.boxes.end(), tails.begin(), tails.end());
  }
  plan.stats.n_pieces = pieces;
  return TPX_OK;
}

}  // namespace tpx

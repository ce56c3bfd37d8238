// Reconfiguration plan generation (paper section 4.2, algorithm 1), specialised to the case where
// every resource is a buffer in one GPU's memory.
//
// The algorithm's three operations collapse into one record per piece:
//   split(v, sigma, sigma')   - the pieces w of a tensor are the non-empty intersections of an old and a
//                               new sub-tensor (boxes of the full tensor);
//   move(w, r_w, r')          - r_w = get_resource(phi, alpha, w) is a surviving holder of w under the old
//                               configuration, chosen for locality; r' is the new holder;
//   merge(W)                  - the pieces of a new sub-tensor are adjacent again simply because each is
//                               written at its own offset inside the new sub-tensor; nothing is staged.
//                               Where the pieces are equal column blocks of the same rows, the GPU tile
//                               covers whole destination rows and reads all of them (a merge tile).
// The result is a list of boxes (tpx_box), which tile_boxes() turns into the flat-box table the kernel
// derives its equal-byte tiles from.
#include <algorithm>
#include <cstring>
#include <map>

#include "tpx_internal.hpp"

namespace tpx {

namespace {

struct Axis {
  uint64_t extent, ss, ds;  // strides in bytes
};

// Element strides (in elements) of each canonical axis inside a stored block.
void stored_strides(const tpx_entry& e, uint64_t stride[4]) {
  uint64_t acc = 1;
  for (int i = int(e.ndim) - 1; i >= 0; --i) {
    const uint32_t ax = e.perm[i];
    stride[ax] = acc;
    acc *= e.hi[ax] - e.lo[ax];
  }
}

// Turn the piece [lo, hi) (canonical coordinates) of tensor blocks `se` (source, may be null for a
// fill) and `de` (destination) into a box: drop unit axes, order by destination stride, fuse axes that
// are nested the same way on both sides, and peel off the innermost run if it is contiguous on both.
tpx_box lower_piece(const uint64_t lo[4], const uint64_t hi[4], const tpx_entry* se, uint32_t src_rank,
                    const tpx_entry& de, uint32_t dst_rank) {
  tpx_box b{};
  const uint64_t eb = de.elem_bytes;
  uint64_t sstr[4] = {0, 0, 0, 0}, dstr[4] = {0, 0, 0, 0};
  stored_strides(de, dstr);
  if (se) stored_strides(*se, sstr);
  b.elem_bytes = uint32_t(eb);
  b.tensor_id = de.tensor_id;
  b.src_rank = se ? src_rank : 0;
  b.dst_rank = dst_rank;
  b.n_dst = 1;
  b.dst_rank_stride = 0;
  b.dst_off = de.offset;
  b.src_off = se ? se->offset : 0;
  Axis ax[4];
  size_t n = 0;
  for (uint32_t k = 0; k < de.ndim; ++k) {
    b.dst_off += (lo[k] - de.lo[k]) * dstr[k] * eb;
    if (se) b.src_off += (lo[k] - se->lo[k]) * sstr[k] * eb;
    if (hi[k] - lo[k] > 1) ax[n++] = Axis{hi[k] - lo[k], (se ? sstr[k] : dstr[k]) * eb, dstr[k] * eb};
  }
  std::sort(ax, ax + n, [](const Axis& x, const Axis& y) { return x.ds != y.ds ? x.ds > y.ds : x.ss > y.ss; });
  for (size_t i = 0; i + 1 < n;) {
    if (ax[i].ss == ax[i + 1].ss * ax[i + 1].extent && ax[i].ds == ax[i + 1].ds * ax[i + 1].extent) {
      ax[i + 1].extent *= ax[i].extent;
      for (size_t j = i; j + 1 < n; ++j) ax[j] = ax[j + 1];
      --n;
      if (i) --i;
    } else {
      ++i;
    }
  }
  b.run_bytes = eb;
  b.kind = se ? TPX_BOX_COPY : TPX_BOX_FILL;
  if (n && ax[n - 1].ds == eb && ax[n - 1].ss == eb) {
    b.run_bytes = ax[n - 1].extent * eb;
    --n;
  } else if (n && se) {
    b.kind = TPX_BOX_TRANSPOSE;
  }
  b.ndim = uint32_t(n);
  for (size_t i = 0; i < n; ++i) {
    b.extent[i] = ax[i].extent;
    b.src_stride[i] = se ? ax[i].ss : 0;
    b.dst_stride[i] = ax[i].ds;
  }
  return b;
}

}  // namespace

uint64_t box_bytes(const tpx_box& b) {
  uint64_t n = b.run_bytes;
  for (uint32_t i = 0; i < b.ndim; ++i) n *= b.extent[i];
  return n;
}

// get_resource(phi, alpha, w): among the surviving old holders of the old sub-tensor that contains
// piece w, prefer (1) the one whose buffer index equals the destination's (the "same device": nothing
// crosses), then (2) one with the destination's tensor-parallel index (only replicated tensors have a
// choice here; it keeps a rank's neighbouring tensors coming from one source buffer, so their moves
// merge), then (3) the lowest rank index.  Returns -1 if no holder survives.
static int get_resource(const Side& src, const Side& dst, const SubTensor& sub, uint32_t dst_rank) {
  int best = -1, best_score = 3;
  const bool tp = src.tp_degree && dst.tp_degree;
  const uint32_t t_dst = tp ? dst_rank % dst.tp_degree : 0;
  for (size_t i = 0; i < sub.holders.size(); ++i) {
    const uint32_t r = sub.holders[i].rank;
    if (!src.alive[r]) continue;
    const int score = r == dst_rank ? 0 : (tp && r % src.tp_degree == t_dst ? 1 : 2);
    if (score < best_score) { best = int(i); best_score = score; }
  }
  return best;
}

namespace {

// SPLIT: W = get_split_tensors(t, sigma, sigma') for the new sub-tensor sn: its intersections with the
// old sub-tensors of the same tensor, in position order.  Calls fn(lo, hi, sub) per piece; sub == nullptr
// marks rows that exist only as new padding (axis 0 of the new tensor is longer than the old one's).
// The old sub-tensors must tile the part of sn that exists in the old tensor.
template <typename Fn>
tpx_status for_each_piece(const tpx_entry& sn, const tpx_entry& any, const std::vector<SubTensor>& subs, Fn&& fn) {
  if (any.ndim != sn.ndim || any.elem_bytes != sn.elem_bytes) return fail(TPX_ERR_INVALID_ARG, "tensor rank or element size differs between configurations");
  for (uint32_t k = 1; k < sn.ndim; ++k)  // only the (padded) extent of axis 0 may differ
    if (any.full_shape[k] != sn.full_shape[k]) return fail(TPX_ERR_INVALID_ARG, "tensor shapes differ between configurations");
  const uint64_t old_rows = any.full_shape[0];
  uint64_t want = 1, got = 0;
  for (uint32_t k = 0; k < sn.ndim; ++k) {
    const uint64_t hi = k == 0 ? std::min(sn.hi[0], old_rows) : sn.hi[k];
    want *= hi > sn.lo[k] ? hi - sn.lo[k] : 0;
  }
  for (const SubTensor& sub : subs) {
    uint64_t lo[4] = {0, 0, 0, 0}, hi[4] = {0, 0, 0, 0}, vol = 1;
    for (uint32_t k = 0; k < sn.ndim; ++k) {
      lo[k] = std::max(sn.lo[k], sub.lo[k]);
      hi[k] = std::min(sn.hi[k], sub.hi[k]);
      vol *= hi[k] > lo[k] ? hi[k] - lo[k] : 0;
    }
    if (!vol) continue;
    got += vol;
    if (tpx_status st = fn(lo, hi, &sub)) return st;
  }
  if (got != want) return fail(TPX_ERR_INVALID_ARG, "the old sub-tensors of tensor " + std::to_string(sn.tensor_id) + " do not tile it");
  if (sn.hi[0] > old_rows) {
    uint64_t lo[4], hi[4];
    for (uint32_t k = 0; k < 4; ++k) { lo[k] = sn.lo[k]; hi[k] = sn.hi[k]; }
    lo[0] = std::max(sn.lo[0], old_rows);
    if (tpx_status st = fn(lo, hi, nullptr)) return st;
  }
  return TPX_OK;
}

}  // namespace

tpx_status plan_model_moves(tpx_plan_s& plan) {
  const Side& S = plan.side[0];
  const Side& Sn = plan.side[1];
  plan.boxes.clear();
  uint64_t n_pieces = 0;
  struct Piece {
    uint64_t lo[4], hi[4];
    const SubTensor* sub;  // nullptr: rows that exist only as new padding
    const tpx_entry* sn;
  };
  std::vector<Piece> pieces;
  std::vector<std::vector<int>> choice;
  const uint64_t max_multicast = plan.opts.max_multicast, share_reads = plan.opts.share_reads;
  auto unrecoverable = [&](const tpx_entry& sn) {
    return fail(TPX_ERR_UNRECOVERABLE, "no surviving holder of a piece of tensor " + std::to_string(sn.tensor_id) +
                                           (sn.name < N_NAMES && S.tp_degree ? std::string(" (") + param_name(sn.name) + ", layer " + std::to_string(sn.layer) + ")" : std::string()));
  };
  auto emit = [&](const Piece& pc, int h, uint32_t rn, uint32_t n_dst, uint32_t stride) {
    tpx_box b;
    if (!pc.sub) {
      b = lower_piece(pc.lo, pc.hi, nullptr, 0, *pc.sn, rn);
    } else {
      const Holder& who = pc.sub->holders[size_t(h)];
      b = lower_piece(pc.lo, pc.hi, &S.ranks[who.rank][who.entry], who.rank, *pc.sn, rn);  // move(w, r_w, r')
    }
    b.n_dst = n_dst;
    b.dst_rank_stride = n_dst > 1 ? stride : 0;
    plan.boxes.push_back(b);
  };
  // RE-PARTITION: foreach r' in R', foreach sub-tensor s' allocated to r'.  Ranks of a replica group hold
  // identical sub-collections at identical offsets; members that also make the same source choices are
  // served by one multicast move (read once, written to each), so a group is planned together.
  for (const ReplicaGroup& g : Sn.groups) {
    const uint32_t r0 = g.first;
    // SPLIT, once per group: the pieces of every sub-tensor of the (shared) manifest
    pieces.clear();
    for (const tpx_entry& sn : Sn.ranks[r0]) {
      const int32_t key = S.find_key(sn.tensor_id, sn.kind);  // get_base_tensor: the same tensor, old side
      if (key < 0) return fail(TPX_ERR_INVALID_ARG, "tensor " + std::to_string(sn.tensor_id) + " is missing from the source configuration");
      const auto& subs = S.subs[size_t(key)];
      const tpx_entry& any = S.ranks[subs[0].holders[0].rank][subs[0].holders[0].entry];
      tpx_status st = for_each_piece(sn, any, subs, [&](const uint64_t* lo, const uint64_t* hi, const SubTensor* sub) -> tpx_status {
        Piece pc;
        for (uint32_t k = 0; k < 4; ++k) { pc.lo[k] = lo[k]; pc.hi[k] = hi[k]; }
        pc.sub = sub;
        pc.sn = &sn;
        pieces.push_back(pc);
        return TPX_OK;
      });
      if (st) return st;
      // merge(W): implicit - the pieces are addressed inside s' itself
    }
    if (g.count == 1) {  // no replicas: choose (get_resource) and move in one go
      for (const Piece& pc : pieces) {
        int h = -1;
        if (pc.sub) {
          h = get_resource(S, Sn, *pc.sub, r0);
          if (h < 0) return unrecoverable(*pc.sn);
          ++n_pieces;
        }
        emit(pc, h, r0, 1, 0);
      }
      continue;
    }
    // every member's source choice for every piece
    choice.assign(g.count, std::vector<int>());
    for (uint32_t dn = 0; dn < g.count; ++dn) {
      const uint32_t rn = r0 + dn * g.stride;
      choice[dn].reserve(pieces.size());
      for (const Piece& pc : pieces) {
        int h = -1;
        if (pc.sub) {
          h = get_resource(S, Sn, *pc.sub, rn);
          if (h < 0) return unrecoverable(*pc.sn);
          ++n_pieces;
        }
        choice[dn].push_back(h);
      }
    }
    // With every buffer in one GPU's memory "the same device" saves nothing, while one shared source
    // makes the whole group one multicast move: each piece is read once instead of once per distinct choice.
    if (share_reads)
      for (uint32_t dn = 1; dn < g.count; ++dn) choice[dn] = choice[0];
    // one set of moves per run of consecutive members with identical choices
    for (uint32_t d0 = 0; d0 < g.count;) {
      uint32_t d1 = d0 + 1;
      while (d1 < g.count && d1 - d0 < max_multicast && choice[d1] == choice[d0]) ++d1;
      const uint32_t rn = r0 + d0 * g.stride;
      for (size_t i = 0; i < pieces.size(); ++i) emit(pieces[i], choice[d0][i], rn, d1 - d0, g.stride);
      d0 = d1;
    }
  }
  plan.stats.n_pieces = n_pieces;
  return TPX_OK;
}

// Two boxes that are plain runs, exact neighbours in both the source and the destination buffer
// (no alignment gap in between), become one.
void coalesce_boxes(std::vector<tpx_box>& boxes) {
  std::vector<tpx_box> out;
  out.reserve(boxes.size());
  for (const tpx_box& b : boxes) {
    if (!out.empty()) {
      tpx_box& a = out.back();
      const bool plain = a.ndim == 0 && b.ndim == 0 && a.kind == b.kind && a.kind != TPX_BOX_TRANSPOSE;
      if (plain && a.dst_rank == b.dst_rank && a.n_dst == b.n_dst && a.dst_rank_stride == b.dst_rank_stride &&
          a.dst_off + a.run_bytes == b.dst_off &&
          (a.kind == TPX_BOX_FILL || (a.src_rank == b.src_rank && a.src_off + a.run_bytes == b.src_off))) {
        a.run_bytes += b.run_bytes;
        a.elem_bytes = std::min(a.elem_bytes, b.elem_bytes);
        continue;
      }
    }
    out.push_back(b);
  }
  boxes.swap(out);
}

namespace {

uint32_t unit_log2_of(uint64_t bits) {  // largest power of two <= 16 dividing everything OR-ed into bits
  uint32_t l = 0;
  while (l < 4 && !(bits & (1ull << l))) ++l;
  return l;
}

// Cut a span of `run` bytes into n near-equal chunks of at most tile_bytes, chunk sizes multiples of `quantum`.
uint64_t chunk_of(uint64_t run, uint64_t tile_bytes, uint64_t quantum) {
  if (run <= tile_bytes) return run;
  const uint64_t n = (run + tile_bytes - 1) / tile_bytes;
  uint64_t c = (run + n - 1) / n;
  c = (c + quantum - 1) / quantum * quantum;
  return std::min(c, tile_bytes);
}

constexpr uint64_t kMaxRunUnits = 0x80000000ull;  // units per row of one flat box

}  // namespace

// Boxes -> flat boxes (at most two-dimensional, with their tiling parameters), tile prefix sums and the
// coarse search table.  Tiles are bounded by tile_bytes; on small jobs the bound is lowered so that
// the launch still has thousands of workgroups.
tpx_status tile_boxes(tpx_plan_s& plan, uint64_t tile_bytes) {
  plan.flat.clear();
  uint64_t total = 0;
  for (const tpx_box& b : plan.boxes) total += box_bytes(b);
  for (const tpx_box& b : plan.boxes)  // a plan with transposing moves runs workgroups sized for their blocks
    if (b.kind == TPX_BOX_TRANSPOSE) tile_bytes = std::min<uint64_t>(tile_bytes, kBlockBytes);
  while (tile_bytes > 16384 && total / tile_bytes < 8192) tile_bytes >>= 1;
  plan.tile_bytes_used = tile_bytes;
  plan.segments.clear();
  plan.uniform_tiles = true;
  for (const tpx_box& b : plan.boxes) plan.uniform_tiles = plan.uniform_tiles && b.n_dst == plan.boxes[0].n_dst;
  // Short contiguous moves (biases, LayerNorm vectors, the replicated tensors of every layer) would each hold a compute
  // unit for a full memory round trip while moving a few KiB: those that go to the same destination buffer(s) are
  // set aside here and share PACK tiles, made after all other boxes.
  const uint64_t pack_limit = plan.opts.pack_bytes ? plan.opts.pack_bytes : tile_bytes / 4;
  std::vector<uint8_t> packed(plan.boxes.size(), 0);
  std::map<uint64_t, std::vector<size_t>> pack_groups;  // (first destination, replicas, their stride) -> boxes, in plan order
  for (size_t bi = 0; bi < plan.boxes.size(); ++bi) {
    const tpx_box& b = plan.boxes[bi];
    if (b.kind != TPX_BOX_COPY || b.ndim != 0 || !b.run_bytes || b.run_bytes > pack_limit || b.run_bytes > tile_bytes) continue;
    if ((b.src_off | b.dst_off | b.run_bytes) % 16 || b.src_rank >= TPX_MAX_RANKS || b.dst_rank >= TPX_MAX_RANKS || b.n_dst > 255 ||
        b.dst_rank_stride > 255)
      continue;
    pack_groups[uint64_t(b.dst_rank) | uint64_t(b.n_dst) << 32 | uint64_t(b.dst_rank_stride) << 48].push_back(bi);
  }
  for (auto it = pack_groups.begin(); it != pack_groups.end();) {
    if (it->second.size() < 2) { it = pack_groups.erase(it); continue; }  // nothing to share a tile with
    for (size_t bi : it->second) packed[bi] = 1;
    ++it;
  }
  for (size_t bi = 0; bi < plan.boxes.size(); ++bi) {
    const tpx_box& b = plan.boxes[bi];
    if (box_bytes(b) == 0 || packed[bi]) continue;
    // merge(W) inside the tile: K consecutive moves that each bring one column block of the same
    // destination rows, together the whole row, become one MERGE box whose tiles write whole destination
    // rows and read K sources.  The blocks may differ in width (T 3 -> 4 cuts rows in thirds and quarters);
    // then the kernel needs the segment table in LDS, which bounds K.
    if (b.kind == TPX_BOX_COPY && b.ndim == 1 && b.run_bytes % 16 == 0 && b.dst_stride[0] > b.run_bytes &&
        b.dst_stride[0] <= tile_bytes && b.dst_stride[0] % 16 == 0 && b.extent[0] <= 0xffffffffull) {
      uint64_t K = 0, width = 0, bits = b.dst_off | b.dst_stride[0];
      bool ok = true, equal = true;
      while (ok && width < b.dst_stride[0]) {
        ok = bi + K < plan.boxes.size() && K < 0xffff;
        if (!ok) break;
        const tpx_box& c = plan.boxes[bi + K];
        ok = c.kind == TPX_BOX_COPY && c.ndim == 1 && c.run_bytes % 16 == 0 && c.extent[0] == b.extent[0] &&
             c.dst_stride[0] == b.dst_stride[0] && c.dst_rank == b.dst_rank && c.n_dst == b.n_dst &&
             c.dst_rank_stride == b.dst_rank_stride && c.dst_off == b.dst_off + width && c.src_rank < TPX_MAX_RANKS;
        bits |= c.src_off | c.src_stride[0];
        equal = equal && c.run_bytes == b.run_bytes;
        width += c.run_bytes;
        ++K;
      }
      ok = ok && width == b.dst_stride[0] && K >= 2 && (equal || K <= kMaxSegLds);
      if (ok && bits % 16 == 0) {
        FlatBox f{};
        f.kind = TPX_TILE_MERGE;
        f.unit_log2 = 4;
        f.dst_rank = uint16_t(b.dst_rank);
        f.n_dst = uint8_t(b.n_dst);
        f.dst_rank_stride = uint8_t(b.dst_rank_stride);
        if (b.dst_rank + uint64_t(b.n_dst - 1) * b.dst_rank_stride >= TPX_MAX_RANKS) return fail(TPX_ERR_INVALID_ARG, "rank out of range");
        f.dst_off = b.dst_off;
        f.dst_pitch = b.dst_stride[0];
        f.src_step = f.dst_step = 16;
        f.nrows = uint32_t(b.extent[0]);
        f.run_units = uint32_t(b.dst_stride[0] / 16);
        f.chunk_units = f.run_units;
        f.chunks_per_row = 1;
        f.rows_per_tile = uint32_t(std::max<uint64_t>(1, tile_bytes / b.dst_stride[0]));
        f.seg_first = uint32_t(plan.segments.size());
        f.n_seg = uint32_t(K);
        f.seg_units = equal ? uint32_t(b.run_bytes / 16) : 0;
        for (uint64_t k = 0; k < K; ++k) {
          const tpx_box& c = plan.boxes[bi + k];
          plan.segments.push_back(tpx_segment{c.src_off, c.src_stride[0], c.src_rank, uint32_t(c.run_bytes / 16), 0});
        }
        plan.flat.push_back(f);
        bi += K - 1;
        continue;
      }
    }
    if (b.src_rank >= TPX_MAX_RANKS || b.dst_rank >= TPX_MAX_RANKS) return fail(TPX_ERR_INVALID_ARG, "rank out of range");
    FlatBox f{};
    f.src_rank = uint16_t(b.src_rank);
    f.dst_rank = uint16_t(b.dst_rank);
    f.n_dst = uint8_t(b.n_dst);
    f.dst_rank_stride = uint8_t(b.dst_rank_stride);
    if (b.dst_rank + uint64_t(b.n_dst - 1) * b.dst_rank_stride >= TPX_MAX_RANKS) return fail(TPX_ERR_INVALID_ARG, "rank out of range");
    uint32_t I = 0, J = 0;     // the two axes a flat box keeps; all others are enumerated
    uint64_t nI = 1, nJ = 1;
    if (b.kind == TPX_BOX_TRANSPOSE) {
      // Plane (I, J): J = axis contiguous on the source, I = axis contiguous on the destination.  When one
      // axis is the finest on both sides (its contiguous partner had extent 1) the plane degenerates and
      // elements are gathered one by one.
      const uint64_t eb = b.elem_bytes;
      for (uint32_t k = 1; k < b.ndim; ++k) {
        if (b.src_stride[k] < b.src_stride[J]) J = k;
        if (b.dst_stride[k] < b.dst_stride[I]) I = k;
      }
      uint32_t ulog = 0;
      while ((1ull << ulog) < eb) ++ulog;
      f.unit_log2 = uint8_t(ulog);
      const bool plane = I != J && b.src_stride[J] == eb && b.dst_stride[I] == eb;
      if (!plane) {
        I = J;
        for (uint32_t k = 0; k < b.ndim; ++k) if (k != J) { I = k; break; }
      }
      f.kind = plane ? TPX_TILE_TRANSPOSE : TPX_TILE_GATHER;
      nI = (I == J) ? 1 : b.extent[I];
      nJ = b.extent[J];
      f.src_step = b.src_stride[J];
      f.dst_step = b.dst_stride[J];
      f.src_pitch = (I == J) ? 0 : b.src_stride[I];
      f.dst_pitch = (I == J) ? 0 : b.dst_stride[I];
      const uint32_t rows = plane ? block_i(uint32_t(eb), nI) : 0;
      if (rows) {  // blocks the kernel moves in one shot
        // consecutive workgroups then write neighbouring segments of the same destination rows: the scattered side
        // is the reads, which take it better (measured: 5.85 -> 6.0 TB/s on the 1.3B-shape transposing reshard)
        f.rows_first = 1;
        f.rows_per_tile = rows;
        f.chunk_units = uint32_t(kBlockBytes / (rows * eb));
      } else {
        f.rows_per_tile = uint32_t(std::min<uint64_t>(nI, 256));
        f.chunk_units = uint32_t(std::max<uint64_t>(64, std::min<uint64_t>(nJ, tile_bytes / (f.rows_per_tile * eb))));
      }
    } else {
      // COPY / FILL: the unit is the widest power of two (<= 16 bytes) that divides every offset, pitch
      // and the run length; buffer bases are required to be 16-byte aligned.
      uint64_t bits = b.dst_off | b.run_bytes | 16;
      if (b.kind == TPX_BOX_COPY) bits |= b.src_off;
      for (uint32_t k = 0; k < b.ndim; ++k) bits |= b.dst_stride[k] | (b.kind == TPX_BOX_COPY ? b.src_stride[k] : 0);
      const uint32_t ulog = unit_log2_of(bits);
      const uint64_t unit = 1ull << ulog;
      f.kind = uint8_t(b.kind == TPX_BOX_COPY ? TPX_TILE_COPY : TPX_TILE_FILL);
      f.unit_log2 = uint8_t(ulog);
      f.src_step = f.dst_step = unit;
      I = J = b.ndim ? b.ndim - 1 : 0;  // rows = the innermost outer axis; the run itself is the "J" extent
      nI = b.ndim ? b.extent[b.ndim - 1] : 1;
      nJ = b.run_bytes >> ulog;
      f.src_pitch = b.ndim ? b.src_stride[b.ndim - 1] : 0;
      f.dst_pitch = b.ndim ? b.dst_stride[b.ndim - 1] : 0;
      if (b.run_bytes > tile_bytes) {  // long rows: each row is cut into contiguous chunks
        const uint64_t quantum = std::max<uint64_t>(unit, (b.run_bytes % 256 == 0) ? 256 : unit);
        f.rows_per_tile = 1;
        f.chunk_units = uint32_t(chunk_of(b.run_bytes, tile_bytes, quantum) >> ulog);
      } else {                         // short rows: several whole rows per tile
        f.rows_per_tile = uint32_t(std::max<uint64_t>(1, tile_bytes / b.run_bytes));
        f.chunk_units = uint32_t(nJ);
      }
    }
    // A contiguous run longer than 32-bit unit counts reach (a whole arena of one rank coalesced into one move)
    // is cut into several flat boxes, each a whole number of chunks long.
    // The same goes for more rows than a 32-bit count holds: several flat boxes of whole tiles of rows.
    const bool linear = f.kind == TPX_TILE_COPY || f.kind == TPX_TILE_FILL;
    const uint64_t piece = linear ? (kMaxRunUnits / f.chunk_units) * f.chunk_units : 0xffffffffull;
    const uint64_t row_piece = linear ? (kMaxRunUnits / f.rows_per_tile) * f.rows_per_tile : 0xffffffffull;
    if (!linear && (nI > row_piece || nJ > piece)) return fail(TPX_ERR_INVALID_ARG, "a transposing move is too large for 32-bit tile indices");
    uint64_t idx[4] = {0, 0, 0, 0};
    for (;;) {  // odometer over the enumerated axes
      f.src_off = b.src_off;
      f.dst_off = b.dst_off;
      for (uint32_t k = 0; k < b.ndim; ++k)
        if (k != I && k != J) { f.src_off += idx[k] * b.src_stride[k]; f.dst_off += idx[k] * b.dst_stride[k]; }
      for (uint64_t i0 = 0; i0 < nI; i0 += row_piece)
        for (uint64_t j0 = 0; j0 < nJ; j0 += piece) {
          FlatBox g = f;
          g.nrows = uint32_t(std::min<uint64_t>(row_piece, nI - i0));
          g.run_units = uint32_t(std::min<uint64_t>(piece, nJ - j0));
          g.chunks_per_row = (g.run_units + g.chunk_units - 1) / g.chunk_units;
          g.src_off += i0 * f.src_pitch + j0 * f.src_step;
          g.dst_off += i0 * f.dst_pitch + j0 * f.dst_step;
          plan.flat.push_back(g);
        }
      int k = int(b.ndim) - 1;
      for (; k >= 0; --k) {
        if (uint32_t(k) == I || uint32_t(k) == J) continue;
        if (++idx[k] < b.extent[k]) break;
        idx[k] = 0;
      }
      if (k < 0) break;
    }
  }
  // PACK boxes: per destination, runs of at most kMaxSegLds moves and tile_bytes bytes, one tile each
  for (const auto& group : pack_groups) {
    size_t k = 0;
    const std::vector<size_t>& ids = group.second;
    while (k < ids.size()) {
      const tpx_box& b0 = plan.boxes[ids[k]];
      FlatBox f{};
      f.kind = TPX_TILE_PACK;
      f.unit_log2 = 4;
      f.dst_rank = uint16_t(b0.dst_rank);
      f.n_dst = uint8_t(b0.n_dst);
      f.dst_rank_stride = uint8_t(b0.dst_rank_stride);
      if (b0.dst_rank + uint64_t(b0.n_dst - 1) * b0.dst_rank_stride >= TPX_MAX_RANKS) return fail(TPX_ERR_INVALID_ARG, "rank out of range");
      f.src_step = f.dst_step = 16;
      f.nrows = f.rows_per_tile = 1;
      f.chunks_per_row = 1;
      f.seg_first = uint32_t(plan.segments.size());
      uint64_t units = 0;
      while (k < ids.size() && f.n_seg < kMaxSegLds && (units + plan.boxes[ids[k]].run_bytes / 16) * 16 <= tile_bytes) {
        const tpx_box& c = plan.boxes[ids[k]];
        plan.segments.push_back(tpx_segment{c.src_off, units, c.src_rank, uint32_t(c.run_bytes / 16), c.dst_off});
        units += c.run_bytes / 16;
        ++f.n_seg;
        ++k;
      }
      f.run_units = f.chunk_units = uint32_t(units);
      plan.flat.push_back(f);
    }
  }
  // prefix sums and coarse table
  uint64_t n_tiles = 0;
  plan.first_tile.resize(plan.flat.size() + 1);
  for (size_t i = 0; i < plan.flat.size(); ++i) {
    plan.flat[i].first_tile = uint32_t(n_tiles);
    plan.first_tile[i] = uint32_t(n_tiles);
    n_tiles += tiles_of(plan.flat[i]);
    if (n_tiles > 0x7fffffffull) return fail(TPX_ERR_INVALID_ARG, "too many tiles for one launch");
  }
  plan.first_tile[plan.flat.size()] = uint32_t(n_tiles);
  plan.n_tiles = n_tiles;
  plan.coarse.assign(size_t((n_tiles >> kCoarseShift) + 2), plan.flat.empty() ? 0 : uint32_t(plan.flat.size() - 1));
  size_t box = 0;
  for (uint64_t t = 0; t < n_tiles; t += (1ull << kCoarseShift)) {
    while (box + 1 < plan.flat.size() && plan.first_tile[box + 1] <= t) ++box;
    plan.coarse[size_t(t >> kCoarseShift)] = uint32_t(box);
  }
  return TPX_OK;
}

// Host-side guard for the kernel: the first and last byte every flat box touches lie inside the rank
// buffers the manifests describe.
tpx_status validate_tiles(tpx_plan_s& plan) {
  plan.needs_lds = false;
  for (const FlatBox& t : plan.flat) {
    const uint64_t unit = 1ull << t.unit_log2;
    if (!t.nrows || !t.run_units || !t.rows_per_tile || !t.chunk_units) return fail(TPX_ERR_INVALID_ARG, "internal: empty flat box");
    const uint64_t dlast = t.dst_off + (t.nrows - 1) * t.dst_pitch + (t.run_units - 1) * t.dst_step + unit;
    if (!t.n_dst) return fail(TPX_ERR_INVALID_ARG, "internal: a move without destination");
    for (uint32_t k = 0; k < t.n_dst; ++k) {
      const uint32_t r = t.dst_rank + k * t.dst_rank_stride;
      if (r >= plan.side[1].bytes.size() || dlast > plan.side[1].bytes[r])
        return fail(TPX_ERR_INVALID_ARG, "internal: a move writes outside its destination buffer");
      if (!plan.side[1].alive[r]) return fail(TPX_ERR_INVALID_ARG, "internal: a move targets a rank that is not to be built");
    }
    if (t.kind == TPX_TILE_PACK) {
      if (!t.n_seg || t.n_seg > kMaxSegLds || uint64_t(t.seg_first) + t.n_seg > plan.segments.size() || t.unit_log2 != 4 || t.nrows != 1)
        return fail(TPX_ERR_INVALID_ARG, "internal: bad pack tile");
      uint64_t first = 0;
      for (uint32_t k = 0; k < t.n_seg; ++k) {
        const tpx_segment& sg = plan.segments[t.seg_first + k];
        if (!sg.units || sg.src_pitch != first) return fail(TPX_ERR_INVALID_ARG, "internal: bad pack segment");
        first += sg.units;
        if (sg.src_rank >= plan.side[0].bytes.size() || sg.src_off + uint64_t(sg.units) * 16 > plan.side[0].bytes[sg.src_rank])
          return fail(TPX_ERR_INVALID_ARG, "internal: a packed move reads outside its source buffer");
        for (uint32_t c = 0; c < t.n_dst; ++c)
          if (sg.dst_off + uint64_t(sg.units) * 16 > plan.side[1].bytes[t.dst_rank + c * t.dst_rank_stride])
            return fail(TPX_ERR_INVALID_ARG, "internal: a packed move writes outside its destination buffer");
      }
      if (first != t.run_units) return fail(TPX_ERR_INVALID_ARG, "internal: the moves of a pack tile do not make up its units");
    } else if (t.kind == TPX_TILE_MERGE) {
      if (!t.n_seg || uint64_t(t.seg_first) + t.n_seg > plan.segments.size() || (!t.seg_units && t.n_seg > kMaxSegLds))
        return fail(TPX_ERR_INVALID_ARG, "internal: bad segment range");
      uint64_t row_units = 0;
      for (uint32_t k = 0; k < t.n_seg; ++k) {
        const tpx_segment& sg = plan.segments[t.seg_first + k];
        if (!sg.units || (t.seg_units && sg.units != t.seg_units)) return fail(TPX_ERR_INVALID_ARG, "internal: bad segment width");
        row_units += sg.units;
      }
      if (row_units != t.run_units) return fail(TPX_ERR_INVALID_ARG, "internal: the segments of a merge do not make up its rows");
      for (uint32_t k = 0; k < t.n_seg; ++k) {
        const tpx_segment& sg = plan.segments[t.seg_first + k];
        const uint64_t slast = sg.src_off + (t.nrows - 1) * sg.src_pitch + uint64_t(sg.units) * unit;
        if (sg.src_rank >= plan.side[0].bytes.size() || slast > plan.side[0].bytes[sg.src_rank])
          return fail(TPX_ERR_INVALID_ARG, "internal: a merge reads outside its source buffer");
      }
    } else if (t.kind != TPX_TILE_FILL) {
      const uint64_t slast = t.src_off + (t.nrows - 1) * t.src_pitch + (t.run_units - 1) * t.src_step + unit;
      if (t.src_rank >= plan.side[0].bytes.size() || slast > plan.side[0].bytes[t.src_rank])
        return fail(TPX_ERR_INVALID_ARG, "internal: a move reads outside its source buffer");
    }
    if (t.kind == TPX_TILE_TRANSPOSE) plan.needs_lds = true;
  }
  return TPX_OK;
}

WorkspaceLayout workspace_layout(const tpx_plan_s& plan) {
  auto up = [](uint64_t x) { return (x + 255) / 256 * 256; };
  WorkspaceLayout w;
  w.header_off = 0;
  w.boxes_off = up(sizeof(WorkspaceHeader));
  w.first_off = w.boxes_off + up(plan.flat.size() * sizeof(FlatBox));
  w.coarse_off = w.first_off + up(plan.first_tile.size() * sizeof(uint32_t));
  w.seg_off = w.coarse_off + up(plan.coarse.size() * sizeof(uint32_t));
  w.total = std::max<uint64_t>(256, w.seg_off + up(plan.segments.size() * sizeof(tpx_segment)));
  return w;
}

void build_image(tpx_plan_s& plan) {
  const WorkspaceLayout w = workspace_layout(plan);
  plan.image.assign(size_t(w.total), 0);
  const WorkspaceHeader h{plan.id, plan.flat.size(), plan.n_tiles, plan.segments.size()};
  std::memcpy(plan.image.data() + w.header_off, &h, sizeof(h));
  if (!plan.flat.empty()) std::memcpy(plan.image.data() + w.boxes_off, plan.flat.data(), plan.flat.size() * sizeof(FlatBox));
  std::memcpy(plan.image.data() + w.first_off, plan.first_tile.data(), plan.first_tile.size() * sizeof(uint32_t));
  std::memcpy(plan.image.data() + w.coarse_off, plan.coarse.data(), plan.coarse.size() * sizeof(uint32_t));
  if (!plan.segments.empty())
    std::memcpy(plan.image.data() + w.seg_off, plan.segments.data(), plan.segments.size() * sizeof(tpx_segment));
}

void finish_stats(tpx_plan_s& plan) {
  tpx_stats_t& s = plan.stats;
  s.n_boxes = plan.boxes.size();
  s.n_tiles = plan.n_tiles;
  s.bytes_read = s.bytes_written = s.bytes_fill = s.bytes_cross_rank = 0;
  for (const tpx_box& b : plan.boxes) {
    const uint64_t n = box_bytes(b);
    s.bytes_written += n * b.n_dst;
    if (b.kind == TPX_BOX_FILL) {
      s.bytes_fill += n * b.n_dst;
    } else {
      s.bytes_read += n;  // a multicast move reads its source once
      for (uint32_t k = 0; k < b.n_dst; ++k)
        if (b.src_rank != b.dst_rank + k * b.dst_rank_stride) s.bytes_cross_rank += n;
    }
  }
}

}  // namespace tpx

// Internal declarations shared by the host planner, the C ABI and the HIP executor.
#pragma once

#include <atomic>
#include <cstdint>
#include <string>
#include <unordered_map>
#include <vector>

#include "tile_math.hpp"
#include "tpx.h"

namespace tpx {

// The 16 parameter tensors of the GPT-style model, in the order a rank buffer packs them.
enum Name : uint32_t {
  WORD_EMB = 0, POS_EMB, LN1_W, LN1_B, QKV_W, QKV_B, DENSE_W, DENSE_B,
  LN2_W, LN2_B, FC1_W, FC1_B, FC2_W, FC2_B, LNF_W, LNF_B, N_NAMES
};
constexpr uint32_t kLayerNames = 12;  // LN1_W .. FC2_B
constexpr uint64_t kAlign = 256;      // every stored tensor starts on a 256-byte boundary

// sigma of one parameter tensor under one configuration: the canonical view of the full tensor,
// the canonical axis that tensor parallelism cuts (or -1: replicated) and the storage order.
struct Sigma {
  uint32_t ndim = 0;
  uint64_t full[4] = {1, 1, 1, 1};
  int split_axis = -1;
  uint32_t perm[4] = {0, 1, 2, 3};
};

struct Holder {
  uint32_t rank;
  uint32_t entry;  // index into Side::ranks[rank]
};

// One distinct sub-tensor of a state tensor (a box of the full tensor) and every rank that stores it
// (data-parallel replicas, replicated tensors, tied copies), in ascending rank order.
struct HolderList {  // the first two holders inline: most sliced sub-tensors have one or two
  uint32_t n = 0;
  Holder inl[2] = {{0, 0}, {0, 0}};
  std::vector<Holder> more;
  void push_back(Holder h) {
    if (n < 2) inl[n] = h; else more.push_back(h);
    ++n;
  }
  size_t size() const { return n; }
  const Holder& operator[](size_t i) const { return i < 2 ? inl[i] : more[i - 2]; }
};

struct SubTensor {
  uint64_t lo[4] = {0, 0, 0, 0}, hi[4] = {0, 0, 0, 0};
  HolderList holders;
};

// Ranks of the new configuration that hold identical sub-collections at identical offsets
// (data-parallel replicas): first, first + stride, ...
struct ReplicaGroup {
  uint32_t first, count, stride;
};

// One PTC evaluated for every rank: sigma (the boxes), phi and alpha (which rank buffer, where).
struct Side {
  uint32_t tp_degree = 0;                     // T of a (T, P, D) configuration, 0 for an explicit PTC
  std::vector<uint8_t> alive;                 // per rank
  std::vector<std::vector<tpx_entry>> ranks;  // manifest of every rank buffer
  std::vector<uint64_t> bytes;                // size of every rank buffer
  // index, built by index_subs(): state tensor (tensor_id, kind) -> dense key -> its distinct sub-tensors,
  // sorted by position
  std::unordered_map<uint64_t, uint32_t> key_of;   // used when the ids are too sparse for the dense table
  std::vector<int32_t> dense_key;                  // [tensor_id * n_kinds + kind] -> key, -1 = absent
  uint32_t dense_kinds = 0;                        // 0 = dense table not in use
  std::vector<std::vector<SubTensor>> subs;
  // key of state tensor (tensor_id, kind), or -1
  int32_t find_key(uint32_t tensor_id, uint32_t kind) const {
    if (dense_kinds) {
      const uint64_t i = uint64_t(tensor_id) * dense_kinds + kind;
      return kind < dense_kinds && i < dense_key.size() ? dense_key[size_t(i)] : -1;
    }
    const auto it = key_of.find((uint64_t(tensor_id) << 8) | kind);
    return it == key_of.end() ? -1 : int32_t(it->second);
  }
  std::vector<ReplicaGroup> groups;           // partition of the ranks into replica groups
};
tpx_status check_entries(Side& side);  // validates every manifest entry, fills nbytes
tpx_status index_subs(Side& side);    // builds key_of / dense_key and subs from ranks (needed on the source side)
tpx_status find_groups(Side& side);   // builds groups from ranks (needed on the destination side)

// Error reporting: sets the thread-local message and returns `st`.
tpx_status fail(tpx_status st, const std::string& msg);
tpx_status resolve_opts(const tpx_plan_opts* in, tpx_plan_opts& out);  // defaults for NULL / zero fields, range checks
const char* last_error_cstr();

const char* param_name(uint32_t name);
uint32_t tensor_id_of(uint32_t name, int32_t layer);
uint32_t n_tensors_of(const tpx_model& m);
tpx_status check_model(const tpx_model& m);
tpx_status sigma_of(const tpx_model& m, const tpx_parallel& par, uint32_t name, Sigma& out);
tpx_status build_side(const tpx_model& m, const tpx_parallel& par, Side& out);

// Process-wide knobs of the executor (tpx_set_option).  Atomic so that one thread may set them while others
// execute: each read sees the old or the new value, never a torn one.
struct Tuning {
  std::atomic<uint64_t> streams{4};        // tile order: workgroup b works on contiguous part b % streams of the plan
  std::atomic<uint64_t> chunk{0};          // tile order: tiles an XCD takes in a row (0 = automatic, 1 = none)
  std::atomic<uint64_t> occupancy{0};      // workgroups per CU, capped through the LDS request (0 = automatic)
  std::atomic<uint64_t> variant{0};        // 0 = chosen from the tile size (512 threads x 8 nontemporal loads for 64 KiB tiles)
};
Tuning& tuning();

}  // namespace tpx

struct tpx_plan_s {
  bool is_dataset = false;
  tpx_model model{};
  tpx::Side side[2];
  std::vector<tpx_box> boxes;
  std::vector<tpx::FlatBox> flat;     // what the GPU executes
  std::vector<tpx_segment> segments;  // sources of MERGE boxes, moves of PACK boxes
  std::vector<uint32_t> first_tile;   // flat.size() + 1 prefix sums of tiles
  std::vector<uint32_t> coarse;       // box index of every 64th tile (+ sentinel)
  uint64_t n_tiles = 0;
  uint64_t tile_bytes_used = 0;
  tpx_stats_t stats{};
  bool needs_lds = false;       // some tile is staged through LDS
  bool uniform_tiles = true;    // every tile has the same number of destinations (same cost per byte)
  tpx_plan_opts opts{65536, 8, 0, 0, 0};  // the caller's options with defaults filled in
  uint64_t id = 0;              // process-unique, never 0: stamps the workspace header
  std::vector<uint8_t> image;   // host image of the whole workspace (header and tables), what an upload copies
};

namespace tpx {

// Planner stages (host).
tpx_status plan_model_moves(tpx_plan_s& plan);                 // split + re-partition + merge -> boxes
void       coalesce_boxes(std::vector<tpx_box>& boxes);        // merge neighbours
tpx_status tile_boxes(tpx_plan_s& plan, uint64_t tile_bytes);  // boxes -> tiles
tpx_status validate_tiles(tpx_plan_s& plan);                    // every access inside its buffer
void       finish_stats(tpx_plan_s& plan);
uint64_t   box_bytes(const tpx_box& b);                          // payload of one move (per destination)
tpx_status plan_dataset_moves(tpx_plan_s& plan, uint64_t n_samples, uint32_t B, uint32_t elem_bytes,
                              uint32_t D_src, uint32_t D_dst, const uint64_t* src_cursors,
                              std::vector<uint64_t>& dst_cursors);

// HIP executor (kernels.hip).
// Workspace layout: flat boxes, then first_tile, then coarse, then segments, each section starting on a 256-byte boundary.
// The workspace starts with a 256-byte header whose first word is the id of the plan whose tables
// follow; the kernel compares it with the id it was launched with and does nothing on a mismatch, so a
// workspace that was overwritten or recycled since the upload cannot steer it out of bounds.
struct WorkspaceLayout {
  uint64_t header_off = 0, boxes_off = 0, first_off = 0, coarse_off = 0, seg_off = 0, total = 0;
};
struct WorkspaceHeader {
  uint64_t plan_id, n_boxes, n_tiles, n_segments;
};
WorkspaceLayout workspace_layout(const tpx_plan_s& plan);
void build_image(tpx_plan_s& plan);  // fills plan.image from id, flat, first_tile, coarse and segments
tpx_status hip_upload_tables(void* workspace, const tpx_plan_s& plan, void* stream);
tpx_status hip_launch_tiles(const void* workspace, const tpx_plan_s& plan, const void* const* src, uint32_t n_src,
                            void* const* dst, uint32_t n_dst, uint64_t variant, void* stream);
tpx_status hip_probe_copy(void* dst, const void* src, uint64_t nbytes, void* stream);
tpx_status hip_probe_read(const void* src, uint64_t nbytes, void* sink, void* stream);
tpx_status hip_probe_fill(void* dst, uint64_t nbytes, uint32_t value, void* stream);
tpx_status hip_read_header(const void* workspace, void* stream, WorkspaceHeader* out);
// Like hip_upload_tables + hip_launch_tiles with the tables in the library's own static device array of
// TPX_STATIC_WORKSPACE_BYTES (one per GPU); allocates nothing.
tpx_status hip_execute_static(const tpx_plan_s& plan, const void* const* src, uint32_t n_src, void* const* dst,
                              uint32_t n_dst, uint64_t variant, void* stream);

}  // namespace tpx

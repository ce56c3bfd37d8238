// C ABI of libtpx (declared in tpx.h): argument checking and hand-off to the planner and the HIP executor.
#include <algorithm>
#include <atomic>
#include <chrono>
#include <cstring>
#include <memory>
#include <exception>
#include <mutex>
#include <new>
#include <string>
#include <unordered_map>

#include "tpx_internal.hpp"

using namespace tpx;

namespace {
uint64_t now_ns() {
  return uint64_t(std::chrono::duration_cast<std::chrono::nanoseconds>(
                      std::chrono::steady_clock::now().time_since_epoch()).count());
}

// Never 0, different for every plan of this process and unlikely to repeat across processes that share a
// device buffer: a counter mixed with the time the library was first used.
uint64_t next_plan_id() {
  static const uint64_t salt = now_ns();
  static std::atomic<uint64_t> counter{0};
  uint64_t x = salt + 0x9e3779b97f4a7c15ull * (counter.fetch_add(1) + 1);
  x = (x ^ (x >> 30)) * 0xbf58476d1ce4e5b9ull;
  x = (x ^ (x >> 27)) * 0x94d049bb133111ebull;
  x ^= x >> 31;
  return x ? x : 1;
}

tpx_status finish_plan(tpx_plan_s& p) {
  p.id = next_plan_id();
  coalesce_boxes(p.boxes);
  if (tpx_status st = tile_boxes(p, p.opts.tile_bytes)) return st;
  if (tpx_status st = validate_tiles(p)) return st;
  finish_stats(p);
  build_image(p);
  return TPX_OK;
}

// Which plan's tables the library last copied to a workspace address.  tpx_prepare consults and updates it under
// the mutex, so any number of threads may execute plans (the plans themselves are never modified), and two
// plans taking turns on one workspace each find out that their tables are gone.
std::mutex g_ws_mutex;
std::unordered_map<const void*, uint64_t> g_ws_plan;
constexpr size_t kMaxTrackedWorkspaces = 4096;  // beyond that everything is forgotten (tables are copied again)
}  // namespace

extern "C" {

tpx_status tpx_plan(const tpx_model* model, const tpx_parallel* src, const tpx_parallel* dst, const tpx_plan_opts* opts,
                    tpx_plan_t** out) {
  if (!model || !src || !dst || !out) return fail(TPX_ERR_INVALID_ARG, "tpx_plan: NULL argument");
  const uint64_t t0 = now_ns();
  try {
    if (tpx_status st = check_model(*model)) return st;
    std::unique_ptr<tpx_plan_s> p(new tpx_plan_s());
    if (tpx_status st = resolve_opts(opts, p->opts)) return st;
    p->model = *model;
    tpx_status st = build_side(*model, *src, p->side[0]);
    if (!st) st = build_side(*model, *dst, p->side[1]);
    if (!st) st = index_subs(p->side[0]);
    if (!st) st = find_groups(p->side[1]);
    if (!st) st = plan_model_moves(*p);
    if (!st) st = finish_plan(*p);
    if (st) return st;
    p->stats.plan_ns = now_ns() - t0;
    *out = p.release();
    return TPX_OK;
  } catch (const std::bad_alloc&) {
    return fail(TPX_ERR_OOM, "tpx_plan: out of host memory");
  } catch (const std::exception& e) {
    return fail(TPX_ERR_INVALID_ARG, std::string("tpx_plan: ") + e.what());
  }
}

static tpx_status side_from_ptc(const tpx_ptc* c, Side& out, const char* which) {
  if (!c->n_ranks || c->n_ranks > TPX_MAX_RANKS) return fail(TPX_ERR_INVALID_ARG, std::string(which) + ": n_ranks must be 1..TPX_MAX_RANKS");
  if (!c->n_entries || !c->entries) return fail(TPX_ERR_INVALID_ARG, std::string(which) + ": NULL entry tables");
  out = Side{};
  out.alive.assign(c->n_ranks, 1);
  if (c->rank_alive) std::copy(c->rank_alive, c->rank_alive + c->n_ranks, out.alive.begin());
  out.ranks.resize(c->n_ranks);
  out.bytes.assign(c->n_ranks, 0);
  for (uint32_t r = 0; r < c->n_ranks; ++r) {
    if (c->n_entries[r] && !c->entries[r]) return fail(TPX_ERR_INVALID_ARG, std::string(which) + ": NULL entries for a rank");
    out.ranks[r].assign(c->entries[r], c->entries[r] + c->n_entries[r]);
    uint64_t end = 0, n_auto = 0;
    for (const tpx_entry& e : out.ranks[r]) n_auto += e.offset == TPX_OFFSET_AUTO;
    if (n_auto && n_auto != out.ranks[r].size())
      return fail(TPX_ERR_INVALID_ARG, std::string(which) + ": a rank's entries must all have TPX_OFFSET_AUTO or none");
    for (tpx_entry& e : out.ranks[r]) {
      uint64_t numel = 1;
      for (uint32_t k = 0; k < e.ndim && k < 4; ++k) numel *= e.hi[k] - e.lo[k];
      if (n_auto) e.offset = (end + kAlign - 1) / kAlign * kAlign;  // alpha left to the library: packed in list order
      end = std::max(end, e.offset + numel * e.elem_bytes);
    }
    out.bytes[r] = c->rank_bytes ? c->rank_bytes[r] : (end + kAlign - 1) / kAlign * kAlign;
  }
  return check_entries(out);
}

tpx_status tpx_plan_ptc(const tpx_ptc* src, const tpx_ptc* dst, const tpx_plan_opts* opts, tpx_plan_t** out) {
  if (!src || !dst || !out) return fail(TPX_ERR_INVALID_ARG, "tpx_plan_ptc: NULL argument");
  const uint64_t t0 = now_ns();
  try {
    std::unique_ptr<tpx_plan_s> p(new tpx_plan_s());
    if (tpx_status st = resolve_opts(opts, p->opts)) return st;
    tpx_status st = side_from_ptc(src, p->side[0], "source");
    if (!st) st = side_from_ptc(dst, p->side[1], "destination");
    if (!st) st = index_subs(p->side[0]);
    if (!st) st = index_subs(p->side[1]);  // only for its checks: equal or disjoint sub-tensors, one shape per tensor
    if (!st) st = find_groups(p->side[1]);
    if (!st) st = plan_model_moves(*p);
    if (!st) st = finish_plan(*p);
    if (st) return st;
    p->stats.plan_ns = now_ns() - t0;
    *out = p.release();
    return TPX_OK;
  } catch (const std::bad_alloc&) {
    return fail(TPX_ERR_OOM, "tpx_plan_ptc: out of host memory");
  } catch (const std::exception& e) {
    return fail(TPX_ERR_INVALID_ARG, std::string("tpx_plan_ptc: ") + e.what());
  }
}

tpx_status tpx_plan_query(const tpx_ptc* src, uint32_t n_queries, const tpx_query* queries, const tpx_plan_opts* opts,
                          tpx_plan_t** out) {
  if (!src || !out || (n_queries && !queries)) return fail(TPX_ERR_INVALID_ARG, "tpx_plan_query: NULL argument");
  if (!src->n_ranks || src->n_ranks > TPX_MAX_RANKS || !src->n_entries || !src->entries)
    return fail(TPX_ERR_INVALID_ARG, "tpx_plan_query: malformed source collection");
  try {
    // the one destination rank: every queried box dense in the tensor's own axis order, placed by the library
    std::vector<tpx_entry> want(n_queries);
    for (uint32_t q = 0; q < n_queries; ++q) {
      const tpx_entry* like = nullptr;
      for (uint32_t r = 0; r < src->n_ranks && !like; ++r)
        for (uint32_t i = 0; i < src->n_entries[r] && src->entries[r]; ++i)
          if (src->entries[r][i].tensor_id == queries[q].tensor_id && src->entries[r][i].kind == queries[q].kind) {
            like = &src->entries[r][i];
            break;
          }
      if (!like)
        return fail(TPX_ERR_INVALID_ARG, "tpx_plan_query: tensor " + std::to_string(queries[q].tensor_id) + " kind " +
                                             std::to_string(queries[q].kind) + " is not in the collection");
      tpx_entry& e = want[q];
      e = tpx_entry{};
      e.tensor_id = like->tensor_id;
      e.kind = like->kind;
      e.elem_bytes = like->elem_bytes;
      e.ndim = like->ndim;
      e.name = like->name;
      e.layer = like->layer;
      e.offset = TPX_OFFSET_AUTO;
      for (uint32_t k = 0; k < 4 && k < like->ndim; ++k) {
        e.full_shape[k] = like->full_shape[k];
        e.lo[k] = queries[q].lo[k];
        e.hi[k] = queries[q].hi[k];
        e.perm[k] = k;
      }
    }
    const uint32_t count = n_queries;
    const tpx_entry* list = want.data();
    const tpx_ptc dst{1, &count, &list, nullptr, nullptr};
    return tpx_plan_ptc(src, &dst, opts, out);
  } catch (const std::bad_alloc&) {
    return fail(TPX_ERR_OOM, "tpx_plan_query: out of host memory");
  }
}

tpx_status tpx_plan_dataset(uint64_t n_samples, uint32_t global_batch, uint32_t index_elem_bytes, uint32_t D_src,
                            uint32_t D_dst, const uint64_t* src_cursors, uint64_t* dst_cursors, const tpx_plan_opts* opts,
                            tpx_plan_t** out) {
  if (!out || !dst_cursors) return fail(TPX_ERR_INVALID_ARG, "tpx_plan_dataset: NULL argument");
  const uint64_t t0 = now_ns();
  try {
    std::unique_ptr<tpx_plan_s> p(new tpx_plan_s());
    if (tpx_status st = resolve_opts(opts, p->opts)) return st;
    p->is_dataset = true;
    std::vector<uint64_t> cur;
    tpx_status st = plan_dataset_moves(*p, n_samples, global_batch, index_elem_bytes, D_src, D_dst, src_cursors, cur);
    if (!st) st = finish_plan(*p);
    if (st) return st;
    std::copy(cur.begin(), cur.end(), dst_cursors);
    p->stats.plan_ns = now_ns() - t0;
    *out = p.release();
    return TPX_OK;
  } catch (const std::bad_alloc&) {
    return fail(TPX_ERR_OOM, "tpx_plan_dataset: out of host memory");
  } catch (const std::exception& e) {
    return fail(TPX_ERR_INVALID_ARG, std::string("tpx_plan_dataset: ") + e.what());
  }
}

uint32_t tpx_num_buffers(const tpx_plan_t* p, int side) {
  return (p && (side == 0 || side == 1)) ? uint32_t(p->side[side].bytes.size()) : 0;
}

uint64_t tpx_buffer_bytes(const tpx_plan_t* p, int side, uint32_t rank) {
  if (!p || (side != 0 && side != 1) || rank >= p->side[side].bytes.size()) return 0;
  return p->side[side].bytes[rank];
}

uint32_t tpx_num_entries(const tpx_plan_t* p, int side, uint32_t rank) {
  if (!p || (side != 0 && side != 1) || rank >= p->side[side].ranks.size()) return 0;
  return uint32_t(p->side[side].ranks[rank].size());
}

tpx_status tpx_manifest(const tpx_plan_t* p, int side, uint32_t rank, uint32_t i, tpx_entry* out) {
  if (!p || !out || (side != 0 && side != 1) || rank >= p->side[side].ranks.size() ||
      i >= p->side[side].ranks[rank].size())
    return fail(TPX_ERR_INVALID_ARG, "tpx_manifest: bad argument");
  *out = p->side[side].ranks[rank][i];
  return TPX_OK;
}

const char* tpx_param_name(uint32_t name) { return param_name(name); }

tpx_status tpx_stats(const tpx_plan_t* p, tpx_stats_t* out) {
  if (!p || !out) return fail(TPX_ERR_INVALID_ARG, "tpx_stats: NULL argument");
  *out = p->stats;
  return TPX_OK;
}

uint64_t tpx_num_boxes(const tpx_plan_t* p) { return p ? p->boxes.size() : 0; }

tpx_status tpx_get_box(const tpx_plan_t* p, uint64_t i, tpx_box* out) {
  if (!p || !out || i >= p->boxes.size()) return fail(TPX_ERR_INVALID_ARG, "tpx_get_box: bad argument");
  *out = p->boxes[i];
  return TPX_OK;
}

uint64_t tpx_num_tiles(const tpx_plan_t* p) { return p ? p->n_tiles : 0; }

tpx_status tpx_get_tile(const tpx_plan_t* p, uint64_t i, tpx_tile* out) {
  if (!p || !out || i >= p->n_tiles) return fail(TPX_ERR_INVALID_ARG, "tpx_get_tile: bad argument");
  // the same search and arithmetic the kernel performs
  const uint32_t box = find_box(p->first_tile.data(), p->coarse.data(), uint32_t(p->flat.size()), uint32_t(i));
  *out = tile_of(p->flat[box], uint32_t(i) - p->flat[box].first_tile);
  return TPX_OK;
}

uint64_t tpx_num_segments(const tpx_plan_t* p) { return p ? p->segments.size() : 0; }

tpx_status tpx_get_segment(const tpx_plan_t* p, uint64_t i, tpx_segment* out) {
  if (!p || !out || i >= p->segments.size()) return fail(TPX_ERR_INVALID_ARG, "tpx_get_segment: bad argument");
  *out = p->segments[i];
  return TPX_OK;
}

tpx_status tpx_traffic(const tpx_plan_t* p, uint64_t* out) {
  if (!p || !out) return fail(TPX_ERR_INVALID_ARG, "tpx_traffic: NULL argument");
  const size_t ns = p->side[0].bytes.size(), nd = p->side[1].bytes.size();
  std::fill(out, out + ns * nd, uint64_t(0));
  for (const tpx_box& b : p->boxes) {
    if (b.kind == TPX_BOX_FILL) continue;
    const uint64_t n = box_bytes(b);
    for (uint32_t k = 0; k < b.n_dst; ++k) out[size_t(b.src_rank) * nd + b.dst_rank + size_t(k) * b.dst_rank_stride] += n;
  }
  return TPX_OK;
}

uint64_t tpx_workspace_bytes(const tpx_plan_t* p) { return p ? workspace_layout(*p).total : 0; }

tpx_status tpx_prepare(const tpx_plan_t* p, void* workspace, void* hip_stream) {
  if (!p || !workspace) return fail(TPX_ERR_INVALID_ARG, "tpx_prepare: NULL argument");
  if (reinterpret_cast<uintptr_t>(workspace) % 64) return fail(TPX_ERR_MISALIGNED, "tpx_prepare: workspace must be 64-byte aligned");
  if (p->n_tiles == 0) return TPX_OK;
  try {
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    const auto it = g_ws_plan.find(workspace);
    if (it != g_ws_plan.end()) {
      if (it->second == p->id) return TPX_OK;
      g_ws_plan.erase(it);  // whatever happens next, the old plan's tables are no longer to be trusted there
    }
    if (tpx_status st = hip_upload_tables(workspace, *p, hip_stream)) return st;
    if (g_ws_plan.size() >= kMaxTrackedWorkspaces) g_ws_plan.clear();
    g_ws_plan.emplace(workspace, p->id);
  } catch (const std::bad_alloc&) {
    return fail(TPX_ERR_OOM, "tpx_prepare: out of host memory");
  }
  return TPX_OK;
}

static tpx_status check_rank_buffers(const tpx_plan_t* p, const void* const* src_bufs, void* const* dst_bufs, const char* who) {
  const std::string w(who);
  const uint32_t ns = uint32_t(p->side[0].bytes.size()), nd = uint32_t(p->side[1].bytes.size());
  for (uint32_t r = 0; r < ns; ++r) {
    if (!src_bufs[r] && p->side[0].alive[r] && p->side[0].bytes[r])
      return fail(TPX_ERR_INVALID_ARG, w + ": NULL source buffer for a live rank");
    if (reinterpret_cast<uintptr_t>(src_bufs[r]) % 16) return fail(TPX_ERR_MISALIGNED, w + ": source buffer not 16-byte aligned");
  }
  for (uint32_t r = 0; r < nd; ++r) {
    if (!dst_bufs[r] && p->side[1].alive[r] && p->side[1].bytes[r])
      return fail(TPX_ERR_INVALID_ARG, w + ": NULL destination buffer for a rank that is to be built");
    if (reinterpret_cast<uintptr_t>(dst_bufs[r]) % 16) return fail(TPX_ERR_MISALIGNED, w + ": destination buffer not 16-byte aligned");
  }
  return TPX_OK;
}

tpx_status tpx_execute(const tpx_plan_t* p, const void* const* src_bufs, void* const* dst_bufs, void* workspace,
                       void* hip_stream) {
  if (!p || !src_bufs || !dst_bufs || !workspace) return fail(TPX_ERR_INVALID_ARG, "tpx_execute: NULL argument");
  if (tpx_status st = check_rank_buffers(p, src_bufs, dst_bufs, "tpx_execute")) return st;
  if (p->n_tiles == 0) return TPX_OK;
  if (tpx_status st = tpx_prepare(p, workspace, hip_stream)) return st;
  return hip_launch_tiles(workspace, *p, src_bufs, uint32_t(p->side[0].bytes.size()), dst_bufs,
                          uint32_t(p->side[1].bytes.size()), tuning().variant, hip_stream);
}

tpx_status tpx_execute_static(const tpx_plan_t* p, const void* const* src_bufs, void* const* dst_bufs, void* hip_stream) {
  if (!p || !src_bufs || !dst_bufs) return fail(TPX_ERR_INVALID_ARG, "tpx_execute_static: NULL argument");
  if (tpx_status st = check_rank_buffers(p, src_bufs, dst_bufs, "tpx_execute_static")) return st;
  return hip_execute_static(*p, src_bufs, uint32_t(p->side[0].bytes.size()), dst_bufs, uint32_t(p->side[1].bytes.size()),
                            tuning().variant, hip_stream);
}

tpx_status tpx_workspace_check(const tpx_plan_t* p, const void* workspace, void* hip_stream) {
  if (!p || !workspace) return fail(TPX_ERR_INVALID_ARG, "tpx_workspace_check: NULL argument");
  if (p->n_tiles == 0) return TPX_OK;  // nothing is ever uploaded for an empty plan
  WorkspaceHeader h{};
  if (tpx_status st = hip_read_header(workspace, hip_stream, &h)) return st;
  if (h.plan_id != p->id || h.n_boxes != p->flat.size() || h.n_tiles != p->n_tiles || h.n_segments != p->segments.size()) {
    tpx_workspace_forget(workspace);
    return fail(TPX_ERR_STALE_WORKSPACE, "the workspace does not hold this plan's tables");
  }
  return TPX_OK;
}

void tpx_workspace_forget(const void* workspace) {
  std::lock_guard<std::mutex> lock(g_ws_mutex);
  if (workspace) g_ws_plan.erase(workspace);
  else g_ws_plan.clear();
}

void tpx_free(tpx_plan_t* p) { delete p; }

const char* tpx_last_error(void) { return last_error_cstr(); }

tpx_status tpx_set_option(const char* key, uint64_t value) {
  if (!key) return fail(TPX_ERR_INVALID_ARG, "tpx_set_option: NULL key");
  if (!std::strcmp(key, "variant")) {
    if (value == 0) { tuning().variant = 0; return TPX_OK; }
    if (value > 95 || (value & 7) < 2 || (value & 7) > 4 || (((value >> 3) & 1) != ((value >> 4) & 1)))
      return fail(TPX_ERR_INVALID_ARG, "variant out of range");
    tuning().variant = value;
    return TPX_OK;
  }
  if (!std::strcmp(key, "chunk")) {
    if (value > 4096) return fail(TPX_ERR_INVALID_ARG, "chunk must be in [0, 4096]");
    tuning().chunk = value;
    return TPX_OK;
  }
  if (!std::strcmp(key, "occupancy")) {
    if (value > 16) return fail(TPX_ERR_INVALID_ARG, "occupancy must be in [0, 16]");
    tuning().occupancy = value;
    return TPX_OK;
  }
  if (!std::strcmp(key, "streams")) {
    if (value < 1 || value > 1024) return fail(TPX_ERR_INVALID_ARG, "streams must be in [1, 1024]");
    tuning().streams = value;
    return TPX_OK;
  }
  return fail(TPX_ERR_INVALID_ARG, std::string("unknown option ") + key);
}

tpx_status tpx_probe_read(const void* src, uint64_t nbytes, void* sink, void* hip_stream) {
  if (!src || !sink) return fail(TPX_ERR_INVALID_ARG, "tpx_probe_read: NULL argument");
  if (nbytes % 16) return fail(TPX_ERR_INVALID_ARG, "tpx_probe_read: size must be a multiple of 16");
  if (reinterpret_cast<uintptr_t>(src) % 16 || reinterpret_cast<uintptr_t>(sink) % 16)
    return fail(TPX_ERR_MISALIGNED, "tpx_probe_read: pointers must be 16-byte aligned");
  return hip_probe_read(src, nbytes, sink, hip_stream);
}

tpx_status tpx_probe_fill(void* dst, uint64_t nbytes, uint32_t value, void* hip_stream) {
  if (!dst) return fail(TPX_ERR_INVALID_ARG, "tpx_probe_fill: NULL argument");
  if (nbytes % 16) return fail(TPX_ERR_INVALID_ARG, "tpx_probe_fill: size must be a multiple of 16");
  if (reinterpret_cast<uintptr_t>(dst) % 16) return fail(TPX_ERR_MISALIGNED, "tpx_probe_fill: the pointer must be 16-byte aligned");
  return hip_probe_fill(dst, nbytes, value, hip_stream);
}

tpx_status tpx_probe_copy(void* dst, const void* src, uint64_t nbytes, void* hip_stream) {
  if (!dst || !src) return fail(TPX_ERR_INVALID_ARG, "tpx_probe_copy: NULL argument");
  if (nbytes % 16) return fail(TPX_ERR_INVALID_ARG, "tpx_probe_copy: size must be a multiple of 16");
  if (reinterpret_cast<uintptr_t>(dst) % 16 || reinterpret_cast<uintptr_t>(src) % 16)
    return fail(TPX_ERR_MISALIGNED, "tpx_probe_copy: pointers must be 16-byte aligned");
  return hip_probe_copy(dst, src, nbytes, hip_stream);
}

}  // extern "C"

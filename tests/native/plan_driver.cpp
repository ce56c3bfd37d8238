// Drives the host side of libtpx through its C ABI under sanitizers: plans the benchmark workloads and a set
// of awkward ones, walks every box and a dense sample of tiles, checks that every tile stays inside the
// buffers the plan itself declares, and pokes the error paths.  Exit status 0 = clean.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "tpx.h"

static int failures = 0;
#define CHECK(c) do { if (!(c)) { std::printf("CHECK failed line %d: %s (%s)\n", __LINE__, #c, tpx_last_error()); ++failures; } } while (0)

static void walk(tpx_plan_t* p, uint64_t stride) {
  tpx_stats_t st;
  CHECK(tpx_stats(p, &st) == TPX_OK);
  CHECK(st.n_boxes == tpx_num_boxes(p) && st.n_tiles == tpx_num_tiles(p));
  uint64_t written = 0;
  for (uint64_t i = 0; i < tpx_num_boxes(p); ++i) {
    tpx_box b;
    CHECK(tpx_get_box(p, i, &b) == TPX_OK);
    uint64_t n = b.run_bytes;
    for (uint32_t k = 0; k < b.ndim; ++k) n *= b.extent[k];
    written += n * b.n_dst;
  }
  CHECK(written == st.bytes_written);
  for (uint64_t i = 0; i < tpx_num_tiles(p); i += stride) {
    tpx_tile t;
    CHECK(tpx_get_tile(p, i, &t) == TPX_OK);
    const uint64_t unit = 1ull << t.unit_log2;
    CHECK(t.nrows && t.run_units && t.n_dst);
    const uint64_t dlast = t.dst_off + (t.nrows - 1ull) * t.dst_pitch + (t.run_units - 1ull) * t.dst_step + unit;
    for (uint32_t c = 0; c < t.n_dst; ++c) CHECK(dlast <= tpx_buffer_bytes(p, TPX_SIDE_DST, t.dst_rank + c * t.dst_rank_stride));
    if (t.kind == TPX_TILE_PACK) {
      uint64_t first = 0;
      for (uint32_t g = 0; g < t.n_seg; ++g) {
        tpx_segment sg;
        CHECK(tpx_get_segment(p, t.seg_first + g, &sg) == TPX_OK);
        CHECK(sg.src_pitch == first && sg.units);
        first += sg.units;
        CHECK(sg.src_off + sg.units * 16ull <= tpx_buffer_bytes(p, TPX_SIDE_SRC, sg.src_rank));
        for (uint32_t c = 0; c < t.n_dst; ++c) CHECK(sg.dst_off + sg.units * 16ull <= tpx_buffer_bytes(p, TPX_SIDE_DST, t.dst_rank + c * t.dst_rank_stride));
      }
      CHECK(first == t.run_units);
    } else if (t.kind == TPX_TILE_MERGE) {
      for (uint32_t g = 0; g < t.n_seg; ++g) {
        tpx_segment sg;
        CHECK(tpx_get_segment(p, t.seg_first + g, &sg) == TPX_OK);
        CHECK(sg.src_off + (t.src_off + t.nrows - 1ull) * sg.src_pitch + uint64_t(t.seg_units) * unit <= tpx_buffer_bytes(p, TPX_SIDE_SRC, sg.src_rank));
      }
    } else if (t.kind != TPX_TILE_FILL) {
      CHECK(t.src_off + (t.nrows - 1ull) * t.src_pitch + (t.run_units - 1ull) * t.src_step + unit <= tpx_buffer_bytes(p, TPX_SIDE_SRC, t.src_rank));
    }
  }
  tpx_tile t;
  CHECK(tpx_get_tile(p, tpx_num_tiles(p), &t) == TPX_ERR_INVALID_ARG);
  for (int side = 0; side < 2; ++side)
    for (uint32_t r = 0; r < tpx_num_buffers(p, side); ++r) {
      tpx_entry e;
      for (uint32_t i = 0; i < tpx_num_entries(p, side, r); ++i) CHECK(tpx_manifest(p, side, r, i, &e) == TPX_OK && e.offset + e.nbytes <= tpx_buffer_bytes(p, side, r));
      CHECK(tpx_manifest(p, side, r, tpx_num_entries(p, side, r), &e) == TPX_ERR_INVALID_ARG);
    }
  CHECK(tpx_workspace_bytes(p) >= 256);
}

static tpx_model model(uint32_t L, uint32_t h, uint32_t a, uint32_t f, uint32_t v, uint32_t div, int kinds, uint32_t flags = 0) {
  tpx_model m{};
  m.n_layers = L; m.hidden = h; m.n_heads = a; m.ffn = f; m.vocab_true = v; m.max_pos = 1024; m.vocab_divisor = div;
  m.n_state_kinds = uint32_t(kinds);
  const uint8_t eb4[4] = {2, 4, 4, 4}, eb3[4] = {4, 4, 4, 0};
  std::memcpy(m.state_elem_bytes, kinds == 4 ? eb4 : eb3, 4);
  m.flags = flags;
  return m;
}

static tpx_parallel par(uint32_t T, uint32_t P, uint32_t D, const uint32_t* stages = nullptr, uint32_t qkv = 0, uint32_t tr = 0, const uint8_t* alive = nullptr) {
  tpx_parallel p{};
  p.T = T; p.P = P; p.D = D; p.stage_first_layer = stages; p.qkv_layout = qkv; p.w_transposed = tr; p.rank_alive = alive;
  return p;
}

static void plan_and_walk(const tpx_model& m, const tpx_parallel& a, const tpx_parallel& b, uint64_t stride,
                          const tpx_plan_opts* opts = nullptr) {
  tpx_plan_t* p = nullptr;
  CHECK(tpx_plan(&m, &a, &b, opts, &p) == TPX_OK);
  if (p) { walk(p, stride); tpx_free(p); }
}

int main() {
  const uint32_t uneven[5] = {0, 7, 16, 25, 32};
  plan_and_walk(model(2, 256, 4, 1024, 1024, 0, 3), par(2, 1, 1), par(4, 2, 1), 1);
  plan_and_walk(model(24, 2048, 16, 8192, 50304, 0, 4), par(4, 2, 1), par(2, 4, 1), 7);
  plan_and_walk(model(32, 2560, 32, 10240, 50304, 0, 4), par(4, 4, 2), par(2, 4, 1, uneven), 13);
  plan_and_walk(model(32, 4096, 32, 16384, 50304, 0, 4), par(8, 1, 1), par(1, 8, 1), 29);
  plan_and_walk(model(24, 3072, 24, 12288, 50257, 128, 4), par(3, 1, 1), par(4, 1, 1), 11);
  plan_and_walk(model(24, 2048, 16, 8192, 50304, 0, 4), par(4, 2, 1), par(4, 2, 4), 17);
  plan_and_walk(model(4, 24, 12, 48, 36, 0, 4, TPX_MODEL_TIED_HEAD), par(2, 2, 2), par(3, 4, 1, nullptr, 1, 1), 1);
  plan_and_walk(model(4, 24, 12, 48, 50, 4, 3), par(4, 1, 1, nullptr, 1, 1), par(3, 2, 3), 1);
  plan_and_walk(model(8, 64, 8, 128, 64, 0, 4), par(8, 4, 4), par(4, 8, 4), 1);
  {  // state kinds cut over the replicas, odd replica counts, with and without share_reads
    tpx_parallel a = par(2, 2, 3), b = par(4, 1, 5, nullptr, 1, 1), c = par(1, 2, 7);
    a.shard_kinds = 14; b.shard_kinds = 6; c.shard_kinds = 15;
    plan_and_walk(model(4, 24, 12, 48, 36, 0, 4), a, b, 1);
    plan_and_walk(model(4, 24, 12, 48, 36, 0, 4), b, c, 1);
    const tpx_plan_opts shared{0, 0, 1};
    plan_and_walk(model(4, 24, 12, 48, 36, 0, 4), c, a, 1, &shared);
    plan_and_walk(model(24, 2048, 16, 8192, 50304, 0, 4), par(4, 2, 2), par(4, 2, 8), 19, &shared);
    tpx_parallel bad = par(2, 1, 2);
    bad.shard_kinds = 16;
    tpx_plan_t* p = nullptr;
    CHECK(tpx_plan(&(const tpx_model&)model(4, 24, 12, 48, 36, 0, 4), &bad, &a, nullptr, &p) == TPX_ERR_INVALID_ARG);
    const tpx_plan_opts odd_tile{5000, 0, 0}, wide{0, 129, 0}, twice{0, 0, 2};
    for (const tpx_plan_opts* o : {&odd_tile, &wide, &twice})
      CHECK(tpx_plan(&(const tpx_model&)model(4, 24, 12, 48, 36, 0, 4), &a, &b, o, &p) == TPX_ERR_INVALID_ARG);
    CHECK(tpx_set_option("tile_bytes", 4096) == TPX_ERR_INVALID_ARG);   // a plan option, not a process-wide knob
  }
  const uint8_t alive[8] = {0, 0, 1, 1, 1, 1, 0, 0};
  plan_and_walk(model(4, 24, 12, 48, 36, 0, 4), par(2, 2, 2, nullptr, 0, 0, alive), par(2, 1, 1), 1);
  for (uint64_t tb : {4096ull, 65536ull, 4194304ull}) {
    const tpx_plan_opts o{tb, 3, 0};
    plan_and_walk(model(2, 256, 4, 1024, 1024, 0, 3), par(2, 1, 1), par(4, 2, 1, nullptr, 1, 1), 1, &o);
  }
  // dataset plans
  {
    const uint64_t cur[6] = {128 * 65000ull, 128 * 65000ull, 128 * 65000ull, 128 * 65000ull, 128 * 65000ull, 128 * 65000ull};
    uint64_t out[4];
    tpx_plan_t* p = nullptr;
    CHECK(tpx_plan_dataset(100000000ull, 768, 8, 6, 4, cur, out, nullptr, &p) == TPX_OK);
    if (p) { CHECK(out[0] == 192 * 65000ull); walk(p, 3); tpx_free(p); }
    const uint64_t zero[3] = {0, 0, 0};
    CHECK(tpx_plan_dataset(0, 12, 8, 3, 2, zero, out, nullptr, &p) == TPX_OK);
    if (p) { CHECK(tpx_num_tiles(p) == 0); tpx_free(p); }
    const uint64_t bad[3] = {1, 0, 0};
    CHECK(tpx_plan_dataset(100, 12, 8, 3, 2, bad, out, nullptr, &p) == TPX_ERR_CURSOR);
    CHECK(tpx_plan_dataset(100, 13, 8, 3, 2, zero, out, nullptr, &p) == TPX_ERR_INDIVISIBLE);
  }
  // explicit collection: a flat optimizer state in uneven chunks, 3 -> 4 ranks, plus errors
  {
    auto entry = [](uint64_t n, uint64_t lo, uint64_t hi) {
      tpx_entry e{};
      e.tensor_id = 7; e.kind = 1; e.elem_bytes = 4; e.ndim = 1; e.full_shape[0] = n; e.lo[0] = lo; e.hi[0] = hi; e.perm[0] = 0;
      return e;
    };
    const uint64_t n = 100003;
    std::vector<tpx_entry> s = {entry(n, 0, 33334), entry(n, 33334, 66668), entry(n, 66668, n)};
    std::vector<tpx_entry> d = {entry(n, 0, 25000), entry(n, 25000, 50001), entry(n, 50001, 75002), entry(n, 75002, n)};
    const uint32_t ones[4] = {1, 1, 1, 1};
    const tpx_entry* sp[3] = {&s[0], &s[1], &s[2]};
    const tpx_entry* dp[4] = {&d[0], &d[1], &d[2], &d[3]};
    tpx_ptc a{3, ones, sp, nullptr, nullptr}, b{4, ones, dp, nullptr, nullptr};
    tpx_plan_t* p = nullptr;
    CHECK(tpx_plan_ptc(&a, &b, nullptr, &p) == TPX_OK);
    if (p) { walk(p, 1); tpx_free(p); }
    tpx_ptc half{2, ones, sp, nullptr, nullptr};
    CHECK(tpx_plan_ptc(&half, &b, nullptr, &p) == TPX_ERR_INVALID_ARG);
    const uint8_t dead[3] = {1, 0, 1};
    tpx_ptc lost{3, ones, sp, nullptr, dead};
    CHECK(tpx_plan_ptc(&lost, &b, nullptr, &p) == TPX_ERR_UNRECOVERABLE);
    // a range query over the three chunks, and offsets left to the library
    const tpx_query qs[2] = {{7, 1, {30000, 0, 0, 0}, {70000, 0, 0, 0}}, {7, 1, {5, 0, 0, 0}, {6, 0, 0, 0}}};
    CHECK(tpx_plan_query(&a, 2, qs, nullptr, &p) == TPX_OK);
    if (p) {
      tpx_entry e{};
      CHECK(tpx_num_buffers(p, TPX_SIDE_DST) == 1 && tpx_num_entries(p, TPX_SIDE_DST, 0) == 2);
      CHECK(tpx_manifest(p, TPX_SIDE_DST, 0, 1, &e) == TPX_OK && e.offset == 160000 && e.nbytes == 4);
      CHECK(tpx_buffer_bytes(p, TPX_SIDE_DST, 0) == 160256);
      walk(p, 1);
      tpx_free(p);
      p = nullptr;
    }
    const tpx_query nope{8, 1, {0, 0, 0, 0}, {1, 0, 0, 0}}, beyond{7, 1, {0, 0, 0, 0}, {n + 1, 0, 0, 0}};
    CHECK(tpx_plan_query(&a, 1, &nope, nullptr, &p) == TPX_ERR_INVALID_ARG);
    CHECK(tpx_plan_query(&a, 1, &beyond, nullptr, &p) == TPX_ERR_INVALID_ARG);
    for (tpx_entry& e : d) e.offset = TPX_OFFSET_AUTO;
    CHECK(tpx_plan_ptc(&a, &b, nullptr, &p) == TPX_OK);
    if (p) { walk(p, 1); tpx_free(p); p = nullptr; }
    s[1].perm[0] = 3;
    CHECK(tpx_plan_ptc(&a, &b, nullptr, &p) == TPX_ERR_INVALID_ARG);
  }
  // error paths of the model planner
  {
    tpx_plan_t* p = nullptr;
    tpx_model m = model(4, 24, 12, 48, 36, 0, 4);
    tpx_parallel one = par(1, 1, 1), five = par(5, 1, 1), three = par(1, 3, 1), big = par(8, 8, 4);
    CHECK(tpx_plan(&m, &five, &one, nullptr, &p) == TPX_ERR_INDIVISIBLE);
    CHECK(tpx_plan(&m, &three, &one, nullptr, &p) == TPX_ERR_INDIVISIBLE);
    CHECK(tpx_plan(&m, &big, &one, nullptr, &p) == TPX_ERR_INVALID_ARG);
    const uint32_t bad[3] = {0, 3, 2};
    tpx_parallel bs = par(1, 2, 1, bad);
    CHECK(tpx_plan(&m, &bs, &one, nullptr, &p) == TPX_ERR_BAD_STAGE_MAP);
    CHECK(tpx_plan(nullptr, &one, &one, nullptr, &p) == TPX_ERR_INVALID_ARG);
    CHECK(p == nullptr);
    // execute without a GPU: argument checks first, then the stub reports the missing device
    CHECK(tpx_plan(&m, &one, &one, nullptr, &p) == TPX_OK);
    void* bufs[1] = {reinterpret_cast<void*>(0x1000)};
    CHECK(tpx_execute(p, bufs, bufs, nullptr, nullptr) == TPX_ERR_INVALID_ARG);
    CHECK(tpx_execute(p, bufs, bufs, reinterpret_cast<void*>(0x1000), nullptr) == TPX_ERR_HIP);
    CHECK(tpx_execute(p, bufs, bufs, reinterpret_cast<void*>(0x1008), nullptr) == TPX_ERR_MISALIGNED);
    void* odd[1] = {reinterpret_cast<void*>(0x1004)};
    CHECK(tpx_execute(p, odd, bufs, reinterpret_cast<void*>(0x1000), nullptr) == TPX_ERR_MISALIGNED);
    CHECK(tpx_execute_static(p, odd, bufs, nullptr) == TPX_ERR_MISALIGNED);
    CHECK(tpx_execute_static(p, bufs, bufs, nullptr) == TPX_ERR_HIP);
    tpx_workspace_forget(reinterpret_cast<void*>(0x1000));
    tpx_workspace_forget(nullptr);
    tpx_free(p);
    tpx_free(nullptr);
  }
  std::printf(failures ? "FAILED: %d checks\n" : "all checks passed%.0d\n", failures);
  return failures ? 1 : 0;
}

// Stand-alone use of the C ABI (no Python, no PyTorch): plan a small reshard, run it with buffers from
// hipMalloc, and check every destination tensor element against a value function of (tensor, kind,
// position in the full tensor).  Build: see paper_2312_05181_amd/build.py (target tpx_selftest).
// Exit status 0 = every byte as expected.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "tpx.h"

#define HIP_OK(x)                                                                      \
  do {                                                                                 \
    hipError_t e_ = (x);                                                               \
    if (e_ != hipSuccess) { std::fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 2; } \
  } while (0)
#define TPX_OK_OR_DIE(x)                                                               \
  do {                                                                                 \
    tpx_status s_ = (x);                                                               \
    if (s_ != TPX_OK) { std::fprintf(stderr, "%s: status %d: %s\n", #x, int(s_), tpx_last_error()); return 3; } \
  } while (0)

// value of element `index` (row-major position in the full tensor) of state tensor (tensor, kind)
static uint64_t value_of(uint32_t tensor, uint32_t kind, uint64_t index) {
  uint64_t x = (uint64_t(tensor) << 40) ^ (uint64_t(kind) << 36) ^ index;
  x ^= x >> 31; x *= 0x7fb5d329728ea185ull; x ^= x >> 27; x *= 0x81dadef4bc2dd44dull; x ^= x >> 33;
  return x;
}

// calls fn(byte offset in the rank buffer, row-major index in the full tensor) for every element of e
template <typename Fn>
static void for_each_element(const tpx_entry& e, Fn fn) {
  uint64_t ext[4] = {1, 1, 1, 1}, idx[4] = {0, 0, 0, 0}, full_stride[4] = {1, 1, 1, 1};
  for (int k = int(e.ndim) - 2; k >= 0; --k) full_stride[k] = full_stride[k + 1] * e.full_shape[k + 1];
  for (uint32_t i = 0; i < e.ndim; ++i) ext[i] = e.hi[e.perm[i]] - e.lo[e.perm[i]];   // stored order
  uint64_t off = e.offset;
  for (;;) {
    uint64_t lin = 0;
    for (uint32_t i = 0; i < e.ndim; ++i) lin += (e.lo[e.perm[i]] + idx[i]) * full_stride[e.perm[i]];
    fn(off, lin);
    off += e.elem_bytes;
    int i = int(e.ndim) - 1;
    for (; i >= 0; --i) {
      if (++idx[i] < ext[i]) break;
      idx[i] = 0;
    }
    if (i < 0) break;
  }
}

int main() {
  tpx_model m{};
  m.n_layers = 2; m.hidden = 240; m.n_heads = 12; m.ffn = 960; m.vocab_true = 1000; m.max_pos = 64;  // divisible by 3 and 4
  m.vocab_divisor = 8;                      // 1000 rows padded to 1008 (T = 3) and 1024 (T = 4): zero rows appear
  m.n_state_kinds = 3;
  m.state_elem_bytes[0] = 2; m.state_elem_bytes[1] = 4; m.state_elem_bytes[2] = 8;
  tpx_parallel src{}, dst{};
  src.T = 3; src.P = 1; src.D = 2; src.shard_kinds = 4;           // the 8-byte kind is cut over the 2 replicas
  dst.T = 4; dst.P = 2; dst.D = 1; dst.qkv_layout = 1; dst.w_transposed = 1;
  tpx_plan_t* plan = nullptr;
  TPX_OK_OR_DIE(tpx_plan(&m, &src, &dst, nullptr, &plan));
  tpx_stats_t st{};
  TPX_OK_OR_DIE(tpx_stats(plan, &st));
  std::printf("plan: %llu moves, %llu tiles, %llu bytes read, %llu written, %llu zero-filled\n", (unsigned long long)st.n_boxes,
              (unsigned long long)st.n_tiles, (unsigned long long)st.bytes_read, (unsigned long long)st.bytes_written,
              (unsigned long long)st.bytes_fill);

  const uint32_t ns = tpx_num_buffers(plan, TPX_SIDE_SRC), nd = tpx_num_buffers(plan, TPX_SIDE_DST);
  std::vector<void*> sbuf(ns, nullptr), dbuf(nd, nullptr);
  uint64_t old_vocab_rows = 0;
  for (uint32_t r = 0; r < ns; ++r) {
    const uint64_t n = tpx_buffer_bytes(plan, TPX_SIDE_SRC, r);
    std::vector<uint8_t> host(n, 0x5a);
    for (uint32_t i = 0; i < tpx_num_entries(plan, TPX_SIDE_SRC, r); ++i) {
      tpx_entry e{};
      TPX_OK_OR_DIE(tpx_manifest(plan, TPX_SIDE_SRC, r, i, &e));
      if (e.tensor_id == 0) old_vocab_rows = e.full_shape[0];
      for_each_element(e, [&](uint64_t off, uint64_t lin) {
        const uint64_t v = value_of(e.tensor_id, e.kind, lin);
        std::memcpy(host.data() + off, &v, e.elem_bytes);       // little endian: the low bytes
      });
    }
    HIP_OK(hipMalloc(&sbuf[r], n ? n : 16));
    HIP_OK(hipMemcpy(sbuf[r], host.data(), n, hipMemcpyHostToDevice));
  }
  for (uint32_t r = 0; r < nd; ++r) {
    const uint64_t n = tpx_buffer_bytes(plan, TPX_SIDE_DST, r);
    HIP_OK(hipMalloc(&dbuf[r], n ? n : 16));
    HIP_OK(hipMemset(dbuf[r], 0xa5, n));
  }
  void* ws = nullptr;
  HIP_OK(hipMalloc(&ws, tpx_workspace_bytes(plan)));
  hipStream_t stream;
  HIP_OK(hipStreamCreate(&stream));
  TPX_OK_OR_DIE(tpx_execute(plan, sbuf.data(), dbuf.data(), ws, stream));
  TPX_OK_OR_DIE(tpx_workspace_check(plan, ws, stream));           // also waits for the stream

  uint64_t bad = 0, checked = 0;
  for (uint32_t r = 0; r < nd; ++r) {
    const uint64_t n = tpx_buffer_bytes(plan, TPX_SIDE_DST, r);
    std::vector<uint8_t> host(n), covered(n, 0);
    HIP_OK(hipMemcpy(host.data(), dbuf[r], n, hipMemcpyDeviceToHost));
    for (uint32_t i = 0; i < tpx_num_entries(plan, TPX_SIDE_DST, r); ++i) {
      tpx_entry e{};
      TPX_OK_OR_DIE(tpx_manifest(plan, TPX_SIDE_DST, r, i, &e));
      const uint64_t row_elems = e.ndim > 1 ? e.full_shape[1] : 1;
      for_each_element(e, [&](uint64_t off, uint64_t lin) {
        // rows of the word embeddings beyond the old padded vocabulary are new padding: zero
        uint64_t v = (e.tensor_id == 0 && lin / row_elems >= old_vocab_rows) ? 0 : value_of(e.tensor_id, e.kind, lin);
        bad += std::memcmp(host.data() + off, &v, e.elem_bytes) != 0;
        std::memset(covered.data() + off, 1, e.elem_bytes);
        ++checked;
      });
    }
    for (uint64_t b = 0; b < n; ++b) bad += !covered[b] && host[b] != 0xa5;   // gaps stay untouched
  }
  std::printf("%llu elements checked, %llu wrong\n", (unsigned long long)checked, (unsigned long long)bad);
  tpx_free(plan);
  for (void* p : sbuf) HIP_OK(hipFree(p));
  for (void* p : dbuf) HIP_OK(hipFree(p));
  HIP_OK(hipFree(ws));
  HIP_OK(hipStreamDestroy(stream));
  return bad ? 1 : 0;
}

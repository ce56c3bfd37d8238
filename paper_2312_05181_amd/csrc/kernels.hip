// HIP executor for gfx950: applies a whole reconfiguration plan (paper section 5.1, step 4: the split,
// re-partition and merge operations of section 4.2) with one kernel launch.
//
// The plan reaches the GPU as a small table of flat boxes with the prefix sums of their tile counts;
// a workgroup finds the box that owns its tile by a short search and derives the tile from the box's
// tiling parameters.  A tile is a bounded piece (at most `tile_bytes`) of one move, so every workgroup has
// about the same amount of work no matter how uneven the moves are.  Nothing is contracted, so there is
// no MFMA work: the kernel is a gather/scatter of 16-byte vectors and is bound by HBM bandwidth.  A
// workgroup loads its whole tile (threads x loads in flight x 16 bytes), then stores it.  LDS holds only
// the segment table of merge tiles and the staging array of transposing tiles.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "tpx_internal.hpp"

// The plan tables of tpx_execute_static: one array per GPU the code object is loaded on, held until the
// process ends.  In host code this name is only a handle for hipGetSymbolAddress; the device address is
// looked up once per device (hip_execute_static) and that pointer is what copies and kernels get.  Host code
// refers to it below, which is what makes the compiler keep it in the code object under a visible name.
static __device__ __align__(256) uint8_t scratch[TPX_STATIC_WORKSPACE_BYTES];

namespace {

typedef unsigned int v4u __attribute__((ext_vector_type(4)));

struct PtrTable {
  const uint8_t* src[TPX_MAX_RANKS];
  uint8_t* dst[TPX_MAX_RANKS];
};

template <typename V, bool NT>
__device__ __forceinline__ V ld(const V* p) {
  if constexpr (NT) return __builtin_nontemporal_load(p);
  else return *p;
}
template <typename V, bool NT>
__device__ __forceinline__ void st(V* p, V v) {
  if constexpr (NT) __builtin_nontemporal_store(v, p);
  else *p = v;
}

template <typename V>
__device__ __forceinline__ V zero_of() {
  V z;
  __builtin_memset(&z, 0, sizeof(V));
  return z;
}

// Destinations of a tile: buffer dst_rank + c * stride for c < n (data-parallel replicas), same offset in each.
struct DstSet {
  uint8_t* const* table;  // rank -> base pointer
  uint64_t off;
  uint32_t rank, stride, n;
  __device__ __forceinline__ uint8_t* base(uint32_t c) const { return table[rank + c * stride] + off; }
};

// The common loop: unit idx (0 <= idx < total) is loaded from src_of(idx) and stored at byte offset
// dst_off_of(idx) of every destination.  Consecutive threads take consecutive units; every thread keeps U
// independent loads in flight before storing them; the ragged end is one more, predicated, block of U.
template <typename V, int kThreads, int U, bool NTL, bool NTS, bool FILL, bool MC, typename SrcOf, typename DstOffOf>
__device__ __forceinline__ void move_units(uint32_t total, const DstSet& ds, SrcOf src_of, DstOffOf dst_off_of) {
  const uint32_t n_dst = MC ? ds.n : 1;
  uint8_t* const d0 = ds.base(0);
  uint32_t i = threadIdx.x;
  for (; i + (U - 1) * kThreads < total; i += U * kThreads) {
    V r[U];
    uint64_t doff[U];
#pragma unroll
    for (int k = 0; k < U; ++k) {
      r[k] = FILL ? zero_of<V>() : ld<V, NTL>(src_of(i + k * kThreads));
      doff[k] = dst_off_of(i + k * kThreads);
    }
    for (uint32_t c = 0; c < n_dst; ++c) {
      uint8_t* d = MC ? ds.base(c) : d0;
#pragma unroll
      for (int k = 0; k < U; ++k) st<V, NTS>(reinterpret_cast<V*>(d + doff[k]), r[k]);
    }
  }
  if (i < total) {
    V r[U];
    uint64_t doff[U];
#pragma unroll
    for (int k = 0; k < U; ++k)
      if (i + k * kThreads < total) {
        r[k] = FILL ? zero_of<V>() : ld<V, NTL>(src_of(i + k * kThreads));
        doff[k] = dst_off_of(i + k * kThreads);
      }
    for (uint32_t c = 0; c < n_dst; ++c) {
      uint8_t* d = MC ? ds.base(c) : d0;
#pragma unroll
      for (int k = 0; k < U; ++k)
        if (i + k * kThreads < total) st<V, NTS>(reinterpret_cast<V*>(d + doff[k]), r[k]);
    }
  }
}

// Copy (or zero-fill) nrows rows of run_units units of type V; rows are contiguous on both sides, so
// accesses are coalesced along each row.  MC: every unit is stored to every destination of the set.
template <typename V, int kThreads, int U, bool NTL, bool NTS, bool FILL, bool MC>
__device__ __forceinline__ void move_rows(const uint8_t* __restrict__ s, const DstSet& ds, uint32_t run_units,
                                          uint32_t nrows, uint64_t sp, uint64_t dp) {
  const uint32_t total = run_units * nrows;
  if (nrows == 1) {
    move_units<V, kThreads, U, NTL, NTS, FILL, MC>(
        total, ds, [&](uint32_t idx) { return reinterpret_cast<const V*>(s) + idx; },
        [&](uint32_t idx) { return uint64_t(idx) * sizeof(V); });
  } else {
    move_units<V, kThreads, U, NTL, NTS, FILL, MC>(
        total, ds,
        [&](uint32_t idx) {
          const uint32_t row = idx / run_units;
          return reinterpret_cast<const V*>(s + row * sp + uint64_t(idx - row * run_units) * sizeof(V));
        },
        [&](uint32_t idx) {
          const uint32_t row = idx / run_units;
          return row * dp + uint64_t(idx - row * run_units) * sizeof(V);
        });
  }
}

template <int kThreads, int U, bool NTL, bool NTS, bool FILL, bool MC>
__device__ __forceinline__ void move_rows_any(uint32_t unit_log2, const uint8_t* s, const DstSet& ds, uint32_t run_units,
                                              uint32_t nrows, uint64_t sp, uint64_t dp) {
  switch (unit_log2) {
    case 4: move_rows<v4u, kThreads, U, NTL, NTS, FILL, MC>(s, ds, run_units, nrows, sp, dp); break;
    case 3: move_rows<uint64_t, kThreads, 2, false, false, FILL, MC>(s, ds, run_units, nrows, sp, dp); break;
    case 2: move_rows<uint32_t, kThreads, 2, false, false, FILL, MC>(s, ds, run_units, nrows, sp, dp); break;
    case 1: move_rows<uint16_t, kThreads, 2, false, false, FILL, MC>(s, ds, run_units, nrows, sp, dp); break;
    default: move_rows<uint8_t, kThreads, 2, false, false, FILL, MC>(s, ds, run_units, nrows, sp, dp); break;
  }
}

// Merge tile: whole destination rows of row_units 16-byte units are written contiguously; every row is the
// concatenation of n_seg column blocks, block g read from segment g.  The per-segment source row pointers (and, when
// the blocks differ in width, their first columns) are staged in LDS because lanes of one wave may read different
// segments.
struct SegLds {
  const uint8_t* base;  // first row of this tile in the segment's source
  uint64_t pitch;
};
using tpx::kMaxSegLds;
constexpr int kSegLdsBytes = int(kMaxSegLds * sizeof(SegLds) + (kMaxSegLds + 1) * sizeof(uint32_t) + 12);  // 1296

template <int kThreads, int U, bool NTL, bool NTS>
__device__ __forceinline__ void merge_tile(const tpx_tile& t, const tpx_segment* __restrict__ segs, const uint8_t* const* src_table,
                                           const DstSet& ds, SegLds* lseg) {
  const uint32_t row_units = t.run_units, seg_units = t.seg_units, n_seg = t.n_seg;
  const bool in_lds = n_seg <= kMaxSegLds;  // always so when the widths differ (seg_units == 0)
  uint32_t* lfirst = reinterpret_cast<uint32_t*>(lseg + kMaxSegLds);  // lfirst[g] = first column of segment g
  if (in_lds) {
    for (uint32_t g = threadIdx.x; g < n_seg; g += kThreads) {
      const tpx_segment sg = segs[t.seg_first + g];
      lseg[g].base = src_table[sg.src_rank] + sg.src_off + t.src_off * sg.src_pitch;  // t.src_off = first row
      lseg[g].pitch = sg.src_pitch;
      if (!seg_units) {
        uint32_t first = 0;
        for (uint32_t k = 0; k < g; ++k) first += segs[t.seg_first + k].units;
        lfirst[g] = first;
        if (g + 1 == n_seg) lfirst[n_seg] = first + sg.units;
      }
    }
    __syncthreads();
  }
  auto src_of = [&](uint32_t idx) -> const v4u* {
    const uint32_t row = idx / row_units;
    const uint32_t c = idx - row * row_units;
    uint32_t g, col;
    if (seg_units) {
      g = c / seg_units;
      col = c - g * seg_units;
    } else {  // a handful of segments: walk their first columns
      g = 0;
      while (c >= lfirst[g + 1]) ++g;
      col = c - lfirst[g];
    }
    if (in_lds) return reinterpret_cast<const v4u*>(lseg[g].base + row * lseg[g].pitch + uint64_t(col) * 16);
    const tpx_segment sg = segs[t.seg_first + g];
    return reinterpret_cast<const v4u*>(src_table[sg.src_rank] + sg.src_off + (t.src_off + row) * sg.src_pitch + uint64_t(col) * 16);
  };
  const uint32_t total = row_units * t.nrows;
  const bool dense = t.dst_pitch == uint64_t(row_units) * 16;  // rows adjacent in the destination
  auto dst_off = [&](uint32_t idx) -> uint64_t {
    if (dense) return uint64_t(idx) * 16;
    const uint32_t row = idx / row_units;
    return row * t.dst_pitch + uint64_t(idx - row * row_units) * 16;
  };
  if (ds.n > 1) move_units<v4u, kThreads, U, NTL, NTS, false, true>(total, ds, src_of, dst_off);
  else move_units<v4u, kThreads, U, NTL, NTS, false, false>(total, ds, src_of, dst_off);
}

// Pack tile: n_seg short contiguous moves into the same destination buffer(s), as one row of units.  Unit idx belongs to
// the segment whose first unit is the largest one <= idx (found by bisection in LDS: entries past n_seg hold a
// sentinel); source pointer and destination offset of every segment are staged in LDS like a merge tile's.
template <int kThreads, int U, bool NTL, bool NTS>
__device__ __forceinline__ void pack_tile(const tpx_tile& t, const tpx_segment* __restrict__ segs, const uint8_t* const* src_table,
                                          const DstSet& ds, SegLds* lseg) {
  uint32_t* lfirst = reinterpret_cast<uint32_t*>(lseg + kMaxSegLds);
  for (uint32_t g = threadIdx.x; g < kMaxSegLds; g += kThreads) {
    if (g < t.n_seg) {
      const tpx_segment sg = segs[t.seg_first + g];
      lseg[g].base = src_table[sg.src_rank] + sg.src_off;
      lseg[g].pitch = sg.dst_off;
      lfirst[g] = uint32_t(sg.src_pitch);  // first unit of the segment within the tile
    } else {
      lfirst[g] = 0xffffffffu;
    }
  }
  __syncthreads();
  auto seg_of = [&](uint32_t idx) -> uint32_t {
    uint32_t g = 0;
#pragma unroll
    for (uint32_t step = kMaxSegLds / 2; step; step >>= 1)
      if (lfirst[g + step] <= idx) g += step;
    return g;
  };
  auto src_of = [&](uint32_t idx) -> const v4u* {
    const uint32_t g = seg_of(idx);
    return reinterpret_cast<const v4u*>(lseg[g].base + uint64_t(idx - lfirst[g]) * 16);
  };
  auto dst_off = [&](uint32_t idx) -> uint64_t {
    const uint32_t g = seg_of(idx);
    return lseg[g].pitch + uint64_t(idx - lfirst[g]) * 16;
  };
  if (ds.n > 1) move_units<v4u, kThreads, U, NTL, NTS, false, true>(t.run_units, ds, src_of, dst_off);
  else move_units<v4u, kThreads, U, NTL, NTS, false, false>(t.run_units, ds, src_of, dst_off);
}

// Transposing tile: element (i, j) is contiguous in j on the source and in i on the destination.
// Square sub-tiles of TS x TS elements (at least 256 bytes a side) go through LDS: 16-byte global loads
// along j, element-wise LDS writes into the transposed position, 16-byte reads along i, 16-byte global
// stores.  Ragged or misaligned sub-tiles take the same route one element at a time.
// lds holds TS x (TS + 1) elements of type E, addressed [j][i].
template <typename E>
struct TransposeShape {
  static constexpr int VE = 16 / int(sizeof(E));                          // elements per 16-byte vector
  static constexpr int TS = sizeof(E) == 1 ? 128 : 256 / int(sizeof(E));  // 128, 128, 64, 32
  static constexpr int LD = TS + 1;
  static constexpr int kBytes = TS * LD * int(sizeof(E));
};

template <typename E, int kThreads, bool NTL, bool NTS>
__device__ __forceinline__ void transpose_tile(const uint8_t* __restrict__ s, uint8_t* __restrict__ d, uint32_t nJ,
                                               uint32_t nI, uint64_t sp, uint64_t dstep, void* lds_raw) {
  using Sh = TransposeShape<E>;
  constexpr int VE = Sh::VE, TS = Sh::TS, LD = Sh::LD;
  E* lds = reinterpret_cast<E*>(lds_raw);
  const bool aligned = reinterpret_cast<uintptr_t>(s) % 16 == 0 && sp % 16 == 0 &&
                       reinterpret_cast<uintptr_t>(d) % 16 == 0 && dstep % 16 == 0;
  for (uint32_t i0 = 0; i0 < nI; i0 += TS)
    for (uint32_t j0 = 0; j0 < nJ; j0 += TS) {
      const uint32_t ni = min(uint32_t(TS), nI - i0), nj = min(uint32_t(TS), nJ - j0);
      if (aligned && ni == TS && nj == TS) {
        for (uint32_t v = threadIdx.x; v < TS * TS / VE; v += kThreads) {
          const uint32_t i = v / (TS / VE), jv = v % (TS / VE);
          const v4u x = ld<v4u, NTL>(reinterpret_cast<const v4u*>(s + uint64_t(i0 + i) * sp + uint64_t(j0 + jv * VE) * sizeof(E)));
          E e[VE];
          __builtin_memcpy(e, &x, 16);
#pragma unroll
          for (int k = 0; k < VE; ++k) lds[(jv * VE + k) * LD + i] = e[k];
        }
        __syncthreads();
        for (uint32_t v = threadIdx.x; v < TS * TS / VE; v += kThreads) {
          const uint32_t j = v / (TS / VE), iv = v % (TS / VE);
          E e[VE];
#pragma unroll
          for (int k = 0; k < VE; ++k) e[k] = lds[j * LD + iv * VE + k];
          v4u x;
          __builtin_memcpy(&x, e, 16);
          st<v4u, NTS>(reinterpret_cast<v4u*>(d + uint64_t(j0 + j) * dstep + uint64_t(i0 + iv * VE) * sizeof(E)), x);
        }
      } else {
        for (uint32_t e = threadIdx.x; e < TS * TS; e += kThreads) {
          const uint32_t i = e / TS, jj = e % TS;
          if (i < ni && jj < nj) lds[jj * LD + i] = *reinterpret_cast<const E*>(s + uint64_t(i0 + i) * sp + uint64_t(j0 + jj) * sizeof(E));
        }
        __syncthreads();
        for (uint32_t e = threadIdx.x; e < TS * TS; e += kThreads) {
          const uint32_t jj = e / TS, i = e % TS;
          if (i < ni && jj < nj) *reinterpret_cast<E*>(d + uint64_t(i0 + i) * sizeof(E) + uint64_t(j0 + jj) * dstep) = lds[jj * LD + i];
        }
      }
      __syncthreads();
    }
}

// ---- one-shot transposing block ---------------------------------------------------------------------------
// A block of TI x TJ elements (tpx::kBlockBytes in all): element (i, j) sits at s + i*sp + j*sizeof(E) and goes to
// d + j*dstep + i*sizeof(E).  Like a copy tile it is moved in one shot: every thread issues all its 16-byte loads
// (the whole block is in flight), the block passes through LDS once, and every thread issues all its 16-byte
// stores.  The unit of the exchange is a micro-block of VE x VE elements (VE = 16 / sizeof(E)): a thread loads its
// VE row vectors (consecutive lanes take consecutive vectors of a row: coalesced), transposes them in registers
// (pure renaming for 4- and 8-byte elements, 16-bit packs for 2-byte ones) and writes VE column vectors to LDS,
// which is laid out like the destination block: TJ rows of TI elements, i.e. IB = TI / VE chunks of 16 bytes.
// Chunk c of row r is kept at position c ^ ((r / VE) & 7): the lanes of a write (same c, rows VE apart) and of a
// read (same r, consecutive c) then fall on different banks, with no padding.
template <typename E>
struct MicroBlock {
  static constexpr int VE = 16 / int(sizeof(E));
  // out[k] = (in[0] element k, in[1] element k, ..., in[VE-1] element k)
  static __device__ __forceinline__ void transpose(const v4u (&in)[VE], v4u (&out)[VE]) {
    if constexpr (sizeof(E) == 4) {
#pragma unroll
      for (int k = 0; k < 4; ++k) out[k] = v4u{in[0][k], in[1][k], in[2][k], in[3][k]};
    } else if constexpr (sizeof(E) == 8) {
      out[0] = v4u{in[0][0], in[0][1], in[1][0], in[1][1]};
      out[1] = v4u{in[0][2], in[0][3], in[1][2], in[1][3]};
    } else {
      static_assert(sizeof(E) == 2, "element size");
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        // halves k of dword k/2: low halves (bytes 0,1 of each source) for even k, high halves (bytes 2,3) for odd k
        const unsigned sel = (k & 1) ? 0x07060302u : 0x05040100u;
#pragma unroll
        for (int w = 0; w < 4; ++w) out[k][w] = __builtin_amdgcn_perm(in[2 * w + 1][k >> 1], in[2 * w][k >> 1], sel);
      }
    }
  }
};

template <typename E, int TI, int TJ, int kThreads, bool NTL, bool NTS>
__device__ __forceinline__ void transpose_block(const uint8_t* __restrict__ s, const DstSet& ds, uint64_t sp, uint64_t dstep,
                                                void* lds_raw) {
  constexpr int VE = MicroBlock<E>::VE;
  constexpr int IB = TI / VE, JB = TJ / VE;   // micro-blocks along i and j; IB is also the 16-byte chunks of an LDS row
  constexpr int PER = IB * JB / kThreads;     // micro-blocks per thread
  static_assert(TI * TJ * int(sizeof(E)) == int(tpx::kBlockBytes) && IB % 8 == 0 && (IB * JB) % kThreads == 0 && PER >= 1, "block shape");
  v4u* lds = reinterpret_cast<v4u*>(lds_raw);
  v4u r[PER][VE];
#pragma unroll
  for (int m = 0; m < PER; ++m) {
    const uint32_t mb = threadIdx.x + m * kThreads, jb = mb % JB, ib = mb / JB;
#pragma unroll
    for (int q = 0; q < VE; ++q)
      r[m][q] = ld<v4u, NTL>(reinterpret_cast<const v4u*>(s + uint64_t(ib * VE + q) * sp + jb * 16));
  }
#pragma unroll
  for (int m = 0; m < PER; ++m) {
    const uint32_t mb = threadIdx.x + m * kThreads, jb = mb % JB, ib = mb / JB;
    v4u c[VE];
    MicroBlock<E>::transpose(r[m], c);
#pragma unroll
    for (int k = 0; k < VE; ++k) lds[(jb * VE + k) * IB + (ib ^ (jb & 7))] = c[k];
  }
  __syncthreads();
  constexpr int NV = PER * VE;  // 16-byte vectors per thread
  v4u w[NV];
#pragma unroll
  for (int n = 0; n < NV; ++n) {
    const uint32_t q = threadIdx.x + n * kThreads, c = q % IB, row = q / IB;
    w[n] = lds[row * IB + (c ^ ((row / VE) & 7))];
  }
  for (uint32_t k = 0; k < ds.n; ++k) {
    uint8_t* d = ds.base(k);
#pragma unroll
    for (int n = 0; n < NV; ++n) {
      const uint32_t q = threadIdx.x + n * kThreads, c = q % IB, row = q / IB;
      st<v4u, NTS>(reinterpret_cast<v4u*>(d + row * dstep + c * 16), w[n]);
    }
  }
}

// True if the tile was a full, 16-byte aligned block of a shape moved in one shot (and has been moved).
template <typename E, int kThreads, bool NTL, bool NTS>
__device__ __forceinline__ bool transpose_one_shot(const uint8_t* s, const DstSet& ds, const tpx_tile& t, void* lds_raw) {
  if constexpr (kThreads != 512 || sizeof(E) == 1) {
    return false;
  } else {
    if (uint64_t(t.nrows) * t.run_units * sizeof(E) != tpx::kBlockBytes) return false;
    uint64_t bits = reinterpret_cast<uintptr_t>(s) | t.src_pitch | t.dst_step;
    for (uint32_t k = 0; k < ds.n; ++k) bits |= reinterpret_cast<uintptr_t>(ds.base(k));
    if (bits % 16) return false;
    constexpr int kElems = int(tpx::kBlockBytes) / int(sizeof(E));
    switch (t.nrows) {  // the shapes tpx::block_i can ask for
      case 64: transpose_block<E, 64, kElems / 64, kThreads, NTL, NTS>(s, ds, t.src_pitch, t.dst_step, lds_raw); break;
      case 128: transpose_block<E, 128, kElems / 128, kThreads, NTL, NTS>(s, ds, t.src_pitch, t.dst_step, lds_raw); break;
      case 256: transpose_block<E, 256, kElems / 256, kThreads, NTL, NTS>(s, ds, t.src_pitch, t.dst_step, lds_raw); break;
      case 512: transpose_block<E, 512, kElems / 512, kThreads, NTL, NTS>(s, ds, t.src_pitch, t.dst_step, lds_raw); break;
      default: return false;
    }
    return true;
  }
}

template <typename E, int kThreads>
__device__ __forceinline__ void gather_tile(const uint8_t* __restrict__ s, uint8_t* __restrict__ d, const tpx_tile& t) {
  const uint32_t total = t.run_units * t.nrows;
  for (uint32_t e = threadIdx.x; e < total; e += kThreads) {
    const uint32_t i = e / t.run_units, j = e - i * t.run_units;
    *reinterpret_cast<E*>(d + i * t.dst_pitch + j * t.dst_step) =
        *reinterpret_cast<const E*>(s + i * t.src_pitch + j * t.src_step);
  }
}

constexpr int kLdsBytes = int(tpx::kBlockBytes);  // a one-shot block; the general path's sub-tiles are smaller
constexpr uint32_t kLdsPerCu = 160 * 1024;        // gfx950
static_assert(kLdsBytes >= TransposeShape<uint8_t>::kBytes && kLdsBytes >= TransposeShape<uint16_t>::kBytes &&
                  kLdsBytes >= TransposeShape<uint32_t>::kBytes && kLdsBytes >= TransposeShape<uint64_t>::kBytes, "LDS budget");

template <int kThreads, int U, bool NTL, bool NTS>
__global__ __launch_bounds__(kThreads) void tpx_execute_tiles(const tpx::WorkspaceHeader* __restrict__ header, uint64_t plan_id,
                                                              const tpx::FlatBox* __restrict__ boxes,
                                                              const uint32_t* __restrict__ first_tile,
                                                              const uint32_t* __restrict__ coarse,
                                                              const tpx_segment* __restrict__ segs, uint32_t n_boxes,
                                                              uint32_t n_tiles, uint32_t order, PtrTable ptrs) {
  // dynamic LDS only: the segment table of a merge tile or the staging block of a transposing tile (a workgroup
  // executes one tile, so the two never coexist)
  extern __shared__ __align__(16) uint8_t lds_raw[];
  SegLds* lseg = reinterpret_cast<SegLds*>(lds_raw);
  // The tables behind `header` must be the ones this launch was made for (a workspace recycled for another
  // plan since the upload would send the moves anywhere): otherwise the whole grid does nothing.
  if (header->plan_id != plan_id) return;
  // Locate this workgroup's tile; everything here is uniform for the workgroup, so these are scalar loads.
  // `order` = S | C << 16.  The tile sequence is cut into S contiguous parts ("streams") that advance side by side, so
  // the workgroups in flight touch S distant regions of the rank buffers instead of one, which spreads the load over
  // HBM channels and banks; all streams advance at the same rate, so they end together.
  // C > 0 (S divides 8): the order is XCD-aware.  Workgroups are dealt round-robin to the 8 XCDs (workgroup b runs on XCD
  // b % 8), so XCD x serves stream x % S together with the 8/S - 1 other XCDs of that stream, and within the stream
  // each XCD takes runs of C consecutive tiles: what one XCD has in flight is contiguous in the plan (and mostly in
  // memory), not every 8th tile.  C = 0: workgroup b simply takes the (b / S)-th tile of stream b % S.
  uint32_t tile_no = blockIdx.x;
  const uint32_t S = order & 0xffff, C = order >> 16;
  if (C) {
    const uint32_t x = blockIdx.x & 7, i = blockIdx.x >> 3, per = 8 / S, stream = x % S, member = x / S;
    const uint32_t q = (n_tiles + S - 1) / S;  // tiles per stream
    const uint32_t j = ((i / C) * per + member) * C + i % C;
    if (j >= q) return;  // slots the grid was rounded up by
    tile_no = stream * q + j;
    if (tile_no >= n_tiles) return;
  } else if (S > 1) {
    tile_no = (blockIdx.x % S) * (gridDim.x / S) + (blockIdx.x / S);
    if (tile_no >= n_tiles) return;
  }
  const uint32_t box = tpx::find_box(first_tile, coarse, n_boxes, tile_no);
  const tpx::FlatBox fb = boxes[box];
  const tpx_tile t = tpx::tile_of(fb, tile_no - fb.first_tile);
  const DstSet ds{ptrs.dst, t.dst_off, t.dst_rank, t.dst_rank_stride, t.n_dst};
  const bool mc = t.n_dst > 1;
  if (t.kind == TPX_TILE_FILL) {
    if (mc) move_rows_any<kThreads, U, NTL, NTS, true, true>(t.unit_log2, nullptr, ds, t.run_units, t.nrows, 0, t.dst_pitch);
    else move_rows_any<kThreads, U, NTL, NTS, true, false>(t.unit_log2, nullptr, ds, t.run_units, t.nrows, 0, t.dst_pitch);
    return;
  }
  if (t.kind == TPX_TILE_MERGE) {
    merge_tile<kThreads, U, NTL, NTS>(t, segs, ptrs.src, ds, lseg);
    return;
  }
  if (t.kind == TPX_TILE_PACK) {
    pack_tile<kThreads, U, NTL, NTS>(t, segs, ptrs.src, ds, lseg);
    return;
  }
  const uint8_t* s = ptrs.src[t.src_rank] + t.src_off;
  if (t.kind == TPX_TILE_COPY) {
    if (mc) move_rows_any<kThreads, U, NTL, NTS, false, true>(t.unit_log2, s, ds, t.run_units, t.nrows, t.src_pitch, t.dst_pitch);
    else move_rows_any<kThreads, U, NTL, NTS, false, false>(t.unit_log2, s, ds, t.run_units, t.nrows, t.src_pitch, t.dst_pitch);
    return;
  }
  if (t.kind == TPX_TILE_TRANSPOSE) {  // full blocks in one shot; ragged or misaligned ones fall through to the general path
    bool done = false;
    switch (t.unit_log2) {
      case 3: done = transpose_one_shot<uint64_t, kThreads, NTL, NTS>(s, ds, t, lds_raw); break;
      case 2: done = transpose_one_shot<uint32_t, kThreads, NTL, NTS>(s, ds, t, lds_raw); break;
      case 1: done = transpose_one_shot<uint16_t, kThreads, NTL, NTS>(s, ds, t, lds_raw); break;
      default: break;
    }
    if (done) return;
  }
  // other transposing tiles and gathering tiles: one pass per destination (they are rare; the source is re-read)
  for (uint32_t c = 0; c < t.n_dst; ++c) {
    uint8_t* d = ds.base(c);
    if (t.kind == TPX_TILE_TRANSPOSE) {
      switch (t.unit_log2) {
        case 3: transpose_tile<uint64_t, kThreads, NTL, NTS>(s, d, t.run_units, t.nrows, t.src_pitch, t.dst_step, lds_raw); break;
        case 2: transpose_tile<uint32_t, kThreads, NTL, NTS>(s, d, t.run_units, t.nrows, t.src_pitch, t.dst_step, lds_raw); break;
        case 1: transpose_tile<uint16_t, kThreads, NTL, NTS>(s, d, t.run_units, t.nrows, t.src_pitch, t.dst_step, lds_raw); break;
        default: transpose_tile<uint8_t, kThreads, NTL, NTS>(s, d, t.run_units, t.nrows, t.src_pitch, t.dst_step, lds_raw); break;
      }
    } else {
      switch (t.unit_log2) {
        case 3: gather_tile<uint64_t, kThreads>(s, d, t); break;
        case 2: gather_tile<uint32_t, kThreads>(s, d, t); break;
        case 1: gather_tile<uint16_t, kThreads>(s, d, t); break;
        default: gather_tile<uint8_t, kThreads>(s, d, t); break;
      }
    }
  }
}

// Read-only and write-only yardsticks: what this memory gives a pure read and a pure write stream in the launch shape
// and tile order of the default copy tile (512 threads x 8 nontemporal 16-byte accesses all issued at once, one
// workgroup per CU, 4 streams, every XCD taking runs of 8 consecutive 64 KiB chunks).  Among 256/512/1024 threads x
// 4/8/16 accesses x 1...256 fronts, with and without the occupancy cap and the per-XCD runs, that shape is within 1 %
// of the best write-only rate found (6.7-6.8 TB/s; without per-XCD runs 5.5-6.1, with more than one workgroup per CU
// 5.2-6.6) and within 3 % of the best read-only rate (7.0-7.2 TB/s in every shape).
constexpr int kOneShotThreads = 512;
constexpr uint64_t kOneShotUnits = uint64_t(kOneShotThreads) * 8;
constexpr uint32_t kOneShotStreams = 4, kOneShotRun = 8;
constexpr uint32_t kOneShotLds = ((kLdsPerCu / 2) & ~255u) + 256;  // one workgroup fits a CU, two do not
// First unit of this workgroup's chunk, or ~0 if the workgroup is one of those the grid was rounded up by.
__device__ __forceinline__ uint64_t one_shot_base(uint64_t n_chunks) {
  const uint32_t x = blockIdx.x & 7, i = blockIdx.x >> 3, per = 8 / kOneShotStreams, stream = x % kOneShotStreams, member = x / kOneShotStreams;
  const uint64_t q = (n_chunks + kOneShotStreams - 1) / kOneShotStreams;
  const uint64_t j = (uint64_t(i / kOneShotRun) * per + member) * kOneShotRun + i % kOneShotRun;
  if (j >= q) return ~0ull;
  return (stream * q + j) * kOneShotUnits + threadIdx.x;  // chunks past the end are caught by the callers' idx < n
}
__global__ __launch_bounds__(kOneShotThreads) void tpx_probe_read_kernel(const v4u* __restrict__ s, uint64_t n, uint64_t n_chunks,
                                                                         v4u* __restrict__ sink) {
  const uint64_t base = one_shot_base(n_chunks);
  if (base == ~0ull) return;
  v4u acc = zero_of<v4u>();
  if (base - threadIdx.x + kOneShotUnits <= n) {  // a whole chunk: all eight loads in flight before the first use
    v4u r[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) r[k] = __builtin_nontemporal_load(s + base + uint64_t(k) * kOneShotThreads);
#pragma unroll
    for (int k = 0; k < 8; ++k) acc ^= r[k];
  } else {
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const uint64_t idx = base + uint64_t(k) * kOneShotThreads;
      if (idx < n) acc ^= __builtin_nontemporal_load(s + idx);
    }
  }
  // keeps the loads alive; for data that is not adversarial the store happens about once in 2^32 threads
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) *sink = acc;
}
__global__ __launch_bounds__(kOneShotThreads) void tpx_probe_fill_kernel(v4u* __restrict__ d, uint64_t n, uint64_t n_chunks, uint32_t value) {
  const uint64_t base = one_shot_base(n_chunks);
  if (base == ~0ull) return;
  const v4u v = {value, value, value, value};
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const uint64_t idx = base + uint64_t(k) * kOneShotThreads;
    if (idx < n) __builtin_nontemporal_store(v, d + idx);
  }
}

// Plain grid-stride copy: each thread moves 4 independent 16-byte vectors per iteration.
constexpr int kProbeThreads = 256;
__global__ __launch_bounds__(kProbeThreads) void tpx_probe_copy_kernel(v4u* __restrict__ d, const v4u* __restrict__ s, uint64_t n) {
  const uint64_t stride = uint64_t(gridDim.x) * kProbeThreads * 4;
  for (uint64_t base = uint64_t(blockIdx.x) * kProbeThreads * 4 + threadIdx.x; base < n; base += stride) {
    v4u r[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (base + uint64_t(k) * kProbeThreads < n) r[k] = s[base + uint64_t(k) * kProbeThreads];
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (base + uint64_t(k) * kProbeThreads < n) d[base + uint64_t(k) * kProbeThreads] = r[k];
  }
}

tpx_status hip_fail(hipError_t e, const char* what) {
  return tpx::fail(TPX_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

using KernelFn = void (*)(const tpx::WorkspaceHeader*, uint64_t, const tpx::FlatBox*, const uint32_t*, const uint32_t*, const tpx_segment*, uint32_t, uint32_t, uint32_t, PtrTable);

template <int T, int U>
KernelFn pick_nt(bool nt) {
  return nt ? tpx_execute_tiles<T, U, true, true> : tpx_execute_tiles<T, U, false, false>;
}

template <int T>
KernelFn pick_unroll(uint64_t variant) {
  const bool nt = (variant >> 3) & 1;
  switch (variant & 7) {
    case 2: return pick_nt<T, 4>(nt);
    case 4: return pick_nt<T, 16>(nt);
    default: return pick_nt<T, 8>(nt);
  }
}

// variant bits: [2:0] log2 of the 16-byte loads in flight per thread (2, 3 or 4); bits 3 and 4 (set
// together or not at all): nontemporal loads and stores; bits [6:5] threads per workgroup (0: 256, 1: 512,
// 2: 1024).
int threads_of(uint64_t variant) {
  switch ((variant >> 5) & 3) {
    case 0: return 256;
    case 1: return 512;
    default: return 1024;
  }
}

KernelFn pick_kernel(uint64_t variant) {
  switch (threads_of(variant)) {
    case 1024: return pick_unroll<1024>(variant);
    case 512: return pick_unroll<512>(variant);
    default: return pick_unroll<256>(variant);
  }
}

}  // namespace

namespace tpx {

tpx_status hip_upload_tables(void* workspace, const tpx_plan_s& plan, void* stream) {
  // the plan keeps one host image of the whole workspace (header, flat boxes, prefix sums, coarse table,
  // segments): one copy
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipError_t e = hipMemcpyAsync(workspace, plan.image.data(), plan.image.size(), hipMemcpyHostToDevice, st);
  if (e != hipSuccess) return hip_fail(e, "copying the plan tables to the workspace");
  e = hipStreamSynchronize(st);  // the plan may be freed as soon as the caller likes
  if (e != hipSuccess) return hip_fail(e, "waiting for the plan table copy");
  return TPX_OK;
}

tpx_status hip_launch_tiles(const void* workspace, const tpx_plan_s& plan, const void* const* src, uint32_t n_src,
                            void* const* dst, uint32_t n_dst, uint64_t variant, void* stream) {
  if (plan.n_tiles == 0) return TPX_OK;
  if (plan.n_tiles > 0x7fffffffull) return fail(TPX_ERR_INVALID_ARG, "too many tiles for one launch");
  if (n_src > TPX_MAX_RANKS || n_dst > TPX_MAX_RANKS) return fail(TPX_ERR_INVALID_ARG, "too many rank buffers");
  PtrTable pt;
  for (uint32_t r = 0; r < TPX_MAX_RANKS; ++r) {
    pt.src[r] = r < n_src ? static_cast<const uint8_t*>(src[r]) : nullptr;
    pt.dst[r] = r < n_dst ? static_cast<uint8_t*>(dst[r]) : nullptr;
  }
  const WorkspaceLayout w = workspace_layout(plan);
  const uint8_t* base = static_cast<const uint8_t*>(workspace);
  const bool automatic = variant == 0;
  if (automatic) {
    // A workgroup loads its whole tile at once (threads x loads in flight x 16 bytes = tile).  64 KiB tiles (the
    // default, and what a plan with transposing blocks always has) go to 512 threads x 8 loads; small jobs have smaller
    // tiles and smaller workgroups; tiles of 128 KiB and more (a plan option) to 1024 threads x 8.
    variant = plan.tile_bytes_used >= 131072 ? (3 | 24 | (2 << 5))   // 1024 threads x 8
            : plan.tile_bytes_used >= 65536  ? (3 | 24 | (1 << 5))   //  512 threads x 8
                                             : (2 | 24);             //  256 threads x 4 (small jobs, small tiles)
  }
  // Workgroups per CU.  The memory side is saturated with about 64 KiB in flight per CU (16 MiB on the chip); more
  // only lengthens the queues in front of DRAM and costs bandwidth (measured: one 512-thread workgroup with 64 KiB in
  // flight per CU beats two of them, and one 1024-thread workgroup with 128 KiB, by 2-3 %).  Registers would allow two
  // 512-thread workgroups, so occupancy is capped through the LDS request: a workgroup that asks for a little more
  // than half of the CU's 160 KiB has the CU to itself.
  uint32_t per_cu = uint32_t(tuning().occupancy.load());
  if (!per_cu && threads_of(variant) == 512) per_cu = 1;
  uint32_t lds_bytes = plan.needs_lds ? kLdsBytes : kSegLdsBytes;
  if (per_cu) lds_bytes = std::max<uint32_t>(lds_bytes, ((kLdsPerCu / (per_cu + 1)) & ~255u) + 256);  // per_cu fit, per_cu + 1 do not
  // Tile order.  Interleaving several parts of the plan pays only when tiles cost the same; a plan that mixes plain
  // and replicated moves runs as one stream.  Runs of 8 tiles per XCD (see the kernel) unless the plan has transposing
  // blocks, whose boxes already order their tiles for the destination.
  const uint32_t streams = plan.uniform_tiles ? uint32_t(std::max<uint64_t>(1, tuning().streams.load())) : 1;
  uint32_t chunk = uint32_t(tuning().chunk.load());
  if (!chunk) chunk = plan.needs_lds ? 1 : 8;  // knob: 0 = automatic, 1 = no XCD-aware runs
  uint32_t grid = uint32_t((plan.n_tiles + streams - 1) / streams * streams);
  uint32_t order = streams;
  if (chunk > 1 && 8 % streams == 0) {
    const uint64_t q = (plan.n_tiles + streams - 1) / streams, unit = uint64_t(8 / streams) * chunk;
    grid = uint32_t((q + unit - 1) / unit * unit * streams);
    order = streams | (chunk << 16);
  }
  KernelFn k = pick_kernel(variant);
  const WorkspaceHeader* a_header = reinterpret_cast<const WorkspaceHeader*>(base + w.header_off);
  uint64_t a_id = plan.id;
  const FlatBox* a_boxes = reinterpret_cast<const FlatBox*>(base + w.boxes_off);
  const uint32_t* a_first = reinterpret_cast<const uint32_t*>(base + w.first_off);
  const uint32_t* a_coarse = reinterpret_cast<const uint32_t*>(base + w.coarse_off);
  const tpx_segment* a_segs = reinterpret_cast<const tpx_segment*>(base + w.seg_off);
  uint32_t a_nboxes = uint32_t(plan.flat.size()), a_ntiles = uint32_t(plan.n_tiles), a_order = order;
  void* args[] = {&a_header, &a_id, &a_boxes, &a_first, &a_coarse, &a_segs, &a_nboxes, &a_ntiles, &a_order, &pt};
  // the launch's own status, not the runtime's last-error slot, which other users of the runtime share
  const hipError_t e = hipLaunchKernel(reinterpret_cast<const void*>(k), dim3(grid), dim3(threads_of(variant)), args,
                                       lds_bytes, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(e, "launching the tile kernel");
  return TPX_OK;
}

namespace {
// Per device: the address of that device's copy of `scratch` and the id of the plan whose tables the
// library last put there (0 = none).  Nobody else knows the address, so the host-side record is exact.
constexpr int kMaxDevices = 64;
struct StaticTables {
  void* ptr = nullptr;
  uint64_t plan_id = 0;
};
StaticTables g_static[kMaxDevices];
std::mutex g_static_mutex;
}  // namespace

tpx_status hip_execute_static(const tpx_plan_s& plan, const void* const* src, uint32_t n_src, void* const* dst,
                              uint32_t n_dst, uint64_t variant, void* stream) {
  if (plan.n_tiles == 0) return TPX_OK;
  if (plan.image.size() > TPX_STATIC_WORKSPACE_BYTES)
    return fail(TPX_ERR_TOO_LARGE, "tpx_execute_static: the plan tables take " + std::to_string(plan.image.size()) +
                                       " bytes, more than TPX_STATIC_WORKSPACE_BYTES (" +
                                       std::to_string(TPX_STATIC_WORKSPACE_BYTES) + "); use tpx_execute with a workspace");
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "tpx_execute_static: asking for the current device");
  if (dev < 0 || dev >= kMaxDevices) return fail(TPX_ERR_INVALID_ARG, "tpx_execute_static: device index out of range");
  if (stream) {
    int sdev = -1;
    e = hipStreamGetDevice(static_cast<hipStream_t>(stream), &sdev);
    if (e != hipSuccess) return hip_fail(e, "tpx_execute_static: asking for the stream's device");
    if (sdev != dev) return fail(TPX_ERR_INVALID_ARG, "tpx_execute_static: hip_stream belongs to another device than the current one");
  }
  void* tables = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_static_mutex);
    StaticTables& s = g_static[dev];
    if (!s.ptr) {  // first call on this device: every GPU holds its own copy of the array at its own address
      void* p = nullptr;
      e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess) return hip_fail(e, "tpx_execute_static: looking up the static table array");
      if (!p) return fail(TPX_ERR_HIP, "tpx_execute_static: the static table array has no device address");
      s.ptr = p;
    }
    if (s.plan_id != plan.id) {  // ordered on `stream` after whatever the caller's earlier launches there still read
      s.plan_id = 0;
      if (tpx_status st = hip_upload_tables(s.ptr, plan, stream)) return st;
      s.plan_id = plan.id;
    }
    tables = s.ptr;
  }
  return hip_launch_tiles(tables, plan, src, n_src, dst, n_dst, variant, stream);
}

tpx_status hip_read_header(const void* workspace, void* stream, WorkspaceHeader* out) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipError_t e = hipMemcpyAsync(out, workspace, sizeof(WorkspaceHeader), hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  if (e != hipSuccess) return hip_fail(e, "reading the workspace header");
  return TPX_OK;
}

namespace {
// Grid of the one-shot probes for n units: per stream ceil(chunks / streams) slots, rounded up to whole runs of all
// the XCDs of the stream (see one_shot_base).  0 = too large for one launch.
uint32_t one_shot_grid(uint64_t n, uint64_t& n_chunks) {
  n_chunks = (n + kOneShotUnits - 1) / kOneShotUnits;
  const uint64_t q = (n_chunks + kOneShotStreams - 1) / kOneShotStreams, unit = uint64_t(8 / kOneShotStreams) * kOneShotRun;
  const uint64_t grid = (q + unit - 1) / unit * unit * kOneShotStreams;
  return grid > 0x7fffffffull ? 0 : uint32_t(grid);
}
}  // namespace

tpx_status hip_probe_read(const void* src, uint64_t nbytes, void* sink, void* stream) {
  if (nbytes == 0) return TPX_OK;
  const v4u* a_src = static_cast<const v4u*>(src);
  uint64_t a_n = nbytes / 16, a_chunks = 0;
  v4u* a_sink = static_cast<v4u*>(sink);
  const uint32_t grid = one_shot_grid(a_n, a_chunks);
  if (!grid) return fail(TPX_ERR_INVALID_ARG, "tpx_probe_read: too many bytes for one launch");
  void* args[] = {&a_src, &a_n, &a_chunks, &a_sink};
  const hipError_t e = hipLaunchKernel(reinterpret_cast<const void*>(tpx_probe_read_kernel), dim3(grid), dim3(kOneShotThreads), args,
                                       kOneShotLds, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(e, "launching the read probe");
  return TPX_OK;
}

tpx_status hip_probe_fill(void* dst, uint64_t nbytes, uint32_t value, void* stream) {
  if (nbytes == 0) return TPX_OK;
  v4u* a_dst = static_cast<v4u*>(dst);
  uint64_t a_n = nbytes / 16, a_chunks = 0;
  uint32_t a_value = value;
  const uint32_t grid = one_shot_grid(a_n, a_chunks);
  if (!grid) return fail(TPX_ERR_INVALID_ARG, "tpx_probe_fill: too many bytes for one launch");
  void* args[] = {&a_dst, &a_n, &a_chunks, &a_value};
  const hipError_t e = hipLaunchKernel(reinterpret_cast<const void*>(tpx_probe_fill_kernel), dim3(grid), dim3(kOneShotThreads), args,
                                       kOneShotLds, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(e, "launching the fill probe");
  return TPX_OK;
}

tpx_status hip_probe_copy(void* dst, const void* src, uint64_t nbytes, void* stream) {
  if (nbytes == 0) return TPX_OK;
  const uint64_t n = nbytes / 16;
  const uint64_t want = (n + kProbeThreads * 4 - 1) / (kProbeThreads * 4);
  const uint32_t grid = uint32_t(want < 256 * 16 ? want : 256 * 16);
  v4u* a_dst = static_cast<v4u*>(dst);
  const v4u* a_src = static_cast<const v4u*>(src);
  uint64_t a_n = n;
  void* args[] = {&a_dst, &a_src, &a_n};
  const hipError_t e = hipLaunchKernel(reinterpret_cast<const void*>(tpx_probe_copy_kernel), dim3(grid), dim3(kProbeThreads),
                                       args, 0, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(e, "launching the probe copy kernel");
  return TPX_OK;
}

}  // namespace tpx

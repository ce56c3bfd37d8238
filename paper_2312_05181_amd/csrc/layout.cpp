// The PTC of one configuration (paper section 4.1, equation 1), evaluated on the host:
// sigma (how each tensor is sliced), phi (which stage and replica holds a slice) and
// alpha (which rank buffer that is, and where inside it).  The paper leaves the concrete
// functions to the model parallelizer; the Megatron-style rules here are this library's
// own convention.
#include <algorithm>
#include <cstring>

#include "tpx_internal.hpp"

namespace tpx {

namespace {
thread_local std::string g_err;
const char* kNames[N_NAMES] = {
    "word_embeddings.weight", "position_embeddings.weight",
    "input_layernorm.weight", "input_layernorm.bias",
    "attention.query_key_value.weight", "attention.query_key_value.bias",
    "attention.dense.weight", "attention.dense.bias",
    "post_attention_layernorm.weight", "post_attention_layernorm.bias",
    "mlp.dense_h_to_4h.weight", "mlp.dense_h_to_4h.bias",
    "mlp.dense_4h_to_h.weight", "mlp.dense_4h_to_h.bias",
    "final_layernorm.weight", "final_layernorm.bias"};
}  // namespace

tpx_status fail(tpx_status st, const std::string& msg) {
  g_err = msg;
  return st;
}
const char* last_error_cstr() { return g_err.c_str(); }

Tuning& tuning() {
  static Tuning t;
  return t;
}

tpx_status resolve_opts(const tpx_plan_opts* in, tpx_plan_opts& out) {
  out = tpx_plan_opts{65536, 8, 0, 0, 0};
  if (!in) return TPX_OK;
  if (in->tile_bytes) {
    if (in->tile_bytes < 4096 || in->tile_bytes > 4194304 || (in->tile_bytes & (in->tile_bytes - 1)))
      return fail(TPX_ERR_INVALID_ARG, "tile_bytes must be a power of two in [4096, 4194304]");
    out.tile_bytes = in->tile_bytes;
  }
  if (in->max_multicast) {
    if (in->max_multicast > 128) return fail(TPX_ERR_INVALID_ARG, "max_multicast must be in [1, 128]");
    out.max_multicast = in->max_multicast;
  }
  if (in->share_reads > 1) return fail(TPX_ERR_INVALID_ARG, "share_reads must be 0 or 1");
  out.share_reads = in->share_reads;
  if (in->reserved_) return fail(TPX_ERR_INVALID_ARG, "the reserved field of tpx_plan_opts must be 0");
  if (in->pack_bytes > out.tile_bytes) return fail(TPX_ERR_INVALID_ARG, "pack_bytes must not exceed tile_bytes");
  out.pack_bytes = in->pack_bytes;  // 0 = a quarter of the tile size in use, decided when the tiles are cut
  return TPX_OK;
}

const char* param_name(uint32_t name) { return name < N_NAMES ? kNames[name] : nullptr; }

uint32_t tensor_id_of(uint32_t name, int32_t layer) {
  switch (name) {
    case WORD_EMB: return 0;
    case POS_EMB: return 1;
    case LNF_W: return 2;
    case LNF_B: return 3;
    default: return 4 + uint32_t(layer) * kLayerNames + (name - LN1_W);
  }
}

uint32_t n_tensors_of(const tpx_model& m) { return 4 + m.n_layers * kLayerNames; }

tpx_status check_model(const tpx_model& m) {
  if (!m.n_layers || !m.hidden || !m.n_heads || !m.ffn || !m.vocab_true || !m.max_pos)
    return fail(TPX_ERR_INVALID_ARG, "model: a dimension is zero");
  if (m.n_state_kinds < 1 || m.n_state_kinds > 4)
    return fail(TPX_ERR_INVALID_ARG, "model: n_state_kinds must be 1..4");
  for (uint32_t k = 0; k < m.n_state_kinds; ++k) {
    uint8_t b = m.state_elem_bytes[k];
    if (b != 1 && b != 2 && b != 4 && b != 8)
      return fail(TPX_ERR_INVALID_ARG, "model: state element size must be 1, 2, 4 or 8 bytes");
  }
  if (m.hidden % m.n_heads) return fail(TPX_ERR_INDIVISIBLE, "model: hidden is not a multiple of n_heads");
  return TPX_OK;
}

static tpx_status padded_vocab(const tpx_model& m, uint32_t T, uint64_t& out) {
  if (m.vocab_divisor == 0) {
    if (m.vocab_true % T) return fail(TPX_ERR_INDIVISIBLE, "vocabulary is not divisible by T and no padding divisor is set");
    out = m.vocab_true;
    return TPX_OK;
  }
  const uint64_t q = uint64_t(m.vocab_divisor) * T;
  out = (m.vocab_true + q - 1) / q * q;
  return TPX_OK;
}

// sigma: the slicing of one parameter tensor.
tpx_status sigma_of(const tpx_model& m, const tpx_parallel& par, uint32_t name, Sigma& s) {
  s = Sigma{};
  const uint64_t h = m.hidden, a = m.n_heads, dh = m.hidden / m.n_heads, f = m.ffn;
  const bool tr = par.w_transposed != 0;
  auto set = [&](std::initializer_list<uint64_t> full, int axis, std::initializer_list<uint32_t> perm) {
    s.ndim = uint32_t(full.size());
    std::copy(full.begin(), full.end(), s.full);
    std::copy(perm.begin(), perm.end(), s.perm);
    s.split_axis = axis;
  };
  switch (name) {
    case WORD_EMB: {  // vocabulary-parallel embedding: rows are cut
      uint64_t vp = 0;
      if (tpx_status st = padded_vocab(m, par.T, vp)) return st;
      set({vp, h}, 0, {0, 1});
      break;
    }
    case POS_EMB: set({m.max_pos, h}, -1, {0, 1}); break;
    case LN1_W: case LN1_B: case LN2_W: case LN2_B: case DENSE_B: case FC2_B: case LNF_W: case LNF_B:
      set({h}, -1, {0});
      break;
    case QKV_W:  // column-parallel, cut by heads; canonical view [head, q/k/v, head_dim, in]
      if (par.qkv_layout == 0) {
        if (tr) set({a, 3, dh, h}, 0, {3, 0, 1, 2}); else set({a, 3, dh, h}, 0, {0, 1, 2, 3});
      } else {
        if (tr) set({a, 3, dh, h}, 0, {3, 1, 0, 2}); else set({a, 3, dh, h}, 0, {1, 0, 2, 3});
      }
      break;
    case QKV_B:
      if (par.qkv_layout == 0) set({a, 3, dh}, 0, {0, 1, 2}); else set({a, 3, dh}, 0, {1, 0, 2});
      break;
    case DENSE_W:  // row-parallel: the input axis is cut
      if (tr) set({h, h}, 1, {1, 0}); else set({h, h}, 1, {0, 1});
      break;
    case FC1_W:    // column-parallel
      if (tr) set({f, h}, 0, {1, 0}); else set({f, h}, 0, {0, 1});
      break;
    case FC1_B: set({f}, 0, {0}); break;
    case FC2_W:    // row-parallel
      if (tr) set({h, f}, 1, {1, 0}); else set({h, f}, 1, {0, 1});
      break;
    default: return fail(TPX_ERR_INVALID_ARG, "unknown parameter name");
  }
  if (s.split_axis >= 0 && s.full[s.split_axis] % par.T)
    return fail(TPX_ERR_INDIVISIBLE, std::string(kNames[name]) + ": sliced axis is not divisible by T");
  return TPX_OK;
}

// phi + alpha: fill the manifests of all rank buffers of one configuration.
tpx_status build_side(const tpx_model& m, const tpx_parallel& par, Side& out) {
  if (!par.T || !par.P || !par.D) return fail(TPX_ERR_INVALID_ARG, "parallel degrees must be >= 1");
  const uint64_t n_ranks = uint64_t(par.T) * par.P * par.D;
  if (n_ranks > TPX_MAX_RANKS) return fail(TPX_ERR_INVALID_ARG, "more than TPX_MAX_RANKS ranks in one configuration");
  if (par.qkv_layout > 1 || par.w_transposed > 1) return fail(TPX_ERR_INVALID_ARG, "unknown layout tag");
  if (par.shard_kinds >> m.n_state_kinds) return fail(TPX_ERR_INVALID_ARG, "shard_kinds names a state kind the model does not have");
  if (m.n_heads % par.T || m.ffn % par.T || m.hidden % par.T)
    return fail(TPX_ERR_INDIVISIBLE, "heads, ffn or hidden not divisible by T");
  out = Side{};
  out.tp_degree = par.T;
  std::vector<uint32_t> stage_first(par.P + 1);
  if (par.layer_stage) {
    for (uint32_t l = 0; l < m.n_layers; ++l)
      if (par.layer_stage[l] >= par.P) return fail(TPX_ERR_BAD_STAGE_MAP, "layer_stage names a stage >= P");
  } else if (par.stage_first_layer) {
    for (uint32_t p = 0; p <= par.P; ++p) stage_first[p] = par.stage_first_layer[p];
    if (stage_first[0] != 0 || stage_first[par.P] != m.n_layers)
      return fail(TPX_ERR_BAD_STAGE_MAP, "stage boundaries must start at 0 and end at n_layers");
    for (uint32_t p = 0; p < par.P; ++p)
      if (stage_first[p] > stage_first[p + 1])
        return fail(TPX_ERR_BAD_STAGE_MAP, "stage boundaries must be ascending");
  } else {
    if (m.n_layers % par.P) return fail(TPX_ERR_INDIVISIBLE, "layers not divisible by P and no stage map given");
    for (uint32_t p = 0; p <= par.P; ++p) stage_first[p] = p * (m.n_layers / par.P);
  }
  out.alive.assign(n_ranks, 1);
  if (par.rank_alive) std::copy(par.rank_alive, par.rank_alive + n_ranks, out.alive.begin());

  Sigma sig[N_NAMES];
  for (uint32_t n = 0; n < N_NAMES; ++n)
    if (tpx_status st = sigma_of(m, par, n, sig[n])) return st;

  out.ranks.resize(n_ranks);
  out.bytes.assign(n_ranks, 0);

  for (uint32_t p = 0; p < par.P; ++p) {
    // the tensors of stage p in packing order
    std::vector<std::pair<uint32_t, int32_t>> held;
    if (p == 0) { held.push_back({WORD_EMB, -1}); held.push_back({POS_EMB, -1}); }
    for (uint32_t l = par.layer_stage ? 0 : stage_first[p]; l < (par.layer_stage ? m.n_layers : stage_first[p + 1]); ++l) {
      if (par.layer_stage && par.layer_stage[l] != p) continue;
      for (uint32_t n = LN1_W; n <= FC2_B; ++n) held.push_back({n, int32_t(l)});
    }
    if (p == par.P - 1) {
      held.push_back({LNF_W, -1});
      held.push_back({LNF_B, -1});
      if ((m.flags & TPX_MODEL_TIED_HEAD) && par.P > 1) held.push_back({WORD_EMB, -1});
    }
    for (uint32_t d = 0; d < par.D; ++d)
      for (uint32_t t = 0; t < par.T; ++t) {
        const uint32_t rank = t + par.T * (d + par.D * p);  // alpha
        auto& man = out.ranks[rank];
        man.reserve(held.size() * m.n_state_kinds);
        uint64_t off = 0;
        for (uint32_t k = 0; k < m.n_state_kinds; ++k) {  // one arena per state kind
          const bool cut_over_d = (par.shard_kinds >> k) & 1;
          for (auto [name, layer] : held) {
            const Sigma& s = sig[name];
            tpx_entry e{};
            e.tensor_id = tensor_id_of(name, layer);
            e.kind = k;
            e.elem_bytes = m.state_elem_bytes[k];
            e.ndim = s.ndim;
            e.name = name;
            e.layer = layer;
            uint64_t numel = 1;
            for (uint32_t ax = 0; ax < s.ndim; ++ax) {
              e.full_shape[ax] = s.full[ax];
              e.lo[ax] = 0;
              e.hi[ax] = s.full[ax];
              e.perm[ax] = s.perm[ax];
              if (int(ax) == s.split_axis) {
                const uint64_t part = s.full[ax] / par.T;
                e.lo[ax] = part * t;
                e.hi[ax] = part * (t + 1);
              }
            }
            if (cut_over_d) {  // replica d keeps chunk d along the outermost stored axis
              const uint32_t ax = s.perm[0];
              const uint64_t n = e.hi[ax] - e.lo[ax], c = (n + par.D - 1) / par.D;
              const uint64_t a = std::min<uint64_t>(n, uint64_t(d) * c), b = std::min<uint64_t>(n, uint64_t(d + 1) * c);
              if (a == b) continue;  // nothing of this tensor on this replica
              e.hi[ax] = e.lo[ax] + b;
              e.lo[ax] += a;
            }
            for (uint32_t ax = 0; ax < s.ndim; ++ax) numel *= e.hi[ax] - e.lo[ax];
            off = (off + kAlign - 1) / kAlign * kAlign;
            e.offset = off;
            e.nbytes = numel * e.elem_bytes;
            off += e.nbytes;
            man.push_back(e);
          }
        }
        out.bytes[rank] = (off + kAlign - 1) / kAlign * kAlign;
      }
  }
  return TPX_OK;
}

// Checks every entry of every manifest: shape, storage order, size, placement inside the rank buffer,
// no two sub-tensors of a rank overlapping.  Fills nbytes.
tpx_status check_entries(Side& side) {
  for (size_t r = 0; r < side.ranks.size(); ++r) {
    std::vector<std::pair<uint64_t, uint64_t>> spans;
    for (tpx_entry& e : side.ranks[r]) {
      const std::string where = "rank " + std::to_string(r) + " tensor " + std::to_string(e.tensor_id);
      if (e.ndim < 1 || e.ndim > 4) return fail(TPX_ERR_INVALID_ARG, where + ": ndim must be 1..4");
      if (e.elem_bytes != 1 && e.elem_bytes != 2 && e.elem_bytes != 4 && e.elem_bytes != 8)
        return fail(TPX_ERR_INVALID_ARG, where + ": element size must be 1, 2, 4 or 8 bytes");
      if (e.kind > 255) return fail(TPX_ERR_INVALID_ARG, where + ": state kind must be < 256");
      uint32_t seen = 0;
      uint64_t numel = 1;
      for (uint32_t k = 0; k < e.ndim; ++k) {
        if (e.perm[k] >= e.ndim || (seen >> e.perm[k]) & 1) return fail(TPX_ERR_INVALID_ARG, where + ": perm is not a permutation");
        seen |= 1u << e.perm[k];
        if (!(e.lo[k] < e.hi[k] && e.hi[k] <= e.full_shape[k])) return fail(TPX_ERR_INVALID_ARG, where + ": need lo < hi <= full_shape");
        numel *= e.hi[k] - e.lo[k];
      }
      if (e.nbytes && e.nbytes != numel * e.elem_bytes) return fail(TPX_ERR_INVALID_ARG, where + ": nbytes does not match its box");
      e.nbytes = numel * e.elem_bytes;
      if (e.offset % e.elem_bytes) return fail(TPX_ERR_INVALID_ARG, where + ": offset is not a multiple of the element size");
      if (e.offset + e.nbytes > side.bytes[r]) return fail(TPX_ERR_INVALID_ARG, where + ": extends past the end of its rank buffer");
      spans.push_back({e.offset, e.offset + e.nbytes});
    }
    std::sort(spans.begin(), spans.end());
    for (size_t i = 1; i < spans.size(); ++i)
      if (spans[i].first < spans[i - 1].second) return fail(TPX_ERR_INVALID_ARG, "rank " + std::to_string(r) + ": two sub-tensors overlap in the buffer");
  }
  return TPX_OK;
}

// Builds the per-tensor index of a side: which distinct boxes of a tensor exist and who holds each.
// Rejects sub-tensors of one tensor that disagree about its shape or overlap without being equal.
tpx_status index_subs(Side& side) {
  side.key_of.clear();
  side.dense_key.clear();
  side.subs.clear();
  uint64_t max_tid = 0, max_kind = 0;
  for (const auto& man : side.ranks)
    for (const tpx_entry& e : man) { max_tid = std::max<uint64_t>(max_tid, e.tensor_id); max_kind = std::max<uint64_t>(max_kind, e.kind); }
  side.dense_kinds = (max_tid + 1) * (max_kind + 1) <= (1u << 22) ? uint32_t(max_kind + 1) : 0;
  if (side.dense_kinds) side.dense_key.assign(size_t((max_tid + 1) * side.dense_kinds), -1);
  for (uint32_t r = 0; r < side.ranks.size(); ++r)
    for (uint32_t i = 0; i < side.ranks[r].size(); ++i) {
      const tpx_entry& e = side.ranks[r][i];
      int32_t key = side.find_key(e.tensor_id, e.kind);
      if (key < 0) {
        key = int32_t(side.subs.size());
        if (side.dense_kinds) side.dense_key[size_t(e.tensor_id) * side.dense_kinds + e.kind] = key;
        else side.key_of.emplace((uint64_t(e.tensor_id) << 8) | e.kind, uint32_t(key));
        side.subs.emplace_back();
        side.subs.back().reserve(side.tp_degree ? side.tp_degree : 4);
      }
      auto& subs = side.subs[size_t(key)];
      if (!subs.empty()) {
        const tpx_entry& f = side.ranks[subs[0].holders[0].rank][subs[0].holders[0].entry];
        bool same = f.ndim == e.ndim && f.elem_bytes == e.elem_bytes;
        for (uint32_t k = 0; same && k < e.ndim; ++k) same = f.full_shape[k] == e.full_shape[k];
        if (!same) return fail(TPX_ERR_INVALID_ARG, "tensor " + std::to_string(e.tensor_id) + ": its sub-tensors disagree about shape or element size");
      }
      SubTensor* found = nullptr;
      for (SubTensor& s : subs) {
        bool equal = true, disjoint = false;
        for (uint32_t k = 0; k < e.ndim; ++k) {
          equal = equal && s.lo[k] == e.lo[k] && s.hi[k] == e.hi[k];
          disjoint = disjoint || s.hi[k] <= e.lo[k] || e.hi[k] <= s.lo[k];
        }
        if (equal) { found = &s; break; }
        if (!disjoint) return fail(TPX_ERR_INVALID_ARG, "tensor " + std::to_string(e.tensor_id) + ": sub-tensors overlap without being equal");
      }
      if (!found) {
        subs.emplace_back();
        found = &subs.back();
        for (uint32_t k = 0; k < e.ndim; ++k) { found->lo[k] = e.lo[k]; found->hi[k] = e.hi[k]; }
      }
      found->holders.push_back({r, i});  // ranks are visited in ascending order
    }
  for (auto& subs : side.subs)
    std::sort(subs.begin(), subs.end(), [](const SubTensor& a, const SubTensor& b) {
      return std::lexicographical_compare(a.lo, a.lo + 4, b.lo, b.lo + 4);
    });
  return TPX_OK;
}

// Partitions the wanted ranks (alive != 0) into replica groups: ranks with identical manifests whose indices
// form an arithmetic progression.
tpx_status find_groups(Side& side) {
  side.groups.clear();
  std::vector<char> done(side.ranks.size(), 0);
  auto same_manifest = [&](uint32_t a, uint32_t b) {
    if (side.bytes[a] != side.bytes[b] || side.ranks[a].size() != side.ranks[b].size()) return false;
    for (size_t i = 0; i < side.ranks[a].size(); ++i) {
      const tpx_entry &x = side.ranks[a][i], &y = side.ranks[b][i];
      if (x.tensor_id != y.tensor_id || x.kind != y.kind || x.offset != y.offset || x.elem_bytes != y.elem_bytes || x.ndim != y.ndim) return false;
      for (uint32_t k = 0; k < x.ndim; ++k)
        if (x.lo[k] != y.lo[k] || x.hi[k] != y.hi[k] || x.perm[k] != y.perm[k] || x.full_shape[k] != y.full_shape[k]) return false;
    }
    return true;
  };
  for (uint32_t r = 0; r < side.ranks.size(); ++r)
    if (!side.alive[r]) done[r] = 1;  // a destination rank that is not to be built belongs to no group: nothing is planned for it
  for (uint32_t r = 0; r < side.ranks.size(); ++r) {
    if (done[r]) continue;
    ReplicaGroup g{r, 1, 0};
    done[r] = 1;
    if (!side.ranks[r].empty())
      for (uint32_t q = r + 1; q < side.ranks.size(); ++q) {
        if (done[q] || !same_manifest(r, q)) continue;
        const uint32_t stride = q - r;
        if (stride > 255) break;
        g.stride = stride;
        for (uint32_t x = q; x < side.ranks.size() && g.count < 255 && !done[x] && same_manifest(r, x); x += stride) {
          done[x] = 1;
          ++g.count;
        }
        break;
      }
    side.groups.push_back(g);
  }
  return TPX_OK;
}

}  // namespace tpx

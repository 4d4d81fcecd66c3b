// Host planner: rank coordinates, tensor tables, copy descriptors and tiles for the
// train <-> generation weight reshard of the HybridFlow 3D-HybridEngine.
//
// Paper passages implemented here (arXiv 2409.19256):
//   Section 5.1  sizes: N = p*t*d = p_g*t_g*d_g*d, d_g = p*t/(p_g*t_g)
//   Section 5.3  grouping: training TP/PP groups are consecutive ranks and DP groups sit
//                at stride p*t; HybridFlow generation TP/PP groups take ranks at stride
//                t/t_g and p/p_g and micro-DP groups are consecutive ranks; the vanilla
//                variant reuses the training rule with the smaller sizes
//   Section 5.2  step 1 = gather of the updated parameters inside each micro-DP group,
//                step 4 = re-partition for training
//   Section 5.4  only the remote parameters of the micro-DP group are collected; the own
//                training shard is reused in place (zero redundancy)
// Pure host code: no HIP calls in this file.
#include "plan.hpp"

#include <algorithm>
#include <cstring>
#include <map>
#include <numeric>
#include <set>
#include <tuple>

namespace hf {

namespace {

constexpr uint64_t kTensorAlign = 256;
constexpr uint64_t kRankAlign = 4096;

uint64_t round_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

const int kTrainLayerIds[] = {HF_T_LN1, HF_T_QKV, HF_T_O, HF_T_LN2, HF_T_GATE_UP, HF_T_DOWN};
const int kGenLayerIds[] = {HF_G_LN1, HF_G_Q, HF_G_K, HF_G_V, HF_G_O, HF_G_LN2, HF_G_GATE, HF_G_UP, HF_G_DOWN};

// [rows, cols] of a training-shard tensor (Megatron layout, TP size t)
void train_shape(const hf_model_desc &m, int t, int id, uint32_t &rows, uint32_t &cols) {
  const uint32_t h = m.hidden, hd = m.head_dim;
  switch (id) {
  case HF_T_EMBED: case HF_T_HEAD: rows = m.vocab / t; cols = h; break;
  case HF_T_LN1: case HF_T_LN2: case HF_T_LNF: rows = 1; cols = h; break;
  case HF_T_QKV: rows = (uint32_t)(m.n_q_heads + 2 * m.n_kv_heads) / t * hd; cols = h; break;
  case HF_T_O: rows = h; cols = (uint32_t)m.n_q_heads * hd / t; break;
  case HF_T_GATE_UP: rows = 2u * m.ffn / t; cols = h; break;
  case HF_T_DOWN: rows = h; cols = (uint32_t)m.ffn / t; break;
  default: rows = cols = 0;
  }
}

// [rows, cols] of a generation-buffer tensor (separate q/k/v/gate/up, TP size tg)
void gen_shape(const hf_model_desc &m, int tg, int id, uint32_t &rows, uint32_t &cols) {
  const uint32_t h = m.hidden, hd = m.head_dim;
  switch (id) {
  case HF_G_EMBED: case HF_G_HEAD: rows = m.vocab / tg; cols = h; break;
  case HF_G_LN1: case HF_G_LN2: case HF_G_LNF: rows = 1; cols = h; break;
  case HF_G_Q: rows = (uint32_t)m.n_q_heads * hd / tg; cols = h; break;
  case HF_G_K: case HF_G_V: rows = (uint32_t)m.n_kv_heads * hd / tg; cols = h; break;
  case HF_G_O: rows = h; cols = (uint32_t)m.n_q_heads * hd / tg; break;
  case HF_G_GATE: case HF_G_UP: rows = (uint32_t)m.ffn / tg; cols = h; break;
  case HF_G_DOWN: rows = h; cols = (uint32_t)m.ffn / tg; break;
  default: rows = cols = 0;
  }
}

template <typename ShapeFn>
void lay_out(RankTable &tab, bool first, bool last, int layer0, int n_layers, const int *layer_ids, int n_ids,
             int id_embed, int id_lnf, int id_head, ShapeFn shape) {
  uint64_t off = 0;
  auto put = [&](int id, int layer) {
    TensorRec r;
    r.id = id;
    r.layer = layer;
    shape(id, r.rows, r.cols);
    off = round_up(off, kTensorAlign);
    r.off = off;
    off += (uint64_t)r.rows * r.cols * 2;
    tab.index[{id, layer}] = (int)tab.tensors.size();
    tab.tensors.push_back(r);
  };
  if (first) put(id_embed, -1);
  for (int l = layer0; l < layer0 + n_layers; ++l)
    for (int k = 0; k < n_ids; ++k) put(layer_ids[k], l);
  if (last) {
    put(id_lnf, -1);
    put(id_head, -1);
  }
  tab.size = round_up(off, kRankAlign);
}

uint32_t align_flag(uint64_t x) {
  if (x % 16 == 0) return HF_DESC_ALIGN16;
  if (x % 8 == 0) return HF_DESC_ALIGN8;
  if (x % 4 == 0) return HF_DESC_ALIGN4;
  return HF_DESC_ALIGN2;
}

// widest vector that divides every offset, size and (used) stride of the descriptor
uint32_t desc_align(const hf_desc &d) {
  uint64_t g = d.src_off | d.dst_off | d.row_bytes;
  if (d.rows > 1) g |= d.src_row_stride | d.dst_row_stride;
  if (d.n_blocks > 1) g |= d.src_block_stride | d.dst_block_stride;
  return align_flag(g); // low set bit of the OR = gcd with a power of two
}

struct Emitter {
  Plan &pl;
  int dst_rank;
  // offsets are relative to the START OF THE TENSOR on either side
  void add(int src_rank, const TensorRec &src_t, const TensorRec &dst_t, uint32_t kind, uint64_t src_delta,
           uint64_t dst_delta, uint32_t n_blocks, uint32_t rows, uint32_t row_bytes, uint64_t sbs, uint64_t dbs,
           uint64_t srs, uint64_t drs) {
    hf_desc d;
    std::memset(&d, 0, sizeof d);
    d.src_rank = src_rank;
    d.dst_rank = dst_rank;
    d.tensor_id = dst_t.id;
    d.layer = dst_t.layer;
    d.kind = kind;
    d.src_off = pl.train_tab[src_rank].base + src_t.off + src_delta;
    d.dst_off = pl.gen_tab[dst_rank].base + dst_t.off + dst_delta;
    d.n_blocks = n_blocks;
    d.rows = rows;
    d.row_bytes = row_bytes;
    d.src_block_stride = sbs;
    d.dst_block_stride = dbs;
    d.src_row_stride = srs;
    d.dst_row_stride = drs;
    if ((pl.flags & HF_GATHER_FROM_GEN) && src_rank != dst_rank) {
      // The peer is a member of the destination's micro-DP group: same generation stage and
      // TP index, hence the same generation tensors at the same offsets inside its region, and
      // the piece it trains sits there exactly where it is wanted here.
      d.src_off = pl.gen_tab[src_rank].base + dst_t.off + dst_delta;
      d.src_block_stride = dbs;
      d.src_row_stride = drs;
    }
    d.flags = desc_align(d) | (src_rank == dst_rank ? HF_DESC_OWN : 0u);
    (src_rank == dst_rank ? pl.fwd_own : pl.fwd_peer).push_back(d);
  }
};

} // namespace

uint64_t desc_bytes(const hf_desc &d) { return (uint64_t)d.n_blocks * d.rows * d.row_bytes; }

uint64_t unique_src_bytes(const std::vector<const hf_desc *> &descs) {
  // pieces read by several destinations are byte-identical descriptors on the source
  // side; different pieces never overlap (checked by validate_plan through coverage)
  std::set<std::tuple<uint64_t, uint64_t, uint32_t, uint32_t, uint32_t>> seen;
  uint64_t total = 0;
  for (const hf_desc *d : descs)
    if (seen.insert({d->src_off, d->src_block_stride, d->n_blocks, d->rows, d->row_bytes}).second)
      total += desc_bytes(*d);
  return total;
}

int build_plan(const hf_model_desc &m, const hf_train_layout &tl, const hf_gen_layout &gl, Plan &pl, std::string &err) {
  // ---- validation -------------------------------------------------------------
  const int32_t sizes[] = {m.n_layers, m.hidden, m.n_q_heads, m.n_kv_heads, m.head_dim, m.ffn, m.vocab,
                           tl.pp, tl.tp, tl.dp, gl.pp, gl.tp};
  for (int32_t v : sizes)
    if (v <= 0) { err = "all model and layout sizes must be positive"; return HF_EINVAL; }
  if (m.elem_bytes != 2) { err = "elem_bytes must be 2 (bf16)"; return HF_EINVAL; }
  if (m.tied_embed != 0) { err = "tied embedding / LM head is not supported"; return HF_EINVAL; }
  if (gl.flags & ~(HF_COPY_OWN | HF_GROUPING_VANILLA | HF_PLAN_HOST_ONLY | HF_PLAN_OFFLOAD | HF_GATHER_FROM_GEN)) { err = "unknown flag bits"; return HF_EINVAL; }
  if ((gl.flags & HF_GATHER_FROM_GEN) && (gl.flags & (HF_COPY_OWN | HF_GROUPING_VANILLA))) {
    err = "HF_GATHER_FROM_GEN needs the HybridFlow grouping and HF_SKIP_OWN: the own pieces are the source";
    return HF_EINVAL;
  }
  if (gl.mat_ranks && gl.n_mat <= 0) { err = "mat_ranks given but n_mat <= 0"; return HF_EINVAL; }
  struct { bool bad; const char *what; } div[] = {
      {tl.tp % gl.tp != 0, "t % t_g"}, {tl.pp % gl.pp != 0, "p % p_g"}, {m.n_layers % tl.pp != 0, "L % p"},
      {m.n_layers % gl.pp != 0, "L % p_g"}, {m.vocab % tl.tp != 0, "V % t"}, {m.ffn % tl.tp != 0, "F % t"},
      {m.n_q_heads % m.n_kv_heads != 0, "n_q % n_kv"}, {m.n_kv_heads % tl.tp != 0, "n_kv % t"},
      {m.n_kv_heads % gl.tp != 0, "n_kv % t_g"}};
  for (auto &c : div)
    if (c.bad) { err = std::string("not divisible: ") + c.what; return HF_EDIVIS; }
  const int64_t n64 = (int64_t)tl.pp * tl.tp * tl.dp;
  if (n64 > (1 << 20)) { err = "too many ranks"; return HF_ERANGE; }
  // row lengths and block strides must fit 32-bit fields of descriptors and tiles
  const uint64_t widest_row = 2ull * std::max<uint64_t>(m.hidden, std::max<uint64_t>(m.ffn, (uint64_t)m.n_q_heads * m.head_dim));
  const uint64_t qkv_group = 2ull * ((uint64_t)m.n_q_heads / m.n_kv_heads + 2) * m.head_dim * m.hidden;
  if (widest_row >= (1ull << 31) || qkv_group >= (1ull << 32)) { err = "tensor rows too long for 32-bit strides"; return HF_ERANGE; }

  pl.m = m;
  pl.p = tl.pp; pl.t = tl.tp; pl.d = tl.dp; pl.pg = gl.pp; pl.tg = gl.tp;
  pl.flags = gl.flags;
  pl.multicast_auto = true; // build_tiles picks the mode from the fan-out of the list
  pl.a = pl.t / pl.tg;
  pl.b = pl.p / pl.pg;
  pl.dg = pl.a * pl.b;
  pl.N = (int)n64;
  pl.lps = m.n_layers / pl.p;
  pl.lpgs = m.n_layers / pl.pg;
  const int N = pl.N, p = pl.p, t = pl.t, pg = pl.pg, tg = pl.tg, a = pl.a, b = pl.b;
  const bool vanilla = (gl.flags & HF_GROUPING_VANILLA) != 0;

  // ---- materialised ranks ------------------------------------------------------
  pl.mat_pos.assign(N, -1);
  if (gl.mat_ranks) {
    for (int i = 0; i < gl.n_mat; ++i) {
      const int r = gl.mat_ranks[i];
      if (r < 0 || r >= N) { err = "materialised rank out of range"; return HF_ERANGE; }
      if (pl.mat_pos[r] >= 0) { err = "materialised rank listed twice"; return HF_ERANGE; }
      pl.mat_pos[r] = i;
      pl.mat.push_back(r);
    }
  } else {
    for (int r = 0; r < N; ++r) { pl.mat_pos[r] = r; pl.mat.push_back(r); }
  }

  // ---- rank coordinates ----------------------------------------------------------
  pl.coords.resize(N);
  for (int r = 0; r < N; ++r) {
    Coords &c = pl.coords[r];
    c.dp = r / (p * t);
    c.pp = (r % (p * t)) / t;
    c.tp = r % t;
    if (!vanilla) {
      // generation TP peers are t/t_g training ranks apart and generation PP peers p/p_g
      // stages apart: quotient = generation index, remainder = place in the micro-DP group
      c.gtp = c.tp / a;
      c.gpp = c.pp / b;
      c.micro = (c.pp % b) * a + (c.tp % a);
    } else {
      const int i = c.pp * t + c.tp; // place inside the replica; consecutive ranks per group
      c.gtp = i % tg;
      c.gpp = (i / tg) % pg;
      c.micro = i / (tg * pg);
    }
  }

  // micro-DP groups: the d_g ranks of a replica that share (gpp, gtp), by micro-DP index
  pl.micro_peers.assign((size_t)N * pl.dg, -1);
  for (int r = 0; r < N; ++r)
    for (int q = 0; q < N; ++q) {
      const Coords &x = pl.coords[r], &y = pl.coords[q];
      if (x.dp == y.dp && x.gpp == y.gpp && x.gtp == y.gtp) pl.micro_peers[(size_t)r * pl.dg + y.micro] = q;
    }
  for (int32_t q : pl.micro_peers)
    if (q < 0) { err = "internal: incomplete micro-DP group"; return HF_EINVAL; }

  // ---- tensor tables -----------------------------------------------------------
  pl.train_tab.assign(N, RankTable());
  pl.gen_tab.assign(N, RankTable());
  uint64_t base = 0;
  for (int r = 0; r < N; ++r) {
    const Coords &c = pl.coords[r];
    lay_out(pl.train_tab[r], c.pp == 0, c.pp == p - 1, c.pp * pl.lps, pl.lps, kTrainLayerIds, 6, HF_T_EMBED, HF_T_LNF,
            HF_T_HEAD, [&](int id, uint32_t &rows, uint32_t &cols) { train_shape(m, t, id, rows, cols); });
    pl.train_tab[r].base = base;
    base += pl.train_tab[r].size;
    lay_out(pl.gen_tab[r], c.gpp == 0, c.gpp == pg - 1, c.gpp * pl.lpgs, pl.lpgs, kGenLayerIds, 9, HF_G_EMBED, HF_G_LNF,
            HF_G_HEAD, [&](int id, uint32_t &rows, uint32_t &cols) { gen_shape(m, tg, id, rows, cols); });
  }
  pl.train_bytes = base;
  base = 0;
  for (int r : pl.mat) {
    pl.gen_tab[r].base = base;
    base += pl.gen_tab[r].size;
  }
  pl.gen_bytes = base;

  // ---- step 1 descriptors: for every materialised rank, every generation tensor, every
  // training shard that contributes to it ------------------------------------------
  const uint64_t h2 = 2ull * m.hidden;                 // bytes of one [*, h] row
  const uint32_t hd = m.head_dim, qpg = m.n_q_heads / m.n_kv_heads;
  const uint32_t ng = m.n_kv_heads / t;                // KV groups per training shard
  const uint64_t grp = (uint64_t)(qpg + 2) * hd * h2;  // bytes of one fused [q..q k v] group
  for (int r : pl.mat) {
    const Coords &c = pl.coords[r];
    Emitter em{pl, r};
    auto rank_of = [&](int pp, int tp) { return c.dp * p * t + pp * t + tp; };
    for (const TensorRec &g : pl.gen_tab[r].tensors) {
      // training stage that owns the tensor
      const int spp = g.id == HF_G_EMBED ? 0 : (g.id == HF_G_LNF || g.id == HF_G_HEAD) ? p - 1 : g.layer / pl.lps;
      if (g.id == HF_G_LN1 || g.id == HF_G_LN2 || g.id == HF_G_LNF) {
        // replicated: take the copy of the rank with the same TP index in the owning stage
        const int q = rank_of(spp, c.tp);
        if ((gl.flags & HF_GATHER_FROM_GEN) && pl.mat_pos[q] < 0) { err = "HF_GATHER_FROM_GEN: a micro-DP peer of a materialised rank is not materialised"; return HF_EINVAL; }
        const int tid = g.id == HF_G_LN1 ? HF_T_LN1 : g.id == HF_G_LN2 ? HF_T_LN2 : HF_T_LNF;
        em.add(q, pl.train_tab[q].at(tid, g.layer), g, HF_REPL, 0, 0, 1, 1, (uint32_t)h2, h2, h2, h2, h2);
        continue;
      }
      for (int k = 0; k < a; ++k) {                    // the a training TP shards inside generation shard gtp
        const int q = rank_of(spp, c.gtp * a + k);
        if ((gl.flags & HF_GATHER_FROM_GEN) && pl.mat_pos[q] < 0) { err = "HF_GATHER_FROM_GEN: a micro-DP peer of a materialised rank is not materialised"; return HF_EINVAL; }
        const RankTable &st = pl.train_tab[q];
        switch (g.id) {
        case HF_G_EMBED: case HF_G_HEAD: {
          const TensorRec &s = st.at(g.id == HF_G_EMBED ? HF_T_EMBED : HF_T_HEAD, -1);
          em.add(q, s, g, HF_COL, 0, (uint64_t)k * s.rows * h2, 1, s.rows, (uint32_t)h2, 0, 0, h2, h2);
          break;
        }
        case HF_G_Q: case HF_G_K: case HF_G_V: {
          const TensorRec &s = st.at(HF_T_QKV, g.layer);
          const uint32_t rows = g.id == HF_G_Q ? qpg * hd : hd;             // rows of one group's piece
          const uint64_t in_group = g.id == HF_G_Q ? 0 : g.id == HF_G_K ? (uint64_t)qpg * hd * h2 : (uint64_t)(qpg + 1) * hd * h2;
          em.add(q, s, g, HF_QKV_DEINT, in_group, (uint64_t)k * ng * rows * h2, ng, rows, (uint32_t)h2, grp,
                 (uint64_t)rows * h2, h2, h2);
          break;
        }
        case HF_G_GATE: case HF_G_UP: {
          const TensorRec &s = st.at(HF_T_GATE_UP, g.layer);
          const uint32_t rows = s.rows / 2;                                  // F/t
          em.add(q, s, g, HF_GATEUP_DEINT, g.id == HF_G_GATE ? 0 : (uint64_t)rows * h2, (uint64_t)k * rows * h2, 1, rows,
                 (uint32_t)h2, 0, 0, h2, h2);
          break;
        }
        case HF_G_O: case HF_G_DOWN: {
          const TensorRec &s = st.at(g.id == HF_G_O ? HF_T_O : HF_T_DOWN, g.layer);
          em.add(q, s, g, HF_ROW, 0, (uint64_t)k * s.cols * 2, 1, s.rows, s.cols * 2, 0, 0, (uint64_t)s.cols * 2,
                 (uint64_t)g.cols * 2);
          break;
        }
        default: err = "internal: unknown generation tensor"; return HF_EINVAL;
        }
      }
    }
  }

  // ---- step 4 descriptors: the own pieces, run backwards ----------------------------
  if (!vanilla) {
    pl.back.reserve(pl.fwd_own.size());
    for (const hf_desc &o : pl.fwd_own) {
      hf_desc d = o;
      std::swap(d.src_off, d.dst_off);
      std::swap(d.src_block_stride, d.dst_block_stride);
      std::swap(d.src_row_stride, d.dst_row_stride);
      pl.back.push_back(d);
    }
  }

  // ---- offload image of the remote pieces (Section 7: the generation copy of the weights
  // leaves the GPU while the model trains).  The peer descriptors of one (rank, generation
  // tensor) are consecutive and ordered by the position of their piece in the tensor, so
  // the remote elements of the tensor in row-major order are: for column-parallel kinds the
  // pieces one after another, for row-parallel kinds a matrix [rows, n_remote * piece cols].
  // Tensor parts start at 256-byte boundaries, rank parts at 4096-byte boundaries.
  {
    uint64_t hoff = 0;
    int cur_rank = -1;
    for (size_t i = 0; i < pl.fwd_peer.size();) {
      const hf_desc &d0 = pl.fwd_peer[i];
      size_t j = i + 1;
      while (j < pl.fwd_peer.size() && pl.fwd_peer[j].dst_rank == d0.dst_rank && pl.fwd_peer[j].tensor_id == d0.tensor_id &&
             pl.fwd_peer[j].layer == d0.layer)
        ++j;
      if (d0.dst_rank != cur_rank) {
        // ranks appear in buffer order; a rank without remote pieces gets an empty part
        while (pl.remote_rank_off.size() <= (size_t)pl.mat_pos[d0.dst_rank]) {
          hoff = round_up(hoff, kRankAlign);
          pl.remote_rank_off.push_back(hoff);
        }
        cur_rank = d0.dst_rank;
      }
      hoff = round_up(hoff, kTensorAlign);
      const uint64_t n_remote = j - i;
      for (size_t k = i; k < j; ++k) {
        const hf_desc &f = pl.fwd_peer[k];
        hf_desc d;
        std::memset(&d, 0, sizeof d);
        d.src_rank = d.dst_rank = f.dst_rank;
        d.tensor_id = f.tensor_id;
        d.layer = f.layer;
        d.kind = f.kind;
        d.src_off = f.dst_off;
        d.n_blocks = 1;
        d.row_bytes = f.row_bytes;
        if (f.kind == HF_ROW) {
          d.rows = f.rows;
          d.src_row_stride = f.dst_row_stride;
          d.dst_row_stride = n_remote * f.row_bytes;
          d.dst_off = hoff + (k - i) * f.row_bytes;
        } else { // contiguous in the generation tensor
          d.rows = f.n_blocks * f.rows;
          d.src_row_stride = d.dst_row_stride = f.row_bytes;
          d.dst_off = hoff + (k - i) * desc_bytes(f);
        }
        d.src_block_stride = (uint64_t)d.rows * d.src_row_stride;
        d.dst_block_stride = (uint64_t)d.rows * d.dst_row_stride;
        d.flags = desc_align(d);
        pl.remote.push_back(d);
      }
      hoff += n_remote * desc_bytes(d0);
      i = j;
    }
    while (pl.remote_rank_off.size() < pl.mat.size()) {
      hoff = round_up(hoff, kRankAlign);
      pl.remote_rank_off.push_back(hoff);
    }
    pl.remote_bytes = round_up(hoff, kRankAlign);
  }
  return build_tiles(pl, err);
}

// ---- tiler --------------------------------------------------------------------------
namespace {

uint32_t vec_of(uint64_t g) { return g % 16 == 0 ? 16 : g % 8 == 0 ? 8 : g % 4 == 0 ? 4 : 2; }

void push_tile(std::vector<hf_tile> &out, uint64_t src, uint64_t dst, uint32_t rows, uint32_t row_bytes, uint32_t sstr,
               uint32_t dstr) {
  hf_tile tl;
  std::memset(&tl, 0, sizeof tl);
  tl.src_off = src;
  tl.dst_off = dst;
  tl.rows = rows;
  tl.row_bytes = row_bytes;
  tl.src_row_stride = rows > 1 ? sstr : row_bytes;
  tl.dst_row_stride = rows > 1 ? dstr : row_bytes;
  uint64_t g = src | dst | row_bytes;
  if (rows > 1) g |= (uint64_t)sstr | dstr;
  tl.vec_bytes = vec_of(g);
  tl.n_dst = 1;
  out.push_back(tl);
}

// one contiguous run of `len` bytes -> chunks of about tile_bytes, cut at 256-byte steps
void tile_run(std::vector<hf_tile> &out, uint64_t src, uint64_t dst, uint64_t len, uint64_t tile_bytes) {
  const uint64_t n = (len + tile_bytes - 1) / tile_bytes;
  const uint64_t chunk = round_up((len + n - 1) / n, 256);
  for (uint64_t o = 0; o < len; o += chunk) push_tile(out, src + o, dst + o, 1, (uint32_t)std::min(chunk, len - o), 0, 0);
}

void tile_desc(std::vector<hf_tile> &out, const hf_desc &d, uint64_t tile_bytes) {
  const bool rows_contig = d.rows == 1 || (d.src_row_stride == d.row_bytes && d.dst_row_stride == d.row_bytes);
  const uint64_t block_len = (uint64_t)d.rows * d.row_bytes;
  const bool blocks_contig = d.n_blocks == 1 || (d.src_block_stride == block_len && d.dst_block_stride == block_len);
  if (rows_contig && blocks_contig) {
    tile_run(out, d.src_off, d.dst_off, block_len * d.n_blocks, tile_bytes);
    return;
  }
  for (uint32_t bidx = 0; bidx < d.n_blocks; ++bidx) {
    const uint64_t s = d.src_off + bidx * d.src_block_stride, t = d.dst_off + bidx * d.dst_block_stride;
    if (rows_contig) {
      tile_run(out, s, t, block_len, tile_bytes);
    } else if (d.row_bytes >= tile_bytes) {
      for (uint32_t r = 0; r < d.rows; ++r) tile_run(out, s + r * d.src_row_stride, t + r * d.dst_row_stride, d.row_bytes, tile_bytes);
    } else {
      // rows per tile: about tile_bytes of payload, and offsets inside a tile below 4 GiB
      // (the kernel computes row*stride in 32 bits)
      const uint64_t widest = std::max(d.src_row_stride, d.dst_row_stride);
      const uint64_t fit = ((1ull << 32) - 1 - d.row_bytes) / std::max<uint64_t>(widest, 1) + 1;
      const uint32_t per = (uint32_t)std::max<uint64_t>(1, std::min(tile_bytes / d.row_bytes, fit));
      for (uint32_t r = 0; r < d.rows; r += per)
        push_tile(out, s + r * d.src_row_stride, t + r * d.dst_row_stride, std::min(per, d.rows - r), d.row_bytes,
                  (uint32_t)d.src_row_stride, (uint32_t)d.dst_row_stride);
    }
  }
}

} // namespace

// Multicast mode when the caller leaves the choice to the library, from the list's fan-out
// (bytes written per distinct byte read).  Measured on the Llama-7B, 13B and 34B shapes under
// training TP 8 (and TP 4 x PP 2) with generation TP 1, 2, 4, own pieces in the list or not, in
// several processes on several machines:
//   2 destinations per piece: registers and prefetched level, cache-blocked 3-5 % behind;
//   3: prefetched 1-3 % ahead of cache-blocked on average and never behind it; registers
//      between 3 % ahead and 10 % behind from process to process;
//   4: prefetched 3-8 % ahead of the others;
//   7 and 8: prefetched and registers level, cache-blocked 10-13 % behind.
int64_t default_multicast(const Plan &pl) {
  if (!pl.unique_bytes[0]) return HF_MULTICAST_PREFETCHED;
  const double fan = (double)pl.moved_bytes[0] / (double)pl.unique_bytes[0];
  return fan < 2.5 ? HF_MULTICAST_REGISTERS : HF_MULTICAST_PREFETCHED;
}

// Copy tiles per chunked load-only tile of the prefetched list when the caller leaves it to
// the library.  Measured on the same workloads: two chunks against one gain 7 % at 3
// destinations per piece (Llama-7B TP8->TP2: 8.29 against 8.88 ms), 3 % at 4, nothing at 7
// and 8; four and eight chunks lose the gain again at 3 and 4 and are level at 7 and 8.
int64_t default_prefetch_merge(const Plan &) { return 2; }

namespace {

bool wanted(const Plan &pl, const hf_desc &d) { return (pl.kind_mask >> d.kind) & 1; }

// one-destination lists in descriptor order, except that a run of row-parallel
// descriptors into the same destination tensor (its column stripes) is tiled round-robin,
// for the DRAM-row reason given at the multicast list below
void tile_list(const Plan &pl, const std::vector<hf_desc> &descs, std::vector<hf_tile> &out) {
  std::vector<std::vector<hf_tile>> run;
  for (size_t i = 0; i < descs.size();) {
    if (!wanted(pl, descs[i])) { ++i; continue; }
    size_t j = i + 1;
    if (descs[i].kind == HF_ROW && pl.row_interleave)
      while (j < descs.size() && descs[j].kind == HF_ROW && descs[j].dst_rank == descs[i].dst_rank &&
             descs[j].tensor_id == descs[i].tensor_id && descs[j].layer == descs[i].layer)
        ++j;
    if (j == i + 1) {
      tile_desc(out, descs[i], (uint64_t)pl.tile_bytes);
    } else {
      run.assign(j - i, {});
      size_t longest = 0;
      for (size_t k = i; k < j; ++k) {
        tile_desc(run[k - i], descs[k], (uint64_t)pl.tile_bytes);
        longest = std::max(longest, run[k - i].size());
      }
      for (size_t t = 0; t < longest; ++t)
        for (auto &r : run)
          if (t < r.size()) out.push_back(r[t]);
    }
    i = j;
  }
}

// one-destination lists of all four directions
void build_plain_lists(Plan &pl) {
  pl.tiles_fwd.clear();
  pl.tiles_back.clear();
  tile_list(pl, pl.fwd_peer, pl.tiles_fwd);
  pl.n_tiles_fwd_peer = pl.tiles_fwd.size();
  tile_list(pl, pl.fwd_own, pl.tiles_fwd);
  tile_list(pl, pl.back, pl.tiles_back);
  pl.tiles_offload.clear();
  pl.tiles_reload.clear();
  if (pl.flags & HF_PLAN_OFFLOAD) {
    for (const hf_desc &d : pl.remote) tile_desc(pl.tiles_offload, d, (uint64_t)pl.tile_bytes);
    pl.tiles_reload = pl.tiles_offload;
    for (hf_tile &t : pl.tiles_reload) {
      std::swap(t.src_off, t.dst_off);
      std::swap(t.src_row_stride, t.dst_row_stride);
    }
  }
}

// totals of the descriptors that take part (queried on the hot path of harnesses)
void cache_totals(Plan &pl) {
  std::vector<const hf_desc *> fwd, back;
  for (const hf_desc &d : pl.fwd_peer) if (wanted(pl, d)) fwd.push_back(&d);
  if (pl.flags & HF_COPY_OWN)
    for (const hf_desc &d : pl.fwd_own) if (wanted(pl, d)) fwd.push_back(&d);
  for (const hf_desc &d : pl.back) if (wanted(pl, d)) back.push_back(&d);
  pl.moved_bytes[0] = pl.moved_bytes[1] = 0;
  for (const hf_desc *d : fwd) pl.moved_bytes[0] += desc_bytes(*d);
  for (const hf_desc *d : back) pl.moved_bytes[1] += desc_bytes(*d);
  pl.unique_bytes[0] = unique_src_bytes(fwd);
  pl.unique_bytes[1] = unique_src_bytes(back);
}

// multicast list over the descriptors execute performs: same source bytes and same
// geometry -> one tile with several destinations, in order of first appearance
int build_multicast_list(Plan &pl, std::string &err) {
  pl.tiles_fwd_mc.clear();
  pl.mc_dst.clear();
  std::vector<const hf_desc *> active;
  for (const hf_desc &d : pl.fwd_peer) if (wanted(pl, d)) active.push_back(&d);
  if (pl.flags & HF_COPY_OWN)
    for (const hf_desc &d : pl.fwd_own) if (wanted(pl, d)) active.push_back(&d);
  typedef std::tuple<uint64_t, uint32_t, uint32_t, uint32_t, uint64_t, uint64_t, uint64_t, uint64_t> Key;
  std::map<Key, size_t> group_of;
  std::vector<std::vector<const hf_desc *>> groups;
  for (const hf_desc *d : active) {
    const Key k{d->src_off, d->n_blocks, d->rows, d->row_bytes, d->src_block_stride, d->src_row_stride,
                d->dst_block_stride, d->dst_row_stride};
    auto it = group_of.find(k);
    if (it == group_of.end()) {
      group_of[k] = groups.size();
      groups.push_back({d});
    } else {
      groups[it->second].push_back(d);
    }
  }
  pl.has_sharing = false;
  for (const auto &g : groups) pl.has_sharing = pl.has_sharing || g.size() > 1;
  // tiles of every group (destinations 2..n already appended to mc_dst)
  std::vector<std::vector<hf_tile>> group_tiles(groups.size());
  for (size_t gi = 0; gi < groups.size(); ++gi) {
    const auto &grp_descs = groups[gi];
    const hf_desc &d0 = *grp_descs[0];
    tile_desc(group_tiles[gi], d0, (uint64_t)pl.tile_bytes);
    for (hf_tile &tl : group_tiles[gi]) {
      tl.n_dst = (uint32_t)grp_descs.size();
      tl.dst_list = (uint32_t)pl.mc_dst.size();
      uint64_t g = tl.vec_bytes; // already covers source, first destination, sizes, strides
      for (size_t j = 1; j < grp_descs.size(); ++j) {
        const uint64_t off = tl.dst_off - d0.dst_off + grp_descs[j]->dst_off;
        pl.mc_dst.push_back(off);
        g |= off;
      }
      tl.vec_bytes = vec_of(g);
    }
  }
  // Row-parallel tensors: the a training pieces of one generation tensor are column
  // stripes of the same destination rows.  Their tiles are emitted round-robin (rows
  // 0..R of every piece, then the next rows of every piece, ...) so that each
  // destination row is completed while it is still open in DRAM, instead of being
  // visited once per stripe with a fraction of a row each time.
  typedef std::tuple<int, int, int, int, int> SibKey; // tensor, layer, dp, gpp, gtp of the destination
  std::map<SibKey, std::vector<size_t>> siblings;
  for (size_t gi = 0; gi < groups.size(); ++gi) {
    const hf_desc &d0 = *groups[gi][0];
    if (d0.kind != HF_ROW || !pl.row_interleave) continue;
    const Coords &c = pl.coords[d0.dst_rank];
    siblings[SibKey{d0.tensor_id, d0.layer, c.dp, c.gpp, c.gtp}].push_back(gi);
  }
  std::vector<char> emitted(groups.size(), 0);
  for (size_t gi = 0; gi < groups.size(); ++gi) {
    if (emitted[gi]) continue;
    const hf_desc &d0 = *groups[gi][0];
    std::vector<size_t> set{gi};
    if (d0.kind == HF_ROW && pl.row_interleave) {
      const Coords &c = pl.coords[d0.dst_rank];
      set = siblings[SibKey{d0.tensor_id, d0.layer, c.dp, c.gpp, c.gtp}];
    }
    size_t longest = 0;
    for (size_t g2 : set) { emitted[g2] = 1; longest = std::max(longest, group_tiles[g2].size()); }
    for (size_t i = 0; i < longest; ++i)
      for (size_t g2 : set)
        if (i < group_tiles[g2].size()) pl.tiles_fwd_mc.push_back(group_tiles[g2][i]);
  }
  if (pl.mc_dst.size() >= (1ull << 32)) { err = "too many multicast destinations; raise the tile size"; return HF_ERANGE; }
  return HF_OK;
}

// cache-blocked multicast order: the same work as one-destination tiles, arranged so that
// a block of at most mc_block_bytes of source is copied to its first destination, then
// the same block to the second, ...: only the first pass reads HBM, the later passes
// find the block in L2 (workgroups are handed out in list order, and the workgroup that
// copies a given source part runs on the same XCD in every pass because each pass spans
// a whole number of tiles with a fixed number of workgroups per tile).
void build_cache_blocked_list(Plan &pl) {
  pl.tiles_fwd_cb.clear();
  std::vector<const hf_tile *> batch;
  uint64_t batch_bytes = 0;
  auto flush = [&]() {
    if (batch.empty()) return;
    for (uint32_t j = 0; j < batch[0]->n_dst; ++j)
      for (const hf_tile *t : batch) {
        hf_tile one = *t;
        one.dst_off = j == 0 ? t->dst_off : pl.mc_dst[t->dst_list + j - 1];
        one.n_dst = 1;
        one.dst_list = 0;
        pl.tiles_fwd_cb.push_back(one);
      }
    batch.clear();
    batch_bytes = 0;
  };
  for (const hf_tile &t : pl.tiles_fwd_mc) {
    const uint64_t payload = (uint64_t)t.rows * t.row_bytes;
    if (!batch.empty() && (t.n_dst != batch[0]->n_dst || batch_bytes + payload > (uint64_t)pl.mc_block_bytes)) flush();
    batch.push_back(&t);
    batch_bytes += payload;
  }
  flush();
}

// prefetched multicast order: the multicast tiles in blocks of at most prefetch_block_bytes of
// source; in front of every block the load-only tiles (n_dst == 0) that bring its shared
// source bytes into L2.  A shared tile whose source is one contiguous run takes part in a
// chunked load-only tile (dst_list = number of chunks): up to prefetch_merge tiles of the
// block that follow one another in the source and have the same size share one, and the
// group with part number k of that tile loads part k of every chunk.  A shared tile with a
// strided source gets a load-only copy of itself.  Every tile, load-only or not, takes the
// same number of workgroups (a multiple of 8), so the group that loads part k of a chunk and
// the group that copies part k of it run on the same XCD and share its L2.
void build_prefetched_list(Plan &pl) {
  pl.tiles_fwd_pf.clear();
  std::vector<const hf_tile *> batch;
  uint64_t batch_bytes = 0;
  const uint32_t merge = (uint32_t)std::max<int64_t>(1, std::min<int64_t>(pl.effective_prefetch_merge(), HF_MAX_PREFETCH_CHUNKS));
  std::map<uint64_t, size_t> open; // source offset a chain would continue at -> its load-only tile
  auto flush = [&]() {
    open.clear();
    for (const hf_tile *t : batch) {
      if (t->n_dst <= 1) continue; // a piece with one destination is read once anyway
      const uint64_t payload = (uint64_t)t->rows * t->row_bytes;
      const bool flat = t->rows == 1 || t->src_row_stride == t->row_bytes;
      if (!flat || t->src_off % 16 || payload % 16) {
        hf_tile pre = *t;
        pre.n_dst = 0;
        pre.dst_list = 0;
        pl.tiles_fwd_pf.push_back(pre);
        continue;
      }
      auto it = open.find(t->src_off);
      if (it != open.end() && pl.tiles_fwd_pf[it->second].row_bytes == payload) {
        const size_t at = it->second;
        hf_tile &pre = pl.tiles_fwd_pf[at];
        pre.rows = ++pre.dst_list;
        open.erase(it);
        if (pre.dst_list < merge) open[t->src_off + payload] = at;
        continue;
      }
      hf_tile pre;
      std::memset(&pre, 0, sizeof pre);
      pre.src_off = t->src_off;
      pre.rows = 1;
      pre.row_bytes = (uint32_t)payload;
      pre.src_row_stride = pre.dst_row_stride = (uint32_t)payload;
      pre.vec_bytes = 16;
      pre.dst_list = 1;
      if (merge > 1) open[t->src_off + payload] = pl.tiles_fwd_pf.size();
      pl.tiles_fwd_pf.push_back(pre);
    }
    for (const hf_tile *t : batch) pl.tiles_fwd_pf.push_back(*t);
    batch.clear();
    batch_bytes = 0;
  };
  for (const hf_tile &t : pl.tiles_fwd_mc) {
    const uint64_t payload = (uint64_t)t.rows * t.row_bytes;
    if (!batch.empty() && batch_bytes + payload > (uint64_t)pl.prefetch_block_bytes) flush();
    batch.push_back(&t);
    batch_bytes += payload;
  }
  flush();
}

} // namespace

int build_tiles(Plan &pl, std::string &err) {
  if (pl.tile_bytes < 4096 || pl.tile_bytes > (4 << 20) || pl.tile_bytes % 4096) {
    err = "tile bytes must be a multiple of 4096 in [4096, 4 MiB]";
    return HF_EINVAL;
  }
  build_plain_lists(pl);
  cache_totals(pl);
  if (int rc = build_multicast_list(pl, err)) return rc;
  build_cache_blocked_list(pl);
  build_prefetched_list(pl);
  if (pl.multicast_auto) pl.multicast = default_multicast(pl);
  if (pl.tiles_fwd.size() >= (1ull << 31) || pl.tiles_back.size() >= (1ull << 31)) {
    err = "too many tiles; raise the tile size";
    return HF_ERANGE;
  }
  return HF_OK;
}

// ---- validation -------------------------------------------------------------------------
namespace {

struct Seg { uint64_t dst, src, len; };

void desc_segments(const hf_desc &d, std::vector<Seg> &out) {
  for (uint32_t b = 0; b < d.n_blocks; ++b)
    for (uint32_t r = 0; r < d.rows; ++r)
      out.push_back({d.dst_off + b * d.dst_block_stride + r * d.dst_row_stride,
                     d.src_off + b * d.src_block_stride + r * d.src_row_stride, d.row_bytes});
}

void tile_segments(const hf_tile &t, std::vector<Seg> &out) {
  for (uint32_t r = 0; r < t.rows; ++r)
    out.push_back({t.dst_off + (uint64_t)r * t.dst_row_stride, t.src_off + (uint64_t)r * t.src_row_stride, t.row_bytes});
}

// sort by destination and merge neighbours that are contiguous on both sides
bool normalise(std::vector<Seg> &v, std::string &err, const char *what) {
  std::sort(v.begin(), v.end(), [](const Seg &x, const Seg &y) { return x.dst < y.dst; });
  std::vector<Seg> m;
  for (const Seg &s : v) {
    if (!m.empty()) {
      Seg &l = m.back();
      if (l.dst + l.len > s.dst) { err = std::string(what) + ": overlapping destinations"; return false; }
      if (l.dst + l.len == s.dst && l.src + l.len == s.src) { l.len += s.len; continue; }
    }
    m.push_back(s);
  }
  v.swap(m);
  return true;
}

bool same(const std::vector<Seg> &x, const std::vector<Seg> &y) {
  if (x.size() != y.size()) return false;
  for (size_t i = 0; i < x.size(); ++i)
    if (x[i].dst != y[i].dst || x[i].src != y[i].src || x[i].len != y[i].len) return false;
  return true;
}

int train_id_of(int gen_id) {
  switch (gen_id) {
  case HF_G_EMBED: return HF_T_EMBED;
  case HF_G_HEAD: return HF_T_HEAD;
  case HF_G_LN1: return HF_T_LN1;
  case HF_G_LN2: return HF_T_LN2;
  case HF_G_LNF: return HF_T_LNF;
  case HF_G_Q: case HF_G_K: case HF_G_V: return HF_T_QKV;
  case HF_G_O: return HF_T_O;
  case HF_G_GATE: case HF_G_UP: return HF_T_GATE_UP;
  case HF_G_DOWN: return HF_T_DOWN;
  }
  return -1;
}

} // namespace

int validate_plan(const Plan &pl, std::string &err) {
  if (pl.kind_mask != 0x1F) { err = "plan is restricted to some descriptor kinds (hf_debug_restrict_kinds)"; return HF_EINVAL; }
  // (1) every descriptor stays inside the payload of the tensors it names
  auto inside = [&](const hf_desc &d, bool forward) -> bool {
    const int train_rank = forward ? d.src_rank : d.dst_rank, gen_rank = forward ? d.dst_rank : d.src_rank;
    const RankTable &tt = pl.train_tab[train_rank], &gt = pl.gen_tab[gen_rank];
    const TensorRec &tr = tt.at(train_id_of(d.tensor_id), d.layer), &gr = gt.at(d.tensor_id, d.layer);
    const uint64_t t0 = tt.base + tr.off, t1 = t0 + 2ull * tr.rows * tr.cols;
    const uint64_t g0 = gt.base + gr.off, g1 = g0 + 2ull * gr.rows * gr.cols;
    const uint64_t s_lo = d.src_off, s_hi = d.src_off + (d.n_blocks - 1) * d.src_block_stride + (d.rows - 1) * d.src_row_stride + d.row_bytes;
    const uint64_t d_lo = d.dst_off, d_hi = d.dst_off + (d.n_blocks - 1) * d.dst_block_stride + (d.rows - 1) * d.dst_row_stride + d.row_bytes;
    if (forward && (pl.flags & HF_GATHER_FROM_GEN) && d.src_rank != d.dst_rank) {
      const RankTable &sg = pl.gen_tab[d.src_rank];
      if (pl.mat_pos[d.src_rank] < 0) return false;
      const TensorRec &sr = sg.at(d.tensor_id, d.layer);
      const uint64_t q0 = sg.base + sr.off, q1 = q0 + 2ull * sr.rows * sr.cols;
      return s_lo >= q0 && s_hi <= q1 && d_lo >= g0 && d_hi <= g1;
    }
    if (forward) return s_lo >= t0 && s_hi <= t1 && d_lo >= g0 && d_hi <= g1;
    return s_lo >= g0 && s_hi <= g1 && d_lo >= t0 && d_hi <= t1;
  };
  for (const hf_desc &d : pl.fwd_peer) if (!inside(d, true)) { err = "peer descriptor leaves its tensor"; return HF_ERANGE; }
  for (const hf_desc &d : pl.fwd_own) if (!inside(d, true)) { err = "own descriptor leaves its tensor"; return HF_ERANGE; }
  for (const hf_desc &d : pl.back) if (!inside(d, false)) { err = "reverse descriptor leaves its tensor"; return HF_ERANGE; }

  // (2) destinations pairwise disjoint, and together exactly the payload
  std::vector<Seg> fwd, fwd_peer_only, back;
  for (const hf_desc &d : pl.fwd_peer) desc_segments(d, fwd);
  fwd_peer_only = fwd;
  for (const hf_desc &d : pl.fwd_own) desc_segments(d, fwd);
  for (const hf_desc &d : pl.back) desc_segments(d, back);
  uint64_t gen_payload = 0, train_payload = 0, fwd_total = 0, back_total = 0;
  for (int r : pl.mat) {
    for (const TensorRec &g : pl.gen_tab[r].tensors) gen_payload += 2ull * g.rows * g.cols;
    for (const TensorRec &s : pl.train_tab[r].tensors) train_payload += 2ull * s.rows * s.cols;
  }
  for (const Seg &s : fwd) fwd_total += s.len;
  for (const Seg &s : back) back_total += s.len;
  if (!normalise(fwd, err, "train->gen") || !normalise(back, err, "gen->train")) return HF_ERANGE;
  if (fwd_total != gen_payload) { err = "train->gen descriptors do not cover the generation payload"; return HF_ERANGE; }
  if (!(pl.flags & HF_GROUPING_VANILLA) && back_total != train_payload) {
    err = "gen->train descriptors do not cover the training payload";
    return HF_ERANGE;
  }

  // (3) the tiles are exactly the descriptors
  std::vector<Seg> tf, tf_peer, tb;
  for (size_t i = 0; i < pl.tiles_fwd.size(); ++i) {
    tile_segments(pl.tiles_fwd[i], tf);
    if (i + 1 == pl.n_tiles_fwd_peer) tf_peer = tf;
  }
  for (const hf_tile &t : pl.tiles_back) tile_segments(t, tb);
  if (!normalise(tf, err, "train->gen tiles") || !normalise(tb, err, "gen->train tiles") ||
      !normalise(tf_peer, err, "peer tiles") || !normalise(fwd_peer_only, err, "peer descriptors"))
    return HF_ERANGE;
  if (!same(tf, fwd) || !same(tb, back) || !same(tf_peer, fwd_peer_only)) { err = "tiles differ from descriptors"; return HF_ERANGE; }
  // the multicast list, expanded per destination, is the list execute would run one by one
  std::vector<Seg> mc;
  for (const hf_tile &t : pl.tiles_fwd_mc) {
    if (t.n_dst == 0 || (t.n_dst > 1 && (uint64_t)t.dst_list + t.n_dst - 1 > pl.mc_dst.size())) { err = "multicast tile: bad destination list"; return HF_ERANGE; }
    for (uint32_t k = 0; k < t.n_dst; ++k) {
      hf_tile one = t;
      one.dst_off = k == 0 ? t.dst_off : pl.mc_dst[t.dst_list + k - 1];
      uint64_t g = one.src_off | one.dst_off | one.row_bytes;
      if (one.rows > 1) g |= (uint64_t)one.src_row_stride | one.dst_row_stride;
      if (g % t.vec_bytes) { err = "multicast tile alignment wrong"; return HF_ERANGE; }
      tile_segments(one, mc);
    }
  }
  if (!normalise(mc, err, "multicast tiles")) return HF_ERANGE;
  if (!same(mc, (pl.flags & HF_COPY_OWN) ? fwd : fwd_peer_only)) { err = "multicast tiles differ from descriptors"; return HF_ERANGE; }
  std::vector<Seg> cb;
  for (const hf_tile &t : pl.tiles_fwd_cb) {
    if (t.n_dst != 1) { err = "cache-blocked tile with several destinations"; return HF_ERANGE; }
    tile_segments(t, cb);
  }
  if (!normalise(cb, err, "cache-blocked tiles")) return HF_ERANGE;
  if (!same(cb, mc)) { err = "cache-blocked tiles differ from descriptors"; return HF_ERANGE; }
  // the prefetched list without its load-only tiles is the multicast list, and in every block
  // the load-only tiles read exactly the source bytes of the block's shared tiles
  {
    size_t k = 0;
    typedef std::pair<uint64_t, uint64_t> Run; // source offset, length
    std::vector<Run> pre, shared;
    auto tidy = [](std::vector<Run> &v) {
      std::sort(v.begin(), v.end());
      std::vector<Run> m;
      for (const Run &r : v) {
        if (!m.empty() && m.back().first + m.back().second == r.first) m.back().second += r.second;
        else m.push_back(r);
      }
      v.swap(m);
    };
    auto close_block = [&]() {
      tidy(pre);
      tidy(shared);
      const bool ok = pre == shared;
      pre.clear();
      shared.clear();
      return ok;
    };
    bool copying = false;
    for (const hf_tile &t : pl.tiles_fwd_pf) {
      if (t.n_dst == 0) {
        if (copying && !close_block()) { err = "prefetched list: load-only tiles do not cover the shared tiles of their block"; return HF_ERANGE; }
        copying = false;
        if (t.dst_list > HF_MAX_PREFETCH_CHUNKS || (t.dst_list && (t.rows != t.dst_list || t.src_off % 16 || t.row_bytes % 16 || t.vec_bytes != 16))) {
          err = "prefetched list: malformed chunked load-only tile";
          return HF_ERANGE;
        }
        for (uint32_t r = 0; r < t.rows; ++r) pre.push_back({t.src_off + (uint64_t)r * t.src_row_stride, t.row_bytes});
        continue;
      }
      copying = true;
      if (k >= pl.tiles_fwd_mc.size() || std::memcmp(&t, &pl.tiles_fwd_mc[k], sizeof t) != 0) { err = "prefetched list differs from the multicast list"; return HF_ERANGE; }
      ++k;
      if (t.n_dst > 1)
        for (uint32_t r = 0; r < t.rows; ++r) shared.push_back({t.src_off + (uint64_t)r * t.src_row_stride, t.row_bytes});
    }
    if (k != pl.tiles_fwd_mc.size() || !close_block()) { err = "prefetched list: load-only tiles do not cover the shared tiles of their block"; return HF_ERANGE; }
  }
  // (3b) gathering out of the generation buffers: every source lies inside an own piece of
  // its rank (resident, and never a destination of the same launch)
  if (pl.flags & HF_GATHER_FROM_GEN) {
    std::vector<Seg> own;
    for (const hf_desc &d : pl.fwd_own) desc_segments(d, own);
    for (Seg &s : own) s.src = s.dst;
    if (!normalise(own, err, "own pieces")) return HF_ERANGE;
    std::vector<Seg> srcs;
    for (const hf_desc &d : pl.fwd_peer) desc_segments(d, srcs);
    for (const Seg &s : srcs) {
      // last own interval that starts at or before the source segment
      auto it = std::upper_bound(own.begin(), own.end(), s.src, [](uint64_t v, const Seg &o) { return v < o.dst; });
      if (it == own.begin() || (--it, s.src + s.len > it->dst + it->len)) { err = "a gather source is not inside an own piece"; return HF_ERANGE; }
    }
  }

  // (4) offload image: its generation side is exactly the peer destinations, its host side
  // is pairwise disjoint and inside the image; the offload tiles are its descriptors
  {
    std::vector<Seg> gen_side, host_side, peers = fwd_peer_only, tiles;
    for (const hf_desc &d : pl.remote) {
      std::vector<Seg> one;
      desc_segments(d, one); // Seg.dst = host image offset, Seg.src = generation offset
      for (const Seg &s : one) {
        if (s.dst + s.len > pl.remote_bytes) { err = "offload descriptor leaves the image"; return HF_ERANGE; }
        host_side.push_back(s);
        gen_side.push_back({s.src, s.src, s.len});
      }
    }
    for (Seg &s : peers) s.src = s.dst; // compare coverage of gen_buf only
    std::vector<Seg> host_sorted = host_side;
    if (!normalise(host_sorted, err, "offload image") || !normalise(gen_side, err, "offload sources") ||
        !normalise(peers, err, "peer destinations"))
      return HF_ERANGE;
    if (!same(gen_side, peers)) { err = "offload image does not cover the remote pieces"; return HF_ERANGE; }
    if (pl.flags & HF_PLAN_OFFLOAD) {
      for (const hf_tile &t : pl.tiles_offload) tile_segments(t, tiles);
      if (!normalise(tiles, err, "offload tiles")) return HF_ERANGE;
      if (!same(tiles, host_sorted)) { err = "offload tiles differ from descriptors"; return HF_ERANGE; }
      if (pl.tiles_reload.size() != pl.tiles_offload.size()) { err = "reload tiles differ from offload tiles"; return HF_ERANGE; }
      for (size_t i = 0; i < pl.tiles_reload.size(); ++i) {
        const hf_tile &x = pl.tiles_offload[i], &y = pl.tiles_reload[i];
        if (x.src_off != y.dst_off || x.dst_off != y.src_off || x.src_row_stride != y.dst_row_stride ||
            x.dst_row_stride != y.src_row_stride || x.rows != y.rows || x.row_bytes != y.row_bytes || x.vec_bytes != y.vec_bytes) {
          err = "reload tiles differ from offload tiles";
          return HF_ERANGE;
        }
      }
    }
  }
  for (const std::vector<hf_tile> *lst : {&pl.tiles_fwd, &pl.tiles_back, &pl.tiles_offload, &pl.tiles_reload})
    for (const hf_tile &t : *lst) {
      uint64_t g = t.src_off | t.dst_off | t.row_bytes;
      if (t.rows > 1) g |= (uint64_t)t.src_row_stride | t.dst_row_stride;
      if (g % t.vec_bytes || t.row_bytes == 0 || t.rows == 0) { err = "tile alignment wrong"; return HF_ERANGE; }
    }
  return HF_OK;
}

} // namespace hf

// Internal representation of a reshard plan (host side).  Not part of the ABI.
#pragma once

#include <cstdint>
#include <map>
#include <string>
#include <utility>
#include <vector>

#include "hfreshard.h"

namespace hf {

// Position of a rank in the training grid and in the generation grid
// (HybridFlow Section 5.1 for the sizes, Section 5.3 for the grouping rules).
struct Coords {
  int dp, pp, tp;      // training: r = dp*p*t + pp*t + tp
  int gpp, gtp, micro; // generation stage, generation TP index, index in the micro-DP group
};

struct TensorRec {
  int id;        // HF_T_* or HF_G_*
  int layer;     // global layer, -1 for embed / lnf / head
  uint32_t rows, cols;
  uint64_t off;  // bytes from the start of the rank region
};

struct RankTable {
  std::vector<TensorRec> tensors;
  std::map<std::pair<int, int>, int> index; // (id, layer) -> position in `tensors`
  uint64_t size = 0;                        // region bytes (multiple of 4096)
  uint64_t base = 0;                        // bytes from the buffer base
  const TensorRec &at(int id, int layer) const { return tensors[index.at({id, layer})]; }
};

struct Plan {
  hf_model_desc m{};
  int p = 0, t = 0, d = 0, pg = 0, tg = 0;
  uint32_t flags = 0;
  int a = 0, b = 0, dg = 0, N = 0;
  int lps = 0, lpgs = 0; // layers per training / generation stage
  std::vector<int> mat;     // materialised ranks in buffer order
  std::vector<int> mat_pos; // rank -> position in `mat`, -1 if absent
  std::vector<Coords> coords;
  std::vector<int32_t> micro_peers; // [rank * dg + j] = rank with micro-DP index j in rank's micro-DP group
  std::vector<RankTable> train_tab, gen_tab; // per rank (gen_tab[r].base valid only if materialised)
  uint64_t train_bytes = 0, gen_bytes = 0;

  // step 1 (train -> gen): pieces from micro-DP peers, and pieces from the rank's own shard
  std::vector<hf_desc> fwd_peer, fwd_own;
  // step 4 (gen -> train): inverse of the own pieces
  std::vector<hf_desc> back;
  // offload image (host side of hf_offload_remote / hf_reload_remote): one descriptor per
  // peer descriptor, src_off = where the piece sits in gen_buf, dst_off = where it sits in
  // the packed host image; remote_rank_off[i] = start of the i-th materialised rank's part
  std::vector<hf_desc> remote;
  std::vector<uint64_t> remote_rank_off;
  uint64_t remote_bytes = 0;

  // device work lists; tiles_fwd = [peer tiles | own tiles], one destination per tile
  std::vector<hf_tile> tiles_fwd, tiles_back;
  size_t n_tiles_fwd_peer = 0;
  // multicast work list for execute: descriptors that read the same training piece are
  // tiled once; destinations 2..n of every tile are in mc_dst
  std::vector<hf_tile> tiles_fwd_mc;
  std::vector<uint64_t> mc_dst;
  // the same work, one destination per tile, in cache-blocked order (see build_tiles)
  std::vector<hf_tile> tiles_fwd_cb;
  // the multicast list with a prefetch tile (n_dst == 0: loaded, stored nowhere) for every tile,
  // block-wise in front of the tiles themselves (see build_tiles)
  std::vector<hf_tile> tiles_fwd_pf;
  // offload / reload work lists (only with HF_PLAN_OFFLOAD): gen_buf -> image and back
  std::vector<hf_tile> tiles_offload, tiles_reload;
  bool has_sharing = false; // some training piece has more than one destination
  // multicast mode that execute really uses: without sharing the multicast lists are the
  // one-destination work in another order, and the plain list with streaming loads is faster
  int64_t effective_prefetch_merge() const;
  int64_t effective_multicast() const { return has_sharing ? multicast : (int64_t)HF_MULTICAST_OFF; }
  // host copy of the work list hf_reshard_execute runs in the current mode, and its length
  const std::vector<hf_tile> &active_fwd() const {
    switch (effective_multicast()) {
    case HF_MULTICAST_REGISTERS: return tiles_fwd_mc;
    case HF_MULTICAST_CACHE_BLOCKED: return tiles_fwd_cb;
    case HF_MULTICAST_PREFETCHED: return tiles_fwd_pf;
    default: return tiles_fwd;
    }
  }
  size_t active_fwd_count() const {
    return effective_multicast() == HF_MULTICAST_OFF && !(flags & HF_COPY_OWN) ? n_tiles_fwd_peer : active_fwd().size();
  }
  bool active_fwd_uses_mc_dst() const {
    return effective_multicast() == HF_MULTICAST_REGISTERS || effective_multicast() == HF_MULTICAST_PREFETCHED;
  }

  int64_t tile_bytes = 128 * 1024;
  int64_t grid_wgs = 2048;
  int64_t variant = HF_VARIANT_PARTS;
  int64_t multicast = HF_MULTICAST_CACHE_BLOCKED;
  bool multicast_auto = true; // the mode follows the list's fan-out until the caller names one
  int64_t mc_block_bytes = 2 << 20;
  int64_t prefetch_block_bytes = 6 << 20; // measured over identical buffer placements: 6 MiB is 0.5-2.6 % ahead of 8 MiB on the 7B and 13B
                                          // shapes at 3 to 7 destinations per piece and level on the 34B shape; 4 MiB and 10+ MiB are behind
  int64_t prefetch_merge = 0; // copy tiles per chunked load-only tile; 0 = chosen from the fan-out
  int64_t cache_policy = -1; // auto
  int64_t part_bytes = 0; // 0 = chosen per launch
  int64_t max_wgs_per_launch = 0xFFFFFFFFll / 256; // a grid holds fewer than 2^32 threads
  int64_t wg_threads = 0; // 0 = chosen per launch
  int64_t kind_mask = 0x1F; // bit k: descriptors of kind k take part (hf_debug_restrict_kinds)
  int64_t offload_wgs = 8; // persistent workgroups of the offload / reload kernels
  int64_t row_interleave = 1; // tiles of the column stripes of one row-parallel tensor go out round-robin
  // totals of the descriptors that take part, per direction (set by build_tiles)
  uint64_t moved_bytes[2] = {0, 0}, unique_bytes[2] = {0, 0};

  // changes whenever the work lists change: tells hf_reshard_execute_static whether the list
  // it staged for this plan is still the current one
  uint64_t serial = 0;

  // device copy (null for HF_PLAN_HOST_ONLY)
  int device = -1;
  // Only the lists the current multicast mode needs are resident: d_tiles_fwd (the whole
  // one-destination list) for HF_MULTICAST_OFF, d_tiles_fwd_mc + d_mc_dst for
  // HF_MULTICAST_REGISTERS, d_tiles_fwd_cb for HF_MULTICAST_CACHE_BLOCKED, d_tiles_fwd_pf +
  // d_mc_dst for HF_MULTICAST_PREFETCHED; the own tiles
  // (hf_reshard_install_own), the reverse list and the group table always.
  hf_tile *d_tiles_fwd = nullptr;
  hf_tile *d_tiles_own = nullptr;
  hf_tile *d_tiles_back = nullptr;
  hf_tile *d_tiles_fwd_mc = nullptr;
  hf_tile *d_tiles_fwd_cb = nullptr;
  hf_tile *d_tiles_fwd_pf = nullptr;
  hf_tile *d_tiles_offload = nullptr;
  hf_tile *d_tiles_reload = nullptr;
  uint64_t *d_mc_dst = nullptr;
  int32_t *d_micro_peers = nullptr;
};

// Builds everything except the device copy.  Returns HF_OK or an error, with `err` set.
int build_plan(const hf_model_desc &m, const hf_train_layout &tl, const hf_gen_layout &gl, Plan &out, std::string &err);
// (Re)creates the tile lists from the descriptors with out.tile_bytes.
int build_tiles(Plan &pl, std::string &err);
int64_t default_multicast(const Plan &pl); // needs the byte totals build_tiles sets
int64_t default_prefetch_merge(const Plan &pl); // likewise
inline int64_t Plan::effective_prefetch_merge() const { return prefetch_merge ? prefetch_merge : default_prefetch_merge(*this); }
// Host-side consistency check (see hf_plan_validate).
int validate_plan(const Plan &pl, std::string &err);
uint64_t desc_bytes(const hf_desc &d);
uint64_t unique_src_bytes(const std::vector<const hf_desc *> &descs);

} // namespace hf

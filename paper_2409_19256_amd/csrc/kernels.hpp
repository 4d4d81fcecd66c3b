// Launch interface between the C ABI and the device code.  Not part of the ABI.
#pragma once
#include <cstddef>
#include <cstdint>

#include "hfreshard.h"

namespace hf {
// Enqueues the kernel(s) that execute tiles[0..n_tiles) (DEVICE pointer) on `stream`;
// extra_dst (DEVICE pointer, may be null if every tile has n_dst == 1) holds the
// destinations 2..n_dst of multicast tiles; src/dst are the buffers the tile offsets are
// relative to (device memory, or pinned host memory through its device address).
// tile_bytes = the tiler's tile size.  HF_VARIANT_PARTS (the default): one short-lived
// workgroup of wg_threads lanes (64 or 256) per part_bytes of every tile, part_bytes =
// 1, 2, 4 or 8 vectors of 16 bytes per lane (1..8 KiB with 64 lanes, 4..32 KiB with 256).
// The persistent variants take grid_wgs workgroups of 256 lanes instead.  Returns a
// hipError_t value (0 = success).  max_wgs_per_launch: upper bound of the grid of one
// launch for the variants whose grid grows with the work (at most (2^32-1)/256).  list_tag
// (HF_VARIANT_PARTS only) goes into the kernel's name and nowhere else: 0 = train->gen
// without own pieces, 1 = train->gen with own pieces, 2 = any other list.  Never allocates
// or synchronises.
int launch_tiles(const hf_tile *d_tiles, size_t n_tiles, const uint64_t *extra_dst, const void *src, void *dst,
                 int variant, int grid_wgs, int cache_policy, uint32_t tile_bytes, uint32_t part_bytes,
                 uint32_t max_wgs_per_launch, int wg_threads, int list_tag, void *stream);
// out slot (pair) <- in slot peers[pair] for pair in [0, n_pairs), slots of slot_bytes bytes
// (multiple of 4).  Returns a hipError_t value.
int launch_gather_slots(const int32_t *d_peers, uint32_t n_pairs, const void *in, void *out, size_t slot_bytes,
                        void *stream);
// One read, n_dst writes of known traffic (see hf_calib_fanout).  Returns a hipError_t value.
int launch_calib_fanout(const void *src, void *dst, size_t bytes, int n_dst, size_t dst_stride, int method, size_t block_bytes,
                        int wg_bytes, void *stream);
// Plain grid-stride 16-byte copy (calibration); src == null: write only, dst == null: read only.
int launch_calib_copy(const void *src, void *dst, size_t bytes, void *stream);
} // namespace hf

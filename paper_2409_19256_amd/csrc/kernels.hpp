// Launch interface between the C ABI and the device code.  Not part of the ABI.
#pragma once
#include <cstddef>
#include <cstdint>

#include "hfreshard.h"

namespace hf {
// Enqueues one kernel that executes tiles[0..n_tiles) (DEVICE pointer) on `stream`;
// extra_dst (DEVICE pointer, may be null if every tile has n_dst == 1) holds the
// destinations 2..n_dst of multicast tiles; src/dst are the device buffers the tile
// offsets are relative to.  tile_bytes = the tiler's tile size, part_bytes = payload per
// workgroup of HF_VARIANT_PARTS (4096, 8192, 16384 or 32768).  Returns a hipError_t value
// (0 = success).  max_wgs_per_launch: upper bound of the grid of one launch for the
// variants whose grid grows with the work (at most (2^32-1)/256).  Never allocates or
// synchronises.  wg_threads: 256, or 64 (HF_VARIANT_PARTS only: part_bytes is then 1..8 KiB).
int launch_tiles(const hf_tile *d_tiles, size_t n_tiles, const uint64_t *extra_dst, const void *src, void *dst,
                 int variant, int grid_wgs, int cache_policy, uint32_t tile_bytes, uint32_t part_bytes,
                 uint32_t max_wgs_per_launch, int wg_threads, void *stream);
// out slot (pair) <- in slot peers[pair] for pair in [0, n_pairs), slots of slot_bytes bytes
// (multiple of 4).  Returns a hipError_t value.
int launch_gather_slots(const int32_t *d_peers, uint32_t n_pairs, const void *in, void *out, size_t slot_bytes,
                        void *stream);
// Plain grid-stride 16-byte copy (calibration); src == null: write only, dst == null: read only.
int launch_calib_copy(const void *src, void *dst, size_t bytes, void *stream);
} // namespace hf

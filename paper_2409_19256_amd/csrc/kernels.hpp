// Launch interface between the C ABI and the device code.  Not part of the ABI.
#pragma once
#include <cstddef>

#include "hfreshard.h"

namespace hf {
// Enqueues one kernel that executes tiles[0..n_tiles) (DEVICE pointer) on `stream`;
// src/dst are the device buffers the tile offsets are relative to.  Returns a hipError_t
// value (0 = success).  Never allocates or synchronises.
int launch_tiles(const hf_tile *d_tiles, size_t n_tiles, const void *src, void *dst, int variant, int grid_wgs,
                 void *stream);
} // namespace hf

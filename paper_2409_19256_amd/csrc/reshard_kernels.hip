// gfx950 copy kernels that execute a reshard plan's tile list.
//
// The work is pure data movement (HybridFlow Section 5.2 steps 1 and 4 re-arrange
// parameters, they compute nothing), so the kernels are shaped for HBM bandwidth:
// every lane moves 16 bytes per access (8/4/2 when a tile is less aligned), a wavefront
// therefore touches 1 KiB of consecutive bytes per instruction, eight independent loads
// are issued per lane before the first store so that each CU keeps tens of KiB in
// flight, and the grid is a fixed number of persistent workgroups that stride over the
// tile list (tile i -> workgroup i mod grid), which keeps the workgroups that run at the
// same time on neighbouring tiles of the same tensors.  No MFMA: there is no arithmetic.
#include <hip/hip_runtime.h>

#include "hfreshard.h"
#include "kernels.hpp"

namespace hf {

namespace {

constexpr int kWG = 256;    // threads per workgroup = 4 wavefronts of 64
constexpr int kUnroll = 8;  // independent accesses in flight per lane

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <typename V> __device__ __forceinline__ V load_stream(const char *p) {
  return __builtin_nontemporal_load(reinterpret_cast<const V *>(p));
}
template <typename V> __device__ __forceinline__ void store_stream(char *p, V v) {
  __builtin_nontemporal_store(v, reinterpret_cast<V *>(p));
}

// rows x row_bytes, element (row, i) at base + row*stride + i on either side.
// Vector index v in [0, rows*vpr) maps to row = v / vpr, column = v % vpr, so lanes of a
// wavefront walk consecutive bytes of a row and spill into the next row at its end.
template <typename V>
__device__ __forceinline__ void copy_tile(const char *__restrict__ src, char *__restrict__ dst, uint32_t rows,
                                          uint32_t row_bytes, uint32_t sstr, uint32_t dstr) {
  const uint32_t vpr = row_bytes / (uint32_t)sizeof(V);
  const uint32_t total = rows * vpr;
  if (rows == 1) {
    for (uint32_t i0 = threadIdx.x; i0 < total; i0 += kUnroll * kWG) {
      V v[kUnroll];
#pragma unroll
      for (int k = 0; k < kUnroll; ++k) {
        const uint32_t i = i0 + k * kWG;
        if (i < total) v[k] = load_stream<V>(src + (uint64_t)i * sizeof(V));
      }
#pragma unroll
      for (int k = 0; k < kUnroll; ++k) {
        const uint32_t i = i0 + k * kWG;
        if (i < total) store_stream<V>(dst + (uint64_t)i * sizeof(V), v[k]);
      }
    }
    return;
  }
  for (uint32_t i0 = threadIdx.x; i0 < total; i0 += kUnroll * kWG) {
    V v[kUnroll];
    uint32_t doff[kUnroll];
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) {
      const uint32_t i = i0 + k * kWG;
      const uint32_t row = i / vpr, col = (i - row * vpr) * (uint32_t)sizeof(V);
      doff[k] = row * dstr + col; // tile extents stay far below 4 GiB
      if (i < total) v[k] = load_stream<V>(src + (row * sstr + col));
    }
#pragma unroll
    for (int k = 0; k < kUnroll; ++k)
      if (i0 + k * kWG < total) store_stream<V>(dst + doff[k], v[k]);
  }
}

__device__ __forceinline__ void run_tile(const hf_tile &tl, const char *__restrict__ src, char *__restrict__ dst) {
  const char *s = src + tl.src_off;
  char *d = dst + tl.dst_off;
  switch (tl.vec_bytes) { // uniform over the workgroup
  case 16: copy_tile<u32x4>(s, d, tl.rows, tl.row_bytes, tl.src_row_stride, tl.dst_row_stride); break;
  case 8: copy_tile<u32x2>(s, d, tl.rows, tl.row_bytes, tl.src_row_stride, tl.dst_row_stride); break;
  case 4: copy_tile<uint32_t>(s, d, tl.rows, tl.row_bytes, tl.src_row_stride, tl.dst_row_stride); break;
  default: copy_tile<uint16_t>(s, d, tl.rows, tl.row_bytes, tl.src_row_stride, tl.dst_row_stride); break;
  }
}

// Persistent workgroups: workgroup w copies tiles w, w+grid, w+2*grid, ...  Every
// workgroup leaves the loop after at most ceil(n/grid) rounds; there is no waiting on
// other workgroups anywhere.
__global__ __launch_bounds__(kWG) void reshard_persistent(const hf_tile *__restrict__ tiles, uint32_t n_tiles,
                                                          const char *__restrict__ src, char *__restrict__ dst) {
  for (uint32_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
    const hf_tile tl = tiles[t];
    run_tile(tl, src, dst);
  }
}

__global__ __launch_bounds__(kWG) void reshard_one_tile(const hf_tile *__restrict__ tiles, uint32_t n_tiles,
                                                        const char *__restrict__ src, char *__restrict__ dst) {
  const uint32_t t = blockIdx.x;
  if (t < n_tiles) {
    const hf_tile tl = tiles[t];
    run_tile(tl, src, dst);
  }
}

// Tile staged through LDS in 16 KiB slabs: global -> registers -> LDS, barrier,
// LDS -> registers -> global.  Exists to measure whether staging buys anything for the
// block-level permutations of this path (it moves the same HBM bytes).
constexpr uint32_t kSlab = 16 * 1024;
template <typename V>
__device__ __forceinline__ void copy_tile_lds(const char *__restrict__ src, char *__restrict__ dst, uint32_t rows,
                                              uint32_t row_bytes, uint32_t sstr, uint32_t dstr, char *lds) {
  const uint32_t vpr = row_bytes / (uint32_t)sizeof(V);
  const uint32_t total = rows * vpr;
  constexpr uint32_t per_slab = kSlab / (uint32_t)sizeof(V);
  V *stage = reinterpret_cast<V *>(lds);
  for (uint32_t base = 0; base < total; base += per_slab) {
    const uint32_t n = min(per_slab, total - base);
    for (uint32_t j = threadIdx.x; j < n; j += kWG) {
      const uint32_t i = base + j;
      const uint32_t row = i / vpr, col = (i - row * vpr) * (uint32_t)sizeof(V);
      stage[j] = load_stream<V>(src + (row * sstr + col));
    }
    __syncthreads();
    for (uint32_t j = threadIdx.x; j < n; j += kWG) {
      const uint32_t i = base + j;
      const uint32_t row = i / vpr, col = (i - row * vpr) * (uint32_t)sizeof(V);
      store_stream<V>(dst + (row * dstr + col), stage[j]);
    }
    __syncthreads();
  }
}

__global__ __launch_bounds__(kWG) void reshard_persistent_lds(const hf_tile *__restrict__ tiles, uint32_t n_tiles,
                                                              const char *__restrict__ src, char *__restrict__ dst) {
  __shared__ __attribute__((aligned(16))) char lds[kSlab];
  for (uint32_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
    const hf_tile tl = tiles[t];
    const char *s = src + tl.src_off;
    char *d = dst + tl.dst_off;
    switch (tl.vec_bytes) {
    case 16: copy_tile_lds<u32x4>(s, d, tl.rows, tl.row_bytes, tl.src_row_stride, tl.dst_row_stride, lds); break;
    case 8: copy_tile_lds<u32x2>(s, d, tl.rows, tl.row_bytes, tl.src_row_stride, tl.dst_row_stride, lds); break;
    case 4: copy_tile_lds<uint32_t>(s, d, tl.rows, tl.row_bytes, tl.src_row_stride, tl.dst_row_stride, lds); break;
    default: copy_tile_lds<uint16_t>(s, d, tl.rows, tl.row_bytes, tl.src_row_stride, tl.dst_row_stride, lds); break;
    }
  }
}

} // namespace

int launch_tiles(const hf_tile *d_tiles, size_t n_tiles, const void *src, void *dst, int variant, int grid_wgs,
                 void *stream) {
  if (n_tiles == 0) return 0;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const char *s = static_cast<const char *>(src);
  char *d = static_cast<char *>(dst);
  const uint32_t n = (uint32_t)n_tiles;
  switch (variant) {
  case HF_VARIANT_ONE_WG_PER_TILE:
    hipLaunchKernelGGL(reshard_one_tile, dim3(n), dim3(kWG), 0, st, d_tiles, n, s, d);
    break;
  case HF_VARIANT_LDS_STAGED:
    hipLaunchKernelGGL(reshard_persistent_lds, dim3((uint32_t)std::min<size_t>(n_tiles, (size_t)grid_wgs)), dim3(kWG), 0, st,
                       d_tiles, n, s, d);
    break;
  default:
    hipLaunchKernelGGL(reshard_persistent, dim3((uint32_t)std::min<size_t>(n_tiles, (size_t)grid_wgs)), dim3(kWG), 0, st,
                       d_tiles, n, s, d);
    break;
  }
  return (int)hipGetLastError();
}

} // namespace hf

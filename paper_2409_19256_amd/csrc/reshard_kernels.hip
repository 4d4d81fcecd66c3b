// gfx950 copy kernels that execute a reshard plan's tile list.
//
// The work is pure data movement (HybridFlow Section 5.2 steps 1 and 4 re-arrange
// parameters, they compute nothing), so the kernels are shaped for HBM bandwidth and use
// no MFMA and, in the default path, no LDS.  Every lane moves 16 bytes per access (8/4/2
// when a tile is less aligned), so a wavefront touches 1 KiB of consecutive bytes per
// instruction.
//
// Default kernel, reshard_parts: the tile list (tiles of about 128 KiB) is cut into parts
// of 1 to 8 KiB and every part gets its own short-lived workgroup of 64 or 256 lanes,
// which loads its one or two vectors per lane, stores them and exits.  The hardware
// dispatcher hands out workgroups in index order, so the chip works on one narrow window
// of source and destination addresses that moves through the list, and a slow CU simply
// takes fewer workgroups.  One training piece wanted by several ranks of a micro-DP group
// (Section 5.3) is served by tiles that name several destinations (loaded once, stored to
// each), by default with load-only tiles in front of every block of the list that bring the
// block into the L2 of the XCD that will copy it (prefetched list), or by listing its tiles
// once per destination in an order that lets L2 serve the re-reads (cache-blocked list).
//
// Kept beside it, selectable per plan, for measurements: persistent workgroups that stride
// over the tile list, the same with one wavefront per stride (wavefront-level dispatch),
// the same staged through LDS, and one workgroup per tile.  The persistent kernel also
// carries the offload / reload of the remote pieces, where the host link is the bound and
// few workgroups are wanted.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "hfreshard.h"
#include "kernels.hpp"

namespace hf {

namespace {

constexpr int kWG = 256;    // threads per workgroup = 4 wavefronts of 64
constexpr int kWave = 64;
constexpr int kMaxUnroll = 8;  // independent accesses in flight per lane (persistent kernels)

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Cache policy of the streaming accesses: bit 0 = plain (temporal) loads instead of
// non-temporal ones; bit 1 = plain stores; bit 2 = non-temporal stores through the
// compiler builtin (`nt`) instead of the default `sc0 sc1 nt` (system-scope, streaming)
// 16-byte store.  Every byte is touched once, so nothing is worth keeping in L2 except the
// source block of the cache-blocked multicast list (plain loads there).  Measured on a
// one-shot 1:1 copy of 8 GiB: stores `sc0 sc1 nt` 6.74 TB/s vs `nt` 6.66 TB/s with 64-lane
// workgroups, 6.66 vs 6.42 TB/s with 256-lane workgroups; plain stores 6.55 / 6.37 TB/s.
template <typename V, int kPolicy> __device__ __forceinline__ V load_stream(const char *p) {
  if constexpr (kPolicy & 1) return *reinterpret_cast<const V *>(p);
  else return __builtin_nontemporal_load(reinterpret_cast<const V *>(p));
}
template <typename V, int kPolicy> __device__ __forceinline__ void store_stream(char *p, V v) {
  if constexpr (kPolicy & 2) {
    *reinterpret_cast<V *>(p) = v;
  } else if constexpr (sizeof(V) == 16 && !(kPolicy & 4)) {
    // a vector store like any other to the hardware; the compiler's own wait counts stay
    // correct because an extra outstanding store can only make its vmcnt waits longer.  The
    // compiler does not see a memory instruction here, so the wait state gfx9 wants between
    // a store of more than 64 bits and a vector instruction that overwrites its data
    // registers is supplied by hand.
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt\n\ts_nop 0" : : "v"(p), "v"(v) : "memory");
  } else {
    __builtin_nontemporal_store(v, reinterpret_cast<V *>(p));
  }
}

// a loaded value is "used" without any store: an empty instruction sequence that takes
// its registers as inputs keeps the load from being optimised away
__device__ __forceinline__ void keep_alive(const u32x4 &v) { asm volatile("" : : "v"(v.x), "v"(v.y), "v"(v.z), "v"(v.w)); }
__device__ __forceinline__ void keep_alive(const u32x2 &v) { asm volatile("" : : "v"(v.x), "v"(v.y)); }
__device__ __forceinline__ void keep_alive(uint32_t v) { asm volatile("" : : "v"(v)); }
__device__ __forceinline__ void keep_alive(uint16_t v) { asm volatile("" : : "v"((uint32_t)v)); }

// rows x row_bytes, byte (row, i) at base + row*stride + i on either side, copied by a
// group of kGroup consecutive lanes (a workgroup or one wavefront); `lane` is the index
// inside the group.  Vector index v in [0, rows*vpr) maps to row = v / vpr, column =
// v % vpr, so the lanes of a wavefront walk consecutive bytes of a row and spill into
// the next row at its end.  The loaded vectors are stored to n_dst destinations; a tile
// with n_dst == 0 is only loaded (it brings its source into L2 for a later tile).
// `part`/`part_bytes`: the group copies only bytes [part*part_bytes, (part+1)*part_bytes)
// of the tile's payload (part_bytes == 0: the whole tile).
template <typename V, int kGroup, int kPolicy, int kUnroll>
__device__ __forceinline__ void copy_tile(const hf_tile &tl, const uint64_t *__restrict__ extra_dst,
                                          const char *__restrict__ src_base, char *__restrict__ dst_base, uint32_t lane,
                                          uint32_t part, uint32_t part_bytes) {
  const char *__restrict__ src = src_base + tl.src_off;
  const uint32_t rows = tl.rows, sstr = tl.src_row_stride, dstr = tl.dst_row_stride;
  const uint32_t vpr = tl.row_bytes / (uint32_t)sizeof(V);
  uint32_t total = rows * vpr, first = 0;
  if (part_bytes) {
    const uint32_t per = part_bytes / (uint32_t)sizeof(V);
    first = min(part * per, total);
    total = min(first + per, total);
  }
  for (uint32_t i0 = first + lane; i0 < total; i0 += kUnroll * kGroup) {
    V v[kUnroll];
    uint32_t doff[kUnroll];
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) {
      const uint32_t i = i0 + k * kGroup;
      uint32_t soff;
      if (rows == 1) {
        soff = doff[k] = i * (uint32_t)sizeof(V);
      } else {
        const uint32_t row = i / vpr, col = (i - row * vpr) * (uint32_t)sizeof(V);
        soff = row * sstr + col; // the tiler keeps offsets inside a tile below 4 GiB
        doff[k] = row * dstr + col;
      }
      if (i < total) v[k] = load_stream<V, kPolicy>(src + soff);
    }
    if (tl.n_dst == 0) { // uniform
#pragma unroll
      for (int k = 0; k < kUnroll; ++k)
        if (i0 + k * kGroup < total) keep_alive(v[k]);
      continue;
    }
    for (uint32_t j = 0; j < tl.n_dst; ++j) { // uniform trip count
      char *__restrict__ dst = dst_base + (j == 0 ? tl.dst_off : extra_dst[tl.dst_list + j - 1]);
#pragma unroll
      for (int k = 0; k < kUnroll; ++k)
        if (i0 + k * kGroup < total) store_stream<V, kPolicy>(dst + doff[k], v[k]);
    }
  }
}

template <int kGroup, int kPolicy, int kUnroll = kMaxUnroll>
__device__ __forceinline__ void run_tile(const hf_tile &tl, const uint64_t *__restrict__ extra_dst,
                                         const char *__restrict__ src, char *__restrict__ dst, uint32_t lane,
                                         uint32_t part = 0, uint32_t part_bytes = 0) {
  switch (tl.vec_bytes) { // uniform over the group
  case 16: copy_tile<u32x4, kGroup, kPolicy, kUnroll>(tl, extra_dst, src, dst, lane, part, part_bytes); break;
  case 8: copy_tile<u32x2, kGroup, kPolicy, kUnroll>(tl, extra_dst, src, dst, lane, part, part_bytes); break;
  case 4: copy_tile<uint32_t, kGroup, kPolicy, kUnroll>(tl, extra_dst, src, dst, lane, part, part_bytes); break;
  default: copy_tile<uint16_t, kGroup, kPolicy, kUnroll>(tl, extra_dst, src, dst, lane, part, part_bytes); break;
  }
}

// Persistent workgroups: workgroup w copies tiles w, w+grid, w+2*grid, ...  Every
// workgroup leaves the loop after at most ceil(n/grid) rounds; there is no waiting on
// other workgroups anywhere.
template <int kPolicy>
__global__ __launch_bounds__(kWG) void reshard_persistent(const hf_tile *__restrict__ tiles, uint32_t n_tiles,
                                                          const uint64_t *__restrict__ extra_dst,
                                                          const char *__restrict__ src, char *__restrict__ dst) {
  for (uint32_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
    const hf_tile tl = tiles[t];
    run_tile<kWG, kPolicy>(tl, extra_dst, src, dst, threadIdx.x);
  }
}

// Same, but every wavefront walks the list on its own: wavefront g of G copies tiles
// g, g+G, ...  (wavefront-level dispatch; pair it with tiles of a few KiB to 32 KiB).
template <int kPolicy>
__global__ __launch_bounds__(kWG) void reshard_wave_persistent(const hf_tile *__restrict__ tiles, uint32_t n_tiles,
                                                               const uint64_t *__restrict__ extra_dst,
                                                               const char *__restrict__ src, char *__restrict__ dst) {
  const uint32_t waves_per_wg = kWG / kWave;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave); // uniform -> scalar tile loads
  const uint32_t g = blockIdx.x * waves_per_wg + wave, G = gridDim.x * waves_per_wg;
  for (uint32_t t = g; t < n_tiles; t += G) {
    const hf_tile tl = tiles[t];
    run_tile<kWave, kPolicy>(tl, extra_dst, src, dst, threadIdx.x % kWave);
  }
}

template <int kPolicy>
__global__ __launch_bounds__(kWG) void reshard_one_tile(const hf_tile *__restrict__ tiles, uint32_t n_tiles,
                                                        const uint64_t *__restrict__ extra_dst,
                                                        const char *__restrict__ src, char *__restrict__ dst) {
  const uint32_t t = blockIdx.x;
  if (t < n_tiles) {
    const hf_tile tl = tiles[t];
    run_tile<kWG, kPolicy>(tl, extra_dst, src, dst, threadIdx.x);
  }
}

// One short-lived workgroup per `part_bytes` of payload: workgroup b copies part b % parts
// of tile b / parts and exits (parts = ceil(tile bytes / part_bytes), the same for every
// tile; parts beyond the end of a short tile are empty).  The hardware dispatcher hands
// out workgroups in index order, so at any moment the chip works on one narrow, moving
// window of source and destination addresses, and a slow CU simply takes fewer
// workgroups.  kUnroll = part_bytes / 4 KiB vectors per lane, all loaded before the
// first store.  kList does not change the code: it names the work list in the kernel's
// name, so that a profiler's per-kernel statistics keep apart what one process launches
// over different lists (0 = train->gen without own pieces, 1 = train->gen with own
// pieces, 2 = any other list: reverse, own pieces alone).
// A prefetch tile that stands for several copy tiles (n_dst == 0, dst_list = number of chunks):
// `dst_list` chunks of row_bytes bytes, src_row_stride apart; the group that has part number
// `part` loads part `part` of EVERY chunk (all loads in flight together).  The copy tiles of
// the chunks follow later in the list with the same number of workgroups each, so that the
// workgroup that copies part k of a chunk runs on the XCD (workgroup index mod 8) whose L2
// this group filled.
template <int kGroup, int kUnroll>
__device__ __forceinline__ void prefetch_chunks(const hf_tile &tl, const char *__restrict__ src_base, uint32_t lane, uint32_t part) {
  constexpr uint32_t kMaxChunks = HF_MAX_PREFETCH_CHUNKS;
  const uint32_t n = tl.dst_list, bytes = tl.row_bytes, stride = tl.src_row_stride;
  const char *__restrict__ src = src_base + tl.src_off;
#pragma unroll
  for (int k = 0; k < kUnroll; ++k) {
    const uint32_t off = ((part * kUnroll + k) * kGroup + lane) * 16u;
    if (off >= bytes) continue;
    u32x4 v[kMaxChunks];
#pragma unroll
    for (uint32_t j = 0; j < kMaxChunks; ++j)
      if (j < n) v[j] = *reinterpret_cast<const u32x4 *>(src + (size_t)j * stride + off);
#pragma unroll
    for (uint32_t j = 0; j < kMaxChunks; ++j)
      if (j < n) keep_alive(v[j]);
  }
}

template <int kPolicy, int kUnroll, int kThreads, int kList>
__global__ __launch_bounds__(kThreads) void reshard_parts(const hf_tile *__restrict__ tiles, uint32_t n_tiles, uint32_t parts,
                                                          const uint64_t *__restrict__ extra_dst,
                                                          const char *__restrict__ src, char *__restrict__ dst) {
  const uint32_t t = blockIdx.x / parts, part = blockIdx.x - t * parts;
  if (t < n_tiles) {
    const hf_tile tl = tiles[t];
    if (tl.n_dst == 0 && tl.dst_list != 0) { // uniform
      prefetch_chunks<kThreads, kUnroll>(tl, src, threadIdx.x, part);
      return;
    }
    run_tile<kThreads, kPolicy, kUnroll>(tl, extra_dst, src, dst, threadIdx.x, part, kUnroll * kThreads * 16);
  }
}

// Tile staged through LDS in 16 KiB slabs: global -> registers -> LDS, barrier,
// LDS -> registers -> global.  Exists to measure whether staging buys anything for the
// block-level permutations of this path (it moves the same HBM bytes).
constexpr uint32_t kSlab = 16 * 1024;
template <typename V>
__device__ __forceinline__ void copy_tile_lds(const hf_tile &tl, const uint64_t *__restrict__ extra_dst,
                                              const char *__restrict__ src_base, char *__restrict__ dst_base, char *lds) {
  const char *__restrict__ src = src_base + tl.src_off;
  const uint32_t sstr = tl.src_row_stride, dstr = tl.dst_row_stride;
  const uint32_t vpr = tl.row_bytes / (uint32_t)sizeof(V);
  const uint32_t total = tl.rows * vpr;
  constexpr uint32_t per_slab = kSlab / (uint32_t)sizeof(V);
  V *stage = reinterpret_cast<V *>(lds);
  for (uint32_t base = 0; base < total; base += per_slab) {
    const uint32_t n = min(per_slab, total - base);
    for (uint32_t j = threadIdx.x; j < n; j += kWG) {
      const uint32_t i = base + j;
      const uint32_t row = i / vpr, col = (i - row * vpr) * (uint32_t)sizeof(V);
      stage[j] = load_stream<V, 0>(src + (row * sstr + col));
    }
    __syncthreads();
    for (uint32_t d = 0; d < tl.n_dst; ++d) {
      char *__restrict__ dst = dst_base + (d == 0 ? tl.dst_off : extra_dst[tl.dst_list + d - 1]);
      for (uint32_t j = threadIdx.x; j < n; j += kWG) {
        const uint32_t i = base + j;
        const uint32_t row = i / vpr, col = (i - row * vpr) * (uint32_t)sizeof(V);
        store_stream<V, 0>(dst + (row * dstr + col), stage[j]);
      }
    }
    __syncthreads();
  }
}

__global__ __launch_bounds__(kWG) void reshard_persistent_lds(const hf_tile *__restrict__ tiles, uint32_t n_tiles,
                                                              const uint64_t *__restrict__ extra_dst,
                                                              const char *__restrict__ src, char *__restrict__ dst) {
  __shared__ __attribute__((aligned(16))) char lds[kSlab];
  for (uint32_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
    const hf_tile tl = tiles[t];
    switch (tl.vec_bytes) {
    case 16: copy_tile_lds<u32x4>(tl, extra_dst, src, dst, lds); break;
    case 8: copy_tile_lds<u32x2>(tl, extra_dst, src, dst, lds); break;
    case 4: copy_tile_lds<uint32_t>(tl, extra_dst, src, dst, lds); break;
    default: copy_tile_lds<uint16_t>(tl, extra_dst, src, dst, lds); break;
    }
  }
}

__global__ __launch_bounds__(kWG) void calib_copy(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, size_t n_vec) {
  const size_t stride = (size_t)gridDim.x * kWG;
  for (size_t i = (size_t)blockIdx.x * kWG + threadIdx.x; i < n_vec; i += stride) dst[i] = src[i];
}

// All-gather of per-rank result slots inside micro-DP groups (HybridFlow Section 5.2
// step 3): output slot `pair` receives input slot peers[pair].  One workgroup per 256
// vectors of a slot; the slots are small (token ids), so this is launch/latency bound.
template <typename V>
__global__ __launch_bounds__(kWG) void gather_slots(const int32_t *__restrict__ peers, uint32_t n_pairs, uint32_t chunks,
                                                    uint64_t slot_vecs, const V *__restrict__ in, V *__restrict__ out) {
  const uint32_t pair = blockIdx.x / chunks, chunk = blockIdx.x - pair * chunks;
  if (pair >= n_pairs) return;
  const uint64_t i = (uint64_t)chunk * kWG + threadIdx.x;
  if (i < slot_vecs) out[(uint64_t)pair * slot_vecs + i] = in[(uint64_t)peers[pair] * slot_vecs + i];
}

// read-only and write-only counterparts of calib_copy (ceilings of one direction)
__global__ __launch_bounds__(kWG) void calib_read(const u32x4 *__restrict__ src, size_t n_vec) {
  const size_t stride = (size_t)gridDim.x * kWG;
  u32x4 acc = {0, 0, 0, 0};
  for (size_t i = (size_t)blockIdx.x * kWG + threadIdx.x; i < n_vec; i += stride) acc ^= __builtin_nontemporal_load(src + i);
  keep_alive(acc);
}
__global__ __launch_bounds__(kWG) void calib_write(u32x4 *__restrict__ dst, size_t n_vec) {
  const size_t stride = (size_t)gridDim.x * kWG;
  const u32x4 v = {0x5A5A5A5Au, 0x5A5A5A5Au, 0x5A5A5A5Au, 0x5A5A5A5Au};
  for (size_t i = (size_t)blockIdx.x * kWG + threadIdx.x; i < n_vec; i += stride) __builtin_nontemporal_store(v, dst + i);
}

// One read, n_dst writes (hf_calib_fanout); src == null: writes only, dst == null: the
// read only.  A workgroup handles kUnroll vectors per lane.  method 0 (registers): every
// workgroup stores its vectors to all n_dst places.  method 1 (cache-blocked): the grid is
// (blocks x n_dst passes x workgroups per block) and a workgroup stores to the place of its
// pass, so that passes 2.. re-read what pass 1 brought into L2.  method 2 (prefetched): the
// grid is (blocks x 2 passes x workgroups per block); pass 0 only loads the block, pass 1
// loads it again (from L2) and stores it to all n_dst places.
template <int kThreads, int kUnroll>
__global__ __launch_bounds__(kThreads) void calib_fanout(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, size_t n_vec,
                                                         uint32_t n_dst, size_t stride_vec, uint32_t block_vecs, int method) {
  constexpr uint32_t per_wg = kThreads * kUnroll;
  size_t first;
  uint32_t pass = 0;
  if (method == 0) {
    first = (size_t)blockIdx.x * per_wg;
  } else {
    const uint32_t wpb = block_vecs / per_wg; // workgroups per block pass
    const uint32_t passes = method == 1 ? n_dst : 2;
    const uint32_t block = blockIdx.x / (wpb * passes), rest = blockIdx.x - block * (wpb * passes);
    pass = rest / wpb;
    first = (size_t)block * block_vecs + (size_t)(rest - pass * wpb) * per_wg;
  }
  u32x4 v[kUnroll];
#pragma unroll
  for (int k = 0; k < kUnroll; ++k) {
    const size_t i = first + (size_t)k * kThreads + threadIdx.x;
    v[k] = u32x4{0x5A5A5A5Au, 0x5A5A5A5Au, 0x5A5A5A5Au, 0x5A5A5A5Au};
    if (src && i < n_vec) v[k] = method ? src[i] : __builtin_nontemporal_load(src + i);
  }
  if (!dst || (method == 2 && pass == 0)) { // read only
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) keep_alive(v[k]);
    return;
  }
  const uint32_t j0 = method == 1 ? pass : 0, j1 = method == 1 ? pass + 1 : n_dst;
  for (uint32_t j = j0; j < j1; ++j)
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) {
      const size_t i = first + (size_t)k * kThreads + threadIdx.x;
      if (i < n_vec) __builtin_nontemporal_store(v[k], dst + (size_t)j * stride_vec + i);
    }
}

template <int kPolicy, int kList>
void launch_parts(const hf_tile *d_tiles, uint32_t n, const uint64_t *extra_dst, const char *s, char *d, uint32_t tile_bytes,
                  uint32_t part_bytes, int wg_threads, hipStream_t st) {
  const uint32_t parts = (tile_bytes + part_bytes - 1) / part_bytes;
  const dim3 g(n * parts);
  if (wg_threads == kWave) { // one wavefront per workgroup: part_bytes = U * 1 KiB
    switch (part_bytes / 1024) {
    case 1: hipLaunchKernelGGL((reshard_parts<kPolicy, 1, kWave, kList>), g, dim3(kWave), 0, st, d_tiles, n, parts, extra_dst, s, d); break;
    case 2: hipLaunchKernelGGL((reshard_parts<kPolicy, 2, kWave, kList>), g, dim3(kWave), 0, st, d_tiles, n, parts, extra_dst, s, d); break;
    case 4: hipLaunchKernelGGL((reshard_parts<kPolicy, 4, kWave, kList>), g, dim3(kWave), 0, st, d_tiles, n, parts, extra_dst, s, d); break;
    default: hipLaunchKernelGGL((reshard_parts<kPolicy, 8, kWave, kList>), g, dim3(kWave), 0, st, d_tiles, n, parts, extra_dst, s, d); break;
    }
  } else {
    switch (part_bytes / 4096) {
    case 1: hipLaunchKernelGGL((reshard_parts<kPolicy, 1, kWG, kList>), g, dim3(kWG), 0, st, d_tiles, n, parts, extra_dst, s, d); break;
    case 2: hipLaunchKernelGGL((reshard_parts<kPolicy, 2, kWG, kList>), g, dim3(kWG), 0, st, d_tiles, n, parts, extra_dst, s, d); break;
    case 4: hipLaunchKernelGGL((reshard_parts<kPolicy, 4, kWG, kList>), g, dim3(kWG), 0, st, d_tiles, n, parts, extra_dst, s, d); break;
    default: hipLaunchKernelGGL((reshard_parts<kPolicy, 8, kWG, kList>), g, dim3(kWG), 0, st, d_tiles, n, parts, extra_dst, s, d); break;
    }
  }
}

template <int kPolicy>
void launch_policy(const hf_tile *d_tiles, uint32_t n, uint32_t grid, const uint64_t *extra_dst, const char *s, char *d,
                   int variant, uint32_t tile_bytes, uint32_t part_bytes, int wg_threads, int list_tag, hipStream_t st) {
  switch (variant) {
  case HF_VARIANT_PARTS:
    switch (list_tag) {
    case 0: launch_parts<kPolicy, 0>(d_tiles, n, extra_dst, s, d, tile_bytes, part_bytes, wg_threads, st); break;
    case 1: launch_parts<kPolicy, 1>(d_tiles, n, extra_dst, s, d, tile_bytes, part_bytes, wg_threads, st); break;
    default: launch_parts<kPolicy, 2>(d_tiles, n, extra_dst, s, d, tile_bytes, part_bytes, wg_threads, st); break;
    }
    break;
  case HF_VARIANT_ONE_WG_PER_TILE:
    hipLaunchKernelGGL(reshard_one_tile<kPolicy>, dim3(n), dim3(kWG), 0, st, d_tiles, n, extra_dst, s, d);
    break;
  case HF_VARIANT_WAVE_PERSISTENT:
    hipLaunchKernelGGL(reshard_wave_persistent<kPolicy>, dim3(grid), dim3(kWG), 0, st, d_tiles, n, extra_dst, s, d);
    break;
  default:
    hipLaunchKernelGGL(reshard_persistent<kPolicy>, dim3(grid), dim3(kWG), 0, st, d_tiles, n, extra_dst, s, d);
    break;
  }
}

} // namespace

int launch_tiles(const hf_tile *d_tiles, size_t n_tiles, const uint64_t *extra_dst, const void *src, void *dst,
                 int variant, int grid_wgs, int cache_policy, uint32_t tile_bytes, uint32_t part_bytes,
                 uint32_t max_wgs_per_launch, int wg_threads, int list_tag, void *stream) {
  if (n_tiles == 0) return 0;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const char *s = static_cast<const char *>(src);
  char *d = static_cast<char *>(dst);
  // A HIP grid holds fewer than 2^32 threads per dimension (a larger one is not refused,
  // its size wraps), so the kernels that take one workgroup per tile or per part go out
  // in several launches of at most max_wgs_per_launch workgroups, in list order.
  size_t tiles_per_launch = n_tiles;
  if (variant == HF_VARIANT_PARTS) {
    const uint32_t parts = (tile_bytes + part_bytes - 1) / part_bytes;
    if (parts > max_wgs_per_launch) return (int)hipErrorInvalidValue;
    tiles_per_launch = max_wgs_per_launch / parts;
  } else if (variant == HF_VARIANT_ONE_WG_PER_TILE) {
    tiles_per_launch = max_wgs_per_launch;
  }
  for (size_t first = 0; first < n_tiles; first += tiles_per_launch) {
    const uint32_t n = (uint32_t)std::min(tiles_per_launch, n_tiles - first);
    const uint32_t grid = (uint32_t)std::min<size_t>(n, (size_t)grid_wgs);
    const hf_tile *t = d_tiles + first;
    if (variant == HF_VARIANT_LDS_STAGED) {
      hipLaunchKernelGGL(reshard_persistent_lds, dim3(grid), dim3(kWG), 0, st, t, n, extra_dst, s, d);
    } else {
      switch (cache_policy) {
      case 1: launch_policy<1>(t, n, grid, extra_dst, s, d, variant, tile_bytes, part_bytes, wg_threads, list_tag, st); break;
      case 2: launch_policy<2>(t, n, grid, extra_dst, s, d, variant, tile_bytes, part_bytes, wg_threads, list_tag, st); break;
      case 3: launch_policy<3>(t, n, grid, extra_dst, s, d, variant, tile_bytes, part_bytes, wg_threads, list_tag, st); break;
      case 4: launch_policy<4>(t, n, grid, extra_dst, s, d, variant, tile_bytes, part_bytes, wg_threads, list_tag, st); break;
      case 5: launch_policy<5>(t, n, grid, extra_dst, s, d, variant, tile_bytes, part_bytes, wg_threads, list_tag, st); break;
      default: launch_policy<0>(t, n, grid, extra_dst, s, d, variant, tile_bytes, part_bytes, wg_threads, list_tag, st); break;
      }
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
  }
  return 0;
}

int launch_gather_slots(const int32_t *d_peers, uint32_t n_pairs, const void *in, void *out, size_t slot_bytes,
                        void *stream) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool wide = slot_bytes % 16 == 0;
  const uint64_t slot_vecs = slot_bytes / (wide ? 16 : 4);
  const uint64_t chunks = (slot_vecs + kWG - 1) / kWG;
  if (chunks * n_pairs > 0xFFFFFFFFull / kWG) return (int)hipErrorInvalidValue; // beyond one HIP grid
  const dim3 grid((uint32_t)(chunks * n_pairs));
  if (wide)
    hipLaunchKernelGGL(gather_slots<u32x4>, grid, dim3(kWG), 0, st, d_peers, n_pairs, (uint32_t)chunks, slot_vecs,
                       static_cast<const u32x4 *>(in), static_cast<u32x4 *>(out));
  else
    hipLaunchKernelGGL(gather_slots<uint32_t>, grid, dim3(kWG), 0, st, d_peers, n_pairs, (uint32_t)chunks, slot_vecs,
                       static_cast<const uint32_t *>(in), static_cast<uint32_t *>(out));
  return (int)hipGetLastError();
}

int launch_calib_fanout(const void *src, void *dst, size_t bytes, int n_dst, size_t dst_stride, int method, size_t block_bytes,
                        int wg_bytes, void *stream) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  const size_t n_vec = bytes / 16, stride_vec = dst_stride / 16;
  const size_t wgs_one_pass = (bytes + wg_bytes - 1) / wg_bytes;
  size_t grid = wgs_one_pass;
  if (method) {
    const size_t blocks = (bytes + block_bytes - 1) / block_bytes;
    grid = blocks * (size_t)(method == 1 ? n_dst : 2) * (block_bytes / wg_bytes);
  }
  const int threads = wg_bytes == 1024 ? kWave : kWG;
  if (grid == 0 || grid > 0xFFFFFFFFull / threads) return (int)hipErrorInvalidValue; // beyond one HIP grid
  const dim3 g((uint32_t)grid);
  const u32x4 *s = static_cast<const u32x4 *>(src);
  u32x4 *d = static_cast<u32x4 *>(dst);
  const uint32_t bv = (uint32_t)(block_bytes / 16);
  if (wg_bytes == 1024) hipLaunchKernelGGL((calib_fanout<kWave, 1>), g, dim3(kWave), 0, st, s, d, n_vec, (uint32_t)n_dst, stride_vec, bv, method);
  else if (wg_bytes == 4096) hipLaunchKernelGGL((calib_fanout<kWG, 1>), g, dim3(kWG), 0, st, s, d, n_vec, (uint32_t)n_dst, stride_vec, bv, method);
  else hipLaunchKernelGGL((calib_fanout<kWG, 2>), g, dim3(kWG), 0, st, s, d, n_vec, (uint32_t)n_dst, stride_vec, bv, method);
  return (int)hipGetLastError();
}

int launch_calib_copy(const void *src, void *dst, size_t bytes, void *stream) {
  if (bytes == 0) return 0;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (src && dst)
    hipLaunchKernelGGL(calib_copy, dim3(4096), dim3(kWG), 0, st, static_cast<const u32x4 *>(src), static_cast<u32x4 *>(dst), bytes / 16);
  else if (src) // read only
    hipLaunchKernelGGL(calib_read, dim3(4096), dim3(kWG), 0, st, static_cast<const u32x4 *>(src), bytes / 16);
  else
    hipLaunchKernelGGL(calib_write, dim3(4096), dim3(kWG), 0, st, static_cast<u32x4 *>(dst), bytes / 16);
  return (int)hipGetLastError();
}

} // namespace hf

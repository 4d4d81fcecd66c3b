// C ABI of libhfreshard (declarations and contracts: include/hfreshard.h).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstring>
#include <mutex>
#include <new>
#include <string>

#include "hfreshard.h"
#include "kernels.hpp"
#include "plan.hpp"

// the Python binding mirrors these layouts field by field
static_assert(sizeof(hf_desc) == 88 && sizeof(hf_tile) == 48 && sizeof(hf_tensor_info) == 32, "ABI struct layout");
static_assert(sizeof(hf_model_desc) == 36 && sizeof(hf_gen_layout) == 32 && sizeof(hf_train_layout) == 12, "ABI struct layout");

struct hf_plan {
  hf::Plan p;
};

// Work-list staging area of hf_reshard_execute_static: device memory that exists from the
// moment the library is loaded, so that the entry point never has to allocate.  In host code
// this name is only a handle for hipGetSymbolAddress; the address the kernels get is looked
// up once per device (scratch_of).
static __device__ __align__(256) unsigned char scratch[HF_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};       // device address of `scratch` on each device
uint64_t g_scratch_serial[kMaxDevices] = {}; // Plan::serial of the work list staged there
std::atomic<uint64_t> g_next_serial{1};

thread_local std::string g_err;

int fail(int code, const std::string &msg) {
  g_err = msg;
  return code;
}

template <typename T> void release(T *&ptr) {
  if (ptr) (void)hipFree(ptr);
  ptr = nullptr;
}

void free_device(hf::Plan &p) {
  release(p.d_tiles_fwd);
  release(p.d_tiles_own);
  release(p.d_tiles_back);
  release(p.d_tiles_fwd_mc);
  release(p.d_mc_dst);
  release(p.d_tiles_fwd_cb);
  release(p.d_tiles_fwd_pf);
  release(p.d_tiles_offload);
  release(p.d_tiles_reload);
  release(p.d_micro_peers);
}

template <typename T> int upload_list(const T *v, size_t n, T **out) {
  release(*out);
  if (n == 0) return HF_OK;
  hipError_t e = hipMalloc(reinterpret_cast<void **>(out), n * sizeof(T));
  if (e != hipSuccess) return fail(e == hipErrorOutOfMemory ? HF_ENOMEM : HF_EHIP, std::string("hipMalloc: ") + hipGetErrorString(e));
  e = hipMemcpy(*out, v, n * sizeof(T), hipMemcpyHostToDevice);
  if (e != hipSuccess) return fail(HF_EHIP, std::string("hipMemcpy: ") + hipGetErrorString(e));
  return HF_OK;
}
template <typename T> int upload_list(const std::vector<T> &v, T **out) { return upload_list(v.data(), v.size(), out); }

// Makes resident exactly the train->gen work list that the current multicast mode runs
// (and frees the others).  Called at plan time and from hf_plan_set_param, never from an
// execution entry point.
int upload_forward_lists(hf::Plan &p) {
  const int64_t mode = p.effective_multicast();
  int rc = HF_OK;
  if (mode == HF_MULTICAST_OFF) rc = upload_list(p.tiles_fwd.data(), (p.flags & HF_COPY_OWN) ? p.tiles_fwd.size() : p.n_tiles_fwd_peer, &p.d_tiles_fwd);
  else release(p.d_tiles_fwd);
  if (rc == HF_OK && mode == HF_MULTICAST_REGISTERS) rc = upload_list(p.tiles_fwd_mc, &p.d_tiles_fwd_mc);
  else release(p.d_tiles_fwd_mc);
  if (rc == HF_OK && mode == HF_MULTICAST_PREFETCHED) rc = upload_list(p.tiles_fwd_pf, &p.d_tiles_fwd_pf);
  else release(p.d_tiles_fwd_pf);
  if (rc == HF_OK && p.active_fwd_uses_mc_dst()) rc = upload_list(p.mc_dst, &p.d_mc_dst);
  else release(p.d_mc_dst);
  if (rc == HF_OK && mode == HF_MULTICAST_CACHE_BLOCKED) rc = upload_list(p.tiles_fwd_cb, &p.d_tiles_fwd_cb);
  else release(p.d_tiles_fwd_cb);
  return rc;
}

int upload(hf::Plan &p) {
  free_device(p);
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(HF_EHIP, std::string("no HIP device: ") + hipGetErrorString(e));
  p.device = dev;
  int rc = upload_forward_lists(p);
  if (rc == HF_OK) rc = upload_list(p.tiles_fwd.data() + p.n_tiles_fwd_peer, p.tiles_fwd.size() - p.n_tiles_fwd_peer, &p.d_tiles_own);
  if (rc == HF_OK) rc = upload_list(p.tiles_back, &p.d_tiles_back);
  if (rc == HF_OK) rc = upload_list(p.tiles_offload, &p.d_tiles_offload);
  if (rc == HF_OK) rc = upload_list(p.tiles_reload, &p.d_tiles_reload);
  if (rc == HF_OK) rc = upload_list(p.micro_peers, &p.d_micro_peers);
  if (rc != HF_OK) free_device(p);
  return rc;
}

// re-tile with a new tile size (and the current multicast block size), then re-upload
int retile(hf::Plan &p, int64_t tile_bytes) {
  const int64_t old = p.tile_bytes;
  p.tile_bytes = tile_bytes;
  std::string err;
  int rc;
  try {
    rc = hf::build_tiles(p, err);
  } catch (const std::bad_alloc &) {
    rc = HF_ENOMEM;
    err = "out of host memory while tiling";
  }
  if (rc != HF_OK) {
    p.tile_bytes = old;
    std::string e2;
    (void)hf::build_tiles(p, e2);
    return fail(rc, err);
  }
  p.serial = g_next_serial++;
  if (!(p.flags & HF_PLAN_HOST_ONLY)) return upload(p);
  return HF_OK;
}

// train_optional: the call does not read or write train_buf (it may then be null)
int check_buffers(const hf::Plan &p, const void *train_buf, const void *gen_buf, bool train_optional) {
  if (!gen_buf || (!train_buf && !train_optional)) return fail(HF_EINVAL, "null plan or buffer");
  if ((reinterpret_cast<uintptr_t>(train_buf) | reinterpret_cast<uintptr_t>(gen_buf)) % 256)
    return fail(HF_EINVAL, "train_buf and gen_buf must be 256-byte aligned");
  const char *t0 = static_cast<const char *>(train_buf), *g0 = static_cast<const char *>(gen_buf);
  if (t0 && t0 < g0 + p.gen_bytes && g0 < t0 + p.train_bytes) return fail(HF_EINVAL, "train_buf and gen_buf overlap");
  return HF_OK;
}

int check_exec(const hf_plan *plan, const void *train_buf, const void *gen_buf, bool train_optional = false) {
  if (!plan) return fail(HF_EINVAL, "null plan or buffer");
  if (int rc = check_buffers(plan->p, train_buf, gen_buf, train_optional)) return rc;
  if (plan->p.flags & HF_PLAN_HOST_ONLY) return fail(HF_EINVAL, "plan was built with HF_PLAN_HOST_ONLY: it has no device copy");
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != plan->p.device)
    return fail(HF_EINVAL, "the current HIP device is not the one the plan was built on");
  return HF_OK;
}

// temporal_loads: the work list counts on re-reads being served by L2
enum { kListTransition = 0, kListFullRefresh = 1, kListOther = 2 }; // names the list in the kernel's name

// How a list wants to be run when the plan leaves the choice to the library.
enum ListShape {
  kShapeStreaming = 0,  // every byte is read once from HBM
  kShapeCacheBlocked,   // later passes re-read from L2: plain loads, 8 KiB workgroups
  kShapePrefetched      // copy workgroups find their source in L2: plain loads, one wavefront per KiB
};

int launch(const hf::Plan &p, const hf_tile *tiles, size_t n, const uint64_t *extra_dst, const void *src, void *dst,
           void *stream, int list_tag, ListShape shape = kShapeStreaming) {
  const bool temporal_loads = shape == kShapeCacheBlocked;
  // Automatic cache policy, measured on the five benchmark shapes: one-to-one streaming
  // lists gain 2 % from system-scope streaming stores (policy 0); the cache-blocked list
  // loses 8 % with them (they disturb the L2-resident source block) and runs with plain
  // loads + compiler non-temporal stores (5); multi-destination tiles take 4.
  const int policy = p.cache_policy >= 0 ? (int)p.cache_policy : (temporal_loads || shape == kShapePrefetched) ? 5 : extra_dst ? 4 : 0;
  // Automatic launch shape, measured on the Llama-7B / 34B transitions: lists whose later
  // passes hit L2 run best with 256 lanes x 2 vectors (8 KiB per workgroup); plain streaming
  // lists with one wavefront x 1 vector (1 KiB per workgroup).
  const int threads = p.wg_threads ? (int)p.wg_threads : (temporal_loads ? 256 : 64);
  uint32_t part = p.part_bytes ? (uint32_t)p.part_bytes : (temporal_loads ? 8192u : threads == 64 ? 1024u : 4096u);
  part = threads == 64 ? std::min(part, 8192u) : std::max(part, 4096u);
  const int e = hf::launch_tiles(tiles, n, extra_dst, src, dst, (int)p.variant, (int)p.grid_wgs, policy,
                                 (uint32_t)p.tile_bytes, part,
                                 (uint32_t)(p.max_wgs_per_launch * (256 / threads)), threads, list_tag, stream);
  if (e != 0) return fail(HF_EHIP, std::string("kernel launch: ") + hipGetErrorString(static_cast<hipError_t>(e)));
  return HF_OK;
}

} // namespace

extern "C" {

int hf_reshard_plan(const hf_model_desc *model, const hf_train_layout *train, const hf_gen_layout *gen, hf_plan **out) {
  if (out) *out = nullptr;
  if (!model || !train || !gen || !out) return fail(HF_EINVAL, "null argument");
  hf_plan *pl = new (std::nothrow) hf_plan();
  if (!pl) return fail(HF_ENOMEM, "out of host memory");
  std::string err;
  int rc;
  try {
    rc = hf::build_plan(*model, *train, *gen, pl->p, err);
  } catch (const std::bad_alloc &) {
    rc = HF_ENOMEM;
    err = "out of host memory while building the plan";
  }
  pl->p.serial = g_next_serial++;
  if (rc == HF_OK && !(gen->flags & HF_PLAN_HOST_ONLY)) {
    rc = upload(pl->p);
    if (rc != HF_OK) err = g_err;
  }
  if (rc != HF_OK) {
    delete pl;
    return fail(rc, err);
  }
  *out = pl;
  return HF_OK;
}

void hf_plan_destroy(hf_plan *plan) {
  if (!plan) return;
  free_device(plan->p);
  delete plan;
}

int hf_reshard_execute(const hf_plan *plan, const void *train_buf, void *gen_buf, void *hip_stream) {
  // gathering out of the generation buffers: gen_buf is source and destination (disjoint
  // pieces), train_buf is not used and need not exist
  const bool from_gen = plan && (plan->p.flags & HF_GATHER_FROM_GEN);
  if (int rc = check_exec(plan, train_buf, gen_buf, from_gen)) return rc;
  if (from_gen) train_buf = gen_buf;
  const hf::Plan &p = plan->p;
  const int tag = (p.flags & HF_COPY_OWN) ? kListFullRefresh : kListTransition;
  if (p.effective_multicast() == HF_MULTICAST_REGISTERS)
    return launch(p, p.d_tiles_fwd_mc, p.tiles_fwd_mc.size(), p.d_mc_dst, train_buf, gen_buf, hip_stream, tag);
  if (p.effective_multicast() == HF_MULTICAST_PREFETCHED)
    return launch(p, p.d_tiles_fwd_pf, p.tiles_fwd_pf.size(), p.d_mc_dst, train_buf, gen_buf, hip_stream, tag, kShapePrefetched);
  if (p.effective_multicast() == HF_MULTICAST_CACHE_BLOCKED)
    return launch(p, p.d_tiles_fwd_cb, p.tiles_fwd_cb.size(), nullptr, train_buf, gen_buf, hip_stream, tag, kShapeCacheBlocked);
  const size_t n = (p.flags & HF_COPY_OWN) ? p.tiles_fwd.size() : p.n_tiles_fwd_peer;
  return launch(p, p.d_tiles_fwd, n, nullptr, train_buf, gen_buf, hip_stream, tag);
}

int hf_reshard_execute_static(const hf_plan *plan, const void *train_buf, void *gen_buf, void *hip_stream) {
  if (!plan) return fail(HF_EINVAL, "null plan or buffer");
  const hf::Plan &p = plan->p;
  const bool from_gen = (p.flags & HF_GATHER_FROM_GEN) != 0;
  if (int rc = check_buffers(p, train_buf, gen_buf, from_gen)) return rc;
  if (from_gen) train_buf = gen_buf; // source and destination are disjoint pieces of gen_buf
  // the work list hf_reshard_execute would run, from the plan's host copy
  const int64_t mode = p.effective_multicast();
  const hf_tile *tiles = p.active_fwd().data();
  const size_t n = p.active_fwd_count();
  const size_t tile_bytes = n * sizeof(hf_tile), extra_at = (tile_bytes + 255) / 256 * 256;
  const size_t extra_bytes = p.active_fwd_uses_mc_dst() ? p.mc_dst.size() * sizeof(uint64_t) : 0;
  if (extra_at + extra_bytes > HF_STATIC_SCRATCH_BYTES)
    return fail(HF_ERANGE, "work list of " + std::to_string(extra_at + extra_bytes) + " bytes does not fit the static scratch of " +
                               std::to_string((size_t)HF_STATIC_SCRATCH_BYTES) + " bytes: raise HF_PARAM_TILE_BYTES or use hf_reshard_execute");
  if (n == 0) return HF_OK;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(HF_EHIP, std::string("no HIP device: ") + hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(HF_ERANGE, "device index beyond the library's table");
  if (p.device >= 0 && dev != p.device) return fail(HF_EINVAL, "the current HIP device is not the one the plan was built on");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  char *base = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) { // once per device, with that device current
      void *ptr = nullptr;
      e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !ptr) return fail(HF_EHIP, std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e));
      g_scratch_ptr[dev] = ptr;
    }
    base = static_cast<char *>(g_scratch_ptr[dev]);
    if (g_scratch_serial[dev] != p.serial) { // another plan's list (or none) is staged: replace it, in stream order
      g_scratch_serial[dev] = 0;
      e = hipMemcpyAsync(base, tiles, tile_bytes, hipMemcpyHostToDevice, st);
      if (e == hipSuccess && extra_bytes) e = hipMemcpyAsync(base + extra_at, p.mc_dst.data(), extra_bytes, hipMemcpyHostToDevice, st);
      if (e != hipSuccess) return fail(HF_EHIP, std::string("staging the work list: ") + hipGetErrorString(e));
      g_scratch_serial[dev] = p.serial;
    }
  }
  return launch(p, reinterpret_cast<const hf_tile *>(base), n, extra_bytes ? reinterpret_cast<const uint64_t *>(base + extra_at) : nullptr,
                train_buf, gen_buf, hip_stream, (p.flags & HF_COPY_OWN) ? kListFullRefresh : kListTransition,
                mode == HF_MULTICAST_CACHE_BLOCKED ? kShapeCacheBlocked : mode == HF_MULTICAST_PREFETCHED ? kShapePrefetched : kShapeStreaming);
}

// host_buf must be pinned host memory; returns the address the device uses for it
static int device_view_of_pinned(const void *host_buf, size_t bytes, void **out) {
  hipPointerAttribute_t at;
  std::memset(&at, 0, sizeof at);
  if (hipPointerGetAttributes(&at, host_buf) != hipSuccess) {
    (void)hipGetLastError(); // an unknown pointer leaves a sticky error behind
    return fail(HF_EINVAL, "host_buf is not known to the HIP runtime: it must be pinned host memory (hipHostMalloc)");
  }
  if (at.type != hipMemoryTypeHost || !at.devicePointer)
    return fail(HF_EINVAL, "host_buf must be pinned host memory that the device can address (hipHostMalloc)");
  void *base = nullptr;
  size_t size = 0;
  if (hipMemGetAddressRange(reinterpret_cast<hipDeviceptr_t *>(&base), &size, at.devicePointer) == hipSuccess && base) {
    const char *lo = static_cast<const char *>(base), *p0 = static_cast<const char *>(at.devicePointer);
    if (p0 < lo || p0 + bytes > lo + size) return fail(HF_EINVAL, "host_buf is shorter than hf_plan_remote_bytes");
  } else {
    (void)hipGetLastError();
  }
  *out = at.devicePointer;
  return HF_OK;
}

static int offload_common(const hf_plan *plan, const void *gen_buf, const void *host_buf, void **host_dev) {
  if (!plan || !gen_buf || !host_buf) return fail(HF_EINVAL, "null plan or buffer");
  const hf::Plan &p = plan->p;
  if (p.flags & HF_PLAN_HOST_ONLY) return fail(HF_EINVAL, "plan was built with HF_PLAN_HOST_ONLY: it has no device copy");
  if (!(p.flags & HF_PLAN_OFFLOAD)) return fail(HF_EINVAL, "plan was built without HF_PLAN_OFFLOAD");
  if (p.kind_mask != 0x1F) return fail(HF_EINVAL, "plan is restricted to some descriptor kinds");
  if ((reinterpret_cast<uintptr_t>(gen_buf) | reinterpret_cast<uintptr_t>(host_buf)) % 256)
    return fail(HF_EINVAL, "gen_buf and host_buf must be 256-byte aligned");
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != p.device)
    return fail(HF_EINVAL, "the current HIP device is not the one the plan was built on");
  return device_view_of_pinned(host_buf, p.remote_bytes, host_dev);
}

// The host link, not HBM, bounds these two: a handful of persistent workgroups (each lane
// with eight 16-byte accesses in flight) keeps it full.  More would only queue host-bound
// writes in the memory fabric ahead of the HBM traffic of kernels on other streams.
static int launch_link(const hf::Plan &p, const hf_tile *tiles, size_t n, const void *src, void *dst, void *stream) {
  const int policy = p.cache_policy >= 0 ? (int)p.cache_policy : 0;
  const int e = hf::launch_tiles(tiles, n, nullptr, src, dst, HF_VARIANT_PERSISTENT, (int)p.offload_wgs, policy,
                                 (uint32_t)p.tile_bytes, 4096u, (uint32_t)p.max_wgs_per_launch, 256, kListOther, stream);
  if (e != 0) return fail(HF_EHIP, std::string("kernel launch: ") + hipGetErrorString(static_cast<hipError_t>(e)));
  return HF_OK;
}

int hf_offload_remote(const hf_plan *plan, const void *gen_buf, void *host_buf, void *hip_stream) {
  void *hd = nullptr;
  if (int rc = offload_common(plan, gen_buf, host_buf, &hd)) return rc;
  return launch_link(plan->p, plan->p.d_tiles_offload, plan->p.tiles_offload.size(), gen_buf, hd, hip_stream);
}

int hf_reload_remote(const hf_plan *plan, const void *host_buf, void *gen_buf, void *hip_stream) {
  void *hd = nullptr;
  if (int rc = offload_common(plan, gen_buf, host_buf, &hd)) return rc;
  return launch_link(plan->p, plan->p.d_tiles_reload, plan->p.tiles_reload.size(), hd, gen_buf, hip_stream);
}

size_t hf_plan_remote_bytes(const hf_plan *plan) { return plan ? plan->p.remote_bytes : 0; }
size_t hf_plan_remote_rank_offset(const hf_plan *plan, int rank) {
  if (!plan || rank < 0 || rank >= plan->p.N || plan->p.mat_pos[rank] < 0) return (size_t)-1;
  return plan->p.remote_rank_off[plan->p.mat_pos[rank]];
}

int hf_plan_check_buffers(const hf_plan *plan, const void *train_buf, size_t train_len, const void *gen_buf, size_t gen_len) {
  if (!plan) return fail(HF_EINVAL, "null plan or buffer");
  const hf::Plan &p = plan->p;
  // a plan that gathers out of the generation buffers never touches train_buf
  if (int rc = check_buffers(p, train_buf, gen_buf, (p.flags & HF_GATHER_FROM_GEN) != 0)) return rc;
  if (train_buf && train_len < p.train_bytes) return fail(HF_EINVAL, "train_buf is shorter than hf_plan_train_bytes");
  if (gen_len < p.gen_bytes) return fail(HF_EINVAL, "gen_buf is shorter than hf_plan_gen_bytes");
  if (p.flags & HF_PLAN_HOST_ONLY) return HF_OK;
  struct { const char *ptr; size_t need; const char *name; } bufs[] = {{static_cast<const char *>(train_buf), p.train_bytes, "train_buf"},
                                                                        {static_cast<const char *>(gen_buf), p.gen_bytes, "gen_buf"}};
  for (auto &b : bufs) {
    if (!b.ptr) continue;
    void *base = nullptr;
    size_t size = 0;
    if (hipMemGetAddressRange(reinterpret_cast<hipDeviceptr_t *>(&base), &size, const_cast<char *>(b.ptr)) != hipSuccess || !base) {
      (void)hipGetLastError();
      return fail(HF_ERANGE, std::string(b.name) + " is not inside a device allocation of the HIP runtime");
    }
    if (b.ptr + b.need > static_cast<const char *>(base) + size)
      return fail(HF_ERANGE, std::string(b.name) + ": the device allocation ends before the bytes the plan needs");
  }
  return HF_OK;
}

int hf_reshard_install_own(const hf_plan *plan, const void *train_buf, void *gen_buf, void *hip_stream) {
  if (int rc = check_exec(plan, train_buf, gen_buf)) return rc;
  const hf::Plan &p = plan->p;
  return launch(p, p.d_tiles_own, p.tiles_fwd.size() - p.n_tiles_fwd_peer, nullptr, train_buf, gen_buf, hip_stream, kListOther);
}

int hf_reshard_back(const hf_plan *plan, void *train_buf, const void *gen_buf, void *hip_stream) {
  if (int rc = check_exec(plan, train_buf, gen_buf)) return rc;
  const hf::Plan &p = plan->p;
  if (p.flags & HF_GROUPING_VANILLA)
    return fail(HF_EINVAL, "vanilla grouping keeps the training shard besides the generation buffer: nothing to re-partition");
  return launch(p, p.d_tiles_back, p.tiles_back.size(), nullptr, gen_buf, train_buf, hip_stream, kListOther);
}

int hf_gather_responses(const hf_plan *plan, const void *resp_in, void *resp_out, size_t slot_bytes, void *hip_stream) {
  if (!plan || !resp_in || !resp_out) return fail(HF_EINVAL, "null plan or buffer");
  const hf::Plan &p = plan->p;
  if (p.flags & HF_PLAN_HOST_ONLY) return fail(HF_EINVAL, "plan was built with HF_PLAN_HOST_ONLY: it has no device copy");
  if (slot_bytes == 0 || slot_bytes % 4) return fail(HF_EINVAL, "slot_bytes must be a positive multiple of 4");
  if ((reinterpret_cast<uintptr_t>(resp_in) | reinterpret_cast<uintptr_t>(resp_out)) % 256)
    return fail(HF_EINVAL, "resp_in and resp_out must be 256-byte aligned");
  const char *a = static_cast<const char *>(resp_in), *b = static_cast<const char *>(resp_out);
  const size_t in_bytes = (size_t)p.N * slot_bytes, out_bytes = in_bytes * p.dg;
  if (a < b + out_bytes && b < a + in_bytes) return fail(HF_EINVAL, "resp_in and resp_out overlap");
  const int e = hf::launch_gather_slots(p.d_micro_peers, (uint32_t)p.micro_peers.size(), resp_in, resp_out, slot_bytes, hip_stream);
  if (e == (int)hipErrorInvalidValue) return fail(HF_ERANGE, "slots too large for one launch");
  if (e != 0) return fail(HF_EHIP, std::string("kernel launch: ") + hipGetErrorString(static_cast<hipError_t>(e)));
  return HF_OK;
}

int hf_plan_micro_dp_peer(const hf_plan *plan, int rank, int j) {
  if (!plan || rank < 0 || rank >= plan->p.N || j < 0 || j >= plan->p.dg) return -1;
  return plan->p.micro_peers[(size_t)rank * plan->p.dg + j];
}

int hf_plan_set_param(hf_plan *plan, int param, int64_t value) {
  if (!plan) return fail(HF_EINVAL, "null plan");
  hf::Plan &p = plan->p;
  switch (param) {
  case HF_PARAM_TILE_BYTES:
    return retile(p, value);
  case HF_PARAM_GRID_WGS:
    if (value < 1 || value > 65536) return fail(HF_EINVAL, "grid workgroups must be in [1, 65536]");
    p.grid_wgs = value;
    return HF_OK;
  case HF_PARAM_VARIANT:
    if (value < HF_VARIANT_PERSISTENT || value > HF_VARIANT_PARTS) return fail(HF_EINVAL, "unknown kernel variant");
    p.variant = value;
    return HF_OK;
  case HF_PARAM_MULTICAST:
    if (value < HF_MULTICAST_AUTO || value > HF_MULTICAST_PREFETCHED) return fail(HF_EINVAL, "unknown multicast mode");
    p.multicast_auto = value == HF_MULTICAST_AUTO;
    p.multicast = p.multicast_auto ? hf::default_multicast(p) : value;
    p.serial = g_next_serial++;
    if (!(p.flags & HF_PLAN_HOST_ONLY)) return upload_forward_lists(p);
    return HF_OK;
  case HF_PARAM_OFFLOAD_WGS:
    if (value < 1 || value > 4096) return fail(HF_EINVAL, "offload workgroups must be in [1, 4096]");
    p.offload_wgs = value;
    return HF_OK;
  case HF_PARAM_PREFETCH_BLOCK_BYTES:
    if (value < (1 << 20) || value > (64 << 20)) return fail(HF_EINVAL, "prefetch block must be in [1 MiB, 64 MiB]");
    p.prefetch_block_bytes = value;
    return retile(p, p.tile_bytes);
  case HF_PARAM_PREFETCH_MERGE:
    if (value < 0 || value > HF_MAX_PREFETCH_CHUNKS) return fail(HF_EINVAL, "prefetch merge must be in [0, 8]");
    p.prefetch_merge = value;
    return retile(p, p.tile_bytes);
  case HF_PARAM_ROW_INTERLEAVE:
    if (value != 0 && value != 1) return fail(HF_EINVAL, "row interleave must be 0 or 1");
    p.row_interleave = value;
    return retile(p, p.tile_bytes);
  case HF_PARAM_MC_BLOCK_BYTES: {
    if (value < (1 << 20) || value > (1ll << 30)) return fail(HF_EINVAL, "multicast block must be in [1 MiB, 1 GiB]");
    p.mc_block_bytes = value;
    return retile(p, p.tile_bytes);
  }
  case HF_PARAM_MAX_WGS_PER_LAUNCH:
    if (value < 1024 || value > 0xFFFFFFFFll / 256) return fail(HF_EINVAL, "workgroups per launch must be in [1024, 16777215]");
    p.max_wgs_per_launch = value;
    return HF_OK;
  case HF_PARAM_WG_THREADS:
    if (value != 0 && value != 64 && value != 256) return fail(HF_EINVAL, "workgroup size must be 0 (automatic), 64 or 256");
    p.wg_threads = value;
    return HF_OK;
  case HF_PARAM_CACHE_POLICY:
    if (value < -1 || value > 5) return fail(HF_EINVAL, "cache policy must be in [-1, 5]");
    p.cache_policy = value;
    return HF_OK;
  case HF_PARAM_PART_BYTES:
    if (value != 0 && value != 1024 && value != 2048 && value != 4096 && value != 8192 && value != 16384 && value != 32768)
      return fail(HF_EINVAL, "part bytes must be 0 (automatic) or a power of two from 1024 to 32768");
    p.part_bytes = value;
    return HF_OK;
  }
  return fail(HF_EINVAL, "unknown parameter");
}

int hf_debug_restrict_kinds(hf_plan *plan, int kind_mask) {
  if (!plan) return fail(HF_EINVAL, "null plan");
  if (kind_mask < 1 || kind_mask > 0x1F) return fail(HF_EINVAL, "kind mask must be in [1, 31]");
  plan->p.kind_mask = kind_mask;
  return retile(plan->p, plan->p.tile_bytes);
}

int64_t hf_plan_get_param(const hf_plan *plan, int param) {
  if (!plan) return -1;
  switch (param) {
  case HF_PARAM_TILE_BYTES: return plan->p.tile_bytes;
  case HF_PARAM_GRID_WGS: return plan->p.grid_wgs;
  case HF_PARAM_VARIANT: return plan->p.variant;
  case HF_PARAM_MULTICAST: return plan->p.effective_multicast();
  case HF_PARAM_MC_BLOCK_BYTES: return plan->p.mc_block_bytes;
  case HF_PARAM_OFFLOAD_WGS: return plan->p.offload_wgs;
  case HF_PARAM_ROW_INTERLEAVE: return plan->p.row_interleave;
  case HF_PARAM_PREFETCH_BLOCK_BYTES: return plan->p.prefetch_block_bytes;
  case HF_PARAM_PREFETCH_MERGE: return plan->p.effective_prefetch_merge();
  case HF_PARAM_WG_THREADS: return plan->p.wg_threads;
  case HF_PARAM_MAX_WGS_PER_LAUNCH: return plan->p.max_wgs_per_launch;
  case HF_PARAM_CACHE_POLICY: return plan->p.cache_policy;
  case HF_PARAM_PART_BYTES: return plan->p.part_bytes;
  }
  return -1;
}

size_t hf_plan_train_bytes(const hf_plan *plan) { return plan ? plan->p.train_bytes : 0; }
size_t hf_plan_gen_bytes(const hf_plan *plan) { return plan ? plan->p.gen_bytes : 0; }
int hf_plan_num_ranks(const hf_plan *plan) { return plan ? plan->p.N : 0; }
int hf_plan_num_mat(const hf_plan *plan) { return plan ? (int)plan->p.mat.size() : 0; }
int hf_plan_mat_rank(const hf_plan *plan, int i) {
  return (plan && i >= 0 && i < (int)plan->p.mat.size()) ? plan->p.mat[i] : -1;
}
int hf_plan_micro_dp_size(const hf_plan *plan) { return plan ? plan->p.dg : 0; }

size_t hf_plan_rank_train_offset(const hf_plan *plan, int rank) {
  if (!plan || rank < 0 || rank >= plan->p.N) return (size_t)-1;
  return plan->p.train_tab[rank].base;
}

size_t hf_plan_rank_gen_offset(const hf_plan *plan, int rank) {
  if (!plan || rank < 0 || rank >= plan->p.N || plan->p.mat_pos[rank] < 0) return (size_t)-1;
  return plan->p.gen_tab[rank].base;
}

int hf_plan_rank_coords(const hf_plan *plan, int rank, int32_t out[6]) {
  if (!plan || !out) return fail(HF_EINVAL, "null argument");
  if (rank < 0 || rank >= plan->p.N) return fail(HF_ERANGE, "rank out of range");
  const hf::Coords &c = plan->p.coords[rank];
  out[0] = c.dp; out[1] = c.pp; out[2] = c.tp; out[3] = c.gpp; out[4] = c.gtp; out[5] = c.micro;
  return HF_OK;
}

size_t hf_plan_num_tensors(const hf_plan *plan, int which_buf, int rank) {
  if (!plan || rank < 0 || rank >= plan->p.N) return 0;
  if (which_buf == HF_BUF_TRAIN) return plan->p.train_tab[rank].tensors.size();
  if (which_buf == HF_BUF_GEN && plan->p.mat_pos[rank] >= 0) return plan->p.gen_tab[rank].tensors.size();
  return 0;
}

int hf_plan_get_tensor(const hf_plan *plan, int which_buf, int rank, size_t i, hf_tensor_info *out) {
  if (!plan || !out) return fail(HF_EINVAL, "null argument");
  if (which_buf != HF_BUF_TRAIN && which_buf != HF_BUF_GEN) return fail(HF_EINVAL, "which_buf must be HF_BUF_TRAIN or HF_BUF_GEN");
  if (rank < 0 || rank >= plan->p.N) return fail(HF_ERANGE, "rank out of range");
  if (which_buf == HF_BUF_GEN && plan->p.mat_pos[rank] < 0) return fail(HF_ERANGE, "rank has no generation buffer");
  const hf::RankTable &tab = which_buf == HF_BUF_TRAIN ? plan->p.train_tab[rank] : plan->p.gen_tab[rank];
  if (i >= tab.tensors.size()) return fail(HF_ERANGE, "tensor index past the end");
  const hf::TensorRec &t = tab.tensors[i];
  const hf::Coords &c = plan->p.coords[rank];
  const bool repl = t.id == HF_T_LN1 || t.id == HF_T_LN2 || t.id == HF_T_LNF || t.id == HF_G_LN1 || t.id == HF_G_LN2 || t.id == HF_G_LNF;
  out->tensor_id = t.id;
  out->layer = t.layer;
  out->rows = t.rows;
  out->cols = t.cols;
  out->offset = tab.base + t.off;
  out->tp_index = repl ? 0 : (which_buf == HF_BUF_TRAIN ? c.tp : c.gtp);
  out->replicated = repl ? 1 : 0;
  return HF_OK;
}

static const hf_desc *desc_at(const hf::Plan &p, int direction, size_t i) {
  if (direction == HF_DIR_TRAIN_TO_GEN) {
    if (i < p.fwd_peer.size()) return &p.fwd_peer[i];
    i -= p.fwd_peer.size();
    if ((p.flags & HF_COPY_OWN) && i < p.fwd_own.size()) return &p.fwd_own[i];
    return nullptr;
  }
  if (direction == HF_DIR_GEN_TO_TRAIN && i < p.back.size()) return &p.back[i];
  if ((direction == HF_DIR_OFFLOAD || direction == HF_DIR_RELOAD) && i < p.remote.size()) return &p.remote[i];
  return nullptr;
}

size_t hf_plan_num_desc(const hf_plan *plan, int direction) {
  if (!plan) return 0;
  const hf::Plan &p = plan->p;
  if (direction == HF_DIR_TRAIN_TO_GEN) return p.fwd_peer.size() + ((p.flags & HF_COPY_OWN) ? p.fwd_own.size() : 0);
  if (direction == HF_DIR_GEN_TO_TRAIN) return p.back.size();
  if (direction == HF_DIR_OFFLOAD || direction == HF_DIR_RELOAD) return p.remote.size();
  return 0;
}

int hf_plan_get_desc(const hf_plan *plan, int direction, size_t i, hf_desc *out) {
  if (!plan || !out) return fail(HF_EINVAL, "null argument");
  const hf_desc *d = desc_at(plan->p, direction, i);
  if (!d) return fail(HF_ERANGE, "no such descriptor");
  *out = *d;
  if (direction == HF_DIR_RELOAD) {
    std::swap(out->src_off, out->dst_off);
    std::swap(out->src_block_stride, out->dst_block_stride);
    std::swap(out->src_row_stride, out->dst_row_stride);
  }
  return HF_OK;
}

// totals are cached when the work lists are built
size_t hf_plan_bytes_moved(const hf_plan *plan, int direction) {
  if (!plan) return 0;
  if (direction == HF_DIR_TRAIN_TO_GEN || direction == HF_DIR_GEN_TO_TRAIN) return plan->p.moved_bytes[direction];
  if (direction == HF_DIR_OFFLOAD || direction == HF_DIR_RELOAD) {
    size_t total = 0;
    for (const hf_desc &d : plan->p.remote) total += hf::desc_bytes(d);
    return total;
  }
  return 0;
}

size_t hf_plan_unique_src_bytes(const hf_plan *plan, int direction) {
  if (!plan) return 0;
  if (direction == HF_DIR_TRAIN_TO_GEN || direction == HF_DIR_GEN_TO_TRAIN) return plan->p.unique_bytes[direction];
  return hf_plan_bytes_moved(plan, direction); // the image holds every remote piece once
}

size_t hf_plan_num_own_view(const hf_plan *plan, int rank) {
  if (!plan || rank < 0 || rank >= plan->p.N) return 0;
  size_t n = 0;
  for (const hf_desc &d : plan->p.fwd_own) n += d.dst_rank == rank;
  return n;
}

int hf_plan_get_own_view(const hf_plan *plan, int rank, size_t i, hf_desc *out) {
  if (!plan || !out) return fail(HF_EINVAL, "null argument");
  if (rank < 0 || rank >= plan->p.N) return fail(HF_ERANGE, "rank out of range");
  for (const hf_desc &d : plan->p.fwd_own)
    if (d.dst_rank == rank && i-- == 0) {
      *out = d;
      return HF_OK;
    }
  return fail(HF_ERANGE, "no such own-view entry");
}

size_t hf_plan_num_tiles(const hf_plan *plan, int direction) {
  if (!plan) return 0;
  const hf::Plan &p = plan->p;
  if (direction == HF_DIR_TRAIN_TO_GEN) return p.active_fwd_count();
  if (direction == HF_DIR_GEN_TO_TRAIN) return p.tiles_back.size();
  if (direction == HF_DIR_OFFLOAD) return p.tiles_offload.size();
  if (direction == HF_DIR_RELOAD) return p.tiles_reload.size();
  return 0;
}

int hf_plan_get_tile(const hf_plan *plan, int direction, size_t i, hf_tile *out) {
  if (!plan || !out) return fail(HF_EINVAL, "null argument");
  if (i >= hf_plan_num_tiles(plan, direction)) return fail(HF_ERANGE, "no such tile");
  const hf::Plan &p = plan->p;
  *out = direction == HF_DIR_GEN_TO_TRAIN                    ? p.tiles_back[i]
         : direction == HF_DIR_OFFLOAD                           ? p.tiles_offload[i]
         : direction == HF_DIR_RELOAD                            ? p.tiles_reload[i]
                                                                 : p.active_fwd()[i];
  return HF_OK;
}

int hf_plan_get_tile_dst(const hf_plan *plan, int direction, size_t i, uint32_t k, uint64_t *out) {
  hf_tile tl;
  if (!out) return fail(HF_EINVAL, "null argument");
  if (int rc = hf_plan_get_tile(plan, direction, i, &tl)) return rc;
  if (k >= tl.n_dst) return fail(HF_ERANGE, "no such destination");
  *out = k == 0 ? tl.dst_off : plan->p.mc_dst[tl.dst_list + k - 1];
  return HF_OK;
}

int hf_calib_copy(const void *src, void *dst, size_t bytes, void *hip_stream) {
  if (!src && !dst) return fail(HF_EINVAL, "null buffers");
  if (bytes % 16 || (reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) % 16)
    return fail(HF_EINVAL, "calibration copy needs 16-byte aligned pointers and size");
  const char *s = static_cast<const char *>(src), *d = static_cast<const char *>(dst);
  if (s && d && s < d + bytes && d < s + bytes) return fail(HF_EINVAL, "calibration copy: buffers overlap");
  const int e = hf::launch_calib_copy(src, dst, bytes, hip_stream);
  if (e != 0) return fail(HF_EHIP, std::string("kernel launch: ") + hipGetErrorString(static_cast<hipError_t>(e)));
  return HF_OK;
}

int hf_calib_fanout(const void *src, void *dst, size_t bytes, int n_dst, size_t dst_stride, int method, size_t block_bytes,
                    int wg_bytes, void *hip_stream) {
  if (!src && !dst) return fail(HF_EINVAL, "null buffers");
  if (method < HF_FANOUT_REGISTERS || method > HF_FANOUT_PREFETCHED) return fail(HF_EINVAL, "unknown fan-out method");
  if ((!src || !dst) && method != HF_FANOUT_REGISTERS) return fail(HF_EINVAL, "fan-out copy: blocks need both a source and destinations");
  if (method != HF_FANOUT_REGISTERS && block_bytes == 0) return fail(HF_EINVAL, "fan-out copy: this method needs a block size");
  if (n_dst < 1 || n_dst > 8) return fail(HF_EINVAL, "n_dst must be in [1, 8]");
  if (wg_bytes != 1024 && wg_bytes != 4096 && wg_bytes != 8192) return fail(HF_EINVAL, "wg_bytes must be 1024, 4096 or 8192");
  if (bytes == 0 || bytes % 8192 || dst_stride % 256 || dst_stride < bytes || block_bytes % 65536 ||
      (reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) % 256)
    return fail(HF_EINVAL, "fan-out copy: sizes or alignment out of contract");
  const char *s0 = static_cast<const char *>(src), *d0 = static_cast<const char *>(dst);
  const size_t span = (size_t)(n_dst - 1) * dst_stride + bytes;
  if (s0 && d0 && s0 < d0 + span && d0 < s0 + bytes) return fail(HF_EINVAL, "fan-out copy: buffers overlap");
  const int e = hf::launch_calib_fanout(src, dst, bytes, n_dst, dst_stride, method, block_bytes, wg_bytes, hip_stream);
  if (e == (int)hipErrorInvalidValue) return fail(HF_ERANGE, "fan-out copy: too many workgroups for one launch");
  if (e != 0) return fail(HF_EHIP, std::string("kernel launch: ") + hipGetErrorString(static_cast<hipError_t>(e)));
  return HF_OK;
}

int hf_plan_validate(const hf_plan *plan) {
  if (!plan) return fail(HF_EINVAL, "null plan");
  std::string err;
  int rc;
  try {
    rc = hf::validate_plan(plan->p, err);
  } catch (const std::bad_alloc &) {
    rc = HF_ENOMEM;
    err = "out of host memory while validating";
  }
  return rc == HF_OK ? HF_OK : fail(rc, err);
}

const char *hf_last_error(void) { return g_err.c_str(); }
const char *hf_version(void) { return "hfreshard 0.1 (gfx950)"; }

} // extern "C"

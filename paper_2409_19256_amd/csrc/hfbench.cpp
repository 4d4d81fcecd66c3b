// hfbench: native driver of the C ABI for profiling runs (rocprofv3 counters and kernel
// traces) without a Python interpreter in the traced process.  It plans one of the five
// benchmark configurations, puts train_buf and gen_buf in one HBM allocation, runs
// hf_reshard_execute / hf_reshard_back and times it with HIP events on the launch stream.
// Further modes: --ceilings (copy ceilings of the box from the library's calibration
// kernels), --offload (offload / reload of the remote pieces over the host link, alone and
// next to hf_reshard_back on a second stream), --graph (HIP-graph replay of the transition),
// --responses (step-3 all-gather).  The buffers hold a constant byte pattern: the copy
// kernels never look at the values.  Parity is the business of the test-suite, not of
// this tool.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "hfreshard.h"

#define HIP_CHECK(x)                                                                          \
  do {                                                                                        \
    hipError_t e_ = (x);                                                                      \
    if (e_ != hipSuccess) {                                                                   \
      std::fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));                     \
      return 1;                                                                               \
    }                                                                                         \
  } while (0)
#define HF_CHECK(x)                                                                           \
  do {                                                                                        \
    int rc_ = (x);                                                                            \
    if (rc_ != HF_OK) {                                                                       \
      std::fprintf(stderr, "%s failed: %d: %s\n", #x, rc_, hf_last_error());                  \
      return 1;                                                                               \
    }                                                                                         \
  } while (0)

struct Config {
  const char *name;
  hf_model_desc m;
  hf_train_layout t;
  int pg, tg;
  std::vector<int32_t> mat;
};

namespace {

double now_ms() {
  return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

// mean duration in ms of `reps` calls of f on stream st, after `warm` untimed calls
template <typename F> int time_calls(hipStream_t st, int warm, int reps, F f, double *mean_ms, double *min_ms = nullptr) {
  for (int i = 0; i < warm; ++i)
    if (int rc = f()) return rc;
  HIP_CHECK(hipStreamSynchronize(st));
  std::vector<hipEvent_t> ev(2 * reps);
  for (auto &e : ev) HIP_CHECK(hipEventCreate(&e));
  for (int i = 0; i < reps; ++i) {
    HIP_CHECK(hipEventRecord(ev[2 * i], st));
    if (int rc = f()) return rc;
    HIP_CHECK(hipEventRecord(ev[2 * i + 1], st));
  }
  HIP_CHECK(hipStreamSynchronize(st));
  double sum = 0, mn = 1e30;
  for (int i = 0; i < reps; ++i) {
    float ms = 0;
    HIP_CHECK(hipEventElapsedTime(&ms, ev[2 * i], ev[2 * i + 1]));
    sum += ms;
    mn = std::min<double>(mn, ms);
  }
  for (auto &e : ev) (void)hipEventDestroy(e);
  *mean_ms = sum / reps;
  if (min_ms) *min_ms = mn;
  return 0;
}

} // namespace

int main(int argc, char **argv) {
  const Config configs[] = {
      {"tiny", {2, 256, 4, 4, 64, 688, 1024, 2, 0}, {1, 4, 1}, 1, 2, {}},
      {"llama7b_tp8_to_tp2", {32, 4096, 32, 32, 128, 11008, 32000, 2, 0}, {1, 8, 1}, 1, 2, {}},
      {"llama13b_tp4pp2_to_tp2", {40, 5120, 40, 40, 128, 13824, 32000, 2, 0}, {2, 4, 1}, 1, 2, {}},
      {"llama34b_gqa_tp8pp2_to_tp4", {48, 8192, 64, 8, 128, 22016, 32000, 2, 0}, {2, 8, 1}, 1, 4, {0, 2, 4, 6}},
      {"llama70b_gqa_tp8pp4_to_tp4", {80, 8192, 64, 8, 128, 28672, 128256, 2, 0}, {4, 8, 1}, 1, 4, {0, 31}},
  };
  int config = 2, steps = 10, warmup = 3, back = 0, install = 0, graph = 0, offload = 0;
  long long multicast = -1, variant = -1, tile_bytes = 0, part_bytes = 0, mc_block = 0, grid = 0, policy = -2, calib = 0, kind_mask = 0,
            wg_threads = 0, resp_tokens = 0, ceilings = 0, offload_wgs = 0, row_interleave = -1, pf_block = 0, pf_merge = 0;
  unsigned flags = HF_SKIP_OWN;
  std::vector<int32_t> mat_override, train_override, gen_override;
  auto int_list = [](const std::string &list) {
    std::vector<int32_t> out;
    for (size_t p0 = 0; p0 < list.size();) {
      size_t p1 = list.find(',', p0);
      if (p1 == std::string::npos) p1 = list.size();
      out.push_back(std::atoi(list.substr(p0, p1 - p0).c_str()));
      p0 = p1 + 1;
    }
    return out;
  };
  for (int i = 1; i < argc; ++i) {
    const std::string a = argv[i];
    auto val = [&]() -> long long { return i + 1 < argc ? std::atoll(argv[++i]) : 0; };
    if (a == "--config") config = (int)val();
    else if (a == "--steps") steps = (int)val();
    else if (a == "--warmup") warmup = (int)val();
    else if (a == "--back") back = 1;
    else if (a == "--install-own") install = 1;
    else if (a == "--copy-own") flags |= HF_COPY_OWN;
    else if (a == "--vanilla") flags |= HF_GROUPING_VANILLA;
    else if (a == "--from-gen") flags |= HF_GATHER_FROM_GEN;
    else if (a == "--multicast") multicast = val();
    else if (a == "--variant") variant = val();
    else if (a == "--tile-bytes") tile_bytes = val();
    else if (a == "--part-bytes") part_bytes = val();
    else if (a == "--mc-block-bytes") mc_block = val();
    else if (a == "--grid") grid = val();
    else if (a == "--cache-policy") policy = val();
    else if (a == "--calib-copy-bytes") calib = val();
    else if (a == "--kind-mask") kind_mask = val();
    else if (a == "--wg-threads") wg_threads = val();
    else if (a == "--responses") resp_tokens = val();
    else if (a == "--ceilings") ceilings = val();
    else if (a == "--graph") graph = 1;
    else if (a == "--offload") { offload = 1; flags |= HF_PLAN_OFFLOAD; }
    else if (a == "--offload-wgs") offload_wgs = val();
    else if (a == "--row-interleave") row_interleave = val();
    else if (a == "--prefetch-block-bytes") pf_block = val();
    else if (a == "--prefetch-merge") pf_merge = val();
    else if (a == "--mat") mat_override = int_list(i + 1 < argc ? argv[++i] : "");     // ranks to materialise instead of the configuration's
    else if (a == "--train") train_override = int_list(i + 1 < argc ? argv[++i] : ""); // p,t,d instead of the configuration's
    else if (a == "--gen") gen_override = int_list(i + 1 < argc ? argv[++i] : "");     // p_g,t_g instead of the configuration's
    else {
      std::fprintf(stderr, "usage: hfbench [--config 1..5] [--steps K] [--warmup W] [--back | --install-own] [--copy-own] [--vanilla] [--from-gen] "
                           "[--multicast 0|1|2|3] [--variant V] [--tile-bytes B] [--part-bytes B] [--mc-block-bytes B] [--grid G] "
                           "[--cache-policy P] [--calib-copy-bytes B] [--kind-mask M] [--wg-threads 64|256] [--mat r0,r1,..] [--train p,t,d] [--gen pg,tg] "
                           "[--responses TOKENS_PER_REPLICA] [--ceilings SOURCE_BYTES] [--graph] [--offload [--offload-wgs G]] [--row-interleave 0|1] [--prefetch-block-bytes B] [--prefetch-merge 1..8]\n");
      return 2;
    }
  }
  if (config < 1 || config > 5 || steps < 1 || warmup < 0) { std::fprintf(stderr, "bad arguments\n"); return 2; }
  if ((!train_override.empty() && train_override.size() != 3) || (!gen_override.empty() && gen_override.size() != 2)) {
    std::fprintf(stderr, "--train takes p,t,d and --gen takes pg,tg\n");
    return 2;
  }
  Config c = configs[config - 1];
  std::string name = c.name;
  if (!train_override.empty() || !gen_override.empty()) {
    if (!train_override.empty()) c.t = hf_train_layout{train_override[0], train_override[1], train_override[2]};
    if (!gen_override.empty()) { c.pg = gen_override[0]; c.tg = gen_override[1]; }
    c.mat.clear(); // the configuration's subset belongs to its own layout
    name = name.substr(0, name.find('_')) + "_p" + std::to_string(c.t.pp) + "t" + std::to_string(c.t.tp) + "d" + std::to_string(c.t.dp) +
           "_to_p" + std::to_string(c.pg) + "t" + std::to_string(c.tg);
    c.name = name.c_str();
  }
  const std::vector<int32_t> &mat = mat_override.empty() ? c.mat : mat_override;
  hf_gen_layout gl{c.pg, c.tg, flags, mat.empty() ? nullptr : mat.data(), (int32_t)mat.size()};
  hf_plan *plan = nullptr;
  const double t_plan0 = now_ms();
  HF_CHECK(hf_reshard_plan(&c.m, &c.t, &gl, &plan));
  const double plan_ms = now_ms() - t_plan0;
  if (multicast >= 0) HF_CHECK(hf_plan_set_param(plan, HF_PARAM_MULTICAST, multicast));
  if (variant >= 0) HF_CHECK(hf_plan_set_param(plan, HF_PARAM_VARIANT, variant));
  if (tile_bytes) HF_CHECK(hf_plan_set_param(plan, HF_PARAM_TILE_BYTES, tile_bytes));
  if (part_bytes) HF_CHECK(hf_plan_set_param(plan, HF_PARAM_PART_BYTES, part_bytes));
  if (mc_block) HF_CHECK(hf_plan_set_param(plan, HF_PARAM_MC_BLOCK_BYTES, mc_block));
  if (grid) HF_CHECK(hf_plan_set_param(plan, HF_PARAM_GRID_WGS, grid));
  if (policy >= -1) HF_CHECK(hf_plan_set_param(plan, HF_PARAM_CACHE_POLICY, policy));
  if (kind_mask) HF_CHECK(hf_debug_restrict_kinds(plan, (int)kind_mask));
  if (wg_threads) HF_CHECK(hf_plan_set_param(plan, HF_PARAM_WG_THREADS, wg_threads));
  if (offload_wgs) HF_CHECK(hf_plan_set_param(plan, HF_PARAM_OFFLOAD_WGS, offload_wgs));
  if (pf_block) HF_CHECK(hf_plan_set_param(plan, HF_PARAM_PREFETCH_BLOCK_BYTES, pf_block));
  if (pf_merge) HF_CHECK(hf_plan_set_param(plan, HF_PARAM_PREFETCH_MERGE, pf_merge));
  if (row_interleave >= 0) HF_CHECK(hf_plan_set_param(plan, HF_PARAM_ROW_INTERLEAVE, row_interleave));

  const size_t tb = hf_plan_train_bytes(plan), gb = hf_plan_gen_bytes(plan);
  const size_t gen_start = (tb + 4095) / 4096 * 4096;
  char *arena = nullptr;
  HIP_CHECK(hipMalloc(reinterpret_cast<void **>(&arena), gen_start + gb));
  HIP_CHECK(hipMemset(arena, 0x11, gen_start + gb));
  hipStream_t st;
  HIP_CHECK(hipStreamCreate(&st)); // default priority
  char *train = arena, *gen = arena + gen_start;
  HF_CHECK(hf_plan_check_buffers(plan, train, tb, gen, gb));
  const int dir = back ? HF_DIR_GEN_TO_TRAIN : HF_DIR_TRAIN_TO_GEN;
  auto step = [&]() -> int {
    return back ? hf_reshard_back(plan, train, gen, st) : install ? hf_reshard_install_own(plan, train, gen, st) : hf_reshard_execute(plan, train, gen, st);
  };
  for (int i = 0; i < warmup; ++i) HF_CHECK(step());
  HIP_CHECK(hipStreamSynchronize(st));
  std::vector<hipEvent_t> ev(2 * steps);
  for (auto &e : ev) HIP_CHECK(hipEventCreate(&e));
  const double t_host0 = now_ms();
  for (int i = 0; i < steps; ++i) {
    HIP_CHECK(hipEventRecord(ev[2 * i], st));
    HF_CHECK(step());
    HIP_CHECK(hipEventRecord(ev[2 * i + 1], st));
  }
  HIP_CHECK(hipStreamSynchronize(st));
  const double wall_ms = (now_ms() - t_host0) / steps;
  std::vector<float> ms(steps);
  for (int i = 0; i < steps; ++i) HIP_CHECK(hipEventElapsedTime(&ms[i], ev[2 * i], ev[2 * i + 1]));
  std::sort(ms.begin(), ms.end());
  double mean = 0;
  for (float v : ms) mean += v;
  mean /= steps;
  size_t W = hf_plan_bytes_moved(plan, dir), R = hf_plan_unique_src_bytes(plan, dir);
  if (install) { // the own pieces: the training shards of the materialised ranks, once each way
    W = R = hf_plan_bytes_moved(plan, HF_DIR_GEN_TO_TRAIN);
  }
  const long long mc = (back || install) ? 0 : hf_plan_get_param(plan, HF_PARAM_MULTICAST);
  const double alg = (double)W + (mc ? (double)R : (double)W);
  if (calib > 0) { // one dispatch of known traffic: calib bytes read + calib bytes written
    const size_t n = std::min<size_t>({(size_t)calib, tb, gb}) / 16 * 16;
    HF_CHECK(hf_calib_copy(train, gen, n, st));
    HIP_CHECK(hipStreamSynchronize(st));
    std::printf("calib_copy_bytes %zu\n", n);
  }
  std::printf("{\"workload\": \"%s%s\", \"direction\": \"%s\", \"flags\": \"%s\", \"multicast\": %lld, \"variant\": %lld, \"tile_bytes\": %lld, "
              "\"part_bytes\": %lld, \"mc_block_bytes\": %lld, \"bytes_written\": %zu, \"unique_bytes_read\": %zu, "
              "\"algorithmic_bytes\": %.0f, \"ms_mean\": %.4f, \"ms_median\": %.4f, \"ms_min\": %.4f, \"GBps\": %.1f, "
              "\"frac_of_8TBps\": %.4f, \"wall_ms_per_call\": %.4f, \"plan_build_upload_ms\": %.1f}\n",
              c.name, (flags & HF_GROUPING_VANILLA) ? " (vanilla grouping)" : "", back ? "back" : install ? "install_own" : "fwd",
              (flags & HF_COPY_OWN) ? "copy_own" : (flags & HF_GATHER_FROM_GEN) ? "skip_own, gathered from gen_buf" : "skip_own", mc, (long long)hf_plan_get_param(plan, HF_PARAM_VARIANT),
              (long long)hf_plan_get_param(plan, HF_PARAM_TILE_BYTES), (long long)hf_plan_get_param(plan, HF_PARAM_PART_BYTES),
              (long long)hf_plan_get_param(plan, HF_PARAM_MC_BLOCK_BYTES), W, R, alg, mean, ms[steps / 2], ms[0], alg / mean / 1e6,
              alg / mean / 1e6 / 8000.0, wall_ms, plan_ms);
  std::fflush(stdout);

  if (graph) { // the same call captured once and replayed: what a launch-bound transition costs without the host
    hipGraph_t g;
    hipGraphExec_t ge;
    HIP_CHECK(hipStreamBeginCapture(st, hipStreamCaptureModeGlobal));
    HF_CHECK(step());
    HIP_CHECK(hipStreamEndCapture(st, &g));
    HIP_CHECK(hipGraphInstantiate(&ge, g, nullptr, nullptr, 0));
    const int reps = 200;
    for (int i = 0; i < 10; ++i) HIP_CHECK(hipGraphLaunch(ge, st));
    HIP_CHECK(hipStreamSynchronize(st));
    HIP_CHECK(hipEventRecord(ev[0], st));
    const double h0 = now_ms();
    for (int i = 0; i < reps; ++i) HIP_CHECK(hipGraphLaunch(ge, st));
    HIP_CHECK(hipEventRecord(ev[1], st));
    HIP_CHECK(hipStreamSynchronize(st));
    const double h1 = now_ms();
    float tg = 0;
    HIP_CHECK(hipEventElapsedTime(&tg, ev[0], ev[1]));
    // eager back-to-back launches of the same call, no events in between
    HIP_CHECK(hipEventRecord(ev[0], st));
    const double e0 = now_ms();
    for (int i = 0; i < reps; ++i) HF_CHECK(step());
    HIP_CHECK(hipEventRecord(ev[1], st));
    HIP_CHECK(hipStreamSynchronize(st));
    const double e1 = now_ms();
    float te = 0;
    HIP_CHECK(hipEventElapsedTime(&te, ev[0], ev[1]));
    std::printf("{\"workload\": \"%s\", \"launch_mode\": \"back-to-back, %d calls\", \"graph_replay_us_per_call\": %.2f, \"graph_host_us_per_call\": %.2f, "
                "\"eager_us_per_call\": %.2f, \"eager_host_us_per_call\": %.2f}\n",
                c.name, reps, tg * 1e3 / reps, (h1 - h0) * 1e3 / reps, te * 1e3 / reps, (e1 - e0) * 1e3 / reps);
    HIP_CHECK(hipGraphExecDestroy(ge));
    HIP_CHECK(hipGraphDestroy(g));
  }

  if (ceilings > 0) {
    // what the box sustains for plain streams of known traffic: source = the training
    // region, destinations inside the generation region
    const size_t S = std::min<size_t>({(size_t)ceilings, tb, gb / 4}) / 65536 * 65536;
    auto report = [&](const char *what, double traffic, double t) {
      std::printf("{\"ceiling\": \"%s\", \"source_bytes\": %zu, \"traffic_bytes\": %.0f, \"ms\": %.4f, \"GBps\": %.1f, \"frac_of_8TBps\": %.4f}\n", what, S,
                  traffic, t, traffic / t / 1e6, traffic / t / 1e6 / 8000.0);
      std::fflush(stdout);
    };
    double t = 0;
    if (time_calls(st, 2, 5, [&]() { return hf_calib_copy(train, nullptr, S, st); }, &t)) return 1;
    report("read only (grid-stride)", (double)S, t);
    if (time_calls(st, 2, 5, [&]() { return hf_calib_copy(nullptr, gen, S, st); }, &t)) return 1;
    report("write only (grid-stride)", (double)S, t);
    if (time_calls(st, 2, 5, [&]() { return hf_calib_copy(train, gen, S, st); }, &t)) return 1;
    report("copy 1:1 (grid-stride)", 2.0 * S, t);
    HIP_CHECK(hipEventRecord(ev[0], st));
    for (int i = 0; i < 5; ++i) HIP_CHECK(hipMemcpyAsync(gen, train, S, hipMemcpyDeviceToDevice, st));
    HIP_CHECK(hipEventRecord(ev[1], st));
    HIP_CHECK(hipStreamSynchronize(st));
    float tm = 0;
    HIP_CHECK(hipEventElapsedTime(&tm, ev[0], ev[1]));
    report("hipMemcpyAsync device to device", 2.0 * S, tm / 5);
    for (int w : {1024, 4096, 8192}) { // one short-lived workgroup per w bytes, like the library's default kernel
      char what[96];
      if (time_calls(st, 2, 5, [&]() { return hf_calib_fanout(train, nullptr, S, 1, S, HF_FANOUT_REGISTERS, 0, w, st); }, &t)) return 1;
      std::snprintf(what, sizeof what, "read only, %d B per workgroup", w);
      report(what, (double)S, t);
      for (int n_dst : {1, 3, 4}) {
        if (time_calls(st, 2, 5, [&]() { return hf_calib_fanout(nullptr, gen, S, n_dst, S, HF_FANOUT_REGISTERS, 0, w, st); }, &t)) return 1;
        std::snprintf(what, sizeof what, "write only, %d streams, %d B per workgroup", n_dst, w);
        report(what, (double)n_dst * S, t);
      }
    }
    const size_t region = gb / std::max<size_t>(1, (size_t)hf_plan_num_mat(plan)); // distance of two ranks' generation buffers
    const size_t strides[] = {S, (S + (1u << 20)) / 256 * 256, std::max(S, region / 256 * 256)};
    const int wgb[] = {1024, 4096, 8192};
    for (int n_dst : {1, 2, 3, 4, 7}) {
      for (size_t stride : strides) {
        if ((size_t)(n_dst - 1) * stride + S > gb) continue;
        for (int w : wgb) {
          struct { int method; size_t block; const char *name; } forms[] = {
              {HF_FANOUT_REGISTERS, 0, "registers"},
              {HF_FANOUT_CACHE_BLOCKED, (size_t)1 << 20, "cache-blocked 1 MiB"},
              {HF_FANOUT_CACHE_BLOCKED, (size_t)2 << 20, "cache-blocked 2 MiB"},
              {HF_FANOUT_CACHE_BLOCKED, (size_t)4 << 20, "cache-blocked 4 MiB"},
              {HF_FANOUT_PREFETCHED, (size_t)4 << 20, "prefetched 4 MiB"},
              {HF_FANOUT_PREFETCHED, (size_t)8 << 20, "prefetched 8 MiB"},
              {HF_FANOUT_PREFETCHED, (size_t)16 << 20, "prefetched 16 MiB"}};
          for (const auto &f : forms) {
            if (n_dst == 1 && f.method != HF_FANOUT_REGISTERS) continue;
            char what[160];
            std::snprintf(what, sizeof what, "fan-out 1 read : %d writes, %s, %d B per workgroup, stride %zu", n_dst, f.name, w, stride);
            int rc = time_calls(st, 1, 4, [&]() {
              const int r = hf_calib_fanout(train, gen, S, n_dst, stride, f.method, f.block, w, st);
              if (r) std::fprintf(stderr, "hf_calib_fanout: %s\n", hf_last_error());
              return r;
            }, &t);
            if (rc) return 1;
            report(what, (1.0 + n_dst) * S, t);
          }
        }
      }
    }
  }

  if (offload) {
    const size_t hb = hf_plan_remote_bytes(plan), moved = hf_plan_bytes_moved(plan, HF_DIR_OFFLOAD);
    char *host = nullptr;
    const double a0 = now_ms();
    HIP_CHECK(hipHostMalloc(reinterpret_cast<void **>(&host), hb, hipHostMallocDefault));
    std::memset(host, 0x33, hb);
    std::printf("{\"offload_image_bytes\": %zu, \"remote_bytes\": %zu, \"pinned_alloc_and_touch_ms\": %.0f}\n", hb, moved, now_ms() - a0);
    std::fflush(stdout);
    hipStream_t st2;
    HIP_CHECK(hipStreamCreate(&st2)); // default priority
    auto line = [&](const char *what, double bytes, double t) {
      std::printf("{\"link\": \"%s\", \"bytes\": %.0f, \"ms\": %.2f, \"GBps\": %.2f}\n", what, bytes, t, bytes / t / 1e6);
      std::fflush(stdout);
    };
    double t = 0;
    // the box's pinned-copy rate: one hipMemcpyAsync of the same number of bytes each way
    const size_t probe = std::min<size_t>(moved, gb) / 4096 * 4096;
    if (time_calls(st, 1, 2, [&]() { return (int)hipMemcpyAsync(host, gen, probe, hipMemcpyDeviceToHost, st); }, &t)) return 1;
    line("hipMemcpyAsync device to pinned host", (double)probe, t);
    if (time_calls(st, 1, 2, [&]() { return (int)hipMemcpyAsync(gen, host, probe, hipMemcpyHostToDevice, st); }, &t)) return 1;
    line("hipMemcpyAsync pinned host to device", (double)probe, t);
    if (time_calls(st, 1, 2, [&]() { return hf_offload_remote(plan, gen, host, st); }, &t)) { std::fprintf(stderr, "%s\n", hf_last_error()); return 1; }
    line("hf_offload_remote", (double)moved, t);
    if (time_calls(st, 1, 2, [&]() { return hf_reload_remote(plan, host, gen, st); }, &t)) { std::fprintf(stderr, "%s\n", hf_last_error()); return 1; }
    line("hf_reload_remote", (double)moved, t);
    // step 4 next to the offload: hf_reshard_back on this stream, the offload on a second one
    double tb_alone = 0;
    if (time_calls(st, 1, 3, [&]() { return hf_reshard_back(plan, train, gen, st); }, &tb_alone)) return 1;
    hipEvent_t b0, b1, o0, o1;
    for (hipEvent_t *e : {&b0, &b1, &o0, &o1}) HIP_CHECK(hipEventCreate(e));
    // mode 0: the library's offload kernel on the second stream; mode 1: the runtime's copy
    // engine moving the same number of bytes, for comparison
    for (int mode = 0; mode < 2; ++mode) {
      HIP_CHECK(hipDeviceSynchronize());
      const double w0 = now_ms();
      HIP_CHECK(hipEventRecord(o0, st2));
      if (mode == 0) HF_CHECK(hf_offload_remote(plan, gen, host, st2));
      else HIP_CHECK(hipMemcpyAsync(host, gen, probe, hipMemcpyDeviceToHost, st2));
      HIP_CHECK(hipEventRecord(o1, st2));
      HIP_CHECK(hipEventRecord(b0, st));
      HF_CHECK(hf_reshard_back(plan, train, gen, st));
      HIP_CHECK(hipEventRecord(b1, st));
      HIP_CHECK(hipDeviceSynchronize());
      const double w1 = now_ms();
      float tbk = 0, tof = 0;
      HIP_CHECK(hipEventElapsedTime(&tbk, b0, b1));
      HIP_CHECK(hipEventElapsedTime(&tof, o0, o1));
      std::printf("{\"overlap\": \"%s on a second stream next to hf_reshard_back\", \"offload_workgroups\": %lld, \"back_alone_ms\": %.3f, "
                  "\"back_next_to_offload_ms\": %.3f, \"offload_next_to_back_ms\": %.2f, \"offload_GBps\": %.2f, \"wall_ms\": %.2f}\n",
                  mode == 0 ? "hf_offload_remote" : "hipMemcpyAsync device to pinned host", (long long)hf_plan_get_param(plan, HF_PARAM_OFFLOAD_WGS),
                  tb_alone, tbk, tof, (mode == 0 ? moved : probe) / tof / 1e6, w1 - w0);
      std::fflush(stdout);
    }
    HIP_CHECK(hipStreamDestroy(st2));
    HIP_CHECK(hipHostFree(host));
  }

  if (resp_tokens > 0) { // step 3: all-gather of int64 token ids inside the micro-DP groups
    const int N = hf_plan_num_ranks(plan), dg = hf_plan_micro_dp_size(plan);
    const size_t slot = (size_t)resp_tokens * 8;
    char *rin = nullptr, *rout = nullptr;
    HIP_CHECK(hipMalloc(reinterpret_cast<void **>(&rin), slot * N));
    HIP_CHECK(hipMalloc(reinterpret_cast<void **>(&rout), slot * N * dg));
    HIP_CHECK(hipMemset(rin, 0x22, slot * N));
    double t = 0;
    if (time_calls(st, 5, 50, [&]() { return hf_gather_responses(plan, rin, rout, slot, st); }, &t)) return 1;
    const double bytes = 2.0 * slot * N * dg; // every output byte is written once and read once (from one of N slots)
    std::printf("{\"step\": \"response all-gather in micro-DP groups\", \"ranks\": %d, \"micro_dp\": %d, \"slot_bytes\": %zu, "
                "\"bytes_written\": %zu, \"ms\": %.4f, \"GBps_read_plus_write\": %.1f}\n",
                N, dg, slot, slot * N * dg, t, bytes / t / 1e6);
    HIP_CHECK(hipFree(rin));
    HIP_CHECK(hipFree(rout));
  }
  for (auto &e : ev) (void)hipEventDestroy(e);
  hf_plan_destroy(plan);
  HIP_CHECK(hipFree(arena));
  return 0;
}

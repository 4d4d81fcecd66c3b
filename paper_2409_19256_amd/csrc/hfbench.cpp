// hfbench: native driver of the C ABI for profiling runs (rocprofv3 counters and kernel
// traces) without a Python interpreter in the traced process.  It plans one of the five
// benchmark configurations, puts train_buf and gen_buf in one HBM allocation, runs
// hf_reshard_execute / hf_reshard_back and times it with HIP events on the launch stream.
// The buffers hold a constant byte pattern: the copy kernels never look at the values.
// Parity is the business of the test-suite, not of this tool.
#include <hip/hip_runtime.h>

#include <algorithm>
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

int main(int argc, char **argv) {
  const Config configs[] = {
      {"tiny", {2, 256, 4, 4, 64, 688, 1024, 2, 0}, {1, 4, 1}, 1, 2, {}},
      {"llama7b_tp8_to_tp2", {32, 4096, 32, 32, 128, 11008, 32000, 2, 0}, {1, 8, 1}, 1, 2, {}},
      {"llama13b_tp4pp2_to_tp2", {40, 5120, 40, 40, 128, 13824, 32000, 2, 0}, {2, 4, 1}, 1, 2, {}},
      {"llama34b_gqa_tp8pp2_to_tp4", {48, 8192, 64, 8, 128, 22016, 32000, 2, 0}, {2, 8, 1}, 1, 4, {0, 2, 4, 6}},
      {"llama70b_gqa_tp8pp4_to_tp4", {80, 8192, 64, 8, 128, 28672, 128256, 2, 0}, {4, 8, 1}, 1, 4, {0, 31}},
  };
  int config = 2, steps = 10, warmup = 3, back = 0;
  long long multicast = -1, variant = -1, tile_bytes = 0, part_bytes = 0, mc_block = 0, grid = 0, policy = -2, calib = 0, kind_mask = 0, wg_threads = 0, resp_tokens = 0;
  unsigned flags = HF_SKIP_OWN;
  for (int i = 1; i < argc; ++i) {
    const std::string a = argv[i];
    auto val = [&]() -> long long { return i + 1 < argc ? std::atoll(argv[++i]) : 0; };
    if (a == "--config") config = (int)val();
    else if (a == "--steps") steps = (int)val();
    else if (a == "--warmup") warmup = (int)val();
    else if (a == "--back") back = 1;
    else if (a == "--copy-own") flags |= HF_COPY_OWN;
    else if (a == "--vanilla") flags |= HF_GROUPING_VANILLA;
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
    else {
      std::fprintf(stderr, "usage: hfbench [--config 1..5] [--steps K] [--warmup W] [--back] [--copy-own] [--vanilla] [--multicast 0|1|2] "
                           "[--variant V] [--tile-bytes B] [--part-bytes B] [--mc-block-bytes B] [--grid G] [--cache-policy P] "
                           "[--calib-copy-bytes B] [--kind-mask M] [--wg-threads 64|256] [--responses TOKENS_PER_REPLICA]\n");
      return 2;
    }
  }
  if (config < 1 || config > 5 || steps < 1 || warmup < 0) { std::fprintf(stderr, "bad arguments\n"); return 2; }
  const Config &c = configs[config - 1];
  hf_gen_layout gl{c.pg, c.tg, flags, c.mat.empty() ? nullptr : c.mat.data(), (int32_t)c.mat.size()};
  hf_plan *plan = nullptr;
  HF_CHECK(hf_reshard_plan(&c.m, &c.t, &gl, &plan));
  if (multicast >= 0) HF_CHECK(hf_plan_set_param(plan, HF_PARAM_MULTICAST, multicast));
  if (variant >= 0) HF_CHECK(hf_plan_set_param(plan, HF_PARAM_VARIANT, variant));
  if (tile_bytes) HF_CHECK(hf_plan_set_param(plan, HF_PARAM_TILE_BYTES, tile_bytes));
  if (part_bytes) HF_CHECK(hf_plan_set_param(plan, HF_PARAM_PART_BYTES, part_bytes));
  if (mc_block) HF_CHECK(hf_plan_set_param(plan, HF_PARAM_MC_BLOCK_BYTES, mc_block));
  if (grid) HF_CHECK(hf_plan_set_param(plan, HF_PARAM_GRID_WGS, grid));
  if (policy >= -1) HF_CHECK(hf_plan_set_param(plan, HF_PARAM_CACHE_POLICY, policy));
  if (kind_mask) HF_CHECK(hf_plan_set_param(plan, HF_PARAM_KIND_MASK, kind_mask));
  if (wg_threads) HF_CHECK(hf_plan_set_param(plan, HF_PARAM_WG_THREADS, wg_threads));

  const size_t tb = hf_plan_train_bytes(plan), gb = hf_plan_gen_bytes(plan);
  const size_t gen_start = (tb + 4095) / 4096 * 4096;
  char *arena = nullptr;
  HIP_CHECK(hipMalloc(reinterpret_cast<void **>(&arena), gen_start + gb));
  HIP_CHECK(hipMemset(arena, 0x11, gen_start + gb));
  hipStream_t st;
  HIP_CHECK(hipStreamCreate(&st)); // default priority
  char *train = arena, *gen = arena + gen_start;
  const int dir = back ? HF_DIR_GEN_TO_TRAIN : HF_DIR_TRAIN_TO_GEN;
  auto step = [&]() { return back ? hf_reshard_back(plan, train, gen, st) : hf_reshard_execute(plan, train, gen, st); };
  for (int i = 0; i < warmup; ++i) HF_CHECK(step());
  HIP_CHECK(hipStreamSynchronize(st));
  std::vector<hipEvent_t> ev(2 * steps);
  for (auto &e : ev) HIP_CHECK(hipEventCreate(&e));
  for (int i = 0; i < steps; ++i) {
    HIP_CHECK(hipEventRecord(ev[2 * i], st));
    HF_CHECK(step());
    HIP_CHECK(hipEventRecord(ev[2 * i + 1], st));
  }
  HIP_CHECK(hipStreamSynchronize(st));
  std::vector<float> ms(steps);
  for (int i = 0; i < steps; ++i) HIP_CHECK(hipEventElapsedTime(&ms[i], ev[2 * i], ev[2 * i + 1]));
  std::sort(ms.begin(), ms.end());
  double mean = 0;
  for (float v : ms) mean += v;
  mean /= steps;
  const size_t W = hf_plan_bytes_moved(plan, dir), R = hf_plan_unique_src_bytes(plan, dir);
  const long long mc = back ? 0 : hf_plan_get_param(plan, HF_PARAM_MULTICAST);
  const double alg = (double)W + (mc ? (double)R : (double)W);
  if (calib > 0) { // one dispatch of known traffic: calib bytes read + calib bytes written
    const size_t n = std::min<size_t>({(size_t)calib, tb, gb}) / 16 * 16;
    HF_CHECK(hf_calib_copy(train, gen, n, st));
    HIP_CHECK(hipStreamSynchronize(st));
    std::printf("calib_copy_bytes %zu\n", n);
  }
  std::printf("{\"workload\": \"%s%s\", \"direction\": \"%s\", \"multicast\": %lld, \"variant\": %lld, \"tile_bytes\": %lld, "
              "\"part_bytes\": %lld, \"mc_block_bytes\": %lld, \"bytes_written\": %zu, \"unique_bytes_read\": %zu, "
              "\"algorithmic_bytes\": %.0f, \"ms_mean\": %.4f, \"ms_median\": %.4f, \"ms_min\": %.4f, \"GBps\": %.1f, "
              "\"frac_of_8TBps\": %.4f}\n",
              c.name, (flags & HF_GROUPING_VANILLA) ? " (vanilla grouping)" : "", back ? "back" : "fwd", mc, (long long)hf_plan_get_param(plan, HF_PARAM_VARIANT),
              (long long)hf_plan_get_param(plan, HF_PARAM_TILE_BYTES), (long long)hf_plan_get_param(plan, HF_PARAM_PART_BYTES),
              (long long)hf_plan_get_param(plan, HF_PARAM_MC_BLOCK_BYTES), W, R, alg, mean, ms[steps / 2], ms[0], alg / mean / 1e6,
              alg / mean / 1e6 / 8000.0);
  if (resp_tokens > 0) { // step 3: all-gather of int64 token ids inside the micro-DP groups
    const int N = hf_plan_num_ranks(plan), dg = hf_plan_micro_dp_size(plan);
    const size_t slot = (size_t)resp_tokens * 8;
    char *rin = nullptr, *rout = nullptr;
    HIP_CHECK(hipMalloc(reinterpret_cast<void **>(&rin), slot * N));
    HIP_CHECK(hipMalloc(reinterpret_cast<void **>(&rout), slot * N * dg));
    HIP_CHECK(hipMemset(rin, 0x22, slot * N));
    for (int i = 0; i < 5; ++i) HF_CHECK(hf_gather_responses(plan, rin, rout, slot, st));
    HIP_CHECK(hipStreamSynchronize(st));
    HIP_CHECK(hipEventRecord(ev[0], st));
    const int reps = 50;
    for (int i = 0; i < reps; ++i) HF_CHECK(hf_gather_responses(plan, rin, rout, slot, st));
    HIP_CHECK(hipEventRecord(ev[1], st));
    HIP_CHECK(hipStreamSynchronize(st));
    float t = 0;
    HIP_CHECK(hipEventElapsedTime(&t, ev[0], ev[1]));
    t /= reps;
    const double bytes = 2.0 * slot * N * dg; // every output byte is written once and read once (from one of N slots)
    std::printf("{\"step\": \"response all-gather in micro-DP groups\", \"ranks\": %d, \"micro_dp\": %d, \"slot_bytes\": %zu, "
                "\"bytes_written\": %zu, \"ms\": %.4f, \"GBps_read_plus_write\": %.1f}\n",
                N, dg, slot, slot * N * dg, t, bytes / t / 1e6);
    HIP_CHECK(hipFree(rin));
    HIP_CHECK(hipFree(rout));
  }
  hf_plan_destroy(plan);
  HIP_CHECK(hipFree(arena));
  return 0;
}

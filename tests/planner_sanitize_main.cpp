// Host-only driver for the sanitizer test: builds and validates plans with the planner
// compiled under AddressSanitizer + UndefinedBehaviorSanitizer (no HIP involved).
#include <cstdio>
#include <string>
#include <vector>

#include "plan.hpp"

static int run(const hf_model_desc &m, hf_train_layout t, int pg, int tg, unsigned flags, std::vector<int32_t> mat,
               long long tile_bytes, bool validate) {
  hf_gen_layout gl{pg, tg, flags, mat.empty() ? nullptr : mat.data(), (int32_t)mat.size()};
  hf::Plan pl;
  pl.tile_bytes = tile_bytes;
  std::string err;
  int rc = hf::build_plan(m, t, gl, pl, err);
  if (rc != HF_OK) { std::printf("plan failed (%d): %s\n", rc, err.c_str()); return 1; }
  if (validate && (rc = hf::validate_plan(pl, err)) != HF_OK) { std::printf("validate failed (%d): %s\n", rc, err.c_str()); return 1; }
  std::printf("ok: N=%d descs=%zu+%zu tiles=%zu/%zu/%zu\n", pl.N, pl.fwd_peer.size(), pl.fwd_own.size(), pl.tiles_fwd.size(),
              pl.tiles_fwd_mc.size(), pl.tiles_fwd_cb.size());
  return 0;
}

int main() {
  int bad = 0;
  const hf_model_desc tiny{2, 256, 4, 4, 64, 688, 1024, 2, 0}, odd{1, 6, 2, 2, 3, 10, 8, 2, 0}, gqa{4, 24, 8, 4, 4, 28, 32, 2, 0},
      mid{4, 512, 16, 8, 32, 2760, 2000, 2, 0}, l7b{32, 4096, 32, 32, 128, 11008, 32000, 2, 0},
      l70b{80, 8192, 64, 8, 128, 28672, 128256, 2, 0};
  bad += run(tiny, {1, 4, 1}, 1, 2, HF_PLAN_HOST_ONLY, {}, 131072, true);
  bad += run(tiny, {1, 4, 1}, 1, 2, HF_PLAN_HOST_ONLY | HF_COPY_OWN | HF_PLAN_OFFLOAD, {3, 0}, 4096, true);
  bad += run(odd, {1, 2, 1}, 1, 1, HF_PLAN_HOST_ONLY | HF_COPY_OWN, {}, 4096, true);
  bad += run(gqa, {4, 4, 2}, 2, 2, HF_PLAN_HOST_ONLY | HF_PLAN_OFFLOAD, {}, 8192, true);
  bad += run(gqa, {4, 4, 1}, 2, 2, HF_PLAN_HOST_ONLY | HF_GROUPING_VANILLA | HF_COPY_OWN, {}, 8192, true);
  bad += run(mid, {2, 8, 1}, 1, 2, HF_PLAN_HOST_ONLY | HF_PLAN_OFFLOAD, {}, 131072, true);
  bad += run(l7b, {1, 8, 1}, 1, 2, HF_PLAN_HOST_ONLY, {}, 131072, false); // full validation is O(rows): too slow here
  bad += run(l70b, {4, 8, 1}, 1, 4, HF_PLAN_HOST_ONLY | HF_PLAN_OFFLOAD, {0, 31}, 131072, false);
  return bad ? 1 : 0;
}

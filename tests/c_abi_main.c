/* A C99 caller of libhfreshard: shows that include/hfreshard.h is a plain C header and that the
 * library can be driven without C++ or Python.  Host-only plan (no GPU needed): builds the plan of
 * the worked example of Section 5.3 (8 ranks, training 1-4-2, generation 1-2-2-2), prints what a
 * test compares: group coordinates, buffer sizes, descriptor and byte totals. */
#include <stdio.h>
#include <string.h>

#include "hfreshard.h"

int main(void) {
  hf_model_desc m;
  hf_train_layout t;
  hf_gen_layout g;
  hf_plan *plan = NULL;
  int32_t c[6];
  hf_desc d;
  int r, rc;
  size_t i, n, bytes = 0;

  memset(&m, 0, sizeof m);
  memset(&g, 0, sizeof g);
  m.n_layers = 2; m.hidden = 64; m.n_q_heads = 8; m.n_kv_heads = 4; m.head_dim = 8; m.ffn = 96; m.vocab = 128;
  m.elem_bytes = 2; m.tied_embed = 0;
  t.pp = 1; t.tp = 4; t.dp = 2;
  g.pp = 1; g.tp = 2; g.flags = HF_SKIP_OWN | HF_PLAN_HOST_ONLY; g.mat_ranks = NULL; g.n_mat = 0;

  rc = hf_reshard_plan(&m, &t, &g, &plan);
  if (rc != HF_OK) { fprintf(stderr, "plan: %d %s\n", rc, hf_last_error()); return 1; }
  printf("ranks %d micro_dp %d train_bytes %lu gen_bytes %lu\n", hf_plan_num_ranks(plan), hf_plan_micro_dp_size(plan),
         (unsigned long)hf_plan_train_bytes(plan), (unsigned long)hf_plan_gen_bytes(plan));
  for (r = 0; r < hf_plan_num_ranks(plan); ++r) {
    if (hf_plan_rank_coords(plan, r, c) != HF_OK) return 2;
    printf("rank %d dp %d pp %d tp %d gpp %d gtp %d micro %d\n", r, c[0], c[1], c[2], c[3], c[4], c[5]);
  }
  n = hf_plan_num_desc(plan, HF_DIR_TRAIN_TO_GEN);
  for (i = 0; i < n; ++i) {
    if (hf_plan_get_desc(plan, HF_DIR_TRAIN_TO_GEN, i, &d) != HF_OK) return 3;
    bytes += (size_t)d.n_blocks * d.rows * d.row_bytes;
  }
  printf("descriptors %lu bytes %lu moved %lu\n", (unsigned long)n, (unsigned long)bytes,
         (unsigned long)hf_plan_bytes_moved(plan, HF_DIR_TRAIN_TO_GEN));
  rc = hf_plan_validate(plan);
  printf("validate %d\n", rc);
  /* an execution call on a host-only plan is an error, not a crash */
  rc = hf_reshard_execute(plan, (const void *)4096, (void *)(1 << 30), NULL);
  printf("execute_on_host_only_plan %d\n", rc);
  hf_plan_destroy(plan);

  t.tp = 3; /* 3 does not divide the heads */
  rc = hf_reshard_plan(&m, &t, &g, &plan);
  printf("bad_layout %d plan_is_null %d\n", rc, plan == NULL);
  return 0;
}

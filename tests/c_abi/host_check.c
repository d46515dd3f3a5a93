/* Plain C (C99) user of the two C ABIs, host-only: proves that the headers are C, that the
 * library can be driven without Python or torch, and that argument checks work before any
 * GPU is touched.  Built and run by tests/test_c_abi.py. */
#include <stdio.h>
#include <string.h>

#include "bca.h"
#include "lbs.h"

#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      printf("FAILED line %d: %s (bca: %s; lbs: %s)\n", __LINE__, #cond, bca_last_error(), lbs_last_error()); \
      return 1;                                                            \
    }                                                                      \
  } while (0)

int main(void) {
  /* two tensors of 3000 and 500 elements in two buckets; tensor 0 is split between them */
  const uint64_t numel[2] = {3000, 500};
  const uint64_t seg_off[3] = {0, 2, 3};
  bca_segment segs[3];
  bca_plan* plan = NULL;
  bca_tuning tune;
  uint32_t tensor = 0, len = 0, bucket = 0, first = 0, count = 0;
  uint64_t begin = 0;
  const uint8_t mask[2] = {1, 0};
  bca_adam hp = {1e-3, 0.9, 0.999, 1e-6, 0.01};
  float dummy = 0.f;

  memset(segs, 0, sizeof segs);
  segs[0].tensor = 1, segs[0].begin = 0, segs[0].len = 500;
  segs[1].tensor = 0, segs[1].begin = 2000, segs[1].len = 1000;
  segs[2].tensor = 0, segs[2].begin = 0, segs[2].len = 2000;
  memset(&tune, 0, sizeof tune);
  tune.chunk_norm = 1024, tune.chunk_apply = 1024;

  printf("sizeof bca_segment %u bca_tuning %u bca_adam %u lbs_run %u\n", (unsigned)sizeof(bca_segment), (unsigned)sizeof(bca_tuning),
         (unsigned)sizeof(bca_adam), (unsigned)sizeof(lbs_run));
  CHECK(bca_version() >= 1);
  CHECK(bca_plan_create(&plan, -1, 2, numel, 2, seg_off, segs, BCA_GRAD_BF16, &tune) == BCA_OK);
  CHECK(bca_plan_num_buckets(plan) == 2);
  /* tensor 0: [0,1024) [1024,2000) in bucket 1, [2000,2048) [2048,3000) in bucket 0; tensor 1: one chunk */
  CHECK(bca_plan_num_chunks(plan, BCA_TABLE_APPLY) == 5);
  CHECK(bca_plan_num_chunks(plan, BCA_TABLE_LAMB) == 5);
  CHECK(bca_plan_chunk_info(plan, BCA_TABLE_APPLY, 0, &tensor, &begin, &len, &bucket) == BCA_OK);
  CHECK(tensor == 1 && begin == 0 && len == 500 && bucket == 0);
  CHECK(bca_plan_chunk_info(plan, BCA_TABLE_LAMB, 0, &tensor, &begin, &len, &bucket) == BCA_OK);
  CHECK(tensor == 0 && begin == 0 && len == 1024 && bucket == 1);
  CHECK(bca_plan_bucket_chunks(plan, BCA_TABLE_LAMB, 1, &first, &count) == BCA_OK && first == 4 && count == 1);
  CHECK(bca_plan_chunk_info(plan, BCA_TABLE_APPLY, 5, NULL, NULL, NULL, NULL) == BCA_ERR_RANGE);
  CHECK(bca_plan_set_decay_mask(plan, mask) == BCA_OK);
  {
    /* the fused step's work list and lamb_step's runs of tensors, read back */
    uint32_t kind = 9, n_items = bca_plan_num_work_items(plan), i, n_norm = 0, n_adam = 0, t0 = 9, t1 = 9;
    CHECK(n_items >= 5 + 2 && bca_plan_norm_item_chunks(plan) >= 1);
    for (i = 0; i < n_items; ++i) {
      CHECK(bca_plan_work_item(plan, i, &kind, &first, &count) == BCA_OK && kind <= 2);
      if (kind == 0) n_norm += count;
      if (kind == 1) n_adam += count;
    }
    CHECK(n_norm == bca_plan_num_chunks(plan, BCA_TABLE_NORM) && n_adam == 5);
    CHECK(bca_plan_work_item(plan, n_items, &kind, NULL, NULL) == BCA_ERR_RANGE);
    CHECK(bca_plan_num_lamb_runs(plan) == 1 && bca_plan_lamb_run(plan, 0, &t0, &t1) == BCA_OK && t0 == 0 && t1 == 2);
    CHECK(bca_plan_lamb_run(plan, 1, NULL, NULL) == BCA_ERR_RANGE);
  }
  CHECK(adam_step(plan, &hp, 1, NULL) == BCA_ERR_UNBOUND);       /* host-only plan: no kernels */
  CHECK(lamb_step(plan, &hp, 0, NULL, NULL) == BCA_ERR_HPARAM);  /* step counts from 1 */
  CHECK(bucket_clip_adam(plan, &dummy, &hp, 1, 64u, NULL, NULL, NULL, NULL) == BCA_ERR_RANGE);
  bca_plan_destroy(plan);
  tune.lamb_group_elems = 600; /* tensor 0 (3000 elements) is a run of its own, tensor 1 (500) the next */
  CHECK(bca_plan_create(&plan, -1, 2, numel, 2, seg_off, segs, BCA_GRAD_F32, &tune) == BCA_OK);
  CHECK(bca_plan_num_lamb_runs(plan) == 2 && bca_plan_lamb_run(plan, 1, &first, &count) == BCA_OK && first == 1 && count == 2);
  bca_plan_destroy(plan);
  tune.lamb_group_elems = 0;
  segs[2].len = 1999; /* one element of tensor 0 not covered */
  CHECK(bca_plan_create(&plan, -1, 2, numel, 2, seg_off, segs, BCA_GRAD_F32, NULL) == BCA_ERR_LAYOUT && plan == NULL);
  CHECK(strstr(bca_last_error(), "tensor 0") != NULL);

  {
    /* Alg. 1's per-bucket thresholds, and the argument checks of the call that allocates nothing (all of them
     * come before anything touches a GPU) */
    float thr[4] = {0.f, 0.f, 0.f, 0.f};
    uint64_t stats[2];
    CHECK(bca_alg1_thresholds(2.0, 4, thr) == BCA_OK && thr[0] == 1.0f && thr[3] == 1.0f);
    CHECK(bca_alg1_thresholds(0.0, 4, thr) == BCA_ERR_HPARAM);
    CHECK(bca_alg1_thresholds(1.0, 4, NULL) == BCA_ERR_NULL);
    CHECK(bucket_clip_flat(&dummy, ((uint64_t)1 << 28) + 1, BCA_GRAD_F32, &dummy, NULL, NULL, NULL, NULL) == BCA_ERR_RANGE);
    CHECK(strstr(bca_last_error(), "at most") != NULL);
    CHECK(bucket_clip_flat(&dummy, 16, 9, &dummy, NULL, NULL, NULL, NULL) == BCA_ERR_DTYPE);
    CHECK(bucket_clip_flat(NULL, 16, BCA_GRAD_F32, &dummy, NULL, NULL, NULL, NULL) == BCA_ERR_NULL);
    CHECK(bucket_clip_flat(&dummy, 16, BCA_GRAD_F32, NULL, NULL, NULL, NULL, NULL) == BCA_ERR_NULL);
    CHECK(bucket_clip_flat((char*)&dummy + 1, 16, BCA_GRAD_F16, &dummy, NULL, NULL, NULL, NULL) == BCA_ERR_ALIGN);
    CHECK(bca_plan_wait_stats(NULL, stats) == BCA_ERR_NULL);
  }

  {
    /* lengths 1..4 with 10, 0, 5, 5 samples; two strata */
    const uint32_t cum[5] = {0, 10, 10, 15, 20};
    const uint32_t ends[2] = {2, 4};
    lbs_dataset* ds = NULL;
    lbs_run run;
    uint64_t sums[2];
    memset(&run, 0, sizeof run);
    CHECK(lbs_dataset_create(&ds, -1, 4, cum, 2, ends) == 0);
    run.method = LBS_LOCAL_SNAKE, run.local_batch = 4, run.gpus_per_node = 2, run.n_gpus = 8;
    run.quota[0] = 2, run.quota[1] = 2, run.seed = 1, run.n_trials = 3;
    CHECK(lbs_simulate(ds, &run, NULL, NULL, sums, NULL) == LBS_ERR_HOST);   /* valid, but no device */
    run.quota[1] = 1;
    CHECK(lbs_simulate(ds, &run, NULL, NULL, sums, NULL) == LBS_ERR_ARG);
    lbs_dataset_destroy(ds);
    CHECK(lbs_dataset_create(&ds, -1, 4, cum, 2, cum) == LBS_ERR_ARG);
  }
  printf("c abi ok\n");
  return 0;
}

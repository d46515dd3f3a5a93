/* lbs.h -- Monte-Carlo simulation of per-GPU load balance under the paper's
 * batch-forming methods, on one MI355X (gfx950).  Part of libbca.so.
 *
 * What is simulated (Sec. 5.2 "Load balancing effect simulation"; App. C, Table 5):
 * in every trial each of n_gpus GPUs retrieves local_batch sequences at random
 * from a dataset given by its length histogram; a load-balancing method
 * redistributes them; the smallest and the largest per-GPU token count (sum of the
 * lengths a GPU ends up with) are recorded.  The paper averages both over 100 000
 * trials.  Methods (Sec. 4.1, Fig. 3 and Fig. 4; Sec. 3.1 for global presorting):
 *   LBS_NONE          every GPU keeps what it drew from the original dataset
 *   LBS_STRATIFIED    every GPU draws quota[s] sequences from length stratum s
 *   LBS_LOCAL_RASTER  stratified draws, then the gpus_per_node GPUs of a node pool
 *   LBS_LOCAL_SNAKE   their sequences, sort them by length and deal the sorted list
 *                     row by row (a row = gpus_per_node entries): raster = every row
 *                     left to right, snake = every second row right to left
 *   LBS_GLOBAL        draws from the original dataset; all GPUs pool, sort and deal
 *                     row by row over all n_gpus GPUs (raster)
 * The packing method of the same figure needs a pre-packed dataset and is not built.
 *
 * Randomness is counter based, so results do not depend on the order of evaluation:
 * draw number k = ((trial * n_gpus + gpu) * local_batch + j) of a run is the
 * (k+1)-th output of SplitMix64 (Steele, Lea, Flood 2014) seeded with `seed`; its
 * upper 32 bits u select entry (u * n) >> 32 of the n candidate dataset entries
 * (ordered by length).  All results are integers and bit-reproducible.
 *
 * Conventions as in bca.h: 0 on success, negative LBS_ERR_* otherwise (nothing
 * enqueued); compute calls only enqueue on `stream`; lbs_last_error() has a message.
 */
#ifndef LBS_H_
#define LBS_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LBS_NONE 0
#define LBS_STRATIFIED 1
#define LBS_LOCAL_RASTER 2
#define LBS_LOCAL_SNAKE 3
#define LBS_GLOBAL 4

#define LBS_ERR_NULL (-1)  /* a required pointer is NULL                                            */
#define LBS_ERR_ARG (-2)   /* histogram not cumulative, strata not increasing / not ending at max_len,
                              quota not adding up to local_batch, empty stratum with a quota, n_gpus
                              not a multiple of gpus_per_node, unknown method, zero sizes            */
#define LBS_ERR_LIMIT (-3) /* beyond what the kernels are built for (see LBS_MAX_*)                  */
#define LBS_ERR_HIP (-4)   /* a HIP runtime call failed                                             */
#define LBS_ERR_HOST (-5)  /* compute call on a host-only dataset (device -1)                       */

#define LBS_MAX_LEN 1024       /* longest sequence                                   */
#define LBS_MAX_STRATA 8
#define LBS_MAX_LOCAL_BATCH 64 /* sequences a GPU retrieves                          */
#define LBS_MAX_NODE_POOL 1024 /* gpus_per_node * local_batch for the LOCAL methods   */

typedef struct lbs_dataset lbs_dataset; /* opaque: histogram + strata, resident on one device */

/* cum is a HOST array of max_len + 1 entries: cum[0] = 0 and cum[l] = number of
 * dataset entries of length <= l (so cum[max_len] is the dataset size, > 0, < 2^32).
 * stratum_end (HOST, n_strata entries, increasing, last == max_len): stratum s holds
 * lengths stratum_end[s-1] + 1 .. stratum_end[s].  Both are copied.  device >= 0:
 * the GPU that will run the simulation; device = -1: host-only (validation only). */
int lbs_dataset_create(lbs_dataset** out, int device, uint32_t max_len, const uint32_t* cum /*HOST*/,
                       uint32_t n_strata, const uint32_t* stratum_end /*HOST*/);
void lbs_dataset_destroy(lbs_dataset* ds);

typedef struct lbs_run {
  uint32_t method;        /* LBS_*                                                            */
  uint32_t local_batch;   /* sequences per GPU per trial (16 in the paper)                    */
  uint32_t gpus_per_node; /* LOCAL methods: GPUs that pool their sequences (8 in the paper)   */
  uint32_t n_gpus;
  uint32_t quota[LBS_MAX_STRATA]; /* stratified methods: sequences per stratum, sum == local_batch
                                     (Fig. 3: 5, 2, 3, 6); ignored by LBS_NONE and LBS_GLOBAL */
  uint64_t seed;
  uint64_t first_trial; /* trials first_trial .. first_trial + n_trials - 1 are run           */
  uint64_t n_trials;    /* < 2^31                                                             */
} lbs_run;

/* Runs the trials.  trial_min / trial_max (DEVICE [n_trials], either may be NULL)
 * receive every trial's smallest / largest per-GPU token count; sums (DEVICE [2],
 * required) receives the totals of the two over the trials (the paper's averages are
 * sums[i] / n_trials).  A call is a small clearing kernel and one simulation kernel whose
 * workgroups each run a share of the trials; it allocates nothing and keeps no state. */
int lbs_simulate(const lbs_dataset* ds, const lbs_run* run /*HOST*/, uint32_t* trial_min /*DEVICE or NULL*/,
                 uint32_t* trial_max /*DEVICE or NULL*/, uint64_t* sums /*DEVICE [2]*/, void* stream);

/* All five methods of one run in method order (run->method is ignored): exactly what five lbs_simulate calls
 * that differ in `method` only compute, since draw number k of a run does not depend on the method -- LBS_NONE
 * and LBS_GLOBAL see the same draws from the whole dataset, LBS_STRATIFIED and the two LOCAL methods the same
 * stratified draws.  When gpus_per_node and local_batch are powers of two (at most 32 and 64) and n_gpus is at
 * most 8192, one kernel makes each set of draws once; otherwise the five methods run one after the other.
 * trial_min / trial_max: DEVICE [5][n_trials] or NULL; sums: DEVICE [5][2]. */
int lbs_simulate_all(const lbs_dataset* ds, const lbs_run* run /*HOST*/, uint32_t* trial_min /*DEVICE or NULL*/,
                     uint32_t* trial_max /*DEVICE or NULL*/, uint64_t* sums /*DEVICE [5][2]*/, void* stream);

/* Measurement only (not part of the method): runs `iters` rounds of eight independent register chains per lane
 * of one instruction kind in n_workgroups workgroups of 256 threads, so that a caller who times it gets the rate
 * at which this GPU issues that kind -- the evidence behind the "alu" roofline peak the simulation is priced on.
 * Per round and chain: XOR_ADD, MUL_HI_ADD, DPP_ADD and BPERMUTE_ADD issue two instructions, the others one.
 * out: DEVICE [n_workgroups * 256] (one word per thread, written so that the arithmetic is kept). */
#define LBS_PROBE_XOR_ADD 0      /* v_xor_b32 + v_add_u32                  */
#define LBS_PROBE_MUL_LO 1       /* v_mul_lo_u32 (+ add)                   */
#define LBS_PROBE_MUL_HI_ADD 2   /* v_mul_hi_u32 + v_add_u32               */
#define LBS_PROBE_MED3 3         /* v_med3_u32                             */
#define LBS_PROBE_DPP_ADD 4      /* v_mov_b32 with a DPP quad permutation + v_add_u32 */
#define LBS_PROBE_BPERMUTE_ADD 5 /* ds_bpermute_b32 + v_add_u32            */
#define LBS_PROBE_FMA_F32 6      /* v_fma_f32                              */
int lbs_issue_rate_probe(int kind, uint32_t n_workgroups, uint32_t iters, uint32_t* out /*DEVICE*/, void* stream);

const char* lbs_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LBS_H_ */

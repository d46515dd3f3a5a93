/* bca.h -- bucket-wise gradient clipping + Adam (or LAMB) on one MI355X (gfx950).
 *
 * C ABI of libbca.so.  Plain pointers and sizes only; every pointer is marked
 * HOST or DEVICE.  The library implements, as hand-written HIP kernels, the
 * per-GPU part of one training iteration of the paper's Alg. 1 (App. B):
 * for every gradient bucket G_b, clip it by its own L2 norm against the
 * bucket's threshold (Sec. 2.3 defines clipping-by-norm; Sec. 4.2 applies it
 * bucket by bucket, before the all-reduce), then update the parameters with
 * Adam (Alg. 1, last line) or with LAMB, the optimizer the paper compares Adam
 * with (Sec. 2.2).  The all-reduce between the two is not part of this library.
 *
 * Conventions
 *   - All compute calls only enqueue kernels on `stream` (a hipStream_t passed
 *     as void*; NULL is the default stream).  Nothing synchronises with the
 *     host; outputs are valid once the caller has synchronised the stream.
 *   - Return value: 0 on success, a negative BCA_ERR_* otherwise.  On error
 *     nothing has been enqueued.  bca_last_error() gives a message.
 *   - Gradients are fp32, fp16 or bf16; parameters and both moments are fp32.
 *   - The caller owns every gradient / parameter / moment / threshold / norm /
 *     coefficient / status buffer.  The library owns only the plan (chunk
 *     table, partial sums, per-bucket scratch), freed by bca_plan_destroy.
 *   - A plan is bound to one device; calls on one plan must not overlap in time
 *     (they share the plan's scratch).  Different plans are independent.
 */
#ifndef BCA_H_
#define BCA_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct bca_plan bca_plan; /* opaque */

/* gradient storage type */
#define BCA_GRAD_F32 0
#define BCA_GRAD_F16 1
#define BCA_GRAD_BF16 2 /* bfloat16: the upper half of a binary32 */

/* error codes */
#define BCA_OK 0
#define BCA_ERR_NULL (-1)    /* a required pointer is NULL                          */
#define BCA_ERR_LAYOUT (-2)  /* segments do not partition the tensors exactly once  */
#define BCA_ERR_RANGE (-3)   /* bucket range b0 > b1 or b1 > n_buckets, bad option  */
#define BCA_ERR_HPARAM (-4)  /* beta outside [0,1), eps < 0, non-finite lr/wd, step 0 */
#define BCA_ERR_UNBOUND (-5) /* compute call before bca_plan_bind, or host-only plan */
#define BCA_ERR_HIP (-6)     /* a HIP runtime call failed (message has its string)  */
#define BCA_ERR_DTYPE (-7)   /* unknown gradient type                               */
#define BCA_ERR_ALIGN (-8)   /* a tensor pointer is not aligned to its element size */
#define BCA_ERR_NOMEM (-9)   /* out of host memory (bca_last_error() may be empty)   */

/* bits of the device status word written by the clip calls */
#define BCA_STATUS_NONFINITE 1     /* some bucket's sum of squares is Inf or NaN          */
#define BCA_STATUS_BAD_THRESHOLD 2 /* some threshold is <= 0 or NaN: that bucket not clipped */
#define BCA_STATUS_TIMEOUT 4       /* a bounded wait inside a pipelined launch expired; the work it
                                      held back was carried out by the call's finish kernel: the
                                      result is complete and the same bits, the call was only slow */
#define BCA_STATUS_INCOMPLETE 8    /* a work item could not be carried out at all: p, m, v (or g) are
                                      partly updated.  Cannot happen by construction; reported
                                      rather than assumed                                       */

/* flags of bucket_clip_adam */
#define BCA_WRITE_BACK_GRADS 1u       /* also store the scaled gradient into g (what Alg. 1
                                         hands to the all-reduce)                          */
#define BCA_CLIP_WHOLE_GRADIENT 4u    /* clip the whole gradient by its norm with ONE threshold instead
                                         of bucket by bucket (the paper's two baselines, Sec. 3.2):
                                         `thresholds` points to a single float c; all coefs[b] are the
                                         same factor; norms, if given, needs n_buckets + 1 entries and
                                         norms[n_buckets] receives the whole-gradient norm              */
#define BCA_SKIP_STEP_ON_NONFINITE 2u /* if any bucket norm is non-finite, leave g, p, m, v
                                         untouched (status still reports it)               */

/* One contiguous piece of one tensor inside a bucket, in elements. */
typedef struct bca_segment {
  uint32_t tensor;   /* index into the tensor list   */
  uint32_t reserved; /* must be 0                    */
  uint64_t begin;    /* first element of the piece   */
  uint64_t len;      /* number of elements (may be 0) */
} bca_segment;

/* Adam hyper-parameters (App. A, Table 4 lists the ones the paper tunes).
 * Read on the host during the call. */
typedef struct bca_adam {
  double lr;           /* learning rate eta, finite                 */
  double beta1;        /* in [0, 1)                                 */
  double beta2;        /* in [0, 1)                                 */
  double eps;          /* >= 0, added to sqrt(vhat)                 */
  double weight_decay; /* decoupled: p <- p - lr * (u + wd * p)     */
} bca_adam;

/* The same hyper-parameters and the step count in DEVICE memory, for callers that replay a captured HIP graph
 * and so cannot change host-side arguments between replays (what frameworks call a capturable optimizer).
 * After bca_plan_set_device_hyper(plan, dev), adam_step, bucket_clip_adam, lamb_step and bucket_clip_lamb
 * ignore their `hp` (may be NULL) and `step` arguments: each call first enqueues a one-thread kernel that
 * reads *dev on the stream and derives the constants the sweeps use, so whatever the caller has written
 * there on that stream before the call (or the replay) applies.  The values are not validated (the ranges
 * of bca_adam, step >= 1): they are the caller's to keep in range.  dev = NULL goes back to host arguments. */
typedef struct bca_adam_device {
  double lr, beta1, beta2, eps, weight_decay;
  uint64_t step; /* >= 1, counts the current update */
} bca_adam_device;

/* Launch tuning; zero in any field means "library default". */
#define BCA_TUNE_MULTI_LAUNCH 1u    /* bucket_clip_adam as separate norm / finalize / Adam launches per
                                       bucket group instead of the single pipelined launch; likewise
                                       bucket_clip_lamb's norms and first sweep (one group)           */
#define BCA_TUNE_TICKETS 4u          /* single launch: work items are handed out through an atomic
                                       ticket instead of by workgroup index                          */
#define BCA_TUNE_STAGE_TABLE_LDS 2u /* multi-launch kernels: persistent workgroups stage chunk-table
                                       slices in LDS                                                 */
typedef struct bca_tuning {
  uint32_t chunk_norm;   /* largest chunk of the squared-norm pass (one set of partial sums each), elements,
                            multiple of 1024; 0: 16 Ki, what a workgroup fetches in one go                 */
  uint32_t chunk_apply;  /* largest chunk of the scale / Adam passes, elements, multiple of 1024 */
  uint32_t grid_norm;    /* workgroups of the squared-norm kernel (0: one per chunk)            */
  uint32_t grid_apply;   /* workgroups of the scale / Adam kernels (0: one per chunk)           */
  uint32_t unroll_apply; /* 128-bit accesses in flight per lane and array in scale / Adam: 1, 2, 4 */
  uint32_t flags;        /* BCA_TUNE_*                                                          */
  uint64_t group_bytes;  /* bucket_clip_adam walks the buckets in groups of at most this many
                            gradient bytes (norms, then Adam, group by group) so that a group's
                            gradients are still in cache when Adam reads them; 0: default      */
  uint32_t adam_lds_reserve; /* adam_step (and any other Adam sweep that streams the gradients): bytes of LDS
                            each workgroup reserves without using them, which caps the workgroups resident
                            per compute unit (160 KiB each) -- the sweep streams fastest with few
                            wavefronts in flight.  0: default (48 KiB); 1: none; at most 65536       */
  uint32_t spin_limit;   /* pipelined calls (bucket_clip_adam, bucket_clip_lamb): polls of a bucket's
                            ready word after which a waiting work item gives up, is handed to the call's finish
                            kernel and BCA_STATUS_TIMEOUT is reported; 0: default (2^18, about a second).  Small
                            values exist for tests of that path: every kernel still ends normally and the
                            result is the same                                                            */
  uint32_t norm_item_chunks; /* fused calls: consecutive squared-norm chunks one work item reads, 1 .. 4;
                            0: chosen from the bucket sizes so that an item reads 16 Ki .. 64 Ki elements
                            (1 when chunk_norm is given)                                               */
  uint32_t norm_lead;    /* fused calls: bucket groups by which the squared-norm items run ahead of the Adam
                            items in the work list (their gradients must stay cached that long); 0: default */
  uint64_t lamb_group_elems; /* lamb_step: the tensors are swept in runs of consecutive tensors of at most this many
                            elements (a larger tensor is a run of its own), both sweeps of a run before the next run, so
                            that the second sweep reads the moments from cache; 0: default (32 Mi); results do not
                            depend on it                                                                        */
} bca_tuning;

/* which chunk table an introspection call looks at */
#define BCA_TABLE_NORM 0
#define BCA_TABLE_APPLY 1
#define BCA_TABLE_LAMB 2 /* the fine cut again, tensor by tensor (bucket-major order does not apply) */

/* ---- plan -----------------------------------------------------------------
 * A plan records the bucket layout of Alg. 1's G = [G_1 ... G_B]: B buckets,
 * bucket b being the concatenation of segments
 * segments[bucket_seg_off[b] .. bucket_seg_off[b+1]-1] in that order.  Bucket 0
 * is the first one backward produces (the paper's loop runs b = B ... 1, so the
 * model's last tensors come first).  Every element of every tensor must lie in
 * exactly one segment, else BCA_ERR_LAYOUT.  All arrays are HOST memory and are
 * copied.  device >= 0 selects the GPU that will run the plan; device = -1
 * builds a host-only plan (layout validation and chunk table only; compute
 * calls return BCA_ERR_UNBOUND) so that the host logic can be exercised without
 * a GPU.  tuning may be NULL. */
int bca_plan_create(bca_plan** out, int device, uint32_t n_tensors, const uint64_t* tensor_numel /*HOST*/,
                    uint32_t n_buckets, const uint64_t* bucket_seg_off /*HOST [n_buckets+1]*/,
                    const bca_segment* segments /*HOST*/, int grad_dtype, const bca_tuning* tuning /*HOST*/);

/* Attach the tensors.  Each argument is a HOST array of n_tensors DEVICE
 * pointers (grads[t] points to tensor_numel[t] values of the plan's gradient
 * type, the others to fp32).  Pointers of empty tensors may be NULL.  Pointers
 * must be aligned to their element size (BCA_ERR_ALIGN); 16-byte alignment
 * of all four arrays of a tensor lets the kernels use 128-bit accesses.  May
 * be called again when the pointers change.  Synchronous (uploads the table). */
int bca_plan_bind(bca_plan* plan, void* const* grads, float* const* params, float* const* exp_avg,
                  float* const* exp_avg_sq);

/* Per-tensor weight-decay mask: decay is a HOST array of n_tensors bytes, non-zero =
 * weight decay applies to that tensor, zero = exempt (the usual treatment of biases
 * and normalisation weights; the paper tunes one weight decay, App. A Table 4, and
 * does not say which tensors it covers).  NULL restores the default, decay everywhere.
 * Affects adam_step, bucket_clip_adam, lamb_step and bucket_clip_lamb.  May be called
 * before or after bca_plan_bind; on a bound plan it is synchronous (rewrites the tables). */
int bca_plan_set_decay_mask(bca_plan* plan, const uint8_t* decay /*HOST [n_tensors] or NULL*/);

/* Take hyper-parameters and step from device memory (see bca_adam_device); dev must stay valid while set.
 * BCA_ERR_UNBOUND on a host-only plan. */
int bca_plan_set_device_hyper(bca_plan* plan, const bca_adam_device* dev /*DEVICE or NULL*/);

void bca_plan_destroy(bca_plan* plan);

/* Introspection of the host-side plan (no GPU needed).  `table` is BCA_TABLE_NORM,
 * BCA_TABLE_APPLY or BCA_TABLE_LAMB: the layout is cut coarsely for the squared-norm
 * pass, finely for the passes that also write, and finely again in tensor-major
 * order for LAMB. */
uint32_t bca_plan_num_buckets(const bca_plan* plan);
uint32_t bca_plan_num_groups(const bca_plan* plan);
uint32_t bca_plan_norm_item_chunks(const bca_plan* plan); /* squared-norm chunks per work item of the fused step */
uint32_t bca_plan_num_chunks(const bca_plan* plan, int table);
/* For chunk i: tensor index, first element, length, bucket.  Any out pointer may be NULL. */
int bca_plan_chunk_info(const bca_plan* plan, int table, uint32_t i, uint32_t* tensor, uint64_t* begin,
                        uint32_t* len, uint32_t* bucket);
/* The runs of tensors in which lamb_step sweeps the plan (bca_tuning.lamb_group_elems): their number, and the
 * tensors [*first_tensor, *end_tensor) of run i (either pointer may be NULL).  Runs are consecutive and cover all
 * tensors.  BCA_ERR_RANGE for i out of range. */
uint32_t bca_plan_num_lamb_runs(const bca_plan* plan);
int bca_plan_lamb_run(const bca_plan* plan, uint32_t i, uint32_t* first_tensor, uint32_t* end_tensor);

/* The work list of the fused step, in the order its workgroups take it: item i is kind 0 = squared norms of
 * `count` consecutive chunks of BCA_TABLE_NORM starting at `first`, kind 1 = Adam on chunk `first` of
 * BCA_TABLE_APPLY (count 1), kind 2 = stand-in for bucket `first`, which has no elements (count 0).  Every
 * squared-norm item of a bucket comes before every Adam item of that bucket. */
uint32_t bca_plan_num_work_items(const bca_plan* plan);
int bca_plan_work_item(const bca_plan* plan, uint32_t i, uint32_t* kind, uint32_t* first, uint32_t* count);
/* Chunks of bucket b are [first, first + count); for BCA_TABLE_LAMB b is a tensor index. */
int bca_plan_bucket_chunks(const bca_plan* plan, int table, uint32_t b, uint32_t* first, uint32_t* count);

/* ---- compute --------------------------------------------------------------*/

/* ||G_b|| for b in [b0, b1)  (the norm in Alg. 1's test and in Sec. 2.3).
 * norms is a DEVICE array of n_buckets floats indexed by bucket; only entries
 * b0..b1-1 are written.  b0 == b1 is a no-op.  Sums are accumulated in fp32
 * per lane, combined in fp64 in a fixed order: results are bit-reproducible. */
int bucket_clip_norms(bca_plan* plan, uint32_t b0, uint32_t b1, float* norms /*DEVICE*/, void* stream);

/* Clip buckets [b0, b1) in place: with n = norms[b] and c = thresholds[b], if
 * n >= c then G_b <- (c / n) * G_b, else G_b is not touched (Sec. 2.3; Alg. 1
 * passes c / sqrt(B) as every bucket's threshold -- that choice is the
 * caller's).  The factor is computed in fp64 from the fp32 norm, rounded once
 * to fp32 and, if coefs is not NULL, stored in coefs[b] (1 for unclipped
 * buckets).  The product is rounded to the gradient's storage type.  status
 * (DEVICE int32, may be NULL) receives BCA_STATUS_* bits for this call. */
int bucket_clip_apply(bca_plan* plan, uint32_t b0, uint32_t b1, const float* thresholds /*DEVICE [B]*/,
                      const float* norms /*DEVICE [B]*/, float* coefs /*DEVICE [B] or NULL*/,
                      int32_t* status /*DEVICE or NULL*/, void* stream);

/* bucket_clip_norms followed by bucket_clip_apply on buckets [b0, b1) in one call, for the
 * paper's use of the method: a bucket is clipped as soon as backward has produced it,
 * before its all-reduce (Sec. 4.2, Alg. 1).  Same norms, coefficients and scaled
 * gradients, bit for bit.  Two launches: the squared-norm partials, then a kernel whose
 * workgroups each derive their bucket's coefficient from the partials and scale a chunk;
 * no workgroup waits for another.  norms / coefs (DEVICE [B], entries b0..b1-1
 * written) and status (DEVICE int32, written: BCA_STATUS_NONFINITE, _BAD_THRESHOLD as in
 * bucket_clip_apply) may each be NULL. */
int bucket_clip(bca_plan* plan, uint32_t b0, uint32_t b1, const float* thresholds /*DEVICE [B]*/, float* norms,
                float* coefs, int32_t* status, void* stream);

/* bucket_clip for callers that cannot allocate or keep a plan: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  One contiguous bucket of n elements of
 * grad_dtype at g (DEVICE) is clipped in place against *threshold (DEVICE, one float): norm and
 * factor as in bucket_clip_apply, written to *norm / *coef / *status (DEVICE, each may be NULL;
 * status is written, not ORed).  The call allocates nothing and calls no allocating routine: its
 * partial sums live in a fixed array of 512.25 KiB inside the library's device image (every GPU
 * the library runs on holds that array until the process ends), looked up once per device at the
 * first call made with that device current.  Limit: n <= 2^28 elements, else BCA_ERR_RANGE and
 * nothing is enqueued.  g must be on the device that is current at the call.  All calls on one
 * GPU share the array: calls that overlap in time on one GPU (different streams) race; calls in
 * stream order are fine, each call writes what it later reads and needs nothing cleared.
 * Results equal bucket_clip's on a one-tensor, one-bucket plan with chunk_norm = 16384, bit for
 * bit.  Only enqueues (two kernels; three beyond 16 Mi elements). */
int bucket_clip_flat(void* g /*DEVICE*/, uint64_t n, int grad_dtype, const float* threshold /*DEVICE*/,
                     float* norm /*DEVICE or NULL*/, float* coef /*DEVICE or NULL*/,
                     int32_t* status /*DEVICE or NULL*/, void* stream);

/* The per-bucket thresholds Alg. 1 (App. B) compares with: out[b] = c / sqrt(n_buckets) for every b,
 * evaluated in fp64 and rounded once to fp32.  The algorithm's test and assignment both
 * divide by sqrt(B); the sentence above it says "divided by B", which is not followed:
 * only the square root gives sum_b ||G_b||^2 <= c^2, i.e. a clipped whole-gradient norm of
 * at most c, which is the stated purpose.  out is a HOST array; the compute calls take
 * thresholds from DEVICE memory, so the caller uploads it.  BCA_ERR_NULL for out == NULL
 * with n_buckets > 0; BCA_ERR_HPARAM unless c > 0 (Inf allowed: never clips). */
int bca_alg1_thresholds(double c, uint32_t n_buckets, float* out /*HOST [n_buckets]*/);

/* theta <- ADAM(theta, eta, G) over every tensor of the plan, reading the
 * gradients as stored (Alg. 1, last line).  Adam as published by Kingma & Ba
 * with bias correction; step >= 1 counts this update:
 *   m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;
 *   p <- p - lr * ( (m/(1-b1^step)) / (sqrt(v/(1-b2^step)) + eps) + wd * p ). */
int adam_step(bca_plan* plan, const bca_adam* hp /*HOST*/, uint64_t step, void* stream);

/* The fused step: one iteration's loop body of Alg. 1 (App. B) without its all-reduce --
 * for every bucket the test ||G_b|| >= c_b and the assignment G_b <- c_b G_b / ||G_b||
 * (clipping-by-norm, Sec. 2.3, per bucket, Sec. 4.2), then theta <- ADAM(theta, eta, G)
 * on G = [G_1 ... G_B] (the algorithm's last line) -- as norms and clip factors of all
 * buckets followed by one sweep that forms ghat = coef_b * g in registers and applies
 * Adam to it.  g is read, not written, unless BCA_WRITE_BACK_GRADS.  norms / coefs
 * (DEVICE [B]) and status (DEVICE int32, BCA_STATUS_* bits of this call) may each be
 * NULL.  With BCA_SKIP_STEP_ON_NONFINITE or BCA_CLIP_WHOLE_GRADIENT all norms are
 * computed before any update (no pipelining of bucket groups). */
int bucket_clip_adam(bca_plan* plan, const float* thresholds /*DEVICE [B]*/, const bca_adam* hp /*HOST*/,
                     uint64_t step, uint32_t flags, float* norms, float* coefs, int32_t* status, void* stream);

/* LAMB in place of Adam (the optimizer the paper compares Adam with, Sec. 2.2, Sec. 5,
 * App. A; taken as published by You et al. 2020, Alg. 2, with bias correction):
 *   m, v as in adam_step;  u = (m/(1-b1^step)) / (sqrt(v/(1-b2^step)) + eps) + wd * p
 *   trust_t = ||p_t|| / ||u_t|| per tensor t (Euclidean, p before the update; 1 if either
 *   norm is 0);  p <- p - lr * trust_t * u.
 * lamb_step reads the gradients as stored.  bucket_clip_lamb first clips bucket by bucket
 * exactly as bucket_clip_adam does (thresholds, norms, coefs, status as there) and feeds
 * LAMB the scaled gradient formed in registers; flags: BCA_WRITE_BACK_GRADS only.
 * trust (DEVICE [n_tensors], may be NULL) receives the ratios.  Two sweeps over p, m, v:
 * moments + per-tensor sums, then the parameter update; lamb_step carries them out run by
 * run of tensors (bca_tuning.lamb_group_elems; results do not depend on the runs);
 * bucket_clip_lamb runs the squared norms and the first sweep as one pipelined launch, as
 * bucket_clip_adam does with Adam (separate launches under BCA_TUNE_MULTI_LAUNCH; same
 * results bit for bit). */
int lamb_step(bca_plan* plan, const bca_adam* hp /*HOST*/, uint64_t step, float* trust /*DEVICE or NULL*/,
              void* stream);
int bucket_clip_lamb(bca_plan* plan, const float* thresholds /*DEVICE [B]*/, const bca_adam* hp /*HOST*/,
                     uint64_t step, uint32_t flags, float* norms, float* coefs, float* trust, int32_t* status,
                     void* stream);

/* ---- per-kernel timing (for benchmarks) -----------------------------------
 * With profiling on, bucket_clip_adam records HIP events on `stream` around each
 * of its kernels (squared norm, finalize, Adam sweep; once per bucket group), for at most
 * `max_calls` calls after it was switched on (max_calls = 0 switches it off and
 * frees the events).  Calls with BCA_SKIP_STEP_ON_NONFINITE or BCA_CLIP_WHOLE_GRADIENT
 * are not recorded.  bca_plan_profile_read waits for the recorded events and
 * returns the summed duration of each kernel in milliseconds in ms[0..2] and the
 * number of calls summed in *n_calls, then starts a new series.  The single pipelined
 * launch (the default) reports its step kernel in ms[2] and its finish kernel in ms[0]. */
int bca_plan_profile(bca_plan* plan, uint32_t max_calls);
int bca_plan_profile_read(bca_plan* plan, double* ms /*HOST [3]*/, uint32_t* n_calls /*HOST*/);

/* Waiting inside the pipelined launches since the plan was created or this was last called: out[0] = work items
 * that found their bucket's coefficient not yet published at their first look, out[1] = polls they made in all
 * (a poll takes about a third of a microsecond; 2^18 of them is the default bound).  Synchronises the device,
 * then clears the two counters.  Measurement only. */
int bca_plan_wait_stats(bca_plan* plan, uint64_t* out /*HOST [2]*/);

/* Plain copy of nbytes from src to dst (both DEVICE, 16-byte aligned, not
 * overlapping) on the current device.  Not part of the method: a kernel with
 * exactly known HBM traffic (nbytes read, nbytes written) against which hardware
 * counter readings are calibrated. */
int bca_copy_bytes(void* dst, const void* src, uint64_t nbytes, void* stream);

/* Message of the calling thread's last error; valid until its next call. */
const char* bca_last_error(void);

/* Library version, for the loader check. */
int bca_version(void);

#ifdef __cplusplus
}
#endif
#endif /* BCA_H_ */

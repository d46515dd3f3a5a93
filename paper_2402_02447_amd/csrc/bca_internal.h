// Internal declarations shared by the host side (plan, argument checks) and the
// kernel launchers of libbca.  Not part of the public ABI.
#ifndef BCA_INTERNAL_H_
#define BCA_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <utility>
#include <vector>

#include "bca.h"

namespace bca {

// One unit of work: at most chunk_elems consecutive elements of one tensor, all
// in one bucket.  Chunks are stored bucket by bucket, so a bucket's chunks (and
// their partial sums) are contiguous.  The four addresses are filled in by
// bca_plan_bind.
struct alignas(16) Chunk {
  uint64_t g, p, m, v;  // device byte addresses of the chunk's first element
  uint32_t len;         // elements
  uint32_t bucket;
  uint32_t tensor;
  uint32_t flags;       // kChunk* bits
};
constexpr uint32_t kChunkNoDecay = 1u;  // the chunk's tensor is exempt from weight decay
static_assert(sizeof(Chunk) == 48, "chunk table entries are 3 x 16 bytes");

struct ChunkInfo {  // host-side description, independent of addresses
  uint32_t tensor;
  uint32_t len;
  uint64_t begin;
  uint32_t bucket;
};

// One cut of the layout into chunks.  A plan holds three: a coarse one for the
// squared-norm pass (fewer partial sums), a fine one for the passes that read
// and write (scale, Adam), where short-lived workgroups stream best, and a fine
// one in tensor-major order for LAMB, whose trust ratio needs per-tensor sums.
struct Table {
  uint32_t chunk_elems = 0;
  std::vector<ChunkInfo> chunks;     // bucket-major
  std::vector<uint32_t> bucket_off;  // [n_buckets + 1] first chunk of each bucket
  Chunk* d_chunks = nullptr;         // device copy with addresses (after bind)
  uint32_t* d_bucket_off = nullptr;
};

// Adam constants, computed in fp64 on the host and rounded once to fp32.
struct AdamK {
  float b1, omb1;    // beta1, 1 - beta1
  float b2, omb2;    // beta2, 1 - beta2
  float rbc1, rbc2;  // 1 / (1 - beta1^t), 1 / (1 - beta2^t)
  float eps;
  float neg_lr;  // -lr
  float wd;
  double lr;     // LAMB: the step -lr * trust_t is formed in fp64 per tensor and rounded once
  const AdamK* from;  // device copy to use instead of this one (hyper-parameters kept in device memory), or null
};

constexpr uint32_t kBlock = 256;          // threads per workgroup (4 wavefronts)
constexpr uint32_t kWaves = kBlock / 64;  // wavefronts per workgroup
constexpr uint32_t kSlice = 64;           // chunk-table entries staged in LDS at a time
// Squared-norm chunk: partial sums are filed per 16 Ki elements (four doubles each).  That is what one
// workgroup fetches in one go (16 or 8 128-bit loads per lane), which is what a single bucket needs to be read
// fast; the fused step hands out 1, 2 or 4 consecutive chunks per work item, so that an item reads
// 16 Ki .. 64 Ki elements.
constexpr uint32_t kDefaultChunkNorm = 16384;
constexpr uint32_t kSmallNormGrid = 2048;       // squared-norm launches of at most this many workgroups fetch 16 pieces per lane at a time
// bucket_clip derives the coefficient in every workgroup from the bucket's partial sums; beyond this many chunks in
// one bucket (64 MiB of fp32) that costs more than a finalize launch of its own
constexpr uint32_t kMaxChunksForInlineFinalize = 1024;
constexpr uint32_t kMaxNormItemChunks = 4;
constexpr uint32_t kMinNormItemElems = 16384, kMaxNormItemElems = 65536;
constexpr uint32_t kDefaultChunkApply = 1024;
// Buckets are pipelined in groups of about this many elements (at least one bucket):
// large enough that a group's norms are done before its Adam items start, small enough
// that two groups' gradients stay in the Infinity Cache (measured optimum on MI355X).
constexpr uint64_t kDefaultGroupElems = 8ull << 20;
// A stand-alone squared-norm pass keeps the gradients cacheable for the pass that follows (scale, Adam) as long as
// the range is at most this many bytes: half of the 256 MB Infinity Cache.  A larger range is gone from the cache
// before it is read again, and streams faster with non-temporal loads (measured on MI355X, BERT-Large, all buckets
// in one call: 202 instead of 225 us).
constexpr uint64_t kKeepCachedBytes = 128ull << 20;
// lamb_step: tensors are swept in runs of at most this many elements, both sweeps of a run before the next run, so
// that the second sweep reads the moments from cache (measured on MI355X, BERT-Large: 16 Mi 2.20 ms, 32 Mi 2.04,
// 48 Mi 2.04, 64 Mi 2.11, one run 2.18; the gain of short runs is eaten by their three launches each).
constexpr uint64_t kLambGroupElems = 32ull << 20;
// The stand-alone Adam sweep streams 3-5 % faster with three workgroups (twelve wavefronts) per compute unit
// than with all eight: fewer requests in flight suit the four-read / three-write mix (measured on MI355X:
// BERT-Large 1.614 -> 1.537 ms, BERT-Base 0.529 -> 0.511 ms).  48 KiB of the 160 KiB LDS per workgroup give that.
// The fused single-launch step does not gain from it (its items wait on each other) and does not use it.
constexpr uint32_t kDefaultAdamLdsReserve = 48u << 10;
constexpr uint32_t kDefaultSpinLimit = 1u << 18;  // polls of a ready word before a waiting item gives up (about a second)

// How a streaming kernel is launched.
struct Launch {
  uint32_t grid;    // workgroups
  uint32_t unroll;  // 128-bit accesses in flight per lane and array in the scale / Adam sweeps: 1, 2 or 4
  bool staged;      // persistent grid staging its table entries in LDS (else one uniform entry load per chunk)
  bool g_keep;      // gradients are loaded with the normal (cacheable) policy because they are read again soon
  uint32_t lds;     // Adam sweep (k_adam) only: bytes of LDS a workgroup reserves without using them, which caps
                    // how many workgroups a compute unit holds at once
};

// Device-side state of the pipelined launch (k_step, followed by its finish kernel).
// Control words, each in its own 128-byte line: eight ticket counters (one per XCD) at
// kCtlTicket + 32 y; the epoch (number of the current call, never 0); the abort flag; the number
// of work items whose wait expired (their indices are in StepState::skipped); the status bits
// collected during the call.  The finish kernel of a call leaves all of them ready for the next call.
enum : uint32_t {
  kCtlTicket = 0,
  kCtlEpoch = 256,
  kCtlAbort = 288,
  kCtlSkipped = 320,
  kCtlStatus = 352,
  // statistics: kStatSlots lines of 32 words, slot = workgroup index mod kStatSlots; word 0: items of that slot that
  // found their bucket not ready at their first look, words 2..3 (64 bits): the polls they made in all.  Only
  // items that waited touch them, and spread over many lines so that they do not queue up behind one address.
  kCtlStats = 384,
  kStatSlots = 256,
  kCtlWords = kCtlStats + 32 * kStatSlots
};
// Work items of k_step: kind in bits 30..31; kItemAdam: apply-table chunk in bits 0..29; kItemNorm: first
// norm-table chunk in bits 0..27 and the number of consecutive chunks minus one in bits 28..29; kItemEmpty: bucket.
constexpr uint32_t kItemNorm = 0u, kItemAdam = 1u, kItemEmpty = 2u;
struct StepState {
  const Chunk* norm_tab;
  const Chunk* apply_tab;
  const uint32_t* norm_bucket_off;  // [B + 1] chunks of the norm table per bucket
  double* partials;                 // kWaves per norm chunk
  uint32_t* arrived;                // [B] squared-norm workgroups done per bucket
  unsigned long long* ready;        // [B] (epoch << 32) | bits of the bucket's coefficient
  uint32_t* ctl;                    // [kCtlWords] see kCtl*
  uint32_t* skipped;                // [chunks of the apply table] apply-table indices of items whose wait expired
  const uint32_t* apply_to_lamb;    // LAMB: place of every apply-table chunk in the tensor-major table
  double* lamb_sums;                // LAMB: two sums per chunk, in tensor-major order
  uint32_t skipped_cap;             // entries of `skipped`
  uint32_t spin_limit;              // polls of a ready word before a waiting item gives up
};

// Kernel launchers (bca_kernels.hip).  All enqueue on `stream` and return the
// launch's hipError_t.  c0/n: first chunk and number of chunks.  partials holds
// kWaves doubles per chunk of the norm table.
hipError_t launch_sqnorm(int gdt, const Chunk* table, uint32_t c0, uint32_t n, double* partials, int32_t* status,
                         const Launch& L, hipStream_t stream);
// norms/coefs/status may alias plan scratch.  thresholds == nullptr: norms only.
// bucket_sq (may be null) receives the buckets' fp64 sums of squares.
hipError_t launch_finalize(const double* partials, const uint32_t* bucket_chunk_off, uint32_t b0, uint32_t b1,
                           const float* thresholds, float* norms, float* coefs, int32_t* status, double* bucket_sq,
                           hipStream_t stream);
// One coefficient for all buckets from the whole-gradient norm and the single threshold *c.
hipError_t launch_whole_coef(const double* bucket_sq, uint32_t n_buckets, const float* c, float* whole_norm,
                             float* coefs, int32_t* status, hipStream_t stream);
hipError_t launch_coefs(uint32_t b0, uint32_t b1, const float* thresholds, const float* norms, float* coefs,
                        int32_t* status, hipStream_t stream);
hipError_t launch_scale(int gdt, const Chunk* table, uint32_t c0, uint32_t n, const float* coefs, const Launch& L,
                        hipStream_t stream);
// coefs == nullptr: plain Adam on the stored gradient.  skip_status != nullptr:
// the kernel returns at once if (*skip_status & BCA_STATUS_NONFINITE).
hipError_t launch_adam(int gdt, const Chunk* table, uint32_t c0, uint32_t n, const float* coefs, bool write_back,
                       const int32_t* skip_status, const AdamK& k, const Launch& L, hipStream_t stream);

// The whole fused step: one k_step workgroup per work item, then the finish kernel.  `between`
// (may be null) is recorded between the two kernels.
hipError_t launch_step(int gdt, const StepState& st, const uint32_t* work, uint32_t n_work, const float* thresholds,
                       float* norms, float* coefs, int32_t* status, bool write_back, const AdamK& k, uint32_t unroll,
                       bool tickets, bool lamb, hipEvent_t between, hipStream_t stream);

// Second launch of bucket_clip (after launch_sqnorm with a status word, which clears it):
// per squared-norm chunk, the bucket's norm and coefficient from the partial sums, then the chunk scaled.
hipError_t launch_clip_scale(int gdt, const Chunk* norm_tab, uint32_t cn0, uint32_t n, const uint32_t* bucket_chunk_off,
                             uint32_t b0, uint32_t b1, const double* partials, const float* thresholds, float* norms,
                             float* coefs, int32_t* status, hipStream_t stream);
hipError_t launch_copy(void* dst, const void* src, uint64_t nbytes, hipStream_t stream);

// bucket_clip_flat: one contiguous bucket of n <= kFlatMaxElems elements at g, clipped in place with partial
// sums in the library's fixed device array.  `device` is the current device, below kFlatMaxDevices.
constexpr uint64_t kFlatMaxElems = 1ull << 28;
constexpr uint32_t kFlatChunkNorm = 16384;
constexpr int kFlatMaxDevices = 64;
hipError_t launch_clip_flat(int device, int gdt, void* g, uint64_t n, const float* threshold, float* norm, float* coef,
                            int32_t* status, hipStream_t stream);

// LAMB (tensor-major table `table` of n chunks; tensor_off[t] = first chunk of tensor t).
// Stage 1: moments, per-chunk sums of p^2 and update^2 (2 doubles per chunk in `sums`);
// coefs == nullptr: gradients as stored.  Trust: per tensor, ratio and step scale.
// Stage 2: p <- p + scale_t * update, the update recomputed from the stored moments.
hipError_t launch_lamb_moments(int gdt, const Chunk* table, uint32_t n, const float* coefs, bool write_back,
                               double* sums, bool keep, const AdamK& k, hipStream_t stream);
// Derives the sweeps' constants from hyper-parameters in device memory (one thread).
hipError_t launch_hyper(const bca_adam_device* dev, AdamK* out, hipStream_t stream);
hipError_t launch_lamb_trust(const double* sums, const uint32_t* tensor_off, uint32_t n_tensors, const AdamK& k,
                             float* trust, float* scale, hipStream_t stream);
hipError_t launch_lamb_update(const Chunk* table, uint32_t n, const float* scale, const AdamK& k,
                              hipStream_t stream);

void set_error(const std::string& msg);

}  // namespace bca

struct bca_plan {
  int device = -1;  // -1: host-only
  int grad_dtype = BCA_GRAD_F32;
  uint32_t n_tensors = 0, n_buckets = 0;
  uint32_t grid_norm = 0, grid_apply = 0;  // 0: one workgroup per chunk
  uint32_t unroll_apply = 1;
  uint32_t adam_lds_reserve = 0;  // bytes; see bca_tuning::adam_lds_reserve
  uint32_t norm_item_chunks = 1;  // consecutive norm-table chunks per squared-norm item of the fused step
  uint32_t norm_lead = 1;         // bucket groups by which the squared-norm items run ahead of the Adam items
  uint32_t spin_limit = 0;        // see bca_tuning::spin_limit (default already applied)
  const bca_adam_device* hyper_dev = nullptr;  // hyper-parameters in device memory, when set
  bca::AdamK* d_adamk = nullptr;  // the constants derived from them by k_hyper
  uint32_t tune_flags = 0;
  bool bound = false;
  std::vector<uint64_t> tensor_numel;
  bca::Table norm_tab, apply_tab;
  // LAMB: the fine cut again, tensor by tensor (chunks of tensor t are tensor_off[t] .. tensor_off[t+1]-1)
  bca::Table lamb_tab;
  std::vector<std::pair<uint32_t, uint32_t>> lamb_groups;  // runs of consecutive tensors [first, last) swept together
  std::vector<uint32_t> tensor_off;
  uint32_t* d_tensor_off = nullptr;
  uint32_t* d_apply_to_lamb = nullptr;  // for every chunk of apply_tab, its index in lamb_tab
  double* d_lamb_sums = nullptr;   // 2 per chunk of lamb_tab: sum p^2, sum update^2
  float* d_trust = nullptr;        // n_tensors
  float* d_lamb_scale = nullptr;   // n_tensors: -lr * trust
  // what bca_plan_bind was given, kept so that the tables can be written again (decay mask)
  std::vector<uint64_t> bound_g, bound_p, bound_m, bound_v;
  std::vector<uint8_t> decay;      // per tensor: 1 = weight decay applies (default), 0 = exempt
  // the fused call walks the buckets in groups [first, last)
  std::vector<std::pair<uint32_t, uint32_t>> groups;
  // work list of the single-launch step: (kind << 30) | index, in pipeline order
  std::vector<uint32_t> work;
  uint32_t* d_work = nullptr;
  uint32_t* d_arrived = nullptr;
  unsigned long long* d_ready = nullptr;
  uint32_t* d_ctl = nullptr;
  uint32_t* d_skipped = nullptr;
  // device memory owned by the plan
  double* d_partials = nullptr;
  float* d_norms = nullptr;        // n_buckets + 1 (the last one: whole-gradient norm)
  double* d_bucket_sq = nullptr;   // n_buckets
  float* d_coefs = nullptr;
  int32_t* d_status = nullptr;
  // per-kernel timing of the fused call: 1 + 3 * groups events per profiled call
  std::vector<hipEvent_t> prof_events;
  uint32_t prof_calls = 0;
};

#endif  // BCA_INTERNAL_H_

// Load-balancing simulation for gfx950 (MI355X): host entry points and kernels.
// See lbs.h for what is simulated and for the contract of every call.
//
// One workgroup (256 threads, four wavefronts) runs one trial.  The dataset's
// cumulative histogram sits in LDS; a draw is one SplitMix64 output (a handful of
// 64-bit integer operations) and a binary search over the histogram.  Nothing here
// is a contraction or a stream over HBM: the work is integer ALU and LDS traffic,
// the outputs are two words per trial.
//   NONE / STRATIFIED : a thread owns whole GPUs; 16 draws, one sum each.
//   LOCAL_*           : a wavefront owns a node: its lanes draw the node's pool into
//                       LDS (padded to a power of two with a sentinel above every
//                       length), sort it there with a bitonic network (log^2 stages
//                       of independent compare-exchanges, one pair per lane), and add
//                       up each GPU's column in raster or snake order.
//   GLOBAL            : lengths are small integers, so the trial's pool of
//                       n_gpus * local_batch draws is sorted by counting: an LDS
//                       histogram, a block-wide prefix sum, and the entry at sorted
//                       position q found by binary search in the running counts.
// Per-trial minimum and maximum are combined with shuffles and LDS; the two sums
// over trials with 64-bit integer atomics (integer addition is associative, so the
// result does not depend on the order).

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cstdio>
#include <new>
#include <string>
#include <vector>

#include "lbs.h"

struct lbs_dataset {
  int device = -1;
  uint32_t max_len = 0, n_strata = 0;
  std::vector<uint32_t> cum, stratum_end;
  uint32_t* d_cum = nullptr;
};

namespace lbs {
namespace {

constexpr uint32_t kBlock = 256, kWaves = 4;

thread_local std::string g_error;
int fail(int code, const std::string& msg) {
  g_error = msg;
  return code;
}

struct Params {  // by-value kernel argument
  uint32_t max_len, local_batch, gpus_per_node, n_gpus, snake, stratified;
  uint32_t total;                             // dataset size
  uint32_t slot_lo[LBS_MAX_LOCAL_BATCH];      // stratified: entries before the stratum of a GPU's j-th draw
  uint32_t slot_size[LBS_MAX_LOCAL_BATCH];    //             entries in that stratum
  uint64_t seed, first_trial;
};

__device__ __forceinline__ uint64_t splitmix64(uint64_t seed, uint64_t k) {
  uint64_t z = seed + (k + 1) * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// Smallest l in [1, max_len] with counts[l] > index (counts is non-decreasing).
__device__ __forceinline__ uint32_t first_above(const uint32_t* counts, uint32_t max_len, uint32_t index) {
  uint32_t lo = 1, hi = max_len;
  while (lo < hi) {
    const uint32_t mid = (lo + hi) >> 1;
    if (counts[mid] > index) hi = mid;
    else lo = mid + 1;
  }
  return lo;
}

// Length of the j-th sequence GPU `gpu` retrieves in trial `trial`.
__device__ __forceinline__ uint32_t draw(const Params& P, const uint32_t* s_cum, uint64_t trial, uint32_t gpu, uint32_t j) {
  const uint64_t k = (trial * P.n_gpus + gpu) * (uint64_t)P.local_batch + j;
  const uint64_t u = splitmix64(P.seed, k) >> 32;
  const uint32_t index = P.stratified ? P.slot_lo[j] + (uint32_t)((u * P.slot_size[j]) >> 32)
                                      : (uint32_t)((u * P.total) >> 32);
  return first_above(s_cum, P.max_len, index);
}

__device__ __forceinline__ void load_histogram(uint32_t* s_cum, const uint32_t* __restrict__ cum, uint32_t max_len) {
  for (uint32_t i = threadIdx.x; i <= max_len; i += kBlock) s_cum[i] = cum[i];
  __syncthreads();
}

// Combines the threads' running minimum and maximum and lets thread 0 publish the trial's result.
__device__ __forceinline__ void finish_trial(uint32_t lo, uint32_t hi, uint32_t* s_lo, uint32_t* s_hi,
                                             uint32_t* trial_min, uint32_t* trial_max, unsigned long long* sums) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    lo = min(lo, (uint32_t)__shfl_xor((int)lo, off, 64));
    hi = max(hi, (uint32_t)__shfl_xor((int)hi, off, 64));
  }
  if ((threadIdx.x & 63u) == 0) s_lo[threadIdx.x >> 6] = lo, s_hi[threadIdx.x >> 6] = hi;
  __syncthreads();
  if (threadIdx.x == 0) {
    lo = min(min(s_lo[0], s_lo[1]), min(s_lo[2], s_lo[3]));
    hi = max(max(s_hi[0], s_hi[1]), max(s_hi[2], s_hi[3]));
    if (trial_min) trial_min[blockIdx.x] = lo;
    if (trial_max) trial_max[blockIdx.x] = hi;
    atomicAdd(&sums[0], (unsigned long long)lo);
    atomicAdd(&sums[1], (unsigned long long)hi);
  }
}

__global__ __launch_bounds__(64) void k_lbs_clear(unsigned long long* sums) {
  if (threadIdx.x < 2) sums[threadIdx.x] = 0ull;
}

// NONE and STRATIFIED: no redistribution.
__global__ __launch_bounds__(kBlock) void k_lbs_keep(const Params P, const uint32_t* __restrict__ cum,
                                                      uint32_t* trial_min, uint32_t* trial_max,
                                                      unsigned long long* sums) {
  __shared__ uint32_t s_cum[LBS_MAX_LEN + 1];
  __shared__ uint32_t s_lo[kWaves], s_hi[kWaves];
  load_histogram(s_cum, cum, P.max_len);
  const uint64_t trial = P.first_trial + blockIdx.x;
  uint32_t lo = 0xffffffffu, hi = 0u;
  for (uint32_t g = threadIdx.x; g < P.n_gpus; g += kBlock) {
    uint32_t tokens = 0;
    for (uint32_t j = 0; j < P.local_batch; ++j) tokens += draw(P, s_cum, trial, g, j);
    lo = min(lo, tokens), hi = max(hi, tokens);
  }
  finish_trial(lo, hi, s_lo, s_hi, trial_min, trial_max, sums);
}

// LOCAL_RASTER and LOCAL_SNAKE: pool, sort and deal within every node.
__global__ __launch_bounds__(kBlock) void k_lbs_local(const Params P, const uint32_t* __restrict__ cum,
                                                       uint32_t* trial_min, uint32_t* trial_max,
                                                       unsigned long long* sums) {
  __shared__ uint32_t s_cum[LBS_MAX_LEN + 1];
  __shared__ uint32_t s_pool[kWaves][LBS_MAX_NODE_POOL];
  __shared__ uint32_t s_lo[kWaves], s_hi[kWaves];
  load_histogram(s_cum, cum, P.max_len);
  const uint64_t trial = P.first_trial + blockIdx.x;
  const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
  const uint32_t n_nodes = P.n_gpus / P.gpus_per_node;
  const uint32_t pool = P.gpus_per_node * P.local_batch;
  uint32_t padded = 2;  // the network sorts a power of two
  while (padded < pool) padded <<= 1;
  uint32_t* mine = s_pool[wave];
  uint32_t lo = 0xffffffffu, hi = 0u;
  // Every wavefront makes the same number of rounds and stages, so the barriers below are
  // met by all; a wavefront without a node in the last round only keeps them company.
  for (uint32_t base = 0; base < n_nodes; base += kWaves) {
    const uint32_t node = base + wave;
    const bool active = node < n_nodes;
    if (active)
      for (uint32_t i = lane; i < padded; i += 64u)
        mine[i] = i < pool ? draw(P, s_cum, trial, node * P.gpus_per_node + i / P.local_batch, i % P.local_batch)
                           : 0xffffffffu;
    __syncthreads();
    for (uint32_t k = 2; k <= padded; k <<= 1)
      for (uint32_t j = k >> 1; j > 0; j >>= 1) {
        if (active)
          for (uint32_t t = lane; t < (padded >> 1); t += 64u) {
            const uint32_t a = ((t & ~(j - 1u)) << 1) | (t & (j - 1u));  // t with a 0 inserted at j's bit
            const uint32_t b = a | j;
            const uint32_t x = mine[a], y = mine[b];
            const bool ascending = (a & k) == 0u;
            if ((x > y) == ascending) mine[a] = y, mine[b] = x;
          }
        __syncthreads();
      }
    if (active)
      for (uint32_t c = lane; c < P.gpus_per_node; c += 64u) {
        uint32_t tokens = 0;
        for (uint32_t r = 0; r < P.local_batch; ++r) {
          const uint32_t col = (P.snake && (r & 1u)) ? P.gpus_per_node - 1u - c : c;  // position in the row dealt to GPU c
          tokens += mine[r * P.gpus_per_node + col];
        }
        lo = min(lo, tokens), hi = max(hi, tokens);
      }
    __syncthreads();
  }
  finish_trial(lo, hi, s_lo, s_hi, trial_min, trial_max, sums);
}

// GLOBAL: pool, sort and deal over all GPUs.
__global__ __launch_bounds__(kBlock) void k_lbs_global(const Params P, const uint32_t* __restrict__ cum,
                                                        uint32_t* trial_min, uint32_t* trial_max,
                                                        unsigned long long* sums) {
  __shared__ uint32_t s_cum[LBS_MAX_LEN + 1];
  __shared__ uint32_t s_cnt[LBS_MAX_LEN + 1];  // first a histogram of the trial's draws, then its running sum
  __shared__ uint32_t s_scan[kBlock];
  __shared__ uint32_t s_lo[kWaves], s_hi[kWaves];
  load_histogram(s_cum, cum, P.max_len);
  const uint64_t trial = P.first_trial + blockIdx.x;
  const uint32_t tid = threadIdx.x;
  for (uint32_t i = tid; i <= P.max_len; i += kBlock) s_cnt[i] = 0u;
  __syncthreads();
  const uint32_t pool = P.n_gpus * P.local_batch;
  for (uint32_t i = tid; i < pool; i += kBlock)
    atomicAdd(&s_cnt[draw(P, s_cum, trial, i / P.local_batch, i % P.local_batch)], 1u);
  __syncthreads();
  // running sum over lengths: thread t owns a contiguous piece, pieces are combined by a doubling scan
  const uint32_t per = (P.max_len + 1u + kBlock - 1u) / kBlock;
  const uint32_t a = tid * per, b = min(a + per, P.max_len + 1u);
  uint32_t piece = 0;
  for (uint32_t i = a; i < b; ++i) piece += s_cnt[i];
  s_scan[tid] = piece;
  __syncthreads();
  for (uint32_t d = 1; d < kBlock; d <<= 1) {
    const uint32_t add = tid >= d ? s_scan[tid - d] : 0u;
    __syncthreads();
    s_scan[tid] += add;
    __syncthreads();
  }
  uint32_t run = s_scan[tid] - piece;  // draws with a length below this thread's piece
  for (uint32_t i = a; i < b; ++i) {
    run += s_cnt[i];
    s_cnt[i] = run;  // draws of length <= i
  }
  __syncthreads();
  uint32_t lo = 0xffffffffu, hi = 0u;
  for (uint32_t c = tid; c < P.n_gpus; c += kBlock) {
    uint32_t tokens = 0;
    for (uint32_t r = 0; r < P.local_batch; ++r) tokens += first_above(s_cnt, P.max_len, r * P.n_gpus + c);
    lo = min(lo, tokens), hi = max(hi, tokens);
  }
  finish_trial(lo, hi, s_lo, s_hi, trial_min, trial_max, sums);
}

}  // namespace
}  // namespace lbs

using namespace lbs;

extern "C" {

const char* lbs_last_error(void) { return g_error.c_str(); }

int lbs_dataset_create(lbs_dataset** out, int device, uint32_t max_len, const uint32_t* cum, uint32_t n_strata,
                       const uint32_t* stratum_end) {
  if (!out) return fail(LBS_ERR_NULL, "out is NULL");
  *out = nullptr;
  if (!cum || !stratum_end) return fail(LBS_ERR_NULL, "cum or stratum_end is NULL");
  if (max_len == 0 || n_strata == 0) return fail(LBS_ERR_ARG, "max_len and n_strata must be positive");
  if (max_len > LBS_MAX_LEN) return fail(LBS_ERR_LIMIT, "max_len exceeds LBS_MAX_LEN");
  if (n_strata > LBS_MAX_STRATA) return fail(LBS_ERR_LIMIT, "n_strata exceeds LBS_MAX_STRATA");
  if (device < -1) return fail(LBS_ERR_ARG, "device must be >= 0, or -1 for a host-only dataset");
  if (cum[0] != 0) return fail(LBS_ERR_ARG, "cum[0] must be 0");
  for (uint32_t l = 1; l <= max_len; ++l)
    if (cum[l] < cum[l - 1]) return fail(LBS_ERR_ARG, "cum must be non-decreasing");
  if (cum[max_len] == 0) return fail(LBS_ERR_ARG, "the dataset is empty");
  for (uint32_t s = 0; s < n_strata; ++s) {
    if (stratum_end[s] == 0 || stratum_end[s] > max_len || (s > 0 && stratum_end[s] <= stratum_end[s - 1]))
      return fail(LBS_ERR_ARG, "stratum_end must be increasing and lie in [1, max_len]");
  }
  if (stratum_end[n_strata - 1] != max_len) return fail(LBS_ERR_ARG, "the last stratum must end at max_len");
  lbs_dataset* ds = new (std::nothrow) lbs_dataset;
  if (!ds) return fail(LBS_ERR_HIP, "out of host memory");
  ds->device = device, ds->max_len = max_len, ds->n_strata = n_strata;
  ds->cum.assign(cum, cum + max_len + 1);
  ds->stratum_end.assign(stratum_end, stratum_end + n_strata);
  if (device >= 0) {
    int prev = -1;
    (void)hipGetDevice(&prev);
    hipError_t e = hipSetDevice(device);
    if (e == hipSuccess) e = hipMalloc((void**)&ds->d_cum, (max_len + 1) * sizeof(uint32_t));
    if (e == hipSuccess) e = hipMemcpy(ds->d_cum, cum, (max_len + 1) * sizeof(uint32_t), hipMemcpyHostToDevice);
    if (prev >= 0 && prev != device) (void)hipSetDevice(prev);
    if (e != hipSuccess) {
      if (ds->d_cum) (void)hipFree(ds->d_cum);
      delete ds;
      return fail(LBS_ERR_HIP, std::string("uploading the histogram: ") + hipGetErrorString(e));
    }
  }
  *out = ds;
  return 0;
}

void lbs_dataset_destroy(lbs_dataset* ds) {
  if (!ds) return;
  if (ds->device >= 0 && ds->d_cum) {
    int prev = -1;
    (void)hipGetDevice(&prev);
    (void)hipSetDevice(ds->device);
    (void)hipDeviceSynchronize();
    (void)hipFree(ds->d_cum);
    if (prev >= 0 && prev != ds->device) (void)hipSetDevice(prev);
  }
  delete ds;
}

int lbs_simulate(const lbs_dataset* ds, const lbs_run* run, uint32_t* trial_min, uint32_t* trial_max, uint64_t* sums,
                 void* stream) {
  if (!ds || !run) return fail(LBS_ERR_NULL, "dataset or run is NULL");
  if (run->method > LBS_GLOBAL) return fail(LBS_ERR_ARG, "unknown method");
  if (run->local_batch == 0 || run->n_gpus == 0) return fail(LBS_ERR_ARG, "local_batch and n_gpus must be positive");
  if (run->local_batch > LBS_MAX_LOCAL_BATCH) return fail(LBS_ERR_LIMIT, "local_batch exceeds LBS_MAX_LOCAL_BATCH");
  if ((uint64_t)run->n_gpus * run->local_batch >= (1ull << 31)) return fail(LBS_ERR_LIMIT, "n_gpus * local_batch must stay below 2^31");
  if (run->n_trials >= (1ull << 31)) return fail(LBS_ERR_LIMIT, "n_trials must stay below 2^31");
  const bool stratified = run->method == LBS_STRATIFIED || run->method == LBS_LOCAL_RASTER || run->method == LBS_LOCAL_SNAKE;
  const bool local = run->method == LBS_LOCAL_RASTER || run->method == LBS_LOCAL_SNAKE;
  Params P{};
  P.max_len = ds->max_len, P.local_batch = run->local_batch, P.gpus_per_node = run->gpus_per_node;
  P.n_gpus = run->n_gpus, P.snake = run->method == LBS_LOCAL_SNAKE, P.stratified = stratified;
  P.total = ds->cum[ds->max_len], P.seed = run->seed, P.first_trial = run->first_trial;
  if (stratified) {
    uint32_t j = 0;
    for (uint32_t s = 0; s < ds->n_strata; ++s) {
      const uint32_t lo = ds->cum[s == 0 ? 0 : ds->stratum_end[s - 1]], size = ds->cum[ds->stratum_end[s]] - lo;
      if (run->quota[s] && size == 0) return fail(LBS_ERR_ARG, "a stratum with a quota has no entries");
      if ((uint64_t)j + run->quota[s] > run->local_batch) return fail(LBS_ERR_ARG, "the quotas exceed local_batch");
      for (uint32_t q = 0; q < run->quota[s]; ++q, ++j) P.slot_lo[j] = lo, P.slot_size[j] = size;
    }
    if (j != run->local_batch) return fail(LBS_ERR_ARG, "the quotas must add up to local_batch");
  }
  if (local) {
    if (run->gpus_per_node == 0 || run->n_gpus % run->gpus_per_node) return fail(LBS_ERR_ARG, "n_gpus must be a multiple of gpus_per_node");
    if ((uint64_t)run->gpus_per_node * run->local_batch > LBS_MAX_NODE_POOL) return fail(LBS_ERR_LIMIT, "gpus_per_node * local_batch exceeds LBS_MAX_NODE_POOL");
  }
  if (!sums) return fail(LBS_ERR_NULL, "sums is NULL");
  if (ds->device < 0) return fail(LBS_ERR_HOST, "host-only dataset (device -1) cannot run kernels");
  int prev = -1;
  (void)hipGetDevice(&prev);
  if (prev != ds->device && hipSetDevice(ds->device) != hipSuccess) return fail(LBS_ERR_HIP, "hipSetDevice failed");
  hipStream_t s = (hipStream_t)stream;
  unsigned long long* ds_sums = reinterpret_cast<unsigned long long*>(sums);
  hipLaunchKernelGGL(k_lbs_clear, dim3(1), dim3(64), 0, s, ds_sums);
  hipError_t e = hipGetLastError();
  if (e == hipSuccess && run->n_trials > 0) {
    const dim3 grid((uint32_t)run->n_trials), block(kBlock);
    if (local) hipLaunchKernelGGL(k_lbs_local, grid, block, 0, s, P, ds->d_cum, trial_min, trial_max, ds_sums);
    else if (run->method == LBS_GLOBAL) hipLaunchKernelGGL(k_lbs_global, grid, block, 0, s, P, ds->d_cum, trial_min, trial_max, ds_sums);
    else hipLaunchKernelGGL(k_lbs_keep, grid, block, 0, s, P, ds->d_cum, trial_min, trial_max, ds_sums);
    e = hipGetLastError();
  }
  if (prev >= 0 && prev != ds->device) (void)hipSetDevice(prev);
  if (e != hipSuccess) return fail(LBS_ERR_HIP, std::string("launching the simulation: ") + hipGetErrorString(e));
  return 0;
}

}  // extern "C"

// Load-balancing simulation for gfx950 (MI355X): host entry points and kernels.
// See lbs.h for what is simulated and for the contract of every call.
//
// A workgroup (256 threads, four wavefronts) runs one trial at a time and a share of
// the call's trials in turn.  Nothing here is a contraction or a stream over HBM: the
// work is integer ALU, cross-lane traffic and LDS, the outputs are two words per trial.
//
// A draw is one SplitMix64 output (a handful of 64-bit integer operations) and the
// inverse of the cumulative histogram at the index it selects.  The histogram sits in
// LDS, and so does a guide table made when the dataset is created: for every range
// the draws can come from (the whole dataset, each stratum) and every value of the
// draw's upper 11 (whole dataset) or 9 (stratum) bits, the smallest and the largest
// length that such a draw can select.  The search for the length then runs over that interval only (mostly one
// or two candidates instead of ten halvings of [1, max_len]).
//   NONE / STRATIFIED : a thread owns whole GPUs; local_batch draws, one sum each.
//   LOCAL_*           : a wavefront owns a node.  Its lanes draw the node's pool into
//                       registers (entry i of the pool in register i / 64 of lane
//                       i % 64, padded to a multiple of 64 with a sentinel above every
//                       length) and sort it there with a bitonic network: a
//                       compare-exchange at distance < 64 is a cross-lane exchange, one
//                       at distance >= 64 pairs two registers of the same lane.  For a
//                       node of 1, 2, 4, ... 32 GPUs each GPU's column of the sorted pool
//                       is then summed across lanes; else the pool goes to LDS once, where
//                       each GPU's column is added up in raster or snake order.
//   GLOBAL            : lengths are small integers, so the trial's pool of
//                       n_gpus * local_batch draws is sorted by counting: an LDS
//                       histogram and a block-wide running sum give every length its
//                       range of sorted positions, which it spreads over the GPUs
//                       (position q goes to GPU q % n_gpus) through a difference array.
// Per-trial minimum and maximum are combined with shuffles and LDS; the two sums
// over trials are kept per workgroup and added up with 64-bit integer atomics at its
// end (integer addition is associative, so the result does not depend on the order).

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <cstdio>
#include <new>
#include <string>
#include <vector>

#include "lbs.h"

namespace lbs {
// guide tables: indexed by a draw's upper 11 bits for the whole dataset, by its upper 9 bits for a stratum
constexpr uint32_t kWholeGuideBits = 11, kWholeGuideSize = 1u << kWholeGuideBits;
constexpr uint32_t kGuideBits = 9, kGuideSize = 1u << kGuideBits;
}

struct lbs_dataset {
  int device = -1;
  uint32_t max_len = 0, n_strata = 0;
  std::vector<uint32_t> cum, stratum_end;
  uint32_t* d_cum = nullptr;
  uint32_t n_cus = 1;           // compute units of the device
  uint32_t* d_guide = nullptr;  // the whole dataset's table (kWholeGuideSize entries), then one of kGuideSize per stratum
};

namespace lbs {
namespace {

constexpr uint32_t kBlock = 256, kWaves = 4;
constexpr uint32_t kMaxSpreadGpus = 8192;  // k_lbs_global keeps one LDS word per GPU up to here
// workgroups launched per compute unit (at most 8 are resident at a time): many short rounds, handed out as slots
// free up, balance better than few long ones (measured: 16 -> 6.4 ms, 32 -> 5.9, 64 -> 5.8, 128 -> 5.7 for the five
// methods at once; beyond that a workgroup runs too few trials to pay for loading the tables)
constexpr uint32_t kGridPerCu = 128;
// ... and with few simulated GPUs a trial is so short that the tables' load has to be spread over more of them:
// a workgroup runs about three trials at 1 024 GPUs and proportionally more below (12 at 256 GPUs and fewer),
// but the grid never falls below four rounds of resident workgroups (32 per compute unit), so that the last
// round is a small part of the whole.
inline uint32_t trial_grid(uint64_t n_trials, uint32_t n_gpus, int n_cus) {
  const uint64_t most = (uint64_t)n_cus * kGridPerCu, least = (uint64_t)n_cus * 32u;
  const uint64_t scaled = n_trials * n_gpus / (3u * 1024u);
  const uint64_t want = std::min(most, std::max(least, scaled));
  return (uint32_t)std::max<uint64_t>(1, std::min<uint64_t>(n_trials, want));
}

thread_local std::string g_error;
int fail(int code, const std::string& msg) {
  g_error = msg;
  return code;
}

struct Params {  // by-value kernel argument
  uint32_t max_len, local_batch, gpus_per_node, n_gpus, snake, stratified;
  uint32_t total;                             // dataset size
  uint32_t guide_words;                       // guide entries the kernel loads (the whole dataset's table, or all strata's)
  uint32_t guide_shift;                       // a draw's upper 32 - guide_shift bits index its table
  uint32_t slot_lo[LBS_MAX_LOCAL_BATCH];      // a GPU's j-th draw: dataset entries before its range (0 / its stratum),
  uint32_t slot_size[LBS_MAX_LOCAL_BATCH];    //   entries in that range,
  uint32_t slot_guide[LBS_MAX_LOCAL_BATCH];   //   and where that range's guide table starts in LDS
  uint64_t seed, first_trial;
  uint32_t n_trials;
};

// SplitMix64: output number k + 1 of the generator seeded with `seed` is mix(state(seed, k)); the state
// advances by kGamma per draw, so consecutive draws cost one 64-bit addition, not a multiplication.
constexpr uint64_t kGamma = 0x9E3779B97F4A7C15ull;
__device__ __forceinline__ uint64_t state(uint64_t seed, uint64_t k) { return seed + (k + 1) * kGamma; }
__device__ __forceinline__ uint64_t mix(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// Smallest l in [lo, hi] with counts[l] > index (counts is non-decreasing and counts[hi] > index).
__device__ __forceinline__ uint32_t first_above(const uint32_t* counts, uint32_t lo, uint32_t hi, uint32_t index) {
  while (lo < hi) {
    const uint32_t mid = (lo + hi) >> 1;
    if (counts[mid] > index) hi = mid;
    else lo = mid + 1;
  }
  return lo;
}

// Length selected by the draw with generator state z out of the `size` dataset entries that follow the
// first `before` ones; `guide` is that range's table.
__device__ __forceinline__ uint32_t draw(const uint32_t* s_cum, const uint32_t* guide, uint32_t guide_shift, uint64_t z,
                                         uint32_t before, uint32_t size) {
  const uint32_t u = (uint32_t)(mix(z) >> 32);
  const uint32_t index = before + __umulhi(u, size);
  const uint32_t span = guide[u >> guide_shift];  // lengths a draw with these upper bits can select
  return first_above(s_cum, span & 0xffffu, span >> 16, index);
}

// Histogram and guide tables into LDS; returns where the guide tables start.
__device__ __forceinline__ uint32_t* load_tables(uint32_t* s_dyn, const Params& P, const uint32_t* __restrict__ cum,
                                                 const uint32_t* __restrict__ guide) {
  uint32_t* s_guide = s_dyn + P.max_len + 1u;
  for (uint32_t i = threadIdx.x; i <= P.max_len; i += kBlock) s_dyn[i] = cum[i];
  const uint32_t* src = guide + (P.stratified ? kWholeGuideSize : 0u);  // the whole dataset's table comes first
  for (uint32_t i = threadIdx.x; i < P.guide_words; i += kBlock) s_guide[i] = src[i];
  __syncthreads();
  return s_guide;
}

// The value that lane ^ 2^LJ holds.  Within a row of 16 lanes the exchange is a data-parallel move of the
// vector unit (quad permutation, shifts by 4 written to alternate banks of four lanes, rotation by 8);
// across rows it goes through the LDS crossbar.
template <int LJ>
__device__ __forceinline__ uint32_t from_partner(uint32_t x) {
  const int v = (int)x;
  if (LJ == 0) return (uint32_t)__builtin_amdgcn_mov_dpp(v, 0xB1, 0xf, 0xf, true);  // quad_perm [1,0,3,2]
  if (LJ == 1) return (uint32_t)__builtin_amdgcn_mov_dpp(v, 0x4E, 0xf, 0xf, true);  // quad_perm [2,3,0,1]
  if (LJ == 2) {
    const int t = __builtin_amdgcn_mov_dpp(v, 0x104, 0xf, 0x5, true);            // lanes 0-3, 8-11 of a row read lane + 4
    return (uint32_t)__builtin_amdgcn_update_dpp(t, v, 0x114, 0xf, 0xA, false);  // lanes 4-7, 12-15 read lane - 4
  }
  if (LJ == 3) return (uint32_t)__builtin_amdgcn_mov_dpp(v, 0x128, 0xf, 0xf, true);  // row_ror:8
  return (uint32_t)__shfl_xor(v, 1 << LJ, 64);
}

__device__ __forceinline__ uint32_t partner_of(uint32_t x, int lj) {  // lj is a constant after unrolling
  switch (lj) {
    case 0: return from_partner<0>(x);
    case 1: return from_partner<1>(x);
    case 2: return from_partner<2>(x);
    case 3: return from_partner<3>(x);
    case 4: return from_partner<4>(x);
    default: return from_partner<5>(x);
  }
}

// Sum of x over the lanes that differ from this one only in lane bits lo_bit .. hi_bit - 1 (the same two numbers
// for the whole workgroup): a butterfly, highest bit first, whose steps inside a row of 16 lanes are DPP moves.
// Written as a switch that is entered at the first step and left after the last, so that only the steps
// asked for are executed.
__device__ __forceinline__ uint32_t butterfly_sum(uint32_t x, uint32_t lo_bit, uint32_t hi_bit) {
  if (hi_bit <= lo_bit) return x;
  switch (hi_bit) {
    default: x += from_partner<5>(x); if (lo_bit == 5u) break; [[fallthrough]];
    case 5: x += from_partner<4>(x); if (lo_bit == 4u) break; [[fallthrough]];
    case 4: x += from_partner<3>(x); if (lo_bit == 3u) break; [[fallthrough]];
    case 3: x += from_partner<2>(x); if (lo_bit == 2u) break; [[fallthrough]];
    case 2: x += from_partner<1>(x); if (lo_bit == 1u) break; [[fallthrough]];
    case 1: x += from_partner<0>(x);
  }
  return x;
}

// The value of the lane whose position inside its group of n lanes (n a power of two up to 32) is mirrored.
__device__ __forceinline__ uint32_t from_mirror(uint32_t x, uint32_t n) {
  const int v = (int)x;
  switch (n) {
    case 1: return x;
    case 2: return (uint32_t)__builtin_amdgcn_mov_dpp(v, 0xB1, 0xf, 0xf, true);   // quad_perm [1,0,3,2]
    case 4: return (uint32_t)__builtin_amdgcn_mov_dpp(v, 0x1B, 0xf, 0xf, true);   // quad_perm [3,2,1,0]
    case 8: return (uint32_t)__builtin_amdgcn_mov_dpp(v, 0x141, 0xf, 0xf, true);  // row_half_mirror
    case 16: return (uint32_t)__builtin_amdgcn_mov_dpp(v, 0x140, 0xf, 0xf, true); // row_mirror
    default: return (uint32_t)__shfl_xor(v, (int)(n - 1u), 64);
  }
}

// Minimum and maximum over the wavefront, in every lane.
__device__ __forceinline__ void wave_min_max(uint32_t& lo, uint32_t& hi) {
#pragma unroll
  for (int lj = 0; lj < 6; ++lj) {
    lo = min(lo, partner_of(lo, lj));
    hi = max(hi, partner_of(hi, lj));
  }
}

// A workgroup loads the tables once and then runs trials blockIdx.x, blockIdx.x + gridDim.x, ... of the
// call, so the grid need only fill the chip, and thread 0 carries the workgroup's share of the two sums.

// Wavefront minima and maxima of a trial, double-buffered by the parity of the workgroup's trial count: a
// wavefront can be one trial ahead of thread 0, never two (the barrier in between needs all of them).
struct Finish {
  uint32_t lo[2][kWaves], hi[2][kWaves];
};

// Combines the threads' minimum and maximum of trial t (the round-th this workgroup runs); thread 0 stores
// them and adds them to its running sums.
__device__ __forceinline__ void finish_trial(uint32_t lo, uint32_t hi, Finish& f, uint32_t round, uint32_t t,
                                             uint32_t* trial_min, uint32_t* trial_max, unsigned long long& sum_lo,
                                             unsigned long long& sum_hi) {
  wave_min_max(lo, hi);
  const uint32_t buf = round & 1u;
  if ((threadIdx.x & 63u) == 0) f.lo[buf][threadIdx.x >> 6] = lo, f.hi[buf][threadIdx.x >> 6] = hi;
  __syncthreads();
  if (threadIdx.x == 0) {
    lo = min(min(f.lo[buf][0], f.lo[buf][1]), min(f.lo[buf][2], f.lo[buf][3]));
    hi = max(max(f.hi[buf][0], f.hi[buf][1]), max(f.hi[buf][2], f.hi[buf][3]));
    if (trial_min) trial_min[t] = lo;
    if (trial_max) trial_max[t] = hi;
    sum_lo += lo, sum_hi += hi;
  }
}

// Thread 0 adds the workgroup's sums to the call's.
__device__ __forceinline__ void publish_sums(unsigned long long* sums, unsigned long long sum_lo,
                                             unsigned long long sum_hi) {
  if (threadIdx.x == 0) {
    atomicAdd(&sums[0], sum_lo);
    atomicAdd(&sums[1], sum_hi);
  }
}

__global__ __launch_bounds__(64) void k_lbs_clear(unsigned long long* sums) {
  if (threadIdx.x < 2) sums[threadIdx.x] = 0ull;
}

// NONE and STRATIFIED: no redistribution.
__global__ __launch_bounds__(kBlock) void k_lbs_keep(const Params P, const uint32_t* __restrict__ cum,
                                                      const uint32_t* __restrict__ guide, uint32_t* trial_min,
                                                      uint32_t* trial_max, unsigned long long* sums) {
  extern __shared__ uint32_t s_dyn[];  // histogram, guide tables
  __shared__ Finish s_finish;
  const uint32_t* s_guide = load_tables(s_dyn, P, cum, guide);
  unsigned long long sum_lo = 0, sum_hi = 0;
  for (uint32_t t = blockIdx.x, round = 0; t < P.n_trials; t += gridDim.x, ++round) {
    const uint64_t k_trial = (P.first_trial + t) * P.n_gpus * (uint64_t)P.local_batch;  // the trial's first draw
    uint32_t lo = 0xffffffffu, hi = 0u;
    for (uint32_t g = threadIdx.x; g < P.n_gpus; g += kBlock) {
      uint64_t z = state(P.seed, k_trial + (uint64_t)g * P.local_batch);
      uint32_t tokens = 0;
      for (uint32_t j = 0; j < P.local_batch; ++j, z += kGamma)
        tokens += draw(s_dyn, s_guide + P.slot_guide[j], P.guide_shift, z, P.slot_lo[j], P.slot_size[j]);
      lo = min(lo, tokens), hi = max(hi, tokens);
    }
    finish_trial(lo, hi, s_finish, round, t, trial_min, trial_max, sum_lo, sum_hi);
  }
  publish_sums(sums, sum_lo, sum_hi);
}

// Median of three: with c = 0 it is min(a, b), with c = 0xffffffff it is max(a, b) (one v_med3_u32).
__device__ __forceinline__ uint32_t median3(uint32_t a, uint32_t b, uint32_t c) {
  return max(min(a, b), min(max(a, b), c));
}

// Sorts the 64 * E values held by a wavefront (value i in v[i / 64] of lane i % 64) into ascending order of i.
// bit[b] is all ones in lanes whose bit b is set and 0 elsewhere (b < 6).
template <int E>
__device__ __forceinline__ void bitonic_sort(uint32_t (&v)[E], const uint32_t (&bit)[6]) {
  constexpr int kLog = 6 + (E == 1 ? 0 : E == 2 ? 1 : E == 4 ? 2 : E == 8 ? 3 : 4);
#pragma unroll
  for (int lk = 1; lk <= kLog; ++lk) {       // merge sorted runs of 2^(lk-1) into runs of k = 2^lk, directions alternating
#pragma unroll
    for (int lj = lk - 1; lj >= 0; --lj) {   // compare-exchange at distance j = 2^lj
      if (lj >= 6) {                         // both entries in this lane
        const int je = 1 << (lj - 6);
#pragma unroll
        for (int e = 0; e < E; ++e) {
          if (e & je) continue;
          const bool ascending = ((e >> (lk - 6)) & 1) == 0;  // lk >= 7: the run's direction depends on e alone
          const uint32_t a = v[e], b = v[e | je];
          v[e] = ascending ? min(a, b) : max(a, b);
          v[e | je] = ascending ? max(a, b) : min(a, b);
        }
      } else {                               // the other entry is in lane ^ j
        // The lane with the pair's smaller index keeps the minimum in an ascending run and the maximum in a
        // descending one; the other lane the opposite: `keep` is 0 where the minimum stays, all ones elsewhere.
#pragma unroll
        for (int e = 0; e < E; ++e) {
          const uint32_t descending = lk < 6 ? bit[lk < 6 ? lk : 0] : (((e >> (lk - 6)) & 1) ? 0xffffffffu : 0u);
          const uint32_t keep = bit[lj] ^ descending;
          v[e] = median3(v[e], partner_of(v[e], lj), keep);
        }
      }
    }
  }
}

// LOCAL_RASTER and LOCAL_SNAKE: pool, sort and deal within every node.  E = registers per lane: 64 * E >= the pool.
// IN_LANES: gpus_per_node is a power of two up to 32.  Then sorted entry i = e * 64 + lane lies in column
// lane % gpus_per_node of row e * (64 / gpus_per_node) + lane / gpus_per_node, whose parity is that of
// lane / gpus_per_node for every e, and the deal is a sum within the lane, a mirror exchange inside odd rows
// (snake) and a butterfly over the lane bits above the column: no LDS and no barrier.  Otherwise the sorted
// pool goes to LDS and one lane per GPU walks its column.
template <int E, bool IN_LANES>
__global__ __launch_bounds__(kBlock) void k_lbs_local(const Params P, const uint32_t* __restrict__ cum,
                                                       const uint32_t* __restrict__ guide, uint32_t* trial_min,
                                                       uint32_t* trial_max, unsigned long long* sums) {
  extern __shared__ uint32_t s_dyn[];  // histogram, guide tables, (not IN_LANES) one sorted pool per wavefront
  __shared__ Finish s_finish;
  const uint32_t* s_guide = load_tables(s_dyn, P, cum, guide);
  const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
  const uint32_t n_nodes = P.n_gpus / P.gpus_per_node;
  const uint32_t pool = P.gpus_per_node * P.local_batch;
  uint32_t* sorted = s_dyn + P.max_len + 1u + P.guide_words + wave * pool;
  // pool entry i = e * 64 + lane is draw i % local_batch of GPU i / local_batch of the node, for every node alike
  uint32_t before[E], size[E], goff[E];
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const uint32_t i = (uint32_t)e * 64u + lane, j = i % P.local_batch;
    const bool real = i < pool;
    before[e] = real ? P.slot_lo[j] : 0u, size[e] = real ? P.slot_size[j] : 0u, goff[e] = real ? P.slot_guide[j] : 0u;
  }
  uint32_t bit[6];
#pragma unroll
  for (int b = 0; b < 6; ++b) bit[b] = 0u - ((lane >> b) & 1u);
  const bool odd_row = ((lane / P.gpus_per_node) & 1u) != 0u;  // IN_LANES only
  const uint32_t gpn_bit = (uint32_t)__ffs((int)P.gpus_per_node) - 1u;  // IN_LANES: gpus_per_node = 2^gpn_bit
  unsigned long long sum_lo = 0, sum_hi = 0;
  for (uint32_t t = blockIdx.x, round = 0; t < P.n_trials; t += gridDim.x, ++round) {
    const uint64_t k_trial = (P.first_trial + t) * P.n_gpus * (uint64_t)P.local_batch;
    uint32_t lo = 0xffffffffu, hi = 0u;
    // Every wavefront makes the same number of rounds, so the barriers below (not IN_LANES) are met by all; a
    // wavefront without a node in the last round only keeps them company.
    for (uint32_t base = 0; base < n_nodes; base += kWaves) {
      const uint32_t node = base + wave;
      const bool active = node < n_nodes;
      if (active) {
        const uint64_t z_node = state(P.seed, k_trial + (uint64_t)node * pool);  // a node's draws are consecutive
        uint32_t v[E];
#pragma unroll
        for (int e = 0; e < E; ++e) {
          const uint32_t i = (uint32_t)e * 64u + lane;
          v[e] = i < pool ? draw(s_dyn, s_guide + goff[e], P.guide_shift, z_node + i * kGamma, before[e], size[e]) : 0xffffffffu;
        }
        bitonic_sort<E>(v, bit);
        if (IN_LANES) {
          uint32_t tokens = 0;
#pragma unroll
          for (int e = 0; e < E; ++e) tokens += (uint32_t)e * 64u + lane < pool ? v[e] : 0u;  // the padding sorts to the end
          if (P.snake) {  // an odd row is dealt right to left: its column c goes to GPU gpus_per_node - 1 - c
            const uint32_t mirrored = from_mirror(tokens, P.gpus_per_node);
            tokens = odd_row ? mirrored : tokens;
          }
          tokens = butterfly_sum(tokens, gpn_bit, 6u);
          lo = min(lo, tokens), hi = max(hi, tokens);  // every lane now holds the total of GPU lane % gpus_per_node
        } else {
#pragma unroll
          for (int e = 0; e < E; ++e) {
            const uint32_t i = (uint32_t)e * 64u + lane;
            if (i < pool) sorted[i] = v[e];
          }
        }
      }
      if (!IN_LANES) {
        __syncthreads();
        if (active)
          for (uint32_t c = lane; c < P.gpus_per_node; c += 64u) {
            uint32_t tokens = 0;
            for (uint32_t r = 0; r < P.local_batch; ++r) {
              const uint32_t col = (P.snake && (r & 1u)) ? P.gpus_per_node - 1u - c : c;  // position in the row dealt to GPU c
              tokens += sorted[r * P.gpus_per_node + col];
            }
            lo = min(lo, tokens), hi = max(hi, tokens);
          }
        __syncthreads();
      }
    }
    finish_trial(lo, hi, s_finish, round, t, trial_min, trial_max, sum_lo, sum_hi);
  }
  publish_sums(sums, sum_lo, sum_hi);
}

// Inclusive running sum over the workgroup of one value per thread; all threads call it.  Within a wavefront
// by shuffles, across the four wavefronts through s_scan (kWaves words): one barrier.  The caller leaves s_scan
// alone until the workgroup has passed another barrier (each use in a trial has words of its own).
__device__ __forceinline__ uint32_t block_running_sum(uint32_t* s_scan, uint32_t value) {
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  uint32_t x = value;
#pragma unroll
  for (uint32_t off = 1; off < 64u; off <<= 1) {
    const uint32_t below = (uint32_t)__shfl_up((int)x, off, 64);
    if (lane >= off) x += below;
  }
  if (lane == 63u) s_scan[wave] = x;
  __syncthreads();
  uint32_t before = 0;
  for (uint32_t w = 0; w < wave; ++w) before += s_scan[w];
  return x + before;
}

// GLOBAL: pool, sort and deal over all GPUs.  The pool is sorted by counting (lengths are small integers):
// after the running sum, the entries of length l hold sorted positions cnt[l-1] .. cnt[l] - 1, and position q
// goes to GPU q % n_gpus.
// SPREAD (n_gpus <= kMaxSpreadGpus): every length adds itself to the GPUs its positions fall on, as a
// difference array over the GPUs: whole turns round all GPUs go to a common base, the rest is a circular
// range [first, first + rest) marked at its two ends; a running sum over the GPUs then gives every GPU's tokens.
// Otherwise every GPU looks up the length at each of its local_batch positions by binary search.
template <bool SPREAD>
__global__ __launch_bounds__(kBlock) void k_lbs_global(const Params P, const uint32_t* __restrict__ cum,
                                                        const uint32_t* __restrict__ guide, uint32_t* trial_min,
                                                        uint32_t* trial_max, unsigned long long* sums) {
  extern __shared__ uint32_t s_dyn[];  // histogram, guide table, the trial's own histogram, (SPREAD) one word per GPU
  __shared__ uint32_t s_scan[2][kWaves];
  __shared__ uint32_t s_base;
  __shared__ Finish s_finish;
  const uint32_t* s_guide = load_tables(s_dyn, P, cum, guide);
  uint32_t* s_cnt = s_dyn + P.max_len + 1u + P.guide_words;  // first counts of the trial's draws, then their running sum
  uint32_t* s_gpu = s_cnt + P.max_len + 1u;                           // SPREAD: difference array over the GPUs
  const uint32_t tid = threadIdx.x;
  const uint32_t pool = P.n_gpus * P.local_batch;
  const uint32_t per = (P.max_len + 1u + kBlock - 1u) / kBlock;  // lengths per thread in the running sum
  const uint32_t a = tid * per, b = min(a + per, P.max_len + 1u);
  const uint32_t per_gpu = (P.n_gpus + kBlock - 1u) / kBlock;    // SPREAD: GPUs per thread in theirs
  const uint32_t ga = min(tid * per_gpu, P.n_gpus), gb = min(ga + per_gpu, P.n_gpus);
  unsigned long long sum_lo = 0, sum_hi = 0;
  for (uint32_t t = blockIdx.x, round = 0; t < P.n_trials; t += gridDim.x, ++round) {
    // the previous trial's last reads of s_cnt and s_gpu lie before the barrier in its finish_trial
    for (uint32_t i = tid; i <= P.max_len; i += kBlock) s_cnt[i] = 0u;
    if (SPREAD) {
      for (uint32_t i = tid; i < P.n_gpus; i += kBlock) s_gpu[i] = 0u;
      if (tid == 0) s_base = 0u;
    }
    __syncthreads();
    uint64_t z = state(P.seed, (P.first_trial + t) * (uint64_t)pool + tid);
    for (uint32_t i = tid; i < pool; i += kBlock, z += kBlock * kGamma)
      atomicAdd(&s_cnt[draw(s_dyn, s_guide, P.guide_shift, z, 0u, P.total)], 1u);
    __syncthreads();
    // running sum over lengths: a thread owns a contiguous piece, the pieces' sums are combined across threads
    uint32_t piece = 0;
    for (uint32_t i = a; i < b; ++i) piece += s_cnt[i];
    uint32_t run = block_running_sum(s_scan[0], piece) - piece;  // draws with a length below this thread's piece
    uint32_t lo = 0xffffffffu, hi = 0u;
    if (SPREAD) {
      uint32_t whole_turns = 0;
      for (uint32_t l = a; l < b; ++l) {  // entries of length l: positions run .. run + n - 1
        const uint32_t n = s_cnt[l];
        if (n != 0u) {
          const uint32_t turns = n / P.n_gpus, rest = n - turns * P.n_gpus, first = run % P.n_gpus;
          whole_turns += turns * l;
          if (rest != 0u) {  // unsigned wrap-around is harmless: the sums that are read come out below 2^32
            const uint32_t end = first + rest;
            atomicAdd(&s_gpu[first], l);
            if (end < P.n_gpus) atomicAdd(&s_gpu[end], 0u - l);
            if (end > P.n_gpus) atomicAdd(&s_gpu[0], l), atomicAdd(&s_gpu[end - P.n_gpus], 0u - l);
          }
        }
        run += n;
      }
      if (whole_turns != 0u) atomicAdd(&s_base, whole_turns);
      __syncthreads();
      uint32_t mine = 0;
      for (uint32_t g = ga; g < gb; ++g) mine += s_gpu[g];
      uint32_t tokens = block_running_sum(s_scan[1], mine) - mine + s_base;  // ... of the GPU before this thread's first
      for (uint32_t g = ga; g < gb; ++g) {
        tokens += s_gpu[g];
        lo = min(lo, tokens), hi = max(hi, tokens);
      }
    } else {
      for (uint32_t i = a; i < b; ++i) {
        run += s_cnt[i];
        s_cnt[i] = run;  // draws of length <= i
      }
      __syncthreads();
      for (uint32_t c = tid; c < P.n_gpus; c += kBlock) {
        uint32_t tokens = 0, l = 1;
        for (uint32_t r = 0; r < P.local_batch; ++r) {  // sorted positions r * n_gpus + c grow with r, and so do their lengths
          l = first_above(s_cnt, l, P.max_len, r * P.n_gpus + c);
          tokens += l;
        }
        lo = min(lo, tokens), hi = max(hi, tokens);
      }
    }
    finish_trial(lo, hi, s_finish, round, t, trial_min, trial_max, sum_lo, sum_hi);
  }
  publish_sums(sums, sum_lo, sum_hi);
}

// ---- all five methods on one set of draws ----------------------------------------
// NONE and GLOBAL use the same draws from the whole dataset, STRATIFIED and the two LOCAL methods the same
// stratified draws (draw number k of a run does not depend on the method), so one pass makes each set once:
// first a thread per GPU draws from the whole dataset, sums its GPU's tokens (NONE) and counts the lengths
// for the counting sort (GLOBAL, as in k_lbs_global<true>); then a wavefront per node draws the stratified
// pool into registers, adds up each GPU's own draws (STRATIFIED: local_batch consecutive pool entries, a
// butterfly over the low lane bits), sorts and deals twice (LOCAL_RASTER, LOCAL_SNAKE, as in
// k_lbs_local<E, true>).  Needs gpus_per_node and local_batch to be powers of two (<= 32 and <= 64).
constexpr uint32_t kMethods = 5;
struct FinishAll {
  uint32_t lo[2][kMethods][kWaves], hi[2][kMethods][kWaves];
};

template <int E>
__global__ __launch_bounds__(kBlock, E <= 2 ? 6 : E == 4 ? 4 : E == 8 ? 3 : 2) void k_lbs_all(const Params P, const uint32_t* __restrict__ cum,
                                                     const uint32_t* __restrict__ guide, uint32_t* trial_min,
                                                     uint32_t* trial_max, unsigned long long* sums) {
  extern __shared__ uint32_t s_dyn[];  // histogram, all guide tables, the trial's own histogram, one word per GPU
  __shared__ uint32_t s_scan[2][kWaves];
  __shared__ uint32_t s_base;
  __shared__ FinishAll s_fin;
  __shared__ unsigned long long s_sum[2u * kMethods];  // the workgroup's share of the sums: thread i keeps sum i
  const uint32_t tid = threadIdx.x, wave = tid >> 6, lane = tid & 63u;
  if (tid < 2u * kMethods) s_sum[tid] = 0ull;
  uint32_t* s_whole = s_dyn + P.max_len + 1u;          // guide table of the whole dataset
  uint32_t* s_strata = s_whole + kWholeGuideSize;      // guide tables of the strata
  uint32_t* s_cnt = s_whole + P.guide_words;
  uint32_t* s_gpu = s_cnt + P.max_len + 1u;
  for (uint32_t i = tid; i <= P.max_len; i += kBlock) s_dyn[i] = cum[i];
  for (uint32_t i = tid; i < P.guide_words; i += kBlock) s_whole[i] = guide[i];
  __syncthreads();

  const uint32_t pool_all = P.n_gpus * P.local_batch;
  const uint32_t per = (P.max_len + 1u + kBlock - 1u) / kBlock;
  const uint32_t a = tid * per, b = min(a + per, P.max_len + 1u);
  const uint32_t per_gpu = (P.n_gpus + kBlock - 1u) / kBlock;
  const uint32_t ga = min(tid * per_gpu, P.n_gpus), gb = min(ga + per_gpu, P.n_gpus);
  const uint32_t n_nodes = P.n_gpus / P.gpus_per_node;
  const uint32_t pool = P.gpus_per_node * P.local_batch;
  uint32_t before[E], size[E], goff[E];
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const uint32_t i = (uint32_t)e * 64u + lane, j = i % P.local_batch;
    const bool real = i < pool;
    before[e] = real ? P.slot_lo[j] : 0u, size[e] = real ? P.slot_size[j] : 0u, goff[e] = real ? P.slot_guide[j] : 0u;
  }
  uint32_t bit[6];
#pragma unroll
  for (int q = 0; q < 6; ++q) bit[q] = 0u - ((lane >> q) & 1u);
  const bool odd_row = ((lane / P.gpus_per_node) & 1u) != 0u;
  const uint32_t gpn_bit = (uint32_t)__ffs((int)P.gpus_per_node) - 1u, batch_bit = (uint32_t)__ffs((int)P.local_batch) - 1u;

  for (uint32_t t = blockIdx.x, round = 0; t < P.n_trials; t += gridDim.x, ++round) {
    const uint32_t buf = round & 1u;
    uint32_t lo[kMethods], hi[kMethods];
#pragma unroll
    for (uint32_t q = 0; q < kMethods; ++q) lo[q] = 0xffffffffu, hi[q] = 0u;
    const uint64_t k_trial = (P.first_trial + t) * (uint64_t)pool_all;  // the trial's first draw
    // ---- draws from the whole dataset: NONE, and the counts for GLOBAL
    for (uint32_t i = tid; i <= P.max_len; i += kBlock) s_cnt[i] = 0u;
    for (uint32_t i = tid; i < P.n_gpus; i += kBlock) s_gpu[i] = 0u;
    if (tid == 0) s_base = 0u;
    __syncthreads();
    for (uint32_t g = tid; g < P.n_gpus; g += kBlock) {
      uint64_t z = state(P.seed, k_trial + (uint64_t)g * P.local_batch);
      uint32_t tokens = 0;
      for (uint32_t j = 0; j < P.local_batch; ++j, z += kGamma) {
        const uint32_t l = draw(s_dyn, s_whole, 32u - kWholeGuideBits, z, 0u, P.total);
        tokens += l;
        atomicAdd(&s_cnt[l], 1u);
      }
      lo[LBS_NONE] = min(lo[LBS_NONE], tokens), hi[LBS_NONE] = max(hi[LBS_NONE], tokens);
    }
    __syncthreads();
    {
      uint32_t piece = 0;
      for (uint32_t i = a; i < b; ++i) piece += s_cnt[i];
      uint32_t run = block_running_sum(s_scan[0], piece) - piece;
      uint32_t whole_turns = 0;
      for (uint32_t l = a; l < b; ++l) {
        const uint32_t n = s_cnt[l];
        if (n != 0u) {
          const uint32_t turns = n / P.n_gpus, rest = n - turns * P.n_gpus, first = run % P.n_gpus;
          whole_turns += turns * l;
          if (rest != 0u) {
            const uint32_t end = first + rest;
            atomicAdd(&s_gpu[first], l);
            if (end < P.n_gpus) atomicAdd(&s_gpu[end], 0u - l);
            if (end > P.n_gpus) atomicAdd(&s_gpu[0], l), atomicAdd(&s_gpu[end - P.n_gpus], 0u - l);
          }
        }
        run += n;
      }
      if (whole_turns != 0u) atomicAdd(&s_base, whole_turns);
      __syncthreads();
      uint32_t mine = 0;
      for (uint32_t g = ga; g < gb; ++g) mine += s_gpu[g];
      uint32_t tokens = block_running_sum(s_scan[1], mine) - mine + s_base;
      for (uint32_t g = ga; g < gb; ++g) {
        tokens += s_gpu[g];
        lo[LBS_GLOBAL] = min(lo[LBS_GLOBAL], tokens), hi[LBS_GLOBAL] = max(hi[LBS_GLOBAL], tokens);
      }
    }
    // these two are filed now, so that they need no registers during the sort
    wave_min_max(lo[LBS_NONE], hi[LBS_NONE]);
    wave_min_max(lo[LBS_GLOBAL], hi[LBS_GLOBAL]);
    if (lane == 0) {
      s_fin.lo[buf][LBS_NONE][wave] = lo[LBS_NONE], s_fin.hi[buf][LBS_NONE][wave] = hi[LBS_NONE];
      s_fin.lo[buf][LBS_GLOBAL][wave] = lo[LBS_GLOBAL], s_fin.hi[buf][LBS_GLOBAL][wave] = hi[LBS_GLOBAL];
    }
    // ---- stratified draws, a wavefront per node: STRATIFIED, LOCAL_RASTER, LOCAL_SNAKE (no LDS writes, no barriers)
    for (uint32_t node = wave; node < n_nodes; node += kWaves) {
      const uint64_t z_node = state(P.seed, k_trial + (uint64_t)node * pool);
      uint32_t v[E];
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const uint32_t i = (uint32_t)e * 64u + lane;
        v[e] = i < pool ? draw(s_dyn, s_strata + goff[e], 32u - kGuideBits, z_node + i * kGamma, before[e], size[e]) : 0xffffffffu;
      }
#pragma unroll
      for (int e = 0; e < E; ++e) {  // a GPU's own draws are local_batch consecutive pool entries
        const bool real = (uint32_t)e * 64u + lane < pool;
        const uint32_t own = butterfly_sum(real ? v[e] : 0u, 0u, batch_bit);
        if (real) lo[LBS_STRATIFIED] = min(lo[LBS_STRATIFIED], own), hi[LBS_STRATIFIED] = max(hi[LBS_STRATIFIED], own);
      }
      bitonic_sort<E>(v, bit);
      uint32_t column = 0;
#pragma unroll
      for (int e = 0; e < E; ++e) column += (uint32_t)e * 64u + lane < pool ? v[e] : 0u;
      const uint32_t mirrored = from_mirror(column, P.gpus_per_node);
      const uint32_t raster = butterfly_sum(column, gpn_bit, 6u);
      const uint32_t snake = butterfly_sum(odd_row ? mirrored : column, gpn_bit, 6u);
      lo[LBS_LOCAL_RASTER] = min(lo[LBS_LOCAL_RASTER], raster), hi[LBS_LOCAL_RASTER] = max(hi[LBS_LOCAL_RASTER], raster);
      lo[LBS_LOCAL_SNAKE] = min(lo[LBS_LOCAL_SNAKE], snake), hi[LBS_LOCAL_SNAKE] = max(hi[LBS_LOCAL_SNAKE], snake);
    }
    // ---- the trial's five results
#pragma unroll
    for (uint32_t q = LBS_STRATIFIED; q <= LBS_LOCAL_SNAKE; ++q) {
      wave_min_max(lo[q], hi[q]);
      if (lane == 0) s_fin.lo[buf][q][wave] = lo[q], s_fin.hi[buf][q][wave] = hi[q];
    }
    __syncthreads();  // also: this trial's last reads of s_cnt and s_gpu lie before the next trial's clearing
    if (tid < 2u * kMethods) {  // thread 2 q: method q's minimum; thread 2 q + 1: its maximum
      const uint32_t q = tid >> 1;
      uint32_t r;
      if (tid & 1u) {
        r = max(max(s_fin.hi[buf][q][0], s_fin.hi[buf][q][1]), max(s_fin.hi[buf][q][2], s_fin.hi[buf][q][3]));
        if (trial_max) trial_max[(size_t)q * P.n_trials + t] = r;
      } else {
        r = min(min(s_fin.lo[buf][q][0], s_fin.lo[buf][q][1]), min(s_fin.lo[buf][q][2], s_fin.lo[buf][q][3]));
        if (trial_min) trial_min[(size_t)q * P.n_trials + t] = r;
      }
      s_sum[tid] += r;
    }
  }
  if (tid < 2u * kMethods) atomicAdd(&sums[tid], s_sum[tid]);
}

__global__ __launch_bounds__(64) void k_lbs_clear_all(unsigned long long* sums) {
  if (threadIdx.x < 2u * kMethods) sums[threadIdx.x] = 0ull;
}

// Host: length of dataset entry `index` (entries ordered by length).
uint32_t length_of(const std::vector<uint32_t>& cum, uint32_t index) {
  return (uint32_t)(std::upper_bound(cum.begin() + 1, cum.end(), index) - cum.begin());
}

// Guide table of the `size` entries after the first `before`: for every value of a draw's upper `bits`
// bits, the smallest (low half) and the largest (high half) length that such a draw selects.  The index a
// draw selects grows with the draw, and the length with the index, so the two ends bound everything between.
void fill_guide(uint32_t* out, uint32_t bits, const std::vector<uint32_t>& cum, uint32_t before, uint32_t size) {
  for (uint32_t ub = 0; ub < (1u << bits); ++ub) {
    const uint64_t u_min = (uint64_t)ub << (32u - bits), u_max = u_min + (1ull << (32u - bits)) - 1u;
    if (size == 0) {
      out[ub] = 1u | (1u << 16);  // never drawn from
      continue;
    }
    const uint32_t l_min = length_of(cum, before + (uint32_t)((u_min * size) >> 32));
    const uint32_t l_max = length_of(cum, before + (uint32_t)((u_max * size) >> 32));
    out[ub] = l_min | (l_max << 16);
  }
}

// Measurement only: how many lane-operations per second the vector units issue for the instruction kinds the
// simulation is made of.  Pure register arithmetic on eight independent chains per lane (enough to cover every
// instruction's latency), one store per thread at the end so that nothing is optimised away.
template <int KIND>
__global__ __launch_bounds__(256) void k_issue_probe(uint32_t* out, uint32_t iters, uint32_t seed) {
  uint32_t a[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = seed * (i + 1) + threadIdx.x;
  const uint32_t c = seed | 1u;
  for (uint32_t it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (KIND == LBS_PROBE_XOR_ADD) a[i] = (a[i] ^ c) + 0x9E3779B9u;
      if (KIND == LBS_PROBE_MUL_LO) a[i] = a[i] * 0x85EBCA6Bu + 1u;
      if (KIND == LBS_PROBE_MUL_HI_ADD) a[i] = __umulhi(a[i], c) + a[i];
      if (KIND == LBS_PROBE_MED3) a[i] = max(min(a[i], c), min(max(a[i], c), it));
      if (KIND == LBS_PROBE_DPP_ADD)
        a[i] = (uint32_t)__builtin_amdgcn_update_dpp((int)a[i], (int)a[i], 0xB1, 0xf, 0xf, false) + 1u;
      if (KIND == LBS_PROBE_BPERMUTE_ADD) a[i] = (uint32_t)__shfl_xor((int)a[i], 16, 64) + 1u;
      if (KIND == LBS_PROBE_FMA_F32) a[i] = __float_as_uint(__fmaf_rn(__uint_as_float(a[i]), 1.0001f, 0.5f));
    }
  }
  uint32_t r = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) r ^= a[i];
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = r;
}

}  // namespace
}  // namespace lbs

using namespace lbs;

extern "C" {

const char* lbs_last_error(void) { return g_error.c_str(); }

int lbs_issue_rate_probe(int kind, uint32_t n_workgroups, uint32_t iters, uint32_t* out, void* stream) {
  if (!out) return fail(LBS_ERR_NULL, "out is NULL");
  if (n_workgroups == 0 || n_workgroups > (1u << 20)) return fail(LBS_ERR_ARG, "n_workgroups must lie in [1, 2^20]");
  void (*kernel)(uint32_t*, uint32_t, uint32_t) = nullptr;
  switch (kind) {
    case LBS_PROBE_XOR_ADD: kernel = k_issue_probe<LBS_PROBE_XOR_ADD>; break;
    case LBS_PROBE_MUL_LO: kernel = k_issue_probe<LBS_PROBE_MUL_LO>; break;
    case LBS_PROBE_MUL_HI_ADD: kernel = k_issue_probe<LBS_PROBE_MUL_HI_ADD>; break;
    case LBS_PROBE_MED3: kernel = k_issue_probe<LBS_PROBE_MED3>; break;
    case LBS_PROBE_DPP_ADD: kernel = k_issue_probe<LBS_PROBE_DPP_ADD>; break;
    case LBS_PROBE_BPERMUTE_ADD: kernel = k_issue_probe<LBS_PROBE_BPERMUTE_ADD>; break;
    case LBS_PROBE_FMA_F32: kernel = k_issue_probe<LBS_PROBE_FMA_F32>; break;
    default: return fail(LBS_ERR_ARG, "unknown probe kind");
  }
  hipLaunchKernelGGL(kernel, dim3(n_workgroups), dim3(256), 0, (hipStream_t)stream, out, iters, 12345u);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(LBS_ERR_HIP, std::string("launching the probe: ") + hipGetErrorString(e));
  return 0;
}

static int dataset_create(lbs_dataset** out, int device, uint32_t max_len, const uint32_t* cum, uint32_t n_strata,
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
  lbs_dataset* ds = new lbs_dataset;
  *out = ds;  // from here on the caller's wrapper frees it on failure
  ds->max_len = max_len, ds->n_strata = n_strata;
  ds->cum.assign(cum, cum + max_len + 1);
  ds->stratum_end.assign(stratum_end, stratum_end + n_strata);
  if (device >= 0) {
    std::vector<uint32_t> guide(kWholeGuideSize + (size_t)n_strata * kGuideSize);
    fill_guide(guide.data(), kWholeGuideBits, ds->cum, 0, cum[max_len]);
    for (uint32_t s = 0; s < n_strata; ++s) {
      const uint32_t before = cum[s == 0 ? 0 : stratum_end[s - 1]];
      fill_guide(guide.data() + kWholeGuideSize + (size_t)s * kGuideSize, kGuideBits, ds->cum, before, cum[stratum_end[s]] - before);
    }
    int prev = -1;
    (void)hipGetDevice(&prev);
    hipError_t e = hipSetDevice(device);
    if (e == hipSuccess) ds->device = device;
    int n_cus = 0;
    if (e == hipSuccess) e = hipDeviceGetAttribute(&n_cus, hipDeviceAttributeMultiprocessorCount, device);
    if (e == hipSuccess) ds->n_cus = (uint32_t)std::max(n_cus, 1);
    if (e == hipSuccess) e = hipMalloc((void**)&ds->d_cum, (max_len + 1) * sizeof(uint32_t));
    if (e == hipSuccess) e = hipMemcpy(ds->d_cum, cum, (max_len + 1) * sizeof(uint32_t), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMalloc((void**)&ds->d_guide, guide.size() * sizeof(uint32_t));
    if (e == hipSuccess) e = hipMemcpy(ds->d_guide, guide.data(), guide.size() * sizeof(uint32_t), hipMemcpyHostToDevice);
    if (prev >= 0 && prev != device) (void)hipSetDevice(prev);
    if (e != hipSuccess) return fail(LBS_ERR_HIP, std::string("uploading the histogram: ") + hipGetErrorString(e));
  }
  return 0;
}

void lbs_dataset_destroy(lbs_dataset* ds) {
  if (!ds) return;
  if (ds->device >= 0 && (ds->d_cum || ds->d_guide)) {
    int prev = -1;
    (void)hipGetDevice(&prev);
    (void)hipSetDevice(ds->device);
    (void)hipDeviceSynchronize();
    if (ds->d_cum) (void)hipFree(ds->d_cum);
    if (ds->d_guide) (void)hipFree(ds->d_guide);
    if (prev >= 0 && prev != ds->device) (void)hipSetDevice(prev);
  }
  delete ds;
}

int lbs_dataset_create(lbs_dataset** out, int device, uint32_t max_len, const uint32_t* cum, uint32_t n_strata,
                       const uint32_t* stratum_end) {
  int rc;
  try {  // no C++ exception crosses the C boundary
    rc = dataset_create(out, device, max_len, cum, n_strata, stratum_end);
  } catch (...) {
    rc = LBS_ERR_HIP;
    g_error.clear();  // out of host memory: nothing is allocated to say so
  }
  if (rc != 0 && out && *out) {
    lbs_dataset_destroy(*out);
    *out = nullptr;
  }
  return rc;
}

// One method of a run (run->method is not looked at).
static int simulate_one(const lbs_dataset* ds, const lbs_run* run, uint32_t method, uint32_t* trial_min, uint32_t* trial_max,
                        uint64_t* sums, void* stream) {
  if (!ds || !run) return fail(LBS_ERR_NULL, "dataset or run is NULL");
  if (method > LBS_GLOBAL) return fail(LBS_ERR_ARG, "unknown method");
  if (run->local_batch == 0 || run->n_gpus == 0) return fail(LBS_ERR_ARG, "local_batch and n_gpus must be positive");
  if (run->local_batch > LBS_MAX_LOCAL_BATCH) return fail(LBS_ERR_LIMIT, "local_batch exceeds LBS_MAX_LOCAL_BATCH");
  if ((uint64_t)run->n_gpus * run->local_batch >= (1ull << 31)) return fail(LBS_ERR_LIMIT, "n_gpus * local_batch must stay below 2^31");
  if (run->n_trials >= (1ull << 31)) return fail(LBS_ERR_LIMIT, "n_trials must stay below 2^31");
  const bool stratified = method == LBS_STRATIFIED || method == LBS_LOCAL_RASTER || method == LBS_LOCAL_SNAKE;
  const bool local = method == LBS_LOCAL_RASTER || method == LBS_LOCAL_SNAKE;
  Params P{};
  P.max_len = ds->max_len, P.local_batch = run->local_batch, P.gpus_per_node = run->gpus_per_node;
  P.n_gpus = run->n_gpus, P.snake = method == LBS_LOCAL_SNAKE, P.stratified = stratified;
  P.total = ds->cum[ds->max_len], P.seed = run->seed;
  P.guide_words = stratified ? ds->n_strata * kGuideSize : kWholeGuideSize;
  P.guide_shift = 32u - (stratified ? kGuideBits : kWholeGuideBits);
  if (stratified) {
    uint32_t j = 0;
    for (uint32_t s = 0; s < ds->n_strata; ++s) {
      const uint32_t lo = ds->cum[s == 0 ? 0 : ds->stratum_end[s - 1]], size = ds->cum[ds->stratum_end[s]] - lo;
      if (run->quota[s] && size == 0) return fail(LBS_ERR_ARG, "a stratum with a quota has no entries");
      if ((uint64_t)j + run->quota[s] > run->local_batch) return fail(LBS_ERR_ARG, "the quotas exceed local_batch");
      for (uint32_t q = 0; q < run->quota[s]; ++q, ++j) P.slot_lo[j] = lo, P.slot_size[j] = size, P.slot_guide[j] = s * kGuideSize;
    }
    if (j != run->local_batch) return fail(LBS_ERR_ARG, "the quotas must add up to local_batch");
  } else {
    for (uint32_t j = 0; j < run->local_batch; ++j) P.slot_lo[j] = 0, P.slot_size[j] = P.total, P.slot_guide[j] = 0;
  }
  uint32_t pool = 0;
  if (local) {
    if (run->gpus_per_node == 0 || run->n_gpus % run->gpus_per_node) return fail(LBS_ERR_ARG, "n_gpus must be a multiple of gpus_per_node");
    if ((uint64_t)run->gpus_per_node * run->local_batch > LBS_MAX_NODE_POOL) return fail(LBS_ERR_LIMIT, "gpus_per_node * local_batch exceeds LBS_MAX_NODE_POOL");
    pool = run->gpus_per_node * run->local_batch;
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
  // dynamic LDS in words: histogram, guide tables, then the sorted pools (local) or the trial's histogram (global)
  const uint32_t tables = ds->max_len + 1u + P.guide_words;
  const bool spread = method == LBS_GLOBAL && run->n_gpus <= kMaxSpreadGpus;
  const size_t lds = sizeof(uint32_t) * (tables + (local ? kWaves * pool : method == LBS_GLOBAL ? ds->max_len + 1u + (spread ? run->n_gpus : 0u) : 0u));
  if (e == hipSuccess && run->n_trials > 0) {
    // trials cost the same, so a few workgroups per resident slot balance; each loops over its share of the trials
    const dim3 grid(trial_grid(run->n_trials, run->n_gpus, ds->n_cus)), block(kBlock);
    P.first_trial = run->first_trial, P.n_trials = (uint32_t)run->n_trials;
    if (local) {
      const uint32_t gpn = run->gpus_per_node;
      const bool in_lanes = gpn <= 32 && (gpn & (gpn - 1u)) == 0;
      void (*kernel)(const Params, const uint32_t*, const uint32_t*, uint32_t*, uint32_t*, unsigned long long*) =
          pool <= 64    ? (in_lanes ? k_lbs_local<1, true> : k_lbs_local<1, false>)
          : pool <= 128 ? (in_lanes ? k_lbs_local<2, true> : k_lbs_local<2, false>)
          : pool <= 256 ? (in_lanes ? k_lbs_local<4, true> : k_lbs_local<4, false>)
          : pool <= 512 ? (in_lanes ? k_lbs_local<8, true> : k_lbs_local<8, false>)
                        : (in_lanes ? k_lbs_local<16, true> : k_lbs_local<16, false>);
      hipLaunchKernelGGL(kernel, grid, block, lds, s, P, ds->d_cum, ds->d_guide, trial_min, trial_max, ds_sums);
    } else if (method == LBS_GLOBAL) {
      hipLaunchKernelGGL(spread ? k_lbs_global<true> : k_lbs_global<false>, grid, block, lds, s, P, ds->d_cum, ds->d_guide, trial_min,
                         trial_max, ds_sums);
    } else {
      hipLaunchKernelGGL(k_lbs_keep, grid, block, lds, s, P, ds->d_cum, ds->d_guide, trial_min, trial_max, ds_sums);
    }
    e = hipGetLastError();
  }
  if (prev >= 0 && prev != ds->device) (void)hipSetDevice(prev);
  if (e != hipSuccess) return fail(LBS_ERR_HIP, std::string("launching the simulation: ") + hipGetErrorString(e));
  return 0;
}

int lbs_simulate(const lbs_dataset* ds, const lbs_run* run, uint32_t* trial_min, uint32_t* trial_max, uint64_t* sums,
                 void* stream) {
  if (!ds || !run) return fail(LBS_ERR_NULL, "dataset or run is NULL");
  return simulate_one(ds, run, run->method, trial_min, trial_max, sums, stream);
}

int lbs_simulate_all(const lbs_dataset* ds, const lbs_run* run, uint32_t* trial_min, uint32_t* trial_max, uint64_t* sums,
                     void* stream) {
  if (!ds || !run) return fail(LBS_ERR_NULL, "dataset or run is NULL");
  if (!sums) return fail(LBS_ERR_NULL, "sums is NULL");
  const uint32_t gpn = run->gpus_per_node, lb = run->local_batch, G = run->n_gpus;
  const uint32_t guide_words = kWholeGuideSize + ds->n_strata * kGuideSize;
  const size_t lds = sizeof(uint32_t) * (2u * (size_t)(ds->max_len + 1u) + guide_words + G);
  const bool one_pass = gpn != 0 && gpn <= 32 && (gpn & (gpn - 1u)) == 0 && lb != 0 && lb <= LBS_MAX_LOCAL_BATCH &&
                        (lb & (lb - 1u)) == 0 && G != 0 && G % gpn == 0 && G <= kMaxSpreadGpus && lds <= (60u << 10) &&
                        (uint64_t)gpn * lb <= LBS_MAX_NODE_POOL && ds->device >= 0 && run->n_trials > 0 &&
                        run->n_trials < (1ull << 31);
  if (!one_pass) {  // every other case, errors included: method by method
    for (uint32_t m = 0; m < kMethods; ++m) {
      const int rc = simulate_one(ds, run, m, trial_min ? trial_min + (size_t)m * run->n_trials : nullptr,
                                  trial_max ? trial_max + (size_t)m * run->n_trials : nullptr, sums + 2u * m, stream);
      if (rc != 0) return rc;
    }
    return 0;
  }
  Params P{};
  P.max_len = ds->max_len, P.local_batch = lb, P.gpus_per_node = gpn, P.n_gpus = G, P.stratified = 1;
  P.total = ds->cum[ds->max_len], P.seed = run->seed, P.first_trial = run->first_trial, P.n_trials = (uint32_t)run->n_trials;
  P.guide_words = guide_words;
  uint32_t j = 0;
  for (uint32_t s = 0; s < ds->n_strata; ++s) {
    const uint32_t lo = ds->cum[s == 0 ? 0 : ds->stratum_end[s - 1]], size = ds->cum[ds->stratum_end[s]] - lo;
    if (run->quota[s] && size == 0) return fail(LBS_ERR_ARG, "a stratum with a quota has no entries");
    if ((uint64_t)j + run->quota[s] > lb) return fail(LBS_ERR_ARG, "the quotas exceed local_batch");
    for (uint32_t q = 0; q < run->quota[s]; ++q, ++j) P.slot_lo[j] = lo, P.slot_size[j] = size, P.slot_guide[j] = s * kGuideSize;
  }
  if (j != lb) return fail(LBS_ERR_ARG, "the quotas must add up to local_batch");
  int prev = -1;
  (void)hipGetDevice(&prev);
  if (prev != ds->device && hipSetDevice(ds->device) != hipSuccess) return fail(LBS_ERR_HIP, "hipSetDevice failed");
  hipStream_t s = (hipStream_t)stream;
  unsigned long long* ds_sums = reinterpret_cast<unsigned long long*>(sums);
  hipLaunchKernelGGL(k_lbs_clear_all, dim3(1), dim3(64), 0, s, ds_sums);
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) {
    const dim3 grid(trial_grid(run->n_trials, run->n_gpus, ds->n_cus)), block(kBlock);
    const uint32_t pool = gpn * lb;
    void (*kernel)(const Params, const uint32_t*, const uint32_t*, uint32_t*, uint32_t*, unsigned long long*) =
        pool <= 64 ? k_lbs_all<1> : pool <= 128 ? k_lbs_all<2> : pool <= 256 ? k_lbs_all<4> : pool <= 512 ? k_lbs_all<8> : k_lbs_all<16>;
    hipLaunchKernelGGL(kernel, grid, block, lds, s, P, ds->d_cum, ds->d_guide, trial_min, trial_max, ds_sums);
    e = hipGetLastError();
  }
  if (prev >= 0 && prev != ds->device) (void)hipSetDevice(prev);
  if (e != hipSuccess) return fail(LBS_ERR_HIP, std::string("launching the simulation: ") + hipGetErrorString(e));
  return 0;
}

}  // extern "C"

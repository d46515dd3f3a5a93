// CPU oracle for the load-balancing simulation (per-GPU token counts under the
// paper's batch-forming methods).
//
// TEST INFRASTRUCTURE ONLY.  Plain, single-threaded, obviously correct; only
// tests, the smoke check and the benchmark's cpu_baseline leg may call it.  The
// HIP library shares no code with it.
//
// What is simulated (Sec. 5.2, "Load balancing effect simulation", and App. C,
// Table 5): every GPU retrieves `local_batch` sequences at random (16 in the
// paper), the sequences are redistributed by a load-balancing method, and the
// largest and the smallest per-GPU token count (sum of the sequence lengths a GPU
// ends up with) are recorded; this is repeated over many trials (100 000 in the
// paper) and the two are averaged.  Methods (Sec. 4.1 and Table 5's rows):
//   NONE        each GPU keeps the sequences it drew from the original dataset
//   STRATIFIED  each GPU draws quota[s] sequences from stratum s of the dataset
//               (strata are length ranges; Fig. 3: 5, 2, 3, 6 of 16) and keeps them
//   LOCAL_RASTER / LOCAL_SNAKE
//               stratified draws; then the GPUs of one node (8 in the paper)
//               gather their sequences, sort them by length and scatter them row
//               by row: row r of the sorted list (gpus_per_node consecutive
//               entries) goes to the node's GPUs left to right (raster) or, on
//               every second row, right to left (snake)  (Fig. 4)
//   GLOBAL      draws from the original dataset; all GPUs gather, sort, and the
//               sorted list is dealt row by row over all GPUs (global presorting,
//               Sec. 3.1 "allocate them to GPUs in the sorted order")
//
// Randomness: a counter-based generator so that the GPU can draw the same numbers
// in any order.  Draw number k of a run is the (k+1)-th output of SplitMix64
// (Steele, Lea, Flood 2014) seeded with `seed`; draw k = ((trial * n_gpus + gpu) *
// local_batch + j) belongs to sequence j of that GPU in that trial.  The upper 32
// bits u of a draw pick index (u * n) >> 32 out of n equally likely dataset
// entries; the dataset is given as a cumulative length histogram.
//
// The dataset's real histogram is not printed in the paper (only four bin
// percentages, Sec. 3.1), so Table 5's absolute numbers are "parity unpinned";
// the pins are the generator's published outputs, hand-worked scatter examples,
// conservation and ordering properties, and an independent brute force.

#include <algorithm>
#include <cstdint>
#include <vector>

extern "C" {

enum { LBS_NONE = 0, LBS_STRATIFIED = 1, LBS_LOCAL_RASTER = 2, LBS_LOCAL_SNAKE = 3, LBS_GLOBAL = 4 };

// The (k+1)-th output of SplitMix64 seeded with `seed`.
uint64_t orc_lbs_splitmix64(uint64_t seed, uint64_t k) {
  uint64_t z = seed + (k + 1) * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// Length of dataset entry `index` when the entries are ordered by length:
// cum[l] = number of entries of length <= l, cum[0] = 0; the answer is the
// smallest l with cum[l] > index.
uint32_t orc_lbs_length_of(const uint32_t* cum, uint32_t max_len, uint32_t index) {
  for (uint32_t l = 1; l <= max_len; ++l)
    if (cum[l] > index) return l;
  return max_len;
}

// The local_batch sequence lengths GPU `gpu` retrieves in trial `trial`.
// Original dataset: every entry equally likely.  Stratified: for stratum s,
// quota[s] entries, each equally likely among the stratum's entries (lengths
// stratum_end[s-1]+1 .. stratum_end[s]); strata in order.
void orc_lbs_draw(const uint32_t* cum, uint32_t max_len, int stratified, uint32_t n_strata,
                  const uint32_t* stratum_end, const uint32_t* quota, uint32_t local_batch, uint32_t n_gpus,
                  uint64_t seed, uint64_t trial, uint32_t gpu, uint32_t* out) {
  const uint64_t k0 = (trial * n_gpus + gpu) * static_cast<uint64_t>(local_batch);
  if (!stratified) {
    const uint64_t total = cum[max_len];
    for (uint32_t j = 0; j < local_batch; ++j) {
      const uint64_t u = orc_lbs_splitmix64(seed, k0 + j) >> 32;
      out[j] = orc_lbs_length_of(cum, max_len, static_cast<uint32_t>((u * total) >> 32));
    }
    return;
  }
  uint32_t j = 0;
  for (uint32_t s = 0; s < n_strata; ++s) {
    const uint32_t lo = cum[s == 0 ? 0 : stratum_end[s - 1]];   // entries before the stratum
    const uint64_t size = cum[stratum_end[s]] - lo;             // entries in the stratum
    for (uint32_t q = 0; q < quota[s]; ++q, ++j) {
      const uint64_t u = orc_lbs_splitmix64(seed, k0 + j) >> 32;
      out[j] = orc_lbs_length_of(cum, max_len, lo + static_cast<uint32_t>((u * size) >> 32));
    }
  }
}

// Sort `n_group` GPUs' sequences together and deal them out row by row.
// lengths: n_group * local_batch values (sorted in place); tokens[g] receives
// the token count of GPU g of the group.
void orc_lbs_presort_scatter(uint32_t* lengths, uint32_t n_group, uint32_t local_batch, int snake, uint64_t* tokens) {
  std::sort(lengths, lengths + static_cast<size_t>(n_group) * local_batch);
  for (uint32_t g = 0; g < n_group; ++g) tokens[g] = 0;
  for (uint32_t r = 0; r < local_batch; ++r)
    for (uint32_t c = 0; c < n_group; ++c) {
      const uint32_t g = (snake && (r % 2 == 1)) ? n_group - 1 - c : c;
      tokens[g] += lengths[static_cast<size_t>(r) * n_group + c];
    }
}

// Runs trials first_trial .. first_trial + n_trials - 1.  trial_min / trial_max
// (may be null) receive each trial's smallest / largest per-GPU token count;
// sums[0], sums[1] their totals over the trials (the paper's averages are these
// divided by n_trials).  Returns 0, or -1 for an argument the definition above
// does not cover.
int orc_lbs_simulate(const uint32_t* cum, uint32_t max_len, uint32_t n_strata, const uint32_t* stratum_end,
                     const uint32_t* quota, uint32_t local_batch, uint32_t gpus_per_node, uint32_t n_gpus,
                     int method, uint64_t seed, uint64_t first_trial, uint64_t n_trials, uint32_t* trial_min,
                     uint32_t* trial_max, uint64_t* sums) {
  if (method < LBS_NONE || method > LBS_GLOBAL || n_gpus == 0 || local_batch == 0 || cum[max_len] == 0) return -1;
  const bool stratified = method == LBS_STRATIFIED || method == LBS_LOCAL_RASTER || method == LBS_LOCAL_SNAKE;
  if (stratified) {
    uint32_t q = 0;
    for (uint32_t s = 0; s < n_strata; ++s) {
      q += quota[s];
      if (quota[s] && cum[stratum_end[s]] == cum[s == 0 ? 0 : stratum_end[s - 1]]) return -1;  // empty stratum
    }
    if (q != local_batch || n_strata == 0 || stratum_end[n_strata - 1] != max_len) return -1;
  }
  const bool local = method == LBS_LOCAL_RASTER || method == LBS_LOCAL_SNAKE;
  if (local && (gpus_per_node == 0 || n_gpus % gpus_per_node != 0)) return -1;

  std::vector<uint32_t> drawn(static_cast<size_t>(n_gpus) * local_batch);
  std::vector<uint64_t> tokens(n_gpus);
  sums[0] = sums[1] = 0;
  for (uint64_t t = 0; t < n_trials; ++t) {
    const uint64_t trial = first_trial + t;
    for (uint32_t g = 0; g < n_gpus; ++g)
      orc_lbs_draw(cum, max_len, stratified, n_strata, stratum_end, quota, local_batch, n_gpus, seed, trial, g,
                   &drawn[static_cast<size_t>(g) * local_batch]);
    if (method == LBS_NONE || method == LBS_STRATIFIED) {
      for (uint32_t g = 0; g < n_gpus; ++g) {
        tokens[g] = 0;
        for (uint32_t j = 0; j < local_batch; ++j) tokens[g] += drawn[static_cast<size_t>(g) * local_batch + j];
      }
    } else if (local) {
      for (uint32_t node = 0; node < n_gpus / gpus_per_node; ++node) {
        const size_t first = static_cast<size_t>(node) * gpus_per_node * local_batch;
        std::vector<uint32_t> gathered(drawn.begin() + first, drawn.begin() + first + static_cast<size_t>(gpus_per_node) * local_batch);
        orc_lbs_presort_scatter(gathered.data(), gpus_per_node, local_batch, method == LBS_LOCAL_SNAKE,
                                &tokens[static_cast<size_t>(node) * gpus_per_node]);
      }
    } else {
      std::vector<uint32_t> gathered(drawn);
      orc_lbs_presort_scatter(gathered.data(), n_gpus, local_batch, 0, tokens.data());
    }
    uint64_t lo = tokens[0], hi = tokens[0];
    for (uint32_t g = 1; g < n_gpus; ++g) lo = std::min(lo, tokens[g]), hi = std::max(hi, tokens[g]);
    if (trial_min) trial_min[t] = static_cast<uint32_t>(lo);
    if (trial_max) trial_max[t] = static_cast<uint32_t>(hi);
    sums[0] += lo;
    sums[1] += hi;
  }
  return 0;
}

}  // extern "C"

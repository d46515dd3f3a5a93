// Host side of libbca: plan construction (layout validation, chunk tables,
// bucket groups), binding, argument checks and the compute entry points.  See
// bca.h for the contract of every call.

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <memory>
#include <new>

#include "bca_internal.h"

namespace bca {

static thread_local std::string g_last_error;
void set_error(const std::string& msg) { g_last_error = msg; }

namespace {

int fail(int code, const std::string& msg) {
  set_error(msg);
  return code;
}

int fail_hip(hipError_t e, const char* what) {
  return fail(BCA_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

// No C++ exception may cross the C boundary: the calls that grow host containers run through this.
template <class F>
int no_throw(F&& body) {
  try {
    return body();
  } catch (const std::bad_alloc&) {
    g_last_error.clear();  // no allocation while reporting the lack of memory
    return BCA_ERR_NOMEM;
  } catch (...) {
    return BCA_ERR_NOMEM;
  }
}

uint64_t grad_bytes(int gdt) { return gdt == BCA_GRAD_F32 ? 4 : 2; }

// Makes the plan's device current for the lifetime of the object.
struct DeviceGuard {
  int prev = -1;
  bool ok = true;
  explicit DeviceGuard(int dev) {
    if (hipGetDevice(&prev) != hipSuccess) prev = -1;
    if (prev != dev) ok = (hipSetDevice(dev) == hipSuccess);
  }
  ~DeviceGuard() {
    int cur = -1;
    if (prev >= 0 && hipGetDevice(&cur) == hipSuccess && cur != prev) (void)hipSetDevice(prev);
  }
};

// Every element of every tensor must be covered by exactly one segment.
int validate_layout(uint32_t n_tensors, const uint64_t* numel, uint32_t n_buckets, const uint64_t* seg_off,
                    const bca_segment* segs) {
  if (seg_off[0] != 0) return fail(BCA_ERR_LAYOUT, "bucket_seg_off[0] must be 0");
  for (uint32_t b = 0; b < n_buckets; ++b)
    if (seg_off[b + 1] < seg_off[b]) return fail(BCA_ERR_LAYOUT, "bucket_seg_off must be non-decreasing");
  const uint64_t n_seg = seg_off[n_buckets];
  std::vector<std::vector<std::pair<uint64_t, uint64_t>>> per_tensor(n_tensors);
  for (uint64_t s = 0; s < n_seg; ++s) {
    const bca_segment& sg = segs[s];
    char buf[160];
    if (sg.tensor >= n_tensors) {
      snprintf(buf, sizeof buf, "segment %llu names tensor %u of %u", (unsigned long long)s, sg.tensor, n_tensors);
      return fail(BCA_ERR_LAYOUT, buf);
    }
    if (sg.reserved != 0) return fail(BCA_ERR_LAYOUT, "segment.reserved must be 0");
    if (sg.begin > numel[sg.tensor] || sg.len > numel[sg.tensor] - sg.begin) {
      snprintf(buf, sizeof buf, "segment %llu [%llu, +%llu) exceeds tensor %u of %llu elements",
               (unsigned long long)s, (unsigned long long)sg.begin, (unsigned long long)sg.len, sg.tensor,
               (unsigned long long)numel[sg.tensor]);
      return fail(BCA_ERR_LAYOUT, buf);
    }
    if (sg.len) per_tensor[sg.tensor].emplace_back(sg.begin, sg.len);
  }
  for (uint32_t t = 0; t < n_tensors; ++t) {
    auto& v = per_tensor[t];
    std::sort(v.begin(), v.end());
    uint64_t pos = 0;
    for (auto& pr : v) {
      if (pr.first != pos) {
        char buf[160];
        snprintf(buf, sizeof buf, "tensor %u: segments %s at element %llu", t, pr.first < pos ? "overlap" : "leave a gap",
                 (unsigned long long)std::min(pos, pr.first));
        return fail(BCA_ERR_LAYOUT, buf);
      }
      pos += pr.second;
    }
    if (pos != numel[t]) {
      char buf[160];
      snprintf(buf, sizeof buf, "tensor %u: segments cover %llu of %llu elements", t, (unsigned long long)pos,
               (unsigned long long)numel[t]);
      return fail(BCA_ERR_LAYOUT, buf);
    }
  }
  return BCA_OK;
}

// Cut every segment at multiples of chunk_elems counted from the start of its
// tensor, so that all chunks but a segment's first start vector-aligned.
void build_table(Table* t, uint32_t chunk_elems, uint32_t n_buckets, const uint64_t* seg_off, const bca_segment* segs) {
  const uint64_t C = chunk_elems;
  t->chunk_elems = chunk_elems;
  t->chunks.clear();
  t->bucket_off.assign(n_buckets + 1, 0);
  for (uint32_t b = 0; b < n_buckets; ++b) {
    t->bucket_off[b] = (uint32_t)t->chunks.size();
    for (uint64_t s = seg_off[b]; s < seg_off[b + 1]; ++s) {
      uint64_t pos = segs[s].begin;
      const uint64_t end = segs[s].begin + segs[s].len;
      while (pos < end) {
        const uint64_t stop = std::min(end, (pos / C + 1) * C);
        t->chunks.push_back(ChunkInfo{segs[s].tensor, (uint32_t)(stop - pos), pos, b});
        pos = stop;
      }
    }
  }
  t->bucket_off[n_buckets] = (uint32_t)t->chunks.size();
}

// The same cut, tensor by tensor: tensor t's pieces in the order of their position in
// the tensor, so that the chunks (and partial sums) of a tensor are contiguous.  A
// chunk still lies in one bucket, because the clip coefficient is the bucket's.
void build_tensor_table(Table* t, std::vector<uint32_t>* tensor_off, uint32_t chunk_elems, uint32_t n_tensors,
                        uint32_t n_buckets, const uint64_t* seg_off, const bca_segment* segs) {
  const uint64_t C = chunk_elems;
  t->chunk_elems = chunk_elems;
  t->chunks.clear();
  t->bucket_off.clear();
  struct Piece {
    uint64_t begin, len;
    uint32_t bucket;
  };
  std::vector<std::vector<Piece>> per_tensor(n_tensors);
  for (uint32_t b = 0; b < n_buckets; ++b)
    for (uint64_t s = seg_off[b]; s < seg_off[b + 1]; ++s)
      if (segs[s].len) per_tensor[segs[s].tensor].push_back(Piece{segs[s].begin, segs[s].len, b});
  tensor_off->assign(n_tensors + 1, 0);
  for (uint32_t ti = 0; ti < n_tensors; ++ti) {
    (*tensor_off)[ti] = (uint32_t)t->chunks.size();
    auto& v = per_tensor[ti];
    std::sort(v.begin(), v.end(), [](const Piece& a, const Piece& b) { return a.begin < b.begin; });
    for (const Piece& pc : v) {
      uint64_t pos = pc.begin;
      const uint64_t end = pc.begin + pc.len;
      while (pos < end) {
        const uint64_t stop = std::min(end, (pos / C + 1) * C);
        t->chunks.push_back(ChunkInfo{ti, (uint32_t)(stop - pos), pos, pc.bucket});
        pos = stop;
      }
    }
  }
  (*tensor_off)[n_tensors] = (uint32_t)t->chunks.size();
}

// Consecutive buckets are put in one group until their gradients exceed
// group_bytes (0: the library default).  A group has at least one bucket.
void build_groups(bca_plan* p, uint64_t group_bytes, const uint64_t* seg_off, const bca_segment* segs) {
  p->groups.clear();
  const uint64_t gsize = grad_bytes(p->grad_dtype);
  if (group_bytes == 0) group_bytes = kDefaultGroupElems * gsize;
  uint32_t first = 0;
  uint64_t acc = 0;
  for (uint32_t b = 0; b < p->n_buckets; ++b) {
    uint64_t bytes = 0;
    for (uint64_t s = seg_off[b]; s < seg_off[b + 1]; ++s) bytes += segs[s].len * gsize;
    if (b > first && acc + bytes > group_bytes) {
      p->groups.emplace_back(first, b);
      first = b;
      acc = 0;
    }
    acc += bytes;
  }
  p->groups.emplace_back(first, p->n_buckets);
}

// lamb_step sweeps the tensors in runs of consecutive tensors of at most `limit` elements (0: the library default; a
// tensor larger than that is a run of its own): the second sweep of a run then finds the moments that the first
// sweep has just written in cache.
void build_lamb_groups(bca_plan* p, uint64_t limit) {
  p->lamb_groups.clear();
  if (limit == 0) limit = kLambGroupElems;
  uint32_t first = 0;
  uint64_t acc = 0;
  for (uint32_t t = 0; t < p->n_tensors; ++t) {
    const uint64_t n = p->tensor_numel[t];
    if (t > first && (acc + n > limit || acc + n < acc)) {
      p->lamb_groups.emplace_back(first, t);
      first = t;
      acc = 0;
    }
    acc += n;
  }
  p->lamb_groups.emplace_back(first, p->n_tensors);
}

// Elements a squared-norm item of the fused step reads when the caller does not say: the largest power of
// two in [16 Ki, 64 Ki] that still gives an average bucket group 160 items or more.  Fewer, larger items
// mean fewer workgroups and arrivals; but a group's squared-norm items are all that keeps its Adam items
// from waiting, and below ~200 of them (256 CUs) they finish late (measured: 64 Ki best for 50 MiB
// buckets, 32 Ki for 25 MiB and 4 MiB ones).
uint32_t default_norm_item_elems(const bca_plan* p, const uint64_t* seg_off, const bca_segment* segs) {
  uint64_t total = 0;
  for (uint64_t s = 0; s < seg_off[p->n_buckets]; ++s) total += segs[s].len;
  const uint64_t per_group = total / std::max<size_t>(p->groups.size(), 1);
  uint32_t c = kMaxNormItemElems;
  while (c > kMinNormItemElems && per_group / c < 160) c >>= 1;
  return c;
}

// Work items of the single-launch step in pipeline order: the squared-norm
// chunks of group i+1 come before the Adam chunks of group i, so that by the
// time a bucket's Adam items start, its norm has long been finished, and its
// gradients are read twice within two groups' worth of traffic.
void build_work(bca_plan* p) {
  p->work.clear();
  const Table& TN = p->norm_tab;
  const Table& TA = p->apply_tab;
  const uint32_t span_all = std::min(std::max(p->norm_item_chunks, 1u), kMaxNormItemChunks);
  auto push_norm = [&](const std::pair<uint32_t, uint32_t>& g) {
    // The launch starts with nothing to do but the first group's squared norms while the first Adam items wait:
    // that group is handed out chunk by chunk, so that more workgroups share it and it is done sooner.
    const uint32_t span = g.first == 0 ? 1u : span_all;
    for (uint32_t b = g.first; b < g.second; ++b) {
      if (TN.bucket_off[b] == TN.bucket_off[b + 1]) p->work.push_back((kItemEmpty << 30) | b);
      // an item is up to `span` consecutive chunks of one bucket: first chunk in bits 0..27, count - 1 in bits 28..29
      for (uint32_t c = TN.bucket_off[b]; c < TN.bucket_off[b + 1]; c += span) {
        const uint32_t cnt = std::min(span, TN.bucket_off[b + 1] - c);
        p->work.push_back((kItemNorm << 30) | ((cnt - 1u) << 28) | c);
      }
    }
  };
  auto push_adam = [&](const std::pair<uint32_t, uint32_t>& g) {
    for (uint32_t c = TA.bucket_off[g.first]; c < TA.bucket_off[g.second]; ++c) p->work.push_back((kItemAdam << 30) | c);
  };
  const size_t G = p->groups.size(), lead = std::max(p->norm_lead, 1u);
  for (size_t i = 0; i < G + lead; ++i) {
    if (i < G) push_norm(p->groups[i]);
    if (i >= lead && i - lead < G) push_adam(p->groups[i - lead]);
  }
}

void free_profile(bca_plan* p) {
  for (hipEvent_t e : p->prof_events) (void)hipEventDestroy(e);
  p->prof_events.clear();
  p->prof_calls = 0;
}

void free_device(bca_plan* p) {
  if (p->device < 0) return;
  DeviceGuard g(p->device);
  free_profile(p);
  for (Table* t : {&p->norm_tab, &p->apply_tab, &p->lamb_tab}) {
    if (t->d_chunks) (void)hipFree(t->d_chunks);
    if (t->d_bucket_off) (void)hipFree(t->d_bucket_off);
    t->d_chunks = nullptr, t->d_bucket_off = nullptr;
  }
  if (p->d_work) (void)hipFree(p->d_work);
  if (p->d_arrived) (void)hipFree(p->d_arrived);
  if (p->d_ready) (void)hipFree(p->d_ready);
  if (p->d_ctl) (void)hipFree(p->d_ctl);
  if (p->d_skipped) (void)hipFree(p->d_skipped);
  p->d_work = nullptr, p->d_arrived = nullptr, p->d_ready = nullptr, p->d_ctl = nullptr, p->d_skipped = nullptr;
  if (p->d_partials) (void)hipFree(p->d_partials);
  if (p->d_norms) (void)hipFree(p->d_norms);
  if (p->d_bucket_sq) (void)hipFree(p->d_bucket_sq);
  p->d_bucket_sq = nullptr;
  if (p->d_tensor_off) (void)hipFree(p->d_tensor_off);
  if (p->d_apply_to_lamb) (void)hipFree(p->d_apply_to_lamb);
  p->d_apply_to_lamb = nullptr;
  if (p->d_lamb_sums) (void)hipFree(p->d_lamb_sums);
  if (p->d_trust) (void)hipFree(p->d_trust);
  if (p->d_lamb_scale) (void)hipFree(p->d_lamb_scale);
  p->d_tensor_off = nullptr, p->d_lamb_sums = nullptr, p->d_trust = nullptr, p->d_lamb_scale = nullptr;
  if (p->d_adamk) (void)hipFree(p->d_adamk);
  p->d_adamk = nullptr;
  if (p->d_coefs) (void)hipFree(p->d_coefs);
  if (p->d_status) (void)hipFree(p->d_status);
  p->d_partials = nullptr, p->d_norms = nullptr, p->d_coefs = nullptr, p->d_status = nullptr;
}

hipError_t alloc_table(Table* t, uint32_t n_buckets) {
  const size_t nc = std::max<size_t>(t->chunks.size(), 1);
  hipError_t e = hipMalloc((void**)&t->d_chunks, nc * sizeof(Chunk));
  if (t->bucket_off.empty()) return e;  // the tensor-major table has no bucket offsets
  if (e == hipSuccess) e = hipMalloc((void**)&t->d_bucket_off, (n_buckets + 1) * sizeof(uint32_t));
  if (e == hipSuccess)
    e = hipMemcpy(t->d_bucket_off, t->bucket_off.data(), (n_buckets + 1) * sizeof(uint32_t), hipMemcpyHostToDevice);
  return e;
}

// Writes a table's device copy from the bound pointers and the decay mask.
hipError_t upload_table(const bca_plan* p, Table* t) {
  const uint64_t gsize = grad_bytes(p->grad_dtype);
  std::vector<Chunk> table(std::max<size_t>(t->chunks.size(), 1));
  memset(table.data(), 0, table.size() * sizeof(Chunk));
  for (size_t i = 0; i < t->chunks.size(); ++i) {
    const ChunkInfo& c = t->chunks[i];
    table[i].g = p->bound_g[c.tensor] + c.begin * gsize;
    table[i].p = p->bound_p[c.tensor] + c.begin * 4;
    table[i].m = p->bound_m[c.tensor] + c.begin * 4;
    table[i].v = p->bound_v[c.tensor] + c.begin * 4;
    table[i].len = c.len;
    table[i].bucket = c.bucket;
    table[i].tensor = c.tensor;
    table[i].flags = p->decay[c.tensor] ? 0u : kChunkNoDecay;
  }
  return hipMemcpy(t->d_chunks, table.data(), table.size() * sizeof(Chunk), hipMemcpyHostToDevice);
}

// Kernels enqueued earlier on any stream may still be reading the old tables, so
// wait for them before the (host-synchronous) copies.
hipError_t upload_all_tables(bca_plan* p) {
  hipError_t e = hipDeviceSynchronize();
  for (Table* t : {&p->norm_tab, &p->apply_tab, &p->lamb_tab})
    if (e == hipSuccess) e = upload_table(p, t);
  return e;
}

StepState step_state(const bca_plan* p) {
  StepState ss;
  ss.norm_tab = p->norm_tab.d_chunks, ss.apply_tab = p->apply_tab.d_chunks;
  ss.norm_bucket_off = p->norm_tab.d_bucket_off;
  ss.partials = p->d_partials, ss.arrived = p->d_arrived, ss.ready = p->d_ready, ss.ctl = p->d_ctl;
  ss.skipped = p->d_skipped, ss.skipped_cap = (uint32_t)std::max<size_t>(p->apply_tab.chunks.size(), 1);
  ss.apply_to_lamb = p->d_apply_to_lamb, ss.lamb_sums = p->d_lamb_sums;
  ss.spin_limit = p->spin_limit;
  return ss;
}

// For every chunk of the apply table, the index of the same chunk (same tensor, same first
// element: both tables cut at the same places) in the tensor-major table.
std::vector<uint32_t> apply_to_lamb_map(const bca_plan* p) {
  const auto& A = p->apply_tab.chunks;
  const auto& L = p->lamb_tab.chunks;
  std::vector<uint32_t> map(A.size());
  for (size_t i = 0; i < A.size(); ++i) {
    uint32_t lo = p->tensor_off[A[i].tensor], hi = p->tensor_off[A[i].tensor + 1];
    while (lo + 1 < hi) {  // chunks of a tensor are sorted by their first element
      const uint32_t mid = lo + (hi - lo) / 2;
      if (L[mid].begin <= A[i].begin) lo = mid;
      else hi = mid;
    }
    map[i] = lo;
  }
  return map;
}

int check_ready(const bca_plan* p) {
  if (!p) return fail(BCA_ERR_NULL, "plan is NULL");
  if (p->device < 0) return fail(BCA_ERR_UNBOUND, "host-only plan (device -1) cannot run kernels");
  if (!p->bound) return fail(BCA_ERR_UNBOUND, "bca_plan_bind has not been called");
  return BCA_OK;
}

int check_range(const bca_plan* p, uint32_t b0, uint32_t b1) {
  if (b0 > b1 || b1 > p->n_buckets) {
    char buf[96];
    snprintf(buf, sizeof buf, "bucket range [%u, %u) outside [0, %u]", b0, b1, p->n_buckets);
    return fail(BCA_ERR_RANGE, buf);
  }
  return BCA_OK;
}

// The constants of one call: from the host arguments, or (hyper-parameters in device memory) a pointer to
// the device copy that enqueue_hyper fills on the call's stream.
int make_adam_constants(const bca_plan* p, const bca_adam* hp, uint64_t step, AdamK* k) {
  *k = AdamK{};
  if (p->hyper_dev != nullptr) {
    k->from = p->d_adamk;
    return BCA_OK;
  }
  if (!hp) return fail(BCA_ERR_NULL, "hyper-parameters are NULL");
  if (step == 0) return fail(BCA_ERR_HPARAM, "step counts from 1");
  if (!(hp->beta1 >= 0.0 && hp->beta1 < 1.0)) return fail(BCA_ERR_HPARAM, "beta1 must lie in [0, 1)");
  if (!(hp->beta2 >= 0.0 && hp->beta2 < 1.0)) return fail(BCA_ERR_HPARAM, "beta2 must lie in [0, 1)");
  if (!(hp->eps >= 0.0) || !std::isfinite(hp->eps)) return fail(BCA_ERR_HPARAM, "eps must be finite and >= 0");
  if (!std::isfinite(hp->lr)) return fail(BCA_ERR_HPARAM, "lr must be finite");
  if (!std::isfinite(hp->weight_decay)) return fail(BCA_ERR_HPARAM, "weight_decay must be finite");
  const double t = (double)step;
  const double bc1 = 1.0 - std::pow(hp->beta1, t);
  const double bc2 = 1.0 - std::pow(hp->beta2, t);
  k->b1 = (float)hp->beta1, k->omb1 = (float)(1.0 - hp->beta1);
  k->b2 = (float)hp->beta2, k->omb2 = (float)(1.0 - hp->beta2);
  k->rbc1 = (float)(1.0 / bc1), k->rbc2 = (float)(1.0 / bc2);
  k->eps = (float)hp->eps;
  k->neg_lr = (float)(-hp->lr);
  k->wd = (float)hp->weight_decay;
  k->lr = hp->lr;
  return BCA_OK;
}

// With hyper-parameters in device memory: the one-thread kernel that derives this call's constants.
int enqueue_hyper(const bca_plan* p, hipStream_t stream) {
  if (p->hyper_dev == nullptr) return BCA_OK;
  const hipError_t e = launch_hyper(p->hyper_dev, p->d_adamk, stream);
  return e == hipSuccess ? BCA_OK : fail_hip(e, "launching the hyper-parameter kernel");
}

// Workgroups of a stand-alone squared-norm launch over n chunks: the plan's grid_norm if the caller set one, else
// as many as the fused step would use items for them (a workgroup then reads several 16 Ki chunks, which streams
// better than one workgroup per chunk once there are thousands of chunks).
uint32_t norm_grid(const bca_plan* p, uint32_t n_chunks) {
  if (p->grid_norm) return p->grid_norm;
  const uint32_t span = std::max(p->norm_item_chunks, 1u);
  return (n_chunks + span - 1) / span;
}

// requested == 0: one workgroup per chunk.
Launch make_launch(const bca_plan* p, uint32_t requested, uint32_t n_chunks, bool g_keep) {
  const uint32_t g = requested ? std::min(requested, n_chunks) : n_chunks;
  Launch L;
  L.grid = std::max(g, 1u);
  L.unroll = p->unroll_apply;
  L.staged = (p->tune_flags & BCA_TUNE_STAGE_TABLE_LDS) != 0;
  L.g_keep = g_keep;
  L.lds = g_keep ? 0 : p->adam_lds_reserve;  // grouped sweeps read g from cache and are fastest at full occupancy
  return L;
}

}  // namespace
}  // namespace bca

using namespace bca;

extern "C" {

int bca_version(void) { return 1; }

const char* bca_last_error(void) { return g_last_error.c_str(); }

static int plan_create(bca_plan** out, int device, uint32_t n_tensors, const uint64_t* tensor_numel, uint32_t n_buckets,
                       const uint64_t* bucket_seg_off, const bca_segment* segments, int grad_dtype,
                       const bca_tuning* tuning) {
  if (!out) return fail(BCA_ERR_NULL, "out is NULL");
  *out = nullptr;
  if (!bucket_seg_off) return fail(BCA_ERR_NULL, "bucket_seg_off is NULL");
  if (n_tensors && !tensor_numel) return fail(BCA_ERR_NULL, "tensor_numel is NULL");
  if (n_buckets == 0) return fail(BCA_ERR_LAYOUT, "a plan needs at least one bucket");
  if (grad_dtype != BCA_GRAD_F32 && grad_dtype != BCA_GRAD_F16 && grad_dtype != BCA_GRAD_BF16)
    return fail(BCA_ERR_DTYPE, "unknown gradient type");
  if (bucket_seg_off[n_buckets] && !segments) return fail(BCA_ERR_NULL, "segments is NULL");
  if (device < -1) return fail(BCA_ERR_RANGE, "device must be >= 0, or -1 for a host-only plan");
  uint32_t chunk_norm = 0, chunk_apply = kDefaultChunkApply, unroll = 0;
  if (tuning) {
    for (uint32_t c : {tuning->chunk_norm, tuning->chunk_apply})
      if (c % 1024u || c > (1u << 24)) return fail(BCA_ERR_RANGE, "chunk sizes must be multiples of 1024, at most 2^24");
    if (tuning->chunk_norm) chunk_norm = tuning->chunk_norm;
    if (tuning->chunk_apply) chunk_apply = tuning->chunk_apply;
    if (tuning->unroll_apply) {
      if (tuning->unroll_apply != 1 && tuning->unroll_apply != 2 && tuning->unroll_apply != 4)
        return fail(BCA_ERR_RANGE, "unroll_apply must be 1, 2 or 4");
      unroll = tuning->unroll_apply;
    }
    if (tuning->flags & ~(BCA_TUNE_MULTI_LAUNCH | BCA_TUNE_STAGE_TABLE_LDS | BCA_TUNE_TICKETS))
      return fail(BCA_ERR_RANGE, "unknown tuning flag bits");
    if (tuning->adam_lds_reserve > 65536) return fail(BCA_ERR_RANGE, "adam_lds_reserve must be at most 65536");
    if (tuning->norm_item_chunks > kMaxNormItemChunks) return fail(BCA_ERR_RANGE, "norm_item_chunks must be at most 4");
    if (tuning->norm_lead > 64) return fail(BCA_ERR_RANGE, "norm_lead must be at most 64");
  }
  if (int rc = validate_layout(n_tensors, tensor_numel, n_buckets, bucket_seg_off, segments)) return rc;

  struct Release {  // a plan that is not handed out is freed, device memory included
    void operator()(bca_plan* q) const {
      free_device(q);
      delete q;
    }
  };
  std::unique_ptr<bca_plan, Release> owner(new bca_plan);
  bca_plan* p = owner.get();
  p->device = -1;  // becomes `device` once that device is known to exist: until then there is nothing to free on it
  p->grad_dtype = grad_dtype;
  p->n_tensors = n_tensors;
  p->n_buckets = n_buckets;
  p->grid_norm = tuning ? tuning->grid_norm : 0;
  p->grid_apply = tuning ? tuning->grid_apply : 0;
  // default: as many 128-bit accesses in flight as one pass over a full chunk needs, at most 4
  p->unroll_apply = unroll ? unroll : (chunk_apply >= 4096 ? 4u : chunk_apply >= 2048 ? 2u : 1u);
  p->tune_flags = tuning ? tuning->flags : 0;
  p->adam_lds_reserve = (tuning && tuning->adam_lds_reserve) ? (tuning->adam_lds_reserve == 1 ? 0 : tuning->adam_lds_reserve)
                                                              : kDefaultAdamLdsReserve;
  p->spin_limit = (tuning && tuning->spin_limit) ? tuning->spin_limit : kDefaultSpinLimit;
  p->tensor_numel.assign(tensor_numel, tensor_numel + n_tensors);
  p->decay.assign(n_tensors, 1);
  build_groups(p, tuning ? tuning->group_bytes : 0, bucket_seg_off, segments);
  // Squared norms run one bucket group ahead of the Adam items; two when groups hold several buckets (measured: with
  // 4 MiB buckets 13 K instead of 2 K Adam items per step find their bucket not ready at one group's lead, and the
  // step takes 2.4 % longer), which leaves three groups' gradients to be kept cached: fine for 8 Mi-element groups,
  // too much for groups that are one 50 MiB bucket.
  p->norm_lead = (tuning && tuning->norm_lead) ? tuning->norm_lead : (p->n_buckets >= 2 * p->groups.size() ? 2 : 1);
  if (tuning && tuning->norm_item_chunks) {
    p->norm_item_chunks = tuning->norm_item_chunks;
  } else if (chunk_norm == 0) {
    p->norm_item_chunks = default_norm_item_elems(p, bucket_seg_off, segments) / kDefaultChunkNorm;
  } else {
    p->norm_item_chunks = 1;  // a caller who names the chunk gets one chunk per item unless told otherwise
  }
  if (chunk_norm == 0) chunk_norm = kDefaultChunkNorm;
  build_table(&p->norm_tab, chunk_norm, n_buckets, bucket_seg_off, segments);
  if (p->norm_tab.chunks.size() >= (1ull << 28))
    return fail(BCA_ERR_RANGE, "too many squared-norm chunks; raise chunk_norm");
  build_table(&p->apply_tab, chunk_apply, n_buckets, bucket_seg_off, segments);
  build_tensor_table(&p->lamb_tab, &p->tensor_off, chunk_apply, n_tensors, n_buckets, bucket_seg_off, segments);
  build_lamb_groups(p, tuning ? tuning->lamb_group_elems : 0);
  build_work(p);
  // A launch holds at most 2^32 threads: with 256 per workgroup that is 2^24 workgroups.
  if (p->work.size() >= (1ull << 24))
    return fail(BCA_ERR_RANGE, "too many chunks for one launch; raise chunk_norm / chunk_apply");

  if (device >= 0) {
    int n_dev = 0;
    hipError_t e = hipGetDeviceCount(&n_dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDeviceCount");
    if (device >= n_dev) return fail(BCA_ERR_RANGE, "no such device");
    DeviceGuard g(device);
    if (!g.ok) return fail(BCA_ERR_HIP, "hipSetDevice failed");
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, device);
    if (e != hipSuccess) return fail_hip(e, "hipGetDeviceProperties");
    if (prop.warpSize != 64) return fail(BCA_ERR_HIP, "the kernels need 64-wide wavefronts (gfx950)");
    p->device = device;
    const size_t np = std::max<size_t>(p->norm_tab.chunks.size(), 1) * kWaves;
    const size_t nb = n_buckets;
    const size_t nl = std::max<size_t>(p->lamb_tab.chunks.size(), 1), nt = std::max<size_t>(n_tensors, 1);
    const std::vector<uint32_t> a2l = apply_to_lamb_map(p);
    const uint32_t first_epoch = 1;  // ready words start at zero: epoch 0 is never current
    if ((e = alloc_table(&p->norm_tab, n_buckets)) != hipSuccess ||
        (e = alloc_table(&p->apply_tab, n_buckets)) != hipSuccess ||
        (e = alloc_table(&p->lamb_tab, n_buckets)) != hipSuccess ||
        (e = hipMalloc((void**)&p->d_tensor_off, (n_tensors + 1) * sizeof(uint32_t))) != hipSuccess ||
        (e = hipMemcpy(p->d_tensor_off, p->tensor_off.data(), (n_tensors + 1) * sizeof(uint32_t),
                       hipMemcpyHostToDevice)) != hipSuccess ||
        (e = hipMalloc((void**)&p->d_apply_to_lamb, nl * sizeof(uint32_t))) != hipSuccess ||
        (e = hipMemcpy(p->d_apply_to_lamb, a2l.data(), a2l.size() * sizeof(uint32_t), hipMemcpyHostToDevice)) !=
            hipSuccess ||
        (e = hipMalloc((void**)&p->d_lamb_sums, nl * 2 * sizeof(double))) != hipSuccess ||
        (e = hipMalloc((void**)&p->d_trust, nt * sizeof(float))) != hipSuccess ||
        (e = hipMalloc((void**)&p->d_lamb_scale, nt * sizeof(float))) != hipSuccess ||
        (e = hipMalloc((void**)&p->d_work, std::max<size_t>(p->work.size(), 1) * sizeof(uint32_t))) != hipSuccess ||
        (e = hipMemcpy(p->d_work, p->work.data(), p->work.size() * sizeof(uint32_t), hipMemcpyHostToDevice)) !=
            hipSuccess ||
        (e = hipMalloc((void**)&p->d_arrived, nb * sizeof(uint32_t))) != hipSuccess ||
        (e = hipMemset(p->d_arrived, 0, nb * sizeof(uint32_t))) != hipSuccess ||
        (e = hipMalloc((void**)&p->d_ready, nb * sizeof(unsigned long long))) != hipSuccess ||
        (e = hipMemset(p->d_ready, 0, nb * sizeof(unsigned long long))) != hipSuccess ||
        (e = hipMalloc((void**)&p->d_ctl, kCtlWords * sizeof(uint32_t))) != hipSuccess ||
        (e = hipMemset(p->d_ctl, 0, kCtlWords * sizeof(uint32_t))) != hipSuccess ||
        (e = hipMemcpy(p->d_ctl + kCtlEpoch, &first_epoch, sizeof first_epoch, hipMemcpyHostToDevice)) != hipSuccess ||
        (e = hipMalloc((void**)&p->d_skipped, std::max<size_t>(p->apply_tab.chunks.size(), 1) * sizeof(uint32_t))) !=
            hipSuccess ||
        (e = hipMalloc((void**)&p->d_partials, np * sizeof(double))) != hipSuccess ||
        (e = hipMalloc((void**)&p->d_norms, (nb + 1) * sizeof(float))) != hipSuccess ||
        (e = hipMalloc((void**)&p->d_bucket_sq, nb * sizeof(double))) != hipSuccess ||
        (e = hipMalloc((void**)&p->d_coefs, nb * sizeof(float))) != hipSuccess ||
        (e = hipMalloc((void**)&p->d_adamk, sizeof(AdamK))) != hipSuccess ||
        (e = hipMalloc((void**)&p->d_status, sizeof(int32_t))) != hipSuccess ||
        (e = hipMemset(p->d_status, 0, sizeof(int32_t))) != hipSuccess)
      return fail_hip(e, "allocating plan memory");
  }
  *out = owner.release();
  return BCA_OK;
}

int bca_plan_create(bca_plan** out, int device, uint32_t n_tensors, const uint64_t* tensor_numel, uint32_t n_buckets,
                    const uint64_t* bucket_seg_off, const bca_segment* segments, int grad_dtype,
                    const bca_tuning* tuning) {
  return no_throw([&] {
    return plan_create(out, device, n_tensors, tensor_numel, n_buckets, bucket_seg_off, segments, grad_dtype, tuning);
  });
}

static int plan_bind(bca_plan* p, void* const* grads, float* const* params, float* const* exp_avg,
                     float* const* exp_avg_sq) {
  if (!p) return fail(BCA_ERR_NULL, "plan is NULL");
  if (p->device < 0) return fail(BCA_ERR_UNBOUND, "host-only plan (device -1) cannot be bound");
  if (p->n_tensors && (!grads || !params || !exp_avg || !exp_avg_sq)) return fail(BCA_ERR_NULL, "a pointer array is NULL");
  const uint64_t gsize = grad_bytes(p->grad_dtype);
  for (uint32_t t = 0; t < p->n_tensors; ++t) {
    if (p->tensor_numel[t] == 0) continue;
    char buf[96];
    if (!grads[t] || !params[t] || !exp_avg[t] || !exp_avg_sq[t]) {
      snprintf(buf, sizeof buf, "tensor %u: NULL device pointer", t);
      return fail(BCA_ERR_NULL, buf);
    }
    if (((uintptr_t)grads[t] % gsize) || ((uintptr_t)params[t] % 4) || ((uintptr_t)exp_avg[t] % 4) ||
        ((uintptr_t)exp_avg_sq[t] % 4)) {
      snprintf(buf, sizeof buf, "tensor %u: pointer not aligned to its element size", t);
      return fail(BCA_ERR_ALIGN, buf);
    }
  }
  DeviceGuard g(p->device);
  p->bound = false;
  p->bound_g.assign(p->n_tensors, 0), p->bound_p.assign(p->n_tensors, 0);
  p->bound_m.assign(p->n_tensors, 0), p->bound_v.assign(p->n_tensors, 0);
  for (uint32_t t = 0; t < p->n_tensors; ++t) {
    p->bound_g[t] = (uint64_t)(uintptr_t)grads[t], p->bound_p[t] = (uint64_t)(uintptr_t)params[t];
    p->bound_m[t] = (uint64_t)(uintptr_t)exp_avg[t], p->bound_v[t] = (uint64_t)(uintptr_t)exp_avg_sq[t];
  }
  hipError_t e = upload_all_tables(p);
  if (e != hipSuccess) return fail_hip(e, "uploading the chunk tables");
  p->bound = true;
  return BCA_OK;
}

int bca_plan_bind(bca_plan* p, void* const* grads, float* const* params, float* const* exp_avg,
                  float* const* exp_avg_sq) {
  return no_throw([&] { return plan_bind(p, grads, params, exp_avg, exp_avg_sq); });
}

int bca_plan_set_decay_mask(bca_plan* p, const uint8_t* decay) {
  if (!p) return fail(BCA_ERR_NULL, "plan is NULL");
  for (uint32_t t = 0; t < p->n_tensors; ++t) p->decay[t] = decay ? (decay[t] != 0) : 1;
  if (p->device < 0 || !p->bound) return BCA_OK;  // the next bind writes the flags
  DeviceGuard g(p->device);
  return no_throw([&] {
    hipError_t e = upload_all_tables(p);
    if (e != hipSuccess) {
      p->bound = false;
      return fail_hip(e, "uploading the chunk tables");
    }
    return (int)BCA_OK;
  });
}

int bca_plan_set_device_hyper(bca_plan* p, const bca_adam_device* dev) {
  if (!p) return fail(BCA_ERR_NULL, "plan is NULL");
  if (p->device < 0) return fail(BCA_ERR_UNBOUND, "host-only plan (device -1) has no device hyper-parameters");
  if (((uintptr_t)dev) % 8u) return fail(BCA_ERR_ALIGN, "dev must be 8-byte aligned");
  p->hyper_dev = dev;
  return BCA_OK;
}

void bca_plan_destroy(bca_plan* p) {
  if (!p) return;
  if (p->device >= 0) {
    DeviceGuard g(p->device);
    (void)hipDeviceSynchronize();
  }
  free_device(p);
  delete p;
}

uint32_t bca_plan_num_buckets(const bca_plan* p) { return p ? p->n_buckets : 0; }

static const Table* pick_table(const bca_plan* p, int which) {
  if (!p) {
    fail(BCA_ERR_NULL, "plan is NULL");
    return nullptr;
  }
  if (which != BCA_TABLE_NORM && which != BCA_TABLE_APPLY && which != BCA_TABLE_LAMB) {
    fail(BCA_ERR_RANGE, "table must be BCA_TABLE_NORM, BCA_TABLE_APPLY or BCA_TABLE_LAMB");
    return nullptr;
  }
  return which == BCA_TABLE_NORM ? &p->norm_tab : which == BCA_TABLE_APPLY ? &p->apply_tab : &p->lamb_tab;
}

uint32_t bca_plan_num_chunks(const bca_plan* p, int which) {
  const Table* t = pick_table(p, which);
  return t ? (uint32_t)t->chunks.size() : 0;
}

uint32_t bca_plan_num_groups(const bca_plan* p) { return p ? (uint32_t)p->groups.size() : 0; }

uint32_t bca_plan_norm_item_chunks(const bca_plan* p) { return p ? p->norm_item_chunks : 0; }

uint32_t bca_plan_num_lamb_runs(const bca_plan* p) { return p ? (uint32_t)p->lamb_groups.size() : 0; }

int bca_plan_lamb_run(const bca_plan* p, uint32_t i, uint32_t* first_tensor, uint32_t* end_tensor) {
  if (!p) return fail(BCA_ERR_NULL, "plan is NULL");
  if (i >= p->lamb_groups.size()) return fail(BCA_ERR_RANGE, "run index out of range");
  if (first_tensor) *first_tensor = p->lamb_groups[i].first;
  if (end_tensor) *end_tensor = p->lamb_groups[i].second;
  return BCA_OK;
}

uint32_t bca_plan_num_work_items(const bca_plan* p) { return p ? (uint32_t)p->work.size() : 0; }

int bca_plan_work_item(const bca_plan* p, uint32_t i, uint32_t* kind, uint32_t* first, uint32_t* count) {
  if (!p) return fail(BCA_ERR_NULL, "plan is NULL");
  if (i >= p->work.size()) return fail(BCA_ERR_RANGE, "work item index out of range");
  const uint32_t item = p->work[i], k = item >> 30;
  if (kind) *kind = k;
  if (first) *first = k == kItemAdam ? (item & 0x3fffffffu) : (item & 0x0fffffffu);
  if (count) *count = k == kItemNorm ? ((item >> 28) & 3u) + 1u : k == kItemAdam ? 1u : 0u;
  return BCA_OK;
}

int bca_plan_chunk_info(const bca_plan* p, int which, uint32_t i, uint32_t* tensor, uint64_t* begin, uint32_t* len,
                        uint32_t* bucket) {
  const Table* t = pick_table(p, which);
  if (!t) return p ? BCA_ERR_RANGE : BCA_ERR_NULL;
  if (i >= t->chunks.size()) return fail(BCA_ERR_RANGE, "chunk index out of range");
  const ChunkInfo& c = t->chunks[i];
  if (tensor) *tensor = c.tensor;
  if (begin) *begin = c.begin;
  if (len) *len = c.len;
  if (bucket) *bucket = c.bucket;
  return BCA_OK;
}

int bca_plan_bucket_chunks(const bca_plan* p, int which, uint32_t b, uint32_t* first, uint32_t* count) {
  const Table* t = pick_table(p, which);
  if (!t) return p ? BCA_ERR_RANGE : BCA_ERR_NULL;
  const std::vector<uint32_t>& off = which == BCA_TABLE_LAMB ? p->tensor_off : t->bucket_off;
  if ((size_t)b + 1 >= off.size()) return fail(BCA_ERR_RANGE, "bucket (or tensor) index out of range");
  if (first) *first = off[b];
  if (count) *count = off[b + 1] - off[b];
  return BCA_OK;
}

// Events one profiled fused call records: one before the first kernel and one after each.
static size_t events_per_call(const bca_plan* p) {
  return (p->tune_flags & BCA_TUNE_MULTI_LAUNCH) ? 1 + 3 * p->groups.size() : 3;
}

int bca_plan_profile(bca_plan* p, uint32_t max_calls) {
  if (!p) return fail(BCA_ERR_NULL, "plan is NULL");
  if (p->device < 0) return fail(BCA_ERR_UNBOUND, "host-only plan");
  if (max_calls > 65536) return fail(BCA_ERR_RANGE, "at most 65536 profiled calls");
  DeviceGuard g(p->device);
  (void)hipDeviceSynchronize();
  free_profile(p);
  const size_t per_call = events_per_call(p);
  return no_throw([&] {
    p->prof_events.reserve(max_calls * per_call);
    for (size_t i = 0; i < max_calls * per_call; ++i) {
      hipEvent_t ev;
      hipError_t e = hipEventCreate(&ev);
      if (e != hipSuccess) {
        free_profile(p);
        return fail_hip(e, "hipEventCreate");
      }
      p->prof_events.push_back(ev);
    }
    return (int)BCA_OK;
  });
}

int bca_plan_profile_read(bca_plan* p, double* ms, uint32_t* n_calls) {
  if (!p || !ms || !n_calls) return fail(BCA_ERR_NULL, "NULL argument");
  ms[0] = ms[1] = ms[2] = 0.0;
  *n_calls = 0;
  if (p->device < 0) return fail(BCA_ERR_UNBOUND, "host-only plan");
  DeviceGuard g(p->device);
  const size_t per_call = events_per_call(p);
  for (uint32_t c = 0; c < p->prof_calls; ++c) {
    hipEvent_t* ev = &p->prof_events[(size_t)c * per_call];
    hipError_t e = hipEventSynchronize(ev[per_call - 1]);
    for (size_t k = 0; k + 1 < per_call && e == hipSuccess; ++k) {
      float t = 0.f;
      e = hipEventElapsedTime(&t, ev[k], ev[k + 1]);
      // multi-launch: squared norm, finalize, Adam in turn; single launch: the step kernel (ms[2]), then the
      // finish kernel (ms[0])
      ms[per_call == 3 ? (k == 0 ? 2 : 0) : k % 3] += t;
    }
    if (e != hipSuccess) return fail_hip(e, "reading profile events");
  }
  *n_calls = p->prof_calls;
  p->prof_calls = 0;
  return BCA_OK;
}

int bca_plan_wait_stats(bca_plan* p, uint64_t* out) {
  if (!p || !out) return fail(BCA_ERR_NULL, "NULL argument");
  out[0] = out[1] = 0;
  if (p->device < 0) return fail(BCA_ERR_UNBOUND, "host-only plan");
  DeviceGuard g(p->device);
  hipError_t e = hipDeviceSynchronize();
  return no_throw([&] {
    std::vector<uint32_t> words(32 * kStatSlots);
    if (e == hipSuccess) e = hipMemcpy(words.data(), p->d_ctl + kCtlStats, words.size() * sizeof(uint32_t), hipMemcpyDeviceToHost);
    if (e == hipSuccess) e = hipMemset(p->d_ctl + kCtlStats, 0, words.size() * sizeof(uint32_t));
    if (e != hipSuccess) return fail_hip(e, "reading the wait statistics");
    for (uint32_t sl = 0; sl < kStatSlots; ++sl) {
      out[0] += words[32 * sl];
      out[1] += (uint64_t)words[32 * sl + 2] | ((uint64_t)words[32 * sl + 3] << 32);
    }
    return (int)BCA_OK;
  });
}

int bca_copy_bytes(void* dst, const void* src, uint64_t nbytes, void* stream) {
  if (nbytes && (!dst || !src)) return fail(BCA_ERR_NULL, "NULL buffer");
  if (((uintptr_t)dst | (uintptr_t)src) & 15u) return fail(BCA_ERR_ALIGN, "buffers must be 16-byte aligned");
  hipError_t e = launch_copy(dst, src, nbytes, (hipStream_t)stream);
  if (e != hipSuccess) return fail_hip(e, "launching the copy kernel");
  return BCA_OK;
}

int bca_alg1_thresholds(double c, uint32_t n_buckets, float* out) {
  if (n_buckets && !out) return fail(BCA_ERR_NULL, "out is NULL");
  if (!(c > 0.0)) return fail(BCA_ERR_HPARAM, "the clipping threshold c must be positive");
  const float each = (float)(c / std::sqrt((double)n_buckets));
  for (uint32_t b = 0; b < n_buckets; ++b) out[b] = each;
  return BCA_OK;
}

int bucket_clip_norms(bca_plan* p, uint32_t b0, uint32_t b1, float* norms, void* stream) {
  if (!p) return fail(BCA_ERR_NULL, "plan is NULL");
  if (int rc = check_range(p, b0, b1)) return rc;
  if (!norms) return fail(BCA_ERR_NULL, "norms is NULL");
  if (int rc = check_ready(p)) return rc;
  if (b0 == b1) return BCA_OK;
  DeviceGuard g(p->device);
  hipStream_t s = (hipStream_t)stream;
  const Table& T = p->norm_tab;
  const uint32_t c0 = T.bucket_off[b0], n = T.bucket_off[b1] - c0;
  // Called per bucket as buckets become ready, bucket_clip_apply follows shortly: keep the gradients cacheable,
  // unless the range is too large to be found in the cache again.
  const bool keep = (uint64_t)n * T.chunk_elems * grad_bytes(p->grad_dtype) <= kKeepCachedBytes;
  hipError_t e = launch_sqnorm(p->grad_dtype, T.d_chunks, c0, n, p->d_partials, nullptr,
                               make_launch(p, norm_grid(p, n), n, keep), s);
  if (e != hipSuccess) return fail_hip(e, "launching the squared-norm kernel");
  e = launch_finalize(p->d_partials, T.d_bucket_off, b0, b1, nullptr, norms, nullptr, nullptr, nullptr, s);
  if (e != hipSuccess) return fail_hip(e, "launching the finalize kernel");
  return BCA_OK;
}

int bucket_clip_apply(bca_plan* p, uint32_t b0, uint32_t b1, const float* thresholds, const float* norms,
                      float* coefs, int32_t* status, void* stream) {
  if (!p) return fail(BCA_ERR_NULL, "plan is NULL");
  if (int rc = check_range(p, b0, b1)) return rc;
  if (!thresholds) return fail(BCA_ERR_NULL, "thresholds is NULL");
  if (!norms) return fail(BCA_ERR_NULL, "norms is NULL");
  if (int rc = check_ready(p)) return rc;
  DeviceGuard g(p->device);
  hipStream_t s = (hipStream_t)stream;
  float* cf = coefs ? coefs : p->d_coefs;
  hipError_t e = launch_coefs(b0, b1, thresholds, norms, cf, status, s);
  if (e != hipSuccess) return fail_hip(e, "launching the coefficient kernel");
  if (b0 == b1) return BCA_OK;
  const Table& T = p->apply_tab;
  const uint32_t c0 = T.bucket_off[b0], n = T.bucket_off[b1] - c0;
  e = launch_scale(p->grad_dtype, T.d_chunks, c0, n, cf, make_launch(p, p->grid_apply, n, true), s);
  if (e != hipSuccess) return fail_hip(e, "launching the scale kernel");
  return BCA_OK;
}

int bucket_clip(bca_plan* p, uint32_t b0, uint32_t b1, const float* thresholds, float* norms, float* coefs,
                int32_t* status, void* stream) {
  if (!p) return fail(BCA_ERR_NULL, "plan is NULL");
  if (int rc = check_range(p, b0, b1)) return rc;
  if (!thresholds) return fail(BCA_ERR_NULL, "thresholds is NULL");
  if (int rc = check_ready(p)) return rc;
  if (b0 == b1) return BCA_OK;
  DeviceGuard g(p->device);
  hipStream_t s = (hipStream_t)stream;
  const Table& TN = p->norm_tab;
  const uint32_t cn0 = TN.bucket_off[b0], nn = TN.bucket_off[b1] - cn0;
  float* nm = norms ? norms : p->d_norms;
  float* cf = coefs ? coefs : p->d_coefs;
  int32_t* st = status ? status : p->d_status;
  uint32_t most = 0;  // chunks of the range's largest bucket
  for (uint32_t b = b0; b < b1; ++b) most = std::max(most, TN.bucket_off[b + 1] - TN.bucket_off[b]);
  // First launch: the squared-norm partials of the range's chunks (one workgroup per chunk: a single bucket has
  // few of them); it also clears the status word.
  const bool keep = (uint64_t)nn * TN.chunk_elems * grad_bytes(p->grad_dtype) <= kKeepCachedBytes;
  hipError_t e = launch_sqnorm(p->grad_dtype, TN.d_chunks, cn0, nn, p->d_partials, st, make_launch(p, 0, nn, keep), s);
  if (e != hipSuccess) return fail_hip(e, "launching the squared-norm kernel");
  if (most <= kMaxChunksForInlineFinalize && !(p->tune_flags & BCA_TUNE_MULTI_LAUNCH)) {
    // Second launch: one workgroup per chunk derives the bucket's coefficient from the partials and scales the chunk.
    e = launch_clip_scale(p->grad_dtype, TN.d_chunks, cn0, nn, TN.d_bucket_off, b0, b1, p->d_partials, thresholds, nm, cf,
                          st, s);
    if (e != hipSuccess) return fail_hip(e, "launching the clip kernel");
    return BCA_OK;
  }
  // Very large buckets: the finalize and scale kernels of bucket_clip_norms / bucket_clip_apply instead.
  e = launch_finalize(p->d_partials, TN.d_bucket_off, b0, b1, thresholds, nm, cf, st, nullptr, s);
  if (e != hipSuccess) return fail_hip(e, "launching the finalize kernel");
  const Table& TA = p->apply_tab;
  const uint32_t ca0 = TA.bucket_off[b0], na = TA.bucket_off[b1] - ca0;
  e = launch_scale(p->grad_dtype, TA.d_chunks, ca0, na, cf, make_launch(p, p->grid_apply, na, true), s);
  if (e != hipSuccess) return fail_hip(e, "launching the scale kernel");
  return BCA_OK;
}

int bucket_clip_flat(void* g, uint64_t n, int grad_dtype, const float* threshold, float* norm, float* coef,
                     int32_t* status, void* stream) {
  if (grad_dtype != BCA_GRAD_F32 && grad_dtype != BCA_GRAD_F16 && grad_dtype != BCA_GRAD_BF16)
    return fail(BCA_ERR_DTYPE, "unknown gradient type");
  if (n > kFlatMaxElems) {
    char buf[128];
    snprintf(buf, sizeof buf, "bucket_clip_flat handles at most %llu elements per call (got %llu)",
             (unsigned long long)kFlatMaxElems, (unsigned long long)n);
    return fail(BCA_ERR_RANGE, buf);
  }
  if (n && !g) return fail(BCA_ERR_NULL, "g is NULL");
  if (!threshold) return fail(BCA_ERR_NULL, "threshold is NULL");
  if ((uintptr_t)g % grad_bytes(grad_dtype)) return fail(BCA_ERR_ALIGN, "g is not aligned to its element size");
  int device = -1;
  hipError_t e = hipGetDevice(&device);
  if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
  if (device < 0 || device >= kFlatMaxDevices) return fail(BCA_ERR_RANGE, "device index beyond what bucket_clip_flat keeps scratch for");
  e = launch_clip_flat(device, grad_dtype, g, n, threshold, norm, coef, status, (hipStream_t)stream);
  if (e != hipSuccess) return fail_hip(e, "bucket_clip_flat");
  return BCA_OK;
}

int adam_step(bca_plan* p, const bca_adam* hp, uint64_t step, void* stream) {
  if (!p) return fail(BCA_ERR_NULL, "plan is NULL");
  AdamK k;
  if (int rc = make_adam_constants(p, hp, step, &k)) return rc;
  if (int rc = check_ready(p)) return rc;
  DeviceGuard g(p->device);
  if (int rc = enqueue_hyper(p, (hipStream_t)stream)) return rc;
  const Table& T = p->apply_tab;
  const uint32_t n = (uint32_t)T.chunks.size();
  hipError_t e = launch_adam(p->grad_dtype, T.d_chunks, 0, n, nullptr, false, nullptr, k,
                             make_launch(p, p->grid_apply, n, false), (hipStream_t)stream);
  if (e != hipSuccess) return fail_hip(e, "launching the Adam kernel");
  return BCA_OK;
}

int bucket_clip_adam(bca_plan* p, const float* thresholds, const bca_adam* hp, uint64_t step, uint32_t flags,
                     float* norms, float* coefs, int32_t* status, void* stream) {
  if (!p) return fail(BCA_ERR_NULL, "plan is NULL");
  if (!thresholds) return fail(BCA_ERR_NULL, "thresholds is NULL");
  if (flags & ~(BCA_WRITE_BACK_GRADS | BCA_SKIP_STEP_ON_NONFINITE | BCA_CLIP_WHOLE_GRADIENT))
    return fail(BCA_ERR_RANGE, "unknown flag bits");
  AdamK k;
  if (int rc = make_adam_constants(p, hp, step, &k)) return rc;
  if (int rc = check_ready(p)) return rc;
  const bool whole = (flags & BCA_CLIP_WHOLE_GRADIENT) != 0;
  const bool skip = (flags & BCA_SKIP_STEP_ON_NONFINITE) != 0 || whole;  // both need every norm before any update
  const bool multi = (p->tune_flags & BCA_TUNE_MULTI_LAUNCH) != 0;
  DeviceGuard g(p->device);
  hipStream_t s = (hipStream_t)stream;
  if (int rc = enqueue_hyper(p, s)) return rc;
  float* nm = norms ? norms : p->d_norms;
  float* cf = coefs ? coefs : p->d_coefs;
  int32_t* st = status ? status : p->d_status;
  const size_t per_call = events_per_call(p);
  // events of this call when profiling has room left; a call that needs every norm first runs as one
  // group whatever the plan's groups are, so it does not fit the per-group event layout: not profiled
  hipEvent_t* ev = nullptr;
  if (!skip && (size_t)(p->prof_calls + 1) * per_call <= p->prof_events.size())
    ev = &p->prof_events[(size_t)p->prof_calls++ * per_call];

  if (!multi && !skip) {
    // One launch for the whole step (plus the small finish kernel behind it).
    const StepState ss = step_state(p);
    if (ev) (void)hipEventRecord(ev[0], s);
    hipError_t e = launch_step(p->grad_dtype, ss, p->d_work, (uint32_t)p->work.size(), thresholds, nm, cf,
                               st, (flags & BCA_WRITE_BACK_GRADS) != 0, k, p->unroll_apply,
                               (p->tune_flags & BCA_TUNE_TICKETS) != 0, false, ev ? ev[1] : nullptr, s);
    if (e != hipSuccess) return fail_hip(e, "launching the fused step kernel");
    if (ev) (void)hipEventRecord(ev[2], s);
    return BCA_OK;
  }

  // Several launches.  The skip decision covers all buckets, so that mode takes one
  // group: all norms first, then one Adam sweep that checks the status word.
  const std::pair<uint32_t, uint32_t> all_buckets(0u, p->n_buckets);
  const std::pair<uint32_t, uint32_t>* groups = skip ? &all_buckets : p->groups.data();
  const size_t n_groups = skip ? 1 : p->groups.size();
  if (ev) (void)hipEventRecord(*ev++, s);
  // With groups, a group's gradients are read twice in quick succession (norm,
  // then Adam) and are kept cacheable; everything else streams.
  const bool keep = n_groups > 1;
  bool first = true;
  for (size_t gi = 0; gi < n_groups; ++gi) {
    const uint32_t b0 = groups[gi].first, b1 = groups[gi].second;
    const Table& TN = p->norm_tab;
    const Table& TA = p->apply_tab;
    const uint32_t cn0 = TN.bucket_off[b0], nn = TN.bucket_off[b1] - cn0;
    const uint32_t ca0 = TA.bucket_off[b0], na = TA.bucket_off[b1] - ca0;
    // the first squared-norm launch of a call also clears the status word
    hipError_t e = launch_sqnorm(p->grad_dtype, TN.d_chunks, cn0, nn, p->d_partials, first ? st : nullptr,
                                 make_launch(p, norm_grid(p, nn), nn, keep), s);
    if (e != hipSuccess) return fail_hip(e, "launching the squared-norm kernel");
    if (ev) (void)hipEventRecord(*ev++, s);
    e = launch_finalize(p->d_partials, TN.d_bucket_off, b0, b1, whole ? nullptr : thresholds, nm, cf, st,
                        whole ? p->d_bucket_sq : nullptr, s);
    if (e == hipSuccess && whole)
      e = launch_whole_coef(p->d_bucket_sq, p->n_buckets, thresholds, nm + p->n_buckets, cf, st, s);
    if (e != hipSuccess) return fail_hip(e, "launching the finalize kernel");
    if (ev) (void)hipEventRecord(*ev++, s);
    e = launch_adam(p->grad_dtype, TA.d_chunks, ca0, na, cf, (flags & BCA_WRITE_BACK_GRADS) != 0,
                    (flags & BCA_SKIP_STEP_ON_NONFINITE) ? st : nullptr,
                    k, make_launch(p, p->grid_apply, na, keep), s);
    if (e != hipSuccess) return fail_hip(e, "launching the Adam kernel");
    if (ev) (void)hipEventRecord(*ev++, s);
    first = false;
  }
  return BCA_OK;
}

// LAMB, with (thresholds != nullptr) or without bucket-wise clipping in front.
static int lamb_impl(bca_plan* p, const float* thresholds, const bca_adam* hp, uint64_t step, uint32_t flags,
                     float* norms, float* coefs, float* trust, int32_t* status, hipStream_t s) {
  AdamK k;
  if (int rc = make_adam_constants(p, hp, step, &k)) return rc;
  if (int rc = check_ready(p)) return rc;
  DeviceGuard g(p->device);
  if (int rc = enqueue_hyper(p, s)) return rc;
  const Table& TL = p->lamb_tab;
  const uint32_t nl = (uint32_t)TL.chunks.size();
  hipError_t e = hipSuccess;
  if (thresholds) {
    float* nm = norms ? norms : p->d_norms;
    float* cw = coefs ? coefs : p->d_coefs;
    int32_t* st = status ? status : p->d_status;
    if (!(p->tune_flags & BCA_TUNE_MULTI_LAUNCH)) {
      // squared norms, coefficients and LAMB's first sweep as one pipelined launch (the fused Adam step's
      // work list and waiting scheme; the first sweep's second read of the gradients is served from cache)
      e = launch_step(p->grad_dtype, step_state(p), p->d_work, (uint32_t)p->work.size(), thresholds, nm, cw,
                      st, (flags & BCA_WRITE_BACK_GRADS) != 0, k, 1, false, true, nullptr, s);
      if (e != hipSuccess) return fail_hip(e, "launching the fused clip + LAMB moments kernel");
    } else {
      const Table& TN = p->norm_tab;
      const uint32_t nn = (uint32_t)TN.chunks.size();
      e = launch_sqnorm(p->grad_dtype, TN.d_chunks, 0, nn, p->d_partials, st, make_launch(p, norm_grid(p, nn), nn, false), s);
      if (e != hipSuccess) return fail_hip(e, "launching the squared-norm kernel");
      e = launch_finalize(p->d_partials, TN.d_bucket_off, 0, p->n_buckets, thresholds, nm, cw, st, nullptr, s);
      if (e != hipSuccess) return fail_hip(e, "launching the finalize kernel");
      e = launch_lamb_moments(p->grad_dtype, TL.d_chunks, nl, cw, (flags & BCA_WRITE_BACK_GRADS) != 0, p->d_lamb_sums, false, k, s);
      if (e != hipSuccess) return fail_hip(e, "launching the LAMB moments kernel");
    }
  } else {
    // Run by run: first sweep, trust ratios, second sweep.  With several runs the first sweep stores the moments with
    // cacheable stores, so that the second sweep, which follows at once, finds them in cache (measured, BERT-Large:
    // 2.05 instead of 2.18 ms; runs with streaming stores 2.21, cacheable stores without runs 2.34).
    float* tr = trust ? trust : p->d_trust;
    const bool keep = p->lamb_groups.size() > 1;
    for (const auto& gr : p->lamb_groups) {
      const uint32_t c0 = p->tensor_off[gr.first], n = p->tensor_off[gr.second] - c0;
      e = launch_lamb_moments(p->grad_dtype, TL.d_chunks + c0, n, nullptr, false, p->d_lamb_sums + (uint64_t)c0 * 2u, keep, k, s);
      if (e != hipSuccess) return fail_hip(e, "launching the LAMB moments kernel");
      e = launch_lamb_trust(p->d_lamb_sums, p->d_tensor_off + gr.first, gr.second - gr.first, k, tr + gr.first,
                            p->d_lamb_scale + gr.first, s);
      if (e != hipSuccess) return fail_hip(e, "launching the LAMB trust-ratio kernel");
      e = launch_lamb_update(TL.d_chunks + c0, n, p->d_lamb_scale, k, s);
      if (e != hipSuccess) return fail_hip(e, "launching the LAMB update kernel");
    }
    return BCA_OK;
  }
  e = launch_lamb_trust(p->d_lamb_sums, p->d_tensor_off, p->n_tensors, k, trust ? trust : p->d_trust,
                        p->d_lamb_scale, s);
  if (e != hipSuccess) return fail_hip(e, "launching the LAMB trust-ratio kernel");
  e = launch_lamb_update(TL.d_chunks, nl, p->d_lamb_scale, k, s);
  if (e != hipSuccess) return fail_hip(e, "launching the LAMB update kernel");
  return BCA_OK;
}

int lamb_step(bca_plan* p, const bca_adam* hp, uint64_t step, float* trust, void* stream) {
  if (!p) return fail(BCA_ERR_NULL, "plan is NULL");
  return lamb_impl(p, nullptr, hp, step, 0, nullptr, nullptr, trust, nullptr, (hipStream_t)stream);
}

int bucket_clip_lamb(bca_plan* p, const float* thresholds, const bca_adam* hp, uint64_t step, uint32_t flags,
                     float* norms, float* coefs, float* trust, int32_t* status, void* stream) {
  if (!p) return fail(BCA_ERR_NULL, "plan is NULL");
  if (!thresholds) return fail(BCA_ERR_NULL, "thresholds is NULL");
  if (flags & ~BCA_WRITE_BACK_GRADS) return fail(BCA_ERR_RANGE, "bucket_clip_lamb knows BCA_WRITE_BACK_GRADS only");
  return lamb_impl(p, thresholds, hp, step, flags, norms, coefs, trust, status, (hipStream_t)stream);
}

}  // extern "C"

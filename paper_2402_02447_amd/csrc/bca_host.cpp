// Host side of libbca: plan construction (layout validation, chunk table),
// binding, argument checks and the four compute entry points.  See bca.h for
// the contract of every call.

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
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
void build_chunks(bca_plan* p, const uint64_t* seg_off, const bca_segment* segs) {
  const uint64_t C = p->chunk_elems;
  p->chunks.clear();
  p->bucket_chunk_off.assign(p->n_buckets + 1, 0);
  for (uint32_t b = 0; b < p->n_buckets; ++b) {
    p->bucket_chunk_off[b] = (uint32_t)p->chunks.size();
    for (uint64_t s = seg_off[b]; s < seg_off[b + 1]; ++s) {
      uint64_t pos = segs[s].begin;
      const uint64_t end = segs[s].begin + segs[s].len;
      while (pos < end) {
        const uint64_t stop = std::min(end, (pos / C + 1) * C);
        p->chunks.push_back(ChunkInfo{segs[s].tensor, (uint32_t)(stop - pos), pos, b});
        pos = stop;
      }
    }
  }
  p->bucket_chunk_off[p->n_buckets] = (uint32_t)p->chunks.size();
}

void free_device(bca_plan* p) {
  if (p->device < 0) return;
  DeviceGuard g(p->device);
  if (p->d_table) (void)hipFree(p->d_table);
  if (p->d_partials) (void)hipFree(p->d_partials);
  if (p->d_bucket_chunk_off) (void)hipFree(p->d_bucket_chunk_off);
  if (p->d_norms) (void)hipFree(p->d_norms);
  if (p->d_coefs) (void)hipFree(p->d_coefs);
  if (p->d_status) (void)hipFree(p->d_status);
  p->d_table = nullptr, p->d_partials = nullptr, p->d_bucket_chunk_off = nullptr;
  p->d_norms = nullptr, p->d_coefs = nullptr, p->d_status = nullptr;
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

int make_adam_constants(const bca_adam* hp, uint64_t step, AdamK* k) {
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
  return BCA_OK;
}

uint32_t pick_grid(uint32_t requested, uint32_t fallback, uint32_t n_chunks) {
  uint32_t g = requested ? requested : fallback;
  g = std::min(g, n_chunks);
  return std::max(g, 1u);
}

}  // namespace
}  // namespace bca

using namespace bca;

extern "C" {

int bca_version(void) { return 1; }

const char* bca_last_error(void) { return g_last_error.c_str(); }

int bca_plan_create(bca_plan** out, int device, uint32_t n_tensors, const uint64_t* tensor_numel, uint32_t n_buckets,
                    const uint64_t* bucket_seg_off, const bca_segment* segments, int grad_dtype,
                    const bca_tuning* tuning) {
  if (!out) return fail(BCA_ERR_NULL, "out is NULL");
  *out = nullptr;
  if (!bucket_seg_off) return fail(BCA_ERR_NULL, "bucket_seg_off is NULL");
  if (n_tensors && !tensor_numel) return fail(BCA_ERR_NULL, "tensor_numel is NULL");
  if (n_buckets == 0) return fail(BCA_ERR_LAYOUT, "a plan needs at least one bucket");
  if (grad_dtype != BCA_GRAD_F32 && grad_dtype != BCA_GRAD_F16) return fail(BCA_ERR_DTYPE, "unknown gradient type");
  if (bucket_seg_off[n_buckets] && !segments) return fail(BCA_ERR_NULL, "segments is NULL");
  if (device < -1) return fail(BCA_ERR_RANGE, "device must be >= 0, or -1 for a host-only plan");
  uint32_t chunk = kDefaultChunk;
  if (tuning && tuning->chunk_elems) {
    if (tuning->chunk_elems % 1024u || tuning->chunk_elems > (1u << 24))
      return fail(BCA_ERR_RANGE, "chunk_elems must be a multiple of 1024 and at most 2^24");
    chunk = tuning->chunk_elems;
  }
  if (int rc = validate_layout(n_tensors, tensor_numel, n_buckets, bucket_seg_off, segments)) return rc;

  bca_plan* p = new (std::nothrow) bca_plan;
  if (!p) return fail(BCA_ERR_HIP, "out of host memory");
  p->device = device;
  p->grad_dtype = grad_dtype;
  p->n_tensors = n_tensors;
  p->n_buckets = n_buckets;
  p->chunk_elems = chunk;
  p->grid_norm = tuning ? tuning->grid_norm : 0;
  p->grid_apply = tuning ? tuning->grid_apply : 0;
  p->tensor_numel.assign(tensor_numel, tensor_numel + n_tensors);
  build_chunks(p, bucket_seg_off, segments);
  if (p->chunks.size() >= (1ull << 31)) {
    delete p;
    return fail(BCA_ERR_RANGE, "too many chunks; raise chunk_elems");
  }

  if (device >= 0) {
    int n_dev = 0;
    hipError_t e = hipGetDeviceCount(&n_dev);
    if (e != hipSuccess || device >= n_dev) {
      delete p;
      return e != hipSuccess ? fail_hip(e, "hipGetDeviceCount") : fail(BCA_ERR_RANGE, "no such device");
    }
    DeviceGuard g(device);
    if (!g.ok) {
      delete p;
      return fail(BCA_ERR_HIP, "hipSetDevice failed");
    }
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, device);
    if (e != hipSuccess) {
      delete p;
      return fail_hip(e, "hipGetDeviceProperties");
    }
    const uint32_t cus = (uint32_t)std::max(prop.multiProcessorCount, 1);
    if (!p->grid_norm) p->grid_norm = cus * 8;
    if (!p->grid_apply) p->grid_apply = cus * 8;
    const size_t nc = std::max<size_t>(p->chunks.size(), 1);
    const size_t nb = n_buckets;
    if ((e = hipMalloc((void**)&p->d_table, nc * sizeof(Chunk))) != hipSuccess ||
        (e = hipMalloc((void**)&p->d_partials, nc * sizeof(double))) != hipSuccess ||
        (e = hipMalloc((void**)&p->d_bucket_chunk_off, (nb + 1) * sizeof(uint32_t))) != hipSuccess ||
        (e = hipMalloc((void**)&p->d_norms, nb * sizeof(float))) != hipSuccess ||
        (e = hipMalloc((void**)&p->d_coefs, nb * sizeof(float))) != hipSuccess ||
        (e = hipMalloc((void**)&p->d_status, sizeof(int32_t))) != hipSuccess ||
        (e = hipMemcpy(p->d_bucket_chunk_off, p->bucket_chunk_off.data(), (nb + 1) * sizeof(uint32_t),
                       hipMemcpyHostToDevice)) != hipSuccess ||
        (e = hipMemset(p->d_status, 0, sizeof(int32_t))) != hipSuccess) {
      free_device(p);
      delete p;
      return fail_hip(e, "allocating plan memory");
    }
  }
  *out = p;
  return BCA_OK;
}

int bca_plan_bind(bca_plan* p, void* const* grads, float* const* params, float* const* exp_avg,
                  float* const* exp_avg_sq) {
  if (!p) return fail(BCA_ERR_NULL, "plan is NULL");
  if (p->device < 0) return fail(BCA_ERR_UNBOUND, "host-only plan (device -1) cannot be bound");
  if (p->n_tensors && (!grads || !params || !exp_avg || !exp_avg_sq)) return fail(BCA_ERR_NULL, "a pointer array is NULL");
  const uint64_t gsize = p->grad_dtype == BCA_GRAD_F16 ? 2 : 4;
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
  std::vector<Chunk> table(std::max<size_t>(p->chunks.size(), 1));
  memset(table.data(), 0, table.size() * sizeof(Chunk));
  for (size_t i = 0; i < p->chunks.size(); ++i) {
    const ChunkInfo& c = p->chunks[i];
    table[i].g = (uint64_t)(uintptr_t)grads[c.tensor] + c.begin * gsize;
    table[i].p = (uint64_t)(uintptr_t)params[c.tensor] + c.begin * 4;
    table[i].m = (uint64_t)(uintptr_t)exp_avg[c.tensor] + c.begin * 4;
    table[i].v = (uint64_t)(uintptr_t)exp_avg_sq[c.tensor] + c.begin * 4;
    table[i].len = c.len;
    table[i].bucket = c.bucket;
  }
  DeviceGuard g(p->device);
  // The copy is synchronous with respect to the host; kernels enqueued earlier
  // on any stream may still be reading the old table, so wait for them first.
  hipError_t e = hipDeviceSynchronize();
  if (e == hipSuccess) e = hipMemcpy(p->d_table, table.data(), table.size() * sizeof(Chunk), hipMemcpyHostToDevice);
  if (e != hipSuccess) return fail_hip(e, "uploading the chunk table");
  p->bound = true;
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
uint32_t bca_plan_num_chunks(const bca_plan* p) { return p ? (uint32_t)p->chunks.size() : 0; }

int bca_plan_chunk_info(const bca_plan* p, uint32_t i, uint32_t* tensor, uint64_t* begin, uint32_t* len,
                        uint32_t* bucket) {
  if (!p) return fail(BCA_ERR_NULL, "plan is NULL");
  if (i >= p->chunks.size()) return fail(BCA_ERR_RANGE, "chunk index out of range");
  const ChunkInfo& c = p->chunks[i];
  if (tensor) *tensor = c.tensor;
  if (begin) *begin = c.begin;
  if (len) *len = c.len;
  if (bucket) *bucket = c.bucket;
  return BCA_OK;
}

int bca_plan_bucket_chunks(const bca_plan* p, uint32_t b, uint32_t* first, uint32_t* count) {
  if (!p) return fail(BCA_ERR_NULL, "plan is NULL");
  if (b >= p->n_buckets) return fail(BCA_ERR_RANGE, "bucket index out of range");
  if (first) *first = p->bucket_chunk_off[b];
  if (count) *count = p->bucket_chunk_off[b + 1] - p->bucket_chunk_off[b];
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
  const uint32_t c0 = p->bucket_chunk_off[b0], n = p->bucket_chunk_off[b1] - c0;
  hipError_t e = launch_sqnorm(p->grad_dtype, p->d_table, c0, n, p->d_partials, nullptr,
                               pick_grid(p->grid_norm, 2048, n), s);
  if (e != hipSuccess) return fail_hip(e, "launching the squared-norm kernel");
  e = launch_finalize(p->d_partials, p->d_bucket_chunk_off, b0, b1, nullptr, norms, nullptr, nullptr, s);
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
  const uint32_t c0 = p->bucket_chunk_off[b0], n = p->bucket_chunk_off[b1] - c0;
  e = launch_scale(p->grad_dtype, p->d_table, c0, n, cf, pick_grid(p->grid_apply, 2048, n), s);
  if (e != hipSuccess) return fail_hip(e, "launching the scale kernel");
  return BCA_OK;
}

int adam_step(bca_plan* p, const bca_adam* hp, uint64_t step, void* stream) {
  if (!p) return fail(BCA_ERR_NULL, "plan is NULL");
  AdamK k;
  if (int rc = make_adam_constants(hp, step, &k)) return rc;
  if (int rc = check_ready(p)) return rc;
  DeviceGuard g(p->device);
  const uint32_t n = (uint32_t)p->chunks.size();
  hipError_t e = launch_adam(p->grad_dtype, p->d_table, 0, n, nullptr, false, nullptr, k,
                             pick_grid(p->grid_apply, 2048, n), (hipStream_t)stream);
  if (e != hipSuccess) return fail_hip(e, "launching the Adam kernel");
  return BCA_OK;
}

int bucket_clip_adam(bca_plan* p, const float* thresholds, const bca_adam* hp, uint64_t step, uint32_t flags,
                     float* norms, float* coefs, int32_t* status, void* stream) {
  if (!p) return fail(BCA_ERR_NULL, "plan is NULL");
  if (!thresholds) return fail(BCA_ERR_NULL, "thresholds is NULL");
  if (flags & ~(BCA_WRITE_BACK_GRADS | BCA_SKIP_STEP_ON_NONFINITE)) return fail(BCA_ERR_RANGE, "unknown flag bits");
  AdamK k;
  if (int rc = make_adam_constants(hp, step, &k)) return rc;
  if (int rc = check_ready(p)) return rc;
  DeviceGuard g(p->device);
  hipStream_t s = (hipStream_t)stream;
  const uint32_t n = (uint32_t)p->chunks.size();
  float* nm = norms ? norms : p->d_norms;
  float* cf = coefs ? coefs : p->d_coefs;
  int32_t* st = status ? status : p->d_status;
  hipError_t e = launch_sqnorm(p->grad_dtype, p->d_table, 0, n, p->d_partials, st, pick_grid(p->grid_norm, 2048, n), s);
  if (e != hipSuccess) return fail_hip(e, "launching the squared-norm kernel");
  e = launch_finalize(p->d_partials, p->d_bucket_chunk_off, 0, p->n_buckets, thresholds, nm, cf, st, s);
  if (e != hipSuccess) return fail_hip(e, "launching the finalize kernel");
  e = launch_adam(p->grad_dtype, p->d_table, 0, n, cf, (flags & BCA_WRITE_BACK_GRADS) != 0,
                  (flags & BCA_SKIP_STEP_ON_NONFINITE) ? st : nullptr, k, pick_grid(p->grid_apply, 2048, n), s);
  if (e != hipSuccess) return fail_hip(e, "launching the Adam kernel");
  return BCA_OK;
}

}  // extern "C"

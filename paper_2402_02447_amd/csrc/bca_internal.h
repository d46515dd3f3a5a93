// Internal declarations shared by the host side (plan, argument checks) and the
// kernel launchers of libbca.  Not part of the public ABI.
#ifndef BCA_INTERNAL_H_
#define BCA_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "bca.h"

namespace bca {

// One unit of work: at most chunk_elems consecutive elements of one tensor, all
// in one bucket.  Chunks are stored bucket by bucket, so chunk index == slot of
// that chunk's partial sum, and a bucket's partials are contiguous.  The four
// addresses are filled in by bca_plan_bind.
struct alignas(16) Chunk {
  uint64_t g, p, m, v;  // device byte addresses of the chunk's first element
  uint32_t len;         // elements
  uint32_t bucket;
  uint32_t pad0, pad1;
};
static_assert(sizeof(Chunk) == 48, "chunk table entries are 3 x 16 bytes");

struct ChunkInfo {  // host-side description, independent of addresses
  uint32_t tensor;
  uint32_t len;
  uint64_t begin;
  uint32_t bucket;
};

// Adam constants, computed in fp64 on the host and rounded once to fp32.
struct AdamK {
  float b1, omb1;    // beta1, 1 - beta1
  float b2, omb2;    // beta2, 1 - beta2
  float rbc1, rbc2;  // 1 / (1 - beta1^t), 1 / (1 - beta2^t)
  float eps;
  float neg_lr;  // -lr
  float wd;
};

constexpr uint32_t kBlock = 256;          // threads per workgroup (4 wavefronts)
constexpr uint32_t kWaves = kBlock / 64;  // wavefronts per workgroup
constexpr uint32_t kSlice = 64;           // chunk-table entries staged in LDS at a time
constexpr uint32_t kDefaultChunk = 16384;

// Kernel launchers (bca_kernels.hip).  All enqueue on `stream` and return the
// launch's hipError_t.  c0/n: first chunk and number of chunks.
hipError_t launch_sqnorm(int gdt, const Chunk* table, uint32_t c0, uint32_t n, double* partials, int32_t* status,
                         uint32_t grid, hipStream_t stream);
// norms/coefs/status may alias plan scratch.  thresholds == nullptr: norms only.
hipError_t launch_finalize(const double* partials, const uint32_t* bucket_chunk_off, uint32_t b0, uint32_t b1,
                           const float* thresholds, float* norms, float* coefs, int32_t* status,
                           hipStream_t stream);
hipError_t launch_coefs(uint32_t b0, uint32_t b1, const float* thresholds, const float* norms, float* coefs,
                        int32_t* status, hipStream_t stream);
hipError_t launch_zero_status(int32_t* status, hipStream_t stream);
hipError_t launch_scale(int gdt, const Chunk* table, uint32_t c0, uint32_t n, const float* coefs, uint32_t grid,
                        hipStream_t stream);
// coefs == nullptr: plain Adam on the stored gradient.  skip_status != nullptr:
// the kernel returns at once if (*skip_status & BCA_STATUS_NONFINITE).
hipError_t launch_adam(int gdt, const Chunk* table, uint32_t c0, uint32_t n, const float* coefs, bool write_back,
                       const int32_t* skip_status, const AdamK& k, uint32_t grid, hipStream_t stream);

void set_error(const std::string& msg);

}  // namespace bca

struct bca_plan {
  int device = -1;  // -1: host-only
  int grad_dtype = BCA_GRAD_F32;
  uint32_t n_tensors = 0, n_buckets = 0;
  uint32_t chunk_elems = bca::kDefaultChunk;
  uint32_t grid_norm = 0, grid_apply = 0;
  bool bound = false;
  std::vector<uint64_t> tensor_numel;
  std::vector<bca::ChunkInfo> chunks;        // bucket-major
  std::vector<uint32_t> bucket_chunk_off;    // [n_buckets + 1]
  // device memory owned by the plan
  bca::Chunk* d_table = nullptr;
  double* d_partials = nullptr;
  uint32_t* d_bucket_chunk_off = nullptr;
  float* d_norms = nullptr;
  float* d_coefs = nullptr;
  int32_t* d_status = nullptr;
};

#endif  // BCA_INTERNAL_H_

// HIP kernels for gfx950 (MI355X): squared-norm partials, per-bucket finalize,
// in-place scale, the two launches of the per-bucket clip (with and without a plan),
// the (optionally clip-fused) Adam sweep, the whole fused step as one pipelined
// launch with its finish kernel, and LAMB's two sweeps.  Gradients are fp32, fp16 or bf16.
//
// All streaming kernels are table driven: the host cuts the bucket layout into
// chunks (<= chunk_elems consecutive elements of one tensor in one bucket,
// bca_internal.h) and workgroup w of a grid of G walks chunks c0+w, c0+w+G, ...
// Neighbouring workgroups therefore stream through neighbouring memory at the
// same time, and which workgroup handles a chunk never changes a result: a
// chunk's partial sums depend only on the chunk.  Two ways to fetch the table
// are compiled (STAGED): a persistent grid that copies its share of entries
// into LDS in slices, or uniform (scalar) loads of one entry per iteration,
// which is what a grid of one workgroup per chunk uses.
//
// Memory access: 128-bit loads/stores, lane-contiguous (a wavefront touches
// 1 KiB per instruction per array), several independent loads in flight per
// lane before first use, streaming (non-temporal) hints on data touched once.
// A chunk whose arrays are not mutually 16-byte congruent falls back to
// element-wise access.  No MFMA: nothing here is a contraction; the path is
// bound by HBM bandwidth.
//
// Arithmetic follows the paper's definitions: clipping-by-norm (Sec. 2.3)
// applied per bucket (Sec. 4.2, Alg. 1) and Adam (Alg. 1, last line; Kingma &
// Ba with bias correction, decoupled weight decay).  Every fp32 operation is
// written as an explicit multiply or fma so that the fused and the unfused
// paths produce the same bits.

#include <hip/hip_runtime.h>

#include <algorithm>
#include <mutex>
#include <type_traits>

#include "bca_internal.h"

namespace bca {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short u16x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));

// ---- streaming accesses ---------------------------------------------------------
// NT = non-temporal: data that is touched once per launch is loaded and stored
// with the streaming hint, which raises HBM throughput on gfx950 and keeps such
// lines from displacing reusable ones in L2 / Infinity Cache.
//
// Tensor addresses come out of the chunk table as integers, so the compiler cannot tell that they are global
// memory and would emit flat accesses; those may complete out of order, which forces a full wait
// (vmcnt(0) lgkmcnt(0)) before the first use of any of them and leaves only two or three of a batch of
// loads in flight.  Every access to tensor memory therefore goes through a pointer that is explicitly in the
// global address space: global_load / global_store, counted waits, all loads of a batch in flight.
// loads_issued(): nothing is scheduled across this point, so a batch of loads written before it is issued as a
// whole before the first instruction that uses one of them (left to itself the scheduler interleaves loads and
// uses in pairs, which leaves two loads in flight where eight or sixteen were meant).
__device__ __forceinline__ void loads_issued() { __builtin_amdgcn_sched_barrier(0); }
#define BCA_GLOBAL __attribute__((address_space(1)))
template <typename T>
__device__ __forceinline__ BCA_GLOBAL T* as_global(T* p) {
  return (BCA_GLOBAL T*)p;
}
template <bool NT, typename T>
__device__ __forceinline__ T ldv(const T* p) {
  if constexpr (NT) return __builtin_nontemporal_load(as_global(p));
  else return *as_global(p);
}
template <bool NT, typename T>
__device__ __forceinline__ void stv(T* p, T x) {
  if constexpr (NT) __builtin_nontemporal_store(x, as_global(p));
  else *as_global(p) = x;
}

// ---- chunk table access -----------------------------------------------------------

struct Entry {  // one chunk, in registers (uniform across the workgroup)
  uint64_t g, p, m, v;
  uint32_t len, bucket, tensor, flags;
};

__device__ __forceinline__ Entry read_entry(const Chunk* e) {
  Entry r;
  r.g = e->g, r.p = e->p, r.m = e->m, r.v = e->v, r.len = e->len, r.bucket = e->bucket;
  r.tensor = e->tensor, r.flags = e->flags;
  return r;
}

// Number of chunks workgroup w of G owns out of n under interleaved assignment.
__device__ __forceinline__ uint32_t my_chunk_count(uint32_t n, uint32_t w, uint32_t G) {
  return n > w ? (n - w + G - 1) / G : 0u;
}

// Copy entries  table[c0 + w + (first + e) * G], e in [0, cnt)  into LDS.
__device__ __forceinline__ void stage_slice(Chunk* s_tab, const Chunk* table, uint32_t c0, uint32_t w, uint32_t G,
                                            uint32_t first, uint32_t cnt) {
  const uint4* src = reinterpret_cast<const uint4*>(table);
  uint4* dst = reinterpret_cast<uint4*>(s_tab);
  for (uint32_t q = threadIdx.x; q < cnt * 3u; q += kBlock) {
    const uint32_t e = q / 3u, piece = q - e * 3u;
    const uint64_t ci = (uint64_t)c0 + w + (uint64_t)(first + e) * G;
    dst[q] = src[ci * 3u + piece];
  }
}

// Calls body(entry, chunk_index) for every chunk of this workgroup.
template <bool STAGED, typename F>
__device__ __forceinline__ void for_each_chunk(const Chunk* __restrict__ table, uint32_t c0, uint32_t n, F body) {
  const uint32_t w = blockIdx.x, Gn = gridDim.x;
  if constexpr (STAGED) {
    __shared__ Chunk s_tab[kSlice];
    const uint32_t mine = my_chunk_count(n, w, Gn);
    for (uint32_t first = 0; first < mine; first += kSlice) {
      const uint32_t cnt = min(kSlice, mine - first);
      stage_slice(s_tab, table, c0, w, Gn, first, cnt);
      __syncthreads();
      for (uint32_t e = 0; e < cnt; ++e) body(read_entry(&s_tab[e]), c0 + w + (first + e) * Gn);
      __syncthreads();
    }
  } else {
    for (uint32_t i = w; i < n; i += Gn) body(read_entry(&table[c0 + i]), c0 + i);
  }
}

// ---- gradient access by storage type -----------------------------------------

template <int GDT>
struct Grad;

// `wide` is the 128-bit piece the squared-norm pass loads; widen() turns it into
// its VE fp32 values (exactly).
template <>
struct Grad<BCA_GRAD_F32> {
  typedef float elem;
  typedef f32x4 wide;
  static constexpr uint32_t VE = 4;
  static __device__ __forceinline__ void widen(const wide& x, float (&f)[VE]) {
    f[0] = x.x, f[1] = x.y, f[2] = x.z, f[3] = x.w;
  }
  static __device__ __forceinline__ wide narrow(const float (&f)[VE]) {
    wide x;
    x.x = f[0], x.y = f[1], x.z = f[2], x.w = f[3];
    return x;
  }
  template <bool NT>
  static __device__ __forceinline__ f32x4 load4(const void* base, uint32_t vec) {
    return ldv<NT>(reinterpret_cast<const f32x4*>(base) + vec);
  }
  template <bool NT>
  static __device__ __forceinline__ void store4(void* base, uint32_t vec, f32x4 x) {
    stv<NT>(reinterpret_cast<f32x4*>(base) + vec, x);
  }
  static __device__ __forceinline__ float load1(const void* base, uint32_t i) {
    return as_global(reinterpret_cast<const float*>(base))[i];
  }
  static __device__ __forceinline__ void store1(void* base, uint32_t i, float x) {
    as_global(reinterpret_cast<float*>(base))[i] = x;
  }
};

template <>
struct Grad<BCA_GRAD_F16> {
  typedef _Float16 elem;
  typedef f16x8 wide;
  static constexpr uint32_t VE = 8;
  static __device__ __forceinline__ void widen(const wide& x, float (&f)[VE]) {
#pragma unroll
    for (int q = 0; q < 8; ++q) f[q] = (float)x[q];
  }
  // fp16 -> fp32 is exact (subnormals included); fp32 -> fp16 rounds to nearest even.  What is stored is the
  // fp32 value rounded once more: settled() keeps the compiler from folding the multiplication that made the
  // value into the conversion (a mixed-precision multiply rounds the exact product to fp16 in one step, which
  // differs from the two roundings on ties of the fp32 product, about one stored value in a thousand).
  static __device__ __forceinline__ float settled(float x) {
    asm volatile("" : "+v"(x));
    return x;
  }
  static __device__ __forceinline__ wide narrow(const float (&f)[VE]) {  // the rounding of store4 / store1
    wide x;
#pragma unroll
    for (int q = 0; q < 8; ++q) x[q] = (_Float16)settled(f[q]);
    return x;
  }
  template <bool NT>
  static __device__ __forceinline__ f32x4 load4(const void* base, uint32_t vec) {
    const f16x4 h = ldv<NT>(reinterpret_cast<const f16x4*>(base) + vec);
    f32x4 r;
    r.x = (float)h.x, r.y = (float)h.y, r.z = (float)h.z, r.w = (float)h.w;
    return r;
  }
  template <bool NT>
  static __device__ __forceinline__ void store4(void* base, uint32_t vec, f32x4 x) {
    f16x4 h;
    h.x = (_Float16)settled(x.x), h.y = (_Float16)settled(x.y), h.z = (_Float16)settled(x.z), h.w = (_Float16)settled(x.w);
    stv<NT>(reinterpret_cast<f16x4*>(base) + vec, h);
  }
  static __device__ __forceinline__ float load1(const void* base, uint32_t i) {
    return (float)as_global(reinterpret_cast<const _Float16*>(base))[i];
  }
  static __device__ __forceinline__ void store1(void* base, uint32_t i, float x) {
    as_global(reinterpret_cast<_Float16*>(base))[i] = (_Float16)settled(x);
  }
};

// bfloat16 is the upper half of a binary32: widening appends 16 zero bits (exact);
// narrowing rounds to nearest, ties to even, in integer arithmetic (the carry out of
// the fraction moves to the exponent and ends at infinity, as it should); NaN stays
// NaN with the quiet bit set.
__device__ __forceinline__ float bf16_to_f32(unsigned short h) { return __uint_as_float((uint32_t)h << 16); }
__device__ __forceinline__ unsigned short f32_to_bf16(float x) {
  const uint32_t u = __float_as_uint(x);
  if (x != x) return (unsigned short)((u >> 16) | 0x40u);
  return (unsigned short)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

template <>
struct Grad<BCA_GRAD_BF16> {
  typedef unsigned short elem;
  typedef u16x8 wide;
  static constexpr uint32_t VE = 8;
  static __device__ __forceinline__ void widen(const wide& x, float (&f)[VE]) {
#pragma unroll
    for (int q = 0; q < 8; ++q) f[q] = bf16_to_f32(x[q]);
  }
  static __device__ __forceinline__ wide narrow(const float (&f)[VE]) {
    wide x;
#pragma unroll
    for (int q = 0; q < 8; ++q) x[q] = f32_to_bf16(f[q]);
    return x;
  }
  template <bool NT>
  static __device__ __forceinline__ f32x4 load4(const void* base, uint32_t vec) {
    const u16x4 h = ldv<NT>(reinterpret_cast<const u16x4*>(base) + vec);
    f32x4 r;
    r.x = bf16_to_f32(h.x), r.y = bf16_to_f32(h.y), r.z = bf16_to_f32(h.z), r.w = bf16_to_f32(h.w);
    return r;
  }
  template <bool NT>
  static __device__ __forceinline__ void store4(void* base, uint32_t vec, f32x4 x) {
    u16x4 h;
    h.x = f32_to_bf16(x.x), h.y = f32_to_bf16(x.y), h.z = f32_to_bf16(x.z), h.w = f32_to_bf16(x.w);
    stv<NT>(reinterpret_cast<u16x4*>(base) + vec, h);
  }
  static __device__ __forceinline__ float load1(const void* base, uint32_t i) {
    return bf16_to_f32(as_global(reinterpret_cast<const unsigned short*>(base))[i]);
  }
  static __device__ __forceinline__ void store1(void* base, uint32_t i, float x) {
    as_global(reinterpret_cast<unsigned short*>(base))[i] = f32_to_bf16(x);
  }
};

// Number of leading elements to handle one by one so that what follows can be
// accessed as aligned vectors (g in g_vec_bytes pieces, the fp32 arrays in 16-byte
// pieces), or `len` if no such head exists (mutually incongruent addresses).
__device__ __forceinline__ uint32_t vector_head(uint32_t len, uint64_t g_addr, uint32_t gsize, uint32_t g_vec_bytes,
                                                bool with_state, uint64_t p, uint64_t m, uint64_t v) {
  const uint32_t mis = (uint32_t)(g_addr & (g_vec_bytes - 1));
  if (mis % gsize) return len;
  const uint32_t h = ((g_vec_bytes - mis) & (g_vec_bytes - 1)) / gsize;
  if (with_state) {
    const uint64_t sh = (uint64_t)h * 4u;
    if (((p + sh) | (m + sh) | (v + sh)) & 15u) return len;
  }
  return h < len ? h : len;
}

// ---- wavefront reduction (fixed order) ----------------------------------------

__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
  return x;
}

// ---- squared-norm partials ------------------------------------------------------

// Adds the squares of one 128-bit piece to the lane's four fp32 accumulators: element q of the piece goes to
// accumulator q mod 4, in element order.  Every squared-norm path goes through this one function, so that a
// chunk's partial sums do not depend on which kernel computed them.
template <int GDT>
__device__ __forceinline__ void add_squares(const typename Grad<GDT>::wide& x, float& a0, float& a1, float& a2, float& a3) {
  constexpr uint32_t VE = Grad<GDT>::VE;
  float f[VE];
  Grad<GDT>::widen(x, f);
#pragma unroll
  for (uint32_t q = 0; q < VE; q += 4) {
    a0 = __fmaf_rn(f[q], f[q], a0), a1 = __fmaf_rn(f[q + 1], f[q + 1], a1);
    a2 = __fmaf_rn(f[q + 2], f[q + 2], a2), a3 = __fmaf_rn(f[q + 3], f[q + 3], a3);
  }
}

// Sum of g^2 over the part of a chunk this wavefront reads, in fp64 (same value
// in every lane).  Per lane the squares are accumulated in fp32 (four independent
// accumulators, at most chunk_elems/1024 terms each), then the lanes are combined
// in fp64 by butterfly shuffles.  Wavefronts never wait for each other.
template <int GDT, bool NT, uint32_t U = 8>  // U: 128-bit loads in flight per lane (the result does not depend on it)
__device__ __forceinline__ double sqnorm_chunk(const Entry& en) {
  typedef Grad<GDT> G;
  constexpr uint32_t gsize = sizeof(typename G::elem);
  constexpr uint32_t VE = G::VE;  // elements per 128-bit load: 4 (fp32) or 8 (fp16, bf16)
  const uint32_t tid = threadIdx.x;
  const uint64_t ga = en.g;
  const uint32_t len = en.len;
  const uint32_t head = vector_head(len, ga, gsize, 16u, false, 0, 0, 0);
  const uint32_t nvec = (len - head) / VE;
  const uint32_t tail0 = head + nvec * VE;
  const void* gbase = reinterpret_cast<const void*>(ga);
  const void* gv = reinterpret_cast<const void*>(ga + (uint64_t)head * gsize);
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;

  typedef typename G::wide wide;
  const wide* gw = reinterpret_cast<const wide*>(gv);
  // Lane t adds pieces t, t + 256, t + 512, ... in that order.  They are fetched U at a time; a slot past the end
  // of the chunk holds zeros, whose squares leave the (non-negative) accumulators as they are.
  for (uint32_t base = 0; base < nvec; base += kBlock * U) {
    const uint32_t j0 = base + tid;
    wide x[U];
    if (base + kBlock * U <= nvec) {
#pragma unroll
      for (uint32_t u = 0; u < U; ++u) x[u] = ldv<NT>(gw + j0 + u * kBlock);
    } else {
#pragma unroll
      for (uint32_t u = 0; u < U; ++u) {
        const uint32_t j = j0 + u * kBlock;
        x[u] = wide{};
        if (j < nvec) x[u] = ldv<NT>(gw + j);
      }
    }
    loads_issued();
#pragma unroll
    for (uint32_t u = 0; u < U; ++u) add_squares<GDT>(x[u], a0, a1, a2, a3);
  }
  // head and tail elements one by one (fewer than VE each unless the chunk is unaligned throughout)
  for (uint32_t i = tid; i < head; i += kBlock) {
    const float x = G::load1(gbase, i);
    a0 = __fmaf_rn(x, x, a0);
  }
  for (uint32_t i = tail0 + tid; i < len; i += kBlock) {
    const float x = G::load1(gbase, i);
    a1 = __fmaf_rn(x, x, a1);
  }
  const double lane = ((double)a0 + (double)a1) + ((double)a2 + (double)a3);
  return wave_sum(lane);
}

// kWaves partials (fp64) per chunk, one per wavefront.  The finalize pass adds a
// bucket's partials in a fixed order.
template <int GDT, bool NT, bool STAGED, uint32_t U>
__global__ __launch_bounds__(kBlock) void k_sqnorm(const Chunk* __restrict__ table, uint32_t c0, uint32_t n,
                                                    double* __restrict__ partials, int32_t* status) {
  const uint32_t tid = threadIdx.x;
  if (status != nullptr && blockIdx.x == 0 && tid == 0) *status = 0;  // finalize ORs into it later on this stream
  for_each_chunk<STAGED>(table, c0, n, [&](const Entry& en, uint32_t ci) {
    const double ws = sqnorm_chunk<GDT, NT, U>(en);
    if ((tid & 63u) == 0) partials[(uint64_t)ci * kWaves + (tid >> 6)] = ws;
  });
}

// ---- clip coefficient -----------------------------------------------------------

// Sec. 2.3: if ||g|| >= c the gradient is multiplied by c / ||g||, else left
// alone.  The quotient is taken in fp64 from the fp32 norm and rounded once.
// A threshold that is not a positive number means "no clipping" and is flagged.
__device__ __forceinline__ float clip_coef(float norm, float c, int32_t& status) {
  if (!(fabsf(norm) <= 3.402823466e38f)) status |= BCA_STATUS_NONFINITE;  // Inf or NaN
  if (!(c > 0.f)) {
    status |= BCA_STATUS_BAD_THRESHOLD;
    return 1.f;
  }
  if (norm >= c) return (float)((double)c / (double)norm);
  return 1.f;
}

// The sum of partials[lo .. hi) in THE order every path uses (thread t adds lo + t, lo + t + 256, ... one after the
// other, lanes by butterfly, wavefronts in index order), computed by the whole workgroup; loads are issued eight
// at a time before the first addition, a slot past the end adding +0.0.  Valid in thread 0.
__device__ __forceinline__ double sum_partials(const double* __restrict__ partials, uint64_t lo, uint64_t hi, double* s_w) {
  const uint32_t tid = threadIdx.x;
  double s = 0.0;
  for (uint64_t i = lo + tid; i < hi; i += 8u * kBlock) {
    double part[8];
#pragma unroll
    for (uint32_t q = 0; q < 8u; ++q) {
      const uint64_t j = i + (uint64_t)q * kBlock;
      part[q] = j < hi ? partials[j] : 0.0;
    }
#pragma unroll
    for (uint32_t q = 0; q < 8u; ++q) s += part[q];
  }
  s = wave_sum(s);
  if ((tid & 63u) == 0) s_w[tid >> 6] = s;
  __syncthreads();
  return ((s_w[0] + s_w[1]) + s_w[2]) + s_w[3];
}

// One workgroup per bucket: threads take the bucket's partials in strides of 256
// in fp64, lanes are combined by a butterfly, the four wavefronts through LDS in
// index order.  Same order on every run, so norms are reproducible.
__global__ __launch_bounds__(kBlock) void k_finalize(const double* __restrict__ partials,
                                                      const uint32_t* __restrict__ bucket_chunk_off, uint32_t b0,
                                                      const float* __restrict__ thresholds, float* __restrict__ norms,
                                                      float* __restrict__ coefs, int32_t* status,
                                                      double* __restrict__ bucket_sq) {
  __shared__ double s_w[kWaves];
  const uint32_t b = b0 + blockIdx.x;
  const uint64_t lo = (uint64_t)bucket_chunk_off[b] * kWaves, hi = (uint64_t)bucket_chunk_off[b + 1] * kWaves;
  const double tot = sum_partials(partials, lo, hi, s_w);
  if (threadIdx.x == 0) {
    const float norm = (float)sqrt(tot);
    norms[b] = norm;
    if (bucket_sq != nullptr) bucket_sq[b] = tot;
    if (thresholds != nullptr) {
      int32_t st = 0;
      const float coef = clip_coef(norm, thresholds[b], st);
      coefs[b] = coef;
      if (st != 0 && status != nullptr) atomicOr(status, st);
    }
  }
}

// Whole-gradient clipping (Sec. 3.2's baselines): the buckets' sums of squares
// are added in index order in fp64, the clipping rule of Sec. 2.3 is applied
// once with the single threshold *c, and every bucket gets that coefficient.
// One workgroup; ORs its status bits into *status.
__global__ __launch_bounds__(kBlock) void k_whole_coef(const double* __restrict__ bucket_sq, uint32_t n_buckets,
                                                        const float* __restrict__ c, float* __restrict__ whole_norm,
                                                        float* __restrict__ coefs, int32_t* status) {
  __shared__ double s_w[kWaves];
  __shared__ float s_coef;
  double s = 0.0;
  for (uint32_t b = threadIdx.x; b < n_buckets; b += kBlock) s += bucket_sq[b];
  s = wave_sum(s);
  if ((threadIdx.x & 63u) == 0) s_w[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    const float norm = (float)sqrt(((s_w[0] + s_w[1]) + s_w[2]) + s_w[3]);
    int32_t st = 0;
    s_coef = clip_coef(norm, *c, st);
    *whole_norm = norm;
    if (st != 0) atomicOr(status, st);
  }
  __syncthreads();
  for (uint32_t b = threadIdx.x; b < n_buckets; b += kBlock) coefs[b] = s_coef;
}

// Coefficients from norms the caller supplies (unfused path).  One workgroup;
// writes (not ORs) the status word of this call.
__global__ __launch_bounds__(kBlock) void k_coefs(uint32_t b0, uint32_t b1, const float* __restrict__ thresholds,
                                                   const float* __restrict__ norms, float* __restrict__ coefs,
                                                   int32_t* status) {
  __shared__ int32_t s_st;
  if (threadIdx.x == 0) s_st = 0;
  __syncthreads();
  int32_t st = 0;
  for (uint32_t b = b0 + threadIdx.x; b < b1; b += kBlock) coefs[b] = clip_coef(norms[b], thresholds[b], st);
  if (st != 0) atomicOr(&s_st, st);
  __syncthreads();
  if (threadIdx.x == 0 && status != nullptr) *status = s_st;
}

// ---- in-place scale -------------------------------------------------------------

// g <- coef * g over one chunk, in the gradient's storage type (Alg. 1, the
// assignment under the if).
template <int GDT, uint32_t U, bool NT>
__device__ __forceinline__ void scale_chunk(const Entry& en, float coef) {
  typedef Grad<GDT> G;
  constexpr uint32_t gsize = sizeof(typename G::elem);
  const uint32_t tid = threadIdx.x;
  const uint64_t ga = en.g;
  const uint32_t len = en.len;
  const uint32_t head = vector_head(len, ga, gsize, 4u * gsize, false, 0, 0, 0);
  const uint32_t nvec = (len - head) / 4u;
  const uint32_t tail0 = head + nvec * 4u;
  void* gbase = reinterpret_cast<void*>(ga);
  void* gv = reinterpret_cast<void*>(ga + (uint64_t)head * gsize);
  for (uint32_t base = 0; base < nvec; base += kBlock * U) {
    const uint32_t j0 = base + tid;
    if (base + kBlock * U <= nvec) {
      f32x4 x[U];
#pragma unroll
      for (uint32_t u = 0; u < U; ++u) x[u] = G::template load4<NT>(gv, j0 + u * kBlock);
      loads_issued();
#pragma unroll
      for (uint32_t u = 0; u < U; ++u) G::template store4<NT>(gv, j0 + u * kBlock, x[u] * coef);
    } else {
      for (uint32_t u = 0; u < U; ++u) {
        const uint32_t j = j0 + u * kBlock;
        if (j < nvec) G::template store4<NT>(gv, j, G::template load4<NT>(gv, j) * coef);
      }
    }
  }
  for (uint32_t i = tid; i < head; i += kBlock) G::store1(gbase, i, G::load1(gbase, i) * coef);
  for (uint32_t i = tail0 + tid; i < len; i += kBlock) G::store1(gbase, i, G::load1(gbase, i) * coef);
}

// Buckets with coef_b == 1 are not read at all.
template <int GDT, uint32_t U, bool NT, bool STAGED>
__global__ __launch_bounds__(kBlock) void k_scale(const Chunk* __restrict__ table, uint32_t c0, uint32_t n,
                                                   const float* __restrict__ coefs) {
  for_each_chunk<STAGED>(table, c0, n, [&](const Entry& en, uint32_t) {
    const float coef = coefs[en.bucket];
    if (coef != 1.f) scale_chunk<GDT, U, NT>(en, coef);
  });
}

// ---- Adam -----------------------------------------------------------------------

// One element of  theta <- ADAM(theta, eta, G)  (Alg. 1, last line):
//   m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2
//   p <- p - lr * ( mhat / (sqrt(vhat) + eps) + wd p ),  mhat = m/(1-b1^t), vhat = v/(1-b2^t)
// Division and square root are the correctly rounded ones.
// wd is the weight decay that applies to the element's tensor: k.wd, or 0 for a
// tensor the decay mask exempts.
// The constants a kernel works with: those passed by value, or the device copy they point to.
__device__ __forceinline__ AdamK resolve(const AdamK& a) {
  if (a.from != nullptr) return *a.from;
  return a;
}

// Hyper-parameters in device memory -> the sweeps' constants, as the host derives them from a bca_adam.
__global__ __launch_bounds__(64) void k_hyper(const bca_adam_device* __restrict__ dev, AdamK* __restrict__ out) {
  if (threadIdx.x != 0) return;
  const double t = (double)dev->step;
  AdamK k;
  k.b1 = (float)dev->beta1, k.omb1 = (float)(1.0 - dev->beta1);
  k.b2 = (float)dev->beta2, k.omb2 = (float)(1.0 - dev->beta2);
  k.rbc1 = (float)(1.0 / (1.0 - pow(dev->beta1, t))), k.rbc2 = (float)(1.0 / (1.0 - pow(dev->beta2, t)));
  k.eps = (float)dev->eps;
  k.neg_lr = (float)(-dev->lr);
  k.wd = (float)dev->weight_decay;
  k.lr = dev->lr;
  k.from = nullptr;
  *out = k;
}

__device__ __forceinline__ void adam_moments(float g, float& m, float& v, const AdamK& k) {
  m = __fmaf_rn(k.b1, m, k.omb1 * g);
  v = __fmaf_rn(k.b2, v, k.omb2 * (g * g));
}
// mhat / (sqrt(vhat) + eps) + wd p: the bracket of Adam's parameter update, which is
// also LAMB's update direction.
__device__ __forceinline__ float adam_direction(float p, float m, float v, const AdamK& k, float wd) {
  const float mhat = m * k.rbc1;
  const float vhat = v * k.rbc2;
  const float denom = __fsqrt_rn(vhat) + k.eps;
  return __fmaf_rn(wd, p, __fdiv_rn(mhat, denom));
}
__device__ __forceinline__ void adam1(float g, float& p, float& m, float& v, const AdamK& k, float wd) {
  adam_moments(g, m, v, k);
  p = __fmaf_rn(k.neg_lr, adam_direction(p, m, v, k, wd), p);
}

__device__ __forceinline__ void adam4(f32x4 g, f32x4& p, f32x4& m, f32x4& v, const AdamK& k, float wd) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float pi = p[i], mi = m[i], vi = v[i];
    adam1(g[i], pi, mi, vi, k, wd);
    p[i] = pi, m[i] = mi, v[i] = vi;
  }
}

__device__ __forceinline__ float chunk_wd(const Entry& en, const AdamK& k) {
  return (en.flags & kChunkNoDecay) ? 0.f : k.wd;
}

// The read-modify-write sweep over one chunk.  coef != 1 only on the fused path:
// ghat = coef_b * g is formed in registers (one fp32 multiply, so it equals what
// k_scale would have stored for fp32 gradients); WB: ghat, rounded to the gradient
// type, also replaces g.  p, m, v are touched once per sweep and always stream;
// GNT says whether g streams too.
template <int GDT, bool FUSED, bool WB, uint32_t U, bool GNT>
__device__ __forceinline__ void adam_chunk(const Entry& en, float coef, const AdamK& k) {
  typedef Grad<GDT> G;
  constexpr uint32_t gsize = sizeof(typename G::elem);
  constexpr bool NT = true;
  const uint32_t tid = threadIdx.x;
  const uint64_t ga = en.g, pa = en.p, ma = en.m, va = en.v;
  const uint32_t len = en.len;
  const bool wb = WB && coef != 1.f;
  const float wd = chunk_wd(en, k);
  const uint32_t head = vector_head(len, ga, gsize, 4u * gsize, true, pa, ma, va);
  const uint32_t nvec = (len - head) / 4u;
  const uint32_t tail0 = head + nvec * 4u;
  void* gv = reinterpret_cast<void*>(ga + (uint64_t)head * gsize);
  f32x4* pv = reinterpret_cast<f32x4*>(pa + (uint64_t)head * 4u);
  f32x4* mv = reinterpret_cast<f32x4*>(ma + (uint64_t)head * 4u);
  f32x4* vv = reinterpret_cast<f32x4*>(va + (uint64_t)head * 4u);

  for (uint32_t base = 0; base < nvec; base += kBlock * U) {
    const uint32_t j0 = base + tid;
    if (base + kBlock * U <= nvec) {
      f32x4 g[U], p[U], m[U], v[U];
#pragma unroll
      for (uint32_t u = 0; u < U; ++u) g[u] = G::template load4<GNT>(gv, j0 + u * kBlock);
#pragma unroll
      for (uint32_t u = 0; u < U; ++u) p[u] = ldv<NT>(pv + j0 + u * kBlock);
#pragma unroll
      for (uint32_t u = 0; u < U; ++u) m[u] = ldv<NT>(mv + j0 + u * kBlock);
#pragma unroll
      for (uint32_t u = 0; u < U; ++u) v[u] = ldv<NT>(vv + j0 + u * kBlock);
      loads_issued();
#pragma unroll
      for (uint32_t u = 0; u < U; ++u) {
        if constexpr (FUSED) g[u] = g[u] * coef;
        adam4(g[u], p[u], m[u], v[u], k, wd);
        const uint32_t j = j0 + u * kBlock;
        stv<NT>(pv + j, p[u]), stv<NT>(mv + j, m[u]), stv<NT>(vv + j, v[u]);
        if (wb) G::template store4<GNT>(gv, j, g[u]);
      }
    } else {
      for (uint32_t u = 0; u < U; ++u) {
        const uint32_t j = j0 + u * kBlock;
        if (j < nvec) {
          f32x4 g = G::template load4<GNT>(gv, j), p = ldv<NT>(pv + j), m = ldv<NT>(mv + j), v = ldv<NT>(vv + j);
          if constexpr (FUSED) g = g * coef;
          adam4(g, p, m, v, k, wd);
          stv<NT>(pv + j, p), stv<NT>(mv + j, m), stv<NT>(vv + j, v);
          if (wb) G::template store4<GNT>(gv, j, g);
        }
      }
    }
  }
  // head and tail, element-wise
  void* gbase = reinterpret_cast<void*>(ga);
  BCA_GLOBAL float* p1 = as_global(reinterpret_cast<float*>(pa));
  BCA_GLOBAL float* m1 = as_global(reinterpret_cast<float*>(ma));
  BCA_GLOBAL float* v1 = as_global(reinterpret_cast<float*>(va));
  for (uint32_t r = tid; r < head + (len - tail0); r += kBlock) {
    const uint32_t i = r < head ? r : tail0 + (r - head);
    float g = G::load1(gbase, i), p = p1[i], m = m1[i], v = v1[i];
    if constexpr (FUSED) g = g * coef;
    adam1(g, p, m, v, k, wd);
    p1[i] = p, m1[i] = m, v1[i] = v;
    if (wb) G::store1(gbase, i, g);
  }
}

template <int GDT, bool FUSED, bool WB, uint32_t U, bool GNT, bool STAGED>
__global__ __launch_bounds__(kBlock) void k_adam(const Chunk* __restrict__ table, uint32_t c0, uint32_t n,
                                                  const float* __restrict__ coefs, const int32_t* skip_status,
                                                  const AdamK ka) {
  if (skip_status != nullptr && (*skip_status & BCA_STATUS_NONFINITE)) return;
  const AdamK k = resolve(ka);
  for_each_chunk<STAGED>(table, c0, n, [&](const Entry& en, uint32_t) {
    float coef = 1.f;
    if constexpr (FUSED) coef = coefs[en.bucket];
    adam_chunk<GDT, FUSED, WB, U, GNT>(en, coef, k);
  });
}

// ---- LAMB -------------------------------------------------------------------------
//
// LAMB (You et al. 2020, the optimizer the paper weighs Adam against in Sec. 2.2 and
// Sec. 5) keeps Adam's moments and direction u = mhat / (sqrt(vhat) + eps) + wd p, and
// scales each tensor's step by the trust ratio ||p|| / ||u||.  The ratio needs sums
// over whole tensors, so the sweep is split in two, over a tensor-major chunk table:
//   k_lamb_moments : g, p, m, v -> m, v; per-chunk sums of p^2 and u^2
//   k_lamb_trust   : per tensor, the sums in chunk order (fp64) -> ratio, -lr * ratio
//   k_lamb_update  : p, m, v -> p + (-lr ratio) u, u recomputed from the stored moments
// (recomputing u costs the same 16 B/element as storing and re-reading it would, and
// leaves the gradients alone).  Both stages evaluate u with the same correctly rounded
// operations on the same fp32 inputs, so the u that is applied is the u that was measured.

// Combines per-lane values of the four wavefronts in a fixed order; the result is valid in thread 0.
__device__ __forceinline__ double block_sum(double x, double* s_w) {
  x = wave_sum(x);
  if ((threadIdx.x & 63u) == 0) s_w[threadIdx.x >> 6] = x;
  __syncthreads();
  return ((s_w[0] + s_w[1]) + s_w[2]) + s_w[3];
}

// LAMB's first sweep over one chunk: moments updated and stored, the chunk's sums of
// p^2 and u^2 written to out[0], out[1] (fp64; per lane 4 * chunk_elems / 1024 squares
// are added in fp32 first).  coef != 1 only behind clipping; WB: the scaled gradient,
// rounded to its storage type, also replaces g.  GNT: whether g streams (it does not
// when the squared-norm pass has just read it and it is still cached).
template <int GDT, bool FUSED, bool WB, bool GNT, bool KEEP = false>
__device__ __forceinline__ void lamb_moments_chunk(const Entry& en, float coef, const AdamK& k, double* s_pp,
                                                   double* s_uu, double* __restrict__ out) {
  typedef Grad<GDT> G;
  constexpr uint32_t gsize = sizeof(typename G::elem);
  const uint32_t tid = threadIdx.x;
  const bool wb = WB && coef != 1.f;
  const float wd = chunk_wd(en, k);
  const uint32_t len = en.len;
  const uint32_t head = vector_head(len, en.g, gsize, 4u * gsize, true, en.p, en.m, en.v);
  const uint32_t nvec = (len - head) / 4u;
  const uint32_t tail0 = head + nvec * 4u;
  void* gv = reinterpret_cast<void*>(en.g + (uint64_t)head * gsize);
  const f32x4* pv = reinterpret_cast<const f32x4*>(en.p + (uint64_t)head * 4u);
  f32x4* mv = reinterpret_cast<f32x4*>(en.m + (uint64_t)head * 4u);
  f32x4* vv = reinterpret_cast<f32x4*>(en.v + (uint64_t)head * 4u);
  float pp = 0.f, uu = 0.f;
  for (uint32_t j = tid; j < nvec; j += kBlock) {
    f32x4 g = G::template load4<GNT>(gv, j), p = ldv<true>(pv + j), m = ldv<true>(mv + j), v = ldv<true>(vv + j);
    loads_issued();
    if constexpr (FUSED) g = g * coef;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float mi = m[i], vi = v[i];
      adam_moments(g[i], mi, vi, k);
      const float u = adam_direction(p[i], mi, vi, k, wd);
      pp = __fmaf_rn(p[i], p[i], pp), uu = __fmaf_rn(u, u, uu);
      m[i] = mi, v[i] = vi;
    }
    stv<!KEEP>(mv + j, m), stv<!KEEP>(vv + j, v);
    if (wb) G::template store4<GNT>(gv, j, g);
  }
  void* gbase = reinterpret_cast<void*>(en.g);
  const BCA_GLOBAL float* p1 = as_global(reinterpret_cast<const float*>(en.p));
  BCA_GLOBAL float* m1 = as_global(reinterpret_cast<float*>(en.m));
  BCA_GLOBAL float* v1 = as_global(reinterpret_cast<float*>(en.v));
  for (uint32_t r = tid; r < head + (len - tail0); r += kBlock) {
    const uint32_t i = r < head ? r : tail0 + (r - head);
    float g = G::load1(gbase, i), m = m1[i], v = v1[i];
    const float p = p1[i];
    if constexpr (FUSED) g = g * coef;
    adam_moments(g, m, v, k);
    const float u = adam_direction(p, m, v, k, wd);
    pp = __fmaf_rn(p, p, pp), uu = __fmaf_rn(u, u, uu);
    m1[i] = m, v1[i] = v;
    if (wb) G::store1(gbase, i, g);
  }
  const double tpp = block_sum((double)pp, s_pp), tuu = block_sum((double)uu, s_uu);
  if (tid == 0) out[0] = tpp, out[1] = tuu;
}

template <int GDT, bool FUSED, bool WB, bool KEEP>
__global__ __launch_bounds__(kBlock) void k_lamb_moments(const Chunk* __restrict__ table, uint32_t n,
                                                          const float* __restrict__ coefs,
                                                          double* __restrict__ sums, const AdamK ka) {
  __shared__ double s_pp[kWaves], s_uu[kWaves];
  const AdamK k = resolve(ka);
  for (uint32_t ci = blockIdx.x; ci < n; ci += gridDim.x) {
    const Entry en = read_entry(&table[ci]);
    float coef = 1.f;
    if constexpr (FUSED) coef = coefs[en.bucket];
    lamb_moments_chunk<GDT, FUSED, WB, true, KEEP>(en, coef, k, s_pp, s_uu, sums + (uint64_t)ci * 2u);
    __syncthreads();  // s_pp / s_uu are reused by the next chunk
  }
}

// One workgroup of 1024 threads per tensor: the chunk sums strided over the threads (two
// independent accumulators each, the word embedding alone has 30 K chunks), butterfly per
// wavefront, the sixteen wavefronts in index order; then trust = ||p|| / ||u||, or 1
// where either norm is zero and the quotient means nothing; scale = -lr * trust in fp64,
// rounded once.  The order is fixed, so the ratios are reproducible.
constexpr uint32_t kTrustBlock = 1024;
__global__ __launch_bounds__(kTrustBlock) void k_lamb_trust(const double* __restrict__ sums,
                                                             const uint32_t* __restrict__ tensor_off, const AdamK ka,
                                                             float* __restrict__ trust, float* __restrict__ scale) {
  __shared__ double s_pp[kTrustBlock / 64], s_uu[kTrustBlock / 64];
  const double lr = resolve(ka).lr;
  const uint32_t t = blockIdx.x, lo = tensor_off[t], hi = tensor_off[t + 1];
  double pp0 = 0.0, uu0 = 0.0, pp1 = 0.0, uu1 = 0.0;
  uint32_t c = lo + threadIdx.x;
  for (; c + kTrustBlock < hi; c += 2u * kTrustBlock) {
    pp0 += sums[(uint64_t)c * 2u], uu0 += sums[(uint64_t)c * 2u + 1u];
    pp1 += sums[(uint64_t)(c + kTrustBlock) * 2u], uu1 += sums[(uint64_t)(c + kTrustBlock) * 2u + 1u];
  }
  if (c < hi) pp0 += sums[(uint64_t)c * 2u], uu0 += sums[(uint64_t)c * 2u + 1u];
  const double pp = wave_sum(pp0 + pp1), uu = wave_sum(uu0 + uu1);
  if ((threadIdx.x & 63u) == 0) s_pp[threadIdx.x >> 6] = pp, s_uu[threadIdx.x >> 6] = uu;
  __syncthreads();
  if (threadIdx.x == 0) {
    double tpp = 0.0, tuu = 0.0;
    for (uint32_t w = 0; w < kTrustBlock / 64; ++w) tpp += s_pp[w], tuu += s_uu[w];
    const double pn = sqrt(tpp), un = sqrt(tuu);
    const double r = (pn > 0.0 && un > 0.0) ? pn / un : 1.0;
    trust[t] = (float)r;
    scale[t] = (float)(-lr * r);
  }
}

__global__ __launch_bounds__(kBlock) void k_lamb_update(const Chunk* __restrict__ table, uint32_t n,
                                                         const float* __restrict__ scale, const AdamK ka) {
  const uint32_t tid = threadIdx.x;
  const AdamK k = resolve(ka);
  for (uint32_t ci = blockIdx.x; ci < n; ci += gridDim.x) {
    const Entry en = read_entry(&table[ci]);
    const float sc = scale[en.tensor];
    const float wd = chunk_wd(en, k);
    const uint32_t len = en.len;
    const uint32_t head = vector_head(len, en.p, 4u, 16u, true, en.p, en.m, en.v);
    const uint32_t nvec = (len - head) / 4u;
    const uint32_t tail0 = head + nvec * 4u;
    f32x4* pv = reinterpret_cast<f32x4*>(en.p + (uint64_t)head * 4u);
    const f32x4* mv = reinterpret_cast<const f32x4*>(en.m + (uint64_t)head * 4u);
    const f32x4* vv = reinterpret_cast<const f32x4*>(en.v + (uint64_t)head * 4u);
    for (uint32_t j = tid; j < nvec; j += kBlock) {
      f32x4 p = ldv<true>(pv + j);
      const f32x4 m = ldv<true>(mv + j), v = ldv<true>(vv + j);
      loads_issued();
#pragma unroll
      for (int i = 0; i < 4; ++i) p[i] = __fmaf_rn(sc, adam_direction(p[i], m[i], v[i], k, wd), p[i]);
      stv<true>(pv + j, p);
    }
    BCA_GLOBAL float* p1 = as_global(reinterpret_cast<float*>(en.p));
    const BCA_GLOBAL float* m1 = as_global(reinterpret_cast<const float*>(en.m));
    const BCA_GLOBAL float* v1 = as_global(reinterpret_cast<const float*>(en.v));
    for (uint32_t r = tid; r < head + (len - tail0); r += kBlock) {
      const uint32_t i = r < head ? r : tail0 + (r - head);
      p1[i] = __fmaf_rn(sc, adam_direction(p1[i], m1[i], v1[i], k, wd), p1[i]);
    }
  }
}

// ---- the whole fused step in one launch ----------------------------------------------
//
// Work items (one per workgroup) are listed by the host in an order that
// pipelines bucket groups:  N(g0) N(g1) A(g0) N(g2) A(g1) ... A(last), where N(g)
// are the squared-norm chunks of group g's buckets and A(g) the Adam chunks.  A
// group's gradients are read by N(g), stay in the Infinity Cache (everything
// else streams past it with non-temporal accesses), and are read again by A(g)
// one group later, so HBM sees the gradients once.
//
// An Adam item needs its bucket's coefficient; it waits on that bucket's ready
// word, which is set by whichever squared-norm workgroup of the bucket finishes
// last (it adds the bucket's partials in the fixed order of k_finalize, so
// results do not depend on who that is).  All squared-norm items of a bucket
// precede its Adam items in the list and never wait themselves.
//
// Which workgroup takes which item:
//  * default: item = workgroup index.  The hardware has been seen to start the
//    workgroups of a grid in index order within each XCD, so that everything an
//    Adam item waits for has been started before it; that is what makes the
//    pipeline fast, but nothing below depends on it for its result.
//  * TICKETS: eight atomic counters, one per XCD; item 8 t + y is the t-th item
//    of list y.  A workgroup draws from its own XCD's list and moves to the next
//    list when that one is used up.  Each list is thus started strictly in order
//    by running workgroups, whatever the dispatcher does.
//
// Every wait is bounded: after StepState::spin_limit polls the item gives up, files
// its index in the skipped list, raises the abort word (every other waiter then
// gives up at its next look) and BCA_STATUS_TIMEOUT, and its workgroup ends, which
// frees the slot for whatever it was waiting for.  Squared-norm items never wait, so
// by the end of the launch every bucket's coefficient exists, and the finish kernel
// that follows every such launch on the stream carries out the skipped items with
// the same code.  The call's result is therefore complete and bit-identical whatever
// the order in which workgroups were started; an expired wait only costs time.
//
// Per-call state needs no kernel in front of the launch: the last squared-norm item of a
// bucket zeroes that bucket's arrival counter, and the finish kernel hands the collected
// status bits to the caller, clears the abort word, the skipped count and the tickets and
// moves the epoch on, so that the state is ready for the next call on the plan.

// Waits until this wavefront's outstanding vector-memory operations have completed (stores
// included: gfx9-family stores are counted by vmcnt until they are acknowledged).
__device__ __forceinline__ void wait_vmem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__device__ __forceinline__ uint32_t ctl_load(const uint32_t* w) {
  return __hip_atomic_load(w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void ctl_store(uint32_t* w, uint32_t x) {
  __hip_atomic_store(w, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void ctl_or(uint32_t* w, uint32_t bits) {
  (void)__hip_atomic_fetch_or(w, bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Shared memory of one k_step workgroup.
struct StepShared {
  uint32_t item;
  uint32_t flag;
  float coef;
  double w[kWaves];
  double pp[kWaves], uu[kWaves];  // LAMB: block sums of p^2 and u^2
};

// Waits (bounded) for bucket b's ready word of this epoch.  Returns true with the
// bucket's coefficient in sh.coef; false when the wait expired, after filing `self`
// (the item's index in the apply table) for the finish kernel.
__device__ __forceinline__ bool wait_for_bucket(const StepState& st, uint32_t b, uint32_t epoch, uint32_t self,
                                                StepShared& sh) {
  if (threadIdx.x == 0) {
    // ready word: (epoch << 32) | bits of the coefficient
    unsigned long long r = 0;
    uint32_t polls = 0;
    for (;;) {
      r = __hip_atomic_load(&st.ready[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if ((uint32_t)(r >> 32) == epoch || ++polls > st.spin_limit) break;
      // once one wait has expired every other waiter gives up at its next look
      if ((polls & 63u) == 0 && ctl_load(&st.ctl[kCtlAbort]) != 0u) break;
      __builtin_amdgcn_s_sleep(8);
    }
    const bool ok = (uint32_t)(r >> 32) == epoch;
    sh.flag = ok ? 1u : 0u;
    sh.coef = __uint_as_float((uint32_t)r);
    if (polls != 0u) {  // statistics (bca_plan_wait_stats); an item that never waited does not come here
      uint32_t* slot = &st.ctl[kCtlStats + 32u * (blockIdx.x % kStatSlots)];
      atomicAdd(slot, 1u);
      atomicAdd(reinterpret_cast<unsigned long long*>(slot + 2), (unsigned long long)polls);
    }
    if (!ok) {
      ctl_store(&st.ctl[kCtlAbort], 1u);
      ctl_or(&st.ctl[kCtlStatus], BCA_STATUS_TIMEOUT);
      // every item is filed at most once, so the list cannot overflow unless an earlier call on the plan was
      // cut short between its two launches; then the item is reported lost rather than written out of bounds
      const uint32_t slot = atomicAdd(&st.ctl[kCtlSkipped], 1u);
      if (slot < st.skipped_cap) st.skipped[slot] = self;  // read by the finish kernel, after this launch has ended
      else ctl_or(&st.ctl[kCtlStatus], BCA_STATUS_INCOMPLETE);
    }
  }
  __syncthreads();
  return sh.flag != 0u;
}

// A squared-norm item (kind kItemNorm, idx = chunk of the norm table) or the
// stand-in for a bucket without elements (kItemEmpty, idx = bucket).  The last
// workgroup of a bucket to get here adds the bucket's partials in the fixed
// order of k_finalize, writes norm and coefficient and publishes the ready word.
//
// Why the last arriver sees every partial.  A partial is written by an agent-scope
// atomic store, which on this target is a write-through store that is acknowledged
// once it has reached the level at which the whole device is coherent; the storing
// wavefront then waits for that acknowledgement (vmcnt(0)) *before* the workgroup
// barrier, so when thread 0 counts the workgroup's arrival (after the barrier) all
// four partials of the chunk are visible to any agent-scope load.  Read-modify-write
// operations on arrived[b] are totally ordered; the workgroup whose increment makes the
// count complete therefore runs after every other arrival, hence after every partial
// of the bucket became visible, and its own loads of the partials (agent scope: they
// do not hit lines a per-XCD L2 may still hold from an earlier call) are issued only
// after its increment has returned.  A workgroup-scope release fence would not do: on
// this target it does not wait for vector stores, so the arrival could be counted
// while a partial is still on its way.
// The tail of every squared-norm item.  `stored` chunks' partials of bucket b have just been written by this
// workgroup (0: a bucket without elements, nothing to count): waits for them, counts the arrival, and if
// this workgroup completes the bucket, finalizes it and publishes the ready word.
__device__ __forceinline__ void norm_arrive(const StepState& st, uint32_t b, uint32_t stored, uint32_t epoch,
                                            const float* __restrict__ thresholds, float* __restrict__ norms,
                                            float* __restrict__ coefs, StepShared& sh) {
  const uint32_t tid = threadIdx.x;
  if (stored != 0) {
    wait_vmem();      // the partials have been acknowledged ...
    __syncthreads();  // ... for every wavefront of the workgroup
    if (tid == 0) {
      const uint32_t total = st.norm_bucket_off[b + 1] - st.norm_bucket_off[b];
      const uint32_t old = atomicAdd(&st.arrived[b], stored);
      const bool last = (old + stored == total);
      // nobody else touches the counter again in this call: leave it at zero for the next one
      if (last) ctl_store(&st.arrived[b], 0u);
      sh.flag = last ? 1u : 0u;
    }
    __syncthreads();
    if (!sh.flag) return;
  }
  // k_finalize's order: thread t adds partials lo + t, lo + t + 256, ... one after the other.  The loads are issued
  // eight at a time before the first addition (this workgroup is the one everybody else is waiting for, and an
  // agent-scope load that misses every cache takes a microsecond or two); a slot past the end adds +0.0, which
  // leaves a sum of squares as it is.
  const uint64_t lo = (uint64_t)st.norm_bucket_off[b] * kWaves, hi = (uint64_t)st.norm_bucket_off[b + 1] * kWaves;
  double s = 0.0;
  for (uint64_t i = lo + tid; i < hi; i += 8u * kBlock) {
    double part[8];
#pragma unroll
    for (uint32_t q = 0; q < 8u; ++q) {
      const uint64_t j = i + (uint64_t)q * kBlock;
      part[q] = j < hi ? __hip_atomic_load(&st.partials[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.0;
    }
#pragma unroll
    for (uint32_t q = 0; q < 8u; ++q) s += part[q];
  }
  s = wave_sum(s);
  if ((tid & 63u) == 0) sh.w[tid >> 6] = s;
  __syncthreads();
  if (tid == 0) {
    const double tot = ((sh.w[0] + sh.w[1]) + sh.w[2]) + sh.w[3];
    const float norm = (float)sqrt(tot);
    int32_t bst = 0;
    const float coef = clip_coef(norm, thresholds[b], bst);
    norms[b] = norm;
    coefs[b] = coef;
    if (bst) ctl_or(&st.ctl[kCtlStatus], (uint32_t)bst);
    // The coefficient travels inside the ready word, so a waiter needs nothing else that this item wrote.
    const unsigned long long word = ((unsigned long long)epoch << 32) | (unsigned long long)__float_as_uint(coef);
    __hip_atomic_store(&st.ready[b], word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

__device__ __forceinline__ void store_partial(const StepState& st, uint32_t chunk, double ws) {
  if ((threadIdx.x & 63u) == 0)
    __hip_atomic_store(&st.partials[(uint64_t)chunk * kWaves + (threadIdx.x >> 6)], ws, __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}

// A squared-norm item of k_step: `count` consecutive chunks of the norm table (all of one bucket), first
// chunk idx; or (kItemEmpty) the stand-in for bucket idx, which has no elements.  A chunk's partials are the
// same whichever item it was part of.
template <int GDT>
__device__ __forceinline__ void norm_item(const StepState& st, uint32_t kind, uint32_t idx, uint32_t count,
                                          uint32_t epoch, const float* __restrict__ thresholds,
                                          float* __restrict__ norms, float* __restrict__ coefs, StepShared& sh) {
  if (kind != kItemNorm) {
    norm_arrive(st, idx, 0u, epoch, thresholds, norms, coefs, sh);
    return;
  }
  uint32_t b = 0;
  for (uint32_t c = idx; c < idx + count; ++c) {
    const Entry en = read_entry(&st.norm_tab[c]);
    b = en.bucket;
    store_partial(st, c, sqnorm_chunk<GDT, false>(en));
  }
  norm_arrive(st, b, count, epoch, thresholds, norms, coefs, sh);
}

// What the items that wait for a coefficient do with it.
constexpr int kModeAdam = 0, kModeLamb = 1;

template <int GDT, bool WB, uint32_t U, int MODE>
__device__ __forceinline__ void apply_item(const StepState& st, const Entry& en, uint32_t idx, float coef,
                                           const AdamK& k, StepShared& sh) {
  if constexpr (MODE == kModeLamb)
    // LAMB's first sweep in place of Adam: moments and the chunk's two sums, filed under the chunk's place in
    // the tensor-major order; the trust ratio and the parameter update follow as launches of their own.
    lamb_moments_chunk<GDT, true, WB, false>(en, coef, k, sh.pp, sh.uu, st.lamb_sums + (uint64_t)st.apply_to_lamb[idx] * 2u);
  else
    adam_chunk<GDT, true, WB, U, false>(en, coef, k);
}

template <int GDT, bool WB, uint32_t U, bool TICKETS, bool LAMB>
__global__ __launch_bounds__(kBlock) void k_step(StepState st, const uint32_t* __restrict__ work, uint32_t n_work,
                                                  const float* __restrict__ thresholds, float* __restrict__ norms,
                                                  float* __restrict__ coefs, const AdamK ka) {
  __shared__ StepShared sh;
  const AdamK k = resolve(ka);
  uint32_t ticket;
  if constexpr (TICKETS) {
    // Eight ticket counters, one per XCD: item 8 t + y is the t-th item of list y.  A
    // workgroup draws from its own XCD's list and moves on to the next list when that
    // one is used up, so every list is started strictly in order and every item is
    // taken by exactly one of the n_work workgroups.
    if (threadIdx.x == 0) {
      const uint32_t xcc = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 7u;  // HW_REG_XCC_ID[3:0]
      uint32_t it = 0xffffffffu;
      for (uint32_t a = 0; a < 8u; ++a) {
        const uint32_t y = (xcc + a) & 7u;
        const uint32_t t = atomicAdd(&st.ctl[kCtlTicket + 32u * y], 1u);
        if ((uint64_t)t * 8u + y < n_work) {
          it = t * 8u + y;
          break;
        }
      }
      sh.item = it;
    }
    __syncthreads();
    ticket = sh.item;
  } else {
    ticket = blockIdx.x;
  }
  if (ticket >= n_work) return;
  const uint32_t epoch = st.ctl[kCtlEpoch];  // left by the previous call's finish kernel, constant during this launch
  const uint32_t item = work[ticket];
  const uint32_t kind = item >> 30;
  if (kind == kItemAdam) {
    const uint32_t idx = item & 0x3fffffffu;
    const Entry en = read_entry(&st.apply_tab[idx]);
    if (wait_for_bucket(st, en.bucket, epoch, idx, sh))
      apply_item<GDT, WB, U, LAMB ? kModeLamb : kModeAdam>(st, en, idx, sh.coef, k, sh);
  } else {
    // squared-norm items carry their chunk count (1 .. 4) in bits 28..29
    norm_item<GDT>(st, kind, item & 0x0fffffffu, ((item >> 28) & 3u) + 1u, epoch, thresholds, norms, coefs, sh);
  }
}

// g <- coef * g over one chunk of the squared-norm cut.  A full, 16-byte aligned chunk of kDefaultChunkNorm
// elements is fetched whole (every load in flight before the first store); anything else goes through scale_chunk.
// Element by element the stored value is the same either way.
template <int GDT>
__device__ __forceinline__ void scale_norm_chunk(const Entry& en, float coef) {
  typedef Grad<GDT> G;
  typedef typename G::wide wide;
  constexpr uint32_t R = kDefaultChunkNorm / (G::VE * kBlock);  // 128-bit pieces per lane: 16 (fp32) or 8 (16-bit types)
  if (en.len == kDefaultChunkNorm && (en.g & 15u) == 0) {
    wide* gw = reinterpret_cast<wide*>(en.g);
    const uint32_t tid = threadIdx.x;
    wide x[R];
#pragma unroll
    for (uint32_t u = 0; u < R; ++u) x[u] = ldv<false>(gw + tid + u * kBlock);
    loads_issued();
#pragma unroll
    for (uint32_t u = 0; u < R; ++u) {
      float f[G::VE];
      G::widen(x[u], f);
#pragma unroll
      for (uint32_t q = 0; q < G::VE; ++q) f[q] = f[q] * coef;
      stv<false>(gw + tid + u * kBlock, G::narrow(f));
    }
  } else {
    scale_chunk<GDT, 4, false>(en, coef);
  }
}

// The second of bucket_clip's two launches (the first is k_sqnorm over the range's chunks): one workgroup per
// squared-norm chunk.  Every workgroup adds up its bucket's partial sums itself, in k_finalize's order, so all of
// them arrive at the same norm and coefficient without exchanging anything (the partials of a 50 MiB bucket
// are 25 KB, read from L2 by every workgroup), and then scales its chunk; the workgroup of a bucket's first
// chunk also writes the bucket's norm and coefficient and ORs its status bits.  No workgroup waits for another.
// Workgroup 0 deals with the range's buckets that have no elements.
template <int GDT>
__global__ __launch_bounds__(kBlock) void k_clip_scale(const Chunk* __restrict__ norm_tab, uint32_t cn0, uint32_t n,
                                                        const uint32_t* __restrict__ bucket_chunk_off, uint32_t b0,
                                                        uint32_t b1, const double* __restrict__ partials,
                                                        const float* __restrict__ thresholds, float* __restrict__ norms,
                                                        float* __restrict__ coefs, int32_t* status) {
  __shared__ double s_w[kWaves];
  __shared__ float s_coef;
  const uint32_t tid = threadIdx.x;
  if (blockIdx.x == 0) {
    int32_t bst = 0;
    for (uint32_t b = b0 + tid; b < b1; b += kBlock) {
      if (bucket_chunk_off[b] == bucket_chunk_off[b + 1]) {
        norms[b] = 0.f;
        coefs[b] = clip_coef(0.f, thresholds[b], bst);
      }
    }
    if (bst != 0 && status != nullptr) atomicOr(status, bst);
  }
  if (blockIdx.x >= n) return;
  const uint32_t idx = cn0 + blockIdx.x;
  const Entry en = read_entry(&norm_tab[idx]);
  const uint32_t b = en.bucket;
  const double tot = sum_partials(partials, (uint64_t)bucket_chunk_off[b] * kWaves, (uint64_t)bucket_chunk_off[b + 1] * kWaves, s_w);
  if (tid == 0) {
    const float norm = (float)sqrt(tot);
    int32_t bst = 0;
    const float coef = clip_coef(norm, thresholds[b], bst);
    s_coef = coef;
    if (idx == bucket_chunk_off[b]) {
      norms[b] = norm;
      coefs[b] = coef;
      if (bst != 0 && status != nullptr) atomicOr(status, bst);
    }
  }
  __syncthreads();
  const float coef = s_coef;
  if (coef != 1.f) scale_norm_chunk<GDT>(en, coef);
}

// Follows every k_step launch on the stream; ONE workgroup, so that it costs a launch and one round trip to
// memory when there is nothing to do.  (1) Carries out the items whose wait expired (none, as a rule; one after
// the other if there are any -- an expired wait has cost about a second already), with the coefficient their
// bucket's ready word holds by now.  (2) Hands the status bits collected during the call to the caller and
// resets the per-call state, epoch included.
template <int GDT, bool WB, uint32_t U, int MODE>
__global__ __launch_bounds__(kBlock) void k_finish(StepState st, int32_t* status, const AdamK ka) {
  __shared__ StepShared sh;
  const uint32_t tid = threadIdx.x;
  const uint32_t epoch = ctl_load(&st.ctl[kCtlEpoch]);
  const uint32_t n_skipped = min(ctl_load(&st.ctl[kCtlSkipped]), st.skipped_cap);
  const uint32_t collected = ctl_load(&st.ctl[kCtlStatus]);  // complete: the launch that ORed into it has ended
  uint32_t bits = 0;
  if (n_skipped != 0) {
    const AdamK k = resolve(ka);
    for (uint32_t i = 0; i < n_skipped; ++i) {
      const uint32_t idx = st.skipped[i];
      const Entry en = read_entry(&st.apply_tab[idx]);
      const unsigned long long r = __hip_atomic_load(&st.ready[en.bucket], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if ((uint32_t)(r >> 32) != epoch) {  // cannot happen: squared-norm items never wait
        bits |= BCA_STATUS_INCOMPLETE;
        continue;
      }
      apply_item<GDT, WB, U, MODE>(st, en, idx, __uint_as_float((uint32_t)r), k, sh);
      __syncthreads();  // LAMB: sh.pp / sh.uu are reused by the next item
    }
  }
  if (tid == 0) {
    if (status != nullptr) *status = (int32_t)(collected | bits);
    ctl_store(&st.ctl[kCtlStatus], 0u);
    ctl_store(&st.ctl[kCtlSkipped], 0u);
    ctl_store(&st.ctl[kCtlAbort], 0u);
    for (uint32_t y = 0; y < 8u; ++y) ctl_store(&st.ctl[kCtlTicket + 32u * y], 0u);
    ctl_store(&st.ctl[kCtlEpoch], epoch + 1u == 0u ? 1u : epoch + 1u);
  }
}

// ---- clipping one contiguous bucket without a plan and without allocating ---------------
//
// For callers that cannot allocate (HIP graph capture, tight loops): the bucket is a
// pointer and a length, chunk bounds are computed from the chunk index instead of read
// from a table, and the partial sums live in a fixed array of this library's device
// image.  Two plain launches (squared norms; coefficient and scale; three for buckets of more than 16 Mi
// elements, whose coefficient gets a launch of its own) with the device functions
// of the plan-based path, so norm, coefficient and scaled gradients are those of
// bucket_clip on a one-tensor, one-bucket plan whose squared-norm chunk is kFlatChunkNorm.

constexpr uint32_t kFlatHeaderBytes = 256;  // one float: the coefficient of a large bucket, handed from its finalize launch to its scale launch
constexpr size_t kFlatScratchBytes = kFlatHeaderBytes + (size_t)(kFlatMaxElems / kFlatChunkNorm) * kWaves * sizeof(double);
static __device__ __align__(256) unsigned char scratch[kFlatScratchBytes];

__device__ __forceinline__ Entry flat_entry(uint64_t g, uint64_t n, uint32_t chunk_elems, uint32_t gsize, uint32_t i) {
  const uint64_t first = (uint64_t)i * chunk_elems;
  Entry e;
  e.g = g + first * gsize, e.p = 0, e.m = 0, e.v = 0;
  e.len = (uint32_t)(n - first < chunk_elems ? n - first : chunk_elems);
  e.bucket = 0, e.tensor = 0, e.flags = 0;
  return e;
}

template <int GDT>
__global__ __launch_bounds__(kBlock) void k_flat_sqnorm(uint64_t g, uint64_t n, double* __restrict__ partials) {
  const Entry en = flat_entry(g, n, kFlatChunkNorm, sizeof(typename Grad<GDT>::elem), blockIdx.x);
  const double ws = sqnorm_chunk<GDT, false, 16>(en);  // cacheable loads: the scale pass reads the bucket again at once
  if ((threadIdx.x & 63u) == 0) partials[(uint64_t)blockIdx.x * kWaves + (threadIdx.x >> 6)] = ws;
}

// Norm, coefficient and status of the bucket from its partial sums (whole workgroup; thread 0 writes the outputs
// if `write_outputs`).  Returns the coefficient to every thread.
__device__ __forceinline__ float flat_coef(const double* __restrict__ partials, uint32_t n_chunks,
                                           const float* __restrict__ threshold, float* norm_out, float* coef_out,
                                           int32_t* status, bool write_outputs, double* s_w, float* s_coef) {
  const double tot = sum_partials(partials, 0, (uint64_t)n_chunks * kWaves, s_w);
  if (threadIdx.x == 0) {
    const float norm = (float)sqrt(tot);
    int32_t st = 0;
    const float coef = clip_coef(norm, *threshold, st);
    *s_coef = coef;
    if (write_outputs) {
      if (norm_out != nullptr) *norm_out = norm;
      if (coef_out != nullptr) *coef_out = coef;
      if (status != nullptr) *status = st;  // written, not ORed
    }
  }
  __syncthreads();
  return *s_coef;
}

// Large buckets only (their partials are too many for every workgroup of the scale launch to add up): one
// workgroup derives the coefficient and leaves it in the scratch header.
__global__ __launch_bounds__(kBlock) void k_flat_finalize(const double* __restrict__ partials, uint32_t n_chunks,
                                                           const float* __restrict__ threshold, float* norm_out,
                                                           float* coef_out, int32_t* status, float* coef_header) {
  __shared__ double s_w[kWaves];
  __shared__ float s_coef;
  const float coef = flat_coef(partials, n_chunks, threshold, norm_out, coef_out, status, true, s_w, &s_coef);
  if (threadIdx.x == 0) *coef_header = coef;
}

// One workgroup per chunk of the squared-norm cut (one workgroup for an empty bucket).  coef_header == nullptr:
// every workgroup derives norm and coefficient from the partial sums itself, as in k_clip_scale, and workgroup 0
// writes the outputs; else the coefficient is read from there.  Then the chunk is scaled.
template <int GDT>
__global__ __launch_bounds__(kBlock) void k_flat_scale(uint64_t g, uint64_t n, uint32_t n_chunks,
                                                        const double* __restrict__ partials,
                                                        const float* __restrict__ threshold, float* norm_out,
                                                        float* coef_out, int32_t* status,
                                                        const float* __restrict__ coef_header) {
  __shared__ double s_w[kWaves];
  __shared__ float s_coef;
  const float coef = coef_header != nullptr
                         ? *coef_header
                         : flat_coef(partials, n_chunks, threshold, norm_out, coef_out, status, blockIdx.x == 0, s_w, &s_coef);
  if (coef == 1.f || blockIdx.x >= n_chunks) return;  // an unclipped bucket is not touched
  scale_norm_chunk<GDT>(flat_entry(g, n, kFlatChunkNorm, sizeof(typename Grad<GDT>::elem), blockIdx.x), coef);
}

// Plain device-to-device copy (16-byte pieces, then single bytes).  It exists so
// that hardware counters can be calibrated against a kernel whose HBM traffic is
// known exactly: nbytes read, nbytes written.
__global__ __launch_bounds__(kBlock) void k_copy(uint8_t* __restrict__ dst, const uint8_t* __restrict__ src,
                                                  uint64_t nbytes) {
  const uint64_t nvec = nbytes / 16u;
  const uint64_t stride = (uint64_t)gridDim.x * kBlock;
  for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < nvec; i += stride)
    reinterpret_cast<uint4*>(dst)[i] = reinterpret_cast<const uint4*>(src)[i];
  for (uint64_t i = nvec * 16u + (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < nbytes; i += stride) dst[i] = src[i];
}

// Compile-time variants are picked from run-time switches through these helpers.
template <typename F>
void pick2(bool a, bool b, F f) {
  if (a) {
    if (b) f(std::true_type{}, std::true_type{});
    else f(std::true_type{}, std::false_type{});
  } else {
    if (b) f(std::false_type{}, std::true_type{});
    else f(std::false_type{}, std::false_type{});
  }
}
template <typename F>
void pick_gdt(int gdt, F f) {
  if (gdt == BCA_GRAD_F32) f(std::integral_constant<int, BCA_GRAD_F32>{});
  else if (gdt == BCA_GRAD_F16) f(std::integral_constant<int, BCA_GRAD_F16>{});
  else f(std::integral_constant<int, BCA_GRAD_BF16>{});
}
template <typename F>
void pick_unroll(uint32_t u, F f) {
  if (u == 1) f(std::integral_constant<uint32_t, 1>{});
  else if (u == 2) f(std::integral_constant<uint32_t, 2>{});
  else f(std::integral_constant<uint32_t, 4>{});
}

}  // namespace

// ---- launchers --------------------------------------------------------------------

hipError_t launch_sqnorm(int gdt, const Chunk* table, uint32_t c0, uint32_t n, double* partials, int32_t* status,
                         const Launch& L, hipStream_t stream) {
  if (n == 0 && status == nullptr) return hipSuccess;  // with a status word the launch still has to clear it
  pick2(!L.g_keep, L.staged, [&](auto nt, auto st) {
    constexpr bool NT = decltype(nt)::value, ST = decltype(st)::value;
    pick_gdt(gdt, [&](auto gd) {
      constexpr int GDT = decltype(gd)::value;
      // a launch that does not fill the GPU (one bucket) keeps a whole 16 Ki chunk in flight per workgroup
      if (L.grid <= kSmallNormGrid)
        hipLaunchKernelGGL((k_sqnorm<GDT, NT, ST, 16>), dim3(L.grid), dim3(kBlock), 0, stream, table, c0, n, partials,
                           status);
      else
        hipLaunchKernelGGL((k_sqnorm<GDT, NT, ST, 8>), dim3(L.grid), dim3(kBlock), 0, stream, table, c0, n, partials,
                           status);
    });
  });
  return hipGetLastError();
}

hipError_t launch_copy(void* dst, const void* src, uint64_t nbytes, hipStream_t stream) {
  if (nbytes == 0) return hipSuccess;
  const uint64_t want = (nbytes / 16u + kBlock - 1) / kBlock;
  const uint32_t grid = (uint32_t)std::min<uint64_t>(std::max<uint64_t>(want, 1), 1u << 20);
  hipLaunchKernelGGL(k_copy, dim3(grid), dim3(kBlock), 0, stream, (uint8_t*)dst, (const uint8_t*)src, nbytes);
  return hipGetLastError();
}

hipError_t launch_clip_scale(int gdt, const Chunk* norm_tab, uint32_t cn0, uint32_t n, const uint32_t* bucket_chunk_off,
                             uint32_t b0, uint32_t b1, const double* partials, const float* thresholds, float* norms,
                             float* coefs, int32_t* status, hipStream_t stream) {
  pick_gdt(gdt, [&](auto gd) {
    hipLaunchKernelGGL((k_clip_scale<decltype(gd)::value>), dim3(std::max(n, 1u)), dim3(kBlock), 0, stream, norm_tab, cn0, n,
                       bucket_chunk_off, b0, b1, partials, thresholds, norms, coefs, status);
  });
  return hipGetLastError();
}

hipError_t launch_step(int gdt, const StepState& st, const uint32_t* work, uint32_t n_work, const float* thresholds,
                       float* norms, float* coefs, int32_t* status, bool write_back, const AdamK& k, uint32_t unroll,
                       bool tickets, bool lamb, hipEvent_t between, hipStream_t stream) {
  if (n_work != 0) {
    if (lamb) {  // one variant per gradient type and write-back setting: items by workgroup index, no unrolling
      pick_gdt(gdt, [&](auto gd) {
        constexpr int GDT = decltype(gd)::value;
        if (write_back)
          hipLaunchKernelGGL((k_step<GDT, true, 1, false, true>), dim3(n_work), dim3(kBlock), 0, stream, st, work, n_work,
                             thresholds, norms, coefs, k);
        else
          hipLaunchKernelGGL((k_step<GDT, false, 1, false, true>), dim3(n_work), dim3(kBlock), 0, stream, st, work, n_work,
                             thresholds, norms, coefs, k);
      });
    } else {
      pick_unroll(unroll, [&](auto uu) {
        constexpr uint32_t U = decltype(uu)::value;
        pick2(tickets, write_back, [&](auto tk, auto wb) {
          constexpr bool TK = decltype(tk)::value, WB = decltype(wb)::value;
          pick_gdt(gdt, [&](auto gd) {
            constexpr int GDT = decltype(gd)::value;
            hipLaunchKernelGGL((k_step<GDT, WB, U, TK, false>), dim3(n_work), dim3(kBlock), 0, stream, st, work, n_work,
                               thresholds, norms, coefs, k);
          });
        });
      });
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (between != nullptr) (void)hipEventRecord(between, stream);
  // the finish kernel: skipped items (same arithmetic whatever the unrolling, so one variant), status, next epoch
  pick2(lamb, write_back, [&](auto lm, auto wb) {
    constexpr bool LM = decltype(lm)::value, WB = decltype(wb)::value;
    pick_gdt(gdt, [&](auto gd) {
      constexpr int GDT = decltype(gd)::value;
      hipLaunchKernelGGL((k_finish<GDT, WB, 1, LM ? kModeLamb : kModeAdam>), dim3(1), dim3(kBlock), 0, stream, st, status,
                         k);
    });
  });
  return hipGetLastError();
}

hipError_t launch_finalize(const double* partials, const uint32_t* bucket_chunk_off, uint32_t b0, uint32_t b1,
                           const float* thresholds, float* norms, float* coefs, int32_t* status, double* bucket_sq,
                           hipStream_t stream) {
  if (b1 <= b0) return hipSuccess;
  hipLaunchKernelGGL(k_finalize, dim3(b1 - b0), dim3(kBlock), 0, stream, partials, bucket_chunk_off, b0, thresholds,
                     norms, coefs, status, bucket_sq);
  return hipGetLastError();
}

hipError_t launch_whole_coef(const double* bucket_sq, uint32_t n_buckets, const float* c, float* whole_norm,
                             float* coefs, int32_t* status, hipStream_t stream) {
  hipLaunchKernelGGL(k_whole_coef, dim3(1), dim3(kBlock), 0, stream, bucket_sq, n_buckets, c, whole_norm, coefs,
                     status);
  return hipGetLastError();
}

hipError_t launch_coefs(uint32_t b0, uint32_t b1, const float* thresholds, const float* norms, float* coefs,
                        int32_t* status, hipStream_t stream) {
  hipLaunchKernelGGL(k_coefs, dim3(1), dim3(kBlock), 0, stream, b0, b1, thresholds, norms, coefs, status);
  return hipGetLastError();
}

hipError_t launch_scale(int gdt, const Chunk* table, uint32_t c0, uint32_t n, const float* coefs, const Launch& L,
                        hipStream_t stream) {
  if (n == 0) return hipSuccess;
  // The scaled gradients are about to be read again (by the all-reduce or by Adam): plain stores.
  pick_unroll(L.unroll, [&](auto uu) {
    constexpr uint32_t U = decltype(uu)::value;
    pick_gdt(gdt, [&](auto gd) {
      constexpr int GDT = decltype(gd)::value;
      if (L.staged)
        hipLaunchKernelGGL((k_scale<GDT, U, false, true>), dim3(L.grid), dim3(kBlock), 0, stream, table, c0, n, coefs);
      else
        hipLaunchKernelGGL((k_scale<GDT, U, false, false>), dim3(L.grid), dim3(kBlock), 0, stream, table, c0, n, coefs);
    });
  });
  return hipGetLastError();
}

template <int GDT, uint32_t U, bool GNT, bool ST>
static void launch_adam_t(const Chunk* table, uint32_t c0, uint32_t n, const float* coefs, bool write_back,
                          const int32_t* skip_status, const AdamK& k, uint32_t grid, uint32_t lds, hipStream_t stream) {
  if (coefs == nullptr)
    hipLaunchKernelGGL((k_adam<GDT, false, false, U, GNT, ST>), dim3(grid), dim3(kBlock), lds, stream, table, c0, n,
                       coefs, skip_status, k);
  else if (!write_back)
    hipLaunchKernelGGL((k_adam<GDT, true, false, U, GNT, ST>), dim3(grid), dim3(kBlock), lds, stream, table, c0, n,
                       coefs, skip_status, k);
  else
    hipLaunchKernelGGL((k_adam<GDT, true, true, U, GNT, ST>), dim3(grid), dim3(kBlock), lds, stream, table, c0, n,
                       coefs, skip_status, k);
}

hipError_t launch_adam(int gdt, const Chunk* table, uint32_t c0, uint32_t n, const float* coefs, bool write_back,
                       const int32_t* skip_status, const AdamK& k, const Launch& L, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  pick_unroll(L.unroll, [&](auto uu) {
    constexpr uint32_t U = decltype(uu)::value;
    pick2(!L.g_keep, L.staged, [&](auto gnt, auto st) {
      constexpr bool GNT = decltype(gnt)::value, ST = decltype(st)::value;
      pick_gdt(gdt, [&](auto gd) {
        launch_adam_t<decltype(gd)::value, U, GNT, ST>(table, c0, n, coefs, write_back, skip_status, k, L.grid, L.lds,
                                                       stream);
      });
    });
  });
  return hipGetLastError();
}

hipError_t launch_lamb_moments(int gdt, const Chunk* table, uint32_t n, const float* coefs, bool write_back,
                               double* sums, bool keep, const AdamK& k, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  pick2(keep, write_back, [&](auto kp, auto wbk) {
    constexpr bool KEEP = decltype(kp)::value, WB = decltype(wbk)::value;
    pick_gdt(gdt, [&](auto gd) {
      constexpr int GDT = decltype(gd)::value;
      if (coefs == nullptr)
        hipLaunchKernelGGL((k_lamb_moments<GDT, false, false, KEEP>), dim3(n), dim3(kBlock), 0, stream, table, n, coefs, sums, k);
      else
        hipLaunchKernelGGL((k_lamb_moments<GDT, true, WB, KEEP>), dim3(n), dim3(kBlock), 0, stream, table, n, coefs, sums, k);
    });
  });
  return hipGetLastError();
}

hipError_t launch_hyper(const bca_adam_device* dev, AdamK* out, hipStream_t stream) {
  hipLaunchKernelGGL(k_hyper, dim3(1), dim3(64), 0, stream, dev, out);
  return hipGetLastError();
}

hipError_t launch_lamb_trust(const double* sums, const uint32_t* tensor_off, uint32_t n_tensors, const AdamK& k,
                             float* trust, float* scale, hipStream_t stream) {
  if (n_tensors == 0) return hipSuccess;
  hipLaunchKernelGGL(k_lamb_trust, dim3(n_tensors), dim3(kTrustBlock), 0, stream, sums, tensor_off, k, trust, scale);
  return hipGetLastError();
}

// Device address of `scratch` on each device, looked up once per device with that device current
// (every device holds its own copy of the array at its own address).  Host code never uses the
// array's name for anything else: as an expression it is a host-side stand-in, not a device address.
static void* g_flat_scratch[kFlatMaxDevices];
static hipError_t g_flat_scratch_err[kFlatMaxDevices];
static std::once_flag g_flat_scratch_once[kFlatMaxDevices];

hipError_t launch_clip_flat(int device, int gdt, void* g, uint64_t n, const float* threshold, float* norm, float* coef,
                            int32_t* status, hipStream_t stream) {
  std::call_once(g_flat_scratch_once[device], [device] {
    void* ptr = nullptr;
    g_flat_scratch_err[device] = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    g_flat_scratch[device] = g_flat_scratch_err[device] == hipSuccess ? ptr : nullptr;
  });
  if (g_flat_scratch_err[device] != hipSuccess) return g_flat_scratch_err[device];
  unsigned char* base = static_cast<unsigned char*>(g_flat_scratch[device]);
  if (base == nullptr) return hipErrorInvalidSymbol;
  float* coef_header = reinterpret_cast<float*>(base);
  double* partials = reinterpret_cast<double*>(base + kFlatHeaderBytes);
  const uint32_t n_norm = (uint32_t)((n + kFlatChunkNorm - 1) / kFlatChunkNorm);
  const uint64_t ga = (uint64_t)(uintptr_t)g;
  const bool large = n_norm > kMaxChunksForInlineFinalize;
  hipError_t e = hipSuccess;
  // Nothing in the scratch array has to start at zero: every partial (and the header) that a later kernel of the
  // call reads is written by an earlier kernel of this same call.
  if (n_norm != 0) {
    pick_gdt(gdt, [&](auto gd) {
      hipLaunchKernelGGL((k_flat_sqnorm<decltype(gd)::value>), dim3(n_norm), dim3(kBlock), 0, stream, ga, n, partials);
    });
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (large) {
    hipLaunchKernelGGL(k_flat_finalize, dim3(1), dim3(kBlock), 0, stream, partials, n_norm, threshold, norm, coef, status,
                       coef_header);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  pick_gdt(gdt, [&](auto gd) {
    hipLaunchKernelGGL((k_flat_scale<decltype(gd)::value>), dim3(std::max(n_norm, 1u)), dim3(kBlock), 0, stream, ga, n, n_norm,
                       partials, threshold, norm, coef, status, large ? coef_header : nullptr);
  });
  return hipGetLastError();
}

hipError_t launch_lamb_update(const Chunk* table, uint32_t n, const float* scale, const AdamK& k, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(k_lamb_update, dim3(n), dim3(kBlock), 0, stream, table, n, scale, k);
  return hipGetLastError();
}

}  // namespace bca

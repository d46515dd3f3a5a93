// HIP kernels for gfx950 (MI355X): squared-norm partials, per-bucket finalize,
// in-place scale, and the (optionally clip-fused) Adam sweep.
//
// All four streaming kernels are table driven: the host cuts the bucket layout
// into chunks (<= chunk_elems consecutive elements of one tensor in one bucket,
// bca_internal.h) and every workgroup of a persistent grid walks a static,
// interleaved share of that table (chunk c0 + w, c0 + w + G, ...), staging its
// entries in LDS.  Neighbouring workgroups therefore stream through
// neighbouring memory at the same time, and which workgroup handles a chunk
// never changes a result: a chunk's partial sum depends only on the chunk.
//
// Memory access: 128-bit loads/stores, lane-contiguous (a wavefront touches
// 1 KiB per instruction per array), several independent loads in flight per
// lane before first use.  A chunk whose arrays are not mutually 16-byte
// congruent falls back to element-wise access.  No MFMA: nothing here is a
// contraction; the path is bound by HBM bandwidth.
//
// Arithmetic follows the paper's definitions: clipping-by-norm (Sec. 2.3)
// applied per bucket (Sec. 4.2, Alg. 1) and Adam (Alg. 1, last line; Kingma &
// Ba with bias correction, decoupled weight decay).  Every fp32 operation is
// written as an explicit multiply or fma so that the fused and the unfused
// paths produce the same bits.

#include <hip/hip_runtime.h>

#include "bca_internal.h"

namespace bca {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// ---- chunk-table slice in LDS ------------------------------------------------

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

// ---- gradient access by storage type -----------------------------------------

template <int GDT>
struct Grad;

template <>
struct Grad<BCA_GRAD_F32> {
  typedef float elem;
  static __device__ __forceinline__ f32x4 load4(const void* base, uint32_t vec) {
    return reinterpret_cast<const f32x4*>(base)[vec];
  }
  static __device__ __forceinline__ void store4(void* base, uint32_t vec, f32x4 x) {
    reinterpret_cast<f32x4*>(base)[vec] = x;
  }
  static __device__ __forceinline__ float load1(const void* base, uint32_t i) {
    return reinterpret_cast<const float*>(base)[i];
  }
  static __device__ __forceinline__ void store1(void* base, uint32_t i, float x) {
    reinterpret_cast<float*>(base)[i] = x;
  }
};

template <>
struct Grad<BCA_GRAD_F16> {
  typedef _Float16 elem;
  // fp16 -> fp32 is exact (subnormals included); fp32 -> fp16 rounds to nearest even.
  static __device__ __forceinline__ f32x4 load4(const void* base, uint32_t vec) {
    const f16x4 h = reinterpret_cast<const f16x4*>(base)[vec];
    f32x4 r;
    r.x = (float)h.x, r.y = (float)h.y, r.z = (float)h.z, r.w = (float)h.w;
    return r;
  }
  static __device__ __forceinline__ void store4(void* base, uint32_t vec, f32x4 x) {
    f16x4 h;
    h.x = (_Float16)x.x, h.y = (_Float16)x.y, h.z = (_Float16)x.z, h.w = (_Float16)x.w;
    reinterpret_cast<f16x4*>(base)[vec] = h;
  }
  static __device__ __forceinline__ float load1(const void* base, uint32_t i) {
    return (float)reinterpret_cast<const _Float16*>(base)[i];
  }
  static __device__ __forceinline__ void store1(void* base, uint32_t i, float x) {
    reinterpret_cast<_Float16*>(base)[i] = (_Float16)x;
  }
};

// Number of leading elements to handle one by one so that what follows can be
// accessed as aligned vectors of `vec_elems` elements in every listed array, or
// `len` if no such head exists (mutually incongruent or misaligned addresses).
// g_addr uses gsize-byte elements, the fp32 arrays 4-byte elements.
__device__ __forceinline__ uint32_t vector_head(uint32_t len, uint64_t g_addr, uint32_t gsize, uint32_t g_vec_bytes,
                                                bool with_state, uint64_t p, uint64_t m, uint64_t v) {
  const uint32_t vec_elems = g_vec_bytes / gsize;
  // smallest h in [0, vec_elems) with (g_addr + h*gsize) % g_vec_bytes == 0
  const uint32_t mis = (uint32_t)(g_addr & (g_vec_bytes - 1));
  if (mis % gsize) return len;
  const uint32_t h = ((g_vec_bytes - mis) & (g_vec_bytes - 1)) / gsize;
  (void)vec_elems;
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

// One partial (fp64) per chunk: sum over the chunk of g^2.  Per lane the squares
// are accumulated in fp32 (four independent accumulators, at most
// chunk_elems/1024 terms each), then combined in fp64: lanes by butterfly
// shuffles, the four wavefronts through LDS in index order.
template <int GDT>
__global__ __launch_bounds__(kBlock) void k_sqnorm(const Chunk* __restrict__ table, uint32_t c0, uint32_t n,
                                                    double* __restrict__ partials, int32_t* status) {
  __shared__ Chunk s_tab[kSlice];
  __shared__ double s_part[kSlice][kWaves];
  typedef Grad<GDT> G;
  constexpr uint32_t gsize = sizeof(typename G::elem);
  constexpr uint32_t VE = 16u / gsize;  // elements per 128-bit load: 4 (fp32) or 8 (fp16)
  constexpr uint32_t U = 8;             // loads in flight per lane

  const uint32_t w = blockIdx.x, Gn = gridDim.x, tid = threadIdx.x;
  if (status != nullptr && w == 0 && tid == 0) *status = 0;  // finalize ORs into it later on this stream
  const uint32_t mine = my_chunk_count(n, w, Gn);

  for (uint32_t first = 0; first < mine; first += kSlice) {
    const uint32_t cnt = min(kSlice, mine - first);
    stage_slice(s_tab, table, c0, w, Gn, first, cnt);
    __syncthreads();
    for (uint32_t e = 0; e < cnt; ++e) {
      const uint64_t ga = s_tab[e].g;
      const uint32_t len = s_tab[e].len;
      const uint32_t head = vector_head(len, ga, gsize, 16u, false, 0, 0, 0);
      const uint32_t nvec = (len - head) / VE;
      const uint32_t tail0 = head + nvec * VE;
      const void* gbase = reinterpret_cast<const void*>(ga);
      const void* gv = reinterpret_cast<const void*>(ga + (uint64_t)head * gsize);
      float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;

      for (uint32_t base = 0; base < nvec; base += kBlock * U) {
        const uint32_t j0 = base + tid;
        if (base + kBlock * U <= nvec) {
          if constexpr (GDT == BCA_GRAD_F32) {
            f32x4 x[U];
#pragma unroll
            for (uint32_t u = 0; u < U; ++u) x[u] = reinterpret_cast<const f32x4*>(gv)[j0 + u * kBlock];
#pragma unroll
            for (uint32_t u = 0; u < U; ++u) {
              a0 = __fmaf_rn(x[u].x, x[u].x, a0), a1 = __fmaf_rn(x[u].y, x[u].y, a1);
              a2 = __fmaf_rn(x[u].z, x[u].z, a2), a3 = __fmaf_rn(x[u].w, x[u].w, a3);
            }
          } else {
            f16x8 x[U];
#pragma unroll
            for (uint32_t u = 0; u < U; ++u) x[u] = reinterpret_cast<const f16x8*>(gv)[j0 + u * kBlock];
#pragma unroll
            for (uint32_t u = 0; u < U; ++u) {
              const float f0 = (float)x[u][0], f1 = (float)x[u][1], f2 = (float)x[u][2], f3 = (float)x[u][3];
              const float f4 = (float)x[u][4], f5 = (float)x[u][5], f6 = (float)x[u][6], f7 = (float)x[u][7];
              a0 = __fmaf_rn(f0, f0, a0), a1 = __fmaf_rn(f1, f1, a1), a2 = __fmaf_rn(f2, f2, a2);
              a3 = __fmaf_rn(f3, f3, a3), a0 = __fmaf_rn(f4, f4, a0), a1 = __fmaf_rn(f5, f5, a1);
              a2 = __fmaf_rn(f6, f6, a2), a3 = __fmaf_rn(f7, f7, a3);
            }
          }
        } else {
          for (uint32_t u = 0; u < U; ++u) {
            const uint32_t j = j0 + u * kBlock;
            if (j < nvec) {
              if constexpr (GDT == BCA_GRAD_F32) {
                const f32x4 x = reinterpret_cast<const f32x4*>(gv)[j];
                a0 = __fmaf_rn(x.x, x.x, a0), a1 = __fmaf_rn(x.y, x.y, a1);
                a2 = __fmaf_rn(x.z, x.z, a2), a3 = __fmaf_rn(x.w, x.w, a3);
              } else {
                const f16x8 x = reinterpret_cast<const f16x8*>(gv)[j];
#pragma unroll
                for (int q = 0; q < 8; q += 4) {
                  const float f0 = (float)x[q], f1 = (float)x[q + 1], f2 = (float)x[q + 2], f3 = (float)x[q + 3];
                  a0 = __fmaf_rn(f0, f0, a0), a1 = __fmaf_rn(f1, f1, a1);
                  a2 = __fmaf_rn(f2, f2, a2), a3 = __fmaf_rn(f3, f3, a3);
                }
              }
            }
          }
        }
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
      const double ws = wave_sum(lane);
      if ((tid & 63u) == 0) s_part[e][tid >> 6] = ws;
    }
    __syncthreads();
    for (uint32_t e = tid; e < cnt; e += kBlock) {
      const uint64_t ci = (uint64_t)c0 + w + (uint64_t)(first + e) * Gn;
      partials[ci] = ((s_part[e][0] + s_part[e][1]) + s_part[e][2]) + s_part[e][3];
    }
    __syncthreads();
  }
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

// One wavefront per bucket: lanes take the bucket's partials in strides of 64 in
// fp64, then a butterfly.  Same order on every run, so norms are reproducible.
__global__ __launch_bounds__(kBlock) void k_finalize(const double* __restrict__ partials,
                                                      const uint32_t* __restrict__ bucket_chunk_off, uint32_t b0,
                                                      uint32_t b1, const float* __restrict__ thresholds,
                                                      float* __restrict__ norms, float* __restrict__ coefs,
                                                      int32_t* status) {
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t b = b0 + blockIdx.x * kWaves + (threadIdx.x >> 6);
  if (b >= b1) return;
  const uint32_t lo = bucket_chunk_off[b], hi = bucket_chunk_off[b + 1];
  double s = 0.0;
  for (uint32_t i = lo + lane; i < hi; i += 64u) s += partials[i];
  s = wave_sum(s);
  if (lane == 0) {
    const float norm = (float)sqrt(s);
    norms[b] = norm;
    if (thresholds != nullptr) {
      int32_t st = 0;
      const float coef = clip_coef(norm, thresholds[b], st);
      coefs[b] = coef;
      if (st != 0 && status != nullptr) atomicOr(status, st);
    }
  }
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

// G_b <- coef_b * G_b for clipped buckets (Alg. 1, the assignment under the if);
// buckets with coef_b == 1 are not read at all.
template <int GDT>
__global__ __launch_bounds__(kBlock) void k_scale(const Chunk* __restrict__ table, uint32_t c0, uint32_t n,
                                                   const float* __restrict__ coefs) {
  __shared__ Chunk s_tab[kSlice];
  typedef Grad<GDT> G;
  constexpr uint32_t gsize = sizeof(typename G::elem);
  constexpr uint32_t U = 4;
  const uint32_t w = blockIdx.x, Gn = gridDim.x, tid = threadIdx.x;
  const uint32_t mine = my_chunk_count(n, w, Gn);
  for (uint32_t first = 0; first < mine; first += kSlice) {
    const uint32_t cnt = min(kSlice, mine - first);
    stage_slice(s_tab, table, c0, w, Gn, first, cnt);
    __syncthreads();
    for (uint32_t e = 0; e < cnt; ++e) {
      const float coef = coefs[s_tab[e].bucket];
      if (coef == 1.f) continue;
      const uint64_t ga = s_tab[e].g;
      const uint32_t len = s_tab[e].len;
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
          for (uint32_t u = 0; u < U; ++u) x[u] = G::load4(gv, j0 + u * kBlock);
#pragma unroll
          for (uint32_t u = 0; u < U; ++u) G::store4(gv, j0 + u * kBlock, x[u] * coef);
        } else {
          for (uint32_t u = 0; u < U; ++u) {
            const uint32_t j = j0 + u * kBlock;
            if (j < nvec) G::store4(gv, j, G::load4(gv, j) * coef);
          }
        }
      }
      for (uint32_t i = tid; i < head; i += kBlock) G::store1(gbase, i, G::load1(gbase, i) * coef);
      for (uint32_t i = tail0 + tid; i < len; i += kBlock) G::store1(gbase, i, G::load1(gbase, i) * coef);
    }
    __syncthreads();
  }
}

// ---- Adam -----------------------------------------------------------------------

// One element of  theta <- ADAM(theta, eta, G)  (Alg. 1, last line):
//   m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2
//   p <- p - lr * ( mhat / (sqrt(vhat) + eps) + wd p ),  mhat = m/(1-b1^t), vhat = v/(1-b2^t)
// Division and square root are the correctly rounded ones.
__device__ __forceinline__ void adam1(float g, float& p, float& m, float& v, const AdamK& k) {
  m = __fmaf_rn(k.b1, m, k.omb1 * g);
  v = __fmaf_rn(k.b2, v, k.omb2 * (g * g));
  const float mhat = m * k.rbc1;
  const float vhat = v * k.rbc2;
  const float denom = __fsqrt_rn(vhat) + k.eps;
  const float upd = __fdiv_rn(mhat, denom);
  p = __fmaf_rn(k.neg_lr, __fmaf_rn(k.wd, p, upd), p);
}

__device__ __forceinline__ void adam4(f32x4 g, f32x4& p, f32x4& m, f32x4& v, const AdamK& k) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float pi = p[i], mi = m[i], vi = v[i];
    adam1(g[i], pi, mi, vi, k);
    p[i] = pi, m[i] = mi, v[i] = vi;
  }
}

// The read-modify-write sweep.  FUSED: ghat = coef_b * g is formed in registers
// (one fp32 multiply, so it equals what k_scale would have stored for fp32
// gradients); WB: ghat, rounded to the gradient type, also replaces g.
template <int GDT, bool FUSED, bool WB>
__global__ __launch_bounds__(kBlock) void k_adam(const Chunk* __restrict__ table, uint32_t c0, uint32_t n,
                                                  const float* __restrict__ coefs, const int32_t* skip_status,
                                                  const AdamK k) {
  __shared__ Chunk s_tab[kSlice];
  typedef Grad<GDT> G;
  constexpr uint32_t gsize = sizeof(typename G::elem);
  constexpr uint32_t U = 4;
  if (skip_status != nullptr && (*skip_status & BCA_STATUS_NONFINITE)) return;
  const uint32_t w = blockIdx.x, Gn = gridDim.x, tid = threadIdx.x;
  const uint32_t mine = my_chunk_count(n, w, Gn);
  for (uint32_t first = 0; first < mine; first += kSlice) {
    const uint32_t cnt = min(kSlice, mine - first);
    stage_slice(s_tab, table, c0, w, Gn, first, cnt);
    __syncthreads();
    for (uint32_t e = 0; e < cnt; ++e) {
      const uint64_t ga = s_tab[e].g, pa = s_tab[e].p, ma = s_tab[e].m, va = s_tab[e].v;
      const uint32_t len = s_tab[e].len;
      float coef = 1.f;
      if constexpr (FUSED) coef = coefs[s_tab[e].bucket];
      const bool wb = WB && coef != 1.f;
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
          for (uint32_t u = 0; u < U; ++u) g[u] = G::load4(gv, j0 + u * kBlock);
#pragma unroll
          for (uint32_t u = 0; u < U; ++u) p[u] = pv[j0 + u * kBlock];
#pragma unroll
          for (uint32_t u = 0; u < U; ++u) m[u] = mv[j0 + u * kBlock];
#pragma unroll
          for (uint32_t u = 0; u < U; ++u) v[u] = vv[j0 + u * kBlock];
#pragma unroll
          for (uint32_t u = 0; u < U; ++u) {
            if constexpr (FUSED) g[u] = g[u] * coef;
            adam4(g[u], p[u], m[u], v[u], k);
            const uint32_t j = j0 + u * kBlock;
            pv[j] = p[u], mv[j] = m[u], vv[j] = v[u];
            if (wb) G::store4(gv, j, g[u]);
          }
        } else {
          for (uint32_t u = 0; u < U; ++u) {
            const uint32_t j = j0 + u * kBlock;
            if (j < nvec) {
              f32x4 g = G::load4(gv, j), p = pv[j], m = mv[j], v = vv[j];
              if constexpr (FUSED) g = g * coef;
              adam4(g, p, m, v, k);
              pv[j] = p, mv[j] = m, vv[j] = v;
              if (wb) G::store4(gv, j, g);
            }
          }
        }
      }
      // head and tail, element-wise
      void* gbase = reinterpret_cast<void*>(ga);
      float* p1 = reinterpret_cast<float*>(pa);
      float* m1 = reinterpret_cast<float*>(ma);
      float* v1 = reinterpret_cast<float*>(va);
      for (uint32_t r = tid; r < head + (len - tail0); r += kBlock) {
        const uint32_t i = r < head ? r : tail0 + (r - head);
        float g = G::load1(gbase, i), p = p1[i], m = m1[i], v = v1[i];
        if constexpr (FUSED) g = g * coef;
        adam1(g, p, m, v, k);
        p1[i] = p, m1[i] = m, v1[i] = v;
        if (wb) G::store1(gbase, i, g);
      }
    }
    __syncthreads();
  }
}

}  // namespace

// ---- launchers --------------------------------------------------------------------

hipError_t launch_sqnorm(int gdt, const Chunk* table, uint32_t c0, uint32_t n, double* partials, int32_t* status,
                         uint32_t grid, hipStream_t stream) {
  if (n == 0 && status == nullptr) return hipSuccess;  // with a status word the launch still has to clear it
  if (gdt == BCA_GRAD_F32)
    hipLaunchKernelGGL(k_sqnorm<BCA_GRAD_F32>, dim3(grid), dim3(kBlock), 0, stream, table, c0, n, partials, status);
  else
    hipLaunchKernelGGL(k_sqnorm<BCA_GRAD_F16>, dim3(grid), dim3(kBlock), 0, stream, table, c0, n, partials, status);
  return hipGetLastError();
}

hipError_t launch_finalize(const double* partials, const uint32_t* bucket_chunk_off, uint32_t b0, uint32_t b1,
                           const float* thresholds, float* norms, float* coefs, int32_t* status,
                           hipStream_t stream) {
  if (b1 <= b0) return hipSuccess;
  const uint32_t grid = (b1 - b0 + kWaves - 1) / kWaves;
  hipLaunchKernelGGL(k_finalize, dim3(grid), dim3(kBlock), 0, stream, partials, bucket_chunk_off, b0, b1, thresholds,
                     norms, coefs, status);
  return hipGetLastError();
}

hipError_t launch_coefs(uint32_t b0, uint32_t b1, const float* thresholds, const float* norms, float* coefs,
                        int32_t* status, hipStream_t stream) {
  hipLaunchKernelGGL(k_coefs, dim3(1), dim3(kBlock), 0, stream, b0, b1, thresholds, norms, coefs, status);
  return hipGetLastError();
}

hipError_t launch_scale(int gdt, const Chunk* table, uint32_t c0, uint32_t n, const float* coefs, uint32_t grid,
                        hipStream_t stream) {
  if (n == 0) return hipSuccess;
  if (gdt == BCA_GRAD_F32)
    hipLaunchKernelGGL(k_scale<BCA_GRAD_F32>, dim3(grid), dim3(kBlock), 0, stream, table, c0, n, coefs);
  else
    hipLaunchKernelGGL(k_scale<BCA_GRAD_F16>, dim3(grid), dim3(kBlock), 0, stream, table, c0, n, coefs);
  return hipGetLastError();
}

template <int GDT>
static hipError_t launch_adam_t(const Chunk* table, uint32_t c0, uint32_t n, const float* coefs, bool write_back,
                                const int32_t* skip_status, const AdamK& k, uint32_t grid, hipStream_t stream) {
  if (coefs == nullptr)
    hipLaunchKernelGGL((k_adam<GDT, false, false>), dim3(grid), dim3(kBlock), 0, stream, table, c0, n, coefs,
                       skip_status, k);
  else if (!write_back)
    hipLaunchKernelGGL((k_adam<GDT, true, false>), dim3(grid), dim3(kBlock), 0, stream, table, c0, n, coefs,
                       skip_status, k);
  else
    hipLaunchKernelGGL((k_adam<GDT, true, true>), dim3(grid), dim3(kBlock), 0, stream, table, c0, n, coefs,
                       skip_status, k);
  return hipGetLastError();
}

hipError_t launch_adam(int gdt, const Chunk* table, uint32_t c0, uint32_t n, const float* coefs, bool write_back,
                       const int32_t* skip_status, const AdamK& k, uint32_t grid, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  return gdt == BCA_GRAD_F32 ? launch_adam_t<BCA_GRAD_F32>(table, c0, n, coefs, write_back, skip_status, k, grid, stream)
                             : launch_adam_t<BCA_GRAD_F16>(table, c0, n, coefs, write_back, skip_status, k, grid, stream);
}

}  // namespace bca

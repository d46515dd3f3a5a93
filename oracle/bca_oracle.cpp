// CPU oracle for bucket-wise gradient clipping followed by Adam.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, single-threaded
// fp64 statement of what the path computes.  Only tests, the smoke check and
// the benchmark's cpu_baseline leg may call it; the product (the HIP library)
// never does, and the two share no code.
//
// What is computed, and where the paper defines it:
//   * clipping-by-norm (Sec. 2.3, the unnumbered equation): if ||g|| >= c then
//     g <- c * g / ||g||.  The norm is read as the Euclidean norm.
//   * bucket-wise application (Sec. 4.2 and Alg. 1 of App. B): the rule is
//     applied to each gradient bucket G_b on its own, with the threshold the
//     caller passes for that bucket (Alg. 1 uses c / sqrt(B) for every b; that
//     choice is the caller's, see orc_alg1_threshold below).
//   * theta <- ADAM(theta, eta, G) after the bucket loop (Alg. 1, last line).
//     The paper does not restate Adam; it tunes lr, beta1, beta2, eps and
//     weight decay (App. A, Table 4).  This file takes Adam as published by
//     Kingma & Ba (Alg. 1 there, with bias correction, eps added to the
//     square root of the corrected second moment) and weight decay in its
//     decoupled form:  p <- p - lr * ( mhat / (sqrt(vhat) + eps) + wd * p ).
//
//   * variants the paper weighs against plain Adam (Sec. 2.2, Sec. 5, App. A): a
//     per-tensor weight-decay mask (decay only where the mask says so), bfloat16
//     gradient storage, and LAMB (You et al. 2020, Alg. 2: Adam's direction with
//     a per-tensor trust ratio ||p|| / ||update||).  The paper only names these;
//     the definitions used are the published ones, restated at each function.
//
// Inputs keep the bit patterns the GPU receives (fp32, fp16 or bf16 gradients, fp32
// thresholds); every value is widened exactly to double before use.  State
// (p, m, v) is held in double by the caller so that multi-step runs accumulate
// no fp32 rounding on the oracle's side.
//
// Parity pins: every function here is pinned by tests/test_oracle_*.py against
// closed forms, invariants, brute force and library routines (orc_compare_f32, the
// acceptance rule of the GPU tests, by tests/test_oracle_compare.py).  Non-finite
// gradients get no special case beyond the status bit and the skip mode: what
// propagates from them is what IEEE arithmetic gives for the formulas as written
// (an Inf makes the norm Inf and the coefficient 0, a NaN makes the comparison with
// the threshold false and the coefficient 1), pinned in tests/test_oracle_adam.py.

#include <cmath>
#include <cstdint>
#include <cstring>

namespace {

// ---- IEEE binary16 <-> wider types, written from the format's definition ----

double half_bits_to_double(uint16_t h) {
  const int sign = (h >> 15) & 1;
  const int expo = (h >> 10) & 0x1f;
  const int frac = h & 0x3ff;
  double mag;
  if (expo == 0) {
    mag = std::ldexp(static_cast<double>(frac), -24);            // subnormal: frac * 2^-24
  } else if (expo == 31) {
    mag = frac ? std::nan("") : INFINITY;
  } else {
    mag = std::ldexp(static_cast<double>(1024 + frac), expo - 25);  // (1 + frac/1024) * 2^(expo-15)
  }
  return sign ? -mag : mag;
}

// Round a float to the nearest binary16, ties to even.
uint16_t float_to_half_bits(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  const uint16_t sign = static_cast<uint16_t>((u >> 16) & 0x8000u);
  if (std::isnan(f)) return sign | 0x7e00u;
  const double a = std::fabs(static_cast<double>(f));
  if (a >= 65520.0) return sign | 0x7c00u;            // at or past the midpoint above the largest finite half
  if (a == 0.0) return sign;
  int e;
  std::frexp(a, &e);                                   // a = x * 2^e, x in [0.5, 1)
  int ulp_exp = e - 11;                                // 11 significant bits for normal halves
  if (ulp_exp < -24) ulp_exp = -24;                    // subnormal spacing
  const double q = std::ldexp(a, -ulp_exp);            // a in units of its ulp, exact
  const double r = std::nearbyint(q);                  // default rounding mode: ties to even
  const double rounded = std::ldexp(r, ulp_exp);
  // re-encode
  if (rounded == 0.0) return sign;
  int e2;
  const double x2 = std::frexp(rounded, &e2);          // rounded = x2 * 2^e2
  const int biased = e2 - 1 + 15;
  if (biased <= 0) {
    const int frac = static_cast<int>(std::ldexp(rounded, 24));
    return sign | static_cast<uint16_t>(frac);
  }
  if (biased >= 31) return sign | 0x7c00u;
  const int frac = static_cast<int>(std::ldexp(x2, 11)) - 1024;
  return sign | static_cast<uint16_t>((biased << 10) | frac);
}

// ---- bfloat16 (1 sign, 8 exponent, 7 fraction bits: the upper half of a binary32) ----

double bf16_bits_to_double(uint16_t h) {
  const int sign = (h >> 15) & 1;
  const int expo = (h >> 7) & 0xff;
  const int frac = h & 0x7f;
  double mag;
  if (expo == 0) {
    mag = std::ldexp(static_cast<double>(frac), -133);            // subnormal: frac * 2^-7 * 2^-126
  } else if (expo == 255) {
    mag = frac ? std::nan("") : INFINITY;
  } else {
    mag = std::ldexp(static_cast<double>(128 + frac), expo - 134);  // (1 + frac/128) * 2^(expo-127)
  }
  return sign ? -mag : mag;
}

// Round a float to the nearest bfloat16, ties to even.
uint16_t float_to_bf16_bits(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  const uint16_t sign = static_cast<uint16_t>((u >> 16) & 0x8000u);
  if (std::isnan(f)) return sign | 0x7fc0u;
  const double a = std::fabs(static_cast<double>(f));
  if (std::isinf(a)) return sign | 0x7f80u;
  if (a == 0.0) return sign;
  int e;
  std::frexp(a, &e);                                   // a = x * 2^e, x in [0.5, 1)
  int ulp_exp = e - 8;                                 // 8 significant bits for normal values
  if (ulp_exp < -133) ulp_exp = -133;                  // subnormal spacing
  const double r = std::nearbyint(std::ldexp(a, -ulp_exp));   // ties to even in the default rounding mode
  const double rounded = std::ldexp(r, ulp_exp);
  if (rounded == 0.0) return sign;
  int e2;
  const double x2 = std::frexp(rounded, &e2);          // rounded = x2 * 2^e2
  const int biased = e2 - 1 + 127;
  if (biased <= 0) return sign | static_cast<uint16_t>(static_cast<int>(std::ldexp(rounded, 133)));
  if (biased >= 255) return sign | 0x7f80u;            // rounded past the largest finite value
  const int frac = static_cast<int>(std::ldexp(x2, 8)) - 128;
  return sign | static_cast<uint16_t>((biased << 7) | frac);
}

enum { GRAD_F32 = 0, GRAD_F16 = 1, GRAD_BF16 = 2 };

inline double load_grad(const void* base, int gdt, uint64_t i) {
  if (gdt == GRAD_F32) return static_cast<double>(static_cast<const float*>(base)[i]);
  if (gdt == GRAD_BF16) return bf16_bits_to_double(static_cast<const uint16_t*>(base)[i]);
  return half_bits_to_double(static_cast<const uint16_t*>(base)[i]);
}

// The scaled gradient as a value of the gradient's storage type.  The product
// of the fp32 coefficient and the stored gradient is formed in fp32 (exactly
// the correctly rounded product, since the double product of two floats is
// exact) and, for fp16 storage, rounded once more to fp16: the decision which
// fp16 value is stored is taken in the precision the kernel works in.  The same
// holds for bf16 storage.
inline void store_scaled_grad(void* base, int gdt, uint64_t i, float coef) {
  if (gdt == GRAD_F32) {
    float* g = static_cast<float*>(base);
    g[i] = static_cast<float>(static_cast<double>(coef) * static_cast<double>(g[i]));
  } else if (gdt == GRAD_BF16) {
    uint16_t* g = static_cast<uint16_t*>(base);
    const float prod = static_cast<float>(static_cast<double>(coef) * bf16_bits_to_double(g[i]));
    g[i] = float_to_bf16_bits(prod);
  } else {
    uint16_t* g = static_cast<uint16_t*>(base);
    const float prod = static_cast<float>(static_cast<double>(coef) * half_bits_to_double(g[i]));
    g[i] = float_to_half_bits(prod);
  }
}

struct Adam {
  double lr, beta1, beta2, eps, wd;
};

// One Adam update of one element (Kingma & Ba Alg. 1 + decoupled decay).
// `t` is the number of updates made so far including this one.
inline void adam_element(double g, double& p, double& m, double& v, const Adam& h, double bc1, double bc2) {
  m = h.beta1 * m + (1.0 - h.beta1) * g;
  v = h.beta2 * v + (1.0 - h.beta2) * g * g;
  const double mhat = m / bc1;
  const double vhat = v / bc2;
  p = p - h.lr * (mhat / (std::sqrt(vhat) + h.eps) + h.wd * p);
}

// Hyper-parameters as they apply to tensor t: with a decay mask (one byte per
// tensor, null = decay everywhere) weight decay acts only on tensors whose byte
// is non-zero (the usual exemption of biases and normalisation weights).
inline Adam for_tensor(const Adam& all, const uint8_t* decay, uint32_t t) {
  Adam h = all;
  if (decay != nullptr && decay[t] == 0) h.wd = 0.0;
  return h;
}

// LAMB on one tensor of n elements (You et al. 2020, Alg. 2, with Adam's bias
// correction and phi = identity):
//   m, v, mhat, vhat as in Adam;  u_i = mhat_i / (sqrt(vhat_i) + eps) + wd * p_i
//   trust = ||p|| / ||u||  (Euclidean norms over the tensor, p before the update;
//           1 if either norm is zero, where the quotient has no meaning)
//   p_i <- p_i - lr * trust * u_i
// g[i] is the gradient Adam sees (already scaled when clipping came first).
// Returns the trust ratio.
double lamb_tensor(uint64_t n, const double* g, double* p, double* m, double* v, const Adam& h, double bc1,
                   double bc2) {
  double* u = new double[n ? n : 1];
  double sum_pp = 0.0, sum_uu = 0.0;
  for (uint64_t i = 0; i < n; ++i) {
    m[i] = h.beta1 * m[i] + (1.0 - h.beta1) * g[i];
    v[i] = h.beta2 * v[i] + (1.0 - h.beta2) * g[i] * g[i];
    const double mhat = m[i] / bc1;
    const double vhat = v[i] / bc2;
    u[i] = mhat / (std::sqrt(vhat) + h.eps) + h.wd * p[i];
    sum_pp += p[i] * p[i];
    sum_uu += u[i] * u[i];
  }
  const double p_norm = std::sqrt(sum_pp), u_norm = std::sqrt(sum_uu);
  const double trust = (p_norm > 0.0 && u_norm > 0.0) ? p_norm / u_norm : 1.0;
  for (uint64_t i = 0; i < n; ++i) p[i] = p[i] - h.lr * trust * u[i];
  delete[] u;
  return trust;
}

}  // namespace

extern "C" {

// status bits shared by the calls below
enum { ORC_STATUS_NONFINITE = 1, ORC_STATUS_BAD_THRESHOLD = 2 };

double orc_half_to_double(uint16_t h) { return half_bits_to_double(h); }
uint16_t orc_float_to_half(float f) { return float_to_half_bits(f); }
double orc_bf16_to_double(uint16_t h) { return bf16_bits_to_double(h); }
uint16_t orc_float_to_bf16(float f) { return float_to_bf16_bits(f); }

// Alg. 1: every bucket is compared against c / sqrt(B).
double orc_alg1_threshold(double c, uint64_t n_buckets) { return c / std::sqrt(static_cast<double>(n_buckets)); }

// ||G_b|| for every bucket: the square root of the sum of squares over the
// bucket's segments, taken in the order given.
void orc_bucket_norms(uint32_t n_buckets, const uint64_t* bucket_seg_off, const uint32_t* seg_tensor,
                      const uint64_t* seg_begin, const uint64_t* seg_len, const void* const* grads, int gdt,
                      double* norms) {
  for (uint32_t b = 0; b < n_buckets; ++b) {
    double s = 0.0;
    for (uint64_t k = bucket_seg_off[b]; k < bucket_seg_off[b + 1]; ++k) {
      const void* g = grads[seg_tensor[k]];
      for (uint64_t i = seg_begin[k]; i < seg_begin[k] + seg_len[k]; ++i) {
        const double x = load_grad(g, gdt, i);
        s += x * x;
      }
    }
    norms[b] = std::sqrt(s);
  }
}

// Clip coefficient of every bucket: c_b / ||G_b|| if ||G_b|| >= c_b, else 1
// (Sec. 2.3).  A zero norm is below any valid threshold, so nothing divides by
// zero.  The coefficient is rounded once to fp32; that fp32 value is what
// multiplies the gradient everywhere below.  A threshold that is not a
// positive number means "do not clip" and raises ORC_STATUS_BAD_THRESHOLD; a
// non-finite norm raises ORC_STATUS_NONFINITE.  Returns the OR of the bits.
int32_t orc_clip_coefs(uint32_t n_buckets, const double* norms, const float* thresholds, float* coefs) {
  int32_t status = 0;
  for (uint32_t b = 0; b < n_buckets; ++b) {
    const double c = static_cast<double>(thresholds[b]);
    const double n = norms[b];
    if (!std::isfinite(n)) status |= ORC_STATUS_NONFINITE;
    double coef = 1.0;
    if (!(c > 0.0)) {
      status |= ORC_STATUS_BAD_THRESHOLD;
    } else if (n >= c) {
      coef = c / n;
    }
    coefs[b] = static_cast<float>(coef);
  }
  return status;
}

// G_b <- coef_b * G_b in place, in the gradient's storage type (Alg. 1, the
// assignment inside the if).  Buckets whose coefficient is exactly 1 are left
// untouched bit for bit.
void orc_bucket_scale(uint32_t n_buckets, const uint64_t* bucket_seg_off, const uint32_t* seg_tensor,
                      const uint64_t* seg_begin, const uint64_t* seg_len, void* const* grads, int gdt,
                      const float* coefs) {
  for (uint32_t b = 0; b < n_buckets; ++b) {
    if (coefs[b] == 1.0f) continue;
    for (uint64_t k = bucket_seg_off[b]; k < bucket_seg_off[b + 1]; ++k) {
      void* g = grads[seg_tensor[k]];
      for (uint64_t i = seg_begin[k]; i < seg_begin[k] + seg_len[k]; ++i) store_scaled_grad(g, gdt, i, coefs[b]);
    }
  }
}

// theta <- ADAM(theta, eta, G) over whole tensors, reading the gradients as
// stored (Alg. 1, last line).  step >= 1 counts this update.  decay (may be
// null) is the per-tensor weight-decay mask.
void orc_adam_step(uint32_t n_tensors, const uint64_t* tensor_numel, const void* const* grads, int gdt,
                   double* const* p, double* const* m, double* const* v, double lr, double beta1, double beta2,
                   double eps, double wd, uint64_t step, const uint8_t* decay) {
  const Adam h_all{lr, beta1, beta2, eps, wd};
  const double bc1 = 1.0 - std::pow(beta1, static_cast<double>(step));
  const double bc2 = 1.0 - std::pow(beta2, static_cast<double>(step));
  for (uint32_t t = 0; t < n_tensors; ++t) {
    const Adam h = for_tensor(h_all, decay, t);
    for (uint64_t i = 0; i < tensor_numel[t]; ++i)
      adam_element(load_grad(grads[t], gdt, i), p[t][i], m[t][i], v[t][i], h, bc1, bc2);
  }
}

// The fused step: per-bucket norm and coefficient, then Adam on
// ghat = coef_b * g formed in working precision (not rounded to the storage
// type).  With write_back the storage-rounded ghat also replaces g, as Alg. 1
// needs before the all-reduce.  With skip_on_nonfinite a non-finite bucket
// norm leaves g, p, m and v untouched.  norms and coefs (either may be null)
// receive the per-bucket values.  decay (may be null) is the per-tensor
// weight-decay mask.  Returns the status bits.
int32_t orc_bucket_clip_adam(uint32_t n_buckets, const uint64_t* bucket_seg_off, const uint32_t* seg_tensor,
                             const uint64_t* seg_begin, const uint64_t* seg_len, void* const* grads, int gdt,
                             double* const* p, double* const* m, double* const* v, const float* thresholds,
                             double lr, double beta1, double beta2, double eps, double wd, uint64_t step,
                             int write_back, int skip_on_nonfinite, double* norms_out, float* coefs_out,
                             const uint8_t* decay) {
  double* norms = new double[n_buckets ? n_buckets : 1];
  float* coefs = new float[n_buckets ? n_buckets : 1];
  orc_bucket_norms(n_buckets, bucket_seg_off, seg_tensor, seg_begin, seg_len, grads, gdt, norms);
  const int32_t status = orc_clip_coefs(n_buckets, norms, thresholds, coefs);
  if (norms_out) std::memcpy(norms_out, norms, sizeof(double) * n_buckets);
  if (coefs_out) std::memcpy(coefs_out, coefs, sizeof(float) * n_buckets);

  if (!(skip_on_nonfinite && (status & ORC_STATUS_NONFINITE))) {
    const Adam h_all{lr, beta1, beta2, eps, wd};
    const double bc1 = 1.0 - std::pow(beta1, static_cast<double>(step));
    const double bc2 = 1.0 - std::pow(beta2, static_cast<double>(step));
    for (uint32_t b = 0; b < n_buckets; ++b) {
      const double coef = static_cast<double>(coefs[b]);
      for (uint64_t k = bucket_seg_off[b]; k < bucket_seg_off[b + 1]; ++k) {
        const uint32_t t = seg_tensor[k];
        const Adam h = for_tensor(h_all, decay, t);
        for (uint64_t i = seg_begin[k]; i < seg_begin[k] + seg_len[k]; ++i) {
          const double ghat = coef * load_grad(grads[t], gdt, i);
          adam_element(ghat, p[t][i], m[t][i], v[t][i], h, bc1, bc2);
          if (write_back && coefs[b] != 1.0f) store_scaled_grad(grads[t], gdt, i, coefs[b]);
        }
      }
    }
  }
  delete[] norms;
  delete[] coefs;
  return status;
}

// Whole-gradient clipping, the two baselines the paper compares with (Sec. 3.2:
// clipping after or before the all-reduce, which coincide on one GPU): the
// clipping-by-norm rule of Sec. 2.3 applied once to the concatenation of all
// buckets with the single threshold c, then Adam on the scaled gradient formed
// in working precision.  norms_out (may be null) receives the per-bucket norms,
// *whole_norm_out the norm of the whole gradient, *coef_out the one coefficient.
int32_t orc_whole_clip_adam(uint32_t n_buckets, const uint64_t* bucket_seg_off, const uint32_t* seg_tensor,
                            const uint64_t* seg_begin, const uint64_t* seg_len, void* const* grads, int gdt,
                            double* const* p, double* const* m, double* const* v, float threshold, double lr,
                            double beta1, double beta2, double eps, double wd, uint64_t step, int write_back,
                            double* norms_out, double* whole_norm_out, float* coef_out, const uint8_t* decay) {
  double total = 0.0;
  for (uint32_t b = 0; b < n_buckets; ++b) {
    double s = 0.0;
    for (uint64_t k = bucket_seg_off[b]; k < bucket_seg_off[b + 1]; ++k)
      for (uint64_t i = seg_begin[k]; i < seg_begin[k] + seg_len[k]; ++i) {
        const double x = load_grad(grads[seg_tensor[k]], gdt, i);
        s += x * x;
      }
    if (norms_out) norms_out[b] = std::sqrt(s);
    total += s;
  }
  const double whole = std::sqrt(total);
  float coef = 1.0f;
  const int32_t status = orc_clip_coefs(1, &whole, &threshold, &coef);
  if (whole_norm_out) *whole_norm_out = whole;
  if (coef_out) *coef_out = coef;
  const Adam h_all{lr, beta1, beta2, eps, wd};
  const double bc1 = 1.0 - std::pow(beta1, static_cast<double>(step));
  const double bc2 = 1.0 - std::pow(beta2, static_cast<double>(step));
  for (uint32_t b = 0; b < n_buckets; ++b)
    for (uint64_t k = bucket_seg_off[b]; k < bucket_seg_off[b + 1]; ++k) {
      const uint32_t t = seg_tensor[k];
      const Adam h = for_tensor(h_all, decay, t);
      for (uint64_t i = seg_begin[k]; i < seg_begin[k] + seg_len[k]; ++i) {
        const double ghat = static_cast<double>(coef) * load_grad(grads[t], gdt, i);
        adam_element(ghat, p[t][i], m[t][i], v[t][i], h, bc1, bc2);
        if (write_back && coef != 1.0f) store_scaled_grad(grads[t], gdt, i, coef);
      }
    }
  return status;
}

// LAMB over whole tensors on the stored gradients (the optimizer the paper
// compares Adam with, Sec. 2.2 and Sec. 5; definition at lamb_tensor above).
// trust_out (may be null) receives one ratio per tensor.
void orc_lamb_step(uint32_t n_tensors, const uint64_t* tensor_numel, const void* const* grads, int gdt,
                   double* const* p, double* const* m, double* const* v, double lr, double beta1, double beta2,
                   double eps, double wd, uint64_t step, const uint8_t* decay, double* trust_out) {
  const Adam h_all{lr, beta1, beta2, eps, wd};
  const double bc1 = 1.0 - std::pow(beta1, static_cast<double>(step));
  const double bc2 = 1.0 - std::pow(beta2, static_cast<double>(step));
  for (uint32_t t = 0; t < n_tensors; ++t) {
    const uint64_t n = tensor_numel[t];
    double* g = new double[n ? n : 1];
    for (uint64_t i = 0; i < n; ++i) g[i] = load_grad(grads[t], gdt, i);
    const double trust = lamb_tensor(n, g, p[t], m[t], v[t], for_tensor(h_all, decay, t), bc1, bc2);
    if (trust_out) trust_out[t] = trust;
    delete[] g;
  }
}

// Bucket-wise clipping (Sec. 2.3, Sec. 4.2, Alg. 1) followed by LAMB instead of
// Adam: norms and coefficients per bucket as in orc_bucket_clip_adam, then
// ghat = coef_b * g in working precision for every element, then LAMB tensor by
// tensor on ghat.  With write_back the storage-rounded ghat replaces g.
int32_t orc_bucket_clip_lamb(uint32_t n_tensors, const uint64_t* tensor_numel, uint32_t n_buckets,
                             const uint64_t* bucket_seg_off, const uint32_t* seg_tensor, const uint64_t* seg_begin,
                             const uint64_t* seg_len, void* const* grads, int gdt, double* const* p,
                             double* const* m, double* const* v, const float* thresholds, double lr, double beta1,
                             double beta2, double eps, double wd, uint64_t step, int write_back,
                             const uint8_t* decay, double* norms_out, float* coefs_out, double* trust_out) {
  double* norms = new double[n_buckets ? n_buckets : 1];
  float* coefs = new float[n_buckets ? n_buckets : 1];
  orc_bucket_norms(n_buckets, bucket_seg_off, seg_tensor, seg_begin, seg_len, grads, gdt, norms);
  const int32_t status = orc_clip_coefs(n_buckets, norms, thresholds, coefs);
  if (norms_out) std::memcpy(norms_out, norms, sizeof(double) * n_buckets);
  if (coefs_out) std::memcpy(coefs_out, coefs, sizeof(float) * n_buckets);

  double** ghat = new double*[n_tensors ? n_tensors : 1];
  for (uint32_t t = 0; t < n_tensors; ++t) ghat[t] = new double[tensor_numel[t] ? tensor_numel[t] : 1]();  // zeros where no segment writes
  for (uint32_t b = 0; b < n_buckets; ++b)
    for (uint64_t k = bucket_seg_off[b]; k < bucket_seg_off[b + 1]; ++k) {
      const uint32_t t = seg_tensor[k];
      for (uint64_t i = seg_begin[k]; i < seg_begin[k] + seg_len[k]; ++i) {
        ghat[t][i] = static_cast<double>(coefs[b]) * load_grad(grads[t], gdt, i);
        if (write_back && coefs[b] != 1.0f) store_scaled_grad(grads[t], gdt, i, coefs[b]);
      }
    }
  const Adam h_all{lr, beta1, beta2, eps, wd};
  const double bc1 = 1.0 - std::pow(beta1, static_cast<double>(step));
  const double bc2 = 1.0 - std::pow(beta2, static_cast<double>(step));
  for (uint32_t t = 0; t < n_tensors; ++t) {
    const double trust = lamb_tensor(tensor_numel[t], ghat[t], p[t], m[t], v[t], for_tensor(h_all, decay, t), bc1, bc2);
    if (trust_out) trust_out[t] = trust;
    delete[] ghat[t];
  }
  delete[] ghat;
  delete[] norms;
  delete[] coefs;
  return status;
}

// Element-wise comparison of a GPU fp32 array with the oracle's fp64 array
// under the acceptance rule: relative error <= rel_tol, or absolute error <=
// abs_tol where |oracle| < small.  Returns the number of failing elements and
// fills out[0..3] = max relative error over |oracle| >= small, max absolute
// error over |oracle| < small, max relative error over all |oracle| > tiny,
// index of the worst failing element (or -1).
uint64_t orc_compare_f32(const float* got, const double* want, uint64_t n, double rel_tol, double abs_tol,
                         double small, double tiny, double* out) {
  uint64_t bad = 0;
  double max_rel_big = 0.0, max_abs_small = 0.0, max_rel_all = 0.0, worst = -1.0, worst_err = -1.0;
  for (uint64_t i = 0; i < n; ++i) {
    const double w = want[i], g = static_cast<double>(got[i]);
    const double err = std::fabs(g - w), aw = std::fabs(w);
    bool ok;
    if (std::isnan(w) || std::isnan(g)) {
      ok = std::isnan(w) && std::isnan(g);
    } else if (std::isinf(w) || std::isinf(g)) {
      ok = (w == g);
    } else {
      const double rel = aw > 0.0 ? err / aw : (err == 0.0 ? 0.0 : INFINITY);
      if (aw >= small) {
        if (rel > max_rel_big) max_rel_big = rel;
      } else if (err > max_abs_small) {
        max_abs_small = err;
      }
      if (aw > tiny && rel > max_rel_all) max_rel_all = rel;
      ok = (rel <= rel_tol) || (aw < small && err <= abs_tol);
      if (!ok && err > worst_err) {
        worst_err = err;
        worst = static_cast<double>(i);
      }
    }
    if (!ok) {
      ++bad;
      if (worst < 0) worst = static_cast<double>(i);
    }
  }
  out[0] = max_rel_big;
  out[1] = max_abs_small;
  out[2] = max_rel_all;
  out[3] = worst;
  return bad;
}

}  // extern "C"

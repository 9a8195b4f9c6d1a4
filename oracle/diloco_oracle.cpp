// CPU oracle for the DiLoCo optimizer hot path.  TEST INFRASTRUCTURE ONLY.
//
// This file is the definition the GPU library is checked against.  It is plain,
// slow, element-at-a-time C++ with no blocking, fusion or vector intrinsics.  It
// shares no code with the HIP path and the product never calls it: only tests,
// the smoke check and the benchmark's cpu_baseline leg load it.
//
// What it follows (OpenDiLoCo, arxiv 2407.07852):
//   * Section "Implementation": two optimizers -- inner AdamW per worker, outer
//     SGD with Nesterov momentum -- and the pseudo-gradient
//     delta = theta(t) - theta(t+h)  (original minus locally updated weight).
//   * Figure 1 (outer optimizer pseudo-code): per parameter, subtract, average
//     over workers, reset the worker's weights to the original, take the outer
//     step, then re-snapshot the original weights.
//   * Paragraph "General Implementation Details": pseudo-gradients are FP32, or
//     optionally FP16; the mixed-precision gradient scaler belongs to the inner
//     step only.
//   * Section "All-Reduce in FP16": the FP16 pseudo-gradient variant.
//   * Appendix A, Table 3: the hyper-parameters (they are arguments here).
//
// AdamW is the decoupled-weight-decay Adam of Loshchilov & Hutter (the paper's
// citation for its inner optimizer); the Nesterov step uses the convention of
// the framework the paper builds on: b <- mu*b + g ; p <- p - lr*(g + mu*b).
//
// Arithmetic: the working type T is float (IEEE binary32, round to nearest
// even, one rounding per written operation -- compile with -ffp-contract=off,
// never -ffast-math) for everything compared with the GPU, and double for the
// tests that pin the formulas against closed forms and library optimizers.
//
// Parity pins: every function below is pinned by tests/test_oracle_*.py
// (hand-computed steps, closed forms, library optimizers in float64,
// the half-precision boundary table and round trip, brute force on tiny inputs).

#include <cmath>
#include <cstdint>
#include <cstring>
#include <cstddef>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

inline uint32_t bits_of(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }
inline float float_of(uint32_t u) { float f; std::memcpy(&f, &u, 4); return f; }

// ---------------------------------------------------------------------------
// IEEE binary16 <-> binary32, integer arithmetic only.
// binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits.  Smallest normal
// 2^-14, smallest subnormal 2^-24, largest finite 65504.  Values at or above
// 65520 (half way between 65504 and 2^16) round to infinity.
// ---------------------------------------------------------------------------
uint16_t f32_to_f16_rne(float f) {
  const uint32_t u = bits_of(f);
  const uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
  const uint32_t a = u & 0x7fffffffu;               // magnitude bits
  if (a > 0x7f800000u) return (uint16_t)(sign | 0x7e00u);   // NaN -> a quiet NaN
  if (a >= 0x477ff000u) return (uint16_t)(sign | 0x7c00u);  // >= 65520, incl. inf
  const uint32_t e = a >> 23;                        // biased binary32 exponent
  if (e == 0) return sign;                           // zero / binary32 subnormal: far below 2^-25
  const uint32_t sig = (a & 0x007fffffu) | 0x00800000u;   // 24-bit significand, value sig * 2^(e-150)
  uint32_t keep, rem, half_way;
  if (e >= 113) {
    // Normal half: drop the low 13 fraction bits.
    keep = ((e - 112) << 10) | ((sig >> 13) & 0x3ffu);
    rem = sig & 0x1fffu;
    half_way = 0x1000u;
  } else {
    // Subnormal half, in units of 2^-24:  sig * 2^(e-150) / 2^-24 = sig >> (126 - e).
    const uint32_t shift = 126 - e;                  // >= 14
    if (shift > 25) return sign;                     // below 2^-26 <= ... < 2^-25: rounds to zero
    keep = sig >> shift;
    rem = sig & ((1u << shift) - 1u);
    half_way = 1u << (shift - 1);
  }
  // Round to nearest, ties to the even code.  A carry out of the fraction moves
  // into the exponent field, which is the correct next binade (or 2^-14 from the
  // subnormal range).
  if (rem > half_way || (rem == half_way && (keep & 1u))) keep += 1;
  return (uint16_t)(sign | keep);
}

float f16_to_f32(uint16_t h) {
  const uint32_t sign = ((uint32_t)h & 0x8000u) << 16;
  const uint32_t e = (h >> 10) & 0x1fu;
  const uint32_t frac = h & 0x3ffu;
  if (e == 0x1f) return float_of(sign | 0x7f800000u | (frac << 13));   // inf / NaN
  if (e != 0) return float_of(sign | ((e + 112) << 23) | (frac << 13)); // normal
  if (frac == 0) return float_of(sign);                                  // signed zero
  // Subnormal: frac * 2^-24, exact in binary32.
  const float mag = (float)frac * float_of(0x33800000u);                 // 2^-24
  return float_of(sign | bits_of(mag));
}

// ---------------------------------------------------------------------------
// bfloat16 = the upper 16 bits of a binary32 (1 sign, 8 exponent, 7 fraction bits), reached by
// round to nearest, ties to even, on the dropped 16 bits.  Same exponent range as binary32, so
// subnormals round on the same grid and only values within half a unit of the largest finite
// bfloat16 of binary32's top binade overflow to infinity.
// ---------------------------------------------------------------------------
uint16_t f32_to_bf16_rne(float f) {
  const uint32_t u = bits_of(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);  // NaN stays NaN
  const uint32_t keep = u >> 16;
  const uint32_t rem = u & 0xffffu;
  uint32_t out = keep;
  if (rem > 0x8000u || (rem == 0x8000u && (keep & 1u))) out += 1;  // carry may reach infinity
  return (uint16_t)out;
}

float bf16_to_f32(uint16_t h) { return float_of((uint32_t)h << 16); }

// ---------------------------------------------------------------------------
// Inner optimizer: one AdamW step of one worker over n elements.
// p1, p2 are the worker's running products beta1^t, beta2^t (double, start 1);
// the step advances them, i.e. the worker's step count t grows by one.
// ---------------------------------------------------------------------------
// The element loop of one AdamW step over [first, first+n) with the scalars of one parameter
// group.  bc1 = 1 - beta1^t, bc2 = 1 - beta2^t.
template <class T>
void adamw_elements(T* theta, T* m, T* v, const T* g, size_t first, size_t n, double lr,
                    double beta1, double beta2, double eps, double weight_decay, T bc1, T bc2) {
  // Hyper-parameters are doubles; each scalar the loop uses is formed in double and
  // rounded to the working type once.
  const T b1 = (T)beta1, b2 = (T)beta2;
  const T one_minus_b1 = (T)(1.0 - beta1);
  const T one_minus_b2 = (T)(1.0 - beta2);
  const T lr_t = (T)lr, eps_t = (T)eps;
  const T lr_wd = (T)(lr * weight_decay);
#pragma omp parallel for schedule(static)
  for (size_t i = first; i < first + n; ++i) {
    const T gi = g[i];
    const T mi = b1 * m[i] + one_minus_b1 * gi;
    const T vi = b2 * v[i] + one_minus_b2 * (gi * gi);
    const T m_hat = mi / bc1;
    const T v_hat = vi / bc2;
    const T decayed = theta[i] - lr_wd * theta[i];
    theta[i] = decayed - lr_t * (m_hat / (std::sqrt(v_hat) + eps_t));
    m[i] = mi;
    v[i] = vi;
  }
}

template <class T>
void adamw_step(T* theta, T* m, T* v, const T* g, size_t n, double lr, double beta1, double beta2,
                double eps, double weight_decay, double* p1, double* p2) {
  *p1 *= beta1;
  *p2 *= beta2;
  const T bc1 = (T)(1.0 - *p1);   // 1 - beta1^t
  const T bc2 = (T)(1.0 - *p2);   // 1 - beta2^t
  adamw_elements<T>(theta, m, v, g, 0, n, lr, beta1, beta2, eps, weight_decay, bc1, bc2);
}

// Parameter groups: tensor t (elements [offset[t], offset[t]+numel[t]) of the flat arrays)
// belongs to group group_of_tensor[t] and is stepped with that group's learning rate
// lr * lr_scale[group] and weight decay weight_decay[group].  One step count per worker.
template <class T>
void adamw_step_groups(T* theta, T* m, T* v, const T* g, uint32_t n_tensors,
                       const uint64_t* offset, const uint64_t* numel,
                       const uint8_t* group_of_tensor, const double* lr_scale,
                       const double* weight_decay, double lr, double beta1, double beta2,
                       double eps, double* p1, double* p2) {
  *p1 *= beta1;
  *p2 *= beta2;
  const T bc1 = (T)(1.0 - *p1);
  const T bc2 = (T)(1.0 - *p2);
  for (uint32_t t = 0; t < n_tensors; ++t) {
    const uint8_t grp = group_of_tensor[t];
    adamw_elements<T>(theta, m, v, g, offset[t], numel[t], lr * lr_scale[grp], beta1, beta2, eps,
                      weight_decay[grp], bc1, bc2);
  }
}

// ---------------------------------------------------------------------------
// Outer optimizer pieces (Figure 1).
// ---------------------------------------------------------------------------
template <class T>
void pseudo_grad(const T* theta0, const T* theta_r, T* delta, size_t n) {
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < n; ++i) delta[i] = theta0[i] - theta_r[i];
}

// Average over k workers: sum in worker order 0..k-1, then divide by k.
template <class T>
void replica_mean(const T* delta /* [k][n] */, size_t k, size_t n, T* mean) {
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < n; ++i) {
    T s = delta[i];
    for (size_t r = 1; r < k; ++r) s = s + delta[r * n + i];
    mean[i] = s / (T)k;
  }
}

// SGD with Nesterov momentum, dampening 0, no weight decay.
template <class T>
void nesterov_step(T* theta0, T* b, const T* grad, size_t n, double lr, double mu) {
  const T lr_t = (T)lr, mu_t = (T)mu;
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < n; ++i) {
    const T bi = mu_t * b[i] + grad[i];
    theta0[i] = theta0[i] - lr_t * (grad[i] + mu_t * bi);
    b[i] = bi;
  }
}

}  // namespace

// Step 2: delayed application.  theta0 holds the new outer weights; theta is [k][n], the
// workers' current weights, updated in place.
template <class T>
static void merge_delayed(const T* theta0, const T* snap, T* theta, size_t k, size_t n) {
  for (size_t r = 0; r < k; ++r) {
    const T* s = snap + r * n;
    T* th = theta + r * n;
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
      const T since_snapshot = s[i] - th[i];  // minus the worker's progress since the snapshot
      th[i] = theta0[i] - since_snapshot;
    }
  }
}
extern "C" {

// ---- binary16 casts --------------------------------------------------------
uint16_t oracle_f32_to_f16_rne(float f) { return f32_to_f16_rne(f); }
float oracle_f16_to_f32(uint16_t h) { return f16_to_f32(h); }

void oracle_cast_f32_to_f16(const float* in, uint16_t* out, size_t n) {
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < n; ++i) out[i] = f32_to_f16_rne(in[i]);
}

// Cast of the n consecutive binary32 bit patterns first, first+1, ...
void oracle_cast_pattern_range(uint32_t first, size_t n, uint16_t* out) {
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < n; ++i) out[i] = f32_to_f16_rne(float_of(first + (uint32_t)i));
}

void oracle_cast_f16_to_f32(const uint16_t* in, float* out, size_t n) {
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < n; ++i) out[i] = f16_to_f32(in[i]);
}

uint16_t oracle_f32_to_bf16_rne(float f) { return f32_to_bf16_rne(f); }
float oracle_bf16_to_f32(uint16_t h) { return bf16_to_f32(h); }

void oracle_cast_f32_to_bf16(const float* in, uint16_t* out, size_t n) {
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < n; ++i) out[i] = f32_to_bf16_rne(in[i]);
}

void oracle_cast_pattern_range_bf16(uint32_t first, size_t n, uint16_t* out) {
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < n; ++i) out[i] = f32_to_bf16_rne(float_of(first + (uint32_t)i));
}

// ---- inner step ------------------------------------------------------------
void oracle_adamw_step_f32(float* theta, float* m, float* v, const float* g, size_t n, double lr,
                           double beta1, double beta2, double eps, double weight_decay,
                           double* p1, double* p2) {
  adamw_step<float>(theta, m, v, g, n, lr, beta1, beta2, eps, weight_decay, p1, p2);
}

void oracle_adamw_step_f64(double* theta, double* m, double* v, const double* g, size_t n,
                           double lr, double beta1, double beta2, double eps, double weight_decay,
                           double* p1, double* p2) {
  adamw_step<double>(theta, m, v, g, n, lr, beta1, beta2, eps, weight_decay, p1, p2);
}

void oracle_adamw_step_groups_f32(float* theta, float* m, float* v, const float* g,
                                  uint32_t n_tensors, const uint64_t* offset,
                                  const uint64_t* numel, const uint8_t* group_of_tensor,
                                  const double* lr_scale, const double* weight_decay, double lr,
                                  double beta1, double beta2, double eps, double* p1, double* p2) {
  adamw_step_groups<float>(theta, m, v, g, n_tensors, offset, numel, group_of_tensor, lr_scale,
                           weight_decay, lr, beta1, beta2, eps, p1, p2);
}

void oracle_adamw_step_groups_f64(double* theta, double* m, double* v, const double* g,
                                  uint32_t n_tensors, const uint64_t* offset,
                                  const uint64_t* numel, const uint8_t* group_of_tensor,
                                  const double* lr_scale, const double* weight_decay, double lr,
                                  double beta1, double beta2, double eps, double* p1, double* p2) {
  adamw_step_groups<double>(theta, m, v, g, n_tensors, offset, numel, group_of_tensor, lr_scale,
                            weight_decay, lr, beta1, beta2, eps, p1, p2);
}

// Learning-rate schedule on the host: linear warm-up from 0 over warmup_steps, then (when
// total_steps > warmup_steps) a half-cosine from base_lr down to base_lr*final_ratio at
// total_steps, constant afterwards; with total_steps == 0 the rate stays at base_lr.
double oracle_lr_at(uint64_t step, uint64_t warmup_steps, uint64_t total_steps, double base_lr,
                    double final_ratio) {
  if (step < warmup_steps) return base_lr * ((double)step / (double)warmup_steps);
  if (total_steps <= warmup_steps) return base_lr;
  if (step >= total_steps) return base_lr * final_ratio;
  const double progress = (double)(step - warmup_steps) / (double)(total_steps - warmup_steps);
  const double pi = 3.14159265358979323846;
  const double cosine = 0.5 * (1.0 + std::cos(pi * progress));
  return base_lr * (final_ratio + (1.0 - final_ratio) * cosine);
}

// Mixed precision: gradients arrive as binary16 multiplied by the loss scale;
// they are widened and multiplied by inv_scale into g32 (n floats of scratch the
// caller provides), then the ordinary step runs.
void oracle_unscale_f16(const uint16_t* g16, float inv_scale, float* g32, size_t n) {
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < n; ++i) g32[i] = f16_to_f32(g16[i]) * inv_scale;
}

// The same for gradients kept in FP32 under a loss scale: the scaler's unscale is
// one multiply per element whatever type the gradients are stored in.
void oracle_unscale_f32(const float* g, float inv_scale, float* g32, size_t n) {
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < n; ++i) g32[i] = g[i] * inv_scale;
}

// found_inf for one worker: 1 if any element is +-inf or NaN, else 0.
int32_t oracle_found_inf_f16(const uint16_t* g16, size_t n) {
  int32_t found = 0;
  for (size_t i = 0; i < n; ++i)
    if ((g16[i] & 0x7c00u) == 0x7c00u) found = 1;
  return found;
}

int32_t oracle_found_inf_f32(const float* g, size_t n) {
  int32_t found = 0;
  for (size_t i = 0; i < n; ++i)
    if (std::isinf(g[i]) || std::isnan(g[i])) found = 1;
  return found;
}

// ---- outer step ------------------------------------------------------------
void oracle_pseudo_grad_f32(const float* theta0, const float* theta_r, float* delta, size_t n) {
  pseudo_grad<float>(theta0, theta_r, delta, n);
}
void oracle_pseudo_grad_f64(const double* theta0, const double* theta_r, double* delta, size_t n) {
  pseudo_grad<double>(theta0, theta_r, delta, n);
}

// In place: delta <- widen(f16_rne(delta)).
void oracle_round_through_f16(float* delta, size_t n) {
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < n; ++i) delta[i] = f16_to_f32(f32_to_f16_rne(delta[i]));
}

// In place: delta <- widen(bf16_rne(delta)).
void oracle_round_through_bf16(float* delta, size_t n) {
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < n; ++i) delta[i] = bf16_to_f32(f32_to_bf16_rne(delta[i]));
}

// pg_dtype: 0 = binary32 (no rounding), 1 = binary16, 2 = bfloat16.
static void round_through(float* x, size_t n, int32_t pg_dtype) {
  if (pg_dtype == 1) oracle_round_through_f16(x, n);
  if (pg_dtype == 2) oracle_round_through_bf16(x, n);
}

void oracle_replica_mean_f32(const float* delta, size_t k, size_t n, float* mean) {
  replica_mean<float>(delta, k, n, mean);
}
void oracle_replica_mean_f64(const double* delta, size_t k, size_t n, double* mean) {
  replica_mean<double>(delta, k, n, mean);
}

void oracle_nesterov_step_f32(float* theta0, float* b, const float* grad, size_t n, double lr,
                              double mu) {
  nesterov_step<float>(theta0, b, grad, n, lr, mu);
}
void oracle_nesterov_step_f64(double* theta0, double* b, const double* grad, size_t n, double lr,
                              double mu) {
  nesterov_step<double>(theta0, b, grad, n, lr, mu);
}

// The whole outer step in Figure 1's order.  theta is [k][n] (the workers' local
// weights), delta_scratch is [k][n] and mean_scratch is [n].  pg_dtype (0 binary32,
// 1 binary16, 2 bfloat16) is the type each worker's pseudo-gradient is rounded through
// before the average; with round_mean != 0 the average itself is rounded through that type
// as well, as the output buffer of a reduced-precision all-reduce would be.
void oracle_outer_step_f32(float* theta0, float* b, float* theta, size_t k, size_t n,
                           double outer_lr, double mu, int32_t pg_dtype, int32_t round_mean,
                           float* delta_scratch, float* mean_scratch) {
  for (size_t r = 0; r < k; ++r) {
    pseudo_grad<float>(theta0, theta + r * n, delta_scratch + r * n, n);
    round_through(delta_scratch + r * n, n, pg_dtype);
  }
  replica_mean<float>(delta_scratch, k, n, mean_scratch);
  if (round_mean) round_through(mean_scratch, n, pg_dtype);
  nesterov_step<float>(theta0, b, mean_scratch, n, outer_lr, mu);
  for (size_t r = 0; r < k; ++r) std::memcpy(theta + r * n, theta0, n * sizeof(float));
}

// ---- delayed application of the outer step --------------------------------
// The paper's future work (Conclusion; Section "Globally Distributed Training Setting", last
// sentence) names averaging the weights asynchronously, interleaved with the computation of the
// next round, without giving an update rule.  The rule taken here: at the round boundary each
// worker's weights are snapshotted (sigma_r); the outer update is computed from the snapshots
// exactly as the outer step computes it from the workers' weights (same pseudo-gradient,
// rounding, average and Nesterov step), but the workers are not reset yet and keep stepping;
// when the update is applied, each worker carries over what it has done since the snapshot:
//     theta_r <- theta0_new - (sigma_r - theta_r).
// With no steps in between, sigma_r - theta_r = +0 and the rule is the outer step of Figure 1.

// Step 1: outer update from the snapshots.  snap is [k][n]; theta0 and b are updated in place;
// the workers' weights are not read or written.
void oracle_outer_update_from_snapshot_f32(float* theta0, float* b, const float* snap, size_t k,
                                           size_t n, double outer_lr, double mu, int32_t pg_dtype,
                                           int32_t round_mean, float* delta_scratch,
                                           float* mean_scratch) {
  for (size_t r = 0; r < k; ++r) {
    pseudo_grad<float>(theta0, snap + r * n, delta_scratch + r * n, n);
    round_through(delta_scratch + r * n, n, pg_dtype);
  }
  replica_mean<float>(delta_scratch, k, n, mean_scratch);
  if (round_mean) round_through(mean_scratch, n, pg_dtype);
  nesterov_step<float>(theta0, b, mean_scratch, n, outer_lr, mu);
}

// Step 2: delayed application (merge_delayed above).
void oracle_merge_delayed_f32(const float* theta0, const float* snap, float* theta, size_t k,
                              size_t n) {
  merge_delayed<float>(theta0, snap, theta, k, n);
}
void oracle_merge_delayed_f64(const double* theta0, const double* snap, double* theta, size_t k,
                              size_t n) {
  merge_delayed<double>(theta0, snap, theta, k, n);
}

// ---- flat layout (written independently of the library's planner) ----------
// Each tensor starts at a multiple of `align` elements; the total is rounded up
// to a multiple of `tile` elements.  Returns the padded length.
uint64_t oracle_plan_layout(const uint64_t* numel, uint32_t n_tensors, uint64_t align,
                            uint64_t tile, uint64_t* offsets) {
  uint64_t cursor = 0;
  for (uint32_t t = 0; t < n_tensors; ++t) {
    while (cursor % align != 0) ++cursor;
    offsets[t] = cursor;
    cursor += numel[t];
  }
  while (cursor % tile != 0) ++cursor;
  return cursor;
}

int oracle_num_threads(void) {
  int n = 1;
#ifdef _OPENMP
#pragma omp parallel
  {
#pragma omp single
    n = omp_get_num_threads();
  }
#endif
  return n;
}

}  // extern "C"

/* Seeded, counter-based synthetic input generator shared by the CPU test harness and the
 * GPU test harness.  It holds none of the optimizer's arithmetic: it only turns
 * (seed, stream, replica, step, element index) into a reproducible input value, with integer
 * arithmetic up to one final float multiply, so the host and the device produce the same bits.
 *
 * Value recipe: a 64-bit hash u of the counter; S = sum of its four 16-bit fields
 * (Irwin-Hall, mean 131070, standard deviation sqrt(4*(65536^2-1)/12) = 37837.227);
 * x = (float)(S - 131070) * c, with c = (float)(sigma / 37837.227).  Bell-shaped, bounded
 * at +-3.46 sigma.
 */
#ifndef SYNTH_MIX_H
#define SYNTH_MIX_H
#include <stdint.h>

#if defined(__HIPCC__)
#define SYNTH_HD __host__ __device__ static inline
#else
#define SYNTH_HD static inline
#endif

#define SYNTH_IRWIN_HALL_SD 37837.22723513447

/* element kinds in the per-element map */
#define SYNTH_KIND_PAD 0    /* padding: always 0 */
#define SYNTH_KIND_NORMAL 1 /* bell-shaped value */
#define SYNTH_KIND_ONE 2    /* weights: 1.0 (norm vectors); gradients: bell-shaped like kind 1 */

/* 64-bit finalizer of the SplitMix64 generator (Steele, Lea, Flood 2014). */
SYNTH_HD uint64_t synth_mix64(uint64_t z) {
  z ^= z >> 30;
  z *= 0xBF58476D1CE4E5B9ull;
  z ^= z >> 27;
  z *= 0x94D049BB133111EBull;
  z ^= z >> 31;
  return z;
}

SYNTH_HD uint64_t synth_key(uint64_t seed, uint64_t stream, uint64_t replica, uint64_t step) {
  uint64_t k = synth_mix64(seed + 0x9E3779B97F4A7C15ull);
  k = synth_mix64(k + stream);
  k = synth_mix64(k + replica);
  k = synth_mix64(k + step);
  return k;
}

SYNTH_HD uint64_t synth_hash(uint64_t key, uint64_t index) {
  return synth_mix64(key + index * 0x9E3779B97F4A7C15ull);
}

/* S - 131070, in [-131070, 131070] */
SYNTH_HD int32_t synth_bell_int(uint64_t key, uint64_t index) {
  const uint64_t u = synth_hash(key, index);
  const int32_t s = (int32_t)(u & 0xffff) + (int32_t)((u >> 16) & 0xffff) +
                    (int32_t)((u >> 32) & 0xffff) + (int32_t)((u >> 48) & 0xffff);
  return s - 131070;
}

SYNTH_HD float synth_bell_f32(uint64_t key, uint64_t index, float c) {
  return (float)synth_bell_int(key, index) * c;
}

/* binary16 code of the exactly representable value j * 2^-3 with j = (S-131070) >> 6, so
 * |j| <= 2048 fits the 11-bit significand: no rounding is involved, the code is built from
 * the integer.  Standard deviation 591.2/8 = 73.9 (a gradient of ~1.1e-3 times a loss scale
 * of 65536). */
SYNTH_HD uint16_t synth_bell_f16_bits(uint64_t key, uint64_t index) {
  const int32_t j = synth_bell_int(key, index) >> 6;
  if (j == 0) return 0;
  const uint16_t sign = j < 0 ? 0x8000u : 0u;
  uint32_t a = (uint32_t)(j < 0 ? -j : j);
  int p = 0; /* position of the leading one */
  while ((a >> (p + 1)) != 0) ++p;
  const uint32_t frac = p <= 10 ? ((a << (10 - p)) & 0x3ffu) : ((a >> (p - 10)) & 0x3ffu);
  return (uint16_t)(sign | ((uint32_t)(p + 12) << 10) | frac);
}

/* Non-finite injection: where hash(inject_key, index) % period == 0 the value becomes
 * +inf, -inf or NaN in rotation.  Returns 0 when the element is left alone, else the
 * binary16 code to store. */
SYNTH_HD uint16_t synth_inject_f16(uint64_t inject_key, uint64_t index, uint32_t period) {
  const uint64_t u = synth_hash(inject_key, index);
  if (u % period != 0) return 0;
  const uint32_t which = (uint32_t)((u / period) % 3);
  return which == 0 ? 0x7C00u : (which == 1 ? 0xFC00u : 0x7E00u);
}

#endif

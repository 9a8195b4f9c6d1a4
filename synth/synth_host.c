/* Host twin of the synthetic input generator (see synth_mix.h). */
#include <stddef.h>
#include "synth_mix.h"

/* out[i] for flat indices first..first+n-1; kind may be NULL (all bell-shaped). */
void synth_host_fill_f32(float* out, const uint8_t* kind, uint64_t first, size_t n, uint64_t key,
                         float c, int ones_as_one) {
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < n; ++i) {
    const uint8_t kd = kind ? kind[i] : SYNTH_KIND_NORMAL;
    float x = 0.0f;
    if (kd == SYNTH_KIND_NORMAL || (kd == SYNTH_KIND_ONE && !ones_as_one))
      x = synth_bell_f32(key, first + i, c);
    else if (kd == SYNTH_KIND_ONE)
      x = 1.0f;
    out[i] = x;
  }
}

/* Same values at an arbitrary list of flat indices; kind_at[j] is the kind of idx[j]. */
void synth_host_gather_f32(float* out, const uint8_t* kind_at, const uint64_t* idx, size_t n_idx,
                           uint64_t key, float c, int ones_as_one) {
#pragma omp parallel for schedule(static)
  for (size_t j = 0; j < n_idx; ++j) {
    const uint8_t kd = kind_at ? kind_at[j] : SYNTH_KIND_NORMAL;
    float x = 0.0f;
    if (kd == SYNTH_KIND_NORMAL || (kd == SYNTH_KIND_ONE && !ones_as_one))
      x = synth_bell_f32(key, idx[j], c);
    else if (kd == SYNTH_KIND_ONE)
      x = 1.0f;
    out[j] = x;
  }
}

void synth_host_fill_f16(uint16_t* out, const uint8_t* kind, uint64_t first, size_t n,
                         uint64_t key, uint64_t inject_key, uint32_t inject_period) {
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < n; ++i) {
    const uint8_t kd = kind ? kind[i] : SYNTH_KIND_NORMAL;
    uint16_t h = 0;
    if (kd != SYNTH_KIND_PAD) {
      h = synth_bell_f16_bits(key, first + i);
      if (inject_period) {
        const uint16_t bad = synth_inject_f16(inject_key, first + i, inject_period);
        if (bad) h = bad;
      }
    }
    out[i] = h;
  }
}

void synth_host_gather_f16(uint16_t* out, const uint8_t* kind_at, const uint64_t* idx,
                           size_t n_idx, uint64_t key, uint64_t inject_key,
                           uint32_t inject_period) {
#pragma omp parallel for schedule(static)
  for (size_t j = 0; j < n_idx; ++j) {
    const uint8_t kd = kind_at ? kind_at[j] : SYNTH_KIND_NORMAL;
    uint16_t h = 0;
    if (kd != SYNTH_KIND_PAD) {
      h = synth_bell_f16_bits(key, idx[j]);
      if (inject_period) {
        const uint16_t bad = synth_inject_f16(inject_key, idx[j], inject_period);
        if (bad) h = bad;
      }
    }
    out[j] = h;
  }
}

uint64_t synth_host_key(uint64_t seed, uint64_t stream, uint64_t replica, uint64_t step) {
  return synth_key(seed, stream, replica, step);
}

uint64_t synth_host_hash(uint64_t key, uint64_t index) { return synth_hash(key, index); }

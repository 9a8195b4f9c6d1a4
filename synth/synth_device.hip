// Device twin of the synthetic input generator (see synth_mix.h): fills device buffers with
// exactly the values synth_host.c produces on the CPU.  Untimed test/benchmark plumbing.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include "synth_mix.h"

namespace {

__global__ void fill_f32_kernel(float* __restrict__ out, const uint8_t* __restrict__ kind,
                                uint64_t first, size_t n, uint64_t key, float c, int ones_as_one) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    const uint8_t kd = kind ? kind[i] : SYNTH_KIND_NORMAL;
    float x = 0.0f;
    if (kd == SYNTH_KIND_NORMAL || (kd == SYNTH_KIND_ONE && !ones_as_one))
      x = synth_bell_f32(key, first + i, c);
    else if (kd == SYNTH_KIND_ONE)
      x = 1.0f;
    out[i] = x;
  }
}

__global__ void fill_f16_kernel(uint16_t* __restrict__ out, const uint8_t* __restrict__ kind,
                                uint64_t first, size_t n, uint64_t key, uint64_t inject_key,
                                uint32_t inject_period) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
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

// Plain copy of n 16-byte vectors: the known-size reference that hardware-counter readings of
// HBM traffic are scaled by.
__global__ void copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

unsigned grid_for(size_t n) {
  size_t blocks = (n + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  if (blocks == 0) blocks = 1;
  return (unsigned)blocks;
}

}  // namespace

extern "C" {

// All pointers are device pointers; stream is a hipStream_t.  Returns the hipError_t of the launch.
int synth_device_fill_f32(void* out, const void* kind, uint64_t first, size_t n, uint64_t key,
                          float c, int ones_as_one, void* stream) {
  if (n == 0) return 0;
  hipLaunchKernelGGL(fill_f32_kernel, dim3(grid_for(n)), dim3(256), 0, (hipStream_t)stream,
                     (float*)out, (const uint8_t*)kind, first, n, key, c, ones_as_one);
  return (int)hipGetLastError();
}

int synth_device_fill_f16(void* out, const void* kind, uint64_t first, size_t n, uint64_t key,
                          uint64_t inject_key, uint32_t inject_period, void* stream) {
  if (n == 0) return 0;
  hipLaunchKernelGGL(fill_f16_kernel, dim3(grid_for(n)), dim3(256), 0, (hipStream_t)stream,
                     (uint16_t*)out, (const uint8_t*)kind, first, n, key, inject_key,
                     inject_period);
  return (int)hipGetLastError();
}

// Copies n_bytes (a multiple of 16) from src to dst, one 16-byte vector per thread.
int synth_device_copy(void* dst, const void* src, size_t n_bytes, void* stream) {
  const size_t n = n_bytes / 16;
  if (n == 0) return 0;
  hipLaunchKernelGGL(copy_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                     (hipStream_t)stream, (const uint4*)src, (uint4*)dst, n);
  return (int)hipGetLastError();
}

}  // extern "C"

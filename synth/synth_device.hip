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

// Streaming-pattern reference kernels for the benchmark: NR read streams and NW write streams in
// the launch shape of the optimizer kernels (one 256-element tile per single-wave workgroup, one
// 128-bit nontemporal access per lane and stream, residency capped through an untouched slice of
// LDS), with no arithmetic beyond a sum that keeps the loads alive.  What these sustain is the
// machine's ceiling for the traffic mix, against which the optimizer kernels are read.
typedef float f32x4 __attribute__((ext_vector_type(4)));
struct StreamPtrs { f32x4* p[20]; };
extern __shared__ float pattern_lds_pad[];

template <int NR, int NW>
__global__ __launch_bounds__(64) void stream_pattern_kernel(StreamPtrs s, float* sink, uint32_t tiles) {
  const size_t i = (size_t)blockIdx.x * 64 + threadIdx.x;
  f32x4 acc = {1.f, 1.f, 1.f, 1.f};
  if (NR == 0) {
    // pure writes: hashed mantissas and signs, because what the memory system sustains depends
    // on the data (all-equal words stream measurably faster than trained-weight-like ones)
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      uint32_t h = ((uint32_t)i * 4u + (uint32_t)c) * 2654435761u;
      h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
      acc[c] = __builtin_bit_cast(float, (h & 0x807fffffu) | 0x3c000000u);
    }
  }
  f32x4 r[NR > 0 ? NR : 1];
#pragma unroll
  for (int j = 0; j < NR; ++j) r[j] = __builtin_nontemporal_load(s.p[j] + i);
#pragma unroll
  for (int j = 0; j < NR; ++j) acc += r[j];
  if (NW == 0) {
    if (acc[0] == 12345.678f) sink[0] = acc[1];  // data-dependent and never true: keeps the loads
  }
#pragma unroll
  for (int j = 0; j < NW; ++j) __builtin_nontemporal_store(acc, s.p[NR + j] + i);
  if (tiles == 0xffffffffu) pattern_lds_pad[threadIdx.x] = 0.f;  // never true: keeps the LDS pad
}

template <int NR, int NW>
int launch_pattern(const StreamPtrs& s, float* sink, size_t n_vec, unsigned lds, hipStream_t st) {
  const uint32_t tiles = (uint32_t)(n_vec / 64);
  hipLaunchKernelGGL((stream_pattern_kernel<NR, NW>), dim3(tiles), dim3(64), lds, st, s, sink, tiles);
  return (int)hipGetLastError();
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

// One launch of a streaming pattern: nr read streams (bufs[0..nr)) and nw write streams
// (bufs[nr..nr+nw)), each n_bytes long (a multiple of 1024), at most waves_per_cu single-wave
// workgroups resident per CU (0 = no cap).  Supported (nr, nw): (1,0) (4,0) (10,0) (0,10) (1,1)
// (4,3) (10,10).
// sink: device, at least 4 bytes.  Returns the hipError_t of the launch, or -1 for an unsupported
// pattern.
int synth_device_stream_pattern(void* const* bufs, int nr, int nw, size_t n_bytes, int waves_per_cu,
                                void* sink, void* stream) {
  if (nr < 0 || nw < 0 || nr + nw > 20 || n_bytes % 1024 != 0 || n_bytes == 0) return -1;
  StreamPtrs s;
  for (int j = 0; j < nr + nw; ++j) s.p[j] = (f32x4*)bufs[j];
  unsigned lds = 0;
  if (waves_per_cu > 0 && waves_per_cu < 32) {
    // whole 1280-byte granules, the unit in which the hardware hands out LDS
    lds = 160u * 1024u / (unsigned)waves_per_cu / 1280u * 1280u;
    if (lds > 64000u) lds = 64000u;
  }
  const size_t n_vec = n_bytes / 16;
  hipStream_t st = (hipStream_t)stream;
  float* sk = (float*)sink;
  if (nr == 1 && nw == 0) return launch_pattern<1, 0>(s, sk, n_vec, lds, st);
  if (nr == 4 && nw == 0) return launch_pattern<4, 0>(s, sk, n_vec, lds, st);
  if (nr == 10 && nw == 0) return launch_pattern<10, 0>(s, sk, n_vec, lds, st);
  if (nr == 0 && nw == 10) return launch_pattern<0, 10>(s, sk, n_vec, lds, st);
  if (nr == 1 && nw == 1) return launch_pattern<1, 1>(s, sk, n_vec, lds, st);
  if (nr == 4 && nw == 3) return launch_pattern<4, 3>(s, sk, n_vec, lds, st);
  if (nr == 10 && nw == 10) return launch_pattern<10, 10>(s, sk, n_vec, lds, st);
  return -1;
}

}  // extern "C"

// gfx950 (MI355X, CDNA4) kernels of the DiLoCo optimizer hot path.
//
// Everything here is elementwise and HBM-bound, so the design is about memory streams, not
// arithmetic: flat padded buffers, one 128-bit load/store per lane per stream, every buffer
// streamed exactly once per step, one 256-element tile per single-wave workgroup handed out in
// address order by the hardware dispatcher, a capped number of waves resident per CU, and
// nontemporal accesses because nothing is reused.  No MFMA: there is no contraction.
//
// Floating point follows the method's definition operation by operation: IEEE binary32,
// round to nearest even, correctly rounded divide and sqrt, no fused multiply-add, no
// flush-to-zero (build with -ffp-contract=off and without any fast-math option).
#include "internal.h"

#pragma clang fp contract(off)

namespace diloco {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

constexpr int kBlock = 256;         // 4 wavefronts of 64 lanes
constexpr int kVecElems = 4;        // floats per 128-bit access

template <bool NT, class T>
__device__ __forceinline__ T ld(const T* p) {
  if constexpr (NT) return __builtin_nontemporal_load(p);
  else return *p;
}
template <bool NT, class T>
__device__ __forceinline__ void st(T* p, T x) {
  if constexpr (NT) __builtin_nontemporal_store(x, p);
  else *p = x;
}

// The mixed read/write streaming kernels run fastest with a LIMITED number of waves resident per
// CU (about 10 MB of loads in flight chip-wide; more in-flight requests lower the sustained HBM
// bandwidth).  Residency is capped by giving every workgroup a slice of the CU's LDS as dynamic
// shared memory that the kernel never touches.
extern __shared__ float occupancy_pad[];

// ------------------------------------------------------------------------------------------
// Inner optimizer: AdamW over all k workers, grid = (tile blocks, k).
// (Section "Implementation": the inner optimizer is AdamW, one step per training step.)
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void adamw_elem(float& th, float& m, float& v, float g,
                                           const InnerArgs& a, float lr, float lr_wd, float bc1,
                                           float bc2) {
  const float mi = a.beta1 * m + a.omb1 * g;
  const float vi = a.beta2 * v + a.omb2 * (g * g);
  const float m_hat = mi / bc1;
  const float v_hat = vi / bc2;
  const float decayed = th - lr_wd * th;
  th = decayed - lr * (m_hat / (sqrtf(v_hat) + a.eps));
  m = mi;
  v = vi;
}

// Step prologue: one thread per worker.  A worker whose found_inf flag is set takes no step:
// its step state stays as it is and its table entry says "inactive".  Otherwise the running
// products beta^t (double) and the step count advance in place, and the table receives the
// bias corrections 1 - beta^t rounded to float once.  Because the state lives on the device
// and is advanced by this kernel, a captured launch sequence replays correctly any number of
// times.
__global__ __launch_bounds__(64) void step_prologue_kernel(RepState* __restrict__ state,
                                                           StepEntry* __restrict__ table,
                                                           const int32_t* __restrict__ found_inf,
                                                           double beta1, double beta2, int k) {
  const int r = (int)threadIdx.x;
  if (r >= k) return;
  const bool skip = found_inf != nullptr && found_inf[r] != 0;
  RepState rs = state[r];
  if (!skip) {
    rs.p1 *= beta1;
    rs.p2 *= beta2;
    rs.step += 1;
    state[r] = rs;
  }
  StepEntry e;
  e.bc1 = (float)(1.0 - rs.p1);  // 1 - beta1^t
  e.bc2 = (float)(1.0 - rs.p2);  // 1 - beta2^t
  e.active = skip ? 0 : 1;
  e.pad = 0;
  table[r] = e;
}

// The group's learning rate and lr*weight_decay (at most 8 groups; the 16 scalars sit in SGPRs).
// With a wave-uniform q this is a chain of scalar selects; with a per-lane q, vector selects.
__device__ __forceinline__ void select_group(const InnerArgs& a, uint32_t q, float& lr,
                                             float& lr_wd) {
  lr = a.lr_g[0];
  lr_wd = a.lr_wd_g[0];
#pragma unroll
  for (uint32_t j = 1; j < 8; ++j) {
    lr = q == j ? a.lr_g[j] : lr;
    lr_wd = q == j ? a.lr_wd_g[j] : lr_wd;
  }
}

// One 128-bit vector per lane per stream; a wave covers 256 consecutive elements, a workgroup
// of B threads B*4.  The grid holds exactly one workgroup per tile: no bounds check.
template <int B, bool G16, bool GROUPS>
__global__ __launch_bounds__(B) void adamw_flat_kernel(const InnerArgs a, uint32_t tiles) {
  constexpr bool NT = true;
  const uint32_t r = blockIdx.y;
  const uint32_t tile = blockIdx.x;

  f32x4* __restrict__ th_p = reinterpret_cast<f32x4*>(a.theta + (size_t)r * a.stride);
  f32x4* __restrict__ m_p = reinterpret_cast<f32x4*>(a.m + (size_t)r * a.stride);
  f32x4* __restrict__ v_p = reinterpret_cast<f32x4*>(a.v + (size_t)r * a.stride);
  const f32x4* __restrict__ g32_p =
      reinterpret_cast<const f32x4*>(static_cast<const float*>(a.g) + (size_t)r * a.g_stride);
  const u32x2* __restrict__ g16_p =
      reinterpret_cast<const u32x2*>(static_cast<const uint16_t*>(a.g) + (size_t)r * a.g_stride);

  // The tile's loads go out first; the worker's table entry and the tile's group word are
  // wave-uniform scalar loads that overlap the HBM latency.
  const size_t i = (size_t)tile * B + threadIdx.x;
  f32x4 th, m, v, g;
  u32x2 graw;
  if constexpr (G16) graw = ld<NT>(g16_p + i);
  else g = ld<NT>(g32_p + i);
  th = ld<NT>(th_p + i);
  m = ld<NT>(m_p + i);
  v = ld<NT>(v_p + i);

  const StepEntry e = a.table[r];
  // A lane's four elements lie inside one 64-element chunk, and a chunk holds one tensor.  A
  // wave's 256 elements are 4 chunks = one 32-bit word of the chunk map.
  uint32_t word = 0;
  if constexpr (GROUPS) {
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    word = a.chunk_group[(size_t)tile * (B / 64) + wave];
  }
  // A worker whose found_inf flag was set takes no step at all: weights and moments stay.
  if (!e.active) return;

  if constexpr (G16) {
    f16x4 h;
    __builtin_memcpy(&h, &graw, 8);
    g = __builtin_convertvector(h, f32x4);
  }
  g = g * a.inv_scale;  // 1.0 unless a scaler check recorded a factor (exact then)

  float lr = a.lr, lr_wd = a.lr_wd;
  if constexpr (GROUPS) {
    // Almost every wave lies inside one tensor: all four chunk ids equal, scalar selects.
    if (word == (word & 0xffu) * 0x01010101u) {
      select_group(a, word & 0xffu, lr, lr_wd);
    } else {
      select_group(a, (word >> (((threadIdx.x & 63u) >> 4) * 8)) & 0xffu, lr, lr_wd);
    }
  }
#pragma unroll
  for (int c = 0; c < kVecElems; ++c) {
    float t = th[c], mm = m[c], vv = v[c];
    adamw_elem(t, mm, vv, g[c], a, lr, lr_wd, e.bc1, e.bc2);
    th[c] = t;
    m[c] = mm;
    v[c] = vv;
  }
  st<NT>(th_p + i, th);
  st<NT>(m_p + i, m);
  st<NT>(v_p + i, v);
  if (tiles == 0xffffffffu) occupancy_pad[threadIdx.x] = 0.f;  // never true: keeps the LDS pad
}

// ------------------------------------------------------------------------------------------
// Outer step (Figure 1), fused: pseudo-gradient, optional binary16 rounding, mean over the k
// workers, Nesterov SGD on theta0, and the reset of every worker to the new theta0.
// The pseudo-gradients never leave registers.
// ------------------------------------------------------------------------------------------
// Rounds x through the pseudo-gradient type PG (0 binary32, 1 binary16, 2 bfloat16) with the
// hardware's round-to-nearest-even conversions (subnormals kept) and widens it back.
template <int PG>
__device__ __forceinline__ float round_through(float x) {
  if constexpr (PG == 1) x = (float)(_Float16)x;  // v_cvt_f16_f32 and back
  if constexpr (PG == 2) x = (float)(__bf16)x;    // v_cvt_pk_bf16_f32 and back
  return x;
}

template <int PG>
__device__ __forceinline__ float pseudo_grad(float th0, float th_r) {
  return round_through<PG>(th0 - th_r);
}

__device__ __forceinline__ void nesterov_elem(float& th0, float& b, float dbar, float lr,
                                              float mu) {
  const float bn = mu * b + dbar;
  th0 = th0 - lr * (dbar + mu * bn);
  b = bn;
}

// sum / k.  For a power-of-two k the quotient and the product with the exactly representable
// 1/k are the same real number, hence the same correctly rounded float (subnormal results
// included); the product costs one instruction instead of an IEEE division sequence.
template <bool POW2>
__device__ __forceinline__ float mean_of_sum(float s, const OuterArgs& a) {
  if constexpr (POW2) return s * a.inv_kf;
  else return s / a.kf;
}

// B/64 waves per workgroup, each wave one 256-element tile: all K+2 loads in flight, then the
// arithmetic, then K+2 stores.  The library launches single-wave workgroups (B = 64); larger B
// exists for the launch-shape sweeps.
// RM: the average is rounded through the pseudo-gradient type as well.
template <int K, int PG, bool RM, int B>
__global__ __launch_bounds__(B) void outer_fused_kernel(const OuterArgs a, uint32_t tiles) {
  constexpr bool NT = true;
  constexpr bool POW2 = (K & (K - 1)) == 0;
  f32x4* __restrict__ t0_p = reinterpret_cast<f32x4*>(a.theta0);
  f32x4* __restrict__ b_p = reinterpret_cast<f32x4*>(a.mom);
  f32x4* __restrict__ th_p = reinterpret_cast<f32x4*>(a.theta);
  const size_t rstride = a.stride / kVecElems;  // replica stride in vectors
  const size_t i = (size_t)blockIdx.x * B + threadIdx.x;  // one workgroup per B*4 elements
  f32x4 t0 = ld<NT>(t0_p + i);
  f32x4 b = ld<NT>(b_p + i);
  f32x4 th[K];
#pragma unroll
  for (int r = 0; r < K; ++r) th[r] = ld<NT>(th_p + (size_t)r * rstride + i);
#pragma unroll
  for (int c = 0; c < kVecElems; ++c) {
    float s = pseudo_grad<PG>(t0[c], th[0][c]);
#pragma unroll
    for (int r = 1; r < K; ++r) s = s + pseudo_grad<PG>(t0[c], th[r][c]);
    float dbar = mean_of_sum<POW2>(s, a);
    if constexpr (RM) dbar = round_through<PG>(dbar);
    float t = t0[c], bb = b[c];
    nesterov_elem(t, bb, dbar, a.lr, a.mu);
    t0[c] = t;
    b[c] = bb;
  }
  st<NT>(t0_p + i, t0);
  st<NT>(b_p + i, b);
#pragma unroll
  for (int r = 0; r < K; ++r) st<NT>(th_p + (size_t)r * rstride + i, t0);
  if (tiles == 0xffffffffu) occupancy_pad[threadIdx.x] = 0.f;  // never true: keeps the LDS pad
}

// Any k (run-time loop over the workers), in batches of up to 16 workers whose loads are all in
// flight together; the sum still runs over the workers in ascending order.
// BCAST = false is the delayed variant: a.theta is a snapshot of the workers' weights, theta0 and
// mom are updated, and no worker is reset.
template <int PG, bool RM, int B, bool BCAST>
__global__ __launch_bounds__(B) void outer_fused_anyk_kernel(const OuterArgs a, uint32_t tiles) {
  constexpr bool NT = true;
  constexpr int kBatch = 16;
  f32x4* __restrict__ t0_p = reinterpret_cast<f32x4*>(a.theta0);
  f32x4* __restrict__ b_p = reinterpret_cast<f32x4*>(a.mom);
  f32x4* __restrict__ th_p = reinterpret_cast<f32x4*>(a.theta);
  const size_t rstride = a.stride / kVecElems;
  const size_t i = (size_t)blockIdx.x * B + threadIdx.x;
  f32x4 t0 = ld<NT>(t0_p + i);
  f32x4 b = ld<NT>(b_p + i);
  f32x4 s = {0.f, 0.f, 0.f, 0.f};
  for (int r0 = 0; r0 < a.k; r0 += kBatch) {
    f32x4 th[kBatch];
#pragma unroll
    for (int j = 0; j < kBatch; ++j)
      if (r0 + j < a.k) th[j] = ld<NT>(th_p + (size_t)(r0 + j) * rstride + i);
#pragma unroll
    for (int j = 0; j < kBatch; ++j) {
      if (r0 + j < a.k) {
#pragma unroll
        for (int c = 0; c < kVecElems; ++c) {
          const float d = pseudo_grad<PG>(t0[c], th[j][c]);
          // the first worker's pseudo-gradient starts the sum (0 + d would lose the sign of -0)
          s[c] = (j == 0 && r0 == 0) ? d : s[c] + d;
        }
      }
    }
  }
  const bool pow2 = (a.k & (a.k - 1)) == 0;
#pragma unroll
  for (int c = 0; c < kVecElems; ++c) {
    float dbar = pow2 ? mean_of_sum<true>(s[c], a) : mean_of_sum<false>(s[c], a);
    if constexpr (RM) dbar = round_through<PG>(dbar);
    float t = t0[c], bb = b[c];
    nesterov_elem(t, bb, dbar, a.lr, a.mu);
    t0[c] = t;
    b[c] = bb;
  }
  st<NT>(t0_p + i, t0);
  st<NT>(b_p + i, b);
  if constexpr (BCAST)
    for (int r = 0; r < a.k; ++r) st<NT>(th_p + (size_t)r * rstride + i, t0);
  if (tiles == 0xffffffffu) occupancy_pad[threadIdx.x] = 0.f;  // never true: keeps the LDS pad
}

// ------------------------------------------------------------------------------------------
// Delayed application of the outer step (the asynchronous weight averaging the paper's
// Conclusion names as future work): snapshot at the round boundary, and the later merge
//   theta_r <- theta0_new - (snapshot_r - theta_r),
// which keeps what each worker did since the snapshot.
// ------------------------------------------------------------------------------------------
template <int B>
__global__ __launch_bounds__(B) void snapshot_kernel(const float* __restrict__ theta,
                                                     float* __restrict__ snap, uint64_t stride,
                                                     uint64_t snap_stride, uint32_t tiles) {
  const size_t e = (size_t)blockIdx.x * B + threadIdx.x;
  const size_t i = (size_t)blockIdx.y * (stride / kVecElems) + e;
  const size_t j = (size_t)blockIdx.y * (snap_stride / kVecElems) + e;
  st<true>(reinterpret_cast<f32x4*>(snap) + j, ld<true>(reinterpret_cast<const f32x4*>(theta) + i));
  if (tiles == 0xffffffffu) occupancy_pad[threadIdx.x] = 0.f;  // never true: keeps the LDS pad
}

// One workgroup per tile for all k workers, so that theta0 is read once per element and not once
// per worker: 1 + 2k read streams and k write streams, (4 + 12k) B per element.  Workers go in
// batches of up to 8 (16 loads in flight per lane beside theta0).
template <int B>
__global__ __launch_bounds__(B) void merge_delayed_kernel(const float* __restrict__ theta0,
                                                          const float* __restrict__ snap,
                                                          float* __restrict__ theta, uint64_t stride,
                                                          uint64_t snap_stride, int k,
                                                          uint32_t tiles) {
  constexpr int kBatch = 8;
  const size_t e = (size_t)blockIdx.x * B + threadIdx.x;
  const size_t rstride = stride / kVecElems, sstride = snap_stride / kVecElems;
  const f32x4* __restrict__ sg_p = reinterpret_cast<const f32x4*>(snap) + e;
  f32x4* __restrict__ th_p = reinterpret_cast<f32x4*>(theta) + e;
  const f32x4 t0 = ld<true>(reinterpret_cast<const f32x4*>(theta0) + e);
  for (int r0 = 0; r0 < k; r0 += kBatch) {
    f32x4 sg[kBatch], th[kBatch];
#pragma unroll
    for (int j = 0; j < kBatch; ++j)
      if (r0 + j < k) {
        sg[j] = ld<true>(sg_p + (size_t)(r0 + j) * sstride);
        th[j] = ld<true>(th_p + (size_t)(r0 + j) * rstride);
      }
#pragma unroll
    for (int j = 0; j < kBatch; ++j)
      if (r0 + j < k) {
#pragma unroll
        for (int c = 0; c < kVecElems; ++c) {
          const float since_snapshot = sg[j][c] - th[j][c];
          th[j][c] = t0[c] - since_snapshot;
        }
        st<true>(th_p + (size_t)(r0 + j) * rstride, th[j]);
      }
  }
  if (tiles == 0xffffffffu) occupancy_pad[threadIdx.x] = 0.f;  // never true: keeps the LDS pad
}

// ------------------------------------------------------------------------------------------
// Gradient-scaler check: found_inf[r] = any element of worker r's gradient is inf or NaN.
// Per lane a "bad" predicate; wave-level ballot; the four waves of a block meet in LDS; one
// atomic per block, and only when something was found.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ bool nonfinite_f16x2(uint32_t w) {
  const uint32_t e = w & 0x7c007c00u;
  return (e & 0xffffu) == 0x7c00u || (e >> 16) == 0x7c00u;
}
__device__ __forceinline__ bool nonfinite_f32(uint32_t w) {
  return (w & 0x7f800000u) == 0x7f800000u;
}

template <int B, int V, bool G16>
__global__ __launch_bounds__(B) void unscale_check_kernel(const void* g, uint64_t g_stride,
                                                          uint32_t tiles, int32_t* found_inf) {
  if (tiles == 0xffffffffu) occupancy_pad[threadIdx.x] = 0.f;  // keeps the LDS pad allocated
  const uint32_t r = blockIdx.y;
  const size_t elem_bytes = G16 ? 2 : 4;
  const u32x4* __restrict__ p = reinterpret_cast<const u32x4*>(
      static_cast<const char*>(g) + (size_t)r * g_stride * elem_bytes);
  constexpr uint32_t kTileVecs = B * V;
  bool bad = false;
  for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    const size_t base = (size_t)tile * kTileVecs + threadIdx.x;
    u32x4 w[V];
#pragma unroll
    for (int j = 0; j < V; ++j) w[j] = ld<true>(p + base + (size_t)j * B);
#pragma unroll
    for (int j = 0; j < V; ++j) {
#pragma unroll
      for (int c = 0; c < 4; ++c) bad |= G16 ? nonfinite_f16x2(w[j][c]) : nonfinite_f32(w[j][c]);
    }
  }
  // Cross-lane any-reduce: ballot inside each wave, LDS across the block's waves, then one
  // atomic per block and only when something was found (so clean gradients cost no atomics).
  const bool wave_any = __ballot(bad) != 0ull;
  if constexpr (B == 64) {
    if (threadIdx.x == 0 && wave_any) atomicOr(found_inf + r, 1);
  } else {
    __shared__ int wave_bad[B / 64];
    if ((threadIdx.x & 63) == 0) wave_bad[threadIdx.x >> 6] = wave_any ? 1 : 0;
    __syncthreads();
    if (threadIdx.x == 0) {
      int any = 0;
#pragma unroll
      for (int w = 0; w < B / 64; ++w) any |= wave_bad[w];
      if (any) atomicOr(found_inf + r, 1);
    }
  }
}

__global__ void zero_flags_kernel(int32_t* flags, int k) {
  if ((int)threadIdx.x < k) flags[threadIdx.x] = 0;
}

// ------------------------------------------------------------------------------------------
// Starting state: every worker's weights = theta0, moments = 0, outer momentum = 0.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void init_state_kernel(const float* theta0, float* mom,
                                                            float* theta, float* m, float* v,
                                                            uint64_t stride, uint32_t tiles,
                                                            int k) {
  const f32x4* t0_p = reinterpret_cast<const f32x4*>(theta0);
  const size_t rstride = stride / kVecElems;
  const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
  for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    const size_t i = (size_t)tile * kBlock + threadIdx.x;
    const f32x4 x = t0_p[i];
    reinterpret_cast<f32x4*>(mom)[i] = zero;
    for (int r = 0; r < k; ++r) {
      reinterpret_cast<f32x4*>(theta)[(size_t)r * rstride + i] = x;
      reinterpret_cast<f32x4*>(m)[(size_t)r * rstride + i] = zero;
      reinterpret_cast<f32x4*>(v)[(size_t)r * rstride + i] = zero;
    }
  }
}

template <int PG>
__global__ __launch_bounds__(kBlock) void cast_kernel(const float* __restrict__ in,
                                                      uint16_t* __restrict__ out, uint64_t n) {
  const size_t step = (size_t)gridDim.x * kBlock;
  for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += step) {
    uint16_t bits;
    if constexpr (PG == 1) {
      const _Float16 h = (_Float16)in[i];
      __builtin_memcpy(&bits, &h, 2);
    } else {
      const __bf16 h = (__bf16)in[i];
      __builtin_memcpy(&bits, &h, 2);
    }
    out[i] = bits;
  }
}

// Residency.  The mixed read/write streaming kernels run fastest with a LIMITED number of waves
// resident per CU (40-50 KiB of loads in flight per CU; more in-flight requests lower the
// sustained HBM bandwidth, fewer starve it).  Measured optima on MI355X, the same at the 150M and
// the 1.1B size: the inner step wants 10 waves of 4 KiB loads each (11 with one or two workers,
// 12 with binary16 gradients, whose waves load 3.5 KiB); the outer step is tabulated per k below.
int inner_waves_auto(int k, bool g16) { return g16 ? 12 : (k <= 2 ? 11 : 10); }

// The hardware hands out LDS in granules of 1280 bytes (160 KiB / 128): a request is rounded up
// to whole granules, and that, not the runtime's occupancy query, decides how many workgroups fit
// (measured: 54272 bytes leave 2 workgroups per CU, 53248 leave 3; 32768 leave 4, 32000 leave 5).
// The pad is therefore a whole number of granules.
constexpr uint32_t kLdsGranule = 1280;

uint32_t pad_lds_bytes(int waves_per_cu, int block, uint32_t lds_per_cu) {
  if (waves_per_cu <= 0) return 0;
  int groups = waves_per_cu / (block / 64);
  if (groups < 1) groups = 1;
  if (groups >= 32) return 0;
  uint32_t bytes = lds_per_cu / (uint32_t)groups / kLdsGranule * kLdsGranule;
  if (bytes > 64000u) bytes = 64000u;  // 50 granules, under the 64 KiB per-workgroup limit: 2 groups
  return bytes;
}

// Grid size in x for `tiles` tiles: one block per tile, or persist*n_cu grid-stride blocks.
uint32_t grid_x(uint64_t tiles, int persist, int n_cu) {
  uint64_t g = tiles;
  if (persist > 0) {
    const uint64_t cap = (uint64_t)persist * (uint64_t)n_cu;
    if (g > cap) g = cap;
  }
  if (g == 0) g = 1;
  return (uint32_t)g;
}

}  // namespace

// ------------------------------------------------------------------------------------------
// Launchers.  n_pad is a multiple of 8192 elements, so every tile size below divides it.
// ------------------------------------------------------------------------------------------
hipError_t launch_prologue(RepState* state, StepEntry* table, const int32_t* found_inf,
                           double beta1, double beta2, int k, hipStream_t s) {
  hipLaunchKernelGGL(step_prologue_kernel, dim3(1), dim3(64), 0, s, state, table, found_inf, beta1,
                     beta2, k);
  return hipGetLastError();
}

template <int B, bool G16, bool GROUPS>
static hipError_t launch_inner_t(const InnerArgs& a, int k, const Tuning& t, hipStream_t s) {
  const uint64_t tiles = a.n_pad / (uint64_t)(B * kVecElems);
  const dim3 grid((uint32_t)tiles, (uint32_t)k);
  const int waves = t.inner_waves < 0 ? inner_waves_auto(k, G16) : t.inner_waves;
  const uint32_t lds = pad_lds_bytes(waves, B, t.lds_per_cu);
  hipLaunchKernelGGL((adamw_flat_kernel<B, G16, GROUPS>), grid, dim3(B), lds, s, a,
                     (uint32_t)tiles);
  return hipGetLastError();
}

template <bool G16, bool GROUPS>
static hipError_t launch_inner_b(const InnerArgs& a, int k, const Tuning& t, hipStream_t s) {
  switch (t.inner_block) {
    case 256: return launch_inner_t<256, G16, GROUPS>(a, k, t, s);
    case 128: return launch_inner_t<128, G16, GROUPS>(a, k, t, s);
    default: return launch_inner_t<64, G16, GROUPS>(a, k, t, s);
  }
}

hipError_t launch_inner(const InnerArgs& a, int k, bool g16, bool groups, const Tuning& t,
                        hipStream_t s) {
  if (groups) return g16 ? launch_inner_b<true, true>(a, k, t, s)
                         : launch_inner_b<false, true>(a, k, t, s);
  return g16 ? launch_inner_b<true, false>(a, k, t, s) : launch_inner_b<false, false>(a, k, t, s);
}

// Launch shape of the outer step: threads per workgroup and resident waves per CU, by k and
// pseudo-gradient type.  Measured optima on MI355X at the 150M and the 1.1B set (medians of 10-16
// launches; the best shape is the same at both sizes): single-wave workgroups throughout (two-wave
// workgroups, which put 2 KiB of every stream in flight from one CU at the same moment, tie at
// k <= 2 and lose 1-15 points from k = 3 on), and 9, 6, 6, 4, 4, 4, 5, 4 waves for k = 1..8.  The
// reduced-precision modes' conversions lengthen each wave's compute phase, which at k = 2, 4, 5
// wants one more wave.  One wave off the optimum costs 0.5-5 points.  The run-time-k kernel
// (k >= 9) has a rule of its own at its launch.
struct OuterShape { int block, waves; };
static bool spread_workers(const OuterArgs& a) {
  return a.worker_major != 0 && a.stride * 4 >= (10ull << 30);
}
static OuterShape outer_shape(const Tuning& t, int k, int pg, bool spread) {
  static const int kWaves32[9] = {0, 9, 6, 6, 4, 4, 4, 5, 4};
  static const int kWaves16[9] = {0, 9, 7, 6, 5, 5, 4, 5, 4};
  OuterShape s;
  s.block = t.outer_block > 0 ? t.outer_block : 64;
  if (t.outer_waves >= 0) s.waves = t.outer_waves;
  else if (k <= 8) s.waves = pg != 0 ? kWaves16[k] : kWaves32[k];
  else s.waves = 4;
  // With the workers' weights 10 GiB or more apart (worker-major arena, multi-GiB slots) the
  // k = 8 step is flat from 5 to 7 waves and 0.3 points better there than at 4 (1.1B set).
  if (t.outer_waves < 0 && spread && k == 8) s.waves = 5;
  return s;
}

template <int K, int PG, bool RM, int B>
static hipError_t launch_outer_t(const OuterArgs& a, const Tuning& t, hipStream_t s) {
  const uint64_t tiles = a.n_pad / (uint64_t)(B * kVecElems);
  const uint32_t lds = pad_lds_bytes(outer_shape(t, K, PG, spread_workers(a)).waves, B, t.lds_per_cu);
  hipLaunchKernelGGL((outer_fused_kernel<K, PG, RM, B>), dim3((uint32_t)tiles), dim3(B), lds, s, a,
                     (uint32_t)tiles);
  return hipGetLastError();
}

template <int PG, bool RM, int B>
static hipError_t launch_outer_k(const OuterArgs& a, const Tuning& t, hipStream_t s) {
  if (!t.outer_anyk) {
    switch (a.k) {
      case 1: return launch_outer_t<1, PG, RM, B>(a, t, s);
      case 2: return launch_outer_t<2, PG, RM, B>(a, t, s);
      case 3: return launch_outer_t<3, PG, RM, B>(a, t, s);
      case 4: return launch_outer_t<4, PG, RM, B>(a, t, s);
      case 5: return launch_outer_t<5, PG, RM, B>(a, t, s);
      case 6: return launch_outer_t<6, PG, RM, B>(a, t, s);
      case 7: return launch_outer_t<7, PG, RM, B>(a, t, s);
      case 8: return launch_outer_t<8, PG, RM, B>(a, t, s);
      default: break;
    }
  }
  const uint64_t tiles = a.n_pad / (uint64_t)(B * kVecElems);
  // the run-time-k kernel's own optimum (measured at k = 2 ... 32, the same in all three
  // pseudo-gradient modes): fewer waves as k grows
  int waves = t.outer_waves;
  if (waves < 0) waves = a.k <= 2 ? 8 : a.k <= 4 ? 6 : a.k <= 6 ? 5 : a.k <= 11 ? 4 : 3;
  const uint32_t lds = pad_lds_bytes(waves, B, t.lds_per_cu);
  hipLaunchKernelGGL((outer_fused_anyk_kernel<PG, RM, B, true>), dim3((uint32_t)tiles), dim3(B), lds,
                     s, a, (uint32_t)tiles);
  return hipGetLastError();
}

template <int PG, bool RM>
static hipError_t launch_outer_b(const OuterArgs& a, const Tuning& t, hipStream_t s) {
  switch (outer_shape(t, a.k, PG, spread_workers(a)).block) {
    case 128: return launch_outer_k<PG, RM, 128>(a, t, s);
    case 256: return launch_outer_k<PG, RM, 256>(a, t, s);
    default: return launch_outer_k<PG, RM, 64>(a, t, s);
  }
}

hipError_t launch_outer(const OuterArgs& a, const Tuning& t, hipStream_t s) {
  const bool rm = a.round_mean != 0;
  switch (a.pg) {
    case 1: return rm ? launch_outer_b<1, true>(a, t, s) : launch_outer_b<1, false>(a, t, s);
    case 2: return rm ? launch_outer_b<2, true>(a, t, s) : launch_outer_b<2, false>(a, t, s);
    default: return launch_outer_b<0, false>(a, t, s);  // FP32: rounding the mean is a no-op
  }
}

// The delayed update: k+2 read streams, 2 write streams; read-heavy traffic sustains more loads
// in flight than the fused step (measured optimum at k = 8: 7 waves per CU against the fused
// step's 4).  The snapshot, a plain copy with one load per wave, wants every wave slot; the
// merge, with up to 17 loads per wave, 3 waves per CU.
template <int PG, bool RM>
static hipError_t launch_outer_update_t(const OuterArgs& a, const Tuning& t, hipStream_t s) {
  constexpr int B = 64;
  const uint64_t tiles = a.n_pad / (uint64_t)(B * kVecElems);
  const int waves = t.update_waves >= 0 ? t.update_waves : 7;
  hipLaunchKernelGGL((outer_fused_anyk_kernel<PG, RM, B, false>), dim3((uint32_t)tiles), dim3(B),
                     pad_lds_bytes(waves, B, t.lds_per_cu), s, a, (uint32_t)tiles);
  return hipGetLastError();
}

hipError_t launch_outer_update(const OuterArgs& a, const Tuning& t, hipStream_t s) {
  const bool rm = a.round_mean != 0;
  switch (a.pg) {
    case 1: return rm ? launch_outer_update_t<1, true>(a, t, s) : launch_outer_update_t<1, false>(a, t, s);
    case 2: return rm ? launch_outer_update_t<2, true>(a, t, s) : launch_outer_update_t<2, false>(a, t, s);
    default: return launch_outer_update_t<0, false>(a, t, s);
  }
}

hipError_t launch_snapshot(const float* theta, float* snap, uint64_t stride, uint64_t snap_stride,
                           uint64_t n_pad, int k, const Tuning& t, hipStream_t s) {
  constexpr int B = 64;
  const uint64_t tiles = n_pad / (uint64_t)(B * kVecElems);
  hipLaunchKernelGGL(snapshot_kernel<B>, dim3((uint32_t)tiles, (uint32_t)k), dim3(B),
                     pad_lds_bytes(t.snapshot_waves >= 0 ? t.snapshot_waves : 0, B, t.lds_per_cu), s,
                     theta, snap, stride, snap_stride, (uint32_t)tiles);
  return hipGetLastError();
}

hipError_t launch_merge_delayed(const float* theta0, const float* snap, float* theta,
                                uint64_t stride, uint64_t snap_stride, uint64_t n_pad, int k,
                                const Tuning& t, hipStream_t s) {
  constexpr int B = 64;
  const uint64_t tiles = n_pad / (uint64_t)(B * kVecElems);
  hipLaunchKernelGGL(merge_delayed_kernel<B>, dim3((uint32_t)tiles), dim3(B),
                     pad_lds_bytes(t.merge_waves >= 0 ? t.merge_waves : 3, B, t.lds_per_cu), s,
                     theta0, snap, theta, stride, snap_stride, k, (uint32_t)tiles);
  return hipGetLastError();
}

template <int B, int V>
static hipError_t launch_check_t(const void* g, uint64_t g_stride, uint64_t n_pad, int k, bool g16,
                                 int32_t* found_inf, const Tuning& t, int n_cu, hipStream_t s) {
  const uint64_t vec_elems = g16 ? 8 : 4;
  const uint64_t tiles = n_pad / (vec_elems * B * V);
  const dim3 grid(grid_x(tiles, t.check_persist, n_cu), (uint32_t)k);
  const uint32_t lds = pad_lds_bytes(t.check_waves, B, t.lds_per_cu);
  if (g16)
    hipLaunchKernelGGL((unscale_check_kernel<B, V, true>), grid, dim3(B), lds, s, g, g_stride,
                       (uint32_t)tiles, found_inf);
  else
    hipLaunchKernelGGL((unscale_check_kernel<B, V, false>), grid, dim3(B), lds, s, g, g_stride,
                       (uint32_t)tiles, found_inf);
  return hipGetLastError();
}

hipError_t launch_check(const void* g, uint64_t g_stride, uint64_t n_pad, int k, bool g16,
                        int32_t* found_inf, const Tuning& t, int n_cu, hipStream_t s) {
  hipLaunchKernelGGL(zero_flags_kernel, dim3(1), dim3(64), 0, s, found_inf, k);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const bool small = t.check_block == 64;
  switch (t.check_vec) {
    case 1: return small ? launch_check_t<64, 1>(g, g_stride, n_pad, k, g16, found_inf, t, n_cu, s)
                         : launch_check_t<256, 1>(g, g_stride, n_pad, k, g16, found_inf, t, n_cu, s);
    case 2: return small ? launch_check_t<64, 2>(g, g_stride, n_pad, k, g16, found_inf, t, n_cu, s)
                         : launch_check_t<256, 2>(g, g_stride, n_pad, k, g16, found_inf, t, n_cu, s);
    case 8: return small ? launch_check_t<64, 8>(g, g_stride, n_pad, k, g16, found_inf, t, n_cu, s)
                         : launch_check_t<256, 4>(g, g_stride, n_pad, k, g16, found_inf, t, n_cu, s);
    default: return small ? launch_check_t<64, 4>(g, g_stride, n_pad, k, g16, found_inf, t, n_cu, s)
                          : launch_check_t<256, 4>(g, g_stride, n_pad, k, g16, found_inf, t, n_cu, s);
  }
}

hipError_t launch_init_state(float* theta0, float* mom, float* theta, float* m, float* v,
                             uint64_t stride, uint64_t n_pad, int k, hipStream_t s) {
  const uint64_t tiles = n_pad / (uint64_t)(kBlock * kVecElems);
  const dim3 grid((uint32_t)(tiles < 65536 ? tiles : 65536));
  hipLaunchKernelGGL(init_state_kernel, grid, dim3(kBlock), 0, s, theta0, mom, theta, m, v,
                     stride, (uint32_t)tiles, k);
  return hipGetLastError();
}

hipError_t launch_cast(const float* in, uint16_t* out, uint64_t n, int pg, hipStream_t s) {
  uint64_t blocks = (n + kBlock - 1) / kBlock;
  if (blocks > 65536) blocks = 65536;
  if (blocks == 0) return hipSuccess;
  if (pg == 2)
    hipLaunchKernelGGL(cast_kernel<2>, dim3((uint32_t)blocks), dim3(kBlock), 0, s, in, out, n);
  else
    hipLaunchKernelGGL(cast_kernel<1>, dim3((uint32_t)blocks), dim3(kBlock), 0, s, in, out, n);
  return hipGetLastError();
}

}  // namespace diloco

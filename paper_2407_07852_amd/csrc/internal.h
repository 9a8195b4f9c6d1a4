// Internal interface between the C-ABI layer (api.hip) and the gfx950 kernels (kernels.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace diloco {

// Per-worker AdamW step state, kept on the device because skip decisions (found_inf) are
// device-side.  p1 = beta1^t, p2 = beta2^t as running products in double.  Same layout as the
// public diloco_step_state.
struct RepState {
  double p1;
  double p2;
  int32_t step;
  int32_t pad;
};

// What one inner step needs to know about a worker, written by the step prologue kernel and read
// by every workgroup of the AdamW kernel: the bias corrections 1 - beta^t of the step being
// taken, and whether the worker steps at all.
struct StepEntry {
  float bc1;
  float bc2;
  int32_t active;
  int32_t pad;
};

// Launch-shape knobs (see diloco_set_tuning).
struct Tuning {
  int inner_block = 64;   // threads per workgroup (64, 128 or 256), one 128-bit vector per lane
  int inner_waves = -1;   // resident waves per CU: -1 = auto, 0 = hardware maximum
  int outer_block = -1;   // threads per workgroup of the outer step (64, 128 or 256): -1 = auto
  int outer_waves = -1;   // resident waves per CU for the outer step: -1 = auto, 0 = maximum
  int outer_anyk = 0;     // 1: use the run-time-k kernel for every k (comparison with the templates)
  int snapshot_waves = -1;  // delayed outer step: resident waves per CU of its three kernels,
  int update_waves = -1;    // -1 = automatic, 0 = hardware maximum
  int merge_waves = -1;
  int check_block = 256;  // 64 or 256
  int check_vec = 4;      // 1, 2, 4 (8 with 64-thread blocks)
  int check_waves = 16;   // resident waves per CU (0 = hardware maximum)
  int check_persist = 0;  // inf/NaN check: grid-stride blocks per CU (0: one tile per block)
  uint32_t lds_per_cu = 160 * 1024;  // set from the device properties at init
};

struct InnerArgs {
  float* theta;        // replica 0
  float* m;
  float* v;
  const void* g;       // replica 0; float or binary16
  uint64_t stride;     // elements between replicas of theta/m/v
  uint64_t g_stride;   // elements between replicas of g
  uint64_t n_pad;
  const StepEntry* table;  // device, [k], written by the prologue launch just before
  float beta1, beta2, omb1, omb2, lr, lr_wd, eps, inv_scale;
  // parameter groups (only read by the grouped kernel variant)
  const uint32_t* chunk_group;  // device, one group id byte per 64-element chunk, 4 per word
  float lr_g[8];
  float lr_wd_g[8];
};

struct OuterArgs {
  float* theta0;
  float* mom;
  float* theta;      // replica 0 (the delayed update reads the snapshot here instead)
  uint64_t stride;
  uint64_t n_pad;
  float lr, mu, kf, inv_kf;  // inv_kf = 1/k, used when k is a power of two (exact)
  int k;
  int pg;          // pseudo-gradient type: 0 binary32, 1 binary16, 2 bfloat16
  int round_mean;  // also round the average through that type
  int worker_major;  // the arena's order (launch shape only): workers 4 slots apart
};

// Advances every worker's step state in place (unless its found_inf flag is set) and writes the
// step table the AdamW launch that follows reads.  One small launch; replay-safe in a HIP graph.
hipError_t launch_prologue(RepState* state, StepEntry* table, const int32_t* found_inf,
                           double beta1, double beta2, int k, hipStream_t s);
hipError_t launch_inner(const InnerArgs& a, int k, bool g16, bool groups, const Tuning& t,
                        hipStream_t s);
hipError_t launch_outer(const OuterArgs& a, const Tuning& t, hipStream_t s);
// Delayed application of the outer step: copy of every worker's weights into the snapshot; the
// outer update computed from the snapshot (a.theta = snapshot; theta0 and mom updated, no
// broadcast); and theta_r <- theta0 - (snapshot_r - theta_r).  The snapshot's rows are
// snap_stride elements apart, the workers' weights stride.
hipError_t launch_snapshot(const float* theta, float* snap, uint64_t stride, uint64_t snap_stride,
                           uint64_t n_pad, int k, const Tuning& t, hipStream_t s);
hipError_t launch_outer_update(const OuterArgs& a, const Tuning& t, hipStream_t s);
hipError_t launch_merge_delayed(const float* theta0, const float* snap, float* theta,
                                uint64_t stride, uint64_t snap_stride, uint64_t n_pad, int k,
                                const Tuning& t, hipStream_t s);
hipError_t launch_check(const void* g, uint64_t g_stride, uint64_t n_pad, int k, bool g16,
                        int32_t* found_inf, const Tuning& t, int n_cu, hipStream_t s);
hipError_t launch_init_state(float* theta0, float* mom, float* theta, float* m, float* v,
                             uint64_t stride, uint64_t n_pad, int k, hipStream_t s);
hipError_t launch_cast(const float* in, uint16_t* out, uint64_t n, int pg, hipStream_t s);

}  // namespace diloco

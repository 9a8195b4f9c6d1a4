// C ABI of the DiLoCo optimizer hot path (see include/diloco.h): argument validation, the
// flat layout planner, the context, and the kernel launches.  Host code only.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/diloco.h"
#include "internal.h"

using namespace diloco;

struct diloco_ctx {
  diloco_config cfg;               // numel pointer re-targeted to `numel` below
  std::vector<uint64_t> numel;
  std::vector<uint64_t> offsets;
  diloco_layout lay;
  hipStream_t stream;
  int device;
  int n_cu;
  RepState* d_state;               // device, [k]: per-worker step state, advanced on the device
  StepEntry* d_table;              // device, [k]: per-step scratch written by the prologue launch
  uint32_t steps_since_outer;
  const void* ok_grads;            // last gradient buffer whose extent was validated ...
  uint64_t ok_grads_bytes;         // ... for at least this many bytes
  bool have_scale;                 // an unscale_check has recorded (flags, inv_scale)
  float inv_scale;
  const int32_t* checked_flags;
  const void* checked_grads;
  // parameter groups
  uint32_t n_groups;               // 0 = single group from cfg
  uint32_t* d_chunk_group;         // device, [n_pad / 64] group id bytes, read as 32-bit words
  double lr_scale[DILOCO_MAX_GROUPS];
  double group_wd[DILOCO_MAX_GROUPS];
  // delayed application of the outer step
  hipEvent_t ev_snapshot;          // main stream: the snapshot is complete
  hipEvent_t ev_update;            // side stream: theta0 and mom hold the new outer state
  bool have_events;
  bool outer_pending;              // between diloco_outer_begin and diloco_outer_finish
  float* pending_snapshot;
  Tuning tune;
  std::string err;
};

namespace {

// Last error of the calling thread for calls without a context: a fixed buffer, so that
// reporting an error never allocates.
thread_local char g_err[512] = "";

int fail(diloco_ctx* ctx, int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  if (ctx) ctx->err = g_err;
  return code;
}

int fail_hip(diloco_ctx* ctx, const char* what, hipError_t e) {
  return fail(ctx, DILOCO_ERR_HIP, "%s: %s (%d)", what, hipGetErrorString(e), (int)e);
}

uint64_t round_up(uint64_t x, uint64_t to) { return (x + to - 1) / to * to; }

bool finite_in(double x, double lo, bool lo_open, double hi, bool hi_open) {
  if (!std::isfinite(x)) return false;
  if (lo_open ? !(x > lo) : !(x >= lo)) return false;
  if (hi_open ? !(x < hi) : !(x <= hi)) return false;
  return true;
}

// Shape / hyper-parameter validation shared by query_layout and init (no GPU involved).
int validate_problem(const diloco_config* cfg) {
  if (!cfg) return fail(nullptr, DILOCO_ERR_INVALID_ARG, "config is NULL");
  if (cfg->n_tensors == 0 || !cfg->numel)
    return fail(nullptr, DILOCO_ERR_INVALID_ARG, "empty parameter tensor list");
  if (cfg->k_workers == 0 || cfg->k_workers > DILOCO_MAX_WORKERS)
    return fail(nullptr, DILOCO_ERR_INVALID_ARG, "k_workers must be in 1..%d, got %u",
                DILOCO_MAX_WORKERS, cfg->k_workers);
  if (cfg->layout_mode != DILOCO_LAYOUT_AUTO && cfg->layout_mode != DILOCO_LAYOUT_BUFFER_MAJOR &&
      cfg->layout_mode != DILOCO_LAYOUT_WORKER_MAJOR)
    return fail(nullptr, DILOCO_ERR_INVALID_ARG, "unknown layout_mode %d", cfg->layout_mode);
  uint64_t total = 0;
  for (uint32_t t = 0; t < cfg->n_tensors; ++t) {
    if (cfg->numel[t] == 0)
      return fail(nullptr, DILOCO_ERR_INVALID_ARG, "tensor %u has zero elements", t);
    // 2^33 elements per replica keeps (workgroups x 64 threads) of the one-tile-per-workgroup
    // launches below 2^32; five FP32 buffers of that size already exceed the GPU's memory.
    if (cfg->numel[t] > (1ull << 33) || (total += cfg->numel[t]) > (1ull << 33))
      return fail(nullptr, DILOCO_ERR_INVALID_ARG, "parameter count exceeds 2^33 per replica");
  }
  return DILOCO_OK;
}

int validate_hyper(const diloco_config* cfg) {
  const double inf = HUGE_VAL;
  if (!finite_in(cfg->inner_lr, 0, false, inf, true) ||
      !finite_in(cfg->outer_lr, 0, false, inf, true))
    return fail(nullptr, DILOCO_ERR_INVALID_ARG, "learning rates must be finite and >= 0");
  if (!finite_in(cfg->beta1, 0, false, 1, true) || !finite_in(cfg->beta2, 0, false, 1, true))
    return fail(nullptr, DILOCO_ERR_INVALID_ARG, "betas must be in [0, 1)");
  if (!finite_in(cfg->eps, 0, true, inf, true))
    return fail(nullptr, DILOCO_ERR_INVALID_ARG, "eps must be finite and > 0");
  if (!finite_in(cfg->weight_decay, 0, false, inf, true))
    return fail(nullptr, DILOCO_ERR_INVALID_ARG, "weight_decay must be finite and >= 0");
  if (!finite_in(cfg->outer_momentum, 0, false, 1, true))
    return fail(nullptr, DILOCO_ERR_INVALID_ARG, "outer_momentum must be in [0, 1)");
  if (cfg->pg_dtype != DILOCO_F32 && cfg->pg_dtype != DILOCO_F16 && cfg->pg_dtype != DILOCO_BF16)
    return fail(nullptr, DILOCO_ERR_INVALID_ARG, "unknown pg_dtype %d", cfg->pg_dtype);
  if (cfg->pg_round_mean != 0 && cfg->pg_round_mean != 1)
    return fail(nullptr, DILOCO_ERR_INVALID_ARG, "pg_round_mean must be 0 or 1");
  return DILOCO_OK;
}

void plan(const diloco_config* cfg, diloco_layout* lay, uint64_t* offsets) {
  uint64_t cursor = 0;
  for (uint32_t t = 0; t < cfg->n_tensors; ++t) {
    cursor = round_up(cursor, DILOCO_TENSOR_ALIGN);
    if (offsets) offsets[t] = cursor;
    cursor += cfg->numel[t];
  }
  const uint64_t n_pad = round_up(cursor, DILOCO_TILE);
  const uint64_t k = cfg->k_workers;
  lay->n_pad = n_pad;
  // All flat buffers start 2 MiB-aligned relative to each other: the streams of a tile then
  // share their offset inside the GPU's 2 MiB page fragments (measured +4 % on the outer step;
  // larger alignments and skews between the buffers measured neutral or worse).
  const uint64_t slot = round_up(n_pad, DILOCO_STRIDE_ALIGN_BYTES / 4);
  const uint64_t sb = slot * 4;  // bytes per slot
  // Which order: measured on MI355X, the inner step sustains most when a worker's four streams
  // are adjacent -- by 1.6 to 3 points for slots of 2 GiB and more (0.6 to 3.5 B parameters,
  // k = 4 and 8), within +-0.5 point for smaller slots -- and the outer step when consecutive
  // workers' weights lie 12-20 GiB apart or, for small slots, directly adjacent (150M set, k = 8:
  // 80.2 % adjacent against 79.1 % with 3.5 GiB between them; 1.1B set: 80.9 % at 16.4 GiB against
  // 79.2 % adjacent).  Worker-major spaces the workers 4 slots apart.  The inner step runs H
  // times per outer step, so it decides from 2 GiB slots on; below that the outer step does --
  // unless the arena outgrows 64 GiB, the period of the memory system's position effect: then
  // buffer-major puts a worker's four streams into different 64 GiB blocks and loses on both
  // steps whatever the slot size (150M set, k = 24: inner 79.0 / outer 74.6 % against 83.1 / 77.9 %).
  int mode = cfg->layout_mode;
  if (mode == DILOCO_LAYOUT_AUTO)
    mode = (sb >= (2ull << 30) || (2 + 4 * k) * sb > (64ull << 30)) ? DILOCO_LAYOUT_WORKER_MAJOR
                                                                   : DILOCO_LAYOUT_BUFFER_MAJOR;
  lay->slot = slot;
  lay->layout_mode = mode;
  lay->reserved = 0;
  lay->off_theta0 = 0;
  lay->off_mom = sb;
  lay->off_theta = 2 * sb;
  if (mode == DILOCO_LAYOUT_WORKER_MAJOR) {
    lay->stride = 4 * slot;
    lay->off_m = lay->off_theta + sb;
    lay->off_v = lay->off_theta + 2 * sb;
    lay->off_grads = lay->off_theta + 3 * sb;
  } else {
    lay->stride = slot;
    lay->off_m = lay->off_theta + k * sb;
    lay->off_v = lay->off_m + k * sb;
    lay->off_grads = lay->off_v + k * sb;
  }
  lay->arena_bytes = (2 + 4 * k) * sb;
}

// The [ptr, ptr+bytes) range must lie inside one device allocation of the current device.
// device >= 0: it must also be memory of that device.
int check_device_range(diloco_ctx* ctx, int device, const void* ptr, uint64_t bytes,
                       const char* name) {
  hipPointerAttribute_t attr;
  hipError_t e = hipPointerGetAttributes(&attr, ptr);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return fail(ctx, DILOCO_ERR_INVALID_ARG, "%s is not a device pointer (%s)", name,
                hipGetErrorString(e));
  }
  if (attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeManaged)
    return fail(ctx, DILOCO_ERR_INVALID_ARG, "%s is not device memory", name);
  if (device >= 0 && attr.type == hipMemoryTypeDevice && attr.device != device)
    return fail(ctx, DILOCO_ERR_INVALID_ARG, "%s lives on device %d, the context on device %d",
                name, attr.device, device);
  hipDeviceptr_t base = nullptr;
  size_t size = 0;
  e = hipMemGetAddressRange(&base, &size, const_cast<void*>(ptr));
  if (e != hipSuccess) {
    // Memory the runtime cannot attribute to one allocation (e.g. virtual-memory mappings):
    // the pointer class and device were verified above, the extent cannot be.
    (void)hipGetLastError();
    return DILOCO_OK;
  }
  const uintptr_t lo = (uintptr_t)base, p = (uintptr_t)ptr;
  if (p < lo || p + bytes > lo + size)
    return fail(ctx, DILOCO_ERR_INVALID_ARG,
                "%s: %llu bytes do not fit its allocation (%zu bytes from its base)", name,
                (unsigned long long)bytes, size - (p - lo));
  return DILOCO_OK;
}

float* buf(const diloco_ctx* c, uint64_t off) {
  return reinterpret_cast<float*>(static_cast<char*>(c->cfg.arena) + off);
}

int check_grads(diloco_ctx* ctx, const void* grads, uint64_t grad_stride, int32_t grad_dtype) {
  if (!grads) return fail(ctx, DILOCO_ERR_INVALID_ARG, "grads is NULL");
  if (grad_dtype != DILOCO_F32 && grad_dtype != DILOCO_F16)
    return fail(ctx, DILOCO_ERR_INVALID_ARG, "unknown grad_dtype %d", grad_dtype);
  if (grad_stride < ctx->lay.n_pad)
    return fail(ctx, DILOCO_ERR_INVALID_ARG, "grad_stride %llu is below n_pad %llu",
                (unsigned long long)grad_stride, (unsigned long long)ctx->lay.n_pad);
  if (((uintptr_t)grads & 15u) != 0 || (grad_stride & 7u) != 0)
    return fail(ctx, DILOCO_ERR_ALIGN,
                "grads must be 16-byte aligned and grad_stride a multiple of 8 elements");
  const uint64_t esz = grad_dtype == DILOCO_F16 ? 2 : 4;
  const uint64_t bytes = ((uint64_t)(ctx->cfg.k_workers - 1) * grad_stride + ctx->lay.n_pad) * esz;
  // Steady state: the same buffer as last time needs no runtime query (a training loop passes
  // one gradient buffer for thousands of steps; the queries cost two driver calls each).
  if (grads == ctx->ok_grads && bytes <= ctx->ok_grads_bytes) return DILOCO_OK;
  const int rc = check_device_range(ctx, ctx->device, grads, bytes, "grads");
  if (rc == DILOCO_OK) {
    ctx->ok_grads = grads;
    ctx->ok_grads_bytes = bytes;
  }
  return rc;
}

// ---- scratch of the entry point that allocates nothing ---------------------------------------
// The per-step table of diloco_inner_step_noalloc: one StepEntry per worker, written by the step
// prologue kernel and read by the AdamW kernel of the same call.  Every GPU the library runs on
// holds its own copy of this array until the process ends.  In host code the array's name is
// only a stand-in; the device address comes from hipGetSymbolAddress, once per device.
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[DILOCO_MAX_WORKERS * sizeof(StepEntry)];
static void* g_scratch_ptr[kMaxDevices];  // per device, resolved with that device current
static std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (resolved on first use); *dev receives the
// device id.  Returns a HIP error code.
hipError_t scratch_on_current_device(void** ptr, int* dev) {
  hipError_t e = hipGetDevice(dev);
  if (e != hipSuccess) return e;
  if (*dev < 0 || *dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[*dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[*dev] = p;
  }
  *ptr = g_scratch_ptr[*dev];
  return hipSuccess;
}

// The AdamW kernel's scalar arguments: each is formed in double and rounded to float once.
void fill_inner_scalars(InnerArgs& a, double lr, double beta1, double beta2, double eps,
                        double weight_decay, float inv_scale) {
  a.beta1 = (float)beta1;
  a.beta2 = (float)beta2;
  a.omb1 = (float)(1.0 - beta1);
  a.omb2 = (float)(1.0 - beta2);
  a.lr = (float)lr;
  a.lr_wd = (float)(lr * weight_decay);
  a.eps = (float)eps;
  a.inv_scale = inv_scale;
}

}  // namespace

extern "C" {

int diloco_query_layout(const diloco_config* cfg, diloco_layout* out, uint64_t* tensor_offsets) {
  int rc = validate_problem(cfg);
  if (rc != DILOCO_OK) return rc;
  if (!out) return fail(nullptr, DILOCO_ERR_INVALID_ARG, "layout output is NULL");
  plan(cfg, out, tensor_offsets);
  return DILOCO_OK;
}

int diloco_init(const diloco_config* cfg, const void* const* init_params, diloco_ctx** out) {
  if (!out) return fail(nullptr, DILOCO_ERR_INVALID_ARG, "out is NULL");
  int rc = validate_problem(cfg);
  if (rc != DILOCO_OK) return rc;
  rc = validate_hyper(cfg);
  if (rc != DILOCO_OK) return rc;
  if (!cfg->arena) return fail(nullptr, DILOCO_ERR_INVALID_ARG, "arena is NULL");
  if (((uintptr_t)cfg->arena & 255u) != 0)
    return fail(nullptr, DILOCO_ERR_ALIGN, "arena must be 256-byte aligned");

  diloco_ctx* c = new (std::nothrow) diloco_ctx();
  if (!c) return fail(nullptr, DILOCO_ERR_INVALID_ARG, "out of host memory");
  c->cfg = *cfg;
  c->numel.assign(cfg->numel, cfg->numel + cfg->n_tensors);
  c->cfg.numel = c->numel.data();
  c->offsets.resize(cfg->n_tensors);
  plan(&c->cfg, &c->lay, c->offsets.data());
  c->stream = (hipStream_t)cfg->stream;
  c->d_state = nullptr;
  c->d_table = nullptr;
  c->steps_since_outer = 0;
  c->ok_grads = nullptr;
  c->ok_grads_bytes = 0;
  c->have_scale = false;
  c->inv_scale = 1.0f;
  c->checked_flags = nullptr;
  c->checked_grads = nullptr;
  c->n_groups = 0;
  c->d_chunk_group = nullptr;
  c->have_events = false;
  c->outer_pending = false;
  c->pending_snapshot = nullptr;

  auto bail = [&](int code) {
    if (c->have_events) {
      (void)hipEventDestroy(c->ev_snapshot);
      (void)hipEventDestroy(c->ev_update);
    }
    if (c->d_state) (void)hipFree(c->d_state);
    if (c->d_chunk_group) (void)hipFree(c->d_chunk_group);
    delete c;  // the message stays in the thread's buffer
    return code;
  };

  if (cfg->arena_bytes < c->lay.arena_bytes)
    return bail(fail(c, DILOCO_ERR_ARENA_TOO_SMALL, "arena has %llu bytes, layout needs %llu",
                     (unsigned long long)cfg->arena_bytes,
                     (unsigned long long)c->lay.arena_bytes));

  hipError_t e = hipGetDevice(&c->device);
  if (e != hipSuccess) return bail(fail_hip(c, "hipGetDevice (no usable GPU runtime)", e));
  hipDeviceProp_t prop;
  e = hipGetDeviceProperties(&prop, c->device);
  if (e != hipSuccess) return bail(fail_hip(c, "hipGetDeviceProperties", e));
  c->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  if (prop.maxSharedMemoryPerMultiProcessor >= 64 * 1024)
    c->tune.lds_per_cu = (uint32_t)prop.maxSharedMemoryPerMultiProcessor;

  rc = check_device_range(c, c->device, cfg->arena, c->lay.arena_bytes, "arena");
  if (rc != DILOCO_OK) return bail(rc);
  {
    // set-up is also where the static step table of diloco_inner_step_noalloc gets its device
    // address on this GPU, so that the first such call has nothing left to resolve
    void* table = nullptr;
    int dev = -1;
    e = scratch_on_current_device(&table, &dev);
    if (e != hipSuccess) return bail(fail_hip(c, "address of the static step table", e));
  }

  e = hipEventCreateWithFlags(&c->ev_snapshot, hipEventDisableTiming);
  if (e != hipSuccess) return bail(fail_hip(c, "hipEventCreate", e));
  e = hipEventCreateWithFlags(&c->ev_update, hipEventDisableTiming);
  if (e != hipSuccess) {
    (void)hipEventDestroy(c->ev_snapshot);
    return bail(fail_hip(c, "hipEventCreate", e));
  }
  c->have_events = true;

  const uint32_t k = cfg->k_workers;
  // One allocation: the step state [k], then the per-step table [k].
  e = hipMalloc(reinterpret_cast<void**>(&c->d_state), k * (sizeof(RepState) + sizeof(StepEntry)));
  if (e != hipSuccess) return bail(fail_hip(c, "hipMalloc(step state)", e));
  c->d_table = reinterpret_cast<StepEntry*>(c->d_state + k);
  std::vector<RepState> st(k);
  for (auto& s : st) { s.p1 = 1.0; s.p2 = 1.0; s.step = 0; s.pad = 0; }
  e = hipMemcpyAsync(c->d_state, st.data(), st.size() * sizeof(RepState), hipMemcpyHostToDevice,
                     c->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(c->stream);  // st is a host temporary
  if (e != hipSuccess) return bail(fail_hip(c, "step state upload", e));

  float* theta0 = buf(c, c->lay.off_theta0);
  // Pack the caller's tensors into theta0, then clear the alignment gaps and the tail.
  if (init_params) {
    for (uint32_t t = 0; t < cfg->n_tensors; ++t) {
      if (!init_params[t]) return bail(fail(c, DILOCO_ERR_INVALID_ARG, "init_params[%u] is NULL", t));
      rc = check_device_range(c, c->device, init_params[t], c->numel[t] * 4, "init_params[t]");
      if (rc != DILOCO_OK) return bail(rc);
      e = hipMemcpyAsync(theta0 + c->offsets[t], init_params[t], c->numel[t] * 4,
                         hipMemcpyDeviceToDevice, c->stream);
      if (e != hipSuccess) return bail(fail_hip(c, "pack tensor into theta0", e));
    }
  }
  for (uint32_t t = 0; t < cfg->n_tensors; ++t) {
    const uint64_t end = c->offsets[t] + c->numel[t];
    const uint64_t next = t + 1 < cfg->n_tensors ? c->offsets[t + 1] : c->lay.n_pad;
    if (next > end) {
      e = hipMemsetAsync(theta0 + end, 0, (next - end) * 4, c->stream);
      if (e != hipSuccess) return bail(fail_hip(c, "clear padding", e));
    }
  }
  e = launch_init_state(theta0, buf(c, c->lay.off_mom), buf(c, c->lay.off_theta),
                        buf(c, c->lay.off_m), buf(c, c->lay.off_v), c->lay.stride, c->lay.n_pad,
                        (int)k, c->stream);
  if (e != hipSuccess) return bail(fail_hip(c, "init_state launch", e));
  *out = c;
  return DILOCO_OK;
}

int diloco_unscale_check(diloco_ctx* ctx, const void* grads, uint64_t grad_stride,
                         int32_t grad_dtype, float inv_scale, int32_t* found_inf) {
  if (!ctx) return fail(nullptr, DILOCO_ERR_INVALID_ARG, "ctx is NULL");
  int rc = check_grads(ctx, grads, grad_stride, grad_dtype);
  if (rc != DILOCO_OK) return rc;
  if (!found_inf) return fail(ctx, DILOCO_ERR_INVALID_ARG, "found_inf is NULL");
  if (((uintptr_t)found_inf & 3u) != 0) return fail(ctx, DILOCO_ERR_ALIGN, "found_inf misaligned");
  if (!std::isfinite(inv_scale) || !(inv_scale > 0.0f))
    return fail(ctx, DILOCO_ERR_INVALID_ARG, "inv_scale must be finite and > 0");
  rc = check_device_range(ctx, ctx->device, found_inf, ctx->cfg.k_workers * 4ull, "found_inf");
  if (rc != DILOCO_OK) return rc;
  hipError_t e = launch_check(grads, grad_stride, ctx->lay.n_pad, (int)ctx->cfg.k_workers,
                              grad_dtype == DILOCO_F16, found_inf, ctx->tune, ctx->n_cu,
                              ctx->stream);
  if (e != hipSuccess) return fail_hip(ctx, "unscale_check launch", e);
  ctx->have_scale = true;
  ctx->inv_scale = inv_scale;
  ctx->checked_flags = found_inf;
  ctx->checked_grads = grads;
  return DILOCO_OK;
}

int diloco_inner_step(diloco_ctx* ctx, const void* grads, uint64_t grad_stride,
                      int32_t grad_dtype, double lr, const int32_t* found_inf) {
  if (!ctx) return fail(nullptr, DILOCO_ERR_INVALID_ARG, "ctx is NULL");
  int rc = check_grads(ctx, grads, grad_stride, grad_dtype);
  if (rc != DILOCO_OK) return rc;
  if (lr < 0) lr = ctx->cfg.inner_lr;
  if (!std::isfinite(lr)) return fail(ctx, DILOCO_ERR_INVALID_ARG, "lr must be finite");
  float inv_scale = 1.0f;
  if (found_inf) {
    if (!ctx->have_scale || ctx->checked_flags != found_inf || ctx->checked_grads != grads)
      return fail(ctx, DILOCO_ERR_STATE,
                  "found_inf given without a preceding diloco_unscale_check of these gradients");
    inv_scale = ctx->inv_scale;
  } else if (grad_dtype == DILOCO_F16) {
    // binary16 gradients exist only under a loss scale: stepping them unchecked and unscaled
    // would corrupt the weights silently
    return fail(ctx, DILOCO_ERR_STATE,
                "binary16 gradients need the found_inf flags of a preceding diloco_unscale_check");
  }
  const diloco_config& cf = ctx->cfg;
  const uint32_t k = cf.k_workers;
  InnerArgs a;
  a.theta = buf(ctx, ctx->lay.off_theta);
  a.m = buf(ctx, ctx->lay.off_m);
  a.v = buf(ctx, ctx->lay.off_v);
  a.g = grads;
  a.stride = ctx->lay.stride;
  a.g_stride = grad_stride;
  a.n_pad = ctx->lay.n_pad;
  a.table = ctx->d_table;
  fill_inner_scalars(a, lr, cf.beta1, cf.beta2, cf.eps, cf.weight_decay, inv_scale);
  a.chunk_group = ctx->d_chunk_group;
  for (uint32_t q = 0; q < DILOCO_MAX_GROUPS; ++q) {
    const bool used = q < ctx->n_groups;
    a.lr_g[q] = used ? (float)(lr * ctx->lr_scale[q]) : 0.0f;
    a.lr_wd_g[q] = used ? (float)(lr * ctx->lr_scale[q] * ctx->group_wd[q]) : 0.0f;
  }
  hipError_t e = launch_prologue(ctx->d_state, ctx->d_table, found_inf, cf.beta1, cf.beta2, (int)k,
                                 ctx->stream);
  if (e != hipSuccess) return fail_hip(ctx, "step prologue launch", e);
  e = launch_inner(a, (int)k, grad_dtype == DILOCO_F16, ctx->n_groups != 0, ctx->tune,
                   ctx->stream);
  if (e != hipSuccess) return fail_hip(ctx, "inner step launch", e);
  ctx->have_scale = false;
  ctx->steps_since_outer += 1;
  if (cf.h_inner_steps != 0 && ctx->steps_since_outer % cf.h_inner_steps == 0)
    return DILOCO_ROUND_COMPLETE;
  return DILOCO_OK;
}

int diloco_inner_step_noalloc(const diloco_inner_call* c) {
  if (!c) return fail(nullptr, DILOCO_ERR_INVALID_ARG, "call is NULL");
  if (!c->theta || !c->m || !c->v || !c->grads || !c->step_state)
    return fail(nullptr, DILOCO_ERR_INVALID_ARG, "NULL buffer in diloco_inner_call");
  if (c->k_workers == 0 || c->k_workers > DILOCO_MAX_WORKERS)
    return fail(nullptr, DILOCO_ERR_INVALID_ARG,
                "k_workers %u is outside 1..%d, the size of the library's static step table",
                c->k_workers, DILOCO_MAX_WORKERS);
  if (c->n_pad == 0 || c->n_pad % DILOCO_TILE != 0 || c->n_pad > (1ull << 33))
    return fail(nullptr, DILOCO_ERR_INVALID_ARG,
                "n_pad must be a positive multiple of %u elements, at most 2^33", DILOCO_TILE);
  if (c->stride < c->n_pad || c->grad_stride < c->n_pad)
    return fail(nullptr, DILOCO_ERR_INVALID_ARG, "stride and grad_stride must be at least n_pad");
  if (c->grad_dtype != DILOCO_F32 && c->grad_dtype != DILOCO_F16)
    return fail(nullptr, DILOCO_ERR_INVALID_ARG, "unknown grad_dtype %d", c->grad_dtype);
  if ((((uintptr_t)c->theta | (uintptr_t)c->m | (uintptr_t)c->v | (uintptr_t)c->grads) & 15u) != 0 ||
      (c->stride & 3u) != 0 || (c->grad_stride & 7u) != 0 || ((uintptr_t)c->step_state & 7u) != 0 ||
      ((uintptr_t)c->found_inf & 3u) != 0)
    return fail(nullptr, DILOCO_ERR_ALIGN,
                "buffers must be 16-byte aligned, stride a multiple of 4 and grad_stride of 8 elements");
  if (!finite_in(c->lr, 0, false, HUGE_VAL, true) || !finite_in(c->beta1, 0, false, 1, true) ||
      !finite_in(c->beta2, 0, false, 1, true) || !finite_in(c->eps, 0, true, HUGE_VAL, true) ||
      !finite_in(c->weight_decay, 0, false, HUGE_VAL, true))
    return fail(nullptr, DILOCO_ERR_INVALID_ARG, "hyper-parameter out of range");
  if (!std::isfinite(c->inv_scale) || !(c->inv_scale > 0.0f))
    return fail(nullptr, DILOCO_ERR_INVALID_ARG, "inv_scale must be finite and > 0");
  if (c->grad_dtype == DILOCO_F16 && !c->found_inf)
    return fail(nullptr, DILOCO_ERR_STATE, "binary16 gradients need found_inf flags of a check");

  void* table = nullptr;
  int dev = -1;
  hipError_t e = scratch_on_current_device(&table, &dev);
  if (e != hipSuccess) return fail_hip(nullptr, "address of the static step table", e);

  InnerArgs a;
  a.theta = c->theta;
  a.m = c->m;
  a.v = c->v;
  a.g = c->grads;
  a.stride = c->stride;
  a.g_stride = c->grad_stride;
  a.n_pad = c->n_pad;
  a.table = static_cast<const StepEntry*>(table);
  fill_inner_scalars(a, c->lr, c->beta1, c->beta2, c->eps, c->weight_decay, c->inv_scale);
  a.chunk_group = nullptr;
  for (uint32_t q = 0; q < DILOCO_MAX_GROUPS; ++q) a.lr_g[q] = a.lr_wd_g[q] = 0.0f;
  const hipStream_t stream = (hipStream_t)c->stream;
  // The prologue overwrites the first k entries of the table, which is all the AdamW kernel of
  // this call reads: nothing of an earlier call's contents is used.
  e = launch_prologue(reinterpret_cast<RepState*>(c->step_state), static_cast<StepEntry*>(table),
                      c->found_inf, c->beta1, c->beta2, (int)c->k_workers, stream);
  if (e != hipSuccess) return fail_hip(nullptr, "step prologue launch", e);
  Tuning tune;  // defaults; the LDS size of gfx950 CUs is the struct's default
  e = launch_inner(a, (int)c->k_workers, c->grad_dtype == DILOCO_F16, false, tune, stream);
  if (e != hipSuccess) return fail_hip(nullptr, "inner step launch", e);
  return DILOCO_OK;
}

int diloco_set_param_groups(diloco_ctx* ctx, const uint8_t* group_of_tensor, uint32_t n_groups,
                            const double* lr_scale, const double* weight_decay) {
  if (!ctx) return fail(nullptr, DILOCO_ERR_INVALID_ARG, "ctx is NULL");
  if (n_groups == 0) {
    ctx->n_groups = 0;
    return DILOCO_OK;
  }
  if (n_groups > DILOCO_MAX_GROUPS)
    return fail(ctx, DILOCO_ERR_INVALID_ARG, "n_groups %u exceeds %d", n_groups, DILOCO_MAX_GROUPS);
  if (!group_of_tensor || !lr_scale || !weight_decay)
    return fail(ctx, DILOCO_ERR_INVALID_ARG, "NULL group table");
  for (uint32_t q = 0; q < n_groups; ++q)
    if (!finite_in(lr_scale[q], 0, false, HUGE_VAL, true) ||
        !finite_in(weight_decay[q], 0, false, HUGE_VAL, true))
      return fail(ctx, DILOCO_ERR_INVALID_ARG, "group %u: lr_scale and weight_decay must be finite and >= 0", q);
  const uint32_t nt = ctx->cfg.n_tensors;
  for (uint32_t t = 0; t < nt; ++t)
    if (group_of_tensor[t] >= n_groups)
      return fail(ctx, DILOCO_ERR_INVALID_ARG, "tensor %u: group %u out of range", t,
                  (unsigned)group_of_tensor[t]);
  // One group id per 64-element chunk; a chunk never holds elements of two tensors because
  // every tensor starts on a 64-element boundary.  Chunks of pure padding take group 0.
  const uint64_t n_chunks = ctx->lay.n_pad / DILOCO_TENSOR_ALIGN;
  std::vector<uint8_t> map(n_chunks, 0);  // n_chunks is a multiple of 128: whole 32-bit words
  for (uint32_t t = 0; t < nt; ++t) {
    const uint64_t first = ctx->offsets[t] / DILOCO_TENSOR_ALIGN;
    const uint64_t last = (ctx->offsets[t] + ctx->numel[t] - 1) / DILOCO_TENSOR_ALIGN;
    for (uint64_t c = first; c <= last; ++c) map[c] = group_of_tensor[t];
  }
  hipError_t e = hipStreamSynchronize(ctx->stream);  // no launch may still read the old map
  if (e != hipSuccess) return fail_hip(ctx, "stream synchronize", e);
  if (!ctx->d_chunk_group) {
    e = hipMalloc(reinterpret_cast<void**>(&ctx->d_chunk_group), n_chunks);
    if (e != hipSuccess) return fail_hip(ctx, "hipMalloc(chunk groups)", e);
  }
  e = hipMemcpy(ctx->d_chunk_group, map.data(), n_chunks, hipMemcpyHostToDevice);
  if (e != hipSuccess) return fail_hip(ctx, "chunk group upload", e);
  for (uint32_t q = 0; q < n_groups; ++q) {
    ctx->lr_scale[q] = lr_scale[q];
    ctx->group_wd[q] = weight_decay[q];
  }
  ctx->n_groups = n_groups;
  return DILOCO_OK;
}

double diloco_lr_at(uint64_t step, uint64_t warmup_steps, uint64_t total_steps, double base_lr,
                    double final_ratio) {
  if (!finite_in(base_lr, 0, false, HUGE_VAL, true) ||
      !finite_in(final_ratio, 0, false, HUGE_VAL, true))
    return NAN;
  if (step < warmup_steps) return base_lr * ((double)step / (double)warmup_steps);
  if (total_steps <= warmup_steps) return base_lr;
  if (step >= total_steps) return base_lr * final_ratio;
  const double progress = (double)(step - warmup_steps) / (double)(total_steps - warmup_steps);
  const double cosine = 0.5 * (1.0 + std::cos(3.14159265358979323846 * progress));
  return base_lr * (final_ratio + (1.0 - final_ratio) * cosine);
}

static OuterArgs outer_args(const diloco_ctx* ctx, float* workers) {
  OuterArgs a;
  a.theta0 = buf(ctx, ctx->lay.off_theta0);
  a.mom = buf(ctx, ctx->lay.off_mom);
  a.theta = workers;
  a.stride = ctx->lay.stride;
  a.n_pad = ctx->lay.n_pad;
  a.lr = (float)ctx->cfg.outer_lr;
  a.mu = (float)ctx->cfg.outer_momentum;
  a.kf = (float)ctx->cfg.k_workers;
  a.inv_kf = 1.0f / a.kf;  // exact when k is a power of two, the only case that uses it
  a.k = (int)ctx->cfg.k_workers;
  a.pg = ctx->cfg.pg_dtype;
  a.round_mean = ctx->cfg.pg_round_mean;
  a.worker_major = ctx->lay.layout_mode == DILOCO_LAYOUT_WORKER_MAJOR;
  return a;
}

int diloco_outer_step(diloco_ctx* ctx) {
  if (!ctx) return fail(nullptr, DILOCO_ERR_INVALID_ARG, "ctx is NULL");
  if (ctx->outer_pending)
    return fail(ctx, DILOCO_ERR_STATE, "a delayed outer step is pending: call diloco_outer_finish");
  const OuterArgs a = outer_args(ctx, buf(ctx, ctx->lay.off_theta));
  hipError_t e = launch_outer(a, ctx->tune, ctx->stream);
  if (e != hipSuccess) return fail_hip(ctx, "outer step launch", e);
  ctx->steps_since_outer = 0;
  return DILOCO_OK;
}

int diloco_outer_begin(diloco_ctx* ctx, void* snapshot, uint64_t snapshot_bytes, void* side_stream) {
  if (!ctx) return fail(nullptr, DILOCO_ERR_INVALID_ARG, "ctx is NULL");
  if (ctx->outer_pending)
    return fail(ctx, DILOCO_ERR_STATE, "a delayed outer step is already pending");
  if (!snapshot) return fail(ctx, DILOCO_ERR_INVALID_ARG, "snapshot is NULL");
  if (((uintptr_t)snapshot & 15u) != 0)
    return fail(ctx, DILOCO_ERR_ALIGN, "snapshot must be 16-byte aligned");
  const uint64_t k = ctx->cfg.k_workers;
  const uint64_t need = ((k - 1) * ctx->lay.slot + ctx->lay.n_pad) * 4;  // dense rows
  if (snapshot_bytes < need)
    return fail(ctx, DILOCO_ERR_INVALID_ARG, "snapshot has %llu bytes, %llu are needed",
                (unsigned long long)snapshot_bytes, (unsigned long long)need);
  int rc = check_device_range(ctx, ctx->device, snapshot, need, "snapshot");
  if (rc != DILOCO_OK) return rc;
  const hipStream_t side = (hipStream_t)side_stream;
  float* snap = static_cast<float*>(snapshot);
  // main stream: snapshot of every worker's weights; everything enqueued earlier precedes it
  hipError_t e = launch_snapshot(buf(ctx, ctx->lay.off_theta), snap, ctx->lay.stride,
                                 ctx->lay.slot, ctx->lay.n_pad, (int)k, ctx->tune, ctx->stream);
  if (e != hipSuccess) return fail_hip(ctx, "snapshot launch", e);
  e = hipEventRecord(ctx->ev_snapshot, ctx->stream);
  if (e != hipSuccess) return fail_hip(ctx, "hipEventRecord", e);
  // side stream: the outer update from the snapshot.  It touches theta0, mom and the snapshot
  // only, none of which an inner step reads or writes, so inner steps enqueued on the main
  // stream from here on may run at the same time.
  e = hipStreamWaitEvent(side, ctx->ev_snapshot, 0);
  if (e != hipSuccess) return fail_hip(ctx, "hipStreamWaitEvent", e);
  OuterArgs upd = outer_args(ctx, snap);
  upd.stride = ctx->lay.slot;  // the snapshot's rows are dense
  e = launch_outer_update(upd, ctx->tune, side);
  if (e != hipSuccess) return fail_hip(ctx, "outer update launch", e);
  e = hipEventRecord(ctx->ev_update, side);
  if (e != hipSuccess) return fail_hip(ctx, "hipEventRecord", e);
  ctx->outer_pending = true;
  ctx->pending_snapshot = snap;
  ctx->steps_since_outer = 0;
  return DILOCO_OK;
}

int diloco_outer_finish(diloco_ctx* ctx) {
  if (!ctx) return fail(nullptr, DILOCO_ERR_INVALID_ARG, "ctx is NULL");
  if (!ctx->outer_pending)
    return fail(ctx, DILOCO_ERR_STATE, "no delayed outer step is pending");
  hipError_t e = hipStreamWaitEvent(ctx->stream, ctx->ev_update, 0);
  if (e != hipSuccess) return fail_hip(ctx, "hipStreamWaitEvent", e);
  e = launch_merge_delayed(buf(ctx, ctx->lay.off_theta0), ctx->pending_snapshot,
                           buf(ctx, ctx->lay.off_theta), ctx->lay.stride, ctx->lay.slot,
                           ctx->lay.n_pad, (int)ctx->cfg.k_workers, ctx->tune, ctx->stream);
  if (e != hipSuccess) return fail_hip(ctx, "merge launch", e);
  ctx->outer_pending = false;
  ctx->pending_snapshot = nullptr;
  return DILOCO_OK;
}

int diloco_get_buffer(diloco_ctx* ctx, int which, uint32_t replica, void** dev_ptr) {
  if (!ctx || !dev_ptr) return fail(ctx, DILOCO_ERR_INVALID_ARG, "NULL argument");
  if ((which == DILOCO_BUF_THETA || which == DILOCO_BUF_M || which == DILOCO_BUF_V ||
       which == DILOCO_BUF_GRADS) &&
      replica >= ctx->cfg.k_workers)
    return fail(ctx, DILOCO_ERR_INVALID_ARG, "replica %u out of range", replica);
  const uint64_t rs = (uint64_t)replica * ctx->lay.stride;
  switch (which) {
    case DILOCO_BUF_THETA0: *dev_ptr = buf(ctx, ctx->lay.off_theta0); break;
    case DILOCO_BUF_MOM: *dev_ptr = buf(ctx, ctx->lay.off_mom); break;
    case DILOCO_BUF_THETA: *dev_ptr = buf(ctx, ctx->lay.off_theta) + rs; break;
    case DILOCO_BUF_M: *dev_ptr = buf(ctx, ctx->lay.off_m) + rs; break;
    case DILOCO_BUF_V: *dev_ptr = buf(ctx, ctx->lay.off_v) + rs; break;
    case DILOCO_BUF_GRADS: *dev_ptr = buf(ctx, ctx->lay.off_grads) + rs; break;
    default: return fail(ctx, DILOCO_ERR_INVALID_ARG, "unknown buffer selector %d", which);
  }
  return DILOCO_OK;
}

int diloco_get_layout(diloco_ctx* ctx, diloco_layout* out) {
  if (!ctx || !out) return fail(ctx, DILOCO_ERR_INVALID_ARG, "NULL argument");
  *out = ctx->lay;
  return DILOCO_OK;
}

int diloco_get_steps(diloco_ctx* ctx, uint32_t* steps) {
  if (!ctx || !steps) return fail(ctx, DILOCO_ERR_INVALID_ARG, "NULL argument");
  const uint32_t k = ctx->cfg.k_workers;
  std::vector<RepState> st(k);
  hipError_t e = hipStreamSynchronize(ctx->stream);
  if (e == hipSuccess)
    e = hipMemcpy(st.data(), ctx->d_state, k * sizeof(RepState), hipMemcpyDeviceToHost);
  if (e != hipSuccess) return fail_hip(ctx, "reading step counts", e);
  for (uint32_t r = 0; r < k; ++r) steps[r] = (uint32_t)st[r].step;
  return DILOCO_OK;
}

static int cast_common(const float* in, uint16_t* out, uint64_t n, int pg, void* stream);

int diloco_cast_f32_to_f16(const float* in, uint16_t* out, uint64_t n, void* stream) {
  return cast_common(in, out, n, DILOCO_F16, stream);
}

int diloco_cast_f32_to_bf16(const float* in, uint16_t* out, uint64_t n, void* stream) {
  return cast_common(in, out, n, DILOCO_BF16, stream);
}

static int cast_common(const float* in, uint16_t* out, uint64_t n, int pg, void* stream) {
  if (n == 0) return DILOCO_OK;
  if (!in || !out) return fail(nullptr, DILOCO_ERR_INVALID_ARG, "NULL argument");
  int rc = check_device_range(nullptr, -1, in, n * 4, "in");
  if (rc != DILOCO_OK) return rc;
  rc = check_device_range(nullptr, -1, out, n * 2, "out");
  if (rc != DILOCO_OK) return rc;
  hipError_t e = launch_cast(in, out, n, pg, (hipStream_t)stream);
  if (e != hipSuccess) return fail_hip(nullptr, "cast launch", e);
  return DILOCO_OK;
}

int diloco_set_tuning(diloco_ctx* ctx, const char* name, int value) {
  if (!ctx || !name) return fail(ctx, DILOCO_ERR_INVALID_ARG, "NULL argument");
  Tuning& t = ctx->tune;
  const std::string n(name);
  const bool block_ok = value == 64 || value == 128 || value == 256;
  if (n == "inner_block" && block_ok) t.inner_block = value;
  else if (n == "outer_block" && (block_ok || value == -1)) t.outer_block = value;
  else if (n == "inner_waves" && value >= -1 && value <= 32) t.inner_waves = value;
  else if (n == "outer_waves" && value >= -1 && value <= 32) t.outer_waves = value;
  else if (n == "outer_anyk" && (value == 0 || value == 1)) t.outer_anyk = value;
  else if (n == "snapshot_waves" && value >= -1 && value <= 32) t.snapshot_waves = value;
  else if (n == "update_waves" && value >= -1 && value <= 32) t.update_waves = value;
  else if (n == "merge_waves" && value >= -1 && value <= 32) t.merge_waves = value;
  else if (n == "check_block" && (value == 64 || value == 256)) t.check_block = value;
  else if (n == "check_vec" && (value == 1 || value == 2 || value == 4 || value == 8)) t.check_vec = value;
  else if (n == "check_waves" && value >= 0 && value <= 32) t.check_waves = value;
  else if (n == "check_persist" && value >= 0 && value <= 64) t.check_persist = value;
  else return fail(ctx, DILOCO_ERR_INVALID_ARG, "unknown tuning knob or value: %s=%d", name, value);
  return DILOCO_OK;
}

const char* diloco_last_error(diloco_ctx* ctx) {
  if (ctx) return ctx->err.c_str();
  return g_err;
}

int diloco_destroy(diloco_ctx* ctx) {
  if (!ctx) return DILOCO_OK;
  hipError_t e = hipStreamSynchronize(ctx->stream);
  if (ctx->outer_pending) (void)hipEventSynchronize(ctx->ev_update);  // side-stream work still reads the arena
  if (ctx->have_events) {
    (void)hipEventDestroy(ctx->ev_snapshot);
    (void)hipEventDestroy(ctx->ev_update);
  }
  hipError_t e2 = hipFree(ctx->d_state);
  if (ctx->d_chunk_group) {
    hipError_t e3 = hipFree(ctx->d_chunk_group);
    if (e2 == hipSuccess) e2 = e3;
  }
  delete ctx;
  if (e != hipSuccess) return fail_hip(nullptr, "stream synchronize at destroy", e);
  if (e2 != hipSuccess) return fail_hip(nullptr, "hipFree at destroy", e2);
  return DILOCO_OK;
}

}  // extern "C"

// Context, error reporting, workspace arena and timing taps of libsignmuon.
#include "common.h"

#include <stdio.h>

#include <algorithm>
#include <mutex>

int sm_fail(signmuon_ctx* ctx, int code, const std::string& msg) {
  if (ctx) ctx->last_error = msg;
  return code;
}

int sm_hip_fail(signmuon_ctx* ctx, hipError_t e, const char* what) {
  std::string msg = std::string(what) + ": " + hipGetErrorString(e);
  if (ctx) ctx->last_error = msg;
  return SM_EHIP;
}

sm_launch_scope::sm_launch_scope(signmuon_ctx* c, int k) : ctx(c), klass(k) {
  if (!((ctx->profiling >> k) & 1u)) return;
  if (ctx->ev_used == ctx->ev_pool.size()) {
    sm_event_pair p;
    if (hipEventCreate(&p.a) != hipSuccess) return;
    if (hipEventCreate(&p.b) != hipSuccess) {
      (void)hipEventDestroy(p.a);
      return;
    }
    ctx->ev_pool.push_back(p);
  }
  idx = (long)ctx->ev_used++;
  (void)hipEventRecord(ctx->ev_pool[idx].a, ctx->stream);
}

sm_launch_scope::~sm_launch_scope() {
  if (idx < 0) return;
  (void)hipEventRecord(ctx->ev_pool[idx].b, ctx->stream);
  ctx->ev_log.emplace_back(klass, (size_t)idx);
}

void sm_plan_free(signmuon_ctx* ctx, int slot);  // api.hip

// Scratch of the entry point that allocates nothing (signmuon_momentum_noalloc): per-chunk partial
// sums of squares.  Every GPU the library runs on holds its own copy of this array until the
// process ends.  Host code never uses the array's name as an address: signmuon_create asks the
// runtime for the device address once per device and kernels receive that pointer as an argument.
static __device__ __align__(256) unsigned char scratch[SM_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[MAX_DEVICES] = {};

// Device address of `scratch` on device `dev`, which must be the current device.
hipError_t static_scratch_address(int dev, void** out) {
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}
}  // namespace

int sm_arena_reserve(signmuon_ctx* ctx, int slot, size_t bytes) {
  signmuon_ctx::workspace& w = ctx->ws[slot];
  if (bytes > w.bytes) {
    sm_plan_free(ctx, slot);  // a plan's zero padding does not survive a new allocation
    if (w.arena) {
      SM_HIP(ctx, hipStreamSynchronize(ctx->stream));
      SM_HIP(ctx, hipFree(w.arena));
      w.arena = nullptr;
      w.bytes = 0;
    }
    void* p = nullptr;
    hipError_t e = hipMalloc(&p, bytes);
    if (e != hipSuccess) {
      (void)hipGetLastError();
      return sm_fail(ctx, SM_ENOMEM, "workspace allocation of " + std::to_string(bytes) + " bytes failed");
    }
    w.arena = p;
    w.bytes = bytes;
  }
  ctx->arena = w.arena;
  return SM_OK;
}

int sm_aux_reserve(signmuon_ctx* ctx, size_t bytes) {
  if (bytes <= ctx->aux_bytes) return SM_OK;
  if (ctx->aux) {
    SM_HIP(ctx, hipStreamSynchronize(ctx->stream));
    SM_HIP(ctx, hipFree(ctx->aux));
    ctx->aux = nullptr;
    ctx->aux_bytes = 0;
  }
  bytes = std::max<size_t>(bytes, 1u << 20);
  void* p = nullptr;
  hipError_t e = hipMalloc(&p, bytes);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return sm_fail(ctx, SM_ENOMEM, "scratch allocation of " + std::to_string(bytes) + " bytes failed");
  }
  ctx->aux = p;
  ctx->aux_bytes = bytes;
  return SM_OK;
}

extern "C" {

int signmuon_create(signmuon_ctx** out, void* hip_stream, size_t workspace_bytes_hint) {
  if (!out) return SM_EINVAL;
  *out = nullptr;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return SM_EHIP;
  hipDeviceProp_t prop;
  e = hipGetDeviceProperties(&prop, dev);
  if (e != hipSuccess) return SM_EHIP;
  if (std::string(prop.gcnArchName).rfind("gfx950", 0) != 0) return SM_EUNSUPPORTED;
  signmuon_ctx* c = new signmuon_ctx();
  c->stream = (hipStream_t)hip_stream;
  c->device = dev;
  c->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  e = static_scratch_address(dev, &c->static_scratch);
  if (e != hipSuccess) {
    delete c;
    return SM_EHIP;
  }
  if (workspace_bytes_hint) {
    const int rc = sm_arena_reserve(c, SM_WS_STEP, workspace_bytes_hint);
    if (rc != SM_OK) {
      delete c;
      return rc;
    }
  }
  *out = c;
  return SM_OK;
}

int signmuon_destroy(signmuon_ctx* ctx) {
  if (!ctx) return SM_EINVAL;
  (void)hipStreamSynchronize(ctx->stream);
  for (int slot = 0; slot < 2; ++slot) {
    sm_plan_free(ctx, slot);
    if (ctx->ws[slot].arena) (void)hipFree(ctx->ws[slot].arena);
  }
  if (ctx->aux) (void)hipFree(ctx->aux);
  for (auto& p : ctx->ev_pool) {
    (void)hipEventDestroy(p.a);
    (void)hipEventDestroy(p.b);
  }
  delete ctx;
  return SM_OK;
}

int signmuon_set_option(signmuon_ctx* ctx, int option, int value) {
  if (!ctx) return SM_EINVAL;
  bool ok = false;
  switch (option) {
    case SM_OPT_GEMM_TILE: ok = (value == 0 || value == 128 || value == 256); break;
    case SM_OPT_NS_PATH: ok = (value >= SM_NS_PATH_PAIRS && value <= SM_NS_PATH_STEPWISE); break;
    case SM_OPT_NS_STORE: ok = (value == SM_NS_STORE_UPPER || value == SM_NS_STORE_FULL); break;
    case SM_OPT_POWER_ITER: ok = (value >= SM_PI_AUTO && value <= SM_PI_SEPARATE); break;
    default: break;
  }
  if (!ok) return sm_fail(ctx, SM_EINVAL, "set_option: unknown option or value");
  ctx->opt[option] = value;
  return SM_OK;
}

int signmuon_get_option(const signmuon_ctx* ctx, int option, int* value) {
  if (!ctx || !value || option < 0 || option >= SM_OPT_COUNT) return SM_EINVAL;
  *value = ctx->opt[option];
  return SM_OK;
}

const char* signmuon_strerror(int status) {
  switch (status) {
    case SM_OK: return "ok";
    case SM_EINVAL: return "invalid argument";
    case SM_EUNSUPPORTED: return "unsupported";
    case SM_ENOMEM: return "out of device memory";
    case SM_EHIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

const char* signmuon_last_error(const signmuon_ctx* ctx) { return ctx ? ctx->last_error.c_str() : ""; }

size_t signmuon_workspace_bytes(const signmuon_ctx* ctx) {
  return ctx ? ctx->ws[0].bytes + ctx->ws[1].bytes + ctx->aux_bytes : 0;
}

int signmuon_profile_enable(signmuon_ctx* ctx, unsigned class_mask) {
  if (!ctx) return SM_EINVAL;
  ctx->profiling = class_mask;
  return SM_OK;
}

int signmuon_profile_reset(signmuon_ctx* ctx) {
  if (!ctx) return SM_EINVAL;
  SM_HIP(ctx, hipStreamSynchronize(ctx->stream));
  ctx->ev_used = 0;
  ctx->ev_log.clear();
  for (int k = 0; k < SM_K_COUNT; ++k) ctx->work_flop[k] = ctx->work_dense[k] = ctx->work_bytes[k] = 0.0;
  return SM_OK;
}

int signmuon_profile_work(signmuon_ctx* ctx, int kernel_class, double* flop_executed, double* flop_dense,
                          double* bytes) {
  if (!ctx || kernel_class < 0 || kernel_class >= SM_K_COUNT) return SM_EINVAL;
  if (flop_executed) *flop_executed = ctx->work_flop[kernel_class];
  if (flop_dense) *flop_dense = ctx->work_dense[kernel_class];
  if (bytes) *bytes = ctx->work_bytes[kernel_class];
  return SM_OK;
}

int signmuon_profile_read(signmuon_ctx* ctx, int kernel_class, int64_t* launches, double* total_ms) {
  if (!ctx || kernel_class < 0 || kernel_class >= SM_K_COUNT) return SM_EINVAL;
  SM_HIP(ctx, hipStreamSynchronize(ctx->stream));
  int64_t n = 0;
  double ms = 0.0;
  for (auto& rec : ctx->ev_log) {
    if (rec.first != kernel_class) continue;
    float t = 0.f;
    SM_HIP(ctx, hipEventElapsedTime(&t, ctx->ev_pool[rec.second].a, ctx->ev_pool[rec.second].b));
    ms += t;
    ++n;
  }
  if (launches) *launches = n;
  if (total_ms) *total_ms = ms;
  return SM_OK;
}

const char* signmuon_kernel_name(int k) {
  switch (k) {
    case SM_K_MOMENTUM: return "sm_momentum_kernel";
    case SM_K_NS_GRAM: return "sm_ns_gemm_kernel (Gram of Y)";
    case SM_K_NS_APPLY: return "sm_ns_gemm_kernel (apply to Y)";
    case SM_K_NS_SMALL: return "sm_ns_gemm_kernel (short-side recurrence)";
    case SM_K_SIGN_PACK: return "sm_sign_pack_kernel";
    case SM_K_VOTE: return "sm_vote_kernel";
    case SM_K_UPDATE: return "sm_update_kernel";
    case SM_K_OTHER: return "other";
    case SM_K_POWER_ITER: return "sm_pi_kernels (PowerIter)";
    default: return "?";
  }
}

}  // extern "C"

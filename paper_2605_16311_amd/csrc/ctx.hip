// Context, error reporting, workspace arena and timing taps of libsignmuon.
#include "common.h"

#include <stdio.h>

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

void sm_plan_free(signmuon_ctx* ctx);  // api.hip

int sm_arena_reserve(signmuon_ctx* ctx, size_t bytes) {
  if (bytes <= ctx->arena_bytes) return SM_OK;
  sm_plan_free(ctx);  // a plan's zero padding does not survive a new allocation
  if (ctx->arena) {
    SM_HIP(ctx, hipStreamSynchronize(ctx->stream));
    SM_HIP(ctx, hipFree(ctx->arena));
    ctx->arena = nullptr;
    ctx->arena_bytes = 0;
  }
  void* p = nullptr;
  hipError_t e = hipMalloc(&p, bytes);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return sm_fail(ctx, SM_ENOMEM, "workspace allocation of " + std::to_string(bytes) + " bytes failed");
  }
  ctx->arena = p;
  ctx->arena_bytes = bytes;
  return SM_OK;
}

extern "C" {

int signmuon_create(signmuon_ctx** out, void* hip_stream) {
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
  *out = c;
  return SM_OK;
}

int signmuon_destroy(signmuon_ctx* ctx) {
  if (!ctx) return SM_EINVAL;
  (void)hipStreamSynchronize(ctx->stream);
  sm_plan_free(ctx);
  if (ctx->arena) (void)hipFree(ctx->arena);
  for (auto& p : ctx->ev_pool) {
    (void)hipEventDestroy(p.a);
    (void)hipEventDestroy(p.b);
  }
  delete ctx;
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

size_t signmuon_workspace_bytes(const signmuon_ctx* ctx) { return ctx ? ctx->arena_bytes : 0; }

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
  for (int k = 0; k < SM_K_COUNT; ++k) ctx->work_flop[k] = ctx->work_bytes[k] = 0.0;
  return SM_OK;
}

int signmuon_profile_work(signmuon_ctx* ctx, int kernel_class, double* flop, double* bytes) {
  if (!ctx || kernel_class < 0 || kernel_class >= SM_K_COUNT) return SM_EINVAL;
  if (flop) *flop = ctx->work_flop[kernel_class];
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
    default: return "?";
  }
}

}  // extern "C"

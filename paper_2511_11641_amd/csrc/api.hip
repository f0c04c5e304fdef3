// Context management and status strings of the C ABI.
#include "common.h"

#include <new>

extern "C" int ecospa_create(ecospa_ctx** out, void* hip_stream) {
  if (!out) return ECOSPA_ERR_NULL;
  ecospa_ctx* c = new (std::nothrow) ecospa_ctx;
  if (!c) return ECOSPA_ERR_NULL;
  c->stream = static_cast<hipStream_t>(hip_stream);
  c->ws = nullptr;
  c->ws_bytes = 0;
  c->err[0] = 0;
  c->prof_on = c->prof_n = c->prof_cap = 0;
  c->prof_ev = nullptr;
  c->prof_flop = nullptr;
  *out = c;
  return ECOSPA_OK;
}

extern "C" void ecospa_destroy(ecospa_ctx* ctx) {
  if (!ctx) return;
  for (int i = 0; i < 2 * ctx->prof_cap; ++i) (void)hipEventDestroy(ctx->prof_ev[i]);
  delete[] ctx->prof_ev;
  delete[] ctx->prof_flop;
  delete ctx;
}

extern "C" int ecospa_profile_gemm(ecospa_ctx* ctx, int enable) {
  if (!ctx) return ECOSPA_ERR_NULL;
  if (enable && !ctx->prof_ev) {
    ctx->prof_ev = new (std::nothrow) hipEvent_t[2 * ECOSPA_PROF_MAX];
    ctx->prof_flop = new (std::nothrow) double[ECOSPA_PROF_MAX];
    if (!ctx->prof_ev || !ctx->prof_flop) return ECOSPA_ERR_NULL;
    for (int i = 0; i < 2 * ECOSPA_PROF_MAX; ++i) {
      hipError_t e = hipEventCreate(&ctx->prof_ev[i]);
      if (e != hipSuccess) return hip_fail(ctx, e, "hipEventCreate");
    }
    ctx->prof_cap = ECOSPA_PROF_MAX;
  }
  ctx->prof_on = enable ? 1 : 0;
  if (enable) ctx->prof_n = 0;
  return ECOSPA_OK;
}

extern "C" int ecospa_profile_gemm_read(ecospa_ctx* ctx, int* launches, double* total_ms, double* total_flop) {
  if (!ctx || !launches || !total_ms || !total_flop) return ECOSPA_ERR_NULL;
  double ms = 0.0, fl = 0.0;
  for (int i = 0; i < ctx->prof_n; ++i) {
    hipError_t e = hipEventSynchronize(ctx->prof_ev[2 * i + 1]);
    if (e != hipSuccess) return hip_fail(ctx, e, "hipEventSynchronize");
    float t = 0.f;
    e = hipEventElapsedTime(&t, ctx->prof_ev[2 * i], ctx->prof_ev[2 * i + 1]);
    if (e != hipSuccess) return hip_fail(ctx, e, "hipEventElapsedTime");
    ms += t;
    fl += ctx->prof_flop[i];
  }
  *launches = ctx->prof_n;
  *total_ms = ms;
  *total_flop = fl;
  return ECOSPA_OK;
}

extern "C" int ecospa_set_workspace(ecospa_ctx* ctx, void* dev, size_t bytes) {
  if (!ctx) return ECOSPA_ERR_NULL;
  if (dev && (reinterpret_cast<uintptr_t>(dev) & 255u)) return ECOSPA_ERR_ALIGN;
  ctx->ws = dev;
  ctx->ws_bytes = dev ? bytes : 0;
  return ECOSPA_OK;
}

extern "C" const char* ecospa_status_string(int code) {
  switch (code) {
    case ECOSPA_OK: return "ok";
    case ECOSPA_ERR_NULL: return "required pointer is NULL";
    case ECOSPA_ERR_SHAPE: return "bad shape or leading dimension";
    case ECOSPA_ERR_DTYPE: return "unsupported dtype, pair kind, block kind or activation";
    case ECOSPA_ERR_K: return "k out of range";
    case ECOSPA_ERR_INDEX: return "bad index";
    case ECOSPA_ERR_WORKSPACE: return "workspace missing or too small";
    case ECOSPA_ERR_ALIGN: return "pointer or leading dimension not aligned";
    case ECOSPA_ERR_HIP: return "HIP runtime error (see ecospa_last_error)";
    default: return "unknown status";
  }
}

extern "C" const char* ecospa_last_error(const ecospa_ctx* ctx) { return ctx ? ctx->err : ""; }

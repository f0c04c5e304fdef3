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
  *out = c;
  return ECOSPA_OK;
}

extern "C" void ecospa_destroy(ecospa_ctx* ctx) { delete ctx; }

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

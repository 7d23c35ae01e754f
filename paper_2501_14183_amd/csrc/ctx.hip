// Context life cycle and error strings of libvardrop.
#include "common.h"
#include <new>

extern "C" int vardrop_create(vardrop_ctx** out, int device_id) {
  if (!out) return VARDROP_EINVAL;
  *out = nullptr;
  int count = 0;
  if (hipGetDeviceCount(&count) != hipSuccess || device_id < 0 || device_id >= count) return VARDROP_EINVAL;
  vardrop_ctx* c = new (std::nothrow) vardrop_ctx();
  if (!c) return VARDROP_EHIP;
  c->device = device_id;
  c->last_hip_error = 0;
  c->twiddle = nullptr;
  c->twiddle_L = 0;
  c->lds_per_block = 65536;
  int prev = 0;
  hipError_t e = hipGetDevice(&prev);
  if (e == hipSuccess) e = hipSetDevice(device_id);
  if (e == hipSuccess) {
    int v = 0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, device_id) == hipSuccess && v > 0)
      c->lds_per_block = v;
    e = hipMalloc((void**)&c->twiddle, sizeof(float) * 2 * kMaxTwiddleL);
    (void)hipSetDevice(prev);
  }
  if (e != hipSuccess) {
    delete c;
    return VARDROP_EHIP;
  }
  *out = c;
  return VARDROP_OK;
}

extern "C" void vardrop_destroy(vardrop_ctx* ctx) {
  if (!ctx) return;
  if (ctx->twiddle) (void)hipFree(ctx->twiddle);
  delete ctx;
}

extern "C" const char* vardrop_strerror(int code) {
  switch (code) {
    case VARDROP_OK: return "ok";
    case VARDROP_EINVAL: return "invalid argument";
    case VARDROP_EWORKSPACE: return "workspace missing, misaligned or too small";
    case VARDROP_EHIP: return "HIP runtime error";
    case VARDROP_EUNSUPPORTED: return "request outside the implemented range";
    default: return "unknown error code";
  }
}

extern "C" int vardrop_last_hip_error(const vardrop_ctx* ctx) { return ctx ? ctx->last_hip_error : 0; }

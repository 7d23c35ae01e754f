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
  c->twiddle_fmin = 0;
  c->twiddle_F = 0;
  c->twiddle_r2 = 0;
  c->prof_kid = -1;
  c->prof_n = 0;
  c->prof_stride = 1;
  c->prof_seen = 0;
  c->prof_ev = nullptr;
  c->prof_kids = nullptr;
  c->prof_e0 = nullptr;
  c->prof_e1 = nullptr;
  for (int i = 0; i < 64; ++i) c->signal_event[i] = nullptr;
  c->lds_per_block = 65536;
  c->num_cus = 256;
  c->static_scratch = nullptr;
  int prev = 0;
  hipError_t e = hipGetDevice(&prev);
  if (e == hipSuccess) e = hipSetDevice(device_id);
  if (e == hipSuccess) {
    int v = 0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, device_id) == hipSuccess && v > 0)
      c->lds_per_block = v;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, device_id) == hipSuccess && v > 0) c->num_cus = v;
    e = hipMalloc(&c->twiddle, kTwiddleBytes);
    // the static scratch array has one copy per device: its address is taken with this context's device current
    if (e == hipSuccess) {
      const int se = vd_static_scratch_address(&c->static_scratch);
      if (se != 0) e = (hipError_t)se;
    }
    if (e != hipSuccess && c->twiddle) (void)hipFree(c->twiddle);
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
  if (ctx->prof_ev) {
    for (int i = 0; i < 2 * kProfPairs; ++i) (void)hipEventDestroy(ctx->prof_ev[i]);
    delete[] ctx->prof_ev;
    delete[] ctx->prof_kids;
  }
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

extern "C" const char* vardrop_kernel_name(int kernel_id) {
  static const char* const names[VARDROP_K_COUNT] = {
      "hash", "sample", "gather", "gemm_qkv", "sdpa_fwd", "gemm_out", "gemm_do",
      "sdpa_bwd_dq", "sdpa_bwd_dkv", "gemm_dw", "reduce_dw", "gemm_dxs", "scatter", "gemm_dw_dxs", "sdpa_bwd", "qkv_sdpa_fwd",
      "embed_rows", "gemm_embed", "gemm_dwe", "sdpa_bwd_dqkv", "embed_fused"};
  return (kernel_id >= 0 && kernel_id < VARDROP_K_COUNT) ? names[kernel_id] : nullptr;
}

extern "C" int vardrop_profile_select(vardrop_ctx* ctx, int kernel_id) {
  if (!ctx || kernel_id < VARDROP_K_ALL || kernel_id >= VARDROP_K_COUNT) return VARDROP_EINVAL;
  if (kernel_id != -1 && !ctx->prof_ev) {
    hipEvent_t* ev = new (std::nothrow) hipEvent_t[2 * kProfPairs];
    short* kids = new (std::nothrow) short[kProfPairs];
    if (!ev || !kids) {
      delete[] ev;
      delete[] kids;
      return VARDROP_EHIP;
    }
    ctx->prof_kids = kids;
    for (int i = 0; i < 2 * kProfPairs; ++i) {
      hipError_t e = hipEventCreate(&ev[i]);
      if (e != hipSuccess) {
        for (int j = 0; j < i; ++j) (void)hipEventDestroy(ev[j]);
        delete[] ev;
        delete[] kids;
        ctx->prof_kids = nullptr;
        ctx->last_hip_error = (int)e;
        return VARDROP_EHIP;
      }
    }
    ctx->prof_ev = ev;
  }
  ctx->prof_kid = kernel_id;
  ctx->prof_n = 0;
  ctx->prof_seen = 0;
  return VARDROP_OK;
}

static_assert(VARDROP_K_COUNT <= 64, "one pending completion signal per kernel id");
extern "C" int vardrop_signal_after(vardrop_ctx* ctx, int kernel_id, void* event) {
  if (!ctx || kernel_id < 0 || kernel_id >= VARDROP_K_COUNT) return VARDROP_EINVAL;
  ctx->signal_event[kernel_id] = (hipEvent_t)event;
  return VARDROP_OK;
}

extern "C" int vardrop_profile_stride(vardrop_ctx* ctx, int stride) {
  if (!ctx || stride < 1) return VARDROP_EINVAL;
  ctx->prof_stride = stride;
  return VARDROP_OK;
}

extern "C" int vardrop_profile_read(vardrop_ctx* ctx, double* total_ms, int* launches) {
  if (!ctx || !total_ms || !launches) return VARDROP_EINVAL;
  double sum = 0.0;
  for (int i = 0; i < ctx->prof_n; ++i) {
    VD_HIP(ctx, hipEventSynchronize(ctx->prof_ev[2 * i + 1]));
    float ms = 0.f;
    VD_HIP(ctx, hipEventElapsedTime(&ms, ctx->prof_ev[2 * i], ctx->prof_ev[2 * i + 1]));
    sum += ms;
  }
  *total_ms = sum;
  *launches = ctx->prof_n;
  ctx->prof_n = 0;
  return VARDROP_OK;
}

extern "C" int vardrop_profile_read_all(vardrop_ctx* ctx, double* total_ms, int* launches) {
  if (!ctx || !total_ms || !launches) return VARDROP_EINVAL;
  for (int k = 0; k < VARDROP_K_COUNT; ++k) {
    total_ms[k] = 0.0;
    launches[k] = 0;
  }
  for (int i = 0; i < ctx->prof_n; ++i) {
    VD_HIP(ctx, hipEventSynchronize(ctx->prof_ev[2 * i + 1]));
    float ms = 0.f;
    VD_HIP(ctx, hipEventElapsedTime(&ms, ctx->prof_ev[2 * i], ctx->prof_ev[2 * i + 1]));
    const int k = ctx->prof_kids[i];
    total_ms[k] += ms;
    ++launches[k];
  }
  ctx->prof_n = 0;
  return VARDROP_OK;
}

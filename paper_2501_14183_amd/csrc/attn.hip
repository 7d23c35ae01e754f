// Entry points of the multi-head attention (Eq. 3): argument checks, buffer sizes and the
// dispatch to the fp32 or bf16 back end.
#include "common.h"

namespace {

int elem_size(int dtype) { return dtype == VARDROP_F32 ? 4 : (dtype == VARDROP_BF16 ? 2 : 0); }

int check_shape(int B, int n, int d, int H, int dtype) {
  if (B < 0 || n < 0 || d < 1 || H < 1 || d % H != 0) return VARDROP_EINVAL;
  if (elem_size(dtype) == 0) return VARDROP_EINVAL;
  if ((long long)B * n * d >= (1ll << 31)) return VARDROP_EUNSUPPORTED;
  const int dh = d / H;
  if (dtype == VARDROP_BF16) {
    if (dh != 64) return VARDROP_EUNSUPPORTED;
  } else if (dh != 16 && dh != 32 && dh != 64 && dh != 128) {
    return VARDROP_EUNSUPPORTED;
  }
  return VARDROP_OK;
}

__global__ void zero_f32_kernel(float* p, long long count) {
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (long long)gridDim.x * blockDim.x)
    p[i] = 0.f;
}

int zero_f32(vardrop_ctx* ctx, float* p, long long count, hipStream_t s) {
  if (!p || count == 0) return VARDROP_OK;
  long long blocks = (count + 255) / 256;
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(zero_f32_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p, count);
  VD_LAUNCH_CHECK(ctx);
  return VARDROP_OK;
}

}  // namespace

extern "C" size_t vardrop_attn_saved_bytes(int B, int n, int d, int H, int dtype) {
  if (check_shape(B, n, d, H, dtype) != VARDROP_OK) return 0;
  const size_t M = (size_t)B * n;
  return vd_align_up(4 * M * d * elem_size(dtype) + (size_t)B * H * n * sizeof(float), 256);
}

extern "C" size_t vardrop_attn_workspace_bytes(int B, int n, int d, int H, int dtype) {
  if (check_shape(B, n, d, H, dtype) != VARDROP_OK) return 0;
  if (dtype == VARDROP_BF16) return vd_attn_bf16_ws_bytes(B, n, d, H);
  return vardrop_attn_saved_bytes(B, n, d, H, dtype);   // dO, dq, dk, dv and D have the same shapes
}

extern "C" int vardrop_attn_fwd(vardrop_ctx* ctx, const void* xs, int B, int n, int d, int H, int dtype,
                                const void* Wq, const void* Wk, const void* Wv, const void* Wo,
                                const void* bq, const void* bk, const void* bv, const void* bo,
                                void* y, void* saved, void* ws, size_t ws_bytes, void* stream) {
  (void)ws_bytes;
  if (!ctx) return VARDROP_EINVAL;
  int rc = check_shape(B, n, d, H, dtype);
  if (rc) return rc;
  if ((long long)B * n == 0) return VARDROP_OK;
  if (!xs || !Wq || !Wk || !Wv || !Wo || !y || !saved) return VARDROP_EINVAL;
  if (!vd_aligned(saved, 256)) return VARDROP_EWORKSPACE;
  if (!vd_aligned(xs, 16) || !vd_aligned(y, 16) || !vd_aligned(Wq, 16) || !vd_aligned(Wk, 16) ||
      !vd_aligned(Wv, 16) || !vd_aligned(Wo, 16))
    return VARDROP_EINVAL;
  const void* W[4] = {Wq, Wk, Wv, Wo};
  const void* bias[4] = {bq, bk, bv, bo};
  hipStream_t s = (hipStream_t)stream;
  if (dtype == VARDROP_F32)
    return vd_attn_fwd_f32(ctx, (const float*)xs, B, n, d, H, (const float* const*)W, (const float* const*)bias,
                           (float*)y, saved, ws, s);
  return vd_attn_fwd_bf16(ctx, xs, B, n, d, H, W, bias, y, saved, ws, s);
}

extern "C" int vardrop_gather_attn_fwd(vardrop_ctx* ctx, const void* tokens, int B, int N, const int32_t* sel, int n,
                                       int d, int H, int dtype,
                                       const void* Wq, const void* Wk, const void* Wv, const void* Wo,
                                       const void* bq, const void* bk, const void* bv, const void* bo,
                                       void* xs, void* y, void* saved, void* ws, size_t ws_bytes, void* stream) {
  if (!ctx) return VARDROP_EINVAL;
  if (N < 0 || n > N) return VARDROP_EINVAL;
  int rc = check_shape(B, n, d, H, dtype);
  if (rc) return rc;
  if ((long long)B * n == 0) return VARDROP_OK;
  if (!tokens || !sel || !xs || !vd_aligned(tokens, 16) || !vd_aligned(xs, 16)) return VARDROP_EINVAL;
  if (dtype == VARDROP_BF16 && (long long)B * N * d >= (1ll << 31)) return VARDROP_EUNSUPPORTED;
  if (dtype == VARDROP_F32) {
    rc = vardrop_gather(ctx, tokens, B, N, d, dtype, sel, n, xs, stream);
    if (rc) return rc;
    return vardrop_attn_fwd(ctx, xs, B, n, d, H, dtype, Wq, Wk, Wv, Wo, bq, bk, bv, bo, y, saved, ws, ws_bytes, stream);
  }
  if (!Wq || !Wk || !Wv || !Wo || !y || !saved) return VARDROP_EINVAL;
  if (!vd_aligned(saved, 256)) return VARDROP_EWORKSPACE;
  if (!vd_aligned(y, 16) || !vd_aligned(Wq, 16) || !vd_aligned(Wk, 16) || !vd_aligned(Wv, 16) || !vd_aligned(Wo, 16))
    return VARDROP_EINVAL;
  const void* W[4] = {Wq, Wk, Wv, Wo};
  const void* bias[4] = {bq, bk, bv, bo};
  return vd_attn_fwd_bf16(ctx, tokens, B, n, d, H, W, bias, y, saved, ws, (hipStream_t)stream, sel, N, xs);
}

extern "C" int vardrop_attn_bwd(vardrop_ctx* ctx, const void* dy, const void* xs,
                                int B, int n, int d, int H, int dtype,
                                const void* Wq, const void* Wk, const void* Wv, const void* Wo,
                                const void* saved,
                                void* dxs, float* dWq, float* dWk, float* dWv, float* dWo,
                                float* dbq, float* dbk, float* dbv, float* dbo,
                                void* ws, size_t ws_bytes, void* stream) {
  if (!ctx) return VARDROP_EINVAL;
  int rc = check_shape(B, n, d, H, dtype);
  if (rc) return rc;
  if (!dWq || !dWk || !dWv || !dWo) return VARDROP_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  float* dW[4] = {dWq, dWk, dWv, dWo};
  float* db[4] = {dbq, dbk, dbv, dbo};
  if ((long long)B * n == 0) {
    for (int i = 0; i < 4; ++i) {
      if ((rc = zero_f32(ctx, dW[i], (long long)d * d, s))) return rc;
      if ((rc = zero_f32(ctx, db[i], d, s))) return rc;
    }
    return VARDROP_OK;
  }
  if (!dy || !xs || !Wq || !Wk || !Wv || !Wo || !saved || !dxs) return VARDROP_EINVAL;
  if (!ws || !vd_aligned(ws, 256) || ws_bytes < vardrop_attn_workspace_bytes(B, n, d, H, dtype))
    return VARDROP_EWORKSPACE;
  if (!vd_aligned(saved, 256)) return VARDROP_EWORKSPACE;
  if (!vd_aligned(xs, 16) || !vd_aligned(dy, 16) || !vd_aligned(dxs, 16) || !vd_aligned(Wq, 16) ||
      !vd_aligned(Wk, 16) || !vd_aligned(Wv, 16) || !vd_aligned(Wo, 16))
    return VARDROP_EINVAL;
  const void* W[4] = {Wq, Wk, Wv, Wo};
  if (dtype == VARDROP_F32)
    return vd_attn_bwd_f32(ctx, (const float*)dy, (const float*)xs, B, n, d, H, (const float* const*)W, saved,
                           (float*)dxs, dW, db, ws, s);
  return vd_attn_bwd_bf16(ctx, dy, xs, B, n, d, H, W, saved, dxs, dW, db, ws, s);
}

// ---------------------------------------------------------------- device-side token count
// The same two steps with the number of kept tokens read by the kernels from device memory (it is a result of the
// sampling step): nothing crosses to the host between sampling and attention, and the launches do not depend on the
// count, so a whole step can be recorded once and replayed.
extern "C" int vardrop_gather_attn_fwd_dev(vardrop_ctx* ctx, const void* tokens, int B, int N, const int32_t* sel,
                                           const int32_t* n_dev, int n_max, int32_t* status,
                                           int d, int H, int dtype,
                                           const void* Wq, const void* Wk, const void* Wv, const void* Wo,
                                           const void* bq, const void* bk, const void* bv, const void* bo,
                                           void* xs, void* y, void* saved, void* ws, size_t ws_bytes, void* stream) {
  (void)ws_bytes;
  if (!ctx || !n_dev) return VARDROP_EINVAL;
  if (N < 0 || n_max < 1 || n_max > N) return VARDROP_EINVAL;
  int rc = check_shape(B, n_max, d, H, dtype);
  if (rc) return rc;
  if (B == 0) return VARDROP_OK;
  if (!tokens || !sel || !xs || !vd_aligned(tokens, 16) || !vd_aligned(xs, 16)) return VARDROP_EINVAL;
  if (dtype == VARDROP_BF16 && (long long)B * N * d >= (1ll << 31)) return VARDROP_EUNSUPPORTED;
  if (!Wq || !Wk || !Wv || !Wo || !y || !saved) return VARDROP_EINVAL;
  if (!vd_aligned(saved, 256)) return VARDROP_EWORKSPACE;
  if (!vd_aligned(y, 16) || !vd_aligned(Wq, 16) || !vd_aligned(Wk, 16) || !vd_aligned(Wv, 16) || !vd_aligned(Wo, 16))
    return VARDROP_EINVAL;
  const void* W[4] = {Wq, Wk, Wv, Wo};
  const void* bias[4] = {bq, bk, bv, bo};
  hipStream_t s = (hipStream_t)stream;
  const VdDevCount dn = {n_dev, status};
  if (dtype == VARDROP_F32) {
    rc = vd_gather(ctx, tokens, B, N, d, dtype, sel, n_max, xs, s, dn);
    if (rc) return rc;
    return vd_attn_fwd_f32(ctx, (const float*)xs, B, n_max, d, H, (const float* const*)W, (const float* const*)bias,
                           (float*)y, saved, ws, s, VdDevCount{n_dev, nullptr});
  }
  return vd_attn_fwd_bf16(ctx, tokens, B, n_max, d, H, W, bias, y, saved, ws, s, sel, N, xs, dn);
}

// The forward pass on tokens that are already packed for the count (as vardrop_embed_fwd_dev writes them).
extern "C" int vardrop_attn_fwd_dev(vardrop_ctx* ctx, const void* xs, int B, const int32_t* n_dev, int n_max, int32_t* status,
                                    int d, int H, int dtype,
                                    const void* Wq, const void* Wk, const void* Wv, const void* Wo,
                                    const void* bq, const void* bk, const void* bv, const void* bo,
                                    void* y, void* saved, void* ws, size_t ws_bytes, void* stream) {
  (void)ws_bytes;
  if (!ctx || !n_dev || n_max < 1) return VARDROP_EINVAL;
  int rc = check_shape(B, n_max, d, H, dtype);
  if (rc) return rc;
  if (B == 0) return VARDROP_OK;
  if (!xs || !Wq || !Wk || !Wv || !Wo || !y || !saved) return VARDROP_EINVAL;
  if (!vd_aligned(saved, 256)) return VARDROP_EWORKSPACE;
  if (!vd_aligned(xs, 16) || !vd_aligned(y, 16) || !vd_aligned(Wq, 16) || !vd_aligned(Wk, 16) ||
      !vd_aligned(Wv, 16) || !vd_aligned(Wo, 16))
    return VARDROP_EINVAL;
  const void* W[4] = {Wq, Wk, Wv, Wo};
  const void* bias[4] = {bq, bk, bv, bo};
  hipStream_t s = (hipStream_t)stream;
  const VdDevCount dn = {n_dev, status};
  if (dtype == VARDROP_F32)
    return vd_attn_fwd_f32(ctx, (const float*)xs, B, n_max, d, H, (const float* const*)W, (const float* const*)bias,
                           (float*)y, saved, ws, s, dn);
  return vd_attn_fwd_bf16(ctx, xs, B, n_max, d, H, W, bias, y, saved, ws, s, nullptr, 0, nullptr, dn);
}

extern "C" int vardrop_attn_bwd_dev(vardrop_ctx* ctx, const void* dy, const void* xs,
                                    int B, const int32_t* n_dev, int n_max, int32_t* status, int d, int H, int dtype,
                                    const void* Wq, const void* Wk, const void* Wv, const void* Wo,
                                    const void* saved,
                                    void* dxs, float* dWq, float* dWk, float* dWv, float* dWo,
                                    float* dbq, float* dbk, float* dbv, float* dbo,
                                    void* ws, size_t ws_bytes, void* stream) {
  if (!ctx || !n_dev || n_max < 1) return VARDROP_EINVAL;
  int rc = check_shape(B, n_max, d, H, dtype);
  if (rc) return rc;
  if (B < 1) return VARDROP_EINVAL;
  if (!dWq || !dWk || !dWv || !dWo) return VARDROP_EINVAL;
  if (!dy || !xs || !Wq || !Wk || !Wv || !Wo || !saved || !dxs) return VARDROP_EINVAL;
  if (!ws || !vd_aligned(ws, 256) || ws_bytes < vardrop_attn_workspace_bytes(B, n_max, d, H, dtype))
    return VARDROP_EWORKSPACE;
  if (!vd_aligned(saved, 256)) return VARDROP_EWORKSPACE;
  if (!vd_aligned(xs, 16) || !vd_aligned(dy, 16) || !vd_aligned(dxs, 16) || !vd_aligned(Wq, 16) ||
      !vd_aligned(Wk, 16) || !vd_aligned(Wv, 16) || !vd_aligned(Wo, 16))
    return VARDROP_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  float* dW[4] = {dWq, dWk, dWv, dWo};
  float* db[4] = {dbq, dbk, dbv, dbo};
  const void* W[4] = {Wq, Wk, Wv, Wo};
  const VdDevCount dn = {n_dev, status};
  if (dtype == VARDROP_F32)
    return vd_attn_bwd_f32(ctx, (const float*)dy, (const float*)xs, B, n_max, d, H, (const float* const*)W, saved,
                           (float*)dxs, dW, db, ws, s, dn);
  return vd_attn_bwd_bf16(ctx, dy, xs, B, n_max, d, H, W, saved, dxs, dW, db, ws, s, dn);
}

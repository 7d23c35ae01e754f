// Token embedding of the kept variates only (Sec. 3.1 / 3.3: the reduction works directly from the raw
// variates, so the tokens of the dropped ones are never formed): xs = z We + be, where z are the kept
// windows, optionally standardised over time, and its weight gradients dWe = z^T dxs, dbe = colsum(dxs).
//
// Two steps.  (1) One wavefront per kept window reads it from the raw batch through `sel` (coalesced:
// consecutive lanes read consecutive samples), takes mean and variance with wavefront reductions in a
// fixed order, and writes the standardised window in the operand type: bf16 rows padded with zeros to a
// multiple of 64 samples, or fp32 rows.  The caller keeps that buffer for the backward pass.  (2) The
// products run on the GEMM kernels of the attention back end: bf16 on the matrix cores (the padding
// lets the 64-deep K slices run past L), fp32 on the plain multiply-add kernel.
#include "bf16_mfma.h"
#include "gemm_bf16.h"

namespace {

constexpr int kMaxEmbedL = 1024;               // 16 samples per lane

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// BF16: out rows are bf16 with pitch `pitch` (zeros from L on); else fp32 rows of pitch L
template <bool BF16>
__global__ __launch_bounds__(256) void embed_rows_kernel(const float* __restrict__ x, void* __restrict__ out,
                                                        const int32_t* __restrict__ sel, int N, int L, int n_sel,
                                                        long long rows, long long sb, long long sn, int pitch,
                                                        int standardise) {
  const int lane = threadIdx.x & 63;
  const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const long long b = row / n_sel;
  const int i = (int)(row - b * n_sel);
  const int n = sel[i];
  const bool ok = (unsigned)n < (unsigned)N;
  const float* p = x + b * sb + (long long)(ok ? n : 0) * sn;
  float v[kMaxEmbedL / 64];
  float sum = 0.f;
#pragma unroll
  for (int u = 0; u < kMaxEmbedL / 64; ++u) {
    const int t = lane + 64 * u;
    v[u] = (ok && t < L) ? p[t] : 0.f;
    sum += v[u];
  }
  if (standardise) {
    const float mean = wave_sum(sum) / (float)L;
    float ss = 0.f;
#pragma unroll
    for (int u = 0; u < kMaxEmbedL / 64; ++u) {
      const int t = lane + 64 * u;
      v[u] = t < L ? v[u] - mean : 0.f;
      ss = fmaf(v[u], v[u], ss);
    }
    const float var = wave_sum(ss) / (float)L;
    const float inv = var > 0.f ? 1.0f / sqrtf(var) : 1.0f;        // (a constant window is all zeros already)
#pragma unroll
    for (int u = 0; u < kMaxEmbedL / 64; ++u) v[u] *= inv;
  }
#pragma unroll
  for (int u = 0; u < kMaxEmbedL / 64; ++u) {
    const int t = lane + 64 * u;
    if (t < pitch) {
      if (BF16) reinterpret_cast<bf16_t*>(out)[row * pitch + t] = f2bf(v[u]);
      else reinterpret_cast<float*>(out)[row * pitch + t] = v[u];
    }
  }
}

// Column sums in two steps with a fixed order: part[j][c] = sum of rows [j * per, (j + 1) * per) of column c
// (a thread per column, rows ascending), then dst[c] = sum_j part[j][c] (j ascending).
constexpr int kColSlices = 64;
template <typename T>
__global__ __launch_bounds__(256) void embed_colsum_part_kernel(const T* __restrict__ src, float* __restrict__ part,
                                                               long long rows, long long per, int d) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= d) return;
  const long long r0 = blockIdx.y * per, r1 = min(rows, r0 + per);
  float s = 0.f;
  for (long long r = r0; r < r1; ++r) {
    if constexpr (sizeof(T) == 2) s += bf2f(src[r * d + c]);
    else s += src[r * d + c];
  }
  part[(long long)blockIdx.y * d + c] = s;
}
__global__ __launch_bounds__(256) void embed_colsum_final_kernel(const float* __restrict__ part, float* __restrict__ dst, int d) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= d) return;
  float s = 0.f;
  for (int j = 0; j < kColSlices; ++j) s += part[(long long)j * d + c];
  dst[c] = s;
}
template <typename T>
int embed_colsum(vardrop_ctx* ctx, const T* src, float* part, float* dst, long long rows, int d, hipStream_t s) {
  const long long per = (rows + kColSlices - 1) / kColSlices;
  hipLaunchKernelGGL(embed_colsum_part_kernel<T>, dim3(vd_ceil_div(d, 256), kColSlices), dim3(256), 0, s, src, part, rows, per, d);
  hipLaunchKernelGGL(embed_colsum_final_kernel, dim3(vd_ceil_div(d, 256)), dim3(256), 0, s, part, dst, d);
  VD_LAUNCH_CHECK(ctx);
  return VARDROP_OK;
}

__global__ void embed_zero_kernel(float* p, long long count) {
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (long long)gridDim.x * blockDim.x)
    p[i] = 0.f;
}

int embed_pitch(int L, int dtype) { return dtype == VARDROP_BF16 ? (int)vd_align_up((size_t)L, 64) : L; }

int check(int B, int n_sel, int L, int d, int dtype) {
  if (B < 0 || n_sel < 0 || L < 2 || d < 1) return VARDROP_EINVAL;
  if (dtype != VARDROP_F32 && dtype != VARDROP_BF16) return VARDROP_EINVAL;
  if (L > kMaxEmbedL) return VARDROP_EUNSUPPORTED;
  const long long M = (long long)B * n_sel;
  if (M * d >= (1ll << 31) || M * (L + 63) >= (1ll << 31)) return VARDROP_EUNSUPPORTED;
  if (dtype == VARDROP_BF16 && (d % 8 != 0 || L % 8 != 0)) return VARDROP_EUNSUPPORTED;
  return VARDROP_OK;
}

// K slices of dWe = z^T dxs (K = B * n_sel rows; tiles of 64 x 128): enough of them to give the chip two
// workgroups per compute unit, at least 128 rows each, at most 16
int embed_splitk(int L, int d, long long M, int* kchunk) {
  const int tiles = vd_ceil_div(L, 64) * vd_ceil_div(d, 128);
  int s = vd_ceil_div(512, tiles);
  if (s > 16) s = 16;
  while (s > 1 && M / s < 128) --s;
  int chunk = (int)vd_align_up((size_t)vd_ceil_div((int)M, s), 64);
  if (chunk < 64) chunk = 64;
  *kchunk = chunk;
  return M > 0 ? vd_ceil_div((int)M, chunk) : 1;
}

size_t embed_colsum_bytes(int d) { return vd_align_up((size_t)kColSlices * d * sizeof(float), 256); }

}  // namespace

extern "C" size_t vardrop_embed_saved_bytes(int B, int n_sel, int L, int dtype) {
  if (check(B, n_sel, L, 8, dtype) != VARDROP_OK) return 0;
  const size_t es = dtype == VARDROP_BF16 ? 2 : 4;
  return vd_align_up((size_t)B * n_sel * embed_pitch(L, dtype) * es, 256);
}

extern "C" size_t vardrop_embed_workspace_bytes(int B, int n_sel, int L, int d, int dtype) {
  if (check(B, n_sel, L, d, dtype) != VARDROP_OK) return 0;
  // partial column sums of dxs (bias gradient), then, for bf16, room for the largest slice count of dWe
  return embed_colsum_bytes(d) + (dtype == VARDROP_BF16 ? vd_align_up((size_t)16 * L * d * sizeof(float), 256) : 0);
}

extern "C" int vardrop_embed_fwd(vardrop_ctx* ctx, const float* x, int B, int N, int L, int64_t sb, int64_t sn,
                                 const int32_t* sel, int n_sel, int standardise,
                                 const void* We, const void* be, int d, int dtype,
                                 void* xs, void* saved, void* stream) {
  if (!ctx) return VARDROP_EINVAL;
  int rc = check(B, n_sel, L, d, dtype);
  if (rc) return rc;
  if (N < 0 || n_sel > N || sb < 0 || sn < 0) return VARDROP_EINVAL;
  const long long M = (long long)B * n_sel;
  if (M == 0) return VARDROP_OK;
  if (!x || !sel || !We || !xs || !saved) return VARDROP_EINVAL;
  if (!vd_aligned(saved, 256)) return VARDROP_EWORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const int pitch = embed_pitch(L, dtype);
  {
    VdTimer timer(ctx, VARDROP_K_EMBED_ROWS, s);
    const dim3 grid((unsigned)((M + 3) / 4));
    if (dtype == VARDROP_BF16)
      VD_KERNEL(ctx, embed_rows_kernel<true>, grid, dim3(256), 0, s, x, saved, sel, N, L, n_sel, M,
                         (long long)sb, (long long)sn, pitch, standardise);
    else
      VD_KERNEL(ctx, embed_rows_kernel<false>, grid, dim3(256), 0, s, x, saved, sel, N, L, n_sel, M,
                         (long long)sb, (long long)sn, pitch, standardise);
  }
  VD_LAUNCH_CHECK(ctx);
  if (dtype == VARDROP_BF16) {
    GemmBf16 g = {};
    g.set(0, saved, We, xs, be);
    g.lda = pitch; g.ldb = d; g.ldc = d;
    g.M = (int)M; g.N = d; g.K = L; g.nseg = 1;
    g.a_kpad = 1;
    return vd_gemm_bf16(ctx, VARDROP_K_GEMM_EMBED, g, 1, false, s);
  }
  return vd_gemm_f32(ctx, VARDROP_K_GEMM_EMBED, (const float*)saved, L, 1, (const float*)We, d, 1,
                     (float*)xs, d, (const float*)be, (int)M, d, L, s);
}

extern "C" int vardrop_embed_bwd(vardrop_ctx* ctx, const void* dxs, int B, int n_sel, int L, int d, int dtype,
                                 const void* saved, float* dWe, float* dbe,
                                 void* ws, size_t ws_bytes, void* stream) {
  if (!ctx) return VARDROP_EINVAL;
  int rc = check(B, n_sel, L, d, dtype);
  if (rc) return rc;
  if (!dWe) return VARDROP_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  const long long M = (long long)B * n_sel;
  if (M == 0) {
    hipLaunchKernelGGL(embed_zero_kernel, dim3(64), dim3(256), 0, s, dWe, (long long)L * d);
    if (dbe) hipLaunchKernelGGL(embed_zero_kernel, dim3(1), dim3(256), 0, s, dbe, (long long)d);
    VD_LAUNCH_CHECK(ctx);
    return VARDROP_OK;
  }
  if (!dxs || !saved) return VARDROP_EINVAL;
  if (!vd_aligned(saved, 256)) return VARDROP_EWORKSPACE;
  if (!ws || !vd_aligned(ws, 256) || ws_bytes < vardrop_embed_workspace_bytes(B, n_sel, L, d, dtype)) return VARDROP_EWORKSPACE;
  float* colpart = (float*)ws;
  float* slices = (float*)((char*)ws + embed_colsum_bytes(d));
  const int pitch = embed_pitch(L, dtype);
  if (dtype == VARDROP_BF16) {
    GemmBf16 g = {};
    g.set(0, saved, dxs, dWe, nullptr);
    g.lda = pitch; g.ldb = d; g.ldc = d;
    g.M = L; g.N = d; g.K = (int)M; g.nseg = 1;
    int kchunk = 0;
    g.splitk = embed_splitk(L, d, M, &kchunk);
    g.kchunk = kchunk;
    if (g.splitk > 1) {
      g.part = slices;
      if ((rc = vd_gemm_bf16_wgrad_split(ctx, VARDROP_K_GEMM_DWE, g, s))) return rc;
      float* out[4] = {dWe, nullptr, nullptr, nullptr};
      if ((rc = vd_gemm_bf16_sum_slices(ctx, slices, out, (long long)L * d, g.splitk, s, 1))) return rc;
    } else if ((rc = vd_gemm_bf16_wgrad_split(ctx, VARDROP_K_GEMM_DWE, g, s))) {
      return rc;
    }
    if (dbe) return embed_colsum(ctx, (const bf16_t*)dxs, colpart, dbe, M, d, s);
    return VARDROP_OK;
  }
  // fp32: dWe(t, c) = sum_r z[r][t] dxs[r][c]
  if ((rc = vd_gemm_f32(ctx, VARDROP_K_GEMM_DWE, (const float*)saved, 1, L, (const float*)dxs, d, 1, dWe, d, nullptr,
                        L, d, (int)M, s)))
    return rc;
  if (dbe) return embed_colsum(ctx, (const float*)dxs, colpart, dbe, M, d, s);
  return VARDROP_OK;
}

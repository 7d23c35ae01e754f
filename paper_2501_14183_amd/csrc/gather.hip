// Gather of the kept variate tokens and its adjoint (Sec. 3.1: only the selected tokens
// enter the attention).  Pure data movement: every row is d * sizeof(elem) contiguous
// bytes, moved with 16-byte accesses when the row size and the pointers allow it.
#include "common.h"

namespace {

// Element types: the kernels move opaque units of 16, 4 or 2 bytes.
template <typename T> __device__ inline T zero_unit() { return T(0); }
template <> __device__ inline uint4 zero_unit<uint4>() { return make_uint4(0, 0, 0, 0); }

// out[b][i][:] = src[b][sel[i]][:].  A workgroup of 256 threads moves blockDim.y rows at a time,
// `row_units` units each; threadIdx.y walks the rows, threadIdx.x the units of a row.
template <typename T>
__global__ __launch_bounds__(256) void gather_kernel(const T* __restrict__ src, T* __restrict__ out,
                                                    const int32_t* __restrict__ sel,
                                                    int B, int N, int n_sel, int row_units,
                                                    const int32_t* n_dev, int32_t* status) {
  if (!vd_count(n_dev, n_sel, n_sel, status)) return;     // device-side count: n_sel was its bound
  const int rows = B * n_sel;
  for (int row = blockIdx.x * blockDim.y + threadIdx.y; row < rows; row += gridDim.x * blockDim.y) {
    const int b = row / n_sel, j = row - b * n_sel;
    const int n = sel[j];
    const bool ok = (unsigned)n < (unsigned)N;
    const T* p = src + ((long long)b * N + (ok ? n : 0)) * row_units;
    T* q = out + (long long)row * row_units;
    for (int c = threadIdx.x; c < row_units; c += blockDim.x) {
      T v = p[c];
      if (!ok) v = zero_unit<T>();
      q[c] = v;
    }
  }
}

// dst[b][n][:] = src[b][i][:] if sel[i] == n for some i (sel ascending), else 0.
template <typename T>
__global__ __launch_bounds__(256) void scatter_kernel(const T* __restrict__ src, T* __restrict__ dst,
                                                     const int32_t* __restrict__ sel,
                                                     int B, int N, int n_sel, int row_units,
                                                     const int32_t* n_dev, int32_t* status) {
  if (!vd_count(n_dev, n_sel, n_sel, status)) return;
  const int rows = B * N;
  for (int row = blockIdx.x * blockDim.y + threadIdx.y; row < rows; row += gridDim.x * blockDim.y) {
    const int b = row / N, n = row - b * N;
    int lo = 0, hi = n_sel;                       // first position with sel[pos] >= n
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (sel[mid] < n) lo = mid + 1; else hi = mid;
    }
    const bool hit = lo < n_sel && sel[lo] == n;
    T* q = dst + (long long)row * row_units;
    if (hit) {
      const T* p = src + ((long long)b * n_sel + lo) * row_units;
      for (int c = threadIdx.x; c < row_units; c += blockDim.x) q[c] = p[c];
    } else {
      for (int c = threadIdx.x; c < row_units; c += blockDim.x) q[c] = zero_unit<T>();
    }
  }
}

typedef uint4 Chunk16;

int elem_size(int dtype) { return dtype == VARDROP_F32 ? 4 : (dtype == VARDROP_BF16 ? 2 : 0); }

template <bool kScatter>
int launch(vardrop_ctx* ctx, const void* src, void* dst, const int32_t* sel, int B, int N, int n_sel,
           int d, int dtype, hipStream_t s, VdDevCount dn = {nullptr, nullptr}) {
  const int es = elem_size(dtype);
  const long long row_bytes = (long long)d * es;
  const long long rows = (long long)B * (kScatter ? N : n_sel);
  if (rows == 0) return VARDROP_OK;
  const bool wide = row_bytes % 16 == 0 && vd_aligned(src, 16) && vd_aligned(dst, 16);
  const int unit = wide ? 16 : es;
  const int row_units = (int)(row_bytes / unit);
  if (rows >= (1ll << 31)) return VARDROP_EUNSUPPORTED;
  int tx = 1;                                     // threads along a row: power of two, at most 64
  while (tx < 64 && tx < row_units) tx <<= 1;
  const int ty = 256 / tx;
  long long blocks = (rows + ty - 1) / ty;
  if (blocks > 256 * 64) blocks = 256 * 64;
  dim3 grid((unsigned)blocks), block(tx, ty);
  VdTimer timer(ctx, kScatter ? VARDROP_K_SCATTER : VARDROP_K_GATHER, s);
  if (wide) {
    if (kScatter) VD_KERNEL(ctx, scatter_kernel<Chunk16>, grid, block, 0, s, (const Chunk16*)src, (Chunk16*)dst, sel, B, N, n_sel, row_units, dn.dev, dn.status);
    else VD_KERNEL(ctx, gather_kernel<Chunk16>, grid, block, 0, s, (const Chunk16*)src, (Chunk16*)dst, sel, B, N, n_sel, row_units, dn.dev, dn.status);
  } else if (es == 4) {
    if (kScatter) VD_KERNEL(ctx, scatter_kernel<uint32_t>, grid, block, 0, s, (const uint32_t*)src, (uint32_t*)dst, sel, B, N, n_sel, row_units, dn.dev, dn.status);
    else VD_KERNEL(ctx, gather_kernel<uint32_t>, grid, block, 0, s, (const uint32_t*)src, (uint32_t*)dst, sel, B, N, n_sel, row_units, dn.dev, dn.status);
  } else {
    if (kScatter) VD_KERNEL(ctx, scatter_kernel<uint16_t>, grid, block, 0, s, (const uint16_t*)src, (uint16_t*)dst, sel, B, N, n_sel, row_units, dn.dev, dn.status);
    else VD_KERNEL(ctx, gather_kernel<uint16_t>, grid, block, 0, s, (const uint16_t*)src, (uint16_t*)dst, sel, B, N, n_sel, row_units, dn.dev, dn.status);
  }
  VD_LAUNCH_CHECK(ctx);
  return VARDROP_OK;
}

int check(vardrop_ctx* ctx, int B, int N, int d, int dtype, int n_sel) {
  if (!ctx) return VARDROP_EINVAL;
  if (B < 0 || N < 0 || d < 1 || n_sel < 0 || n_sel > N) return VARDROP_EINVAL;
  if (elem_size(dtype) == 0) return VARDROP_EINVAL;
  return VARDROP_OK;
}

}  // namespace

extern "C" int vardrop_gather(vardrop_ctx* ctx, const void* tokens, int B, int N, int d, int dtype,
                              const int32_t* sel, int n_sel, void* out, void* stream) {
  int rc = check(ctx, B, N, d, dtype, n_sel);
  if (rc != VARDROP_OK) return rc;
  if ((long long)B * n_sel == 0) return VARDROP_OK;
  if (!tokens || !out || !sel) return VARDROP_EINVAL;
  return launch<false>(ctx, tokens, out, sel, B, N, n_sel, d, dtype, (hipStream_t)stream);
}

int vd_gather(vardrop_ctx* ctx, const void* tokens, int B, int N, int d, int dtype, const int32_t* sel, int n_sel,
              void* out, hipStream_t s, VdDevCount dn) {
  return launch<false>(ctx, tokens, out, sel, B, N, n_sel, d, dtype, s, dn);
}

extern "C" int vardrop_gather_dev(vardrop_ctx* ctx, const void* tokens, int B, int N, int d, int dtype,
                                  const int32_t* sel, const int32_t* n_sel_dev, int n_sel_max, int32_t* status,
                                  void* out, void* stream) {
  int rc = check(ctx, B, N, d, dtype, n_sel_max);
  if (rc != VARDROP_OK) return rc;
  if (!n_sel_dev) return VARDROP_EINVAL;
  if ((long long)B * n_sel_max == 0) return VARDROP_OK;
  if (!tokens || !out || !sel) return VARDROP_EINVAL;
  return launch<false>(ctx, tokens, out, sel, B, N, n_sel_max, d, dtype, (hipStream_t)stream, VdDevCount{n_sel_dev, status});
}

extern "C" int vardrop_scatter_dev(vardrop_ctx* ctx, const void* dxs, int B, int N, int d, int dtype,
                                   const int32_t* sel, const int32_t* n_sel_dev, int n_sel_max, int32_t* status,
                                   void* dtokens, void* stream) {
  int rc = check(ctx, B, N, d, dtype, n_sel_max);
  if (rc != VARDROP_OK) return rc;
  if (!n_sel_dev) return VARDROP_EINVAL;
  if ((long long)B * N == 0) return VARDROP_OK;
  if (!dtokens || !dxs || !sel) return VARDROP_EINVAL;
  return launch<true>(ctx, dxs, dtokens, sel, B, N, n_sel_max, d, dtype, (hipStream_t)stream, VdDevCount{n_sel_dev, status});
}

extern "C" int vardrop_scatter(vardrop_ctx* ctx, const void* dxs, int B, int N, int d, int dtype,
                               const int32_t* sel, int n_sel, void* dtokens, void* stream) {
  int rc = check(ctx, B, N, d, dtype, n_sel);
  if (rc != VARDROP_OK) return rc;
  if ((long long)B * N == 0) return VARDROP_OK;
  if (!dtokens || (n_sel > 0 && (!dxs || !sel))) return VARDROP_EINVAL;
  return launch<true>(ctx, dxs, dtokens, sel, B, N, n_sel, d, dtype, (hipStream_t)stream);
}

// fp32 back end of the multi-head attention (Eq. 3), forward and backward.
//
// Plain fp32 multiply-add kernels: an LDS-tiled strided GEMM for the four projections and
// their gradients, and row-per-thread attention kernels with an online softmax (forward)
// and recomputed probabilities (backward).  This back end serves fp32 callers and small
// problems; the bf16 matrix-core back end carries the large ones.
#include "common.h"

namespace {

// ------------------------------------------------------------------ strided GEMM
// C[z][m][n] = sum_seg sum_k A[seg or z](m, k) * B[seg or z](k, n) (+ bias[z][n])
struct GemmF32 {
  const float* A[3];
  const float* B[3];
  float* C[3];
  const float* bias[3];
  long long sam, sak, sbk, sbn;   // element strides of A(m,k) and B(k,n)
  int M, N, K, ldc;
  int nseg;                       // > 1: segments accumulate into C[0] (grid z must be 1)
  // device-side token count (see vd_count): M (n_role 0) or K (n_role 1) becomes n_mul * n, at most its host value
  const int32_t* n_dev;
  int32_t* status;
  int n_max, n_mul, n_role;
  void count(const VdDevCount& dn, bool give_status, int nmax, int mul, int role) {
    n_dev = dn.dev; status = give_status ? dn.status : nullptr; n_max = nmax; n_mul = mul; n_role = role;
  }
};

__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmF32 g) {
  __shared__ float As[16][64 + 1];
  __shared__ float Bs[16][64 + 1];
  if (g.n_dev) {
    int n;
    if (!vd_count(g.n_dev, g.n_max, n, g.status)) return;
    if (g.n_role == 0) g.M = g.n_mul * n; else g.K = g.n_mul * n;
  }
  const int z = blockIdx.z;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  if (m0 >= g.M) return;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4] = {};
  const int nseg = g.nseg > 1 ? g.nseg : 1;
  for (int seg = 0; seg < nseg; ++seg) {
    const float* A = g.A[g.nseg > 1 ? seg : z];
    const float* Bm = g.B[g.nseg > 1 ? seg : z];
    for (int k0 = 0; k0 < g.K; k0 += 16) {
      for (int i = threadIdx.x; i < 16 * 64; i += 256) {
        const int kk = i & 15, mm = i >> 4;       // consecutive threads walk k (fast when sak == 1)
        const int kk2 = i >> 6, nn = i & 63;      // consecutive threads walk n (fast when sbn == 1)
        float av = 0.f, bv = 0.f;
        if (g.sak == 1) {
          if (m0 + mm < g.M && k0 + kk < g.K) av = A[(long long)(m0 + mm) * g.sam + (k0 + kk)];
          As[kk][mm] = av;
        } else {
          if (m0 + nn < g.M && k0 + kk2 < g.K) av = A[(long long)(m0 + nn) * g.sam + (long long)(k0 + kk2) * g.sak];
          As[kk2][nn] = av;
        }
        if (g.sbn == 1) {
          if (n0 + nn < g.N && k0 + kk2 < g.K) bv = Bm[(long long)(k0 + kk2) * g.sbk + (n0 + nn)];
          Bs[kk2][nn] = bv;
        } else {
          if (n0 + mm < g.N && k0 + kk < g.K) bv = Bm[(long long)(k0 + kk) * g.sbk + (long long)(n0 + mm) * g.sbn];
          Bs[kk][mm] = bv;
        }
      }
      __syncthreads();
#pragma unroll
      for (int kk = 0; kk < 16; ++kk) {
        float a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
        for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
      }
      __syncthreads();
    }
  }
  float* C = g.C[g.nseg > 1 ? 0 : z];
  const float* bias = g.bias[g.nseg > 1 ? 0 : z];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < g.M && n < g.N) C[(long long)m * g.ldc + n] = acc[i][j] + (bias ? bias[n] : 0.f);
    }
}

int launch_gemm(vardrop_ctx* ctx, int kid, const GemmF32& g, int nz, hipStream_t s) {
  if (g.M == 0 || g.N == 0) return VARDROP_OK;
  dim3 grid(vd_ceil_div(g.N, 64), vd_ceil_div(g.M, 64), nz);
  VdTimer timer(ctx, kid, s);
  VD_KERNEL(ctx, gemm_f32_kernel, grid, dim3(256), 0, s, g);
  VD_LAUNCH_CHECK(ctx);
  return VARDROP_OK;
}

}  // namespace

// C[m][n] = sum_k A(m, k) B(k, n) (+ bias[n]) with element strides (sam, sak) and (sbk, sbn)
int vd_gemm_f32(vardrop_ctx* ctx, int kid, const float* A, long long sam, long long sak,
                const float* B, long long sbk, long long sbn, float* C, int ldc, const float* bias,
                int M, int N, int K, hipStream_t s) {
  GemmF32 g = {};
  g.A[0] = A; g.B[0] = B; g.C[0] = C; g.bias[0] = bias;
  g.sam = sam; g.sak = sak; g.sbk = sbk; g.sbn = sbn;
  g.M = M; g.N = N; g.K = K; g.ldc = ldc; g.nseg = 1;
  return launch_gemm(ctx, kid, g, 1, s);
}

namespace {

// ------------------------------------------------------------------ attention core
// q, k, v, o: [B][n][d], head h at columns h*DH .. h*DH+DH-1.  One query (or key) per thread.
constexpr int kTile = 32;

template <int DH>
__global__ __launch_bounds__(64) void sdpa_fwd_f32(const float* __restrict__ q, const float* __restrict__ k,
                                                  const float* __restrict__ v, float* __restrict__ o,
                                                  float* __restrict__ lse, int n, int d, int H, float scale,
                                                  const int32_t* n_dev) {
  __shared__ float Ks[kTile][DH];
  __shared__ float Vs[kTile][DH];
  if (!vd_count(n_dev, n, n) || (int)blockIdx.x * 64 >= n) return;
  const int b = blockIdx.z, h = blockIdx.y;
  const int i = blockIdx.x * 64 + threadIdx.x;
  const long long base = (long long)b * n * d + h * DH;
  float qr[DH], acc[DH];
#pragma unroll
  for (int c = 0; c < DH; ++c) {
    qr[c] = i < n ? q[base + (long long)i * d + c] : 0.f;
    acc[c] = 0.f;
  }
  float m = -INFINITY, l = 0.f;
  for (int j0 = 0; j0 < n; j0 += kTile) {
    __syncthreads();
    for (int t = threadIdx.x; t < kTile * DH; t += 64) {
      const int jj = t / DH, c = t % DH;
      const bool ok = j0 + jj < n;
      Ks[jj][c] = ok ? k[base + (long long)(j0 + jj) * d + c] : 0.f;
      Vs[jj][c] = ok ? v[base + (long long)(j0 + jj) * d + c] : 0.f;
    }
    __syncthreads();
    const int jn = min(kTile, n - j0);
    for (int jj = 0; jj < jn; ++jj) {
      float s = 0.f;
#pragma unroll
      for (int c = 0; c < DH; ++c) s = fmaf(qr[c], Ks[jj][c], s);
      s *= scale;
      const float mn = fmaxf(m, s);
      const float alpha = expf(m - mn);
      const float p = expf(s - mn);
      l = l * alpha + p;
#pragma unroll
      for (int c = 0; c < DH; ++c) acc[c] = fmaf(p, Vs[jj][c], acc[c] * alpha);
      m = mn;
    }
  }
  if (i < n) {
    const float inv = 1.f / l;
#pragma unroll
    for (int c = 0; c < DH; ++c) o[base + (long long)i * d + c] = acc[c] * inv;
    lse[((long long)b * H + h) * n + i] = m + logf(l);
  }
}

// dQ and D = rowsum(dO * O); one query per thread, loop over keys.
template <int DH>
__global__ __launch_bounds__(64) void sdpa_bwd_dq_f32(const float* __restrict__ q, const float* __restrict__ k,
                                                     const float* __restrict__ v, const float* __restrict__ o,
                                                     const float* __restrict__ dout, const float* __restrict__ lse,
                                                     float* __restrict__ dq, float* __restrict__ Dsum,
                                                     int n, int d, int H, float scale, const int32_t* n_dev) {
  __shared__ float Ks[kTile][DH];
  __shared__ float Vs[kTile][DH];
  if (!vd_count(n_dev, n, n) || (int)blockIdx.x * 64 >= n) return;
  const int b = blockIdx.z, h = blockIdx.y;
  const int i = blockIdx.x * 64 + threadIdx.x;
  const long long base = (long long)b * n * d + h * DH;
  float qr[DH], dor[DH], acc[DH];
  float D = 0.f;
#pragma unroll
  for (int c = 0; c < DH; ++c) {
    qr[c] = i < n ? q[base + (long long)i * d + c] : 0.f;
    dor[c] = i < n ? dout[base + (long long)i * d + c] : 0.f;
    const float oc = i < n ? o[base + (long long)i * d + c] : 0.f;
    D = fmaf(dor[c], oc, D);
    acc[c] = 0.f;
  }
  const float li = i < n ? lse[((long long)b * H + h) * n + i] : 0.f;
  for (int j0 = 0; j0 < n; j0 += kTile) {
    __syncthreads();
    for (int t = threadIdx.x; t < kTile * DH; t += 64) {
      const int jj = t / DH, c = t % DH;
      const bool ok = j0 + jj < n;
      Ks[jj][c] = ok ? k[base + (long long)(j0 + jj) * d + c] : 0.f;
      Vs[jj][c] = ok ? v[base + (long long)(j0 + jj) * d + c] : 0.f;
    }
    __syncthreads();
    const int jn = min(kTile, n - j0);
    for (int jj = 0; jj < jn; ++jj) {
      float s = 0.f, dp = 0.f;
#pragma unroll
      for (int c = 0; c < DH; ++c) {
        s = fmaf(qr[c], Ks[jj][c], s);
        dp = fmaf(dor[c], Vs[jj][c], dp);
      }
      const float p = expf(s * scale - li);
      const float ds = p * (dp - D) * scale;
#pragma unroll
      for (int c = 0; c < DH; ++c) acc[c] = fmaf(ds, Ks[jj][c], acc[c]);
    }
  }
  if (i < n) {
#pragma unroll
    for (int c = 0; c < DH; ++c) dq[base + (long long)i * d + c] = acc[c];
    Dsum[((long long)b * H + h) * n + i] = D;
  }
}

// dK and dV; one key per thread, loop over queries.
template <int DH>
__global__ __launch_bounds__(64) void sdpa_bwd_dkv_f32(const float* __restrict__ q, const float* __restrict__ k,
                                                      const float* __restrict__ v, const float* __restrict__ dout,
                                                      const float* __restrict__ lse, const float* __restrict__ Dsum,
                                                      float* __restrict__ dk, float* __restrict__ dv,
                                                      int n, int d, int H, float scale, const int32_t* n_dev) {
  __shared__ float Qs[kTile][DH];
  __shared__ float Os[kTile][DH];
  __shared__ float Ls[kTile], Ds[kTile];
  if (!vd_count(n_dev, n, n) || (int)blockIdx.x * 64 >= n) return;
  const int b = blockIdx.z, h = blockIdx.y;
  const int j = blockIdx.x * 64 + threadIdx.x;
  const long long base = (long long)b * n * d + h * DH;
  float kr[DH], vr[DH], ak[DH], av[DH];
#pragma unroll
  for (int c = 0; c < DH; ++c) {
    kr[c] = j < n ? k[base + (long long)j * d + c] : 0.f;
    vr[c] = j < n ? v[base + (long long)j * d + c] : 0.f;
    ak[c] = 0.f;
    av[c] = 0.f;
  }
  for (int i0 = 0; i0 < n; i0 += kTile) {
    __syncthreads();
    for (int t = threadIdx.x; t < kTile * DH; t += 64) {
      const int ii = t / DH, c = t % DH;
      const bool ok = i0 + ii < n;
      Qs[ii][c] = ok ? q[base + (long long)(i0 + ii) * d + c] : 0.f;
      Os[ii][c] = ok ? dout[base + (long long)(i0 + ii) * d + c] : 0.f;
    }
    if (threadIdx.x < kTile) {
      const bool ok = i0 + threadIdx.x < n;
      Ls[threadIdx.x] = ok ? lse[((long long)b * H + h) * n + i0 + threadIdx.x] : 0.f;
      Ds[threadIdx.x] = ok ? Dsum[((long long)b * H + h) * n + i0 + threadIdx.x] : 0.f;
    }
    __syncthreads();
    const int in = min(kTile, n - i0);
    for (int ii = 0; ii < in; ++ii) {
      float s = 0.f, dp = 0.f;
#pragma unroll
      for (int c = 0; c < DH; ++c) {
        s = fmaf(Qs[ii][c], kr[c], s);
        dp = fmaf(Os[ii][c], vr[c], dp);
      }
      const float p = expf(s * scale - Ls[ii]);
      const float ds = p * (dp - Ds[ii]) * scale;
#pragma unroll
      for (int c = 0; c < DH; ++c) {
        av[c] = fmaf(p, Os[ii][c], av[c]);
        ak[c] = fmaf(ds, Qs[ii][c], ak[c]);
      }
    }
  }
  if (j < n) {
#pragma unroll
    for (int c = 0; c < DH; ++c) {
      dk[base + (long long)j * d + c] = ak[c];
      dv[base + (long long)j * d + c] = av[c];
    }
  }
}

// column sums of up to four [rows][d] matrices (bias gradients)
struct ColSumF32 {
  const float* src[4];
  float* dst[4];
  long long rows;
  int d;
  const int32_t* n_dev;           // device-side token count: rows = n_mul * n
  int n_max, n_mul;
};
__global__ __launch_bounds__(256) void colsum_f32_kernel(ColSumF32 a) {
  const float* src = a.src[blockIdx.y];
  float* dst = a.dst[blockIdx.y];
  if (!dst) return;
  if (a.n_dev) {
    int n;
    if (!vd_count(a.n_dev, a.n_max, n)) return;
    a.rows = (long long)a.n_mul * n;
  }
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= a.d) return;
  float s = 0.f;
  for (long long r = 0; r < a.rows; ++r) s += src[r * a.d + c];
  dst[c] = s;
}

template <int DH>
int run_fwd_core(vardrop_ctx* ctx, const float* q, const float* k, const float* v, float* o, float* lse,
                 int B, int n, int d, int H, hipStream_t s, const int32_t* n_dev) {
  VdTimer timer(ctx, VARDROP_K_SDPA_FWD, s);
  VD_KERNEL(ctx, sdpa_fwd_f32<DH>, dim3(vd_ceil_div(n, 64), H, B), dim3(64), 0, s, q, k, v, o, lse, n, d, H,
                     1.0f / sqrtf((float)DH), n_dev);
  VD_LAUNCH_CHECK(ctx);
  return VARDROP_OK;
}

template <int DH>
int run_bwd_core(vardrop_ctx* ctx, const float* q, const float* k, const float* v, const float* o, const float* dO,
                 const float* lse, float* dq, float* dk, float* dv, float* D, int B, int n, int d, int H,
                 hipStream_t s, const int32_t* n_dev) {
  const float scale = 1.0f / sqrtf((float)DH);
  dim3 grid(vd_ceil_div(n, 64), H, B);
  {
    VdTimer timer(ctx, VARDROP_K_SDPA_BWD_DQ, s);
    VD_KERNEL(ctx, sdpa_bwd_dq_f32<DH>, grid, dim3(64), 0, s, q, k, v, o, dO, lse, dq, D, n, d, H, scale, n_dev);
  }
  VD_LAUNCH_CHECK(ctx);
  VdTimer timer(ctx, VARDROP_K_SDPA_BWD_DKV, s);
  VD_KERNEL(ctx, sdpa_bwd_dkv_f32<DH>, grid, dim3(64), 0, s, q, k, v, dO, lse, D, dk, dv, n, d, H, scale, n_dev);
  VD_LAUNCH_CHECK(ctx);
  return VARDROP_OK;
}

}  // namespace

// saved: q, k, v, o ([M][d] fp32 each, M = B*n) then lse [B][H][n]
int vd_attn_fwd_f32(vardrop_ctx* ctx, const float* xs, int B, int n, int d, int H,
                    const float* const W[4], const float* const bias[4],
                    float* y, void* saved, void* ws, hipStream_t s, VdDevCount dn) {
  (void)ws;
  const long long M = (long long)B * n;
  float* q = (float*)saved;
  float* k = q + M * d;
  float* v = k + M * d;
  float* o = v + M * d;
  float* lse = o + M * d;
  GemmF32 g = {};
  for (int z = 0; z < 3; ++z) {
    g.A[z] = xs;
    g.B[z] = W[z];
    g.bias[z] = bias[z];
  }
  g.C[0] = q;
  g.C[1] = k;
  g.C[2] = v;
  g.sam = d; g.sak = 1; g.sbk = d; g.sbn = 1;
  g.M = (int)M; g.N = d; g.K = d; g.ldc = d; g.nseg = 1;
  g.count(dn, true, n, B, 0);
  int rc = launch_gemm(ctx, VARDROP_K_GEMM_QKV, g, 3, s);
  if (rc) return rc;
  const int dh = d / H;
  switch (dh) {
    case 16: rc = run_fwd_core<16>(ctx, q, k, v, o, lse, B, n, d, H, s, dn.dev); break;
    case 32: rc = run_fwd_core<32>(ctx, q, k, v, o, lse, B, n, d, H, s, dn.dev); break;
    case 64: rc = run_fwd_core<64>(ctx, q, k, v, o, lse, B, n, d, H, s, dn.dev); break;
    case 128: rc = run_fwd_core<128>(ctx, q, k, v, o, lse, B, n, d, H, s, dn.dev); break;
    default: return VARDROP_EUNSUPPORTED;
  }
  if (rc) return rc;
  GemmF32 go = {};
  go.A[0] = o; go.B[0] = W[3]; go.C[0] = y; go.bias[0] = bias[3];
  go.sam = d; go.sak = 1; go.sbk = d; go.sbn = 1;
  go.M = (int)M; go.N = d; go.K = d; go.ldc = d; go.nseg = 1;
  go.count(dn, false, n, B, 0);
  return launch_gemm(ctx, VARDROP_K_GEMM_OUT, go, 1, s);
}

// ws: dO, dq, dk, dv ([M][d] fp32 each) then D [B][H][n]
int vd_attn_bwd_f32(vardrop_ctx* ctx, const float* dy, const float* xs, int B, int n, int d, int H,
                    const float* const W[4], const void* saved, float* dxs,
                    float* const dW[4], float* const db[4], void* ws, hipStream_t s, VdDevCount dn) {
  const long long M = (long long)B * n;
  const float* q = (const float*)saved;
  const float* k = q + M * d;
  const float* v = k + M * d;
  const float* o = v + M * d;
  const float* lse = o + M * d;
  float* dO = (float*)ws;
  float* dq = dO + M * d;
  float* dk = dq + M * d;
  float* dv = dk + M * d;
  float* D = dv + M * d;
  int rc;
  {  // dO = dy Wo^T
    GemmF32 g = {};
    g.A[0] = dy; g.B[0] = W[3]; g.C[0] = dO;
    g.sam = d; g.sak = 1; g.sbk = 1; g.sbn = d;      // B(k, n) = Wo[n][k]
    g.M = (int)M; g.N = d; g.K = d; g.ldc = d; g.nseg = 1;
    g.count(dn, true, n, B, 0);
    if ((rc = launch_gemm(ctx, VARDROP_K_GEMM_DO, g, 1, s))) return rc;
  }
  const int dh = d / H;
  switch (dh) {
    case 16: rc = run_bwd_core<16>(ctx, q, k, v, o, dO, lse, dq, dk, dv, D, B, n, d, H, s, dn.dev); break;
    case 32: rc = run_bwd_core<32>(ctx, q, k, v, o, dO, lse, dq, dk, dv, D, B, n, d, H, s, dn.dev); break;
    case 64: rc = run_bwd_core<64>(ctx, q, k, v, o, dO, lse, dq, dk, dv, D, B, n, d, H, s, dn.dev); break;
    case 128: rc = run_bwd_core<128>(ctx, q, k, v, o, dO, lse, dq, dk, dv, D, B, n, d, H, s, dn.dev); break;
    default: return VARDROP_EUNSUPPORTED;
  }
  if (rc) return rc;
  {  // dWo = o^T dy
    GemmF32 g = {};
    g.A[0] = o; g.B[0] = dy; g.C[0] = dW[3];
    g.sam = 1; g.sak = d; g.sbk = d; g.sbn = 1;      // A(m, k) = o[k][m]
    g.M = d; g.N = d; g.K = (int)M; g.ldc = d; g.nseg = 1;
    g.count(dn, false, n, B, 1);
    if ((rc = launch_gemm(ctx, VARDROP_K_GEMM_DW, g, 1, s))) return rc;
  }
  {  // dWq, dWk, dWv = xs^T dq, xs^T dk, xs^T dv
    GemmF32 g = {};
    const float* grads[3] = {dq, dk, dv};
    for (int z = 0; z < 3; ++z) {
      g.A[z] = xs; g.B[z] = grads[z]; g.C[z] = dW[z];
    }
    g.sam = 1; g.sak = d; g.sbk = d; g.sbn = 1;
    g.M = d; g.N = d; g.K = (int)M; g.ldc = d; g.nseg = 1;
    g.count(dn, false, n, B, 1);
    if ((rc = launch_gemm(ctx, VARDROP_K_GEMM_DW, g, 3, s))) return rc;
  }
  {  // dxs = dq Wq^T + dk Wk^T + dv Wv^T
    GemmF32 g = {};
    const float* grads[3] = {dq, dk, dv};
    for (int z = 0; z < 3; ++z) {
      g.A[z] = grads[z]; g.B[z] = W[z];
    }
    g.C[0] = dxs;
    g.sam = d; g.sak = 1; g.sbk = 1; g.sbn = d;
    g.M = (int)M; g.N = d; g.K = d; g.ldc = d; g.nseg = 3;
    g.count(dn, false, n, B, 0);
    if ((rc = launch_gemm(ctx, VARDROP_K_GEMM_DXS, g, 1, s))) return rc;
  }
  if (db[0] || db[1] || db[2] || db[3]) {
    ColSumF32 c = {};
    c.src[0] = dq; c.src[1] = dk; c.src[2] = dv; c.src[3] = dy;
    for (int z = 0; z < 4; ++z) c.dst[z] = db[z];
    c.rows = M; c.d = d;
    c.n_dev = dn.dev; c.n_max = n; c.n_mul = B;
    hipLaunchKernelGGL(colsum_f32_kernel, dim3(vd_ceil_div(d, 256), 4), dim3(256), 0, s, c);
    VD_LAUNCH_CHECK(ctx);
  }
  return VARDROP_OK;
}

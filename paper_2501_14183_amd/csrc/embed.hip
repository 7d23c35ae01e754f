// Token embedding of the kept variates only (Sec. 3.1 / 3.3: the reduction works directly from the raw
// variates, so the tokens of the dropped ones are never formed): xs = z We + be, where z are the kept
// windows, optionally standardised over time, and its weight gradients dWe = z^T dxs, dbe = colsum(dxs).
//
// Short windows in bf16 (at most 383 samples) take one kernel forward: the standardisation happens inside the
// operand load of the product (embed_fwd_fused_kernel below), and one product backward, which also yields the bias
// gradient (a column of ones rides beside the window in the saved operand).  Everything else takes two steps.
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


// ------------------------------------------------------------------ fused forward (bf16, short windows)
// xs[m][:] = z[m][:] We + be for a tile of 64 kept windows x 128 columns, with z formed inside the kernel: the
// workgroup requests the whole We panel of its columns ([Lp][128], asynchronous copies into LDS), and while that
// travels four threads per window read the tile's 64 windows from the raw batch through `sel`, standardise them
// (mean and variance: partial sums of the four threads, joined in a fixed order) and write them as bf16 into the LDS tile the
// matrix instruction reads its left operand from; the column tile 0 also writes them to `saved` for the backward
// pass, with a one at sample position L (so that z^T dxs has the column sums of dxs, the bias gradient, as row L).
// LDS: KT = Lp / 64 slices of the z tile ([64][64] bf16, 16-byte chunk position XORed with row % 8) and of the We
// panel ([64][128] bf16, chunk position XORed as in the GEMM's n-contiguous operands), then reused for the output tile.
struct EmbedFused {
  const float* x;
  const int32_t* sel;
  const bf16_t* We;
  const bf16_t* be;
  bf16_t* xs;
  bf16_t* saved;
  long long sb, sn;
  int N, L, Lp, n_sel, d, standardise;
  int vec;                    // rows can be read as aligned float4 (x, sb, sn multiples of 4 elements)
  long long M;
  const int32_t* n_dev;       // device-side count of kept windows (then n_sel is its bound, see vd_count)
  int32_t* status;
  int B;
};
constexpr int kEmbedMaxKT = 6;

template <int UL>   // samples per lane: Lp / 64
__global__ __launch_bounds__(256, 2) void embed_fwd_fused_kernel(EmbedFused a) {
  constexpr int BM = 64, BN = 128, A_SLICE = BM * 64 * 2, B_SLICE = 64 * BN * 2, CPITCH = BN * 2 + 16;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  int n_sel;
  if (!vd_count(a.n_dev, a.n_sel, n_sel, a.status) || n_sel == 0) return;
  const long long M = a.n_dev ? (long long)a.B * n_sel : a.M;
  const int gx = (a.d + BN - 1) / BN, gy = (int)((M + BM - 1) / BM);
  if ((int)blockIdx.x >= gx * gy) return;
  const int t = xcd_contiguous(blockIdx.x, gx * gy);
  const int bx = t % gx, by = t / gx;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int col = lane & 31, half = lane >> 5;
  const int m0 = by * BM, n0 = bx * BN;
  const int L = a.L, KT = a.Lp >> 6;
  unsigned char* Az = smem;
  unsigned char* Bs = smem + KT * A_SLICE;

  // ---- the We panel: rows 64 kt .. 64 kt + 63 (clamped to the last row: those meet zeros of z), columns n0 .. n0 + 127
  {
    const int krow = wave * 4 + (lane >> 4);              // copy u covers k-rows 16 u + 4 wave .. + 3
    for (int kt = 0; kt < KT; ++kt)
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int kr = u * 16 + krow;
        const int cc = min(n0 + (((lane & 15) ^ swz_nc<BN>(kr)) * 8), a.d - 8);
        dma16(a.We + (long long)min(kt * 64 + kr, L - 1) * a.d + cc, Bs + kt * B_SLICE + u * 4096 + wave * 1024);
      }
  }
  // ---- the windows: four threads per row of the tile, thread j of a row takes its 16-byte chunks (8 samples)
  // j, j + 4, ...; sums meet by two exchanges inside the group of four, in a fixed order
  {
    const int r = threadIdx.x >> 2, j = threadIdx.x & 3;
    const long long m = m0 + r;
    bool live = m < M;
    const long long b = live ? m / n_sel : 0;
    const int i = live ? (int)(m - b * n_sel) : 0;
    const int n = live ? a.sel[i] : 0;
    live = live && (unsigned)n < (unsigned)a.N;            // an index out of range stands for a zero window
    const float* p = a.x + b * a.sb + (long long)(live ? n : 0) * a.sn;
    const int nchunk = L >> 3;                             // (L is a multiple of 8)
    float v[2 * UL][8];
    float sum = 0.f;
#pragma unroll
    for (int c2 = 0; c2 < 2 * UL; ++c2) {
      const int c = j + 4 * c2;
      const bool in = live && c < nchunk;
      if (a.vec) {
        const float4* q = reinterpret_cast<const float4*>(p + 8 * (in ? c : 0));
        const float4 lo = q[0], hi = q[1];
        v[c2][0] = lo.x; v[c2][1] = lo.y; v[c2][2] = lo.z; v[c2][3] = lo.w;
        v[c2][4] = hi.x; v[c2][5] = hi.y; v[c2][6] = hi.z; v[c2][7] = hi.w;
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[c2][e] = p[8 * (in ? c : 0) + e];
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        v[c2][e] = in ? v[c2][e] : 0.f;
        sum += v[c2][e];
      }
    }
    if (a.standardise) {
      sum += __shfl_xor(sum, 1, 64);
      sum += __shfl_xor(sum, 2, 64);
      const float mean = sum / (float)L;
      float ss = 0.f;
#pragma unroll
      for (int c2 = 0; c2 < 2 * UL; ++c2) {
        const bool in = j + 4 * c2 < nchunk;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          v[c2][e] = in ? v[c2][e] - mean : 0.f;
          ss = fmaf(v[c2][e], v[c2][e], ss);
        }
      }
      ss += __shfl_xor(ss, 1, 64);
      ss += __shfl_xor(ss, 2, 64);
      const float var = ss / (float)L;
      const float inv = var > 0.f ? 1.0f / sqrtf(var) : 1.0f;      // (a constant window is all zeros already)
#pragma unroll
      for (int c2 = 0; c2 < 2 * UL; ++c2)
#pragma unroll
        for (int e = 0; e < 8; ++e) v[c2][e] *= inv;
    }
#pragma unroll
    for (int c2 = 0; c2 < 2 * UL; ++c2) {
      const int c = j + 4 * c2;                            // chunk of the row: samples 8 c .. 8 c + 7, slice c / 8
      u32x4 z;
      z.x = pack2(v[c2][0], v[c2][1]); z.y = pack2(v[c2][2], v[c2][3]);
      z.z = pack2(v[c2][4], v[c2][5]); z.w = pack2(v[c2][6], v[c2][7]);
      *reinterpret_cast<u32x4*>(Az + (c >> 3) * A_SLICE + r * 128 + (((c & 7) ^ swz_kc<64>(r)) * 16)) = z;
      if (bx == 0 && m < M) {
        if (c == nchunk) z.x = 0x3F80u;                    // a bf16 one at sample position L (see above)
        *reinterpret_cast<u32x4*>(a.saved + m * a.Lp + 8 * c) = z;
      }
    }
  }
  wait_vm<0>();
  __syncthreads();

  // ---- product: wavefront (wm, wn) takes rows 32 wm .. + 31, columns 64 wn .. + 63; formed transposed so that a
  // lane owns an output row
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
  const int ra = wm * 32 + col;
  uint32_t addrB[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int krow = 8 * half + ((lane & 15) >> 2);
    const int mn = wn * 64 + j * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
    addrB[j] = lds0 + KT * A_SLICE + krow * (BN * 2) + (((mn >> 3) ^ swz_nc<BN>(krow)) * 16) + ((mn >> 2) & 1) * 8;
  }
  floatx16 acc[2] = {zero16(), zero16()};
  for (int kt = 0; kt < KT; ++kt) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      Frag fa, fb[2];
      lds_read16(fa.q, lds0 + kt * A_SLICE + ra * 128 + (((2 * ks + half) ^ swz_kc<64>(ra)) * 16));
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const uint32_t base = addrB[j] + kt * B_SLICE + ks * 16 * BN * 2;
        lds_read8_tr<0>(fb[j].d[0], base);
        lds_read8_tr<4 * BN * 2>(fb[j].d[1], base);
      }
      wait_lds<0>(fa, fb[0], fb[1]);
      acc[0] = mfma(fb[0], fa, acc[0]);
      acc[1] = mfma(fb[1], fa, acc[1]);
    }
  }
  // ---- output tile through LDS (bias added), then 16-byte chunks of whole rows
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int nl = wn * 64 + j * 32 + 8 * q4 + 4 * half;
      float bv[4] = {0.f, 0.f, 0.f, 0.f};
      if (a.be && n0 + nl < a.d) {
        const u32x2 b4 = *reinterpret_cast<const u32x2*>(a.be + n0 + nl);
        bv[0] = __uint_as_float(b4.x << 16); bv[1] = __uint_as_float(b4.x & 0xffff0000u);
        bv[2] = __uint_as_float(b4.y << 16); bv[3] = __uint_as_float(b4.y & 0xffff0000u);
      }
      u32x2 o;
      o.x = pack2(acc[j][4 * q4] + bv[0], acc[j][4 * q4 + 1] + bv[1]);
      o.y = pack2(acc[j][4 * q4 + 2] + bv[2], acc[j][4 * q4 + 3] + bv[3]);
      *reinterpret_cast<u32x2*>(smem + ra * CPITCH + nl * 2) = o;
    }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < BM * 16 / 256; ++u) {
    const int idx = u * 256 + threadIdx.x;
    const int row = idx >> 4, c = idx & 15;
    if (m0 + row < M && n0 + c * 8 < a.d) {
      const u32x4 v = *reinterpret_cast<const u32x4*>(smem + row * CPITCH + c * 16);
      *reinterpret_cast<u32x4*>(a.xs + (m0 + row) * (long long)a.d + n0 + c * 8) = v;
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

// bf16 windows short enough for the single-kernel forward (its LDS holds kEmbedMaxKT slices of 64 samples, one
// position past the window included)
bool embed_fused(int L, int dtype) { return dtype == VARDROP_BF16 && (L + 1 + 63) / 64 <= kEmbedMaxKT; }
// row pitch of the saved windows: bf16 rows are padded to a multiple of 64 samples (fused path: of L + 1, the extra
// position holds a one)
int embed_pitch(int L, int dtype) {
  if (dtype != VARDROP_BF16) return L;
  return (int)vd_align_up((size_t)(embed_fused(L, dtype) ? L + 1 : L), 64);
}

int check(int B, int n_sel, int L, int d, int dtype) {
  if (B < 0 || n_sel < 0 || L < 2 || d < 1) return VARDROP_EINVAL;
  if (dtype != VARDROP_F32 && dtype != VARDROP_BF16) return VARDROP_EINVAL;
  if (L > kMaxEmbedL) return VARDROP_EUNSUPPORTED;
  const long long M = (long long)B * n_sel;
  if (M * d >= (1ll << 31) || M * (L + 63) >= (1ll << 31)) return VARDROP_EUNSUPPORTED;
  if (dtype == VARDROP_BF16 && (d % 8 != 0 || L % 8 != 0)) return VARDROP_EUNSUPPORTED;
  return VARDROP_OK;
}

// (the K slices of dWe = z^T dxs follow vd_embed_splitk, common.h)
int embed_splitk(int L, int d, long long M, int* kchunk) { return vd_embed_splitk(L, d, M, kchunk); }

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
  return embed_colsum_bytes(d) + (dtype == VARDROP_BF16 ? vd_align_up((size_t)16 * (L + 8) * d * sizeof(float), 256) : 0);
}

namespace {
template <int UL>
int launch_embed_fused(vardrop_ctx* ctx, const EmbedFused& a, long long M_bound, hipStream_t s) {
  const int lds = UL * (64 * 64 * 2 + 64 * 128 * 2);
  if (lds > 65536)
    VD_HIP(ctx, hipFuncSetAttribute((const void*)embed_fwd_fused_kernel<UL>, hipFuncAttributeMaxDynamicSharedMemorySize, lds));
  const long long grid = (long long)vd_ceil_div(a.d, 128) * ((M_bound + 63) / 64);
  {
    VdTimer timer(ctx, VARDROP_K_EMBED_FUSED, s);
    VD_KERNEL(ctx, embed_fwd_fused_kernel<UL>, dim3((unsigned)grid), dim3(256), lds, s, a);
  }
  VD_LAUNCH_CHECK(ctx);
  return VARDROP_OK;
}

// n_sel is the count, or with dn.dev its bound
int embed_fwd(vardrop_ctx* ctx, const float* x, int B, int N, int L, int64_t sb, int64_t sn,
              const int32_t* sel, int n_sel, int standardise, const void* We, const void* be, int d, int dtype,
              void* xs, void* saved, hipStream_t s, VdDevCount dn) {
  int rc = check(B, n_sel, L, d, dtype);
  if (rc) return rc;
  if (N < 0 || n_sel > N || sb < 0 || sn < 0) return VARDROP_EINVAL;
  const long long M = (long long)B * n_sel;
  if (M == 0) return VARDROP_OK;
  if (!x || !sel || !We || !xs || !saved) return VARDROP_EINVAL;
  if (!vd_aligned(saved, 256)) return VARDROP_EWORKSPACE;
  const int pitch = embed_pitch(L, dtype);
  if (embed_fused(L, dtype)) {
    if (!vd_aligned(We, 16) || !vd_aligned(xs, 16)) return VARDROP_EINVAL;
    EmbedFused a = {};
    a.x = x; a.sel = sel; a.We = (const bf16_t*)We; a.be = (const bf16_t*)be;
    a.xs = (bf16_t*)xs; a.saved = (bf16_t*)saved;
    a.sb = sb; a.sn = sn; a.N = N; a.L = L; a.Lp = pitch; a.n_sel = n_sel; a.d = d; a.standardise = standardise;
    a.M = M; a.n_dev = dn.dev; a.status = dn.status; a.B = B;
    a.vec = vd_aligned(x, 16) && sb % 4 == 0 && sn % 4 == 0;
    switch (pitch / 64) {
      case 1: return launch_embed_fused<1>(ctx, a, M, s);
      case 2: return launch_embed_fused<2>(ctx, a, M, s);
      case 3: return launch_embed_fused<3>(ctx, a, M, s);
      case 4: return launch_embed_fused<4>(ctx, a, M, s);
      case 5: return launch_embed_fused<5>(ctx, a, M, s);
      default: return launch_embed_fused<6>(ctx, a, M, s);
    }
  }
  if (dn.dev) return VARDROP_EUNSUPPORTED;      // the two-step path takes a host count
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

int embed_bwd(vardrop_ctx* ctx, const void* dxs, int B, int n_sel, int L, int d, int dtype,
              const void* saved, float* dWe, float* dbe, void* ws, size_t ws_bytes, hipStream_t s, VdDevCount dn) {
  int rc = check(B, n_sel, L, d, dtype);
  if (rc) return rc;
  if (!dWe) return VARDROP_EINVAL;
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
  if (embed_fused(L, dtype)) {
    // One product: [dWe ; dbe] = [z | 1]^T dxs, the operand rows L + 1 .. up to the next multiple of 8 are zeros.
    // Its K slices always go through the partial sums (the result is not one contiguous matrix of the caller's).
    GemmBf16 g = {};
    g.set(0, saved, dxs, nullptr, nullptr);
    g.lda = pitch; g.ldb = d; g.ldc = d;
    g.M = (int)vd_align_up((size_t)L + 1, 8); g.N = d; g.K = (int)M; g.nseg = 1;
    int kchunk = 0;
    g.splitk = embed_splitk(g.M, d, M, &kchunk);
    g.kchunk = kchunk;
    g.part = slices;
    g.force_part = 1;
    if (dn.dev) {
      g.count_k(dn.dev, n_sel, B);
      g.n_role = 2;                                  // the slices follow the embedding's rule
      g.splitk = 16;                                 // (the grid is sized for the largest number of slices)
    }
    if ((rc = vd_gemm_bf16_wgrad_split(ctx, VARDROP_K_GEMM_DWE, g, s))) return rc;
    return vd_gemm_bf16_sum_rows(ctx, slices, dWe, (long long)L * d, dbe, d, (long long)g.M * d, g.splitk, s,
                                 dn.dev ? &g : nullptr);
  }
  if (dn.dev) return VARDROP_EUNSUPPORTED;
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
}  // namespace

extern "C" int vardrop_embed_fwd(vardrop_ctx* ctx, const float* x, int B, int N, int L, int64_t sb, int64_t sn,
                                 const int32_t* sel, int n_sel, int standardise,
                                 const void* We, const void* be, int d, int dtype,
                                 void* xs, void* saved, void* stream) {
  if (!ctx) return VARDROP_EINVAL;
  return embed_fwd(ctx, x, B, N, L, sb, sn, sel, n_sel, standardise, We, be, d, dtype, xs, saved, (hipStream_t)stream,
                   VdDevCount{nullptr, nullptr});
}

extern "C" int vardrop_embed_fwd_dev(vardrop_ctx* ctx, const float* x, int B, int N, int L, int64_t sb, int64_t sn,
                                     const int32_t* sel, const int32_t* n_dev, int n_max, int32_t* status, int standardise,
                                     const void* We, const void* be, int d, int dtype,
                                     void* xs, void* saved, void* stream) {
  if (!ctx || !n_dev || n_max < 1) return VARDROP_EINVAL;
  return embed_fwd(ctx, x, B, N, L, sb, sn, sel, n_max, standardise, We, be, d, dtype, xs, saved, (hipStream_t)stream,
                   VdDevCount{n_dev, status});
}

extern "C" int vardrop_embed_bwd_dev(vardrop_ctx* ctx, const void* dxs, int B, const int32_t* n_dev, int n_max, int L, int d,
                                     int dtype, const void* saved, float* dWe, float* dbe,
                                     void* ws, size_t ws_bytes, void* stream) {
  if (!ctx || !n_dev || n_max < 1 || B < 1) return VARDROP_EINVAL;
  return embed_bwd(ctx, dxs, B, n_max, L, d, dtype, saved, dWe, dbe, ws, ws_bytes, (hipStream_t)stream,
                   VdDevCount{n_dev, nullptr});
}

extern "C" int vardrop_embed_bwd(vardrop_ctx* ctx, const void* dxs, int B, int n_sel, int L, int d, int dtype,
                                 const void* saved, float* dWe, float* dbe,
                                 void* ws, size_t ws_bytes, void* stream) {
  if (!ctx) return VARDROP_EINVAL;
  return embed_bwd(ctx, dxs, B, n_sel, L, d, dtype, saved, dWe, dbe, ws, ws_bytes, (hipStream_t)stream,
                   VdDevCount{nullptr, nullptr});
}

// k-dominant frequency hashing (Alg. 1, Def. 1) as one fused gfx950 kernel.
//
// Mapping.  A workgroup of four wavefronts owns a block of 32 (variate, window) rows: all B
// windows of one variate when B >= 32 (several blocks in sequence when B > 32), or 32/Bp variates
// with Bp = B rounded up to a power of two when B < 32.  The block's windows are staged in LDS
// (time-major, padded), and the amplitude spectrum on the candidate bins is a dense contraction of
// the folded window with a cosine / sine table:
//     Re X_f =  x[0] + (-1)^f x[L/2] + sum_{0<t<L/2} (x[t] + x[L-t]) cos(2 pi f t / L)
//     Im X_f = -sum_{0<t<L/2} (x[t] - x[L-t]) sin(2 pi f t / L)
// evaluated with the fp32 matrix instruction v_mfma_f32_16x16x4_f32 (rows = windows, columns = bins,
// contraction = folded time).  Each of the four wavefronts owns a 16 x 16 quadrant of the block's
// 32 windows x 32 bins and runs the whole contraction on it, so loads, folding and matrix work of
// a block run four wide and nothing is reduced across wavefronts.  The bins above the cut-off are never produced (Alg. 1
// step 2).  Amplitudes are summed over the batch in ascending window order in fp32 (step 3), and
// the ranked top-k (step 4) is k rounds of a wavefront arg-max with the lower bin winning ties; the
// hash is the tuple in radix R (step 5).
#include "common.h"

typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kTilePad = 33;     // LDS row stride of the time-major tile (32 rows + 1)
constexpr int kMaxBinsPerLane = 8;
constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;

__global__ void twiddle_kernel(float* tw, int L) {
  int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < L) {
    double s, c;
    sincospi(2.0 * (double)j / (double)L, &s, &c);
    tw[j] = (float)c;
    tw[L + j] = (float)s;
  }
}

struct KdfhArgs {
  const float* x;
  const float* tw;
  int32_t* topk;
  uint64_t* hash;
  float* abar;
  long long sb, sn;
  int B, N, L, k, f_min, F;
  int log2_rpv;   // rows per variate inside a 32-row block = 1 << log2_rpv
  int nrb;        // 32-row blocks per variate group (> 1 only when B > 32)
  int vec;        // rows can be read as aligned float4
  float inv_B;
};

__global__ __launch_bounds__(kThreads) void kdfh_kernel(KdfhArgs a) {
  extern __shared__ float lds[];
  const int L = a.L, F = a.F;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, half = lane >> 5;
  const int rpv = 1 << a.log2_rpv;
  const int Vb = 32 >> a.log2_rpv;               // variates per block
  const int n0 = blockIdx.x * Vb;
  float* cosT = lds;
  float* sinT = lds + L;
  float* tile = sinT + L;                        // [L + 1][kTilePad], last row zero
  float* ampT = tile + (L + 1) * kTilePad;       // [32][kTilePad]
  float* psum = ampT + 32 * kTilePad;            // [8][32] partial batch sums
  float* asum = psum + 8 * 32;                   // [Vb][F]

  for (int i = tid; i < 2 * L; i += kThreads) lds[i] = a.tw[i];
  for (int i = tid; i < Vb * F; i += kThreads) asum[i] = 0.f;

  const int Lh = L >> 1;
  const int S4 = (Lh + 4) >> 2;                  // steps of four folded time samples: t = 0 .. floor(L/2)
  const int nct = (F + 31) >> 5;

  for (int rb = 0; rb < a.nrb; ++rb) {
    __syncthreads();
    // ---- stage 32 windows in LDS, time-major: tile[t][row]
    if (a.vec) {
      const int L4 = L >> 2;
      const int items = 32 * L4;
      for (int base = 0; base < items; base += kThreads * 4) {
        float4 v[4];
        int rr[4], cc[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int i = base + u * kThreads + tid;
          const int ic = i < items ? i : 0;                      // clamped: the load is unconditional
          const int r = ic / L4;
          const int c = ic - r * L4;
          rr[u] = i < items ? r : -1;
          cc[u] = c;
          const int n = min(n0 + (r >> a.log2_rpv), a.N - 1);
          const int b = min(rb * 32 + (r & (rpv - 1)), a.B - 1);
          const bool ok = (n0 + (r >> a.log2_rpv) < a.N) && (rb * 32 + (r & (rpv - 1)) < a.B);
          const float4 t = *reinterpret_cast<const float4*>(a.x + (long long)b * a.sb + (long long)n * a.sn + 4 * c);
          v[u] = make_float4(ok ? t.x : 0.f, ok ? t.y : 0.f, ok ? t.z : 0.f, ok ? t.w : 0.f);   // rows past the end are zero windows
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (rr[u] >= 0) {
            float* p = tile + (4 * cc[u]) * kTilePad + rr[u];
            p[0] = v[u].x;
            p[kTilePad] = v[u].y;
            p[2 * kTilePad] = v[u].z;
            p[3 * kTilePad] = v[u].w;
          }
        }
      }
    } else {
      for (int r = wave; r < 32; r += kWaves) {
        const int n = n0 + (r >> a.log2_rpv);
        const int b = rb * 32 + (r & (rpv - 1));
        const bool ok = n < a.N && b < a.B;
        const float* p = a.x + (long long)b * a.sb + (long long)n * a.sn;
        for (int t = lane; t < L; t += 64) tile[t * kTilePad + r] = ok ? p[t] : 0.f;
      }
    }
    __syncthreads();
    // ---- fold in place: row t becomes x[t] + x[L-t] and row L-t becomes x[t] - x[L-t] for
    // 0 < t < L/2 (rows 0 and L/2 stay); row L is a zero row for steps past the end.
    const bool folded = nct > 1;      // one column tile reads every sample once: folding on the fly is cheaper
    if (folded) {
      const int npair = (L - 1) >> 1;
      for (int i = tid; i < npair * 32; i += kThreads) {
        const int t = 1 + (i >> 5), r = i & 31;
        const float p = tile[t * kTilePad + r], q = tile[(L - t) * kTilePad + r];
        tile[t * kTilePad + r] = p + q;
        tile[(L - t) * kTilePad + r] = p - q;
      }
    }
    if (tid < 32) tile[L * kTilePad + tid] = 0.f;
    __syncthreads();

    // ---- spectrum of the 32 rows, 32 bins at a time.  The four wavefronts take one 16 x 16 quadrant of
    // the 32 x 32 (window, bin) tile each and run the whole contraction on it with
    // v_mfma_f32_16x16x4_f32 (four folded time samples per instruction), so no partial sums are exchanged.
    // Operand layout: A[i][k] lane holds row i = lane % 16, k = lane / 16; B[k][j] lane holds column
    // j = lane % 16, the same k; C[i][j] lane holds column j = lane % 16, register r holds row 4*(lane/16) + r.
    for (int ct = 0; ct < nct; ++ct) {
      const int i16 = lane & 15, kq = lane >> 4;
      const int rh = wave & 1, ch = wave >> 1;
      const int f = a.f_min + ct * 32 + ch * 16 + i16;
      const int step4 = (4 * f) % L;             // advancing one step moves t by 4
      int m = (f * kq) % L;                      // (f t) mod L: index into both tables
      floatx4 re = {0.f, 0.f, 0.f, 0.f}, im = re;
      // Re uses rows t <= L/2 (x[0], the sums, x[L/2]); Im uses rows L - t for 0 < 2t < L (the
      // differences); every other step reads the zero row L.  Software pipeline: the operands of the
      // next step are read from LDS while the matrix instructions of this one run.
      const int arow = rh * 16 + i16;
      int t = kq;
      // p = row t (or zero past L/2), q = row L - t when 0 < 2t < L (else zero); folded rows already hold
      // p + q and p - q, unfolded ones are combined here
      float p = tile[(t <= Lh ? t : L) * kTilePad + arow];
      float q = tile[((t > 0 && 2 * t < L) ? L - t : L) * kTilePad + arow];
      float ac = folded ? p : p + q;
      float as = folded ? q : ((t > 0 && 2 * t < L) ? p - q : 0.f);
      float bc = cosT[m], bs = sinT[m];
      for (int s = 0; s < S4; ++s) {
        const float ac0 = ac, as0 = as, bc0 = bc, bs0 = bs;
        t += 4;
        m += step4;
        if (m >= L) m -= L;
        p = tile[(t <= Lh ? t : L) * kTilePad + arow];
        q = tile[(2 * t < L ? L - t : L) * kTilePad + arow];
        ac = folded ? p : p + q;
        as = folded ? q : (2 * t < L ? p - q : 0.f);
        bc = cosT[m];
        bs = sinT[m];
        __builtin_amdgcn_sched_barrier(0);
        re = __builtin_amdgcn_mfma_f32_16x16x4f32(ac0, bc0, re, 0, 0, 0);
        im = __builtin_amdgcn_mfma_f32_16x16x4f32(as0, bs0, im, 0, 0, 0);
        // (keeps the reads above in this iteration: without it the compiler folds them back into
        //  the top of the next one, in front of the instructions that need them)
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("" : "+v"(ac), "+v"(as), "+v"(bc), "+v"(bs));
      }
#pragma unroll
      for (int r = 0; r < 4; ++r)
        ampT[(rh * 16 + 4 * kq + r) * kTilePad + ch * 16 + i16] = sqrtf(re[r] * re[r] + im[r] * im[r]);
      __syncthreads();
      // batch sums (Alg. 1 step 3).  The eight 32-lane groups add four windows each, ascending; with
      // fewer than eight variates in the block the groups of a variate then add their partial sums,
      // ascending again, so the order of the additions is fixed.
      const int bin = ct * 32 + col;
      const int grp = tid >> 5;
      if (Vb <= 8) {
        float sum = 0.f;
#pragma unroll
        for (int b = 0; b < 4; ++b) sum += ampT[(grp * 4 + b) * kTilePad + col];
        psum[grp * 32 + col] = sum;
        __syncthreads();
        const int gpv = 8 / Vb;                   // groups per variate
        if (grp % gpv == 0 && bin < F) {
          float total = 0.f;
          for (int u = 0; u < gpv; ++u) total += psum[(grp + u) * 32 + col];
          asum[(grp / gpv) * F + bin] += total;
        }
      } else {
        for (int v = grp; v < Vb; v += kThreads / 32) {
          float sum = 0.f;
          for (int b = 0; b < rpv; ++b) sum += ampT[(v * rpv + b) * kTilePad + col];
          if (bin < F) asum[v * F + bin] += sum;
        }
      }
      __syncthreads();                            // ampT and psum are rewritten by the next column tile
    }
  }
  __syncthreads();

  // ---- ranked top-k and hash; the variates of the block are shared out over the wavefronts
  const unsigned long long R = (unsigned long long)(L / 2 + 1);
  for (int v = wave; v < Vb; v += kWaves) {
    const int n = n0 + v;
    if (n >= a.N) break;
    float vals[kMaxBinsPerLane];
#pragma unroll
    for (int j = 0; j < kMaxBinsPerLane; ++j) {
      const int idx = lane + 64 * j;
      vals[j] = idx < F ? asum[v * F + idx] : -2.f;
    }
    unsigned long long h = 0;
    if (F <= 64) {
      // every lane holds one bin: its rank is the number of bins that beat it (larger mean amplitude, or
      // equal and lower index); the lanes of rank 0 .. k-1 are the ranked top-k
      const float mine = vals[0];
      int rank = 0;
      for (int j = 0; j < F; ++j) {
        const float vj = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mine), j));
        rank += (vj > mine || (vj == mine && j < lane)) ? 1 : 0;
      }
      for (int r = 0; r < a.k; ++r) {
        const unsigned long long mask = __ballot(lane < F && rank == r);
        const int fsel = a.f_min + (__ffsll((long long)mask) - 1);
        if (lane == 0) a.topk[(long long)n * a.k + r] = fsel;
        h = h * R + (unsigned long long)(unsigned)fsel;
      }
    } else
    for (int r = 0; r < a.k; ++r) {
      float best = -3.f;
      int bi = 0x7fffffff;
#pragma unroll
      for (int j = 0; j < kMaxBinsPerLane; ++j) {
        if (vals[j] > best) {
          best = vals[j];
          bi = lane + 64 * j;
        }
      }
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(best, off, 64);
        const int oi = __shfl_xor(bi, off, 64);
        if (ov > best || (ov == best && oi < bi)) {
          best = ov;
          bi = oi;
        }
      }
#pragma unroll
      for (int j = 0; j < kMaxBinsPerLane; ++j)
        if (bi == lane + 64 * j) vals[j] = -2.f;
      const int fsel = a.f_min + bi;
      if (lane == 0) a.topk[(long long)n * a.k + r] = fsel;
      h = h * R + (unsigned long long)(unsigned)fsel;
    }
    if (lane == 0) a.hash[n] = h;
    if (a.abar)
      for (int idx = lane; idx < F; idx += 64) a.abar[(long long)n * F + idx] = asum[v * F + idx] * a.inv_B;
  }
}

size_t kdfh_lds_bytes(int L, int F, int Vb) {
  return sizeof(float) * ((size_t)2 * L + (size_t)(L + 1) * kTilePad + 32 * kTilePad + 8 * 32 + (size_t)Vb * F);
}

}  // namespace

extern "C" size_t vardrop_hash_workspace_bytes(int, int, int, int, int, int) { return 0; }

extern "C" int vardrop_hash(vardrop_ctx* ctx, const float* x, int B, int N, int L,
                            int64_t sb, int64_t sn, int64_t st, int k, int f_min, int f_max,
                            int32_t* topk, uint64_t* hash, float* abar,
                            void* ws, size_t ws_bytes, void* stream) {
  (void)ws;
  (void)ws_bytes;
  if (!ctx) return VARDROP_EINVAL;
  if (B < 1 || N < 0 || L < 2) return VARDROP_EINVAL;
  if (f_min < 0 || f_max < f_min || f_max > L / 2) return VARDROP_EINVAL;
  const int F = f_max - f_min + 1;
  if (k < 1 || k > F) return VARDROP_EINVAL;
  {
    const unsigned long long R = (unsigned long long)(L / 2 + 1);
    unsigned long long p = 1;
    for (int j = 0; j < k; ++j) {
      if (p > (1ull << 63) / R) return VARDROP_EINVAL;
      p *= R;
    }
    if (p >= (1ull << 63)) return VARDROP_EINVAL;
  }
  if (N == 0) return VARDROP_OK;
  if (!x || !topk || !hash) return VARDROP_EINVAL;
  if (sb < 0 || sn < 0) return VARDROP_EINVAL;
  if (st != 1) return VARDROP_EUNSUPPORTED;
  if (L > 1024 || F > 64 * kMaxBinsPerLane) return VARDROP_EUNSUPPORTED;

  int log2_rpv = 5, nrb = vd_ceil_div(B, 32);
  if (B < 32) {
    log2_rpv = 0;
    while ((1 << log2_rpv) < B) ++log2_rpv;
    nrb = 1;
  }
  const int Vb = 32 >> log2_rpv;
  const size_t lds = kdfh_lds_bytes(L, F, Vb);
  if (lds > (size_t)ctx->lds_per_block) return VARDROP_EUNSUPPORTED;

  hipStream_t s = (hipStream_t)stream;
  if (ctx->twiddle_L != L) {
    hipLaunchKernelGGL(twiddle_kernel, dim3(vd_ceil_div(L, 256)), dim3(256), 0, s, ctx->twiddle, L);
    VD_LAUNCH_CHECK(ctx);
    ctx->twiddle_L = L;
  }
  KdfhArgs a;
  a.x = x;
  a.tw = ctx->twiddle;
  a.topk = topk;
  a.hash = hash;
  a.abar = abar;
  a.sb = sb;
  a.sn = sn;
  a.B = B;
  a.N = N;
  a.L = L;
  a.k = k;
  a.f_min = f_min;
  a.F = F;
  a.log2_rpv = log2_rpv;
  a.nrb = nrb;
  a.vec = (L % 4 == 0 && sb % 4 == 0 && sn % 4 == 0 && vd_aligned(x, 16)) ? 1 : 0;
  a.inv_B = 1.0f / (float)B;
  if (lds > 65536)
    VD_HIP(ctx, hipFuncSetAttribute((const void*)kdfh_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  {
    VdTimer timer(ctx, VARDROP_K_HASH, s);
    hipLaunchKernelGGL(kdfh_kernel, dim3(vd_ceil_div(N, Vb)), dim3(kThreads), lds, s, a);
  }
  VD_LAUNCH_CHECK(ctx);
  return VARDROP_OK;
}

// k-dominant frequency hashing (Alg. 1, Def. 1) as one fused gfx950 kernel.
//
// Mapping.  A workgroup of four wavefronts owns a block of 32 (variate, window) rows: all B
// windows of one variate when B >= 32 (several blocks in sequence when B > 32), or 32/Bp variates
// with Bp = B rounded up to a power of two when B < 32.  The amplitude spectrum on the candidate
// bins is a dense contraction of the folded window with a cosine / sine table:
//     Re X_f =  x[0] + (-1)^f x[L/2] + sum_{0<t<L/2} (x[t] + x[L-t]) cos(2 pi f t / L)
//     Im X_f = -sum_{0<t<L/2} (x[t] - x[L-t]) sin(2 pi f t / L)
// (rows = windows, columns = bins, contraction = folded time; the x[L/2] term is added afterwards).
// When L is a multiple of 8 (and the rows can be read as aligned float4) one radix-2 step comes first:
// with M = L/2, u[t] = x[t] + x[t+M] and v[t] = x[t] - x[t+M], the even bins are the spectrum of u at
// f/2 and the odd bins that of v with an odd twist, and both fold once more (t <-> M - t):
//     even f:  Re =  u[0] + (-1)^(f/2) u[M/2] + sum_{0<t<M/2} (u[t] + u[M-t]) cos(2 pi f t / L)
//              Im = -sum_{0<t<M/2} (u[t] - u[M-t]) sin(2 pi f t / L)
//     odd f:   Re =  v[0] + sum_{0<t<M/2} (v[t] - v[M-t]) cos(2 pi f t / L)
//              Im = -sum_{0<t<M/2} (v[t] + v[M-t]) sin(2 pi f t / L) - v[M/2] sin(pi f / 2)
// so every bin is a contraction over L/4 samples instead of L/2; even and odd bins get tiles of their own.
// One or two bins that a parity set has left after its full tiles (bin 129 of the 129 candidates of a
// 512-sample window) are contracted by the vector units from the same folded samples instead of occupying
// a tile, and a wavefront, of their own.
//
// Arithmetic.  The contraction runs on the half-precision matrix cores at fp32 quality: every
// operand is split as  v = hi + lo  with hi = fp16(v) and lo = fp16(v - hi), and
//     sum v w  ~=  sum hi_v hi_w  +  sum hi_v lo_w  +  sum lo_v hi_w
// accumulated in fp32 by v_mfma_f32_32x32x16_f16; the dropped lo_v lo_w term is 2^-22 of a product.
// A window is first scaled by a power of two (exact) that brings its largest magnitude to
// [2^12, 2^13), so that the fp16 range holds both pieces whatever the input's scale is, and the
// amplitude is scaled back before the batch sum.  The low piece of a cosine or sine is below 2^-12,
// where fp16 loses precision, so the table stores it times 2^11 and the window's high piece is
// multiplied by 2^-11 (exact) for that product.  The bins above the cut-off are never produced
// (Alg. 1 step 2).  Amplitudes are summed over the batch in a fixed order in fp32 (step 3), the
// ranked top-k (step 4) lets the lower bin win ties, and the hash is the tuple in radix R (step 5).
//
// Data flow.  Every thread reads 8 consecutive samples of a row and the 8 mirrored ones straight
// from global memory, folds them, and writes the four half-precision operand pieces (sum hi / lo,
// difference hi / lo) to LDS in the layout the matrix instruction reads (row-major, 16 bytes per
// lane).  The cosine / sine pieces come from a table in global memory that is laid out in
// matrix-fragment order (it stays in L2) and is rebuilt when L or the candidate bins change.  A
// wavefront owns a tile of 32 bins at a time and runs the whole contraction for it, real and
// imaginary part together, so nothing is exchanged between wavefronts until the batch sums.
#include "common.h"

typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int kMaxBinsPerLane = 8;
constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;
constexpr float kLoUnscale = 1.f / 2048.f;   // 2^-11: the table's low pieces are stored times 2^11

struct Pieces {
  halfx8 hi, lo;
};

__device__ inline void split8(const float (&v)[8], Pieces& p) {
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const _Float16 h = (_Float16)v[j];
    p.hi[j] = h;
    p.lo[j] = (_Float16)(v[j] - (float)h);
  }
}
// The same split with fewer instructions, for values scaled into the normal range of fp16: the high piece is the
// value truncated to fp16 (one conversion instruction per pair, and its float value is the input with the low 13
// mantissa bits cleared), the low piece the remainder, which is exact in fp32, rounded to nearest.  A value below
// 2^-14 loses part of its high piece (the truncating conversion then yields a subnormal): an absolute error below
// 2^-24, against row maxima of at least 2^12.
typedef _Float16 halfx2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
__device__ inline void split8_trunc(const float (&v)[8], Pieces& p) {
#pragma unroll
  for (int j = 0; j < 8; j += 2) {
    const halfx2 h = __builtin_bit_cast(halfx2, __builtin_amdgcn_cvt_pkrtz(v[j], v[j + 1]));
    const floatx2 rem = {v[j] - __uint_as_float(__float_as_uint(v[j]) & 0xffffe000u),
                         v[j + 1] - __uint_as_float(__float_as_uint(v[j + 1]) & 0xffffe000u)};
    const halfx2 lo = __builtin_convertvector(rem, halfx2);
    p.hi[j] = h[0];
    p.hi[j + 1] = h[1];
    p.lo[j] = lo[0];
    p.lo[j + 1] = lo[1];
  }
}

// Table of the twiddle pieces in fragment order: entry ((s * nct + ct) * 4 + kind) * 64 + lane holds,
// for contraction step s and bin tile ct, the 8 halves of lane `lane` of the right-hand operand
// (column = the bin of column lane % 32 of that tile, rows t = 16 s + 8 (lane / 32) + 0..7); kind 0 / 1 = cosine
// hi / lo, 2 / 3 = sine hi / lo.  Entries past the last contracted sample or the last bin are zero.
// Bin of column `c` of bin tile `ct`.  Plain: consecutive bins from f_min.  Radix-2: the first nct_e tiles
// hold the even candidate bins (from fe0, step 2), the rest the odd ones (from fo0).
// With the radix-2 step, one or two bins of a parity set left over after its full tiles of 32 ("stray" bins: bin 129
// of the 129 candidates of a 512-sample window) do not get a tile of their own: the vector units contract them.
constexpr int kMaxStray = 4;
struct BinMap {
  int r2, f_min, nct_e, fe0, fo0;
  int n_stray, stray_f[kMaxStray];
};
__device__ inline int bin_of(const BinMap& m, int ct, int c) {
  if (!m.r2) return m.f_min + ct * 32 + c;
  return ct < m.nct_e ? m.fe0 + 2 * (ct * 32 + c) : m.fo0 + 2 * ((ct - m.nct_e) * 32 + c);
}

__global__ void twiddle_kernel(halfx8* tw, int L, BinMap m, int f_max, int T, int steps, int nct) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= steps * nct * 64) return;
  const int lane = i & 63;
  const int ct = (i >> 6) % nct;
  const int s = (i >> 6) / nct;
  const int f = bin_of(m, ct, lane & 31);
  halfx8 out[4];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int t = 16 * s + 8 * (lane >> 5) + j;
    double sn = 0.0, cs = 0.0;
    if (t < T && f <= f_max) sincospi(2.0 * (double)(((long long)f * t) % L) / (double)L, &sn, &cs);
    const _Float16 ch = (_Float16)(float)cs, sh = (_Float16)(float)sn;
    out[0][j] = ch;
    out[1][j] = (_Float16)(float)((cs - (double)(float)ch) * 2048.0);
    out[2][j] = sh;
    out[3][j] = (_Float16)(float)((sn - (double)(float)sh) * 2048.0);
  }
  const size_t base = ((size_t)(s * nct + ct) * 4) * 64 + lane;
#pragma unroll
  for (int q = 0; q < 4; ++q) tw[base + (size_t)q * 64] = out[q];
}

// Windows whose time stride is not 1 (time-major batches [B][L][N], as forecasting loaders hand them over) are
// first copied into time-contiguous rows: 32 x 32 tiles through LDS, read with the variate index fastest
// (coalesced when the variate stride is 1), written with time fastest.
__global__ __launch_bounds__(256) void time_contiguous_kernel(const float* x, float* out, int N, int L,
                                                              long long sb, long long sn, long long st) {
  __shared__ float tile[32][33];
  const int n0 = blockIdx.x * 32, t0 = blockIdx.y * 32, b = blockIdx.z;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  for (int j = ty; j < 32; j += 8) {
    const int t = t0 + j, n = n0 + tx;
    tile[j][tx] = (t < L && n < N) ? x[(long long)b * sb + (long long)n * sn + (long long)t * st] : 0.f;
  }
  __syncthreads();
  for (int i = ty; i < 32; i += 8) {
    const int n = n0 + i, t = t0 + tx;
    if (n < N && t < L) out[((long long)b * N + n) * L + t] = tile[tx][i];
  }
}

// cosine and sine of the stray bins as plain floats: stw[(i * Tp + t) * 2 + {0, 1}] for stray bin i, t < Tp
__global__ void stray_twiddle_kernel(float* stw, int L, BinMap m, int T, int Tp) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= m.n_stray * Tp) return;
  const int si = i / Tp, t = i - si * Tp;
  double sn = 0.0, cs = 0.0;
  if (t < T) sincospi(2.0 * (double)(((long long)m.stray_f[si] * t) % L) / (double)L, &sn, &cs);
  stw[2 * i] = (float)cs;
  stw[2 * i + 1] = (float)sn;
}

struct KdfhArgs {
  const float* x;
  const halfx8* tw;
  const float* stw;    // twiddles of the stray bins (BinMap::n_stray > 0)
  int32_t* topk;
  uint64_t* hash;
  float* abar;
  long long sb, sn;
  int B, N, L, k, f_min, F;
  BinMap bins;
  int log2_rpv;   // rows per variate inside a 32-row block = 1 << log2_rpv
  int nrb;        // 32-row blocks per variate group (> 1 only when B > 32)
  int T;          // folded samples in the contraction: t = 0 .. T-1, T = ceil(L / 2), or L / 4 after the radix-2 step
  int KS;         // contraction steps of 16 that hold them
  int steps;      // steps the kernel runs (KS rounded up to the unroll; the table is zero there)
  int nct;        // bin tiles of 32
  int pitch;      // LDS row pitch of an operand piece, in 16-byte units (odd)
  float inv_B;
};

// One step's right-hand pieces of a wavefront.
struct Tw {
  halfx8 ch, cl, sh, sl;
};

// One step's left-hand pieces: folded sums (for the cosine) hi / lo, folded differences (for the sine) hi / lo.
struct Left {
  halfx8 sh, sl, dh, dl;
};

__device__ inline void load_tw(Tw& w, const halfx8* p) {
  w.ch = p[0];
  w.cl = p[64];
  w.sh = p[128];
  w.sl = p[192];
}

// Maximum or minimum of an integer over the 64 lanes, returned to all of them: four shifts inside the
// rows of 16 lanes, then the last lane of a row is passed on to the next row, then to the upper half;
// lane 63 ends up with the result.  Lanes that a step does not reach keep their own value.
template <bool MAX>
__device__ inline int wave_reduce(int v) {
#define KDFH_RED(CTRL, ROWS)                                                      \
  {                                                                               \
    const int t = __builtin_amdgcn_update_dpp(v, v, CTRL, ROWS, 0xF, false);      \
    v = MAX ? max(v, t) : min(v, t);                                              \
  }
  KDFH_RED(0x111, 0xF)   // row_shr:1
  KDFH_RED(0x112, 0xF)   // row_shr:2
  KDFH_RED(0x114, 0xF)   // row_shr:4
  KDFH_RED(0x118, 0xF)   // row_shr:8
  KDFH_RED(0x142, 0xA)   // row_bcast:15 into rows 1 and 3
  KDFH_RED(0x143, 0xC)   // row_bcast:31 into rows 2 and 3
#undef KDFH_RED
  return __builtin_amdgcn_readlane(v, 63);
}

// VEC: rows can be read as aligned float4 (L and the strides multiples of 4, aligned base).
// R2: radix-2 step before the fold (needs VEC, L a multiple of 8 and at least 64).
// ITEMS: 8-sample items a thread reads per row block; RING: contraction steps whose table pieces are in
// flight (2 for the short-window instance, which has to stay inside 128 registers).
// WPE: wavefronts per SIMD the register budget is set for.  The short-window instances (ITEMS = 1) take four: at
// 862 variates of 32 windows the grid is 3448 wavefronts, which only then are all resident at once (3 per SIMD
// leave 376 of them waiting for a second round: 14.9 us instead of 11.7).  (Three for ITEMS = 2, which the LDS
// would hold at L = 336, costs spills and was slower.)
// STRAY: the instance that also contracts stray bins (R2 only).
template <int ITEMS, int RING, bool VEC, bool R2, bool STRAY = false, int WPE = (ITEMS == 1 ? 4 : (ITEMS <= 4 ? 2 : 1))>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(WPE))) void kdfh_kernel(KdfhArgs a) {
  extern __shared__ halfx8 lds8[];
  const int L = a.L, F = a.F, T = a.T;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, half = lane >> 5;
  const int rpv = 1 << a.log2_rpv;
  const int Vb = 32 >> a.log2_rpv;               // variates per block
  const int n0 = blockIdx.x * Vb;
  const int KG = 2 * a.KS;                       // groups of 8 folded samples per row
  const int pitch = a.pitch;
  // [4][32][pitch]: cosine operand hi, lo, sine operand hi, lo; with R2 a second set of four for the odd bins
  halfx8* opnd = lds8;
  unsigned* rowmax = reinterpret_cast<unsigned*>(opnd + (R2 ? 8 : 4) * 32 * pitch);   // [32] bits of the largest |x| of a row
  float* rowinv = reinterpret_cast<float*>(rowmax + 32);                   // [32] 1 / scale of a row
  float* xn1 = rowinv + 32;      // [32] scaled middle term of the cosine sum: x[L/2] (0 when L is odd); R2: u[L/4], even bins
  float* xn2 = xn1 + 32;         // [32] R2: scaled middle term of the sine sum, v[L/4], odd bins
  float* samp = xn2 + 32;        // [kMaxStray][32] amplitudes of the stray bins, per row
  float* asum = samp + kMaxStray * 32;                                     // [Vb][F]

  for (int i = tid; i < Vb * F; i += kThreads) asum[i] = 0.f;
  const bool even = (L & 1) == 0;
  // which wavefront takes the odd bin tile out rotates with the block, so that the blocks that share a
  // compute unit do not all load the same one of its four matrix pipelines
  const int rot = (blockIdx.x + (blockIdx.x >> 8)) & (kWaves - 1);
  const int ct0 = (wave + rot) & (kWaves - 1);                       // first bin tile of this wavefront
  const int nt = ct0 < a.nct ? (a.nct - ct0 + kWaves - 1) / kWaves : 0;   // and how many it takes
  Tw w0, w1, w2, w3;                                                 // right-hand pieces in flight (w2, w3: RING = 4)
  const int ctp = min(ct0, a.nct - 1);                               // (a wavefront without a tile loads one all the same)

  for (int rb = 0; rb < a.nrb; ++rb) {
    __syncthreads();                             // the operands of the previous block have been used
    if (tid < 32) rowmax[tid] = 0u;
    // In the short-window instances the item coordinates and row addresses below are formed from an opaque copy
    // of the thread index, so that they are computed here and not ahead of the loop: hoisted, they would live
    // across it (most launches run it once) and cost registers these instances do not have (they spilled).  The
    // long-window instances have the registers and are faster with the addresses ready.
    int tl = tid;
    if constexpr (ITEMS == 1) asm volatile("" : "+v"(tl));
    // the first steps of the wavefront's first bin tile are requested before the windows are when
    // the windows leave the registers for it (short windows), else right before the contraction
    constexpr bool kEarly = false;
#define KDFH_PRIME()                                        \
  {                                                         \
    const halfx8* tb = a.tw + (size_t)ctp * 256 + lane;     \
    const size_t sstride = (size_t)a.nct * 256;             \
    load_tw(w0, tb);                                        \
    load_tw(w1, tb + sstride);                              \
    if (RING == 4) {                                        \
      load_tw(w2, tb + 2 * sstride);                        \
      load_tw(w3, tb + 3 * sstride);                        \
    }                                                       \
  }
    if (kEarly) KDFH_PRIME()
    __syncthreads();

    if constexpr (R2) {
      // ---- read, radix-2: item (r, g) = samples t = 8g .. 8g+7 of row r, the ones half a window later, and
      // the mirror images M - t and L - t (M = L/2); all loads unconditional and in bounds for L >= 64
      const int M = L >> 1;
      float xa[ITEMS][8], xb[ITEMS][8], xc[ITEMS][8], xd[ITEMS][8];
      int ir[ITEMS], ig[ITEMS];
      float n1 = 0.f, n2 = 0.f;                    // x[L/4] and x[3L/4] of row tid (threads 0..31)
      {
        int row = tid;
        asm volatile("" : "+v"(row));              // (keeps this address out of the registers that live across the loop)
        const int nn = n0 + (row >> a.log2_rpv), bb = rb * 32 + (row & (rpv - 1));
        if (tid < 32 && nn < a.N && bb < a.B) {
          const float* p = a.x + (long long)bb * a.sb + (long long)nn * a.sn;
          n1 = p[T];
          n2 = p[T + M];
        }
      }
#pragma unroll
      for (int it = 0; it < ITEMS; ++it) {
        const int i = min(it * kThreads + tl, 32 * KG - 1);    // (a thread past the last item repeats it and stores nothing)
        const int r = i / KG;
        const int g = i - r * KG;
        ir[it] = r;
        ig[it] = g;
        const int t0 = 8 * g;
        const int nn = n0 + (r >> a.log2_rpv), bb = rb * 32 + (r & (rpv - 1));
        const float* p = a.x + (long long)min(bb, a.B - 1) * a.sb + (long long)min(nn, a.N - 1) * a.sn;
        const float4* pa4 = reinterpret_cast<const float4*>(p + t0);
        const float4* pb4 = reinterpret_cast<const float4*>(p + M + t0);
        const float4* pc4 = reinterpret_cast<const float4*>(p + (M - 8 - t0));     // x[M - t0 - 8 .. M - t0 - 1]
        const float4* pd4 = reinterpret_cast<const float4*>(p + (L - 8 - t0));     // x[L - t0 - 8 .. L - t0 - 1]
        const float4 a0 = pa4[0], a1 = pa4[1], b0 = pb4[0], b1 = pb4[1];
        const float4 c0 = pc4[0], c1 = pc4[1], d0 = pd4[0], d1 = pd4[1];
        xc[it][0] = p[M - t0];
        xd[it][0] = p[min(L - t0, L - 1)];         // (t = 0 has no mirror image)
        xa[it][0] = a0.x; xa[it][1] = a0.y; xa[it][2] = a0.z; xa[it][3] = a0.w;
        xa[it][4] = a1.x; xa[it][5] = a1.y; xa[it][6] = a1.z; xa[it][7] = a1.w;
        xb[it][0] = b0.x; xb[it][1] = b0.y; xb[it][2] = b0.z; xb[it][3] = b0.w;
        xb[it][4] = b1.x; xb[it][5] = b1.y; xb[it][6] = b1.z; xb[it][7] = b1.w;
        xc[it][1] = c1.w; xc[it][2] = c1.z; xc[it][3] = c1.y; xc[it][4] = c1.x;
        xc[it][5] = c0.w; xc[it][6] = c0.z; xc[it][7] = c0.y;
        xd[it][1] = d1.w; xd[it][2] = d1.z; xd[it][3] = d1.y; xd[it][4] = d1.x;
        xd[it][5] = d0.w; xd[it][6] = d0.z; xd[it][7] = d0.y;
      }
      // ---- zero what lies outside the fold or the input; largest magnitude of every row; the four folded
      // sequences replace the samples: cosine / sine operand of the even bins, then of the odd bins
#pragma unroll
      for (int it = 0; it < ITEMS; ++it) {
        const int r = ir[it], t0 = 8 * ig[it];
        const int nn = n0 + (r >> a.log2_rpv), bb = rb * 32 + (r & (rpv - 1));
        const bool ok = nn < a.N && bb < a.B;                  // rows past the end are zero windows
        float mx = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int t = t0 + j;
          const bool vd = ok && t < T, vm = vd && t >= 1;
          const float xa_ = vd ? xa[it][j] : 0.f, xb_ = vd ? xb[it][j] : 0.f;
          const float xc_ = vm ? xc[it][j] : 0.f, xd_ = vm ? xd[it][j] : 0.f;
          mx = fmaxf(fmaxf(mx, fmaxf(fabsf(xa_), fabsf(xb_))), fmaxf(fabsf(xc_), fabsf(xd_)));
          const float u = xa_ + xb_, v = xa_ - xb_, um = xc_ + xd_, vm_ = xc_ - xd_;
          xa[it][j] = u + um;                      // even bins, cosine
          xb[it][j] = vm ? u - um : 0.f;           // even bins, sine
          xc[it][j] = v - vm_;                     // odd bins, cosine
          xd[it][j] = vm ? v + vm_ : 0.f;          // odd bins, sine
        }
        atomicMax(&rowmax[r], __float_as_uint(mx));
      }
      if (tid < 32) atomicMax(&rowmax[tid], __float_as_uint(fmaxf(fabsf(n1), fabsf(n2))));
      __syncthreads();

      // ---- scale by a power of two (the folded values are sums of four samples: below 2^15), split, store
      if (tid < 32) {
        const int se = min(max(266 - (int)(rowmax[tid] >> 23), 1), 253);
        const float sc = __uint_as_float((unsigned)se << 23);
        rowinv[tid] = __uint_as_float((unsigned)(254 - se) << 23);
        xn1[tid] = (n1 + n2) * sc;
        xn2[tid] = (n1 - n2) * sc;
      }
#pragma unroll
      for (int it = 0; it < ITEMS; ++it) {
        const int r = ir[it], g = ig[it];
        const int se = min(max(266 - (int)(rowmax[r] >> 23), 1), 253);
        const float sc = __uint_as_float((unsigned)se << 23);
        float s0[8], s1[8], s2[8], s3[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          s0[j] = xa[it][j] * sc;
          s1[j] = xb[it][j] * sc;
          s2[j] = xc[it][j] * sc;
          s3[j] = xd[it][j] * sc;
        }
        Pieces p0, p1, p2, p3;
        split8(s0, p0);
        split8(s1, p1);
        split8(s2, p2);
        split8(s3, p3);
        if (it * kThreads + tid < 32 * KG) {
          halfx8* q = opnd + r * pitch + g;
          q[0] = p0.hi;
          q[32 * pitch] = p0.lo;
          q[64 * pitch] = p1.hi;
          q[96 * pitch] = p1.lo;
          q[128 * pitch] = p2.hi;
          q[160 * pitch] = p2.lo;
          q[192 * pitch] = p3.hi;
          q[224 * pitch] = p3.lo;
        }
      }
    } else {
    // ---- read: item (r, g) = samples t = 8g .. 8g+7 of row r and their mirror images L - t.  Every load is
    // unconditional (addresses are clamped into the row, rows into the input) and issued before any is used.
    float dv[ITEMS][8], mv[ITEMS][8];
    int ir[ITEMS], ig[ITEMS];
    float nyv = 0.f;                               // x[L/2] of row tid (threads 0..31, even L)
    {
      int row = tid;
      asm volatile("" : "+v"(row));                // (keeps this address out of the registers that live across the loop)
      const int nn = n0 + (row >> a.log2_rpv), bb = rb * 32 + (row & (rpv - 1));
      if (tid < 32 && even && nn < a.N && bb < a.B) nyv = a.x[(long long)bb * a.sb + (long long)nn * a.sn + (L >> 1)];
    }
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
      const int i = min(it * kThreads + tl, 32 * KG - 1);    // (a thread past the last item repeats it and stores nothing)
      const int r = i / KG;
      const int g = i - r * KG;
      ir[it] = r;
      ig[it] = g;
      const int t0 = 8 * g;
      const int nn = n0 + (r >> a.log2_rpv), bb = rb * 32 + (r & (rpv - 1));
      const float* p = a.x + (long long)min(bb, a.B - 1) * a.sb + (long long)min(nn, a.N - 1) * a.sn;
      if (VEC) {
        // L is a multiple of 4 and at least 8 here.  The mirror images x[L - t0 - 7 .. L - t0] are the aligned
        // float4 at L - t0 - 8 (its last three samples), the one at L - t0 - 4 and one more sample.  An item that
        // starts past L - 8 reads the row's last 8 samples instead: none of its samples is inside the fold.
        const int tc = min(t0, L - 8);
        const float4* pd = reinterpret_cast<const float4*>(p + tc);
        const float4* pm = reinterpret_cast<const float4*>(p + (L - 8 - tc));
        const float4 u0 = pd[0], u1 = pd[1], ua = pm[0], ub = pm[1];
        mv[it][0] = p[min(L - tc, L - 1)];
        dv[it][0] = u0.x; dv[it][1] = u0.y; dv[it][2] = u0.z; dv[it][3] = u0.w;
        dv[it][4] = u1.x; dv[it][5] = u1.y; dv[it][6] = u1.z; dv[it][7] = u1.w;
        mv[it][1] = ub.w; mv[it][2] = ub.z; mv[it][3] = ub.y; mv[it][4] = ub.x;
        mv[it][5] = ua.w; mv[it][6] = ua.z; mv[it][7] = ua.y;
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          dv[it][j] = p[min(t0 + j, L - 1)];
          mv[it][j] = p[min(max(L - t0 - j, 0), L - 1)];
        }
      }
    }
    // ---- zero what lies outside the window or the input; largest magnitude of every row
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
      const int r = ir[it], t0 = 8 * ig[it];
      const int nn = n0 + (r >> a.log2_rpv), bb = rb * 32 + (r & (rpv - 1));
      const bool ok = nn < a.N && bb < a.B;                  // rows past the end are zero windows
      float mx = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int t = t0 + j;
        dv[it][j] = (ok && t < T) ? dv[it][j] : 0.f;
        mv[it][j] = (ok && t >= 1 && t < T) ? mv[it][j] : 0.f;
        mx = fmaxf(mx, fmaxf(fabsf(dv[it][j]), fabsf(mv[it][j])));
      }
      atomicMax(&rowmax[r], __float_as_uint(mx));
    }
    if (tid < 32) atomicMax(&rowmax[tid], __float_as_uint(fabsf(nyv)));
    __syncthreads();

    // ---- scale by a power of two, fold, split, store the operand pieces
    if (tid < 32) {
      const int se = min(max(266 - (int)(rowmax[tid] >> 23), 1), 253);
      rowinv[tid] = __uint_as_float((unsigned)(254 - se) << 23);
      xn1[tid] = nyv * __uint_as_float((unsigned)se << 23);
      xn2[tid] = 0.f;
    }
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
      const int r = ir[it], g = ig[it];
      const int e = (int)(rowmax[r] >> 23);                  // biased exponent of the row's largest magnitude
      const int se = min(max(266 - e, 1), 253);              // scale = 2^(12 - (e - 127)), clamped to normal numbers
      const float sc = __uint_as_float((unsigned)se << 23);
      float sum[8], dif[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int t = 8 * g + j;
        const float d = dv[it][j] * sc, m = mv[it][j] * sc;
        sum[j] = d + m;
        dif[j] = (t >= 1 && t < T) ? d - m : 0.f;
      }
      Pieces ps, pd;
      split8(sum, ps);
      split8(dif, pd);
      if (it * kThreads + tid < 32 * KG) {
        halfx8* q = opnd + r * pitch + g;
        q[0] = ps.hi;
        q[32 * pitch] = ps.lo;
        q[64 * pitch] = pd.hi;
        q[96 * pitch] = pd.lo;
      }
    }
    }
    if (!kEarly) KDFH_PRIME()
#undef KDFH_PRIME
    __syncthreads();

    // ---- spectrum of the 32 rows; a wavefront takes 32 bins at a time.
    // Operand layout of v_mfma_f32_32x32x16_f16: left lane holds row lane % 32, k = 8 (lane / 32) + 0..7;
    // right lane holds column lane % 32, the same k; result lane holds column lane % 32, register r holds
    // row 8 (r / 4) + 4 (lane / 32) + r % 4.
    Left la, lb;
    for (int ti = 0; ti < nt; ++ti) {
      const int ct = ct0 + kWaves * ti;
      floatx16 re = {}, im = {};
      // left operands of this tile and of the wavefront's next one (even and odd bins have sets of their own)
      const halfx8* pa = opnd + ((R2 && ct >= a.bins.nct_e) ? 128 * pitch : 0) + col * pitch;
      const halfx8* pn = opnd + ((R2 && ct + kWaves >= a.bins.nct_e) ? 128 * pitch : 0) + col * pitch;
      const halfx8 lo_unscale = {(_Float16)kLoUnscale, (_Float16)kLoUnscale, (_Float16)kLoUnscale, (_Float16)kLoUnscale,
                                 (_Float16)kLoUnscale, (_Float16)kLoUnscale, (_Float16)kLoUnscale, (_Float16)kLoUnscale};
      // the pieces of step S + RING replace those of step S; past the tile's last step they are the first of
      // the wavefront's next tile (of its last step again when there is none: loaded, never used)
      // With RING = 4 the left pieces of step S + 1 are read from LDS while the matrix instructions of step S run
      // (the first step of the next tile after the last).
#define KDFH_READ_LEFT(A, S)                                                              \
  {                                                                                       \
    const bool nx = (S) >= a.steps;           /* first step of the wavefront's next tile */ \
    const halfx8* pl = nx ? pn : pa;                                                      \
    const int g = min(2 * (nx ? 0 : (S)) + half, KG - 1); /* steps past KS: the table is zero there */ \
    A.sh = pl[g];                                                                         \
    A.sl = pl[32 * pitch + g];                                                            \
    A.dh = pl[64 * pitch + g];                                                            \
    A.dl = pl[96 * pitch + g];                                                            \
  }
#define KDFH_STEP(W, A, AN, S)                                                            \
  {                                                                                       \
    if (RING == 4) KDFH_READ_LEFT(AN, (S) + 1) else KDFH_READ_LEFT(A, S)                  \
    const halfx8 shs = A.sh * lo_unscale, dhs = A.dh * lo_unscale;                        \
    __builtin_amdgcn_sched_barrier(0);                                                    \
    re = __builtin_amdgcn_mfma_f32_32x32x16_f16(A.sh, W.ch, re, 0, 0, 0);                 \
    im = __builtin_amdgcn_mfma_f32_32x32x16_f16(A.dh, W.sh, im, 0, 0, 0);                 \
    re = __builtin_amdgcn_mfma_f32_32x32x16_f16(shs, W.cl, re, 0, 0, 0);                  \
    im = __builtin_amdgcn_mfma_f32_32x32x16_f16(dhs, W.sl, im, 0, 0, 0);                  \
    re = __builtin_amdgcn_mfma_f32_32x32x16_f16(A.sl, W.ch, re, 0, 0, 0);                 \
    im = __builtin_amdgcn_mfma_f32_32x32x16_f16(A.dl, W.sh, im, 0, 0, 0);                 \
    __builtin_amdgcn_sched_barrier(0);                                                    \
    {                                                                                     \
      const bool wrap = (S) + RING >= a.steps;                                            \
      const int s2 = wrap ? (ti + 1 < nt ? (S) + RING - a.steps : a.steps - 1) : (S) + RING; \
      const int c2 = (wrap && ti + 1 < nt) ? ct + kWaves : ct;                            \
      load_tw(W, a.tw + ((size_t)s2 * a.nct + c2) * 256 + lane);                          \
    }                                                                                     \
    __builtin_amdgcn_sched_barrier(0);                                                    \
  }
      if (RING == 4 && ti == 0) KDFH_READ_LEFT(la, 0)
      for (int s = 0; s < a.steps; s += 4) {
        if (RING == 4) {
          KDFH_STEP(w0, la, lb, s)
          KDFH_STEP(w1, lb, la, s + 1)
          KDFH_STEP(w2, la, lb, s + 2)
          KDFH_STEP(w3, lb, la, s + 3)
        } else {
          KDFH_STEP(w0, la, lb, s)
          KDFH_STEP(w1, lb, la, s + 1)
          KDFH_STEP(w0, la, lb, s + 2)
          KDFH_STEP(w1, lb, la, s + 3)
        }
      }
#undef KDFH_READ_LEFT
#undef KDFH_STEP

      // ---- amplitudes, scaled back, and the batch sums (Alg. 1 step 3) of this bin tile
      const int f = bin_of(a.bins, ct, col);
      const int c = f - a.f_min;                   // index of this lane's bin among the candidates
      // middle terms of the two sums: plain (-1)^f x[L/2] in the cosine sum; radix-2 (-1)^(f/2) u[L/4] in the
      // cosine sum of an even bin, sin(pi f / 2) v[L/4] in the sine sum of an odd one
      float cr, ci;
      if (!R2) {
        cr = (f & 1) ? -1.f : 1.f;
        ci = 0.f;
      } else if (ct < a.bins.nct_e) {
        cr = (f & 2) ? -1.f : 1.f;
        ci = 0.f;
      } else {
        cr = 0.f;
        ci = (f & 2) ? -1.f : 1.f;
      }
      float amp[16];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 inv4 = *reinterpret_cast<const float4*>(rowinv + 8 * q + 4 * half);
        const float4 m14 = *reinterpret_cast<const float4*>(xn1 + 8 * q + 4 * half);
        const float4 m24 = *reinterpret_cast<const float4*>(xn2 + 8 * q + 4 * half);
        const float inv[4] = {inv4.x, inv4.y, inv4.z, inv4.w};
        const float m1[4] = {m14.x, m14.y, m14.z, m14.w};
        const float m2[4] = {m24.x, m24.y, m24.z, m24.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int r = 4 * q + e;
          const float rv = re[r] + cr * m1[e];
          const float iv = im[r] + ci * m2[e];
          amp[r] = sqrtf(rv * rv + iv * iv) * inv[e];
        }
      }
      float qs[4];                                 // rows 8q + 4 half + 0..3
#pragma unroll
      for (int q = 0; q < 4; ++q) qs[q] = (amp[4 * q] + amp[4 * q + 1]) + (amp[4 * q + 2] + amp[4 * q + 3]);
      const bool live = c < F;                     // (bins step by 2 with R2, so the tile's last columns may lie past f_max)
      if (a.log2_rpv >= 3) {
        // a variate spans 8, 16 or 32 rows: both lane halves hold four rows of every 8
        float vs[4];
        if (a.log2_rpv == 3) {
          vs[0] = qs[0]; vs[1] = qs[1]; vs[2] = qs[2]; vs[3] = qs[3];
        } else if (a.log2_rpv == 4) {
          vs[0] = qs[0] + qs[1]; vs[1] = qs[2] + qs[3]; vs[2] = 0.f; vs[3] = 0.f;
        } else {
          vs[0] = (qs[0] + qs[1]) + (qs[2] + qs[3]); vs[1] = 0.f; vs[2] = 0.f; vs[3] = 0.f;
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const float tot = vs[v] + __shfl_xor(vs[v], 32, 64);
          if (live && half == 0 && v < Vb) asum[v * F + c] += tot;
        }
      } else if (a.log2_rpv == 2) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (live) asum[(2 * q + half) * F + c] += qs[q];
      } else if (a.log2_rpv == 1) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (live) {
            asum[(4 * q + 2 * half) * F + c] += amp[4 * q] + amp[4 * q + 1];
            asum[(4 * q + 2 * half + 1) * F + c] += amp[4 * q + 2] + amp[4 * q + 3];
          }
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (live) asum[(8 * (r >> 2) + 4 * half + (r & 3)) * F + c] += amp[r];
      }
    }

    // ---- stray bins on the vector units: eight threads per row share the folded samples (operand pieces added
    // back together), then one thread per (bin, variate) adds the rows of the variate in ascending order
    if constexpr (R2 && STRAY) {
      {
        const int r = tid >> 3, part = tid & 7;
        const int Tp = 8 * KG;
        for (int si = 0; si < a.bins.n_stray; ++si) {
          const int f = a.bins.stray_f[si];
          const halfx8* base = opnd + ((f & 1) ? 128 * pitch : 0) + r * pitch;
          const float4* tw4 = reinterpret_cast<const float4*>(a.stw + (size_t)si * Tp * 2);
          float re = 0.f, im = 0.f;
          for (int g = part; g < KG; g += 8) {
            const halfx8 ch = base[g], cl = base[32 * pitch + g], sh = base[64 * pitch + g], sl = base[96 * pitch + g];
#pragma unroll
            for (int j2 = 0; j2 < 4; ++j2) {
              const float4 w = tw4[4 * g + j2];            // cos, sin of t = 8 g + 2 j2 and of the next sample
              re = fmaf((float)ch[2 * j2] + (float)cl[2 * j2], w.x, re);
              im = fmaf((float)sh[2 * j2] + (float)sl[2 * j2], w.y, im);
              re = fmaf((float)ch[2 * j2 + 1] + (float)cl[2 * j2 + 1], w.z, re);
              im = fmaf((float)sh[2 * j2 + 1] + (float)sl[2 * j2 + 1], w.w, im);
            }
          }
#pragma unroll
          for (int o = 1; o <= 4; o <<= 1) {
            re += __shfl_xor(re, o, 64);
            im += __shfl_xor(im, o, 64);
          }
          if (part == 0) {
            const float sg = (f & 2) ? -1.f : 1.f;           // (-1)^(f/2) for an even bin, sin(pi f / 2) for an odd one
            const float rv = (f & 1) ? re : re + sg * xn1[r];
            const float iv = (f & 1) ? im + sg * xn2[r] : im;
            samp[si * 32 + r] = sqrtf(rv * rv + iv * iv) * rowinv[r];
          }
        }
        __syncthreads();
        for (int i = tid; i < a.bins.n_stray * Vb; i += kThreads) {
          const int si = i / Vb, v = i - si * Vb;
          float tot = 0.f;
          for (int rr = 0; rr < rpv; ++rr) tot += samp[si * 32 + v * rpv + rr];
          asum[v * F + (a.bins.stray_f[si] - a.f_min)] += tot;
        }
      }
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
    } else {
      // k rounds of a wavefront-wide arg-max.  Mean amplitudes are not negative, so their bit patterns order
      // like signed integers (the -2 of a used or absent bin is below all of them).
      for (int r = 0; r < a.k; ++r) {
        int best = (int)0x80000000;
#pragma unroll
        for (int j = 0; j < kMaxBinsPerLane; ++j) best = max(best, __float_as_int(vals[j]));
        const int top = wave_reduce<true>(best);
        int bi = 0x7fffffff;
#pragma unroll
        for (int j = kMaxBinsPerLane - 1; j >= 0; --j)
          if (__float_as_int(vals[j]) == top) bi = lane + 64 * j;
        bi = wave_reduce<false>(bi);                       // the lowest bin that holds it
#pragma unroll
        for (int j = 0; j < kMaxBinsPerLane; ++j)
          if (bi == lane + 64 * j) vals[j] = -2.f;
        const int fsel = a.f_min + bi;
        if (lane == 0) a.topk[(long long)n * a.k + r] = fsel;
        h = h * R + (unsigned long long)(unsigned)fsel;
      }
    }
    if (lane == 0) a.hash[n] = h;
    if (a.abar)
      for (int idx = lane; idx < F; idx += 64) a.abar[(long long)n * F + idx] = asum[v * F + idx] * a.inv_B;
  }
}


// ================================================================== pipelined variant
// The same computation for inputs whose rows can be read as aligned float4 (VEC), arranged so that the memory
// reads, the vector work (fold, scale, split) and the matrix work of different row blocks overlap instead of
// following each other.  A workgroup of eight wavefronts is persistent: it walks over variate groups
// g = blockIdx.x, blockIdx.x + gridDim.x, ... and their row blocks.  Wavefronts 0-3 are producers: each owns 8 of
// the 32 rows of a block, requests the rows of block t + 2 from memory while it folds, scales and splits block t + 1
// into one of two LDS operand buffers (the row maximum is an LDS exchange inside the wavefront: no workgroup
// barrier), and ranks the top-k of the group that block t - 1 completed.  Wavefronts 4-7 are consumers: they contract
// block t from the other buffer on the matrix cores and add the amplitudes to the batch sums.  One workgroup barrier
// per block hands the buffers over.
constexpr int kPipeThreads = 512;

template <int IW, bool R2>
struct RawRows {
  float a[IW][8], b[IW][8];                       // samples t0 .. t0+7 and (R2) the ones half a window later
  float c[IW][8], d[IW][8];                       // mirror images (plain: c only)
  float n1, n2;                                   // middle samples of the row of lanes 0..7
};

// requests the samples of this lane's items of row block (n0, rb): rows 8 pw .. 8 pw + 7 of the block
template <int IW, bool R2>
__device__ __forceinline__ void pipe_load(RawRows<IW, R2>& w, const KdfhArgs& a, int n0, int rb, int pw, int lane) {
  const int L = a.L, T = a.T, KG = 2 * a.KS, rpv = 1 << a.log2_rpv;
  const int M = L >> 1;
  w.n1 = 0.f;
  w.n2 = 0.f;
  if (lane < 8) {
    const int r = 8 * pw + lane;
    const int nn = n0 + (r >> a.log2_rpv), bb = rb * 32 + (r & (rpv - 1));
    if (nn < a.N && bb < a.B) {
      const float* p = a.x + (long long)bb * a.sb + (long long)nn * a.sn;
      if (R2) {
        w.n1 = p[T];
        w.n2 = p[T + M];
      } else if ((L & 1) == 0) {
        w.n1 = p[M];
      }
    }
  }
#pragma unroll
  for (int it = 0; it < IW; ++it) {
    const int i = min(it * 64 + lane, 8 * KG - 1);      // (a lane past the last item repeats it and stores nothing)
    const int rl = i / KG;
    const int g = i - rl * KG;
    const int r = 8 * pw + rl;
    const int t0 = 8 * g;
    const int nn = n0 + (r >> a.log2_rpv), bb = rb * 32 + (r & (rpv - 1));
    const float* p = a.x + (long long)min(bb, a.B - 1) * a.sb + (long long)min(nn, a.N - 1) * a.sn;
    if constexpr (R2) {
      const float4* pa4 = reinterpret_cast<const float4*>(p + t0);
      const float4* pb4 = reinterpret_cast<const float4*>(p + M + t0);
      const float4* pc4 = reinterpret_cast<const float4*>(p + (M - 8 - t0));     // x[M - t0 - 8 .. M - t0 - 1]
      const float4* pd4 = reinterpret_cast<const float4*>(p + (L - 8 - t0));     // x[L - t0 - 8 .. L - t0 - 1]
      const float4 a0 = pa4[0], a1 = pa4[1], b0 = pb4[0], b1 = pb4[1];
      const float4 c0 = pc4[0], c1 = pc4[1], d0 = pd4[0], d1 = pd4[1];
      w.c[it][0] = p[M - t0];
      w.d[it][0] = p[min(L - t0, L - 1)];          // (t = 0 has no mirror image)
      w.a[it][0] = a0.x; w.a[it][1] = a0.y; w.a[it][2] = a0.z; w.a[it][3] = a0.w;
      w.a[it][4] = a1.x; w.a[it][5] = a1.y; w.a[it][6] = a1.z; w.a[it][7] = a1.w;
      w.b[it][0] = b0.x; w.b[it][1] = b0.y; w.b[it][2] = b0.z; w.b[it][3] = b0.w;
      w.b[it][4] = b1.x; w.b[it][5] = b1.y; w.b[it][6] = b1.z; w.b[it][7] = b1.w;
      w.c[it][1] = c1.w; w.c[it][2] = c1.z; w.c[it][3] = c1.y; w.c[it][4] = c1.x;
      w.c[it][5] = c0.w; w.c[it][6] = c0.z; w.c[it][7] = c0.y;
      w.d[it][1] = d1.w; w.d[it][2] = d1.z; w.d[it][3] = d1.y; w.d[it][4] = d1.x;
      w.d[it][5] = d0.w; w.d[it][6] = d0.z; w.d[it][7] = d0.y;
    } else {
      // mirror images x[L - t0 - 7 .. L - t0]: the aligned float4 at L - t0 - 8 (its last three samples), the one
      // at L - t0 - 4 and one more sample; an item that starts past L - 8 reads the row's last 8 samples instead
      // (none of its samples is inside the fold)
      const int tc = min(t0, L - 8);
      const float4* pd = reinterpret_cast<const float4*>(p + tc);
      const float4* pm = reinterpret_cast<const float4*>(p + (L - 8 - tc));
      const float4 u0 = pd[0], u1 = pd[1], ua = pm[0], ub = pm[1];
      w.c[it][0] = p[min(L - tc, L - 1)];
      w.a[it][0] = u0.x; w.a[it][1] = u0.y; w.a[it][2] = u0.z; w.a[it][3] = u0.w;
      w.a[it][4] = u1.x; w.a[it][5] = u1.y; w.a[it][6] = u1.z; w.a[it][7] = u1.w;
      w.c[it][1] = ub.w; w.c[it][2] = ub.z; w.c[it][3] = ub.y; w.c[it][4] = ub.x;
      w.c[it][5] = ua.w; w.c[it][6] = ua.z; w.c[it][7] = ua.y;
    }
  }
}

// LDS of the pipelined kernel: two operand buffers, two sets of per-block floats, then the producers' row maxima.
// (Accessors compute addresses from the set number: a struct of pointer arrays indexed at run time would live in
// private memory.)
struct PipeLds {
  halfx8* base;
  float* fbase;
  int opnd_elems;           // halfx8 elements of one operand buffer: (R2 ? 8 : 4) * 32 * pitch
  int set_floats;           // floats of one set: (3 + kMaxStray) * 32 + Vb * F
  __device__ halfx8* opnd(int b) const { return base + b * opnd_elems; }
  __device__ float* rowinv(int b) const { return fbase + b * set_floats; }                    // [32] 1 / scale of a row
  __device__ float* xn1(int b) const { return fbase + b * set_floats + 32; }                  // [32] middle term, cosine sum
  __device__ float* xn2(int b) const { return fbase + b * set_floats + 64; }                  // [32] middle term, sine sum (R2)
  __device__ float* samp(int b) const { return fbase + b * set_floats + 96; }                 // [kMaxStray][32] stray bins per row
  __device__ float* asum(int b) const { return fbase + b * set_floats + 96 + kMaxStray * 32; }   // [Vb][F] batch sums
  __device__ unsigned* rowmax() const { return reinterpret_cast<unsigned*>(fbase + 2 * set_floats); }   // [32]
  __device__ float* stw() const { return fbase + 2 * set_floats + 32; }    // [kMaxStray][2 Tp] cosine, sine of the stray bins (R2)
};
__host__ __device__ inline size_t pipe_lds_bytes(int pitch, int F, int Vb, bool r2) {
  const size_t opnd = (size_t)(r2 ? 8 : 4) * 32 * pitch * 16;
  return 2 * (opnd + sizeof(float) * ((3 + kMaxStray) * 32 + (size_t)Vb * F)) + 32 * sizeof(unsigned) +
         (r2 ? sizeof(float) * kMaxStray * 2 * 8 * (size_t)(pitch - 1) : 0);      // pitch = 2 KS | 1: Tp = 8 (pitch - 1)
}
__device__ inline PipeLds pipe_lds(halfx8* base, int pitch, int F, int Vb, bool r2) {
  PipeLds l;
  l.base = base;
  l.opnd_elems = (r2 ? 8 : 4) * 32 * pitch;
  l.fbase = reinterpret_cast<float*>(base + 2 * l.opnd_elems);
  l.set_floats = (3 + kMaxStray) * 32 + Vb * F;
  return l;
}

// folds, scales and splits the rows `w` holds into operand buffer `b`
template <int IW, bool R2>
__device__ __forceinline__ void pipe_produce(RawRows<IW, R2>& w, const KdfhArgs& a, const PipeLds& l, int b,
                                             int n0, int rb, int pw, int lane) {
  const int T = a.T, KG = 2 * a.KS, rpv = 1 << a.log2_rpv, pitch = a.pitch;
  // ---- largest magnitude of every row: the rows of this wavefront are its own, and LDS operations of one
  // wavefront take effect in program order, so the exchange needs no workgroup barrier
  unsigned* rowmax = l.rowmax();
  if (lane < 8) rowmax[8 * pw + lane] = __float_as_uint(fmaxf(fabsf(w.n1), fabsf(w.n2)));
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  // Samples at t >= T need no masking: the loads read samples of the same row (so the row maximum is unchanged)
  // and the table is zero there.  What does: rows past the end of the input are zero windows, and t = 0 has no
  // mirror image.
#pragma unroll
  for (int it = 0; it < IW; ++it) {
    const int i = min(it * 64 + lane, 8 * KG - 1);
    const int rl = i / KG, g = i - rl * KG, r = 8 * pw + rl;
    const int nn = n0 + (r >> a.log2_rpv), bb = rb * 32 + (r & (rpv - 1));
    const bool ok = nn < a.N && bb < a.B;
    if (__builtin_amdgcn_ballot_w64(!ok) != 0) {           // (uniform: only a group at the end of the input has such rows)
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        w.a[it][j] = ok ? w.a[it][j] : 0.f;
        w.c[it][j] = ok ? w.c[it][j] : 0.f;
        if (R2) {
          w.b[it][j] = ok ? w.b[it][j] : 0.f;
          w.d[it][j] = ok ? w.d[it][j] : 0.f;
        }
      }
    }
    if (g == 0) {
      w.c[it][0] = 0.f;
      if (R2) w.d[it][0] = 0.f;
    }
    float mx = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if constexpr (R2) {
        const float xa_ = w.a[it][j], xb_ = w.b[it][j], xc_ = w.c[it][j], xd_ = w.d[it][j];
        mx = fmaxf(fmaxf(mx, fmaxf(fabsf(xa_), fabsf(xb_))), fmaxf(fabsf(xc_), fabsf(xd_)));
        const float u = xa_ + xb_, v = xa_ - xb_, um = xc_ + xd_, vm_ = xc_ - xd_;
        w.a[it][j] = u + um;                      // even bins, cosine
        w.b[it][j] = u - um;                      // even bins, sine   (t = 0: times sin 0)
        w.c[it][j] = v - vm_;                     // odd bins, cosine
        w.d[it][j] = v + vm_;                     // odd bins, sine
      } else {
        const float d = w.a[it][j], m = w.c[it][j];
        mx = fmaxf(mx, fmaxf(fabsf(d), fabsf(m)));
        w.a[it][j] = d + m;                       // cosine operand
        w.c[it][j] = d - m;                       // sine operand   (t = 0: times sin 0)
      }
    }
    if (it * 64 + lane < 8 * KG) atomicMax(&rowmax[r], __float_as_uint(mx));
  }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  // ---- scale by a power of two that brings the row's largest magnitude to [2^12, 2^13) (the folded values are
  // sums of up to four samples: below 2^15), split, store
  if (lane < 8) {
    const int r = 8 * pw + lane;
    const int se = min(max(266 - (int)(rowmax[r] >> 23), 1), 253);
    const float sc = __uint_as_float((unsigned)se << 23);
    l.rowinv(b)[r] = __uint_as_float((unsigned)(254 - se) << 23);
    if (R2) {
      l.xn1(b)[r] = (w.n1 + w.n2) * sc;
      l.xn2(b)[r] = (w.n1 - w.n2) * sc;
    } else {
      l.xn1(b)[r] = w.n1 * sc;
      l.xn2(b)[r] = 0.f;
    }
  }
  halfx8* opnd = l.opnd(b);
#pragma unroll
  for (int it = 0; it < IW; ++it) {
    const int i = min(it * 64 + lane, 8 * KG - 1);
    const int rl = i / KG, g = i - rl * KG, r = 8 * pw + rl;
    const int se = min(max(266 - (int)(rowmax[r] >> 23), 1), 253);
    const float sc = __uint_as_float((unsigned)se << 23);
    float s0[8], s1[8], s2[8], s3[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      s0[j] = w.a[it][j] * sc;
      s1[j] = (R2 ? w.b[it][j] : w.c[it][j]) * sc;
      if (R2) {
        s2[j] = w.c[it][j] * sc;
        s3[j] = w.d[it][j] * sc;
      }
    }
    Pieces p0, p1, p2, p3;
    split8_trunc(s0, p0);
    split8_trunc(s1, p1);
    if (R2) {
      split8_trunc(s2, p2);
      split8_trunc(s3, p3);
    }
    if (it * 64 + lane < 8 * KG) {
      halfx8* q = opnd + r * pitch + g;
      q[0] = p0.hi;
      q[32 * pitch] = p0.lo;
      q[64 * pitch] = p1.hi;
      q[96 * pitch] = p1.lo;
      if (R2) {
        q[128 * pitch] = p2.hi;
        q[160 * pitch] = p2.lo;
        q[192 * pitch] = p3.hi;
        q[224 * pitch] = p3.lo;
      }
    }
  }
}

// ranked top-k and hash (Alg. 1 steps 4-5) of the variates v = cw, cw + 4, ... of a group, from its batch sums;
// (the stray bins' row amplitudes of the group's last block have been added by the caller)
__device__ __forceinline__ void pipe_rank(const KdfhArgs& a, float* asum, int n0, int cw, int lane) {
  const int F = a.F, Vb = 32 >> a.log2_rpv;
  const unsigned long long R = (unsigned long long)(a.L / 2 + 1);
  for (int v = cw; v < Vb; v += 4) {
    const int n = n0 + v;
    if (n < a.N) {
      const int nslot = (F + 63) >> 6;             // bin lane + 64 j lives in slot j: only these slots hold bins
      float vals[kMaxBinsPerLane];
#pragma unroll
      for (int j = 0; j < kMaxBinsPerLane; ++j) {
        const int idx = lane + 64 * j;
        vals[j] = (j < nslot && idx < F) ? asum[v * F + idx] : -2.f;
      }
      unsigned long long h = 0;
      if (F <= 64) {
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
      } else {
        // k rounds: the largest value by one wavefront reduction, then the lowest bin that holds it: bin lane + 64 j
        // grows with j before it grows with the lane, so it is the first set lane of the first non-empty ballot
        for (int r = 0; r < a.k; ++r) {
          int best = (int)0x80000000;
#pragma unroll
          for (int j = 0; j < kMaxBinsPerLane; ++j)
            if (j < nslot) best = max(best, __float_as_int(vals[j]));
          const int top = wave_reduce<true>(best);
          int bi = -1;
#pragma unroll
          for (int j = kMaxBinsPerLane - 1; j >= 0; --j)
            if (j < nslot) {
              const unsigned long long m = __ballot(__float_as_int(vals[j]) == top);
              if (m) bi = (__ffsll((long long)m) - 1) + 64 * j;
            }
#pragma unroll
          for (int j = 0; j < kMaxBinsPerLane; ++j)
            if (j < nslot && bi == lane + 64 * j) vals[j] = -2.f;
          const int fsel = a.f_min + bi;
          if (lane == 0) a.topk[(long long)n * a.k + r] = fsel;
          h = h * R + (unsigned long long)(unsigned)fsel;
        }
      }
      if (lane == 0) a.hash[n] = h;
      if (a.abar)
        for (int idx = lane; idx < F; idx += 64) a.abar[(long long)n * F + idx] = asum[v * F + idx] * a.inv_B;
    }
  }
}

// Workgroup barrier that orders LDS accesses only: outstanding global loads (the next block's rows, the table
// pieces) and stores (the previous group's results) stay in flight across it.
__device__ inline void pipe_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int IW, bool R2, bool STRAY, int WPE>
__global__ __launch_bounds__(kPipeThreads) __attribute__((amdgpu_waves_per_eu(WPE))) void kdfh_pipe_kernel(KdfhArgs a, int ngroups) {
  extern __shared__ halfx8 lds8[];
  const int F = a.F;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, half = lane >> 5;
  const int rpv = 1 << a.log2_rpv;
  const int Vb = 32 >> a.log2_rpv;               // variates per group
  const int KG = 2 * a.KS;
  const int pitch = a.pitch;
  const PipeLds l = pipe_lds(lds8, pitch, F, Vb, R2);
  if constexpr (R2 && STRAY)
    for (int i = tid; i < a.bins.n_stray * 2 * 8 * KG; i += kPipeThreads) l.stw()[i] = a.stw[i];
  // this workgroup's groups: blockIdx.x, blockIdx.x + gridDim.x, ...; block t of its sequence is row block
  // t % nrb of its group number t / nrb
  const int my_groups = ((int)blockIdx.x < ngroups) ? (ngroups - 1 - (int)blockIdx.x) / (int)gridDim.x + 1 : 0;
  const int nblk = my_groups * a.nrb;
  __syncthreads();
  // What block u leaves to do once every consumer is done with it (the producers do it, so that no store of results
  // sits in front of a consumer's table read): the wavefront's variates (v = w4, w4 + 4, ...) get
  // their stray bins' row amplitudes added to the batch sums, and, when u was the last row block of its group,
  // their ranked top-k and hash.
  auto post = [&](int u, int w4) {
    const int gq = u / a.nrb, rbp = u - gq * a.nrb;
    float* asum = l.asum(gq & 1);
    if constexpr (STRAY) {
      const float* samp = l.samp(u & 1);
      for (int v = w4; v < Vb; v += 4)
        if (lane < a.bins.n_stray) {
          float tot = 0.f;
          for (int rr = 0; rr < rpv; ++rr) tot += samp[lane * 32 + v * rpv + rr];
          float& dst = asum[v * F + (a.bins.stray_f[lane] - a.f_min)];
          dst = rbp == 0 ? tot : dst + tot;      // (the first row block of a group starts its sums)
        }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
    if (rbp == a.nrb - 1) pipe_rank(a, asum, ((int)blockIdx.x + gq * (int)gridDim.x) * Vb, w4, lane);
  };
  if (wave < 4) {
    // ================================================================ producers
    const int pw = wave;
    RawRows<IW, R2> w0, w1;
    if (nblk > 0) pipe_load(w0, a, (int)blockIdx.x * Vb, 0, pw, lane);
#define KDFH_PRODUCE(CUR, NXT, T_)                                                                        \
  {                                                                                                      \
    const int t_ = (T_);                                                                                 \
    if (t_ + 1 < nblk) {                                                                                 \
      const int gq = (t_ + 1) / a.nrb;                                                                   \
      pipe_load(NXT, a, ((int)blockIdx.x + gq * (int)gridDim.x) * Vb, (t_ + 1) - gq * a.nrb, pw, lane);  \
    }                                                                                                    \
    if (t_ >= 2) post(t_ - 2, pw);                   /* (the consumers finished block t_ - 2 before the last barrier) */ \
    const int gq0 = t_ / a.nrb;                                                                          \
    pipe_produce(CUR, a, l, t_ & 1, ((int)blockIdx.x + gq0 * (int)gridDim.x) * Vb, t_ - gq0 * a.nrb, pw, lane); \
    pipe_barrier();                       /* block t_ is ready; the consumers are done with block t_ - 1 */ \
  }
    for (int t = 0; t < nblk; t += 2) {
      KDFH_PRODUCE(w0, w1, t)
      if (t + 1 < nblk) KDFH_PRODUCE(w1, w0, t + 1)
    }
#undef KDFH_PRODUCE
    if (nblk >= 2) post(nblk - 2, pw);
    pipe_barrier();                       // the consumers are done with the last block
    if (nblk >= 1) post(nblk - 1, pw);
    return;
  }
  // ================================================================== consumers
  const int cw = wave - 4;
  const int rot = (blockIdx.x + (blockIdx.x >> 8)) & 3;
  const int ct0 = (cw + rot) & 3;                                    // first bin tile of this wavefront
  const int nt = ct0 < a.nct ? (a.nct - ct0 + 3) / 4 : 0;            // and how many it takes
  const int ctp = min(ct0, a.nct - 1);                               // (a wavefront without a tile loads one all the same)
  Tw w0, w1, w2, w3;
  for (int t = 0; t <= nblk; ++t) {
    pipe_barrier();                       // block t is ready (t < nblk); every consumer is done with block t - 1
    if (t == nblk) break;
    const int b = t & 1, gq = t / a.nrb;
    const halfx8* opnd = l.opnd(b);
    float* asum = l.asum(gq & 1);
    // the first row block of a group starts its batch sums (a plain store: no read in front of it), later ones add
    const bool first_rb = t - gq * a.nrb == 0;
    auto acc = [&](float& dst, float v) { dst = first_rb ? v : dst + v; };
    const float* rowinv = l.rowinv(b);
    const float* xn1 = l.xn1(b);
    const float* xn2 = l.xn2(b);
    // the table pieces of the wavefront's first tile are requested once; from then on the last steps of a block
    // request those of the next block's first steps (the table does not depend on the block), so a block starts on
    // pieces that are already there
    if (t == 0) {
      const halfx8* tb = a.tw + (size_t)ctp * 256 + lane;
      const size_t sstride = (size_t)a.nct * 256;
      load_tw(w0, tb);
      load_tw(w1, tb + sstride);
      load_tw(w2, tb + 2 * sstride);
      load_tw(w3, tb + 3 * sstride);
    }
    Left la, lb;
    for (int ti = 0; ti < nt; ++ti) {
      const int ct = ct0 + 4 * ti;
      floatx16 re = {}, im = {};
      const halfx8* pa = opnd + ((R2 && ct >= a.bins.nct_e) ? 128 * pitch : 0) + col * pitch;
      const halfx8* pn = opnd + ((R2 && ct + 4 >= a.bins.nct_e) ? 128 * pitch : 0) + col * pitch;
      const halfx8 lo_unscale = {(_Float16)kLoUnscale, (_Float16)kLoUnscale, (_Float16)kLoUnscale, (_Float16)kLoUnscale,
                                 (_Float16)kLoUnscale, (_Float16)kLoUnscale, (_Float16)kLoUnscale, (_Float16)kLoUnscale};
#define KDFH_READ_LEFT(A, S)                                                              \
  {                                                                                       \
    const bool nx = (S) >= a.steps;           /* first step of the wavefront's next tile */ \
    const halfx8* pl = nx ? pn : pa;                                                      \
    const int g = min(2 * (nx ? 0 : (S)) + half, KG - 1); /* steps past KS: the table is zero there */ \
    A.sh = pl[g];                                                                         \
    A.sl = pl[32 * pitch + g];                                                            \
    A.dh = pl[64 * pitch + g];                                                            \
    A.dl = pl[96 * pitch + g];                                                            \
  }
#define KDFH_STEP(W, A, AN, S)                                                            \
  {                                                                                       \
    KDFH_READ_LEFT(AN, (S) + 1)                                                           \
    const halfx8 shs = A.sh * lo_unscale, dhs = A.dh * lo_unscale;                        \
    __builtin_amdgcn_sched_barrier(0);                                                    \
    re = __builtin_amdgcn_mfma_f32_32x32x16_f16(A.sh, W.ch, re, 0, 0, 0);                 \
    im = __builtin_amdgcn_mfma_f32_32x32x16_f16(A.dh, W.sh, im, 0, 0, 0);                 \
    re = __builtin_amdgcn_mfma_f32_32x32x16_f16(shs, W.cl, re, 0, 0, 0);                  \
    im = __builtin_amdgcn_mfma_f32_32x32x16_f16(dhs, W.sl, im, 0, 0, 0);                  \
    re = __builtin_amdgcn_mfma_f32_32x32x16_f16(A.sl, W.ch, re, 0, 0, 0);                 \
    im = __builtin_amdgcn_mfma_f32_32x32x16_f16(A.dl, W.sh, im, 0, 0, 0);                 \
    __builtin_amdgcn_sched_barrier(0);                                                    \
    {                                                                                     \
      const bool wrap = (S) + 4 >= a.steps;   /* then: the next tile, or the first tile again for the next block */ \
      const int s2 = wrap ? (S) + 4 - a.steps : (S) + 4;                                  \
      const int c2 = wrap ? (ti + 1 < nt ? ct + 4 : ctp) : ct;                            \
      load_tw(W, a.tw + ((size_t)s2 * a.nct + c2) * 256 + lane);                          \
    }                                                                                     \
    __builtin_amdgcn_sched_barrier(0);                                                    \
  }
      if (ti == 0) KDFH_READ_LEFT(la, 0)
      for (int s = 0; s < a.steps; s += 4) {
        KDFH_STEP(w0, la, lb, s)
        KDFH_STEP(w1, lb, la, s + 1)
        KDFH_STEP(w2, la, lb, s + 2)
        KDFH_STEP(w3, lb, la, s + 3)
      }
#undef KDFH_READ_LEFT
#undef KDFH_STEP
      // ---- amplitudes, scaled back, and the batch sums (Alg. 1 step 3) of this bin tile
      const int f = bin_of(a.bins, ct, col);
      const int c = f - a.f_min;
      float cr, ci;
      if (!R2) {
        cr = (f & 1) ? -1.f : 1.f;
        ci = 0.f;
      } else if (ct < a.bins.nct_e) {
        cr = (f & 2) ? -1.f : 1.f;
        ci = 0.f;
      } else {
        cr = 0.f;
        ci = (f & 2) ? -1.f : 1.f;
      }
      float amp[16];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 inv4 = *reinterpret_cast<const float4*>(rowinv + 8 * q + 4 * half);
        const float4 m14 = *reinterpret_cast<const float4*>(xn1 + 8 * q + 4 * half);
        const float4 m24 = *reinterpret_cast<const float4*>(xn2 + 8 * q + 4 * half);
        const float inv[4] = {inv4.x, inv4.y, inv4.z, inv4.w};
        const float m1[4] = {m14.x, m14.y, m14.z, m14.w};
        const float m2[4] = {m24.x, m24.y, m24.z, m24.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int r = 4 * q + e;
          const float rv = re[r] + cr * m1[e];
          const float iv = im[r] + ci * m2[e];
          amp[r] = sqrtf(rv * rv + iv * iv) * inv[e];
        }
      }
      float qs[4];                                 // rows 8q + 4 half + 0..3
#pragma unroll
      for (int q = 0; q < 4; ++q) qs[q] = (amp[4 * q] + amp[4 * q + 1]) + (amp[4 * q + 2] + amp[4 * q + 3]);
      const bool live = c < F;
      if (a.log2_rpv >= 3) {
        float vs[4];
        if (a.log2_rpv == 3) {
          vs[0] = qs[0]; vs[1] = qs[1]; vs[2] = qs[2]; vs[3] = qs[3];
        } else if (a.log2_rpv == 4) {
          vs[0] = qs[0] + qs[1]; vs[1] = qs[2] + qs[3]; vs[2] = 0.f; vs[3] = 0.f;
        } else {
          vs[0] = (qs[0] + qs[1]) + (qs[2] + qs[3]); vs[1] = 0.f; vs[2] = 0.f; vs[3] = 0.f;
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const float tot = vs[v] + __shfl_xor(vs[v], 32, 64);
          if (live && half == 0 && v < Vb) acc(asum[v * F + c], tot);
        }
      } else if (a.log2_rpv == 2) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (live) acc(asum[(2 * q + half) * F + c], qs[q]);
      } else if (a.log2_rpv == 1) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (live) {
            acc(asum[(4 * q + 2 * half) * F + c], amp[4 * q] + amp[4 * q + 1]);
            acc(asum[(4 * q + 2 * half + 1) * F + c], amp[4 * q + 2] + amp[4 * q + 3]);
          }
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (live) acc(asum[(8 * (r >> 2) + 4 * half + (r & 3)) * F + c], amp[r]);
      }
    }
    // ---- stray bins on the vector units: eight consumer threads per row share the folded samples (operand pieces
    // added back together); their row amplitudes go to LDS and are added to the batch sums after the next barrier
    if constexpr (R2 && STRAY) {
      const int ctid = tid - 256;
      const int r = ctid >> 3, part = ctid & 7;
      const int Tp = 8 * KG;
      float* samp = l.samp(b);
      for (int si = 0; si < a.bins.n_stray; ++si) {
        const int f = a.bins.stray_f[si];
        const halfx8* base = opnd + ((f & 1) ? 128 * pitch : 0) + r * pitch;
        const float4* tw4 = reinterpret_cast<const float4*>(l.stw() + (size_t)si * Tp * 2);   // (the copy in LDS)
        float re = 0.f, im = 0.f;
        for (int g = part; g < KG; g += 8) {
          const halfx8 ch = base[g], cl = base[32 * pitch + g], sh = base[64 * pitch + g], sl = base[96 * pitch + g];
#pragma unroll
          for (int j2 = 0; j2 < 4; ++j2) {
            const float4 tw = tw4[4 * g + j2];            // cos, sin of t = 8 g + 2 j2 and of the next sample
            re = fmaf((float)ch[2 * j2] + (float)cl[2 * j2], tw.x, re);
            im = fmaf((float)sh[2 * j2] + (float)sl[2 * j2], tw.y, im);
            re = fmaf((float)ch[2 * j2 + 1] + (float)cl[2 * j2 + 1], tw.z, re);
            im = fmaf((float)sh[2 * j2 + 1] + (float)sl[2 * j2 + 1], tw.w, im);
          }
        }
#pragma unroll
        for (int o = 1; o <= 4; o <<= 1) {
          re += __shfl_xor(re, o, 64);
          im += __shfl_xor(im, o, 64);
        }
        if (part == 0) {
          const float sg = (f & 2) ? -1.f : 1.f;           // (-1)^(f/2) for an even bin, sin(pi f / 2) for an odd one
          const float rv = (f & 1) ? re : re + sg * xn1[r];
          const float iv = (f & 1) ? im + sg * xn2[r] : im;
          samp[si * 32 + r] = sqrtf(rv * rv + iv * iv) * rowinv[r];
        }
      }
    }
  }
}

size_t kdfh_lds_bytes(int pitch, int F, int Vb, bool r2) {
  return (size_t)(r2 ? 8 : 4) * 32 * pitch * 16 + sizeof(float) * ((4 + kMaxStray) * 32 + (size_t)Vb * F);
}

// Pipelined kernel: workgroups persistent over the variate groups, as many as stay resident at once.
template <int IW, bool R2, bool STRAY>
int launch_kdfh_pipe(vardrop_ctx* ctx, const KdfhArgs& a, int ngroups, size_t lds, hipStream_t s) {
  constexpr int WPE = 2;                                   // eight wavefronts of up to 256 registers: one workgroup per compute unit
  if (lds > 65536)
    VD_HIP(ctx, hipFuncSetAttribute((const void*)kdfh_pipe_kernel<IW, R2, STRAY, WPE>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  const int grid = ngroups < ctx->num_cus ? ngroups : ctx->num_cus;
  {
    VdTimer timer(ctx, VARDROP_K_HASH, s);
    VD_KERNEL(ctx, (kdfh_pipe_kernel<IW, R2, STRAY, WPE>), dim3(grid), dim3(kPipeThreads), lds, s, a, ngroups);
  }
  VD_LAUNCH_CHECK(ctx);
  return VARDROP_OK;
}

template <int ITEMS, int RING, bool VEC, bool R2, bool STRAY = false, int WPE = (ITEMS == 1 ? 4 : (ITEMS <= 4 ? 2 : 1))>
int launch_kdfh(vardrop_ctx* ctx, const KdfhArgs& a, int grid, size_t lds, hipStream_t s) {
  if (lds > 65536)
    VD_HIP(ctx, hipFuncSetAttribute((const void*)kdfh_kernel<ITEMS, RING, VEC, R2, STRAY, WPE>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  {
    VdTimer timer(ctx, VARDROP_K_HASH, s);
    VD_KERNEL(ctx, (kdfh_kernel<ITEMS, RING, VEC, R2, STRAY, WPE>), dim3(grid), dim3(kThreads), lds, s, a);
  }
  VD_LAUNCH_CHECK(ctx);
  return VARDROP_OK;
}

}  // namespace

extern "C" size_t vardrop_hash_workspace_bytes(int, int, int, int, int, int) { return 0; }

extern "C" size_t vardrop_hash_strided_workspace_bytes(int B, int N, int L) {
  if (B < 1 || N < 0 || L < 2) return 0;
  return vd_align_up((size_t)B * (size_t)N * (size_t)L * sizeof(float), 256);
}

// Default cut-off (App. E: 25 at T = 96, "half of the number of positive frequencies"): half of the
// floor(L/2) + 1 bins of the real spectrum, rounded up; with the first candidate at bin 1 it is also their number.
extern "C" int vardrop_hash_default_cutoff(int L) { return L < 2 ? 0 : (L / 2 + 2) / 2; }

extern "C" int vardrop_hash(vardrop_ctx* ctx, const float* x, int B, int N, int L,
                            int64_t sb, int64_t sn, int64_t st, int k, int f_min, int f_max,
                            int32_t* topk, uint64_t* hash, float* abar,
                            void* ws, size_t ws_bytes, void* stream) {
  if (!ctx) return VARDROP_EINVAL;
  if (B < 1 || N < 0 || L < 2) return VARDROP_EINVAL;
  if (f_min < 0) f_min = 1;
  if (f_max < 0) f_max = vardrop_hash_default_cutoff(L);
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
  if (sb < 0 || sn < 0 || st < 1) return VARDROP_EINVAL;
  if (L > kMaxHashL || F > 64 * kMaxBinsPerLane) return VARDROP_EUNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  if (st != 1) {
    // time-contiguous copy of the windows in the workspace; the kernel below then reads that
    if (!ws || ws_bytes < vardrop_hash_strided_workspace_bytes(B, N, L) || !vd_aligned(ws, 16)) return VARDROP_EWORKSPACE;
    if (B > 65535) return VARDROP_EUNSUPPORTED;
    hipLaunchKernelGGL(time_contiguous_kernel, dim3(vd_ceil_div(N, 32), vd_ceil_div(L, 32), B), dim3(256), 0, s,
                       x, (float*)ws, N, L, (long long)sb, (long long)sn, (long long)st);
    VD_LAUNCH_CHECK(ctx);
    x = (const float*)ws;
    sb = (int64_t)N * L;
    sn = L;
    st = 1;
  }

  int log2_rpv = 5, nrb = vd_ceil_div(B, 32);
  if (B < 32) {
    log2_rpv = 0;
    while ((1 << log2_rpv) < B) ++log2_rpv;
    nrb = 1;
  }
  const int Vb = 32 >> log2_rpv;
  const bool vec = L % 4 == 0 && L >= 8 && sb % 4 == 0 && sn % 4 == 0 && vd_aligned(x, 16);
  // the radix-2 step pays when it saves contraction steps (they come in fours): from L = 136 on
  const bool r2 = vec && L % 8 == 0 && L >= 64 &&
                  ((vd_ceil_div(L / 4, 16) + 3) & ~3) < ((vd_ceil_div((L + 1) / 2, 16) + 3) & ~3);
  BinMap bins;
  bins.r2 = r2 ? 1 : 0;
  bins.f_min = f_min;
  bins.fe0 = f_min + (f_min & 1);                      // first even and first odd candidate bin
  bins.fo0 = f_min + 1 - (f_min & 1);
  const int n_even = bins.fe0 <= f_max ? (f_max - bins.fe0) / 2 + 1 : 0;
  const int n_odd = bins.fo0 <= f_max ? (f_max - bins.fo0) / 2 + 1 : 0;
  // tiles per parity set; one or two bins left over by a set that fills at least one tile are stray bins
  int tiles_e = vd_ceil_div(n_even, 32), tiles_o = vd_ceil_div(n_odd, 32);
  bins.n_stray = 0;
  if (r2) {
    if (n_even >= 32 && n_even % 32 >= 1 && n_even % 32 <= 2) {
      tiles_e = n_even / 32;
      for (int i = 0; i < n_even % 32; ++i) bins.stray_f[bins.n_stray++] = bins.fe0 + 2 * (tiles_e * 32 + i);
    }
    if (n_odd >= 32 && n_odd % 32 >= 1 && n_odd % 32 <= 2) {
      tiles_o = n_odd / 32;
      for (int i = 0; i < n_odd % 32; ++i) bins.stray_f[bins.n_stray++] = bins.fo0 + 2 * (tiles_o * 32 + i);
    }
  }
  for (int i = bins.n_stray; i < kMaxStray; ++i) bins.stray_f[i] = 0;
  bins.nct_e = r2 ? tiles_e : 0;
  const int T = r2 ? L / 4 : (L + 1) / 2;
  const int KS = vd_ceil_div(T, 16);
  const int steps = (KS + 3) & ~3;
  const int nct = r2 ? tiles_e + tiles_o : vd_ceil_div(F, 32);
  const int Tp = 16 * KS;                                 // samples per row the operand entries cover
  const size_t stw_off = (size_t)steps * nct * 4096;     // the stray bins' twiddles follow the table
  const int pitch = (2 * KS) | 1;
  const size_t lds = kdfh_lds_bytes(pitch, F, Vb, r2);
  if (lds > (size_t)ctx->lds_per_block) return VARDROP_EUNSUPPORTED;
  if (stw_off + (size_t)kMaxStray * Tp * 2 * sizeof(float) > kTwiddleBytes) return VARDROP_EUNSUPPORTED;   // (cannot happen within the limits above)

  if (ctx->twiddle_L != L || ctx->twiddle_fmin != f_min || ctx->twiddle_F != F || ctx->twiddle_r2 != bins.r2) {
    const int entries = steps * nct * 64;
    hipLaunchKernelGGL(twiddle_kernel, dim3(vd_ceil_div(entries, 256)), dim3(256), 0, s,
                       (halfx8*)ctx->twiddle, L, bins, f_max, T, steps, nct);
    if (bins.n_stray > 0)
      hipLaunchKernelGGL(stray_twiddle_kernel, dim3(vd_ceil_div(bins.n_stray * Tp, 256)), dim3(256), 0, s,
                         (float*)((char*)ctx->twiddle + stw_off), L, bins, T, Tp);
    VD_LAUNCH_CHECK(ctx);
    ctx->twiddle_L = L;
    ctx->twiddle_fmin = f_min;
    ctx->twiddle_F = F;
    ctx->twiddle_r2 = bins.r2;
  }
  KdfhArgs a;
  a.x = x;
  a.tw = (const halfx8*)ctx->twiddle;
  a.stw = (const float*)((const char*)ctx->twiddle + stw_off);
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
  a.bins = bins;
  a.log2_rpv = log2_rpv;
  a.nrb = nrb;
  a.T = T;
  a.KS = KS;
  a.steps = steps;
  a.nct = nct;
  a.pitch = pitch;
  a.inv_B = 1.0f / (float)B;
  const int grid = vd_ceil_div(N, Vb);
  const int items = vd_ceil_div(32 * 2 * KS, kThreads);
  // Long aligned windows with several row blocks per compute unit: the pipelined kernel (measured at 8192 variates
  // of 8 windows of 512 samples: 61 against 67 microseconds; at 336 samples and below the one-block-per-workgroup
  // kernel is as fast or faster and stays).
  const size_t plds = pipe_lds_bytes(pitch, F, Vb, r2);
  const int iw = vd_ceil_div(8 * 2 * KS, 64);             // items per producer lane: two sets of them must fit the registers
  if (r2 && L >= 384 && iw <= 2 && plds <= (size_t)ctx->lds_per_block && (long long)grid * nrb >= 4ll * ctx->num_cus) {
    if (bins.n_stray > 0) return launch_kdfh_pipe<2, true, true>(ctx, a, grid, plds, s);
    return launch_kdfh_pipe<2, true, false>(ctx, a, grid, plds, s);
  }
  if (r2 && bins.n_stray > 0) {
    if (items <= 1) return launch_kdfh<1, 2, true, true, true>(ctx, a, grid, lds, s);
    if (items <= 2) return launch_kdfh<2, 4, true, true, true>(ctx, a, grid, lds, s);
    return launch_kdfh<4, 4, true, true, true>(ctx, a, grid, lds, s);
  }
  if (r2) {
    if (items <= 1) return launch_kdfh<1, 2, true, true>(ctx, a, grid, lds, s);
    if (items <= 2) return launch_kdfh<2, 4, true, true>(ctx, a, grid, lds, s);
    return launch_kdfh<4, 4, true, true>(ctx, a, grid, lds, s);
  }
  if (vec) {
    if (items <= 1) return launch_kdfh<1, 2, true, false>(ctx, a, grid, lds, s);
    if (items <= 2) return launch_kdfh<2, 4, true, false>(ctx, a, grid, lds, s);
    if (items <= 4) return launch_kdfh<4, 4, true, false>(ctx, a, grid, lds, s);
    return launch_kdfh<8, 4, true, false>(ctx, a, grid, lds, s);
  }
  if (items <= 1) return launch_kdfh<1, 2, false, false>(ctx, a, grid, lds, s);
  if (items <= 2) return launch_kdfh<2, 4, false, false>(ctx, a, grid, lds, s);
  if (items <= 4) return launch_kdfh<4, 4, false, false>(ctx, a, grid, lds, s);
  return launch_kdfh<8, 4, false, false>(ctx, a, grid, lds, s);
}

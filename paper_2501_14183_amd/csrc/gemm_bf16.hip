// bf16 GEMMs of the attention back end on v_mfma_f32_32x32x16_bf16: projections, their input and
// weight gradients, and the sum of K slices.
#include "bf16_mfma.h"
#include "gemm_bf16.h"

namespace {

// out[z][i] = sum_s part[(z * splitk + s)][i], slices added in ascending order
struct SplitkReduce {
  const float* part;
  float* out[4];
  long long count;     // elements per matrix
  int splitk;
  // device-side token count: the slice count is the one the weight-gradient kernel derived from it (d = dn_d)
  const int32_t* n_dev;
  int n_max, n_mul, dn_d;
};
// One matrix of `stride` elements per slice, always `splitk` partial products (no direct result): its first count0
// elements go to out0, the next count1 to out1 (nullable).  With a device-side count the slices follow the
// embedding's rule (M = dn_m rows, N = dn_n columns).
struct SplitkReduceRows {
  const float* part;
  float* out0;
  float* out1;
  long long count0, count1, stride;
  int splitk;
  const int32_t* n_dev;
  int n_max, n_mul, dn_m, dn_n;
};
__global__ __launch_bounds__(256) void splitk_reduce_rows_kernel(SplitkReduceRows a) {
  int splitk = a.splitk;
  if (a.n_dev) {
    int n;
    if (!vd_count(a.n_dev, a.n_max, n)) return;
    splitk = n == 0 ? 0 : vd_embed_splitk(a.dn_m, a.dn_n, (long long)a.n_mul * n, nullptr);   // no tokens: zero gradients
  }
  const long long total = a.count0 + (a.out1 ? a.count1 : 0);
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    const float* p = a.part + i;
    float s = 0.f;
    int k = 0;
    for (; k + 4 <= splitk; k += 4) {            // four loads in flight, added in slice order
      const float p0 = p[(long long)k * a.stride], p1 = p[(long long)(k + 1) * a.stride];
      const float p2 = p[(long long)(k + 2) * a.stride], p3 = p[(long long)(k + 3) * a.stride];
      s = ((s + p0) + p1) + p2 + p3;
    }
    for (; k < splitk; ++k) s += p[(long long)k * a.stride];
    if (i < a.count0) a.out0[i] = s; else a.out1[i - a.count0] = s;
  }
}
__global__ __launch_bounds__(256) void splitk_reduce_kernel(SplitkReduce a) {
  if (a.n_dev) {
    int n;
    if (!vd_count(a.n_dev, a.n_max, n)) return;
    a.splitk = vd_attn_bf16_splitk(a.dn_d, (long long)a.n_mul * n, nullptr);
    if (a.splitk <= 1 && n > 0) return;          // a single slice was written as the result itself
    if (n == 0) a.splitk = 0;                    // no tokens: the gradients are zero
  }
  const int z = blockIdx.y;
  const float4* src = reinterpret_cast<const float4*>(a.part + (long long)z * a.splitk * a.count);
  float4* dst = reinterpret_cast<float4*>(a.out[z]);
  const long long n4 = a.count >> 2;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (long long)gridDim.x * blockDim.x) {
    float4 s = a.splitk > 0 ? src[i] : make_float4(0.f, 0.f, 0.f, 0.f);
    for (int k = 1; k < a.splitk; ++k) {
      const float4 v = src[(long long)k * n4 + i];
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    dst[i] = s;
  }
}

// ================================================================== GEMM with asynchronous LDS fill
// C[z] = op(A[z]) * op(B[z]) (+ bias[z]) in bf16, the sum over up to three segments into C[0], or
// (SPLIT) an fp32 partial product per K slice.  Each operand is either k-contiguous ([M][K] / [N][K])
// or mn-contiguous ([K][M] / [K][N]).
//
// Global memory is copied straight into LDS (global_load_lds_dwordx4: every lane names its own 16
// source bytes, the wavefront's 64 chunks land in 1 KB of consecutive LDS), NS stages deep, so
// that the copies of the next NS-1 slices are in flight while the matrix cores work on the
// current one and no register or LDS-store instruction is spent on staging.  Because the LDS side
// of a copy is fixed, the bank swizzle is applied on the source side: LDS chunk position p of a row
// holds source chunk p ^ pattern(row).
//   k-contiguous operand:  LDS tile [row][BK], fragments are 16-byte reads (row = lane % 32,
//                          chunk 2*ks + lane / 32), pattern chosen so that eight consecutive rows
//                          spread over all banks.
//   mn-contiguous operand: LDS tile [k][W]; fragments come from the transposing read
//                          ds_read_b64_tr_b16, in which, inside each group of 16 lanes, lane s names
//                          four consecutive columns of k-row s / 4 at column block s % 4, and lane j
//                          receives column j of the four k-rows.  A slice that reaches past the end
//                          of K (weight gradients: K is the token count) is copied from clamped
//                          rows and the left operand's fragments are masked.
// Fragment reads and the wait counters are written out by hand: the compiler would otherwise wait
// for every outstanding copy before any LDS read.
// The product is formed transposed (the B fragment is the left operand of the instruction), so a
// lane owns one output row and four consecutive columns per register quad; the tile goes through
// LDS once more so that global stores are whole 16-byte chunks of consecutive rows.
// The dimensions a kernel works with: those of the argument block, or what a device-side token count makes of them.
// waits until at most min(ahead, A) * LPS of this wavefront's copies are still in flight
template <int A, int LPS>
__device__ __forceinline__ void wait_ahead(int ahead) {
  if constexpr (A <= 0) {
    wait_vm<0>();
  } else {
    if (ahead >= A) wait_vm<A * LPS>();
    else wait_ahead<A - 1, LPS>(ahead);
  }
}
constexpr int kGemmThreads = 512;     // four computing wavefronts and four copy wavefronts
struct GemmDims {
  int M, K, splitk, kchunk, rs_n;
};
// KH (a 64-row tile of fp32 partial products from mn-contiguous operands on 64-k stages): the four computing
// wavefronts are two column halves x two halves of every K slice instead of 2 x 2 blocks of the tile.  A wavefront
// then owns all 64 rows, reads 2 KB + 2 KB of fragments per 16-k step instead of 1 KB + 2 KB for half the matrix
// instructions' worth of it (32 KB of LDS reads per slice instead of 48 KB, which is what bounds this tile), and
// the two K halves are added through LDS before the epilogue, lower half first.
template <bool AKC, bool BKC, bool SPLIT, int BM, int BK, int NS, bool KH = false>
__device__ __forceinline__ void gemm_async_tile(const GemmBf16& g, const GemmDims& dm, const int bx, const int by, const int bz) {
  static_assert(!KH || (!AKC && !BKC && SPLIT && BM == 64 && BK == 64), "K halves: 64-row weight-gradient tiles on 64-k stages");
  constexpr int BN = 128, MI = KH ? 2 : BM / 64, KS = BK / 16;
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;
  constexpr int IA = A_BYTES / 4096, IB = B_BYTES / 4096, LPS = IA + IB;   // 1 KB copies per wavefront and stage
  constexpr int CH = BK / 8;                                              // 16-byte chunks per k-contiguous row
  constexpr int RPI = 64 / CH;                                            // ... and rows per copy instruction
  constexpr int CHA = BM / 8, RPA = 64 / CHA;                             // the same for an [k][BM] tile
  constexpr int CHB = BN / 8, RPB = 64 / CHB;                             // and an [k][BN] tile
  constexpr int OPK = (AKC ? MI : 2 * MI) + (BKC ? 2 : 4);                // LDS reads per 16-k step
  constexpr int ES = SPLIT ? 4 : 2;                                       // output element size
  constexpr int CPITCH = BN * ES + 16;                                    // LDS row pitch of the output tile
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = KH ? 0 : (wave >> 1) & 1, wn = wave & 1;
  const int kh = KH ? (wave >> 1) & 1 : 0;                                // which two of a slice's four 16-k steps
  constexpr int MROWS = KH ? BM : BM / 2;                                 // tile rows a computing wavefront covers
  const int col = lane & 31, half = lane >> 5;
  const int zb = SPLIT ? bz / dm.splitk : bz;
  const int kbeg = SPLIT ? (bz % dm.splitk) * dm.kchunk : 0;
  const int kend = SPLIT ? min(dm.K, kbeg + dm.kchunk) : dm.K;
  const int m0 = by * BM, n0 = bx * BN;
  const int nseg = g.nseg > 1 ? g.nseg : 1;
  const int nk = (kend - kbeg + BK - 1) / BK;
  const int total = nseg * nk;
  const int zsel = g.nseg > 1 ? 0 : zb;
  const bf16_t* A1 = g.A1; const bf16_t* B1 = g.B1;
  const bf16_t* A2 = g.A2; const bf16_t* B2 = g.B2;
  const bf16_t* A0 = zsel == 0 ? g.A0 : (zsel == 1 ? A1 : (zsel == 2 ? A2 : g.A3));
  const bf16_t* B0 = zsel == 0 ? g.B0 : (zsel == 1 ? B1 : (zsel == 2 ? B2 : g.B3));

  // ---- the copy wavefronts.  Wavefronts 4-7 do nothing but issue the asynchronous copies; wavefronts 0-3 never touch
  // global memory inside the loop.  A copy instruction holds its wavefront until the memory pipeline takes it
  // (300-500 clocks per slice for a wavefront's share), which would otherwise be time in which that wavefront
  // issues neither LDS reads nor matrix instructions; one wavefront alone cannot issue a whole slice fast enough
  // (about 32 bytes per clock), four reach the pipeline's 64-74.
  const bool producer = wave >= 4;
  const int w4 = wave & 3;
  // source offsets (elements) of this copy wavefront's share: copy u fills LDS bytes [1024 (4 u + w4), + 1024) of the operand
  //   k-contiguous: clamped row * ld + chunk * 8, the slice start is added per stage
  //   mn-contiguous: column offset; the k-row krowX + u * 4 * RPx is clamped per stage
  static_assert((NS - 2) * LPS < 64, "the copy counter holds at most 63");
  int goffA[IA], goffB[IB];
  int krowA = 0, krowB = 0;
  if (producer) {
#pragma unroll
    for (int u = 0; u < IA; ++u) {
      if constexpr (AKC) {
        const int row = (u * 4 + w4) * RPI + lane / CH;
        goffA[u] = min(m0 + row, dm.M - 1) * g.lda + ((lane % CH) ^ swz_kc<BK>(row)) * 8;
      } else {
        const int krow = (u * 4 + w4) * RPA + lane / CHA;
        if (u == 0) krowA = krow;
        goffA[u] = min(m0 + ((lane % CHA) ^ swz_nc<BM>(krow)) * 8, dm.M - 8);
      }
    }
#pragma unroll
    for (int u = 0; u < IB; ++u) {
      if constexpr (BKC) {
        const int row = (u * 4 + w4) * RPI + lane / CH;
        goffB[u] = min(n0 + row, g.N - 1) * g.ldb + ((lane % CH) ^ swz_kc<BK>(row)) * 8;
      } else {
        const int krow = (u * 4 + w4) * RPB + lane / CHB;
        if (u == 0) krowB = krow;
        goffB[u] = min(n0 + ((lane % CHB) ^ swz_nc<BN>(krow)) * 8, g.N - 8);
      }
    }
  }
  // ---- fragment addresses (LDS bytes relative to a stage)
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
  uint32_t addrA[MI][AKC ? KS : 1], addrB[2][BKC ? KS : 1];
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    if constexpr (AKC) {
      const int ra = wm * MROWS + i * 32 + col;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) addrA[i][ks] = lds0 + ra * (BK * 2) + (((2 * ks + half) ^ swz_kc<BK>(ra)) * 16);
    } else {
      const int krow = 8 * half + ((lane & 15) >> 2);
      const int mn = wm * MROWS + i * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
      addrA[i][0] = lds0 + krow * (BM * 2) + (((mn >> 3) ^ swz_nc<BM>(krow)) * 16) + ((mn >> 2) & 1) * 8 + kh * 32 * BM * 2;
    }
  }
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    if constexpr (BKC) {
      const int rb = wn * 64 + j * 32 + col;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        addrB[j][ks] = lds0 + A_BYTES + rb * (BK * 2) + (((2 * ks + half) ^ swz_kc<BK>(rb)) * 16);
    } else {
      const int krow = 8 * half + ((lane & 15) >> 2);
      const int mn = wn * 64 + j * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
      addrB[j][0] = lds0 + A_BYTES + krow * (BN * 2) + (((mn >> 3) ^ swz_nc<BN>(krow)) * 16) + ((mn >> 2) & 1) * 8 + kh * 32 * BN * 2;
    }
  }

  floatx16 acc[MI][2];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = zero16();

  // ---- copy cursor (copy wavefront)
  int fseg = 0, fk = kbeg;
  const bf16_t* Ap = A0;
  const bf16_t* Bp = B0;
#define VD_ISSUE_STAGE(BUF)                                                                        \
  {                                                                                                \
    unsigned char* sp = smem + (BUF) * STAGE + w4 * 1024;                                          \
    _Pragma("unroll") for (int u = 0; u < IA; ++u) {                                               \
      const bf16_t* p;                                                                             \
      if constexpr (AKC) p = Ap + fk + goffA[u];                                                   \
      else p = Ap + (long long)min(fk + krowA + u * 4 * RPA, kend - 1) * g.lda + goffA[u];         \
      dma16(p, sp + u * 4096);                                                                     \
    }                                                                                              \
    _Pragma("unroll") for (int u = 0; u < IB; ++u) {                                               \
      const bf16_t* p;                                                                             \
      if constexpr (BKC) p = Bp + fk + goffB[u];                                                   \
      else p = Bp + (long long)min(fk + krowB + u * 4 * RPB, kend - 1) * g.ldb + goffB[u];         \
      dma16(p, sp + A_BYTES + u * 4096);                                                           \
    }                                                                                              \
    fk += BK;                                                                                      \
    if (fk >= kend) {                                                                              \
      fk = kbeg;                                                                                   \
      ++fseg;                                                                                      \
      Ap = fseg == 1 ? A1 : A2;                                                                    \
      Bp = fseg == 1 ? B1 : B2;                                                                    \
    }                                                                                              \
  }
  if (producer) {
#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
      if (s < total) VD_ISSUE_STAGE(s)
    for (int t0 = 0; t0 < total; t0 += NS) {
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        const int t = t0 + s;
        if (t < total) {
          // slice t has landed once at most `ahead` younger stages are still in flight
          const int ahead = min(total - 1 - t, NS - 2);
          wait_ahead<NS - 2, LPS>(ahead);
          __builtin_amdgcn_s_barrier();     // slice t is in; everyone is done with slice t-1, whose buffer is filled next
          if (t + NS - 1 < total) VD_ISSUE_STAGE((s + NS - 1) % NS)
        }
      }
    }
  } else {
  for (int t0 = 0; t0 < total; t0 += NS) {
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const int t = t0 + s;
      if (t < total) {
        __builtin_amdgcn_s_barrier();     // the copy wavefront has seen slice t land
        const uint32_t so = s * STAGE;
        // valid k of this lane's first fragment; only the last slice of an mn-contiguous A can fall short
        int kvalid = 8;
        if constexpr (!AKC) kvalid = t == total - 1 ? kend - (kbeg + (nk - 1) * BK + 8 * half + 32 * kh) : 8 + 16 * KS;
        Frag fa[2][2], fb[2][2];
#define VD_READ_STEP(KS_, SET)                                                                     \
  {                                                                                                \
    _Pragma("unroll") for (int i = 0; i < MI; ++i) {                                               \
      if constexpr (AKC) {                                                                         \
        lds_read16(fa[SET][i].q, addrA[i][AKC ? (KS_) : 0] + so);                                  \
      } else {                                                                                     \
        lds_read8_tr<(KS_) * 16 * BM * 2>(fa[SET][i].d[0], addrA[i][0] + so);                      \
        lds_read8_tr<(KS_) * 16 * BM * 2 + 4 * BM * 2>(fa[SET][i].d[1], addrA[i][0] + so);         \
      }                                                                                            \
    }                                                                                              \
    _Pragma("unroll") for (int j = 0; j < 2; ++j) {                                                \
      if constexpr (BKC) {                                                                         \
        lds_read16(fb[SET][j].q, addrB[j][BKC ? (KS_) : 0] + so);                                  \
      } else {                                                                                     \
        lds_read8_tr<(KS_) * 16 * BN * 2>(fb[SET][j].d[0], addrB[j][0] + so);                      \
        lds_read8_tr<(KS_) * 16 * BN * 2 + 4 * BN * 2>(fb[SET][j].d[1], addrB[j][0] + so);         \
      }                                                                                            \
    }                                                                                              \
  }
#define VD_MFMA_STEP(KS_, SET, PENDING)                                                            \
  {                                                                                                \
    if constexpr (MI == 2) wait_lds<PENDING>(fa[SET][0], fa[SET][1], fb[SET][0], fb[SET][1]);      \
    else wait_lds<PENDING>(fa[SET][0], fb[SET][0], fb[SET][1]);                                    \
    if constexpr (!AKC) {                                                                          \
      if (kvalid - 16 * (KS_) < 8) {                                                               \
        _Pragma("unroll") for (int i = 0; i < MI; ++i) mask_frag(fa[SET][i], kvalid - 16 * (KS_)); \
      }                                                                                            \
    }                                                                                              \
    _Pragma("unroll") for (int i = 0; i < MI; ++i)                                                 \
      _Pragma("unroll") for (int j = 0; j < 2; ++j) acc[i][j] = mfma(fb[SET][j], fa[SET][i], acc[i][j]); \
    __builtin_amdgcn_sched_barrier(0);                                                             \
  }
        VD_READ_STEP(0, 0)
        if constexpr (KS == 2 || KH) {
          VD_READ_STEP(1, 1)
          VD_MFMA_STEP(0, 0, OPK)
          VD_MFMA_STEP(1, 1, 0)
        } else {
          VD_READ_STEP(1, 1)
          VD_MFMA_STEP(0, 0, OPK)
          VD_READ_STEP(2, 0)
          VD_MFMA_STEP(1, 1, OPK)
          VD_READ_STEP(3, 1)
          VD_MFMA_STEP(2, 0, OPK)
          VD_MFMA_STEP(3, 1, 0)
        }
#undef VD_READ_STEP
#undef VD_MFMA_STEP
      }
    }
  }
  }
#undef VD_ISSUE_STAGE

  // ---- epilogue.  acc[i][j] register 4*q4 + e is C[wm*MROWS + i*32 + col][wn*64 + j*32 + 8*q4 + 4*half + e]
  // of the tile; it is written to LDS (with the bias), then stored as 16-byte chunks of whole rows.
  const bf16_t* bias = SPLIT ? nullptr : (zsel == 0 ? g.bias0 : (zsel == 1 ? g.bias1 : (zsel == 2 ? g.bias2 : g.bias3)));
  __syncthreads();                        // every wavefront is done reading the last slice
  if constexpr (KH) {
    // the upper K half hands its sums over through LDS; the lower half adds them to its own (lower + upper)
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      if (!producer && kh == 1 - pass) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
            for (int i = 0; i < MI; ++i) {
              float4* p = reinterpret_cast<float4*>(smem + (i * 32 + col) * CPITCH + (wn * 64 + j * 32 + 8 * q4 + 4 * half) * 4);
              if (pass == 0) {
                *p = make_float4(acc[i][j][4 * q4], acc[i][j][4 * q4 + 1], acc[i][j][4 * q4 + 2], acc[i][j][4 * q4 + 3]);
              } else {
                const float4 v = *p;
                acc[i][j][4 * q4] += v.x; acc[i][j][4 * q4 + 1] += v.y; acc[i][j][4 * q4 + 2] += v.z; acc[i][j][4 * q4 + 3] += v.w;
              }
            }
      }
      if (pass == 0) __syncthreads();
    }
    // (a lane of the lower half reads and rewrites only its own elements: no barrier in between)
  }
  if (!producer && kh == 0)
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int nl = wn * 64 + j * 32 + 8 * q4 + 4 * half;
      float bv[4] = {0.f, 0.f, 0.f, 0.f};
      if (bias && n0 + nl < g.N) {                 // N is a multiple of 8: a quad is inside or outside
        const u32x2 b4 = *reinterpret_cast<const u32x2*>(bias + n0 + nl);
        bv[0] = __uint_as_float(b4.x << 16); bv[1] = __uint_as_float(b4.x & 0xffff0000u);
        bv[2] = __uint_as_float(b4.y << 16); bv[3] = __uint_as_float(b4.y & 0xffff0000u);
      }
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        unsigned char* p = smem + (wm * MROWS + i * 32 + col) * CPITCH + nl * ES;
        if constexpr (SPLIT) {
          float4 o = make_float4(acc[i][j][4 * q4], acc[i][j][4 * q4 + 1], acc[i][j][4 * q4 + 2], acc[i][j][4 * q4 + 3]);
          *reinterpret_cast<float4*>(p) = o;
        } else {
          u32x2 o;
          o.x = pack2(acc[i][j][4 * q4] + bv[0], acc[i][j][4 * q4 + 1] + bv[1]);
          o.y = pack2(acc[i][j][4 * q4 + 2] + bv[2], acc[i][j][4 * q4 + 3] + bv[3]);
          *reinterpret_cast<u32x2*>(p) = o;
        }
      }
    }
  __syncthreads();
  constexpr int CPR = BN * ES / 16;          // 16-byte chunks per tile row
  constexpr int EPC = 16 / ES;               // elements per chunk
  unsigned char* Cb;
  long long ldc_bytes;
  if constexpr (SPLIT) {
    if (dm.splitk > 1 || g.force_part) {      // partial product of slice bz % splitk of matrix bz / splitk
      Cb = reinterpret_cast<unsigned char*>(g.part) + (long long)bz * dm.M * g.N * 4;
      ldc_bytes = (long long)g.N * 4;
    } else {                 // a single slice is the result itself
      Cb = reinterpret_cast<unsigned char*>(zsel == 0 ? g.C0 : (zsel == 1 ? g.C1 : (zsel == 2 ? g.C2 : g.C3)));
      ldc_bytes = (long long)g.ldc * 4;
    }
  } else {
    Cb = reinterpret_cast<unsigned char*>(zsel == 0 ? g.C0 : (zsel == 1 ? g.C1 : (zsel == 2 ? g.C2 : g.C3)));
    ldc_bytes = (long long)g.ldc * 2;
  }
  if (producer) return;                   // (no barrier follows)
#pragma unroll
  for (int u = 0; u < BM * CPR / 256; ++u) {
    const int idx = u * 256 + threadIdx.x;
    const int row = idx / CPR, c = idx % CPR;
    if (m0 + row < dm.M && n0 + c * EPC < g.N) {
      const u32x4 v = *reinterpret_cast<const u32x4*>(smem + row * CPITCH + c * 16);
      *reinterpret_cast<u32x4*>(Cb + (long long)(m0 + row) * ldc_bytes + (long long)(n0 + c * EPC) * ES) = v;
    }
  }
  if constexpr (!SPLIT) {
    // per-head row sums of C * rs_o (see GemmBf16) from the rounded tile in LDS: a pair of neighbouring lanes
    // takes the two 32-column halves of one head of one row, each in ascending column order
    if (g.rs_out) {
#pragma unroll
      for (int u = 0; u < BM * 4 / 256; ++u) {
        const int idx = u * 256 + threadIdx.x;
        const int row = idx >> 2, c0 = ((idx >> 1) & 1) * 64 + (idx & 1) * 32;
        const int m = m0 + row;
        const bool live = m < dm.M && n0 + c0 < g.N;
        float p = 0.f;
        if (live) {
          const bf16_t* orow = g.rs_o + (long long)m * g.ldc + n0 + c0;
#pragma unroll
          for (int v4 = 0; v4 < 4; ++v4) {
            const u32x4 cv = *reinterpret_cast<const u32x4*>(smem + row * CPITCH + (c0 + 8 * v4) * 2);
            const u32x4 ov = *reinterpret_cast<const u32x4*>(orow + 8 * v4);
#pragma unroll
            for (int w = 0; w < 4; ++w) {
              p = fmaf(__uint_as_float(cv[w] << 16), __uint_as_float(ov[w] << 16), p);
              p = fmaf(__uint_as_float(cv[w] & 0xffff0000u), __uint_as_float(ov[w] & 0xffff0000u), p);
            }
          }
        }
        p += __shfl_xor(p, 1, 64);
        if (live && (idx & 1) == 0) {
          const int b = m / dm.rs_n;
          const long long i = ((long long)b * g.rs_H + ((n0 + c0) >> 6)) * dm.rs_n + (m - b * dm.rs_n);
          g.rs_out[i] = p;
          if (g.rs_aux_out) g.rs_aux_out[i] = g.rs_aux_mul * g.rs_aux_in[i];
        }
      }
    }
  }
}

// LDS a workgroup of the asynchronous GEMM needs: the staging ring, or the output tile if that is larger
template <bool SPLIT, int BM, int BK, int NS>
constexpr int gemm_async_lds() {
  constexpr int ring = NS * (BM + 128) * BK * 2, out = BM * (128 * (SPLIT ? 4 : 2) + 16);
  return ring > out ? ring : out;
}
template <bool SPLIT, int BM, int BK, int NS>
constexpr int gemm_async_lds_v = gemm_async_lds<SPLIT, BM, BK, NS>();
// The product's dimensions, with a device-side token count (GemmBf16::n_dev) resolved; false: nothing to do.
__device__ __forceinline__ bool gemm_resolve(const GemmBf16& g, GemmDims& dm) {
  dm.M = g.M; dm.K = g.K; dm.splitk = g.splitk; dm.kchunk = g.kchunk; dm.rs_n = g.rs_n;
  if (!g.n_dev) return true;
  int n;
  if (!vd_count(g.n_dev, g.n_max, n, g.status)) return false;
  if (g.n_role == 0) {
    dm.M = g.n_mul * n;
    dm.rs_n = n;
  } else {
    dm.K = g.n_mul * n;
    int kchunk = 64;
    dm.splitk = g.n_role == 2 ? vd_embed_splitk(g.M, g.N, (long long)dm.K, &kchunk)
                              : vd_attn_bf16_splitk(g.M, (long long)dm.K, &kchunk);
    dm.kchunk = kchunk;
  }
  // (no tokens: an input gradient has no rows to write; a weight gradient is all zeros, which its tiles write
  // themselves: a product over no slices)
  if (g.n_role != 0 && dm.K == 0) {
    dm.splitk = 1;
    dm.kchunk = 64;
    return dm.M > 0;
  }
  return dm.M > 0 && dm.K > 0;
}
// One-dimensional grid of at least nz * tiles workgroups (more when the launch was sized for the bound of a
// device-side count: the surplus returns at once).
template <bool AKC, bool BKC, bool SPLIT, int BM, int BK, int NS>
__global__ __launch_bounds__(kGemmThreads, 2) void gemm_async_kernel(GemmBf16 g, int nz) {
  GemmDims dm;
  if (!gemm_resolve(g, dm)) return;
  // tiles in the order n fastest, then m, then batch entry: a die's range shares its rows of A
  const int gx = (g.N + 127) >> 7, gy = (dm.M + BM - 1) / BM;
  const int total = gx * gy * nz * (SPLIT ? dm.splitk : 1);
  if ((int)blockIdx.x >= total) return;
  const int t = xcd_contiguous(blockIdx.x, total);
  gemm_async_tile<AKC, BKC, SPLIT, BM, BK, NS>(g, dm, t % gx, (t / gx) % gy, t / (gx * gy));
}
// The input gradient (gx: k-contiguous operands, up to three accumulated segments) and the weight
// gradients (gw: mn-contiguous operands, K slices, fp32 partial products) depend on the same dQ, dK,
// dV and on nothing of each other, so they share one launch: workgroups [0, nx) take tiles of gx,
// the rest tiles of gw.  The longer-running input-gradient tiles are dispatched first.
// Tile shapes of the two kinds of workgroup: rows, k per copy stage, stages (BN = 128 always).
template <int BMX_, int BKX_, int NSX_, int BMW_, int BKW_, int NSW_, bool KHW_ = false>
struct PairCfg {
  static constexpr int BMX = BMX_, BKX = BKX_, NSX = NSX_, BMW = BMW_, BKW = BKW_, NSW = NSW_;
  static constexpr bool KHW = KHW_;                // the weight-gradient tiles' wavefronts split every K slice in halves
  static constexpr int ldsx = gemm_async_lds_v<false, BMX_, BKX_, NSX_>, ldsw = gemm_async_lds_v<true, BMW_, BKW_, NSW_>;
  static constexpr int lds = ldsx > ldsw ? ldsx : ldsw;
};
// few tokens: 128-row input-gradient tiles beside 64-row weight-gradient tiles (wavefronts in K halves), both on
// three 64-k stages (96 KB of LDS; with two stages an input-gradient tile waits 1000 of 1700 clocks per slice for
// its copies), one slice;
// many tokens: 128-row tiles on four 32-k stages for both (64 KB)
typedef PairCfg<128, 64, 3, 64, 64, 3, true> PairSmall;
typedef PairCfg<128, 32, 4, 128, 32, 4> PairLarge;
template <typename CFG>
__global__ __launch_bounds__(kGemmThreads, 2) void gemm_bwd_pair_kernel(GemmBf16 gx, GemmBf16 gw, int nzw) {
  // Each die takes a contiguous range of the input-gradient tiles (n fastest: a range shares its rows
  // of dQ, dK, dV) and a contiguous range of the weight-gradient tiles (n, then m, then K slice, then
  // matrix: a range shares its K slice of both operands); its input-gradient tiles come first.
  GemmDims dx, dw;
  const bool has_x = gemm_resolve(gx, dx);
  if (!gemm_resolve(gw, dw)) return;          // (an invalid count; with no tokens only the weight-gradient tiles run)
  if (!has_x) dx.M = 0;
  constexpr int BMX = CFG::BMX, BMW = CFG::BMW;
  const int gxn = (gx.N + 127) >> 7, gwn = (gw.N + 127) >> 7, gwm = (dw.M + BMW - 1) / BMW;
  const int nx = gxn * ((dx.M + BMX - 1) / BMX), nw = gwn * gwm * nzw * dw.splitk;
  if ((int)blockIdx.x >= nx + nw) return;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int cntx = (nx >> 3) + (xcd < (nx & 7) ? 1 : 0);
  const int startx = xcd_range_start(xcd, nx);
  if (slot < cntx) {
    const int t = startx + slot;
    gemm_async_tile<true, true, false, BMX, CFG::BKX, CFG::NSX>(gx, dx, t % gxn, t / gxn, 0);
  } else {
    const int t = xcd_range_start(xcd, nx + nw) - startx + (slot - cntx);
    gemm_async_tile<false, false, true, BMW, CFG::BKW, CFG::NSW, CFG::KHW>(gw, dw, t % gwn, (t / gwn) % gwm, t / (gwn * gwm));
  }
}

// Tile and pipeline depth of the asynchronous GEMM: 128 x 128 tiles once there are enough of them to
// keep every compute unit busy with two workgroups; otherwise 64 x 128 tiles, three stages deep while
// two workgroups still fit beside each other in LDS (at most 512 tiles), else two stages and three
// workgroups per compute unit.
template <bool AKC, bool BKC, bool SPLIT, int BM, int NS>
int launch_gemm_async_cfg(vardrop_ctx* ctx, int kid, const GemmBf16& g, int nz, hipStream_t s) {
  constexpr int BK = 64;
  constexpr int lds = gemm_async_lds<SPLIT, BM, BK, NS>();
  static int configured_device = -1;     // raising the dynamic LDS limit is a per-device, per-function setting
  if (configured_device != ctx->device) {
    VD_HIP(ctx, hipFuncSetAttribute((const void*)gemm_async_kernel<AKC, BKC, SPLIT, BM, BK, NS>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    configured_device = ctx->device;
  }
  // (with a device-side count g.M or g.K and g.splitk hold the bounds the grid is sized for)
  const long long grid = (long long)vd_ceil_div(g.N, 128) * vd_ceil_div(g.M, BM) * nz * (SPLIT ? g.splitk : 1);
  if (grid >= (1ll << 31)) return VARDROP_EUNSUPPORTED;
  {
    VdTimer timer(ctx, kid, s);
    VD_KERNEL(ctx, (gemm_async_kernel<AKC, BKC, SPLIT, BM, BK, NS>), dim3((unsigned)grid), dim3(kGemmThreads), lds, s, g, nz);
  }
  VD_LAUNCH_CHECK(ctx);
  return VARDROP_OK;
}
// one launch for the input gradient gx and the sliced weight gradients gw (nzw matrices)
template <typename CFG>
int launch_gemm_bwd_pair_cfg(vardrop_ctx* ctx, const GemmBf16& gx, const GemmBf16& gw, int nzw, hipStream_t s) {
  constexpr int lds = CFG::lds;
  static int configured_device = -1;
  if (configured_device != ctx->device) {
    VD_HIP(ctx, hipFuncSetAttribute((const void*)gemm_bwd_pair_kernel<CFG>, hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    configured_device = ctx->device;
  }
  const int gxn = vd_ceil_div(gx.N, 128), gxm = vd_ceil_div(gx.M, CFG::BMX);
  const int gwn = vd_ceil_div(gw.N, 128), gwm = vd_ceil_div(gw.M, CFG::BMW);
  const int nx = gxn * gxm, nw = gwn * gwm * nzw * gw.splitk;
  {
    VdTimer timer(ctx, VARDROP_K_GEMM_DW_DXS, s);
    VD_KERNEL(ctx, gemm_bwd_pair_kernel<CFG>, dim3(nx + nw), dim3(kGemmThreads), lds, s, gx, gw, nzw);
  }
  VD_LAUNCH_CHECK(ctx);
  return VARDROP_OK;
}
int launch_gemm_bwd_pair(vardrop_ctx* ctx, const GemmBf16& gx, const GemmBf16& gw, int nzw, hipStream_t s) {
  if (gx.K % 64 != 0 || gx.N % 8 != 0 || (long long)gx.M * gx.lda >= (1ll << 31) || (long long)gx.N * gx.ldb >= (1ll << 31) ||
      gw.M % 8 != 0 || gw.N % 8 != 0 || gw.kchunk % 64 != 0 || gw.splitk < 1 ||
      (long long)gw.K * gw.lda >= (1ll << 31) || (long long)gw.K * gw.ldb >= (1ll << 31))
    return VARDROP_EUNSUPPORTED;
  // (with a device-side count gx.M is the bound: a count in the few-token range under a bound in the other one
  // still runs correctly on the many-token tiles, with the single slice its own rule gives it)
  if (vd_attn_bf16_many_tokens(gx.N, gx.M)) return launch_gemm_bwd_pair_cfg<PairLarge>(ctx, gx, gw, nzw, s);
  return launch_gemm_bwd_pair_cfg<PairSmall>(ctx, gx, gw, nzw, s);
}

template <bool BKC>
int launch_gemm_async(vardrop_ctx* ctx, int kid, const GemmBf16& g, int nz, hipStream_t s) {
  if (g.M == 0 || g.N == 0) return VARDROP_OK;
  if ((g.K % 64 != 0 && (BKC || !g.a_kpad)) || g.N % 8 != 0 || (long long)g.M * g.lda >= (1ll << 31) ||
      (long long)g.K * g.ldb >= (1ll << 31))
    return VARDROP_EUNSUPPORTED;
  if (g.rs_out && (nz != 1 || g.nseg > 1 || g.N % 64 != 0 || g.rs_n <= 0 || g.M % g.rs_n != 0)) return VARDROP_EUNSUPPORTED;
  const long long t128 = (long long)vd_ceil_div(g.N, 128) * vd_ceil_div(g.M, 128) * nz;
  const long long t64 = (long long)vd_ceil_div(g.N, 128) * vd_ceil_div(g.M, 64) * nz;
  if (t128 >= 512) return launch_gemm_async_cfg<true, BKC, false, 128, 2>(ctx, kid, g, nz, s);
  if (t64 <= 512) return launch_gemm_async_cfg<true, BKC, false, 64, 3>(ctx, kid, g, nz, s);
  return launch_gemm_async_cfg<true, BKC, false, 64, 2>(ctx, kid, g, nz, s);
}

}  // namespace

int vd_gemm_bf16(vardrop_ctx* ctx, int kid, const GemmBf16& g, int nz, bool b_k_contiguous, hipStream_t s) {
  return b_k_contiguous ? launch_gemm_async<true>(ctx, kid, g, nz, s) : launch_gemm_async<false>(ctx, kid, g, nz, s);
}

int vd_gemm_bf16_bwd_pair(vardrop_ctx* ctx, const GemmBf16& gx, const GemmBf16& gw, int nzw, hipStream_t s) {
  return launch_gemm_bwd_pair(ctx, gx, gw, nzw, s);
}

int vd_gemm_bf16_wgrad_split(vardrop_ctx* ctx, int kid, const GemmBf16& g, hipStream_t s) {
  if (g.M == 0 || g.N == 0) return VARDROP_OK;
  if (g.M % 8 != 0 || g.N % 8 != 0 || g.splitk < 1 || g.kchunk % 64 != 0 ||
      (long long)g.K * g.lda >= (1ll << 31) || (long long)g.K * g.ldb >= (1ll << 31))
    return VARDROP_EUNSUPPORTED;
  return launch_gemm_async_cfg<false, false, true, 64, 2>(ctx, kid, g, 1, s);
}

int vd_gemm_bf16_sum_rows(vardrop_ctx* ctx, const float* part, float* out0, long long count0, float* out1, long long count1,
                          long long stride, int splitk, hipStream_t s, const GemmBf16* like) {
  SplitkReduceRows r = {};
  if (like && like->n_dev) {
    r.n_dev = like->n_dev;
    r.n_max = like->n_max;
    r.n_mul = like->n_mul;
    r.dn_m = like->M;
    r.dn_n = like->N;
  }
  r.part = part;
  r.out0 = out0;
  r.out1 = out1;
  r.count0 = count0;
  r.count1 = count1;
  r.stride = stride;
  r.splitk = splitk;
  {
    VdTimer timer(ctx, VARDROP_K_REDUCE_DW, s);
    VD_KERNEL(ctx, splitk_reduce_rows_kernel, dim3((unsigned)((count0 + count1 + 255) / 256)), dim3(256), 0, s, r);
  }
  VD_LAUNCH_CHECK(ctx);
  return VARDROP_OK;
}

int vd_gemm_bf16_sum_slices(vardrop_ctx* ctx, const float* part, float* const out[4], long long count, int splitk,
                            hipStream_t s, int nz, const GemmBf16* like) {
  SplitkReduce r = {};
  if (like && like->n_dev) {
    r.n_dev = like->n_dev;
    r.n_max = like->n_max;
    r.n_mul = like->n_mul;
    r.dn_d = like->M;
  }
  r.part = part;
  for (int z = 0; z < nz; ++z) r.out[z] = out[z];
  r.count = count;
  r.splitk = splitk;
  {
    VdTimer timer(ctx, VARDROP_K_REDUCE_DW, s);
    VD_KERNEL(ctx, splitk_reduce_kernel, dim3(vd_ceil_div((int)(count / 4), 256), nz), dim3(256), 0, s, r);
  }
  VD_LAUNCH_CHECK(ctx);
  return VARDROP_OK;
}

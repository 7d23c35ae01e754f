// bf16 matrix-core back end of the multi-head attention (Eq. 3), forward and backward.
//
//   * softmax(Q K^T / sqrt(d_k)) V works on the TRANSPOSED score tile S^T = K Q^T: in the accumulator
//     layout of the 32x32 instruction a lane then owns one query, so maximum, sum and rescaling are
//     per-lane scalars, and the probability registers are directly the right-hand operand of
//     O^T = V^T P^T;
//   * the backward recomputes the probabilities from Q, K and the saved log-sum-exp; no atomics, so
//     the result is deterministic;
//   * short selections (n <= 128, what variate dropping leaves) have kernels of their own that keep a
//     whole head in LDS: projection + attention forward, and dO + the whole attention backward;
//   * the projections and their gradients are the GEMMs of gemm_bf16.hip.
#include <algorithm>
#include "bf16_mfma.h"
#include "gemm_bf16.h"

namespace {

// ================================================================== attention core (d_k = 64)
constexpr int kDh = 64;
constexpr float kLog2e = 1.4426950408889634f;

// a lane's row of a head slice as four right-hand (or left-hand) operands: k = 16*s + 8*half + e
__device__ inline void row_frags(Frag f[4], const bf16_t* P, long long ld, int row, int n, int half) {
  const bool ok = row < n;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const u32x4 v = *reinterpret_cast<const u32x4*>(P + (long long)(ok ? row : 0) * ld + s * 16 + half * 8);
    f[s].q = ok ? v : u32x4{0u, 0u, 0u, 0u};
  }
}
// accumulator (transposed: rows = head dims, column = this lane's token) -> out[token][32*ct + ...]
__device__ inline void store_accT(bf16_t* out_row, const floatx16& acc, int ct, int half, float mul) {
#pragma unroll
  for (int g4 = 0; g4 < 4; ++g4) {
    u32x2 w;
    w.x = pack2(acc[4 * g4] * mul, acc[4 * g4 + 1] * mul);
    w.y = pack2(acc[4 * g4 + 2] * mul, acc[4 * g4 + 3] * mul);
    *reinterpret_cast<u32x2*>(out_row + ct * 32 + 8 * g4 + 4 * half) = w;
  }
}

struct SdpaArgs {
  const bf16_t *q, *k, *v, *o, *dout;
  const bf16_t *dy, *wo;          // short selections: dO is formed inside the kernel from dy and Wo
  bf16_t *out, *dq, *dk, *dv;
  float *lse, *Dsum;
  float* nlse2;                   // long selections: -log2(e) * lse, for the dK/dV part
  int n, d, H;
  float scale;
  const int32_t* n_dev;           // device-side token count (then n is its bound, see vd_count)
  int32_t* status;
  int B;
};

// ---- kernels for long selections (n > 128): staging ring.  A stage holds two [64 tokens][64] bf16 tiles of a
// head (8 KB each, 128-byte rows, the 16-byte chunk position XORed with a permutation of token % 8) and 2 x 64 floats; it is
// filled by asynchronous copies, three stages deep, so that a block of tokens costs one workgroup barrier
// and no staging registers.  Row-major fragments are 16-byte reads, transposed fragments come from the
// transposing read; LDS reads and their wait counters are written by hand (the compiler would wait for
// every outstanding copy before any LDS read).
constexpr int kRingTile = 64 * kDh * 2;
// (chunk position p of token row r holds source chunk p ^ tile_swz(r))
constexpr int kRingStage = 2 * kRingTile + 512;
constexpr int kRingStages = 3;
constexpr int kRingLds = kRingStages * kRingStage;
constexpr float kSlack = 8.f;                   // log2 of the largest unnormalised probability (see the forward kernel)

// copies rows [j0, j0 + 64) of two head slices into a stage; a wavefront-wide copy fills 8 token rows and
// rows past n repeat row n-1
template <int NW>
__device__ inline void ring_issue(const bf16_t* p0, const bf16_t* p1, long long ld, int j0, int n,
                                  unsigned char* stage, int wave, int lane) {
#pragma unroll
  for (int u = 0; u < 8 / NW; ++u) {
    const int rb = u * NW + wave;
    const int row = rb * 8 + (lane >> 3);
    const long long off = (long long)min(j0 + row, n - 1) * ld + (((lane & 7) ^ tile_swz(row)) * 8);
    dma16(p0 + off, stage + rb * 1024);
    dma16(p1 + off, stage + kRingTile + rb * 1024);
  }
}
// Per-lane LDS addresses (relative to a stage's first tile) of the two fragment kinds:
//   row[s]: token row `col` of a 32-row sub-tile, k = 16 s + 8 half .. +7 (add 4096 per sub-tile);
//   tr[dt]: transposed fragment, head dimensions 32 dt .. +31 as rows, four token rows 4 half + {0..3}
//           (add 128 * 16 per further 16-row group); tr8[dt]: the same for token rows 8 + 4 half + {0..3}.
struct RingAddr {
  uint32_t lds0, row[4], tr[2], tr8[2];
};
__device__ inline RingAddr ring_addr(const unsigned char* smem, int lane) {
  RingAddr r;
  const int col = lane & 31, half = lane >> 5;
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const unsigned char*)smem;
  r.lds0 = lds0;
#pragma unroll
  for (int s = 0; s < 4; ++s) r.row[s] = lds0 + col * 128 + (((2 * s + half) ^ tile_swz(col)) * 16);
  const int kr = 4 * half + ((lane & 15) >> 2);
#pragma unroll
  for (int dt = 0; dt < 2; ++dt) {
    const int mn = dt * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
    r.tr[dt] = lds0 + kr * 128 + (((mn >> 3) ^ tile_swz(kr)) * 16) + ((mn >> 2) & 1) * 8;
    r.tr8[dt] = lds0 + (kr + 8) * 128 + (((mn >> 3) ^ tile_swz(kr + 8)) * 16) + ((mn >> 2) & 1) * 8;
  }
  return r;
}
// The workgroup's place in an order in which each die works through whole (batch, head) pairs: gx workgroups per
// pair, one-dimensional grid.  Resolves a device-side token count first (a.n becomes the count).  False: this
// workgroup has nothing to do (surplus of a grid sized for the count's bound, or an invalid count).
__device__ inline bool ring_block(SdpaArgs& a, int rows, int parts, int& xb, int& h, int& b) {
  int n;
  if (!vd_count(a.n_dev, a.n, n, a.status)) return false;
  a.n = n;
  const int gx = parts * ((n + rows - 1) / rows);
  const int total = gx * a.H * a.B;
  if ((int)blockIdx.x >= total) return false;
  const int t = xcd_contiguous(blockIdx.x, total);
  xb = t % gx;
  h = (t / gx) % a.H;
  b = t / (gx * a.H);
  return true;
}

// four row-major fragments (k steps 0..3) of sub-tile KT of tile TILE
#define VD_ROW4(F, TILE, KT, SO)                                                        \
  lds_read16_at<(TILE) * kRingTile + (KT) * 4096>(F[0].q, ra.row[0] + (SO));            \
  lds_read16_at<(TILE) * kRingTile + (KT) * 4096>(F[1].q, ra.row[1] + (SO));            \
  lds_read16_at<(TILE) * kRingTile + (KT) * 4096>(F[2].q, ra.row[2] + (SO));            \
  lds_read16_at<(TILE) * kRingTile + (KT) * 4096>(F[3].q, ra.row[3] + (SO));
// four transposed fragments of the 32 token rows KT of tile TILE: F[2 * s2 + dt] = rows 16 s2 .., dimensions 32 dt ..
#define VD_TR4(F, TILE, KT, SO)                                                                              \
  lds_read8_tr<(TILE) * kRingTile + ((KT) * 32) * 128>(F[0].d[0], ra.tr[0] + (SO));                          \
  lds_read8_tr<(TILE) * kRingTile + ((KT) * 32) * 128>(F[0].d[1], ra.tr8[0] + (SO));                      \
  lds_read8_tr<(TILE) * kRingTile + ((KT) * 32) * 128>(F[1].d[0], ra.tr[1] + (SO));                          \
  lds_read8_tr<(TILE) * kRingTile + ((KT) * 32) * 128>(F[1].d[1], ra.tr8[1] + (SO));                      \
  lds_read8_tr<(TILE) * kRingTile + ((KT) * 32 + 16) * 128>(F[2].d[0], ra.tr[0] + (SO));                     \
  lds_read8_tr<(TILE) * kRingTile + ((KT) * 32 + 16) * 128>(F[2].d[1], ra.tr8[0] + (SO));                     \
  lds_read8_tr<(TILE) * kRingTile + ((KT) * 32 + 16) * 128>(F[3].d[0], ra.tr[1] + (SO));                     \
  lds_read8_tr<(TILE) * kRingTile + ((KT) * 32 + 16) * 128>(F[3].d[1], ra.tr8[1] + (SO));

// ---- forward: a wavefront owns 32 QG queries (lane = query of each group), NW wavefronts share the K / V stages.
// S^T = K q^T, online softmax on per-lane scalars, O^T = V^T P^T with the probability registers as the
// right-hand operand; every K or V fragment read from LDS serves all QG query groups.
template <int NW, int QG>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(2))) void sdpa_fwd_bf16(SdpaArgs a) {
  constexpr int NS = kRingStages;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int LPS = 16 / NW;                 // copies per wavefront and stage
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 31, half = lane >> 5;
  int qb, h, b;
  if (!ring_block(a, NW * 32 * QG, 1, qb, h, b)) return;
  const int n = a.n;
  const long long ld = a.d;
  const long long base = (long long)b * n * ld + h * kDh;
  const bf16_t* kp = a.k + base;
  const bf16_t* vp = a.v + base;
  const int q0 = (qb * NW + wave) * (32 * QG);
  const int nb = (n + 63) >> 6;
  ring_issue<NW>(kp, vp, ld, 0, n, smem, wave, lane);
  if (NS > 2 && nb > 1) ring_issue<NW>(kp, vp, ld, 64, n, smem + kRingStage, wave, lane);
  Frag qf[QG][4];
#pragma unroll
  for (int g = 0; g < QG; ++g) row_frags(qf[g], a.q + base, ld, q0 + 32 * g + col, n, half);
  const RingAddr ra = ring_addr(smem, lane);
  floatx16 acc[QG][2];
  float m[QG], l[QG];
#pragma unroll
  for (int g = 0; g < QG; ++g) {
    acc[g][0] = zero16();
    acc[g][1] = zero16();
    m[g] = -INFINITY;
    l[g] = 0.f;
  }
  const float c = a.scale * kLog2e;
  int buf = 0;
  for (int j = 0; j < nb; ++j) {
    // block j has landed once only the copies of block j+1 are in flight; behind the barrier everyone's have,
    // and everyone is done with block j-1, whose stage block j+2 takes
    if (NS > 2 && j + 1 < nb) wait_vm<LPS>(); else wait_vm<0>();
    __builtin_amdgcn_s_barrier();
    if (j + NS - 1 < nb) ring_issue<NW>(kp, vp, ld, (j + NS - 1) * 64, n, smem + ((buf + NS - 1) % NS) * kRingStage, wave, lane);
    const uint32_t so = buf * kRingStage;
    buf = buf == NS - 1 ? 0 : buf + 1;
    floatx16 st[QG][2];
    Frag fa[4], fb[4];
    VD_ROW4(fa, 0, 0, so)
    VD_ROW4(fb, 0, 1, so)
#pragma unroll
    for (int g = 0; g < QG; ++g) {
      st[g][0] = zero16();
      st[g][1] = zero16();
    }
#define VD_S_STEP(F, KT, S, PENDING)                                                    \
  wait_lds<PENDING>(F[S]);                                                              \
  _Pragma("unroll") for (int g = 0; g < QG; ++g) st[g][KT] = mfma(F[S], qf[g][S], st[g][KT]);
    __builtin_amdgcn_s_setprio(1);              // a wavefront feeding the matrix pipeline goes first
    VD_S_STEP(fa, 0, 0, 7) VD_S_STEP(fa, 0, 1, 6) VD_S_STEP(fa, 0, 2, 5) VD_S_STEP(fa, 0, 3, 4)
    VD_S_STEP(fb, 1, 0, 3) VD_S_STEP(fb, 1, 1, 2) VD_S_STEP(fb, 1, 2, 1) VD_S_STEP(fb, 1, 3, 0)
#undef VD_S_STEP
    __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
    VD_TR4(fa, 1, 0, so)                        // V^T fragments of the first 32 keys travel during the softmax
    // online softmax on the raw scores: exp2(c s - reference) as one fused multiply-add per score.  The
    // reference of a query is a past maximum of its scaled scores; it moves up (and the running sum and output
    // are rescaled, for the whole wavefront) only when a new score exceeds it by more than kSlack, so
    // probabilities stay below 2^kSlack and, after the first blocks, rescaling is rare.  The result is the same
    // as with the exact running maximum: numerator and denominator share the reference.
    // Keys past the end exist only in the last block.
    const bool tail = j * 64 + 64 > n;
#pragma unroll
    for (int g = 0; g < QG; ++g) {
      if (tail) {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = j * 64 + kt * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
            st[g][kt][r] = key < n ? st[g][kt][r] : -INFINITY;
          }
      }
      float mt = -INFINITY;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) mt = fmaxf(mt, st[g][kt][r]);
      mt = fmaxf(mt, __shfl_xor(mt, 32, 64));
      const float mc = mt * c;                        // c > 0: scaling commutes with the maximum
      const float mn = mc > m[g] + kSlack ? mc : m[g];
      float rs = 0.f;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          st[g][kt][r] = fast_exp2(fmaf(st[g][kt][r], c, -mn));
          rs += st[g][kt][r];
        }
      if (__any(mn != m[g])) {
        const float alpha = fast_exp2(m[g] - mn);
        l[g] *= alpha;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[g][dt][r] *= alpha;
      }
      l[g] += rs;
      m[g] = mn;
    }
    __builtin_amdgcn_sched_barrier(0);
    wait_lds_count<7>();                        // (the counter holds 15)
    VD_TR4(fb, 1, 1, so)
#define VD_PV_STEP(F, KT, I, PENDING)                                                   \
  wait_lds<PENDING>(F[I]);                                                              \
  _Pragma("unroll") for (int g = 0; g < QG; ++g)                                        \
    acc[g][(I) & 1] = mfma(F[I], regs_to_frag(st[g][KT], (I) >> 1), acc[g][(I) & 1]);
    __builtin_amdgcn_s_setprio(1);
    VD_PV_STEP(fa, 0, 0, 8) VD_PV_STEP(fa, 0, 1, 8) VD_PV_STEP(fa, 0, 2, 8) VD_PV_STEP(fa, 0, 3, 8)
    VD_PV_STEP(fb, 1, 0, 6) VD_PV_STEP(fb, 1, 1, 4) VD_PV_STEP(fb, 1, 2, 2) VD_PV_STEP(fb, 1, 3, 0)
#undef VD_PV_STEP
    __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
  }
#pragma unroll
  for (int g = 0; g < QG; ++g) {
    const int qi = q0 + 32 * g + col;
    const float lt = l[g] + __shfl_xor(l[g], 32, 64);
    if (qi < n) {
      const float inv = 1.f / lt;
      bf16_t* orow = a.out + base + (long long)qi * ld;
      store_accT(orow, acc[g][0], 0, half, inv);
      store_accT(orow, acc[g][1], 1, half, inv);
      if (half == 0) a.lse[((long long)b * a.H + h) * n + qi] = (m[g] + log2f(lt)) * 0.6931471805599453f;
    }
  }
}

// ---- backward, part 1: dQ (D = rowsum(dO * O) comes with dO from the GEMM before).  A wavefront owns 32 QG queries (lane = query), loop over
// key blocks: S^T = K q^T and dP^T = V dO^T from row fragments of the K and V tiles, dS^T in registers as the
// right-hand operand of dQ^T = K^T dS^T, whose left operand is the K tile again, read transposed.
template <int NW, int QG, bool DLOCAL>
__device__ __forceinline__ void sdpa_bwd_dq_body(const SdpaArgs& a, int qb, int h, int b) {
  constexpr int NS = kRingStages;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int LPS = 16 / NW;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 31, half = lane >> 5;
  const int n = a.n;
  const long long ld = a.d;
  const long long base = (long long)b * n * ld + h * kDh;
  const long long srow = ((long long)b * a.H + h) * n;
  const bf16_t* kp = a.k + base;
  const bf16_t* vp = a.v + base;
  const int q0 = (qb * NW + wave) * (32 * QG);
  const int nb = (n + 63) >> 6;
  ring_issue<NW>(kp, vp, ld, 0, n, smem, wave, lane);
  if (NS > 2 && nb > 1) ring_issue<NW>(kp, vp, ld, 64, n, smem + kRingStage, wave, lane);
  Frag qf[QG][4], dof[QG][4];
  float D[QG], nlse2[QG];                      // nlse2 = -log2(e) * log-sum-exp (-inf for a query past the end)
#pragma unroll
  for (int g = 0; g < QG; ++g) {
    const int qi = q0 + 32 * g + col;
    row_frags(qf[g], a.q + base, ld, qi, n, half);
    row_frags(dof[g], a.dout + base, ld, qi, n, half);
    if constexpr (DLOCAL) {   // D = rowsum(dO * O) formed here and left for the dK/dV kernel
      Frag of[4];
      row_frags(of, a.o + base, ld, qi, n, half);
      float dsum = 0.f;
#pragma unroll
      for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int e = 0; e < 8; ++e) dsum = fmaf(bf2f(dof[g][s].h[e]), bf2f(of[s].h[e]), dsum);
      D[g] = dsum + __shfl_xor(dsum, 32, 64);
    } else {
      D[g] = a.Dsum[srow + min(qi, n - 1)];
    }
    nlse2[g] = qi < n ? -a.lse[srow + qi] * kLog2e : -INFINITY;
  }
  const RingAddr ra = ring_addr(smem, lane);
  floatx16 acc[QG][2];
#pragma unroll
  for (int g = 0; g < QG; ++g) {
    acc[g][0] = zero16();
    acc[g][1] = zero16();
  }
  const float c = a.scale * kLog2e;
  int buf = 0;
  for (int j = 0; j < nb; ++j) {
    if (NS > 2 && j + 1 < nb) wait_vm<LPS>(); else wait_vm<0>();
    __builtin_amdgcn_s_barrier();
    if (j + NS - 1 < nb) ring_issue<NW>(kp, vp, ld, (j + NS - 1) * 64, n, smem + ((buf + NS - 1) % NS) * kRingStage, wave, lane);
    const uint32_t so = buf * kRingStage;
    buf = buf == NS - 1 ? 0 : buf + 1;
    const bool tail = j * 64 + 64 > n;
#define VD_DQ_HALF(KT)                                                                                   \
  {                                                                                                      \
    floatx16 st[QG], dp[QG];                                                                             \
    Frag fk[4], fv[4], ft[4];                                                                            \
    VD_ROW4(fk, 0, KT, so)                                                                               \
    VD_ROW4(fv, 1, KT, so)                                                                               \
    _Pragma("unroll") for (int g = 0; g < QG; ++g) {                                                     \
      st[g] = zero16();                                                                                  \
      dp[g] = zero16();                                                                                  \
    }                                                                                                    \
    __builtin_amdgcn_s_setprio(1);                                                                       \
    VD_DQ_STEP(st, fk, qf, 0, 7) VD_DQ_STEP(st, fk, qf, 1, 6) VD_DQ_STEP(st, fk, qf, 2, 5) VD_DQ_STEP(st, fk, qf, 3, 4) \
    VD_DQ_STEP(dp, fv, dof, 0, 3) VD_DQ_STEP(dp, fv, dof, 1, 2) VD_DQ_STEP(dp, fv, dof, 2, 1) VD_DQ_STEP(dp, fv, dof, 3, 0) \
    __builtin_amdgcn_s_setprio(0);                                                                       \
    __builtin_amdgcn_sched_barrier(0);                                                                   \
    VD_TR4(ft, 0, KT, so)                                                                                \
    _Pragma("unroll") for (int g = 0; g < QG; ++g)                                                       \
      _Pragma("unroll") for (int r = 0; r < 16; ++r)                                                     \
        st[g][r] = fast_exp2(fmaf(st[g][r], c, nlse2[g])) * (dp[g][r] - D[g]);                           \
    if (tail) {                                 /* a key past the end repeats the last one: its dS is dropped */ \
      _Pragma("unroll") for (int g = 0; g < QG; ++g)                                                     \
        _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                                 \
          const int key = j * 64 + (KT) * 32 + 8 * (r >> 2) + 4 * half + (r & 3);                        \
          st[g][r] = key < n ? st[g][r] : 0.f;                                                           \
        }                                                                                                \
    }                                                                                                    \
    __builtin_amdgcn_sched_barrier(0);                                                                   \
    __builtin_amdgcn_s_setprio(1);                                                                       \
    VD_DQ_ACC(ft, 0, 6) VD_DQ_ACC(ft, 1, 4) VD_DQ_ACC(ft, 2, 2) VD_DQ_ACC(ft, 3, 0)                       \
    __builtin_amdgcn_s_setprio(0);                                                                       \
    __builtin_amdgcn_sched_barrier(0);                                                                   \
  }
#define VD_DQ_STEP(ACC, F, RHS, S, PENDING)                                             \
  wait_lds<PENDING>(F[S]);                                                              \
  _Pragma("unroll") for (int g = 0; g < QG; ++g) ACC[g] = mfma(F[S], RHS[g][S], ACC[g]);
#define VD_DQ_ACC(F, I, PENDING)                                                        \
  wait_lds<PENDING>(F[I]);                                                              \
  _Pragma("unroll") for (int g = 0; g < QG; ++g)                                        \
    acc[g][(I) & 1] = mfma(F[I], regs_to_frag(st[g], (I) >> 1), acc[g][(I) & 1]);
    VD_DQ_HALF(0)
    VD_DQ_HALF(1)
#undef VD_DQ_HALF
#undef VD_DQ_STEP
#undef VD_DQ_ACC
  }
#pragma unroll
  for (int g = 0; g < QG; ++g) {
    const int qi = q0 + 32 * g + col;
    if (qi < n) {
      bf16_t* row = a.dq + base + (long long)qi * ld;
      store_accT(row, acc[g][0], 0, half, a.scale);
      store_accT(row, acc[g][1], 1, half, a.scale);
      if (DLOCAL && half == 0) {
        a.Dsum[srow + qi] = D[g];
        a.nlse2[srow + qi] = nlse2[g];
      }
    }
  }
}

// ---- backward, part 2: dK and dV.  A wavefront owns 32 keys (lane = key), loop over query blocks: a stage holds
// the Q and dO tiles of 64 queries, their log-sum-exp and their D.  S = Q k^T and dP = dO v^T from row
// fragments; P and dS in registers are the right-hand operands of dV^T = dO^T P and dK^T = Q^T dS, whose left
// operands are the same tiles read transposed.
template <int NW>
__device__ __forceinline__ void sdpa_bwd_dkv_body(const SdpaArgs& a, int kb, int h, int b) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int LPS = 16 / NW + 1;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 31, half = lane >> 5;
  const int n = a.n;
  const long long ld = a.d;
  const long long base = (long long)b * n * ld + h * kDh;
  const long long srow = ((long long)b * a.H + h) * n;
  const bf16_t* qp = a.q + base;
  const bf16_t* op = a.dout + base;
  const int kj = (kb * NW + wave) * 32 + col;
  const int nb = (n + 63) >> 6;
  // even wavefronts copy the block's -log2(e) * log-sum-exp values, odd ones its D (NW is even); queries past n
  // repeat the last
  const float* stat = (wave & 1) ? a.Dsum + srow : a.nlse2 + srow;
  const int stat_off = 2 * kRingTile + (wave & 1) * 256;
#define VD_ISSUE_Q(J, BUF)                                                                            \
  {                                                                                                   \
    unsigned char* sp = smem + (BUF) * kRingStage;                                                    \
    ring_issue<NW>(qp, op, ld, (J) * 64, n, sp, wave, lane);                                          \
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(stat + min((J) * 64 + lane, n - 1)), \
                                     (__attribute__((address_space(3))) void*)(sp + stat_off), 4, 0, 0); \
  }
  VD_ISSUE_Q(0, 0)
  if (nb > 1) VD_ISSUE_Q(1, 1)
  Frag kf[4], vf[4];
  row_frags(kf, a.k + base, ld, kj, n, half);
  row_frags(vf, a.v + base, ld, kj, n, half);
  const RingAddr ra = ring_addr(smem, lane);
  const uint32_t stat_addr = ra.lds0 + 2 * kRingTile + 16 * half;   // + 32 per 8 queries
  floatx16 accK[2] = {zero16(), zero16()}, accV[2] = {zero16(), zero16()};
  const float c = a.scale * kLog2e;
  int buf = 0;
  for (int i = 0; i < nb; ++i) {
    if (i + 1 < nb) wait_vm<LPS>(); else wait_vm<0>();
    __builtin_amdgcn_s_barrier();
    if (i + 2 < nb) VD_ISSUE_Q(i + 2, (buf + 2) % kRingStages)
    const uint32_t so = buf * kRingStage;
    buf = buf == kRingStages - 1 ? 0 : buf + 1;
    const bool tail = i * 64 + 64 > n;
#define VD_DKV_HALF(QT)                                                                                  \
  {                                                                                                      \
    floatx16 st = zero16(), dp = zero16();                                                               \
    Frag fq[4], fo[4], ls[4], ds_[4];                                                                    \
    VD_ROW4(fq, 0, QT, so)                                                                               \
    VD_ROW4(fo, 1, QT, so)                                                                               \
    __builtin_amdgcn_s_setprio(1);                                                                       \
    wait_lds<7>(fq[0]); st = mfma(fq[0], kf[0], st);                                                     \
    wait_lds<6>(fq[1]); st = mfma(fq[1], kf[1], st);                                                     \
    wait_lds<5>(fq[2]); st = mfma(fq[2], kf[2], st);                                                     \
    wait_lds<4>(fq[3]); st = mfma(fq[3], kf[3], st);                                                     \
    __builtin_amdgcn_sched_barrier(0);                                                                   \
    /* log-sum-exp and D of queries 32 QT + 8 q4 + 4 half + 0..3, the rows of registers 4 q4 .. 4 q4 + 3 */ \
    lds_read16_at<(QT) * 128>(ls[0].q, stat_addr + so);                                                  \
    lds_read16_at<(QT) * 128 + 32>(ls[1].q, stat_addr + so);                                             \
    lds_read16_at<(QT) * 128 + 64>(ls[2].q, stat_addr + so);                                             \
    lds_read16_at<(QT) * 128 + 96>(ls[3].q, stat_addr + so);                                             \
    lds_read16_at<(QT) * 128 + 256>(ds_[0].q, stat_addr + so);                                           \
    lds_read16_at<(QT) * 128 + 256 + 32>(ds_[1].q, stat_addr + so);                                      \
    lds_read16_at<(QT) * 128 + 256 + 64>(ds_[2].q, stat_addr + so);                                      \
    lds_read16_at<(QT) * 128 + 256 + 96>(ds_[3].q, stat_addr + so);                                      \
    wait_lds<11>(fo[0]); dp = mfma(fo[0], vf[0], dp);                                                    \
    wait_lds<10>(fo[1]); dp = mfma(fo[1], vf[1], dp);                                                    \
    wait_lds<9>(fo[2]); dp = mfma(fo[2], vf[2], dp);                                                     \
    wait_lds<8>(fo[3]); dp = mfma(fo[3], vf[3], dp);                                                     \
    __builtin_amdgcn_s_setprio(0);                                                                       \
    __builtin_amdgcn_sched_barrier(0);                                                                   \
    wait_lds_count<7>();                        /* (the counter holds 15) */                             \
    VD_TR4(fo, 1, QT, so)                       /* dO^T */                                               \
    wait_lds<8>(ls[0], ls[1], ls[2], ls[3]);                                                             \
    wait_lds<8>(ds_[0], ds_[1], ds_[2], ds_[3]);                                                         \
    _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                                     \
      const float p = fast_exp2(fmaf(st[r], c, __uint_as_float(ls[r >> 2].w[r & 3])));                   \
      st[r] = p;                                                                                         \
      dp[r] = p * (dp[r] - __uint_as_float(ds_[r >> 2].w[r & 3]));                                       \
    }                                                                                                    \
    if (tail) {                                 /* a query past the end repeats the last one: dropped */ \
      _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                                   \
        const int iq = i * 64 + (QT) * 32 + 8 * (r >> 2) + 4 * half + (r & 3);                           \
        st[r] = iq < n ? st[r] : 0.f;                                                                    \
        dp[r] = iq < n ? dp[r] : 0.f;                                                                    \
      }                                                                                                  \
    }                                                                                                    \
    __builtin_amdgcn_sched_barrier(0);                                                                   \
    wait_lds_count<7>();                                                                                 \
    VD_TR4(fq, 0, QT, so)                       /* Q^T */                                                \
    __builtin_amdgcn_s_setprio(1);                                                                       \
    wait_lds<8>(fo[0]); accV[0] = mfma(fo[0], regs_to_frag(st, 0), accV[0]);                             \
    wait_lds<8>(fo[1]); accV[1] = mfma(fo[1], regs_to_frag(st, 0), accV[1]);                             \
    wait_lds<8>(fo[2]); accV[0] = mfma(fo[2], regs_to_frag(st, 1), accV[0]);                             \
    wait_lds<8>(fo[3]); accV[1] = mfma(fo[3], regs_to_frag(st, 1), accV[1]);                             \
    wait_lds<6>(fq[0]); accK[0] = mfma(fq[0], regs_to_frag(dp, 0), accK[0]);                             \
    wait_lds<4>(fq[1]); accK[1] = mfma(fq[1], regs_to_frag(dp, 0), accK[1]);                             \
    wait_lds<2>(fq[2]); accK[0] = mfma(fq[2], regs_to_frag(dp, 1), accK[0]);                             \
    wait_lds<0>(fq[3]); accK[1] = mfma(fq[3], regs_to_frag(dp, 1), accK[1]);                             \
    __builtin_amdgcn_s_setprio(0);                                                                       \
    __builtin_amdgcn_sched_barrier(0);                                                                   \
  }
    VD_DKV_HALF(0)
    VD_DKV_HALF(1)
#undef VD_DKV_HALF
  }
#undef VD_ISSUE_Q
  if (kj < n) {
    bf16_t* rk = a.dk + base + (long long)kj * ld;
    bf16_t* rv = a.dv + base + (long long)kj * ld;
    store_accT(rk, accK[0], 0, half, a.scale);
    store_accT(rk, accK[1], 1, half, a.scale);
    store_accT(rv, accV[0], 0, half, 1.f);
    store_accT(rv, accV[1], 1, half, 1.f);
  }
}
#undef VD_ROW4
#undef VD_TR4

// Many workgroups: two launches, D = rowsum(dO * O) and -log2(e) * lse written by the dQ kernel, whose matrix work
// hides the read of O.
template <int NW>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(2))) void sdpa_bwd_dq_bf16(SdpaArgs a) {
  int xb, h, b;
  if (!ring_block(a, NW * 32, 1, xb, h, b)) return;
  sdpa_bwd_dq_body<NW, 1, true>(a, xb, h, b);
}
template <int NW>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(2))) void sdpa_bwd_dkv_bf16(SdpaArgs a) {
  int xb, h, b;
  if (!ring_block(a, NW * 32, 1, xb, h, b)) return;
  sdpa_bwd_dkv_body<NW>(a, xb, h, b);
}
// Few workgroups: one launch, so that the two parts fill the chip's places together.  Of the workgroups of a
// (batch, head) pair the first half take query blocks (dQ), the second half key blocks (dK, dV); neither part
// reads what the other writes: D and -log2(e) * lse come with dO from the GEMM before.
template <int NW>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(2))) void sdpa_bwd_dqkv_bf16(SdpaArgs a) {
  int xb, h, b;
  if (!ring_block(a, NW * 32, 2, xb, h, b)) return;
  const int nblk = (a.n + NW * 32 - 1) / (NW * 32);
  if (xb < nblk) sdpa_bwd_dq_body<NW, 1, false>(a, xb, h, b);
  else sdpa_bwd_dkv_body<NW>(a, xb - nblk, h, b);
}

// ---- backward for short selections (n <= 128, the regime variate dropping produces): one workgroup
// per (batch, head) holds Q, K, V and O of the head in LDS (asynchronous copies), forms the head's dO tile
// from dy and Wo itself (dO never goes to memory), and forms S and dP once for all three gradients.
//   phase 1, a wavefront owns 32 keys (lane = key):  S^T-free orientation S[query][key] = Q k^T and
//            dP = dO v^T with the key fragments in registers; P and dS feed dV^T = dO^T P and
//            dK^T = Q^T dS, whose left operands (contraction over queries) are transposing reads of
//            the dO and Q tiles; dS goes to LDS as dS^T[key][query].
//   phase 2, a wavefront owns 32 queries (lane = query): dQ^T = K^T dS^T, both operands transposing
//            reads (contraction over keys).
// Tiles are [token][64] with the 16-byte chunk position XORed with token % 8, as the copies write them.
constexpr int kSmallN = 128;
constexpr int kDsPitch = 272;                 // bytes per dS^T row: 128 queries * 2 + 16
constexpr int kSmallTile = kSmallN * kDh * 2;  // bytes of one [128][64] tile
constexpr int kBwdStage = kSmallN * 64 * 2 + 64 * 64 * 2;        // dy tile + Wo tile of one 64-k slice: 24 KB
constexpr int kBwdStages = 2;
constexpr int kSmallLds = 5 * kSmallTile + kBwdStages * kBwdStage;   // the ring overlays dS^T and the statistics

typedef short s16x4 __attribute__((ext_vector_type(4)));
// 16-byte chunk (k = 8*chunk ..) of a token row of a swizzled tile
__device__ inline Frag small_row_frag(const unsigned char* tile, int row, int chunk) {
  Frag f;
  f.q = *reinterpret_cast<const u32x4*>(tile + row * 128 + ((chunk ^ tile_swz(row)) * 16));
  return f;
}
// transposing read of a swizzled tile: this lane receives, for column mn0 + lane % 16 of the 16-lane
// group's column block, the four token rows krow0 .. krow0+3 and krow0+8 .. krow0+11
__device__ inline Frag small_tr_frag(const unsigned char* tile, int krow0, int mn0, int lane) {
  Frag f;
  const int mn = mn0 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
#pragma unroll
  for (int rd = 0; rd < 2; ++rd) {
    const int krow = krow0 + 8 * rd + ((lane & 15) >> 2);
    const unsigned char* p = tile + krow * 128 + (((mn >> 3) ^ tile_swz(krow)) * 16) + ((mn >> 2) & 1) * 8;
    const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p);
    f.d[rd] = __builtin_bit_cast(u32x2, v);
  }
  return f;
}
__global__ __launch_bounds__(512) void sdpa_bwd_small_bf16(SdpaArgs a) {
  // Eight wavefronts, two per SIMD so that one's LDS and conversion work hides behind the other's matrix
  // instructions.  Wavefront w works on token block w % 4; in phase 1 the two wavefronts of a key block
  // split the query tiles between them (their partial dK, dV meet in LDS), in phase 2 the two
  // wavefronts of a query block take one 32-wide half of the head dimension each.
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* Ks = smem;
  unsigned char* Qs = Ks + kSmallTile;
  unsigned char* Vs = Qs + kSmallTile;
  unsigned char* dOs = Vs + kSmallTile;
  unsigned char* Os = dOs + kSmallTile;
  unsigned char* dSt = Os + kSmallTile;                                   // [key][kDsPitch]
  float* Ls = reinterpret_cast<float*>(dSt + kSmallN * kDsPitch);
  float* Ds = Ls + kSmallN;
  float* scratch = reinterpret_cast<float*>(Qs);                          // Q, V, dO, O tiles: free after phase 1
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int blk = wave & 3, part = wave >> 2;
  const int col = lane & 31, half = lane >> 5;
  // heads fastest: a die's contiguous range covers whole batches, whose dy rows it then fetches once
  const int tix = xcd_contiguous(blockIdx.x + gridDim.x * blockIdx.y, gridDim.x * gridDim.y);
  const int h = tix % a.H, b = tix / a.H;
  int n;
  if (!vd_count(a.n_dev, a.n, n, a.status) || n == 0) return;
  const long long ld = a.d;
  const long long base = (long long)b * n * ld + h * kDh;
  const long long srow = ((long long)b * a.H + h) * n;

  // ---- dO tile of this head: dO[token][i] = sum_j dy[token][j] Wo[64 h + i][j], both operands k-contiguous,
  // 64-k slices two stages deep in a ring that overlays the (not yet used) dS^T buffer.  Wavefront w
  // computes token rows 32*(w % 4) .. +31, columns 32*(w / 4) .. +31.
  {
    constexpr int NS = kBwdStages, STAGE = kBwdStage, A_BYTES = kSmallN * 64 * 2, LPS = 3;
    unsigned char* ring = dSt;
    const bf16_t* dy_b = a.dy + (long long)b * n * ld;
    const bf16_t* srcA[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int row = (u * 8 + wave) * 8 + (lane >> 3);
      srcA[u] = dy_b + (long long)min(row, n - 1) * ld + (((lane & 7) ^ tile_swz(row)) * 8);
    }
    const int rowB = wave * 8 + (lane >> 3);
    const bf16_t* srcB = a.wo + (long long)(h * kDh + rowB) * ld + (((lane & 7) ^ tile_swz(rowB)) * 8);
    const uint32_t ring0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)ring;
    uint32_t addrA[4], addrB[4];
    {
      const int ra = blk * 32 + col, rb = part * 32 + col;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        addrA[ks] = ring0 + ra * 128 + (((2 * ks + half) ^ tile_swz(ra)) * 16);
        addrB[ks] = ring0 + A_BYTES + rb * 128 + (((2 * ks + half) ^ tile_swz(rb)) * 16);
      }
    }
    floatx16 acc = zero16();
    const int total = a.d / 64;
    int fk = 0;
#define VD_ISSUE(BUF)                                                                               \
  {                                                                                                \
    unsigned char* sp = ring + (BUF) * STAGE + wave * 1024;                                        \
    dma16(srcA[0] + fk * 64, sp);                                                                  \
    dma16(srcA[1] + fk * 64, sp + 8192);                                                           \
    dma16(srcB + fk * 64, sp + A_BYTES);                                                           \
    ++fk;                                                                                          \
  }
    VD_ISSUE(0)                         // the first slice goes ahead of the tile copies: the product starts on it
    // copies of K, Q, V, O.  A wavefront-wide copy fills 8 token rows; rows past n repeat row n-1.
    {
      const bf16_t* src[5] = {a.k + base, a.q + base, a.v + base, nullptr, a.o + base};
#pragma unroll
      for (int t = 0; t < 5; ++t) {
        if (t == 3) continue;           // the dO tile is what this block computes
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int row = (u * 8 + wave) * 8 + (lane >> 3);
          const int chunk = (lane & 7) ^ tile_swz(row);
          dma16(src[t] + (long long)min(row, n - 1) * ld + chunk * 8, smem + t * kSmallTile + (u * 8 + wave) * 1024);
        }
      }
    }
    constexpr int kTileCopies = 8;      // per wavefront
#pragma unroll
    for (int s = 1; s < NS - 1; ++s)
      if (s < total) VD_ISSUE(s)
    for (int t0 = 0; t0 < total; t0 += NS) {
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        const int t = t0 + s;
        if (t < total) {
          // slice t has landed once only younger copies are in flight: after slice 0 the tile copies and
          // the slices issued with them, later the slices issued since (the tile copies are older: done too)
          if (t == 0) {
            if (NS >= 3 && total >= 2) wait_vm<kTileCopies + LPS>(); else wait_vm<kTileCopies>();
          } else if (NS >= 3 && total - 1 - t >= 1) wait_vm<LPS>(); else wait_vm<0>();
          __builtin_amdgcn_s_barrier();
          if (t + NS - 1 < total) VD_ISSUE((s + NS - 1) % NS)
          const uint32_t so = s * STAGE;
          Frag fa[2], fb[2];
          lds_read16(fa[0].q, addrA[0] + so); lds_read16(fb[0].q, addrB[0] + so);
          lds_read16(fa[1].q, addrA[1] + so); lds_read16(fb[1].q, addrB[1] + so);
          wait_lds<2>(fa[0], fb[0]);
          acc = mfma(fb[0], fa[0], acc);
          __builtin_amdgcn_sched_barrier(0);
          lds_read16(fa[0].q, addrA[2] + so); lds_read16(fb[0].q, addrB[2] + so);
          wait_lds<2>(fa[1], fb[1]);
          acc = mfma(fb[1], fa[1], acc);
          __builtin_amdgcn_sched_barrier(0);
          lds_read16(fa[1].q, addrA[3] + so); lds_read16(fb[1].q, addrB[3] + so);
          wait_lds<2>(fa[0], fb[0]);
          acc = mfma(fb[0], fa[0], acc);
          __builtin_amdgcn_sched_barrier(0);
          wait_lds<0>(fa[1], fb[1]);
          acc = mfma(fb[1], fa[1], acc);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
#undef VD_ISSUE
#undef VD_ISSUE_W
#undef VD_ISSUE_X
    wait_vm<0>();                       // (with a single slice the tile copies can still be in flight here)
    // register 4*q4 + e of the accumulator is dO[32*blk + col][32*part + 8*q4 + 4*half + e]
    const int row = blk * 32 + col;
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int dim = part * 32 + 8 * q4 + 4 * half;
      u32x2 o;
      o.x = pack2(acc[4 * q4], acc[4 * q4 + 1]);
      o.y = pack2(acc[4 * q4 + 2], acc[4 * q4 + 3]);
      *reinterpret_cast<u32x2*>(dOs + row * 128 + (((dim >> 3) ^ tile_swz(row)) * 16) + ((dim >> 2) & 1) * 8) = o;
    }
  }
  __syncthreads();                      // the ring is free: the statistics and later dS^T may use its place
  if (threadIdx.x < kSmallN) {
    const int i = threadIdx.x;
    Ls[i] = i < n ? a.lse[srow + i] * kLog2e : INFINITY;
  }
  __syncthreads();
  // D = rowsum(dO * O), one query per lane pair
  if (part == 0) {
    const int qi = blk * 32 + col;
    float D = 0.f;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const Frag x = small_row_frag(dOs, qi, 2 * s + half), y = small_row_frag(Os, qi, 2 * s + half);
#pragma unroll
      for (int e = 0; e < 8; ++e) D = fmaf(bf2f(x.h[e]), bf2f(y.h[e]), D);
    }
    D += __shfl_xor(D, 32, 64);
    if (half == 0) Ds[qi] = D;
  }
  __syncthreads();

  // ---- phase 1: lane = key; this wavefront's query tiles are 2*part and 2*part + 1
  const float c = a.scale * kLog2e;
  const int kj = blk * 32 + col;
  floatx16 accK[2] = {zero16(), zero16()}, accV[2] = {zero16(), zero16()};
  {
    Frag kf[4], vf[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      kf[s] = small_row_frag(Ks, kj, 2 * s + half);
      vf[s] = small_row_frag(Vs, kj, 2 * s + half);
    }
#pragma unroll
    for (int q2 = 0; q2 < 2; ++q2) {
      const int qt = 2 * part + q2;
      if (qt * 32 >= n) break;
      floatx16 st = zero16(), dp = zero16();
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        st = mfma(small_row_frag(Qs, qt * 32 + col, 2 * s + half), kf[s], st);     // S[query][key]
        dp = mfma(small_row_frag(dOs, qt * 32 + col, 2 * s + half), vf[s], dp);    // dP[query][key]
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int iq = qt * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
        const float p = kj < n ? fast_exp2(st[r] * c - Ls[iq]) : 0.f;      // Ls = +inf past the last query
        st[r] = p;
        dp[r] = p * (dp[r] - Ds[iq]);
      }
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        u32x2 w;
        w.x = pack2(dp[4 * q4], dp[4 * q4 + 1]);
        w.y = pack2(dp[4 * q4 + 2], dp[4 * q4 + 3]);
        *reinterpret_cast<u32x2*>(dSt + kj * kDsPitch + (qt * 32 + 8 * q4 + 4 * half) * 2) = w;
      }
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        // registers 8*s2 .. 8*s2+7 hold queries qt*32 + 16*s2 + 4*half + {0..3} and the same + 8
        const Frag pf = regs_to_frag(st, s2);
        const Frag dsf = regs_to_frag(dp, s2);
        const int krow0 = qt * 32 + 16 * s2 + 4 * half;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) {
          accV[dt] = mfma(small_tr_frag(dOs, krow0, dt * 32, lane), pf, accV[dt]);
          accK[dt] = mfma(small_tr_frag(Qs, krow0, dt * 32, lane), dsf, accK[dt]);
        }
      }
    }
  }
  // query tiles that phase 1 skipped were never written: their dS^T columns are read below only for
  // queries >= n, whose results are not stored
  __syncthreads();                      // dS^T is complete; nobody reads the Q, V, dO, O tiles any more
  // The two wavefronts of a key block join their partial sums through LDS: the lower one hands over its
  // dV^T, the upper one its dK^T; then the lower one finishes and stores dK, the upper one dV.
  // scratch[blk][part][16-byte register quad][lane]
  {
    float4* sp = reinterpret_cast<float4*>(scratch) + (blk * 2 + part) * (8 * 64) + lane;
    const floatx16* give = part == 0 ? accV : accK;
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4)
        sp[(dt * 4 + q4) * 64] = make_float4(give[dt][4 * q4], give[dt][4 * q4 + 1], give[dt][4 * q4 + 2], give[dt][4 * q4 + 3]);
  }
  __syncthreads();
  {
    const float4* sp = reinterpret_cast<const float4*>(scratch) + (blk * 2 + (1 - part)) * (8 * 64) + lane;
    floatx16* mine = part == 0 ? accK : accV;
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const float4 v = sp[(dt * 4 + q4) * 64];
        mine[dt][4 * q4] += v.x; mine[dt][4 * q4 + 1] += v.y; mine[dt][4 * q4 + 2] += v.z; mine[dt][4 * q4 + 3] += v.w;
      }
    if (kj < n) {
      bf16_t* row = (part == 0 ? a.dk : a.dv) + base + (long long)kj * ld;
      const float mul = part == 0 ? a.scale : 1.f;
      store_accT(row, mine[0], 0, half, mul);
      store_accT(row, mine[1], 1, half, mul);
    }
  }

  // ---- phase 2: lane = query; this wavefront's half of the head dimension is dt = part
  {
    const int qi = blk * 32 + col;
    const int dt = part;
    floatx16 acc = zero16();
#pragma unroll
    for (int ks = 0; ks < kSmallN / 16; ++ks) {
      if (ks * 16 >= n) break;
      // right operand: dS^T[key][query], keys 16*ks + 8*half + e
      Frag dsf, kf;
      {
        const int mn = blk * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
#pragma unroll
        for (int rd = 0; rd < 2; ++rd) {
          const int krow = 16 * ks + 8 * half + 4 * rd + ((lane & 15) >> 2);
          const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (__attribute__((address_space(3))) s16x4*)(dSt + krow * kDsPitch + mn * 2));
          dsf.d[rd] = __builtin_bit_cast(u32x2, v);
        }
      }
      {
        // left operand: K^T[dim][key] with the standard k order: rows 16*ks + 8*half + {0..3}, + {4..7}
        const int mn = dt * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
#pragma unroll
        for (int rd = 0; rd < 2; ++rd) {
          const int krow = 16 * ks + 8 * half + 4 * rd + ((lane & 15) >> 2);
          const unsigned char* p = Ks + krow * 128 + (((mn >> 3) ^ tile_swz(krow)) * 16) + ((mn >> 2) & 1) * 8;
          const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p);
          kf.d[rd] = __builtin_bit_cast(u32x2, v);
        }
      }
      acc = mfma(kf, dsf, acc);
    }
    if (qi < n) store_accT(a.dq + base + (long long)qi * ld, acc, dt, half, a.scale);
  }
}

// ---- forward for short selections (n <= 128): one workgroup per (batch, head) computes the head's
// Q, K and V (a 128 x 192 x d product: xs of the batch times the head's columns of Wq | Wk | Wv,
// asynchronous copies four stages deep), leaves them in LDS, and runs the attention of the head on
// them; Q, K, V, O and the log-sum-exp are written for the backward pass.  Compared with a projection
// GEMM followed by an attention kernel this saves a launch and the round trip of Q, K, V through memory.
// With a selection it also gathers: the token rows are fetched through `sel`, and workgroup (batch, head)
// writes the head's 64 columns of the gathered tokens for the backward pass.
//   projection: eight wavefronts as 4 x 2, each 32 tokens x 96 columns (three matrix-instruction tiles);
//               xs tile [token][64 k] read as 16-byte fragments, weight tiles [64 k][64 columns]
//               through transposing reads; product formed transposed so that a lane owns a token.
//   attention:  a wavefront owns 32 queries (lane = query) and half of the keys; S^T = K q^T, softmax
//               over its keys, O^T = V^T P^T with V^T taken from the V tile by transposing reads; the two
//               halves of a query block are merged through LDS (maxima, sums, rescaled outputs).
struct FusedFwdArgs {
  const bf16_t* xs;               // [B][n][d]; with `sel` the tokens of all variates, [B][N][d]
  const int32_t* sel;             // optional: token row i of a batch is row sel[i] of `xs` (the gather of the
  bf16_t* xs_out;                 //   kept tokens is then part of this kernel, and they are written to xs_out)
  int N;
  const bf16_t *Wq, *Wk, *Wv;
  const bf16_t *bq, *bk, *bv;
  bf16_t *q, *k, *v, *o;
  float* lse;
  int n, d, H;
  float scale;
  const int32_t* n_dev;           // device-side token count (then n is its bound, see vd_count)
  int32_t* status;
};
constexpr int kFusedStage = kSmallN * 64 * 2 + 3 * 64 * 64 * 2;     // xs tile + three weight tiles: 40 KB
constexpr int kFusedStages = 4;                    // 160 KB: all of a compute unit's LDS (three stages: 1.5 us more per step)
constexpr int kFusedLds = kFusedStages * kFusedStage;

__global__ __launch_bounds__(512) void attn_fwd_small_bf16(FusedFwdArgs a) {
  // Eight wavefronts (two per SIMD).  Projection: wavefront w computes token rows 32*(w % 4) .. +31 of the
  // column tiles 3*(w / 4) .. +2 of [q | k | v].  Attention: wavefront w owns the queries 32*(w % 4) .. +31
  // and the key tiles 2*(w / 4), 2*(w / 4) + 1; the two partial softmax results of a query block are merged
  // through LDS.
  constexpr int NS = kFusedStages, STAGE = kFusedStage, A_BYTES = kSmallN * 64 * 2, BT = 64 * 64 * 2;
  constexpr int LPS = 5;                                        // copies per wavefront and stage: 2 of xs, 3 of weights
  constexpr int OPK = 7;                                        // LDS reads per 16-k step: 1 + 3 * 2
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wr = wave & 3, wc = wave >> 2;
  const int col = lane & 31, half = lane >> 5;
  // heads fastest: a die's contiguous range covers whole batches, whose tokens it then fetches once
  const int tix = xcd_contiguous(blockIdx.x + gridDim.x * blockIdx.y, gridDim.x * gridDim.y);
  const int h = tix % a.H, b = tix / a.H;
  const int d = a.d;
  const long long ld = d;
  const int total = d / 64;

  // ---- Start-up.  The token count and the token indices come from memory that an earlier kernel wrote, two
  // dependent round trips before the first token row can be requested.  Nothing of the weight tiles depends on
  // them: the weight copies of the first slice go out first.  The indices are requested together with the count,
  // at positions clamped by the bound of the count (the caller's `sel` is readable that far); the entries at and
  // past the count are replaced once it is known.
  const bf16_t* srcB[3];
#pragma unroll
  for (int u = 0; u < 3; ++u) {
    const bf16_t* Wz = u == 0 ? a.Wq : (u == 1 ? a.Wk : a.Wv);
    const int krow = wave * 8 + (lane >> 3);
    srcB[u] = Wz + (long long)krow * ld + h * kDh + (((lane & 7) ^ swz_nc<64>(krow)) * 8);
  }
  int fk = 0;        // slice whose copies are issued next
#define VD_ISSUE_W(BUF)                                                                             \
  {                                                                                                \
    unsigned char* sp = smem + (BUF) * STAGE + wave * 1024;                                        \
    _Pragma("unroll") for (int u = 0; u < 3; ++u)                                                  \
      dma16(srcB[u] + (long long)fk * 64 * ld, sp + A_BYTES + u * BT);                             \
  }
  VD_ISSUE_W(0)
  const int own_row = (wave & 3) * 32 + (lane & 31);         // the token this lane owns in the product below
  int spec[2] = {0, 0}, spec_own = 0, spec_first = 0;
  if (a.sel) {
#pragma unroll
    for (int u = 0; u < 2; ++u) spec[u] = a.sel[min((u * 8 + wave) * 8 + (lane >> 3), a.n - 1)];
    spec_own = a.sel[min(own_row, a.n - 1)];
    spec_first = a.sel[0];
  }
  int n;
  if (!vd_count(a.n_dev, a.n, n, a.status) || n == 0) {
    wait_vm<0>();                          // (the copies in flight write into this workgroup's LDS)
    return;
  }
  const bf16_t* xs_b = a.xs + (long long)b * (a.sel ? a.N : n) * ld;

  // ---- copy sources of the token rows.  Copy u covers token rows 8*(8u + wave) .. +7; rows past the count stand
  // for the first token (any real token: they only have to be finite, every use of them is masked).
  const bf16_t* srcA[2];
  u32x4 kept[2];                  // this thread's 16 bytes of two gathered rows, columns of head h
  int src_row[2];                 // requested here, used after the first weight copies have been issued
  bool src_ok[2] = {true, true};  // an index outside [0, N) reads row 0 and stands for a zero row, as in the gather kernel
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int row = (u * 8 + wave) * 8 + (lane >> 3);
    src_row[u] = min(row, n - 1);
    if (a.sel) {
      const int sidx = row < n ? spec[u] : spec_first;
      src_ok[u] = (unsigned)sidx < (unsigned)a.N;
      src_row[u] = src_ok[u] ? sidx : 0;
    }
  }
  // is the index of the token this lane owns valid?  (rows past the count: no matter)
  bool own_ok = true;
  if (a.sel) own_ok = own_row >= n || (unsigned)spec_own < (unsigned)a.N;
  // ---- fragment addresses relative to a stage
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
  uint32_t addrA[4], addrB[3];
  {
    const int ra = wr * 32 + col;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) addrA[ks] = lds0 + ra * 128 + (((2 * ks + half) ^ tile_swz(ra)) * 16);
  }
#pragma unroll
  for (int j = 0; j < 3; ++j) {
    const int ct = 3 * wc + j;                                   // 32-column tile of [q | k | v]
    const int krow = 8 * half + ((lane & 15) >> 2);
    const int mn = (ct & 1) * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
    addrB[j] = lds0 + A_BYTES + (ct >> 1) * BT + krow * 128 + (((mn >> 3) ^ swz_nc<64>(krow)) * 16) + ((mn >> 2) & 1) * 8;
  }
  floatx16 acc[3] = {zero16(), zero16(), zero16()};

#define VD_ISSUE_X(BUF)                                                                             \
  {                                                                                                \
    unsigned char* sp = smem + (BUF) * STAGE + wave * 1024;                                        \
    _Pragma("unroll") for (int u = 0; u < 2; ++u) dma16(srcA[u] + fk * 64, sp + u * 8192);         \
    ++fk;                                                                                          \
  }
#define VD_ISSUE(BUF) { VD_ISSUE_W(BUF) VD_ISSUE_X(BUF) }
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int row = (u * 8 + wave) * 8 + (lane >> 3);
    srcA[u] = xs_b + (long long)src_row[u] * ld + (((lane & 7) ^ tile_swz(row)) * 8);
  }
  VD_ISSUE_X(0)
#pragma unroll
  for (int s = 1; s < NS - 1; ++s)
    if (s < total) VD_ISSUE(s)
  if (a.sel) {
#pragma unroll
    for (int u = 0; u < 2; ++u)
      kept[u] = *reinterpret_cast<const u32x4*>(xs_b + (long long)src_row[u] * ld + h * kDh + (lane & 7) * 8);
  }
  for (int t0 = 0; t0 < total; t0 += NS) {
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const int t = t0 + s;
      if (t < total) {
        // slice t has landed once at most `ahead` younger slices are still in flight
        const int ahead = min(total - 1 - t, NS - 2);
        if (NS >= 4 && ahead >= 2) wait_vm<2 * LPS>();
        else if (NS >= 3 && ahead == 1) wait_vm<LPS>();
        else wait_vm<0>();
        __builtin_amdgcn_s_barrier();
        if (t + NS - 1 < total) VD_ISSUE((s + NS - 1) % NS)
        const uint32_t so = s * STAGE;
        Frag fa[2], fb[2][3];
#define VD_READ(KS_, SET)                                                                          \
  {                                                                                                \
    lds_read16(fa[SET].q, addrA[KS_] + so);                                                        \
    _Pragma("unroll") for (int j = 0; j < 3; ++j) {                                                \
      lds_read8_tr<(KS_) * 2048>(fb[SET][j].d[0], addrB[j] + so);                                  \
      lds_read8_tr<(KS_) * 2048 + 512>(fb[SET][j].d[1], addrB[j] + so);                            \
    }                                                                                              \
  }
#define VD_MMA(SET, PENDING)                                                                       \
  {                                                                                                \
    wait_lds<PENDING>(fa[SET], fb[SET][0], fb[SET][1], fb[SET][2]);                                \
    _Pragma("unroll") for (int j = 0; j < 3; ++j) acc[j] = mfma(fb[SET][j], fa[SET], acc[j]);      \
    __builtin_amdgcn_sched_barrier(0);                                                             \
  }
        VD_READ(0, 0)
        VD_READ(1, 1)
        VD_MMA(0, OPK)
        VD_READ(2, 0)
        VD_MMA(1, OPK)
        VD_READ(3, 1)
        VD_MMA(0, OPK)
        VD_MMA(1, 0)
#undef VD_READ
#undef VD_MMA
      }
    }
  }
#undef VD_ISSUE

  // a token whose index was out of range is a zero row: its products are exactly zero (the bias is still added)
  if (!own_ok) {
    acc[0] = zero16();
    acc[1] = zero16();
    acc[2] = zero16();
  }
  // ---- Q, K, V tiles (bf16, with bias) into LDS: [token][64], 16-byte chunk position XORed with token % 8
  unsigned char* Qs = smem;
  unsigned char* Ks = Qs + kSmallTile;
  unsigned char* Vs = Ks + kSmallTile;
  float* merge = reinterpret_cast<float*>(Vs + kSmallTile);     // 16-byte aligned, 4 * 2 * 5 * 64 * 16 bytes
  __syncthreads();                       // every wavefront is done with the last slice
#pragma unroll
  for (int j = 0; j < 3; ++j) {
    const int ct = 3 * wc + j, z = ct >> 1;
    const bf16_t* bias = z == 0 ? a.bq : (z == 1 ? a.bk : a.bv);
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int dim = (ct & 1) * 32 + 8 * q4 + 4 * half;
      float bv[4] = {0.f, 0.f, 0.f, 0.f};
      if (bias) {
        const u32x2 b4 = *reinterpret_cast<const u32x2*>(bias + h * kDh + dim);
        bv[0] = __uint_as_float(b4.x << 16); bv[1] = __uint_as_float(b4.x & 0xffff0000u);
        bv[2] = __uint_as_float(b4.y << 16); bv[3] = __uint_as_float(b4.y & 0xffff0000u);
      }
      const int row = wr * 32 + col;
      u32x2 o;
      o.x = pack2(acc[j][4 * q4] + bv[0], acc[j][4 * q4 + 1] + bv[1]);
      o.y = pack2(acc[j][4 * q4 + 2] + bv[2], acc[j][4 * q4 + 3] + bv[3]);
      *reinterpret_cast<u32x2*>(smem + z * kSmallTile + row * 128 + (((dim >> 3) ^ tile_swz(row)) * 16) + ((dim >> 2) & 1) * 8) = o;
    }
  }
  __syncthreads();
  // copy the tiles out for the backward pass: 16-byte chunks, eight per token row
  const long long base = (long long)b * n * ld + h * kDh;
  if (a.sel) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int row = (u * 8 + wave) * 8 + (lane >> 3);
      if (row < n)
        *reinterpret_cast<u32x4*>(a.xs_out + base + (long long)row * ld + (lane & 7) * 8) = src_ok[u] ? kept[u] : u32x4{0u, 0u, 0u, 0u};
    }
  }
#pragma unroll
  for (int u = 0; u < 3 * kSmallN * 8 / 512; ++u) {
    const int idx = u * 512 + threadIdx.x;
    const int z = idx / (kSmallN * 8), row = (idx / 8) % kSmallN, c = idx & 7;
    if (row < n) {
      bf16_t* dst = z == 0 ? a.q : (z == 1 ? a.k : a.v);
      const u32x4 v = *reinterpret_cast<const u32x4*>(smem + z * kSmallTile + row * 128 + ((c ^ tile_swz(row)) * 16));
      *reinterpret_cast<u32x4*>(dst + base + (long long)row * ld + c * 8) = v;
    }
  }

  // ---- attention: lane = query, this wavefront's key tiles are 2*wc and 2*wc + 1
  const int qi = wr * 32 + col;
  Frag qf[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) qf[s] = small_row_frag(Qs, qi, 2 * s + half);
  const float c = a.scale * kLog2e;
  floatx16 st[2];
  float m = -INFINITY;
#pragma unroll
  for (int k2 = 0; k2 < 2; ++k2) {
    const int kt = 2 * wc + k2;
    st[k2] = zero16();
    if (kt * 32 < n) {
#pragma unroll
      for (int s = 0; s < 4; ++s) st[k2] = mfma(small_row_frag(Ks, kt * 32 + col, 2 * s + half), qf[s], st[k2]);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int j = kt * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
      st[k2][r] = j < n ? st[k2][r] * c : -INFINITY;
      m = fmaxf(m, st[k2][r]);
    }
  }
  m = fmaxf(m, __shfl_xor(m, 32, 64));
  // a wavefront whose key tiles are all past n has m = -inf: its probabilities must be zero, not NaN
  const float mref = m == -INFINITY ? 0.f : m;
  float l = 0.f;
#pragma unroll
  for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      st[k2][r] = fast_exp2(st[k2][r] - mref);
      l += st[k2][r];
    }
  l += __shfl_xor(l, 32, 64);
  floatx16 out[2] = {zero16(), zero16()};
#pragma unroll
  for (int k2 = 0; k2 < 2; ++k2) {
    const int kt = 2 * wc + k2;
    if (kt * 32 < n) {
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const Frag pf = regs_to_frag(st[k2], s2);
        const int krow0 = kt * 32 + 16 * s2 + 4 * half;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) out[dt] = mfma(small_tr_frag(Vs, krow0, dt * 32, lane), pf, out[dt]);
      }
    }
  }
  // Merge the two key halves of a query block through LDS: each wavefront hands over its maximum, its
  // sum and the half of its output that the other one finishes (the lower wavefront finishes head
  // dimensions 0..31, the upper one 32..63).  merge[query block][giver][5 quads][lane]
  {
    float4* mp = reinterpret_cast<float4*>(merge) + (wr * 2 + wc) * (5 * 64) + lane;
    const floatx16& give = wc == 0 ? out[1] : out[0];
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4)
      mp[q4 * 64] = make_float4(give[4 * q4], give[4 * q4 + 1], give[4 * q4 + 2], give[4 * q4 + 3]);
    mp[4 * 64] = make_float4(m, l, 0.f, 0.f);
  }
  __syncthreads();
  {
    const float4* mp = reinterpret_cast<const float4*>(merge) + (wr * 2 + (1 - wc)) * (5 * 64) + lane;
    const float4 stat = mp[4 * 64];
    const float mm = fmaxf(m, stat.x);                   // finite: key 0 belongs to the lower half
    const float f0 = fast_exp2(m - mm), f1 = fast_exp2(stat.x - mm);
    const float lsum = l * f0 + stat.y * f1;
    if (qi < n) {
      floatx16 fin = wc == 0 ? out[0] : out[1];
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const float4 v = mp[q4 * 64];
        fin[4 * q4] = fin[4 * q4] * f0 + v.x * f1;
        fin[4 * q4 + 1] = fin[4 * q4 + 1] * f0 + v.y * f1;
        fin[4 * q4 + 2] = fin[4 * q4 + 2] * f0 + v.z * f1;
        fin[4 * q4 + 3] = fin[4 * q4 + 3] * f0 + v.w * f1;
      }
      store_accT(a.o + base + (long long)qi * ld, fin, wc, half, 1.f / lsum);
      if (wc == 0 && half == 0) a.lse[((long long)b * a.H + h) * n + qi] = (mm + log2f(lsum)) * 0.6931471805599453f;
    }
  }
}

// column sums of up to four bf16 [rows][d] matrices (bias gradients)
struct ColSumBf16 {
  const bf16_t* src[4];
  float* dst[4];
  long long rows;
  int d;
  const int32_t* n_dev;           // device-side token count: rows = n_mul * n
  int n_max, n_mul;
};
__global__ __launch_bounds__(256) void colsum_bf16_kernel(ColSumBf16 a) {
  const bf16_t* src = a.src[blockIdx.y];
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
  for (long long r = 0; r < a.rows; ++r) s += bf2f(src[r * a.d + c]);
  dst[c] = s;
}

// Launches of the kernels for long selections.  A workgroup of four wavefronts takes 128 queries (or keys)
// when that still gives the chip two workgroups per compute unit, else two wavefronts take 64.  (Two query
// groups per wavefront, QG = 2, halve the LDS reads per matrix instruction; measured, the kernels are not
// bound by those: equal at 1936 tokens, slower at 862.)  With a device-side count a.n is its bound: the grid
// and the choices below are made for the bound, and the workgroups the actual count does not need return at once.
template <typename K>
int launch_ring(vardrop_ctx* ctx, int kid, K kernel, int rows, int parts, const SdpaArgs& a, hipStream_t s) {
  const long long grid = (long long)parts * vd_ceil_div(a.n, rows) * a.H * a.B;
  if (grid >= (1ll << 31)) return VARDROP_EUNSUPPORTED;
  VdTimer timer(ctx, kid, s);
  VD_KERNEL(ctx, kernel, dim3((unsigned)grid), dim3(rows >= 128 ? 256 : 128), kRingLds, s, a);
  VD_LAUNCH_CHECK(ctx);
  return VARDROP_OK;
}
bool ring_fills(const SdpaArgs& a, int rows) { return (long long)vd_ceil_div(a.n, rows) * a.H * a.B >= 512; }
int launch_sdpa_fwd(vardrop_ctx* ctx, const SdpaArgs& a, hipStream_t s) {
  if (ring_fills(a, 128)) return launch_ring(ctx, VARDROP_K_SDPA_FWD, sdpa_fwd_bf16<4, 1>, 128, 1, a, s);
  return launch_ring(ctx, VARDROP_K_SDPA_FWD, sdpa_fwd_bf16<2, 1>, 64, 1, a, s);
}
// Fewer than three rounds of the chip's 512 workgroup places per part: both parts in one launch.  Measured per step
// at B = 32, H = 8: 1.2-1.8 % faster at 173, 205 and 321 tokens, 1.3 % at 422 (1024 workgroups per part), 0.9 % at 543
// (1280); 1 % slower at 862 (1792) and at 1936 tokens with B = 8, H = 12 (1536), where the single launch gains
// nothing and the row sums cost the dO GEMM more than they do inside the dQ kernel.
bool sdpa_bwd_paired(const SdpaArgs& a) {
  return !ring_fills(a, 128) || (long long)vd_ceil_div(a.n, 128) * a.H * a.B < 1536;   // (64-row blocks: always)
}
int launch_sdpa_bwd(vardrop_ctx* ctx, const SdpaArgs& a, hipStream_t s) {
  if (!sdpa_bwd_paired(a)) {
    const int rc = launch_ring(ctx, VARDROP_K_SDPA_BWD_DQ, sdpa_bwd_dq_bf16<4>, 128, 1, a, s);
    return rc ? rc : launch_ring(ctx, VARDROP_K_SDPA_BWD_DKV, sdpa_bwd_dkv_bf16<4>, 128, 1, a, s);
  }
  if (ring_fills(a, 128)) return launch_ring(ctx, VARDROP_K_SDPA_BWD_DQKV, sdpa_bwd_dqkv_bf16<4>, 128, 2, a, s);
  return launch_ring(ctx, VARDROP_K_SDPA_BWD_DQKV, sdpa_bwd_dqkv_bf16<2>, 64, 2, a, s);
}

}  // namespace

// largest slice count the rule above gives for any token count
// largest slice count of any token count up to n_max (the rule is not monotone)
static int splitk_bound(int d, int B, int n_max) {
  int s = 1;
  for (int n = 1; n <= n_max; ++n) s = std::max(s, vd_attn_bf16_splitk(d, (long long)B * n, nullptr));
  return s;
}
size_t vd_attn_bf16_partial_offset(int B, int n, int d, int H) {
  const size_t M = (size_t)B * n;
  return vd_align_up(4 * M * d * 2 + (size_t)2 * B * H * n * sizeof(float), 256);
}
// Room for the largest slice count, so that a workspace sized for n tokens also serves any smaller
// selection (the slice count is not monotone in the token count).
size_t vd_attn_bf16_ws_bytes(int B, int n, int d, int H) {
  return vd_attn_bf16_partial_offset(B, n, d, H) + (size_t)4 * 8 * d * d * sizeof(float);
}

// saved: q, k, v, o ([M][d] bf16 each, M = B*n) then lse fp32 [B][H][n]
// With `sel` (device, n ascending rows of [0, N)), `xs` holds the tokens of all N variates and the kept ones are
// gathered on the way: inside the fused kernel for short selections, by the gather kernel otherwise; either
// way `xs_out` [B][n][d] receives them.
// With a device-side count (dn.dev) n is its bound: the five sub-buffers of `saved` start where they would for n
// tokens, each holds its rows packed for the actual count, and the kernel path (short or long selection) is
// chosen for the bound.
int vd_attn_fwd_bf16(vardrop_ctx* ctx, const void* xs, int B, int n, int d, int H,
                     const void* const W[4], const void* const bias[4],
                     void* y, void* saved, void* ws, hipStream_t s,
                     const int32_t* sel, int N, void* xs_out, VdDevCount dn) {
  (void)ws;
  bool counted = false;          // has a kernel of this call been given dn.status yet?
  if (sel && n > kSmallN) {
    const int grc = vd_gather(ctx, xs, B, N, d, VARDROP_BF16, sel, n, xs_out, s, dn);
    if (grc) return grc;
    counted = true;
    xs = xs_out;
    sel = nullptr;
  }
  const long long M = (long long)B * n;
  bf16_t* q = (bf16_t*)saved;
  bf16_t* k = q + M * d;
  bf16_t* v = k + M * d;
  bf16_t* o = v + M * d;
  float* lse = (float*)(o + M * d);
  int rc;
  if (n <= kSmallN) {
    FusedFwdArgs f = {};
    f.xs = (const bf16_t*)xs;
    f.sel = sel;
    f.xs_out = (bf16_t*)xs_out;
    f.N = N;
    f.Wq = (const bf16_t*)W[0]; f.Wk = (const bf16_t*)W[1]; f.Wv = (const bf16_t*)W[2];
    f.bq = (const bf16_t*)bias[0]; f.bk = (const bf16_t*)bias[1]; f.bv = (const bf16_t*)bias[2];
    f.q = q; f.k = k; f.v = v; f.o = o; f.lse = lse;
    f.n = n; f.d = d; f.H = H; f.scale = 1.0f / sqrtf((float)kDh);
    f.n_dev = dn.dev; f.status = dn.status;
    static int configured_device = -1;
    if (configured_device != ctx->device) {
      VD_HIP(ctx, hipFuncSetAttribute((const void*)attn_fwd_small_bf16, hipFuncAttributeMaxDynamicSharedMemorySize, kFusedLds));
      configured_device = ctx->device;
    }
    {
      VdTimer timer(ctx, VARDROP_K_QKV_SDPA_FWD, s);
      VD_KERNEL(ctx, attn_fwd_small_bf16, dim3(H, B), dim3(512), kFusedLds, s, f);
    }
    VD_LAUNCH_CHECK(ctx);
  } else {
    GemmBf16 g = {};
    bf16_t* qkv[3] = {q, k, v};
    for (int z = 0; z < 3; ++z) g.set(z, xs, W[z], qkv[z], bias[z]);
    g.lda = d; g.ldb = d; g.ldc = d;
    g.M = (int)M; g.N = d; g.K = d; g.nseg = 1;
    if (dn.dev) g.count_rows(dn.dev, counted ? nullptr : dn.status, n, B);
    rc = vd_gemm_bf16(ctx, VARDROP_K_GEMM_QKV, g, 3, false, s);
    if (rc) return rc;
    SdpaArgs a = {};
    a.q = q; a.k = k; a.v = v; a.out = o; a.lse = lse;
    a.n = n; a.d = d; a.H = H; a.B = B; a.scale = 1.0f / sqrtf((float)kDh);
    a.n_dev = dn.dev;
    rc = launch_sdpa_fwd(ctx, a, s);
    if (rc) return rc;
  }
  GemmBf16 go = {};
  go.set(0, o, W[3], y, bias[3]);
  go.lda = d; go.ldb = d; go.ldc = d;
  go.M = (int)M; go.N = d; go.K = d; go.nseg = 1;
  if (dn.dev) go.count_rows(dn.dev, nullptr, n, B);
  return vd_gemm_bf16(ctx, VARDROP_K_GEMM_OUT, go, 1, false, s);
}

// ws: dO, dq, dk, dv ([M][d] bf16 each), D and -log2(e) lse, fp32 [B][H][n] each, then the split-K partial products
// (with a device-side count: sub-buffers placed for the bound n, rows packed for the actual count, as in the forward)
int vd_attn_bwd_bf16(vardrop_ctx* ctx, const void* dy, const void* xs, int B, int n, int d, int H,
                     const void* const W[4], const void* saved, void* dxs,
                     float* const dW[4], float* const db[4], void* ws, hipStream_t s, VdDevCount dn) {
  const long long M = (long long)B * n;
  const bf16_t* q = (const bf16_t*)saved;
  const bf16_t* k = q + M * d;
  const bf16_t* v = k + M * d;
  const bf16_t* o = v + M * d;
  const float* lse = (const float*)(o + M * d);
  bf16_t* dO = (bf16_t*)ws;
  bf16_t* dq = dO + M * d;
  bf16_t* dk = dq + M * d;
  bf16_t* dv = dk + M * d;
  float* D = (float*)(dv + M * d);
  float* nlse2 = D + (size_t)B * H * n;
  int rc;
  SdpaArgs a = {};
  a.n = n; a.d = d; a.H = H; a.B = B;
  a.n_dev = dn.dev;
  const bool paired = sdpa_bwd_paired(a);
  if (n > kSmallN) {  // dO = dy Wo^T (short selections form their dO tiles inside the attention kernel)
    GemmBf16 g = {};
    g.set(0, dy, W[3], dO, nullptr);
    g.lda = d; g.ldb = d; g.ldc = d;
    g.M = (int)M; g.N = d; g.K = d; g.nseg = 1;
    if (paired) {     // D = rowsum(dO * O) per head from the same tiles, and -log2(e) * lse beside it
      g.rs_o = o; g.rs_out = D; g.rs_n = n; g.rs_H = H;
      g.rs_aux_in = lse; g.rs_aux_out = nlse2; g.rs_aux_mul = -kLog2e;
    }
    if (dn.dev) g.count_rows(dn.dev, dn.status, n, B);
    if ((rc = vd_gemm_bf16(ctx, VARDROP_K_GEMM_DO, g, 1, true, s))) return rc;
  } else {
    a.status = dn.status;
  }
  a.q = q; a.k = k; a.v = v; a.o = o; a.dout = dO; a.lse = const_cast<float*>(lse);
  a.dq = dq; a.dk = dk; a.dv = dv; a.Dsum = D; a.nlse2 = nlse2;
  a.dy = (const bf16_t*)dy; a.wo = (const bf16_t*)W[3];
  a.scale = 1.0f / sqrtf((float)kDh);
  if (n <= kSmallN) {
    static int configured_device = -1;
    if (configured_device != ctx->device) {
      VD_HIP(ctx, hipFuncSetAttribute((const void*)sdpa_bwd_small_bf16, hipFuncAttributeMaxDynamicSharedMemorySize, kSmallLds));
      configured_device = ctx->device;
    }
    {
      VdTimer timer(ctx, VARDROP_K_SDPA_BWD, s);
      VD_KERNEL(ctx, sdpa_bwd_small_bf16, dim3(H, B), dim3(512), kSmallLds, s, a);
    }
    VD_LAUNCH_CHECK(ctx);
  } else {
    if ((rc = launch_sdpa_bwd(ctx, a, s))) return rc;
  }
  {
    // dxs = dq Wq^T + dk Wk^T + dv Wv^T
    GemmBf16 gx = {};
    const bf16_t* grads[3] = {dq, dk, dv};
    for (int z = 0; z < 3; ++z) gx.set(z, grads[z], W[z], z == 0 ? dxs : nullptr, nullptr);
    gx.lda = d; gx.ldb = d; gx.ldc = d;
    gx.M = (int)M; gx.N = d; gx.K = d; gx.nseg = 3;
    // dWq, dWk, dWv, dWo = xs^T dq, xs^T dk, xs^T dv, o^T dy, K = B*n cut into slices
    GemmBf16 gw = {};
    const bf16_t* lhs[4] = {(const bf16_t*)xs, (const bf16_t*)xs, (const bf16_t*)xs, o};
    const bf16_t* rhs[4] = {dq, dk, dv, (const bf16_t*)dy};
    for (int z = 0; z < 4; ++z) gw.set(z, lhs[z], rhs[z], dW[z], nullptr);
    gw.lda = d; gw.ldb = d; gw.ldc = d;
    gw.M = d; gw.N = d; gw.K = (int)M; gw.nseg = 1;
    int kchunk = 0;
    gw.splitk = vd_attn_bf16_splitk(d, M, &kchunk);
    gw.kchunk = kchunk;
    float* part = (float*)((char*)ws + vd_attn_bf16_partial_offset(B, n, d, H));
    gw.part = part;
    if (dn.dev) {
      // the kernels derive the slices from the count; the grid is sized for the largest number of them
      gx.count_rows(dn.dev, nullptr, n, B);
      gw.count_k(dn.dev, n, B);
      gw.splitk = splitk_bound(d, B, n);
    }
    if ((rc = vd_gemm_bf16_bwd_pair(ctx, gx, gw, 4, s))) return rc;
    // a single slice is written as the result itself
    if (gw.splitk > 1 && (rc = vd_gemm_bf16_sum_slices(ctx, part, dW, (long long)d * d, gw.splitk, s, 4, dn.dev ? &gw : nullptr))) return rc;
  }
  if (db[0] || db[1] || db[2] || db[3]) {
    ColSumBf16 c = {};
    c.src[0] = dq; c.src[1] = dk; c.src[2] = dv; c.src[3] = (const bf16_t*)dy;
    for (int z = 0; z < 4; ++z) c.dst[z] = db[z];
    c.rows = M; c.d = d;
    c.n_dev = dn.dev; c.n_max = n; c.n_mul = B;
    hipLaunchKernelGGL(colsum_bf16_kernel, dim3(vd_ceil_div(d, 256), 4), dim3(256), 0, s, c);
    VD_LAUNCH_CHECK(ctx);
  }
  return VARDROP_OK;
}

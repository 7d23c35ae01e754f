// bf16 GEMM entry points shared by the attention back end (gemm_bf16.hip).
#ifndef VARDROP_GEMM_BF16_H
#define VARDROP_GEMM_BF16_H
#include "common.h"

typedef uint16_t bf16_t;   // raw storage

// Up to four batch entries (grid z) or three accumulated segments.  Named fields rather than arrays so
// that the argument block is never indexed at run time (that would force it into private memory).
struct GemmBf16 {
  const bf16_t *A0, *A1, *A2, *A3;
  const bf16_t *B0, *B1, *B2, *B3;
  void *C0, *C1, *C2, *C3;
  const bf16_t *bias0, *bias1, *bias2, *bias3;
  int lda, ldb, ldc;
  int M, N, K;
  int nseg;           // > 1: segments accumulate into C0
  int splitk;         // > 1: every matrix z is cut into splitk K slices, slice s writes fp32 to part + (z * splitk + s) * M * N
  float* part;        //      (the partial products; with splitk == 1 the result goes to C[z] itself,
  int force_part;     //       unless force_part: then a single slice is a partial product as well)
  int kchunk;         // K elements per slice (multiple of 64)
  int a_kpad;         // != 0: the rows of a k-contiguous A hold zeros from K up to the next multiple of 64, so K
                      // itself need not be one (B must then be n-contiguous: its last k-row is re-read, times zero)
  // rs_out != nullptr (bf16 output, one matrix, N a multiple of 64): the epilogue also writes, per row m = b * rs_n + q
  // and per 64-column head h, rs_out[(b * rs_H + h) * rs_n + q] = sum_c C[m][64 h + c] * rs_o[m][64 h + c] in fp32
  // from the rounded C (rs_o has C's shape and leading dimension)
  // and, when rs_aux_out != nullptr, rs_aux_out[i] = rs_aux_mul * rs_aux_in[i] at the same index i
  const bf16_t* rs_o;
  float* rs_out;
  int rs_n, rs_H;
  const float* rs_aux_in;
  float* rs_aux_out;
  float rs_aux_mul;
  // Device-side token count (n_dev != nullptr): the kernels read n = *n_dev (at most n_max, see vd_count) and the
  // token dimension of the product becomes n_mul * n: M when n_role == 0 (with rs_n = n), K when n_role >= 1, where
  // the number and length of the K slices then follow on the device as well: from vd_attn_bf16_splitk (n_role 1)
  // or vd_embed_splitk (n_role 2).
  const int32_t* n_dev;
  int32_t* status;
  int n_max, n_mul, n_role;
  void count_rows(const int32_t* dev, int32_t* st, int nmax, int mul) { n_dev = dev; status = st; n_max = nmax; n_mul = mul; n_role = 0; }
  void count_k(const int32_t* dev, int nmax, int mul) { n_dev = dev; status = nullptr; n_max = nmax; n_mul = mul; n_role = 1; }
  void set(int z, const void* a, const void* b, void* c, const void* bias) {
    const bf16_t* pa = (const bf16_t*)a;
    const bf16_t* pb = (const bf16_t*)b;
    const bf16_t* pbias = (const bf16_t*)bias;
    switch (z) {
      case 0: A0 = pa; B0 = pb; C0 = c; bias0 = pbias; break;
      case 1: A1 = pa; B1 = pb; C1 = c; bias1 = pbias; break;
      case 2: A2 = pa; B2 = pb; C2 = c; bias2 = pbias; break;
      default: A3 = pa; B3 = pb; C3 = c; bias3 = pbias; break;
    }
  }
};

// C[z] = A[z] * op(B[z]) (+ bias) in bf16 for nz batch entries, or the sum over g.nseg segments into C[0].
// A is k-contiguous [M][K]; B is k-contiguous [N][K] (b_k_contiguous) or n-contiguous [K][N].
int vd_gemm_bf16(vardrop_ctx* ctx, int kid, const GemmBf16& g, int nz, bool b_k_contiguous, hipStream_t s);
// One launch for the input gradient gx (k-contiguous operands, up to three segments) and the nzw weight
// gradients gw (mn-contiguous operands, gw.splitk K slices, fp32 partial products in gw.part).
int vd_gemm_bf16_bwd_pair(vardrop_ctx* ctx, const GemmBf16& gx, const GemmBf16& gw, int nzw, hipStream_t s);
// out[z][i] = sum_s part[z * splitk + s][i] for four matrices of `count` elements, slices in ascending order.
// With `like` (a weight-gradient product with a device-side count) the slice count is the one that product's
// kernel derives from the count; a single slice means the product wrote its result itself and nothing is done.
int vd_gemm_bf16_sum_slices(vardrop_ctx* ctx, const float* part, float* const out[4], long long count, int splitk,
                            hipStream_t s, int nz = 4, const GemmBf16* like = nullptr);
// C = A^T * B in fp32 for one matrix, both operands mn-contiguous, K cut into g.splitk slices of g.kchunk: the
// partial products go to g.part ([splitk][M][N] fp32) when splitk > 1, the result itself (C0, ldc) when it is 1.
int vd_gemm_bf16_wgrad_split(vardrop_ctx* ctx, int kid, const GemmBf16& g, hipStream_t s);
// Sums `splitk` partial matrices ([splitk][stride] fp32, slices in ascending order) into two destinations: the first
// `count0` elements of a matrix go to out0, the next `count1` to out1 (nullable); `like`: as for vd_gemm_bf16_sum_slices.
int vd_gemm_bf16_sum_rows(vardrop_ctx* ctx, const float* part, float* out0, long long count0, float* out1, long long count1,
                          long long stride, int splitk, hipStream_t s, const GemmBf16* like);
#endif  // VARDROP_GEMM_BF16_H

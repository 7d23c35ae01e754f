// Shared device helpers of the bf16 matrix-core kernels: storage types, conversions, the operand
// fragment of v_mfma_f32_32x32x16_bf16, asynchronous global-to-LDS copies, hand-written LDS reads
// and wait counters, bank swizzles, XCD-aware workgroup order.
//
// Operand layout of the instruction (64 lanes, half = lane / 32):
//   A[i][k]: lane holds row i = lane % 32, eight k values of group `half`
//   B[k][j]: lane holds column j = lane % 32, the same eight k values
//   C[i][j]: lane holds column j = lane % 32, register r holds row 8*(r/4) + 4*half + r%4
#ifndef VARDROP_BF16_MFMA_H
#define VARDROP_BF16_MFMA_H
#include "common.h"

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // 16-byte unit of data movement (a native vector,
                                                               // so that staging arrays stay in registers)
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint16_t bf16_t;   // raw storage

namespace {



// fp32 -> bf16, round to nearest even (v_cvt_pk_bf16_f32)
__device__ inline bf16_t f2bf(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }
__device__ inline float bf2f(bf16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ inline uint32_t pack2(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  typedef float floatx2 __attribute__((ext_vector_type(2)));
  const floatx2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// 2^x on the transcendental unit (v_exp_f32, 1 ulp): arguments here are <= 0 or -inf, results below the
// normal range may flush to zero
__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

union Frag {
  u32x4 q;
  u32x2 d[2];
  uint32_t w[4];
  bf16_t h[8];
  bf16x8 v;
};

__device__ inline floatx16 zero16() {
  floatx16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  return z;
}
__device__ inline floatx16 mfma(const Frag& a, const Frag& b, floatx16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, b.v, c, 0, 0, 0);
}
// eight accumulator registers (8*s2 .. 8*s2+7) as a bf16 right-hand operand
__device__ inline Frag regs_to_frag(const floatx16& p, int s2) {
  Frag f;
#pragma unroll
  for (int e = 0; e < 4; ++e) f.w[e] = pack2(p[8 * s2 + 2 * e], p[8 * s2 + 2 * e + 1]);
  return f;
}

// ---- asynchronous copies and hand-written LDS access (see gemm_bf16.hip for why)
__device__ inline void dma16(const bf16_t* gp, unsigned char* lp) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gp,
                                   (__attribute__((address_space(3))) void*)lp, 16, 0, 0);
}
__device__ inline void lds_read16(u32x4& dst, uint32_t addr) {
  asm volatile("ds_read_b128 %0, %1" : "=v"(dst) : "v"(addr) : "memory");
}
template <int OFF>
__device__ inline void lds_read16_at(u32x4& dst, uint32_t addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF) : "memory");
}
template <int OFF>
__device__ inline void lds_read8_tr(u32x2& dst, uint32_t addr) {
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF) : "memory");
}
template <int N>
__device__ inline void wait_vm() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
// waits until at most N LDS reads are outstanding; the fragments are operands so that their uses stay behind it
template <int N>
__device__ inline void wait_lds(Frag& a, Frag& b, Frag& c, Frag& d) {
  asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a.q), "+v"(b.q), "+v"(c.q), "+v"(d.q) : "n"(N));
}
template <int N>
__device__ inline void wait_lds(Frag& a, Frag& b, Frag& c) {
  asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(a.q), "+v"(b.q), "+v"(c.q) : "n"(N));
}
template <int N>
__device__ inline void wait_lds(Frag& a, Frag& b) {
  asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a.q), "+v"(b.q) : "n"(N));
}
template <int N>
__device__ inline void wait_lds(Frag& a) {
  asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(a.q) : "n"(N));
}

// waits until at most N LDS reads are outstanding (nothing tied to it: it only keeps the counter in range)
template <int N>
__device__ inline void wait_lds_count() { asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory"); }

// Bank swizzles.  The LDS has 64 banks of 4 bytes: a 16-byte read is served 16 lanes per clock, an 8-byte read 32
// lanes per clock, and either runs at full rate when those lanes touch 256 distinct bytes modulo 256.
//   k-contiguous tile [row][BK]: 16 consecutive lanes read one 16-byte chunk of 16 consecutive rows.  With 128-byte
//   rows (BK = 64) rows r and r + 2 share their 128-byte half of the banks, so the chunk index is XORed with
//   (r >> 1) % 8; with 64-byte rows (BK = 32) four rows share 256 bytes and the XOR is (r >> 2) % 4.
//   mn-contiguous tile [k][W]: 32 consecutive lanes of a transposing read take 64 consecutive bytes of each of the
//   k-rows kr .. kr + 3 (the other half of the wavefront: kr + 8 ..).  The XOR depends on kr % 4 (and on bit 3 of kr
//   where that costs nothing), so that the +4 and +16 row offsets of a fragment's further reads keep the pattern.
template <int BK>
__device__ inline int swz_kc(int row) { return BK == 32 ? (row >> 2) & 3 : (row >> 1) & 7; }
template <int W>
__device__ inline int swz_nc(int krow) { return W == 128 ? ((krow & 3) << 2) : ((krow & 3) << 1); }
// Tile [row][64] (128-byte rows) that is read both ways, by rows (16-byte chunks of 16 consecutive rows) and by the
// transposing read (64 consecutive bytes of four consecutive rows): chunk position p of row r holds chunk
// p ^ tile_swz(r).  Bit 2 of the XOR is bit 1 of r (rows r and r + 2 share a 128-byte half of the banks; a
// transposing read then finds them in different 64-byte quarters), bits 1 and 0 are bits 2 and 3 of r, so the eight
// rows of equal parity among 16 consecutive ones all differ.  Invariant under r += 16.
__device__ inline int tile_swz(int row) { return ((row & 2) << 1) | ((row >> 1) & 2) | ((row >> 3) & 1); }
// zeroes the elements k >= kvalid of a fragment holding k = 0..7
__device__ inline void mask_frag(Frag& f, int kvalid) {
#pragma unroll
  for (int e = 0; e < 4; ++e)
    f.w[e] &= kvalid >= 2 * e + 2 ? 0xffffffffu : (kvalid == 2 * e + 1 ? 0x0000ffffu : 0u);
}

// Workgroups are handed to the eight accelerator dies (XCDs) in turn, and every die has an L2 of its
// own.  These helpers turn a workgroup's linear id into its place in an order in which each die works
// through ONE contiguous range of the tiles, so that tiles sharing an operand meet in the same L2
// instead of each die fetching its own copy from memory.
__device__ inline int xcd_range_start(int xcd, int total) { return xcd * (total >> 3) + min(xcd, total & 7); }
__device__ inline int xcd_contiguous(int id, int total) { return xcd_range_start(id & 7, total) + (id >> 3); }


}  // namespace
#endif  // VARDROP_BF16_MFMA_H

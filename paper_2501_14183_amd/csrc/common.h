// Shared host-side declarations of libvardrop (context, error plumbing, small helpers).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>
#include "../../include/vardrop.h"

static const int kProfPairs = 4096;   // event pairs held between two vardrop_profile_read calls

struct vardrop_ctx {
  int device;
  int last_hip_error;
  int prof_kid;          // kernel whose launches are bracketed by events (-1: none)
  int prof_n;            // pairs recorded since the last read
  int prof_stride;       // every prof_stride-th launch of the selected kernel is bracketed
  int prof_seen;         // launches of the selected kernel seen since it was selected
  hipEvent_t* prof_ev;   // 2 * kProfPairs events, created on first use
  short* prof_kids;      // kernel id of every recorded pair
  hipEvent_t prof_e0, prof_e1;   // the pair the next launch is to be given (null: launch untimed)
  hipEvent_t signal_event[64];   // vardrop_signal_after: the next launch of kernel id i carries signal_event[i] (null: none)
                                 // as the completion event of its own dispatch
  void* twiddle;         // device: k-DFH cosine / sine table in matrix-fragment order (kTwiddleBytes)
  int twiddle_L;         // window length the table currently holds (0: none),
  int twiddle_fmin;      //   its first candidate bin
  int twiddle_F;         //   its number of candidate bins
  int twiddle_r2;        //   and whether it is laid out for the radix-2 kernel
  int lds_per_block;     // bytes of LDS one workgroup may use
  int num_cus;           // compute units of the device
  void* static_scratch;  // device address, on this context's device, of the static scratch array of sample.hip
};

static const int kMaxHashL = 1024;                    // longest window vardrop_hash takes
static const size_t kTwiddleBytes = (size_t)2 << 20;   // 32 contraction steps x 16 bin tiles x 4 KiB

#define VD_HIP(ctx, call)                                   \
  do {                                                      \
    hipError_t e__ = (call);                                \
    if (e__ != hipSuccess) {                                \
      (ctx)->last_hip_error = (int)e__;                     \
      return VARDROP_EHIP;                                  \
    }                                                       \
  } while (0)

#define VD_LAUNCH_CHECK(ctx) VD_HIP(ctx, hipGetLastError())

// Per-kernel timing.  While the context is profiling kernel `kid` (or all kernels), a VdTimer in scope hands the one
// launch issued through VD_KERNEL during its lifetime a pair of events that the runtime ties to that dispatch itself
// (hipExtLaunchKernelGGL): their difference is the kernel's own execution time, as a profiler's kernel trace reports
// it, with no extra packet on the stream.  Costs one integer compare otherwise.
static const int kProfAll = -2;
struct VdTimer {
  vardrop_ctx* ctx;
  bool active;
  bool signal;
  VdTimer(vardrop_ctx* c, int kid, hipStream_t) : ctx(c), active(false), signal(false) {
    if (kid >= 0 && kid < 64 && c->signal_event[kid]) {     // (a launch that signals is not timed)
      signal = true;
      c->prof_e0 = nullptr;
      c->prof_e1 = c->signal_event[kid];
      c->signal_event[kid] = nullptr;
      return;
    }
    if ((c->prof_kid == kid || c->prof_kid == kProfAll) && c->prof_ev && c->prof_n < kProfPairs &&
        (c->prof_seen++ % c->prof_stride) == 0) {
      active = true;
      c->prof_kids[c->prof_n] = (short)kid;
      c->prof_e0 = c->prof_ev[2 * c->prof_n];
      c->prof_e1 = c->prof_ev[2 * c->prof_n + 1];
    }
  }
  ~VdTimer() {
    if (active) {
      ++ctx->prof_n;
      ctx->prof_e0 = ctx->prof_e1 = nullptr;
    }
    if (signal) ctx->prof_e1 = nullptr;
  }
};
#define VD_KERNEL(ctx, kernel, grid, block, lds, s, ...)                                                        \
  do {                                                                                                          \
    if ((ctx)->prof_e1) hipExtLaunchKernelGGL(kernel, grid, block, lds, s, (ctx)->prof_e0, (ctx)->prof_e1, 0, __VA_ARGS__); \
    else hipLaunchKernelGGL(kernel, grid, block, lds, s, __VA_ARGS__);                                          \
  } while (0)

// Token count of a call.  It is either the host integer `bound` itself (n_dev == nullptr) or an int32 in device
// memory that every kernel of the call reads, with `bound` as its upper limit (what the buffers were sized for).
// Returns false when the device value lies outside [0, bound]: the kernel then returns without writing to memory,
// and the first workgroup of the kernel that was handed `status` raises it.
__device__ inline bool vd_count(const int32_t* n_dev, int bound, int& n, int32_t* status = nullptr) {
  n = bound;
  if (!n_dev) return true;
  n = *n_dev;
  if ((unsigned)n <= (unsigned)bound) return true;
  if (status && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x == 0 && threadIdx.y == 0) *status = 1;
  return false;
}

__host__ __device__ static inline size_t vd_align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline bool vd_aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }
__host__ __device__ static inline int vd_ceil_div(int a, int b) { return (a + b - 1) / b; }

// Number of K slices of the weight-gradient GEMMs (K = M = B*n rows).  They share a launch with the input gradient.
// Few tokens (fewer than 512 input-gradient tiles of 128 rows): the 64 x 128 weight-gradient tiles walk over K
// beside 128-row input-gradient tiles, one workgroup per compute unit, in slices of at most 4608 rows: one slice
// up to there, so that no partial products exist (a second slice makes that launch 3.5 us shorter at the Traffic
// shape and costs a 5 us launch that sums the slices).  Many tokens: enough slices of 128 x 128 tiles for two
// workgroups per compute unit (counted as twice as many 64-row tiles), at least 256 rows each.  Slices are a
// multiple of the 64-row stage.
// (Host and device: with a device-side token count the kernels evaluate it themselves.)
__host__ __device__ static inline bool vd_attn_bf16_many_tokens(int d, long long M) {
  return (long long)vd_ceil_div((int)M, 128) * vd_ceil_div(d, 128) >= 512;
}
__host__ __device__ static inline int vd_attn_bf16_splitk(int d, long long M, int* kchunk) {
  int s;
  if (vd_attn_bf16_many_tokens(d, M)) {
    const int tiles = vd_ceil_div(d, 64) * vd_ceil_div(d, 128) * 4;
    s = vd_ceil_div(512, tiles);
    if (s > 8) s = 8;
    while (s > 1 && M / s < 256) --s;
  } else {
    s = vd_ceil_div((int)M, 4608);
  }
  if (s < 1) s = 1;
  int chunk = (int)vd_align_up((size_t)vd_ceil_div((int)M, s), 64);
  if (chunk < 64) chunk = 64;
  s = M > 0 ? vd_ceil_div((int)M, chunk) : 1;
  if (kchunk) *kchunk = chunk;
  return s;
}
size_t vd_attn_bf16_partial_offset(int B, int n, int d, int H);
size_t vd_attn_bf16_ws_bytes(int B, int n, int d, int H);

// device address of the static scratch array (sample.hip) on the current device; 0 or the hipError_t
int vd_static_scratch_address(void** out);

// strided fp32 GEMM of the fp32 back end (attn_f32.hip)
int vd_gemm_f32(vardrop_ctx*, int kid, const float* A, long long sam, long long sak,
                const float* B, long long sbk, long long sbn, float* C, int ldc, const float* bias,
                int M, int N, int K, hipStream_t s);

// attention back ends (attn_f32.hip, attn_bf16.hip); argument checks are done by the caller
// K slices of the embedding's weight gradient dWe = z^T dxs (K = B * n_sel rows; tiles of 64 x 128): enough of them
// to give the chip two workgroups per compute unit, at least 128 rows each, at most 16.  (Host and device.)
__host__ __device__ static inline int vd_embed_splitk(int L, int d, long long M, int* kchunk) {
  const int tiles = vd_ceil_div(L, 64) * vd_ceil_div(d, 128);
  int s = vd_ceil_div(512, tiles);
  if (s > 16) s = 16;
  while (s > 1 && M / s < 128) --s;
  int chunk = (int)vd_align_up((size_t)vd_ceil_div((int)M, s), 64);
  if (chunk < 64) chunk = 64;
  if (kchunk) *kchunk = chunk;
  return M > 0 ? vd_ceil_div((int)M, chunk) : 1;
}

// A count that may live in device memory (see vd_count): with dev != nullptr the `n` of the call is its bound.
struct VdDevCount {
  const int32_t* dev;
  int32_t* status;
};
int vd_attn_fwd_f32(vardrop_ctx*, const float* xs, int B, int n, int d, int H,
                    const float* const W[4], const float* const bias[4],
                    float* y, void* saved, void* ws, hipStream_t s, VdDevCount dn = {nullptr, nullptr});
int vd_attn_bwd_f32(vardrop_ctx*, const float* dy, const float* xs, int B, int n, int d, int H,
                    const float* const W[4], const void* saved, float* dxs,
                    float* const dW[4], float* const db[4], void* ws, hipStream_t s, VdDevCount dn = {nullptr, nullptr});
int vd_attn_fwd_bf16(vardrop_ctx*, const void* xs, int B, int n, int d, int H,
                     const void* const W[4], const void* const bias[4],
                     void* y, void* saved, void* ws, hipStream_t s,
                     const int32_t* sel = nullptr, int N = 0, void* xs_out = nullptr, VdDevCount dn = {nullptr, nullptr});
int vd_attn_bwd_bf16(vardrop_ctx*, const void* dy, const void* xs, int B, int n, int d, int H,
                     const void* const W[4], const void* saved, void* dxs,
                     float* const dW[4], float* const db[4], void* ws, hipStream_t s, VdDevCount dn = {nullptr, nullptr});
// gather / scatter with an optional device-side count (gather.hip); argument checks are done by the caller
int vd_gather(vardrop_ctx*, const void* tokens, int B, int N, int d, int dtype, const int32_t* sel, int n_sel,
              void* out, hipStream_t s, VdDevCount dn = {nullptr, nullptr});

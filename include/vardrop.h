/*
 * vardrop.h -- C ABI of the VarDrop training hot path for AMD MI355X (gfx950).
 *
 * One training step of VarDrop (arXiv 2501.14183, Sec. 3, Fig. 2) is
 *   k-dominant frequency hashing of every variate of a batch  (vardrop_hash)
 *   -> grouping by hash + stratified sampling of representatives (vardrop_sample)
 *   -> gather of the kept variate tokens                       (vardrop_gather)
 *   -> multi-head scaled dot-product attention over the kept tokens, forward and
 *      backward                                               (vardrop_attn_fwd / _bwd).
 *
 * General rules
 *   - Every pointer is a DEVICE pointer owned by the caller unless its name ends in
 *     "_host".  The library never frees or keeps caller memory.
 *   - Every call only enqueues work on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream) and returns without waiting, except where stated.
 *   - Scratch memory comes from the caller: ask the matching *_workspace_bytes function
 *     and pass a buffer of at least that size, 256-byte aligned.  The library allocates
 *     device memory only inside vardrop_create.
 *   - Return value: VARDROP_OK (0) or a negative error code.  On an argument error
 *     nothing is enqueued and no output is touched.  Nothing throws, nothing aborts.
 *   - A context serves one device and one host thread at a time.  Work enqueued through one context on
 *     different streams may overlap on the device, with one exception: the context keeps ONE cosine / sine
 *     table for vardrop_hash, rebuilt (on the call's stream) whenever L, f_min or f_max differ from the
 *     previous vardrop_hash call, so two vardrop_hash calls with different (L, f_min, f_max) must be ordered
 *     by their streams (same stream, or an event between them); give each stream a context of its own to
 *     lift that.  The timing hook below is host-side state of the context.
 *   - Device-side token count.  The number of kept tokens N' is a result of vardrop_sample and lives in
 *     device memory (counts[0]).  The entry points whose names end in _dev take a pointer to it instead of
 *     a host integer, plus an upper bound n_max that sizes buffers and launches: nothing has to cross to the
 *     host between sampling and attention, and since no launch parameter depends on N' a whole step can be
 *     recorded once (a HIP graph) and replayed.  Rows are packed for the actual count, [B][N'][d], exactly
 *     as the host-count entry points lay them out, in buffers sized for n_max.  If the device value is
 *     outside [0, n_max] the call's kernels do nothing, and *status (device int32, optional) is set to 1;
 *     the library never clears it.
 */
#ifndef VARDROP_H
#define VARDROP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct vardrop_ctx vardrop_ctx;

enum {
  VARDROP_OK = 0,
  VARDROP_EINVAL = -1,       /* null pointer, size or parameter out of range            */
  VARDROP_EWORKSPACE = -2,   /* workspace missing, misaligned or too small               */
  VARDROP_EHIP = -3,         /* a HIP call failed; see vardrop_last_hip_error            */
  VARDROP_EUNSUPPORTED = -4  /* valid request outside what the kernels implement         */
};

enum { VARDROP_F32 = 0, VARDROP_BF16 = 1 };   /* element type of tokens / weights */

/* Creates a context on HIP device `device_id` (allocates a 2 MiB cosine / sine table there).
 * Synchronous. */
int vardrop_create(vardrop_ctx** out, int device_id);
void vardrop_destroy(vardrop_ctx* ctx);
/* Static, never-null description of an error code. */
const char* vardrop_strerror(int code);
/* hipError_t of the last failed HIP call made through this context (0 if none). */
int vardrop_last_hip_error(const vardrop_ctx* ctx);

/* ---------------------------------------------------------------------------------
 * Per-kernel timing for benchmarks.  While a kernel id is selected, every launch of that kernel is issued
 * with a pair of HIP events tied to the dispatch itself (hipExtLaunchKernelGGL), whose difference is the
 * kernel's own execution time: no extra packet goes onto the stream, and the figure is the one a profiler's
 * kernel trace reports.  At most 4096 launches are recorded between two reads.  VARDROP_K_ALL times every
 * kernel.  vardrop_profile_read waits for the recorded launches, returns their summed duration in
 * milliseconds and their number, and starts a new collection; vardrop_profile_read_all does the same per
 * kernel id (both arrays hold VARDROP_K_COUNT entries).  Selecting -1 switches the timing off (the default).
 * vardrop_profile_stride(ctx, s) times only every s-th eligible launch (s >= 1, default 1; takes effect at the
 * next vardrop_profile_select).  Launches recorded into a HIP graph are not timed: select -1 before a capture.
 */
enum { VARDROP_K_ALL = -2 };
enum {
  VARDROP_K_HASH = 0,        /* k-DFH: spectrum, batch mean, ranked top-k, hash            */
  VARDROP_K_SAMPLE,          /* grouping + stratified sampling                              */
  VARDROP_K_GATHER,          /* gather of the kept tokens                                   */
  VARDROP_K_GEMM_QKV,        /* [Q|K|V] = xs [Wq|Wk|Wv]                                     */
  VARDROP_K_SDPA_FWD,        /* softmax(Q K^T / sqrt(d_k)) V                                */
  VARDROP_K_GEMM_OUT,        /* y = O Wo                                                    */
  VARDROP_K_GEMM_DO,         /* dO = dy Wo^T                                                */
  VARDROP_K_SDPA_BWD_DQ,     /* dQ and rowsum(dO * O)                                       */
  VARDROP_K_SDPA_BWD_DKV,    /* dK, dV                                                      */
  VARDROP_K_GEMM_DW,         /* dWq, dWk, dWv, dWo (K slices)                               */
  VARDROP_K_REDUCE_DW,       /* sum of the K slices                                         */
  VARDROP_K_GEMM_DXS,        /* dxs = dQ Wq^T + dK Wk^T + dV Wv^T                           */
  VARDROP_K_SCATTER,         /* adjoint of the gather                                       */
  VARDROP_K_GEMM_DW_DXS,     /* weight gradients (K slices) and dxs in one launch           */
  VARDROP_K_SDPA_BWD,        /* dQ, dK, dV of a short selection (n <= 128) in one launch    */
  VARDROP_K_QKV_SDPA_FWD,    /* Q, K, V projection and attention of a short selection       */
  VARDROP_K_EMBED_ROWS,      /* kept windows: gather from the raw batch, standardise, convert */
  VARDROP_K_GEMM_EMBED,      /* xs = z We + be                                              */
  VARDROP_K_GEMM_DWE,        /* dWe = z^T dxs (K slices)                                    */
  VARDROP_K_SDPA_BWD_DQKV,   /* bf16, n > 128, few workgroups: dQ, dK, dV in one launch (GEMM_DO then forms rowsum(dO * O)) */
  VARDROP_K_EMBED_FUSED,     /* kept windows gathered, standardised and embedded in one launch (bf16, short windows) */
  VARDROP_K_COUNT
};
int vardrop_profile_select(vardrop_ctx* ctx, int kernel_id);
int vardrop_profile_read(vardrop_ctx* ctx, double* total_ms, int* launches);
int vardrop_profile_read_all(vardrop_ctx* ctx, double* total_ms, int* launches);
int vardrop_profile_stride(vardrop_ctx* ctx, int stride);
/* Completion signal without a stream packet.  The next launch of kernel `kernel_id` through this context carries
 * `event` (a hipEvent_t created by the caller; NULL cancels) as the completion event of its own dispatch: the event
 * is complete when that kernel has finished, exactly as if it had been recorded on the stream right behind the
 * kernel, but no packet of its own is put between two kernels of the stream (a recorded event holds the next kernel
 * up by a few microseconds).  One-shot: the request is consumed by that launch, which is then not timed by the
 * profiling hook; one request can be pending per kernel id.  A second stream can wait for the event (hipStreamWaitEvent after the call that launched the
 * kernel has returned) to start work beside a chosen kernel of this stream.  Launches recorded into a HIP graph
 * must not carry one.  Returns VARDROP_EINVAL for an unknown id. */
int vardrop_signal_after(vardrop_ctx* ctx, int kernel_id, void* event);
/* Static name of a kernel id ("hash", "gemm_qkv", ...), or NULL when out of range. */
const char* vardrop_kernel_name(int kernel_id);

/* ---------------------------------------------------------------------------------
 * k-dominant frequency hashing -- Alg. 1 and Def. 1 of the paper.
 *
 * For every variate n: amplitude spectrum |X_f| of each of its B windows (step 1) on the
 * candidate bins f_min..f_max only (low-pass, step 2; the paper's cut-off epsilon is the
 * number of candidate bins, 25 for T = 96, App. E), mean over the B windows (step 3), the
 * k bins of largest mean amplitude in descending order, ties to the lower bin (step 4),
 * and hash[n] = sum_j topk[n][j] * R^(k-1-j) with R = floor(L/2)+1 (step 5).
 *
 *   x      fp32 [B][N][L] with element strides sb, sn >= 0 and st >= 1.  The kernel reads time-contiguous
 *          rows (st = 1).  Any other layout -- in particular a time-major batch [B][L][N], sb = L N,
 *          sn = 1, st = N -- is first copied into time-contiguous rows in the workspace `ws`, which
 *          must then hold vardrop_hash_strided_workspace_bytes(B, N, L) bytes, 16-byte aligned
 *          (EWORKSPACE otherwise; B <= 65535 on this path); with st = 1 no workspace is used
 *   topk   int32 [N][k]   bin indices, rank 1 first
 *   hash   uint64 [N]
 *   abar   fp32 [N][f_max-f_min+1] mean amplitudes, or NULL
 * f_max < 0 selects the paper's default cut-off, vardrop_hash_default_cutoff(L) = ceil((floor(L/2)+1)/2)
 * ("half of the number of positive frequencies", 25 at T = 96, App. E); f_min < 0 selects 1 (the mean, bin 0,
 * is not a candidate: App. G prints the hash of a flat variate as 1-2-3).
 * Requires 1 <= k <= f_max-f_min+1, 0 <= f_min <= f_max <= floor(L/2), R^k < 2^63,
 * 2 <= L <= 1024, at most 512 candidate bins, and operand buffers that fit the 160 KiB LDS:
 * 2048 P + 1024 + 4 V (f_max-f_min+1) bytes with P = 2 ceil(ceil(L/2) / 16) + 1, or
 * 4096 P + 1024 + 4 V (f_max-f_min+1) with P = 2 ceil(L / 64) + 1 when the window length is a multiple
 * of 8 from 136 on and the rows are 16-byte aligned (x, sb, sn), where the kernel halves the
 * contraction length; V = 32/min(32, B rounded up to a power of two).  Always true for L <= 768 (EUNSUPPORTED
 * otherwise).  N == 0 is a no-op.  Arithmetic: the spectrum is contracted on the half-precision
 * matrix cores with every operand split into two fp16 pieces and fp32 accumulation, which is
 * as exact as fp32 arithmetic (mean amplitudes within 1e-6 of the largest one of the variate);
 * ranks agree with an exact evaluation whenever neighbouring amplitudes differ by much more than 1e-6
 * relative.  Non-finite inputs give unspecified ranks.
 */
size_t vardrop_hash_workspace_bytes(int B, int N, int L, int k, int f_min, int f_max);   /* st = 1: none */
size_t vardrop_hash_strided_workspace_bytes(int B, int N, int L);                          /* st != 1 */
int vardrop_hash_default_cutoff(int L);                                                    /* 0 when L < 2 */
int vardrop_hash(vardrop_ctx* ctx, const float* x, int B, int N, int L,
                 int64_t sb, int64_t sn, int64_t st, int k, int f_min, int f_max,
                 int32_t* topk, uint64_t* hash, float* abar,
                 void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------
 * Grouping and stratified sampling -- Sec. 3.3, Eq. 1-2.
 *
 * Variates with equal hash form a group; group ids number the distinct hashes in
 * ascending order.  A group of size g keeps
 *     n_i = min(g, gs', max(1, ceil(g * ratio_num / ratio_den)))   (gs' = gs, or no cap if gs == 0)
 * members; ratio 1/1 leaves Eq. 1, |S_i| = min(|G_i|, gs), as printed.  "Random": variate n
 * draws u[n] = r0<<32|r1 from Philox4x32-10 with counter (n, 0, step_lo, step_hi) and key
 * (seed_lo, seed_hi); a group keeps the members with the smallest (u[n], n).
 *
 *   hash      uint64 [N]
 *   group_id  int32 [N]
 *   sel       int32 [N] capacity; the first N' entries are the kept variates, ascending
 *   counts    int32 [2] = {N', G}
 *   counts_host  optional HOST pointer (pinned memory recommended): receives the same two
 *             values through an asynchronous copy on `stream`; valid after the stream is
 *             synchronised.
 * Requires 1 <= N <= 8192 (EUNSUPPORTED above), ratio_num <= ratio_den, ratio_den > 0.
 */
size_t vardrop_sample_workspace_bytes(int N);
int vardrop_sample(vardrop_ctx* ctx, const uint64_t* hash, int N,
                   uint32_t gs, uint32_t ratio_num, uint32_t ratio_den,
                   uint64_t seed, uint64_t step,
                   int32_t* group_id, int32_t* sel, int32_t* counts, int32_t* counts_host,
                   void* ws, size_t ws_bytes, void* stream);

/* vardrop_sample with the Philox step counter in device memory: the kernel reads *step_dev (8-byte aligned
 * device uint64) where vardrop_sample takes `step`, and with advance != 0 stores *step_dev + 1 back once the
 * draw is done, so that a recorded launch draws a new selection at every replay (Sec. 3.3: a fresh random
 * sample per training step).  No host copy of the counts: they stay in `counts`.  Calls that share a step_dev
 * must be ordered by their streams. */
int vardrop_sample_dev(vardrop_ctx* ctx, const uint64_t* hash, int N,
                       uint32_t gs, uint32_t ratio_num, uint32_t ratio_den,
                       uint64_t seed, uint64_t* step_dev, int advance,
                       int32_t* group_id, int32_t* sel, int32_t* counts,
                       void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------
 * Deterministic representatives -- Sec. 3.3 leaves the sampling method open ("not limited to any
 * specific sampling method").  Groups, group ids and the number n_i a group keeps are those of
 * vardrop_sample; instead of a random draw a group keeps the n_i members whose mean amplitude spectrum
 * (abar of vardrop_hash) lies closest to the group's mean spectrum, ties to the lower variate index:
 *     mean_g[f] = (sum of abar[n][f] over the members n of g, ascending n) / |g|
 *     d[n]      = sum over f (ascending) of (abar[n][f] - mean_g[f])^2
 * in IEEE single precision without fused multiply-add, so that the selection is reproducible bit for
 * bit by any implementation that follows this order.
 *
 *   abar   fp32 [N][F], F = number of candidate bins
 *   ws     vardrop_sample_nearest_workspace_bytes(N, F), 256-byte aligned
 * Other arguments, outputs and limits as vardrop_sample.  Cost: the grouping pass runs twice and the
 * group means take O(G N F) operations; meant for the selection of fixed representatives, not tuned
 * like the random sampler.
 */
size_t vardrop_sample_nearest_workspace_bytes(int N, int F);
int vardrop_sample_nearest(vardrop_ctx* ctx, const uint64_t* hash, const float* abar, int N, int F,
                           uint32_t gs, uint32_t ratio_num, uint32_t ratio_den,
                           int32_t* group_id, int32_t* sel, int32_t* counts_dev, int32_t* counts_host,
                           void* ws, size_t ws_bytes, void* stream);

/* vardrop_sample_nearest for callers that cannot allocate device memory or hand over a workspace (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the group means and the distance keys
 * live in a static device array of the library (4 MiB + 64 KiB per device, held until the process ends), whose
 * address vardrop_create takes for its device.  Limits: N <= 8192 and N * F <= 2^20 (EUNSUPPORTED beyond).  The call
 * itself allocates nothing and has no host copy of the counts.  Every call on a device shares that array: calls that
 * overlap in time on one device (any contexts, any streams) race and must be ordered by the caller.  Results are
 * identical to vardrop_sample_nearest. */
int vardrop_sample_nearest_noalloc(vardrop_ctx* ctx, const uint64_t* hash, const float* abar, int N, int F,
                                   uint32_t gs, uint32_t ratio_num, uint32_t ratio_den,
                                   int32_t* group_id, int32_t* sel, int32_t* counts_dev, void* stream);

/* ---------------------------------------------------------------------------------
 * Gather of the kept tokens (Sec. 3.1: attention runs on the selected tokens only) and
 * its adjoint.
 *
 *   gather :  out[b][i][:]     = tokens[b][sel[i]][:]          out [B][n_sel][d]
 *   scatter:  dtokens[b][n][:] = dxs[b][i][:] if n == sel[i], else 0   (every row written)
 * tokens / dtokens are [B][N][d]; dtype is VARDROP_F32 or VARDROP_BF16.  sel must be
 * ascending and within 0..N-1 (as vardrop_sample writes it); an out-of-range entry
 * yields a zero row.  n_sel == 0 is a no-op for gather; scatter then zero-fills.
 */
int vardrop_gather(vardrop_ctx* ctx, const void* tokens, int B, int N, int d, int dtype,
                   const int32_t* sel, int n_sel, void* out, void* stream);
int vardrop_scatter(vardrop_ctx* ctx, const void* dxs, int B, int N, int d, int dtype,
                    const int32_t* sel, int n_sel, void* dtokens, void* stream);

/* The same with a device-side token count (see the general rules): n_sel_dev points to N' (device int32),
 * n_sel_max <= N bounds it; out is [B][N'][d] packed, in a buffer of at least B * n_sel_max * d elements. */
int vardrop_gather_dev(vardrop_ctx* ctx, const void* tokens, int B, int N, int d, int dtype,
                       const int32_t* sel, const int32_t* n_sel_dev, int n_sel_max, int32_t* status,
                       void* out, void* stream);
int vardrop_scatter_dev(vardrop_ctx* ctx, const void* dxs, int B, int N, int d, int dtype,
                        const int32_t* sel, const int32_t* n_sel_dev, int n_sel_max, int32_t* status,
                        void* dtokens, void* stream);

/* ---------------------------------------------------------------------------------
 * Token embedding of the kept variates only -- Sec. 3.1 / 3.3: the reduction works directly from the raw
 * variates, so the tokens of the dropped ones never have to be formed.  A token is the shared linear map
 * R^L -> R^d of one variate's whole lookback window (the variate tokenisation of the backbone, Sec. 4.1):
 *
 *   z[b][i][:]  = window sel[i] of batch element b; with standardise != 0 brought to zero mean and unit
 *                 (population) variance over time, a constant window becoming zeros
 *   xs[b][i][:] = z[b][i][:] We (+ be)                         xs [B][n_sel][d], element type `dtype`
 *   backward:     dWe = sum_{b,i} z[b][i][:]^T dxs[b][i][:],  dbe = sum_{b,i} dxs[b][i][:]
 *                 (the windows are data: there is no gradient with respect to x)
 *
 *   x      fp32 [B][N][L], element strides sb, sn, time contiguous
 *   sel    device int32 [n_sel], entries within 0..N-1 (an out-of-range entry gives a zero window)
 *   We     [L][d] row-major, `dtype`;  be [d], `dtype`, NULL = none
 *   saved  vardrop_embed_saved_bytes: the windows z in `dtype` (VARDROP_BF16: rows zero-padded to a
 *          multiple of 64 samples; windows of at most 383 samples carry a one at position L, which makes the
 *          bias gradient a row of the same product as dWe); written by fwd, read by bwd; 256-byte aligned
 *   dWe    fp32 [L][d], overwritten;  dbe fp32 [d], overwritten, NULL = skip
 *   ws     bwd only: vardrop_embed_workspace_bytes (partial sums of the gradients), 256-byte aligned
 * VARDROP_BF16 rounds z to bf16 and multiplies on the matrix cores with fp32 accumulation; it requires
 * d % 8 == 0, L % 8 == 0 and B*n_sel*max(d, L+63) < 2^31.  VARDROP_F32 is plain fp32.  2 <= L <= 1024.
 * n_sel == 0 is a no-op for fwd; bwd then zero-fills the gradients.
 * VARDROP_BF16 windows of at most 383 samples take one kernel forward (gather through sel, standardisation and
 * the product: the standardised window is formed inside the product's operand load and written to `saved` on
 * the way) and one product plus its slice sum backward; longer windows and VARDROP_F32 take a standardisation
 * kernel followed by the product.  The _dev variants read the count of kept windows on the device (see the
 * general rules; xs and dxs packed [B][N'][d]; sizes for n_max; single-kernel path only, EUNSUPPORTED otherwise).
 */
size_t vardrop_embed_saved_bytes(int B, int n_sel, int L, int dtype);
size_t vardrop_embed_workspace_bytes(int B, int n_sel, int L, int d, int dtype);
int vardrop_embed_fwd(vardrop_ctx* ctx, const float* x, int B, int N, int L, int64_t sb, int64_t sn,
                      const int32_t* sel, int n_sel, int standardise,
                      const void* We, const void* be, int d, int dtype,
                      void* xs, void* saved, void* stream);
int vardrop_embed_bwd(vardrop_ctx* ctx, const void* dxs, int B, int n_sel, int L, int d, int dtype,
                      const void* saved, float* dWe, float* dbe,
                      void* ws, size_t ws_bytes, void* stream);
int vardrop_embed_fwd_dev(vardrop_ctx* ctx, const float* x, int B, int N, int L, int64_t sb, int64_t sn,
                          const int32_t* sel, const int32_t* n_dev, int n_max, int32_t* status, int standardise,
                          const void* We, const void* be, int d, int dtype,
                          void* xs, void* saved, void* stream);
int vardrop_embed_bwd_dev(vardrop_ctx* ctx, const void* dxs, int B, const int32_t* n_dev, int n_max, int L, int d,
                          int dtype, const void* saved, float* dWe, float* dbe,
                          void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------
 * Multi-head scaled dot-product attention over the kept tokens -- Eq. 3,
 * softmax(Q K^T / sqrt(d_k)) V, with d_k = d / H; no mask, no dropout.
 *
 *   Q = xs Wq (+bq), K = xs Wk (+bk), V = xs Wv (+bv), heads = H contiguous chunks of d,
 *   O = concat_h softmax(Q_h K_h^T / sqrt(d_k)) V_h,  y = O Wo (+bo).
 *
 *   xs, y, dy, dxs   [B][n][d]        element type `dtype`
 *   Wq, Wk, Wv, Wo   [d][d] row-major (y = x W), `dtype`; biases [d], `dtype`, NULL = none
 *   saved            vardrop_attn_saved_bytes: Q, K, V, O in `dtype` and the row log-sum-exp
 *                    in fp32; written by fwd, read by bwd
 *   dWq..dWo         fp32 [d][d], overwritten;  dbq..dbo fp32 [d], overwritten, NULL = skip
 * VARDROP_BF16 multiplies bf16 operands on the matrix cores with fp32 accumulation and
 * fp32 softmax, and requires d_k == 64 and d % 64 == 0; VARDROP_F32 is plain fp32 and
 * requires d_k in {16, 32, 64, 128}.  n == 0 is a no-op (weight gradients zero-filled).
 * The backward recomputes the attention probabilities from Q, K and the saved
 * log-sum-exp; it does not store them.  VARDROP_BF16 also requires B*n*d < 2^31
 * (EUNSUPPORTED otherwise).  Sizes returned for n tokens also serve any call with fewer
 * tokens (same B, d, H), so buffers can be sized once for the largest selection.
 */
size_t vardrop_attn_saved_bytes(int B, int n, int d, int H, int dtype);
size_t vardrop_attn_workspace_bytes(int B, int n, int d, int H, int dtype);
int vardrop_attn_fwd(vardrop_ctx* ctx, const void* xs, int B, int n, int d, int H, int dtype,
                     const void* Wq, const void* Wk, const void* Wv, const void* Wo,
                     const void* bq, const void* bk, const void* bv, const void* bo,
                     void* y, void* saved, void* ws, size_t ws_bytes, void* stream);
/* vardrop_gather followed by vardrop_attn_fwd in one call (Sec. 3.3: attention runs on the selected
 * tokens): `tokens` [B][N][d] holds all variates, `sel` (device, int32) the n kept rows in ascending
 * order; `xs` [B][n][d] receives the kept tokens (the backward pass needs them), y and `saved` are
 * those of vardrop_attn_fwd.  For VARDROP_BF16 and n <= 128 the gather happens inside the forward
 * kernel, which saves a launch; otherwise the two steps run one after the other.  Results are
 * identical to the two separate calls.  Also requires n <= N and, for VARDROP_BF16, B*N*d < 2^31. */
int vardrop_gather_attn_fwd(vardrop_ctx* ctx, const void* tokens, int B, int N, const int32_t* sel, int n,
                            int d, int H, int dtype,
                            const void* Wq, const void* Wk, const void* Wv, const void* Wo,
                            const void* bq, const void* bk, const void* bv, const void* bo,
                            void* xs, void* y, void* saved, void* ws, size_t ws_bytes, void* stream);
int vardrop_attn_bwd(vardrop_ctx* ctx, const void* dy, const void* xs,
                     int B, int n, int d, int H, int dtype,
                     const void* Wq, const void* Wk, const void* Wv, const void* Wo,
                     const void* saved,
                     void* dxs, float* dWq, float* dWk, float* dWv, float* dWo,
                     float* dbq, float* dbk, float* dbv, float* dbo,
                     void* ws, size_t ws_bytes, void* stream);

/* vardrop_gather_attn_fwd and vardrop_attn_bwd with a device-side token count (see the general rules; Eq. 2:
 * the selection S, and with it N' = |S|, is data of the step, not a host quantity).  n_dev points to N',
 * 1 <= n_max <= N bounds it.  `sel` must be readable up to n_max entries (those from N' on are ignored; the
 * selection vardrop_sample writes has N).  xs, y, dy, dxs are [B][N'][d] packed in buffers of at least B * n_max * d
 * elements; `saved` and `ws` are sized by vardrop_attn_saved_bytes / vardrop_attn_workspace_bytes for n_max, and
 * the backward call must be given the same n_max as the forward call that wrote `saved`.  The kernels are chosen
 * for n_max (VARDROP_BF16: the single-kernel path of short selections when n_max <= 128), results are those of
 * the host-count entry points called with N'.  N' == 0 leaves y, xs, dxs untouched and zero-fills the weight
 * gradients.  *status as in the general rules (forward and backward may share one). */
int vardrop_gather_attn_fwd_dev(vardrop_ctx* ctx, const void* tokens, int B, int N, const int32_t* sel,
                                const int32_t* n_dev, int n_max, int32_t* status,
                                int d, int H, int dtype,
                                const void* Wq, const void* Wk, const void* Wv, const void* Wo,
                                const void* bq, const void* bk, const void* bv, const void* bo,
                                void* xs, void* y, void* saved, void* ws, size_t ws_bytes, void* stream);
/* vardrop_attn_fwd with a device-side token count, for tokens that are already packed [B][N'][d]. */
int vardrop_attn_fwd_dev(vardrop_ctx* ctx, const void* xs, int B, const int32_t* n_dev, int n_max, int32_t* status,
                         int d, int H, int dtype,
                         const void* Wq, const void* Wk, const void* Wv, const void* Wo,
                         const void* bq, const void* bk, const void* bv, const void* bo,
                         void* y, void* saved, void* ws, size_t ws_bytes, void* stream);
int vardrop_attn_bwd_dev(vardrop_ctx* ctx, const void* dy, const void* xs,
                         int B, const int32_t* n_dev, int n_max, int32_t* status, int d, int H, int dtype,
                         const void* Wq, const void* Wk, const void* Wv, const void* Wo,
                         const void* saved,
                         void* dxs, float* dWq, float* dWk, float* dWv, float* dWo,
                         float* dbq, float* dbk, float* dbv, float* dbo,
                         void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* VARDROP_H */

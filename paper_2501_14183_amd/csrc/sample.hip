// Grouping by hash and stratified sampling (Sec. 3.3, Eq. 1-2) in one workgroup.
//
// N <= 8192 variates fit the LDS of one compute unit, so a single workgroup does the whole
// step without global round trips:
//   1. order the variates by (hash, n): 1024 order-preserving buckets over [min, max] of the hashes, the
//      place of a pair inside its bucket by counting; inputs that crowd one bucket fall back to a bitonic
//      sort of packed (hash, n) keys (registers, lane shuffles, LDS for the widest strides)
//   2. head flags + block scan              -> dense group id (ascending hash), start, size
//   3. u[n] from Philox4x32-10, counter (n, 0, step_lo, step_hi), key (seed_lo, seed_hi); the rank of a
//      member inside its group by counting over the group (groups above 1024 members: a second sort by
//      (group, u[n], n)); a member is kept when its rank is below n_i.
//      Up to 4096 variates steps 1 and 3 are one: u[n] is drawn while the hashes are on their way from memory, the
//      count inside a bucket orders by (hash, u[n], n), and the rank of a member inside its group is its
//      distance from the group's start.
//   4. flags by variate + block scan        -> sel ascending, N'
#include "common.h"

namespace {

constexpr int kMaxN = 8192;

__device__ inline void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                     uint32_t k0, uint32_t k1, uint32_t& r0, uint32_t& r1) {
  const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
    const uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
    c0 = hi1 ^ c1 ^ k0;
    c1 = lo1;
    c2 = hi0 ^ c3 ^ k1;
    c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  r0 = c0;
  r1 = c1;
}

// order of sort 1: (key, payload) lexicographic; payload = variate index (padding: >= N)
__device__ inline bool less_hash(uint64_t ka, uint32_t pa, uint64_t kb, uint32_t pb) {
  return ka < kb || (ka == kb && pa < pb);
}
// order of sort 2: payload = group << 16 | n; (group, key, n) lexicographic
__device__ inline bool less_group(uint64_t ka, uint32_t pa, uint64_t kb, uint32_t pb) {
  const uint32_t ga = pa >> 16, gb = pb >> 16;
  if (ga != gb) return ga < gb;
  if (ka != kb) return ka < kb;
  return (pa & 0xffffu) < (pb & 0xffffu);
}

// Bitonic sort of npad = E * blockDim.x (key, payload) pairs, E consecutive elements per thread
// (element i = tid * E + e).  A compare-exchange with partner i ^ stride stays inside the thread
// for stride < E, inside the wavefront (lane shuffles) for stride < 64 * E, and only goes through
// LDS above that, which leaves a handful of barrier-separated passes instead of log^2(npad) / 2.
template <bool kByGroup>
__device__ inline bool pair_less(uint64_t ka, uint32_t pa, uint64_t kb, uint32_t pb) {
  return kByGroup ? less_group(ka, pa, kb, pb) : less_hash(ka, pa, kb, pb);
}

// compare-exchange of the register pairs (e, e ^ S) of one thread; all indices are compile-time
template <int E, int S, bool kByGroup>
__device__ inline void in_thread_exchange(uint64_t (&k)[E], uint32_t (&p)[E], int tid, int size) {
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const int f = e ^ S;
    if (f > e && f < E) {
      const bool up = ((tid * E + e) & size) == 0;
      const bool f_less = pair_less<kByGroup>(k[f], p[f], k[e], p[e]);
      if (f_less == up) {
        const uint64_t tk = k[e];
        const uint32_t tp = p[e];
        k[e] = k[f];
        p[e] = p[f];
        k[f] = tk;
        p[f] = tp;
      }
    }
  }
}

// The same network for bare keys of type K (uint32_t or uint64_t), ascending: one or two shuffles
// and one compare per exchange.
__device__ inline uint32_t lane_xor(uint32_t v, int d) { return __shfl_xor(v, d, 64); }
__device__ inline uint64_t lane_xor(uint64_t v, int d) {
  const uint32_t lo = __shfl_xor((uint32_t)v, d, 64);
  const uint32_t hi = __shfl_xor((uint32_t)(v >> 32), d, 64);
  return ((uint64_t)hi << 32) | lo;
}

template <typename K, int E, int S>
__device__ inline void in_thread_exchange_keys(K (&k)[E], int tid, int size) {
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const int f = e ^ S;
    if (f > e && f < E) {
      const bool up = ((tid * E + e) & size) == 0;
      if ((k[f] < k[e]) == up) {
        const K t = k[e];
        k[e] = k[f];
        k[f] = t;
      }
    }
  }
}

template <typename K, int E>
__device__ void bitonic_sort_keys(K* key, int npad) {
  const int tid = threadIdx.x;
  K k[E];
  __syncthreads();
#pragma unroll
  for (int e = 0; e < E; ++e) k[e] = key[tid * E + e];
  for (int size = 2; size <= npad; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      if (stride >= 64 * E) {
        __syncthreads();
#pragma unroll
        for (int e = 0; e < E; ++e) key[tid * E + e] = k[e];
        __syncthreads();
#pragma unroll
        for (int e = 0; e < E; ++e) {
          const int i = tid * E + e;
          const K ok = key[i ^ stride];
          const bool keep_min = ((i & stride) == 0) == ((i & size) == 0);
          if ((ok < k[e]) == keep_min) k[e] = ok;
        }
      } else if (stride >= E) {
        const int d = stride / E;
#pragma unroll
        for (int e = 0; e < E; ++e) {
          const int i = tid * E + e;
          const K ok = lane_xor(k[e], d);
          const bool keep_min = ((i & stride) == 0) == ((i & size) == 0);
          if ((ok < k[e]) == keep_min) k[e] = ok;
        }
      } else if (stride == 4) {
        if constexpr (E > 4) in_thread_exchange_keys<K, E, 4>(k, tid, size);
      } else if (stride == 2) {
        if constexpr (E > 2) in_thread_exchange_keys<K, E, 2>(k, tid, size);
      } else {
        if constexpr (E > 1) in_thread_exchange_keys<K, E, 1>(k, tid, size);
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int e = 0; e < E; ++e) key[tid * E + e] = k[e];
  __syncthreads();
}

template <int E, bool kByGroup>
__device__ void bitonic_sort(uint64_t* key, uint32_t* pay, int npad) {
  const int tid = threadIdx.x;
  uint64_t k[E];
  uint32_t p[E];
  __syncthreads();                               // the arrays were filled by other threads
#pragma unroll
  for (int e = 0; e < E; ++e) {
    k[e] = key[tid * E + e];
    p[e] = pay[tid * E + e];
  }
  for (int size = 2; size <= npad; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      if (stride >= 64 * E) {
        // partner lives in another wavefront: exchange through LDS
        __syncthreads();
#pragma unroll
        for (int e = 0; e < E; ++e) {
          key[tid * E + e] = k[e];
          pay[tid * E + e] = p[e];
        }
        __syncthreads();
#pragma unroll
        for (int e = 0; e < E; ++e) {
          const int i = tid * E + e, j = i ^ stride;
          const uint64_t ok = key[j];
          const uint32_t op = pay[j];
          const bool keep_min = ((i & stride) == 0) == ((i & size) == 0);
          const bool other_less = pair_less<kByGroup>(ok, op, k[e], p[e]);
          if (other_less == keep_min) {
            k[e] = ok;
            p[e] = op;
          }
        }
      } else if (stride >= E) {
        const int d = stride / E;             // lane distance
#pragma unroll
        for (int e = 0; e < E; ++e) {
          const int i = tid * E + e;
          const uint32_t lo = __shfl_xor((uint32_t)k[e], d, 64);
          const uint32_t hi = __shfl_xor((uint32_t)(k[e] >> 32), d, 64);
          const uint32_t op = __shfl_xor(p[e], d, 64);
          const uint64_t ok = ((uint64_t)hi << 32) | lo;
          const bool keep_min = ((i & stride) == 0) == ((i & size) == 0);
          const bool other_less = pair_less<kByGroup>(ok, op, k[e], p[e]);
          if (other_less == keep_min) {
            k[e] = ok;
            p[e] = op;
          }
        }
      } else if (stride == 4) {
        if constexpr (E > 4) in_thread_exchange<E, 4, kByGroup>(k, p, tid, size);
      } else if (stride == 2) {
        if constexpr (E > 2) in_thread_exchange<E, 2, kByGroup>(k, p, tid, size);
      } else {
        if constexpr (E > 1) in_thread_exchange<E, 1, kByGroup>(k, p, tid, size);
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int e = 0; e < E; ++e) {
    key[tid * E + e] = k[e];
    pay[tid * E + e] = p[e];
  }
  __syncthreads();
}

// Inclusive prefix sum over the 64 lanes: four shifts inside the rows of 16 lanes, then the last lane of a row is
// added to the next row and lane 31 to the upper half (lanes a step does not reach add zero).
__device__ inline int wave_inclusive_sum(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, false);   // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, false);   // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, false);   // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, false);   // row_shr:8
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false);   // row_bcast:15 into rows 1 and 3
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false);   // row_bcast:31 into rows 2 and 3
  return v;
}
// Minimum and maximum of a 64-bit value over the 64 lanes (same steps; lanes a step does not reach keep their
// own value); valid in lane 63.
__device__ inline void wave_minmax64(unsigned long long& lo, unsigned long long& hi) {
#define VD_MM(CTRL, ROWS)                                                                                     \
  {                                                                                                           \
    const uint32_t l0 = (uint32_t)lo, l1 = (uint32_t)(lo >> 32), h0 = (uint32_t)hi, h1 = (uint32_t)(hi >> 32); \
    const unsigned long long ol = ((unsigned long long)(uint32_t)__builtin_amdgcn_update_dpp((int)l1, (int)l1, CTRL, ROWS, 0xF, false) << 32) | \
                                  (uint32_t)__builtin_amdgcn_update_dpp((int)l0, (int)l0, CTRL, ROWS, 0xF, false);  \
    const unsigned long long oh = ((unsigned long long)(uint32_t)__builtin_amdgcn_update_dpp((int)h1, (int)h1, CTRL, ROWS, 0xF, false) << 32) | \
                                  (uint32_t)__builtin_amdgcn_update_dpp((int)h0, (int)h0, CTRL, ROWS, 0xF, false);  \
    lo = ol < lo ? ol : lo;                                                                                   \
    hi = oh > hi ? oh : hi;                                                                                   \
  }
  VD_MM(0x111, 0xF)
  VD_MM(0x112, 0xF)
  VD_MM(0x114, 0xF)
  VD_MM(0x118, 0xF)
  VD_MM(0x142, 0xA)
  VD_MM(0x143, 0xC)
#undef VD_MM
}

// Exclusive prefix sum over vals[0..count) (count <= per * blockDim.x), in place; returns the total
// to every thread.  `wsum` holds one slot per wavefront plus one.
__device__ int block_exclusive_scan(int* vals, int count, int* wsum) {
  const int tid = threadIdx.x, nt = blockDim.x;
  const int per = (count + nt - 1) / nt;
  const int begin = tid * per;
  int local = 0;
  for (int i = 0; i < per; ++i)
    if (begin + i < count) local += vals[begin + i];
  const int incl = wave_inclusive_sum(local);
  const int lane = tid & 63, wave = tid >> 6;
  if (lane == 63) wsum[wave] = incl;
  __syncthreads();
  if (tid < 64) {                                   // at most 16 wavefront totals: one scan of the first wavefront
    const int nw = (nt + 63) >> 6;
    const int t = tid < nw ? wsum[tid] : 0;
    const int inc = wave_inclusive_sum(t);
    if (tid < nw) wsum[tid] = inc - t;
    if (tid == nw - 1) wsum[nw] = inc;
  }
  __syncthreads();
  int run = wsum[wave] + incl - local;
  const int total = wsum[(nt + 63) >> 6];
  for (int i = 0; i < per; ++i)
    if (begin + i < count) {
      const int t = vals[begin + i];
      vals[begin + i] = run;
      run += t;
    }
  __syncthreads();
  return total;
}

constexpr int kBuckets = 1024;              // order-preserving buckets of the first sort
constexpr int kCountMax = 1024;             // largest group ranked by counting instead of sorting

struct SampleArgs {
  const uint64_t* hash;
  int32_t* group_id;
  int32_t* sel;
  int32_t* counts;
  int N, npad;
  int index_bits;      // log2(npad): room for a variate (or padding) index below the hash in a packed key
  uint32_t gs, num, den;
  uint32_t seed_lo, seed_hi, step_lo, step_hi;
  const uint64_t* ext_keys;   // optional: key of variate n that orders the members of a group, instead of a Philox draw
  uint64_t* step_dev;         // optional: the step counter lives in device memory (read here instead of step_lo / step_hi)
  int advance;                //   and is incremented once the draw is done, so that a recorded launch draws anew when replayed
};

// members kept from a group of `size` (Eq. 1 with the optional keep ratio)
__device__ inline uint32_t keep_count(uint32_t size, const SampleArgs& a) {
  uint64_t by_ratio = ((uint64_t)size * a.num + a.den - 1) / a.den;
  if (by_ratio < 1) by_ratio = 1;
  uint32_t keep = by_ratio < size ? (uint32_t)by_ratio : size;
  if (a.gs != 0 && keep > a.gs) keep = a.gs;
  return keep;
}

// Number of pairs (key[q], idx(q)) with q in [s0, s1) that order before (kp, np), where idx(q) is
// pay[q] & mask.  Four independent LDS reads are in flight per round: the loop is latency-bound.
__device__ inline int count_before(const uint64_t* key, const uint32_t* pay, uint32_t mask, int s0, int s1,
                                   uint64_t kp, uint32_t np) {
  int r = 0;
  int q = s0;
  for (; q + 4 <= s1; q += 4) {
    uint64_t kq[4];
    uint32_t nq[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      kq[u] = key[q + u];
      nq[u] = pay[q + u] & mask;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) r += (kq[u] < kp || (kq[u] == kp && nq[u] < np)) ? 1 : 0;
  }
  for (; q < s1; ++q) {
    const uint64_t kq = key[q];
    r += (kq < kp || (kq == kp && (pay[q] & mask) < np)) ? 1 : 0;
  }
  return r;
}

// Two 8-byte records per variate for the count inside a bucket: first = (the hash's bits below the bucket index, all
// that differs inside a bucket; the upper half of u[n]), second = (the lower half of u[n], n).  Number of records q
// in [s0, s1) that order before the record at p by (hash, u[n], n): the first records decide unless they are equal
// (one pair in 2^32; the record itself is left out by its position), so the count reads 8 bytes per comparison.
__device__ inline int before_rec(unsigned long long ko, unsigned long long km, const uint2* second, int q, int p, uint2 me2) {
  int r = ko < km ? 1 : 0;
  if (ko == km && q != p) {
    const uint2 o2 = second[q];
    r = (o2.x < me2.x || (o2.x == me2.x && o2.y < me2.y)) ? 1 : 0;
  }
  return r;
}
__device__ inline int count_before_rec(const uint2* first, const uint2* second, int s0, int s1, int p) {
  const uint2 me1 = first[p], me2 = second[p];
  const unsigned long long km = ((unsigned long long)me1.x << 32) | me1.y;
  int r = 0;
  int q = s0;
  for (; q + 4 <= s1; q += 4) {
    uint2 o[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) o[u] = first[q + u];
#pragma unroll
    for (int u = 0; u < 4; ++u) r += before_rec(((unsigned long long)o[u].x << 32) | o[u].y, km, second, q + u, p, me2);
  }
  for (; q < s1; ++q) {
    const uint2 o = first[q];
    r += before_rec(((unsigned long long)o.x << 32) | o.y, km, second, q, p, me2);
  }
  return r;
}

// FUSED: one ordering by (hash, u[n], n) instead of one by (hash, n) and a ranking by (u[n], n) inside every group
// (needs another 16 bytes of LDS per variate, two records of 8: up to 4096 of them; the hash's bits below the bucket index must fit
// 32 bits, i.e. the hashes span less than 2^42, else the sorting networks take over).
template <int E, bool FUSED>
__global__ __launch_bounds__(1024) void sample_kernel(SampleArgs a) {
  extern __shared__ unsigned char smem[];
  const int N = a.N, npad = a.npad;
  uint64_t* key = reinterpret_cast<uint64_t*>(smem);                   // [npad]
  uint32_t* pay = reinterpret_cast<uint32_t*>(key + npad);             // [npad]
  int* scan = reinterpret_cast<int*>(pay + npad);                      // [npad]: flags -> ids / offsets
  int* wsum = scan + npad;                                             // [20]
  uint16_t* gstart = reinterpret_cast<uint16_t*>(wsum + 20);           // [npad + 1], values <= 8192
  unsigned long long* mm = reinterpret_cast<unsigned long long*>(
      smem + (((size_t)npad * 16 + 80 + (size_t)(npad + 1) * 2 + 7) & ~(size_t)7));   // [2]: min, max hash
  int* bstart = reinterpret_cast<int*>(mm + 2);                        // [kBuckets + 1]
  int* bcur = bstart + kBuckets + 1;                                   // [kBuckets]
  int* bmax = bcur + kBuckets;                                         // [1]
  uint2* rec1 = reinterpret_cast<uint2*>(
      reinterpret_cast<unsigned char*>(bmax + 1) + ((16 - (reinterpret_cast<uintptr_t>(bmax + 1) & 15)) & 15));   // [npad], FUSED only
  uint2* rec2 = rec1 + npad;                                            // [npad], FUSED only
  const int tid = threadIdx.x, nt = blockDim.x;
  // every thread's E hashes (variates tid, tid + nt, ...; npad = E * nt), read from memory once
  uint64_t hreg[E];
#pragma unroll
  for (int e = 0; e < E; ++e) hreg[e] = tid + e * nt < N ? a.hash[tid + e * nt] : 0ull;
  // ... and, while they travel, the keys that order the members of a group
  unsigned long long ureg[FUSED ? E : 1];
  if constexpr (FUSED) {
    if (a.step_dev) {
      const uint64_t step = *a.step_dev;
      a.step_lo = (uint32_t)step;
      a.step_hi = (uint32_t)(step >> 32);
    }
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const uint32_t n = (uint32_t)(tid + e * nt);
      ureg[e] = 0ull;
      if (n < (uint32_t)N) {
        if (a.ext_keys) {
          ureg[e] = a.ext_keys[n];
        } else {
          uint32_t r0, r1;
          philox4x32_10(n, 0u, a.step_lo, a.step_hi, a.seed_lo, a.seed_hi, r0, r1);
          ureg[e] = ((unsigned long long)r0 << 32) | r1;
        }
      }
    }
  }

  // Sort 1, usual path.  (hash, n) pairs are dropped into kBuckets order-preserving buckets (equal
  // width over [min, max] of the hashes, a shift instead of a division); inside a bucket the position
  // of a pair is a count over the bucket.  The result is the same total order as the sorting
  // networks below, which remain for inputs that crowd one bucket.
  bool sorted = false;
  {
    if (tid == 0) {
      mm[0] = ~0ull;
      mm[1] = 0ull;
      *bmax = 0;
    }
    for (int i = tid; i <= kBuckets; i += nt) bstart[i] = 0;
    __syncthreads();
    unsigned long long lo = ~0ull, hi = 0ull;
#pragma unroll
    for (int e = 0; e < E; ++e)
      if (tid + e * nt < N) {
        const unsigned long long h = hreg[e];
        lo = h < lo ? h : lo;
        hi = h > hi ? h : hi;
      }
    // one atomic per wavefront, not per thread: same-address LDS atomics serialise
    wave_minmax64(lo, hi);
    if ((tid & 63) == 63) {
      atomicMin(&mm[0], lo);
      atomicMax(&mm[1], hi);
    }
    __syncthreads();
    const unsigned long long hmin = mm[0], range = mm[1] - mm[0];
    int shift = 0;
    while ((range >> shift) >= (unsigned long long)kBuckets) ++shift;
#pragma unroll
    for (int e = 0; e < E; ++e)
      if (tid + e * nt < N) atomicAdd(&bstart[(int)((hreg[e] - hmin) >> shift)], 1);
    __syncthreads();
    {
      int m = 0;
      for (int i = tid; i < kBuckets; i += nt) m = max(m, bstart[i]);
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) m = max(m, __shfl_xor(m, off, 64));
      if ((tid & 63) == 0) atomicMax(bmax, m);
    }
    __syncthreads();
    if (*bmax <= kCountMax && (!FUSED || shift <= 32)) {
      block_exclusive_scan(bstart, kBuckets, wsum);                    // counts -> bucket starts
      for (int i = tid; i < kBuckets; i += nt) bcur[i] = bstart[i];
      __syncthreads();
#pragma unroll
      for (int e = 0; e < E; ++e)
        if (tid + e * nt < N) {
          const unsigned long long h = hreg[e];
          const int pos = atomicAdd(&bcur[(int)((h - hmin) >> shift)], 1);
          key[pos] = h;
          pay[pos] = (uint32_t)(tid + e * nt);
          if constexpr (FUSED) {
            rec1[pos] = make_uint2((uint32_t)((h - hmin) & ((1ull << shift) - 1ull)), (uint32_t)(ureg[e] >> 32));
            rec2[pos] = make_uint2((uint32_t)ureg[e], (uint32_t)(tid + e * nt));
          }
        }
      __syncthreads();
      for (int p = tid; p < N; p += nt) {
        const uint64_t kp = key[p];
        const uint32_t np = pay[p];
        const int b = (int)((kp - hmin) >> shift);
        const int s0 = bstart[b], s1 = bcur[b];
        if constexpr (FUSED) scan[p] = s0 + count_before_rec(rec1, rec2, s0, s1, p);
        else scan[p] = s0 + count_before(key, pay, 0xffffffffu, s0, s1, kp, np);
      }
      __syncthreads();
      uint64_t rk[E];
      uint32_t rp[E];
      int rpos[E];
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const int p = tid + e * nt;
        rpos[e] = -1;
        if (p < N) {
          rk[e] = key[p];
          rp[e] = pay[p];
          rpos[e] = scan[p];
        }
      }
      __syncthreads();
#pragma unroll
      for (int e = 0; e < E; ++e)
        if (rpos[e] >= 0) {
          key[rpos[e]] = rk[e];
          pay[rpos[e]] = rp[e];
        }
      __syncthreads();
      sorted = true;
    }
  }

  // Sort 1, sorting networks.  Hash and variate index share one key when they fit: 32 bits (one shuffle per exchange;
  // the radix-R code of three bins of a 96-sample window needs 17 bits), else 64 bits, else the pair
  // network.  Padding keys are all ones and sort last.
  const int ib = a.index_bits;
  int too_wide = 0;                                   // bit 0: not in 32 bits, bit 1: not in 64 bits
  if (!sorted) {                                      // (uniform: every thread took the same branch above)
#pragma unroll
    for (int e = 0; e < E; ++e)
      if (tid + e * nt < N) too_wide |= ((hreg[e] >> (32 - ib)) != 0 ? 1 : 0) | ((hreg[e] >> (64 - ib)) != 0 ? 2 : 0);
    // (the block-wide OR is a logical one: reduce the two bits separately)
    const int over32 = __syncthreads_or(too_wide & 1);
    const int over64 = __syncthreads_or(too_wide & 2);
    too_wide = (over32 ? 1 : 0) | (over64 ? 2 : 0);
  }
  if (sorted) {
    // nothing left to do
  } else if (too_wide == 0) {
    uint32_t* key32 = reinterpret_cast<uint32_t*>(key) + npad;      // upper half of the key array
    for (int i = tid; i < npad; i += nt) key32[i] = i < N ? (((uint32_t)a.hash[i] << ib) | (uint32_t)i) : ~0u;
    bitonic_sort_keys<uint32_t, E>(key32, npad);
    for (int i = tid; i < npad; i += nt) {
      const uint32_t v = key32[i];
      pay[i] = v & ((1u << ib) - 1);
      scan[i] = (int)(v >> ib);                       // parked: key32 overlaps key[npad/2 ..]
    }
    __syncthreads();
    for (int i = tid; i < npad; i += nt) key[i] = (uint64_t)(uint32_t)scan[i];
    __syncthreads();
  } else if ((too_wide & 2) == 0) {
    for (int i = tid; i < npad; i += nt) key[i] = i < N ? ((a.hash[i] << ib) | (uint64_t)i) : ~0ull;
    bitonic_sort_keys<uint64_t, E>(key, npad);
    for (int i = tid; i < npad; i += nt) {
      const uint64_t v = key[i];
      pay[i] = (uint32_t)(v & ((1u << ib) - 1));
      key[i] = v >> ib;
    }
    __syncthreads();
  } else {
    for (int i = tid; i < npad; i += nt) {
      key[i] = i < N ? a.hash[i] : ~0ull;
      pay[i] = (uint32_t)i;
    }
    bitonic_sort<E, false>(key, pay, npad);
  }

  // segment heads -> dense group ids
  for (int p = tid; p < N; p += nt) scan[p] = (p == 0 || key[p] != key[p - 1]) ? 1 : 0;
  __syncthreads();
  const int G = block_exclusive_scan(scan, N, wsum);    // scan[p] = heads before p
  for (int p = tid; p < N; p += nt) {
    const bool head = (p == 0 || key[p] != key[p - 1]);
    const int g = scan[p] - (head ? 0 : 1);              // heads at or before p, minus one
    if (head) gstart[g] = (uint16_t)p;
    scan[p] = g;
  }
  if (tid == 0) {
    gstart[G] = (uint16_t)N;
    wsum[18] = 0;
  }
  __syncthreads();
  {
    int m = 0;
    for (int g = tid; g < G; g += nt) m = max(m, (int)gstart[g + 1] - (int)gstart[g]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = max(m, __shfl_xor(m, off, 64));
    if ((tid & 63) == 0) atomicMax(&wsum[18], m);
  }
  const bool ranked = FUSED && sorted;          // the order inside every group is already that of (u[n], n)
  if (!FUSED && a.step_dev) {
    const uint64_t step = *a.step_dev;
    a.step_lo = (uint32_t)step;
    a.step_hi = (uint32_t)(step >> 32);
  }
  for (int p = tid; p < N; p += nt) {
    const uint32_t n = pay[p];
    const int g = scan[p];
    a.group_id[n] = g;
    if (ranked) {
      // nothing to draw
    } else if (a.ext_keys) {
      key[p] = a.ext_keys[n];
    } else {
      uint32_t r0, r1;
      philox4x32_10(n, 0u, a.step_lo, a.step_hi, a.seed_lo, a.seed_hi, r0, r1);
      key[p] = ((uint64_t)r0 << 32) | r1;
    }
    pay[p] = ((uint32_t)g << 16) | n;
  }
  __syncthreads();
  const int max_group = wsum[18];
  if (ranked) {
    for (int p = tid; p < N; p += nt) {
      const uint32_t g = pay[p] >> 16, n = pay[p] & 0xffffu;
      const int s0 = gstart[g], s1 = gstart[g + 1];
      scan[n] = (uint32_t)(p - s0) < keep_count((uint32_t)(s1 - s0), a) ? 1 : 0;
    }
  } else if (max_group <= kCountMax) {
    // Groups are short: the rank of a member inside its group is a count over the group.
    for (int p = tid; p < N; p += nt) {
      const uint32_t g = pay[p] >> 16, n = pay[p] & 0xffffu;
      const int s0 = gstart[g], s1 = gstart[g + 1];
      const uint64_t ku = key[p];
      const uint32_t rank = (uint32_t)count_before(key, pay, 0xffffu, s0, s1, ku, n);
      scan[n] = rank < keep_count((uint32_t)(s1 - s0), a) ? 1 : 0;
    }
  } else {
    for (int p = N + tid; p < npad; p += nt) {
      key[p] = ~0ull;
      pay[p] = 0xffffffffu;                               // group 65535 sorts after every real group
    }
    bitonic_sort<E, true>(key, pay, npad);
    // keep the first n_i members of every segment; flags indexed by variate
    for (int p = tid; p < N; p += nt) {
      const uint32_t g = pay[p] >> 16, n = pay[p] & 0xffffu;
      const uint32_t size = (uint32_t)gstart[g + 1] - (uint32_t)gstart[g];
      scan[n] = ((uint32_t)p - (uint32_t)gstart[g] < keep_count(size, a)) ? 1 : 0;
    }
  }
  __syncthreads();
  // the flags are needed after the scan as well: keep a copy in the payload array
  for (int n = tid; n < N; n += nt) pay[n] = (uint32_t)scan[n];
  __syncthreads();
  const int n_sel = block_exclusive_scan(scan, N, wsum);
  for (int n = tid; n < N; n += nt)
    if (pay[n]) a.sel[scan[n]] = n;
  if (tid == 0) {
    a.counts[0] = n_sel;
    a.counts[1] = G;
    // (every thread read the counter before the barriers of the scans above)
    if (a.step_dev && a.advance) *a.step_dev = (((uint64_t)a.step_hi << 32) | a.step_lo) + 1;
  }
}

int next_pow2(int v) {
  int p = 1;
  while (p < v) p <<= 1;
  return p;
}

}  // namespace

extern "C" size_t vardrop_sample_workspace_bytes(int) { return 0; }

namespace {

// ---- deterministic representatives: keys from the distance to the group's mean spectrum.
// The first member of a group (lowest variate index) computes the group's mean spectrum: one thread per
// candidate bin adds the members' values in ascending variate index and divides by the group size.
// Single-precision IEEE operations without fused multiply-add throughout: these values decide which
// members are kept, and the test oracle evaluates them in the same arithmetic and order.
__global__ __launch_bounds__(256) void group_mean_kernel(const int32_t* __restrict__ gid, const float* __restrict__ abar,
                                                        float* __restrict__ mean, int N, int F) {
  __shared__ int earlier;
  const int n = blockIdx.x, g = gid[n];
  if (threadIdx.x == 0) earlier = 0;
  __syncthreads();
  for (int m = threadIdx.x; m < n; m += 256)
    if (gid[m] == g) earlier = 1;
  __syncthreads();
  if (earlier) return;
  for (int f = threadIdx.x; f < F; f += 256) {
    float acc = 0.f;
    int size = 0;
    for (int m = n; m < N; ++m)
      if (gid[m] == g) {
        acc = acc + abar[(long long)m * F + f];
        ++size;
      }
    mean[(long long)g * F + f] = acc / (float)size;       // (correctly rounded: the compiler's default for fp32 division)
  }
}
// key[n] = bits of sum_f (abar[n][f] - mean[g][f])^2 (ascending f) in the upper half: non-negative floats order
// like their bit patterns
__global__ __launch_bounds__(256) void distance_key_kernel(const int32_t* __restrict__ gid, const float* __restrict__ abar,
                                                          const float* __restrict__ mean, uint64_t* __restrict__ keys,
                                                          int N, int F) {
  const int n = blockIdx.x * 256 + threadIdx.x;
  if (n >= N) return;
  const float* row = abar + (long long)n * F;
  const float* mu = mean + (long long)gid[n] * F;
  float d = 0.f;
  {
#pragma clang fp contract(off)                  // product and sum are rounded separately (no fused multiply-add)
    for (int f = 0; f < F; ++f) {
      const float t = row[f] - mu[f];
      const float sq = t * t;
      d = d + sq;
    }
  }
  keys[n] = (uint64_t)__float_as_uint(d) << 32;
}

int run_sample(vardrop_ctx* ctx, const uint64_t* hash, int N,
               uint32_t gs, uint32_t ratio_num, uint32_t ratio_den,
               uint64_t seed, uint64_t step, const uint64_t* ext_keys,
               int32_t* group_id, int32_t* sel, int32_t* counts, int32_t* counts_host, void* stream,
               uint64_t* step_dev = nullptr, int advance = 0) {
  if (!ctx || !hash || !group_id || !sel || !counts) return VARDROP_EINVAL;
  if (N < 1) return VARDROP_EINVAL;
  if (ratio_den == 0 || ratio_num > ratio_den) return VARDROP_EINVAL;
  if (N > kMaxN) return VARDROP_EUNSUPPORTED;
  int npad = next_pow2(N);
  if (npad < 128) npad = 128;
  const bool fused = npad <= 4096;
  const size_t lds = (size_t)npad * 16 + 20 * 4 + (size_t)(npad + 1) * 2 + 14 + 16 + (2 * kBuckets + 2) * 4 + (fused ? (size_t)npad * 16 + 16 : 0);
  if (lds > (size_t)ctx->lds_per_block) return VARDROP_EUNSUPPORTED;
  // elements per thread of the sort: as many threads as the workgroup may have, so that the counting loops are short
  const int E = npad <= 1024 ? 1 : (npad <= 2048 ? 2 : (npad == 4096 ? 4 : 8));
  const int threads = npad / E;
  SampleArgs a;
  a.hash = hash;
  a.group_id = group_id;
  a.sel = sel;
  a.counts = counts;
  a.N = N;
  a.npad = npad;
  a.index_bits = 0;
  while ((1 << a.index_bits) < npad) ++a.index_bits;
  a.gs = gs;
  a.num = ratio_num;
  a.den = ratio_den;
  a.seed_lo = (uint32_t)seed;
  a.seed_hi = (uint32_t)(seed >> 32);
  a.step_lo = (uint32_t)step;
  a.step_hi = (uint32_t)(step >> 32);
  a.ext_keys = ext_keys;
  a.step_dev = step_dev;
  a.advance = advance;
  hipStream_t s = (hipStream_t)stream;
  const void* fn = E == 1 ? (const void*)sample_kernel<1, true> : E == 2 ? (const void*)sample_kernel<2, true> : (E == 4 ? (const void*)sample_kernel<4, true> : (const void*)sample_kernel<8, false>);
  if (lds > 65536)
    VD_HIP(ctx, hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  {
    VdTimer timer(ctx, VARDROP_K_SAMPLE, s);
    if (E == 1) VD_KERNEL(ctx, (sample_kernel<1, true>), dim3(1), dim3(threads), lds, s, a);
    else if (E == 2) VD_KERNEL(ctx, (sample_kernel<2, true>), dim3(1), dim3(threads), lds, s, a);
    else if (E == 4) VD_KERNEL(ctx, (sample_kernel<4, true>), dim3(1), dim3(threads), lds, s, a);
    else VD_KERNEL(ctx, (sample_kernel<8, false>), dim3(1), dim3(threads), lds, s, a);
  }
  VD_LAUNCH_CHECK(ctx);
  if (counts_host)
    VD_HIP(ctx, hipMemcpyAsync(counts_host, counts, 2 * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  return VARDROP_OK;
}

}  // namespace

extern "C" int vardrop_sample(vardrop_ctx* ctx, const uint64_t* hash, int N,
                              uint32_t gs, uint32_t ratio_num, uint32_t ratio_den,
                              uint64_t seed, uint64_t step,
                              int32_t* group_id, int32_t* sel, int32_t* counts, int32_t* counts_host,
                              void* ws, size_t ws_bytes, void* stream) {
  (void)ws;
  (void)ws_bytes;
  return run_sample(ctx, hash, N, gs, ratio_num, ratio_den, seed, step, nullptr, group_id, sel, counts, counts_host, stream);
}

extern "C" int vardrop_sample_dev(vardrop_ctx* ctx, const uint64_t* hash, int N,
                                  uint32_t gs, uint32_t ratio_num, uint32_t ratio_den,
                                  uint64_t seed, uint64_t* step_dev, int advance,
                                  int32_t* group_id, int32_t* sel, int32_t* counts,
                                  void* ws, size_t ws_bytes, void* stream) {
  (void)ws;
  (void)ws_bytes;
  if (!step_dev || !vd_aligned(step_dev, 8)) return VARDROP_EINVAL;
  return run_sample(ctx, hash, N, gs, ratio_num, ratio_den, seed, 0, nullptr, group_id, sel, counts, nullptr, stream,
                    step_dev, advance);
}

namespace {
int run_sample_nearest(vardrop_ctx* ctx, const uint64_t* hash, const float* abar, int N, int F,
                       uint32_t gs, uint32_t ratio_num, uint32_t ratio_den,
                       int32_t* group_id, int32_t* sel, int32_t* counts, int32_t* counts_host,
                       float* mean, uint64_t* keys, void* stream) {
  // group ids first (the members kept by this pass are overwritten below)
  int rc = run_sample(ctx, hash, N, gs, ratio_num, ratio_den, 0, 0, nullptr, group_id, sel, counts, nullptr, stream);
  if (rc) return rc;
  hipStream_t s = (hipStream_t)stream;
  hipLaunchKernelGGL(group_mean_kernel, dim3(N), dim3(256), 0, s, group_id, abar, mean, N, F);
  hipLaunchKernelGGL(distance_key_kernel, dim3(vd_ceil_div(N, 256)), dim3(256), 0, s, group_id, abar, mean, keys, N, F);
  VD_LAUNCH_CHECK(ctx);
  return run_sample(ctx, hash, N, gs, ratio_num, ratio_den, 0, 0, keys, group_id, sel, counts, counts_host, stream);
}

// Scratch of the entry point that allocates nothing: the group means ([G][F] floats, G F <= N F <= kStaticMeanFloats)
// followed by the distance keys ([N] uint64, N <= kMaxN).  Part of the code object, one copy per device, held until
// the process ends; every call on a device uses it, so calls that overlap on one device race.
constexpr size_t kStaticMeanFloats = (size_t)1 << 20;
constexpr size_t kStaticScratchBytes = kStaticMeanFloats * sizeof(float) + (size_t)kMaxN * sizeof(uint64_t);
}  // namespace
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Device address of the scratch array on the current device (the array's name is only a host-side stand-in for it).
int vd_static_scratch_address(void** out) {
  void* p = nullptr;
  const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
  if (e != hipSuccess || !p) return (int)(e != hipSuccess ? e : hipErrorInvalidSymbol);
  *out = p;
  return 0;
}

extern "C" int vardrop_sample_nearest_noalloc(vardrop_ctx* ctx, const uint64_t* hash, const float* abar, int N, int F,
                                              uint32_t gs, uint32_t ratio_num, uint32_t ratio_den,
                                              int32_t* group_id, int32_t* sel, int32_t* counts, void* stream) {
  if (!ctx || !abar || F < 1) return VARDROP_EINVAL;
  if (N > kMaxN || (N >= 1 && (size_t)N * (size_t)F > kStaticMeanFloats)) return VARDROP_EUNSUPPORTED;   // beyond the static scratch
  if (!ctx->static_scratch) return VARDROP_EHIP;             // its address could not be taken when the context was made
  float* mean = (float*)ctx->static_scratch;
  uint64_t* keys = (uint64_t*)((char*)ctx->static_scratch + kStaticMeanFloats * sizeof(float));
  return run_sample_nearest(ctx, hash, abar, N, F, gs, ratio_num, ratio_den, group_id, sel, counts, nullptr, mean, keys, stream);
}

extern "C" size_t vardrop_sample_nearest_workspace_bytes(int N, int F) {
  if (N < 1 || F < 1) return 0;
  return vd_align_up((size_t)N * F * sizeof(float), 256) + vd_align_up((size_t)N * sizeof(uint64_t), 256);
}

extern "C" int vardrop_sample_nearest(vardrop_ctx* ctx, const uint64_t* hash, const float* abar, int N, int F,
                                      uint32_t gs, uint32_t ratio_num, uint32_t ratio_den,
                                      int32_t* group_id, int32_t* sel, int32_t* counts, int32_t* counts_host,
                                      void* ws, size_t ws_bytes, void* stream) {
  if (!ctx || !abar || F < 1) return VARDROP_EINVAL;
  if (N >= 1 && (!ws || !vd_aligned(ws, 256) || ws_bytes < vardrop_sample_nearest_workspace_bytes(N, F))) return VARDROP_EWORKSPACE;
  float* mean = (float*)ws;
  uint64_t* keys = (uint64_t*)((char*)ws + vd_align_up((size_t)N * F * sizeof(float), 256));
  return run_sample_nearest(ctx, hash, abar, N, F, gs, ratio_num, ratio_den, group_id, sel, counts, counts_host, mean, keys, stream);
}

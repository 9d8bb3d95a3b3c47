// Block-wide selection helpers: pull the `want` lowest of n fp32 values (with
// their indices) into LDS as sorted 64-bit (value image << 32 | index) keys.
//
// Method: a value-linear histogram between the block's min and max finds the
// bucket d* that holds the want-th lowest value; everything in buckets <= d* is
// compacted and bitonic-sorted.  Ties need no special care: the composite key is
// unique, so the sort alone yields (value ascending, index ascending).
//
// A thread keeps PER values in registers (at most 16), so a block of THREADS threads handles
// n <= PER*THREADS values (1024 threads and PER = 16 for the 16384-token limit).  PER is a
// template parameter chosen by the host from the longest sample: the loops over a thread's
// values are unrolled and a slot past the sample's end still issues its instructions with
// every lane switched off (measured on 2880-token samples: PER = 4 instead of 16 takes 1.9 us
// off pivot selection and 1.7 us off the ordering kernel).
#pragma once
#include "common.hpp"

namespace dart {

constexpr int kSelPerThread = 16;  // most values a thread keeps in registers
constexpr int pow2_at_least(int v) { int p = 1; while (p < v) p <<= 1; return p; }
constexpr int kSelBuckets = 1024;
// Requests for more than kSelCountMin keys are put in order by counting instead of a bitonic
// sort (measured cross-over), unless one fine histogram bucket holds more than kSelMaxSeg of them (massive ties).
constexpr int kSelCountMin = 128, kSelMaxSeg = 64;

template <int THREADS, int PER = kSelPerThread>
struct SelectShared {
  static constexpr int kBuf = pow2_at_least(THREADS * PER);  // (the sorts pad to a power of two)
  unsigned long long buf[kBuf];  // compacted keys, then sorted
  int hist[kSelBuckets];
  float redf[2 * (THREADS / kWave)];
  float redg[THREADS / kWave];
  int redi[THREADS / kWave];
  int count;
  int dstar;
  int count2, dmid, cmid, cstar;  // two-part sort: see collect_sorted
  int clim;                       // keys selected (ordering by counting)
};

template <int THREADS>
__device__ __forceinline__ int block_sum(int v, int tid, int* red) {
  constexpr int kSelWaves = THREADS / kWave;
  const int lane = tid & 63, w = tid >> 6;
  v = wave_sum(v);
  __syncthreads();  // red may still be read from a previous call
  if (lane == 0) red[w] = v;
  __syncthreads();
  int s = 0;
#pragma unroll
  for (int i = 0; i < kSelWaves; ++i) s += red[i];
  return s;
}

// Where the want-th lowest of n values sits in a value-linear histogram of kSelBuckets buckets
// between the block's minimum and maximum: its bucket d*, and how many values lie in the
// buckets below d*.  For callers that need a set of lowest values rather than a sorted list:
// the buckets below d* belong to it outright and only bucket d* needs a closer look.
struct BucketSplit {
  float lo, scale;  // bucket(x) = clamp((x - lo) * scale)
  int dstar, below;
  __device__ __forceinline__ int bucket(float x) const {
    float f = (x - lo) * scale;  // non-finite input lands in a valid bucket too
    int d = f >= (float)(kSelBuckets - 1) ? kSelBuckets - 1 : (int)f;
    d = d < 0 ? 0 : d;
    return d > kSelBuckets - 1 ? kSelBuckets - 1 : d;
  }
};

// v[e] belongs to index tid + e*THREADS; the same result on every thread (four barriers).
// (collect_sorted below repeats these steps because it goes on to use every thread's own
// bucket counts.)
template <int THREADS, int PER>
__device__ __forceinline__ BucketSplit bucket_split(const float (&v)[PER], int n, int want,
                                                    int tid, SelectShared<THREADS, PER>& sh) {
  constexpr int kSelWaves = THREADS / kWave;
  constexpr int kSelBucketsPerThread = kSelBuckets / THREADS;
  const int lane = tid & 63, w = tid >> 6;
  const int ne = __builtin_amdgcn_readfirstlane((n + THREADS - 1) / THREADS);
  float lo = INFINITY, hi = -INFINITY;
#pragma unroll
  for (int e = 0; e < PER; ++e)
    if (e < ne && tid + e * THREADS < n) {
      lo = fminf(lo, v[e]);
      hi = fmaxf(hi, v[e]);
    }
  lo = wave_min(lo);
  hi = wave_max(hi);
  __syncthreads();
  if (lane == 0) {
    sh.redf[2 * w] = lo;
    sh.redf[2 * w + 1] = hi;
  }
#pragma unroll
  for (int q = 0; q < kSelBucketsPerThread; ++q) sh.hist[tid + q * THREADS] = 0;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < kSelWaves; ++i) {
    lo = fminf(lo, sh.redf[2 * i]);
    hi = fmaxf(hi, sh.redf[2 * i + 1]);
  }
  const float range = hi - lo;
  BucketSplit bs;
  bs.lo = lo;
  bs.scale = range > 0.f ? (float)kSelBuckets / range : 0.f;
#pragma unroll
  for (int e = 0; e < PER; ++e)
    if (e < ne && tid + e * THREADS < n) atomicAdd(&sh.hist[bs.bucket(v[e])], 1);
  __syncthreads();
  int h[kSelBucketsPerThread], mine = 0;
#pragma unroll
  for (int q = 0; q < kSelBucketsPerThread; ++q) {
    h[q] = sh.hist[tid * kSelBucketsPerThread + q];
    mine += h[q];
  }
  int run = wave_excl_scan(mine, lane);
  if (lane == 63) sh.redi[w] = run + mine;
  if (tid == 0) {  // (kept if no count crosses the target: values that are not numbers)
    sh.dstar = kSelBuckets - 1;
    sh.cstar = 0;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < kSelWaves; ++i)
    if (i < w) run += sh.redi[i];
  const int target = want < n ? want : n;
#pragma unroll
  for (int q = 0; q < kSelBucketsPerThread; ++q) {
    const int before = run;
    run += h[q];
    if (before < target && run >= target) {
      sh.dstar = tid * kSelBucketsPerThread + q;
      sh.cstar = before;
    }
  }
  __syncthreads();
  bs.dstar = sh.dstar;
  bs.below = sh.cstar;
  return bs;
}

// An upper bound of the want-th lowest of the n values that is itself one of the values: the
// largest value of the buckets up to d*.  For callers that need a superset of the `want`
// lowest, not their order (five barriers, no sort).
template <int THREADS, int PER>
__device__ __forceinline__ float rank_upper_bound(const float (&v)[PER], int n, int want,
                                                  int tid, SelectShared<THREADS, PER>& sh) {
  constexpr int kSelWaves = THREADS / kWave;
  const int lane = tid & 63, w = tid >> 6;
  const BucketSplit bs = bucket_split<THREADS, PER>(v, n, want, tid, sh);
  float top = -INFINITY;  // largest value of the buckets <= d*
#pragma unroll
  for (int e = 0; e < PER; ++e)
    if (e * THREADS < n && tid + e * THREADS < n && bs.bucket(v[e]) <= bs.dstar)
      top = fmaxf(top, v[e]);
  top = wave_max(top);
  if (lane == 0) sh.redg[w] = top;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < kSelWaves; ++i) top = fmaxf(top, sh.redg[i]);
  return top;
}

// v[e] belongs to index tid + e*THREADS (n <= PER*THREADS); entries with index >= n are ignored.
// Compacts every entry whose bucket is <= d* and sorts;
// returns how many were compacted (>= min(want, n)); the same value on every thread.
// part2 (optional): when more than THREADS keys are compacted
// and a bucket boundary cuts them into two runs of at most THREADS keys each, the runs are
// sorted separately (two short sorts instead of one of twice the size; the histogram
// already orders them by value): the first *part2 keys are at buf[0..), the others at
// buf[THREADS..).  Otherwise *part2 is the returned count (one run at buf[0..)).
// COUNTING: long requests may be ordered by counting (see below); callers that only ever ask for
// a few keys leave it off and keep the shorter code.
template <int THREADS, bool COUNTING = false, int PER = kSelPerThread>
__device__ __forceinline__ int collect_sorted(const float (&v)[PER], int n, int want,
                                              int tid, SelectShared<THREADS, PER>& sh,
                                              int* part2 = nullptr) {
  constexpr int kSelThreads = THREADS;
  constexpr int kSelWaves = THREADS / kWave;
  constexpr int kSelBucketsPerThread = kSelBuckets / THREADS;
  const int lane = tid & 63, w = tid >> 6;
  const int ne = __builtin_amdgcn_readfirstlane((n + kSelThreads - 1) / kSelThreads);
  // block min / max
  float lo = INFINITY, hi = -INFINITY;
#pragma unroll
  for (int e = 0; e < PER; ++e)
    if (e < ne && tid + e * kSelThreads < n) {
      lo = fminf(lo, v[e]);
      hi = fmaxf(hi, v[e]);
    }
  lo = wave_min(lo);
  hi = wave_max(hi);
  __syncthreads();
  if (lane == 0) {
    sh.redf[2 * w] = lo;
    sh.redf[2 * w + 1] = hi;
  }
#pragma unroll
  for (int q = 0; q < kSelBucketsPerThread; ++q) sh.hist[tid + q * kSelThreads] = 0;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < kSelWaves; ++i) {
    lo = fminf(lo, sh.redf[2 * i]);
    hi = fmaxf(hi, sh.redf[2 * i + 1]);
  }
  const float range = hi - lo;
  const float scale = range > 0.f ? (float)kSelBuckets / range : 0.f;
  auto bucket = [&](float x) -> int {
    float f = (x - lo) * scale;  // non-finite input lands in a valid bucket too
    int d = f >= (float)(kSelBuckets - 1) ? kSelBuckets - 1 : (int)f;
    d = d < 0 ? 0 : d;
    return d > kSelBuckets - 1 ? kSelBuckets - 1 : d;
  };
#pragma unroll
  for (int e = 0; e < PER; ++e)
    if (e < ne && tid + e * kSelThreads < n) atomicAdd(&sh.hist[bucket(v[e])], 1);
  __syncthreads();
  // inclusive scan of the histogram: thread t owns kSelBucketsPerThread consecutive buckets
  int h[kSelBucketsPerThread], mine = 0;
#pragma unroll
  for (int q = 0; q < kSelBucketsPerThread; ++q) {
    h[q] = sh.hist[tid * kSelBucketsPerThread + q];
    mine += h[q];
  }
  int run = wave_excl_scan(mine, lane);
  if (lane == 63) sh.redi[w] = run + mine;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < kSelWaves; ++i)
    if (i < w) run += sh.redi[i];
  // d* = first bucket whose inclusive count reaches `want`: exactly one thread sees the
  // running count cross the target inside its own buckets
  const int target = want < n ? want : n;
  if (tid == 0) {
    sh.count = 0;
    sh.count2 = 0;
    sh.dmid = -1;
  }
#pragma unroll
  for (int q = 0; q < kSelBucketsPerThread; ++q) {
    const int before = run;
    run += h[q];
    if (before < target && run >= target) {
      sh.dstar = tid * kSelBucketsPerThread + q;
      sh.cstar = run;
    }
  }
  __syncthreads();
  if (COUNTING && want > kSelCountMin) {
    // Ordering by counting instead of a sorting network (long requests only).  The selected keys
    // -- those of the coarse buckets <= dl -- get a second, finer histogram over their own value
    // range (a bucket is a monotone function of the value, so bucket order is value order);
    // its prefix sums are the positions where the buckets' keys start; the keys are scattered
    // there and every key finds its rank inside its bucket's segment.  Six barriers instead of
    // a bitonic network's dozens.  A segment longer than kSelMaxSeg (massive ties) sends the
    // list to the network below.
    constexpr int kCap = SelectShared<THREADS, PER>::kBuf / 2;  // keys that fit twice in buf
    int dl = sh.dstar;
    dl = dl < 0 ? 0 : (dl < kSelBuckets ? dl : kSelBuckets - 1);  // (want >= 1 makes it valid anyway)
    {
      int through = run;  // count up to and including the thread's last bucket
#pragma unroll
      for (int q = kSelBucketsPerThread - 1; q >= 0; --q) {
        if (tid * kSelBucketsPerThread + q == dl) sh.clim = through;
        through -= h[q];
      }
    }
    __syncthreads();
    const int c = __builtin_amdgcn_readfirstlane(sh.clim);  // selected keys
    if (c <= kCap) {
      const float scale2 = scale * ((float)kSelBuckets / (float)(dl + 1));
      auto fine = [&](float x) -> int {
        const float f = (x - lo) * scale2;
        int d = f >= (float)(kSelBuckets - 1) ? kSelBuckets - 1 : (int)f;
        d = d < 0 ? 0 : d;
        return d > kSelBuckets - 1 ? kSelBuckets - 1 : d;
      };
#pragma unroll
      for (int q = 0; q < kSelBucketsPerThread; ++q) sh.hist[tid + q * kSelThreads] = 0;
      __syncthreads();
#pragma unroll
      for (int e = 0; e < PER; ++e)
        if (e < ne && tid + e * kSelThreads < n && bucket(v[e]) <= dl)
          atomicAdd(&sh.hist[fine(v[e])], 1);
      __syncthreads();
      int hh[kSelBucketsPerThread], mine2 = 0, big = 0;
#pragma unroll
      for (int q = 0; q < kSelBucketsPerThread; ++q) {
        hh[q] = sh.hist[tid * kSelBucketsPerThread + q];
        mine2 += hh[q];
        big |= hh[q] > kSelMaxSeg ? 1 : 0;
      }
      int run2 = wave_excl_scan(mine2, lane);
      if (lane == 63) sh.redi[w] = run2 + mine2;
      big = __syncthreads_or(big);
      if (!big) {
#pragma unroll
        for (int i = 0; i < kSelWaves; ++i)
          if (i < w) run2 += sh.redi[i];
#pragma unroll
        for (int q = 0; q < kSelBucketsPerThread; ++q) {
          sh.hist[tid * kSelBucketsPerThread + q] = run2;  // where the bucket's keys start
          run2 += hh[q];
        }
        __syncthreads();
        unsigned long long* tmp = sh.buf + kCap;
#pragma unroll
        for (int e = 0; e < PER; ++e) {
          const int j = tid + e * kSelThreads;
          if (e < ne && j < n && bucket(v[e]) <= dl) {
            const int pos = atomicAdd(&sh.hist[fine(v[e])], 1);
            tmp[pos] = ((unsigned long long)mono_of(v[e]) << 32) | (unsigned)j;
          }
        }
        __syncthreads();
        // every cell now holds the end of its bucket's segment = the start of the next one
        for (int t = tid; t < c; t += kSelThreads) {
          const unsigned long long key = tmp[t];
          const int d = fine(mono_inv((uint32_t)(key >> 32)));
          const int start = d > 0 ? sh.hist[d - 1] : 0, end = sh.hist[d];
          int rank = 0;
          for (int u = start; u < end; ++u) rank += tmp[u] < key ? 1 : 0;
          sh.buf[start + rank] = key;
        }
        __syncthreads();
        if (part2) *part2 = c;
        return c;
      }
    }
  }
  // last bucket whose inclusive count still fits one run (none if bucket 0 alone does not)
  if (part2) {
    int run2 = run;
#pragma unroll
    for (int q = kSelBucketsPerThread - 1; q >= 0; --q) {
      const int incl = run2;
      run2 -= h[q];
      // incl = count through this bucket, run2 = count before it
      if (run2 <= kSelThreads && incl > kSelThreads && tid * kSelBucketsPerThread + q > 0) {
        sh.dmid = tid * kSelBucketsPerThread + q - 1;
        sh.cmid = run2;
      }
    }
    __syncthreads();
  }
  const int dlim = sh.dstar;
  if (part2) {
    const int dmid = sh.dmid, cmid = sh.cmid, cstar = sh.cstar;
    if (cstar > kSelThreads && dmid >= 0 && dmid < dlim && cmid > 0 && cstar - cmid <= kSelThreads) {
      // two runs: buckets <= dmid (cmid keys) and (dmid, dlim] (cstar - cmid keys)
#pragma unroll
      for (int e = 0; e < PER; ++e) {
        const int j = tid + e * kSelThreads;
        if (e < ne && j < n) {
          const int d = bucket(v[e]);
          if (d <= dlim) {
            const unsigned long long key = ((unsigned long long)mono_of(v[e]) << 32) | (unsigned)j;
            if (d <= dmid) sh.buf[atomicAdd(&sh.count, 1)] = key;
            else sh.buf[kSelThreads + atomicAdd(&sh.count2, 1)] = key;
          }
        }
      }
      __syncthreads();
      const int c1 = cmid, c2 = cstar - cmid;
      const int np1 = next_pow2(c1 < kWave ? kWave : c1), np2 = next_pow2(c2 < kWave ? kWave : c2);
      for (int t = c1 + tid; t < np1; t += kSelThreads) sh.buf[t] = ~0ull;
      for (int t = c2 + tid; t < np2; t += kSelThreads) sh.buf[kSelThreads + t] = ~0ull;
      __syncthreads();
      block_bitonic_sort<kSelThreads, SelectShared<THREADS, PER>::kBuf / THREADS>(sh.buf, np1, tid);
      block_bitonic_sort<kSelThreads, SelectShared<THREADS, PER>::kBuf / THREADS>(sh.buf + kSelThreads, np2, tid);
      *part2 = c1;
      return cstar;
    }
  }
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    const int j = tid + e * kSelThreads;
    if (e < ne && j < n && bucket(v[e]) <= dlim) {
      const int slot = atomicAdd(&sh.count, 1);
      sh.buf[slot] = ((unsigned long long)mono_of(v[e]) << 32) | (unsigned)j;
    }
  }
  __syncthreads();
  const int c = __builtin_amdgcn_readfirstlane(sh.count);
  const int np = next_pow2(c < kWave ? kWave : c);
  for (int t = c + tid; t < np; t += kSelThreads) sh.buf[t] = ~0ull;
  __syncthreads();
  block_bitonic_sort<kSelThreads, SelectShared<THREADS, PER>::kBuf / THREADS>(sh.buf, np, tid);
  if (part2) *part2 = c;
  return c;
}

}  // namespace dart

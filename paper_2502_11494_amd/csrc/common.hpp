// Device-side helpers shared by the DART kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dart {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4v __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
constexpr int kMaxP = 64;        // pivots per sample
constexpr int kMaxN = 16384;     // tokens per sample
constexpr int kTileRows = 64;    // token rows per score tile (4 waves x 16)

enum { kF32 = 0, kBF16 = 1 };
enum { kMaxL1 = 0, kMinL1 = 1 };

// Shape of one call, passed to every kernel by value.
struct Geo {
  int B, D, P, Ppad;
  int N;            // dense tokens per sample (0 when ragged)
  int total_N;
  int max_N;
  int K;            // dense / uniform budget, 0 = ratio
  int keep_num, keep_den;
  int dtype, mode;
  long ld;          // X row stride, elements
  const int* cu;    // device cu_seqlens, nullptr = dense
  // ragged only, filled by k_prepare: packed offsets of keep and of score tiles
  const int* cu_keep;
  const int* tile_start;
};

struct Sample {
  int row0;  // first row of the sample in X
  int n;     // tokens
  int k;     // tokens to keep (0: skip the sample)
  int keep0; // first row of the sample in keep / Y / pos_out
};

__device__ __forceinline__ int budget_of(const Geo& g, int n) {
  return g.K > 0 ? g.K : (int)(((long)n * g.keep_num) / g.keep_den);
}

// A ragged sample is processed only if its sizes respect the limits and the budget.
__device__ __forceinline__ bool sample_ok(const Geo& g, int n, int k) {
  return n > 0 && n <= g.max_N && g.P <= n && k >= g.P && k <= n;
}

// Dense: arithmetic.  Ragged: k_prepare has validated the offsets and stored the
// per-sample budgets as differences of cu_keep (0 for a skipped sample).
__device__ __forceinline__ Sample sample_of(const Geo& g, int b) {
  Sample s;
  if (g.cu == nullptr) {
    s.row0 = b * g.N;
    s.n = g.N;
    s.k = g.K;
    s.keep0 = b * g.K;
  } else {
    s.row0 = g.cu[b];
    s.n = g.cu[b + 1] - s.row0;
    s.keep0 = g.cu_keep[b];
    s.k = g.cu_keep[b + 1] - s.keep0;
  }
  return s;
}

// Stage quota of Eq. (9)-(10) under an even split of the K-P non-pivot slots.
__device__ __forceinline__ int quota_of(int k, int P, int i) {
  int m = k - P;
  return m / P + (i < m % P ? 1 : 0);
}
// Slots filled once stages 0..i are done, pivots included.
__device__ __forceinline__ int filled_after(int k, int P, int i) {
  int m = k - P, q = m / P, r = m % P;
  return P + q * (i + 1) + (i + 1 < r ? i + 1 : r);
}

// ---- element access --------------------------------------------------------------

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// ---- order-preserving integer image of a float ----------------------------------
// -0 and +0 must compare equal, so callers add +0.0f first.
__device__ __forceinline__ uint32_t mono_of(float f) {
  uint32_t u = __float_as_uint(f);
  return u ^ ((u >> 31) ? 0xffffffffu : 0x80000000u);
}
__device__ __forceinline__ float mono_inv(uint32_t m) {
  uint32_t u = m ^ ((m >> 31) ? 0x80000000u : 0xffffffffu);
  return __uint_as_float(u);
}

// ---- wave reductions (butterfly: every lane ends with the result) ---------------

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ int wave_excl_scan(int v, int lane) {
  int x = v;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    int y = __shfl_up(x, o, kWave);
    if (lane >= o) x += y;
  }
  return x - v;
}

// ---- fp64 re-evaluation of one row (used where an fp32 decision is too close) ----
// Each lane walks the row in 16-byte pieces, lane-strided, one fp64 chain per
// quantity; the butterfly makes the result a pure function of the row's bytes.

template <int DT>
__device__ __forceinline__ void row_l1_l2_f64(const void* row, int D, int lane, double& l1,
                                              double& l2) {
  double a = 0.0, b = 0.0;
  if (DT == kBF16) {
    const u32x4* p = reinterpret_cast<const u32x4*>(row);
    for (int t = lane; t < D / 8; t += kWave) {
      u32x4 v = p[t];
      uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        double x0 = (double)bf16_lo(w[e]), x1 = (double)bf16_hi(w[e]);
        a += fabs(x0);
        a += fabs(x1);
        b = fma(x0, x0, b);
        b = fma(x1, x1, b);
      }
    }
  } else {
    const f32x4v* p = reinterpret_cast<const f32x4v*>(row);
    for (int t = lane; t < D / 4; t += kWave) {
      f32x4v v = p[t];
      float w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        double x = (double)w[e];
        a += fabs(x);
        b = fma(x, x, b);
      }
    }
  }
  l1 = wave_sum(a);
  l2 = wave_sum(b);
}

// Cosine of Eq. (7) between rows p and x in fp64; 0 if either norm is 0.
template <int DT>
__device__ __forceinline__ double row_cosine_f64(const void* prow, const void* xrow, int D,
                                                 int lane) {
  double dot = 0.0, pp = 0.0, xx = 0.0;
  if (DT == kBF16) {
    const u32x4* p = reinterpret_cast<const u32x4*>(prow);
    const u32x4* x = reinterpret_cast<const u32x4*>(xrow);
    for (int t = lane; t < D / 8; t += kWave) {
      u32x4 pv = p[t], xv = x[t];
      uint32_t pw[4] = {pv.x, pv.y, pv.z, pv.w}, xw[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        double p0 = (double)bf16_lo(pw[e]), p1 = (double)bf16_hi(pw[e]);
        double x0 = (double)bf16_lo(xw[e]), x1 = (double)bf16_hi(xw[e]);
        dot = fma(p0, x0, dot);
        dot = fma(p1, x1, dot);
        pp = fma(p0, p0, pp);
        pp = fma(p1, p1, pp);
        xx = fma(x0, x0, xx);
        xx = fma(x1, x1, xx);
      }
    }
  } else {
    const f32x4v* p = reinterpret_cast<const f32x4v*>(prow);
    const f32x4v* x = reinterpret_cast<const f32x4v*>(xrow);
    for (int t = lane; t < D / 4; t += kWave) {
      f32x4v pv = p[t], xv = x[t];
      float pw[4] = {pv.x, pv.y, pv.z, pv.w}, xw[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        double p0 = (double)pw[e], x0 = (double)xw[e];
        dot = fma(p0, x0, dot);
        pp = fma(p0, p0, pp);
        xx = fma(x0, x0, xx);
      }
    }
  }
  dot = wave_sum(dot);
  pp = wave_sum(pp);
  xx = wave_sum(xx);
  double den = sqrt(pp) * sqrt(xx);
  return den > 0.0 ? dot / den : 0.0;
}

// ---- block-wide bitonic sort of 64-bit keys in LDS -------------------------------
// n must be a power of two; all threads of the block must call.
template <int THREADS>
__device__ __forceinline__ void block_bitonic_sort(unsigned long long* s, int n, int tid) {
  for (int k = 2; k <= n; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int t = tid; t < (n >> 1); t += THREADS) {
        int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
        int l = i | j;
        unsigned long long a = s[i], b = s[l];
        bool up = (i & k) == 0;
        if ((a > b) == up) {
          s[i] = b;
          s[l] = a;
        }
      }
      __syncthreads();
    }
  }
}

__device__ __forceinline__ int next_pow2(int v) {
  int p = 1;
  while (p < v) p <<= 1;
  return p;
}

}  // namespace dart

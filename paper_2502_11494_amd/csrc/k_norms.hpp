// Row L1 norms of the criterion tensor: the pivot criterion of DART (footnote of
// Section 3.3: the K-norm is an L1 norm; Table 1 caption: pivots have the largest
// norm).  One streaming pass over [rows, Dc]; HBM-bound.
#pragma once
#include "common.hpp"

namespace dart {

// Sum of |x| over one 16-byte piece, as a fixed pairwise tree (3 roundings for
// 8 bf16 values, 2 for 4 floats).  |x| of a bf16 widened to fp32 is exact.
template <int DT>
__device__ __forceinline__ float piece_abs_sum(const u32x4& v) {
  if (DT == kBF16) {
    float a0 = fabsf(bf16_lo(v.x)) + fabsf(bf16_hi(v.x));
    float a1 = fabsf(bf16_lo(v.y)) + fabsf(bf16_hi(v.y));
    float a2 = fabsf(bf16_lo(v.z)) + fabsf(bf16_hi(v.z));
    float a3 = fabsf(bf16_lo(v.w)) + fabsf(bf16_hi(v.w));
    return (a0 + a1) + (a2 + a3);
  } else {
    float a0 = fabsf(__uint_as_float(v.x)) + fabsf(__uint_as_float(v.y));
    float a1 = fabsf(__uint_as_float(v.z)) + fabsf(__uint_as_float(v.w));
    return a0 + a1;
  }
}

// Sum of x^2 over one 16-byte piece of bf16 values: the squares are exact in fp32 (8-bit
// significands), the pairwise tree rounds three times (relative error <= 3 * 2^-24).
__device__ __forceinline__ float piece_sq_sum_bf16(const u32x4& v) {
  const float x0 = bf16_lo(v.x), x1 = bf16_hi(v.x), x2 = bf16_lo(v.y), x3 = bf16_hi(v.y);
  const float x4 = bf16_lo(v.z), x5 = bf16_hi(v.z), x6 = bf16_lo(v.w), x7 = bf16_hi(v.w);
  const float a0 = x0 * x0 + x1 * x1, a1 = x2 * x2 + x3 * x3;
  const float a2 = x4 * x4 + x5 * x5, a3 = x6 * x6 + x7 * x7;
  return (a0 + a1) + (a2 + a3);
}

// Relative bound on |fp32 norm - exact norm| for k_row_l1: piece tree, then one
// add per piece a lane owns, then the 6-step butterfly, each rounding at most
// 2^-24 relative on a sum of non-negative terms.
inline double l1_rel_bound(int dtype, int Dc) {
  int per_piece = dtype == kBF16 ? 8 : 4;
  int pieces = Dc / per_piece;
  int chain = (pieces + kWave - 1) / kWave;
  int tree = dtype == kBF16 ? 3 : 2;
  return (double)(tree + chain + 6 + 1) * 5.9604644775390625e-08;
}

// grid: ceil(rows / (4 * ROWS)) blocks of 256 threads, rounded up to a multiple of 8; wave w
// of the grid (after xcd_contiguous) owns
// rows [w*ROWS, (w+1)*ROWS).  Per row, lane l reads the pieces l, l+64, ... so a
// wave's loads are 1 KiB contiguous; 8*ROWS loads are in flight per lane.
// KEEP: ordinary loads, which leave the rows in the memory-side cache for the score
// kernel's second pass (worth it only if the whole matrix fits there); otherwise
// streaming (non-temporal) loads, which read faster.
// SPAN: the samples' rows are spans of C (Geo::span); packed row r belongs to the sample b
// with cu[b] <= r < cu[b+1] and lives at row span[b] + (r - cu[b]) of C.  Rows of a sample
// that keeps nothing (skipped: its span may be invalid) are not read.
// L2SQ (bf16 only, when the rows are the hidden states themselves): also the squared
// Euclidean norm of every row, which the score kernel divides by: piece sums in fp32 (see
// piece_sq_sum_bf16), added in fp64 in a fixed lane-strided order plus butterfly, so the
// result is a function of the row's bytes with a relative error of at most 3.5 * 2^-24.
template <int DT, int ROWS, bool KEEP, bool SPAN, bool L2SQ = false>
__global__ __launch_bounds__(256) void k_row_l1(const void* __restrict__ C, int Dc, long ldc,
                                                int rows, float* __restrict__ l1, Geo g,
                                                double* __restrict__ l2sq = nullptr) {
  const int lane = threadIdx.x & 63;
  // (ordinary loads: the plain order measured faster; streaming loads: a die per eighth)
  const long blk = KEEP ? (long)blockIdx.x : xcd_contiguous(blockIdx.x, gridDim.x);
  const long wave = blk * 4 + (threadIdx.x >> 6);
  const int esz = DT == kBF16 ? 2 : 4;
  const int pieces = Dc * esz / 16;
  const long rowbytes = ldc * esz;
  const unsigned char* base = static_cast<const unsigned char*>(C);
  const u32x4 zero = {0u, 0u, 0u, 0u};

  float acc[ROWS];
  double sq[ROWS];
  const unsigned char* rp[ROWS];
  bool live[ROWS];
#pragma unroll
  for (int r = 0; r < ROWS; ++r) {
    long row = wave * ROWS + r;
    live[r] = row < rows;
    long crow = live[r] ? row : 0;
    if (SPAN && live[r]) {
      int lo = 0, hi = g.B;
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (g.cu[mid] <= row) lo = mid; else hi = mid;
      }
      live[r] = g.cu_keep[lo + 1] != g.cu_keep[lo];
      crow = live[r] ? (long)g.span[lo] + (row - g.cu[lo]) : 0;
    }
    rp[r] = base + crow * rowbytes;
    acc[r] = 0.f;
    sq[r] = 0.0;
  }
  for (int t0 = 0; t0 < pieces; t0 += kWave * 8) {
    u32x4 v[ROWS][8];
#pragma unroll
    for (int r = 0; r < ROWS; ++r)
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        int t = t0 + u * kWave + lane;
        const u32x4* src = reinterpret_cast<const u32x4*>(rp[r]) + t;
        if (live[r] && t < pieces) v[r][u] = KEEP ? *src : __builtin_nontemporal_load(src);
        else v[r][u] = zero;
      }
#pragma unroll
    for (int r = 0; r < ROWS; ++r)
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        acc[r] += piece_abs_sum<DT>(v[r][u]);
        if (L2SQ) sq[r] += (double)piece_sq_sum_bf16(v[r][u]);
      }
  }
#pragma unroll
  for (int r = 0; r < ROWS; ++r) {
    float s = wave_sum(acc[r]);
    if (lane == 0 && live[r]) l1[wave * ROWS + r] = s;
    if (L2SQ) {
      const double q = wave_sum(sq[r]);
      if (lane == 0 && live[r]) l2sq[wave * ROWS + r] = q;
    }
  }
}

}  // namespace dart

// Retained set under ONE threshold common to all pivots: Eq. (9)-(10) with the same
// epsilon for every pivot keep token j iff its aggregate score over the pivots (the
// minimum, or the maximum: a token duplicates the context as soon as it duplicates any
// pivot) is below epsilon, and the budget sets epsilon: R = pivots + the K-P non-pivot
// tokens of lowest aggregate, ties to the lowest index.  One workgroup per sample.
//
// The aggregate of fp32 scores that each err by at most tau errs by at most tau (min
// and max are 1-Lipschitz), so the scheme of the staged kernel applies to the single
// decision: if the last aggregate taken and the first refused differ by more than
// 2*tau the fp32 order stands; otherwise every token within 2*tau of the boundary gets
// its aggregate recomputed in fp64 from the rows (only the cosines of the pivots that can
// hold it) and the band is ranked on (fp64 aggregate, index).
#pragma once
#include "common.hpp"
#include "k_select.hpp"

namespace dart {

enum { kAggMin = 1, kAggMax = 2 };

template <int PER>
struct SingleShared {
  SelectShared<1024, PER> sel;
  uint32_t R[kMaxN / 32];
  int piv[kMaxP];
  int wcnt[16];
  int below, nband;
};

// grid: B blocks of 1024.  S: pivot-major scores.  X may be nullptr (scores exact).
// PER (a multiple of 4): values per thread, PER*1024 >= the longest sample.
// scr_f64 [2*total_N]: per sample, fp64 aggregates of the band at row0 and their
// indices (as ints) at total_N + row0.
template <int DT, int PER>
__global__ __launch_bounds__(1024) void k_keep_single(
    Geo g, const float* __restrict__ S, const int* __restrict__ piv, const void* __restrict__ X,
    int* __restrict__ keep, int* __restrict__ cu_keep_out, double* __restrict__ scr_f64,
    float two_tau, int agg) {
  static_assert(PER % 4 == 0, "the score loads go four slots at a time");
  __shared__ SingleShared<PER> sh;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.x;
  const Sample sm = sample_of(g, b);
  if (cu_keep_out && tid == 0) {
    cu_keep_out[b] = sm.keep0;
    if (b == g.B - 1) cu_keep_out[g.B] = sm.keep0 + sm.k;
  }
  if (sm.k == 0) return;
  const int n = sm.n, P = g.P, m = sm.k - g.Pin;  // pivots from outside hold no slot
  const int words = (n + 31) >> 5;
  const int esz = DT == kBF16 ? 2 : 4;
  const long rowbytes = g.ld * esz;
  const unsigned char* Xb =
      X ? static_cast<const unsigned char*>(X) + (long)sm.xrow * rowbytes : nullptr;
  double* band_v = scr_f64 + sm.row0;
  int* band_j = reinterpret_cast<int*>(scr_f64 + g.total_N + sm.row0);

  for (int t = tid; t < words; t += 1024) sh.R[t] = 0u;
  if (tid < g.Pin) {
    int p = piv[b * P + tid];
    sh.piv[tid] = p < 0 ? 0 : (p < n ? p : n - 1);  // a caller's bad index must not leave X
  }
  __syncthreads();
  if (tid < g.Pin) atomicOr(&sh.R[sh.piv[tid] >> 5], 1u << (sh.piv[tid] & 31));
  __syncthreads();

  if (m > 0) {
    // aggregate of every token; pivots get 2 (above any cosine), so they sort last
    const float* Sb = S + (long)P * sm.row0;
    // Latency-bound (a few workgroups on the whole chip): 4 slots x 8 pivots = 32 independent
    // loads per batch.  Indices are clamped instead of predicated so that the loads of a
    // batch issue together; re-reading an element does not change a minimum or maximum.
    float v[PER];
    const float none = agg == kAggMin ? INFINITY : -INFINITY;
#pragma unroll
    for (int e = 0; e < PER; ++e) v[e] = none;
    for (int i0 = 0; i0 < P; i0 += 8) {
#pragma unroll
      for (int e0 = 0; e0 < PER; e0 += 4) {
        if (e0 * 1024 < n) {
          float s[4][8];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int j = tid + (e0 + e) * 1024;
            const float* col = Sb + (j < n ? j : n - 1);
#pragma unroll
            for (int q = 0; q < 8; ++q) s[e][q] = col[(long)(i0 + q < P ? i0 + q : P - 1) * n];
          }
#pragma unroll
          for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int q = 0; q < 8; ++q)
              v[e0 + e] = agg == kAggMin ? fminf(v[e0 + e], s[e][q] + 0.0f) : fmaxf(v[e0 + e], s[e][q] + 0.0f);
        }
      }
    }
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      const int j = tid + e * 1024;
      if (!(e * 1024 < n && j < n) || ((sh.R[j >> 5] >> (j & 31)) & 1u)) v[e] = 2.0f;
    }
    // Only the set of the m lowest is needed, not their order: the histogram buckets below
    // the one (d*) that holds the (m+1)-th lowest aggregate belong to it outright; bucket d*
    // alone is put in order, and its r-th and (r+1)-th keys are the last taken (fa) and the
    // first refused (fb).
    const int want = m + 1 < n ? m + 1 : n;
    const BucketSplit bs = bucket_split<1024, PER>(v, n, want, tid, sh.sel);
    if (tid == 0) {
      sh.sel.count = 0;
      sh.below = 0;
      sh.nband = 0;
    }
    __syncthreads();
    float max_below = -INFINITY;  // largest aggregate of the buckets below d* (fa if r == 0)
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      const int j = tid + e * 1024;
      if (e * 1024 < n && j < n) {
        const int d = bs.bucket(v[e]);
        if (d == bs.dstar)
          sh.sel.buf[atomicAdd(&sh.sel.count, 1)] = ((unsigned long long)mono_of(v[e]) << 32) | (unsigned)j;
        else if (d < bs.dstar)
          max_below = fmaxf(max_below, v[e]);
      }
    }
    max_below = wave_max(max_below);
    if (lane == 0) sh.sel.redg[wave] = max_below;
    __syncthreads();
    const int hs = __builtin_amdgcn_readfirstlane(sh.sel.count);  // keys of bucket d*
#pragma unroll
    for (int i = 0; i < 16; ++i) max_below = fmaxf(max_below, sh.sel.redg[i]);
    const int np = next_pow2(hs < kWave ? kWave : hs);
    for (int t = hs + tid; t < np; t += 1024) sh.sel.buf[t] = ~0ull;
    __syncthreads();
    block_bitonic_sort<1024>(sh.sel.buf, np, tid);
    const int r = m - bs.below;  // taken from bucket d*: 0 <= r <= hs
    const float fa = r > 0 ? mono_inv((uint32_t)(sh.sel.buf[r - 1] >> 32)) : max_below;
    float fb = r < hs ? mono_inv((uint32_t)(sh.sel.buf[r] >> 32)) : INFINITY;
    if (fb >= 2.0f) fb = INFINITY;  // only pivots are left
    const bool certain = Xb == nullptr || fb - fa > two_tau;
    if (certain) {
#pragma unroll
      for (int e = 0; e < PER; ++e) {
        const int j = tid + e * 1024;
        if (e * 1024 < n && j < n && bs.bucket(v[e]) < bs.dstar) atomicOr(&sh.R[j >> 5], 1u << (j & 31));
      }
      for (int t = tid; t < r; t += 1024) {
        const uint32_t j = (uint32_t)sh.sel.buf[t];
        atomicOr(&sh.R[j >> 5], 1u << (j & 31));
      }
    } else {
      // every token whose aggregate can still be on either side of the boundary goes to the
      // band; those certainly below it are taken
      const float lo = fa - two_tau, hi = fb + two_tau;
      int taken = 0;
#pragma unroll
      for (int e = 0; e < PER; ++e) {
        const int j = tid + e * 1024;
        if (e * 1024 < n && j < n) {
          const float a = v[e];
          if (a < lo) {  // certainly among the m lowest
            atomicOr(&sh.R[j >> 5], 1u << (j & 31));
            ++taken;
          } else if (a <= hi) {
            band_j[atomicAdd(&sh.nband, 1)] = j;
          }
        }
      }
      taken = wave_sum(taken);
      if (lane == 0 && taken > 0) atomicAdd(&sh.below, taken);
      __syncthreads();
      const int nband = sh.nband, need = m - sh.below;
      // fp64 aggregate of every band token, recomputed from the rows: a token per wave.  Only a
      // pivot whose fp32 score is within 2*tau of the token's fp32 aggregate can hold the
      // exact minimum (maximum): s64_k >= s32_k - tau > a32 + tau >= s64 of the fp32 argmin for
      // every other pivot k.  Usually that leaves one or two of the P cosines to compute.
      for (int u = wave; u < nband; u += 16) {
        const int j = band_j[u];
        const unsigned char* xrow = Xb + (long)j * rowbytes;
        const float none = agg == kAggMin ? INFINITY : -INFINITY;
        const float s32 = lane < P ? Sb[(long)lane * n + j] + 0.0f : none;  // lane i: pivot i
        const float a32 = agg == kAggMin ? wave_min(s32) : wave_max(s32);
        const bool near = lane < P && (agg == kAggMin ? s32 <= a32 + two_tau : s32 >= a32 - two_tau);
        unsigned long long todo = __ballot(near);
        double a = agg == kAggMin ? INFINITY : -INFINITY;
        while (todo != 0ull) {
          const int i = __ffsll((long long)todo) - 1;
          todo &= todo - 1ull;
          const double s = row_cosine_f64<DT>(pivot_row(g, X, esz, sm, b, i, piv), xrow, g.D, lane);
          a = agg == kAggMin ? fmin(a, s) : fmax(a, s);
        }
        if (lane == 0) band_v[u] = a;
      }
      __syncthreads();
      for (int u = tid; u < nband; u += 1024) {
        const double au = band_v[u];
        const int ju = band_j[u];
        int beaten = 0;
        for (int o = 0; o < nband && beaten < need; ++o) {
          const double ao = band_v[o];
          const int jo = band_j[o];
          beaten += (ao < au || (ao == au && jo < ju)) ? 1 : 0;
        }
        if (beaten < need) atomicOr(&sh.R[ju >> 5], 1u << (ju & 31));
      }
    }
  }
  __syncthreads();

  // emit the retained indices in ascending order
  const int per = (words + 1023) / 1024;
  const int w0 = tid * per;
  int mine = 0;
  for (int t = w0; t < w0 + per && t < words; ++t) mine += __popc(sh.R[t]);
  int off = wave_excl_scan(mine, lane);
  const int wtotal = __builtin_amdgcn_readlane(off + mine, 63);
  if (lane == 0) sh.wcnt[wave] = wtotal;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < 16; ++w) off += w < wave ? sh.wcnt[w] : 0;
  int* out = keep + sm.keep0 + off;
  for (int t = w0; t < w0 + per && t < words; ++t) {
    uint32_t mk = sh.R[t];
    while (mk) {
      const int bit = __ffs(mk) - 1;
      *out++ = t * 32 + bit;
      mk &= mk - 1;
    }
  }
}

}  // namespace dart

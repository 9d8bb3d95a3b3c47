// Pivot selection (Definition 1; Table 1 caption: the P tokens of largest
// criterion norm), one workgroup per sample.
//
// The fp32 norms of k_row_l1 carry a relative error of at most `tau`.  Every
// token whose fp32 norm is within that error of the P-th best could belong to
// the exact top P, so all of them are re-evaluated in fp64 and ranked by
// (fp64 norm, index).  The fp64 pass also yields the squared Euclidean norm of
// every pivot, which the score kernel divides by.
#pragma once
#include "common.hpp"
#include "k_select.hpp"

namespace dart {

constexpr int kPivLdsCand = 512;  // candidates whose fp64 norms fit in LDS

template <int THREADS, int PER = kSelPerThread>
struct PivotShared {
  SelectShared<THREADS, PER> sel;
  double c64[kPivLdsCand];
  double l2[kPivLdsCand];
  int nU;
};

// Pivot selection of sample b by one workgroup of THREADS (1024) threads.
// l1 [total_N] fp32 criterion norms; piv [B*P] (the first Pin entries of a sample are
// written); pl2 [B*Ppad] squared L2 norms of the pivots' hidden-state rows (0 for the
// other slots); scr [2*total_N] doubles.
// COH: l1 was written, and piv / pl2 will be read, by other workgroups of this launch.
template <int DT, int THREADS, bool COH, int PER = kSelPerThread>
__device__ __forceinline__ void select_pivots_body(
    const Geo& g, int b, const void* X, const void* C, int Dc, long ldc, const float* l1,
    int* piv, double* pl2, double* scr, float tau, PivotShared<THREADS, PER>& sh) {
  constexpr int kSelThreads = THREADS;
  constexpr int kSelWaves = THREADS / kWave;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const Sample sm = sample_of(g, b);
  if (tid < g.Ppad) st_dev<COH>(&pl2[b * g.Ppad + tid], 0.0);
  if (sm.k == 0) return;
  if (COH) stores_done();
  __syncthreads();  // the zeros are ordered before the pivots' norms below
  const int n = sm.n, P = g.Pin;  // pivots chosen among the tokens; stride of piv is g.P
  const float sign = g.mode == kMaxL1 ? -1.f : 1.f;  // "lowest" of -norm = largest norm

  float v[PER];
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    int j = tid + e * kSelThreads;
    v[e] = (e * kSelThreads < n && j < n) ? sign * ld_dev<COH>(&l1[sm.row0 + j]) + 0.0f : 0.f;
  }
  // Candidates: every token that may belong to the exact top P.  With vsel >= the P-th lowest
  // fp32 value, {v <= vsel + 2.5 tau |vsel|} holds every token within the norm pass's error of
  // the P-th best: usually P and a handful more.  They are ranked in fp64 below, so neither
  // their order nor the exact P-th value is needed here.
  const float vsel = rank_upper_bound<THREADS, PER>(v, n, P, tid, sh.sel);
  const float thr = vsel + 2.5f * tau * fabsf(vsel);
  if (tid == 0) sh.nU = 0;
  __syncthreads();
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    const int j = tid + e * kSelThreads;
    if (e * kSelThreads < n && j < n && v[e] <= thr)
      sh.sel.buf[atomicAdd(&sh.nU, 1)] = ((unsigned long long)mono_of(v[e]) << 32) | (unsigned)j;
  }
  __syncthreads();
  const int nU = sh.nU;  // 0 only if the norms are not numbers: then no pivot is written

  double* c64 = nU <= kPivLdsCand ? sh.c64 : scr + sm.row0;
  double* l2s = nU <= kPivLdsCand ? sh.l2 : scr + g.total_N + sm.row0;
  const int esz = DT == kBF16 ? 2 : 4;
  const unsigned char* Xb = static_cast<const unsigned char*>(X) + (long)sm.xrow * g.ld * esz;
  const unsigned char* Cb = static_cast<const unsigned char*>(C) + (long)sm.xrow * ldc * esz;
  // R candidates per wave at a time: 16 rows in flight per block with 4 or 16 waves
  constexpr int R = 16 / kSelWaves;
  for (int u0 = w * R; u0 < nU; u0 += kSelWaves * R) {
    const int live = nU - u0 < R ? nU - u0 : R;
    const void* crow[R];
    const void* xrow[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int j = (int)(uint32_t)sh.sel.buf[u0 + (r < live ? r : 0)];
      crow[r] = Cb + (long)j * ldc * esz;
      xrow[r] = Xb + (long)j * g.ld * esz;
    }
    double a[R], q[R];
    rows_l1_l2_f64<DT, R>(crow, live, Dc, lane, a, q);
    if (C != X) {
      double dummy[R];
      rows_l1_l2_f64<DT, R>(xrow, live, g.D, lane, dummy, q);
    }
    if (lane == 0) {
#pragma unroll
      for (int r = 0; r < R; ++r)
        if (r < live) {
          c64[u0 + r] = g.mode == kMaxL1 ? -a[r] : a[r];
          l2s[u0 + r] = q[r];
        }
    }
  }
  __syncthreads();
  // rank by (fp64 value, index); only ranks < P matter
  if (nU <= kWave) {
    // a wave per candidate: lane o compares candidate o with it, the ballot counts
    const bool on = lane < nU;
    const double co = on ? c64[lane] : 0.0;
    const int jo = on ? (int)(uint32_t)sh.sel.buf[lane] : 0;
    for (int u = w; u < nU; u += kSelWaves) {
      const double cu = c64[u];
      const int ju = (int)(uint32_t)sh.sel.buf[u];
      const int cnt = __popcll(__ballot(on && (co < cu || (co == cu && jo < ju))));
      if (lane == 0 && cnt < P) {
        st_dev<COH>(&piv[b * g.P + cnt], ju);
        st_dev<COH>(&pl2[b * g.Ppad + cnt], l2s[u]);
      }
    }
    return;
  }
  for (int u = tid; u < nU; u += kSelThreads) {
    const double cu = c64[u];
    const int ju = (int)(uint32_t)sh.sel.buf[u];
    int cnt = 0;
    for (int o = 0; o < nU && cnt < P; ++o) {
      const double co = c64[o];
      const int jo = (int)(uint32_t)sh.sel.buf[o];
      cnt += (co < cu || (co == cu && jo < ju)) ? 1 : 0;
    }
    if (cnt < P) {
      st_dev<COH>(&piv[b * g.P + cnt], ju);
      st_dev<COH>(&pl2[b * g.Ppad + cnt], l2s[u]);
    }
  }
}

// grid: B blocks of THREADS (1024): block b selects the pivots of sample b.
// PER*THREADS >= the longest sample.
template <int DT, int THREADS, int PER>
__global__ __launch_bounds__(THREADS) void k_select_pivots(
    Geo g, const void* __restrict__ X, const void* __restrict__ C, int Dc, long ldc,
    const float* __restrict__ l1, int* __restrict__ piv, double* __restrict__ pl2,
    double* __restrict__ scr, float tau) {
  __shared__ PivotShared<THREADS, PER> sh;
  select_pivots_body<DT, THREADS, false, PER>(g, blockIdx.x, X, C, Dc, ldc, l1, piv, pl2, scr, tau,
                                              sh);
}

}  // namespace dart

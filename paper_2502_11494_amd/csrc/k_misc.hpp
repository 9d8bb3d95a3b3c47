// Small kernels around the main passes: per-sample offsets for ragged batches,
// pivot norms for the stand-alone score entry point, and the row gather that
// compacts the retained tokens (the shortened sequence of Appendix D).
#pragma once
#include "common.hpp"

namespace dart {

// Ragged batches only.  One block of 1024 threads: validates the offsets and every
// sample and writes the packed offsets cu_keep[B+1] (retained rows; a skipped
// sample keeps 0) and tile_start[B+1] (score tiles of g.tile_rows rows).  status[0] becomes
// 1 if a non-empty sample was rejected, 2 if cu_seqlens itself is not a
// non-decreasing sequence from 0 to total_N (then every sample is skipped).
__global__ __launch_bounds__(1024) void k_prepare(Geo g, int* __restrict__ cu_keep,
                                                  int* __restrict__ tile_start,
                                                  int* __restrict__ status) {
  __shared__ int red[2][16];
  __shared__ int carry[2];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  int broken = 0;
  for (int b = tid; b < g.B; b += 1024) broken |= g.cu[b + 1] < g.cu[b] ? 1 : 0;
  if (tid == 0) {
    carry[0] = 0;
    carry[1] = 0;
    broken |= (g.cu[0] != 0 || g.cu[g.B] != g.total_N) ? 1 : 0;
  }
  broken = __syncthreads_or(broken);
  int bad = 0;
  for (int b0 = 0; b0 < g.B; b0 += 1024) {
    const int b = b0 + tid;
    int k = 0, tiles = 0;
    if (b < g.B && !broken) {
      int n = g.cu[b + 1] - g.cu[b];
      int kb = budget_of(g, n);
      if (sample_ok(g, n, kb)) {
        k = kb;
        tiles = (n + g.tile_rows - 1) / g.tile_rows;
      } else if (n != 0) {
        bad = 1;
      }
    }
    int sk = wave_excl_scan(k, lane), st = wave_excl_scan(tiles, lane);
    if (lane == 63) {
      red[0][w] = sk + k;
      red[1][w] = st + tiles;
    }
    __syncthreads();
    int bk = carry[0], bt = carry[1], tk = 0, tt = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      bk += i < w ? red[0][i] : 0;
      bt += i < w ? red[1][i] : 0;
      tk += red[0][i];
      tt += red[1][i];
    }
    if (b < g.B) {
      cu_keep[b] = bk + sk;
      tile_start[b] = bt + st;
    }
    __syncthreads();
    if (tid == 0) {
      carry[0] += tk;
      carry[1] += tt;
    }
    __syncthreads();
  }
  bad = __syncthreads_or(bad);
  if (tid == 0) {
    cu_keep[g.B] = carry[0];
    tile_start[g.B] = carry[1];
    status[0] = broken ? 2 : bad;
  }
}

// Caller-supplied pivots: status[1] = 1 if any processed sample's Pin indices are not
// distinct indices inside the sample, else 0.  grid: 1 block of 1024.
__global__ __launch_bounds__(1024) void k_check_pivots(Geo g, const int* __restrict__ piv,
                                                       int* __restrict__ status) {
  int bad = 0;
  for (int idx = threadIdx.x; idx < g.B * g.P; idx += 1024) {
    const int b = idx / g.P, i = idx - b * g.P;
    if (i >= g.Pin) continue;  // a pivot from outside the sample: nothing to check
    const Sample sm = sample_of(g, b);
    if (sm.k == 0) continue;
    const int p = piv[idx];
    bad |= (p < 0 || p >= sm.n) ? 1 : 0;
    for (int o = 0; o < i; ++o) bad |= piv[b * g.P + o] == p ? 1 : 0;
  }
  bad = __syncthreads_or(bad);
  if (threadIdx.x == 0) status[1] = bad ? 1 : 0;
}

// Squared Euclidean norms of the rows of pivots first..Ppad-1 in fp64 (0 for padding
// slots).  piv_mark (optional): entry i of a pivot from outside the sample is set to
// -1 - (its row in the sample's share of E).  grid: B blocks of 256.
template <int DT>
__global__ __launch_bounds__(256) void k_pivot_norms(Geo g, const void* __restrict__ X,
                                                     const int* __restrict__ piv, int first,
                                                     double* __restrict__ pl2,
                                                     int* __restrict__ piv_mark) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.x;
  const Sample sm = sample_of(g, b);
  const int esz = DT == kBF16 ? 2 : 4;
  if (piv_mark && tid >= g.Pin && tid < g.P) piv_mark[b * g.P + tid] = -1 - (tid - g.Pin);
  for (int i = first + wave; i < g.Ppad; i += 4) {
    double l1 = 0.0, l2 = 0.0;
    if (sm.k != 0 && i < g.P) row_l1_l2_f64<DT>(pivot_row(g, X, esz, sm, b, i, piv), g.D, lane, l1, l2);
    if (lane == 0) pl2[b * g.Ppad + i] = l2;
  }
}

// Compaction: one wave per retained row.  grid: ceil(rows_bound / 4) blocks of 256.
// Y rows are packed (stride D); copies are 16 bytes per lane, 1 KiB per wave access.
__global__ __launch_bounds__(256) void k_gather(Geo g, int esz, const void* __restrict__ X,
                                                const long long* __restrict__ pos,
                                                const int* __restrict__ keep,
                                                void* __restrict__ Y,
                                                long long* __restrict__ pos_out) {
  const int lane = threadIdx.x & 63;
  const long r = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  int b;
  if (g.cu == nullptr) {
    if (r >= (long)g.B * g.K) return;
    b = (int)(r / g.K);
  } else {
    if (r >= g.cu_keep[g.B]) return;
    int lo = 0, hi = g.B;
    while (hi - lo > 1) {
      int mid = (lo + hi) >> 1;
      if (g.cu_keep[mid] <= r) lo = mid; else hi = mid;
    }
    b = lo;
  }
  const int row0 = g.cu ? g.cu[b] : b * g.N;
  const int n = g.cu ? g.cu[b + 1] - row0 : g.N;
  int kr = keep[r];
  kr = kr < 0 ? 0 : (kr < n ? kr : n - 1);  // a caller's bad index must not leave X
  const long src = (long)row0 + kr;
  const u32x4* in = reinterpret_cast<const u32x4*>(static_cast<const unsigned char*>(X) +
                                                   src * g.ld * esz);
  u32x4* out = reinterpret_cast<u32x4*>(static_cast<unsigned char*>(Y) + r * (long)g.D * esz);
  const int pieces = g.D * esz / 16;
  for (int t0 = 0; t0 < pieces; t0 += kWave * 8) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      int t = t0 + u * kWave + lane;
      v[u] = t < pieces ? in[t] : u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      int t = t0 + u * kWave + lane;
      if (t < pieces) out[t] = v[u];
    }
  }
  if (pos && lane == 0) pos_out[r] = pos[src];
}

}  // namespace dart

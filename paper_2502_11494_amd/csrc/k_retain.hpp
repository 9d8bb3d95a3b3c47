// Retained set of Eq. (9)-(10), one workgroup per sample.
//
// R starts as the pivots.  Stage i (pivot order) walks pivot i's ascending score
// list, skips tokens already in R and takes the first quota_i others -- the
// per-pivot threshold "determined by the reduction ratio".  The walk is pure
// integer work on the lists k_order_scores prepared.
//
// The scores are fp32 with absolute error <= tau.  A stage's outcome is certain
// when the last score taken and the first one refused differ by more than 2*tau.
// Otherwise every candidate within 2*tau of that boundary is re-scored in fp64
// from its hidden-state row and the stage is decided on (fp64 score, index).
#pragma once
#include "common.hpp"

namespace dart {

constexpr int kRetThreads = 256;
constexpr int kRetWaves = kRetThreads / kWave;
constexpr int kRetWords = kMaxN / 32;

struct RetainShared {
  uint32_t R[kRetWords];
  uint32_t stage[kRetWords];
  int wsum[kRetWaves];
  int cnt;
  unsigned long long a, b;
};

__device__ __forceinline__ int block_sum_ret(int v, int tid, int* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((tid & 63) == 0) red[tid >> 6] = v;
  __syncthreads();
  int s = 0;
#pragma unroll
  for (int i = 0; i < kRetWaves; ++i) s += red[i];
  return s;
}

// grid: B blocks of kRetThreads.
// lists / S: pivot-major per sample (see k_order_scores).  X may be nullptr: then
// scores are taken as exact.  keep: packed, ascending per sample.  cu_keep_out
// (optional) [B+1].  scr_idx [total_N], scr_f64 [total_N]: per-sample scratch.
template <int DT>
__global__ __launch_bounds__(kRetThreads) void k_retain(
    Geo g, const float* __restrict__ S, const unsigned long long* __restrict__ lists,
    const int* __restrict__ piv, const void* __restrict__ X, int* __restrict__ keep,
    int* __restrict__ cu_keep_out, int* __restrict__ scr_idx, double* __restrict__ scr_f64,
    float two_tau) {
  __shared__ RetainShared sh;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.x;
  const Sample sm = sample_of(g, b);
  if (cu_keep_out && tid == 0) {
    cu_keep_out[b] = sm.keep0;
    if (b == g.B - 1) cu_keep_out[g.B] = sm.keep0 + sm.k;
  }
  if (sm.k == 0) return;
  const int n = sm.n, P = g.P, k = sm.k;
  const int words = (n + 31) >> 5;
  for (int t = tid; t < words; t += kRetThreads) {
    sh.R[t] = 0u;
    sh.stage[t] = 0u;
  }
  __syncthreads();
  if (tid < P) {
    int p = piv[b * P + tid];
    if (p >= 0 && p < n) atomicOr(&sh.R[p >> 5], 1u << (p & 31));
  }
  __syncthreads();

  const int esz = DT == kBF16 ? 2 : 4;
  const long rowbytes = g.ld * esz;
  const unsigned char* Xb =
      X ? static_cast<const unsigned char*>(X) + (long)sm.row0 * rowbytes : nullptr;

  for (int i = 0; i < P; ++i) {
    const int quota = quota_of(k, P, i);
    if (quota == 0) continue;
    const long base = (long)P * sm.row0 + (long)i * n;
    const unsigned long long* list = lists + base;
    int len = filled_after(k, P, i) + 1;
    len = len < n ? len : n;
    int taken = 0;
    bool have_b = false;
    for (int pos = 0; pos < len && !have_b; pos += kRetThreads) {
      const int t = pos + tid;
      const unsigned long long e = t < len ? list[t] : 0ull;
      const uint32_t idx = (uint32_t)e;
      const bool cand = t < len && !((sh.R[idx >> 5] >> (idx & 31)) & 1u);
      const unsigned long long bal = __ballot(cand);
      if (lane == 0) sh.wsum[wave] = __popcll(bal);
      __syncthreads();
      int before = taken, total = 0;
#pragma unroll
      for (int w = 0; w < kRetWaves; ++w) {
        before += w < wave ? sh.wsum[w] : 0;
        total += sh.wsum[w];
      }
      const int rank = before + __popcll(bal & ((1ull << lane) - 1ull));
      if (cand) {
        if (rank < quota) atomicOr(&sh.stage[idx >> 5], 1u << (idx & 31));
        if (rank == quota - 1) sh.a = e;
        if (rank == quota) sh.b = e;
      }
      taken += total;
      have_b = taken > quota;
      __syncthreads();
    }
    bool certain = true;
    float fa = 0.f, fb = 0.f;
    if (have_b && Xb) {
      fa = mono_inv((uint32_t)(sh.a >> 32));
      fb = mono_inv((uint32_t)(sh.b >> 32));
      certain = (fb - fa) > two_tau;
    }
    if (certain) {
      for (int t = tid; t < words; t += kRetThreads) {
        sh.R[t] |= sh.stage[t];
        sh.stage[t] = 0u;
      }
      __syncthreads();
      continue;
    }
    // ---- too close to call in fp32: decide the boundary band in fp64 ----
    for (int t = tid; t < words; t += kRetThreads) sh.stage[t] = 0u;
    if (tid == 0) sh.cnt = 0;
    __syncthreads();
    const float lo = fa - two_tau, hi = fb + two_tau;
    const float* Srow = S + base;
    int n_in = 0;
    for (int j = tid; j < n; j += kRetThreads) {
      if ((sh.R[j >> 5] >> (j & 31)) & 1u) continue;
      const float s = Srow[j] + 0.0f;
      if (s < lo) {  // below the band: certainly among the quota lowest
        atomicOr(&sh.R[j >> 5], 1u << (j & 31));
        ++n_in;
      } else if (s <= hi) {
        int slot = atomicAdd(&sh.cnt, 1);
        scr_idx[sm.row0 + slot] = j;
      }
    }
    const int need = quota - block_sum_ret(n_in, tid, sh.wsum);
    const int nU = sh.cnt;
    int pi = piv[b * P + i];
    pi = pi < 0 ? 0 : (pi < n ? pi : n - 1);
    const unsigned char* prow = Xb + (long)pi * rowbytes;
    for (int u = wave; u < nU; u += kRetWaves) {
      const int j = scr_idx[sm.row0 + u];
      const double s64 = row_cosine_f64<DT>(prow, Xb + (long)j * rowbytes, g.D, lane);
      if (lane == 0) scr_f64[sm.row0 + u] = s64;
    }
    __syncthreads();
    for (int u = tid; u < nU; u += kRetThreads) {
      const double su = scr_f64[sm.row0 + u];
      const int ju = scr_idx[sm.row0 + u];
      int cntb = 0;
      for (int o = 0; o < nU && cntb < need; ++o) {
        const double so = scr_f64[sm.row0 + o];
        const int jo = scr_idx[sm.row0 + o];
        cntb += (so < su || (so == su && jo < ju)) ? 1 : 0;
      }
      if (cntb < need) atomicOr(&sh.R[ju >> 5], 1u << (ju & 31));
    }
    __syncthreads();
  }

  // emit the retained indices in ascending order
  const int per = (words + kRetThreads - 1) / kRetThreads;
  const int w0 = tid * per;
  int mine = 0;
  for (int t = w0; t < w0 + per && t < words; ++t) mine += __popc(sh.R[t]);
  int off = wave_excl_scan(mine, lane);
  const int wtotal = __shfl(off + mine, 63, kWave);
  __syncthreads();
  if (lane == 0) sh.wsum[wave] = wtotal;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kRetWaves; ++w) off += w < wave ? sh.wsum[w] : 0;
  int* out = keep + sm.keep0 + off;
  for (int t = w0; t < w0 + per && t < words; ++t) {
    uint32_t m = sh.R[t];
    while (m) {
      int bit = __ffs(m) - 1;
      *out++ = t * 32 + bit;
      m &= m - 1;
    }
  }
}

}  // namespace dart

// Retained set of Eq. (9)-(10), one workgroup of four waves per sample.
//
// R starts as the pivots.  Stage i (pivot order) walks pivot i's ascending score
// list, skips tokens already in R and takes the first quota_i others -- the
// per-pivot threshold "determined by the reduction ratio".  The walk is pure
// integer work on the lists k_order_scores prepared, 64 entries per step.
//
// All four waves run the same walk redundantly, each on its own copy of the R
// bitmap, so the common path needs no barrier at all.  They only meet when a
// decision is too close for fp32:
// the scores carry an absolute error <= tau, so a stage is certain when the last
// score taken and the first one refused differ by more than 2*tau.  Otherwise
// every candidate within 2*tau of that boundary is re-scored in fp64 from its
// hidden-state row (the waves share these rows out) and the stage is decided on
// (fp64 score, index).
#pragma once
#include "common.hpp"

namespace dart {

constexpr int kRetThreads = 256;
constexpr int kRetWaves = kRetThreads / kWave;
constexpr int kRetWords = kMaxN / 32;
constexpr int kRetBand = 128;  // boundary-band candidates held in LDS

struct RetainShared {
  uint32_t R[kRetWaves][kRetWords];
  int uidx[kRetBand];
  double us64[kRetBand];
  int wsum[kRetWaves];
};

__device__ __forceinline__ bool bit_of(const uint32_t* R, uint32_t j) {
  return (R[j >> 5] >> (j & 31)) & 1u;
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
  const unsigned long long lt_mask = (1ull << lane) - 1ull;
  const int b = blockIdx.x;
  const Sample sm = sample_of(g, b);
  if (cu_keep_out && tid == 0) {
    cu_keep_out[b] = sm.keep0;
    if (b == g.B - 1) cu_keep_out[g.B] = sm.keep0 + sm.k;
  }
  if (sm.k == 0) return;
  const int n = sm.n, P = g.P, k = sm.k;
  const int words = (n + 31) >> 5;
  uint32_t* Rw = sh.R[wave];
  for (int t = lane; t < words; t += kWave) Rw[t] = 0u;
  if (lane < P) {
    int p = piv[b * P + lane];
    if (p >= 0 && p < n) atomicOr(&Rw[p >> 5], 1u << (p & 31));
  }

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

    // pass 1: find the last key taken (a) and the first key refused (b)
    unsigned long long ka = 0ull, kb = 0ull;
    bool have_b = false;
    int taken = 0;
    for (int pos = 0; pos < len && !have_b; pos += kWave) {
      const int t = pos + lane;
      const unsigned long long e = t < len ? list[t] : 0ull;
      const bool cand = t < len && !bit_of(Rw, (uint32_t)e);
      const unsigned long long bal = __ballot(cand);
      const int rank = taken + __popcll(bal & lt_mask);
      const unsigned long long ma = __ballot(cand && rank == quota - 1);
      const unsigned long long mb = __ballot(cand && rank == quota);
      if (ma) ka = __shfl(e, __ffsll((long long)ma) - 1, kWave);
      if (mb) {
        kb = __shfl(e, __ffsll((long long)mb) - 1, kWave);
        have_b = true;
      }
      taken += __popcll(bal);
    }
    const float fa = mono_inv((uint32_t)(ka >> 32)), fb = mono_inv((uint32_t)(kb >> 32));
    const bool certain = !(have_b && Xb) || (fb - fa) > two_tau;
    if (certain) {
      // pass 2: commit the first `quota` candidates
      taken = 0;
      for (int pos = 0; pos < len && taken < quota; pos += kWave) {
        const int t = pos + lane;
        const unsigned long long e = t < len ? list[t] : 0ull;
        const uint32_t idx = (uint32_t)e;
        const bool cand = t < len && !bit_of(Rw, idx);
        const unsigned long long bal = __ballot(cand);
        const int rank = taken + __popcll(bal & lt_mask);
        if (cand && rank < quota) atomicOr(&Rw[idx >> 5], 1u << (idx & 31));
        taken += __popcll(bal);
      }
      continue;
    }

    // ---- too close to call in fp32: decide the boundary band in fp64 ----
    const float lo = fa - two_tau, hi = fb + two_tau;
    int n_in = 0, nU = 0;
    bool closed = false;  // saw a key above the band: the band lies inside the list
    for (int pos = 0; pos < len && !closed; pos += kWave) {
      const int t = pos + lane;
      const unsigned long long e = t < len ? list[t] : 0ull;
      const uint32_t idx = (uint32_t)e;
      const float key = mono_inv((uint32_t)(e >> 32));
      const bool cand = t < len && !bit_of(Rw, idx);
      const bool below = cand && key < lo;              // certainly among the quota lowest
      const bool band = cand && key >= lo && key <= hi;
      const unsigned long long mband = __ballot(band);
      if (below) atomicOr(&Rw[idx >> 5], 1u << (idx & 31));
      n_in += __popcll(__ballot(below));
      const int slot = nU + __popcll(mband & lt_mask);
      if (band && slot < kRetBand) sh.uidx[slot] = (int)idx;  // every wave writes the same
      nU += __popcll(mband);
      closed = __ballot(t < len && key > hi) != 0ull;
    }
    int* uidx = sh.uidx;
    double* us64 = sh.us64;
    if ((!closed && len < n) || nU > kRetBand) {
      // the band may reach past the stored list (or is huge): sweep the whole score row
      uidx = scr_idx + sm.row0;
      us64 = scr_f64 + sm.row0;
      const float* Srow = S + base;
      nU = 0;
      for (int j0 = 0; j0 < n; j0 += kWave) {
        const int j = j0 + lane;
        const bool cand = j < n && !bit_of(Rw, (uint32_t)j);
        const float s = cand ? Srow[j] + 0.0f : 0.f;
        const bool below = cand && s < lo;
        const bool band = cand && s >= lo && s <= hi;
        const unsigned long long mband = __ballot(band);
        if (below) atomicOr(&Rw[j >> 5], 1u << (j & 31));
        n_in += __popcll(__ballot(below));
        if (band) uidx[nU + __popcll(mband & lt_mask)] = j;  // every wave writes the same
        nU += __popcll(mband);
      }
    }
    __syncthreads();  // the band list (LDS or global scratch) is complete and visible
    const int need = quota - n_in;
    int pi = piv[b * P + i];
    pi = pi < 0 ? 0 : (pi < n ? pi : n - 1);
    const unsigned char* prow = Xb + (long)pi * rowbytes;
    for (int u = wave; u < nU; u += kRetWaves) {
      const int j = uidx[u];
      const double s64 = row_cosine_f64<DT>(prow, Xb + (long)j * rowbytes, g.D, lane);
      if (lane == 0) us64[u] = s64;
    }
    __syncthreads();
    // the `need` lowest of the band by (fp64 score, index) join R, in every wave's copy
    for (int u = tid; u < nU; u += kRetThreads) {
      const double su = us64[u];
      const int ju = uidx[u];
      int beaten = 0;
      for (int o = 0; o < nU && beaten < need; ++o) {
        const double so = us64[o];
        const int jo = uidx[o];
        beaten += (so < su || (so == su && jo < ju)) ? 1 : 0;
      }
      if (beaten < need) {
#pragma unroll
        for (int w = 0; w < kRetWaves; ++w) atomicOr(&sh.R[w][ju >> 5], 1u << (ju & 31));
      }
    }
    __syncthreads();
  }

  // emit the retained indices in ascending order (each wave reads its own copy)
  const int per = (words + kRetThreads - 1) / kRetThreads;
  const int w0 = tid * per;
  int mine = 0;
  for (int t = w0; t < w0 + per && t < words; ++t) mine += __popc(Rw[t]);
  int off = wave_excl_scan(mine, lane);
  const int wtotal = __shfl(off + mine, 63, kWave);
  if (lane == 0) sh.wsum[wave] = wtotal;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kRetWaves; ++w) off += w < wave ? sh.wsum[w] : 0;
  int* out = keep + sm.keep0 + off;
  for (int t = w0; t < w0 + per && t < words; ++t) {
    uint32_t m = Rw[t];
    while (m) {
      int bit = __ffs(m) - 1;
      *out++ = t * 32 + bit;
      m &= m - 1;
    }
  }
}

}  // namespace dart

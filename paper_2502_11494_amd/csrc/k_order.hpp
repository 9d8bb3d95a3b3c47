// Score ordering: for every (sample, pivot) row of the score matrix, the lowest
// scores in ascending (score, index) order -- as many as stage i of the retained-set
// construction (Eq. 9-10) can possibly look at: the slots filled once stage i is
// done, plus one entry beyond to measure the margin of the stage's last decision.
#pragma once
#include "common.hpp"
#include "k_select.hpp"

namespace dart {

// grid: B*P blocks of THREADS (1024); block (b, i).
// S: pivot-major scores.  lists: 64-bit (score image << 32 | index) entries; the
// region of sample b starts at P*row0(b) and holds the stage lists back to back
// (see list_offset).
template <int THREADS>
__global__ __launch_bounds__(THREADS) void k_order_scores(
    Geo g, const float* __restrict__ S, unsigned long long* __restrict__ lists) {
  constexpr int kSelThreads = THREADS;
  __shared__ SelectShared<THREADS> sh;
  const int tid = threadIdx.x;
  const int b = blockIdx.x / g.P, i = blockIdx.x % g.P;
  const Sample sm = sample_of(g, b);
  if (sm.k == 0) return;
  const int n = sm.n;
  const Split sp(sm.k, g.P, g.Pin);
  const int want = sp.stage_len(n, i);
  if (want == 0) return;  // the stage takes nothing
  const float* row = S + (long)g.P * sm.row0 + (long)i * n;
  float v[kSelPerThread];
#pragma unroll
  for (int e = 0; e < kSelPerThread; ++e) {
    int j = tid + e * kSelThreads;
    v[e] = (e * kSelThreads < n && j < n) ? row[j] + 0.0f : 0.f;
  }
  int first = 0;  // keys of the first sorted run (all of them unless the sort was split)
  collect_sorted<THREADS, true>(v, n, want, tid, sh, &first);
  // offset of this stage's list = sum of the earlier stages' lengths: lane s of every wave
  // computes stage s's length, a wave scan adds them up (no loop over the stages)
  const int len_v = (tid & 63) < g.P ? sp.stage_len(n, tid & 63) : 0;
  const int off_v = wave_excl_scan(len_v, tid & 63);
  unsigned long long* out = lists + (long)g.P * sm.row0 + __builtin_amdgcn_readfirstlane(__shfl(off_v, i, kWave));
  for (int t = tid; t < want; t += kSelThreads)
    out[t] = t < first ? sh.buf[t] : sh.buf[kSelThreads + (t - first)];
}

}  // namespace dart

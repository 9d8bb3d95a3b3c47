// Score ordering: for every (sample, pivot) row of the score matrix, the lowest
// scores in ascending (score, index) order -- as many as stage i of the retained-set
// construction (Eq. 9-10) can possibly look at: the slots filled once stage i is
// done, plus one entry beyond to measure the margin of the stage's last decision.
#pragma once
#include "common.hpp"
#include "k_select.hpp"

namespace dart {

// The list of stage i of sample b, by one workgroup of THREADS (1024) threads.
// S: pivot-major scores.  lists: 64-bit (score image << 32 | index) entries; the
// region of sample b starts at P*row0(b) and holds the stage lists back to back
// (see list_offset).
// COH: S was written, and lists will be read, by other workgroups of this launch.
template <int THREADS, bool COH, int PER = kSelPerThread>
__device__ __forceinline__ void order_scores_body(const Geo& g, int b, int i, const float* S,
                                                  unsigned long long* lists,
                                                  SelectShared<THREADS, PER>& sh) {
  constexpr int kSelThreads = THREADS;
  const int tid = threadIdx.x;
  const Sample sm = sample_of(g, b);
  if (sm.k == 0) return;
  const int n = sm.n;
  const Split sp(sm.k, g.P, g.Pin);
  const int want = sp.stage_len(n, i);
  if (want == 0) return;  // the stage takes nothing
  const float* row = S + (long)g.P * sm.row0 + (long)i * n;
  float v[PER];
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    int j = tid + e * kSelThreads;
    v[e] = (e * kSelThreads < n && j < n) ? ld_dev<COH>(&row[j]) + 0.0f : 0.f;
  }
  int first = 0;  // keys of the first sorted run (all of them unless the sort was split)
  collect_sorted<THREADS, true, PER>(v, n, want, tid, sh, &first);
  // offset of this stage's list = sum of the earlier stages' lengths: lane s of every wave
  // computes stage s's length, a wave scan adds them up (no loop over the stages)
  const int len_v = (tid & 63) < g.P ? sp.stage_len(n, tid & 63) : 0;
  const int off_v = wave_excl_scan(len_v, tid & 63);
  unsigned long long* out = lists + (long)g.P * sm.row0 + __builtin_amdgcn_readfirstlane(__shfl(off_v, i, kWave));
  for (int t = tid; t < want; t += kSelThreads)
    st_dev<COH>(&out[t], t < first ? sh.buf[t] : sh.buf[kSelThreads + (t - first)]);
}

// grid: B*P blocks of THREADS (1024); block (b, i), the samples from the longest to the
// shortest where g.by_size says so.  PER*THREADS >= the longest sample.
template <int THREADS, int PER>
__global__ __launch_bounds__(THREADS) void k_order_scores(
    Geo g, const float* __restrict__ S, unsigned long long* __restrict__ lists) {
  __shared__ SelectShared<THREADS, PER> sh;
  const int slot = blockIdx.x / g.P;
  const int b = g.by_size ? g.by_size[slot] : slot;
  order_scores_body<THREADS, false, PER>(g, b, blockIdx.x % g.P, S, lists, sh);
}

}  // namespace dart

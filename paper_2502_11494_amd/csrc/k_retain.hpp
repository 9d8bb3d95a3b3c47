// Retained set of Eq. (9)-(10), one workgroup of 4 waves per sample.
//
// R starts as the pivots.  Stage i (pivot order) walks pivot i's ascending score
// list, skips tokens already in R and takes the first quota_i others -- the
// per-pivot threshold "determined by the reduction ratio".
//
// The scores are fp32 with absolute error <= tau, so a stage's outcome is certain
// only when the last score taken and the first one refused differ by more than
// 2*tau.  Decisions closer than that are settled in fp64 from the hidden-state
// rows, on (fp64 score, index).  To keep the serial part short the kernel
// speculates:
//   1. the stage lists are staged in LDS (in groups that fit);
//   2. the block walks the stages in fp32 order, 256 list entries per step (one per
//      thread, ranks by ballot + a prefix over the waves), committing what that order
//      says and queueing, for every uncertain stage, the candidates within 2*tau of
//      its boundary;
//   3. the waves re-score the queued (pivot, token) pairs in fp64, in parallel;
//   4. every uncertain stage is checked: if the fp64 order picks the same tokens
//      the speculation stands; at the first stage where it does not, that stage is
//      corrected, the later stages are undone and walked again.
// A boundary band that does not fit the queue or runs past the stored list (only
// with massive ties) is resolved by a block-wide sweep of the whole score row.
#pragma once
#include "common.hpp"

namespace dart {

constexpr int kRetThreads = 256;  // one wave per SIMD: the walk is issue-bound
constexpr int kRetWaves = kRetThreads / kWave;
constexpr int kRetWords = kMaxN / 32;
constexpr int kRetList = 12288;  // list entries staged in LDS at a time
constexpr int kRetQ = 1024;      // band candidates awaiting an fp64 score
constexpr unsigned char kOwnNone = 0xff, kOwnPivot = 0xfe;

struct RetainShared {
  unsigned long long list[kRetList];
  uint32_t R[kRetWords];
  unsigned char owner[kMaxN];  // stage that took the token (kOwnPivot, kOwnNone)
  double q_s64[kRetQ];
  int q_idx[kRetQ];
  unsigned char q_stage[kRetQ];
  unsigned char q_taken[kRetQ];
  int st_off[kMaxP];  // offset of the stage's list inside the sample's list region
  int st_len[kMaxP];
  int st_qlo[kMaxP], st_qhi[kMaxP];
  unsigned char st_unc[kMaxP];
  __attribute__((aligned(16))) int wcnt[2][kRetWaves];
  unsigned long long ka, kb;
  int qn, need, cnt, bad_first;
};

__device__ __forceinline__ bool bit_of(const uint32_t* R, uint32_t j) {
  return (R[j >> 5] >> (j & 31)) & 1u;
}
__device__ __forceinline__ void set_bit(uint32_t* R, uint32_t j) {
  atomicOr(&R[j >> 5], 1u << (j & 31));
}
__device__ __forceinline__ void clear_bit(uint32_t* R, uint32_t j) {
  atomicAnd(&R[j >> 5], ~(1u << (j & 31)));
}

// (score, index) pairs compare lexicographically
__device__ __forceinline__ bool pair_less(double sa, int ja, double sb, int jb) {
  return sa < sb || (sa == sb && ja < jb);
}

// grid: B blocks of kRetThreads.
// lists: per sample at P*row0, stage lists back to back (see k_order_scores).
// S: pivot-major scores.  X may be nullptr: then scores are taken as exact.
// keep: packed, ascending per sample.  cu_keep_out (optional) [B+1].
// scr_f64 [2*total_N] doubles: per-sample scratch at row0 (fallback sweep only).
template <int DT>
__global__ __launch_bounds__(kRetThreads) void k_retain(
    Geo g, const float* __restrict__ S, const unsigned long long* __restrict__ lists,
    const int* __restrict__ piv, const void* __restrict__ X, int* __restrict__ keep,
    int* __restrict__ cu_keep_out, double* __restrict__ scr_f64, float two_tau) {
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
  const int esz = DT == kBF16 ? 2 : 4;
  const long rowbytes = g.ld * esz;
  const unsigned char* Xb =
      X ? static_cast<const unsigned char*>(X) + (long)sm.row0 * rowbytes : nullptr;
  const unsigned long long* glist = lists + (long)P * sm.row0;
  double* sweep_s64 = scr_f64 + sm.row0;                                   // fallback sweep
  int* sweep_idx = reinterpret_cast<int*>(scr_f64 + g.total_N + sm.row0);  // fallback sweep

  const Split sp(k, P);
  for (int t = tid; t < words; t += kRetThreads) sh.R[t] = 0u;
  for (int t = tid; t < (n + 3) / 4; t += kRetThreads)
    reinterpret_cast<uint32_t*>(sh.owner)[t] = 0xffffffffu;
  if (tid < P) {
    sh.st_len[tid] = sp.stage_len(n, tid);
    sh.st_off[tid] = (int)sp.list_offset(n, tid);
  }
  __syncthreads();
  if (tid < P) {
    int p = piv[b * P + tid];
    if (p >= 0 && p < n) {
      set_bit(sh.R, (uint32_t)p);
      sh.owner[p] = kOwnPivot;
    }
  }
  __syncthreads();

  // Rank, within one step of the walk, of this thread's candidate among all the
  // block's candidates, offset by `taken`; `total` = candidates of the step.
  // One barrier (the per-wave counts alternate between two buffers, so a slow wave
  // still reading one step's counts is never overrun); every thread must call.
  static_assert(kRetWaves == 4, "the wave prefix below reads four counts at once");
  int parity = 0;
  auto step_rank = [&](bool cand, int taken, int& total) -> int {
    const unsigned long long bal = __ballot(cand);
    if (lane == 0) sh.wcnt[parity][wave] = __popcll(bal);
    __syncthreads();
    const int c0 = sh.wcnt[parity][0], c1 = sh.wcnt[parity][1], c2 = sh.wcnt[parity][2],
              c3 = sh.wcnt[parity][3];
    parity ^= 1;
    total = c0 + c1 + c2 + c3;
    const int before = (wave > 0 ? c0 : 0) + (wave > 1 ? c1 : 0) + (wave > 2 ? c2 : 0);
    return taken + before + __popcll(bal & lt_mask);
  };

  int next = 0;      // first stage not yet final (block-uniform)
  int group_hi = 0;  // stages whose lists are staged: [stage at staging time, group_hi)
  int group_base = 0, staged_total = 0;
  while (next < P) {
    if (next >= group_hi) {
      // stage the lists of as many further stages as fit (the first one maybe partly)
      group_base = sh.st_off[next];
      int tot = sh.st_len[next] < kRetList ? sh.st_len[next] : kRetList;
      group_hi = next + 1;
      while (group_hi < P && tot + sh.st_len[group_hi] <= kRetList) tot += sh.st_len[group_hi++];
      staged_total = tot;
      for (int t0 = 0; t0 < tot; t0 += 12 * kRetThreads) {
        unsigned long long v[12];  // 24 KiB of loads in flight per step
#pragma unroll
        for (int u = 0; u < 12; ++u) {
          const int t = t0 + u * kRetThreads + tid;
          v[u] = t < tot ? glist[group_base + t] : 0ull;
        }
#pragma unroll
        for (int u = 0; u < 12; ++u) {
          const int t = t0 + u * kRetThreads + tid;
          if (t < tot) sh.list[t] = v[u];
        }
      }
    }
    if (tid == 0) sh.qn = 0;
    __syncthreads();

    // ------------------------------------------------------------------ speculative walk
    int walk_end = group_hi, fb_stage = -1;
    float fb_a = 0.f, fb_b = 0.f;
    for (int i = next; i < group_hi; ++i) {
      const int quota = sp.quota(i);
      if (tid == 0) sh.st_unc[i] = 0;
      if (quota == 0) continue;
      const int len = sh.st_len[i];
      const int off = sh.st_off[i] - group_base;  // position of the list in sh.list
      const unsigned long long* gl = glist + sh.st_off[i];
      auto entry = [&](int p) -> unsigned long long {
        if (off + p < staged_total) return sh.list[off + p];
        return gl[p];
      };
      // commit the first `quota` candidates of the fp32 order; a = last key taken,
      // b = first key refused
      bool have_b = false;
      int taken = 0, pos = 0, rank = 0;
      unsigned long long e = 0ull;
      bool cand = false;
      const bool staged = off + len <= staged_total;  // the usual case: plain LDS reads
      for (; pos < len && !have_b; pos += kRetThreads) {
        const int t = pos + tid;
        if (staged) e = t < len ? sh.list[off + t] : 0ull;
        else e = t < len ? entry(t) : 0ull;
        cand = t < len && !bit_of(sh.R, (uint32_t)e);
        int total;
        rank = step_rank(cand, taken, total);
        if (cand) {
          if (rank < quota) {
            set_bit(sh.R, (uint32_t)e);
            sh.owner[(uint32_t)e] = (unsigned char)i;
          }
          if (rank == quota - 1) sh.ka = e;
          if (rank == quota) sh.kb = e;
        }
        taken += total;
        have_b = taken > quota;
      }
      __syncthreads();
      const float fa = mono_inv((uint32_t)(sh.ka >> 32)), fb = mono_inv((uint32_t)(sh.kb >> 32));
      const bool unc = have_b && Xb && !((fb - fa) > two_tau);
      if (!unc) continue;

      // queue the candidates within 2*tau of the boundary for an fp64 score
      const float lo = fa - two_tau, hi = fb + two_tau;
      const int qlo = sh.qn;
      const int pos0 = pos - kRetThreads;  // the step that found b; its registers are live
      const float key = mono_inv((uint32_t)(e >> 32));
      const bool live = pos0 + tid < len;
      // does the band start inside this step?  (a candidate of it lies below the band)
      const bool starts_here = __syncthreads_or((pos0 == 0) || (cand && key < lo));
      bool closed = __syncthreads_or(live && key > hi);
      if (tid == 0) sh.need = 0;
      __syncthreads();
      if (starts_here) {
        if (cand && key >= lo && key <= hi) {
          const int slot = atomicAdd(&sh.qn, 1);
          if (slot < kRetQ) {
            sh.q_idx[slot] = (int)(uint32_t)e;
            sh.q_stage[slot] = (unsigned char)i;
            sh.q_taken[slot] = rank < quota ? 1 : 0;
          }
        }
        // the band may go on past this step: nothing there was committed
        for (int p2 = pos; p2 < len && !closed; p2 += kRetThreads) {
          const int t = p2 + tid;
          const unsigned long long e2 = t < len ? entry(t) : 0ull;
          const float key2 = mono_inv((uint32_t)(e2 >> 32));
          if (t < len && !bit_of(sh.R, (uint32_t)e2) && key2 <= hi) {
            const int slot = atomicAdd(&sh.qn, 1);
            if (slot < kRetQ) {
              sh.q_idx[slot] = (int)(uint32_t)e2;
              sh.q_stage[slot] = (unsigned char)i;
              sh.q_taken[slot] = 0;
            }
          }
          closed = __syncthreads_or(t < len && key2 > hi);
        }
      } else {
        // rare: the band reaches back into earlier steps.  Take the stage's commits
        // back and scan its list from the start.
        for (int j = tid; j < n; j += kRetThreads)
          if (sh.owner[j] == (unsigned char)i) clear_bit(sh.R, (uint32_t)j);
        __syncthreads();
        closed = false;
        int tk = 0;
        for (int p2 = 0; p2 < len && !closed; p2 += kRetThreads) {
          const int t = p2 + tid;
          const unsigned long long e2 = t < len ? entry(t) : 0ull;
          const float key2 = mono_inv((uint32_t)(e2 >> 32));
          const bool c2 = t < len && !bit_of(sh.R, (uint32_t)e2);
          int total;
          const int rk = step_rank(c2, tk, total);
          if (c2 && key2 >= lo && key2 <= hi) {
            const int slot = atomicAdd(&sh.qn, 1);
            if (slot < kRetQ) {
              sh.q_idx[slot] = (int)(uint32_t)e2;
              sh.q_stage[slot] = (unsigned char)i;
              sh.q_taken[slot] = rk < quota ? 1 : 0;
            }
          }
          tk += total;
          closed = __syncthreads_or(t < len && key2 > hi);
        }
        for (int j = tid; j < n; j += kRetThreads)
          if (sh.owner[j] == (unsigned char)i) set_bit(sh.R, (uint32_t)j);
      }
      __syncthreads();
      if (sh.qn > kRetQ || (!closed && len < n)) {
        // too many ties for the queue, or the band runs past the stored list:
        // take the stage back and leave it to the block-wide sweep
        for (int j = tid; j < n; j += kRetThreads)
          if (sh.owner[j] == (unsigned char)i) {
            clear_bit(sh.R, (uint32_t)j);
            sh.owner[j] = kOwnNone;
          }
        __syncthreads();
        if (tid == 0) sh.qn = qlo;
        fb_stage = i;
        walk_end = i;
        fb_a = fa;
        fb_b = fb;
        __syncthreads();
        break;
      }
      if (tid == 0) {
        sh.st_unc[i] = 1;
        sh.st_qlo[i] = qlo;
        sh.st_qhi[i] = sh.qn;
      }
      __syncthreads();
    }

    // ------------------------------------------------------------------ fp64 scores of the queue
    const int qn = sh.qn;
    for (int q = wave; q < qn; q += kRetWaves) {
      int pi = piv[b * P + sh.q_stage[q]];
      pi = pi < 0 ? 0 : (pi < n ? pi : n - 1);
      const double s64 = row_cosine_f64<DT>(Xb + (long)pi * rowbytes,
                                            Xb + (long)sh.q_idx[q] * rowbytes, g.D, lane);
      if (lane == 0) sh.q_s64[q] = s64;
    }
    if (tid == 0) sh.bad_first = walk_end;
    __syncthreads();

    // ------------------------------------------------------------------ check the speculation
    // wave w checks the uncertain stages next+w, next+w+4, ...: the fp64 order agrees
    // with the fp32 order iff the largest pair taken is below the smallest pair refused
    for (int i = next + wave; i < walk_end; i += kRetWaves) {
      if (!sh.st_unc[i]) continue;
      const int qlo = sh.st_qlo[i], qhi = sh.st_qhi[i];
      double mt_s = -INFINITY, mu_s = INFINITY;
      int mt_j = -1, mu_j = 0x7fffffff;
      for (int q = qlo + lane; q < qhi; q += kWave) {
        const double s = sh.q_s64[q];
        const int j = sh.q_idx[q];
        if (sh.q_taken[q]) {
          if (pair_less(mt_s, mt_j, s, j)) { mt_s = s; mt_j = j; }
        } else {
          if (pair_less(s, j, mu_s, mu_j)) { mu_s = s; mu_j = j; }
        }
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        const double s1 = __shfl_xor(mt_s, o, kWave), s2 = __shfl_xor(mu_s, o, kWave);
        const int j1 = __shfl_xor(mt_j, o, kWave), j2 = __shfl_xor(mu_j, o, kWave);
        if (pair_less(mt_s, mt_j, s1, j1)) { mt_s = s1; mt_j = j1; }
        if (pair_less(s2, j2, mu_s, mu_j)) { mu_s = s2; mu_j = j2; }
      }
      if (!pair_less(mt_s, mt_j, mu_s, mu_j) && lane == 0) atomicMin(&sh.bad_first, i);
    }
    __syncthreads();
    const int bad = sh.bad_first;
    if (bad < walk_end) {
      // fp64 picks other tokens at stage `bad`: undo the later stages, correct this one
      for (int j = tid; j < n; j += kRetThreads) {
        const unsigned char o = sh.owner[j];
        if (o < kOwnPivot && (int)o > bad) {
          clear_bit(sh.R, (uint32_t)j);
          sh.owner[j] = kOwnNone;
        }
      }
      const int qlo = sh.st_qlo[bad], qhi = sh.st_qhi[bad];
      int need = 0;
      for (int q = qlo; q < qhi; ++q) need += sh.q_taken[q];
      __syncthreads();
      for (int q = qlo + tid; q < qhi; q += kRetThreads) {
        const double s = sh.q_s64[q];
        const int j = sh.q_idx[q];
        int beaten = 0;
        for (int o = qlo; o < qhi && beaten < need; ++o)
          beaten += pair_less(sh.q_s64[o], sh.q_idx[o], s, j) ? 1 : 0;
        const bool chosen = beaten < need;
        if (sh.q_taken[q] && !chosen) {
          clear_bit(sh.R, (uint32_t)j);
          sh.owner[j] = kOwnNone;
        }
        if (!sh.q_taken[q] && chosen) {
          set_bit(sh.R, (uint32_t)j);
          sh.owner[j] = (unsigned char)bad;
        }
      }
      next = bad + 1;
      __syncthreads();
      continue;
    }
    next = walk_end;
    if (fb_stage != walk_end || walk_end >= P) continue;

    // ------------------------------------------------------------------ block-wide fallback
    {
      const int i = fb_stage;
      const int quota = sp.quota(i);
      const float lo = fb_a - two_tau, hi = fb_b + two_tau;
      const float* Srow = S + (long)P * sm.row0 + (long)i * n;
      if (tid == 0) sh.cnt = 0;
      __syncthreads();
      int n_in = 0;
      for (int j = tid; j < n; j += kRetThreads) {
        if (bit_of(sh.R, (uint32_t)j)) continue;
        const float s = Srow[j] + 0.0f;
        if (s < lo) {  // below the band: certainly among the quota lowest
          set_bit(sh.R, (uint32_t)j);
          sh.owner[j] = (unsigned char)i;
          ++n_in;
        } else if (s <= hi) {
          sweep_idx[atomicAdd(&sh.cnt, 1)] = j;
        }
      }
      n_in = wave_sum(n_in);
      if (lane == 0) sh.wcnt[0][wave] = n_in;
      __syncthreads();
      int need = quota;
#pragma unroll
      for (int w = 0; w < kRetWaves; ++w) need -= sh.wcnt[0][w];
      const int nU = sh.cnt;
      int pi = piv[b * P + i];
      pi = pi < 0 ? 0 : (pi < n ? pi : n - 1);
      const unsigned char* prow = Xb + (long)pi * rowbytes;
      for (int u = wave; u < nU; u += kRetWaves) {
        const double s64 =
            row_cosine_f64<DT>(prow, Xb + (long)sweep_idx[u] * rowbytes, g.D, lane);
        if (lane == 0) sweep_s64[u] = s64;
      }
      __syncthreads();
      for (int u = tid; u < nU; u += kRetThreads) {
        const double su = sweep_s64[u];
        const int ju = sweep_idx[u];
        int beaten = 0;
        for (int o = 0; o < nU && beaten < need; ++o)
          beaten += pair_less(sweep_s64[o], sweep_idx[o], su, ju) ? 1 : 0;
        if (beaten < need) {
          set_bit(sh.R, (uint32_t)ju);
          sh.owner[ju] = (unsigned char)i;
        }
      }
      next = i + 1;
      __syncthreads();
    }
  }
  __syncthreads();

  // emit the retained indices in ascending order
  const int per = (words + kRetThreads - 1) / kRetThreads;
  const int w0 = tid * per;
  int mine = 0;
  for (int t = w0; t < w0 + per && t < words; ++t) mine += __popc(sh.R[t]);
  int off = wave_excl_scan(mine, lane);
  const int wtotal = __shfl(off + mine, 63, kWave);
  if (lane == 0) sh.wcnt[0][wave] = wtotal;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kRetWaves; ++w) off += w < wave ? sh.wcnt[0][w] : 0;
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

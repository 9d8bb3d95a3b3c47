// Retained set of Eq. (9)-(10), one workgroup per sample.
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
//   2. wave 0 walks the stages in fp32 order, 64 entries per step, committing what
//      that order says and queueing, for every uncertain stage, the candidates
//      within 2*tau of its boundary;
//   3. all waves re-score the queued (pivot, token) pairs in fp64, in parallel;
//   4. wave 0 checks every uncertain stage in order: if the fp64 order picks the
//      same tokens the speculation stands; at the first stage where it does not,
//      that stage is corrected, the later stages are undone and walked again.
// A boundary band that does not fit the queue or runs past the stored list (only
// with massive ties) is resolved by a block-wide sweep of the whole score row.
#pragma once
#include "common.hpp"

namespace dart {

constexpr int kRetThreads = 1024;
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
  int st_off[kMaxP];   // offset of the stage's list inside the sample's list region
  int st_len[kMaxP];
  int st_qlo[kMaxP], st_qhi[kMaxP], st_nin[kMaxP];
  unsigned char st_unc[kMaxP];
  int red[kRetWaves];
  int cnt;
  // block-uniform control, written by wave 0 between barriers
  int next, walk_end, q_count, fb_stage, need_fb;
  float fb_a, fb_b;
};

__device__ __forceinline__ bool bit_of(const uint32_t* R, uint32_t j) {
  return (R[j >> 5] >> (j & 31)) & 1u;
}
__device__ __forceinline__ void set_bit(uint32_t* R, uint32_t j) { atomicOr(&R[j >> 5], 1u << (j & 31)); }
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
    int* __restrict__ cu_keep_out, double* __restrict__ scr_f64,
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
  const int esz = DT == kBF16 ? 2 : 4;
  const long rowbytes = g.ld * esz;
  const unsigned char* Xb =
      X ? static_cast<const unsigned char*>(X) + (long)sm.row0 * rowbytes : nullptr;
  const unsigned long long* glist = lists + (long)P * sm.row0;
  double* sweep_s64 = scr_f64 + sm.row0;         // fallback sweep: fp64 scores
  int* sweep_idx = reinterpret_cast<int*>(scr_f64 + g.total_N + sm.row0);  // and tokens

  const Split sp(k, P);
  for (int t = tid; t < words; t += kRetThreads) sh.R[t] = 0u;
  for (int t = tid; t < (n + 3) / 4; t += kRetThreads)
    reinterpret_cast<uint32_t*>(sh.owner)[t] = 0xffffffffu;
  if (tid < P) {
    sh.st_len[tid] = sp.stage_len(n, tid);
    sh.st_off[tid] = (int)sp.list_offset(n, tid);
  }
  if (tid == 0) sh.next = 0;
  __syncthreads();
  if (tid < P) {
    int p = piv[b * P + tid];
    if (p >= 0 && p < n) {
      set_bit(sh.R, (uint32_t)p);
      sh.owner[p] = kOwnPivot;
    }
  }
  int group_hi = 0;                // stages whose lists are staged: [next at staging, group_hi)
  int group_base = 0;              // list-region offset of the first staged entry
  int staged_total = 0;
  __syncthreads();

  while (true) {
    const int next = sh.next;
    if (next >= P) break;
    if (next >= group_hi) {
      // stage the lists of as many further stages as fit (the first one maybe partly)
      group_base = sh.st_off[next];
      int tot = sh.st_len[next] < kRetList ? sh.st_len[next] : kRetList;
      group_hi = next + 1;
      while (group_hi < P && tot + sh.st_len[group_hi] <= kRetList) tot += sh.st_len[group_hi++];
      staged_total = tot;
      __syncthreads();  // nobody still reads the previous group
      for (int t0 = 0; t0 < tot; t0 += 4 * kRetThreads) {
        unsigned long long v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int t = t0 + u * kRetThreads + tid;
          v[u] = t < tot ? glist[group_base + t] : 0ull;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int t = t0 + u * kRetThreads + tid;
          if (t < tot) sh.list[t] = v[u];
        }
      }
      __syncthreads();
    }

    // ---------------------------------------------------------------- speculative walk
    if (wave == 0) {
      int qn = 0, fb_stage = -1, walk_end = group_hi;
      for (int i = next; i < group_hi; ++i) {
        const int quota = sp.quota(i);
        sh.st_unc[i] = 0;
        if (quota == 0) continue;
        const int len = sh.st_len[i];
        const int off = sh.st_off[i] - group_base;  // position of the list in sh.list
        const unsigned long long* gl = glist + sh.st_off[i];
        auto entry = [&](int p) -> unsigned long long {
          return (off + p < staged_total) ? sh.list[off + p] : gl[p];
        };
        // One pass, 256 entries per step: commit the first `quota` candidates of the
        // fp32 order and find the last key taken (a) and the first key refused (b).
        unsigned long long ka = 0ull, kb = 0ull;
        bool have_b = false;
        int taken = 0, pos = 0;
        unsigned long long e[4];
        bool cand[4];
        int rank[4];
        for (; pos < len && !have_b; pos += 4 * kWave) {
          const bool in_lds = off + pos + 4 * kWave <= staged_total;
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const int t = pos + c * kWave + lane;
            if (in_lds) e[c] = sh.list[off + t];
            else e[c] = t < len ? entry(t) : 0ull;
          }
          unsigned long long bal[4];
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const int t = pos + c * kWave + lane;
            cand[c] = t < len && !bit_of(sh.R, (uint32_t)e[c]);
            bal[c] = __ballot(cand[c]);
          }
          int before = taken;
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            rank[c] = before + __popcll(bal[c] & lt_mask);
            before += __popcll(bal[c]);
          }
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            if (cand[c] && rank[c] < quota) {
              set_bit(sh.R, (uint32_t)e[c]);
              sh.owner[(uint32_t)e[c]] = (unsigned char)i;
            }
            const unsigned long long ma = __ballot(cand[c] && rank[c] == quota - 1);
            const unsigned long long mb = __ballot(cand[c] && rank[c] == quota);
            if (ma) ka = __shfl(e[c], __ffsll((long long)ma) - 1, kWave);
            if (mb) {
              kb = __shfl(e[c], __ffsll((long long)mb) - 1, kWave);
              have_b = true;
            }
          }
          taken = before;
        }
        const float fa = mono_inv((uint32_t)(ka >> 32)), fb = mono_inv((uint32_t)(kb >> 32));
        const bool unc = have_b && Xb && !((fb - fa) > two_tau);
        if (unc) {
          // queue the candidates within 2*tau of the boundary for an fp64 score
          const float lo = fa - two_tau, hi = fb + two_tau;
          const int qlo = qn;
          const int pos0 = pos - 4 * kWave;  // the step that found b; its registers are live
          // does the band start inside this step?  (some candidate of it lies below the band)
          bool starts_here = pos0 == 0;
          bool closed = false;
          int need = 0;
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const int t = pos0 + c * kWave + lane;
            const float key = mono_inv((uint32_t)(e[c] >> 32));
            starts_here = starts_here || __ballot(cand[c] && key < lo) != 0ull;
            closed = closed || __ballot(t < len && key > hi) != 0ull;
          }
          if (starts_here) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
              const float key = mono_inv((uint32_t)(e[c] >> 32));
              const bool band = cand[c] && key >= lo && key <= hi;
              const unsigned long long mband = __ballot(band);
              const int slot = qn + __popcll(mband & lt_mask);
              if (band && slot < kRetQ) {
                sh.q_idx[slot] = (int)(uint32_t)e[c];
                sh.q_stage[slot] = (unsigned char)i;
                sh.q_taken[slot] = rank[c] < quota ? 1 : 0;
              }
              need += __popcll(__ballot(band && rank[c] < quota));
              qn += __popcll(mband);
            }
            // the band may go on past this step: nothing there was committed
            for (int p2 = pos; p2 < len && !closed; p2 += kWave) {
              const int t = p2 + lane;
              const unsigned long long e2 = t < len ? entry(t) : 0ull;
              const float key = mono_inv((uint32_t)(e2 >> 32));
              const bool band = t < len && !bit_of(sh.R, (uint32_t)e2) && key <= hi;
              const unsigned long long mband = __ballot(band);
              const int slot = qn + __popcll(mband & lt_mask);
              if (band && slot < kRetQ) {
                sh.q_idx[slot] = (int)(uint32_t)e2;
                sh.q_stage[slot] = (unsigned char)i;
                sh.q_taken[slot] = 0;
              }
              qn += __popcll(mband);
              closed = __ballot(t < len && key > hi) != 0ull;
            }
          } else {
            // rare: the band reaches back into earlier steps.  Take the stage's commits
            // back and scan its list from the start.
            for (int j = lane; j < n; j += kWave)
              if (sh.owner[j] == (unsigned char)i) clear_bit(sh.R, (uint32_t)j);
            closed = false;
            taken = 0;
            for (int p2 = 0; p2 < len && !closed; p2 += kWave) {
              const int t = p2 + lane;
              const unsigned long long e2 = t < len ? entry(t) : 0ull;
              const uint32_t idx = (uint32_t)e2;
              const float key = mono_inv((uint32_t)(e2 >> 32));
              const bool cnd = t < len && !bit_of(sh.R, idx);
              const unsigned long long bal = __ballot(cnd);
              const int rk = taken + __popcll(bal & lt_mask);
              const bool band = cnd && key >= lo && key <= hi;
              const unsigned long long mband = __ballot(band);
              const int slot = qn + __popcll(mband & lt_mask);
              if (band && slot < kRetQ) {
                sh.q_idx[slot] = (int)idx;
                sh.q_stage[slot] = (unsigned char)i;
                sh.q_taken[slot] = rk < quota ? 1 : 0;
              }
              need += __popcll(__ballot(band && rk < quota));
              qn += __popcll(mband);
              taken += __popcll(bal);
              closed = __ballot(t < len && key > hi) != 0ull;
            }
            for (int j = lane; j < n; j += kWave)
              if (sh.owner[j] == (unsigned char)i) set_bit(sh.R, (uint32_t)j);
          }
          if (qn > kRetQ || (!closed && len < n)) {
            // too many ties for the queue, or the band runs past the stored list:
            // take the stage back and leave it to the block-wide sweep
            for (int j = lane; j < n; j += kWave)
              if (sh.owner[j] == (unsigned char)i) {
                clear_bit(sh.R, (uint32_t)j);
                sh.owner[j] = kOwnNone;
              }
            qn = qlo;
            fb_stage = i;
            walk_end = i;
            if (lane == 0) {
              sh.fb_a = fa;
              sh.fb_b = fb;
            }
            break;
          }
          sh.st_unc[i] = 1;
          sh.st_qlo[i] = qlo;
          sh.st_qhi[i] = qn;
          sh.st_nin[i] = quota - need;
        }
      }
      if (lane == 0) {
        sh.walk_end = walk_end;
        sh.q_count = qn;
        sh.fb_stage = fb_stage;
      }
    }
    __syncthreads();

    // ---------------------------------------------------------------- fp64 scores of the queue
    {
      const int qn = sh.q_count;
      for (int q = wave; q < qn; q += kRetWaves) {
        int pi = piv[b * P + sh.q_stage[q]];
        pi = pi < 0 ? 0 : (pi < n ? pi : n - 1);
        const double s64 = row_cosine_f64<DT>(Xb + (long)pi * rowbytes,
                                              Xb + (long)sh.q_idx[q] * rowbytes, g.D, lane);
        if (lane == 0) sh.q_s64[q] = s64;
      }
    }
    __syncthreads();

    // ---------------------------------------------------------------- check the speculation
    if (wave == 0) {
      const int walk_end = sh.walk_end;
      int new_next = walk_end;
      bool fixed = false;
      for (int i = next; i < walk_end && !fixed; ++i) {
        if (!sh.st_unc[i]) continue;
        const int qlo = sh.st_qlo[i], qhi = sh.st_qhi[i];
        // largest pair among the taken, smallest among the refused
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
        if (pair_less(mt_s, mt_j, mu_s, mu_j)) continue;  // fp64 agrees with the fp32 order

        // fp64 picks other tokens: undo the later stages, then correct this one
        for (int j = lane; j < n; j += kWave) {
          const unsigned char o = sh.owner[j];
          if (o < kOwnPivot && (int)o > i) {
            clear_bit(sh.R, (uint32_t)j);
            sh.owner[j] = kOwnNone;
          }
        }
        int need = 0;
        for (int q = qlo + lane; q < qhi; q += kWave) need += sh.q_taken[q];
        need = wave_sum(need);
        for (int q = qlo + lane; q < qhi; q += kWave) {
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
            sh.owner[j] = (unsigned char)i;
          }
        }
        new_next = i + 1;
        fixed = true;
      }
      if (lane == 0) {
        sh.next = new_next;
        sh.need_fb = (!fixed && sh.fb_stage == walk_end && walk_end < P) ? 1 : 0;
      }
    }
    __syncthreads();

    // ---------------------------------------------------------------- block-wide fallback
    if (sh.need_fb) {
      const int i = sh.next;
      const int quota = sp.quota(i);
      const float lo = sh.fb_a - two_tau, hi = sh.fb_b + two_tau;
      const float* Srow = S + (long)P * sm.row0 + (long)i * n;
      if (tid == 0) sh.cnt = 0;
      __syncthreads();
      int n_in = 0;
      for (int j = tid; j < n; j += kRetThreads) {
        if (bit_of(sh.R, (uint32_t)j)) continue;
        const float s = Srow[j] + 0.0f;
        if (s < lo) {  // below the band: certainly among the quota lowest
          set_bit(sh.R, (uint32_t)j);
          ++n_in;
        } else if (s <= hi) {
          sweep_idx[atomicAdd(&sh.cnt, 1)] = j;
        }
      }
      n_in = wave_sum(n_in);
      if (lane == 0) sh.red[wave] = n_in;
      __syncthreads();
      int need = quota;
#pragma unroll
      for (int w = 0; w < kRetWaves; ++w) need -= sh.red[w];
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
        if (beaten < need) set_bit(sh.R, (uint32_t)ju);
      }
      __syncthreads();
      if (tid == 0) sh.next = i + 1;
      __syncthreads();
    }
  }

  // emit the retained indices in ascending order
  const int per = (words + kRetThreads - 1) / kRetThreads;
  const int w0 = tid * per;
  int mine = 0;
  for (int t = w0; t < w0 + per && t < words; ++t) mine += __popc(sh.R[t]);
  int off = wave_excl_scan(mine, lane);
  const int wtotal = __shfl(off + mine, 63, kWave);
  if (lane == 0) sh.red[wave] = wtotal;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kRetWaves; ++w) off += w < wave ? sh.red[w] : 0;
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

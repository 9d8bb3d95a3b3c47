// Retained set of Eq. (9)-(10), one workgroup of 16 waves per sample.
//
// R starts as the pivots.  Stage i (pivot order) walks pivot i's ascending score
// list, skips tokens already in R and takes the first quota_i others: the threshold of
// Eq. (9) is set per pivot by the reduction ratio, i.e. by that quota.
//
// The scores are fp32 with absolute error <= tau, so a stage's outcome is certain
// only when the last score taken and the first one refused differ by more than
// 2*tau.  Decisions closer than that are settled in fp64 from the hidden-state
// rows, on (fp64 score, index).  The stages depend on each other, so the walk is
// a serial chain of LDS round trips; to keep it short the kernel speculates:
//   1. the stage lists are staged in LDS (in groups that fit);
//   2. the block walks the stages in fp32 order, 1024 list entries per step (one per
//      thread; ranks by ballot + a prefix over the 16 wave counts), committing what
//      that order says and noting each stage's last key taken and first key refused;
//   3. the waves then look at the stages in parallel: a stage whose two keys are
//      within 2*tau is uncertain, and its candidates within 2*tau of the boundary
//      are queued (who was a candidate is known from the per-token owner stage);
//   4. the waves re-score the queued (pivot, token) pairs in fp64, in parallel;
//   5. every uncertain stage is checked: if the fp64 order picks the same tokens
//      the speculation stands; at the first stage where it does not, that stage is
//      corrected, the later stages are undone and walked again.
// A boundary band that does not fit the queue or runs past the stored list (only
// with massive ties) is resolved by a block-wide sweep of the whole score row.
#pragma once
#include "common.hpp"

namespace dart {

constexpr int kRetThreads = 1024;  // 16 waves for staging, the band phase and the fp64 re-scoring
constexpr int kRetWaves = kRetThreads / kWave;
constexpr int kRetWords = kMaxN / 32;
// List entries staged in LDS at a time.  Two layouts of the same LDS region: whole 8-byte
// entries (one LDS read each) when the lists of the batch's largest sample fit kRetList of
// them, else a 32-bit score image and a 16-bit token index per entry (6 bytes, two LDS reads:
// measured 0.5 us slower on a 2880-token sample), so that the 32 lists of a 9216-token video
// sample (17424 entries) or the 16 lists of a 16384-token sample at one ninth (15.6 K) are
// still staged in one go instead of two (measured: -3 and -5 us).
constexpr int kRetList = 12288;
constexpr int kRetListPacked = 18432;
constexpr int kRetQ = 1024;      // band candidates awaiting an fp64 score
constexpr int kRetInFlight = 4;  // 16-byte pieces per row and lane in flight in the fp64 re-scoring
constexpr unsigned char kOwnNone = 0xff, kOwnPivot = 0xfe;
constexpr unsigned long long kNoKey = ~0ull;  // no list entry looks like this (index < 2^14)

struct RetainShared {
  union {
    unsigned long long list[kRetList];
    struct {
      uint32_t lkey[kRetListPacked];        // score images of the staged entries
      unsigned short lidx[kRetListPacked];  // their token indices (< kMaxN = 2^14)
    } pk;
  };
  uint32_t R[kRetWords];
  unsigned char owner[kMaxN];  // stage that took the token (kOwnPivot, kOwnNone)
  double q_s64[kRetQ];
  int q_idx[kRetQ];
  unsigned char q_stage[kRetQ];
  unsigned char q_taken[kRetQ];
  int st_off[kMaxP];  // offset of the stage's list inside the sample's list region
  int st_len[kMaxP];
  // per stage: [0] last key taken, [1] first key refused (kNoKey: the walk met none)
  unsigned long long st_kab[kMaxP][2];
  int st_qlo[kMaxP], st_qhi[kMaxP];
  unsigned char st_unc[kMaxP];
  int wcnt[kRetWaves];
  int qn, cnt, bad_first, fb_first, walk_taken;
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

// The retained set of sample b by one workgroup of kRetThreads threads.
// lists: per sample at P*row0, stage lists back to back (see k_order_scores).
// S: pivot-major scores.  X may be nullptr: then scores are taken as exact.
// pl2 [B*Ppad] (optional): fp64 squared norms of the pivots' rows, if this call computed them
// (the fp64 re-scoring then skips those products).
// keep: packed, ascending per sample.  cu_keep_out (optional) [B+1].
// scr_f64 [2*total_N] doubles: per-sample scratch at row0 (fallback sweep only).
// COH: S, lists and piv were written, and keep will be read, by other workgroups of this
// launch.  PACKED: the 6-byte layout of the staged lists (see kRetList).
template <int DT, bool COH, bool PACKED = false>
__device__ __forceinline__ void retain_body(
    const Geo& g, int b, const float* S, const unsigned long long* lists, const int* piv,
    const void* X, int* keep, int* cu_keep_out, double* scr_f64, float two_tau,
    RetainShared& sh, const double* pl2 = nullptr) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const unsigned long long lt_mask = (1ull << lane) - 1ull;
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
      X ? static_cast<const unsigned char*>(X) + (long)sm.xrow * rowbytes : nullptr;
  const unsigned long long* glist = lists + (long)P * sm.row0;
  double* sweep_s64 = scr_f64 + sm.row0;                                   // fallback sweep
  int* sweep_idx = reinterpret_cast<int*>(scr_f64 + g.total_N + sm.row0);  // fallback sweep

  const Split sp(k, P, g.Pin);
  constexpr int kCap = PACKED ? kRetListPacked : kRetList;  // staged entries at a time
  // staged entry o in the form of the global lists (score image << 32 | index)
  auto staged_entry = [&](int o) -> unsigned long long {
    if (PACKED) return ((unsigned long long)sh.pk.lkey[o] << 32) | sh.pk.lidx[o];
    return sh.list[o];
  };
  // stage constants in the lanes of every wave: lane i holds stage i's quota, list
  // length and list offset (the offsets are the prefix sums of the lengths)
  int quota_v = 0, len_v = 0;
  if (lane < P) {
    quota_v = sp.quota(lane);
    len_v = sp.stage_len(n, lane);
  }
  const int off_v = wave_excl_scan(len_v, lane);
  // Lists of the stages [first, group_hi) that fit in LDS together (the first one maybe
  // only in part); block-uniform arithmetic on the lane constants, no memory access.
  int group_hi = 0, group_base = 0, staged_total = 0;
  auto plan_group = [&](int first_any) {
    // (lane broadcasts by shuffle + readfirstlane: a readlane with a computed lane index did
    // not always compile here)
    const int first = __builtin_amdgcn_readfirstlane(first_any);  // block-uniform: keep it scalar
    group_base = __builtin_amdgcn_readfirstlane(__shfl(off_v, first, kWave));
    const int l0 = __builtin_amdgcn_readfirstlane(__shfl(len_v, first, kWave));
    const int l0c = l0 < kCap ? l0 : kCap;
    // a later stage s joins the group while everything up to the end of its list fits; the
    // list ends grow with s, so the stages that fit are the lanes first+1 .. group_hi-1
    const int rel_end = off_v + len_v - group_base - l0 + l0c;  // staged entries through stage `lane`
    const bool fits = lane > first && lane < P && rel_end <= kCap;
    const int extra = __builtin_amdgcn_readfirstlane(__popcll(__ballot(fits)));
    group_hi = first + 1 + extra;
    const int through = __builtin_amdgcn_readfirstlane(__shfl(rel_end, first + extra, kWave));
    staged_total = extra > 0 ? through : l0c;
  };
  // a group moves in two halves of kStageLoads loads per thread (48 or 72 KiB in flight each)
  constexpr int kStageLoads = kCap / kRetThreads / 2;
  unsigned long long staged[kStageLoads];
  auto load_half = [&](int h) {
#pragma unroll
    for (int u = 0; u < kStageLoads; ++u) {
      const int t = (h * kStageLoads + u) * kRetThreads + tid;
      staged[u] = t < staged_total ? ld_dev<COH>(&glist[group_base + t]) : 0ull;
    }
  };
  auto store_half = [&](int h) {
#pragma unroll
    for (int u = 0; u < kStageLoads; ++u) {
      const int t = (h * kStageLoads + u) * kRetThreads + tid;
      if (t < staged_total) {
        if (PACKED) {
          sh.pk.lkey[t] = (uint32_t)(staged[u] >> 32);
          sh.pk.lidx[t] = (unsigned short)staged[u];
        } else {
          sh.list[t] = staged[u];
        }
      }
    }
  };

  // the first group's lists and the pivots are requested before LDS is cleared, so
  // the kernel waits for global memory once
  plan_group(0);
  load_half(0);
  int my_pivot = -1;
  if (tid < g.Pin) my_pivot = ld_dev<COH>(&piv[b * P + tid]);  // pivots from outside hold no slot
  for (int t = tid; t < words; t += kRetThreads) sh.R[t] = 0u;
  for (int t = tid; t < (n + 3) / 4; t += kRetThreads)
    reinterpret_cast<uint32_t*>(sh.owner)[t] = 0xffffffffu;
  if (tid < P) {  // wave 0: its lanes hold the stage constants
    sh.st_len[tid] = len_v;
    sh.st_off[tid] = off_v;
  }
  store_half(0);
  if (staged_total > kStageLoads * kRetThreads) {
    load_half(1);
    store_half(1);
  }
  __syncthreads();
  if (my_pivot >= 0 && my_pivot < n) {
    set_bit(sh.R, (uint32_t)my_pivot);
    sh.owner[my_pivot] = kOwnPivot;
  }

  int next = 0;  // first stage not yet final (block-uniform)
  while (next < P) {
    if (next >= group_hi) {
      plan_group(next);
      load_half(0);
      __syncthreads();  // nobody reads the old group any more
      store_half(0);
      if (staged_total > kStageLoads * kRetThreads) {
        load_half(1);
        store_half(1);
      }
    }
    if (tid == 0) {
      sh.qn = 0;
      sh.bad_first = group_hi;
      sh.fb_first = group_hi;
    }
    if (tid >= next && tid < group_hi) sh.st_kab[tid][1] = kNoKey;
    __syncthreads();
    const int walk_end = group_hi;
    // The global pointer carries its address space: with a generic one the compiler may fold
    // the two returns into one flat load from a selected pointer (and its LDS-to-flat cast
    // did not compile in every context).
    typedef const unsigned long long __attribute__((address_space(1)))* GlobalList;
    const GlobalList glist_g = (GlobalList)glist;
    auto entry_of = [&](int i, int p) -> unsigned long long {
      const int o = sh.st_off[i] - group_base + p;  // position among the staged entries
      if (o < staged_total) return staged_entry(o);
      if (COH) return ld_dev<true>(&glist[sh.st_off[i] + p]);
      return glist_g[sh.st_off[i] + p];
    };

    // ------------------------------------------------------------------ speculative walk
    // All 16 waves walk together, 1024 list entries per step (one per thread): one step per
    // stage unless a list is longer.  On the critical path of a step: read R, ballot,
    // exchange the 16 wave counts (barrier), commit, barrier.  The step is bound by the
    // number of instructions a wave issues, so the one-step case is kept free of loops and
    // of everything the general case needs; the next stage's entries are read ahead.
    {
      // entries [0, 1024) of a stage's list (threads past its end read the group's entry 0)
      auto first_entries = [&](int st) -> unsigned long long {
        const int len = __builtin_amdgcn_readlane(len_v, st);
        const int off = __builtin_amdgcn_readlane(off_v, st) - group_base;
        int idx = tid < len ? off + tid : 0;
        idx = idx < kCap ? idx : 0;
        return staged_entry(idx);
      };
      const int wv = __builtin_amdgcn_readfirstlane(wave);
      unsigned long long e_pre = first_entries(next);
      for (int i = next; i < walk_end; ++i) {
        const int quota = __builtin_amdgcn_readlane(quota_v, i);
        const int len = __builtin_amdgcn_readlane(len_v, i);
        const int off = __builtin_amdgcn_readlane(off_v, i) - group_base;
        const unsigned long long e0 = e_pre;
        const int inext = i + 1 < walk_end ? i + 1 : i;
        if (quota == 0) {
          e_pre = first_entries(inext);
          continue;
        }
        const bool staged_all = off + len <= staged_total;  // the usual case: plain LDS reads
        if (staged_all && len <= kRetThreads) {
          // The whole list in one step, straight-line: the prefetched entries are the
          // list.  Waves past the list's end only write a zero count and keep the barriers.
          const uint32_t j = (uint32_t)e0;
          const bool busy = wv * kWave < len;  // wave-uniform
          unsigned long long bal = 0ull;
          bool cand = false;
          if (busy) {
            const uint32_t rw = sh.R[j >> 5];
            cand = tid < len && ((rw >> (j & 31)) & 1u) == 0u;
            bal = __ballot(cand);
          }
          if (lane == 0) sh.wcnt[wv] = __popcll(bal);
          __syncthreads();
          // the next stage's entries (they do not depend on this stage's commits) travel
          // together with the wave counts
          if (wv * kWave < __builtin_amdgcn_readlane(len_v, inext)) e_pre = first_entries(inext);
          if (busy) {
            // inclusive prefix of the 16 wave counts in lanes 0..15
            int x = lane < kRetWaves ? sh.wcnt[lane] : 0;
            x += dpp_move<kDppShr1>(0, x);
            x += dpp_move<kDppShr2>(0, x);
            x += dpp_move<kDppShr4>(0, x);
            x += dpp_move<kDppShr8>(0, x);
            const int before = wv > 0 ? __builtin_amdgcn_readlane(x, wv > 0 ? wv - 1 : 0) : 0;
            const int rank = before + __popcll(bal & lt_mask);
            if (cand) {
              if (rank < quota) {
                set_bit(sh.R, j);
                sh.owner[j] = (unsigned char)i;
              }
              const uint32_t rel = (uint32_t)(rank - (quota - 1));  // 0: last taken, 1: first refused
              if (rel < 2u) sh.st_kab[i][rel] = e0;
            }
          }
          __syncthreads();  // the commits are visible before anyone tests R again
          continue;
        }
        e_pre = first_entries(inext);
        bool have_b = false;
        int taken = 0;
        for (int pos = 0; pos < len && !have_b; pos += kRetThreads) {
          if (pos + wv * kWave >= len) {
            // this wave's 64 entries are past the list's end: it only keeps the barriers
            if (lane == 0) sh.wcnt[wv] = 0;
            __syncthreads();
            __syncthreads();
            taken = sh.walk_taken;
            have_b = taken > quota;
            continue;
          }
          const int t = pos + tid;
          const bool in = t < len;
          unsigned long long e;
          if (staged_all) e = staged_entry(in ? off + t : 0);
          else e = in ? entry_of(i, t) : staged_entry(0);  // a list longer than the LDS region
          const uint32_t j = (uint32_t)e;
          const uint32_t rw = sh.R[j >> 5];
          const bool cand = in && ((rw >> (j & 31)) & 1u) == 0u;
          const unsigned long long bal = __ballot(cand);
          if (lane == 0) sh.wcnt[wv] = __popcll(bal);
          __syncthreads();
          int x = lane < kRetWaves ? sh.wcnt[lane] : 0;
          x += dpp_move<kDppShr1>(0, x);
          x += dpp_move<kDppShr2>(0, x);
          x += dpp_move<kDppShr4>(0, x);
          x += dpp_move<kDppShr8>(0, x);
          const int total = __builtin_amdgcn_readlane(x, kRetWaves - 1);
          const int before = wv > 0 ? __builtin_amdgcn_readlane(x, wv > 0 ? wv - 1 : 0) : 0;
          const int rank = taken + before + __popcll(bal & lt_mask);
          if (cand) {
            if (rank < quota) {
              set_bit(sh.R, j);
              sh.owner[j] = (unsigned char)i;
            }
            const uint32_t rel = (uint32_t)(rank - (quota - 1));
            if (rel < 2u) sh.st_kab[i][rel] = e;
          }
          taken += total;
          have_b = taken > quota;
          if (tid == 0) sh.walk_taken = taken;  // for the waves that sat this step out
          __syncthreads();  // the commits are visible before anyone tests R again
        }
      }
    }
    __syncthreads();

    // ------------------------------------------------------------------ uncertain stages
    // wave w looks at stages next+w, next+w+16, ...; R and owner are only read here
    for (int i = next + wave; i < walk_end; i += kRetWaves) {
      bool unc = false;
      uint32_t lo_m = 0, hi_m = 0;
      if (Xb && sp.quota(i) > 0 && sh.st_kab[i][1] != kNoKey) {
        const float fa = mono_inv((uint32_t)(sh.st_kab[i][0] >> 32));
        const float fb = mono_inv((uint32_t)(sh.st_kab[i][1] >> 32));
        unc = !((fb - fa) > two_tau);
        lo_m = mono_of((fa - two_tau) + 0.0f);
        hi_m = mono_of((fb + two_tau) + 0.0f);
      }
      if (lane == 0) sh.st_unc[i] = unc ? 1 : 0;
      if (!unc) continue;
      const int len = sh.st_len[i];
      // first list position whose key reaches the band (64-ary search on the sorted keys)
      int lo_pos = 0, span = len;
      while (span > kWave) {
        const int stride = (span + kWave - 1) / kWave;
        const int p = lo_pos + lane * stride;
        const bool below = p < len && p < lo_pos + span &&
                           (uint32_t)(entry_of(i, p) >> 32) < lo_m;
        const int m = __popcll(__ballot(below));
        if (m > 0) lo_pos += (m - 1) * stride;
        span = stride;
      }
      // candidates of stage i = tokens no earlier stage owned
      auto scan = [&](int qbase) -> int {
        int cnt = 0;
        bool closed = false;
        for (int p0 = lo_pos; p0 < len && !closed; p0 += kWave) {
          const int p = p0 + lane;
          const unsigned long long e = p < len ? entry_of(i, p) : 0ull;
          const uint32_t key = (uint32_t)(e >> 32), idx = (uint32_t)e;
          const unsigned char own = p < len ? sh.owner[idx] : kOwnPivot;
          const bool band = p < len && key >= lo_m && key <= hi_m &&
                            (own == kOwnNone || (own < kOwnPivot && (int)own >= i));
          const unsigned long long mb = __ballot(band);
          if (qbase >= 0 && band) {
            const int slot = qbase + cnt + __popcll(mb & lt_mask);
            sh.q_idx[slot] = (int)idx;
            sh.q_stage[slot] = (unsigned char)i;
            sh.q_taken[slot] = own == (unsigned char)i ? 1 : 0;
          }
          cnt += __popcll(mb);
          closed = __ballot(p < len && key > hi_m) != 0ull;
        }
        return closed ? cnt : -1 - cnt;  // negative: the band reached the end of the list
      };
      int cnt = scan(-1);
      const bool open = cnt < 0 && len < n;  // the band may run past the stored list
      cnt = cnt < 0 ? -1 - cnt : cnt;
      // reserve cnt queue slots, only if they fit (so every reserved slot gets written)
      int qlo = kRetQ + 1;
      if (lane == 0 && !open) {
        int old = sh.qn;
        while (old + cnt <= kRetQ) {
          const int seen = atomicCAS(&sh.qn, old, old + cnt);
          if (seen == old) {
            qlo = old;
            break;
          }
          old = seen;
        }
      }
      qlo = __builtin_amdgcn_readfirstlane(qlo);
      if (qlo + cnt > kRetQ) {
        // too many ties for the queue (or an open band): leave it to the block-wide sweep
        if (lane == 0) atomicMin(&sh.fb_first, i);
        continue;
      }
      scan(qlo);
      if (lane == 0) {
        sh.st_qlo[i] = qlo;
        sh.st_qhi[i] = qlo + cnt;
      }
    }
    __syncthreads();

    // ------------------------------------------------------------------ fp64 scores of the queue
    // block-uniform values read from LDS are made scalar explicitly: they end up as lane
    // indices of readlane, which must be scalar registers
    const int fb_first = __builtin_amdgcn_readfirstlane(sh.fb_first);
    const int qn = __builtin_amdgcn_readfirstlane(sh.qn);
    for (int q = wave; q < qn; q += kRetWaves) {  // a pair per wave: 16 row pairs in flight
      const int st = sh.q_stage[q];
      if (st >= fb_first) continue;  // will be walked again anyway
      const unsigned char* prow = pivot_row<COH>(g, X, esz, sm, b, st, piv);
      const unsigned char* xrow = Xb + (long)sh.q_idx[q] * rowbytes;
      const double s0 =
          pl2 ? row_cosine_f64<DT, true, kRetInFlight>(prow, xrow, g.D, lane, ld_dev<COH>(&pl2[b * g.Ppad + st]))
              : row_cosine_f64<DT, false, kRetInFlight>(prow, xrow, g.D, lane);
      if (lane == 0) sh.q_s64[q] = s0;
    }
    __syncthreads();

    // ------------------------------------------------------------------ check the speculation
    // the fp64 order agrees with the fp32 order iff the largest pair taken is below
    // the smallest pair refused
    for (int i = next + wave; i < walk_end && i < fb_first; i += kRetWaves) {
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
#define DART_PAIR_STEP(J)                                                                      \
  {                                                                                            \
    const double s1 = lane_xor<J>(mt_s, lane), s2 = lane_xor<J>(mu_s, lane);                   \
    const int j1 = lane_xor<J>(mt_j, lane), j2 = lane_xor<J>(mu_j, lane);                      \
    if (pair_less(mt_s, mt_j, s1, j1)) { mt_s = s1; mt_j = j1; }                               \
    if (pair_less(s2, j2, mu_s, mu_j)) { mu_s = s2; mu_j = j2; }                               \
  }
      DART_PAIR_STEP(32) DART_PAIR_STEP(16) DART_PAIR_STEP(8) DART_PAIR_STEP(4) DART_PAIR_STEP(2)
      DART_PAIR_STEP(1)
#undef DART_PAIR_STEP
      if (!pair_less(mt_s, mt_j, mu_s, mu_j) && lane == 0) atomicMin(&sh.bad_first, i);
    }
    __syncthreads();
    const int bad = __builtin_amdgcn_readfirstlane(sh.bad_first);
    if (bad >= walk_end && fb_first >= walk_end) {
      next = walk_end;  // everything stands
      continue;
    }
    if (bad < fb_first) {
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

    // ------------------------------------------------------------------ block-wide fallback
    {
      // stage i and everything after it is taken back; stage i is decided on the
      // whole score row, then the walk goes on from i+1
      const int i = fb_first;
      for (int j = tid; j < n; j += kRetThreads) {
        const unsigned char o = sh.owner[j];
        if (o < kOwnPivot && (int)o >= i) {
          clear_bit(sh.R, (uint32_t)j);
          sh.owner[j] = kOwnNone;
        }
      }
      const int quota = sp.quota(i);
      const float lo = mono_inv((uint32_t)(sh.st_kab[i][0] >> 32)) - two_tau;
      const float hi = mono_inv((uint32_t)(sh.st_kab[i][1] >> 32)) + two_tau;
      const float* Srow = S + (long)P * sm.row0 + (long)i * n;
      if (tid == 0) sh.cnt = 0;
      __syncthreads();
      int n_in = 0;
      for (int j = tid; j < n; j += kRetThreads) {
        if (bit_of(sh.R, (uint32_t)j)) continue;
        const float s = ld_dev<COH>(&Srow[j]) + 0.0f;
        if (s < lo) {  // below the band: certainly among the quota lowest
          set_bit(sh.R, (uint32_t)j);
          sh.owner[j] = (unsigned char)i;
          ++n_in;
        } else if (s <= hi) {
          sweep_idx[atomicAdd(&sh.cnt, 1)] = j;
        }
      }
      n_in = wave_sum(n_in);
      if (lane == 0) sh.wcnt[wave] = n_in;
      __syncthreads();
      int need = quota;
#pragma unroll
      for (int w = 0; w < kRetWaves; ++w) need -= sh.wcnt[w];
      const int nU = sh.cnt;
      const unsigned char* prow = pivot_row<COH>(g, X, esz, sm, b, i, piv);
      const double pp_i = pl2 ? ld_dev<COH>(&pl2[b * g.Ppad + i]) : 0.0;
      for (int u = wave; u < nU; u += kRetWaves) {
        const unsigned char* xrow = Xb + (long)sweep_idx[u] * rowbytes;
        const double s64 = pl2 ? row_cosine_f64<DT, true, kRetInFlight>(prow, xrow, g.D, lane, pp_i)
                               : row_cosine_f64<DT, false, kRetInFlight>(prow, xrow, g.D, lane);
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
  const int wtotal = __builtin_amdgcn_readlane(off + mine, 63);
  if (lane == 0) sh.wcnt[wave] = wtotal;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kRetWaves; ++w) off += w < wave ? sh.wcnt[w] : 0;
  int* out = keep + sm.keep0 + off;
  for (int t = w0; t < w0 + per && t < words; ++t) {
    uint32_t m = sh.R[t];
    while (m) {
      int bit = __ffs(m) - 1;
      st_dev<COH>(out++, t * 32 + bit);
      m &= m - 1;
    }
  }
}

// grid: B blocks of kRetThreads: block b builds the retained set of sample b.
template <int DT, bool PACKED>
__global__ __launch_bounds__(kRetThreads) void k_retain(
    Geo g, const float* __restrict__ S, const unsigned long long* __restrict__ lists,
    const int* __restrict__ piv, const void* __restrict__ X, int* __restrict__ keep,
    int* __restrict__ cu_keep_out, double* __restrict__ scr_f64, float two_tau,
    const double* __restrict__ pl2) {
  __shared__ RetainShared sh;
  retain_body<DT, false, PACKED>(g, blockIdx.x, S, lists, piv, X, keep, cu_keep_out, scr_f64,
                                 two_tau, sh, pl2);
}

}  // namespace dart

// The whole step of Section 3.3 in one launch: row norms, pivot selection (Definition 1),
// duplication scores (Definition 2 / Eq. 7), score ordering and the retained set (Eq. 9-10),
// compaction (Appendix D).
//
// The steps depend on each other sample by sample, not batch by batch: the scores of sample b
// need only the pivots of sample b.  Launched as separate kernels every dependent step waits
// for the slowest sample of the step before it, and the on-chip steps (selection, ordering,
// retained set: a handful of workgroups each) leave the other compute units idle.  Here one
// persistent workgroup of 1024 threads per compute unit takes work items from two sources:
//   * the streaming queue: norm items, then score items, then gather items, sample after
//     sample, handed out in that order by one ticket counter.  An item whose sample is not
//     ready yet (scores need the sample's pivots, the gather needs its retained set) is held
//     by its workgroup until it is;
//   * the chain batches: a sample's pivot selection (1 item), its ordering (P items) and its
//     retained set (1 item), each pushed as a batch by whoever completes the last item it
//     depends on (the last norm item pushes the selection, the last score item the ordering,
//     the last ordering item the retained set).  A batch carries its own claim counter: a
//     workgroup that is between two items, or holds an item that is not ready, adds one to the
//     counter of the oldest batch it has not found exhausted and owns the item of that index if
//     the index is below the batch's size (a larger index means "nothing left here": claims
//     never fail and never consume anything that is not there yet).
// So the on-chip work of one sample runs beside the streaming work of the others, and nothing
// waits for a whole batch.  Every wait is on work that a running workgroup has already taken,
// so it ends; it is also bounded (spin limit): a workgroup that exceeds the limit raises the
// abort flag, everyone leaves at the next scheduling point and dart_device_status reports it.
//
// What one workgroup hands to another goes through device-scope loads and stores (see
// ld_dev / st_dev); a completion is published as: every thread waits for its own stores,
// workgroup barrier, one thread bumps the counter or pushes the batch.
//
// The kernel's parameters live in LDS, and every step makes its own scalar copies of the few
// it uses: held in scalar registers for the whole kernel they (some 70 of the 102 there are)
// drove the register allocator to hundreds of spills.
#pragma once
#include "common.hpp"
#include "k_norms.hpp"
#include "k_order.hpp"
#include "k_pivots.hpp"
#include "k_retain.hpp"
#include "k_scores.hpp"

namespace dart {

constexpr int kFuThreads = 1024, kFuWaves = kFuThreads / kWave;
// Rows per norm / gather item, 4 per wave.  Every item pays a fixed price of several device-
// scope round trips of 1-2 us each (claim, completion count, write-through of its results):
// with 16-row items that price was most of an item (11 us for 128 KB, the norm phase of the
// B=8 N=2880 batch 98 us instead of 52), so the items stay this large.
constexpr int kFuNormRows = 64;
constexpr int kFuGatherRows = 64;
constexpr int kFuMaxB = 4096;      // samples per call the one-launch path accepts
constexpr int kFuAborted = 0x0DA27ABE;  // status word: a bounded wait ran out
constexpr int kFuTabB = 256;       // batches of up to this many samples keep the item tables in LDS

// Sync area (ints, zeroed by k_fused_init before every launch): a header, then five
// per-sample words, then the chain batches (two ints each: code, claims).
enum {
  kSyTicket = 0,  // next streaming item
  kSyTail = 2,    // chain batches pushed            } one aligned 8-byte word, polled together
  kSyDone = 3,    // samples whose retained set is complete; kFuAbortBit: a bounded wait ran out }
  kSyTotalN = 4,  // norm / score / gather items of the call (set by k_fused_init)
  kSyTotalS,
  kSyTotalG,
  kSyLive,        // samples that take part (a rejected or empty ragged sample does not)
  kSyHeader = 16
};
constexpr int kFuAbortBit = 1 << 30;
__host__ __device__ inline long fused_sync_ints(int B, int P) {
  (void)P;
  return kSyHeader + 5L * B + 2L * 3 * B;
}
enum { kWkExit = 0, kWkNorm, kWkScore, kWkGather, kWkSelect, kWkOrder, kWkRetain };

struct FusedArgs {
  const void* X;
  const long long* pos;
  void* Y;  // nullptr: no compaction
  long long* pos_out;
  int* keep;
  int* piv;
  float* S;
  float* l1;
  double* l2sq;
  double* pl2;
  unsigned long long* lists;
  double* scr;
  int* sync;
  const int* norm_start;    // [B+1] first norm item of every sample (k_fused_init)
  const int* score_start;   // [B+1] first score item
  const int* gather_start;  // [B+1] first gather item
  int* status;
  float tau_l1, two_tau;
  int keep_cached;  // the norm items use ordinary loads (the rows stay in the memory-side cache)
  int spin_limit;   // polls of a bounded wait
};

// Rows per score item: the 16 waves of the workgroup split into KS groups that share the
// same 256/KS token rows and each take a contiguous 1/KS of the D-chunks.
template <int NB>
struct FusedScoreCfg {
  static constexpr int KS = NB <= 2 ? 4 : 2;
  static constexpr int ROWS = 256 / KS;
};

// One workgroup, 1024 threads.  Fills the per-sample item tables, the totals and the packed
// offsets a caller may ask for, and zeroes the sync area.  Ragged batches: after k_prepare.
__global__ __launch_bounds__(1024) void k_fused_init(Geo g, int score_rows, int have_y,
                                                     int* __restrict__ sync,
                                                     int* __restrict__ norm_start,
                                                     int* __restrict__ score_start,
                                                     int* __restrict__ gather_start,
                                                     int* __restrict__ cu_keep_out,
                                                     int* __restrict__ status) {
  __shared__ int red[4][16];
  __shared__ int carry[4];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const long ints = fused_sync_ints(g.B, g.P);
  for (long t = tid; t < ints; t += 1024) sync[t] = 0;
  if (tid < 4) carry[tid] = 0;
  __syncthreads();
  for (int b0 = 0; b0 < g.B; b0 += 1024) {
    const int b = b0 + tid;
    int v[4] = {0, 0, 0, 0};
    Sample sm;
    sm.k = 0;
    sm.keep0 = 0;
    if (b < g.B) {
      sm = sample_of(g, b);
      if (sm.k > 0) {
        v[0] = (sm.n + kFuNormRows - 1) / kFuNormRows;
        v[1] = (sm.n + score_rows - 1) / score_rows;
        v[2] = have_y ? (sm.k + kFuGatherRows - 1) / kFuGatherRows : 0;
        v[3] = 1;
      }
    }
    int sc[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      sc[q] = wave_excl_scan(v[q], lane);
      if (lane == 63) red[q][w] = sc[q] + v[q];
    }
    __syncthreads();
    int base[4], tot[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      base[q] = carry[q];
      tot[q] = 0;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        base[q] += i < w ? red[q][i] : 0;
        tot[q] += red[q][i];
      }
    }
    if (b < g.B) {
      norm_start[b] = base[0] + sc[0];
      score_start[b] = base[1] + sc[1];
      gather_start[b] = base[2] + sc[2];
      if (cu_keep_out) cu_keep_out[b] = sm.keep0;
      if (cu_keep_out && b == g.B - 1) cu_keep_out[g.B] = sm.keep0 + sm.k;
    }
    __syncthreads();
    if (tid < 4) carry[tid] += tot[tid];
    __syncthreads();
  }
  if (tid == 0) {
    norm_start[g.B] = carry[0];
    score_start[g.B] = carry[1];
    gather_start[g.B] = carry[2];
    sync[kSyTotalN] = carry[0];
    sync[kSyTotalS] = carry[1];
    sync[kSyTotalG] = carry[2];
    sync[kSyLive] = carry[3];
    status[3] = 0;
  }
}

// Largest b with start[b] <= t (start is non-decreasing, start[0] = 0 <= t < start[B]).
__device__ __forceinline__ int fused_sample_of_item(const int* start, int B, int t) {
  int lo = 0, hi = B;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (start[mid] <= t) lo = mid; else hi = mid;
  }
  return lo;
}

// A scalar-register copy of a parameter block that lives in LDS (only the fields a step uses
// are actually read).
template <typename T>
__device__ __forceinline__ T lds_uniform(const T& src) {
  static_assert(sizeof(T) % 4 == 0, "whole dwords");
  T out;
  const int* s = reinterpret_cast<const int*>(&src);
  int* o = reinterpret_cast<int*>(&out);
#pragma unroll
  for (unsigned i = 0; i < sizeof(T) / 4; ++i) o[i] = __builtin_amdgcn_readfirstlane(s[i]);
  return out;
}

// ---- the items ---------------------------------------------------------------------------

// Norm item: L1 norm (fp32, the order of k_row_l1) and squared Euclidean norm (fp64 over fp32
// piece sums) of the token rows [r0, r0 + 64) of one sample; a wave takes 4 rows in turn.
__device__ __forceinline__ void fused_norm_item(const Geo& g, const Sample& sm, int r0,
                                                const FusedArgs& a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int pieces = g.D / 8;
  const long rowbytes = g.ld * 2;
  const unsigned char* Xb = static_cast<const unsigned char*>(a.X) + (long)sm.xrow * rowbytes;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  for (int q = 0; q < kFuNormRows / kFuWaves; ++q) {
    const int j = r0 + wave * (kFuNormRows / kFuWaves) + q;
    if (j >= sm.n) break;  // wave-uniform
    const u32x4* src = reinterpret_cast<const u32x4*>(Xb + (long)j * rowbytes);
    float acc = 0.f;
    double sq = 0.0;
    for (int t0 = 0; t0 < pieces; t0 += kWave * 8) {
      u32x4 v[8];
      if (a.keep_cached) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int t = t0 + u * kWave + lane;
          v[u] = t < pieces ? src[t] : zero;
        }
      } else {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int t = t0 + u * kWave + lane;
          v[u] = t < pieces ? __builtin_nontemporal_load(src + t) : zero;
        }
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        acc += piece_abs_sum<kBF16>(v[u]);
        sq += (double)piece_sq_sum_bf16(v[u]);
      }
    }
    const float s = wave_sum(acc);
    const double q2 = wave_sum(sq);
    if (lane == 0) {
      st_dev<true>(&a.l1[sm.row0 + j], s);
      st_dev<true>(&a.l2sq[sm.row0 + j], q2);
    }
  }
}

// Gather item: retained rows [r0, r0 + 64) of one sample (bit copies), a wave takes 4 in turn.
__device__ __forceinline__ void fused_gather_item(const Geo& g, const Sample& sm, int r0,
                                                  const FusedArgs& a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int pieces = g.D / 8;
  const long rowbytes = g.ld * 2;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  for (int q = 0; q < kFuGatherRows / kFuWaves; ++q) {
    const int r = r0 + wave * (kFuGatherRows / kFuWaves) + q;
    if (r >= sm.k) break;  // wave-uniform
    int kr = ld_dev<true>(&a.keep[sm.keep0 + r]);
    kr = kr < 0 ? 0 : (kr < sm.n ? kr : sm.n - 1);
    const long src = (long)sm.xrow + kr;
    const u32x4* in = reinterpret_cast<const u32x4*>(static_cast<const unsigned char*>(a.X) +
                                                     src * rowbytes);
    u32x4* out = reinterpret_cast<u32x4*>(static_cast<unsigned char*>(a.Y) +
                                          (long)(sm.keep0 + r) * g.D * 2);
    for (int t0 = 0; t0 < pieces; t0 += kWave * 8) {
      u32x4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int t = t0 + u * kWave + lane;
        v[u] = t < pieces ? __builtin_nontemporal_load(in + t) : zero;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int t = t0 + u * kWave + lane;
        if (t < pieces) out[t] = v[u];
      }
    }
    if (a.pos && lane == 0) a.pos_out[sm.keep0 + r] = a.pos[src];
  }
}

// ---- the scheduler -----------------------------------------------------------------------

// LDS of the persistent workgroup: one region that the steps use in turn, and the kernel's
// parameters.  (The largest score-item layout, NB = 4, is smaller than the selection's.)
union FusedShared {
  PivotShared<kFuThreads> piv;
  SelectShared<kFuThreads> sel;
  RetainShared ret;
  KSplitShared<1, FusedScoreCfg<1>::KS, kFuWaves> sc1;
  KSplitShared<2, FusedScoreCfg<2>::KS, kFuWaves> sc2;
  KSplitShared<3, FusedScoreCfg<3>::KS, kFuWaves> sc3;
  KSplitShared<4, FusedScoreCfg<4>::KS, kFuWaves> sc4;
};
struct FusedParams {
  Geo g;
  FusedArgs a;
};
__shared__ FusedShared fu_sh;
__shared__ FusedParams fu_prm;
// [0..2] the item to run (kind, sample, index); [3] in: take the next streaming ticket while
// running it; [4] out: that ticket (-1: none); [5..6] out: the poll word read while running it
__shared__ int fu_ctl[8];

template <int NB> __device__ __forceinline__ auto& fused_score_lds();
template <> __device__ __forceinline__ auto& fused_score_lds<1>() { return fu_sh.sc1; }
template <> __device__ __forceinline__ auto& fused_score_lds<2>() { return fu_sh.sc2; }
template <> __device__ __forceinline__ auto& fused_score_lds<3>() { return fu_sh.sc3; }
template <> __device__ __forceinline__ auto& fused_score_lds<4>() { return fu_sh.sc4; }

// One function per kind of item, each compiled on its own: inlined into the scheduler's loop
// the steps' loop-invariant values were hoisted out of it and kept alive across all of them
// (hundreds of register spills).  Each takes its parameters from LDS.
#define DART_FUSED_PARAMS(b_in, i_in)                           \
  const int b = __builtin_amdgcn_readfirstlane(b_in);           \
  const int idx = __builtin_amdgcn_readfirstlane(i_in);         \
  (void)idx;                                                    \
  const Geo g = lds_uniform(fu_prm.g);                          \
  const FusedArgs a = lds_uniform(fu_prm.a)

// While an item runs, its first thread already asks for the workgroup's next streaming ticket
// and reads the poll word (chain batches pushed, samples done): the answers arrive during the
// item instead of costing a memory round trip or two between items.
#define DART_FUSED_PREFETCH_BEGIN()                                                            \
  int pre_t = -1;                                                                              \
  unsigned long long pre_p = 0;                                                                \
  if (threadIdx.x == 0) {                                                                      \
    if (fu_ctl[3]) pre_t = atomicAdd(&a.sync[kSyTicket], 1);                                   \
    pre_p = ld_dev<true>(reinterpret_cast<const unsigned long long*>(&a.sync[kSyTail]));       \
  }
#define DART_FUSED_PREFETCH_END()                                                              \
  if (threadIdx.x == 0) {                                                                      \
    fu_ctl[4] = pre_t;                                                                         \
    fu_ctl[5] = (int)(uint32_t)pre_p;                                                          \
    fu_ctl[6] = (int)(uint32_t)(pre_p >> 32);                                                  \
  }

__device__ __attribute__((noinline)) void fused_do_norm(int b_in, int i_in) {
  DART_FUSED_PARAMS(b_in, i_in);
  DART_FUSED_PREFETCH_BEGIN();
  fused_norm_item(g, sample_of(g, b), idx * kFuNormRows, a);
  stores_done();
  DART_FUSED_PREFETCH_END();
}
__device__ __attribute__((noinline)) void fused_do_select(int b_in, int i_in) {
  DART_FUSED_PARAMS(b_in, i_in);
  DART_FUSED_PREFETCH_BEGIN();
  select_pivots_body<kBF16, kFuThreads, true>(g, b, a.X, a.X, g.D, g.ld, a.l1, a.piv, a.pl2, a.scr,
                                              a.tau_l1, fu_sh.piv);
  stores_done();
  DART_FUSED_PREFETCH_END();
}
template <int NB, bool TAIL>
__device__ __attribute__((noinline)) void fused_do_score(int b_in, int i_in) {
  DART_FUSED_PARAMS(b_in, i_in);
  DART_FUSED_PREFETCH_BEGIN();
  score_tile_ksplit<NB, FusedScoreCfg<NB>::KS, kFuWaves, TAIL, true, true>(
      g, sample_of(g, b), b, idx, a.X, a.piv, a.pl2, a.l2sq, a.S, fused_score_lds<NB>());
  stores_done();
  DART_FUSED_PREFETCH_END();
}
__device__ __attribute__((noinline)) void fused_do_order(int b_in, int i_in) {
  DART_FUSED_PARAMS(b_in, i_in);
  DART_FUSED_PREFETCH_BEGIN();
  order_scores_body<kFuThreads, true>(g, b, idx, a.S, a.lists, fu_sh.sel);
  stores_done();
  DART_FUSED_PREFETCH_END();
}
__device__ __attribute__((noinline)) void fused_do_retain(int b_in, int i_in) {
  DART_FUSED_PARAMS(b_in, i_in);
  DART_FUSED_PREFETCH_BEGIN();
  retain_body<kBF16, true, false>(g, b, a.S, a.lists, a.piv, a.X, a.keep, nullptr, a.scr,
                                  a.two_tau, fu_sh.ret, a.pl2);
  stores_done();
  DART_FUSED_PREFETCH_END();
}
__device__ __attribute__((noinline)) void fused_do_gather(int b_in, int i_in) {
  DART_FUSED_PARAMS(b_in, i_in);
  DART_FUSED_PREFETCH_BEGIN();
  fused_gather_item(g, sample_of(g, b), idx * kFuGatherRows, a);
  DART_FUSED_PREFETCH_END();
}
#undef DART_FUSED_PARAMS

#undef DART_FUSED_PREFETCH_BEGIN
#undef DART_FUSED_PREFETCH_END

// Pushes a chain batch: `count` items (kind, b, 0..count-1).  One thread.
__device__ __forceinline__ void fused_push(int* sy, int* batches, int kind, int b, int count) {
  const int j = atomicAdd(&sy[kSyTail], 1);
  st_dev<true>(&batches[2 * j], ((kind << 28) | (b << 8) | count) + 1);
}

// grid: one workgroup of 1024 threads per compute unit (any number works: workgroups that
// start late simply find less left to do).  bf16 hidden states, pivots chosen among the
// tokens by the norms of the hidden states themselves, the staged rule of Eq. (9)-(10).
template <int NB, bool TAIL>
__global__ __launch_bounds__(kFuThreads) void k_fused(Geo g_arg, FusedArgs a_arg) {
  __shared__ int tab[3][kFuTabB + 1];  // the item tables of small batches
  const int tid = threadIdx.x;
  if (tid == 0) {
    fu_prm.g = g_arg;
    fu_prm.a = a_arg;
  }
  const int B = g_arg.B, P = g_arg.P;
  int* const sy = a_arg.sync;
  const bool tabbed = B <= kFuTabB;
  if (tabbed) {
    for (int t = tid; t <= B; t += kFuThreads) {
      tab[0][t] = a_arg.norm_start[t];
      tab[1][t] = a_arg.score_start[t];
      tab[2][t] = a_arg.gather_start[t];
    }
  }
  const int* const nstart = tabbed ? tab[0] : a_arg.norm_start;
  const int* const sstart = tabbed ? tab[1] : a_arg.score_start;
  const int* const gstart = tabbed ? tab[2] : a_arg.gather_start;
  const int spin_limit = a_arg.spin_limit;
  int* const norm_done = sy + kSyHeader;
  int* const piv_ready = norm_done + B;
  int* const score_done = piv_ready + B;
  int* const order_done = score_done + B;
  int* const retain_done = order_done + B;
  int* const batches = retain_done + B;  // {code, claims} per batch
  // totals: written by k_fused_init, an earlier launch
  const int totN = sy[kSyTotalN], totS = sy[kSyTotalS], totG = sy[kSyTotalG], live = sy[kSyLive];
  const int totA = totN + totS + totG;

  // thread 0's scheduling state: the streaming item it holds (kind 0 = none), the oldest
  // chain batch it has not found exhausted, and what the last item read ahead
  int h_kind = 0, h_b = 0, h_idx = 0, cursor = 0;
  bool exhausted = totA == 0;
  bool have_pre = false;
  auto take_ticket = [&](int t) {
    if (t >= totA) {
      exhausted = true;
    } else if (t < totN) {
      h_kind = kWkNorm;
      h_b = fused_sample_of_item(nstart, B, t);
      h_idx = t - nstart[h_b];
    } else if (t < totN + totS) {
      h_kind = kWkScore;
      h_b = fused_sample_of_item(sstart, B, t - totN);
      h_idx = t - totN - sstart[h_b];
    } else {
      h_kind = kWkGather;
      h_b = fused_sample_of_item(gstart, B, t - totN - totS);
      h_idx = t - totN - totS - gstart[h_b];
    }
  };

  for (;;) {
    __syncthreads();  // the previous item is done with LDS and with fu_ctl
    if (tid == 0) {
      int kind = kWkExit, wb = 0, widx = 0;
      if (have_pre && fu_ctl[4] >= 0) take_ticket(fu_ctl[4]);
      for (int spins = 0;; ++spins) {
        // the poll word: the one the last item read ahead on the first round, fresh after that
        unsigned long long td;
        if (have_pre) {
          td = ((unsigned long long)(uint32_t)fu_ctl[6] << 32) | (uint32_t)fu_ctl[5];
          have_pre = false;
        } else {
          td = ld_dev<true>(reinterpret_cast<const unsigned long long*>(&sy[kSyTail]));
        }
        const int tail = (int)(uint32_t)td, done = (int)(uint32_t)(td >> 32);
        if ((done & kFuAbortBit) || spins >= spin_limit) {
          if (!(done & kFuAbortBit)) atomicOr(&sy[kSyDone], kFuAbortBit);
          break;
        }
        // chain items first: they are few, long, and other samples' progress hangs on them
        bool got = false;
        while (cursor < tail) {
          const unsigned long long cc =
              ld_dev<true>(reinterpret_cast<const unsigned long long*>(&batches[2 * cursor]));
          const int code = (int)(uint32_t)cc - 1, claims = (int)(uint32_t)(cc >> 32);
          if (code < 0) break;  // pushed, its code not yet visible: look again next round
          const int count = code & 0xff;
          if (claims < count) {
            const int i = atomicAdd(&batches[2 * cursor + 1], 1);
            if (i < count) {
              kind = code >> 28;
              wb = (code >> 8) & 0xfffff;
              widx = i;
              got = true;
              break;
            }
          }
          ++cursor;  // exhausted: never look at it again
        }
        if (got) break;
        if (h_kind == 0 && !exhausted) take_ticket(atomicAdd(&sy[kSyTicket], 1));
        if (h_kind != 0) {
          const bool ready = h_kind == kWkNorm ||
                             (h_kind == kWkScore ? ld_dev<true>(&piv_ready[h_b]) != 0
                                                 : ld_dev<true>(&retain_done[h_b]) != 0);
          if (ready) {
            kind = h_kind;
            wb = h_b;
            widx = h_idx;
            h_kind = 0;
            break;
          }
        } else if (done >= live) {
          break;  // no streaming item left for this workgroup and no chain item can appear
        }
        // idle: back off (0.4 us at first, 3 us after a few rounds)
        if (spins < 4) __builtin_amdgcn_s_sleep(16);
        else if (spins < 16) __builtin_amdgcn_s_sleep(48);
        else __builtin_amdgcn_s_sleep(127);
      }
      fu_ctl[0] = kind;
      fu_ctl[1] = wb;
      fu_ctl[2] = widx;
      // a streaming item frees the ticket slot: let it fetch the next ticket while it runs
      fu_ctl[3] = (h_kind == 0 && !exhausted) ? 1 : 0;
      have_pre = kind != kWkExit;
    }
    __syncthreads();
    const int kind = fu_ctl[0], b = fu_ctl[1], idx = fu_ctl[2];
    if (kind == kWkExit) break;
    if (kind == kWkNorm) {
      fused_do_norm(b, idx);
      __syncthreads();
      if (tid == 0 && atomicAdd(&norm_done[b], 1) + 1 == nstart[b + 1] - nstart[b])
        fused_push(sy, batches, kWkSelect, b, 1);
    } else if (kind == kWkSelect) {
      fused_do_select(b, idx);
      __syncthreads();
      if (tid == 0) st_dev<true>(&piv_ready[b], 1);
    } else if (kind == kWkScore) {
      fused_do_score<NB, TAIL>(b, idx);
      __syncthreads();
      if (tid == 0 && atomicAdd(&score_done[b], 1) + 1 == sstart[b + 1] - sstart[b])
        fused_push(sy, batches, kWkOrder, b, P);
    } else if (kind == kWkOrder) {
      fused_do_order(b, idx);
      __syncthreads();
      if (tid == 0 && atomicAdd(&order_done[b], 1) + 1 == P)
        fused_push(sy, batches, kWkRetain, b, 1);
    } else if (kind == kWkRetain) {
      fused_do_retain(b, idx);
      __syncthreads();
      if (tid == 0) {
        st_dev<true>(&retain_done[b], 1);
        atomicAdd(&sy[kSyDone], 1);
      }
    } else {
      fused_do_gather(b, idx);
    }
  }
  if (tid == 0 && (ld_dev<true>(&sy[kSyDone]) & kFuAbortBit)) a_arg.status[3] = kFuAborted;
}

}  // namespace dart

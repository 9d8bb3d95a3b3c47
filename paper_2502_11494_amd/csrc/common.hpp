// Device-side helpers shared by the DART kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dart {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4v __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
constexpr int kMaxP = 64;        // pivots per sample
constexpr int kMaxN = 16384;     // tokens per sample
constexpr int kMaxBySize = 256;  // samples a ragged batch may have to be ordered by length

enum { kF32 = 0, kBF16 = 1 };

// The hardware deals the workgroups of a launch to the chip's 8 accelerator dies (XCDs, each
// with its own L2) round-robin by workgroup id.  For a streaming kernel whose block id
// selects a contiguous range of rows, this permutation of the ids gives every die one
// contiguous eighth of the rows instead of every eighth range (measured on the batches of
// 0.26-1.7 GB: -3..5 % on the norm and score passes, -3 % on the gather).  The grid must
// be a multiple of 8 blocks (round_up8); ids past the kernel's work fall out at its own
// bounds check.
constexpr int kXcds = 8;
#ifdef __HIPCC__
__device__ __forceinline__ long xcd_contiguous(unsigned bid, unsigned nblocks) {
  return (long)(bid % kXcds) * (nblocks / kXcds) + bid / kXcds;
}
#endif
inline long round_up8(long n) { return (n + kXcds - 1) / kXcds * kXcds; }
enum { kMaxL1 = 0, kMinL1 = 1, kGiven = 2, kRandom = 3 };

// ---- memory that another workgroup of the same launch wrote ------------------------------
// The chip has eight L2 caches (one per accelerator die) that are not kept coherent for
// ordinary loads and stores inside one kernel, and a cache-wide fence (write back and
// invalidate a whole L2) costs tens of microseconds under streaming load.  The one-launch
// path therefore moves everything one workgroup hands to another through device-scope
// accesses (`sc1` loads and stores: written through to memory, read past the caches), the
// same instructions the atomics use, one value at a time.  COH = false gives the plain
// access for kernels whose inputs were written by an earlier launch.
template <bool COH, typename T>
__device__ __forceinline__ T ld_dev(const T* p) {
  if (COH) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return *p;
}
template <bool COH, typename T>
__device__ __forceinline__ void st_dev(T* p, T v) {
  if (COH) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else *p = v;
}
// Every store this thread has issued has reached the point where other dies read it.  With
// a workgroup barrier after it, one thread may then raise a flag for other workgroups.
__device__ __forceinline__ void stores_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Shape of one call, passed to every kernel by value.
struct Geo {
  int B, D, P, Ppad;
  int N;            // dense tokens per sample (0 when ragged)
  int total_N;
  int max_N;
  int K;            // dense / uniform budget, 0 = ratio
  int keep_num, keep_den;
  int dtype, mode;
  int score_mode;   // 0: a threshold per pivot (staged rule); 1/2: one threshold on the min/max
  int tile_rows;    // token rows per score tile: 16 per wave of the score kernel's workgroup
  long ld;          // X row stride, elements
  const int* cu;    // device cu_seqlens, nullptr = dense
  // ragged only, filled by k_prepare: packed offsets of keep and of score tiles
  const int* cu_keep;
  const int* tile_start;
  // ragged batches of at most kMaxBySize samples, filled by k_prepare: the samples from the
  // longest to the shortest (nullptr: batch order)
  const int* by_size;
  // Pivots from outside the scored tokens (text-token pivots): the last Pe of the P pivots
  // of every sample are rows of E (sample b, outside pivot e at row b*Pe + e, stride lde
  // elements); the first Pin = P - Pe are tokens of the sample.
  int Pe, Pin;
  long lde;
  const void* E;
  // Ragged only, optional: sample b's tokens are rows span[b] .. span[b]+N_b-1 of X (of
  // the criterion tensor, of the position ids), X having x_rows rows; nullptr: the samples
  // are packed back to back (row cu[b]).  Workspace arrays are always indexed by cu[b].
  const int* span;
  int x_rows;
};

struct Sample {
  int row0;  // first row of the sample in the packed per-token arrays (scores, norms, ...)
  int xrow;  // first row of the sample in X
  int n;     // tokens
  int k;     // tokens to keep (0: skip the sample)
  int keep0; // first row of the sample in keep / Y / pos_out
};

__device__ __forceinline__ int budget_of(const Geo& g, int n) {
  return g.K > 0 ? g.K : (int)(((long)n * g.keep_num) / g.keep_den);
}

// A ragged sample is processed only if its sizes respect the limits and the budget.
__device__ __forceinline__ bool sample_ok(const Geo& g, int n, int k) {
  return n > 0 && n <= g.max_N && g.Pin <= n && k >= g.Pin && k <= n;
}

// Dense: arithmetic.  Ragged: k_prepare has validated the offsets and stored the
// per-sample budgets as differences of cu_keep (0 for a skipped sample).
__device__ __forceinline__ Sample sample_of(const Geo& g, int b) {
  Sample s;
  if (g.cu == nullptr) {
    s.row0 = b * g.N;
    s.xrow = s.row0;
    s.n = g.N;
    s.k = g.K;
    s.keep0 = b * g.K;
  } else {
    s.row0 = g.cu[b];
    s.xrow = g.span ? g.span[b] : s.row0;
    s.n = g.cu[b + 1] - s.row0;
    s.keep0 = g.cu_keep[b];
    s.k = g.cu_keep[b + 1] - s.keep0;
  }
  return s;
}

// Row of pivot i of sample b: a token of the sample (index piv[b*P + i], clamped so that a
// caller's bad index cannot leave X) or, for the last Pe pivots, a row of E.
// (COH: piv was written by another workgroup of this launch)
template <bool COH = false>
__device__ __forceinline__ const unsigned char* pivot_row(const Geo& g, const void* X, int esz,
                                                          const Sample& sm, int b, int i,
                                                          const int* piv) {
  if (i >= g.Pin)
    return static_cast<const unsigned char*>(g.E) + ((long)b * g.Pe + (i - g.Pin)) * g.lde * esz;
  int p = ld_dev<COH>(&piv[b * g.P + i]);
  p = p < 0 ? 0 : (p < sm.n ? p : sm.n - 1);
  return static_cast<const unsigned char*>(X) + ((long)sm.xrow + p) * g.ld * esz;
}

// Even split of the K-Pin non-pivot slots over the P stages of Eq. (9)-(10): stage i
// takes q (+1 for the first r stages).  Pin <= P pivots are tokens of the sample and hold
// a slot each; the others come from outside.  Built once per sample (two divisions).
struct Split {
  int pin, q, r;  // pin: slots held by pivots; q, r: quotient and remainder over the stages
  __device__ __forceinline__ Split(int k, int stages, int Pin)
      : pin(Pin), q((k - Pin) / stages), r((k - Pin) % stages) {}
  __device__ __forceinline__ int quota(int i) const { return q + (i < r ? 1 : 0); }
  // slots filled once stages 0..i are done, pivots included
  __device__ __forceinline__ int filled_after(int i) const {
    return pin + q * (i + 1) + (i + 1 < r ? i + 1 : r);
  }
  // tokens taken by the stages before stage i (pivots not counted)
  __device__ __forceinline__ int taken_before(int i) const { return q * i + (i < r ? i : r); }
  // Entries of pivot i's ascending score list that stage i may look at: the slots
  // filled once the stage is done plus one beyond (the first refused candidate),
  // or nothing if the stage takes nothing.
  __device__ __forceinline__ int stage_len(int n, int i) const {
    if (quota(i) == 0) return 0;
    int len = filled_after(i) + 1;
    return len < n ? len : n;
  }
  // The stage lists of one sample are stored back to back: offset of stage i's list.
  __device__ __forceinline__ long list_offset(int n, int i) const {
    long off = 0;
    for (int s = 0; s < i; ++s) off += stage_len(n, s);
    return off;
  }
};

// ---- element access --------------------------------------------------------------

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// ---- order-preserving integer image of a float ----------------------------------
// -0 and +0 must compare equal, so callers add +0.0f first.
__device__ __forceinline__ uint32_t mono_of(float f) {
  uint32_t u = __float_as_uint(f);
  return u ^ ((u >> 31) ? 0xffffffffu : 0x80000000u);
}
__device__ __forceinline__ float mono_inv(uint32_t m) {
  uint32_t u = m ^ ((m >> 31) ? 0x80000000u : 0xffffffffu);
  return __uint_as_float(u);
}

// ---- lane exchange on the vector ALU ------------------------------------------------
// lane_xor<J>(v, lane) returns v of lane (lane ^ J).  Inside a row of 16 lanes these
// are data-parallel-primitive moves (quad permutes, row rotations); across rows the
// gfx950 row / half swaps.  None of them goes through the LDS crossbar, so a
// butterfly costs a few ALU cycles per step.  Every lane of the wave must be active.
template <int CTRL>
__device__ __forceinline__ int dpp_move(int old, int v) {
  return __builtin_amdgcn_update_dpp(old, v, CTRL, 0xf, 0xf, false);
}
constexpr int kDppXor1 = 0xB1;       // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;       // quad_perm [2,3,0,1]
constexpr int kDppRor4 = 0x124;      // lane i <- lane (i-4) mod 16 of its row
constexpr int kDppRor8 = 0x128;      // lane i <- lane i^8
constexpr int kDppRor12 = 0x12C;     // lane i <- lane (i+4) mod 16 of its row
constexpr int kDppShr1 = 0x111, kDppShr2 = 0x112, kDppShr4 = 0x114, kDppShr8 = 0x118;

template <int J>
__device__ __forceinline__ int lane_xor(int v, int lane) {
  static_assert(J == 1 || J == 2 || J == 4 || J == 8 || J == 16 || J == 32, "one bit");
  if (J == 1) return dpp_move<kDppXor1>(v, v);
  if (J == 2) return dpp_move<kDppXor2>(v, v);
  if (J == 4) {
    const int dn = dpp_move<kDppRor4>(v, v), up = dpp_move<kDppRor12>(v, v);
    return (lane & 4) ? dn : up;
  }
  if (J == 8) return dpp_move<kDppRor8>(v, v);
  if (J == 16) {  // .x = rows 0,0,2,2   .y = rows 1,1,3,3
    const auto sw = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    return (lane & 16) ? (int)sw[0] : (int)sw[1];
  }
  // .x = lower half twice, .y = upper half twice
  const auto sw = __builtin_amdgcn_permlane32_swap(v, v, false, false);
  return (lane & 32) ? (int)sw[0] : (int)sw[1];
}
template <int J>
__device__ __forceinline__ float lane_xor(float v, int lane) {
  return __int_as_float(lane_xor<J>(__float_as_int(v), lane));
}
template <int J>
__device__ __forceinline__ unsigned long long lane_xor(unsigned long long v, int lane) {
  const uint32_t lo = (uint32_t)lane_xor<J>((int)(uint32_t)v, lane);
  const uint32_t hi = (uint32_t)lane_xor<J>((int)(uint32_t)(v >> 32), lane);
  return ((unsigned long long)hi << 32) | lo;
}
template <int J>
__device__ __forceinline__ double lane_xor(double v, int lane) {
  return __longlong_as_double((long long)lane_xor<J>((unsigned long long)__double_as_longlong(v), lane));
}

// ---- wave reductions (butterfly: every lane ends with the same bits) ------------------

#define DART_WAVE_BUTTERFLY(v, OP)          \
  {                                         \
    const int l_ = threadIdx.x & 63;        \
    v = OP(v, lane_xor<1>(v, l_));          \
    v = OP(v, lane_xor<2>(v, l_));          \
    v = OP(v, lane_xor<4>(v, l_));          \
    v = OP(v, lane_xor<8>(v, l_));          \
    v = OP(v, lane_xor<16>(v, l_));         \
    v = OP(v, lane_xor<32>(v, l_));         \
  }
#define DART_OP_ADD(a, b) ((a) + (b))
__device__ __forceinline__ float wave_sum(float v) {
  DART_WAVE_BUTTERFLY(v, DART_OP_ADD);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
  DART_WAVE_BUTTERFLY(v, DART_OP_ADD);
  return v;
}
__device__ __forceinline__ int wave_sum(int v) {
  DART_WAVE_BUTTERFLY(v, DART_OP_ADD);
  return v;
}
__device__ __forceinline__ float wave_min(float v) {
  DART_WAVE_BUTTERFLY(v, fminf);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
  DART_WAVE_BUTTERFLY(v, fmaxf);
  return v;
}
#undef DART_OP_ADD
#undef DART_WAVE_BUTTERFLY

// Exclusive prefix sum over the lanes of a wave: a shift-and-add scan inside every row
// of 16 lanes (lanes without a source add 0), then the totals of the rows before.
__device__ __forceinline__ int wave_excl_scan(int v, int lane) {
  int x = v;
  x += dpp_move<kDppShr1>(0, x);
  x += dpp_move<kDppShr2>(0, x);
  x += dpp_move<kDppShr4>(0, x);
  x += dpp_move<kDppShr8>(0, x);
  const int t0 = __builtin_amdgcn_readlane(x, 15), t1 = __builtin_amdgcn_readlane(x, 31),
            t2 = __builtin_amdgcn_readlane(x, 47);
  const int row = lane >> 4;
  x += (row >= 1 ? t0 : 0) + (row >= 2 ? t1 : 0) + (row >= 3 ? t2 : 0);
  return x - v;
}

// ---- fp64 re-evaluation of one row (used where an fp32 decision is too close) ----
// Each lane walks the row in 16-byte pieces, lane-strided (piece t belongs to lane
// t % 64), eight loads in flight at a time, one fp64 chain per quantity in piece
// order; the butterfly makes the result a pure function of the row's bytes.

template <int DT>
__device__ __forceinline__ void piece_to_f64(const u32x4& v, double (&x)[8]) {
  if (DT == kBF16) {
    x[0] = (double)bf16_lo(v.x); x[1] = (double)bf16_hi(v.x);
    x[2] = (double)bf16_lo(v.y); x[3] = (double)bf16_hi(v.y);
    x[4] = (double)bf16_lo(v.z); x[5] = (double)bf16_hi(v.z);
    x[6] = (double)bf16_lo(v.w); x[7] = (double)bf16_hi(v.w);
  } else {
    x[0] = (double)__uint_as_float(v.x); x[1] = (double)__uint_as_float(v.y);
    x[2] = (double)__uint_as_float(v.z); x[3] = (double)__uint_as_float(v.w);
    x[4] = x[5] = x[6] = x[7] = 0.0;
  }
}

template <int DT>
__device__ __forceinline__ void row_l1_l2_f64(const void* row, int D, int lane, double& l1,
                                              double& l2) {
  const int pieces = D * (DT == kBF16 ? 2 : 4) / 16;
  const u32x4* p = reinterpret_cast<const u32x4*>(row);
  const u32x4 zero = {0u, 0u, 0u, 0u};
  double a = 0.0, b = 0.0;
  for (int t0 = 0; t0 < pieces; t0 += kWave * 8) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      int t = t0 + u * kWave + lane;
      v[u] = t < pieces ? p[t] : zero;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      double x[8];
      piece_to_f64<DT>(v[u], x);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        a += fabs(x[e]);
        b = fma(x[e], x[e], b);
      }
    }
  }
  l1 = wave_sum(a);
  l2 = wave_sum(b);
}

// The same for R rows at once (all their loads in flight together).  Rows past
// `live` are skipped; each row's result is identical to row_l1_l2_f64's.
template <int DT, int R>
__device__ __forceinline__ void rows_l1_l2_f64(const void* const (&row)[R], int live, int D,
                                               int lane, double (&l1)[R], double (&l2)[R]) {
  const int pieces = D * (DT == kBF16 ? 2 : 4) / 16;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  double a[R], b[R];
#pragma unroll
  for (int r = 0; r < R; ++r) a[r] = b[r] = 0.0;
  for (int t0 = 0; t0 < pieces; t0 += kWave * 8) {
    u32x4 v[R][8];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        int t = t0 + u * kWave + lane;
        v[r][u] = (r < live && t < pieces) ? reinterpret_cast<const u32x4*>(row[r])[t] : zero;
      }
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        double x[8];
        piece_to_f64<DT>(v[r][u], x);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          a[r] += fabs(x[e]);
          b[r] = fma(x[e], x[e], b[r]);
        }
      }
  }
#pragma unroll
  for (int r = 0; r < R; ++r) {
    l1[r] = wave_sum(a[r]);
    l2[r] = wave_sum(b[r]);
  }
}

// Cosine of Eq. (7) between rows p and x in fp64; 0 if either norm is 0.
// PPG: the squared norm of p is given (pp_given, an fp64 sum over the same row) and its
// products are left out (a sixth of the arithmetic).
// INF: 16-byte pieces of each row a lane keeps in flight (8: a whole 8 KiB row pair at once;
// fewer where registers are short).  The sums run in piece order whatever INF is.
template <int DT, bool PPG = false, int INF = 8>
__device__ __forceinline__ double row_cosine_f64(const void* prow, const void* xrow, int D,
                                                 int lane, double pp_given = 0.0) {
  const int pieces = D * (DT == kBF16 ? 2 : 4) / 16;
  const u32x4* p = reinterpret_cast<const u32x4*>(prow);
  const u32x4* x = reinterpret_cast<const u32x4*>(xrow);
  const u32x4 zero = {0u, 0u, 0u, 0u};
  double dot = 0.0, pp = 0.0, xx = 0.0;
  for (int t0 = 0; t0 < pieces; t0 += kWave * INF) {
    u32x4 pv[INF], xv[INF];
#pragma unroll
    for (int u = 0; u < INF; ++u) {
      int t = t0 + u * kWave + lane;
      pv[u] = t < pieces ? p[t] : zero;
      xv[u] = t < pieces ? x[t] : zero;
    }
#pragma unroll
    for (int u = 0; u < INF; ++u) {
      double pe[8], xe[8];
      piece_to_f64<DT>(pv[u], pe);
      piece_to_f64<DT>(xv[u], xe);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        dot = fma(pe[e], xe[e], dot);
        if (!PPG) pp = fma(pe[e], pe[e], pp);
        xx = fma(xe[e], xe[e], xx);
      }
    }
  }
  dot = wave_sum(dot);
  pp = PPG ? pp_given : wave_sum(pp);
  xx = wave_sum(xx);
  double den = sqrt(pp) * sqrt(xx);
  return den > 0.0 ? dot / den : 0.0;
}

// ---- block-wide bitonic sort of 64-bit keys -----------------------------------------
// Thread t keeps elements t, t+THREADS, ... (M of them) in registers.  A
// compare-exchange at distance j is done in registers when j >= THREADS, by lane
// exchanges on the vector ALU when j < 64, and through LDS (two barriers) only for 64 <= j < THREADS.

template <int THREADS, int M, int JM>
__device__ __forceinline__ void reg_compare_exchange(unsigned long long (&v)[M], int k, int tid) {
#pragma unroll
  for (int m = 0; m < M; ++m) {
    if ((m & JM) == 0 && (m | JM) < M) {
      const bool up = (((m * THREADS + tid) & k) == 0);
      const unsigned long long a = v[m], b = v[m | JM];
      if ((a > b) == up) {
        v[m] = b;
        v[m | JM] = a;
      }
    }
  }
}

// Compare-exchange at lane distance J < 64 (partner in the same wave).
template <int THREADS, int M, int J>
__device__ __forceinline__ void lane_compare_exchange(unsigned long long (&v)[M], int k, int tid) {
#pragma unroll
  for (int m = 0; m < M; ++m) {
    const int e = m * THREADS + tid;
    const unsigned long long o = lane_xor<J>(v[m], tid & 63);
    const bool keep_min = ((tid & J) == 0) == ((e & k) == 0);
    v[m] = keep_min ? (v[m] < o ? v[m] : o) : (v[m] > o ? v[m] : o);
  }
}

// Merge stage k >= 64, distances 32..1: all partners are in the same wave.
template <int THREADS, int M>
__device__ __forceinline__ void wave_merge_tail(unsigned long long (&v)[M], int k, int tid) {
  lane_compare_exchange<THREADS, M, 32>(v, k, tid);
  lane_compare_exchange<THREADS, M, 16>(v, k, tid);
  lane_compare_exchange<THREADS, M, 8>(v, k, tid);
  lane_compare_exchange<THREADS, M, 4>(v, k, tid);
  lane_compare_exchange<THREADS, M, 2>(v, k, tid);
  lane_compare_exchange<THREADS, M, 1>(v, k, tid);
}

// Stages k = 2..64 (21 compare-exchanges, straight-line): every run of 64 consecutive
// elements ends up sorted, ascending or descending as stage 128 needs it.
template <int THREADS, int M>
__device__ __forceinline__ void wave_sort_runs(unsigned long long (&v)[M], int tid) {
  lane_compare_exchange<THREADS, M, 1>(v, 2, tid);
  lane_compare_exchange<THREADS, M, 2>(v, 4, tid);
  lane_compare_exchange<THREADS, M, 1>(v, 4, tid);
  lane_compare_exchange<THREADS, M, 4>(v, 8, tid);
  lane_compare_exchange<THREADS, M, 2>(v, 8, tid);
  lane_compare_exchange<THREADS, M, 1>(v, 8, tid);
  lane_compare_exchange<THREADS, M, 8>(v, 16, tid);
  lane_compare_exchange<THREADS, M, 4>(v, 16, tid);
  lane_compare_exchange<THREADS, M, 2>(v, 16, tid);
  lane_compare_exchange<THREADS, M, 1>(v, 16, tid);
  lane_compare_exchange<THREADS, M, 16>(v, 32, tid);
  lane_compare_exchange<THREADS, M, 8>(v, 32, tid);
  lane_compare_exchange<THREADS, M, 4>(v, 32, tid);
  lane_compare_exchange<THREADS, M, 2>(v, 32, tid);
  lane_compare_exchange<THREADS, M, 1>(v, 32, tid);
  wave_merge_tail<THREADS, M>(v, 64, tid);
}

// Sorts s[0..n) ascending.  n is a power of two with 64 <= n; n == M*THREADS, or
// n < THREADS with M == 1.  n must be the same on every thread; all threads call.
template <int THREADS, int M>
__device__ __forceinline__ void block_bitonic_sort_m(unsigned long long* s, int n, int tid) {
  static_assert(M <= 16, "register distances 1..8 are handled");
  const bool live = (tid & ~(kWave - 1)) < n;  // waves past the data only keep the barriers
  unsigned long long v[M];
#pragma unroll
  for (int m = 0; m < M; ++m) v[m] = (m * THREADS + tid < n) ? s[m * THREADS + tid] : ~0ull;
  if (live) wave_sort_runs<THREADS, M>(v, tid);
  for (int k = 128; k <= n; k <<= 1) {
    for (int j = k >> 1; j >= kWave; j >>= 1) {
      if (j >= THREADS) {
        switch (j / THREADS) {
          case 1: reg_compare_exchange<THREADS, M, 1>(v, k, tid); break;
          case 2: reg_compare_exchange<THREADS, M, 2>(v, k, tid); break;
          case 4: reg_compare_exchange<THREADS, M, 4>(v, k, tid); break;
          default: reg_compare_exchange<THREADS, M, 8>(v, k, tid); break;
        }
      } else {
        __syncthreads();
        if (live) {
#pragma unroll
          for (int m = 0; m < M; ++m) s[m * THREADS + tid] = v[m];
        }
        __syncthreads();
        if (live) {
#pragma unroll
          for (int m = 0; m < M; ++m) {
            const int e = m * THREADS + tid;
            const unsigned long long o = s[e ^ j];
            const bool keep_min = ((tid & j) == 0) == ((e & k) == 0);
            v[m] = keep_min ? (v[m] < o ? v[m] : o) : (v[m] > o ? v[m] : o);
          }
        }
      }
    }
    if (live) wave_merge_tail<THREADS, M>(v, k, tid);
  }
  __syncthreads();
#pragma unroll
  for (int m = 0; m < M; ++m)
    if (m * THREADS + tid < n) s[m * THREADS + tid] = v[m];
  __syncthreads();
}

// Plain LDS bitonic sort (one barrier per compare-exchange distance): used only for
// the huge lists that massive ties or a keep-everything budget produce.
template <int THREADS>
__device__ __forceinline__ void block_bitonic_sort_lds(unsigned long long* s, int n, int tid) {
  for (int k = 2; k <= n; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int t = tid; t < (n >> 1); t += THREADS) {
        const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
        const int l = i | j;
        const unsigned long long a = s[i], b = s[l];
        if ((a > b) == ((i & k) == 0)) {
          s[i] = b;
          s[l] = a;
        }
      }
      __syncthreads();
    }
  }
}

// n: power of two, n >= 64, identical on every thread; s holds n keys (LDS).
// MAXM: the caller's n never exceeds MAXM*THREADS (the larger variants, which need the most
// registers, are then not compiled into its kernel).
template <int THREADS, int MAXM = 16>
__device__ __forceinline__ void block_bitonic_sort(unsigned long long* s, int n, int tid) {
  n = __builtin_amdgcn_readfirstlane(n);
  if (n <= THREADS) {
    block_bitonic_sort_m<THREADS, 1>(s, n, tid);
    return;
  }
  if constexpr (MAXM >= 2) {
    if (n == 2 * THREADS) {
      block_bitonic_sort_m<THREADS, 2>(s, n, tid);
      return;
    }
  }
  if constexpr (MAXM >= 4) {
    if (n == 4 * THREADS) {
      block_bitonic_sort_m<THREADS, 4>(s, n, tid);
      return;
    }
  }
  if constexpr (MAXM >= 8) {
    if (n == 8 * THREADS) {
      block_bitonic_sort_m<THREADS, 8>(s, n, tid);
      return;
    }
  }
  if constexpr (MAXM >= 16) {
    if (n == 16 * THREADS) {
      block_bitonic_sort_m<THREADS, 16>(s, n, tid);
      return;
    }
  }
  block_bitonic_sort_lds<THREADS>(s, n, tid);
}

__device__ __forceinline__ int next_pow2(int v) {
  int p = 1;
  while (p < v) p <<= 1;
  return p;
}

}  // namespace dart

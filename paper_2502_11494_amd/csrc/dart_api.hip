// Host side of the DART C ABI (include/dart.h): argument checks, workspace
// carving and kernel launches.  No allocation, no synchronisation except in
// dart_device_status.
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <mutex>

#include "../../include/dart.h"
#include "common.hpp"
#include "k_fused.hpp"
#include "k_misc.hpp"
#include "k_norms.hpp"
#include "k_order.hpp"
#include "k_pivots.hpp"
#include "k_retain.hpp"
#include "k_scores.hpp"
#include "k_single.hpp"

using namespace dart;

// Scratch of dart_reduce_static: one copy per GPU, at an address of its own on each.  In host
// code this name is only a handle for hipGetSymbolAddress, never a device address.
constexpr size_t kStaticScratchBytes = size_t(32) << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr size_t kAlign = 256;
// Row strides (elements) are bounded so that rows * stride * element size stays far inside 64
// bits on the host and in the kernels' byte offsets.
constexpr int64_t kMaxLd = int64_t(1) << 24;
constexpr int kMaxB = 1 << 20;  // samples per call (grids and offset tables are sized by B)
inline size_t up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Plan {
  Geo g;
  int esz;
  long keep_rows_bound;  // upper bound of the total number of retained rows
  int tiles_bound;       // upper bound of the number of score tiles (g.tile_rows rows each)
  // workspace offsets
  size_t o_status, o_cu_keep, o_tile_start, o_l1, o_piv, o_pl2, o_S, o_lists, o_scr_f64,
      o_l2, o_sync, o_nstart, o_sstart, o_gstart, o_by_size, total;
  bool fusable;  // the shape and modes the one-launch path covers (see reduce_impl)
  bool norms_given;  // this call's norm pass also leaves the squared token norms
  int ks_waves, ks_split;  // bf16 score kernel: waves per workgroup and groups of them (fp32: 0)
  bool retain_packed;      // the largest sample's stage lists need the 6-byte LDS layout
  unsigned long long seed; // DART_PIVOT_RANDOM: the seed of the draw
};

// Compute units of the current GPU looked up once per GPU.
int compute_units() {
  static std::mutex m;
  static int cached[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  std::lock_guard<std::mutex> lock(m);
  if (cached[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      n = 256;
    cached[dev] = n;
  }
  return cached[dev];
}

// ---- tile shape of the bf16 score kernel ----------------------------------------------------
// k_scores_ksplit takes any number of waves W per workgroup and splits the D-chunks over KS
// groups of them, so a tile has R = 16*W/KS rows.  Measured on the benchmark shapes the kernel
// runs at the speed of the busiest compute unit: about 6 TB/s for the chip as a whole (pivot
// chunks, served by L2, count about a fifth of their bytes), plus 48 GB/s for whatever rows
// the busiest unit holds beyond the average (the units take ceil(tiles/256) or one fewer tiles
// each), and never faster than a wave's chain of chunks (0.55 us each).  Tile heights that
// divide the batch evenly over the 256 units therefore win: 9 waves (144 rows) for four
// samples of 9216 tokens (47 us against 55 with 64-row tiles), 12 waves in 4 groups (48 rows)
// for sixteen of 576 (18 us against 27 for four workgroups per tile and a finishing pass).
// The candidates are the shapes instantiated below.
struct KsChoice { int waves, split; };
#define DART_KS_SHAPES(X_)                                                                   \
  X_(3, 1) X_(4, 1) X_(5, 1) X_(6, 1) X_(8, 1) X_(9, 1) X_(10, 1) X_(11, 1) X_(12, 1)        \
  X_(4, 2) X_(6, 2) X_(8, 2) X_(12, 2) X_(6, 3) X_(9, 3) X_(12, 3)                          \
  X_(8, 4) X_(12, 4) X_(16, 4)
constexpr KsChoice kKsShapes[] = {
#define DART_KS_ENTRY(W, KS) {W, KS},
    DART_KS_SHAPES(DART_KS_ENTRY)
#undef DART_KS_ENTRY
};
constexpr size_t kKsLdsLimit = 150 * 1024;  // of the 160 KB of a compute unit

// first_read: the score pass is the first pass of the call over X (pivots given or drawn, a
// separate criterion tensor, the stage entry point), so no norm pass has left the rows in the
// memory-side cache.
KsChoice choose_score_tiles(const Geo& g, int units, bool first_read) {
  const int NB = g.Ppad / 16;
  const double rowbytes = (double)g.D * 2;
  const int chunks = (g.D + kKsCH - 1) / kKsCH;
  struct Cost {
    double t, rows_busiest;
    bool fits;
  };
  auto cost = [&](const KsChoice& c) -> Cost {
    const int R = 16 * c.waves / c.split;
    const size_t lds = ksplit_lds_bytes(NB, c.split, c.waves);
    if (lds > kKsLdsLimit) return {1e30, 0.0, false};
    const double tiles = g.cu == nullptr ? (double)g.B * ((g.N + R - 1) / R)
                                         : (double)g.total_N / R + 0.5 * g.B;
    const double per_unit = std::ceil(tiles / units);
    const double rows_busiest = per_unit * R;
    const double rows_avg = (double)g.total_N / units;
    const double weight = 1.0 + 0.2 * NB * 16 / R;  // pivot chunks come from L2
    double t = g.total_N * rowbytes * weight / 6.0e12;
    if (rows_busiest > rows_avg) t += (rows_busiest - rows_avg) * rowbytes * weight / 48e9;
    const int resident = (int)std::max<size_t>(1, std::min<size_t>(kKsLdsLimit / lds, 16 / c.waves));
    const double chain = std::ceil(per_unit / resident) * ((chunks + c.split - 1) / c.split) * 0.55e-6 + 4e-6;
    t = std::max(t, chain);
    t += 1e-9 * (256 - R) / 256;  // ties: the taller tile (less pivot traffic)
    return {t, rows_busiest, true};
  };
  KsChoice best = {4, 1};
  double best_t = 1e30;
  for (const KsChoice& c : kKsShapes) {
    const Cost k = cost(c);
    if (k.fits && k.t < best_t) {
      best_t = k.t;
      best = c;
    }
  }
  // What the model does not see, measured with every shape forced in turn (score pass by the
  // launch's own events): where a wave's chain of chunks matters, four groups of waves per
  // tile beat two or three of the same tile height (32 rows: 8 waves in 4 groups 15.9 us
  // against 17.4 for 6 in 3 on 32 samples of 256 tokens; 48 rows: 12 in 4 groups 15.2 against
  // 17.2 for 6 in 2 on sixteen 576-token images, 22.1 against 25.2 at a hidden size of 5120) ...
  const int R_best = 16 * best.waves / best.split;
  if (best.split >= 2 && best.split < 4 && (R_best == 32 || R_best == 48)) {
    const KsChoice four = {R_best / 4, 4};
    if (cost(four).fits) return four;
  }
  // ... and on a first read of X they also beat the single group on small dense batches as
  // long as no compute unit gets more rows than with the model's pick (eight samples of 2880
  // tokens: 34.7-35.5 us against 38.6 for 6 waves in one group; with 32 pivots or thousands
  // of tiles the single group stays ahead: 45.6 against 59.5, 276 against 324 us).
  if (first_read && best.split == 1 && NB == 1 && g.cu == nullptr) {
    const Cost picked = cost(best);
    if (picked.rows_busiest <= 128) {
      // (of the two, the one that loads the busiest unit less; equal: the 32-row tiles, two
      // workgroups of which share a unit: 34.7 against 35.5-36.3 us on the headline batch)
      KsChoice alt = best;
      double alt_rows = picked.rows_busiest + 1;
      for (const KsChoice& c : {KsChoice{8, 4}, KsChoice{12, 4}}) {
        const Cost k = cost(c);
        if (k.fits && k.rows_busiest <= picked.rows_busiest && k.rows_busiest < alt_rows) {
          alt_rows = k.rows_busiest;
          alt = c;
        }
      }
      return alt;
    }
  }
  return best;
}

// Upper bound of the number of score tiles for the tile height in p.g.tile_rows.
void size_score_tiles(Plan& p) {
  if (p.g.cu == nullptr)
    p.tiles_bound = p.g.B * ((p.g.N + p.g.tile_rows - 1) / p.g.tile_rows);
  else
    p.tiles_bound = (int)(p.g.total_N / p.g.tile_rows) + p.g.B;
}

// DART_SCORE_TILE="W,KS" in the environment names the shape instead (for tuning, and for the
// tests that run every instantiated shape); a value that is not one of the shapes above, or
// does not fit the LDS with this many pivots, is an error of the call.
dart_status plan_score_tiles(Plan& p, bool first_read) {
  KsChoice c = choose_score_tiles(p.g, compute_units(), first_read);
  if (const char* v = std::getenv("DART_SCORE_TILE")) {
    int w = 0, ks = 0;
    bool known = false;
    if (std::sscanf(v, "%d,%d", &w, &ks) == 2)
      for (const KsChoice& k : kKsShapes) known = known || (k.waves == w && k.split == ks);
    if (!known || ksplit_lds_bytes(p.g.Ppad / 16, ks, w) > kKsLdsLimit) return DART_ERR_SHAPE;
    c = {w, ks};
  }
  p.ks_waves = c.waves;
  p.ks_split = c.split;
  p.g.tile_rows = 16 * c.waves / c.split;
  size_score_tiles(p);
  return DART_OK;
}

// An entry point whose score pass is the first pass over X plans its tiles again (make_plan
// assumes a norm pass over X before it).
dart_status replan_first_read(Plan& p) {
  return p.g.dtype == kBF16 ? plan_score_tiles(p, true) : DART_OK;
}

// Entries of all stage lists of a sample of n tokens that keeps k of them with P pivots, Pin
// of them among the tokens (the sum of Split::stage_len over the stages).
long retain_list_entries(int n, int k, int P, int Pin) {
  if (k <= Pin) return 0;
  const int q = (k - Pin) / P, r = (k - Pin) % P;
  long total = 0;
  for (int i = 0; i < P; ++i) {
    if (q + (i < r ? 1 : 0) == 0) continue;
    const int filled = Pin + q * (i + 1) + (i + 1 < r ? i + 1 : r);
    total += std::min(filled + 1, n);
  }
  return total;
}

dart_status make_plan(const dart_desc* d, Plan& p) {
  if (!d) return DART_ERR_NULL;
  if (d->dtype != DART_F32 && d->dtype != DART_BF16) return DART_ERR_DTYPE;
  if (d->pivot_mode != DART_PIVOT_MAX_L1 && d->pivot_mode != DART_PIVOT_MIN_L1 &&
      d->pivot_mode != DART_PIVOT_GIVEN && d->pivot_mode != DART_PIVOT_RANDOM)
    return DART_ERR_DTYPE;
  if (d->B < 0 || d->B > kMaxB || d->D <= 0 || d->D > 65536 || d->P < 1 || d->P > kMaxP || d->ld < d->D ||
      d->ld > kMaxLd || d->score_mode < 0 || d->score_mode > 2 || d->P_ext < 0 || d->P_ext > d->P)
    return DART_ERR_SHAPE;
  const int Pin = d->P - d->P_ext;  // pivots that are tokens of the sample
  const bool ragged = d->cu_seqlens != nullptr;
  long total;
  int maxn;
  if (!ragged) {
    if (d->N < 0 || d->N > kMaxN) return DART_ERR_SHAPE;
    total = (long)d->B * d->N;
    if (d->total_N != 0 && d->total_N != total) return DART_ERR_SHAPE;
    maxn = d->N;
  } else {
    if (d->total_N < 0 || d->max_N < 1 || d->max_N > kMaxN) return DART_ERR_SHAPE;
    total = d->total_N;
    maxn = d->max_N;
  }
  if (total > (1L << 27)) return DART_ERR_SHAPE;
  if (d->span_start) {  // spans of a larger tensor: packed lengths required, X_rows bounds them
    if (!ragged) return DART_ERR_NULL;
    if (d->X_rows < total || d->X_rows > (1 << 30)) return DART_ERR_SHAPE;
  }
  if (d->K < 0) return DART_ERR_BUDGET;
  if (d->K == 0 && (d->keep_den <= 0 || d->keep_num < 0 || d->keep_num > d->keep_den))
    return DART_ERR_BUDGET;
  int K = d->K;
  if (!ragged) {
    if (K == 0) K = (int)(((long)d->N * d->keep_num) / d->keep_den);
    if (d->B > 0 && (Pin > d->N || K < Pin || K > d->N)) return DART_ERR_BUDGET;
  } else if (K > 0 && (K < Pin || K > maxn)) {
    return DART_ERR_BUDGET;
  }
  const int esz = d->dtype == DART_BF16 ? 2 : 4;
  if (((long)d->ld * esz) % 16 != 0 || ((long)d->D * esz) % 16 != 0) return DART_ERR_ALIGN;
  if (d->P_ext > 0) {
    if (!d->ext_pivots) return DART_ERR_NULL;
    if (d->ext_ld < d->D || d->ext_ld > kMaxLd) return DART_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(d->ext_pivots) & 15u) != 0 || ((long)d->ext_ld * esz) % 16 != 0)
      return DART_ERR_ALIGN;
  }

  Geo& g = p.g;
  g.B = d->B;
  g.D = d->D;
  g.P = d->P;
  g.Ppad = (d->P + 15) / 16 * 16;
  g.N = ragged ? 0 : d->N;
  g.total_N = (int)total;
  g.max_N = maxn;
  g.K = ragged ? d->K : K;
  g.keep_num = d->keep_num;
  g.keep_den = d->keep_den > 0 ? d->keep_den : 1;
  g.dtype = d->dtype;
  g.mode = d->pivot_mode;
  p.seed = d->seed;
  g.score_mode = d->score_mode;
  g.ld = d->ld;
  g.cu = d->cu_seqlens;
  g.cu_keep = nullptr;
  g.tile_start = nullptr;
  g.by_size = nullptr;
  g.Pe = d->P_ext;
  g.Pin = Pin;
  g.lde = d->P_ext > 0 ? d->ext_ld : 0;
  g.E = d->P_ext > 0 ? d->ext_pivots : nullptr;
  g.span = d->span_start;
  g.x_rows = d->span_start ? d->X_rows : (int)total;
  // score tiles: fp32 rows are scored 4 to a block, counted in tiles of 64; bf16 tiles take
  // the shape chosen for this batch
  g.tile_rows = 64;
  p.ks_waves = p.ks_split = 0;
  if (d->dtype == DART_BF16) {
    // (pivots given, drawn or all from outside: no norm pass reads X before the score pass)
    const dart_status ts = plan_score_tiles(p, d->pivot_mode == DART_PIVOT_GIVEN ||
                                                   d->pivot_mode == DART_PIVOT_RANDOM || Pin == 0);
    if (ts != DART_OK) return ts;
  }
  p.esz = esz;
  {
    const int n_big = ragged ? maxn : d->N;
    const int k_big = ragged ? (d->K > 0 ? d->K : (int)(((long)maxn * d->keep_num) / g.keep_den)) : K;
    p.retain_packed = retain_list_entries(n_big, k_big, d->P, Pin) > kRetList;
  }
  if (!ragged) {
    p.keep_rows_bound = (long)d->B * K;
  } else {
    p.keep_rows_bound = d->K > 0 ? (long)d->B * d->K
                                 : (long)(((__int128)total * d->keep_num) / g.keep_den);
    if (p.keep_rows_bound > total) p.keep_rows_bound = total;
  }
  size_score_tiles(p);
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += up(bytes); return at; };
  p.o_status = take(kAlign);
  p.o_cu_keep = take(sizeof(int) * ((size_t)d->B + 1));
  p.o_tile_start = take(sizeof(int) * ((size_t)d->B + 1));
  p.o_l1 = take(sizeof(float) * (size_t)total);
  p.o_piv = take(sizeof(int) * (size_t)d->B * d->P);
  p.o_pl2 = take(sizeof(double) * (size_t)d->B * g.Ppad);
  p.o_S = take(sizeof(float) * (size_t)total * d->P);
  p.o_lists = take(sizeof(unsigned long long) * (size_t)total * d->P);
  p.o_scr_f64 = take(sizeof(double) * 2 * (size_t)total);
  p.o_l2 = take(sizeof(double) * (size_t)total);
  // one-launch path: bf16, pivots chosen among the tokens, the staged rule, packed samples
  p.fusable = d->dtype == DART_BF16 && d->pivot_mode != DART_PIVOT_GIVEN &&
              d->pivot_mode != DART_PIVOT_RANDOM && d->P_ext == 0 &&
              d->score_mode == 0 && d->span_start == nullptr && d->B <= kFuMaxB;
  if (d->B <= kFuMaxB) {  // (the same workspace size whatever the modes)
    p.o_sync = take(sizeof(int) * (size_t)fused_sync_ints(d->B, d->P));
    p.o_nstart = take(sizeof(int) * ((size_t)d->B + 1));
    p.o_sstart = take(sizeof(int) * ((size_t)d->B + 1));
    p.o_gstart = take(sizeof(int) * ((size_t)d->B + 1));
  } else {
    p.o_sync = p.o_nstart = p.o_sstart = p.o_gstart = o;
  }
  p.o_by_size = take(sizeof(int) * kMaxBySize);
  p.norms_given = false;
  p.total = o;
  return DART_OK;
}

inline bool misaligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

dart_status check_ws(const Plan& p, const void* ws, size_t ws_bytes) {
  if (!ws || (reinterpret_cast<uintptr_t>(ws) % kAlign) != 0 || ws_bytes < p.total)
    return DART_ERR_WORKSPACE;
  return DART_OK;
}

template <typename T>
inline T* at(void* ws, size_t off) {
  return reinterpret_cast<T*>(static_cast<unsigned char*>(ws) + off);
}

#define DART_LAUNCH_CHECK()                              \
  do {                                                   \
    if (hipGetLastError() != hipSuccess) return DART_ERR_HIP; \
  } while (0)

// Stage events of dart_reduce_profiled.  While they are set, every kernel this thread launches
// stamps them with its own begin and end (the start/stop events of hipExtLaunchKernel: the
// times are the dispatch's, and no marker packet goes between the kernels, so a stage's
// elapsed time is what a kernel trace shows for it); the first kernel of a stage takes the
// start event, every kernel of the stage the stop event (the last one's time stays).
struct StageEvents {
  hipEvent_t start = nullptr, stop = nullptr;
};
thread_local StageEvents t_stage;

#define DART_LAUNCH(kernel, grid, block, shmem, st, ...)                                        \
  do {                                                                                          \
    if (t_stage.stop != nullptr) {                                                              \
      hipExtLaunchKernelGGL(kernel, grid, block, shmem, st, t_stage.start, t_stage.stop, 0,     \
                            __VA_ARGS__);                                                       \
      t_stage.start = nullptr;                                                                  \
    } else {                                                                                    \
      hipLaunchKernelGGL(kernel, grid, block, shmem, st, __VA_ARGS__);                          \
    }                                                                                           \
  } while (0)

// Fills the ragged offsets (no-op for dense batches) and points g at them.
dart_status launch_prepare(Plan& p, void* ws, hipStream_t st) {
  if (p.g.cu == nullptr) return DART_OK;
  int* cu_keep = at<int>(ws, p.o_cu_keep);
  int* tile_start = at<int>(ws, p.o_tile_start);
  // (only where the ordering kernel's B*P workgroups, one per compute unit, need several rounds)
  int* by_size = p.g.B <= kMaxBySize && (long)p.g.B * p.g.P > compute_units()
                     ? at<int>(ws, p.o_by_size) : nullptr;
  DART_LAUNCH(k_prepare, dim3(1), dim3(1024), 0, st, p.g, cu_keep, tile_start,
              at<int>(ws, p.o_status), by_size);
  DART_LAUNCH_CHECK();
  p.g.cu_keep = cu_keep;
  p.g.tile_start = tile_start;
  p.g.by_size = by_size;
  return DART_OK;
}

// keep_cached: the rows will be read again soon (they are the hidden states themselves).
dart_status launch_row_l1(const Plan& p, const void* C, int Dc, long ldc, float* l1,
                          bool keep_cached, hipStream_t st, double* l2sq = nullptr) {
  constexpr int ROWS = 1;  // one row per wave measured best (more, shorter-lived waves)
  const int rows = p.g.total_N;
  if (rows == 0) return DART_OK;
  const int blocks = (int)round_up8((rows + 4 * ROWS - 1) / (4 * ROWS));
  // The 256 MB memory-side cache serves the score kernel's second pass if this pass leaves
  // the rows there: measured 31 instead of 38 us on that kernel for 0.7 us more on this one
  // at 189 MB; at 264 MB this pass loses 7 us and that one gains 0.7; a loss for matrices
  // that cannot fit.
  // With spans the caller moves whole sequences afterwards, which sweeps that cache anyway:
  // measured slower with ordinary loads there.
  const bool keep = keep_cached && (double)rows * ldc * p.esz <= 224e6;
  double* const no_l2sq = nullptr;
#define DART_LAUNCH_L1(DT)                                                                       \
  do {                                                                                           \
    if (l2sq && p.g.span)                                                                        \
      DART_LAUNCH((k_row_l1<kBF16, ROWS, false, true, true>), dim3(blocks), dim3(256), 0,        \
                  st, C, Dc, ldc, rows, l1, p.g, l2sq);                                          \
    else if (l2sq && keep)                                                                       \
      DART_LAUNCH((k_row_l1<kBF16, ROWS, true, false, true>), dim3(blocks), dim3(256), 0,        \
                  st, C, Dc, ldc, rows, l1, p.g, l2sq);                                          \
    else if (l2sq)                                                                               \
      DART_LAUNCH((k_row_l1<kBF16, ROWS, false, false, true>), dim3(blocks), dim3(256),          \
                  0, st, C, Dc, ldc, rows, l1, p.g, l2sq);                                       \
    else if (p.g.span)                                                                           \
      DART_LAUNCH((k_row_l1<DT, ROWS, false, true>), dim3(blocks), dim3(256), 0, st, C,          \
                  Dc, ldc, rows, l1, p.g, no_l2sq);                                              \
    else if (keep)                                                                               \
      DART_LAUNCH((k_row_l1<DT, ROWS, true, false>), dim3(blocks), dim3(256), 0, st, C,          \
                  Dc, ldc, rows, l1, p.g, no_l2sq);                                              \
    else                                                                                         \
      DART_LAUNCH((k_row_l1<DT, ROWS, false, false>), dim3(blocks), dim3(256), 0, st, C,         \
                  Dc, ldc, rows, l1, p.g, no_l2sq);                                              \
  } while (0)
  if (p.g.dtype == kBF16) DART_LAUNCH_L1(kBF16); else DART_LAUNCH_L1(kF32);
#undef DART_LAUNCH_L1
  DART_LAUNCH_CHECK();
  return DART_OK;
}

// Values a thread of the selection kernels keeps in registers: 1024 threads times this many
// cover the longest sample (see k_select.hpp); instantiated for 1, 2, 3, 4, 6, 8, 10, 12, 16.
int values_per_thread(int max_n) {
  const int need = (max_n + 1023) / 1024;
  for (int per : {1, 2, 3, 4, 6, 8, 10, 12, 16})
    if (per >= need) return per;
  return 16;
}
#define DART_FOR_VALUES_PER_THREAD(per, LAUNCH)                                                  \
  switch (per) {                                                                                 \
    case 1: LAUNCH(1); break;                                                                    \
    case 2: LAUNCH(2); break;                                                                    \
    case 3: LAUNCH(3); break;                                                                    \
    case 4: LAUNCH(4); break;                                                                    \
    case 6: LAUNCH(6); break;                                                                    \
    case 8: LAUNCH(8); break;                                                                    \
    case 10: LAUNCH(10); break;                                                                  \
    case 12: LAUNCH(12); break;                                                                  \
    default: LAUNCH(16); break;                                                                  \
  }

// l1_rel_err < 0: the norms are the norm pass's own (its rounding bound applies); otherwise the
// caller's, good to that relative error.
dart_status launch_select_pivots(const Plan& p, const void* X, const void* C, int Dc, long ldc,
                                 const float* l1, int* piv, void* ws, hipStream_t st,
                                 double l1_rel_err = -1.0) {
  // (the caller's bound plus the rounding of the threshold arithmetic itself, so that a bound
  // of zero -- exact norms rounded to fp32 -- still holds every exact pivot)
  const float tau = (float)(l1_rel_err < 0 ? l1_rel_bound(p.g.dtype, Dc) : l1_rel_err + 1.2e-7);
  double* pl2 = at<double>(ws, p.o_pl2);
  double* scr = at<double>(ws, p.o_scr_f64);
  // 1024 threads: a 256-thread variant measured slower even for short samples
#define DART_LAUNCH_PIVOTS(PER)                                                                  \
  do {                                                                                           \
    if (p.g.dtype == kBF16)                                                                      \
      DART_LAUNCH((k_select_pivots<kBF16, 1024, PER>), dim3(p.g.B), dim3(1024), 0, st,           \
                  p.g, X, C, Dc, ldc, l1, piv, pl2, scr, tau);                                   \
    else                                                                                         \
      DART_LAUNCH((k_select_pivots<kF32, 1024, PER>), dim3(p.g.B), dim3(1024), 0, st,            \
                  p.g, X, C, Dc, ldc, l1, piv, pl2, scr, tau);                                   \
  } while (0)
  DART_FOR_VALUES_PER_THREAD(values_per_thread(p.g.max_N), DART_LAUNCH_PIVOTS);
#undef DART_LAUNCH_PIVOTS
  DART_LAUNCH_CHECK();
  return DART_OK;
}

// Norms of the pivots first..P-1; piv_mark (optional) receives the marks of the pivots from
// outside the samples.
dart_status launch_pivot_norms(const Plan& p, const void* X, const int* piv, int first,
                               int* piv_mark, void* ws, hipStream_t st) {
  double* pl2 = at<double>(ws, p.o_pl2);
  if (p.g.dtype == kBF16)
    DART_LAUNCH((k_pivot_norms<kBF16>), dim3(p.g.B), dim3(1024), 0, st, p.g, X, piv, first,
                pl2, piv_mark);
  else
    DART_LAUNCH((k_pivot_norms<kF32>), dim3(p.g.B), dim3(1024), 0, st, p.g, X, piv, first,
                pl2, piv_mark);
  DART_LAUNCH_CHECK();
  return DART_OK;
}

// The pivots of DART_PIVOT_RANDOM, drawn on the device (the first Pin entries of every sample).
// DART_RANDOM_DRAW_LIMIT=n in the environment lowers the rule's limit of 4096 draws per sample
// (0..4096; for the test of the fill that follows the last draw, which no input reaches).
dart_status launch_random_pivots(const Plan& p, int* piv, hipStream_t st) {
  if (p.g.Pin == 0) return DART_OK;
  int limit = kRandomDraws;
  if (const char* v = std::getenv("DART_RANDOM_DRAW_LIMIT")) {
    const int n = std::atoi(v);
    if (n < 0 || n > kRandomDraws) return DART_ERR_SHAPE;
    limit = n;
  }
  DART_LAUNCH(k_random_pivots, dim3(p.g.B), dim3(64), 0, st, p.g, p.seed, limit, piv);
  DART_LAUNCH_CHECK();
  return DART_OK;
}

// Leaves the pivot flag of dart_device_status defined for a DART_PIVOT_GIVEN descriptor: the
// list the entry point reads is validated, or the flag is cleared if it reads none.
dart_status launch_given_status(const Plan& p, const int* piv, void* ws, hipStream_t st) {
  if (p.g.mode != kGiven) return DART_OK;
  if (piv)
    DART_LAUNCH(k_check_pivots, dim3(1), dim3(1024), 0, st, p.g, piv,
                at<int>(ws, p.o_status));
  else
    DART_LAUNCH(k_clear_pivot_status, dim3(1), dim3(1), 0, st, at<int>(ws, p.o_status));
  DART_LAUNCH_CHECK();
  return DART_OK;
}

template <int NB, bool TAIL, bool XN>
dart_status launch_scores_ksplit_nb(const Plan& p, const void* X, const int* piv,
                                    const double* pl2, const double* l2sq, float* S,
                                    hipStream_t st) {
  const dim3 grid((unsigned)round_up8(p.tiles_bound)), block(64 * p.ks_waves);
#define DART_KS_LAUNCH(W, KS)                                                                   \
  if (p.ks_waves == W && p.ks_split == KS) {                                                    \
    if constexpr (ksplit_lds_bytes(NB, KS, W) <= kKsLdsLimit) {                                 \
      DART_LAUNCH((k_scores_ksplit<NB, KS, W, TAIL, XN>), grid, block, 0, st, p.g, X,           \
                  piv, pl2, l2sq, S);                                                           \
      DART_LAUNCH_CHECK();                                                                      \
      return DART_OK;                                                                           \
    }                                                                                           \
  }
  DART_KS_SHAPES(DART_KS_LAUNCH)
#undef DART_KS_LAUNCH
  return DART_ERR_SHAPE;
}

template <int NB>
dart_status launch_scores_ksplit_tx(const Plan& p, const void* X, const int* piv,
                                    const double* pl2, const double* l2sq, float* S,
                                    hipStream_t st) {
  const bool tail = p.g.D % kKsCH != 0;
  if (l2sq)
    return tail ? launch_scores_ksplit_nb<NB, true, true>(p, X, piv, pl2, l2sq, S, st)
                : launch_scores_ksplit_nb<NB, false, true>(p, X, piv, pl2, l2sq, S, st);
  return tail ? launch_scores_ksplit_nb<NB, true, false>(p, X, piv, pl2, l2sq, S, st)
              : launch_scores_ksplit_nb<NB, false, false>(p, X, piv, pl2, l2sq, S, st);
}

// l2sq: the squared token norms if this call's norm pass left them (else the score kernel
// takes them from its own Gram products).
dart_status launch_scores(const Plan& p, const void* X, const int* piv, float* S, void* ws,
                          hipStream_t st) {
  if (p.tiles_bound == 0) return DART_OK;
  const double* pl2 = at<double>(ws, p.o_pl2);
  const double* l2sq = p.norms_given ? at<double>(ws, p.o_l2) : nullptr;
  if (p.g.dtype == kF32) {
    // two rows per block while four would not give every compute unit two blocks
    if (p.g.total_N <= 4 * 2 * compute_units())
      DART_LAUNCH(k_scores_f32<2>, dim3(p.tiles_bound * (p.g.tile_rows / 2)), dim3(256), 0,
                  st, p.g, X, piv, S);
    else
      DART_LAUNCH(k_scores_f32<4>, dim3(p.tiles_bound * (p.g.tile_rows / 4)), dim3(256), 0,
                  st, p.g, X, piv, S);
    DART_LAUNCH_CHECK();
    return DART_OK;
  }
  switch (p.g.Ppad / 16) {
    case 1: return launch_scores_ksplit_tx<1>(p, X, piv, pl2, l2sq, S, st);
    case 2: return launch_scores_ksplit_tx<2>(p, X, piv, pl2, l2sq, S, st);
    case 3: return launch_scores_ksplit_tx<3>(p, X, piv, pl2, l2sq, S, st);
    default: return launch_scores_ksplit_tx<4>(p, X, piv, pl2, l2sq, S, st);
  }
}

dart_status launch_order(const Plan& p, const float* S, void* ws, hipStream_t st) {
  if (p.g.score_mode != 0) return DART_OK;  // the single-threshold rule orders nothing per pivot
  unsigned long long* lists = at<unsigned long long>(ws, p.o_lists);
  // 1024 threads: a 256-thread variant measured slower even for short samples
#define DART_LAUNCH_ORDER(PER)                                                                   \
  DART_LAUNCH((k_order_scores<1024, PER>), dim3(p.g.B * p.g.P), dim3(1024), 0, st, p.g, S,       \
              lists)
  // samples of at most 1024 tokens: 512 threads with two values each (measured on 576-token
  // samples: 8.9 against 9.6 us; pivot selection is slower that way, 3072-token samples too)
  if (p.g.max_N <= 1024)
    DART_LAUNCH((k_order_scores<512, 2>), dim3(p.g.B * p.g.P), dim3(512), 0, st, p.g, S,
                lists);
  else
    DART_FOR_VALUES_PER_THREAD(values_per_thread(p.g.max_N), DART_LAUNCH_ORDER);
#undef DART_LAUNCH_ORDER
  DART_LAUNCH_CHECK();
  return DART_OK;
}

// pivot_norms_ready: this call has left the pivots' fp64 squared norms in the workspace.
dart_status launch_retain(const Plan& p, const float* S, const int* piv, const void* X, int* keep,
                          int* cu_keep, void* ws, hipStream_t st, bool pivot_norms_ready) {
  const double* pl2 = pivot_norms_ready ? at<double>(ws, p.o_pl2) : nullptr;
  const float two_tau = (float)(2.0 * 1.01 * score_abs_bound(p.g.dtype, p.norms_given));
  const unsigned long long* lists = at<unsigned long long>(ws, p.o_lists);
  double* scr_f64 = at<double>(ws, p.o_scr_f64);
  if (p.g.score_mode != 0) {  // one threshold for all pivots: no stage lists
#define DART_LAUNCH_SINGLE(PER)                                                                  \
  do {                                                                                           \
    if (p.g.dtype == kBF16)                                                                      \
      DART_LAUNCH((k_keep_single<kBF16, PER>), dim3(p.g.B), dim3(1024), 0, st, p.g, S,           \
                  piv, X, keep, cu_keep, scr_f64, two_tau, p.g.score_mode);                      \
    else                                                                                         \
      DART_LAUNCH((k_keep_single<kF32, PER>), dim3(p.g.B), dim3(1024), 0, st, p.g, S,            \
                  piv, X, keep, cu_keep, scr_f64, two_tau, p.g.score_mode);                      \
  } while (0)
    {
      const int per = values_per_thread(p.g.max_N);
      if (per <= 4) DART_LAUNCH_SINGLE(4);
      else if (per <= 8) DART_LAUNCH_SINGLE(8);
      else if (per <= 12) DART_LAUNCH_SINGLE(12);
      else DART_LAUNCH_SINGLE(16);
    }
#undef DART_LAUNCH_SINGLE
    DART_LAUNCH_CHECK();
    return DART_OK;
  }
#define DART_LAUNCH_RETAIN(DT, PK)                                                               \
  DART_LAUNCH((k_retain<DT, PK>), dim3(p.g.B), dim3(kRetThreads), 0, st, p.g, S, lists,          \
              piv, X, keep, cu_keep, scr_f64, two_tau, pl2)
  if (p.g.dtype == kBF16) {
    if (p.retain_packed) DART_LAUNCH_RETAIN(kBF16, true); else DART_LAUNCH_RETAIN(kBF16, false);
  } else {
    if (p.retain_packed) DART_LAUNCH_RETAIN(kF32, true); else DART_LAUNCH_RETAIN(kF32, false);
  }
#undef DART_LAUNCH_RETAIN
  DART_LAUNCH_CHECK();
  return DART_OK;
}

dart_status launch_gather(const Plan& p, const void* X, const int64_t* pos, const int* keep,
                          void* Y, int64_t* pos_out, hipStream_t st) {
  if (p.keep_rows_bound == 0) return DART_OK;
  const int blocks = (int)round_up8((p.keep_rows_bound + 3) / 4);
  DART_LAUNCH(k_gather, dim3(blocks), dim3(256), 0, st, p.g, p.esz, X,
              reinterpret_cast<const long long*>(pos), keep, Y,
              reinterpret_cast<long long*>(pos_out));
  DART_LAUNCH_CHECK();
  return DART_OK;
}

// The whole step as one persistent kernel (after a one-workgroup set-up kernel).
dart_status launch_fused(Plan& p, const void* X, const int64_t* pos, void* Y, int64_t* pos_out,
                         int32_t* keep, int32_t* cu_keep, int* piv, float* S, void* ws,
                         hipStream_t st) {
  const int NB = p.g.Ppad / 16;
  const int score_rows = NB <= 2 ? FusedScoreCfg<1>::ROWS : FusedScoreCfg<3>::ROWS;
  int* sync = at<int>(ws, p.o_sync);
  int* nstart = at<int>(ws, p.o_nstart);
  int* sstart = at<int>(ws, p.o_sstart);
  int* gstart = at<int>(ws, p.o_gstart);
  DART_LAUNCH(k_fused_init, dim3(1), dim3(1024), 0, st, p.g, score_rows, Y ? 1 : 0, sync,
              nstart, sstart, gstart, cu_keep, at<int>(ws, p.o_status));
  DART_LAUNCH_CHECK();
  FusedArgs a;
  a.X = X;
  a.pos = reinterpret_cast<const long long*>(pos);
  a.Y = Y;
  a.pos_out = reinterpret_cast<long long*>(pos_out);
  a.keep = keep;
  a.piv = piv;
  a.S = S;
  a.l1 = at<float>(ws, p.o_l1);
  a.l2sq = at<double>(ws, p.o_l2);
  a.pl2 = at<double>(ws, p.o_pl2);
  a.lists = at<unsigned long long>(ws, p.o_lists);
  a.scr = at<double>(ws, p.o_scr_f64);
  a.sync = sync;
  a.norm_start = nstart;
  a.score_start = sstart;
  a.gather_start = gstart;
  a.status = at<int>(ws, p.o_status);
  a.tau_l1 = (float)l1_rel_bound(p.g.dtype, p.g.D);
  a.two_tau = (float)(2.0 * 1.01 * score_abs_bound(p.g.dtype, true));
  a.keep_cached = (double)p.g.total_N * p.g.ld * p.esz <= 224e6 ? 1 : 0;
  a.spin_limit = 1 << 20;
  const dim3 grid(compute_units()), block(kFuThreads);
  const bool tail = p.g.D % kKsCH != 0;
#define DART_LAUNCH_FUSED(NBV)                                                        \
  do {                                                                                \
    if (tail) DART_LAUNCH((k_fused<NBV, true>), grid, block, 0, st, p.g, a);          \
    else DART_LAUNCH((k_fused<NBV, false>), grid, block, 0, st, p.g, a);              \
  } while (0)
  switch (NB) {
    case 1: DART_LAUNCH_FUSED(1); break;
    case 2: DART_LAUNCH_FUSED(2); break;
    case 3: DART_LAUNCH_FUSED(3); break;
    default: DART_LAUNCH_FUSED(4); break;
  }
#undef DART_LAUNCH_FUSED
  DART_LAUNCH_CHECK();
  return DART_OK;
}

// DART_FUSED=1 in the environment sends dart_reduce through the one-launch kernel where it
// applies (a switch between two complete implementations of the same step; the kernel-per-step
// path is the default because it measured faster on every benchmark shape).
bool fused_enabled() {
  const char* v = std::getenv("DART_FUSED");
  return v && v[0] == '1';
}

#define DART_TRY(expr)                    \
  do {                                    \
    dart_status _s = (expr);              \
    if (_s != DART_OK) return _s;         \
  } while (0)

dart_status check_crit(const Plan& p, const void* X, const void*& crit, int32_t& crit_D,
                       int64_t& crit_ld) {
  if (!crit) {
    crit = X;
    crit_D = p.g.D;
    crit_ld = p.g.ld;
    return DART_OK;
  }
  if (crit_D <= 0 || crit_D > 65536 || crit_ld < crit_D || crit_ld > kMaxLd) return DART_ERR_SHAPE;
  if (misaligned16(crit) || (crit_ld * p.esz) % 16 != 0 || ((long)crit_D * p.esz) % 16 != 0)
    return DART_ERR_ALIGN;
  return DART_OK;
}

dart_status reduce_impl(const dart_desc* desc, const void* X, const void* crit, int32_t crit_D,
                        int64_t crit_ld, const int64_t* pos, void* Y, int64_t* pos_out,
                        int32_t* keep, int32_t* cu_keep, int32_t* piv_out, float* S_out, void* ws,
                        size_t ws_bytes, void* stream, void* const* events,
                        const float* l1_given = nullptr, double l1_rel_err = 0.0) {
  Plan p;
  DART_TRY(make_plan(desc, p));
  if (l1_given && (p.g.mode == kGiven || p.g.mode == kRandom)) return DART_ERR_DTYPE;
  if (l1_given && !(l1_rel_err >= 0.0 && l1_rel_err <= 0.1)) return DART_ERR_SHAPE;
  if (p.g.B == 0) return DART_OK;
  if (!X || !keep || (Y && (pos != nullptr) != (pos_out != nullptr))) return DART_ERR_NULL;
  if (p.g.mode == kGiven && !piv_out) return DART_ERR_NULL;
  if (misaligned16(X) || (Y && misaligned16(Y))) return DART_ERR_ALIGN;
  // pivots drawn at random: the library writes the list, then the step runs as with a
  // caller's list (no pass over a criterion, no check of a list that is valid by construction)
  const bool random = p.g.mode == kRandom;
  if (random) p.g.mode = kGiven;
  if (p.g.mode == kGiven) crit = nullptr;
  DART_TRY(check_crit(p, X, crit, crit_D, crit_ld));
  DART_TRY(check_ws(p, ws, ws_bytes));
  // (the norm pass reads the criterion, not X, or there is none: the caller brought the norms)
  if (crit != X || l1_given) DART_TRY(replan_first_read(p));
  hipStream_t st = static_cast<hipStream_t>(stream);
  // profiled calls: the kernels launched from here on belong to stage k
  struct StageGuard {
    ~StageGuard() { t_stage = StageEvents{}; }
  } stage_guard;
  auto stage = [&](int k) {
    if (events)
      t_stage = {static_cast<hipEvent_t>(events[2 * k]),
                 static_cast<hipEvent_t>(events[2 * k + 1])};
  };
  int* piv = piv_out ? piv_out : at<int>(ws, p.o_piv);
  float* S = S_out ? S_out : at<float>(ws, p.o_S);
  float* l1 = at<float>(ws, p.o_l1);
  // hidden states as their own criterion: the norm pass also leaves the squared token norms,
  // which saves the score pass its Gram products (measured: the extra arithmetic costs the
  // norm pass 1-3 % up to 264 MB and 5 % at 1.7 GB, where it runs at the memory's speed and
  // the gain of the score pass does not pay for it; the tighter error bound also saves the
  // retained-set kernel 10 % on near-duplicate video frames)
  p.norms_given = p.g.mode != kGiven && p.g.Pin > 0 && crit == X && p.g.dtype == kBF16 &&
                  !l1_given && (double)p.g.total_N * p.g.ld * p.esz <= 1e9;
  DART_TRY(launch_prepare(p, ws, st));
  stage(0);
  // (the one-launch path computes its own norms: not for profiled calls or the caller's norms)
  if (p.fusable && crit == X && events == nullptr && !l1_given && p.g.total_N > 0 &&
      fused_enabled())
    return launch_fused(p, X, pos, Y, pos_out, keep, cu_keep, piv, S, ws, st);
  if (p.g.mode == kGiven) {
    // the caller's pivots: check them, compute their norms; no pass over the criterion
    if (random) {
      DART_TRY(launch_random_pivots(p, piv, st));
    } else {
      DART_LAUNCH(k_check_pivots, dim3(1), dim3(1024), 0, st, p.g, piv,
                  at<int>(ws, p.o_status));
      DART_LAUNCH_CHECK();
    }
    stage(1);
    DART_TRY(launch_pivot_norms(p, X, piv, 0, piv, ws, st));
  } else {
    // pivots chosen among the tokens (none if all of them come from outside) ...
    if (p.g.Pin > 0 && !l1_given)
      DART_TRY(launch_row_l1(p, crit, crit_D, crit_ld, l1, crit == X, st,
                             p.norms_given ? at<double>(ws, p.o_l2) : nullptr));
    stage(1);
    if (p.g.Pin > 0)
      DART_TRY(launch_select_pivots(p, X, crit, crit_D, crit_ld, l1_given ? l1_given : l1, piv, ws,
                                    st, l1_given ? l1_rel_err : -1.0));
    // ... then the norms and marks of those from outside
    if (p.g.Pe > 0) DART_TRY(launch_pivot_norms(p, X, piv, p.g.Pin, piv, ws, st));
  }
  stage(2);
  DART_TRY(launch_scores(p, X, piv, S, ws, st));
  stage(3);
  DART_TRY(launch_order(p, S, ws, st));
  stage(4);
  DART_TRY(launch_retain(p, S, piv, X, keep, cu_keep, ws, st, true));
  stage(5);
  if (Y) DART_TRY(launch_gather(p, X, pos, keep, Y, pos_out, st));  // NULL: the caller compacts
  return DART_OK;
}

// Device address of `scratch` on the current GPU, resolved once per GPU with that GPU current.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

dart_status static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return DART_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr)
      return DART_ERR_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return DART_OK;
}

}  // namespace

extern "C" {

size_t dart_workspace_bytes(const dart_desc* desc) {
  Plan p;
  if (make_plan(desc, p) != DART_OK) return 0;
  return p.total;
}

dart_status dart_score_tile_shape(const dart_desc* desc, int32_t* waves, int32_t* split) {
  if (!waves || !split) return DART_ERR_NULL;
  Plan p;
  DART_TRY(make_plan(desc, p));
  *waves = p.ks_waves;
  *split = p.ks_split;
  return DART_OK;
}

dart_status dart_score_tile_shape_first_read(const dart_desc* desc, int32_t* waves,
                                             int32_t* split) {
  if (!waves || !split) return DART_ERR_NULL;
  Plan p;
  DART_TRY(make_plan(desc, p));
  DART_TRY(replan_first_read(p));
  *waves = p.ks_waves;
  *split = p.ks_split;
  return DART_OK;
}

dart_status dart_select_pivots(const dart_desc* desc, const void* X, const void* crit,
                               int32_t crit_D, int64_t crit_ld, int32_t* piv, float* l1_out,
                               void* ws, size_t ws_bytes, void* stream) {
  Plan p;
  DART_TRY(make_plan(desc, p));
  if (p.g.mode == kGiven) return DART_ERR_DTYPE;  // nothing to select
  if (p.g.B == 0) return DART_OK;
  if (!X || !piv) return DART_ERR_NULL;
  if (misaligned16(X)) return DART_ERR_ALIGN;
  if (p.g.mode == kRandom) crit = nullptr;
  DART_TRY(check_crit(p, X, crit, crit_D, crit_ld));
  DART_TRY(check_ws(p, ws, ws_bytes));
  hipStream_t st = static_cast<hipStream_t>(stream);
  float* l1 = l1_out ? l1_out : at<float>(ws, p.o_l1);
  DART_TRY(launch_prepare(p, ws, st));
  if (p.g.mode == kRandom) {  // no criterion is read and l1_out is left as it is
    DART_TRY(launch_random_pivots(p, piv, st));
  } else if (p.g.Pin > 0) {
    DART_TRY(launch_row_l1(p, crit, crit_D, crit_ld, l1, false, st));
    DART_TRY(launch_select_pivots(p, X, crit, crit_D, crit_ld, l1, piv, ws, st));
  }
  if (p.g.Pe > 0) DART_TRY(launch_pivot_norms(p, X, piv, p.g.Pin, piv, ws, st));
  return DART_OK;
}

dart_status dart_duplication_scores(const dart_desc* desc, const void* X, const int32_t* piv,
                                    float* S, void* ws, size_t ws_bytes, void* stream) {
  Plan p;
  DART_TRY(make_plan(desc, p));
  if (p.g.B == 0) return DART_OK;
  if (!X || !piv || !S) return DART_ERR_NULL;
  if (misaligned16(X)) return DART_ERR_ALIGN;
  DART_TRY(check_ws(p, ws, ws_bytes));
  DART_TRY(replan_first_read(p));
  hipStream_t st = static_cast<hipStream_t>(stream);
  DART_TRY(launch_prepare(p, ws, st));
  DART_TRY(launch_given_status(p, piv, ws, st));
  DART_TRY(launch_pivot_norms(p, X, piv, 0, nullptr, ws, st));
  return launch_scores(p, X, piv, S, ws, st);
}

dart_status dart_topk_keep(const dart_desc* desc, const float* S, const int32_t* piv,
                           const void* X, int32_t* keep, int32_t* cu_keep, void* ws,
                           size_t ws_bytes, void* stream) {
  Plan p;
  DART_TRY(make_plan(desc, p));
  if (p.g.B == 0) return DART_OK;
  if (!S || !piv || !keep) return DART_ERR_NULL;
  if (X && misaligned16(X)) return DART_ERR_ALIGN;
  DART_TRY(check_ws(p, ws, ws_bytes));
  hipStream_t st = static_cast<hipStream_t>(stream);
  DART_TRY(launch_prepare(p, ws, st));
  DART_TRY(launch_given_status(p, piv, ws, st));
  DART_TRY(launch_order(p, S, ws, st));
  return launch_retain(p, S, piv, X, keep, cu_keep, ws, st, false);
}

dart_status dart_gather_compact(const dart_desc* desc, const void* X, const int64_t* pos,
                                const int32_t* keep, void* Y, int64_t* pos_out, void* ws,
                                size_t ws_bytes, void* stream) {
  Plan p;
  DART_TRY(make_plan(desc, p));
  if (p.g.B == 0) return DART_OK;
  if (!X || !keep || !Y || (pos != nullptr) != (pos_out != nullptr)) return DART_ERR_NULL;
  if (misaligned16(X) || misaligned16(Y)) return DART_ERR_ALIGN;
  DART_TRY(check_ws(p, ws, ws_bytes));
  hipStream_t st = static_cast<hipStream_t>(stream);
  DART_TRY(launch_prepare(p, ws, st));
  DART_TRY(launch_given_status(p, nullptr, ws, st));
  return launch_gather(p, X, pos, keep, Y, pos_out, st);
}

dart_status dart_compact_sequences(const dart_desc* desc, const int32_t* seq_cu,
                                   const int32_t* keep, int32_t n_tensors,
                                   const dart_row_tensor* tensors, const int64_t* pos,
                                   int32_t pos_planes, int64_t pos_plane_stride, int64_t* pos_out,
                                   int64_t pos_out_plane_stride, int32_t* seq_cu_out,
                                   int32_t* row_map, void* ws, size_t ws_bytes, void* stream) {
  Plan p;
  DART_TRY(make_plan(desc, p));
  if (!desc->span_start) return DART_ERR_NULL;  // sequences exist only around spans
  if (n_tensors < 0 || pos_planes < 0) return DART_ERR_SHAPE;
  if (!seq_cu || !keep || !seq_cu_out || !row_map || (n_tensors > 0 && !tensors) ||
      (pos_planes > 0 && (!pos || !pos_out)))
    return DART_ERR_NULL;
  for (int i = 0; i < n_tensors; ++i) {
    const dart_row_tensor& t = tensors[i];
    if (!t.src || !t.dst) return DART_ERR_NULL;
    if (t.row_bytes <= 0 || t.src_ld_bytes < t.row_bytes || t.dst_ld_bytes < t.row_bytes)
      return DART_ERR_SHAPE;
    if (misaligned16(t.src) || misaligned16(t.dst) || t.row_bytes % 16 || t.src_ld_bytes % 16 ||
        t.dst_ld_bytes % 16)
      return DART_ERR_ALIGN;
  }
  if (pos_planes > 0 && (pos_plane_stride < p.g.x_rows || pos_out_plane_stride < 0))
    return DART_ERR_SHAPE;
  DART_TRY(check_ws(p, ws, ws_bytes));
  hipStream_t st = static_cast<hipStream_t>(stream);
  DART_TRY(launch_prepare(p, ws, st));
  DART_TRY(launch_given_status(p, nullptr, ws, st));
  // every sequence loses its pruned vision tokens; at most this many rows remain
  const long rows_bound = (long)p.g.x_rows - p.g.total_N + p.keep_rows_bound;
  DART_LAUNCH(k_seq_offsets, dim3(1), dim3(1024), 0, st, p.g, seq_cu, seq_cu_out,
              at<int>(ws, p.o_status));
  DART_LAUNCH_CHECK();
  if (p.g.B == 0 || rows_bound <= 0) return DART_OK;
  DART_LAUNCH(k_seq_row_map, dim3((unsigned)((rows_bound + 255) / 256)), dim3(256), 0, st,
              p.g, seq_cu, seq_cu_out, keep, row_map);
  DART_LAUNCH_CHECK();
  const int* n_rows = seq_cu_out + p.g.B;
  for (int i0 = 0; i0 < n_tensors; i0 += kSeqOps) {
    SeqOps ops;
    const int cnt = n_tensors - i0 < kSeqOps ? n_tensors - i0 : kSeqOps;
    for (int i = 0; i < kSeqOps; ++i) {
      const dart_row_tensor& t = tensors[i0 + (i < cnt ? i : 0)];
      ops.src[i] = static_cast<const unsigned char*>(t.src);
      ops.dst[i] = static_cast<unsigned char*>(t.dst);
      ops.row_bytes[i] = t.row_bytes;
      ops.src_ld[i] = t.src_ld_bytes;
      ops.dst_ld[i] = t.dst_ld_bytes;
    }
    DART_LAUNCH(k_gather_rows, dim3((unsigned)round_up8((rows_bound + 3) / 4), cnt), dim3(256), 0,
                st, ops, n_rows, row_map);
    DART_LAUNCH_CHECK();
  }
  if (pos_planes > 0) {
    DART_LAUNCH(k_gather_pos, dim3((unsigned)((rows_bound + 255) / 256), pos_planes),
                dim3(256), 0, st, n_rows, row_map,
                reinterpret_cast<const long long*>(pos), (long)pos_plane_stride,
                reinterpret_cast<long long*>(pos_out), (long)pos_out_plane_stride);
    DART_LAUNCH_CHECK();
  }
  return DART_OK;
}

dart_status dart_reduce(const dart_desc* desc, const void* X, const void* crit, int32_t crit_D,
                        int64_t crit_ld, const int64_t* pos, void* Y, int64_t* pos_out,
                        int32_t* keep, int32_t* cu_keep, int32_t* piv_out, float* S_out, void* ws,
                        size_t ws_bytes, void* stream) {
  return reduce_impl(desc, X, crit, crit_D, crit_ld, pos, Y, pos_out, keep, cu_keep, piv_out,
                     S_out, ws, ws_bytes, stream, nullptr);
}

dart_status dart_reduce_profiled(const dart_desc* desc, const void* X, const void* crit,
                                 int32_t crit_D, int64_t crit_ld, const int64_t* pos, void* Y,
                                 int64_t* pos_out, int32_t* keep, int32_t* cu_keep,
                                 int32_t* piv_out, float* S_out, void* ws, size_t ws_bytes,
                                 void* stream, void* const* events) {
  if (!events) return DART_ERR_NULL;
  for (int k = 0; k < 12; ++k)
    if (!events[k]) return DART_ERR_NULL;
  return reduce_impl(desc, X, crit, crit_D, crit_ld, pos, Y, pos_out, keep, cu_keep, piv_out,
                     S_out, ws, ws_bytes, stream, events);
}

dart_status dart_reduce_with_norms(const dart_desc* desc, const void* X, const void* crit,
                                   int32_t crit_D, int64_t crit_ld, const float* l1,
                                   double l1_rel_err, const int64_t* pos, void* Y,
                                   int64_t* pos_out, int32_t* keep, int32_t* cu_keep,
                                   int32_t* piv_out, float* S_out, void* ws, size_t ws_bytes,
                                   void* stream) {
  if (!l1) return DART_ERR_NULL;
  return reduce_impl(desc, X, crit, crit_D, crit_ld, pos, Y, pos_out, keep, cu_keep, piv_out,
                     S_out, ws, ws_bytes, stream, nullptr, l1, l1_rel_err);
}

size_t dart_static_scratch_bytes(void) { return kStaticScratchBytes; }

dart_status dart_reduce_static(const dart_desc* desc, const void* X, const void* crit,
                               int32_t crit_D, int64_t crit_ld, const int64_t* pos, void* Y,
                               int64_t* pos_out, int32_t* keep, int32_t* cu_keep,
                               int32_t* piv_out, float* S_out, void* stream) {
  Plan p;
  DART_TRY(make_plan(desc, p));
  if (p.total > kStaticScratchBytes) return DART_ERR_STATIC_LIMIT;
  void* ws = nullptr;
  DART_TRY(static_scratch(&ws));
  return reduce_impl(desc, X, crit, crit_D, crit_ld, pos, Y, pos_out, keep, cu_keep, piv_out,
                     S_out, ws, kStaticScratchBytes, stream, nullptr);
}

dart_status dart_device_status_static(const dart_desc* desc, void* stream) {
  void* ws = nullptr;
  DART_TRY(static_scratch(&ws));
  return dart_device_status(desc, ws, stream);
}

dart_status dart_device_status(const dart_desc* desc, const void* ws, void* stream) {
  Plan p;
  DART_TRY(make_plan(desc, p));
  if (!ws) return DART_ERR_WORKSPACE;
  if (p.g.B == 0 || (p.g.cu == nullptr && p.g.mode != kGiven && !p.fusable)) return DART_OK;
  // [0] ragged offsets / budgets / spans, [1] given pivots, [2] sequences around the spans,
  // [3] the one-launch path gave up a bounded wait (its outputs are then unspecified)
  int flag[4] = {0, 0, 0, 0};
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (hipMemcpyAsync(flag, static_cast<const unsigned char*>(ws) + p.o_status, sizeof(flag),
                     hipMemcpyDeviceToHost, st) != hipSuccess)
    return DART_ERR_HIP;
  if (hipStreamSynchronize(st) != hipSuccess) return DART_ERR_HIP;
  if (p.g.cu == nullptr) flag[0] = 0;
  if (p.g.mode != kGiven) flag[1] = 0;
  if (p.g.span == nullptr) flag[2] = 0;
  flag[3] = (p.fusable && flag[3] == kFuAborted) ? 1 : 0;
  return (flag[0] | flag[1] | flag[2] | flag[3]) ? DART_ERR_DEVICE : DART_OK;
}

dart_status dart_probe_mfma_dot32(const void* A, const void* B, float* out, int32_t tiles,
                                  void* stream) {
  if (tiles < 0) return DART_ERR_SHAPE;
  if (tiles == 0) return DART_OK;
  if (!A || !B || !out) return DART_ERR_NULL;
  if (misaligned16(A) || misaligned16(B) || misaligned16(out)) return DART_ERR_ALIGN;
  DART_LAUNCH(k_probe_mfma_dot32, dim3(tiles), dim3(64), 0, static_cast<hipStream_t>(stream),
              static_cast<const unsigned char*>(A), static_cast<const unsigned char*>(B),
              out);
  DART_LAUNCH_CHECK();
  return DART_OK;
}

double dart_score_tolerance(int32_t dtype) {
  return score_abs_bound(dtype == DART_BF16 ? kBF16 : kF32);
}

const char* dart_strerror(dart_status status) {
  switch (status) {
    case DART_OK: return "ok";
    case DART_ERR_NULL: return "a required pointer is NULL";
    case DART_ERR_SHAPE: return "a size or stride is out of range";
    case DART_ERR_BUDGET: return "the keep budget violates P <= K <= N";
    case DART_ERR_DTYPE: return "unknown dtype or pivot mode";
    case DART_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case DART_ERR_ALIGN: return "row starts are not 16-byte aligned";
    case DART_ERR_HIP: return "a HIP call or kernel launch failed";
    case DART_ERR_STATIC_LIMIT:
      return "the problem needs more scratch than the built-in buffer of dart_reduce_static "
             "holds (dart_static_scratch_bytes); use dart_reduce with a workspace";
    case DART_ERR_DEVICE:
      return "a ragged sample violated the size or budget limits, a span or sequence is invalid, "
             "or a given pivot list is invalid";
  }
  return "unknown status";
}

}  // extern "C"

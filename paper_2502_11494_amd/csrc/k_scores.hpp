// Duplication scores of Definition 2 / Eq. (7): the cosine between every pivot
// and every token of its sample.
//
// bf16 hidden states: the tokens x pivots x D contraction runs on the matrix
// cores (v_mfma_f32_16x16x32_bf16).  A workgroup of 4 or 8 waves owns 64 or 128 token
// rows; a wave owns 16 of them and walks D in chunks of 128 or 256 elements:
//   HBM -> registers (two or four rows per load instruction, 256-512 B contiguous
//       each, two chunks ahead) -> LDS (row-padded) -> MFMA A fragments
//       (ds_read_b128, conflict-free).
// The pivot rows of the chunk are staged once per workgroup in LDS (double
// buffered) and serve as B fragments.  Feeding the token fragment as both
// operands yields the tile's Gram matrix, whose diagonal is |x_j|^2, at no extra
// memory traffic.  Every MFMA starts from a zero accumulator and its 32-term sums
// are added up in fp64 on the vector ALU.  bf16 x bf16 products are exact in fp32,
// so the only rounding is inside the matrix core's 32-term sum: see
// score_abs_bound().
//
// fp32 hidden states: plain fp64 arithmetic on the vector ALU (products of two
// floats are exact in fp64).
#pragma once
#include "common.hpp"

namespace dart {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Absolute bound on |stored fp32 score - exact cosine|.
// bf16: one MFMA returns the sum of 32 exact products with an error of at most
// kMfmaUlps * 2^-24 times the sum of their magnitudes.  The matrix core's internal
// rounding is not documented; measured over millions of random, wide-range and
// cancelling inputs the worst case is 6 * 2^-24, and 16 is assumed here.  The
// partial sums are added in fp64, so the dot product errs by at most
// 16 * 2^-24 * sum|p_d x_d| <= 16 * 2^-24 |p||x|.  The token norm comes from the
// same kind of sum and enters through a square root (half the relative error).
// Two more units for rounding the quotient to fp32 and the fp64 steps.
// fp32 inputs: all fp64, only the final rounding to fp32 counts.
// norms_given: the token norms come from k_row_l1 (relative error 3.5 * 2^-24 on the square,
// half of it on the norm; 2 units are counted) instead of the Gram diagonal.
constexpr double kMfmaUlps = 16.0;
inline double score_abs_bound(int dtype, bool norms_given = false) {
  const double u = 5.9604644775390625e-08;  // 2^-24
  if (dtype != kBF16) return 4.0 * u;
  return (norms_given ? kMfmaUlps + 2.0 + 2.0 : kMfmaUlps * 1.5 + 2.0) * u;
}

// LDS of one workgroup: CH = elements of D per chunk; rows are padded by 16 bytes
// so that the 16-row x 64-byte fragment reads hit distinct banks.
template <int NB, int CH, int WAVES>
struct ScoreShared {
  static constexpr int kRowB = CH * 2 + 16;
  unsigned char a[WAVES * 16 * kRowB];   // per-wave token chunk
  unsigned char p[2 * NB * 16 * kRowB];  // pivot chunk, double buffered
  const unsigned char* pivptr[NB * 16];  // pivot rows (nullptr: padding slot)
};

// Tile -> (sample, tile inside the sample).  Returns false for surplus blocks.
__device__ __forceinline__ bool locate_tile(const Geo& g, int tile, int& b, int& tl) {
  if (g.cu == nullptr) {
    int tps = (g.N + g.tile_rows - 1) / g.tile_rows;
    b = tile / tps;
    tl = tile - b * tps;
    return b < g.B;
  }
  if (tile >= g.tile_start[g.B]) return false;
  int lo = 0, hi = g.B;  // largest b with tile_start[b] <= tile
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (g.tile_start[mid] <= tile) lo = mid; else hi = mid;
  }
  b = lo;
  tl = tile - g.tile_start[lo];
  return true;
}

// Scores of one wave's 16 rows from the accumulated dot products and Gram diagonal.
// Output tile: lane holds column (lane&15) and rows 4*(lane>>4)..+3 of each 16x16 block.
// With tokens as the A operand, rows are tokens and columns are pivots (Gram: columns are
// tokens too, so |x_m|^2 sits in lane (m/4)*16+m, slot m%4).
// COH: pl2 and l2sq were written, and S will be read, by other workgroups of this launch.
template <int NB, bool COH = false>
__device__ __forceinline__ void store_scores(const Geo& g, const Sample& sm, int b, int j0,
                                             int lane, const double (&acc64)[NB][4],
                                             const double (&gram64)[4], const double* pl2,
                                             float* S, const double* l2sq) {
  const int n = sm.n, P = g.P;
  const int g4 = lane >> 4;
  double xn[4];
  if (l2sq != nullptr) {  // squared token norms from the norm pass (packed rows)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int j = j0 + g4 * 4 + r;
      xn[r] = sqrt(ld_dev<COH>(&l2sq[sm.row0 + (j < n ? j : n - 1)]));
    }
  } else {
#pragma unroll
    for (int r = 0; r < 4; ++r) xn[r] = sqrt(__shfl(gram64[r], g4 * 16 + g4 * 4 + r, kWave));
  }
  float* Sb = S + (long)P * sm.row0;
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int i = nb * 16 + (lane & 15);
    if (i < P) {
      const double pn = sqrt(ld_dev<COH>(&pl2[b * g.Ppad + i]));
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int j = j0 + g4 * 4 + r;
        if (j < n) {
          const double den = pn * xn[r];
          const double s = den > 0.0 ? acc64[nb][r] / den : 0.0;
          st_dev<COH>(&Sb[(long)i * n + j], (float)s + 0.0f);
        }
      }
    }
  }
}

// grid: number of tiles of g.tile_rows = 16*WAVES rows (dense: B*ceil(N/tile_rows);
// ragged: an upper bound): a workgroup of WAVES waves owns one tile, a wave 16 rows.
// NB = Ppad/16 pivot column blocks; CH = elements of D per chunk (128 or 256);
// TAIL = D is not a multiple of CH (then the last chunk's missing pieces are zeroed).
// DEPTH chunks per wave are in flight in registers: the token pieces (the only HBM
// traffic) and, requested just before them, the chunk's pivot pieces.  All loads are
// unconditional straight-line code, so the compiler's wait counts let the prefetched
// chunks stay in flight.
// SPLIT > 1 (small batches, which cannot fill the chip with one wave per 16 rows): SPLIT
// workgroups share a tile, each takes a contiguous run of the chunks and leaves its partial
// sums in `part` ([tile][slice][wave][lane][NB*4 + 4] doubles); k_scores_finish adds them in
// slice order and stores the scores.  grid: tiles * SPLIT.
// XN: the squared token norms are given (l2sq, from the norm pass): the Gram products and
// their accumulation are left out.
template <int NB, int CH, bool TAIL, int WAVES, int DEPTH, int SPLIT = 1, bool XN = false>
__global__ __launch_bounds__(WAVES * 64) void k_scores_bf16(Geo g, const void* __restrict__ X,
                                                     const int* __restrict__ piv,
                                                     const double* __restrict__ pl2,
                                                     float* __restrict__ S,
                                                     double* __restrict__ part = nullptr,
                                                     const double* __restrict__ l2sq = nullptr) {
  constexpr int kRowB = CH * 2 + 16;   // LDS row stride, bytes
  constexpr int PC = CH / 8;           // 16-byte pieces per row per chunk
  constexpr int RPI = kWave / PC;      // rows covered by one load instruction
  constexpr int LA = 16 / RPI;         // token loads per lane per chunk
  constexpr int THREADS = WAVES * 64;
  constexpr int LP = NB * 16 * PC / THREADS;  // pivot loads per thread per chunk
  constexpr int KS = CH / 32;          // MFMA k-steps per chunk
  __shared__ __align__(16) ScoreShared<NB, CH, WAVES> sh;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int b, tl;
  // (whole-row tiles: a die per contiguous eighth of the tiles; the grid is a multiple of 8)
  const int tile = SPLIT == 1 ? (int)xcd_contiguous(blockIdx.x, gridDim.x) : blockIdx.x / SPLIT;
  const int slice = SPLIT == 1 ? 0 : blockIdx.x - tile * SPLIT;
  if (!locate_tile(g, tile, b, tl)) return;
  const Sample sm = sample_of(g, b);
  if (sm.k == 0) return;
  const int n = sm.n, P = g.P;
  const int block_row0 = tl * (16 * WAVES);
  if (block_row0 >= n) return;
  if (tid < NB * 16) sh.pivptr[tid] = tid < P ? pivot_row(g, X, 2, sm, b, tid, piv) : nullptr;
  __syncthreads();

  const long rowbytes = g.ld * 2;
  const unsigned char* Xb = static_cast<const unsigned char*>(X) + (long)sm.xrow * rowbytes;
  const int pieces = g.D / 8;  // 16-byte pieces per row
  const int chunks_all = (g.D + CH - 1) / CH;
  // this workgroup's chunks [c_first, nchunks)
  const int c_first = SPLIT == 1 ? 0 : slice * chunks_all / SPLIT;
  const int nchunks = SPLIT == 1 ? chunks_all : (slice + 1) * chunks_all / SPLIT;
  const int col16 = lane % PC, rowsub = lane / PC;
  const int j0 = block_row0 + wave * 16;
  const u32x4 zero = {0u, 0u, 0u, 0u};

  // token loads: instruction t covers rows t*RPI .. t*RPI+RPI-1 of the wave's 16
  const unsigned char* aptr[LA];
#pragma unroll
  for (int t = 0; t < LA; ++t) {
    int r = j0 + t * RPI + rowsub;
    r = r < n ? r : n - 1;  // rows past the sample's end re-read its last row; never stored
    aptr[t] = Xb + (long)r * rowbytes + (TAIL ? 0 : col16 * 16);
  }
  // With TAIL the lane's column offset is added per chunk instead: a piece past the end of
  // the row must re-read the row's first 16 bytes, not bytes behind a row shorter than a chunk
  const int tail_col = TAIL ? col16 * 16 : 0;
  // pivot loads: piece id = tid + THREADS*k -> pivot row id/PC, piece id%PC (== col16);
  // padding slots read the sample's first row and are zeroed after the load
  const unsigned char* pptr[LP];
  bool preal[LP];
#pragma unroll
  for (int k = 0; k < LP; ++k) {
    const unsigned char* pr = sh.pivptr[(tid + THREADS * k) / PC];
    preal[k] = pr != nullptr;
    pptr[k] = (pr != nullptr ? pr : Xb) + (TAIL ? 0 : col16 * 16);
  }

  u32x4 ra[DEPTH][LA], rp[DEPTH][LP];
  // With TAIL, a piece past the end of the row re-reads the row's first piece; it is
  // replaced by zeros (as are the padding pivot slots) only when the registers go to LDS:
  // the load stays unconditional and nothing touches its result while it is in flight.
#define DART_LOAD_A(c, buf)                                                                    \
  {                                                                                            \
    const bool in_ = !TAIL || (c) * PC + col16 < pieces;                                       \
    const long off_ = in_ ? (long)(c) * (CH * 2) + tail_col : 0;                               \
    _Pragma("unroll") for (int t = 0; t < LA; ++t) ra[buf][t] =                                \
        __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(aptr[t] + off_));            \
  }
#define DART_STORE_A(c, buf)                                                                   \
  {                                                                                            \
    const bool in_ = !TAIL || (c) * PC + col16 < pieces;                                       \
    _Pragma("unroll") for (int t = 0; t < LA; ++t)                                             \
        *reinterpret_cast<u32x4*>(la + (t * RPI + rowsub) * kRowB + col16 * 16) =              \
            in_ ? ra[buf][t] : zero;                                                           \
  }
#define DART_LOAD_P(c, rbuf)                                                                   \
  {                                                                                            \
    const bool in_ = !TAIL || (c) * PC + col16 < pieces;                                       \
    const long off_ = in_ ? (long)(c) * (CH * 2) + tail_col : 0;                               \
    _Pragma("unroll") for (int k = 0; k < LP; ++k) rp[rbuf][k] =                               \
        *reinterpret_cast<const u32x4*>(pptr[k] + off_);                                       \
  }
#define DART_STORE_P(c, rbuf, buf)                                                             \
  {                                                                                            \
    const bool in_ = !TAIL || (c) * PC + col16 < pieces;                                       \
    _Pragma("unroll") for (int k = 0; k < LP; ++k)                                             \
        *reinterpret_cast<u32x4*>(sh.p + (buf) * (NB * 16 * kRowB) +                           \
                                  ((tid + THREADS * k) / PC) * kRowB + col16 * 16) =           \
            (in_ && preal[k]) ? rp[rbuf][k] : zero;                                            \
  }

  double acc64[NB][4], gram64[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    gram64[r] = 0.0;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc64[nb][r] = 0.0;
  }

  unsigned char* la = sh.a + wave * (16 * kRowB);
  const int frag_off = (lane & 15) * kRowB + (lane >> 4) * 16;
  const f32x4 fzero = {0.f, 0.f, 0.f, 0.f};

  // One chunk c (register slot buf = c % DEPTH): the wave's rows go registers -> its own
  // LDS region (in-order LDS ops within a wave make that safe); the freed slot takes the
  // pivot and token pieces of chunk c + DEPTH (vector loads return in order: each chunk's
  // pivot pieces are requested just before its token pieces, so waiting for the pivots of
  // chunk c + 1 leaves the younger chunks in flight); MFMAs on chunk c; then the pivot
  // registers of chunk c + 1 go to the other LDS pivot buffer.
#define DART_CHUNK(c, buf, nbuf, DO_P, DO_A)                                                   \
  {                                                                                            \
    DART_STORE_A(c, buf);                                                                      \
    if (DO_A) {                                                                                \
      DART_LOAD_P((c) + DEPTH, buf);                                                           \
      DART_LOAD_A((c) + DEPTH, buf);                                                           \
    }                                                                                          \
    __syncthreads(); /* pivot buffer c%2 is complete; buffer (c+1)%2 is no longer read */      \
    const unsigned char* lp = sh.p + ((c) & 1) * (NB * 16 * kRowB);                            \
    _Pragma("unroll") for (int s = 0; s < KS; ++s) {                                           \
      bf16x8 af = *reinterpret_cast<const bf16x8*>(la + frag_off + s * 64);                    \
      f32x4 gram = fzero;                                                                      \
      if (!XN) gram = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, af, fzero, 0, 0, 0);         \
      f32x4 acc[NB];                                                                           \
      _Pragma("unroll") for (int nb = 0; nb < NB; ++nb) {                                      \
        bf16x8 pf =                                                                            \
            *reinterpret_cast<const bf16x8*>(lp + nb * (16 * kRowB) + frag_off + s * 64);      \
        acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, pf, fzero, 0, 0, 0);             \
      }                                                                                        \
      _Pragma("unroll") for (int r = 0; r < 4; ++r) {                                          \
        if (!XN) gram64[r] += (double)gram[r];                                                 \
        _Pragma("unroll") for (int nb = 0; nb < NB; ++nb) acc64[nb][r] += (double)acc[nb][r];  \
      }                                                                                        \
    }                                                                                          \
    if (DO_P) DART_STORE_P((c) + 1, nbuf, ((c) + 1) & 1);                                               \
  }

  // DEPTH chunks (pivot and token pieces) are in flight per wave (register ring, static
  // indices)
  // (a row shorter than DEPTH chunks re-reads chunk 0 into the unused slots: the loads
  // stay unconditional, so every path into the loop has the same loads outstanding and
  // the compiler's wait counts at the loop head stay exact)
#pragma unroll
  for (int d = 0; d < DEPTH; ++d) {
    const int cc = c_first + d < nchunks ? c_first + d : c_first;
    DART_LOAD_P(cc, d);
    DART_LOAD_A(cc, d);
  }
  DART_STORE_P(c_first, 0, c_first & 1);
  int c = c_first;
  for (; c + 2 * DEPTH - 1 < nchunks; c += DEPTH) {  // steady state: every load is issued
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) DART_CHUNK(c + d, d, (d + 1) % DEPTH, true, true);
  }
#pragma unroll
  for (int r = 0; r < 2 * DEPTH - 1; ++r) {  // the last chunks: loads only while chunks remain
    if (c + r < nchunks)
      DART_CHUNK(c + r, r % DEPTH, (r + 1) % DEPTH, c + r + 1 < nchunks, c + r + DEPTH < nchunks);
  }
#undef DART_CHUNK
#undef DART_LOAD_A
#undef DART_STORE_A
#undef DART_LOAD_P
#undef DART_STORE_P

  if (SPLIT == 1) {
    store_scores<NB>(g, sm, b, j0, lane, acc64, gram64, pl2, S, XN ? l2sq : nullptr);
  } else {
    double* out = part + (((long)blockIdx.x * WAVES + wave) * kWave + lane) * (NB * 4 + 4);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      out[r] = gram64[r];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) out[4 + nb * 4 + r] = acc64[nb][r];
    }
  }
}

// Adds the SPLIT partial sums of every (tile, wave, lane) in slice order and stores the
// scores.  grid: tiles blocks of WAVES*64 (the same tiles as k_scores_bf16).
template <int NB, int WAVES, int SPLIT>
__global__ __launch_bounds__(WAVES * 64) void k_scores_finish(Geo g, const double* __restrict__ part,
                                                        const double* __restrict__ pl2,
                                                        float* __restrict__ S,
                                                        const double* __restrict__ l2sq) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int b, tl;
  if (!locate_tile(g, blockIdx.x, b, tl)) return;
  const Sample sm = sample_of(g, b);
  if (sm.k == 0) return;
  const int block_row0 = tl * (16 * WAVES);
  if (block_row0 >= sm.n) return;
  const int j0 = block_row0 + wave * 16;
  double acc64[NB][4], gram64[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    gram64[r] = 0.0;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc64[nb][r] = 0.0;
  }
#pragma unroll
  for (int sl = 0; sl < SPLIT; ++sl) {
    const double* in =
        part + ((((long)blockIdx.x * SPLIT + sl) * WAVES + wave) * kWave + lane) * (NB * 4 + 4);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      gram64[r] += in[r];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) acc64[nb][r] += in[4 + nb * 4 + r];
    }
  }
  store_scores<NB>(g, sm, b, j0, lane, acc64, gram64, pl2, S, l2sq);
}

// ---- score tiles with the D-chunks split inside the workgroup ---------------------------------
// The WAVES waves of a workgroup form KS groups that share the same 16*WAVES/KS token rows;
// group gk walks the D-chunks [gk*chunks/KS, (gk+1)*chunks/KS) with its own pivot chunks, and
// the groups' partial sums are added in group order at the end.  A tile of few rows (many tiles:
// every compute unit busy, a sample's scores done early) then still has WAVES waves' worth of
// loads in flight, at the pivot traffic of its row count.  The token norms come from the norm
// pass (l2sq); the arithmetic is that of k_scores_bf16 (exact bf16 products, 32-term sums on
// the matrix cores, fp64 accumulation).
constexpr int kKsCH = 128;  // elements of D per chunk

// LDS: token chunks of the waves, pivot chunks of the KS groups (double buffered), the
// pivots' row addresses.  Rows padded by 16 bytes as in ScoreShared.
template <int NB, int KS, int WAVES>
struct KSplitShared {
  static constexpr int kRowB = kKsCH * 2 + 16;
  unsigned char a[WAVES * 16 * kRowB];
  unsigned char p[KS * 2 * NB * 16 * kRowB];
  const unsigned char* pivptr[NB * 16];
};

// Tile tl (16*WAVES/KS rows) of sample b.  COH: piv, pl2 and l2sq were written, and S will be
// read, by other workgroups of this launch.
template <int NB, int KS, int WAVES, bool TAIL, bool COH>
__device__ __forceinline__ void score_tile_ksplit(const Geo& g, const Sample& sm, int b, int tl,
                                                  const void* X, const int* piv, const double* pl2,
                                                  const double* l2sq, float* S,
                                                  KSplitShared<NB, KS, WAVES>& sh) {
  constexpr int ROWS = 16 * WAVES / KS;
  constexpr int WG = WAVES / KS;        // waves per group
  constexpr int TG = WG * kWave;        // threads per group
  constexpr int kRowB = kKsCH * 2 + 16;
  constexpr int PC = kKsCH / 8;         // 16-byte pieces per row per chunk
  constexpr int RPI = kWave / PC;       // rows covered by one load instruction
  constexpr int LA = 16 / RPI;          // token loads per lane per chunk
  constexpr int PP = NB * 16 * PC;      // pivot pieces per chunk
  constexpr int LP = (PP + TG - 1) / TG;
  constexpr int KSTEPS = kKsCH / 32;    // matrix-core steps per chunk
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int gk = wave / WG, wi = wave - gk * WG, tg = tid - gk * TG;
  const int n = sm.n, P = g.P;
  if (tid < NB * 16) sh.pivptr[tid] = tid < P ? pivot_row<COH>(g, X, 2, sm, b, tid, piv) : nullptr;
  __syncthreads();

  const long rowbytes = g.ld * 2;
  const unsigned char* Xb = static_cast<const unsigned char*>(X) + (long)sm.xrow * rowbytes;
  const int pieces = g.D / 8;
  const int chunks_all = (g.D + kKsCH - 1) / kKsCH;
  const int c_first = gk * chunks_all / KS, c_end = (gk + 1) * chunks_all / KS;
  const int my_cnt = c_end - c_first;
  const int max_cnt = (chunks_all + KS - 1) / KS;  // every group runs this many rounds
  const int col16 = lane % PC, rowsub = lane / PC;
  const int j0 = tl * ROWS + wi * 16;
  const u32x4 zero = {0u, 0u, 0u, 0u};

  const unsigned char* aptr[LA];
#pragma unroll
  for (int t = 0; t < LA; ++t) {
    int r = j0 + t * RPI + rowsub;
    r = r < n ? r : n - 1;  // rows past the sample's end re-read its last row; never stored
    aptr[t] = Xb + (long)r * rowbytes + (TAIL ? 0 : col16 * 16);
  }
  const int tail_col = TAIL ? col16 * 16 : 0;
  const unsigned char* pptr[LP];
  bool preal[LP], pmine[LP];
#pragma unroll
  for (int k = 0; k < LP; ++k) {
    const int pid = tg + TG * k;
    pmine[k] = pid < PP;
    const unsigned char* pr = pmine[k] ? sh.pivptr[pid / PC] : nullptr;
    preal[k] = pr != nullptr;
    pptr[k] = (pr != nullptr ? pr : Xb) + (TAIL ? 0 : col16 * 16);
  }
  unsigned char* la = sh.a + wave * (16 * kRowB);
  unsigned char* lpg = sh.p + gk * (2 * NB * 16 * kRowB);
  const int frag_off = (lane & 15) * kRowB + (lane >> 4) * 16;
  const f32x4 fzero = {0.f, 0.f, 0.f, 0.f};

  double acc64[NB][4];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int r = 0; r < 4; ++r) acc64[nb][r] = 0.0;

  u32x4 ra[LA], rp[LP];
  // chunk c of this group (clamped to a chunk it owns, so that every load is unconditional
  // and in bounds; the surplus rounds of a group with fewer chunks compute nothing)
  auto load_chunk = [&](int c) {
    const bool in = !TAIL || c * PC + col16 < pieces;
    const long off = in ? (long)c * (kKsCH * 2) + tail_col : 0;
#pragma unroll
    for (int k = 0; k < LP; ++k) rp[k] = *reinterpret_cast<const u32x4*>(pptr[k] + off);
#pragma unroll
    for (int t = 0; t < LA; ++t)
      ra[t] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(aptr[t] + off));
  };
  auto store_p = [&](int c, int buf) {
    const bool in = !TAIL || c * PC + col16 < pieces;
#pragma unroll
    for (int k = 0; k < LP; ++k)
      if (pmine[k])
        *reinterpret_cast<u32x4*>(lpg + buf * (NB * 16 * kRowB) + ((tg + TG * k) / PC) * kRowB +
                                  col16 * 16) = (in && preal[k]) ? rp[k] : zero;
  };
  const int c_last = my_cnt > 0 ? c_end - 1 : 0;
  load_chunk(my_cnt > 0 ? c_first : 0);
  store_p(c_first, 0);
  for (int it = 0; it < max_cnt; ++it) {
    const int c = c_first + it;
    const bool live = it < my_cnt;
    {
      const bool in = !TAIL || c * PC + col16 < pieces;
#pragma unroll
      for (int t = 0; t < LA; ++t)
        *reinterpret_cast<u32x4*>(la + (t * RPI + rowsub) * kRowB + col16 * 16) =
            (in && live) ? ra[t] : zero;
    }
    const bool more = it + 1 < my_cnt;
    if (it + 1 < max_cnt) load_chunk(more ? c + 1 : c_last);
    __syncthreads();  // pivot buffer it%2 is complete; buffer (it+1)%2 is no longer read
    const unsigned char* lp = lpg + (it & 1) * (NB * 16 * kRowB);
    if (live) {
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s) {
        const bf16x8 af = *reinterpret_cast<const bf16x8*>(la + frag_off + s * 64);
        f32x4 acc[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          const bf16x8 pf =
              *reinterpret_cast<const bf16x8*>(lp + nb * (16 * kRowB) + frag_off + s * 64);
          acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, pf, fzero, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) acc64[nb][r] += (double)acc[nb][r];
      }
    }
    if (it + 1 < max_cnt) store_p(more ? c + 1 : c_last, (it + 1) & 1);
  }
  // the groups' partial sums: groups 1.. leave theirs in LDS (over the token chunks, which
  // nobody reads any more), group 0 adds them in group order and stores the scores
  __syncthreads();
  double* part = reinterpret_cast<double*>(sh.a);
  if (KS > 1 && gk > 0) {
    double* out = part + ((long)((gk - 1) * WG + wi) * kWave + lane) * (NB * 4);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int r = 0; r < 4; ++r) out[nb * 4 + r] = acc64[nb][r];
  }
  __syncthreads();
  if (gk == 0) {
#pragma unroll
    for (int o = 1; o < KS; ++o) {
      const double* in = part + ((long)((o - 1) * WG + wi) * kWave + lane) * (NB * 4);
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc64[nb][r] += in[nb * 4 + r];
    }
    const double gram_unused[4] = {0.0, 0.0, 0.0, 0.0};
    if (j0 < n) store_scores<NB, COH>(g, sm, b, j0, lane, acc64, gram_unused, pl2, S, l2sq);
  }
}

// grid: the tiles of 16*WAVES/KS rows (dense: B*ceil(N/rows); ragged: an upper bound), rounded
// up to a multiple of 8 blocks (a die per contiguous eighth of the tiles); WAVES*64 threads.
template <int NB, int KS, int WAVES, bool TAIL>
__global__ __launch_bounds__(WAVES * 64) void k_scores_ksplit(Geo g, const void* __restrict__ X,
                                                       const int* __restrict__ piv,
                                                       const double* __restrict__ pl2,
                                                       const double* __restrict__ l2sq,
                                                       float* __restrict__ S) {
  __shared__ __align__(16) KSplitShared<NB, KS, WAVES> sh;
  int b, tl;
  const int tile = (int)xcd_contiguous(blockIdx.x, gridDim.x);
  if (!locate_tile(g, tile, b, tl)) return;
  const Sample sm = sample_of(g, b);
  if (sm.k == 0 || tl * (16 * WAVES / KS) >= sm.n) return;
  score_tile_ksplit<NB, KS, WAVES, TAIL, false>(g, sm, b, tl, X, piv, pl2, l2sq, S, sh);
}

// fp32 hidden states, fp64 arithmetic on the vector ALU.  grid: tiles * (tile_rows / 4)
// blocks of 256: a block owns 4 consecutive token rows of one sample and 8 pivots at a
// time; its 4 waves split D (piece t of a row goes to wave (t / 64) % 4), so that small
// batches -- the only ones this path is meant for -- still spread over the chip and a wave's
// chain of dependent loads is a quarter as long.  The next pieces are requested before the
// current ones are used.  The 4 partial sums of a dot product are added in wave order, each
// wave's own sum is a fixed lane-strided order plus butterfly: a score depends only on the
// two rows' bytes.
constexpr int kF32Rows = 4, kF32Piv = 8;
__global__ __launch_bounds__(256) void k_scores_f32(Geo g, const void* __restrict__ X,
                                                    const int* __restrict__ piv,
                                                    float* __restrict__ S) {
  // per wave: dot[4][8], pp[8], xx[4]
  __shared__ double red[4][kF32Rows * kF32Piv + kF32Piv + kF32Rows];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int b, tl;
  const int parts = g.tile_rows / kF32Rows;
  const int tile = blockIdx.x / parts;
  if (!locate_tile(g, tile, b, tl)) return;
  const Sample sm = sample_of(g, b);
  if (sm.k == 0) return;
  const int n = sm.n, P = g.P;
  const int j0 = tl * g.tile_rows + (blockIdx.x - tile * parts) * kF32Rows;  // block-uniform
  if (j0 >= n) return;
  const float* Xb = static_cast<const float*>(X) + (long)sm.xrow * g.ld;
  const int pieces = g.D / 4;
  const f32x4v* xr[kF32Rows];
#pragma unroll
  for (int r = 0; r < kF32Rows; ++r) {
    const int j = j0 + r < n ? j0 + r : n - 1;  // rows past the end re-read the last; never stored
    xr[r] = reinterpret_cast<const f32x4v*>(Xb + (long)j * g.ld);
  }
  float* Sb = S + (long)P * sm.row0;
  const f32x4v fz = {0.f, 0.f, 0.f, 0.f};
  for (int i0 = 0; i0 < P; i0 += kF32Piv) {
    const f32x4v* pr[kF32Piv];
#pragma unroll
    for (int q = 0; q < kF32Piv; ++q) {
      const int i = i0 + q < P ? i0 + q : P - 1;
      pr[q] = reinterpret_cast<const f32x4v*>(pivot_row(g, X, 4, sm, b, i, piv));
    }
    double dot[kF32Rows][kF32Piv], xx[kF32Rows], pp[kF32Piv];
#pragma unroll
    for (int r = 0; r < kF32Rows; ++r) {
      xx[r] = 0.0;
#pragma unroll
      for (int q = 0; q < kF32Piv; ++q) dot[r][q] = 0.0;
    }
#pragma unroll
    for (int q = 0; q < kF32Piv; ++q) pp[q] = 0.0;
    f32x4v xv[kF32Rows], pv[kF32Piv], xn[kF32Rows], pn[kF32Piv];
    int t = tid;  // piece index: 256 apart per step
    auto fetch = [&](int tt, f32x4v (&xo)[kF32Rows], f32x4v (&po)[kF32Piv]) {
      const bool in = tt < pieces;
      const int ts = in ? tt : 0;  // a piece past the end re-reads piece 0 and counts as zero
#pragma unroll
      for (int r = 0; r < kF32Rows; ++r) {
        const f32x4v v = xr[r][ts];
        xo[r] = in ? v : fz;
      }
#pragma unroll
      for (int q = 0; q < kF32Piv; ++q) {
        const f32x4v v = pr[q][ts];
        po[q] = in ? v : fz;
      }
    };
    fetch(t, xv, pv);
    for (; t < pieces; t += 256) {
      fetch(t + 256, xn, pn);
#pragma unroll
      for (int q = 0; q < kF32Piv; ++q) {
        const double p0 = pv[q].x, p1 = pv[q].y, p2 = pv[q].z, p3 = pv[q].w;
        pp[q] = fma(p0, p0, pp[q]);
        pp[q] = fma(p1, p1, pp[q]);
        pp[q] = fma(p2, p2, pp[q]);
        pp[q] = fma(p3, p3, pp[q]);
#pragma unroll
        for (int r = 0; r < kF32Rows; ++r) {
          dot[r][q] = fma(p0, (double)xv[r].x, dot[r][q]);
          dot[r][q] = fma(p1, (double)xv[r].y, dot[r][q]);
          dot[r][q] = fma(p2, (double)xv[r].z, dot[r][q]);
          dot[r][q] = fma(p3, (double)xv[r].w, dot[r][q]);
        }
      }
#pragma unroll
      for (int r = 0; r < kF32Rows; ++r) {
        const double x0 = xv[r].x, x1 = xv[r].y, x2 = xv[r].z, x3 = xv[r].w;
        xx[r] = fma(x0, x0, xx[r]);
        xx[r] = fma(x1, x1, xx[r]);
        xx[r] = fma(x2, x2, xx[r]);
        xx[r] = fma(x3, x3, xx[r]);
      }
#pragma unroll
      for (int r = 0; r < kF32Rows; ++r) xv[r] = xn[r];
#pragma unroll
      for (int q = 0; q < kF32Piv; ++q) pv[q] = pn[q];
    }
    // the wave's sums, then the four waves' partials in wave order
#pragma unroll
    for (int r = 0; r < kF32Rows; ++r) {
#pragma unroll
      for (int q = 0; q < kF32Piv; ++q) {
        const double d = wave_sum(dot[r][q]);
        if (lane == 0) red[wave][r * kF32Piv + q] = d;
      }
      const double x2 = wave_sum(xx[r]);
      if (lane == 0) red[wave][kF32Rows * kF32Piv + kF32Piv + r] = x2;
    }
#pragma unroll
    for (int q = 0; q < kF32Piv; ++q) {
      const double p2 = wave_sum(pp[q]);
      if (lane == 0) red[wave][kF32Rows * kF32Piv + q] = p2;
    }
    __syncthreads();
    if (tid < kF32Rows * kF32Piv) {
      const int r = tid / kF32Piv, q = tid - r * kF32Piv;
      double d = 0.0, p2 = 0.0, x2 = 0.0;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        d += red[w][r * kF32Piv + q];
        p2 += red[w][kF32Rows * kF32Piv + q];
        x2 += red[w][kF32Rows * kF32Piv + kF32Piv + r];
      }
      const double den = sqrt(p2) * sqrt(x2);
      const double sc = den > 0.0 ? d / den : 0.0;
      if (i0 + q < P && j0 + r < n) Sb[(long)(i0 + q) * n + j0 + r] = (float)sc + 0.0f;
    }
    __syncthreads();  // red is reused by the next group of pivots
  }
}

}  // namespace dart

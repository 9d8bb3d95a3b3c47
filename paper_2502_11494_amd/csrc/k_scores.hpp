// Duplication scores of Definition 2 / Eq. (7): the cosine between every pivot
// and every token of its sample.
//
// bf16 hidden states: the tokens x pivots x D contraction runs on the matrix
// cores (v_mfma_f32_16x16x32_bf16).  A workgroup of W waves in KS groups owns
// 16*W/KS token rows; a wave owns 16 of them and walks its group's share of D in
// chunks of 128 elements:
//   HBM -> registers (four rows per load instruction, 256 B contiguous each, one
//       chunk ahead) -> LDS (row-padded) -> MFMA A fragments (ds_read_b128,
//       conflict-free).
// The pivot rows of the chunk are staged once per group in LDS (double buffered)
// and serve as B fragments.  The squared token norms come from the norm pass
// when it has read the same rows; otherwise the token fragment is fed as both
// operands, which yields the tile's Gram matrix, whose diagonal is |x_j|^2, at
// no extra memory traffic.  Every MFMA starts from a zero accumulator and its
// 32-term sums are added up in fp64 on the vector ALU.  bf16 x bf16 products are
// exact in fp32, so the only rounding is inside the matrix core's 32-term sum:
// see score_abs_bound().
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

// ---- bf16 score tiles ------------------------------------------------------------------------
// The WAVES waves of a workgroup form KS groups that share the same 16*WAVES/KS token rows;
// group gk walks the D-chunks [gk*chunks/KS, (gk+1)*chunks/KS) with its own pivot chunks, and
// the groups' partial sums are added in group order at the end.  A tile of few rows (many tiles:
// every compute unit busy, a sample's scores done early) then still has WAVES waves' worth of
// loads in flight, at the pivot traffic of its row count.  KS = 1 is the plain tile of 16*WAVES
// rows.
constexpr int kKsCH = 128;  // elements of D per chunk

// LDS: token chunks of the waves, pivot chunks of the KS groups (double buffered), the
// pivots' row addresses.  Rows are padded by 16 bytes so that the 16-row x 64-byte fragment
// reads hit distinct banks.  After the last chunk the groups' partial sums (kPartB bytes per
// wave of the groups 1..KS-1) overlay a and, for the widest shapes, the start of p.
template <int NB, int KS, int WAVES>
struct KSplitShared {
  static constexpr int kRowB = kKsCH * 2 + 16;
  static constexpr int kPartB = kWave * (NB * 4 + 4) * 8;
  unsigned char a[WAVES * 16 * kRowB];
  unsigned char p[KS * 2 * NB * 16 * kRowB];
  const unsigned char* pivptr[NB * 16];
  static_assert((WAVES - WAVES / KS) * kPartB <= WAVES * 16 * kRowB + KS * 2 * NB * 16 * kRowB,
                "the groups' partial sums must fit in the token and pivot chunks they overlay");
};

// LDS bytes of a shape (host side: which shapes fit a compute unit).
constexpr size_t ksplit_lds_bytes(int NB, int KS, int WAVES) {
  return (size_t)(WAVES * 16 + KS * 2 * NB * 16) * (kKsCH * 2 + 16) + (size_t)NB * 16 * 8;
}

// Tile tl (16*WAVES/KS rows) of sample b.
// TAIL: D is not a multiple of the chunk (the last chunk's missing pieces are zeroed).
// XN: the squared token norms are given (l2sq, from the norm pass): the Gram products and
// their accumulation are left out.
// COH: piv, pl2 and l2sq were written, and S will be read, by other workgroups of this launch.
template <int NB, int KS, int WAVES, bool TAIL, bool XN, bool COH>
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
  constexpr int PV = NB * 4 + (XN ? 0 : 4);  // partial sums per lane
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
  // With TAIL the lane's column offset is added per chunk instead: a piece past the end of
  // the row must re-read the row's first 16 bytes, not bytes behind a row shorter than a chunk
  const int tail_col = TAIL ? col16 * 16 : 0;
  // pivot pieces: piece id = tg + TG*k -> pivot row id/PC, piece id%PC (== col16); padding
  // slots read the sample's first row and are zeroed when the registers go to LDS
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

  double acc64[NB][4], gram64[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    gram64[r] = 0.0;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc64[nb][r] = 0.0;
  }

  u32x4 ra[LA], rp[LP];
  // chunk c of this group (clamped to a chunk it owns, so that every load is unconditional
  // and in bounds; the surplus rounds of a group with fewer chunks compute nothing).  The
  // chunk's pivot pieces are requested just before its token pieces (vector loads return in
  // order), and nothing touches a load's result while it is in flight.
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
      // the wave's rows go registers -> its own LDS region (LDS operations of one wave
      // complete in order, so the fragment reads below need no barrier of their own)
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
        f32x4 gram = fzero;
        if (!XN) gram = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, af, fzero, 0, 0, 0);
        f32x4 acc[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          const bf16x8 pf =
              *reinterpret_cast<const bf16x8*>(lp + nb * (16 * kRowB) + frag_off + s * 64);
          acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, pf, fzero, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          if (!XN) gram64[r] += (double)gram[r];
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) acc64[nb][r] += (double)acc[nb][r];
        }
      }
    }
    if (it + 1 < max_cnt) store_p(more ? c + 1 : c_last, (it + 1) & 1);
  }
  if (KS > 1) {
    // the groups' partial sums: groups 1.. leave theirs in LDS (over the chunks, which nobody
    // reads any more), group 0 adds them in group order
    __syncthreads();
    double* part = reinterpret_cast<double*>(sh.a);
    if (gk > 0) {
      double* out = part + ((long)((gk - 1) * WG + wi) * kWave + lane) * PV;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int r = 0; r < 4; ++r) out[nb * 4 + r] = acc64[nb][r];
      if (!XN) {
#pragma unroll
        for (int r = 0; r < 4; ++r) out[NB * 4 + r] = gram64[r];
      }
    }
    __syncthreads();
    if (gk == 0) {
#pragma unroll
      for (int o = 1; o < KS; ++o) {
        const double* in = part + ((long)((o - 1) * WG + wi) * kWave + lane) * PV;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int r = 0; r < 4; ++r) acc64[nb][r] += in[nb * 4 + r];
        if (!XN) {
#pragma unroll
          for (int r = 0; r < 4; ++r) gram64[r] += in[NB * 4 + r];
        }
      }
    }
  }
  if (gk == 0 && j0 < n)
    store_scores<NB, COH>(g, sm, b, j0, lane, acc64, gram64, pl2, S, XN ? l2sq : nullptr);
}

// grid: the tiles of g.tile_rows = 16*WAVES/KS rows (dense: B*ceil(N/rows); ragged: an upper
// bound), rounded up to a multiple of 8 blocks (a die per contiguous eighth of the tiles);
// WAVES*64 threads.  NB = Ppad/16 pivot column blocks.
template <int NB, int KS, int WAVES, bool TAIL, bool XN>
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
  score_tile_ksplit<NB, KS, WAVES, TAIL, XN, false>(g, sm, b, tl, X, piv, pl2, l2sq, S, sh);
}

// fp32 hidden states, fp64 arithmetic on the vector ALU.  grid: tiles * (tile_rows / ROWS)
// blocks of 256: a block owns ROWS (4 or 2) consecutive token rows of one sample and 8 pivots
// at a time; its 4 waves split D (piece t of a row goes to wave (t / 64) % 4), so that small
// batches -- the only ones this path is meant for -- still spread over the chip and a wave's
// chain of dependent loads is a quarter as long.  The next pieces are requested before the
// current ones are used.  The 4 partial sums of a dot product are added in wave order, each
// wave's own sum is a fixed lane-strided order plus butterfly: a score depends only on the
// two rows' bytes.  (Rows per block, measured on one 576-token image: 1, 2, 4, 8 rows give
// 19.4, 15.6, 16.3, 26.8 us by events; 2 rows where 4 would leave compute units idle.)
constexpr int kF32Piv = 8;
template <int kF32Rows>
__global__ __launch_bounds__(256) void k_scores_f32(Geo g, const void* __restrict__ X,
                                                    const int* __restrict__ piv,
                                                    float* __restrict__ S) {
  // per wave: dot[ROWS][8], pp[8], xx[ROWS]
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

// CPU oracle for the duplication-aware token reduction step of DART
// (arXiv 2502.11494, Section 3.3).
//
// THIS IS TEST INFRASTRUCTURE, not part of the product.  It is the yardstick the
// GPU library is compared with: plain loops, fp64 arithmetic, one sample at a
// time, nothing blocked, fused or reordered.  Only the test-suite, the smoke
// check and the benchmark's CPU-baseline leg may call it.  It shares no code
// with the GPU path.
//
// The method is a heuristic, so the oracle is the algorithm taken step by step:
//   1. criterion c_j = L1 norm of token j's criterion row        (Sec. 3.3 footnote)
//   2. pivots = the P tokens of largest c_j                       (Def. 1, Table 1 caption)
//   3. dup(p_i, x_j) = <p_i, x_j> / (|p_i| |x_j|)                 (Def. 2, Eq. 7)
//   4. R = pivots U_i R_i, with R_i the tokens of lowest dup(p_i, .) and the
//      per-pivot threshold set by the reduction ratio             (Eq. 9-10)
//   5. later layers see only the retained tokens, in order        (Appendix D)
// Readings where the paper is silent (all listed in the design notes):
//   * the budget K is split evenly over the pivots, q = floor((K-P)/P), the first
//     (K-P) mod P pivots take one more; pivots are processed in rank order and a
//     token retained earlier is no longer a candidate, so |R| = K exactly;
//   * ties are broken towards the lowest token index, everywhere;
//   * a zero-norm row scores 0 against everything;
//   * the retained tokens keep their original order and their position ids;
//   * pivots may also come from outside the scored tokens (text-token pivots): they are
//     scored against and have their stage, after the pivots chosen among the tokens, but
//     take no slot of the budget.
//
// Parity status: every step below is pinned by closed forms, invariants, a
// library cosine for P = 1 and brute-force enumeration on tiny inputs.  The
// pipeline as a whole is "parity unpinned" against the paper's own numbers: the
// paper prints no pivot list, score or retained set for any input.
//
// Threads: the two loops over tokens carry an OpenMP pragma; every token's
// arithmetic is still one sequential fp64 loop, so results do not depend on the
// thread count.

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

enum { kF32 = 0, kBF16 = 1 };
enum { kMaxL1 = 0, kMinL1 = 1 };

// Exact widening of one stored element to double.
inline double elem(const void* base, int dtype, int64_t idx) {
  if (dtype == kBF16) {
    uint32_t bits = static_cast<uint32_t>(static_cast<const uint16_t*>(base)[idx]) << 16;
    float f;
    std::memcpy(&f, &bits, sizeof f);
    return static_cast<double>(f);
  }
  return static_cast<double>(static_cast<const float*>(base)[idx]);
}

inline size_t elem_size(int dtype) { return dtype == kBF16 ? 2 : 4; }

}  // namespace

extern "C" {

// Number of threads the token loops use (0 = leave OpenMP's default). Returns the
// count that will be used.
int oracle_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
  return omp_get_max_threads();
#else
  (void)n;
  return 1;
#endif
}

// Step 1: c[j] = sum_d |C[j][d]|  (L1 norm; footnote of Sec. 3.3).
void oracle_l1_norms(const void* C, int dtype, int64_t N, int64_t D, int64_t ld, double* c) {
#pragma omp parallel for schedule(static)
  for (int64_t j = 0; j < N; ++j) {
    double s = 0.0;
    for (int64_t d = 0; d < D; ++d) s += std::fabs(elem(C, dtype, j * ld + d));
    c[j] = s;
  }
}

// Step 2: the P tokens of largest criterion, ordered by (c descending, index
// ascending); smallest first for mode kMinL1 (Table 8's "heart" rows).
void oracle_select_pivots(const double* c, int64_t N, int P, int mode, int32_t* piv) {
  std::vector<int32_t> order(N);
  for (int64_t j = 0; j < N; ++j) order[j] = static_cast<int32_t>(j);
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
    if (c[a] != c[b]) return mode == kMinL1 ? c[a] < c[b] : c[a] > c[b];
    return a < b;
  });
  for (int i = 0; i < P; ++i) piv[i] = order[i];
}

// Step 3: S[i*N + j] = <x_piv[i], x_j> / (|x_piv[i]| * |x_j|), 0 if a norm is 0 (Eq. 7).
void oracle_scores(const void* X, int dtype, int64_t N, int64_t D, int64_t ld,
                   const int32_t* piv, int P, double* S) {
  std::vector<double> norm(N);
#pragma omp parallel for schedule(static)
  for (int64_t j = 0; j < N; ++j) {
    double s = 0.0;
    for (int64_t d = 0; d < D; ++d) {
      double v = elem(X, dtype, j * ld + d);
      s += v * v;
    }
    norm[j] = std::sqrt(s);
  }
  for (int i = 0; i < P; ++i) {
    const int64_t p = piv[i];
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < N; ++j) {
      double dot = 0.0;
      for (int64_t d = 0; d < D; ++d) dot += elem(X, dtype, p * ld + d) * elem(X, dtype, j * ld + d);
      double den = norm[p] * norm[j];
      S[i * N + j] = den > 0.0 ? dot / den : 0.0;
    }
  }
}

// Step 3 for pivots that are not tokens of the scored set (Table 8 mixes 4 visual with 4
// text pivots; the section on the modalities of pivot tokens draws them from text alone):
// S[e*N + j] = <E[e], x_j> / (|E[e]| * |x_j|), 0 if a norm is 0 (Eq. 7).  E holds Pe rows
// of D elements, row stride lde.
void oracle_scores_rows(const void* X, int dtype, int64_t N, int64_t D, int64_t ld, const void* E,
                        int Pe, int64_t lde, double* S) {
  for (int e = 0; e < Pe; ++e) {
    double pp = 0.0;
    for (int64_t d = 0; d < D; ++d) {
      double v = elem(E, dtype, e * lde + d);
      pp += v * v;
    }
    const double pnorm = std::sqrt(pp);
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < N; ++j) {
      double dot = 0.0, xx = 0.0;
      for (int64_t d = 0; d < D; ++d) {
        double x = elem(X, dtype, j * ld + d);
        dot += elem(E, dtype, e * lde + d) * x;
        xx += x * x;
      }
      double den = pnorm * std::sqrt(xx);
      S[e * N + j] = den > 0.0 ? dot / den : 0.0;
    }
  }
}

// Step 4: the retained set (Eq. 9-10).  Returns 0, or -1 if P <= K <= N fails.
// keep[K]: retained indices ascending.
// Optional diagnostics, each of length P (pass NULL to skip): for stage i,
//   stage_last[i]  = token taken last (highest score taken), -1 if the stage took none
//   stage_next[i]  = best candidate NOT taken, -1 if none was left
//   stage_gap[i]   = S[i][stage_next] - S[i][stage_last]  (+inf if either is missing)
//
// piv[i] < 0 marks a pivot that is not one of the N tokens (a text-token pivot, Table 8):
// tokens are scored against it and it has its stage like any pivot, but it holds no slot
// of R, so R starts as the Pin <= P pivots inside the sample, Pin <= K <= N is required
// and the stages share K - Pin slots.
int oracle_retain(const double* S, int64_t N, const int32_t* piv, int P, int K, int32_t* keep,
                  int32_t* stage_last, int32_t* stage_next, double* stage_gap) {
  if (P < 1) return -1;
  int Pin = 0;
  for (int i = 0; i < P; ++i) Pin += piv[i] >= 0 ? 1 : 0;
  if (K < Pin || K > N) return -1;
  std::vector<char> in_R(N, 0);
  for (int i = 0; i < P; ++i)
    if (piv[i] >= 0) in_R[piv[i]] = 1;
  const int m = K - Pin, q = m / P, r = m % P;
  for (int i = 0; i < P; ++i) {
    const int quota = q + (i < r ? 1 : 0);
    std::vector<int32_t> cand;
    for (int64_t j = 0; j < N; ++j)
      if (!in_R[j]) cand.push_back(static_cast<int32_t>(j));
    const double* s = S + static_cast<int64_t>(i) * N;
    std::stable_sort(cand.begin(), cand.end(), [&](int32_t a, int32_t b) {
      if (s[a] != s[b]) return s[a] < s[b];
      return a < b;
    });
    for (int t = 0; t < quota; ++t) in_R[cand[t]] = 1;
    const int32_t last = quota > 0 ? cand[quota - 1] : -1;
    const int32_t next = quota < static_cast<int>(cand.size()) ? cand[quota] : -1;
    if (stage_last) stage_last[i] = last;
    if (stage_next) stage_next[i] = next;
    if (stage_gap) stage_gap[i] = (last >= 0 && next >= 0) ? s[next] - s[last] : INFINITY;
  }
  int n = 0;
  for (int64_t j = 0; j < N; ++j)
    if (in_R[j]) keep[n++] = static_cast<int32_t>(j);
  return n == K ? 0 : -2;
}

// Step 4 under ONE threshold common to all pivots (a second reading of Eq. 9-10: Section 1
// describes the retained tokens by a single similarity to the pivot set as a whole).  With
// the same epsilon for every pivot, Eq. (9)-(10) retain token j iff min_i dup(p_i, x_j)
// <= epsilon (agg = 1); agg = 2 aggregates with max_i instead (a token counts as a
// duplicate as soon as it duplicates any pivot).  The budget sets the threshold: R =
// pivots + the K-P non-pivot tokens of lowest aggregate, ties to the lowest index.
// Optional diagnostics (one decision): last = token taken last, next = best token not
// taken (-1 if none), gap = aggregate(next) - aggregate(last) (+inf if either is missing).
int oracle_retain_single(const double* S, int64_t N, const int32_t* piv, int P, int K, int agg,
                         int32_t* keep, int32_t* last, int32_t* next, double* gap) {
  if (P < 1 || (agg != 1 && agg != 2)) return -1;
  int Pin = 0;  // pivots inside the sample (piv[i] < 0: a pivot from outside, see oracle_retain)
  for (int i = 0; i < P; ++i) Pin += piv[i] >= 0 ? 1 : 0;
  if (K < Pin || K > N) return -1;
  std::vector<char> in_R(N, 0);
  for (int i = 0; i < P; ++i)
    if (piv[i] >= 0) in_R[piv[i]] = 1;
  std::vector<double> a(N);
  for (int64_t j = 0; j < N; ++j) {
    double v = S[j];
    for (int i = 1; i < P; ++i) {
      const double s = S[static_cast<int64_t>(i) * N + j];
      v = agg == 1 ? std::min(v, s) : std::max(v, s);
    }
    a[j] = v;
  }
  std::vector<int32_t> cand;
  for (int64_t j = 0; j < N; ++j)
    if (!in_R[j]) cand.push_back(static_cast<int32_t>(j));
  std::stable_sort(cand.begin(), cand.end(), [&](int32_t x, int32_t y) {
    if (a[x] != a[y]) return a[x] < a[y];
    return x < y;
  });
  const int m = K - Pin;
  for (int t = 0; t < m; ++t) in_R[cand[t]] = 1;
  const int32_t l = m > 0 ? cand[m - 1] : -1;
  const int32_t nx = m < static_cast<int>(cand.size()) ? cand[m] : -1;
  if (last) *last = l;
  if (next) *next = nx;
  if (gap) *gap = (l >= 0 && nx >= 0) ? a[nx] - a[l] : INFINITY;
  int n = 0;
  for (int64_t j = 0; j < N; ++j)
    if (in_R[j]) keep[n++] = static_cast<int32_t>(j);
  return n == K ? 0 : -2;
}

// Step 5: Y[r][:] = X[keep[r]][:] (bit copy, Y rows packed with stride D),
// pos_out[r] = pos[keep[r]] (skipped when pos is NULL).
void oracle_gather(const void* X, int dtype, int64_t D, int64_t ld, const int64_t* pos,
                   const int32_t* keep, int K, void* Y, int64_t* pos_out) {
  const size_t es = elem_size(dtype);
  for (int r = 0; r < K; ++r) {
    std::memcpy(static_cast<char*>(Y) + static_cast<size_t>(r) * D * es,
                static_cast<const char*>(X) + static_cast<size_t>(keep[r]) * ld * es, D * es);
    if (pos) pos_out[r] = pos[keep[r]];
  }
}

// Step 5 for a whole sequence (Appendix D: the layers after the step see the text tokens
// and the retained vision tokens; Table 2's KV-cache column shrinks the same way).  The
// sequence has T rows; its vision tokens are rows [vs, vs + N); keep[K] are the retained
// vision tokens (ascending, local to the span).  row_map[T - N + K] receives, for every row
// of the shortened sequence, the row of the original sequence it comes from: the text
// before the span, the retained vision tokens, the text after the span, all in order.
// Returns the new length, or -1 if the span does not fit the sequence.
int64_t oracle_sequence_map(int64_t T, int64_t vs, int64_t N, const int32_t* keep, int K,
                            int32_t* row_map) {
  if (vs < 0 || N < 0 || vs + N > T || K < 0 || K > N) return -1;
  int64_t r = 0;
  for (int64_t t = 0; t < vs; ++t) row_map[r++] = static_cast<int32_t>(t);
  for (int k = 0; k < K; ++k) row_map[r++] = static_cast<int32_t>(vs + keep[k]);
  for (int64_t t = vs + N; t < T; ++t) row_map[r++] = static_cast<int32_t>(t);
  return r;
}

// dst row r = src row row_map[r], bit copy of row_bytes bytes (hidden states, the key and
// value rows of the layers before the step, any per-token tensor).
void oracle_gather_rows(const void* src, int64_t row_bytes, int64_t src_ld_bytes,
                        const int32_t* row_map, int64_t n, void* dst, int64_t dst_ld_bytes) {
  for (int64_t r = 0; r < n; ++r)
    std::memcpy(static_cast<char*>(dst) + r * dst_ld_bytes,
                static_cast<const char*>(src) + static_cast<int64_t>(row_map[r]) * src_ld_bytes,
                static_cast<size_t>(row_bytes));
}

// One block of the Philox4x32 counter-based generator with 10 rounds (Salmon, Moraes, Dror,
// Shaw: "Parallel random numbers: as easy as 1, 2, 3", SC'11): a round replaces the counter
// words (c0, c1, c2, c3) by (hi(M1*c2) ^ c1 ^ k0, lo(M1*c2), hi(M0*c0) ^ c3 ^ k1, lo(M0*c0))
// and the key words grow by the Weyl constants between rounds.
void oracle_philox4x32_10(const uint32_t* counter, const uint32_t* key, uint32_t* out) {
  const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
  uint32_t c0 = counter[0], c1 = counter[1], c2 = counter[2], c3 = counter[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    if (round > 0) {
      k0 += 0x9E3779B9u;
      k1 += 0xBB67AE85u;
    }
    const uint64_t p0 = M0 * c0, p1 = M1 * c2;
    const uint32_t n0 = static_cast<uint32_t>(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = static_cast<uint32_t>(p0 >> 32) ^ c3 ^ k1;
    c1 = static_cast<uint32_t>(p1);
    c3 = static_cast<uint32_t>(p0);
    c0 = n0;
    c2 = n2;
  }
  out[0] = c0;
  out[1] = c1;
  out[2] = c2;
  out[3] = c3;
}

// Pivots drawn at random (the random rows of the pivot ablation, Sec. 4.3 / Table 8; the
// paper names no generator, so the draw is defined here): sample b draws tokens
// d_t = floor(w_t * N / 2^32), t = 0, 1, ..., where w_t is word t mod 4 of the Philox4x32-10
// block with counter (t div 4, b, 0, 0) and key (low, high half of seed); its pivots are the
// first P distinct draws, in the order they appear.  After 4096 draws (never reached in
// practice) the lowest unused tokens fill the list.  Returns the number of draws used.
int oracle_random_pivots_limited(uint64_t seed, int64_t b, int64_t N, int P, int max_draws,
                                 int32_t* piv);
int oracle_random_pivots(uint64_t seed, int64_t b, int64_t N, int P, int32_t* piv) {
  return oracle_random_pivots_limited(seed, b, N, P, 4096, piv);
}

// The same with the draw limit as an argument (the rule's own limit is 4096), so that the
// fill that follows the last draw can be exercised by a test.
int oracle_random_pivots_limited(uint64_t seed, int64_t b, int64_t N, int P, int max_draws,
                                 int32_t* piv) {
  const int kMaxDraws = max_draws;
  if (P < 0 || N < P || max_draws < 0) return -1;
  const uint32_t key[2] = {static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32)};
  std::vector<char> used(N, 0);
  int have = 0, t = 0;
  uint32_t words[4] = {0, 0, 0, 0};
  for (; t < kMaxDraws && have < P; ++t) {
    if (t % 4 == 0) {
      const uint32_t counter[4] = {static_cast<uint32_t>(t / 4), static_cast<uint32_t>(b), 0u, 0u};
      oracle_philox4x32_10(counter, key, words);
    }
    const int64_t d = static_cast<int64_t>((static_cast<uint64_t>(words[t % 4]) *
                                            static_cast<uint64_t>(N)) >> 32);
    if (!used[d]) {
      used[d] = 1;
      piv[have++] = static_cast<int32_t>(d);
    }
  }
  for (int64_t j = 0; j < N && have < P; ++j)
    if (!used[j]) {
      used[j] = 1;
      piv[have++] = static_cast<int32_t>(j);
    }
  return t;
}

// Steps 1-5 for one sample.  crit == NULL means the hidden-state rows are their
// own criterion.  Optional outputs may be NULL: c [N], S [P*N], Y, pos_out,
// piv_gap [P] (c[piv[i]] - c[next in rank], sign-corrected for kMinL1),
// stage_last/stage_next/stage_gap [P] as in oracle_retain.
int oracle_reduce(const void* X, int dtype, int64_t N, int64_t D, int64_t ld, const void* crit,
                  int64_t crit_D, int64_t crit_ld, const int64_t* pos, int P, int K, int mode,
                  int32_t* piv, int32_t* keep, double* c_out, double* S_out, void* Y,
                  int64_t* pos_out, double* piv_gap, int32_t* stage_last, int32_t* stage_next,
                  double* stage_gap) {
  if (P < 1 || K < P || K > N) return -1;
  std::vector<double> c(N);
  if (crit)
    oracle_l1_norms(crit, dtype, N, crit_D, crit_ld, c.data());
  else
    oracle_l1_norms(X, dtype, N, D, ld, c.data());
  if (c_out) std::memcpy(c_out, c.data(), sizeof(double) * N);
  // Rank P+1 tokens so that the margin behind the last pivot can be reported.
  const int P1 = static_cast<int>(std::min<int64_t>(N, P + 1));
  std::vector<int32_t> ranked(P1);
  oracle_select_pivots(c.data(), N, P1, mode, ranked.data());
  for (int i = 0; i < P; ++i) piv[i] = ranked[i];
  if (piv_gap)
    for (int i = 0; i < P; ++i)
      piv_gap[i] = i + 1 < P1 ? std::fabs(c[ranked[i]] - c[ranked[i + 1]]) : INFINITY;
  std::vector<double> S(static_cast<size_t>(P) * N);
  oracle_scores(X, dtype, N, D, ld, piv, P, S.data());
  if (S_out) std::memcpy(S_out, S.data(), sizeof(double) * S.size());
  int rc = oracle_retain(S.data(), N, piv, P, K, keep, stage_last, stage_next, stage_gap);
  if (rc != 0) return rc;
  if (Y) oracle_gather(X, dtype, D, ld, pos, keep, K, Y, pos_out);
  return 0;
}

}  // extern "C"

// AddressSanitizer / UndefinedBehaviorSanitizer run of the CPU oracle (test infrastructure,
// like the oracle itself).  Built together with dart_oracle.cpp by oracle.build_sanitized()
// with -fsanitize=address,undefined -fno-sanitize-recover=all and executed by the CPU test
// suite: every oracle function runs on exactly sized heap buffers over a set of shapes that
// covers both element types, padded row strides, single-token samples, keep-everything and
// pivots-only budgets, the remainder rule, pivots from outside the sample, pivots drawn at
// random and whole-sequence maps.  Any out-of-bounds access, use of uninitialised size arithmetic that overflows, or
// other undefined behaviour aborts the program; on success it prints "sanitize ok".
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

extern "C" {
int oracle_set_threads(int n);
void oracle_l1_norms(const void* C, int dtype, int64_t N, int64_t D, int64_t ld, double* c);
void oracle_select_pivots(const double* c, int64_t N, int P, int mode, int32_t* piv);
void oracle_scores(const void* X, int dtype, int64_t N, int64_t D, int64_t ld, const int32_t* piv,
                   int P, double* S);
void oracle_scores_rows(const void* X, int dtype, int64_t N, int64_t D, int64_t ld, const void* E,
                        int Pe, int64_t lde, double* S);
int oracle_retain(const double* S, int64_t N, const int32_t* piv, int P, int K, int32_t* keep,
                  int32_t* stage_last, int32_t* stage_next, double* stage_gap);
int oracle_retain_single(const double* S, int64_t N, const int32_t* piv, int P, int K, int agg,
                         int32_t* keep, int32_t* last, int32_t* next, double* gap);
void oracle_gather(const void* X, int dtype, int64_t D, int64_t ld, const int64_t* pos,
                   const int32_t* keep, int K, void* Y, int64_t* pos_out);
int64_t oracle_sequence_map(int64_t T, int64_t vs, int64_t N, const int32_t* keep, int K,
                            int32_t* row_map);
void oracle_gather_rows(const void* src, int64_t row_bytes, int64_t src_ld_bytes,
                        const int32_t* row_map, int64_t n, void* dst, int64_t dst_ld_bytes);
int oracle_reduce(const void* X, int dtype, int64_t N, int64_t D, int64_t ld, const void* crit,
                  int64_t crit_D, int64_t crit_ld, const int64_t* pos, int P, int K, int mode,
                  int32_t* piv, int32_t* keep, double* c_out, double* S_out, void* Y,
                  int64_t* pos_out, double* piv_gap, int32_t* stage_last, int32_t* stage_next,
                  double* stage_gap);
void oracle_philox4x32_10(const uint32_t* counter, const uint32_t* key, uint32_t* out);
int oracle_random_pivots(uint64_t seed, int64_t b, int64_t N, int P, int32_t* piv);
}

namespace {

uint64_t g_state = 0x9E3779B97F4A7C15ull;
uint32_t next_u32() {  // splitmix64, upper half
  uint64_t z = (g_state += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return static_cast<uint32_t>((z ^ (z >> 31)) >> 32);
}
float next_unit() { return (static_cast<float>(next_u32() >> 8) / 8388608.0f) - 1.0f; }

int failures = 0;
#define CHECK(cond)                                                          \
  do {                                                                       \
    if (!(cond)) {                                                           \
      std::fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond); \
      ++failures;                                                            \
    }                                                                        \
  } while (0)

// One whole step on a random sample; every buffer has exactly the size the interface states.
void one_case(int dtype, int N, int D, int pad, int P, int K, int mode, bool with_crit) {
  const int ld = D + pad, cD = 8, cld = 8 + pad;
  const size_t es = dtype == 1 ? 2 : 4;
  std::vector<unsigned char> X(static_cast<size_t>(N - 1) * ld * es + D * es);  // no pad after the last row
  std::vector<unsigned char> C(static_cast<size_t>(N - 1) * cld * es + cD * es);
  auto fill = [&](std::vector<unsigned char>& buf) {
    for (size_t i = 0; i + es <= buf.size(); i += es) {
      const float f = next_unit();
      if (dtype == 1) {
        uint32_t u;
        std::memcpy(&u, &f, 4);
        const uint16_t h = static_cast<uint16_t>(u >> 16);
        std::memcpy(&buf[i], &h, 2);
      } else {
        std::memcpy(&buf[i], &f, 4);
      }
    }
  };
  fill(X);
  fill(C);
  std::vector<int64_t> pos(N), pos_out(K);
  for (int j = 0; j < N; ++j) pos[j] = 1000 + j;
  std::vector<int32_t> piv(P), keep(K), last(P), nxt(P);
  std::vector<double> c(N), S(static_cast<size_t>(P) * N), pgap(P), sgap(P);
  std::vector<unsigned char> Y(static_cast<size_t>(K) * D * es);
  const int rc = oracle_reduce(X.data(), dtype, N, D, ld, with_crit ? C.data() : nullptr, cD, cld,
                               pos.data(), P, K, mode, piv.data(), keep.data(), c.data(), S.data(),
                               Y.data(), pos_out.data(), pgap.data(), last.data(), nxt.data(),
                               sgap.data());
  CHECK(rc == 0);
  for (int r = 1; r < K; ++r) CHECK(keep[r] > keep[r - 1]);
  for (int r = 0; r < K; ++r) CHECK(pos_out[r] == 1000 + keep[r]);
  // the single-threshold rule and the stage functions on the same scores
  for (int agg = 1; agg <= 2; ++agg) {
    int32_t l = 0, n2 = 0;
    double g = 0;
    CHECK(oracle_retain_single(S.data(), N, piv.data(), P, K, agg, keep.data(), &l, &n2, &g) == 0);
  }
  // pivots from outside: the last pivot becomes an outside row (a copy of token 0)
  if (P >= 2 && K >= P - 1) {
    std::vector<unsigned char> E(static_cast<size_t>(D) * es);
    std::memcpy(E.data(), X.data(), E.size());
    std::vector<double> S2(static_cast<size_t>(P) * N);
    oracle_scores(X.data(), dtype, N, D, ld, piv.data(), P - 1, S2.data());
    oracle_scores_rows(X.data(), dtype, N, D, ld, E.data(), 1, D, S2.data() + static_cast<size_t>(P - 1) * N);
    std::vector<int32_t> piv2(piv);
    piv2[P - 1] = -1;
    std::vector<int32_t> keep2(K);
    CHECK(oracle_retain(S2.data(), N, piv2.data(), P, K, keep2.data(), nullptr, nullptr, nullptr) == 0);
  }
  // whole-sequence map and row gather around the span
  const int before = 3, after = 2, T = before + N + after;
  std::vector<int32_t> map(T - N + K);
  CHECK(oracle_sequence_map(T, before, N, keep.data(), K, map.data()) == T - N + K);
  std::vector<unsigned char> src(static_cast<size_t>(T) * 16), dst(map.size() * 16);
  oracle_gather_rows(src.data(), 16, 16, map.data(), static_cast<int64_t>(map.size()), dst.data(), 16);
  CHECK(oracle_sequence_map(T, before + after + 1, N, keep.data(), K, map.data()) == -1);
}

}  // namespace

int main(int argc, char** argv) {
  if (argc > 1 && std::strcmp(argv[1], "plant") == 0) {
    // proof that the sanitizer is live: the oracle is handed a buffer one row too short and
    // must be stopped when it reads past it
    std::vector<float> X(3 * 4);
    std::vector<double> c(4);
    oracle_l1_norms(X.data(), 0, 4, 4, 4, c.data());
    std::puts("planted overrun went unnoticed");
    return 0;
  }
  oracle_set_threads(2);
  for (int dtype = 0; dtype <= 1; ++dtype) {
    one_case(dtype, 1, 8, 0, 1, 1, 0, false);       // a single token
    one_case(dtype, 37, 24, 8, 4, 4, 0, true);      // pivots only
    one_case(dtype, 37, 24, 8, 4, 37, 1, false);    // keep everything, min-norm pivots
    one_case(dtype, 64, 40, 0, 5, 23, 0, true);     // remainder rule: (23 - 5) mod 5 = 3
    one_case(dtype, 200, 16, 16, 16, 60, 0, false);
  }
  // rejected budgets return an error code and touch nothing
  double s1[4] = {0, 0, 0, 0};
  int32_t p1[1] = {0}, k1[4];
  CHECK(oracle_retain(s1, 4, p1, 1, 5, k1, nullptr, nullptr, nullptr) == -1);
  CHECK(oracle_retain(s1, 4, p1, 1, 0, k1, nullptr, nullptr, nullptr) == -1);
  CHECK(oracle_retain_single(s1, 4, p1, 1, 2, 3, k1, nullptr, nullptr, nullptr) == -1);
  // random pivots: exactly sized lists, every token drawn, the largest seed and sample index
  for (int n : {1, 2, 64, 1000}) {
    for (int P : {0, 1, n < 64 ? n : 64}) {
      std::vector<int32_t> piv(static_cast<size_t>(P));
      CHECK(oracle_random_pivots(~0ull, (1 << 20) - 1, n, P, piv.data()) >= P);
      for (int32_t j : piv) CHECK(j >= 0 && j < n);
    }
  }
  CHECK(oracle_random_pivots(1, 0, 3, 4, p1) == -1);
  if (failures) return 1;
  std::puts("sanitize ok");
  return 0;
}

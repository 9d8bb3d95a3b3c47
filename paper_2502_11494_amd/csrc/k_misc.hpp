// Small kernels around the main passes: per-sample offsets for ragged batches,
// pivot norms for the stand-alone score entry point, and the row gather that
// compacts the retained tokens (the shortened sequence of Appendix D).
#pragma once
#include "common.hpp"

namespace dart {

// Ragged batches only.  One block of 1024 threads: validates the offsets and every
// sample and writes the packed offsets cu_keep[B+1] (retained rows; a skipped
// sample keeps 0) and tile_start[B+1] (score tiles of g.tile_rows rows).  status[0] becomes
// 1 if a non-empty sample was rejected (its sizes or budget, or a span that leaves X), 2 if
// cu_seqlens itself is not a non-decreasing sequence from 0 to total_N (then every sample
// is skipped).
// by_size (optional, B <= kMaxBySize): the samples ordered from the longest to the shortest
// (ties in batch order).  The ordering kernel runs one workgroup per compute unit, a list's
// time grows with its sample's length, and workgroups start in id order: with the long
// samples first the short ones fill the gaps at the end instead of the other way round.
__global__ __launch_bounds__(1024) void k_prepare(Geo g, int* __restrict__ cu_keep,
                                                  int* __restrict__ tile_start,
                                                  int* __restrict__ status,
                                                  int* __restrict__ by_size) {
  __shared__ int red[2][16];
  __shared__ int carry[2];
  __shared__ int len_of[kMaxBySize];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  int broken = 0;
  for (int b = tid; b < g.B; b += 1024) broken |= g.cu[b + 1] < g.cu[b] ? 1 : 0;
  if (tid == 0) {
    carry[0] = 0;
    carry[1] = 0;
    broken |= (g.cu[0] != 0 || g.cu[g.B] != g.total_N) ? 1 : 0;
  }
  broken = __syncthreads_or(broken);
  int bad = 0;
  for (int b0 = 0; b0 < g.B; b0 += 1024) {
    const int b = b0 + tid;
    int k = 0, tiles = 0;
    if (b < g.B && !broken) {
      int n = g.cu[b + 1] - g.cu[b];
      int kb = budget_of(g, n);
      // a span must lie inside X (long arithmetic: the caller's start may be anything)
      const bool inside = g.span == nullptr ||
                          (g.span[b] >= 0 && (long)g.span[b] + n <= (long)g.x_rows);
      if (inside && sample_ok(g, n, kb)) {
        k = kb;
        tiles = (n + g.tile_rows - 1) / g.tile_rows;
      } else if (n != 0) {
        bad = 1;
      }
    }
    int sk = wave_excl_scan(k, lane), st = wave_excl_scan(tiles, lane);
    if (lane == 63) {
      red[0][w] = sk + k;
      red[1][w] = st + tiles;
    }
    __syncthreads();
    int bk = carry[0], bt = carry[1], tk = 0, tt = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      bk += i < w ? red[0][i] : 0;
      bt += i < w ? red[1][i] : 0;
      tk += red[0][i];
      tt += red[1][i];
    }
    if (b < g.B) {
      cu_keep[b] = bk + sk;
      tile_start[b] = bt + st;
    }
    __syncthreads();
    if (tid == 0) {
      carry[0] += tk;
      carry[1] += tt;
    }
    __syncthreads();
  }
  bad = __syncthreads_or(bad);
  if (by_size != nullptr) {  // (block-uniform; g.B <= kMaxBySize)
    const int n = tid < g.B && !broken ? g.cu[tid + 1] - g.cu[tid] : 0;
    if (tid < g.B) len_of[tid] = n;
    __syncthreads();
    if (tid < g.B) {
      int rank = 0;
      for (int o = 0; o < g.B; ++o) rank += (len_of[o] > n || (len_of[o] == n && o < tid)) ? 1 : 0;
      by_size[rank] = tid;
    }
  }
  if (tid == 0) {
    cu_keep[g.B] = carry[0];
    tile_start[g.B] = carry[1];
    status[0] = broken ? 2 : bad;
    status[2] = 0;  // set by k_seq_offsets if it runs after this
  }
}

// Caller-supplied pivots: status[1] = 1 if any processed sample's Pin indices are not
// distinct indices inside the sample, else 0.  grid: 1 block of 1024.
__global__ __launch_bounds__(1024) void k_check_pivots(Geo g, const int* __restrict__ piv,
                                                       int* __restrict__ status) {
  int bad = 0;
  for (int idx = threadIdx.x; idx < g.B * g.P; idx += 1024) {
    const int b = idx / g.P, i = idx - b * g.P;
    if (i >= g.Pin) continue;  // a pivot from outside the sample: nothing to check
    const Sample sm = sample_of(g, b);
    if (sm.k == 0) continue;
    const int p = piv[idx];
    bad |= (p < 0 || p >= sm.n) ? 1 : 0;
    for (int o = 0; o < i; ++o) bad |= piv[b * g.P + o] == p ? 1 : 0;
  }
  bad = __syncthreads_or(bad);
  if (threadIdx.x == 0) status[1] = bad ? 1 : 0;
}

// Pivots drawn at random (the random rows of the pivot ablation, Section 4.3 / Table 8).
// The generator is Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11): a round maps
// the counter words (c0, c1, c2, c3) to (hi(M1 c2) ^ c1 ^ k0, lo(M1 c2), hi(M0 c0) ^ c3 ^ k1,
// lo(M0 c0)); the key words grow by the two Weyl constants between rounds.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4]) {
  constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    if (round > 0) {
      k0 += 0x9E3779B9u;
      k1 += 0xBB67AE85u;
    }
    const uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
    const uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
    c0 = hi1 ^ c1 ^ k0;
    c1 = lo1;
    c2 = hi0 ^ c3 ^ k1;
    c3 = lo0;
  }
  out[0] = c0;
  out[1] = c1;
  out[2] = c2;
  out[3] = c3;
}

// Sample b draws tokens d_t = floor(w_t * N_b / 2^32), t = 0, 1, ..., with w_t word t mod 4 of
// the Philox block of counter (t div 4, b, 0, 0) and key (low, high half of the seed); its
// Pin pivots are the first Pin distinct draws in the order they appear.  After draw_limit
// draws (kRandomDraws, a bound for the loop: 64 pivots among 64 tokens need about 300; a test
// may lower it) the lowest unused tokens fill the list.  grid: B blocks of one wave: the lanes
// compute 256 draws at a time, lane 0 walks them.
constexpr int kRandomDraws = 4096;
__global__ __launch_bounds__(64) void k_random_pivots(Geo g, unsigned long long seed,
                                                      int draw_limit, int* __restrict__ piv) {
  __shared__ uint32_t used[kMaxN / 32];
  __shared__ int draws[256];
  __shared__ int have_sh;
  const int b = blockIdx.x, lane = threadIdx.x;
  const Sample sm = sample_of(g, b);
  if (sm.k == 0 || g.Pin == 0) return;
  const int n = sm.n, want = g.Pin;
  int* out = piv + (long)b * g.P;
  for (int t = lane; t < (n + 31) / 32; t += 64) used[t] = 0u;
  int have = 0;
  for (int base = 0; base < draw_limit && have < want; base += 256) {
    uint32_t w[4];
    philox4x32_10((uint32_t)(base / 4 + lane), (uint32_t)b, 0u, 0u, (uint32_t)seed,
                  (uint32_t)(seed >> 32), w);
#pragma unroll
    for (int u = 0; u < 4; ++u) draws[4 * lane + u] = (int)__umulhi(w[u], (uint32_t)n);
    __syncthreads();
    if (lane == 0) {
      for (int t = 0; t < 256 && base + t < draw_limit && have < want; ++t) {
        const int d = draws[t];
        const uint32_t bit = 1u << (d & 31);
        if ((used[d >> 5] & bit) == 0u) {
          used[d >> 5] |= bit;
          out[have++] = d;
        }
      }
      have_sh = have;
    }
    __syncthreads();
    have = have_sh;
  }
  if (lane == 0)
    for (int j = 0; j < n && have < want; ++j)
      if ((used[j >> 5] & (1u << (j & 31))) == 0u) out[have++] = j;
}

// status[1] = 0: for entry points that read no pivot list (one thread).
__global__ void k_clear_pivot_status(int* __restrict__ status) { status[1] = 0; }

// The raw matrix-core sums the bf16 score kernel is built on, for the test of its rounding
// bound: tile t of A and B is [16][32] bf16 (k contiguous); out[t][i][j] = sum_k A[i][k] *
// B[j][k] from a zero accumulator.  grid: tiles blocks of 64.
typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));
typedef float probe_f32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(64) void k_probe_mfma_dot32(const unsigned char* __restrict__ A,
                                                        const unsigned char* __restrict__ B,
                                                        float* __restrict__ out) {
  const int lane = threadIdx.x;
  const long tile = blockIdx.x;
  const long off = tile * (16 * 32 * 2) + (lane & 15) * 64 + (lane >> 4) * 16;
  const probe_bf16x8 af = *reinterpret_cast<const probe_bf16x8*>(A + off);
  const probe_bf16x8 bf = *reinterpret_cast<const probe_bf16x8*>(B + off);
  const probe_f32x4 zero = {0.f, 0.f, 0.f, 0.f};
  const probe_f32x4 c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, bf, zero, 0, 0, 0);
#pragma unroll
  for (int r = 0; r < 4; ++r) out[tile * 256 + ((lane >> 4) * 4 + r) * 16 + (lane & 15)] = c[r];
}

// Squared Euclidean norms of the rows of pivots first..Ppad-1 in fp64 (0 for padding
// slots).  piv_mark (optional): entry i of a pivot from outside the sample is set to
// -1 - (its row in the sample's share of E).  grid: B blocks of 1024: a wave per pivot, so
// that up to 16 rows are in flight at once (64 pivots: four rounds).
template <int DT>
__global__ __launch_bounds__(1024) void k_pivot_norms(Geo g, const void* __restrict__ X,
                                                     const int* __restrict__ piv, int first,
                                                     double* __restrict__ pl2,
                                                     int* __restrict__ piv_mark) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.x;
  const Sample sm = sample_of(g, b);
  const int esz = DT == kBF16 ? 2 : 4;
  if (piv_mark && tid >= g.Pin && tid < g.P) piv_mark[b * g.P + tid] = -1 - (tid - g.Pin);
  for (int i = first + wave; i < g.Ppad; i += 16) {
    double l1 = 0.0, l2 = 0.0;
    if (sm.k != 0 && i < g.P) row_l1_l2_f64<DT>(pivot_row(g, X, esz, sm, b, i, piv), g.D, lane, l1, l2);
    if (lane == 0) pl2[b * g.Ppad + i] = l2;
  }
}

// Compaction: one wave per retained row.  grid: ceil(rows_bound / 4) blocks of 256, rounded up
// to a multiple of 8 (xcd_contiguous).
// Y rows are packed (stride D); copies are 16 bytes per lane, 1 KiB per wave access.
// The rows are read once: streaming (non-temporal) loads measured 20 % faster on the
// largest batch than ordinary ones; streaming stores did not help.
__global__ __launch_bounds__(256) void k_gather(Geo g, int esz, const void* __restrict__ X,
                                                const long long* __restrict__ pos,
                                                const int* __restrict__ keep,
                                                void* __restrict__ Y,
                                                long long* __restrict__ pos_out) {
  const int lane = threadIdx.x & 63;
  const long r = xcd_contiguous(blockIdx.x, gridDim.x) * 4 + (threadIdx.x >> 6);
  int b;
  if (g.cu == nullptr) {
    if (r >= (long)g.B * g.K) return;
    b = (int)(r / g.K);
  } else {
    if (r >= g.cu_keep[g.B]) return;
    int lo = 0, hi = g.B;
    while (hi - lo > 1) {
      int mid = (lo + hi) >> 1;
      if (g.cu_keep[mid] <= r) lo = mid; else hi = mid;
    }
    b = lo;
  }
  const int row0 = g.cu ? g.cu[b] : b * g.N;
  const int n = g.cu ? g.cu[b + 1] - row0 : g.N;
  int kr = keep[r];
  kr = kr < 0 ? 0 : (kr < n ? kr : n - 1);  // a caller's bad index must not leave X
  const long src = (long)(g.span ? g.span[b] : row0) + kr;
  const u32x4* in = reinterpret_cast<const u32x4*>(static_cast<const unsigned char*>(X) +
                                                   src * g.ld * esz);
  u32x4* out = reinterpret_cast<u32x4*>(static_cast<unsigned char*>(Y) + r * (long)g.D * esz);
  const int pieces = g.D * esz / 16;
  for (int t0 = 0; t0 < pieces; t0 += kWave * 8) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      int t = t0 + u * kWave + lane;
      v[u] = t < pieces ? __builtin_nontemporal_load(in + t) : u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      int t = t0 + u * kWave + lane;
      if (t < pieces) out[t] = v[u];
    }
  }
  if (pos && lane == 0) pos_out[r] = pos[src];
}

// ---- whole-sequence compaction (Appendix D: text before the vision span, the retained
// vision tokens, text after it) ------------------------------------------------------

// One block of 1024.  Sequence b is rows [seq_cu[b], seq_cu[b+1]) of the caller's per-token
// tensors and must contain its span [span[b], span[b] + N_b).  Writes the new offsets
// seq_cu_out[B+1]: sequence b shrinks by N_b - K_b rows (K_b = 0 for a skipped sample, whose
// vision tokens are all dropped).  status[2] = 1 and all-zero offsets if seq_cu is not a
// non-decreasing sequence from 0 to x_rows or a span is not inside its sequence.
__global__ __launch_bounds__(1024) void k_seq_offsets(Geo g, const int* __restrict__ seq_cu,
                                                      int* __restrict__ seq_cu_out,
                                                      int* __restrict__ status) {
  __shared__ int red[16];
  __shared__ int carry;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  int bad = 0;
  for (int b = tid; b < g.B; b += 1024) {
    const int lo = seq_cu[b], hi = seq_cu[b + 1];
    const int n = g.cu[b + 1] - g.cu[b];
    bad |= (hi < lo || g.span[b] < lo || (long)g.span[b] + n > (long)hi) ? 1 : 0;
  }
  if (tid == 0) {
    carry = 0;
    // status[0] == 2: k_prepare found cu_seqlens itself broken (lengths are meaningless)
    bad |= (status[0] == 2 || seq_cu[0] != 0 || seq_cu[g.B] != g.x_rows) ? 1 : 0;
  }
  bad = __syncthreads_or(bad);
  for (int b0 = 0; b0 < g.B; b0 += 1024) {
    const int b = b0 + tid;
    int len = 0;
    if (b < g.B && !bad) {
      const int n = g.cu[b + 1] - g.cu[b];
      len = (seq_cu[b + 1] - seq_cu[b]) - n + (g.cu_keep[b + 1] - g.cu_keep[b]);
    }
    const int sc = wave_excl_scan(len, lane);
    if (lane == 63) red[w] = sc + len;
    __syncthreads();
    int base = carry, tot = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      base += i < w ? red[i] : 0;
      tot += red[i];
    }
    if (b < g.B) seq_cu_out[b] = base + sc;
    __syncthreads();
    if (tid == 0) carry += tot;
    __syncthreads();
  }
  if (tid == 0) {
    seq_cu_out[g.B] = carry;
    status[2] = bad;
  }
}

// row_map[r] = row of the original tensors that row r of the shortened ones comes from.
// grid: ceil(rows_bound / 256) blocks of 256; rows beyond seq_cu_out[B] are left alone.
__global__ __launch_bounds__(256) void k_seq_row_map(Geo g, const int* __restrict__ seq_cu,
                                                     const int* __restrict__ seq_cu_out,
                                                     const int* __restrict__ keep,
                                                     int* __restrict__ row_map) {
  const long r = (long)blockIdx.x * 256 + threadIdx.x;
  if (r >= seq_cu_out[g.B]) return;
  int lo = 0, hi = g.B;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (seq_cu_out[mid] <= r) lo = mid; else hi = mid;
  }
  const int b = lo;
  const int t = (int)(r - seq_cu_out[b]);
  const int n = g.cu[b + 1] - g.cu[b];
  const int k = g.cu_keep[b + 1] - g.cu_keep[b];
  const int before = g.span[b] - seq_cu[b];  // text rows ahead of the span
  int src;
  if (t < before) {
    src = seq_cu[b] + t;
  } else if (t < before + k) {
    int kr = keep[g.cu_keep[b] + (t - before)];
    kr = kr < 0 ? 0 : (kr < n ? kr : n - 1);  // a caller's bad index must not leave the span
    src = g.span[b] + kr;
  } else {
    src = g.span[b] + n + (t - before - k);
  }
  row_map[r] = src;
}

constexpr int kSeqOps = 8;  // tensors one gather launch moves
struct SeqOps {
  const unsigned char* src[kSeqOps];
  unsigned char* dst[kSeqOps];
  long row_bytes[kSeqOps], src_ld[kSeqOps], dst_ld[kSeqOps];  // bytes, multiples of 16
};

// dst row r = src row row_map[r] for every tensor of ops.  One wave per (row, tensor):
// grid (ceil(rows_bound / 4) rounded up to a multiple of 8, tensors) blocks of 256 (with a
// multiple of 8 in x the die of a block depends on its x only: xcd_contiguous); 16 bytes per
// lane, 1 KiB per access.
__global__ __launch_bounds__(256) void k_gather_rows(SeqOps ops, const int* __restrict__ n_rows,
                                                     const int* __restrict__ row_map) {
  const int lane = threadIdx.x & 63, o = blockIdx.y;
  const long r = xcd_contiguous(blockIdx.x, gridDim.x) * 4 + (threadIdx.x >> 6);
  if (r >= *n_rows) return;
  const long src = row_map[r];
  const u32x4* in = reinterpret_cast<const u32x4*>(ops.src[o] + src * ops.src_ld[o]);
  u32x4* out = reinterpret_cast<u32x4*>(ops.dst[o] + r * ops.dst_ld[o]);
  const int pieces = (int)(ops.row_bytes[o] / 16);
  for (int t0 = 0; t0 < pieces; t0 += kWave * 8) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int t = t0 + u * kWave + lane;
      v[u] = t < pieces ? __builtin_nontemporal_load(in + t) : u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int t = t0 + u * kWave + lane;
      if (t < pieces) out[t] = v[u];
    }
  }
}

// Position ids, plane-major: pos_out[p*out_stride + r] = pos[p*in_stride + row_map[r]].
// grid: (ceil(rows_bound / 256), planes) blocks of 256.
__global__ __launch_bounds__(256) void k_gather_pos(const int* __restrict__ n_rows,
                                                    const int* __restrict__ row_map,
                                                    const long long* __restrict__ pos,
                                                    long in_stride, long long* __restrict__ pos_out,
                                                    long out_stride) {
  const long r = (long)blockIdx.x * 256 + threadIdx.x;
  if (r >= *n_rows) return;
  const long p = blockIdx.y;
  pos_out[p * out_stride + r] = pos[p * in_stride + row_map[r]];
}

}  // namespace dart

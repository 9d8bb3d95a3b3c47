/* Host-side sweep of the C ABI under AddressSanitizer and UndefinedBehaviorSanitizer.
 * Linked against a build of the library whose host code carries the same sanitizers.  Every
 * call below returns on the host before anything is enqueued (an invalid descriptor, a NULL
 * or misaligned required pointer, or a workspace that is too small), so no GPU is needed; what
 * runs is the descriptor validation and the workspace arithmetic, on tens of thousands of
 * descriptors that include the extremes of every integer field.  Prints "abi sanitize ok". */
#include <limits.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "dart.h"

static uint64_t state = 0x243F6A8885A308D3ull;
static uint32_t rnd(void) { /* splitmix64, upper half */
  uint64_t z = (state += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return (uint32_t)((z ^ (z >> 31)) >> 32);
}
static int32_t pick(const int32_t* v, int n) { return v[rnd() % (uint32_t)n]; }

int main(void) {
  static const int32_t sizes[] = {INT_MIN, -1, 0, 1, 2, 7, 8, 16, 17, 64, 65, 576, 2880, 4096,
                                  16384, 16385, 65536, 65537, 1 << 20, 1 << 27, (1 << 27) + 1,
                                  INT_MAX};
  static const int64_t strides[] = {INT64_MIN, -1, 0, 8, 4096, 4104, 65536, 1ll << 40, INT64_MAX};
  const int ns = (int)(sizeof sizes / sizeof sizes[0]);
  long valid = 0, invalid = 0;
  void* fake = (void*)(uintptr_t)0x10000;
  for (int it = 0; it < 60000; ++it) {
    dart_desc d;
    memset(&d, 0, sizeof d);
    d.B = pick(sizes, ns);
    d.D = pick(sizes, ns);
    d.P = pick(sizes, ns);
    d.N = pick(sizes, ns);
    d.total_N = rnd() % 3 ? 0 : pick(sizes, ns);
    d.max_N = pick(sizes, ns);
    d.ld = rnd() % 2 ? d.D : strides[rnd() % 9];
    d.dtype = (int32_t)(rnd() % 4) - 1;
    d.K = pick(sizes, ns);
    d.keep_num = pick(sizes, ns);
    d.keep_den = pick(sizes, ns);
    d.pivot_mode = (int32_t)(rnd() % 6) - 1;
    d.seed = ((uint64_t)rnd() << 32) ^ rnd();
    d.score_mode = (int32_t)(rnd() % 5) - 1;
    d.P_ext = rnd() % 4 ? 0 : pick(sizes, ns);
    d.ext_ld = strides[rnd() % 9];
    d.ext_pivots = rnd() % 2 ? fake : NULL;
    d.cu_seqlens = rnd() % 3 == 0 ? (const int32_t*)fake : NULL;
    d.span_start = rnd() % 5 == 0 ? (const int32_t*)fake : NULL;
    d.X_rows = pick(sizes, ns);
    if (it % 4 == 0) { /* bias a quarter of the draws towards plausible shapes */
      d.B = 1 + (int32_t)(rnd() % 32);
      d.D = 8 * (1 + (int32_t)(rnd() % 512));
      d.ld = d.D;
      d.P = 1 + (int32_t)(rnd() % 64);
      d.N = d.P + (int32_t)(rnd() % 16000);
      d.K = d.P + (int32_t)(rnd() % (uint32_t)(d.N - d.P + 1));
      d.dtype = (int32_t)(rnd() % 2);
      d.pivot_mode = (int32_t)(rnd() % 4);
      d.score_mode = (int32_t)(rnd() % 3);
      d.P_ext = 0;
      d.cu_seqlens = NULL;
      d.span_start = NULL;
      d.total_N = 0;
    }
    const size_t ws = dart_workspace_bytes(&d);
    if (ws == 0) {
      ++invalid;
      /* an invalid descriptor is refused by every entry point, whatever else is passed */
      if (dart_reduce(&d, fake, NULL, 0, 0, NULL, fake, NULL, (int32_t*)fake, NULL,
                      (int32_t*)fake, NULL, fake, (size_t)1 << 40, NULL) >= 0 && d.B != 0)
        return 2;
      (void)dart_reduce_static(&d, fake, NULL, 0, 0, NULL, fake, NULL, (int32_t*)fake, NULL,
                               (int32_t*)fake, NULL, NULL);
      continue;
    }
    ++valid;
    if (ws % 256 != 0) return 3;
    if (d.B == 0) continue; /* an empty batch is a valid no-op */
    /* a valid descriptor: NULL X, then a workspace one byte short, then a misaligned X */
    if (dart_reduce(&d, NULL, NULL, 0, 0, NULL, fake, NULL, (int32_t*)fake, NULL, (int32_t*)fake,
                    NULL, fake, ws, NULL) != DART_ERR_NULL)
      return 4;
    if (dart_reduce(&d, fake, NULL, 0, 0, NULL, fake, NULL, (int32_t*)fake, NULL, (int32_t*)fake,
                    NULL, fake, ws - 1, NULL) != DART_ERR_WORKSPACE)
      return 5;
    if (dart_reduce(&d, (char*)fake + 2, NULL, 0, 0, NULL, fake, NULL, (int32_t*)fake, NULL,
                    (int32_t*)fake, NULL, fake, ws, NULL) != DART_ERR_ALIGN)
      return 6;
    if (dart_select_pivots(&d, fake, NULL, 0, 0, NULL, NULL, fake, ws, NULL) >= 0) return 7;
    if (dart_duplication_scores(&d, fake, NULL, NULL, fake, ws, NULL) != DART_ERR_NULL) return 8;
    if (dart_topk_keep(&d, NULL, NULL, NULL, NULL, NULL, fake, ws, NULL) != DART_ERR_NULL) return 9;
    if (dart_gather_compact(&d, fake, NULL, NULL, fake, NULL, fake, ws, NULL) != DART_ERR_NULL)
      return 10;
    /* caller-supplied norms: missing norms, then an error bound that is none (or a pivot mode
       that ranks no norms) */
    if (dart_reduce_with_norms(&d, fake, NULL, 0, 0, NULL, 1e-6, NULL, fake, NULL, (int32_t*)fake,
                               NULL, (int32_t*)fake, NULL, fake, ws, NULL) != DART_ERR_NULL)
      return 13;
    if (dart_reduce_with_norms(&d, fake, NULL, 0, 0, (const float*)fake, -1.0, NULL, fake, NULL,
                               (int32_t*)fake, NULL, (int32_t*)fake, NULL, fake, ws, NULL) !=
        (d.pivot_mode >= DART_PIVOT_GIVEN ? DART_ERR_DTYPE : DART_ERR_SHAPE))
      return 14;
    {
      int32_t w1 = -1, k1 = -1, w2 = -1, k2 = -1;
      if (dart_score_tile_shape(&d, &w1, &k1) != DART_OK) return 15;
      if (dart_score_tile_shape_first_read(&d, &w2, &k2) != DART_OK) return 16;
      if (d.dtype == DART_BF16 ? (w1 < 1 || k1 < 1 || w1 % k1 || w2 < 1 || k2 < 1 || w2 % k2)
                               : (w1 | k1 | w2 | k2) != 0)
        return 17;
    }
  }
  if (valid < 10000 || invalid < 10000) return 11;
  for (int s = 1; s >= -12; --s)
    if (strlen(dart_strerror((dart_status)s)) == 0) return 12;
  printf("abi sanitize ok: %ld valid and %ld invalid descriptors\n", valid, invalid);
  return 0;
}

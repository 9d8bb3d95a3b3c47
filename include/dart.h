/*
 * dart.h -- C ABI of the duplication-aware token reduction step (DART,
 * arXiv 2502.11494, Section 3.3) for AMD MI355X (gfx950).
 *
 * The step runs between two decoder layers of a multimodal LLM.  Per sample it
 *   (a) picks P pivot tokens by the largest L1 norm of a criterion row
 *       (Definition 1; Table 1 caption; the footnote of Section 3.3 that
 *       defines the K-norm as an L1 norm),
 *   (b) scores every token against every pivot with the cosine similarity of
 *       Definition 2 / Eq. (7),
 *   (c) retains the pivots plus, pivot by pivot, the tokens that duplicate that
 *       pivot least, until the keep budget is met (Eq. (9)-(10) with the
 *       per-pivot threshold fixed by the reduction ratio),
 *   (d) compacts hidden-state rows and position ids to the retained tokens in
 *       their original order, so the remaining layers run on the shorter
 *       sequence (Appendix D, post-pruning sequence length).
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 * Memory.  `desc` is host memory, read during the call only; the device arrays it
 *   names (cu_seqlens, ext_pivots, span_start) are read by the enqueued kernels and must
 *   stay valid and unchanged until that work has finished.  Every other
 *   pointer is DEVICE memory owned by the caller unless stated otherwise.  The
 *   library never allocates, frees or keeps a pointer; scratch comes from the
 *   caller's workspace `ws` of at least dart_workspace_bytes(desc) bytes,
 *   256-byte aligned.  Inputs are never written.  Outputs must not alias inputs.
 * Layout.  X holds `total_N` token rows of D elements, row stride `ld`
 *   elements, sample after sample.  Dense: sample b owns rows [b*N, (b+1)*N).
 *   Ragged: sample b owns rows [cu_seqlens[b], cu_seqlens[b+1]).  Row starts
 *   must be 16-byte aligned (X base, ld*elemsize and D*elemsize multiples of 16).
 * Budget.  Sample b keeps K_b tokens: K_b = K if K > 0, otherwise
 *   K_b = floor(N_b * keep_num / keep_den).  P <= K_b <= N_b is required.
 *   keep/pos_out/Y are packed: sample b owns rows [cu_keep[b], cu_keep[b+1]),
 *   cu_keep[b] = sum of K_b' over b' < b (dense with K > 0: b*K).
 * Streams.  `stream` is a hipStream_t passed as void* (NULL = default stream).
 *   Calls only enqueue work; outputs are valid once the stream reaches that
 *   point.  No call synchronises except dart_device_status.
 * Errors.  Violations visible on the host return a negative dart_status and
 *   enqueue nothing.  In ragged mode the per-sample sizes live on the device:
 *   a sample with N_b > max_N, N_b < P, K_b < P or K_b > N_b (N_b == 0 is a
 *   valid empty sample), or whose span (desc.span_start) leaves X, is skipped -- it
 *   keeps zero tokens -- and a flag is raised in the workspace that
 *   dart_device_status reports.
 *   Non-finite input values give unspecified (but memory-safe) results.
 * Value range.  The fp32 arithmetic of the bf16 path (exact products of two bf16 values,
 *   32-term sums of them, row sums of |x| and x^2) must neither overflow nor lose bits to
 *   underflow, or the rounding bound the decisions are certified against does not hold:
 *   every non-zero element must satisfy 2^-55 <= |x| <= 2^55 (zeros are fine), for either
 *   dtype.  Inside that range a common power-of-two factor on a sample changes no output
 *   bit.  Outside it the retained set may differ from the exact one (memory-safe, not
 *   detected: the library does not scan its input).
 * Determinism.  Same inputs give bit-identical outputs, call after call, and a
 *   row's score depends only on its bytes and the pivot's bytes, not on where
 *   the row sits in the batch.  (Different entry points or pivot modes may take the
 *   token norms from different passes: their scores agree within
 *   dart_score_tolerance, not necessarily in the last bit.)
 * Limits.  B <= 2^20, 1 <= P <= 64, N_b <= 16384, D <= 65536, total_N <= 2^27, row strides (ld, crit_ld,
 *   ext_ld) <= 2^24 elements.
 * Pivots from outside (desc.P_ext > 0).  Tokens are scored against such a pivot and it
 *   has its stage in step (c) like any pivot -- after the pivots that are tokens, in the
 *   order of its rows -- but it is no token: it is never retained and holds no slot of
 *   the budget.  With P_in = P - P_ext, R starts as the P_in pivots inside the sample, the
 *   P stages share K_b - P_in slots (floor((K_b - P_in)/P) each, +1 for the first
 *   (K_b - P_in) mod P stages) and P_in <= K_b <= N_b is required instead of
 *   P <= K_b <= N_b.  In every piv array entry i >= P_in of a sample is not read; where
 *   the library writes piv it sets that entry to -1 - (i - P_in).  Step (a) chooses P_in
 *   pivots (none if P_ext == P).
 */
#ifndef DART_H_
#define DART_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define DART_API __attribute__((visibility("default")))
#else
#define DART_API
#endif

typedef enum dart_status {
  DART_OK = 0,
  DART_ERR_NULL = -1,      /* a required pointer is NULL                          */
  DART_ERR_SHAPE = -2,     /* B, N, D, P, ld, total_N or max_N out of range        */
  DART_ERR_BUDGET = -3,    /* P <= K <= N violated, or bad keep_num/keep_den       */
  DART_ERR_DTYPE = -4,     /* unknown dtype or pivot mode                          */
  DART_ERR_WORKSPACE = -5, /* ws NULL, misaligned or smaller than required         */
  DART_ERR_ALIGN = -6,     /* a row start would not be 16-byte aligned             */
  DART_ERR_HIP = -7,       /* a HIP call or kernel launch failed                   */
  DART_ERR_DEVICE = -8,    /* dart_device_status: a ragged sample or a given pivot
                              list was rejected on the device                      */
  DART_ERR_STATIC_LIMIT = -9 /* dart_reduce_static: the problem needs more scratch than
                              the library's built-in buffer holds                  */
} dart_status;

typedef enum dart_dtype {
  DART_F32 = 0,  /* IEEE binary32 hidden states                                    */
  DART_BF16 = 1  /* bfloat16 hidden states (upper half of a binary32)              */
} dart_dtype;

typedef enum dart_pivot_mode {
  DART_PIVOT_MAX_L1 = 0, /* largest criterion L1 norm first (Table 1 caption)      */
  DART_PIVOT_MIN_L1 = 1, /* smallest first (the "heart" rows of the pivot ablation) */
  DART_PIVOT_GIVEN = 2,  /* dart_reduce only: the caller supplies the pivots; see dart_reduce */
  DART_PIVOT_RANDOM = 3  /* dart_select_pivots and dart_reduce: drawn at random from desc.seed
                            (the random rows of the pivot ablation, Section 4.3 / Table 8).
                            The paper names no generator; the draw is defined here: sample
                            b draws tokens d_t = floor(w_t * N_b / 2^32), t = 0, 1, ..., where
                            w_t is word t mod 4 of the Philox4x32-10 block (Salmon et al.,
                            SC'11) with counter (t div 4, b, 0, 0) and key (low, high 32 bits
                            of seed); the sample's P - P_ext pivots are its first distinct
                            draws, in the order they appear, which is also their stage order
                            in step (c).  (After 4096 draws, which 64 pivots among 64 tokens
                            reach with probability below 1e-25, the lowest unused tokens
                            complete the list; DART_RANDOM_DRAW_LIMIT=n in the environment,
                            0 <= n <= 4096, lowers that limit so that a test can reach the
                            completion.)  No criterion is read: crit is ignored.            */
} dart_pivot_mode;

typedef enum dart_score_mode {
  DART_SCORE_PER_PIVOT = 0, /* Eq. (9)-(10) with a threshold per pivot: the staged rule  */
  DART_SCORE_MIN = 1,       /* one threshold for all pivots on min_i S[i][j]             */
  DART_SCORE_MAX = 2        /* one threshold for all pivots on max_i S[i][j]             */
} dart_score_mode;

/* Problem descriptor (host memory, plain data). */
typedef struct dart_desc {
  int32_t B;        /* samples in the batch, >= 0 (0 is a valid no-op)              */
  int32_t D;        /* hidden size: elements per token row                          */
  int32_t P;        /* pivots per sample (Definition 1), 1..64                      */
  int32_t N;        /* tokens per sample, dense layout; ignored when ragged         */
  const int32_t* cu_seqlens; /* DEVICE int32[B+1] row offsets, or NULL for dense    */
  int32_t total_N;  /* rows of X; dense: B*N (0 means "derive"); ragged: required   */
  int32_t max_N;    /* ragged: host-known upper bound of every N_b; dense: ignored  */
  int64_t ld;       /* row stride of X in elements, >= D                            */
  int32_t dtype;    /* dart_dtype of X, crit and Y                                  */
  int32_t K;        /* keep budget per sample (pivots included); 0 = use the ratio  */
  int32_t keep_num; /* K == 0: K_b = floor(N_b * keep_num / keep_den)               */
  int32_t keep_den;
  int32_t pivot_mode; /* dart_pivot_mode                                            */
  int32_t score_mode; /* dart_score_mode (0 = the default staged rule)              */
  /* Pivots from outside the scored tokens (the text-token pivots of the pivot ablation,
   * Table 8, and of the study of the pivots' modality): of the P pivots of every sample
   * the LAST P_ext are rows of ext_pivots, the first P - P_ext are tokens of the sample.
   * 0 = all pivots are tokens of the sample (then the two fields below are ignored).    */
  int32_t P_ext;
  int64_t ext_ld;         /* row stride of ext_pivots in elements, >= D                  */
  const void* ext_pivots; /* DEVICE rows [B*P_ext, D] of X's dtype, 16-byte aligned row
                             starts: sample b's outside pivot e is row b*P_ext + e        */
  /* Samples that are spans of a larger tensor (the vision tokens inside whole sequences of
   * text and vision tokens): with span_start != NULL (ragged layout required) sample b's
   * N_b = cu_seqlens[b+1] - cu_seqlens[b] tokens are rows span_start[b] .. span_start[b] +
   * N_b - 1 of X -- and of crit and pos, which are indexed like X -- and X has X_rows rows.
   * S, l1_out and keep stay packed by cu_seqlens.  A span that leaves [0, X_rows) makes its
   * sample a skipped one (see Errors).  NULL: the samples are packed back to back.        */
  const int32_t* span_start; /* DEVICE int32[B], or NULL                                   */
  int32_t X_rows;            /* rows of X when span_start != NULL (>= total_N)             */
  uint64_t seed;             /* DART_PIVOT_RANDOM: the seed of the draw (ignored otherwise) */
} dart_desc;

/* Bytes of workspace every entry point below accepts for this descriptor
 * (host arithmetic only; 0 if the descriptor is invalid). */
DART_API size_t dart_workspace_bytes(const dart_desc* desc);

/* The tile of the score kernel (step (b), Eq. 7) this library would use for the descriptor on
 * the current GPU (256 compute units assumed when there is none): *waves wavefronts per
 * workgroup in *split groups that share 16 * waves / split token rows and split the hidden
 * dimension among them; both 0 for fp32 descriptors, whose score kernel has one shape.  This
 * is the shape of dart_reduce with the hidden states as their own criterion.  Host
 * arithmetic only; waves and split are HOST pointers.  The choice is a cost model over the
 * batch's shape (see the library's source); DART_SCORE_TILE="W,KS" in the environment names
 * one of the built shapes instead, and a value that names none, or one whose tiles do not fit
 * the LDS with this many pivots, makes every entry point return DART_ERR_SHAPE.  The results of
 * the step do not depend on the shape (decisions are certified in fp64). */
DART_API dart_status dart_score_tile_shape(const dart_desc* desc, int32_t* waves, int32_t* split);

/* The same for calls whose score pass is the first pass over X: dart_reduce with a separate
 * criterion tensor (its norm pass reads crit, not X) and dart_duplication_scores.  Such calls
 * find no row of X in the memory-side cache, and small dense batches then do better with
 * four groups of waves per tile (measured; see the library's source).  For descriptors whose
 * pivots are given, drawn at random or all from outside, dart_score_tile_shape already
 * reports this shape (no norm pass over X exists for them). */
DART_API dart_status dart_score_tile_shape_first_read(const dart_desc* desc, int32_t* waves,
                                                      int32_t* split);

/* (a) Pivot selection -- Definition 1 with the max-L1-norm criterion of the
 * Table 1 caption.  crit: criterion rows [total_N, crit_D] with row stride
 * crit_ld (same dtype as X, e.g. the layer's key states), or NULL to use the
 * hidden-state rows themselves (then crit_D/crit_ld are ignored).
 * DART_PIVOT_RANDOM: the pivots are drawn from desc.seed instead (see dart_pivot_mode), in
 * draw order; crit is ignored and l1_out is not written.
 * Output piv[b*P + i] = index, local to sample b, of its i-th pivot, ordered by
 * (L1 norm descending, index ascending) -- ascending norm for DART_PIVOT_MIN_L1.
 * Norms are accumulated in fp32 and every token whose fp32 norm could still
 * reach the top P within the rounding bound is re-evaluated in fp64, so the
 * order is that of the exact norms.  l1_out (optional, float[total_N]) receives
 * the fp32 L1 norm of every criterion row. */
DART_API dart_status dart_select_pivots(const dart_desc* desc, const void* X, const void* crit,
                               int32_t crit_D, int64_t crit_ld, int32_t* piv, float* l1_out,
                               void* ws, size_t ws_bytes, void* stream);

/* (b) Duplication scores -- Eq. (7): S = <p_i, x_j> / (|p_i| |x_j|), Euclidean
 * norms, 0 when either norm is 0.  piv as produced by dart_select_pivots.
 * S is pivot-major per sample: sample b, pivot i, token j at
 * S[P*row0(b) + i*N_b + j] with row0(b) the sample's first row in X.
 * bf16 inputs: exact bf16 products summed 32 at a time on the matrix cores in
 * fp32, those partial sums added in fp64; fp32 inputs: fp64 throughout.  The
 * stored value is rounded to fp32. */
DART_API dart_status dart_duplication_scores(const dart_desc* desc, const void* X, const int32_t* piv,
                                    float* S, void* ws, size_t ws_bytes, void* stream);

/* (c) Retained set -- Eq. (9)-(10).  R starts as the pivots; with m = K_b - P,
 * pivot i (in pivot order) adds the floor(m/P) (+1 for the first m mod P
 * pivots) not-yet-retained tokens of lowest S[i][.], ties to the lowest index.
 * keep receives each sample's retained indices (local to the sample) in
 * ascending order; cu_keep (optional, int32[B+1]) receives the packed offsets.
 * X == NULL: S is taken as exact.  X != NULL: wherever two fp32 scores at a
 * decision boundary are closer than the rounding bound of
 * dart_duplication_scores, the candidates involved are re-scored in fp64 from
 * the rows of X before deciding.
 * DART_SCORE_MIN / DART_SCORE_MAX: a second reading of Eq. (9)-(10), one threshold
 * common to all pivots: R = the pivots plus the K_b - P other tokens whose aggregate
 * score over the pivots (minimum or maximum) is lowest, ties to the lowest index. */
DART_API dart_status dart_topk_keep(const dart_desc* desc, const float* S, const int32_t* piv,
                           const void* X, int32_t* keep, int32_t* cu_keep, void* ws,
                           size_t ws_bytes, void* stream);

/* (d) Compaction -- the shortened sequence of Appendix D.  For sample b and
 * r < K_b: Y[cu_keep[b]+r][:] = X[row0(b)+keep[cu_keep[b]+r]][:] (D elements,
 * bit copy, Y rows densely packed with stride D) and
 * pos_out[cu_keep[b]+r] = pos[row0(b)+keep[...]].  pos/pos_out may both be NULL. */
DART_API dart_status dart_gather_compact(const dart_desc* desc, const void* X, const int64_t* pos,
                                const int32_t* keep, void* Y, int64_t* pos_out, void* ws,
                                size_t ws_bytes, void* stream);

/* (a)-(d) in one call.  Optional outputs (NULL to skip): pos/pos_out, cu_keep,
 * piv_out [B*P], S_out [P*total_N].  Y == NULL skips step (d) (pos/pos_out are then
 * ignored): for callers that compact whole sequences with dart_compact_sequences.
 * DART_PIVOT_GIVEN: step (a) is skipped and piv_out (required) is READ: piv_out[b*P + i]
 * is the index, local to sample b, of the pivot of stage i; crit is ignored.  The P
 * indices of a sample must be distinct and inside the sample: a list that is not makes
 * dart_device_status report DART_ERR_DEVICE and leaves that call's outputs unspecified
 * (nothing is read or written out of bounds).
 * DART_PIVOT_RANDOM: step (a) draws the pivots from desc.seed (see dart_pivot_mode) instead
 * of ranking norms; piv_out, if given, receives them; crit is ignored. */
DART_API dart_status dart_reduce(const dart_desc* desc, const void* X, const void* crit, int32_t crit_D,
                        int64_t crit_ld, const int64_t* pos, void* Y, int64_t* pos_out,
                        int32_t* keep, int32_t* cu_keep, int32_t* piv_out, float* S_out,
                        void* ws, size_t ws_bytes, void* stream);

/* dart_reduce for callers that already hold the criterion norms, e.g. from an epilogue of the
 * projection that produced the criterion rows (the K-norm of the Section 3.3 footnote computed
 * where the keys are computed): l1[j] (DEVICE float[total_N], packed like S) approximates the
 * L1 norm of criterion row j with a relative error of at most l1_rel_err (0 <= l1_rel_err <=
 * 0.1; the caller's promise, not checked; the rounding of an exact norm to fp32 is allowed for
 * on top of it).  The norm pass is skipped, so the hidden states
 * are read once, by the score pass.  The pivots are still those of the exact norms: every
 * token whose approximate norm could reach the top P within that error is re-evaluated in
 * fp64 from its criterion row (crit, or X when crit is NULL) and ranked by (exact norm, index),
 * so a loose bound costs time (more rows to re-read), a wrong one can cost the right pivots.
 * DART_PIVOT_MAX_L1 / DART_PIVOT_MIN_L1 only (DART_ERR_DTYPE otherwise); everything else as
 * dart_reduce. */
DART_API dart_status dart_reduce_with_norms(const dart_desc* desc, const void* X, const void* crit,
                                            int32_t crit_D, int64_t crit_ld, const float* l1,
                                            double l1_rel_err, const int64_t* pos, void* Y,
                                            int64_t* pos_out, int32_t* keep, int32_t* cu_keep,
                                            int32_t* piv_out, float* S_out, void* ws,
                                            size_t ws_bytes, void* stream);

/* dart_reduce for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and kernels as dart_reduce, but the scratch memory is a buffer built
 * into the library (a file-scope device array of dart_static_scratch_bytes() bytes -- 32 MiB
 * -- that every GPU the library runs on holds until the process ends) instead of `ws`.  The
 * call allocates and frees nothing.
 *   - A descriptor whose dart_workspace_bytes() exceeds dart_static_scratch_bytes() is
 *     refused with DART_ERR_STATIC_LIMIT and nothing is enqueued (the five benchmark shapes
 *     except the 1.7 GB ragged batch fit).
 *   - All calls on one GPU share that GPU's buffer: two calls whose work overlaps in time on
 *     the same GPU (different streams, or threads) race on it.  Calls on one stream are safe.
 *   - dart_device_status for such a call: pass ws = NULL to dart_device_status_static.
 * The buffer keeps the previous call's contents; the kernels initialise every word they
 * read. */
DART_API dart_status dart_reduce_static(const dart_desc* desc, const void* X, const void* crit,
                               int32_t crit_D, int64_t crit_ld, const int64_t* pos, void* Y,
                               int64_t* pos_out, int32_t* keep, int32_t* cu_keep,
                               int32_t* piv_out, float* S_out, void* stream);

/* Size of the built-in scratch buffer of dart_reduce_static (host arithmetic only). */
DART_API size_t dart_static_scratch_bytes(void);

/* dart_device_status for the last dart_reduce_static call on the current GPU. */
DART_API dart_status dart_device_status_static(const dart_desc* desc, void* stream);

/* One per-token tensor for dart_compact_sequences: rows of row_bytes bytes (a multiple of
 * 16), row r of src at src + r*src_ld_bytes, likewise dst; bases and strides multiples of
 * 16.  src has desc.X_rows rows; dst needs room for the shortened batch. */
typedef struct dart_row_tensor {
  const void* src;      /* DEVICE */
  void* dst;            /* DEVICE, must not overlap src */
  int64_t row_bytes;
  int64_t src_ld_bytes;
  int64_t dst_ld_bytes;
} dart_row_tensor;

/* (d) for whole sequences -- Appendix D: the layers after the step see the text tokens and
 * the retained vision tokens; the key/value rows cached by the layers before it shrink the
 * same way (Table 2, KV-cache column).  Needs desc.span_start.  Sequence b is rows
 * [seq_cu[b], seq_cu[b+1]) of every per-token tensor (seq_cu: DEVICE int32[B+1], from 0 to
 * desc.X_rows, non-decreasing) and must contain its span; keep as produced by dart_reduce /
 * dart_topk_keep for the same descriptor.  Outputs:
 *   seq_cu_out [B+1]  offsets of the shortened sequences (the cu_seqlens a variable-length
 *                     attention kernel takes): sequence b keeps its rows before the span,
 *                     then rows span_start[b] + keep[.] in ascending order, then its rows
 *                     after the span;
 *   row_map [X_rows - total_N + sum of K_b at most]  row_map[r] = the row of the original
 *                     tensors that row r of the shortened batch is a copy of;
 *   tensors[i].dst    the n_tensors (HOST array, may be 0) tensors gathered by row_map, bit
 *                     copies (hidden states, per-layer key and value rows, ...);
 *   pos_out           pos_planes planes of position ids (plane p at pos + p*pos_plane_stride,
 *                     X_rows entries; e.g. 3 planes for multimodal rotary embeddings),
 *                     gathered into pos_out + p*pos_out_plane_stride; pos_planes may be 0.
 * A seq_cu that is not as described, or a span outside its sequence, sets every entry of
 * seq_cu_out to 0, copies nothing and makes dart_device_status report DART_ERR_DEVICE. */
DART_API dart_status dart_compact_sequences(const dart_desc* desc, const int32_t* seq_cu,
                                   const int32_t* keep, int32_t n_tensors,
                                   const dart_row_tensor* tensors, const int64_t* pos,
                                   int32_t pos_planes, int64_t pos_plane_stride, int64_t* pos_out,
                                   int64_t pos_out_plane_stride, int32_t* seq_cu_out,
                                   int32_t* row_map, void* ws, size_t ws_bytes, void* stream);

/* dart_reduce that also stamps the caller's HIP events with the begin and end of its
 * kernels: events is a HOST array of 12 hipEvent_t (as void*, created with timing enabled);
 * events[2k] takes the begin of the first kernel of stage k and events[2k+1] the end of its
 * last kernel (0 row norms, 1 pivot selection, 2 scores, 3 score ordering, 4 retained set,
 * 5 compaction), so hipEventElapsedTime(events[2k], events[2k+1]) is the stage's duration as
 * a kernel trace shows it: the times are the dispatches' own and nothing is enqueued between
 * the kernels.  A stage that launches no kernel for this descriptor (e.g. the ordering under
 * the single-threshold rule, the gather with Y == NULL) leaves its two events untouched.
 * The one-launch path (DART_FUSED=1) is not taken. */
DART_API dart_status dart_reduce_profiled(const dart_desc* desc, const void* X, const void* crit,
                                 int32_t crit_D, int64_t crit_ld, const int64_t* pos, void* Y,
                                 int64_t* pos_out, int32_t* keep, int32_t* cu_keep,
                                 int32_t* piv_out, float* S_out, void* ws, size_t ws_bytes,
                                 void* stream, void* const* events);

/* Waits for `stream`, then reports DART_ERR_DEVICE if the last call that used
 * `ws` (with this descriptor) skipped a ragged sample or met an invalid given pivot
 * list, DART_OK otherwise.  Every entry point that takes `ws` leaves these flags defined:
 * with DART_PIVOT_GIVEN, dart_reduce, dart_duplication_scores and dart_topk_keep validate the
 * piv array they read; an entry point that reads no pivots clears the pivot flag. */
DART_API dart_status dart_device_status(const dart_desc* desc, const void* ws, void* stream);

/* The absolute bound on |fp32 score - exact score| that dart_topk_keep and
 * dart_reduce certify decisions against, for this dtype. */
DART_API double dart_score_tolerance(int32_t dtype);

/* Diagnostic: the raw 32-term sums of the matrix-core instruction the bf16 score path is built
 * on (v_mfma_f32_16x16x32_bf16 from a zero accumulator).  A, B: DEVICE bf16 [tiles][16][32]
 * (k contiguous), out: DEVICE float [tiles][16][16], out[t][i][j] = sum_k A[t][i][k] *
 * B[t][j][k] as the hardware rounds it.  The bound of dart_score_tolerance assumes that this
 * sum errs by at most 16 * 2^-24 * sum_k |A B| (the instruction's internal rounding is not
 * documented); the test-suite checks that assumption through this call on the GPU it runs
 * on.  tiles >= 0; A, B, out 16-byte aligned. */
DART_API dart_status dart_probe_mfma_dot32(const void* A, const void* B, float* out,
                                           int32_t tiles, void* stream);

/* Static, NUL-terminated description of a status code. */
DART_API const char* dart_strerror(dart_status status);

#ifdef __cplusplus
}
#endif
#endif /* DART_H_ */

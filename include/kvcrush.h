/*
 * kvcrush.h -- C ABI of the MI355X (gfx950) KVCrush per-layer KV-cache
 * compression library (KVCrush, arXiv 2503.00022).
 *
 * One layer's compression is three calls on one HIP stream:
 *
 *   kvcrush_scores   attention each cached token receives, per head
 *                    (Alg. 1, attention weights; Sec. 2.3 / 4.1.1: H2O's
 *                    accumulated attention)
 *   kvcrush_select   important tokens (baseline top-n, Sec. 3 first
 *                    paragraph), head-behaviour bit vectors (Alg. 1, Sec. 3.1),
 *                    Hamming grouping and one representative per bucket
 *                    (Alg. 2, Sec. 3.2)
 *   kvcrush_compact  the reduced cache: retained K/V rows gathered into a
 *                    dense layout (Sec. 3.2, last step)
 *
 * Conventions common to every entry point
 *   - All data pointers are DEVICE pointers unless a comment says "host".
 *     The argument structs themselves are host memory, read during the call.
 *   - The caller owns every buffer.  The library allocates, frees and keeps
 *     nothing; scratch memory is passed in as `workspace` whose size the
 *     matching *_workspace() function returns.  Pointers must be 16-byte
 *     aligned.
 *   - Calls only enqueue work on `hip_stream` (a hipStream_t passed as void*)
 *     and return without synchronising.  Outputs are complete when the stream
 *     reaches the end of the enqueued work.  NULL names the legacy default
 *     stream, as it does in every HIP call; the library itself never picks a
 *     stream, so pass your own to stay off the default one.
 *   - Errors are return codes.  Arguments are validated on the host before
 *     anything is launched: INVALID_ARG, UNSUPPORTED and WORKSPACE mean that
 *     nothing has been enqueued.  KVCRUSH_ERR_HIP means that the runtime
 *     refused a launch or a query of THIS call; earlier kernels of the same
 *     call may already be enqueued and the outputs are then unspecified.
 *   - Size limits of the launches (KVCRUSH_ERR_UNSUPPORTED beyond them):
 *     B * Hq <= 65535 and B * Hq * ceil(S / 64) <= 2^30 in the score calls,
 *     B <= 65535 in kvcrush_select and in the gathers (kvcrush_compact,
 *     kvcrush_compact_cache), Hkv + Hs <= 65535 in kvcrush_compact_cache.
 *     kvcrush_select keeps a table of (V + 1) x ceil(n / 1024) x 4 counters in
 *     the LDS of a workgroup, V = Hs * unit bits per vector, n = (S - n_sink -
 *     n_recent) / unit items: at most 30720 counters (Hs = 8: about 870 000
 *     tokens; Hs = 128: about 60 000).  kvcrush_select_workspace returns 0 and
 *     kvcrush_select KVCRUSH_ERR_UNSUPPORTED beyond that.
 *     Offsets inside the arrays are 64-bit: the arrays themselves may exceed
 *     4 GiB.
 *   - Inputs are assumed finite.  NaN scores give an unspecified (but memory
 *     safe) selection.  -0.0 and +0.0 compare equal.
 *   - Overlapping calls that share a workspace race; give each concurrent
 *     stream its own workspace.
 */
#ifndef KVCRUSH_H
#define KVCRUSH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  KVCRUSH_OK = 0,
  KVCRUSH_ERR_INVALID_ARG = 1, /* a size, pointer or enum value is not allowed   */
  KVCRUSH_ERR_UNSUPPORTED = 2, /* legal in the method, not built (e.g. D = 96)   */
  KVCRUSH_ERR_WORKSPACE = 3,   /* workspace NULL or smaller than required        */
  KVCRUSH_ERR_HIP = 4          /* the HIP runtime refused a launch or a query    */
} kvcrush_status;

typedef enum { KVCRUSH_F32 = 0, KVCRUSH_BF16 = 1, KVCRUSH_F16 = 2 /* IEEE half */ } kvcrush_dtype;

/* Anchor vector of Alg. 2: the three strategies it names, plus a caller-supplied one. */
typedef enum {
  KVCRUSH_ANCHOR_RANDOM = 0,      /* word w of sequence b = output w+1 of splitmix64 seeded
                                     with anchor_seed + b, masked to Hs bits           */
  KVCRUSH_ANCHOR_MEAN = 1,        /* bit r = 1 iff more than half of the grouped (non-
                                     important) tokens have bit r set                  */
  KVCRUSH_ANCHOR_ALTERNATING = 2, /* bit r = r & 1 (head 0 -> 0, head 1 -> 1, ...)     */
  KVCRUSH_ANCHOR_EXPLICIT = 3     /* caller supplies anchor_bits                       */
} kvcrush_anchor;

/* Problem shape of one layer.  Query head h reads KV head h / (Hq / Hkv). */
typedef struct {
  int32_t B;             /* independent sequences                                     */
  int32_t Hq;            /* query heads                                               */
  int32_t Hkv;           /* key/value heads, divides Hq                               */
  int32_t S;             /* tokens per sequence (all sequences equal length)          */
  int32_t D;             /* head dimension: 64 or 128                                 */
  int32_t dtype;         /* kvcrush_dtype of Q and K                                  */
  int32_t reduce_groups; /* 1: sum each KV group's query heads -> Hs = Hkv score rows
                            0: one score row per query head    -> Hs = Hq            */
  int32_t obs_window;    /* 0: every query position contributes to the scores.
                            W > 0: only the last min(W, S) query positions do (the
                            observation window of the SnapKV baseline, Sec. 2.3);
                            every score row then totals W instead of S, and lse rows
                            before the window are unspecified / not needed.           */
  float softmax_scale;   /* factor on Q . K before the softmax; 0 means 1 / sqrt(D).
                            Heads of another size are scored by zero-padding them to
                            64 or 128 values and passing 1 / sqrt(true size) here
                            (e.g. 96-value heads: D = 128, softmax_scale = 1/sqrt(96));
                            models with their own attention scale pass that.          */
  int64_t q_stride[3];   /* memory layout of q: elements (not bytes) between consecutive
                            sequences, heads and tokens, in this order; the D values of
                            one (sequence, head, token) are always contiguous.  All three
                            zero: the packed layout [B, Hq, S, D].  A projection output
                            kept token-major, [B, S, Hq, D], is {S*Hq*D, D, Hq*D}; a
                            slice of a longer or padded buffer keeps that buffer's
                            strides.  Each stride is positive and a multiple of 16 bytes,
                            the token stride at least D and at most 2^24 bytes.  Only
                            kvcrush_scores and kvcrush_row_lse read these fields.        */
  int64_t k_stride[3];   /* the same for k ([B, Hkv, S, D] when all zero)                */
} kvcrush_shape;

/* ---------------------------------------------------------------- stage 1 --
 * scores[b, r, t] = sum over the query heads h of row r, and over query
 * positions i >= t, of softmax_i(Q_h K^T / sqrt(D), causal)[t]
 * (Alg. 1's attention weights A_h, accumulated over the queries as H2O does;
 * no 1/S factor; the S x S matrix is never written to memory).
 * Every row of every head sums to one, so each score row totals S (times the
 * group size when reduce_groups = 1).
 *
 *   q       [B, Hq,  S, D]  row-major, D contiguous, dtype as in shape (or any
 *           layout shape->q_stride describes)
 *   k       [B, Hkv, S, D]  (or as shape->k_stride describes)
 *   lse     nullable [B, Hq, S] fp32: natural-log sum-exp of each query row's
 *           scaled causal logits, as an attention forward pass leaves it.
 *           NULL: computed here (one more pass over Q K^T) and left in the
 *           first B*Hq*S floats of the workspace.
 *   scores  [B, Hs, S] fp32, fully overwritten
 *   workspace  kvcrush_scores_workspace(shape) bytes, always required: the
 *           row log-sum-exps first, then partial column sums of long sequences
 * Accuracy: exact bf16 / fp16 (or fp32) products, fp32 accumulation; each score is within
 * 2e-3 relative of the exact value.
 */
size_t kvcrush_scores_workspace(const kvcrush_shape* shape);
kvcrush_status kvcrush_scores(const kvcrush_shape* shape, const void* q, const void* k,
                              const float* lse, float* scores, void* workspace,
                              size_t workspace_bytes, void* hip_stream);

/* First half of stage 1 on its own: lse_out[b, h, i] = natural log of
 * sum_{j <= i} exp(Q_h[i] . K[j] / sqrt(D))  (the normaliser of row i of Alg. 1's
 * A_h), fp32 [B, Hq, S], fully overwritten (with shape->obs_window = W > 0 only
 * the rows i >= S - W are guaranteed to be written; the others are never read).
 * Callers whose attention kernel already produced these values skip this call
 * and hand them to kvcrush_scores as `lse`.  shape->reduce_groups is ignored.
 *
 *   workspace  device scratch of kvcrush_row_lse_workspace(shape) bytes (may be 0),
 *              16-byte aligned, or NULL.  With it, launches that would leave most
 *              of the chip idle (short observation windows, few heads) cut each
 *              row's keys into slices handled by separate workgroups and merge the
 *              slices' sums afterwards; without it every row's keys are walked by
 *              one workgroup.  Both are deterministic; they differ by rounding, and
 *              kvcrush_scores with lse = NULL computes exactly what this call
 *              computes WITH a workspace.
 * Errors: as kvcrush_scores; KVCRUSH_ERR_WORKSPACE if a workspace is given but is
 * too small or misaligned. */
size_t kvcrush_row_lse_workspace(const kvcrush_shape* shape);
kvcrush_status kvcrush_row_lse(const kvcrush_shape* shape, const void* q, const void* k,
                               float* lse_out, void* workspace, size_t workspace_bytes,
                               void* hip_stream);

/* Optional step between stages 1 and 2 for SnapKV-style selection (Sec. 2.3 /
 * 4.1.1: max pooling so that the neighbours of strong tokens are kept too):
 * out[r, t] = max over |u - t| <= kernel / 2, 0 <= u < S, of in[r, u].
 *   in, out  [rows, S] fp32, must not overlap; kernel odd, 1 <= kernel <= 1023. */
kvcrush_status kvcrush_pool_scores(int32_t rows, int32_t S, int32_t kernel, const float* in,
                                   float* out, void* hip_stream);

/* ------------------------------------------------------------ stages 2-4 --
 * Per sequence b, from scores[b] ([Hs, S] fp32):
 *   bits[t] bit r   = 1 iff t is among the bit_topk largest of row r
 *                     (Alg. 1's per-head threshold keeping a fixed fraction)
 *   importance[t]   = ((row0[t] + row1[t]) + row2[t]) + ...  in fp32
 *   important       = the n_important largest importance values
 *   grouped tokens  = all others, N = S - n_important of them
 *   d[t]            = popcount(bits[t] XOR anchor)             (Alg. 2)
 *   buckets         = grouped tokens ordered by (d, t), cut into
 *                     Br = budget - n_important rank ranges
 *                     [floor(j N / Br), floor((j+1) N / Br))
 *   representative  = bucket member with the least summed Hamming distance to
 *                     the bucket's members (nearest the centroid)
 *   idx             = important and representatives merged, ascending
 * Every tie (equal scores, equal costs) goes to the lower token index, so the
 * result is unique for a given score tensor.
 */
typedef struct {
  int32_t B, Hs, S;        /* Hs score rows per sequence, 1 <= Hs <= 1024              */
  int32_t budget;          /* tokens kept per sequence, 0 <= budget <= S               */
  int32_t n_important;     /* 0 <= n_important <= budget; the rest are representatives */
  int32_t bit_topk;        /* per-head top-k that sets a bit; 0 means `budget`         */
  int32_t anchor;          /* kvcrush_anchor                                           */
  int32_t score_stride;    /* floats between consecutive score rows; 0 means S (rows of */
                           /* a capacity-strided decoding cache: capacity)              */
  int32_t n_sink;          /* protected ends (the cache layout of Table 1: initial +   */
  int32_t n_recent;        /* middle + recent tokens): the first n_sink and the last   */
                           /* n_recent tokens are always kept, n_sink + n_recent <=    */
                           /* budget.  The tokens between them are compressed to       */
                           /* budget - n_sink - n_recent tokens exactly as a sequence  */
                           /* of their own: n_important <= that number, bit_topk = 0   */
                           /* means that number, bit_topk <= middle length.  0, 0: off */
  int32_t unit;            /* 0 or 1: tokens are selected.  P > 1: chunk- / page-level  */
                           /* selection (Sec. 4.3.4, 4.3.5) on units of P consecutive   */
                           /* middle tokens: a unit's importance is the sum of its      */
                           /* tokens' importances (token order), its bit vector the     */
                           /* concatenation of its tokens' head vectors (bit j * Hs + r */
                           /* = head r of its j-th token; anchors have Hs * P bits),    */
                           /* and Alg. 2 runs on units.  budget, n_important and the    */
                           /* middle's length stay in tokens and must be multiples of   */
                           /* P; Hs * P <= 1024.  idx lists every token of a kept unit. */
  uint64_t anchor_seed;    /* RANDOM only                                              */
  const uint64_t* anchor_bits; /* EXPLICIT only: device [B, W], W = ceil(Hs / 64)      */
                           /* (ceil(Hs * P / 64) with unit = P > 1)                    */
} kvcrush_select_args;

size_t kvcrush_select_workspace(const kvcrush_select_args* args);
/*   scores  [B, Hs, S] fp32 (rows score_stride floats apart when that is set)
 *   idx     [B, budget] int32, ascending token positions
 *   kind    nullable [B, budget] uint8: 0 kept as important, 1 as representative,
 *           2 protected (n_sink / n_recent)
 *   bits    nullable [B, S, W] uint64: head r is bit r % 64 of word r / 64; zero
 *           words for protected tokens.  With unit = P > 1: [B, Nu, Wu], one
 *           vector of Wu = ceil(Hs * P / 64) words per unit of the middle
 *           (Nu = (S - n_sink - n_recent) / P)
 */
kvcrush_status kvcrush_select(const kvcrush_select_args* args, const float* scores, int32_t* idx,
                              uint8_t* kind, uint64_t* bits, void* workspace,
                              size_t workspace_bytes, void* hip_stream);

/* kvcrush_select for callers that cannot allocate device memory and therefore have
 * no workspace to pass: code running under HIP graph capture, tight serving loops,
 * harnesses that forbid allocation.  Identical arguments and results; the scratch
 * memory is a fixed array of KVCRUSH_SELECT_STATIC_MAX_BYTES inside the library's
 * device image (every GPU the library runs on holds one until the process ends).
 * The call allocates and frees nothing.  The first call on a device looks up the
 * array's address (do that first call outside a capture).
 *   - KVCRUSH_ERR_WORKSPACE when the problem needs more scratch than the array
 *     holds, i.e. when kvcrush_select_workspace(args) exceeds
 *     KVCRUSH_SELECT_STATIC_MAX_BYTES; nothing is enqueued then.
 *   - All calls on one GPU share the array: calls that overlap in time on one GPU
 *     (different streams, different host threads) race.  Calls on one stream, or
 *     otherwise ordered, are safe; nothing needs clearing between them. */
#define KVCRUSH_SELECT_STATIC_MAX_BYTES (4u << 20)
kvcrush_status kvcrush_select_static(const kvcrush_select_args* args, const float* scores,
                                     int32_t* idx, uint8_t* kind, uint64_t* bits,
                                     void* hip_stream);

/* ---------------------------------------------------------------- stage 5 --
 * k_out[b, h, j, :] = K[b, h, idx[b, j], :], same for V (Sec. 3.2: the
 * retained tokens form the final cache).  Pure copy, bit exact.
 *
 *   dense source  (block_table == NULL): k, v [B, Hkv, S, D]
 *   paged source  (block_table != NULL): k, v are pools
 *                 [n_blocks, block_size, Hkv, D]; block_table [B, S / block_size]
 *                 int32 holds the pool block of each logical block;
 *                 S % block_size == 0; entries must be valid pool blocks
 *                 (not checked on the device).
 *   idx     [B, budget] int32 with 0 <= idx < S (as written by kvcrush_select); a value
 *           outside that range is clamped into it, never followed out of the arrays
 *   k_out, v_out [B, Hkv, budget, D], same dtype
 *   D * sizeof(dtype) must be a multiple of 16.
 */
kvcrush_status kvcrush_compact(int32_t B, int32_t Hkv, int32_t S, int32_t D, int32_t dtype,
                               int32_t budget, const void* k, const void* v, const int32_t* idx,
                               const int32_t* block_table, int32_t block_size, void* k_out,
                               void* v_out, void* hip_stream);

/* Page-level eviction on a paged pool (Sec. 4.3.5): when kvcrush_select ran with
 * unit == block_size on a sequence without protected ends, every kept unit is one
 * pool block and the reduced cache needs no copy at all, only its block table:
 *   block_table_out[b, j] = block_table[b, idx[b, j * block_size] / block_size],
 *   j < budget / block_size.
 *   idx          [B, budget] int32 as written by kvcrush_select (whole units)
 *   block_table  [B, S / block_size] int32;  block_table_out [B, budget / block_size]
 * S and budget must be multiples of block_size. */
kvcrush_status kvcrush_compact_block_table(int32_t B, int32_t S, int32_t budget,
                                           int32_t block_size, const int32_t* idx,
                                           const int32_t* block_table, int32_t* block_table_out,
                                           void* hip_stream);

/* ------------------------------------------------------------- decoding --
 * The cache of a sequence that is being generated grows by one token per step
 * (Sec. 1) and the accumulated-attention importance keeps accumulating over
 * those steps (H2O as summarised in Sec. 2.3).  Caches used here are
 * capacity-strided: k, v [B, Hkv, capacity, D] and scores [B, Hs, capacity], of
 * which the first S tokens are valid.
 *
 * kvcrush_scores_append: one decoding step.  shape->S counts the new token (its
 * key is already at position S - 1 of k); q_new [B, Hq, D] holds its queries.
 * For every score row the probabilities softmax_j(q_h . K[j] / sqrt(D)), j < S,
 * of the row's head(s) are added to scores[b, r, 0 .. S-2]; scores[b, r, S-1]
 * (the new token, which had no score) is overwritten with its probability;
 * entries at or beyond S are not touched.  Appending tokens S0+1 .. S one by one
 * to the scores of a prefix of length S0 gives kvcrush_scores of the whole
 * sequence (to rounding).  shape->obs_window must be 0; D in {64, 128}.
 *   lengths    NULL, or device int32 [B]: the number of valid tokens of each
 *              sequence, read by the kernels when they run; shape->S is then
 *              only their upper bound (it sizes the launch and the workspace;
 *              values are clamped to [1, shape->S]).  A serving loop can so
 *              replay one captured launch sequence for every step and for
 *              sequences of different lengths, updating `lengths` on the device.
 *   block_table  NULL: k is dense [B, Hkv, capacity, D].  Otherwise k is a paged
 *              pool [n_blocks, block_size, Hkv, D] (the layout kvcrush_compact
 *              reads) and block_table [B, capacity / block_size] int32 names the
 *              pool block of each logical block; capacity % block_size == 0;
 *              entries must be valid pool blocks (not checked on the device).
 *              scores stay dense [B, Hs, capacity].
 *   workspace  kvcrush_scores_append_workspace(shape, capacity) bytes, 16-byte
 *              aligned (base-2 logits and per-block partial normalisers).
 * Errors as kvcrush_scores.
 */
size_t kvcrush_scores_append_workspace(const kvcrush_shape* shape, int32_t capacity);
kvcrush_status kvcrush_scores_append(const kvcrush_shape* shape, int32_t capacity,
                                     const int32_t* lengths, const void* q_new, const void* k,
                                     const int32_t* block_table, int32_t block_size,
                                     float* scores, void* workspace, size_t workspace_bytes,
                                     void* hip_stream);

/* Eviction while decoding: once kvcrush_select (run on the valid part of the
 * score rows, see kvcrush_select_args.score_stride) has chosen `budget` tokens,
 * they and their running scores move to the front of a second cache:
 *   k_out[b, h, j, :] = k[b, h, idx[b, j], :]  (same for v),
 *   scores_out[b, r, j] = scores[b, r, idx[b, j]],  j < budget.
 * Sources have cap_src tokens per row, destinations cap_dst; only the first
 * `budget` tokens of each destination row are written.  Not in place: outputs
 * must not alias inputs.  0 <= idx < cap_src is the caller's responsibility, as
 * in kvcrush_compact.
 */
kvcrush_status kvcrush_compact_cache(int32_t B, int32_t Hkv, int32_t Hs, int32_t D, int32_t dtype,
                                     int32_t cap_src, int32_t cap_dst, int32_t budget,
                                     const void* k, const void* v, const float* scores,
                                     const int32_t* idx, void* k_out, void* v_out,
                                     float* scores_out, void* hip_stream);

const char* kvcrush_status_string(kvcrush_status status);

/* Library version: 100 * minor + 10 * patch (120 = 0.1.2); changes whenever a struct or
 * a signature of this header changes. */
int32_t kvcrush_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KVCRUSH_H */

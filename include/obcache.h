/*
 * obcache.h -- C ABI of the MI355X (gfx950) OBCache hot path.
 *
 * Implements, for one attention layer, the data-parallel part of
 * "OBCache: Optimal Brain KV Cache Pruning" (arxiv 2510.07651):
 *
 *   obc_score   window attention of the last W queries against all cached keys
 *               (Section 3: Z = QK^T/sqrt(d), A = softmax(Z), O = AV), then the
 *               closed-form saliency scores of Propositions 1-3 (Eq. 4-6) summed
 *               over the perturbation window (Eq. 9) and over the query heads of
 *               each KV head (Appendix A.5);
 *   obc_select  per (sequence, KV head) top-`budget` tokens by score, kept
 *               indices in ascending order (Section 3 "Cache Eviction";
 *               Appendix E, Algorithm 2: topk then sort);
 *   obc_compact gather of the surviving K and V rows (Algorithm 2: gather).
 *
 * General conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller unless its name
 *     ends in `_host`.  Tensors are contiguous, row-major, in the stated shape;
 *     q, k, v and the compacted outputs start on 16-byte boundaries (OBC_EINVAL
 *     otherwise), fp32 and int32 arrays on 4-byte boundaries.
 *   - Nothing here allocates, frees or synchronises.  All work is enqueued on
 *     `hip_stream` (a hipStream_t passed as void*; NULL = the default stream).
 *     Outputs are valid once that stream has reached the end of the call's work.
 *     A call only launches kernels (no memset, no copy), so it may be made while
 *     `hip_stream` is being captured into a HIP graph; the lengths in
 *     `seq_lens_host` are then baked into the captured launches.  No call
 *     configures anything on first use, so a capture needs no warm-up call.
 *   - `seq_lens_host` is a HOST array of B true lengths (W <= len_b <= N, at
 *     most OBC_MAX_RAGGED_BATCH entries) read before the call returns, or NULL
 *     when every sequence has length N.  The W window queries of sequence b sit
 *     at absolute positions len_b-W .. len_b-1; query row r sees keys
 *     p <= len_b-W+r.  Rows p >= len_b of k and v are never interpreted (they may
 *     hold anything, NaN included).
 *   - Query head h reads KV head h / (Hq/Hkv).
 *   - Return value: OBC_OK or a negative obc_status_t.  Argument errors are
 *     detected on the host before anything is launched.
 *   - Same inputs give bit-identical outputs (no floating-point atomics).
 *   - The library targets gfx950 only and has no CPU fallback.
 *   - obc_score picks its kernels from the shapes: bf16 with head_dim 128 runs on the matrix
 *     cores; a one-row window (W = 1, the decoding case) over a bf16 cache of up to ~1e5
 *     head-tokens runs on kernels shaped for memory round trips; everything else (fp32,
 *     bf16 with head_dim 64 and W > 1) on general vector-ALU kernels.  The routing depends
 *     on the arguments only (and on obc_set_score_path, a test hook declared at the end of
 *     this file); the process environment is never read.
 */
#ifndef OBCACHE_H_
#define OBCACHE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    OBC_OK = 0,
    OBC_EINVAL = -1,        /* null pointer, non-positive size, Hq % Hkv != 0, W > len, budget > len ... */
    OBC_EUNSUPPORTED = -2,  /* head_dim / dtype / window / batch outside what the kernels are built for */
    OBC_EWORKSPACE = -3,    /* workspace missing, misaligned (256 B) or too small */
    OBC_ELAUNCH = -4        /* the HIP runtime reported an error when enqueuing */
} obc_status_t;

typedef enum {
    OBC_VALUE = 0,  /* Eq. 4: sum_i A_ip^2 ||v_p||^2 */
    OBC_KEY = 1,    /* Eq. 5: sum_i A_ip^2 Z_ip^2 ||v_p - o_i||^2 */
    OBC_JOINT = 2,  /* Eq. 6: value + key + 2 sum_i A_ip^2 Z_ip (||v_p||^2 - v_p.o_i) */
    OBC_ALL = 3,    /* all three; scores is [3][B][Hkv][N] in the order value, key, joint */
    OBC_ATTN = 4,   /* Eq. 8 (Section 4.3): sum_i |A_ip|, the attention-only score the method generalises */
    OBC_VATP = 5    /* Appendix C, "VATP": the value score with the l1 norm, sum_i |A_ip| ||v_p||_1 */
} obc_variant_t;

typedef enum {
    OBC_F32 = 0,   /* q,k,v fp32; head_dim 64 or 128; fp32 arithmetic */
    OBC_BF16 = 1   /* q,k,v bf16; head_dim 64 or 128; fp32 accumulation */
} obc_dtype_t;

#define OBC_MAX_RAGGED_BATCH 128  /* largest B accepted together with seq_lens_host */
#define OBC_MAX_WINDOW 64         /* largest W */
#define OBC_MAX_GROUP_ROWS 512    /* largest (Hq/Hkv) * W */

/*
 * Bytes of device workspace obc_score needs for these sizes (Section 3's O and
 * softmax statistics of the window rows, plus split-sequence partial results).
 * *bytes_out is a multiple of 256.  Host-only; returns OBC_EINVAL /
 * OBC_EUNSUPPORTED like obc_score would for the same sizes.
 */
int obc_score_workspace_bytes(int B, int N, int W, int Hq, int Hkv, int d,
                              int dtype, int variant, size_t *bytes_out);

/*
 * Saliency scores (Propositions 1-3 / Eq. 4-6, windowed per Eq. 9, GQA-summed per
 * Appendix A.5).
 *   q        [B, Hq, W, d]   the last W query rows of every sequence
 *   k, v     [B, Hkv, N, d]  the KV cache (N = padded length)
 *   scores   [B, Hkv, N] fp32 (or [3, B, Hkv, N] for OBC_ALL), written in full:
 *            positions p >= len_b get 0.  Must not alias the inputs.
 *   workspace  >= obc_score_workspace_bytes(...) bytes, 256-byte aligned; its
 *            contents are scratch (overwritten, no state carried between calls).
 * Z in Eq. 5-6 is the raw scaled logit q.k/sqrt(d).  (query, key) pairs hidden by
 * the causal mask contribute exactly 0.  NaN/Inf inside the first len_b rows give
 * undefined scores.
 */
int obc_score(const void *q, const void *k, const void *v,
              int N, int W, int Hq, int Hkv, int d, int variant, float *scores,
              int B, int dtype, const int32_t *seq_lens_host,
              void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Decoding-time accumulation (Section 4.2, closing remark: during decoding the scores are
 * accumulated over time; Appendix C, decoding setup: an eviction decision at every step).
 * Same arguments as obc_score, but the scores of this call are ADDED to what `scores`
 * already holds: scores[b,g,p] += S_p for p < len_b, and positions p >= len_b are left
 * untouched (they belong to tokens that do not exist yet).  A decode step passes the new
 * token's query with W = 1 and len_b = its position + 1; by Eq. 9 the score of a W-row
 * window equals the sum of the W single-row calls with growing length.
 */
int obc_score_accumulate(const void *q, const void *k, const void *v,
                         int N, int W, int Hq, int Hkv, int d, int variant, float *scores,
                         int B, int dtype, const int32_t *seq_lens_host,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * For callers that cannot allocate or size a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid device allocation.  obc_score (accumulate = 0) or
 * obc_score_accumulate (accumulate = 1) with the library's own scratch in place of the
 * `workspace` argument: a device array of OBC_STATIC_SCRATCH_BYTES that is part of the loaded
 * library (one copy per GPU, held until the process ends).  Same inputs, outputs, checks and
 * results as those calls; nothing is allocated, freed, copied or synchronised.
 *   - Shapes whose obc_score_workspace_bytes exceeds OBC_STATIC_SCRATCH_BYTES are rejected with
 *     OBC_EWORKSPACE before anything is launched (the metric's workload, 4 x 32768 tokens of a
 *     32/8-head layer, needs ~35 MiB and fits; decode steps need well under 1 MiB).
 *   - Every call on one GPU shares that GPU's array.  The scratch carries no state between
 *     calls (each call overwrites what it reads), but two calls in flight on the same GPU at
 *     the same time (different streams, or graphs replayed concurrently) race on it: keep calls
 *     of this entry point on one GPU ordered.
 *   - obc_init() looks the array's device address up for the current device (once per device);
 *     without it the first obc_score_static call on a device does so itself.  Call obc_init()
 *     before capturing a graph that contains this call.  OBC_ELAUNCH if the lookup fails.
 */
#define OBC_STATIC_SCRATCH_BYTES (48u << 20)
int obc_init(void);
int obc_score_static(const void *q, const void *k, const void *v,
                     int N, int W, int Hq, int Hkv, int d, int variant, float *scores,
                     int B, int dtype, const int32_t *seq_lens_host, int accumulate, void *hip_stream);

/*
 * Optional workspace of the three selection calls below.  Heads longer than 32768 tokens
 * do not fit one block's registers; given *bytes_out bytes of 256-byte aligned device
 * scratch their selection is cut into slices of 8192 tokens that run on separate blocks.
 * *bytes_out is 0 for shapes that do not profit.  The results do not depend on whether the
 * workspace is given.
 */
int obc_select_workspace_bytes(int B, int Hkv, int N, size_t *bytes_out);

/*
 * Top-`budget` selection per (b, KV head) (Section 3 "Cache Eviction";
 * Algorithm 2).
 *   scores    [B, Hkv, N] fp32
 *   keep_idx  [B, Hkv, budget] int32, ascending token indices of the `budget`
 *             highest scores among p < len_b; equal scores are won by the lower
 *             index; -0.0 equals +0.0; NaN ranks below every number.
 *   workspace NULL, or obc_select_workspace_bytes(...) bytes of scratch (a smaller one is
 *             ignored; a misaligned one is OBC_EWORKSPACE).
 * Requires 1 <= budget <= len_b for every b.
 */
int obc_select(const float *scores, int budget, int32_t *keep_idx,
               int B, int Hkv, int N, const int32_t *seq_lens_host,
               void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Selection with protected regions (Appendix E, Algorithm 2: only positions below
 * cutoff = len_b - num_recent + num_coming compete for the num_hh heavy-hitter slots and
 * the tail [cutoff, len_b) is always kept; Appendix C, decoding setup: the first tokens are
 * always kept as attention sinks).  Per (b, KV head) the kept set is
 *   {0 .. num_sinks-1}  +  the num_hh highest scores among num_sinks <= p < cutoff
 *   (ties: lowest index)  +  {cutoff .. len_b-1},
 * written ascending to keep_idx [B, Hkv, num_sinks + num_hh + num_recent - num_coming];
 * obc_compact with these indices yields Algorithm 2's [heavy hitters ; recent rows].
 * num_sinks = num_recent = num_coming = 0 is obc_select.  Requires
 * 0 <= num_coming <= num_recent, num_hh >= 0, num_sinks >= 0, a non-empty kept set, and
 * num_sinks + num_hh <= cutoff for every sequence.  Scores and ordering as in obc_select.
 */
int obc_select_protected(const float *scores, int num_hh, int num_sinks, int num_recent, int num_coming,
                         int32_t *keep_idx, int B, int Hkv, int N, const int32_t *seq_lens_host,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Pooled selection (Appendix C, "SnapKV": the scores are smoothed by a one-dimensional
 * average-pooling filter, kernel size 5 in the paper's experiments, before eviction).
 * Same kept set and output as obc_select_protected, but the competing tokens
 * num_sinks <= p < cutoff are ranked by the sum of the scores in their centred window of
 * `pool` positions (stride 1; positions outside the competing range count as zero).  The
 * sum is taken in fp32 in ascending position order; it ranks tokens as the average does
 * and involves no division.  `pool` is odd, 1 <= pool <= OBC_MAX_POOL; pool = 1 is
 * obc_select_protected.  `scores` itself is not modified.
 */
#define OBC_MAX_POOL 15
int obc_select_pooled(const float *scores, int num_hh, int num_sinks, int num_recent, int num_coming, int pool,
                      int32_t *keep_idx, int B, int Hkv, int N, const int32_t *seq_lens_host,
                      void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Head-adaptive selection (Appendix C, "AdaKV": head-wise budgets from a global ranking of
 * the scores across all heads of the layer, with a safeguard, 0.2 in the paper's
 * experiments).  Per sequence the layer keeps Hkv * budget tokens: every KV head first
 * keeps its own n_safe best (the safeguard; floor(0.2 * budget) reproduces the paper's
 * setting), and the remaining Hkv * (budget - n_safe) slots go to the highest scores among
 * all other live (head, token) pairs; equal scores are won by the lower head, then the
 * lower index.  Outputs, per (b, KV head):
 *   counts    [B, Hkv] int32       tokens kept by this head (their sum over the heads of a
 *                                  sequence is Hkv * budget)
 *   keep_idx  [B, Hkv, cap] int32  their indices, ascending, followed by -1
 * `cap` must hold the most one head can receive, min(len_b, Hkv*budget - (Hkv-1)*n_safe).
 * obc_compact turns the -1 entries into all-zero rows.  n_safe = budget is obc_select.
 * Requires 0 <= n_safe <= budget <= len_b and a workspace of
 * obc_select_adaptive_workspace_bytes(...) bytes, 256-byte aligned.
 */
int obc_select_adaptive_workspace_bytes(int B, int Hkv, int N, int budget, int n_safe, size_t *bytes_out);
int obc_select_adaptive(const float *scores, int budget, int n_safe, int32_t *keep_idx, int32_t *counts, int cap,
                        int B, int Hkv, int N, const int32_t *seq_lens_host,
                        void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Compaction (Algorithm 2's gather; with indices from obc_select_protected the recent rows come along):
 *   k_out[b,g,j,:] = k[b,g,keep_idx[b,g,j],:]   and the same for v.
 *   k, v          [B, Hkv, N, d] of `dtype`
 *   keep_idx      [B, Hkv, budget] int32, entries in [0, N), or -1 for an all-zero
 *                 output row (the padding of obc_select_adaptive's lists).  Device data,
 *                 not checked on the host: entries >= N are clamped to N-1.
 *   k_out, v_out  [B, Hkv, budget, d]; must not overlap k, v.
 * d * element size must be a multiple of 16 bytes.
 */
int obc_compact(const void *k, const void *v, const int32_t *keep_idx,
                void *k_out, void *v_out,
                int B, int Hkv, int N, int budget, int d, int dtype, void *hip_stream);

/*
 * Compaction where the cache lies (the specialised eviction kernel Appendix D asks for in
 * place of gather + concatenate; Section 4.2, closing remark: an eviction at every decode
 * step):
 *   k[b,g,j,:] = k[b,g,keep_idx[b,g,j],:]  for j < budget, the same for v, and, when
 *   `scores` is not NULL, scores[b,g,j] = scores[b,g,keep_idx[b,g,j]] for j < budget and
 *   scores[b,g,j] = 0 for budget <= j < N (slots of tokens still to come).
 *   k, v      [B, Hkv, N, d] of `dtype`, updated in place; rows budget..N-1 keep their old
 *             (now stale) contents.
 *   scores    [B, Hkv, N] fp32 or NULL.
 *   keep_idx  [B, Hkv, budget] int32, per head strictly ascending as every obc_select*
 *             call returns it (so keep_idx[j] >= j), optionally followed by -1 entries,
 *             which give all-zero rows and zero scores.  Device data, not checked: entries
 *             >= N are clamped to N-1; for a list that is not ascending the call stays
 *             inside the buffers but the result is unspecified.
 * Rows that already sit in their place (keep_idx[j] == j) are not rewritten.
 * d * element size must be a multiple of 16 bytes; B * Hkv <= 65535.
 */
int obc_compact_inplace(void *k, void *v, float *scores, const int32_t *keep_idx,
                        int B, int Hkv, int N, int budget, int d, int dtype, void *hip_stream);

/*
 * One decoding step in one call (Section 4.2, closing remark: scores accumulate over the decoding steps; Appendix C,
 * decoding setup: an eviction decision at every step, the first tokens kept as attention sinks and the most recent
 * ones kept as well; Appendix D asks for specialised kernels for score computation and cache eviction).  Equivalent
 * to, on the same stream,
 *   obc_score_accumulate(q, k, v, W = 1, ...)                          the new token's query row against len_b rows,
 *   obc_select_protected(num_hh = len_b - 1 - num_sinks - num_recent)  every competing token but one is kept,
 *   obc_compact_inplace(k, v, scores, that list)                       the gap is closed in place,
 * without forming the index lists: per (b, KV head) the dropped token is the one with the lowest running score among
 * num_sinks <= p < len_b - num_recent, the highest index among equal scores (selection lets the lower index win a
 * tie; -0 equals +0, NaN ranks lowest); rows and scores after it move down by one and scores[len_b - 1 .. N) become 0.
 *   q        [B, Hq, 1, d]    k, v  [B, Hkv, N, d], updated in place (row len_b - 1 keeps a stale copy)
 *   scores   [B, Hkv, N] fp32 running scores, updated in place
 *   evicted  [B, Hkv] int32 (device) receives the dropped positions; may be NULL
 *   variant  any single score (not OBC_ALL)
 * Requires num_sinks + num_recent < len_b for every sequence and a workspace of obc_decode_step_workspace_bytes(...)
 * bytes, 256-byte aligned.  Argument errors are found before anything is launched.
 */
int obc_decode_step_workspace_bytes(int B, int N, int Hq, int Hkv, int d, int dtype, int variant, size_t *bytes_out);
int obc_decode_step(const void *q, void *k, void *v, float *scores, int32_t *evicted,
                    int N, int Hq, int Hkv, int d, int variant, int B, int dtype, const int32_t *seq_lens_host,
                    int num_sinks, int num_recent, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Running scores follow their tokens through an eviction (Section 4.2, closing remark, and
 * Appendix C, decoding setup: scores accumulate over time and an eviction is made at every
 * step, so a kept token keeps its accumulated score):
 *   scores_out[b,g,j] = scores[b,g,keep_idx[b,g,j]]  for j < budget,   0 for budget <= j < N_out.
 *   scores      [B, Hkv, N] fp32        keep_idx [B, Hkv, budget] int32 (as for obc_compact)
 *   scores_out  [B, Hkv, N_out] fp32, N_out >= budget; must not overlap scores.
 * The zero tail leaves room for the tokens still to come in a cache of N_out slots.
 */
int obc_compact_scores(const float *scores, const int32_t *keep_idx, float *scores_out,
                       int B, int Hkv, int N, int budget, int N_out, void *hip_stream);

/* ------------------------------------------------------------------------------------
 * Measurement and test hooks.  None of these is part of the method; a caller of the
 * library needs none of them.  They exist so that the benchmark can time single kernels
 * and the tests can compare the scoring paths with each other.
 * ------------------------------------------------------------------------------------ */

/*
 * Measurement hook: obc_score restricted to some of its stages, so that each kernel
 * of the two-sweep scoring path can be timed on its own with events around the call.
 * Same arguments and checks as obc_score; `stage_mask` is a bit set of
 *   OBC_STAGE_SWEEP1   window attention statistics and outputs (Section 3), per sequence split
 *   OBC_STAGE_COMBINE  merge of the splits into per-row constants
 *   OBC_STAGE_SWEEP2   the scores of Eq. 4-6 from those constants
 * A later stage reads what the earlier ones left in `workspace`, so the first call on a
 * workspace must include all earlier stages.  obc_score == all three.
 */
#define OBC_STAGE_SWEEP1 1
#define OBC_STAGE_COMBINE 2
#define OBC_STAGE_SWEEP2 4
#define OBC_STAGE_ALL 7
int obc_score_stages(const void *q, const void *k, const void *v,
                     int N, int W, int Hq, int Hkv, int d, int variant, float *scores,
                     int B, int dtype, const int32_t *seq_lens_host,
                     void *workspace, size_t workspace_bytes, void *hip_stream, int stage_mask);

/*
 * Measurement hook (not part of the method): reads `bytes` bytes (a multiple of 16, 16-byte
 * aligned, device) once with 128-bit loads and writes one folded word per thread to
 * `sink` (device, OBC_PROBE_BLOCKS * 256 uint32).  Timed with events around the call it
 * gives the streaming-read rate this GPU actually sustains, which the benchmark prints
 * next to the nominal HBM peak.
 */
#define OBC_PROBE_BLOCKS 2048
int obc_probe_read_bandwidth(const void *buf, size_t bytes, uint32_t *sink, void *hip_stream);

/*
 * Test hook: pins the kernels obc_score* uses, process-wide, for every later size query and
 * scoring call (both read the same setting, so a workspace sized by obc_score_workspace_bytes
 * always fits the call that follows unless the setting is changed in between).
 *   OBC_PATH_AUTO    routing by shape (the default)
 *   OBC_PATH_PLAIN   the general vector-ALU kernels for every shape
 *   OBC_PATH_MFMA    one-row windows stay on the matrix-core kernels
 *   OBC_PATH_DECODE  one-row windows go to the decode kernels whatever the cache size
 * Returns OBC_EINVAL for any other value.  Results of all paths agree within the dtype's tolerance.
 */
typedef enum { OBC_PATH_AUTO = 0, OBC_PATH_PLAIN = 1, OBC_PATH_MFMA = 2, OBC_PATH_DECODE = 3 } obc_path_t;
int obc_set_score_path(int path);

/*
 * Tuning hook: forces the number of sequence splits of the first sweep and the token range of
 * one workgroup of the second sweep (a multiple of 64 in [64, 65536]) on the matrix-core path,
 * process-wide; 0 restores the automatic choice.  Values a shape cannot take are ignored for it.
 */
int obc_set_score_tuning(int splits, int range_len);

/*
 * Test hook: form of the matrix-core path's second sweep for the variants with a cross term (key, joint, all),
 * process-wide.  0: chosen by shape; 1: 32 window rows per wave, two workgroups per compute unit; 2: 64 rows per
 * wave with the stationary operands in the accumulator registers, one workgroup per compute unit, wherever the
 * row count allows (every 128-row chunk at least three quarters full).  Both forms meet the same tolerance; their
 * sums run in different orders, so their low bits differ.
 */
int obc_set_sweep2_form(int form);

/* Static, human-readable name of a status code. */
const char *obc_status_string(int status);

/* Library ABI version (major * 100 + minor). */
int obc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* OBCACHE_H_ */

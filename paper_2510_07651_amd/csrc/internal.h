// Internal declarations shared by the translation units of libobcache (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "obcache.h"

namespace obc {

// True lengths travel to the kernels by value (kernel-argument memory), so the
// library needs no device allocation and no host-to-device copy of its own.
struct SeqLens {
    int32_t len[OBC_MAX_RAGGED_BATCH];
};

struct ScoreArgs {
    const void *q, *k, *v;
    float *scores;
    int B, N, W, Hq, Hkv, d, G;
    int variant;      // obc_variant_t
    int dtype;        // obc_dtype_t
    int ragged;       // 0: every sequence has length N
    int stage_mask;   // OBC_STAGE_* bits to run
    int accumulate;   // 1: add to the scores already in `scores` (positions beyond the true length untouched)
    SeqLens lens;     // valid for b < B when ragged
};

// Workspace carve-up for obc_score; offsets in bytes from a 256-byte aligned base.
struct ScoreWorkspace {
    size_t row_max;    // float [B*Hq*W]      max over visible keys of the scaled logit (natural log units)
    size_t row_sum;    // float [B*Hq*W]      sum over visible keys of exp(z - row_max)
    size_t out_f32;    // float [B*Hq*W*d]    o_i = sum_p A_ip v_p
    size_t out_rest_f32;  // float [B*Hq*W*d] attention output of the row over every key but its top-logit one
    size_t rest_frac;  // float [B*Hq*W]      1 - A_{i,p*}: share of the row's attention not on its top-logit key
    size_t top_token;  // int32 [B*Hq*W]      p*: lowest index among the keys attaining the row max
    size_t out_bf16;   // bf16  [2][B*Hkv*m_pad*d]  o_i as two bf16 pieces (high, residual); rows of a KV head padded to a multiple of 32
    size_t row_const;  // float [B*Hkv*m_pad*4]  per padded row: 2*(max + log2 sum) in log2 units, ||o||^2, last visible key, spare
    size_t part_ml;    // float [B*Hkv*splits*m_pad*4]  per sequence split: row max (raw q.k), row sum, spare x2
    size_t special;    // float [B*Hkv*m_pad*4]  per padded row: separately scored top key (token or -1) and its value/key/joint terms
    size_t part_o;     // float [B*Hkv*splits*m_pad*d]  per sequence split: unnormalised output
    size_t planes;     // float [n_chunks*nv*B*Hkv*N]   per row-chunk partial scores (only when n_chunks > 1)
    size_t total;
    int m_pad;         // padded rows per KV head (multiple of 32)
    int n_chunks;      // row chunks of 128 rows per KV head
    int splits;        // sequence splits in the first sweep
    int split_len;     // tokens per split (multiple of 64)
    int range_len;     // tokens per workgroup in the second sweep (multiple of 64)
    int use_mfma;      // 1: matrix-core path, 0: plain path
    int use_wide;      // 1: the second sweep runs in its register-blocked form (score_mfma_wide.hip)
    // Decode path (one window row per query head): see score_decode.hip.
    size_t dec_z;      // float [B*Hkv*N*dec_rows]  scaled logits, token-major
    size_t dec_part;   // float [B*Hkv*dec_splits*dec_rows*(d+4)]  per-range partial records
    size_t dec_final;  // float [B*Hkv*dec_rows*(2d+4)]  merged row records
    int use_decode;    // 1: decode path (takes precedence over the other two)
    int dec_rows;      // query heads per KV head, padded to 1, 2, 4 or 8
    int dec_range;     // tokens per workgroup (multiple of 32)
    int dec_splits;    // ranges per KV head
    int dec_merge_inline;  // 1: the scoring kernel merges the ranges itself
};

constexpr int kDecodeMaxGroup = 8;   // query heads per KV head the decode path is built for

// Sweep-1 split count and sweep-2 token range forced through obc_set_score_tuning (0: automatic).
int tuned_splits();
int tuned_range();
int tuned_sweep2_form();     // 0: by shape, 1: 32 rows per wave, 2: 64 rows per wave where the shape allows

int plan_score_workspace(int B, int N, int W, int Hq, int Hkv, int d, int dtype, int variant, ScoreWorkspace *ws);
// Adds the matrix-core path's buffers to the plan, advancing *off (bytes).
void mfma_plan(int B, int N, int W, int Hq, int Hkv, int d, int variant, ScoreWorkspace *ws, size_t *off);

// Decode path: whether it covers the shape, its buffers (advancing *off), its launcher.
bool decode_path_covers(int B, int N, int W, int Hq, int Hkv, int d, int dtype, int variant, bool any_size);
void decode_plan(int B, int N, int Hq, int Hkv, int d, ScoreWorkspace *ws, size_t *off);
hipError_t launch_score_decode(const ScoreArgs &a, const ScoreWorkspace &ws, char *ws_base, hipStream_t stream);

// Launchers.  Each enqueues on `stream` and returns hipSuccess or the launch error.
hipError_t launch_score_plain(const ScoreArgs &a, const ScoreWorkspace &ws, char *ws_base, hipStream_t stream);
hipError_t launch_score_mfma(const ScoreArgs &a, const ScoreWorkspace &ws, char *ws_base, hipStream_t stream);
// Register-blocked second sweep: whether it serves the variant and row count, and its launcher (same arguments
// and outputs as the 32-rows-per-wave kernel it stands in for).
bool sweep2_wide_covers(int variant, int m_pad, int M);
hipError_t launch_sweep2_wide(const ScoreArgs &a, const ScoreWorkspace &ws, char *base, float *dst, size_t plane_elems,
                              size_t chunk_stride, hipStream_t stream);
hipError_t launch_select(const float *scores, int budget, int32_t *keep_idx, int B, int Hkv, int N, int ragged,
                         const SeqLens &lens, int first, int tail, int radius, void *workspace,
                         size_t workspace_bytes, hipStream_t stream, int keys_in = 0);
size_t select_adaptive_workspace_bytes(int B, int Hkv, int N, int budget, int n_safe);
hipError_t launch_select_adaptive(const float *scores, int budget, int n_safe, int cap, int32_t *keep_idx,
                                  int32_t *counts, int B, int Hkv, int N, int ragged, const SeqLens &lens,
                                  void *workspace, hipStream_t stream);
size_t select_workspace_bytes(int B, int Hkv, int N);
bool select_prefers_slices(int B, int Hkv, int N);
hipError_t launch_compact(const void *k, const void *v, const int32_t *keep_idx, void *k_out, void *v_out, int B,
                          int Hkv, int N, int budget, int row_bytes, hipStream_t stream);
hipError_t launch_compact_in_place(void *k, void *v, float *scores, const int32_t *keep_idx, int B, int Hkv, int N,
                                   int budget, int row_bytes, hipStream_t stream);
// Evict-one of a decoding step: picks, per (sequence, KV head), the lowest-scored token among first <= p < len - tail
// (ties: the highest index) into `evicted`, then closes the gap in k, v and scores.
hipError_t launch_evict_one(void *k, void *v, float *scores, int32_t *evicted, int B, int Hkv, int N, int ragged,
                            const SeqLens &lens, int first, int tail, int row_bytes, hipStream_t stream);
hipError_t launch_gather_scores(const float *in, const int32_t *keep_idx, float *out, int BH, int N, int budget,
                                 int n_out, hipStream_t stream);
hipError_t launch_stream_read(const void *src, size_t bytes, uint32_t *sink, int blocks, hipStream_t stream);

__device__ __forceinline__ int seq_len_of(const SeqLens &lens, int ragged, int b, int N) {
    return ragged ? lens.len[b] : N;
}

__device__ __forceinline__ float bf16_bits_to_float(uint16_t h) {
    return __uint_as_float(((uint32_t)h) << 16);
}

}  // namespace obc

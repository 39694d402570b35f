// Decode-time scoring: a perturbation window of ONE query row per head (W = 1, the setting
// Section 3.2 and Appendix C use while generating), bf16 cache.
//
// With one row per query head a KV head sees only G = Hq/Hkv rows, far too few to fill a
// matrix-core tile, and at the cache sizes of decoding the call is bound by memory round
// trips, not by bandwidth.  The path is vector-ALU kernels with 128-bit coalesced loads (one
// token row spread over d/8 lanes) in which a workgroup owns a short range of tokens and every
// lane issues ALL its loads of the range before it computes:
//   decode_partial   per range: scaled logits Z = q.k/sqrt(d) (Section 3), kept in the
//                    workspace so K is read once; range max, sum and unnormalised output
//                    (the range's top-logit token is held out of both sums, see below)
//   decode_merge     per KV head: log-sum-exp merge of the ranges into the row max, 1/sum,
//                    o_i and v_p* - o_i (folded into decode_score when the ranges are few)
//   decode_score     Eq. 4-6 in their direct forms ||v_p||^2, ||v_p - o_i||^2 and
//                    ||v_p + Z (v_p - o_i)||^2 (the completed square of Eq. 6), Eq. 8 and
//                    the l1-weighted variant of Appendix C, summed over the query heads of
//                    the KV head (Appendix A.5), written or added to the running scores.
//
// Cancellation guard.  When one key takes almost all of a row's attention, o_i is almost
// v_p* and fp32 cannot hold their difference.  Every range keeps its top-logit token out of
// its sums; the merge adds the held-out tokens of all ranges but the winning one back, so
// with l' and o' the sum and the mean over every key but p*,
//     v_p* - o_i = (l' / (1 + l')) (v_p* - o')        (no cancellation)
//     o_i        = v_p* - (v_p* - o_i)
// and the (row, p*) pair is scored from the first identity.
// Every sum runs in a fixed order: results are bit-reproducible.
#include "internal.h"

namespace obc {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kSteps = 8;            // token rows per lane: a range is kSteps workgroup-wide steps
constexpr int kRecHead = 4;          // floats ahead of the vectors in a partial or final record
constexpr int kInlineSplits = 16;    // most ranges per head the scoring kernel merges itself
constexpr int kMergeThreads = 1024;
constexpr int kMergeOwn = 4;         // ranges per merging thread
constexpr int kMaxSplits = kMergeThreads * kMergeOwn;

__host__ __device__ constexpr int tokens_per_step(int d) { return kWaves * (64 / (d / 8)); }
__host__ __device__ constexpr int range_tokens(int d) { return kSteps * tokens_per_step(d); }
// Partial record of (KV head, range, row): {range max, sum without the top token, top token
// (int bits, -1 for an empty range), spare, unnormalised output without the top token [d]}.
__host__ __device__ constexpr int part_stride(int d) { return d + kRecHead; }
// Final record of (KV head, row): {row max, 1/sum, top token (int bits), spare, o_i [d],
// v_p* - o_i [d]}.
__host__ __device__ constexpr int final_stride(int d) { return 2 * d + kRecHead; }

__device__ __forceinline__ void unpack8(const uint4 w, float *x) {
    x[0] = __uint_as_float(w.x << 16); x[1] = __uint_as_float(w.x & 0xffff0000u);
    x[2] = __uint_as_float(w.y << 16); x[3] = __uint_as_float(w.y & 0xffff0000u);
    x[4] = __uint_as_float(w.z << 16); x[5] = __uint_as_float(w.z & 0xffff0000u);
    x[6] = __uint_as_float(w.w << 16); x[7] = __uint_as_float(w.w & 0xffff0000u);
}

// x + (x of the lane a data-parallel-primitive control pairs this lane with); register-to-register,
// no trip through LDS.  Call with every lane of the wave active.
template <int kCtrl>
__device__ __forceinline__ float dpp_pair_sum(float x) {
    const int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), kCtrl, 0xf, 0xf, false);
    return x + __int_as_float(y);
}
// Sum over the `kLanes` (8 or 16) consecutive lanes that share a token; all of them end with the
// same bits.  Lane pairings: neighbours, neighbouring pairs (quad permutes 1032 and 2301), then
// the mirror image inside each half row of 8 lanes and inside each row of 16.
template <int kLanes>
__device__ __forceinline__ float group_sum(float x) {
    x = dpp_pair_sum<0xB1>(x);
    x = dpp_pair_sum<0x4E>(x);
    x = dpp_pair_sum<0x141>(x);
    if (kLanes == 16) x = dpp_pair_sum<0x140>(x);
    return x;
}
// Butterfly sum over the token slots of a wave (lanes with equal position inside their group).
template <int kLanes>
__device__ __forceinline__ float slot_sum(float x) {
#pragma unroll
    for (int off = kLanes; off < 64; off <<= 1) x += __shfl_xor(x, off);
    return x;
}
// (larger value, lower index on ties) of two candidates.
__device__ __forceinline__ void take_better(float &bm, int &ba, float om, int oa) {
    if (om > bm || (om == bm && oa < ba)) { bm = om; ba = oa; }
}

// Token of step u for this lane: steps interleave the waves so that a step of the workgroup
// covers consecutive rows.
template <int kD>
__device__ __forceinline__ int token_of(int t0, int u, int wave, int slot) {
    return t0 + u * tokens_per_step(kD) + wave * (64 / (kD / 8)) + slot;
}

// The scaled logits of the range, its row maxima and the unnormalised sums around them.
template <int kG, int kD, bool kNeedO>
__global__ __launch_bounds__(kThreads) void decode_partial(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, const uint16_t *__restrict__ v, int N, int G,
    int Hkv, int ragged, SeqLens lens, int splits, float *__restrict__ z_buf, float *__restrict__ part) {
    constexpr int kLpt = kD / 8;        // lanes per token row
    __shared__ float red_m[kWaves * kG];
    __shared__ int red_a[kWaves * kG];
    __shared__ float red_l[kWaves * kG];
    __shared__ float red_o[kWaves * kG * kD];

    const int bh = blockIdx.y, b = bh / Hkv, split = blockIdx.x;
    const int len = seq_len_of(lens, ragged, b, N);
    const int t0 = split * range_tokens(kD);
    const int t1 = min(t0 + range_tokens(kD), len);
    float *rec = part + ((size_t)bh * splits + split) * kG * part_stride(kD);
    if (t0 >= len) {                                // nothing of this sequence falls in the range
        for (int e = threadIdx.x; e < kG * part_stride(kD); e += kThreads) {
            const int c = e % part_stride(kD);
            rec[e] = c == 0 ? -INFINITY : (c == 2 ? __int_as_float(-1) : 0.f);
        }
        return;
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane % kLpt, slot = lane / kLpt;
    const float scale = kD == 128 ? 0.088388347648318440550f : 0.125f;
    const uint16_t *kg = k + (size_t)bh * N * kD;
    const uint16_t *vg = v + (size_t)bh * N * kD;

    // Every load of the range up front.
    uint4 qw[kG], kw[kSteps], vw[kSteps];
#pragma unroll
    for (int r = 0; r < kG; ++r) {
        qw[r] = make_uint4(0, 0, 0, 0);
        if (r < G) qw[r] = *(const uint4 *)(q + ((size_t)bh * G + r) * kD + sub * 8);
    }
#pragma unroll
    for (int u = 0; u < kSteps; ++u) {
        const int p = token_of<kD>(t0, u, wave, slot);
        kw[u] = make_uint4(0, 0, 0, 0);
        if (p < t1) kw[u] = *(const uint4 *)(kg + (size_t)p * kD + sub * 8);
    }
#pragma unroll
    for (int u = 0; u < kSteps; ++u) {
        const int p = token_of<kD>(t0, u, wave, slot);
        vw[u] = make_uint4(0, 0, 0, 0);
        if (kNeedO && p < t1) vw[u] = *(const uint4 *)(vg + (size_t)p * kD + sub * 8);
    }

    float qr[kG][8];
#pragma unroll
    for (int r = 0; r < kG; ++r) unpack8(qw[r], qr[r]);
    float z[kSteps][kG];
#pragma unroll
    for (int u = 0; u < kSteps; ++u) {
        const int p = token_of<kD>(t0, u, wave, slot);
        float kk[8];
        unpack8(kw[u], kk);
        float mine = 0.f;
#pragma unroll
        for (int r = 0; r < kG; ++r) {
            float dot = 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) dot = fmaf(qr[r][j], kk[j], dot);
            z[u][r] = group_sum<kLpt>(dot) * scale;
            if (sub == r) mine = z[u][r];
        }
        if (p < t1 && sub < kG) z_buf[((size_t)bh * N + p) * kG + sub] = mine;
    }

    // Row maxima of the range and the lowest token attaining each.
    float m[kG];
    int top[kG];
#pragma unroll
    for (int r = 0; r < kG; ++r) {
        float bm = -INFINITY;
        int ba = 0x7fffffff;
#pragma unroll
        for (int u = 0; u < kSteps; ++u) {          // tokens ascend with u: a strict compare keeps the lowest
            const int p = token_of<kD>(t0, u, wave, slot);
            if (p < t1 && z[u][r] > bm) { bm = z[u][r]; ba = p; }
        }
#pragma unroll
        for (int off = kLpt; off < 64; off <<= 1) take_better(bm, ba, __shfl_xor(bm, off), __shfl_xor(ba, off));
        if (lane == 0) { red_m[wave * kG + r] = bm; red_a[wave * kG + r] = ba; }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kG; ++r) {
        float bm = red_m[r];
        int ba = red_a[r];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) take_better(bm, ba, red_m[w * kG + r], red_a[w * kG + r]);
        m[r] = bm;
        top[r] = ba;
    }

    // Sums of exp(z - m) and of exp(z - m) v over the range without the top token.
    float lsum[kG], acc[kG][8];
#pragma unroll
    for (int r = 0; r < kG; ++r) {
        lsum[r] = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[r][j] = 0.f;
    }
#pragma unroll
    for (int u = 0; u < kSteps; ++u) {
        const int p = token_of<kD>(t0, u, wave, slot);
        if (p < t1) {
            float vv[8];
            if (kNeedO) unpack8(vw[u], vv);
#pragma unroll
            for (int r = 0; r < kG; ++r) {
                const float w = p == top[r] ? 0.f : __expf(z[u][r] - m[r]);
                lsum[r] += w;
                if (kNeedO) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[r][j] = fmaf(w, vv[j], acc[r][j]);
                }
            }
        }
    }
#pragma unroll
    for (int r = 0; r < kG; ++r) {
        const float l = slot_sum<kLpt>(lsum[r]);
        if (lane == 0) red_l[wave * kG + r] = l;
        if (kNeedO) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float o = slot_sum<kLpt>(acc[r][j]);
                if (slot == 0) red_o[(wave * kG + r) * kD + sub * 8 + j] = o;
            }
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < kG * kD; e += kThreads) {
        const int r = e / kD, c = e % kD;
        float o = 0.f;
        if (kNeedO) {
            o = red_o[r * kD + c];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) o += red_o[(w * kG + r) * kD + c];
        }
        rec[r * part_stride(kD) + kRecHead + c] = o;
        if (c == 0) {
            float l = red_l[r];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) l += red_l[w * kG + r];
            rec[r * part_stride(kD) + 0] = m[r];
            rec[r * part_stride(kD) + 1] = l;
            rec[r * part_stride(kD) + 2] = __int_as_float(top[r]);
            rec[r * part_stride(kD) + 3] = 0.f;
        }
    }
}

// Closing step of a merge for column c of row r: from the sum l_rest and the weighted vector
// sum o_rest over every key but the top one, the final record's entries of that column (and the
// record's head when c == 0).
template <int kD, bool kNeedO>
__device__ __forceinline__ void merge_finish(float m, int top, float l_rest, float o_rest, float v_top, int r, int c,
                                             float *fin) {
    const float inv_l = 1.f / (1.f + l_rest);
    float *out = fin + (size_t)r * final_stride(kD);
    if (kNeedO) {
        const float d_top = l_rest > 0.f ? (l_rest * inv_l) * (v_top - o_rest / l_rest) : 0.f;
        out[kRecHead + c] = v_top - d_top;
        out[kRecHead + kD + c] = d_top;
    }
    if (c == 0) {
        out[0] = m;
        out[1] = inv_l;
        out[2] = __int_as_float(top);
        out[3] = 0.f;
    }
}

// Merge of at most kInlineSplits ranges of one KV head for column c of row r, by one thread.
// The loads come in two batches (the records; then the rows of the held-out tokens, whose
// addresses the records give), so the merge costs two memory round trips.
template <int kD, bool kNeedO>
__device__ __forceinline__ void merge_few(const float *__restrict__ part_head, int splits, int kG, int r, int c,
                                          const uint16_t *__restrict__ vg, float *fin) {
    constexpr int ps = part_stride(kD);
    float hm[kInlineSplits], hl[kInlineSplits], o_s[kInlineSplits], v_s[kInlineSplits];
    int ht[kInlineSplits];
#pragma unroll
    for (int s = 0; s < kInlineSplits; ++s) {
        hm[s] = -INFINITY; hl[s] = 0.f; ht[s] = -1; o_s[s] = 0.f;
        if (s < splits) {
            const float *rec = part_head + ((size_t)s * kG + r) * ps;
            hm[s] = rec[0];
            hl[s] = rec[1];
            ht[s] = __float_as_int(rec[2]);
            if (kNeedO) o_s[s] = rec[kRecHead + c];
        }
    }
    float m = -INFINITY;
    int s_top = 0;
#pragma unroll
    for (int s = 0; s < kInlineSplits; ++s)
        if (hm[s] > m) { m = hm[s]; s_top = s; }    // first range attaining the max: lowest token index
#pragma unroll
    for (int s = 0; s < kInlineSplits; ++s) {
        v_s[s] = 0.f;
        if (kNeedO && ht[s] >= 0) v_s[s] = bf16_bits_to_float(vg[(size_t)ht[s] * kD + c]);
    }
    int top = -1;
    float v_top = 0.f, l_rest = 0.f, o_rest = 0.f;
#pragma unroll
    for (int s = 0; s < kInlineSplits; ++s) {
        if (s == s_top) { top = ht[s]; v_top = v_s[s]; }
        if (hm[s] == -INFINITY) continue;
        const float w = __expf(hm[s] - m);
        l_rest = fmaf(w, hl[s], l_rest);
        if (kNeedO) o_rest = fmaf(w, o_s[s], o_rest);
        if (s != s_top) {                           // this range's held-out token is an ordinary one after all
            l_rest += w;
            if (kNeedO) o_rest = fmaf(w, v_s[s], o_rest);
        }
    }
    merge_finish<kD, kNeedO>(m, top, l_rest, o_rest, v_top, r, c, fin);
}

// Merge of many ranges: one workgroup per (row, KV head); up to kMergeOwn ranges per thread for
// the scalar part, then columns x segments of ranges for the vector part; fixed summation order.
template <int kG, int kD, bool kNeedO>
__global__ __launch_bounds__(kMergeThreads) void decode_merge(const uint16_t *__restrict__ v, int N, int splits,
                                                              const float *__restrict__ part,
                                                              float *__restrict__ fin) {
    constexpr int ps = part_stride(kD);
    constexpr int kSeg = kMergeThreads / kD;
    constexpr int kMergeWaves = kMergeThreads / 64;
    constexpr int kBatch = 8;
    __shared__ float w_s[kMaxSplits];
    __shared__ int tok_s[kMaxSplits];
    __shared__ float red_m[kMergeWaves];
    __shared__ int red_a[kMergeWaves];
    __shared__ float red_l[kMergeWaves];
    __shared__ float red_o[kSeg * kD];
    const int r = blockIdx.x, bh = blockIdx.y;
    const float *part_head = part + (size_t)bh * splits * kG * ps;
    const uint16_t *vg = v + (size_t)bh * N * kD;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    float hm[kMergeOwn], hl[kMergeOwn];
    int ht[kMergeOwn];
#pragma unroll
    for (int i = 0; i < kMergeOwn; ++i) {
        const int s = i * kMergeThreads + threadIdx.x;
        hm[i] = -INFINITY; hl[i] = 0.f; ht[i] = -1;
        if (s < splits) {
            const float *rec = part_head + ((size_t)s * kG + r) * ps;
            hm[i] = rec[0];
            hl[i] = rec[1];
            ht[i] = __float_as_int(rec[2]);
        }
    }
    float bm = -INFINITY;
    int ba = 0x7fffffff;
#pragma unroll
    for (int i = 0; i < kMergeOwn; ++i) take_better(bm, ba, hm[i], i * kMergeThreads + (int)threadIdx.x);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) take_better(bm, ba, __shfl_xor(bm, off), __shfl_xor(ba, off));
    if (lane == 0) { red_m[wave] = bm; red_a[wave] = ba; }
    __syncthreads();
    bm = red_m[0];
    ba = red_a[0];
#pragma unroll
    for (int w = 1; w < kMergeWaves; ++w) take_better(bm, ba, red_m[w], red_a[w]);
    const float m = bm;
    const int s_top = ba;                           // first range attaining the max: lowest token index

    float l = 0.f;
#pragma unroll
    for (int i = 0; i < kMergeOwn; ++i) {
        const int s = i * kMergeThreads + threadIdx.x;
        const float w = hm[i] == -INFINITY ? 0.f : __expf(hm[i] - m);
        if (s < splits) { w_s[s] = w; tok_s[s] = ht[i]; }
        // ranges other than the winning one give their held-out token back
        l += fmaf(w, hl[i], s != s_top ? w : 0.f);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) l += __shfl_xor(l, off);
    if (lane == 0) red_l[wave] = l;
    __syncthreads();
    float l_rest = red_l[0];
#pragma unroll
    for (int x = 1; x < kMergeWaves; ++x) l_rest += red_l[x];
    const int top = tok_s[s_top];

    const int c = threadIdx.x % kD, seg = threadIdx.x / kD;
    float v_top = 0.f;
    if (kNeedO) {
        if (seg == 0) v_top = bf16_bits_to_float(vg[(size_t)top * kD + c]);
        float o = 0.f;
        for (int s0 = seg; s0 < splits; s0 += kBatch * kSeg) {
            float po[kBatch], pv[kBatch], pw[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int si = s0 + u * kSeg;
                po[u] = 0.f; pv[u] = 0.f; pw[u] = 0.f;
                if (si < splits && tok_s[si] >= 0) {
                    pw[u] = w_s[si];
                    po[u] = part_head[((size_t)si * kG + r) * ps + kRecHead + c];
                    if (si != s_top) pv[u] = bf16_bits_to_float(vg[(size_t)tok_s[si] * kD + c]);
                }
            }
#pragma unroll
            for (int u = 0; u < kBatch; ++u) o = fmaf(pw[u], po[u] + pv[u], o);
        }
        red_o[seg * kD + c] = o;
    }
    __syncthreads();
    if (seg == 0) {
        float o_rest = 0.f;
        if (kNeedO) {
            o_rest = red_o[c];
#pragma unroll
            for (int x = 1; x < kSeg; ++x) o_rest += red_o[x * kD + c];
        }
        merge_finish<kD, kNeedO>(m, top, l_rest, o_rest, v_top, r, c, fin + (size_t)bh * kG * final_stride(kD));
    }
}

template <int kVariant>
struct DecodeNeeds {
    static constexpr bool o = kVariant == OBC_KEY || kVariant == OBC_JOINT || kVariant == OBC_ALL;
    static constexpr bool v = kVariant != OBC_ATTN;
};

// Scores of the range's tokens from the stored logits, the merged row statistics and V.
template <int kG, int kD, int kVariant>
__global__ __launch_bounds__(kThreads) void decode_score(
    const uint16_t *__restrict__ v, int N, int G, int Hkv, int ragged, SeqLens lens, int splits,
    const float *__restrict__ z_buf, const float *__restrict__ part, const float *__restrict__ fin_global,
    int merge_here, float *__restrict__ scores, size_t plane_stride, int accumulate) {
    constexpr int kLpt = kD / 8;
    constexpr bool kNeedO = DecodeNeeds<kVariant>::o;
    constexpr bool kNeedV = DecodeNeeds<kVariant>::v;
    constexpr bool kDoV = kVariant == OBC_VALUE || kVariant == OBC_ALL;
    constexpr bool kDoK = kVariant == OBC_KEY || kVariant == OBC_ALL;
    constexpr bool kDoJ = kVariant == OBC_JOINT || kVariant == OBC_ALL;
    constexpr int kPlanes = kVariant == OBC_ALL ? 3 : 1;
    constexpr int kFs = final_stride(kD);
    __shared__ float fin[kG * kFs];

    const int bh = blockIdx.y, b = bh / Hkv;
    const int len = seq_len_of(lens, ragged, b, N);
    const int t0 = blockIdx.x * range_tokens(kD);
    const int t1 = min(t0 + range_tokens(kD), N);
    const uint16_t *vg = v + (size_t)bh * N * kD;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane % kLpt, slot = lane / kLpt;
    float *out = scores + (size_t)bh * N;

    if (t0 >= len) {                                // only padding here
        if (!accumulate) {
            for (int p = t0 + threadIdx.x; p < t1; p += kThreads) {
#pragma unroll
                for (int x = 0; x < kPlanes; ++x) out[x * plane_stride + p] = 0.f;
            }
        }
        return;
    }

    // Every load of the range up front; they are in flight while the ranges are merged.
    uint4 vw[kSteps];
    float z[kSteps][kG], old[kSteps][kPlanes];
#pragma unroll
    for (int u = 0; u < kSteps; ++u) {
        const int p = token_of<kD>(t0, u, wave, slot);
        vw[u] = make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < kG; ++r) z[u][r] = 0.f;
#pragma unroll
        for (int x = 0; x < kPlanes; ++x) old[u][x] = 0.f;
        if (p < len) {
            if (kNeedV) vw[u] = *(const uint4 *)(vg + (size_t)p * kD + sub * 8);
            const float *zp = z_buf + ((size_t)bh * N + p) * kG;
#pragma unroll
            for (int r = 0; r < kG; ++r) z[u][r] = zp[r];
            if (accumulate && sub == 0) {
#pragma unroll
                for (int x = 0; x < kPlanes; ++x) old[u][x] = out[x * plane_stride + p];
            }
        }
    }

    if (merge_here) {
        const float *part_head = part + (size_t)bh * splits * kG * part_stride(kD);
#pragma unroll
        for (int e0 = 0; e0 < kG * kD; e0 += kThreads) {       // unrolled: the loads of all passes go out together
            const int e = e0 + threadIdx.x;
            if (e < G * kD) merge_few<kD, kNeedO>(part_head, splits, kG, e / kD, e % kD, vg, fin);
        }
    } else {
        const float *src = fin_global + (size_t)bh * kG * kFs;
        for (int e = threadIdx.x; e < G * kFs; e += kThreads) fin[e] = src[e];
    }
    __syncthreads();

    float m[kG], inv_l[kG], o[kG][8];
    int top[kG];
#pragma unroll
    for (int r = 0; r < kG; ++r) {
        if (r < G) {
            m[r] = fin[r * kFs];
            inv_l[r] = fin[r * kFs + 1];
            top[r] = __float_as_int(fin[r * kFs + 2]);
        } else {
            m[r] = 0.f; inv_l[r] = 0.f; top[r] = -1;
        }
        if (kNeedO) {
#pragma unroll
            for (int j = 0; j < 8; ++j) o[r][j] = r < G ? fin[r * kFs + kRecHead + sub * 8 + j] : 0.f;
        }
    }

#pragma unroll
    for (int u = 0; u < kSteps; ++u) {
        const int p = token_of<kD>(t0, u, wave, slot);
        float s_v = 0.f, s_k = 0.f, s_j = 0.f, s_a = 0.f;
        if (p < len) {
            float vv[8];
            if (kNeedV) unpack8(vw[u], vv);
            float a2_sum = 0.f, a_sum = 0.f;
#pragma unroll
            for (int r = 0; r < kG; ++r) {
                if (r < G) {
                    const float zz = z[u][r];
                    const float a = __expf(zz - m[r]) * inv_l[r];
                    const float a2 = a * a;
                    a_sum += a;
                    a2_sum += a2;
                    if (kNeedO) {
                        float dlt[8];
                        if (p == top[r]) {
#pragma unroll
                            for (int j = 0; j < 8; ++j) dlt[j] = fin[r * kFs + kRecHead + kD + sub * 8 + j];
                        } else {
#pragma unroll
                            for (int j = 0; j < 8; ++j) dlt[j] = vv[j] - o[r][j];
                        }
                        float dk = 0.f, dj = 0.f;
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            if (kDoK) dk = fmaf(dlt[j], dlt[j], dk);
                            if (kDoJ) {
                                const float t = fmaf(zz, dlt[j], vv[j]);
                                dj = fmaf(t, t, dj);
                            }
                        }
                        if (kDoK) s_k = fmaf(a2 * zz * zz, dk, s_k);
                        if (kDoJ) s_j = fmaf(a2, dj, s_j);
                    }
                }
            }
            if (kDoV) {
                float n2 = 0.f;
#pragma unroll
                for (int j = 0; j < 8; ++j) n2 = fmaf(vv[j], vv[j], n2);
                s_v = a2_sum * n2;
            }
            if (kVariant == OBC_VATP) {
                float n1 = 0.f;
#pragma unroll
                for (int j = 0; j < 8; ++j) n1 += fabsf(vv[j]);
                s_a = a_sum * n1;
            }
            if (kVariant == OBC_ATTN) s_a = a_sum;
        }
        // per-lane pieces cover 8 of the d columns: add the pieces of the lanes sharing the token
        if (kDoV) s_v = group_sum<kLpt>(s_v);
        if (kDoK) s_k = group_sum<kLpt>(s_k);
        if (kDoJ) s_j = group_sum<kLpt>(s_j);
        if (kVariant == OBC_VATP) s_a = group_sum<kLpt>(s_a);
        if (sub == 0 && p < t1 && (p < len || !accumulate)) {   // padding: zeroed by a plain call, left alone by an accumulating one
            if (kVariant == OBC_ALL) {
                out[p] = old[u][0] + s_v;
                out[plane_stride + p] = old[u][kPlanes > 1 ? 1 : 0] + s_k;
                out[2 * plane_stride + p] = old[u][kPlanes > 2 ? 2 : 0] + s_j;
            } else {
                const float sc = kVariant == OBC_VALUE ? s_v : kVariant == OBC_KEY ? s_k
                               : kVariant == OBC_JOINT ? s_j : s_a;
                out[p] = old[u][0] + sc;
            }
        }
    }
}

template <int kG, int kD, int kVariant>
hipError_t launch_decode_variant(const ScoreArgs &a, const ScoreWorkspace &ws, char *base, hipStream_t stream) {
    constexpr bool kNeedO = DecodeNeeds<kVariant>::o;
    const int BH = a.B * a.Hkv;
    float *z_buf = (float *)(base + ws.dec_z);
    float *part = (float *)(base + ws.dec_part);
    float *fin = (float *)(base + ws.dec_final);
    const dim3 grid(ws.dec_splits, BH);
    if (ws.dec_splits > kMaxSplits || (long long)ws.dec_splits * range_tokens(kD) < a.N) return hipErrorInvalidValue;
    if (a.stage_mask & OBC_STAGE_SWEEP1) {
        decode_partial<kG, kD, kNeedO><<<grid, dim3(kThreads), 0, stream>>>(
            (const uint16_t *)a.q, (const uint16_t *)a.k, (const uint16_t *)a.v, a.N, a.G, a.Hkv, a.ragged, a.lens,
            ws.dec_splits, z_buf, part);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if ((a.stage_mask & OBC_STAGE_COMBINE) && !ws.dec_merge_inline) {
        decode_merge<kG, kD, kNeedO><<<dim3(a.G, BH), dim3(kMergeThreads), 0, stream>>>((const uint16_t *)a.v, a.N,
                                                                                        ws.dec_splits, part, fin);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (a.stage_mask & OBC_STAGE_SWEEP2) {
        decode_score<kG, kD, kVariant><<<grid, dim3(kThreads), 0, stream>>>(
            (const uint16_t *)a.v, a.N, a.G, a.Hkv, a.ragged, a.lens, ws.dec_splits, z_buf, part, fin,
            ws.dec_merge_inline, a.scores, (size_t)a.B * a.Hkv * a.N, a.accumulate);
        return hipGetLastError();
    }
    return hipSuccess;
}

template <int kG, int kD>
hipError_t launch_decode_rows(const ScoreArgs &a, const ScoreWorkspace &ws, char *base, hipStream_t stream) {
    switch (a.variant) {
        case OBC_VALUE: return launch_decode_variant<kG, kD, OBC_VALUE>(a, ws, base, stream);
        case OBC_KEY: return launch_decode_variant<kG, kD, OBC_KEY>(a, ws, base, stream);
        case OBC_JOINT: return launch_decode_variant<kG, kD, OBC_JOINT>(a, ws, base, stream);
        case OBC_ATTN: return launch_decode_variant<kG, kD, OBC_ATTN>(a, ws, base, stream);
        case OBC_VATP: return launch_decode_variant<kG, kD, OBC_VATP>(a, ws, base, stream);
        default: return launch_decode_variant<kG, kD, OBC_ALL>(a, ws, base, stream);
    }
}

template <int kD>
hipError_t launch_decode_dim(const ScoreArgs &a, const ScoreWorkspace &ws, char *base, hipStream_t stream) {
    switch (ws.dec_rows) {
        case 1: return launch_decode_rows<1, kD>(a, ws, base, stream);
        case 2: return launch_decode_rows<2, kD>(a, ws, base, stream);
        case 4: return launch_decode_rows<4, kD>(a, ws, base, stream);
        default: return launch_decode_rows<8, kD>(a, ws, base, stream);
    }
}

size_t align256(size_t x) { return (x + 255) / 256 * 256; }

int splits_for(int N, int d) { return (N + range_tokens(d) - 1) / range_tokens(d); }

}  // namespace

bool decode_path_covers(int B, int N, int W, int Hq, int Hkv, int d, int dtype, int variant, bool any_size) {
    if (dtype != OBC_BF16 || W != 1 || Hq / Hkv > kDecodeMaxGroup || (d != 64 && d != 128)) return false;
    if (splits_for(N, d) > kMaxSplits) return false;            // what one merging workgroup takes
    // These kernels win while the call is bound by round trips.  On long caches the direct forms
    // of the norms make them vector-ALU bound and the matrix-core path is faster (measured
    // crossover on gfx950: about 1e5 head-tokens when o_i is needed, 2.6e5 when it is not).
    const bool need_o = variant == OBC_KEY || variant == OBC_JOINT || variant == OBC_ALL;
    const long long head_tokens = (long long)B * Hkv * N;
    return any_size || d != 128 || head_tokens <= (need_o ? 98304 : 262144);   // (head_dim 64 has no matrix-core path)
}

void decode_plan(int B, int N, int Hq, int Hkv, int d, ScoreWorkspace *ws, size_t *off) {
    const int G = Hq / Hkv;
    const int BH = B * Hkv;
    const int splits = splits_for(N, d);
    ws->dec_rows = G <= 1 ? 1 : G <= 2 ? 2 : G <= 4 ? 4 : 8;
    ws->dec_range = range_tokens(d);
    ws->dec_splits = splits;
    ws->dec_merge_inline = splits <= kInlineSplits ? 1 : 0;
    ws->dec_z = *off;      *off = align256(*off + (size_t)BH * N * ws->dec_rows * sizeof(float));
    ws->dec_part = *off;   *off = align256(*off + (size_t)BH * splits * ws->dec_rows * part_stride(d) * sizeof(float));
    ws->dec_final = *off;  *off = align256(*off + (size_t)BH * ws->dec_rows * final_stride(d) * sizeof(float));
}

hipError_t launch_score_decode(const ScoreArgs &a, const ScoreWorkspace &ws, char *base, hipStream_t stream) {
    return a.d == 128 ? launch_decode_dim<128>(a, ws, base, stream) : launch_decode_dim<64>(a, ws, base, stream);
}

}  // namespace obc

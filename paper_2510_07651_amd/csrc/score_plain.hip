// Plain (vector-ALU) scoring path: direct evaluation of every norm, fp32 arithmetic with
// the logit dot products accumulated in fp64.
//
// Used for fp32 inputs and for shapes the matrix-core path is not built for.  Two
// kernels:
//   plain_window_attention  Section 3 of the paper for the W window rows of one
//                           query head: row max, row sum, o_i = sum_p A_ip v_p.
//   plain_score             Eq. 4-6 per (window row, token) in their direct forms
//                           ||v_p||^2, ||v_p - o_i||^2, ||(1+Z)v_p - Z o_i||^2 (the
//                           completed square of Eq. 6), summed over the window
//                           (Eq. 9) and the query heads of the KV head (Appendix A.5).
//
// Cancellation guard.  When one key takes almost all of a row's attention, o_i is almost
// v_p and fp32 cannot hold their difference.  Each row therefore keeps its top-logit
// token p* out of the running sums: with l' = sum_{q != p*} exp(z_q - z_p*) and
// o' = sum_{q != p*} exp(z_q - z_p*) v_q / l',
//     v_p* - o_i = (l' / (1 + l')) (v_p* - o')        (exact, no cancellation)
//     o_i        = v_p* - (v_p* - o_i)
// and the (row, p*) pair is scored from the first identity.  For every pair,
// (1+Z) v_p - Z o_i is formed as v_p + Z (v_p - o_i).
// Sums run in a fixed order, so results are bit-reproducible.
#include "internal.h"

namespace obc {
namespace {

constexpr int kTile = 64;        // tokens per tile
constexpr int kThreads = 256;    // 4 waves

template <typename T> __device__ __forceinline__ float load_as_float(const T *p);
template <> __device__ __forceinline__ float load_as_float<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float load_as_float<uint16_t>(const uint16_t *p) { return bf16_bits_to_float(*p); }

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x = fmaxf(x, __shfl_xor(x, off));
    return x;
}
__device__ __forceinline__ int wave_min(int x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x = min(x, __shfl_xor(x, off));
    return x;
}
// Fixed-order tree sum over the 64 lanes.
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
    return x;
}

// Scaled logit q.k/sqrt(D) (Section 3).  Products of fp32 values are exact in fp64, so the
// only rounding is the final one to fp32; both kernels call this with identical operands
// and get identical bits.
template <int D>
__device__ __forceinline__ float scaled_logit(const float *__restrict__ qrow, const float *__restrict__ krow) {
    double dot = 0.0;
    for (int j = 0; j < D; ++j) dot = fma((double)qrow[j], (double)krow[j], dot);
    return (float)(dot * (1.0 / sqrt((double)D)));
}

// Copies `kTile` rows starting at token t0 into LDS as fp32 with row stride D+1;
// rows at or beyond `len` are zero-filled (their memory is never read).
template <typename T, int D>
__device__ __forceinline__ void stage_rows(const T *__restrict__ base, int t0, int len, float *dst) {
    for (int e = threadIdx.x; e < kTile * D; e += kThreads) {
        const int row = e / D, col = e % D;
        const int p = t0 + row;
        dst[row * (D + 1) + col] = p < len ? load_as_float(base + (size_t)p * D + col) : 0.f;
    }
}

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void plain_window_attention(
    const T *__restrict__ q, const T *__restrict__ k, const T *__restrict__ v, int N, int W, int Hq, int Hkv,
    int ragged, SeqLens lens, float *__restrict__ row_max, float *__restrict__ row_sum, float *__restrict__ out,
    float *__restrict__ out_rest, float *__restrict__ rest_frac, int32_t *__restrict__ top_token) {
    __shared__ float smem[OBC_MAX_WINDOW * D + kTile * (D + 1) + OBC_MAX_WINDOW * (kTile + 1) + 2 * OBC_MAX_WINDOW];
    float *qs = smem;                                // [OBC_MAX_WINDOW][D]
    float *ts = qs + OBC_MAX_WINDOW * D;             // [kTile][D+1]  K tile, then V tile
    float *ps = ts + kTile * (D + 1);                // [OBC_MAX_WINDOW][kTile+1] unnormalised weights of the tile
    float *ms = ps + OBC_MAX_WINDOW * (kTile + 1);   // [OBC_MAX_WINDOW] row max
    int *top = (int *)(ms + OBC_MAX_WINDOW);         // [OBC_MAX_WINDOW] lowest token index attaining the row max

    const int bh = blockIdx.x;
    const int b = bh / Hq, h = bh % Hq, g = h / (Hq / Hkv);
    const int len = seq_len_of(lens, ragged, b, N);
    const T *kg = k + ((size_t)b * Hkv + g) * (size_t)N * D;
    const T *vg = v + ((size_t)b * Hkv + g) * (size_t)N * D;
    const T *qh = q + (size_t)bh * W * D;

    const int tok = threadIdx.x % kTile;
    const int rq = threadIdx.x / kTile;              // == wave index: rows rq, rq+4, ...
    constexpr int kRowsPerThread = OBC_MAX_WINDOW / 4;

    for (int e = threadIdx.x; e < W * D; e += kThreads) qs[e] = load_as_float(qh + e);

    // Sweep 1: row maxima of the scaled logits over the visible keys, and where they sit.
    float mymax[kRowsPerThread];
    int myarg[kRowsPerThread];
#pragma unroll
    for (int i = 0; i < kRowsPerThread; ++i) { mymax[i] = -INFINITY; myarg[i] = 0x7fffffff; }
    for (int t0 = 0; t0 < len; t0 += kTile) {
        __syncthreads();
        stage_rows<T, D>(kg, t0, len, ts);
        __syncthreads();
        const int p = t0 + tok;
#pragma unroll
        for (int i = 0; i < kRowsPerThread; ++i) {
            const int r = rq + 4 * i;
            if (r < W && p <= len - W + r) {
                const float z = scaled_logit<D>(qs + r * D, ts + tok * (D + 1));
                if (z > mymax[i]) { mymax[i] = z; myarg[i] = p; }     // strict: keeps the thread's lowest index
            }
        }
    }
#pragma unroll
    for (int i = 0; i < kRowsPerThread; ++i) {
        const float m = wave_max(mymax[i]);
        const int arg = wave_min(mymax[i] == m ? myarg[i] : 0x7fffffff);
        if (tok == 0 && rq + 4 * i < W) { ms[rq + 4 * i] = m; top[rq + 4 * i] = arg; }
    }

    // Sweep 2: weights exp(z - max) of every visible key except the top one, their sums,
    // and the weighted sum of V rows.
    float mysum[kRowsPerThread];
#pragma unroll
    for (int i = 0; i < kRowsPerThread; ++i) mysum[i] = 0.f;
    constexpr int kColsPerThread = D / 4;            // thread owns out[row = tid/4][cols (tid%4)*D/4 ...)
    const int orow = threadIdx.x / 4, ocol0 = (threadIdx.x % 4) * kColsPerThread;
    float oacc[kColsPerThread];
#pragma unroll
    for (int j = 0; j < kColsPerThread; ++j) oacc[j] = 0.f;

    for (int t0 = 0; t0 < len; t0 += kTile) {
        __syncthreads();
        stage_rows<T, D>(kg, t0, len, ts);
        __syncthreads();
        const int p = t0 + tok;
#pragma unroll
        for (int i = 0; i < kRowsPerThread; ++i) {
            const int r = rq + 4 * i;
            if (r < W) {
                float w = 0.f;
                if (p <= len - W + r && p != top[r])
                    w = expf(scaled_logit<D>(qs + r * D, ts + tok * (D + 1)) - ms[r]);
                mysum[i] += w;
                ps[r * (kTile + 1) + tok] = w;
            }
        }
        __syncthreads();
        stage_rows<T, D>(vg, t0, len, ts);
        __syncthreads();
        if (orow < W) {
            for (int t = 0; t < kTile; ++t) {
                const float w = ps[orow * (kTile + 1) + t];
#pragma unroll
                for (int j = 0; j < kColsPerThread; ++j) oacc[j] = fmaf(w, ts[t * (D + 1) + ocol0 + j], oacc[j]);
            }
        }
    }
    __syncthreads();
    float *ls = ps;                                   // reuse: [OBC_MAX_WINDOW] sums without the top token
#pragma unroll
    for (int i = 0; i < kRowsPerThread; ++i) {
        const float s = wave_sum(mysum[i]);
        if (tok == 0 && rq + 4 * i < W) ls[rq + 4 * i] = s;
    }
    __syncthreads();
    if ((int)threadIdx.x < W) {
        const size_t row = (size_t)bh * W + threadIdx.x;
        const float lr = ls[threadIdx.x];
        row_max[row] = ms[threadIdx.x];
        row_sum[row] = 1.0f + lr;                     // the top token's own weight is exp(0) = 1
        rest_frac[row] = lr / (1.0f + lr);            // 1 - A_{i,p*}
        top_token[row] = top[threadIdx.x];
    }
    if (orow < W) {
        const float lr = ls[orow];
        const float inv = lr > 0.f ? 1.0f / lr : 0.f;
        const float frac = lr / (1.0f + lr);
        const T *vtop = vg + (size_t)top[orow] * D + ocol0;
        const size_t off = ((size_t)bh * W + orow) * D + ocol0;
#pragma unroll
        for (int j = 0; j < kColsPerThread; ++j) {
            const float orest = oacc[j] * inv;        // attention output over everything but the top token
            const float vt = load_as_float(vtop + j);
            out_rest[off + j] = orest;
            out[off + j] = vt - frac * (vt - orest);
        }
    }
}

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void plain_score(
    const T *__restrict__ q, const T *__restrict__ k, const T *__restrict__ v, int N, int W, int Hq, int Hkv,
    int ragged, SeqLens lens, int variant, const float *__restrict__ row_max, const float *__restrict__ row_sum,
    const float *__restrict__ out, const float *__restrict__ out_rest, const float *__restrict__ rest_frac,
    const int32_t *__restrict__ top_token, float *__restrict__ scores, size_t variant_stride, int accumulate) {
    __shared__ float smem[2 * kTile * (D + 1) + 4 * D + 4 * kTile * 3];
    float *ks = smem;                          // [kTile][D+1]
    float *vs = ks + kTile * (D + 1);          // [kTile][D+1]
    float *qs = vs + kTile * (D + 1);          // [4][D] the query row each wave is working on
    float *red = qs + 4 * D;                   // [4][kTile][3]

    const int bg = blockIdx.y;
    const int b = bg / Hkv, g = bg % Hkv, G = Hq / Hkv;
    const int len = seq_len_of(lens, ragged, b, N);
    const int t0 = blockIdx.x * kTile;
    const int tok = threadIdx.x % kTile;
    const int rq = __builtin_amdgcn_readfirstlane(threadIdx.x / kTile);
    const int p = t0 + tok;

    const bool attn_like = variant == OBC_ATTN || variant == OBC_VATP;   // these use the first accumulator
    float acc_v = 0.f, acc_k = 0.f, acc_j = 0.f;
    if (t0 < len) {                            // uniform per block
        stage_rows<T, D>(k + (size_t)bg * N * D, t0, len, ks);
        stage_rows<T, D>(v + (size_t)bg * N * D, t0, len, vs);
        __syncthreads();
        const float *kp = ks + tok * (D + 1), *vp = vs + tok * (D + 1);
        float *qw = qs + rq * D;               // private to this wave: no block barrier needed around it
        float vv = 0.f, l1 = 0.f;
        for (int j = 0; j < D; ++j) { vv = fmaf(vp[j], vp[j], vv); l1 += fabsf(vp[j]); }
        for (int hh = 0; hh < G; ++hh) {
            const int h = g * G + hh;
            for (int r = rq; r < W; r += 4) {
                if (t0 > len - W + r) continue;            // uniform: whole tile hidden from this row
                const size_t row = ((size_t)b * Hq + h) * W + r;
                for (int j = tok; j < D; j += kTile) qw[j] = load_as_float(q + row * D + j);
                const float *orow = out + row * D, *orest = out_rest + row * D;
                const float m = row_max[row], inv_l = 1.0f / row_sum[row], frac = rest_frac[row];
                const int ptop = top_token[row];
                if (p <= len - W + r) {
                    const float z = scaled_logit<D>(qw, kp);
                    const bool is_top = p == ptop;
                    const float a = is_top ? inv_l : expf(z - m) * inv_l;
                    if (attn_like) {                       // Eq. 8: only the weight itself is summed
                        acc_v += a;
                        continue;
                    }
                    const float a2 = a * a;
                    const float f = is_top ? frac : 1.0f;
                    float dk = 0.f, dj = 0.f;
                    for (int j = 0; j < D; ++j) {
                        const float ref = is_top ? orest[j] : orow[j];
                        const float diff = f * (vp[j] - ref);        // v_p - o_i
                        const float comb = fmaf(z, diff, vp[j]);     // (1+Z) v_p - Z o_i
                        dk = fmaf(diff, diff, dk);
                        dj = fmaf(comb, comb, dj);
                    }
                    acc_v = fmaf(a2, vv, acc_v);
                    acc_k = fmaf(a2 * z * z, dk, acc_k);
                    acc_j = fmaf(a2, dj, acc_j);
                }
            }
        }
        if (variant == OBC_VATP) acc_v *= l1;
    }
    red[(rq * kTile + tok) * 3 + 0] = acc_v;
    red[(rq * kTile + tok) * 3 + 1] = acc_k;
    red[(rq * kTile + tok) * 3 + 2] = acc_j;
    __syncthreads();
    if (threadIdx.x < kTile && p < N) {
        float s[3];
#pragma unroll
        for (int c = 0; c < 3; ++c)
            s[c] = (red[(0 * kTile + tok) * 3 + c] + red[(1 * kTile + tok) * 3 + c]) +
                   (red[(2 * kTile + tok) * 3 + c] + red[(3 * kTile + tok) * 3 + c]);
        const size_t idx = (size_t)bg * N + p;
        const bool live = p < len;
        if (accumulate) {                       // running scores: add this call's increment, leave the padding alone
            if (live) {
                if (variant == OBC_ALL) {
#pragma unroll
                    for (int c = 0; c < 3; ++c) scores[c * variant_stride + idx] += s[c];
                } else {
                    scores[idx] += s[attn_like ? 0 : variant];
                }
            }
        } else if (variant == OBC_ALL) {
#pragma unroll
            for (int c = 0; c < 3; ++c) scores[c * variant_stride + idx] = live ? s[c] : 0.f;
        } else {
            scores[idx] = live ? s[attn_like ? 0 : variant] : 0.f;
        }
    }
}

template <typename T, int D>
hipError_t run(const ScoreArgs &a, const ScoreWorkspace &ws, char *base, hipStream_t stream) {
    float *row_max = (float *)(base + ws.row_max), *row_sum = (float *)(base + ws.row_sum);
    float *out = (float *)(base + ws.out_f32), *out_rest = (float *)(base + ws.out_rest_f32);
    float *rest_frac = (float *)(base + ws.rest_frac);
    int32_t *top_token = (int32_t *)(base + ws.top_token);
    hipError_t e;      // (both kernels size their LDS statically: nothing to configure before a launch)
    if (a.stage_mask & OBC_STAGE_SWEEP1) {      // the plain path has no separate combine stage
        plain_window_attention<T, D><<<dim3(a.B * a.Hq), dim3(kThreads), 0, stream>>>(
            (const T *)a.q, (const T *)a.k, (const T *)a.v, a.N, a.W, a.Hq, a.Hkv, a.ragged, a.lens, row_max, row_sum,
            out, out_rest, rest_frac, top_token);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (!(a.stage_mask & OBC_STAGE_SWEEP2)) return hipSuccess;
    const dim3 grid((a.N + kTile - 1) / kTile, a.B * a.Hkv);
    plain_score<T, D><<<grid, dim3(kThreads), 0, stream>>>(
        (const T *)a.q, (const T *)a.k, (const T *)a.v, a.N, a.W, a.Hq, a.Hkv, a.ragged, a.lens, a.variant, row_max,
        row_sum, out, out_rest, rest_frac, top_token, a.scores, (size_t)a.B * a.Hkv * a.N, a.accumulate);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_score_plain(const ScoreArgs &a, const ScoreWorkspace &ws, char *ws_base, hipStream_t stream) {
    if (a.dtype == OBC_F32) {
        if (a.d == 64) return run<float, 64>(a, ws, ws_base, stream);
        if (a.d == 128) return run<float, 128>(a, ws, ws_base, stream);
    } else {
        if (a.d == 64) return run<uint16_t, 64>(a, ws, ws_base, stream);
        if (a.d == 128) return run<uint16_t, 128>(a, ws, ws_base, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace obc

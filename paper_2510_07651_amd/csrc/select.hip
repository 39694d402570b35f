// Per-head top-`budget` selection (Section 3 "Cache Eviction"; Appendix E, Algorithm 2:
// topk followed by an ascending sort of the kept indices).
//
// One workgroup per (sequence, KV head).  The budget-th largest score is found by a
// most-significant-digit-first radix select over order-preserving 32-bit keys (digits of
// 11, 11 and 10 bits; histograms are integer LDS atomics, and after the first pass only
// the keys inside the selected digit class take part).  A final ordered sweep emits, in index
// order, every token above the threshold plus the first tokens equal to it until the
// budget is filled -- which is both the lowest-index tie-break and the ascending output
// order.  Integer-only bookkeeping: results are exact and reproducible.
//
// Protected regions (Appendix E, Algorithm 2: only positions below the cutoff compete and the
// recent tail is always kept; Appendix C: leading attention-sink tokens are always kept):
// tokens p < first or p >= len - tail get the key 0xffffffff, which no score maps to, so
// they outrank every competitor and the same select keeps them all when the budget is
// first + heavy hitters + tail.
//
// Pooling (Appendix C, SnapKV paragraph: average pooling of the scores, kernel size 5, before
// eviction): with radius r > 0 a competing token is ranked by the fp32 sum of the scores in
// its centred window of 2r+1 positions, taken in ascending position order, positions
// outside the competing range counting as zero.  The sum orders tokens as the average does
// and needs no division.
//
// Heads of up to 65536 tokens are read from memory once (128-bit loads) and their keys
// stay in registers for all passes; longer heads are streamed again in every pass.
#include "internal.h"

namespace obc {
namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kItems = 4;                              // consecutive scores per thread and chunk
constexpr int kChunk = kSelThreads * kItems;           // 4096 scores per chunk

// Monotone map float -> uint32: larger float <=> larger key.  -0.0 is folded onto +0.0,
// every NaN maps to 0 (below -inf).
__device__ __forceinline__ uint32_t order_key(float f) {
    uint32_t u = __float_as_uint(f);
    if (f != f) return 0u;
    if (u == 0x80000000u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

constexpr int kBins = 2048;
constexpr int kMaxRadius = 7;                           // largest pooling window: 15 scores

struct SelectShared {
    int hist[kBins];
    int wave_tot[kSelWaves];
    uint32_t sel_digit;
    int sel_remaining;
};

__device__ __forceinline__ void histogram_add(int *hist, uint32_t digit, bool active) {
    if (__ballot(active) == 0ull) return;              // uniform: nothing of this wave is in the class
    if (active) atomicAdd(&hist[digit], 1);
}

// After a histogram pass over `bins` bins: which digit holds the element of rank `remaining`
// (from the top), and that element's rank inside the digit.  All threads get the same answer.
__device__ __forceinline__ void pick_digit(SelectShared &sh, int remaining, uint32_t *digit, int *new_remaining) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    __syncthreads();
    // thread t owns digits 2t (lo) and 2t+1 (hi); suffix sums over threads t' > t
    const int lo = sh.hist[2 * tid], hi = sh.hist[2 * tid + 1];
    const int mine = lo + hi;
    int incl = mine;                    // inclusive suffix scan inside the wave (towards higher lanes)
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int t = __shfl_down(incl, off);
        if (lane + off < 64) incl += t;
    }
    if (lane == 0) sh.wave_tot[wave] = incl;
    __syncthreads();
    int above = incl - mine;            // elements in digits of higher threads
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w)
        if (w > wave) above += sh.wave_tot[w];
    if (above < remaining && remaining <= above + mine) {        // exactly one thread satisfies this
        if (remaining <= above + hi) {
            sh.sel_digit = 2u * tid + 1u;
            sh.sel_remaining = remaining - above;
        } else {
            sh.sel_digit = 2u * tid;
            sh.sel_remaining = remaining - above - hi;
        }
    }
    __syncthreads();
    *digit = sh.sel_digit;
    *new_remaining = sh.sel_remaining;
    __syncthreads();
}

// Ordered emission of one chunk: position = #greater before + min(#equal before, need_eq).
__device__ __forceinline__ void emit_chunk(SelectShared &sh, const uint32_t (&key)[kItems], int i0, int len,
                                           uint32_t thr, int need_eq, int budget, int &gt_base, int &eq_base,
                                           int32_t *out) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    bool gt[kItems], eq[kItems];
    int packed = 0;                     // low 16 bits: #equal, high 16 bits: #greater (both <= 4096 per chunk)
#pragma unroll
    for (int e = 0; e < kItems; ++e) {
        gt[e] = i0 + e < len && key[e] > thr;
        eq[e] = i0 + e < len && key[e] == thr;
        packed += (gt[e] ? 0x10000 : 0) + (eq[e] ? 1 : 0);
    }
    int incl = packed;                  // inclusive scan inside the wave
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int t = __shfl_up(incl, off);
        if (lane >= off) incl += t;
    }
    if (lane == 63) sh.wave_tot[wave] = incl;
    __syncthreads();
    int before = incl - packed, total = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
        const int t = sh.wave_tot[w];
        if (w < wave) before += t;
        total += t;
    }
    int gt_before = gt_base + (before >> 16), eq_before = eq_base + (before & 0xffff);
#pragma unroll
    for (int e = 0; e < kItems; ++e) {
        if (gt[e] || (eq[e] && eq_before < need_eq)) {
            const int pos = gt_before + min(eq_before, need_eq);
            if (pos < budget) out[pos] = i0 + e;          // always true; guards the store
        }
        gt_before += gt[e] ? 1 : 0;
        eq_before += eq[e] ? 1 : 0;
    }
    gt_base += total >> 16;
    eq_base += total & 0xffff;
    __syncthreads();
}

// Keys of chunks c0 .. c0 + kRegChunks - 1 of one head (128-bit loads where possible).
template <int kRegChunks>
__device__ __forceinline__ void load_batch(uint32_t (&keys)[kRegChunks][kItems], const float *__restrict__ s, int c0,
                                           int n_chunks, int len, bool vec_ok, int first, int cutoff, int radius) {
#pragma unroll
    for (int c = 0; c < kRegChunks; ++c) {
        if (c0 + c < n_chunks) {                          // uniform
            const int i0 = (c0 + c) * kChunk + (int)threadIdx.x * kItems;
            if (radius > 0) {                             // uniform: pooled ranking
                float w[kItems + 2 * kMaxRadius];
#pragma unroll
                for (int j = 0; j < kItems + 2 * kMaxRadius; ++j) {
                    const int idx = i0 - radius + j;
                    const bool ok = j < kItems + 2 * radius && idx >= first && idx < cutoff;
                    w[j] = ok ? s[idx] : 0.f;
                }
#pragma unroll
                for (int e = 0; e < kItems; ++e) {
                    float sum = w[e];
#pragma unroll
                    for (int j = 1; j <= 2 * kMaxRadius; ++j)
                        if (j <= 2 * radius) sum = __fadd_rn(sum, w[e + j]);
                    keys[c][e] = i0 + e < len ? order_key(sum) : 0u;
                }
            } else if (vec_ok && i0 + kItems <= len) {
                const float4 f = *(const float4 *)(s + i0);
                keys[c][0] = order_key(f.x); keys[c][1] = order_key(f.y);
                keys[c][2] = order_key(f.z); keys[c][3] = order_key(f.w);
            } else {
#pragma unroll
                for (int e = 0; e < kItems; ++e) keys[c][e] = i0 + e < len ? order_key(s[i0 + e]) : 0u;
            }
            if (i0 < first || i0 + kItems > cutoff) {     // some of these tokens are protected
#pragma unroll
                for (int e = 0; e < kItems; ++e)
                    if (i0 + e < first || (i0 + e >= cutoff && i0 + e < len)) keys[c][e] = 0xffffffffu;
            }
        }
    }
}

// kResident: the head has at most kRegChunks * 4096 tokens; its keys are loaded once and
// live in registers.  Otherwise every pass streams the head in batches of kRegChunks
// chunks (all loads of a batch are issued before any is used).
template <int kRegChunks, bool kResident>
__global__ __launch_bounds__(kSelThreads) void select_topk(const float *__restrict__ scores, int N, int budget,
                                                           int Hkv, int ragged, SeqLens lens, int first, int tail,
                                                           int radius, int32_t *__restrict__ keep_idx) {
    __shared__ SelectShared sh;
    const int bg = blockIdx.x;
    const int len = seq_len_of(lens, ragged, bg / Hkv, N);
    const int cutoff = len - tail;                        // tokens at or beyond it are always kept
    const float *s = scores + (size_t)bg * N;
    int32_t *out = keep_idx + (size_t)bg * budget;
    const int tid = threadIdx.x;
    const int n_chunks = (len + kChunk - 1) / kChunk;
    const bool vec_ok = (((size_t)bg * N) & 3) == 0;      // the head starts on a 16-byte boundary

    uint32_t keys[kRegChunks][kItems];
#pragma unroll
    for (int c = 0; c < kRegChunks; ++c)
#pragma unroll
        for (int e = 0; e < kItems; ++e) keys[c][e] = 0u;
    if (kResident) load_batch<kRegChunks>(keys, s, 0, n_chunks, len, vec_ok, first, cutoff, radius);

    // ---- radix select: key of the budget-th largest element ----
    uint32_t prefix = 0, mask = 0;
    int remaining = budget;             // rank (1-based, from the top) still to resolve inside the prefix class
    for (int pass = 0; pass < 3; ++pass) {
        const int shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0);
        const uint32_t dmask = pass == 2 ? 1023u : 2047u;
        sh.hist[2 * tid] = 0;
        sh.hist[2 * tid + 1] = 0;
        __syncthreads();
        if constexpr (kResident) {
#pragma unroll
            for (int c = 0; c < kRegChunks; ++c) {
                if (c < n_chunks) {                       // uniform
#pragma unroll
                    for (int e = 0; e < kItems; ++e) {
                        const bool in = c * kChunk + tid * kItems + e < len;
                        histogram_add(sh.hist, (keys[c][e] >> shift) & dmask, in && ((keys[c][e] & mask) == prefix));
                    }
                }
            }
        } else {
            for (int c0 = 0; c0 < n_chunks; c0 += kRegChunks) {
                load_batch<kRegChunks>(keys, s, c0, n_chunks, len, vec_ok, first, cutoff, radius);
#pragma unroll
                for (int c = 0; c < kRegChunks; ++c) {
                    if (c0 + c < n_chunks) {              // uniform
#pragma unroll
                        for (int e = 0; e < kItems; ++e) {
                            const bool in = (c0 + c) * kChunk + tid * kItems + e < len;
                            histogram_add(sh.hist, (keys[c][e] >> shift) & dmask, in && ((keys[c][e] & mask) == prefix));
                        }
                    }
                }
            }
        }
        uint32_t digit;
        pick_digit(sh, remaining, &digit, &remaining);
        prefix |= digit << shift;
        mask |= dmask << shift;
    }
    const uint32_t thr = prefix;        // key of the budget-th largest score
    const int need_eq = remaining;      // how many tokens equal to it are kept (lowest indices first)

    // ---- ordered sweep ----
    int gt_base = 0, eq_base = 0;
    if constexpr (kResident) {
#pragma unroll
        for (int c = 0; c < kRegChunks; ++c)
            if (c < n_chunks)
                emit_chunk(sh, keys[c], c * kChunk + tid * kItems, len, thr, need_eq, budget, gt_base, eq_base, out);
    } else {
        for (int c0 = 0; c0 < n_chunks; c0 += kRegChunks) {
            load_batch<kRegChunks>(keys, s, c0, n_chunks, len, vec_ok, first, cutoff, radius);
#pragma unroll
            for (int c = 0; c < kRegChunks; ++c)
                if (c0 + c < n_chunks)
                    emit_chunk(sh, keys[c], (c0 + c) * kChunk + tid * kItems, len, thr, need_eq, budget, gt_base, eq_base, out);
        }
    }
}

}  // namespace

hipError_t launch_select(const float *scores, int budget, int32_t *keep_idx, int B, int Hkv, int N, int ragged,
                         const SeqLens &lens, int first, int tail, int radius, hipStream_t stream) {
    const dim3 grid(B * Hkv), block(kSelThreads);
    if (N <= 8 * kChunk)
        select_topk<8, true><<<grid, block, 0, stream>>>(scores, N, budget, Hkv, ragged, lens, first, tail, radius, keep_idx);
    else if (N <= 16 * kChunk)
        select_topk<16, true><<<grid, block, 0, stream>>>(scores, N, budget, Hkv, ragged, lens, first, tail, radius, keep_idx);
    else
        select_topk<8, false><<<grid, block, 0, stream>>>(scores, N, budget, Hkv, ragged, lens, first, tail, radius, keep_idx);
    return hipGetLastError();
}

}  // namespace obc

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
#include <cstring>

#include "internal.h"

namespace obc {
namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kItems = 4;                              // consecutive scores per thread and chunk
constexpr int kChunk = kSelThreads * kItems;           // 4096 scores per chunk

// Monotone map float -> uint32: larger float <=> larger key.  -0.0 is folded onto +0.0,
// every NaN maps to 1 (below -inf, whose key is 0x007fffff).  No score maps to 0: that key marks
// positions that do not exist (past a sequence's length), which therefore rank below every token
// and never reach a threshold as long as the budget does not exceed the length.
__device__ __forceinline__ uint32_t order_key(float f) {
    uint32_t u = __float_as_uint(f);
    if (f != f) return 1u;
    if (u == 0x80000000u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

constexpr int kBins = 2048;
constexpr int kMaxRadius = 7;                           // largest pooling window: 15 scores

constexpr int kMaxRegChunks = 16;                       // chunks a block can keep in registers (64K scores)

struct SelectShared {
    int hist[kBins];
    int wave_tot[kSelWaves];
    uint32_t sel_digit;
    int sel_remaining;
    // ordered emission of a register-resident head: per (chunk, wave) the packed counts, then the
    // numbers of greater / equal keys that come before that (chunk, wave)
    int cw_tot[kMaxRegChunks * kSelWaves];
    int cw_gt[kMaxRegChunks * kSelWaves], cw_eq[kMaxRegChunks * kSelWaves];
};

__device__ __forceinline__ void histogram_add(int *hist, uint32_t digit, bool active) {
    if (__ballot(active) == 0ull) return;              // uniform: nothing of this wave is in the class
    if (active) atomicAdd(&hist[digit], 1);
}

// Inclusive scan of one int per lane over the wave, register to register: four data-parallel-primitive steps inside
// each row of 16 lanes (shifts by 1, 2, 4, 8, lanes outside the row reading zero), then the totals of the rows on the
// far side, read from their end lanes.  kSuffix: lane l gets the sum over lanes >= l; otherwise over lanes <= l.
template <bool kSuffix>
__device__ __forceinline__ int wave_scan(int x, int lane) {
    constexpr int kShift = kSuffix ? 0x100 : 0x110;        // row_shl : row_shr
    x += __builtin_amdgcn_update_dpp(0, x, kShift + 1, 0xf, 0xf, true);
    x += __builtin_amdgcn_update_dpp(0, x, kShift + 2, 0xf, 0xf, true);
    x += __builtin_amdgcn_update_dpp(0, x, kShift + 4, 0xf, 0xf, true);
    x += __builtin_amdgcn_update_dpp(0, x, kShift + 8, 0xf, 0xf, true);
    const int row = lane >> 4;
    if (kSuffix) {
        const int t1 = __builtin_amdgcn_readlane(x, 16), t2 = __builtin_amdgcn_readlane(x, 32), t3 = __builtin_amdgcn_readlane(x, 48);
        x += row == 0 ? t1 + t2 + t3 : row == 1 ? t2 + t3 : row == 2 ? t3 : 0;
    } else {
        const int t0 = __builtin_amdgcn_readlane(x, 15), t1 = __builtin_amdgcn_readlane(x, 31), t2 = __builtin_amdgcn_readlane(x, 47);
        x += row == 3 ? t0 + t1 + t2 : row == 2 ? t0 + t1 : row == 1 ? t0 : 0;
    }
    return x;
}

// After a histogram pass over `bins` bins: which digit holds the element of rank `remaining`
// (from the top), and that element's rank inside the digit.  All threads get the same answer.
__device__ __forceinline__ void pick_digit(SelectShared &sh, int remaining, uint32_t *digit, int *new_remaining) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    __syncthreads();
    // thread t owns digits 2t (lo) and 2t+1 (hi); suffix sums over threads t' > t
    const int lo = sh.hist[2 * tid], hi = sh.hist[2 * tid + 1];
    const int mine = lo + hi;
    const int incl = wave_scan<true>(mine, lane);          // inclusive suffix scan inside the wave (towards higher lanes)
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
    const int incl = wave_scan<false>(packed, lane);       // inclusive scan inside the wave
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

// Ordered emission of a head whose keys all sit in registers: the same positions as emit_chunk chunk after
// chunk, with three barriers in all.  Every wave scans its 256 keys of every chunk; the first wave then
// scans the (chunk, wave) totals in emission order; every thread places its keys.
template <int kRegChunks>
__device__ __forceinline__ void emit_resident(SelectShared &sh, const uint32_t (&keys)[kRegChunks][kItems], int n_chunks,
                                              int len, uint32_t thr, int need_eq, int budget, int32_t *out) {
    static_assert(kRegChunks <= kMaxRegChunks, "cw_tot is sized for kMaxRegChunks chunks");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int before[kRegChunks];                     // packed counts: low 16 bits #equal, high 16 bits #greater (<= 256 per wave)
#pragma unroll
    for (int c = 0; c < kRegChunks; ++c) {
        // Counts over the lower lanes and over the wave from the lane masks of the comparisons (no shuffles).
        int gt_lower = 0, eq_lower = 0, gt_wave = 0, eq_wave = 0;
#pragma unroll
        for (int e = 0; e < kItems; ++e) {
            // (no range checks: positions past the length and chunks past the head hold key 0 < thr)
            const unsigned long long mg = __ballot(keys[c][e] > thr), me = __ballot(keys[c][e] == thr);
            gt_lower += __builtin_amdgcn_mbcnt_hi((uint32_t)(mg >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mg, 0));
            eq_lower += __builtin_amdgcn_mbcnt_hi((uint32_t)(me >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)me, 0));
            gt_wave += __popcll(mg);
            eq_wave += __popcll(me);
        }
        if (lane == 0) sh.cw_tot[c * kSelWaves + wave] = (gt_wave << 16) | eq_wave;
        before[c] = (gt_lower << 16) | eq_lower;
    }
    __syncthreads();
    if (wave == 0) {
        // entries in emission order: j = chunk * kSelWaves + wave; lane l owns kPer consecutive ones
        constexpr int kPer = kRegChunks * kSelWaves / 64 > 0 ? kRegChunks * kSelWaves / 64 : 1;
        constexpr int kEntries = kRegChunks * kSelWaves;
        int gt[kPer], eq[kPer], gsum = 0, esum = 0;
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            const int j = lane * kPer + u;
            const int t = j < kEntries ? sh.cw_tot[j] : 0;
            gt[u] = t >> 16; eq[u] = t & 0xffff;
            gsum += gt[u]; esum += eq[u];
        }
        const int ginc = wave_scan<false>(gsum, lane), einc = wave_scan<false>(esum, lane);
        int g = ginc - gsum, q = einc - esum;       // exclusive
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            const int j = lane * kPer + u;
            if (j < kEntries) { sh.cw_gt[j] = g; sh.cw_eq[j] = q; }
            g += gt[u]; q += eq[u];
        }
    }
    __syncthreads();
    // (the comparisons are taken again rather than kept: 128 lane masks would not fit the scalar registers)
    uint32_t thr_again = thr;
    asm volatile("" : "+v"(thr_again));
#pragma unroll
    for (int c = 0; c < kRegChunks; ++c) {
        if (c >= n_chunks) continue;              // uniform
        const int i0 = c * kChunk + tid * kItems;
        int gt_before = sh.cw_gt[c * kSelWaves + wave] + (before[c] >> 16);
        int eq_before = sh.cw_eq[c * kSelWaves + wave] + (before[c] & 0xffff);
#pragma unroll
        for (int e = 0; e < kItems; ++e) {
            const bool gt = keys[c][e] > thr_again, eq = keys[c][e] == thr_again;
            if (gt || (eq && eq_before < need_eq)) {
                const int pos = gt_before + min(eq_before, need_eq);
                if (pos < budget) out[pos] = i0 + e;          // always true; guards the store
            }
            gt_before += gt ? 1 : 0;
            eq_before += eq ? 1 : 0;
        }
    }
}

// The same when every key equal to the threshold is kept (no tie is cut: the usual case): a key is kept iff it is
// >= the threshold, so one comparison and one count per key do.
template <int kRegChunks>
__device__ __forceinline__ void emit_resident_uncut(SelectShared &sh, const uint32_t (&keys)[kRegChunks][kItems],
                                                    int n_chunks, uint32_t thr, int budget, int32_t *out) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int before[kRegChunks];                     // kept keys of the wave's lower lanes in chunk c
#pragma unroll
    for (int c = 0; c < kRegChunks; ++c) {
        int lower = 0, in_wave = 0;
#pragma unroll
        for (int e = 0; e < kItems; ++e) {
            const unsigned long long m = __ballot(keys[c][e] >= thr);
            lower += __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0));
            in_wave += __popcll(m);
        }
        if (lane == 0) sh.cw_tot[c * kSelWaves + wave] = in_wave;
        before[c] = lower;
    }
    __syncthreads();
    if (wave == 0) {
        constexpr int kPer = kRegChunks * kSelWaves / 64 > 0 ? kRegChunks * kSelWaves / 64 : 1;
        constexpr int kEntries = kRegChunks * kSelWaves;
        int n[kPer], sum = 0;
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            const int j = lane * kPer + u;
            n[u] = j < kEntries ? sh.cw_tot[j] : 0;
            sum += n[u];
        }
        int g = wave_scan<false>(sum, lane) - sum;  // exclusive
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            const int j = lane * kPer + u;
            if (j < kEntries) sh.cw_gt[j] = g;
            g += n[u];
        }
    }
    __syncthreads();
    uint32_t thr_again = thr;                       // (compared again rather than kept: the lane masks would not fit)
    asm volatile("" : "+v"(thr_again));
#pragma unroll
    for (int c = 0; c < kRegChunks; ++c) {
        if (c >= n_chunks) continue;                // uniform
        const int i0 = c * kChunk + tid * kItems;
        int pos = sh.cw_gt[c * kSelWaves + wave] + before[c];
#pragma unroll
        for (int e = 0; e < kItems; ++e) {
            const bool keep = keys[c][e] >= thr_again;
            if (keep && pos < budget) out[pos] = i0 + e;      // (pos < budget always holds; it guards the store)
            pos += keep ? 1 : 0;
        }
    }
}

// Keys of chunks c0 .. c0 + kRegChunks - 1 of one head (128-bit loads where possible).
template <int kRegChunks>
__device__ __forceinline__ void load_batch(uint32_t (&keys)[kRegChunks][kItems], const float *__restrict__ s, int c0,
                                           int n_chunks, int len, bool vec_ok, int first, int cutoff, int radius,
                                           bool keys_in = false) {
    if (radius == 0 && !keys_in && vec_ok) {              // uniform: plain scores of an aligned head, the usual case
        // Every load of the batch goes out before any key is formed: one memory round trip, not one per chunk.
        float4 f[kRegChunks];
#pragma unroll
        for (int c = 0; c < kRegChunks; ++c) {
            const int i0 = (c0 + c) * kChunk + (int)threadIdx.x * kItems;
            f[c] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (c0 + c < n_chunks) {                      // uniform
                if (i0 + kItems <= len) {
                    f[c] = *(const float4 *)(s + i0);
                } else {                                  // the head's last, partial group of four
                    if (i0 < len) f[c].x = s[i0];
                    if (i0 + 1 < len) f[c].y = s[i0 + 1];
                    if (i0 + 2 < len) f[c].z = s[i0 + 2];
                }
            }
        }
#pragma unroll
        for (int c = 0; c < kRegChunks; ++c) {
            if (c0 + c < n_chunks) {                      // uniform
                const int i0 = (c0 + c) * kChunk + (int)threadIdx.x * kItems;
                keys[c][0] = order_key(f[c].x); keys[c][1] = order_key(f[c].y);
                keys[c][2] = order_key(f[c].z); keys[c][3] = order_key(f[c].w);
                if (i0 + kItems > len) {                  // positions past the length
#pragma unroll
                    for (int e = 0; e < kItems; ++e)
                        if (i0 + e >= len) keys[c][e] = 0u;
                }
                if (i0 < first || i0 + kItems > cutoff) { // some of these tokens are protected
#pragma unroll
                    for (int e = 0; e < kItems; ++e)
                        if (i0 + e < first || (i0 + e >= cutoff && i0 + e < len)) keys[c][e] = 0xffffffffu;
                }
            }
        }
        return;
    }
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
            } else if (keys_in) {                         // uniform: the input already holds order-preserving keys
                const uint32_t *kin = (const uint32_t *)s;
#pragma unroll
                for (int e = 0; e < kItems; ++e) keys[c][e] = i0 + e < len ? kin[i0 + e] : 0u;
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
                                                           int radius, int keys_in, int32_t *__restrict__ keep_idx) {
    __shared__ SelectShared sh;
    const int bg = blockIdx.x;
    const int len = seq_len_of(lens, ragged, bg / Hkv, N);
    const int cutoff = len - tail;                        // tokens at or beyond it are always kept
    const float *s = scores + (size_t)bg * N;
    int32_t *out = keep_idx + (size_t)bg * budget;
    const int tid = threadIdx.x;
    const int n_chunks = (len + kChunk - 1) / kChunk;
    const bool vec_ok = ((size_t)s & 15) == 0;            // the head starts on a 16-byte boundary

    uint32_t keys[kRegChunks][kItems];
#pragma unroll
    for (int c = 0; c < kRegChunks; ++c)
#pragma unroll
        for (int e = 0; e < kItems; ++e) keys[c][e] = 0u;
    if (kResident) load_batch<kRegChunks>(keys, s, 0, n_chunks, len, vec_ok, first, cutoff, radius, keys_in != 0);

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
            // (positions past the length hold key 0: they land in the lowest class and are never reached)
#pragma unroll
            for (int c = 0; c < kRegChunks; ++c) {
                if (c < n_chunks) {                       // uniform
#pragma unroll
                    for (int e = 0; e < kItems; ++e)
                        if ((keys[c][e] & mask) == prefix) atomicAdd(&sh.hist[(keys[c][e] >> shift) & dmask], 1);
                }
            }
        } else {
            for (int c0 = 0; c0 < n_chunks; c0 += kRegChunks) {
                load_batch<kRegChunks>(keys, s, c0, n_chunks, len, vec_ok, first, cutoff, radius, keys_in != 0);
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
        // (the last pass's counters are still in place: the threshold's own counter is the number of keys equal to it)
        if (need_eq == sh.hist[thr & 1023u]) emit_resident_uncut<kRegChunks>(sh, keys, n_chunks, thr, budget, out);
        else emit_resident<kRegChunks>(sh, keys, n_chunks, len, thr, need_eq, budget, out);
    } else {
        for (int c0 = 0; c0 < n_chunks; c0 += kRegChunks) {
            load_batch<kRegChunks>(keys, s, c0, n_chunks, len, vec_ok, first, cutoff, radius, keys_in != 0);
#pragma unroll
            for (int c = 0; c < kRegChunks; ++c)
                if (c0 + c < n_chunks)
                    emit_chunk(sh, keys[c], (c0 + c) * kChunk + tid * kItems, len, thr, need_eq, budget, gt_base, eq_base, out);
        }
    }
}

// ------------------------------------------------------------------------------------
// Sliced variant for few, long heads: one block per (slice of 8192 tokens, head), five
// short kernels instead of one long block per head.  The same radix select, with the
// per-pass histograms written per slice to a workspace and summed by every block of the
// next kernel (no global atomics, nothing to clear, fixed order of integer sums):
//   stage 0    histogram of digit 0                               -> hist A
//   stage 1    pick digit 0 from A;  histogram of digit 1         -> hist B, state
//   stage 2    pick digit 1 from B;  histogram of digit 2         -> hist A, state
//   stage 3    pick digit 2 from A = threshold; count (above, equal) per slice -> counts, state
//   stage 4    ordered emission, each slice starting at the totals of the slices before it
// ------------------------------------------------------------------------------------
constexpr int kSliceChunks = 2;
constexpr int kSliceTok = kSliceChunks * kChunk;          // 8192 tokens per block

struct SliceState {      // per (stage, head), in the workspace: stage k reads slot k-1 and writes slot k
    uint32_t prefix;     // digits picked so far, in place
    int remaining;       // rank still to resolve inside the prefix class; after stage 3: how many equal keys are kept
};

// Sums the slices' histograms of one head into sh.hist (thread t: bins 2t and 2t+1).
__device__ __forceinline__ void sum_slice_histograms(SelectShared &sh, const int *__restrict__ hist, int n_slices) {
    const int tid = threadIdx.x;
    int lo = 0, hi = 0;
    for (int sl = 0; sl < n_slices; ++sl) {
        const int2 h = *(const int2 *)(hist + (size_t)sl * kBins + 2 * tid);
        lo += h.x;
        hi += h.y;
    }
    sh.hist[2 * tid] = lo;
    sh.hist[2 * tid + 1] = hi;
}

template <int kStage>
__global__ __launch_bounds__(kSelThreads) void select_sliced(const float *__restrict__ scores, int N, int budget,
                                                             int Hkv, int ragged, SeqLens lens, int first, int tail,
                                                             int radius, int keys_in, int n_slices, int *__restrict__ hist_a,
                                                             int *__restrict__ hist_b, SliceState *__restrict__ state,
                                                             int *__restrict__ counts,
                                                             int32_t *__restrict__ keep_idx) {
    __shared__ SelectShared sh;
    const int slice = blockIdx.x, bg = blockIdx.y;
    const int len = seq_len_of(lens, ragged, bg / Hkv, N);
    const int cutoff = len - tail;
    const float *s = scores + (size_t)bg * N;
    const int tid = threadIdx.x;
    const int n_chunks = (len + kChunk - 1) / kChunk;     // of the whole head
    const int c0 = slice * kSliceChunks;                   // first chunk of this slice
    const bool vec_ok = ((size_t)s & 15) == 0;
    // which histogram buffer this stage reads and which it writes
    const int *hist_in = (kStage == 1 || kStage == 3) ? hist_a : hist_b;
    int *hist_out = (kStage == 0 || kStage == 2) ? hist_a : hist_b;
    const SliceState *state_in = state + (size_t)(kStage > 0 ? kStage - 1 : 0) * gridDim.y;
    SliceState *state_out = state + (size_t)(kStage < 4 ? kStage : 0) * gridDim.y;
    hist_in += (size_t)bg * n_slices * kBins;
    hist_out += ((size_t)bg * n_slices + slice) * kBins;

    uint32_t keys[kSliceChunks][kItems];
#pragma unroll
    for (int c = 0; c < kSliceChunks; ++c)
#pragma unroll
        for (int e = 0; e < kItems; ++e) keys[c][e] = 0u;
    load_batch<kSliceChunks>(keys, s, c0, n_chunks, len, vec_ok, first, cutoff, radius, keys_in != 0);

    // ---- the digit the previous stage's histograms decide ----
    uint32_t prefix = 0, mask = 0;
    int remaining = budget;
    if (kStage >= 1 && kStage <= 3) {
        if (kStage >= 2) { prefix = state_in[bg].prefix; remaining = state_in[bg].remaining; }
        mask = kStage == 1 ? 0u : (kStage == 2 ? (2047u << 21) : ((2047u << 21) | (2047u << 10)));
        sum_slice_histograms(sh, hist_in, n_slices);
        uint32_t digit;
        pick_digit(sh, remaining, &digit, &remaining);
        const int shift_prev = kStage == 1 ? 21 : (kStage == 2 ? 10 : 0);
        prefix |= digit << shift_prev;
        mask |= (kStage == 3 ? 1023u : 2047u) << shift_prev;
    }
    if (kStage == 4) { prefix = state_in[bg].prefix; remaining = state_in[bg].remaining; }

    if (kStage <= 2) {
        // ---- histogram of this stage's digit over the slice, restricted to the prefix class ----
        const int shift = kStage == 0 ? 21 : (kStage == 1 ? 10 : 0);
        const uint32_t dmask = kStage == 2 ? 1023u : 2047u;
        __syncthreads();
        sh.hist[2 * tid] = 0;
        sh.hist[2 * tid + 1] = 0;
        __syncthreads();
#pragma unroll
        for (int c = 0; c < kSliceChunks; ++c) {
            if (c0 + c < n_chunks) {                      // uniform
#pragma unroll
                for (int e = 0; e < kItems; ++e) {
                    const bool in = (c0 + c) * kChunk + tid * kItems + e < len;
                    histogram_add(sh.hist, (keys[c][e] >> shift) & dmask, in && ((keys[c][e] & mask) == prefix));
                }
            }
        }
        __syncthreads();
        *(int2 *)(hist_out + 2 * tid) = make_int2(sh.hist[2 * tid], sh.hist[2 * tid + 1]);
        if (kStage >= 1 && slice == 0 && tid == 0) { state_out[bg].prefix = prefix; state_out[bg].remaining = remaining; }
    } else if (kStage == 3) {
        // ---- threshold known: how many keys of this slice lie above it, how many equal it ----
        int packed = 0;
#pragma unroll
        for (int c = 0; c < kSliceChunks; ++c)
#pragma unroll
            for (int e = 0; e < kItems; ++e) {
                const bool in = (c0 + c) * kChunk + tid * kItems + e < len;
                packed += (in && keys[c][e] > prefix ? 0x10000 : 0) + (in && keys[c][e] == prefix ? 1 : 0);
            }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) packed += __shfl_xor(packed, off);
        __syncthreads();
        if ((tid & 63) == 0) sh.wave_tot[tid >> 6] = packed;
        __syncthreads();
        if (tid == 0) {
            int tot = 0;
#pragma unroll
            for (int w = 0; w < kSelWaves; ++w) tot += sh.wave_tot[w];
            counts[((size_t)bg * n_slices + slice) * 2 + 0] = tot >> 16;
            counts[((size_t)bg * n_slices + slice) * 2 + 1] = tot & 0xffff;
            if (slice == 0) { state_out[bg].prefix = prefix; state_out[bg].remaining = remaining; }
        }
    } else {
        // ---- ordered emission ----
        int gt_base = 0, eq_base = 0;
        for (int sl = 0; sl < slice; ++sl) {
            gt_base += counts[((size_t)bg * n_slices + sl) * 2 + 0];
            eq_base += counts[((size_t)bg * n_slices + sl) * 2 + 1];
        }
        int32_t *out = keep_idx + (size_t)bg * budget;
#pragma unroll
        for (int c = 0; c < kSliceChunks; ++c)
            if (c0 + c < n_chunks)
                emit_chunk(sh, keys[c], (c0 + c) * kChunk + tid * kItems, len, prefix, remaining, budget, gt_base, eq_base, out);
    }
}

// ------------------------------------------------------------------------------------
// Head-adaptive budgets (Appendix C, AdaKV paragraph): the layer's budget is spread over the
// KV heads by ranking all (head, token) scores of a sequence together, after each head's own
// top n_safe tokens (the safeguard) have been put beyond competition.  Done with the
// selection above on a sequence's heads laid end to end, over order-preserving keys:
//   adaptive_keys   key of every live token (>= 1), 0 for positions beyond the true length
//   adaptive_mark   0xffffffff for every head's n_safe best (found by the per-head select)
//   select          top Hkv * budget of the Hkv * N keys: ascending flat positions
//   adaptive_split  flat positions -> per-head index lists and counts
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void adaptive_keys(const float *__restrict__ scores, int N, int Hkv, int ragged,
                                                     SeqLens lens, size_t total, uint32_t *__restrict__ keys) {
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= total) return;
    const int p = (int)(t % N);
    const int b = (int)(t / ((size_t)N * Hkv));
    const uint32_t key = order_key(scores[t]);
    keys[t] = p < seq_len_of(lens, ragged, b, N) ? (key < 1u ? 1u : key) : 0u;
}

__global__ __launch_bounds__(256) void adaptive_mark(const int32_t *__restrict__ safe_idx, int N, int n_safe,
                                                     size_t total, uint32_t *__restrict__ keys) {
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;       // (bg, j)
    if (t >= total) return;
    const size_t bg = t / n_safe;
    const int p = safe_idx[t];
    if (p >= 0 && p < N) keys[bg * N + p] = 0xffffffffu;
}

// One block per (head, sequence): the head's share of the ascending flat list is the run of
// positions in [g N, (g+1) N); its ends are found by bisection.
__global__ __launch_bounds__(256) void adaptive_split(const int32_t *__restrict__ flat_idx, int N, int total_budget,
                                                      int cap, int32_t *__restrict__ keep_idx,
                                                      int32_t *__restrict__ counts) {
    const int g = blockIdx.x, b = blockIdx.y, Hkv = gridDim.x;
    const int32_t *flat = flat_idx + (size_t)b * total_budget;
    auto lower_bound = [&](int value) {
        int lo = 0, hi = total_budget;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (flat[mid] < value) lo = mid + 1; else hi = mid;
        }
        return lo;
    };
    const int begin = lower_bound(g * N), end = lower_bound((g + 1) * N);
    const int count = min(end - begin, cap);
    int32_t *out = keep_idx + ((size_t)b * Hkv + g) * cap;
    for (int j = threadIdx.x; j < cap; j += 256) out[j] = j < count ? flat[begin + j] - g * N : -1;
    if (threadIdx.x == 0) counts[(size_t)b * Hkv + g] = count;
}

}  // namespace

static size_t up256(size_t x) { return (x + 255) / 256 * 256; }

size_t select_adaptive_workspace_bytes(int B, int Hkv, int N, int budget, int n_safe) {
    const size_t BH = (size_t)B * Hkv;
    size_t bytes = up256(BH * (size_t)(n_safe > 0 ? n_safe : 1) * sizeof(int32_t));     // safeguard indices
    bytes += up256(BH * N * sizeof(uint32_t));                                           // keys
    bytes += up256((size_t)B * Hkv * budget * sizeof(int32_t));                          // flat positions
    if (select_prefers_slices(B, 1, Hkv * N)) bytes += select_workspace_bytes(B, 1, Hkv * N);
    if (select_prefers_slices(B, Hkv, N)) bytes += select_workspace_bytes(B, Hkv, N);
    return bytes;
}

hipError_t launch_select_adaptive(const float *scores, int budget, int n_safe, int cap, int32_t *keep_idx,
                                  int32_t *counts, int B, int Hkv, int N, int ragged, const SeqLens &lens,
                                  void *workspace, hipStream_t stream) {
    const size_t BH = (size_t)B * Hkv;
    char *base = (char *)workspace;
    int32_t *safe_idx = (int32_t *)base;   base += up256(BH * (size_t)(n_safe > 0 ? n_safe : 1) * sizeof(int32_t));
    uint32_t *keys = (uint32_t *)base;     base += up256(BH * N * sizeof(uint32_t));
    int32_t *flat_idx = (int32_t *)base;   base += up256((size_t)B * Hkv * budget * sizeof(int32_t));
    void *ws_flat = nullptr, *ws_head = nullptr;
    size_t ws_flat_bytes = 0, ws_head_bytes = 0;
    if (select_prefers_slices(B, 1, Hkv * N)) { ws_flat = base; ws_flat_bytes = select_workspace_bytes(B, 1, Hkv * N); base += ws_flat_bytes; }
    if (select_prefers_slices(B, Hkv, N)) { ws_head = base; ws_head_bytes = select_workspace_bytes(B, Hkv, N); }
    hipError_t e;
    const size_t total = BH * N;
    adaptive_keys<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream>>>(scores, N, Hkv, ragged, lens, total, keys);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (n_safe > 0) {
        e = launch_select(scores, n_safe, safe_idx, B, Hkv, N, ragged, lens, 0, 0, 0, ws_head, ws_head_bytes, stream, 0);
        if (e != hipSuccess) return e;
        const size_t marks = BH * n_safe;
        adaptive_mark<<<dim3((unsigned)((marks + 255) / 256)), dim3(256), 0, stream>>>(safe_idx, N, n_safe, marks, keys);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    SeqLens none;
    std::memset(&none, 0, sizeof(none));
    e = launch_select((const float *)keys, Hkv * budget, flat_idx, B, 1, Hkv * N, 0, none, 0, 0, 0, ws_flat, ws_flat_bytes,
                      stream, 1);
    if (e != hipSuccess) return e;
    adaptive_split<<<dim3(Hkv, B), dim3(256), 0, stream>>>(flat_idx, N, Hkv * budget, cap, keep_idx, counts);
    return hipGetLastError();
}

size_t select_workspace_bytes(int B, int Hkv, int N) {
    const size_t BH = (size_t)B * Hkv;
    const size_t n_slices = ((size_t)N + kSliceTok - 1) / kSliceTok;
    auto up = [](size_t x) { return (x + 255) / 256 * 256; };
    return 2 * up(BH * n_slices * kBins * sizeof(int)) + up(4 * BH * sizeof(SliceState)) + up(BH * n_slices * 2 * sizeof(int));
}

// Long heads take the sliced path: one block per head keeps a 32K-token head in registers
// (27 us, about what five launches cost), but beyond that it spills or re-streams the head
// in every pass (53 us at 64K, 390 us at 128K measured) while the slices stay at 35-55 us.
bool select_prefers_slices(int B, int Hkv, int N) {
    const long long BH = (long long)B * Hkv;
    return N > 8 * kChunk && BH * ((N + kSliceTok - 1) / kSliceTok) <= 2048;
}

hipError_t launch_select_sliced(const float *scores, int budget, int32_t *keep_idx, int B, int Hkv, int N, int ragged,
                                const SeqLens &lens, int first, int tail, int radius, int keys_in, void *workspace,
                                hipStream_t stream) {
    const size_t BH = (size_t)B * Hkv;
    const int n_slices = (N + kSliceTok - 1) / kSliceTok;
    auto up = [](size_t x) { return (x + 255) / 256 * 256; };
    char *base = (char *)workspace;
    int *hist_a = (int *)base;                      base += up(BH * n_slices * kBins * sizeof(int));
    int *hist_b = (int *)base;                      base += up(BH * n_slices * kBins * sizeof(int));
    SliceState *state = (SliceState *)base;         base += up(4 * BH * sizeof(SliceState));
    int *counts = (int *)base;
    const dim3 grid(n_slices, (unsigned)BH), block(kSelThreads);
#define OBC_SLICED_ARGS scores, N, budget, Hkv, ragged, lens, first, tail, radius, keys_in, n_slices, hist_a, hist_b, state, counts, keep_idx
    select_sliced<0><<<grid, block, 0, stream>>>(OBC_SLICED_ARGS);
    select_sliced<1><<<grid, block, 0, stream>>>(OBC_SLICED_ARGS);
    select_sliced<2><<<grid, block, 0, stream>>>(OBC_SLICED_ARGS);
    select_sliced<3><<<grid, block, 0, stream>>>(OBC_SLICED_ARGS);
    select_sliced<4><<<grid, block, 0, stream>>>(OBC_SLICED_ARGS);
#undef OBC_SLICED_ARGS
    return hipGetLastError();
}

hipError_t launch_select(const float *scores, int budget, int32_t *keep_idx, int B, int Hkv, int N, int ragged,
                         const SeqLens &lens, int first, int tail, int radius, void *workspace,
                         size_t workspace_bytes, hipStream_t stream, int keys_in) {
    if (workspace && select_prefers_slices(B, Hkv, N) && workspace_bytes >= select_workspace_bytes(B, Hkv, N))
        return launch_select_sliced(scores, budget, keep_idx, B, Hkv, N, ragged, lens, first, tail, radius, keys_in,
                                    workspace, stream);
    const dim3 grid(B * Hkv), block(kSelThreads);
    if (N <= kChunk)             // (short heads: fewer unrolled chunk bodies to step through)
        select_topk<1, true><<<grid, block, 0, stream>>>(scores, N, budget, Hkv, ragged, lens, first, tail, radius, keys_in, keep_idx);
    else if (N <= 2 * kChunk)
        select_topk<2, true><<<grid, block, 0, stream>>>(scores, N, budget, Hkv, ragged, lens, first, tail, radius, keys_in, keep_idx);
    else if (N <= 8 * kChunk)
        select_topk<8, true><<<grid, block, 0, stream>>>(scores, N, budget, Hkv, ragged, lens, first, tail, radius, keys_in, keep_idx);
    else if (N <= 16 * kChunk)
        select_topk<16, true><<<grid, block, 0, stream>>>(scores, N, budget, Hkv, ragged, lens, first, tail, radius, keys_in, keep_idx);
    else
        select_topk<8, false><<<grid, block, 0, stream>>>(scores, N, budget, Hkv, ragged, lens, first, tail, radius, keys_in, keep_idx);
    return hipGetLastError();
}

}  // namespace obc

// Per-head top-`budget` selection (Section 3 "Cache Eviction"; Appendix E, Algorithm 2:
// topk followed by an ascending sort of the kept indices).
//
// One workgroup per (sequence, KV head).  The budget-th largest score is found by a
// most-significant-digit-first radix select over order-preserving 32-bit keys (four
// 8-bit digits; histograms are built with wavefront ballots so that equal digits cost
// one LDS atomic per wave, not one per lane).  A final ordered sweep emits, in index
// order, every token above the threshold plus the first tokens equal to it until the
// budget is filled -- which is both the lowest-index tie-break and the ascending output
// order.  Integer-only bookkeeping: results are exact and reproducible.
#include "internal.h"

namespace obc {
namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kItems = 4;   // consecutive scores per thread in the ordered sweep

// Monotone map float -> uint32: larger float <=> larger key.  -0.0 is folded onto +0.0,
// every NaN maps to 0 (below -inf).
__device__ __forceinline__ uint32_t order_key(float f) {
    uint32_t u = __float_as_uint(f);
    if (f != f) return 0u;
    if (u == 0x80000000u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Adds 1 to hist[digit] for every active lane, one atomic per distinct digit in the wave.
__device__ __forceinline__ void wave_histogram_add(int *hist, uint32_t digit, bool active) {
    unsigned long long peers = __ballot(active);
#pragma unroll
    for (int bit = 0; bit < 8; ++bit) {
        const bool mine = (digit >> bit) & 1u;
        const unsigned long long b = __ballot(mine && active);
        peers &= mine ? b : ~b;
    }
    if (active) {
        const int leader = __ffsll((long long)peers) - 1;
        if ((int)(threadIdx.x & 63) == leader) atomicAdd(&hist[digit], __popcll(peers));
    }
}

__global__ __launch_bounds__(kSelThreads) void select_topk(const float *__restrict__ scores, int N, int budget,
                                                           int Hkv, int ragged, SeqLens lens,
                                                           int32_t *__restrict__ keep_idx) {
    __shared__ int hist[256];
    __shared__ uint32_t sel_digit;
    __shared__ int sel_remaining;
    __shared__ int wave_tot[kSelWaves];

    const int bg = blockIdx.x;
    const int len = seq_len_of(lens, ragged, bg / Hkv, N);
    const float *s = scores + (size_t)bg * N;
    int32_t *out = keep_idx + (size_t)bg * budget;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // ---- radix select: key of the budget-th largest element ----
    uint32_t prefix = 0, mask = 0;
    int remaining = budget;             // rank (1-based, from the top) still to resolve inside the prefix class
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        for (int i0 = 0; i0 < len; i0 += kSelThreads) {     // uniform trip count: ballots see whole waves
            const int i = i0 + tid;
            const bool in = i < len;
            const uint32_t key = in ? order_key(s[i]) : 0u;
            const bool active = in && ((key & mask) == prefix);
            wave_histogram_add(hist, (key >> shift) & 255u, active);
        }
        __syncthreads();
        if (tid < 256) {
            int above = 0;
            for (int j = tid + 1; j < 256; ++j) above += hist[j];
            if (above < remaining && remaining <= above + hist[tid]) {   // exactly one digit satisfies this
                sel_digit = (uint32_t)tid;
                sel_remaining = remaining - above;
            }
        }
        __syncthreads();
        prefix |= sel_digit << shift;
        mask |= 255u << shift;
        remaining = sel_remaining;
        __syncthreads();
    }
    const uint32_t thr = prefix;        // key of the budget-th largest score
    const int need_eq = remaining;      // how many tokens equal to it are kept (lowest indices first)

    // ---- ordered sweep: position = #greater before + min(#equal before, need_eq) ----
    int gt_base = 0, eq_base = 0;
    for (int c0 = 0; c0 < len; c0 += kSelThreads * kItems) {
        const int i0 = c0 + tid * kItems;
        bool gt[kItems], eq[kItems];
        int packed = 0;                 // low 16 bits: #equal, high 16 bits: #greater (both <= 4096 per chunk)
#pragma unroll
        for (int e = 0; e < kItems; ++e) {
            const int i = i0 + e;
            const uint32_t key = i < len ? order_key(s[i]) : 0u;
            gt[e] = i < len && key > thr;
            eq[e] = i < len && key == thr;
            packed += (gt[e] ? 0x10000 : 0) + (eq[e] ? 1 : 0);
        }
        int incl = packed;              // inclusive scan inside the wave
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int t = __shfl_up(incl, off);
            if (lane >= off) incl += t;
        }
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        int before = incl - packed, total = 0;
#pragma unroll
        for (int w = 0; w < kSelWaves; ++w) {
            const int t = wave_tot[w];
            if (w < wave) before += t;
            total += t;
        }
        int gt_before = gt_base + (before >> 16), eq_before = eq_base + (before & 0xffff);
#pragma unroll
        for (int e = 0; e < kItems; ++e) {
            if (gt[e] || (eq[e] && eq_before < need_eq)) {
                const int pos = gt_before + min(eq_before, need_eq);
                if (pos < budget) out[pos] = i0 + e;      // always true; guards the store
            }
            gt_before += gt[e] ? 1 : 0;
            eq_before += eq[e] ? 1 : 0;
        }
        gt_base += total >> 16;
        eq_base += total & 0xffff;
        __syncthreads();
    }
}

}  // namespace

hipError_t launch_select(const float *scores, int budget, int32_t *keep_idx, int B, int Hkv, int N, int ragged,
                         const SeqLens &lens, hipStream_t stream) {
    select_topk<<<dim3(B * Hkv), dim3(kSelThreads), 0, stream>>>(scores, N, budget, Hkv, ragged, lens, keep_idx);
    return hipGetLastError();
}

}  // namespace obc

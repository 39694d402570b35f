// Matrix-core scoring path for bf16 caches with head_dim 128 (gfx950, wave64).
//
// The scores of Eq. 4-6 need, for every (window row i, token p) pair, the softmax weight
// A_ip, the logit Z_ip and the cross term v_p . o_i, where A and o_i depend on sums over
// ALL tokens of the row (Section 3).  So the cache is swept twice:
//
//   sweep 1  (mfma_sweep1)   per (KV head, 128-row chunk, sequence split): S^T = K Q^T on
//            the matrix cores, online softmax per row, O^T += V^T P^T on the matrix cores;
//            emits a partial (row max, row sum, unnormalised O) per split.
//   combine  (mfma_combine, mfma_combine_hold)  merges the splits: final sum, o_i as a pair
//            of bf16 pieces, ||o_i||^2, and the constants the second sweep needs per row.
//   sweep 2  (mfma_sweep2)   per (KV head, chunk, token range): Z = Q K^T and the cross
//            terms O V^T on the matrix cores, with tokens on the lane axis of the
//            accumulators so that the sum over window rows and query heads (Eq. 9,
//            Appendix A.5) runs down registers; A^2 = exp2(2 log2e Z - 2 log2(max-shifted
//            sum)) and the three scores are formed in fp32.  The attention-only score
//            of Eq. 8 and its l1-weighted form need Z only and skip the cross terms.
//
// Both sweeps walk their tokens in blocks of 32.  Sweep 1 is software-pipelined inside a
// wave: while the vector ALUs turn block n's accumulators into softmax weights, the matrix
// cores already work on block n+1's K Q^T and on block n-1's P V product; the streams of
// one step are independent, sit in one basic block, and the instruction scheduler
// interleaves them.  Sweep 2 exists in two forms.  The one in this file gives a wave 32 rows, runs
// a block's matrix phase and vector phase back to back and leaves the overlap to the second wave
// on the SIMD (its stationary operands and row constants leave no registers for a second set of
// accumulators).  The register-blocked form (score_mfma_wide.hip: 64 rows per wave, stationary
// operands in the accumulator file, the wave pipelined against itself) serves the key, joint and
// all-three variants whenever every 128-row chunk is at least three quarters full.  K and V travel
// HBM -> LDS with direct-to-LDS loads: in sweep 1 as 32-token blocks through four-slot rings, three
// batches in flight; in sweep 2 as 64-token tiles, double-buffered here, a four-slot ring there.
//
// Precision.  The matrix cores take bf16 operands, and rows whose attention is
// concentrated on a few keys are sensitive to that rounding (the scores of those keys
// depend on v_p - o_i, a difference of nearly equal vectors).  Two operands are therefore
// fed as an exact-enough pair of bf16 pieces (high part + residual, 16 significant bits):
// the softmax weights P in O^T += V^T P^T, and o_i in the cross term O V^T.  Both pieces
// reuse the same LDS operand, so the cost is matrix-core issue slots only.
// ||v_p - o_i||^2 is evaluated as ||v_p||^2 - 2 v_p.o^_i + ||o^_i||^2 with o^_i the
// two-piece value used by the matrix cores in BOTH the cross term and the norm, so the
// expression is the exact squared distance to o^_i.
//
// Rows dominated by one key (an attention sink, the token's own key) would still lose
// v_p - o_i of that key to cancellation: o_i is then v_p plus a small remainder.  The first
// sweep therefore keeps, per row, the one key that may end up dominant out of its sums (a new
// running maximum that clears the old one by ln 9: no other key can reach a share of 0.9), and the
// combine step forms v_p - o_i = (1 - A_ip)(v_p - mean of the others) for that key directly.
// The (row, key) pair is scored there in fp32 when its share is large, and the second sweep
// skips it.  One pass serves every input: nothing is rescanned for rows that turn out dominated.
//
// A and Z never touch HBM.  All sums have a fixed order: results are bit-reproducible.
#include "internal.h"
#include "mfma_util.h"

namespace obc {
using namespace mfma;
namespace {

// ------------------------------------------------------------------------------------
// Sweep 1
// ------------------------------------------------------------------------------------
struct Sweep1Regs {
    bf16x8 q[8];          // stationary B operand: this lane's query row, pieces 2 kk + half
    f32x16 oacc[4];       // O^T accumulators: head_dim block x 16 registers
    f32x16 s_cur;         // raw q.k of the block whose softmax is due
    PiecePair phi[2], plo[2];   // two-piece softmax weights of the previous block, per k-step
    float p[16];          // the same weights in fp32, from the step that formed them to the step that packs them
    float m_ref, m_true;  // reference of the running sums (raw q.k units, see kLazyRescale); true running max
    float lsum;           // this lane's share of the running sum
    float alpha;          // rescale of oacc still owed from the previous step (1 = none)
    bool rescale;         // uniform: some row of the wave owes a rescale
    // With kNeedO only: the row's candidate for a dominant key, kept out of lsum and oacc.
    float cand_val;       // its raw q.k (-inf: none yet)
    int cand_tok;         // its token (-1: none yet)
    int n_ev;             // former candidates parked in this lane's LDS list, to be added back at the end
};

// A key can end up with more than a share s of a row's attention only if its logit exceeds every
// other one by ln(s / (1 - s)); a new running maximum that clears the old one by less can never
// get there and stays an ordinary key.  The margin below is the one for s = 0.9: rows without a held
// key have no key above that share, which bounds the cancellation in v_p - o_i to a factor 10.
constexpr float kCandMargin = 2.1972245773362196f / kInvSqrtD;   // ln(0.9 / 0.1), in raw q.k units
constexpr float kSeparateShare = 0.5f;   // a candidate holding at least this share of its row is scored by the combine step
constexpr int kEvents = 4;               // former candidates a lane can park

// Adds a former candidate (token `tok`, raw logit `val`) back into this lane's sums: weight
// exp2((val - ref_l) c2) into lsum (one half-wave only, the halves are added at the end) and
// exp2((val - ref_o) c2) v_tok into the lane's 64 entries of O^T.
__device__ __forceinline__ void add_back_fetch(uint2 (&x)[16], const char *vh, int tok, int half) {
    const char *vrow = vh + (size_t)tok * kRowBytes;
#pragma unroll
    for (int ddb = 0; ddb < 4; ++ddb)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) x[ddb * 4 + r4] = *(const uint2 *)(vrow + (ddb * 32 + 8 * r4 + 4 * half) * 2);
}

__device__ __forceinline__ void add_back_apply(Sweep1Regs &R, const uint2 (&x)[16], float val, float ref_l, float ref_o,
                                               int half) {
    const float c2 = kLog2e * kInvSqrtD;
    const float w_o = __builtin_amdgcn_exp2f((val - ref_o) * c2);
    if (half == 0) R.lsum += __builtin_amdgcn_exp2f((val - ref_l) * c2);
#pragma unroll
    for (int ddb = 0; ddb < 4; ++ddb)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            const uint2 w = x[ddb * 4 + r4];
            R.oacc[ddb][4 * r4 + 0] = fmaf(w_o, __uint_as_float(w.x << 16), R.oacc[ddb][4 * r4 + 0]);
            R.oacc[ddb][4 * r4 + 1] = fmaf(w_o, __uint_as_float(w.x & 0xffff0000u), R.oacc[ddb][4 * r4 + 1]);
            R.oacc[ddb][4 * r4 + 2] = fmaf(w_o, __uint_as_float(w.y << 16), R.oacc[ddb][4 * r4 + 2]);
            R.oacc[ddb][4 * r4 + 3] = fmaf(w_o, __uint_as_float(w.y & 0xffff0000u), R.oacc[ddb][4 * r4 + 3]);
        }
}

__device__ __forceinline__ void add_back(Sweep1Regs &R, const char *vh, int tok, float val, float ref_l, float ref_o,
                                         int half) {
    uint2 x[16];
    add_back_fetch(x, vh, tok, half);
    add_back_apply(R, x, val, ref_l, ref_o, half);
}

// P = hi + lo for the matrix cores: hi keeps the top 16 bits of the fp32 weight (a bf16 by truncation), lo is the
// exact remainder rounded to bf16.
__device__ __forceinline__ void pack_weights(Sweep1Regs &R) {
#pragma unroll
    for (int sx = 0; sx < 2; ++sx)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float p0 = R.p[8 * sx + 2 * e], p1 = R.p[8 * sx + 2 * e + 1];
            const uint32_t h0 = __float_as_uint(p0) & 0xffff0000u, h1 = __float_as_uint(p1) & 0xffff0000u;
            R.phi[sx].u[e] = __builtin_amdgcn_perm(h1, h0, 0x07060302u);     // {h0 >> 16, h1 >> 16}
            R.plo[sx].u[e] = pack_bf16(p0 - __uint_as_float(h0), p1 - __uint_as_float(h1));
        }
}

// One pipeline step n of sweep 1 (PH = n mod 4 fixes every LDS slot at compile time):
//   matrix cores: O^T += V^T P^T of block n-1, S^T = K Q^T of block n+1
//   vector ALUs : online softmax of block n
// Every step first waits for the two blocks it reads, meets the other waves at a barrier and
// starts the loads of the blocks three steps ahead.
//
// With kNeedO (Eq. 5, 6) every row keeps its candidate for a dominant key (see kCandMargin) out of
// its sums.  The step is then cut in two: K Q^T and the block's row maxima first; a vote whether
// some row of the wave meets a new candidate in block n, and (rarely) the branch that deals with
// it; then V^T P^T and the weights.  Without kNeedO the step is one basic block.
template <int PH, bool kMasked, bool kNeedO>
__device__ __forceinline__ void sweep1_step(Sweep1Regs &R, const char *smem, uint32_t lds0, int n, int t_begin,
                                            int t_end, int last_row, int vis, const char *kh, const char *vh,
                                            const int (&koff)[8], const int (&voff)[4], const uint32_t (&kdoff)[2],
                                            const uint32_t (&vdoff)[2], int wave, int lane, bool wave_active,
                                            int2 *events) {
    // K and V blocks live in rings of four 8 KB slots each (block j in slot j mod 4): K block
    // n+1 and V block n-1, both started three steps ago, are waited for here while the two
    // younger batches stay in flight; then K block n+4 and V block n+2 start in the slots
    // the previous step has finished with.  Blocks past the end of the split are fetched
    // too (rows clamp to the last one), so that every batch has the same number of transfers.
    constexpr int kKBase = ((PH + 1) & 3) * kBlkBytes;                  // block n+1
    constexpr int kVBase = (4 + ((PH + 3) & 3)) * kBlkBytes;            // block n-1
    const float c2 = kLog2e * kInvSqrtD;
    const int half = lane >> 5;

    wait_async_loads_keep<kNeedO ? 8 : 4>();
    __syncthreads();
    block_load_async<kXor16>(kh, t_begin + (n + 4) * 32, last_row, lds0 + PH * kBlkBytes, wave, lane, kdoff);
    if (kNeedO)
        block_load_async<kRot4>(vh, t_begin + (n + 2) * 32, last_row, lds0 + (4 + ((PH + 2) & 3)) * kBlkBytes, wave, lane, vdoff);
    if (!wave_active) return;

    // ---- matrix cores: block n+1 ----
    // (with kNeedO the operand reads of the whole chain are issued up front, so that one LDS latency is exposed
    // instead of one per pair of matrix ops, and the first value operands follow them ahead of the vote below)
    f32x16 s_next = zero16();
    bf16x8 ka[8], va0[4];
    if (kNeedO) {
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) ka[kk] = lds_read16(smem + kKBase + koff[kk]);
#pragma unroll
        for (int ddb = 0; ddb < 4; ++ddb) va0[ddb] = lds_read_vt(smem + kVBase + voff[ddb]);
        __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
        const bf16x8 a = kNeedO ? ka[kk] : lds_read16(smem + kKBase + koff[kk]);
        s_next = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, R.q[kk], s_next, 0, 0, 0);
    }
    // ---- vector ALUs: block n-1's weights into operand form, in the shadow of the chain above (the second part of
    // the step, whose matrix ops they feed, has the exponentials of block n for company) ----
    if (kNeedO) {
        pack_weights(R);
#pragma unroll
        for (int sx = 0; sx < 2; ++sx)
#pragma unroll
            for (int e = 0; e < 4; ++e) {       // (pinned here: left alone, the packing sinks into the step's second part)
                asm volatile("" : "+v"(R.phi[sx].u[e]));
                asm volatile("" : "+v"(R.plo[sx].u[e]));
            }
#pragma unroll
        for (int i = 0; i < 8; ++i) {           // one matrix op, then its share of the packing
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 7, 0);
        }
    }
    // ---- vector ALUs: block n ----
    f32x16 s = R.s_cur;
    if (kMasked) {
        const int tok0 = t_begin + n * 32;      // register r holds token tok0 + 8 (r / 4) + 4 half + r % 4
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int tok = tok0 + 8 * (r >> 2) + 4 * half + (r & 3);
            if (tok > vis || tok >= t_end) s[r] = -INFINITY;
        }
    }
    float mx = max3(s[0], s[1], s[2]);
#pragma unroll
    for (int r = 3; r < 15; r += 2) mx = max3(mx, s[r], s[r + 1]);
    mx = fmaxf(mx, s[15]);
    mx = halves_max(mx);
    if (kNeedO) {
        // Rows whose block maximum clears their running maximum (and the block's other keys) by the margin
        // take the block's first key of that logit as their candidate: its logit becomes -inf before the
        // weights are formed, so it never enters this block's P or sum, and the previous candidate is parked
        // (or, with the list full, added back on the spot).  (-inf + margin = -inf: in a row's first visible
        // block only the block's other keys decide.)
        const float m_true_before = R.m_true;
        if (R.rescale || __any(mx > m_true_before + kCandMargin)) {    // uniform; one branch for both rare events
            // The running max moved in the previous step: bring the accumulated O^T (blocks <= n-2)
            // to the new reference before block n-1, whose weights already use it, is added.
            if (R.rescale) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) R.oacc[i][r] *= R.alpha;
            }
            if (mx > m_true_before + kCandMargin) {
                uint32_t hit = 0;
#pragma unroll
                for (int r = 0; r < 16; ++r) hit |= s[r] == mx ? (1u << r) : 0u;
                // (a lane's registers ascend with their tokens: its lowest set bit is its first such key)
                const int rc_own = hit ? __builtin_ctz(hit) : 0;
                const int off_own = hit ? 8 * (rc_own >> 2) + 4 * half + (rc_own & 3) : 64;
                float off_lower, off_upper;
                both_halves(__int_as_float(off_own), off_lower, off_upper);      // (bits only)
                const int off_first = min(__float_as_int(off_lower), __float_as_int(off_upper));
                const int rc = off_own == off_first ? rc_own : -1;              // its register, if in this lane
                // It must clear the other keys of its own block by the margin as well.
                float others = -INFINITY;
#pragma unroll
                for (int r = 0; r < 16; ++r) others = fmaxf(others, r == rc ? -INFINITY : s[r]);
                others = halves_max(others);
                if (mx > others + kCandMargin) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) s[r] = r == rc ? -INFINITY : s[r];
                    if (R.cand_tok >= 0) {                             // the previous candidate is an ordinary key after all
                        if (R.n_ev < kEvents) {
                            events[R.n_ev] = make_int2(R.cand_tok, __float_as_int(R.cand_val));
                            R.n_ev += 1;
                        } else {
                            // (sum and O^T both stand at the current reference: the owed rescale was applied above)
                            add_back(R, vh, R.cand_tok, R.cand_val, R.m_ref, R.m_ref, half);
                        }
                    }
                    R.cand_tok = t_begin + n * 32 + off_first;
                    R.cand_val = mx;
                }
            }
        }
        // ---- matrix cores: block n-1 ----
#pragma unroll
        for (int sx = 0; sx < 2; ++sx)
#pragma unroll
            for (int ddb = 0; ddb < 4; ++ddb) {
                const bf16x8 a = sx == 0 ? va0[ddb] : lds_read_vt(smem + kVBase + 16 * kRowBytes + voff[ddb]);
                R.oacc[ddb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, R.phi[sx].v, R.oacc[ddb], 0, 0, 0);
                R.oacc[ddb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, R.plo[sx].v, R.oacc[ddb], 0, 0, 0);
            }
    }
    // The reference may follow a candidate's logit: it only has to bound the weights from above.
    R.m_true = fmaxf(R.m_true, mx);
    const bool moved = mx > R.m_ref + kLazyRescale;                    // also true for the first visible key
    const float m_new = moved ? mx : R.m_ref;
    float alpha = __builtin_amdgcn_exp2f((R.m_ref - m_new) * c2);      // 1 when the reference stays; exp2(-inf) = 0
    float mref = m_new * c2;
    if (kMasked) {                                                     // rows with nothing visible yet
        alpha = moved ? alpha : 1.0f;
        mref = m_new == -INFINITY ? 0.f : mref;
    }
    R.m_ref = m_new;
    float psum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        R.p[r] = __builtin_amdgcn_exp2f(fmaf(s[r], c2, -mref));
        psum += R.p[r];
    }
    R.lsum = fmaf(R.lsum, alpha, psum);
    if (kNeedO) {
        R.alpha = alpha;
        R.rescale = __any(moved);      // uniform and rare once the running max has settled
    }
    R.s_cur = s_next;
    if (kNeedO) {
        // second part: the remaining value operands first, then one matrix op per three vector ops (the exponentials go along)
        __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);
        }
    } else {
        interleave_hint<8, 12, 1>();
    }
}

// Grid: x = sequence split, y = 128-row chunk, z = (b, KV head).
// With kNeedO every row keeps its candidate for a dominant key (see kCandMargin) out of its sums and
// reports it with the partial record; the combine step then forms v_cand - o_i without
// cancellation for every row, and no row ever needs a second pass.
template <bool kNeedO>
__global__ __launch_bounds__(kThreads, 2) void mfma_sweep1(const uint16_t *__restrict__ q,
                                                           const uint16_t *__restrict__ k,
                                                           const uint16_t *__restrict__ v, int N, int W, int Hq,
                                                           int Hkv, int ragged, SeqLens lens, int split_len,
                                                           int n_splits, int m_pad, float *__restrict__ part_ml,
                                                           float *__restrict__ part_o) {
    __shared__ __attribute__((aligned(1024))) char smem[kLdsTiles];
    __shared__ int2 ev_list[kNeedO ? kThreads * kEvents : 1];   // per lane: parked former candidates (token, logit bits)
    int2 *events = ev_list + (kNeedO ? threadIdx.x * kEvents : 0);

    const int split = blockIdx.x, chunk = blockIdx.y, bg = blockIdx.z;
    const int b = bg / Hkv, g = bg % Hkv, G = Hq / Hkv, M = G * W;
    const int len = seq_len_of(lens, ragged, b, N);
    const int t_begin = split * split_len;
    if (t_begin >= len) return;                                  // uniform: nothing of this split is live
    const int t_end = min(t_begin + split_len, len);

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63, half = lane >> 5;
    const int rb = chunk * 4 + wave;                             // row block of this wave
    const int row = rb * 32 + (lane & 31);                       // window row (i) owned by this lane
    const bool wave_active = rb * 32 < M;                        // uniform
    const bool row_valid = row < M;
    // Last key the row may see (Eq. 9 window rows are causal).  Padded rows carry a zero
    // query and see everything: they stay finite and are discarded later.
    const int vis = row_valid ? len - W + (row % W) : len - 1;
    int vis_min = vis;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) vis_min = min(vis_min, __shfl_xor(vis_min, off));
    vis_min = __builtin_amdgcn_readfirstlane(min(vis_min, t_end - 1));

    const char *kh = (const char *)k + (size_t)bg * N * kRowBytes;
    const char *vh = (const char *)v + (size_t)bg * N * kRowBytes;
    const uint32_t lds0 = lds_offset_of(smem);

    int koff[8], voff[4];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) koff[kk] = row_piece_offset(lane, kk);
#pragma unroll
    for (int ddb = 0; ddb < 4; ++ddb) voff[ddb] = vt_piece_offset(lane, ddb);

    Sweep1Regs R;
    {
        const char *qrow = (const char *)q + (((size_t)b * Hq + (size_t)g * G) * W + row) * kRowBytes;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            if (row_valid) R.q[kk] = *(const bf16x8 *)(qrow + (2 * kk + half) * 16);
            else R.q[kk] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) R.oacc[i] = zero16();
#pragma unroll
    for (int sx = 0; sx < 2; ++sx)
#pragma unroll
        for (int e = 0; e < 4; ++e) { R.phi[sx].u[e] = 0; R.plo[sx].u[e] = 0; }
#pragma unroll
    for (int r = 0; r < 16; ++r) R.p[r] = 0.f;
    R.m_ref = -INFINITY;
    R.m_true = -INFINITY;
    R.lsum = 0.f;
    R.alpha = 1.0f;
    R.rescale = false;
    R.cand_val = -INFINITY;
    R.cand_tok = -1;
    R.n_ev = 0;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) settle(R.q[kk]);

    // Prologue.  Step 0 multiplies zero weights with whatever "V block -1" (slot 3 of the V ring)
    // holds, so that slot is cleared.  K blocks 0..3 and V blocks 0..1 are started (the batches
    // the steps -4..-1 would have started), K block 0 is waited for and block 0's S^T formed.
    uint32_t kdoff[2], vdoff[2];
    block_lane_offsets<kXor16>(kdoff, wave, lane);
    block_lane_offsets<kRot4>(vdoff, wave, lane);
    for (int e = threadIdx.x; e < kBlkBytes / 16; e += kThreads) ((uint4 *)(smem + 7 * kBlkBytes))[e] = make_uint4(0, 0, 0, 0);
    block_load_async<kXor16>(kh, t_begin, len - 1, lds0, wave, lane, kdoff);
    block_load_async<kXor16>(kh, t_begin + 32, len - 1, lds0 + kBlkBytes, wave, lane, kdoff);
    block_load_async<kXor16>(kh, t_begin + 64, len - 1, lds0 + 2 * kBlkBytes, wave, lane, kdoff);
    if (kNeedO) block_load_async<kRot4>(vh, t_begin, len - 1, lds0 + 4 * kBlkBytes, wave, lane, vdoff);
    block_load_async<kXor16>(kh, t_begin + 96, len - 1, lds0 + 3 * kBlkBytes, wave, lane, kdoff);
    if (kNeedO) block_load_async<kRot4>(vh, t_begin + 32, len - 1, lds0 + 5 * kBlkBytes, wave, lane, vdoff);
    wait_async_loads_keep<kNeedO ? 10 : 6>();         // everything after K block 0 may still be in flight
    __syncthreads();
    R.s_cur = zero16();
    if (wave_active) {
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            const bf16x8 a = lds_read16(smem + koff[kk]);
            R.s_cur = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, R.q[kk], R.s_cur, 0, 0, 0);
        }
    }

    const int n_blk = (t_end - t_begin + 31) / 32;
    const int n_total = (n_blk + 3) & ~3;
    int n_plain = (vis_min + 1 - t_begin) / 32;       // leading blocks every row of this wave sees in full
    n_plain = max(0, min(n_plain, n_blk)) & ~3;
#define OBC_S1_ARGS smem, lds0, n, t_begin, t_end, len - 1, vis, kh, vh, koff, voff, kdoff, vdoff, wave, lane, wave_active, events
    int n = 0;
    for (; n < n_plain; n += 4) {
        sweep1_step<0, false, kNeedO>(R, OBC_S1_ARGS); ++n;
        sweep1_step<1, false, kNeedO>(R, OBC_S1_ARGS); ++n;
        sweep1_step<2, false, kNeedO>(R, OBC_S1_ARGS); ++n;
        sweep1_step<3, false, kNeedO>(R, OBC_S1_ARGS); n -= 3;
    }
    for (; n < n_total; n += 4) {
        sweep1_step<0, true, kNeedO>(R, OBC_S1_ARGS); ++n;
        sweep1_step<1, true, kNeedO>(R, OBC_S1_ARGS); ++n;
        sweep1_step<2, true, kNeedO>(R, OBC_S1_ARGS); ++n;
        sweep1_step<3, true, kNeedO>(R, OBC_S1_ARGS); n -= 3;
    }
#undef OBC_S1_ARGS
    // A final candidate that holds less than half of its own split's weight cannot dominate the
    // row; it joins the parked former candidates, which are ordinary keys and are added back below, now that
    // the reference is final.  The first one's value row is fetched ahead of the waits that follow.
    uint2 first_row[16];
    int2 first_ev = make_int2(-1, 0);
    if (kNeedO && wave_active) {
        const float c2 = kLog2e * kInvSqrtD;
        const float l_rest = halves_sum(R.lsum);
        if (R.cand_tok >= 0 && __builtin_amdgcn_exp2f((R.cand_val - R.m_ref) * c2) < l_rest) {
            if (R.n_ev < kEvents) {
                events[R.n_ev] = make_int2(R.cand_tok, __float_as_int(R.cand_val));
                R.n_ev += 1;
                R.cand_tok = -1;
            }
        }
        if (R.n_ev > 0) {
            first_ev = events[0];
            add_back_fetch(first_row, vh, first_ev.x, half);
        }
    }
    wait_async_loads();        // the blocks fetched past the end must have landed before the LDS is given back
    if (kNeedO && wave_active) {      // drain: P V of the last block (n_total - 1, in slot 3 of the V ring)
        pack_weights(R);
        if (R.rescale) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) R.oacc[i][r] *= R.alpha;
        }
#pragma unroll
        for (int ddb = 0; ddb < 4; ++ddb)
#pragma unroll
            for (int sx = 0; sx < 2; ++sx) {
                const bf16x8 a = lds_read_vt(smem + 7 * kBlkBytes + 16 * sx * kRowBytes + voff[ddb]);
                R.oacc[ddb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, R.phi[sx].v, R.oacc[ddb], 0, 0, 0);
                R.oacc[ddb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, R.plo[sx].v, R.oacc[ddb], 0, 0, 0);
            }
        if (first_ev.x >= 0) add_back_apply(R, first_row, __int_as_float(first_ev.y), R.m_ref, R.m_ref, half);
        for (int e = 1; e < kEvents; ++e) {
            if (!__any(e < R.n_ev)) break;       // uniform
            if (e < R.n_ev) {
                const int2 ev = events[e];
                add_back(R, vh, ev.x, __int_as_float(ev.y), R.m_ref, R.m_ref, half);
            }
        }
    }
    if (kNeedO) __syncthreads();      // every wave is done with the rings: their space now stages the output rows
    if (!wave_active) return;
    const float lrow = halves_sum(R.lsum);
    const size_t prow0 = ((size_t)bg * n_splits + split) * m_pad + rb * 32;     // the wave's first row
    if (half == 0)                    // reference in raw q.k units (-inf when the split holds no visible key), sum, candidate
        *(float4 *)(part_ml + (prow0 + (lane & 31)) * 4) =
            make_float4(R.m_ref, lrow, kNeedO ? R.cand_val : R.m_true, __int_as_float(kNeedO ? R.cand_tok : 0));
    if (kNeedO) {
        // A lane holds 64 scattered entries of its row: written straight out, every store would touch 64 rows' worth of
        // cache lines 16 bytes at a time.  The wave's 32 rows pass through its own 16 KB of LDS instead (16-byte slot c
        // of row r at slot c ^ r: conflict-free both ways) and leave as whole rows, 1 KB per store.
        char *stage = smem + wave * (32 * kD * 4);
        const int r = lane & 31;
#pragma unroll
        for (int ddb = 0; ddb < 4; ++ddb)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const int c = ddb * 8 + 2 * r4 + half;
                *(float4 *)(stage + r * (kD * 4) + ((c ^ r) << 4)) =
                    make_float4(R.oacc[ddb][4 * r4], R.oacc[ddb][4 * r4 + 1], R.oacc[ddb][4 * r4 + 2], R.oacc[ddb][4 * r4 + 3]);
            }
        // (a wave's LDS operations complete in order: its reads below see its writes above; no other wave touches them)
        float *dst = part_o + prow0 * kD;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int row_i = 2 * i + half, c = lane & 31;
            const f32x4 x = *(const f32x4 *)(stage + row_i * (kD * 4) + ((c ^ row_i) << 4));
            // (streaming store: the partials are read once, by the combine step, and 35 MB of them kept dirty in the
            // L2 would all be written back when the kernel ends)
            __builtin_nontemporal_store(x, (f32x4 *)(dst + row_i * kD + 4 * c));
        }
    }
}

// ------------------------------------------------------------------------------------
// Combine: one 128-thread block per (KV head, padded row); thread = head_dim element.
// ------------------------------------------------------------------------------------
// Variants that need no o_i (Eq. 4, Eq. 8 and its l1-weighted form): the splits' row sums are merged into the
// one constant per row the second sweep turns logits into weights with.
__global__ __launch_bounds__(128) void mfma_combine(const float *__restrict__ part_ml, int N, int W, int Hq, int Hkv,
                                                    int ragged, SeqLens lens, int split_len, int n_splits,
                                                    int m_pad, uint16_t *__restrict__ out_bf16,
                                                    float *__restrict__ row_const, float *__restrict__ special) {
    const int row = blockIdx.x, bg = blockIdx.y;
    const int b = bg / Hkv, G = Hq / Hkv, M = G * W;
    const int len = seq_len_of(lens, ragged, b, N);
    const int dd = threadIdx.x;
    const size_t crow = (size_t)bg * m_pad + row;
    const size_t lo_plane = (size_t)gridDim.y * m_pad * kD;   // residual pieces follow the high pieces
    out_bf16[crow * kD + dd] = 0;                     // (no cross term: the operand is never read, and stays defined)
    out_bf16[lo_plane + crow * kD + dd] = 0;
    if (dd != 0) return;
    special[crow * 4 + 0] = __int_as_float(-1);       // no separately scored (row, token) pair
    row_const[crow * 4 + 1] = 0.f;
    row_const[crow * 4 + 3] = 0.f;
    if (row >= M) {                                   // padded row: weightless in the second sweep
        row_const[crow * 4 + 0] = 1e30f;
        row_const[crow * 4 + 2] = __int_as_float(-1);
        return;
    }
    const int live_splits = (len + split_len - 1) / split_len;
    const float c2 = kLog2e * kInvSqrtD;
    // Splits are merged sixteen at a time, every load of a batch issued before the first use.  The running sum
    // follows the running max of the raw dot products; a split's sum is relative to its own reference.
    float m_raw = -INFINITY, l = 0.f;
    for (int s0 = 0; s0 < live_splits; s0 += 16) {
        float4 ml[16];
#pragma unroll
        for (int j = 0; j < 16; ++j)      // (clamped slots are ignored below)
            ml[j] = ((const float4 *)part_ml)[((size_t)bg * n_splits + min(s0 + j, live_splits - 1)) * m_pad + row];
        float m_new = m_raw;
#pragma unroll
        for (int j = 0; j < 16; ++j)
            if (s0 + j < live_splits) m_new = fmaxf(m_new, ml[j].z);
        l *= m_raw == -INFINITY ? 0.f : exp2f((m_raw - m_new) * c2);
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            if (s0 + j >= live_splits) continue;
            l = fmaf(ml[j].x == -INFINITY ? 0.f : exp2f((ml[j].x - m_new) * c2), ml[j].y, l);
        }
        m_raw = m_new;
    }
    row_const[crow * 4 + 0] = 2.0f * (m_raw * c2 + log2f(l));   // A_ip^2 = exp2(2 log2e Z_ip - this)
    row_const[crow * 4 + 2] = __int_as_float(len - W + (row % W));
}

// Variants that need o_i (Eq. 5, 6): the same grid.  Every split reports, per row, its sums without its
// candidate key and the candidate itself.  The candidate with the largest logit (the first split on
// ties) stays held out; the others are ordinary keys and are added back from the value cache.  With
// l' and O' the sums over every key but that one, relative to a common reference T,
//     w = exp2((z_cand - T) c2),   A_cand = w / (w + l'),
//     v_cand - o_i = l' / (w + l') * (v_cand - O' / l'),      o_i = v_cand - (v_cand - o_i)
// without cancellation however much of the row's attention the candidate holds.  A candidate that
// holds a large share is scored here from these (`special`) and skipped by the second sweep.
// Grid: x = group of four padded rows, y = (b, KV head); 32 lanes per row, four head_dim elements per lane.
__global__ __launch_bounds__(128) void mfma_combine_hold(const uint16_t *__restrict__ v,
                                                         const float *__restrict__ part_ml,
                                                         const float *__restrict__ part_o, int N, int W, int Hq,
                                                         int Hkv, int ragged, SeqLens lens, int split_len,
                                                         int n_splits, int m_pad, uint16_t *__restrict__ out_bf16,
                                                         float *__restrict__ row_const,
                                                         float *__restrict__ special) {
    const int row = blockIdx.x * 4 + (threadIdx.x >> 5), bg = blockIdx.y;
    const int b = bg / Hkv, G = Hq / Hkv, M = G * W;
    const int len = seq_len_of(lens, ragged, b, N);
    const int sub = threadIdx.x & 31, dd = sub * 4;   // this lane's elements dd .. dd + 3
    const size_t crow = (size_t)bg * m_pad + row;
    const size_t lo_plane = (size_t)gridDim.y * m_pad * kD;
    const bool live = row < M;                        // the same for the 32 lanes of a row
    const int live_splits = (len + split_len - 1) / split_len;
    const float c2 = kLog2e * kInvSqrtD;
    const uint16_t *vg = v + (size_t)bg * N * kD;
    // First the common reference T (no sum lies more than the lazy-rescale slack above its own
    // reference, so the largest reference or candidate logit will do) and the winning candidate.
    // The first 16 splits' records and sums are fetched in one go and stay in registers.
    float T = -INFINITY, c_val = -INFINITY;
    int c_tok = -1, s_star = -1;
    float4 ml[16], po[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        const size_t prow = ((size_t)bg * n_splits + min(j, live_splits - 1)) * m_pad + row;
        ml[j] = ((const float4 *)part_ml)[prow];
        po[j] = *(const float4 *)(part_o + prow * kD + dd);
    }
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        if (j >= live_splits) continue;
        T = fmaxf(T, fmaxf(ml[j].x, ml[j].z));
        const int tok = __float_as_int(ml[j].w);
        if (tok >= 0 && ml[j].z > c_val) { c_val = ml[j].z; c_tok = tok; s_star = j; }
    }
    for (int s0 = 16; s0 < live_splits; s0 += 16) {
        float4 mm[16];
#pragma unroll
        for (int j = 0; j < 16; ++j)
            mm[j] = ((const float4 *)part_ml)[((size_t)bg * n_splits + min(s0 + j, live_splits - 1)) * m_pad + row];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            if (s0 + j >= live_splits) continue;
            T = fmaxf(T, fmaxf(mm[j].x, mm[j].z));
            const int tok = __float_as_int(mm[j].w);
            if (tok >= 0 && mm[j].z > c_val) { c_val = mm[j].z; c_tok = tok; s_star = s0 + j; }
        }
    }
    if (!live) { c_tok = -1; s_star = -1; }           // padded rows: zero queries, nothing of theirs is used
    const uint2 vt_bits = c_tok >= 0 ? *(const uint2 *)(vg + (size_t)c_tok * kD + dd) : make_uint2(0u, 0u);
    float l = 0.f, o[4] = {0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < live_splits; s0 += 16) {
        uint2 vo[16];
        if (s0 > 0) {
#pragma unroll
            for (int j = 0; j < 16; ++j) {         // (the records are in cache from the pass above)
                const size_t prow = ((size_t)bg * n_splits + min(s0 + j, live_splits - 1)) * m_pad + row;
                ml[j] = ((const float4 *)part_ml)[prow];
                po[j] = *(const float4 *)(part_o + prow * kD + dd);
            }
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int tok = __float_as_int(ml[j].w);
            const bool back = live && s0 + j < live_splits && s0 + j != s_star && tok >= 0;
            vo[j] = back ? *(const uint2 *)(vg + (size_t)tok * kD + dd) : make_uint2(0u, 0u);
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            if (s0 + j >= live_splits) continue;
            const float w = ml[j].x == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((ml[j].x - T) * c2);
            l = fmaf(w, ml[j].y, l);
            o[0] = fmaf(w, po[j].x, o[0]);
            o[1] = fmaf(w, po[j].y, o[1]);
            o[2] = fmaf(w, po[j].z, o[2]);
            o[3] = fmaf(w, po[j].w, o[3]);
            if (live && s0 + j != s_star && __float_as_int(ml[j].w) >= 0) {   // this split's candidate is an ordinary key
                const float wc = __builtin_amdgcn_exp2f((ml[j].z - T) * c2);
                l += wc;
                o[0] = fmaf(wc, __uint_as_float(vo[j].x << 16), o[0]);
                o[1] = fmaf(wc, __uint_as_float(vo[j].x & 0xffff0000u), o[1]);
                o[2] = fmaf(wc, __uint_as_float(vo[j].y << 16), o[2]);
                o[3] = fmaf(wc, __uint_as_float(vo[j].y & 0xffff0000u), o[3]);
            }
        }
    }
    // (no split may have kept a candidate: then w = 0 and o_i = O' / l' as usual)
    const float wc = c_tok >= 0 ? __builtin_amdgcn_exp2f((c_val - T) * c2) : 0.f;
    const float ltot = wc + l;
    const float inv = 1.0f / ltot;
    const float inv_l = l > 0.f ? 1.0f / l : 0.f;
    const float z = c_val * kInvSqrtD;               // Z of the (row, candidate) pair
    const float vt[4] = {__uint_as_float(vt_bits.x << 16), __uint_as_float(vt_bits.x & 0xffff0000u),
                         __uint_as_float(vt_bits.y << 16), __uint_as_float(vt_bits.y & 0xffff0000u)};
    uint16_t ob[4], olo[4];
    float s_oo = 0.f, s_vv = 0.f, s_dd = 0.f, s_cc = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float diff = (l * inv) * (vt[e] - o[e] * inv_l);     // (v_cand - o_i)[dd + e]
        const float oi = vt[e] - diff;
        const float comb = fmaf(z, diff, vt[e]);                   // ((1+Z) v_cand - Z o_i)[dd + e]
        // o^ = hi + lo, the pair of bf16 pieces the second sweep feeds to the matrix cores.
        ob[e] = (uint16_t)(__float_as_uint(oi) >> 16);
        const float ohi = bf16_bits_to_float(ob[e]);
        olo[e] = (uint16_t)(pack_bf16(oi - ohi, 0.f) & 0xffffu);
        const float of = ohi + bf16_bits_to_float(olo[e]);
        s_oo = fmaf(of, of, s_oo);
        s_vv = fmaf(vt[e], vt[e], s_vv);
        s_dd = fmaf(diff, diff, s_dd);
        s_cc = fmaf(comb, comb, s_cc);
    }
    // A candidate with a small share is scored by the second sweep like any other key (its o_i is exact either
    // way); one that may dominate is scored here and skipped there.
    const float a = wc * inv;
    const bool separate = live && a >= kSeparateShare;
    s_oo = row_sum32(s_oo);
    if (__any(separate)) { s_vv = row_sum32(s_vv); s_dd = row_sum32(s_dd); s_cc = row_sum32(s_cc); }
    uint2 hi_bits, lo_bits;
    hi_bits.x = live ? (uint32_t)cross_operand_bf16(ob[0]) | ((uint32_t)cross_operand_bf16(ob[1]) << 16) : 0u;
    hi_bits.y = live ? (uint32_t)cross_operand_bf16(ob[2]) | ((uint32_t)cross_operand_bf16(ob[3]) << 16) : 0u;
    lo_bits.x = live ? (uint32_t)cross_operand_bf16(olo[0]) | ((uint32_t)cross_operand_bf16(olo[1]) << 16) : 0u;
    lo_bits.y = live ? (uint32_t)cross_operand_bf16(olo[2]) | ((uint32_t)cross_operand_bf16(olo[3]) << 16) : 0u;
    *(uint2 *)(out_bf16 + crow * kD + dd) = hi_bits;
    *(uint2 *)(out_bf16 + lo_plane + crow * kD + dd) = lo_bits;
    if (sub != 0) return;
    if (!live) {                                      // padded row: weightless in the second sweep
        row_const[crow * 4 + 0] = 1e30f;
        row_const[crow * 4 + 1] = 0.f;
        row_const[crow * 4 + 2] = __int_as_float(-1);
        row_const[crow * 4 + 3] = 0.f;
        special[crow * 4 + 0] = __int_as_float(-1);
        return;
    }
    const float a2 = a * a;
    row_const[crow * 4 + 0] = 2.0f * (T * c2 + log2f(ltot));   // A_ip^2 = exp2(2 log2e Z_ip - this)
    row_const[crow * 4 + 1] = s_oo * kCrossScale;              // ||o^_i||^2 / 128
    row_const[crow * 4 + 2] = __int_as_float(len - W + (row % W));
    row_const[crow * 4 + 3] = 0.f;
    special[crow * 4 + 0] = __int_as_float(separate ? c_tok : -1);
    if (separate) {
        special[crow * 4 + 1] = a2 * s_vv;             // Eq. 4 term of the pair
        special[crow * 4 + 2] = a2 * z * z * s_dd;     // Eq. 5 term
        special[crow * 4 + 3] = a2 * s_cc;             // Eq. 6 term (completed square)
    }
}

// ------------------------------------------------------------------------------------
// Sweep 2
// ------------------------------------------------------------------------------------
struct Sweep2Regs {
    bf16x8 q[8], ohi[8], olo[8];   // stationary A operands of this wave's row block
    float c_m2[16], c_oo[16];      // per accumulator register: 2 (max + log2 sum), ||o^||^2 of its row
};

// Adds up, in wave order, the four waves' partial scores of one tile (64 tokens starting at
// `tok0`, staged in LDS as [wave][variant][64]) and writes them out; wave c handles variant c.
template <int kNv>
__device__ __forceinline__ void sweep2_flush(const float *stage, float *out, size_t variant_stride, int tok0,
                                             int t_end, int wave, int lane, bool accumulate) {
    if (wave < kNv && tok0 + lane < t_end) {
        const float *p = stage + wave * 64 + lane;
        float *o = out + wave * variant_stride + tok0 + lane;
        const float sum = (p[0] + p[kNv * 64]) + (p[2 * kNv * 64] + p[3 * kNv * 64]);
        *o = accumulate ? *o + sum : sum;
    }
}

// One step of sweep 2 = one block of 32 tokens (PH = n mod 4 fixes the LDS slot):
//   matrix cores: Z = Q K^T and O V^T of the block (+ ||v||^2 on the dot-product unit)
//   vector ALUs : its scores, summed over this wave's 32 rows, parked in LDS
// The two phases of one wave do not overlap; the second wave on the SIMD runs in the gaps
// (on this hardware a 32x32x16 matrix op blocks most vector-ALU issue anyway).
// Even steps first wait for the tile issued two steps earlier and start the next one.
template <int PH, bool kMasked, int kVariant>
__device__ __forceinline__ void sweep2_step(Sweep2Regs &R, const char *smem, uint32_t lds0, int n, int n_blk,
                                            int t_begin, int t_end, int last_row, const int *vis_i,
                                            const int *excl_i, const char *kh, const char *vh,
                                            const char *const (&kp)[8], const uint32_t (&kdoff)[4], int wave, int lane,
                                            bool wave_active, float *part, float *out, size_t variant_stride, bool accumulate,
                                            int spec_lo_blk, int spec_hi_blk) {
    constexpr int kNv = kVariant == OBC_ALL ? 3 : 1;
    constexpr bool kDoV = kVariant == OBC_VALUE || kVariant == OBC_ALL;
    constexpr bool kDoK = kVariant == OBC_KEY || kVariant == OBC_ALL;
    constexpr bool kDoJ = kVariant == OBC_JOINT || kVariant == OBC_ALL;
    constexpr bool kDoA = kVariant == OBC_ATTN || kVariant == OBC_VATP;   // Eq. 8 and its l1-weighted form
    constexpr bool kNeedVO = kDoK || kDoJ;
    constexpr int kSlot = PH >> 1, kBlk = PH & 1;
    constexpr int kKBase = (kSlot ? kLdsK1 : kLdsK0) + kBlk * 32 * kRowBytes;
    constexpr int kVBase = (kSlot ? kLdsV1 : kLdsV0) + kBlk * 32 * kRowBytes;
    const int half = lane >> 5;
    const float c2x2 = 2.0f * kLog2e * kInvSqrtD;

    if ((PH & 1) == 0) {
        wait_async_loads();
        __syncthreads();
        const int tn = t_begin + ((n >> 1) + 1) * kTileTok;           // first token of the tile to start now
        if (tn < t_end) {
            tile_load_async<kXor16>(kh, tn, last_row, lds0 + (PH == 0 ? kLdsK1 : kLdsK0), wave, lane, kdoff);
            if (kVariant != OBC_ATTN)
                tile_load_async<kXor16>(vh, tn, last_row, lds0 + (PH == 0 ? kLdsV1 : kLdsV0), wave, lane, kdoff);
        }
        if (n >= 2) sweep2_flush<kNv>(part + (kSlot ^ 1) * 4 * kNv * 64, out, variant_stride, t_begin + (n - 2) * 32, t_end, wave, lane, accumulate);
    }
    if (n >= n_blk) return;                                            // uniform
    float acc_v = 0.f, acc_k = 0.f, acc_j = 0.f;
    if (wave_active) {
        // ---- matrix cores ----
        f32x16 z = zero16(), vo = zero16();
        float vv = 0.f;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            const bf16x8 kb = lds_read16(kp[kk] + kKBase);
            z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(R.q[kk], kb, z, 0, 0, 0);
        }
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            if (kVariant == OBC_ATTN) break;                           // no use for V at all
            const bf16x8 vb = lds_read16(kp[kk] + kVBase);
            vv = kVariant == OBC_VATP ? sumabs8(vb, vv) : sumsq8(vb, vv);
            if (kNeedVO) {
                vo = __builtin_amdgcn_mfma_f32_32x32x16_bf16(R.ohi[kk], vb, vo, 0, 0, 0);
                vo = __builtin_amdgcn_mfma_f32_32x32x16_bf16(R.olo[kk], vb, vo, 0, 0, 0);
            }
        }
        vv += __shfl_xor(vv, 32);                                         // ||v_p||^2 of this lane's token
        if (!kMasked && kNeedVO && n >= spec_lo_blk && n <= spec_hi_blk) {      // uniform, rare
            // This fully visible block may hold a (row, key) pair that is scored separately: such a pair gets a
            // logit so low that its weight is exactly 0 (and low enough only for that: every product below stays finite).
            const int tokx = t_begin + n * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int i = wave * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                if (tokx == excl_i[i]) z[r] = kHiddenLogit;
            }
        }
        // ---- vector ALUs ----
        // vo holds -2 v_p.o^_i / 128 and c_oo holds ||o^_i||^2 / 128 (see kCrossScale), so with
        // w7 = ||v_p - o^_i||^2 / 128 = (||v_p||^2 / 128 + c_oo) + vo and z the raw dot product (Z = z / sqrt(128)):
        //   Eq. 5 term  A^2 Z^2 w = A^2 z^2 w7
        //   Eq. 6 term  A^2 ||(1+Z) v - Z o^||^2 = A^2 (||v||^2 + Z (2 (||v||^2 - v.o^) + Z w))
        //                                        = A^2 (||v||^2 + z (2 ||v||^2 / sqrt(128) + sqrt(128) vo + z w7))
        // Rounding can leave a term a hair below zero; the sums are clamped once at the end.
        const int tok = t_begin + n * 32 + (lane & 31);
        const float vv7 = vv * kCrossScale, vv2s = vv * (2.0f * kInvSqrtD);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            // A_ip^2, or A_ip itself (half the exponent) for the attention-only scores
            float a2 = kDoA ? __builtin_amdgcn_exp2f(fmaf(z[r], 0.5f * c2x2, -0.5f * R.c_m2[r]))
                            : __builtin_amdgcn_exp2f(fmaf(z[r], c2x2, -R.c_m2[r]));
            if (kMasked) {
                const int i = wave * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                if (tok > vis_i[i] || tok >= t_end || tok == excl_i[i]) a2 = 0.f; // hidden, padded, or scored separately
            }
            if (kDoV || kDoA) acc_v += a2;
            if (kNeedVO) {
                const float w7 = (vv7 + R.c_oo[r]) + vo[r];                       // ||v_p - o^_i||^2 / 128
                if (kDoK) acc_k = fmaf(a2 * z[r] * z[r], w7, acc_k);
                if (kDoJ) {
                    const float h = fmaf(z[r], w7, fmaf(vo[r], kSqrtD, vv2s));
                    acc_j = fmaf(a2, fmaf(z[r], h, vv), acc_j);
                }
            }
        }
        if (kDoV || kVariant == OBC_VATP) acc_v *= vv;                 // ||v_p||^2, or ||v_p||_1 for the l1 form
        if (kDoV || kDoA) acc_v += __shfl_xor(acc_v, 32);
        if (kDoK) { acc_k += __shfl_xor(acc_k, 32); acc_k = fmaxf(acc_k, 0.f); }
        if (kDoJ) { acc_j += __shfl_xor(acc_j, 32); acc_j = fmaxf(acc_j, 0.f); }
    }
    if (half == 0) {
        float *pw = part + ((kSlot * 4 + wave) * kNv) * 64 + kBlk * 32 + lane;
        int c = 0;
        if (kDoV || kDoA) pw[64 * c++] = acc_v;
        if (kDoK) pw[64 * c++] = acc_k;
        if (kDoJ) pw[64 * c++] = acc_j;
    }
}

// kVariant: OBC_VALUE / OBC_KEY / OBC_JOINT / OBC_ALL / OBC_ATTN / OBC_VATP.  Grid: x = token range, y = chunk, z = (b, KV head).
// With one chunk the scores go straight to `scores`; with several, each chunk writes its
// own plane and mfma_sum_planes adds them in chunk order.
template <int kVariant>
__global__ __launch_bounds__(kThreads, 2) void mfma_sweep2(const uint16_t *__restrict__ q,
                                                           const uint16_t *__restrict__ k,
                                                           const uint16_t *__restrict__ v, int N, int W, int Hq,
                                                           int Hkv, int ragged, SeqLens lens, int range_len, int m_pad,
                                                           const uint16_t *__restrict__ out_bf16,
                                                           const float *__restrict__ row_const,
                                                           const float *__restrict__ special,
                                                           float *__restrict__ dst, size_t variant_stride,
                                                           size_t chunk_stride, int accumulate_flag) {
    const bool accumulate = accumulate_flag != 0;      // add to what `dst` holds; padded positions stay untouched
    constexpr int kNv = kVariant == OBC_ALL ? 3 : 1;
    constexpr bool kNeedVO = kVariant == OBC_KEY || kVariant == OBC_JOINT || kVariant == OBC_ALL;
    // the K and V tiles, then 256 row constants and the staged partial scores of two tiles
    __shared__ __attribute__((aligned(1024))) char smem[kLdsTiles + 256 * sizeof(float) + 2 * 4 * kNv * 64 * sizeof(float)];
    float *vis_s = (float *)(smem + kLdsTiles);                // [128] last visible key of each row of the chunk
    float *excl_s = vis_s + 128;                               // [128] key of the row that is scored separately, or -1
    float *part = excl_s + 128;                                // [2 tiles][4 waves][kNv][64] partial scores

    const int range = blockIdx.x, chunk = blockIdx.y, bg = blockIdx.z;
    const int b = bg / Hkv, g = bg % Hkv, G = Hq / Hkv, M = G * W;
    const int len = seq_len_of(lens, ragged, b, N);
    const int t_begin = range * range_len;
    const int t_stop = min(t_begin + range_len, N);            // scores are written for [t_begin, t_stop)
    float *out = dst + (size_t)chunk * chunk_stride + (size_t)bg * N;

    if (t_begin >= len) {                                      // uniform: only padded positions here
        if (accumulate) return;
        for (int t = t_begin + threadIdx.x; t < t_stop; t += kThreads)
#pragma unroll
            for (int c = 0; c < kNv; ++c) out[c * variant_stride + t] = 0.f;
        return;
    }
    const int t_end = min(t_begin + range_len, len);

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63, half = lane >> 5;
    const int rb = chunk * 4 + wave;
    const bool wave_active = rb * 32 < M;                      // uniform
    const int arow = rb * 32 + (lane & 31);                    // row whose A-operand pieces this lane holds
    const size_t cbase = (size_t)bg * m_pad;

    const char *kh = (const char *)k + (size_t)bg * N * kRowBytes;
    const char *vh = (const char *)v + (size_t)bg * N * kRowBytes;
    const uint32_t lds0 = lds_offset_of(smem);

    // Tile 0 is started before anything else so that its latency hides behind the loads of
    // this wave's stationary operands; step 0 waits for it.
    uint32_t kdoff[4];
    tile_lane_offsets<kXor16>(kdoff, wave, lane);
    tile_load_async<kXor16>(kh, t_begin, len - 1, lds0 + kLdsK0, wave, lane, kdoff);
    if (kVariant != OBC_ATTN) tile_load_async<kXor16>(vh, t_begin, len - 1, lds0 + kLdsV0, wave, lane, kdoff);

    // (fetched with the stationary operands below, in one memory round trip; used after them)
    float my_vis = __int_as_float(-1);
    int my_excl = -1;
    if (threadIdx.x < 128) {
        const int i = chunk * 128 + threadIdx.x;
        if (i < m_pad) my_vis = row_const[(cbase + i) * 4 + 2];
        if (kNeedVO && i < m_pad) my_excl = __float_as_int(special[(cbase + i) * 4 + 0]);
    }

    int koff[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) koff[kk] = row_piece_offset(lane, kk);

    const char *kp[8];                                         // LDS address of this lane's operand piece kk in a tile at offset 0
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) kp[kk] = smem + koff[kk];

    Sweep2Regs R;
    {
        const bool ok = arow < M;
        const char *qrow = (const char *)q + (((size_t)b * Hq + (size_t)g * G) * W + arow) * kRowBytes;
        const char *orow = (const char *)out_bf16 + (cbase + arow) * kRowBytes;
        const size_t lo_plane = (size_t)gridDim.z * m_pad * kRowBytes;
        // One array after the other: the four loads that share a 128-byte line of a row follow each other closely.
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
            R.q[kk] = ok ? *(const bf16x8 *)(qrow + (2 * kk + half) * 16) : bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        if (kNeedVO) {
#pragma unroll
            for (int kk = 0; kk < 8; ++kk)
                R.ohi[kk] = ok ? *(const bf16x8 *)(orow + (2 * kk + half) * 16) : bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int kk = 0; kk < 8; ++kk)
                R.olo[kk] = ok ? *(const bf16x8 *)(orow + lo_plane + (2 * kk + half) * 16) : bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        }
    }
    // Constants of the 16 rows this lane meets in the accumulators: row rb*32 + 8 (r/4) + 4 half + r%4.
    int vis_min = 0x7fffffff;                                  // first key some row of this wave cannot see
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int i = rb * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
        const bool ok = wave_active && i < m_pad;
        const float4 rc = ok ? ((const float4 *)row_const)[cbase + i] : make_float4(1e30f, 0.f, __int_as_float(-1), 0.f);
        R.c_m2[r] = rc.x;                                              // padded rows (1e30) weigh nothing
        R.c_oo[r] = rc.y;
        const int vi = __float_as_int(rc.z);
        if (vi >= 0) vis_min = min(vis_min, vi);
    }
    vis_min = min(vis_min, __shfl_xor(vis_min, 32));
    vis_min = __builtin_amdgcn_readfirstlane(min(vis_min, t_end - 1));
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
        settle(R.q[kk]);
        if (kNeedVO) { settle(R.ohi[kk]); settle(R.olo[kk]); }
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) { settle(R.c_m2[r]); settle(R.c_oo[r]); }
    // First and last block (of 32 tokens, counted from t_begin) that hold a separately scored (row, key) pair.
    __shared__ int spec_lo, spec_hi;
    if (threadIdx.x == 0) { spec_lo = 0x7fffffff; spec_hi = -1; }
    __syncthreads();
    int mine_special = 0;
    if (threadIdx.x < 128) {
        const int ex = my_excl;
        vis_s[threadIdx.x] = my_vis;
        excl_s[threadIdx.x] = __int_as_float(ex);
        mine_special = ex >= t_begin && ex < t_end;
        if (mine_special) {
            atomicMin(&spec_lo, (ex - t_begin) >> 5);
            atomicMax(&spec_hi, (ex - t_begin) >> 5);
        }
    }
    const int *vis_i = (const int *)vis_s, *excl_i = (const int *)excl_s;
    // Uniform: some (row, key) pair of this chunk and token range is scored separately.
    const bool has_special = __syncthreads_or(mine_special) != 0;

    const int n_blk = (t_end - t_begin + 31) / 32;
    const int n_total = (n_blk + 3) & ~3;
    int n_plain = (vis_min + 1 - t_begin) / 32;       // leading blocks every row of this wave sees in full
    n_plain = max(0, min(n_plain, n_blk)) & ~3;
    // Blocks m_lo .. m_hi span the separately scored pairs of this range (none: an empty span).
    const int m_lo = has_special ? __builtin_amdgcn_readfirstlane(spec_lo) : 1;
    const int m_hi = has_special ? __builtin_amdgcn_readfirstlane(spec_hi) : 0;
#define OBC_S2_ARGS smem, lds0, n, n_blk, t_begin, t_end, len - 1, vis_i, excl_i, kh, vh, kp, kdoff, wave, lane, wave_active, part, out, variant_stride, accumulate, m_lo, m_hi
    int n = 0;
    for (; n < n_plain; n += 4) {
        sweep2_step<0, false, kVariant>(R, OBC_S2_ARGS); ++n;
        sweep2_step<1, false, kVariant>(R, OBC_S2_ARGS); ++n;
        sweep2_step<2, false, kVariant>(R, OBC_S2_ARGS); ++n;
        sweep2_step<3, false, kVariant>(R, OBC_S2_ARGS); n -= 3;
    }
    for (; n < n_total; n += 4) {
        sweep2_step<0, true, kVariant>(R, OBC_S2_ARGS); ++n;
        sweep2_step<1, true, kVariant>(R, OBC_S2_ARGS); ++n;
        sweep2_step<2, true, kVariant>(R, OBC_S2_ARGS); ++n;
        sweep2_step<3, true, kVariant>(R, OBC_S2_ARGS); n -= 3;
    }
#undef OBC_S2_ARGS
    __syncthreads();
    // The last tile's partial sums (second staging slot: n_total is a multiple of 4), then zeros for the padding.
    sweep2_flush<kNv>(part + 4 * kNv * 64, out, variant_stride, t_begin + (n_total - 2) * 32, t_end, wave, lane, accumulate);
    if (!accumulate)
        for (int t = t_end + threadIdx.x; t < t_stop; t += kThreads)
#pragma unroll
            for (int c = 0; c < kNv; ++c) out[c * variant_stride + t] = 0.f;
    if (has_special) {
        // Add the separately scored pairs: staged in LDS (the tiles are done with), then summed by one
        // thread in row order; consecutive rows that share their key (a sink, typically) cost one update.
        wait_async_loads();
        __syncthreads();
        float4 *staged = (float4 *)smem;
        if (threadIdx.x < 128) {
            const int i = chunk * 128 + threadIdx.x;
            staged[threadIdx.x] = i < m_pad ? ((const float4 *)special)[cbase + i] : make_float4(__int_as_float(-1), 0.f, 0.f, 0.f);
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            int cur = -1;
            float acc[3] = {0.f, 0.f, 0.f};
            for (int i = 0; i <= 128; ++i) {
                const float4 sp = i < 128 ? staged[i] : make_float4(__int_as_float(-2), 0.f, 0.f, 0.f);
                const int ex = __float_as_int(sp.x);
                const bool mine = ex >= t_begin && ex < t_end;
                if (i < 128 && !mine) continue;
                if (ex != cur) {
                    if (cur >= 0) {
                        int c = 0;
                        if (kVariant == OBC_VALUE || kVariant == OBC_ALL) out[(c++) * variant_stride + cur] += acc[0];
                        if (kVariant == OBC_KEY || kVariant == OBC_ALL) out[(c++) * variant_stride + cur] += acc[1];
                        if (kVariant == OBC_JOINT || kVariant == OBC_ALL) out[(c++) * variant_stride + cur] += acc[2];
                    }
                    cur = i < 128 ? ex : -1;
                    acc[0] = acc[1] = acc[2] = 0.f;
                }
                acc[0] += sp.y; acc[1] += sp.z; acc[2] += sp.w;
            }
        }
    }
}

// scores[c][idx] = sum over chunks of planes[chunk][c][idx], in chunk order.
__global__ __launch_bounds__(256) void mfma_sum_planes(const float *__restrict__ planes, int n_chunks,
                                                       size_t chunk_stride, size_t total, float *__restrict__ scores,
                                                       int accumulate) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    float s = 0.f;
    for (int c = 0; c < n_chunks; ++c) s += planes[(size_t)c * chunk_stride + i];
    scores[i] = accumulate ? scores[i] + s : s;        // the planes hold 0 beyond the true length
}

template <int kVariant>
hipError_t launch_sweep2(const ScoreArgs &a, const ScoreWorkspace &ws, char *base, hipStream_t stream) {
    constexpr int nv = kVariant == OBC_ALL ? 3 : 1;
    hipError_t e;      // (the kernels size their LDS statically: nothing to configure before a launch)
    const size_t plane_elems = (size_t)a.B * a.Hkv * a.N;
    float *dst = ws.n_chunks > 1 ? (float *)(base + ws.planes) : a.scores;
    const size_t chunk_stride = ws.n_chunks > 1 ? plane_elems * nv : 0;
    const dim3 grid((a.N + ws.range_len - 1) / ws.range_len, ws.n_chunks, a.B * a.Hkv);
    if (ws.use_wide) {
        e = launch_sweep2_wide(a, ws, base, dst, plane_elems, chunk_stride, stream);
    } else {
        mfma_sweep2<kVariant><<<grid, dim3(kThreads), 0, stream>>>(
            (const uint16_t *)a.q, (const uint16_t *)a.k, (const uint16_t *)a.v, a.N, a.W, a.Hq, a.Hkv, a.ragged, a.lens,
            ws.range_len, ws.m_pad, (const uint16_t *)(base + ws.out_bf16), (const float *)(base + ws.row_const),
            (const float *)(base + ws.special), dst, plane_elems, chunk_stride,
            ws.n_chunks == 1 ? a.accumulate : 0);
        e = hipGetLastError();
    }
    if (e != hipSuccess || ws.n_chunks == 1) return e;
    const size_t total = plane_elems * nv;
    mfma_sum_planes<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream>>>(dst, ws.n_chunks, chunk_stride, total, a.scores,
                                                                                 a.accumulate);
    return hipGetLastError();
}

}  // namespace

void mfma_plan(int B, int N, int W, int Hq, int Hkv, int d, int variant, ScoreWorkspace *ws, size_t *off) {
    auto align_up = [](size_t x, size_t a) { return (x + a - 1) / a * a; };
    const int BH = B * Hkv;
    const int nv = variant == OBC_ALL ? 3 : 1;
    ws->n_chunks = (ws->m_pad + 127) / 128;
    int splits = (512 + BH * ws->n_chunks - 1) / (BH * ws->n_chunks);
    const int max_splits = (N + 511) / 512;
    splits = splits < 1 ? 1 : (splits > max_splits ? max_splits : splits);
    if (const int v = tuned_splits(); v >= 1 && v <= max_splits) splits = v;    // obc_set_score_tuning
    ws->split_len = ((N + splits - 1) / splits + kTileTok - 1) / kTileTok * kTileTok;
    ws->splits = (N + ws->split_len - 1) / ws->split_len;
    // Token range of one sweep-2 block: about two blocks per compute unit over the whole launch; the
    // register-blocked form runs one workgroup per compute unit and gets one block each.
    const int form = tuned_sweep2_form();
    ws->use_wide = (form != 1 && sweep2_wide_covers(variant, ws->m_pad, (Hq / Hkv) * W)) ? 1 : 0;
    {
        const long long units = (long long)N * BH * ws->n_chunks;
        const long long blocks = ws->use_wide ? 256 : 512;
        long long r = ((units + blocks - 1) / blocks + 63) / 64 * 64;
        ws->range_len = (int)(r < 128 ? 128 : (r > 8192 ? 8192 : r));
    }
    if (const int v = tuned_range(); v >= 64 && v <= 65536 && v % 64 == 0) ws->range_len = v;
    const size_t rows = (size_t)BH * ws->m_pad;
    ws->out_bf16 = *off;  *off = align_up(*off + 2 * rows * d * 2, 256);   // high pieces, then residual pieces
    ws->row_const = *off; *off = align_up(*off + rows * 4 * sizeof(float), 256);
    ws->part_ml = *off;   *off = align_up(*off + rows * ws->splits * 4 * sizeof(float), 256);
    ws->special = *off;   *off = align_up(*off + rows * 4 * sizeof(float), 256);
    ws->part_o = *off;    *off = align_up(*off + rows * ws->splits * d * sizeof(float), 256);
    ws->planes = *off;
    if (ws->n_chunks > 1) *off = align_up(*off + (size_t)ws->n_chunks * nv * BH * N * sizeof(float), 256);
}

hipError_t launch_score_mfma(const ScoreArgs &a, const ScoreWorkspace &ws, char *base, hipStream_t stream) {
    const bool need_o = a.variant == OBC_KEY || a.variant == OBC_JOINT || a.variant == OBC_ALL;
    float *part_ml = (float *)(base + ws.part_ml), *part_o = (float *)(base + ws.part_o);
    hipError_t e = hipSuccess;
    if (a.stage_mask & OBC_STAGE_SWEEP1) {
        const dim3 grid(ws.splits, ws.n_chunks, a.B * a.Hkv);
        if (need_o)
            mfma_sweep1<true><<<grid, dim3(kThreads), 0, stream>>>(
                (const uint16_t *)a.q, (const uint16_t *)a.k, (const uint16_t *)a.v, a.N, a.W, a.Hq, a.Hkv, a.ragged,
                a.lens, ws.split_len, ws.splits, ws.m_pad, part_ml, part_o);
        else
            mfma_sweep1<false><<<grid, dim3(kThreads), 0, stream>>>(
                (const uint16_t *)a.q, (const uint16_t *)a.k, (const uint16_t *)a.v, a.N, a.W, a.Hq, a.Hkv, a.ragged,
                a.lens, ws.split_len, ws.splits, ws.m_pad, part_ml, part_o);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (a.stage_mask & OBC_STAGE_COMBINE) {
        const dim3 grid(ws.m_pad, a.B * a.Hkv);
        if (need_o)
            mfma_combine_hold<<<dim3(ws.m_pad / 4, a.B * a.Hkv), dim3(128), 0, stream>>>(      // (m_pad: a multiple of 32)
                (const uint16_t *)a.v, part_ml, part_o, a.N, a.W, a.Hq, a.Hkv, a.ragged, a.lens, ws.split_len,
                ws.splits, ws.m_pad, (uint16_t *)(base + ws.out_bf16), (float *)(base + ws.row_const),
                (float *)(base + ws.special));
        else
            mfma_combine<<<grid, dim3(128), 0, stream>>>(
                part_ml, a.N, a.W, a.Hq, a.Hkv, a.ragged, a.lens, ws.split_len, ws.splits, ws.m_pad,
                (uint16_t *)(base + ws.out_bf16), (float *)(base + ws.row_const), (float *)(base + ws.special));
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (!(a.stage_mask & OBC_STAGE_SWEEP2)) return hipSuccess;
    switch (a.variant) {
        case OBC_VALUE: return launch_sweep2<OBC_VALUE>(a, ws, base, stream);
        case OBC_KEY: return launch_sweep2<OBC_KEY>(a, ws, base, stream);
        case OBC_JOINT: return launch_sweep2<OBC_JOINT>(a, ws, base, stream);
        case OBC_ATTN: return launch_sweep2<OBC_ATTN>(a, ws, base, stream);
        case OBC_VATP: return launch_sweep2<OBC_VATP>(a, ws, base, stream);
        default: return launch_sweep2<OBC_ALL>(a, ws, base, stream);
    }
}

}  // namespace obc

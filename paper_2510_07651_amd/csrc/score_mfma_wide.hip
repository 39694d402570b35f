// Second sweep of the matrix-core scoring path, register-blocked form for the variants that need
// the cross term v_p . o_i (Eq. 5, Eq. 6, and all three scores at once).
//
// Same mathematics as mfma_sweep2 (score_mfma.hip): per (window row i, token p) the logit Z_ip
// and -2 v_p.o^_i come off the matrix cores with tokens on the lane axis, A_ip^2 and the terms
// of Eq. 4-6 are formed in fp32, and the sum over window rows and query heads (Eq. 9,
// Appendix A.5) runs down accumulator registers.  What differs is the blocking:
//
//   * One workgroup per compute unit, one wave per SIMD.  A wave owns 64 window rows (two
//     32-row sets, A and B) and one 32-token block of every 64-token tile, so each K/V operand
//     piece read from LDS feeds two matrix ops instead of one, and ||v_p||^2 is formed once
//     per 64 rows instead of once per 32.
//   * The wave's 192 registers of stationary operands (Q and the two bf16 pieces of o_i for
//     its 64 rows) live in the accumulator half of the register file.  The matrix ops read
//     them from there directly (inline assembly: the compiler would otherwise copy each
//     operand into the other half before every matrix op), leaving the architectural
//     registers to accumulators, row constants and the streamed K/V pieces.
//   * With one wave per SIMD the overlap of matrix cores and vector ALUs comes from a
//     software pipeline inside the wave: while the matrix cores form set A's logits and
//     cross terms of block n, the vector ALUs score set B of block n-1; then the roles swap.
//     The two streams are interleaved slot by slot (one matrix op, then a slice of the vector
//     work) and the compiler's scheduler is kept from moving anything across a slot boundary.
//   * K and V tiles travel HBM -> LDS through a ring of four 32 KB slots, three tiles in
//     flight per compute unit.
//
// Blocks that hold a causally hidden (row, key) pair, the ragged end of a sequence or a
// separately scored pair run the same pipeline with the masks applied to every pair.
// All sums have a fixed order: results are bit-reproducible.
#include "internal.h"
#include "mfma_util.h"

namespace obc {
using namespace mfma;
namespace {

typedef const __attribute__((address_space(3))) char *lds_ptr;

constexpr int kSlots = 4;                       // tiles in the ring
constexpr int kSlotBytes = 2 * kTileBytes;      // 32 KB: a K tile, then the V tile of the same 64 tokens
constexpr int kRing = kSlots * kSlotBytes;      // 128 KB
constexpr int kTilePerWave = 8;                 // direct-to-LDS transfers a wave issues per tile (4 K + 4 V)

// acc = A * B (first op of a chain) and acc += A * B, with the 16-byte A operand in four accumulator-file
// registers and B in four architectural ones.
__device__ __forceinline__ void mma_first(f32x16 &acc, const f32x4 &a, const bf16x8 &b) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(acc) : "a"(a), "v"(b));
}
__device__ __forceinline__ void mma_next(f32x16 &acc, const f32x4 &a, const bf16x8 &b) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "a"(a), "v"(b));
}
// Moves a 16-byte operand into the accumulator file, where it stays.
__device__ __forceinline__ f32x4 park(const bf16x8 &x) {
    union { bf16x8 v; float f[4]; } u;
    u.v = x;
    f32x4 r;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float t;
        asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(t) : "v"(u.f[e]));
        r[e] = t;
    }
    return r;
}
// The matrix ops above are opaque to the compiler, which therefore cannot count the cycles a
// vector instruction must keep away from a matrix op's result (the last pass of a 32x32x16 op
// lands ten issue slots after the op).  Wherever vector code may follow a matrix op closely,
// this spends those slots explicitly.
__device__ __forceinline__ void matrix_results_land() { asm volatile("s_nop 7\n\ts_nop 4" ::: "memory"); }

// Ties a value to this point of the instruction stream (no instruction is emitted): the compiler's passes would
// otherwise gather the vector work that is spread between the matrix ops next to its first use.
__device__ __forceinline__ void stay(float &x) { asm volatile("" : "+v"(x)); }

__device__ __forceinline__ bf16x8 lds_piece(lds_ptr p, int imm) {
    return *(const __attribute__((address_space(3))) bf16x8 *)(p + imm);
}

// Row constants live in LDS as [128 rows][2] = {2 (max + log2 sum), ||o^||^2}.  Accumulator registers 4 g .. 4 g + 3
// of row set S hold four consecutive rows: their constants are two 16-byte reads, the same address for the 32 lanes
// of a half-wave.
struct RowConsts { f32x4 a, b; };      // {m2_0, oo_0, m2_1, oo_1}, {m2_2, oo_2, m2_3, oo_3}
__device__ __forceinline__ RowConsts row_consts(lds_ptr cp, int S, int g) {
    RowConsts c;
    c.a = *(const __attribute__((address_space(3))) f32x4 *)(cp + (32 * S + 8 * g) * 8);
    c.b = *(const __attribute__((address_space(3))) f32x4 *)(cp + (32 * S + 8 * g) * 8 + 16);
    return c;
}
__device__ __forceinline__ float m2_of(const RowConsts &c, int e) { return e == 0 ? c.a[0] : e == 1 ? c.a[2] : e == 2 ? c.b[0] : c.b[2]; }
__device__ __forceinline__ float oo_of(const RowConsts &c, int e) { return e == 0 ? c.a[1] : e == 1 ? c.a[3] : e == 2 ? c.b[1] : c.b[3]; }

struct Stationary {          // per 32-row set S: Q, high and residual pieces of -2 o^ (accumulator file)
    f32x4 q[2][8], hi[2][8], lo[2][8];
};

struct WideState {
    f32x16 zA, voA, zB, voB;             // logits and cross terms of the two row sets
    bf16x8 kreg[8], vreg[8];             // this lane's operand pieces of the current block
    lds_ptr kp[8];                       // LDS address of operand piece kk of this lane's block in the tile read next
    lds_ptr cp;                          // LDS address of this lane's first row constants
    RowConsts c0;                        // row constants of the first four registers of the set that is scored next
    float sv, sk, sj;                    // set A's sums of the block whose set B is still due
    float vv_prev;                       // ||v_p||^2 (or ||v_p||_1) of that block's token
    bool pend;                           // uniform: set B of the previous block is still due
};

// The vector work for one accumulator register (one (row, token) pair per lane), cut into three tasks of about equal
// cost so that it can be dealt evenly over the slots between the matrix ops.  With z the raw dot product
// (Z = z / sqrt(128)), vo = -2 v_p.o^_i / 128 and oo = ||o^_i||^2 / 128 (see kCrossScale):
//   task 0   A^2 = exp2(2 log2e Z - m2)
//   task 1   w7 = ||v_p - o^_i||^2 / 128 = (||v_p||^2 / 128 + oo) + vo,   sg = 2 ||v_p||^2 / sqrt(128) + sqrt(128) vo
//   task 2   Eq. 5 term  A^2 Z^2 w = A^2 z^2 w7
//            Eq. 6 term  A^2 ||(1+Z) v - Z o^||^2 = A^2 (||v||^2 + z (sg + z w7))
struct TokenConsts { float vv, vv7, vv2s; };      // ||v_p||^2, that / 128, 2 ||v_p||^2 / sqrt(128)
__device__ __forceinline__ TokenConsts token_consts(float vv) { return {vv, vv * kCrossScale, vv * (2.0f * kInvSqrtD)}; }
struct PairWork { float a2, w7, sg; };
template <int kVariant>
__device__ __forceinline__ void pair_task(int task, PairWork &p, float z, float vo, float m2, float oo, const TokenConsts &t,
                                          float &acc_v, float &acc_k, float &acc_j) {
    constexpr bool kDoV = kVariant == OBC_ALL;
    constexpr bool kDoK = kVariant == OBC_KEY || kVariant == OBC_ALL;
    constexpr bool kDoJ = kVariant == OBC_JOINT || kVariant == OBC_ALL;
    if (task == 0) {
        p.a2 = __builtin_amdgcn_exp2f(fmaf(z, 2.0f * kLog2e * kInvSqrtD, -m2));
        stay(p.a2);
    } else if (task == 1) {
        p.w7 = (t.vv7 + oo) + vo;
        stay(p.w7);
        if (kDoJ) { p.sg = fmaf(vo, kSqrtD, t.vv2s); stay(p.sg); }
    } else {
        if (kDoV) { acc_v += p.a2; stay(acc_v); }
        if (kDoK) { acc_k = fmaf(p.a2 * z * z, p.w7, acc_k); stay(acc_k); }
        if (kDoJ) { acc_j = fmaf(p.a2, fmaf(z, fmaf(z, p.w7, p.sg), t.vv), acc_j); stay(acc_j); }
    }
}

// Adds the two row sets' sums of one block, folds the wave's halves (lanes l and l + 32 hold the same token) and
// parks the wave's 32 partial scores in the staging slot of the block's tile: [row half][variant][64 tokens].
template <int kVariant>
__device__ __forceinline__ void park_block(float *stage_slot, int rh, int th, int lane, float vv, float av, float ak,
                                           float aj, float bv, float bk, float bj) {
    constexpr int kNv = kVariant == OBC_ALL ? 3 : 1;
    constexpr bool kDoV = kVariant == OBC_ALL;
    constexpr bool kDoK = kVariant == OBC_KEY || kVariant == OBC_ALL;
    constexpr bool kDoJ = kVariant == OBC_JOINT || kVariant == OBC_ALL;
    float sv = 0.f, sk = 0.f, sj = 0.f;
    if (kDoV) sv = halves_sum((av + bv) * vv);
    if (kDoK) sk = fmaxf(halves_sum(ak + bk), 0.f);      // (rounding can leave a sum a hair below zero)
    if (kDoJ) sj = fmaxf(halves_sum(aj + bj), 0.f);
    if (lane < 32) {
        float *pw = stage_slot + rh * kNv * 64 + th * 32 + lane;
        int c = 0;
        if (kDoV) pw[64 * c++] = sv;
        if (kDoK) pw[64 * c++] = sk;
        if (kDoJ) pw[64 * c++] = sj;
    }
}

// Adds the two row halves' partial scores of one tile (64 tokens from `tok0`) and writes them out; wave c handles
// variant c.
template <int kNv>
__device__ __forceinline__ void flush_tile(const float *stage_slot, float *out, size_t variant_stride, int tok0,
                                           int t_end, int wave, int lane, bool accumulate) {
    if (wave < kNv && tok0 + lane < t_end) {
        const float *p = stage_slot + wave * 64 + lane;
        float *o = out + wave * variant_stride + tok0 + lane;
        const float sum = p[0] + p[kNv * 64];
        *o = accumulate ? *o + sum : sum;
    }
}

// Vector work of one row set of one block outside the pipeline (the last block's second set).
template <int kVariant>
__device__ __forceinline__ void score_set(const f32x16 &z, const f32x16 &vo, lds_ptr cp, int S, float vv, float &av,
                                          float &ak, float &aj) {
    const TokenConsts t = token_consts(vv);
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const RowConsts c = row_consts(cp, S, g);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            PairWork p;
#pragma unroll
            for (int task = 0; task < 3; ++task)
                pair_task<kVariant>(task, p, z[4 * g + e], vo[4 * g + e], m2_of(c, e), oo_of(c, e), t, av, ak, aj);
        }
    }
}

// The 24 matrix ops of row set S on the block held in (kreg, vreg): slot j issues op j, then runs `work(j)`.
template <int S, typename Work>
__device__ __forceinline__ void matrix_phase(const Stationary &A, f32x16 &z, f32x16 &vo, const bf16x8 (&kreg)[8],
                                             const bf16x8 (&vreg)[8], Work &&work) {
#pragma unroll
    for (int j = 0; j < 24; ++j) {
        if (j == 0) mma_first(z, A.q[S][0], kreg[0]);
        else if (j < 8) mma_next(z, A.q[S][j], kreg[j]);
        else if (j == 8) mma_first(vo, A.hi[S][0], vreg[0]);
        else if (j & 1) mma_next(vo, A.lo[S][(j - 8) >> 1], vreg[(j - 8) >> 1]);
        else mma_next(vo, A.hi[S][(j - 8) >> 1], vreg[(j - 8) >> 1]);
        work(j);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Pairs that must not count (causally hidden, past the sequence's end, or scored separately) get a logit so low that
// their weight is exactly 0, and low enough only for that: every product formed from it stays finite.  Applied to the
// logits of row set S of one block (lane's token `tok`) between the matrix ops that formed them and their scoring.
__device__ __forceinline__ void hide_pairs(f32x16 &z, int S, int tok, int t_end, int rh, int half, const int *vis_i,
                                           const int *excl_i) {
    typedef int i32x4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int i0 = rh * 64 + 32 * S + 8 * g + 4 * half;             // four consecutive rows of the 128-row chunk
        const i32x4 vis = *(const i32x4 *)(vis_i + i0), excl = *(const i32x4 *)(excl_i + i0);
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (tok > vis[e] || tok >= t_end || tok == excl[e]) z[4 * g + e] = kHiddenLogit;
    }
}

// Sum of squares of dwords 2 q and 2 q + 1 (four bf16 values) of a 16-byte operand piece.
__device__ __forceinline__ float sumsq_quarter(const bf16x8 x, int q, float acc) {
    union { bf16x8 v; bf16x2 h[4]; } u;
    u.v = x;
    acc = __builtin_amdgcn_fdot2_f32_bf16(u.h[2 * q], u.h[2 * q], acc, false);
    return __builtin_amdgcn_fdot2_f32_bf16(u.h[2 * q + 1], u.h[2 * q + 1], acc, false);
}

// What a wave needs to start one of its eight transfers of the tile that is fetched during a step.
struct TileFetch {
    const char *k_base, *v_base;     // first byte of the tile's first row in K and in V (uniform)
    uint32_t voff[4];                // per-lane byte offset of transfer n inside the tile (rows past the end clamped)
    uint32_t lds;                    // LDS byte address of the ring slot (K tile; the V tile follows)
};
__device__ __forceinline__ void fetch_one(const TileFetch &f, int n, int wave) {       // n = 0..3: K, 4..7: V
    dma16_based(n < 4 ? f.k_base : f.v_base, f.voff[n & 3], f.lds + (n < 4 ? 0 : kTileBytes) + (wave * 4 + (n & 3)) * 1024);
}

// The pipelined work of one wave on one block (32 tokens, lane's token `tok`), operands already in registers:
//   phase 1: matrix cores on set A of this block, vector ALUs on set B of the block before;
//   phase 2: matrix cores on set B of this block, vector ALUs on set A of it; each operand piece is replaced by the
//            next block's (R.kp points into the next tile) as soon as its last matrix op has been issued.
// A phase has 24 slots (one matrix op each) and 48 vector tasks (three per accumulator register): slot j runs tasks
// 2 j and 2 j + 1.  Phase 1 also forms ||v_p||^2 of this block (two dot-product ops in each of the first 16 slots) and
// starts the wave's eight transfers of the tile three steps ahead (one in each of the last eight slots).
// The row constants of four accumulator registers are fetched from LDS six slots before their first use.
// `masks`: some (row, key) pair of this block is causally hidden, past the sequence's end or scored separately.
template <int kVariant>
__device__ __forceinline__ void pipelined_block(WideState &R, const Stationary &A, const TileFetch &fetch, float *stage_prev,
                                                int tok, int t_end, int rh, int th, int wave, int lane, bool masks,
                                                const int *vis_i, const int *excl_i) {
    const int half = lane >> 5;
    float vvn = 0.f, bv = 0.f, bk = 0.f, bj = 0.f;
    const TokenConsts tp = token_consts(R.vv_prev);
    RowConsts cB[4], cA[4];
    PairWork pw[16];
    cB[0] = R.c0;
    matrix_phase<0>(A, R.zA, R.voA, R.kreg, R.vreg, [&](int j) __attribute__((always_inline)) {
        if (j % 6 == 0 && j < 18) cB[j / 6 + 1] = row_consts(R.cp, 1, j / 6 + 1);
        if (j == 18) cA[0] = row_consts(R.cp, 0, 0);
        if (j < 16) { vvn = sumsq_quarter(R.vreg[j >> 1], j & 1, vvn); stay(vvn); }
        else fetch_one(fetch, j - 16, wave);
#pragma unroll
        for (int t = 2 * j; t < 2 * j + 2; ++t) {
            const int r = t / 3;
            pair_task<kVariant>(t % 3, pw[r], R.zB[r], R.voB[r], m2_of(cB[r >> 2], r & 3), oo_of(cB[r >> 2], r & 3), tp, bv, bk, bj);
        }
    });
    // (unconditional, so that the vector work above stays where it is: with no block before, `stage_prev` is a spare slot)
    park_block<kVariant>(stage_prev, rh, th, lane, tp.vv, R.sv, R.sk, R.sj, bv, bk, bj);
    if (masks) {                                               // uniform for the wave, rare
        matrix_results_land();
        hide_pairs(R.zA, 0, tok, t_end, rh, half, vis_i, excl_i);
    }
    const TokenConsts tc = token_consts(halves_sum(vvn));
    float av = 0.f, ak = 0.f, aj = 0.f;
    matrix_phase<1>(A, R.zB, R.voB, R.kreg, R.vreg, [&](int j) __attribute__((always_inline)) {
        if (j % 6 == 0 && j < 18) cA[j / 6 + 1] = row_consts(R.cp, 0, j / 6 + 1);
        if (j == 18) R.c0 = row_consts(R.cp, 1, 0);
        if (j < 8) R.kreg[j] = lds_piece(R.kp[j], 0);
        else if (j & 1) R.vreg[(j - 8) >> 1] = lds_piece(R.kp[(j - 8) >> 1], kTileBytes);
#pragma unroll
        for (int t = 2 * j; t < 2 * j + 2; ++t) {
            const int r = t / 3;
            pair_task<kVariant>(t % 3, pw[r], R.zA[r], R.voA[r], m2_of(cA[r >> 2], r & 3), oo_of(cA[r >> 2], r & 3), tc, av, ak, aj);
        }
    });
    if (masks) {
        matrix_results_land();
        hide_pairs(R.zB, 1, tok, t_end, rh, half, vis_i, excl_i);
    }
    R.sv = av; R.sk = ak; R.sj = aj;
    R.vv_prev = tc.vv;
    R.pend = true;
}

// The workgroups of a launch walk their token ranges in step, and ranges start at multiples of a large power of two:
// walking every range front to back would send all compute units to the same few memory channels at any moment.
// Each workgroup therefore starts at its own tile and wraps around (the order of tokens is free: every token's score
// is a sum over rows).  Tile visited at position t of the walk (t may run past the end: the ring prefetches ahead).
__device__ __forceinline__ int tile_at(int t, int first, int n_tiles) {
    int a = t + first;
    while (a >= n_tiles) a -= n_tiles;      // uniform; at most a few rounds
    return a;
}
__device__ __forceinline__ int next_tile(int a, int n_tiles) { return a + 1 == n_tiles ? 0 : a + 1; }

// One tile step of a wave: this block's operands are in registers already; the next tile (ring slot (s+1) mod 4,
// where R.kp points) is read during the step.
template <int kVariant>
__device__ __forceinline__ void wide_step(WideState &R, const Stationary &A, const uint32_t lds0, int s, int tile,
                                          int tile_fetch, int tile_flush, int t_begin,
                                          int t_end, int last_row, const int *vis_i, const int *excl_i, const char *kh,
                                          const char *vh, const uint32_t (&kdoff)[4], int wave, int lane, int vis_min,
                                          int m_lo, int m_hi, float *stage, float *out, size_t variant_stride,
                                          bool accumulate) {
    constexpr int kNv = kVariant == OBC_ALL ? 3 : 1;
    const int rh = wave & 1, th = wave >> 1;

    // Tile s+1 has landed once at most the two younger tiles' transfers are in flight; the barrier also tells that
    // every wave is done with tile s, whose slot the tile fetched during this step reuses.  (The walk wraps around, so
    // the ring also prefetches past its end: every step waits for the same number of transfers.)
    wait_async_loads_keep<2 * kTilePerWave>();
    __syncthreads();
    TileFetch fetch;
    {
        const int tn = t_begin + tile_fetch * kTileTok;                          // (<= last_row: the tile exists)
        fetch.k_base = kh + (size_t)tn * kRowBytes;
        fetch.v_base = vh + (size_t)tn * kRowBytes;
        fetch.lds = lds0 + ((s + 3) & 3) * kSlotBytes;                        // (the slot of tile s)
        const int rmax = last_row - tn;                                    // last row of the tile that exists
#pragma unroll
        for (int n = 0; n < 4; ++n) fetch.voff[n] = kdoff[n];
        if (rmax < kTileTok - 1) {                                         // uniform, rare: rows past the end re-read the last one
#pragma unroll
            for (int n = 0; n < 4; ++n) {
                const int Rn = (wave * 4 + n) * 4 + (lane >> 4);
                fetch.voff[n] -= (uint32_t)(max(Rn - rmax, 0) * kRowBytes);
            }
        }
    }
    if (s >= 2) flush_tile<kNv>(stage + ((s - 2) & 3) * 2 * kNv * 64, out, variant_stride, t_begin + tile_flush * kTileTok, t_end, wave, lane, accumulate);

    const int tok0 = t_begin + tile * kTileTok + th * 32;                // this wave's block
    const int blk = 2 * tile + th;
    // Blocks every row of the wave sees in full and that hold no separately scored pair need no masks.
    const bool masks = !(tok0 + 31 <= vis_min) || (blk >= m_lo && blk <= m_hi);      // uniform for the wave
    float *stage_prev = stage + (R.pend ? (s - 1) & 3 : kSlots) * 2 * kNv * 64;      // (slot 4: never flushed)
    pipelined_block<kVariant>(R, A, fetch, stage_prev, tok0 + (lane & 31), t_end, rh, th, wave, lane, masks, vis_i, excl_i);
    // On to the slot of tile s+2 (the ring wraps after slot 3).
    const int hop = ((s + 1) & 3) == 0 ? -(kSlots - 1) * kSlotBytes : kSlotBytes;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) R.kp[kk] += hop;
}

// kVariant: OBC_KEY / OBC_JOINT / OBC_ALL.  Grid: x = token range, y = 128-row chunk, z = (b, KV head).
template <int kVariant>
__global__ __launch_bounds__(kThreads, 1) void mfma_sweep2_wide(const uint16_t *__restrict__ q,
                                                                const uint16_t *__restrict__ k,
                                                                const uint16_t *__restrict__ v, int N, int W, int Hq,
                                                                int Hkv, int ragged, SeqLens lens, int range_len, int m_pad,
                                                                const uint16_t *__restrict__ out_bf16,
                                                                const float *__restrict__ row_const,
                                                                const float *__restrict__ special,
                                                                float *__restrict__ dst, size_t variant_stride,
                                                                size_t chunk_stride, int accumulate_flag) {
    const bool accumulate = accumulate_flag != 0;
    constexpr int kNv = kVariant == OBC_ALL ? 3 : 1;
    // the ring of K/V tiles, four constants per row of the chunk, the staged partial scores of four tiles (+ a spare slot)
    __shared__ __attribute__((aligned(1024))) char smem[kRing + 512 * sizeof(float) + 5 * 2 * kNv * 64 * sizeof(float)];
    float *rc_s = (float *)(smem + kRing);                     // [128][2] 2 (max + log2 sum) and ||o^||^2 of each row
    float *vis_s = rc_s + 256;                                 // [128] last visible key of each row of the chunk
    float *excl_s = vis_s + 128;                               // [128] key of the row that is scored separately, or -1
    float *stage = excl_s + 128;                               // [4 tiles + 1][2 row halves][kNv][64]

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
    const int rh = wave & 1, th = wave >> 1;
    const int row0 = chunk * 128 + rh * 64;                    // first of this wave's 64 rows
    const size_t cbase = (size_t)bg * m_pad;

    const char *kh = (const char *)k + (size_t)bg * N * kRowBytes;
    const char *vh = (const char *)v + (size_t)bg * N * kRowBytes;
    const uint32_t lds0 = lds_offset_of(smem);

    // Tile t of the walk lives in ring slot (t + 3) mod 4.  The first tile goes out before anything else (slot 3); the
    // other three slots first serve as a staging area for the stationary operands of the chunk's 128 rows: Q, then the
    // high and the residual pieces of o_i, each as two 64-row tiles in the K tiles' layout, brought in by the same
    // coalesced direct-to-LDS transfers (per-lane loads of 16-byte pieces from 32 rows each would take ten times as long).
    uint32_t kdoff[4];
    tile_lane_offsets<kXor16>(kdoff, wave, lane);
    const int n_tiles = (t_end - t_begin + kTileTok - 1) / kTileTok;
    // (consecutive workgroups start 13 tiles apart: coprime to the power-of-two tile counts of the usual shapes)
    const int first = (int)((13u * (blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z))) % (unsigned)n_tiles);
    {
        const int tt = t_begin + first * kTileTok;
        tile_load_async<kXor16>(kh, tt, len - 1, lds0 + 3 * kSlotBytes, wave, lane, kdoff);
        tile_load_async<kXor16>(vh, tt, len - 1, lds0 + 3 * kSlotBytes + kTileBytes, wave, lane, kdoff);
    }
    const size_t lo_plane = (size_t)gridDim.z * m_pad * kRowBytes;
    {
        const char *q_rows = (const char *)q + ((size_t)b * Hq + (size_t)g * G) * W * kRowBytes;      // the KV head's M rows
        const char *o_rows = (const char *)out_bf16 + cbase * kRowBytes;                             // its m_pad rows
#pragma unroll
        for (int t = 0; t < 2; ++t) {              // rows past the last one re-read it (and are zeroed below, for Q)
            tile_load_async<kXor16>(q_rows, chunk * 128 + 64 * t, M - 1, lds0 + t * kTileBytes, wave, lane, kdoff);
            tile_load_async<kXor16>(o_rows, chunk * 128 + 64 * t, m_pad - 1, lds0 + kSlotBytes + t * kTileBytes, wave, lane, kdoff);
            tile_load_async<kXor16>(o_rows + lo_plane, chunk * 128 + 64 * t, m_pad - 1, lds0 + 2 * kSlotBytes + t * kTileBytes, wave, lane, kdoff);
        }
    }

    float4 my_rc = make_float4(1e30f, 0.f, __int_as_float(-1), 0.f);   // padded rows (1e30) weigh nothing
    int my_excl = -1;
    if (threadIdx.x < 128) {
        const int i = chunk * 128 + threadIdx.x;
        if (i < m_pad) my_rc = ((const float4 *)row_const)[cbase + i];
        if (i < m_pad) my_excl = __float_as_int(special[(cbase + i) * 4 + 0]);
    }

    WideState R;
    // LDS address of this lane's operand piece kk of its block (tokens 32 th .. 32 th + 31 of a tile) in ring slot 3,
    // where the first tile lands; the V tile of a slot is reached with an immediate offset, the other slots by moving
    // the addresses.
    lds_ptr base = (lds_ptr)smem;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) R.kp[kk] = base + 3 * kSlotBytes + th * 32 * kRowBytes + row_piece_offset(lane, kk);
    R.cp = base + kRing + (rh * 64 + 4 * half) * 8;

    // First key some valid row of this wave cannot see (rows row0 .. row0 + 63; lane l looks at row l).
    int vis_min = 0x7fffffff;
    {
        const int i = row0 + lane;
        const int vi = i < m_pad ? __float_as_int(row_const[(cbase + i) * 4 + 2]) : -1;
        if (vi >= 0) vis_min = vi;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) vis_min = min(vis_min, __shfl_xor(vis_min, off));
        vis_min = __builtin_amdgcn_readfirstlane(min(vis_min, t_end - 1));
    }

    // First and last block (of 32 tokens, counted from t_begin) that hold a separately scored (row, key) pair.
    __shared__ int spec_lo, spec_hi;
    if (threadIdx.x == 0) { spec_lo = 0x7fffffff; spec_hi = -1; }
    wait_async_loads();                                        // the first tile and the staged operands have landed
    __syncthreads();
    // Stationary operands: rows row0 + 32 S + (lane % 32), pieces 2 kk + half, parked in the accumulator file.
    Stationary A;
#pragma unroll
    for (int S = 0; S < 2; ++S) {
        const bool ok = row0 + 32 * S + (lane & 31) < M;       // (o_i of a padded row is stored as zeros; Q has no such row)
        const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            lds_ptr piece = base + rh * kTileBytes + S * 32 * kRowBytes + row_piece_offset(lane, kk);
            const bf16x8 tq = lds_piece(piece, 0);
            A.q[S][kk] = park(ok ? tq : zero);
            A.hi[S][kk] = park(lds_piece(piece, kSlotBytes));
            A.lo[S][kk] = park(lds_piece(piece + 2 * kSlotBytes, 0));
        }
    }
    int mine_special = 0;
    if (threadIdx.x < 128) {
        const int ex = my_excl;
        rc_s[2 * threadIdx.x] = my_rc.x;
        rc_s[2 * threadIdx.x + 1] = my_rc.y;
        vis_s[threadIdx.x] = my_rc.z;
        excl_s[threadIdx.x] = __int_as_float(ex);
        mine_special = ex >= t_begin && ex < t_end;
        if (mine_special) {
            atomicMin(&spec_lo, (ex - t_begin) >> 5);
            atomicMax(&spec_hi, (ex - t_begin) >> 5);
        }
    }
    const int *vis_i = (const int *)vis_s, *excl_i = (const int *)excl_s;
    const bool has_special = __syncthreads_or(mine_special) != 0;
    const int m_lo = has_special ? __builtin_amdgcn_readfirstlane(spec_lo) : 1;
    const int m_hi = has_special ? __builtin_amdgcn_readfirstlane(spec_hi) : 0;

    // Every wave has its stationary operands (the barrier above): the staging slots take the next three tiles.
#pragma unroll
    for (int t = 1; t < kSlots; ++t) {
        const int tt = t_begin + tile_at(t, first, n_tiles) * kTileTok;
        tile_load_async<kXor16>(kh, tt, len - 1, lds0 + (t - 1) * kSlotBytes, wave, lane, kdoff);
        tile_load_async<kXor16>(vh, tt, len - 1, lds0 + (t - 1) * kSlotBytes + kTileBytes, wave, lane, kdoff);
    }
    // The first block's operand pieces (slot 3).
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
        R.kreg[kk] = lds_piece(R.kp[kk], 0);
        R.vreg[kk] = lds_piece(R.kp[kk], kTileBytes);
        R.kp[kk] -= 3 * kSlotBytes;                            // step 0 reads the second tile (slot 0)
    }
    R.zA = zero16(); R.voA = zero16(); R.zB = zero16(); R.voB = zero16();
    R.sv = R.sk = R.sj = 0.f;
    R.vv_prev = 0.f;
    R.pend = false;
    R.c0 = row_consts(R.cp, 1, 0);

    // Positions of the walk: the tile worked on, the one fetched during the step (four ahead), the one flushed (two back).
    int tile = first, tile_fetch = tile_at(4, first, n_tiles), tile_flush = tile_at(2 * n_tiles - 2, first, n_tiles);
    for (int s = 0; s < n_tiles; ++s, tile = next_tile(tile, n_tiles), tile_fetch = next_tile(tile_fetch, n_tiles), tile_flush = next_tile(tile_flush, n_tiles))
        wide_step<kVariant>(R, A, lds0, s, tile, tile_fetch, tile_flush, t_begin, t_end, len - 1, vis_i, excl_i, kh, vh, kdoff, wave, lane, vis_min, m_lo,
                            m_hi, stage, out, variant_stride, accumulate);
    if (R.pend) {                                              // set B of the last block
        matrix_results_land();
        float bv = 0.f, bk = 0.f, bj = 0.f;
        score_set<kVariant>(R.zB, R.voB, R.cp, 1, R.vv_prev, bv, bk, bj);
        park_block<kVariant>(stage + ((n_tiles - 1) & 3) * 2 * kNv * 64, rh, th, lane, R.vv_prev, R.sv, R.sk, R.sj, bv, bk, bj);
    }
    wait_async_loads();        // the tiles fetched past the end must have landed before the LDS is given back
    __syncthreads();
    if (n_tiles >= 2) flush_tile<kNv>(stage + ((n_tiles - 2) & 3) * 2 * kNv * 64, out, variant_stride, t_begin + tile_at(n_tiles - 2, first, n_tiles) * kTileTok, t_end, wave, lane, accumulate);
    flush_tile<kNv>(stage + ((n_tiles - 1) & 3) * 2 * kNv * 64, out, variant_stride, t_begin + tile_at(n_tiles - 1, first, n_tiles) * kTileTok, t_end, wave, lane, accumulate);
    if (!accumulate)
        for (int t = t_end + threadIdx.x; t < t_stop; t += kThreads)
#pragma unroll
            for (int c = 0; c < kNv; ++c) out[c * variant_stride + t] = 0.f;
    if (has_special) {
        // Add the separately scored pairs: staged in LDS (the tiles are done with), then summed by one
        // thread in row order; consecutive rows that share their key (a sink, typically) cost one update.
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
                        if (kVariant == OBC_ALL) out[(c++) * variant_stride + cur] += acc[0];
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

}  // namespace

bool sweep2_wide_covers(int variant, int m_pad, int M) {
    if (variant != OBC_KEY && variant != OBC_JOINT && variant != OBC_ALL) return false;
    return M % 128 == 0 || M % 128 > 64;        // every 128-row chunk at least three quarters full
}

template <int kVariant>
static hipError_t launch_wide(const ScoreArgs &a, const ScoreWorkspace &ws, char *base, float *dst, size_t plane_elems,
                              size_t chunk_stride, hipStream_t stream) {
    const dim3 grid((a.N + ws.range_len - 1) / ws.range_len, ws.n_chunks, a.B * a.Hkv);
    mfma_sweep2_wide<kVariant><<<grid, dim3(kThreads), 0, stream>>>(
        (const uint16_t *)a.q, (const uint16_t *)a.k, (const uint16_t *)a.v, a.N, a.W, a.Hq, a.Hkv, a.ragged, a.lens,
        ws.range_len, ws.m_pad, (const uint16_t *)(base + ws.out_bf16), (const float *)(base + ws.row_const),
        (const float *)(base + ws.special), dst, plane_elems, chunk_stride, ws.n_chunks == 1 ? a.accumulate : 0);
    return hipGetLastError();
}

hipError_t launch_sweep2_wide(const ScoreArgs &a, const ScoreWorkspace &ws, char *base, float *dst, size_t plane_elems,
                              size_t chunk_stride, hipStream_t stream) {
    switch (a.variant) {
        case OBC_KEY: return launch_wide<OBC_KEY>(a, ws, base, dst, plane_elems, chunk_stride, stream);
        case OBC_JOINT: return launch_wide<OBC_JOINT>(a, ws, base, dst, plane_elems, chunk_stride, stream);
        case OBC_ALL: return launch_wide<OBC_ALL>(a, ws, base, dst, plane_elems, chunk_stride, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace obc

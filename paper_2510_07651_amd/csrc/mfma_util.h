// Device helpers shared by the matrix-core scoring kernels (gfx950, wave64): vector types, the LDS tile
// layout and its swizzles, direct-to-LDS transfers, operand-piece addressing, lane exchanges.
// Internal to the library; every function is inline device code.
#pragma once

#include "internal.h"

namespace obc {
namespace mfma {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short i16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __bf16 bf16_2 __attribute__((ext_vector_type(2)));
typedef float f32_2 __attribute__((ext_vector_type(2)));

constexpr int kD = 128;                 // head_dim
constexpr int kRowBytes = kD * 2;       // one bf16 K or V row
constexpr int kTileTok = 64;            // tokens per LDS tile (two blocks of 32)
constexpr int kTileBytes = kTileTok * kRowBytes;   // 16 KB
constexpr int kThreads = 256;           // 4 waves; wave w owns row block 4*chunk + w (32 window rows)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kInvSqrtD = 0.08838834764831845f;   // 1/sqrt(128)
// The running softmax sums of sweep 1 are kept relative to a reference that follows the
// running max lazily: it only moves (and the accumulated O is only rescaled) when the max
// has grown by more than 8 in log2 units, so weights stay below 2^8 and the 64-register
// rescale becomes rare instead of happening whenever any of a wave's 32 rows sees a new max.
constexpr float kLazyRescale = 8.0f / (kLog2e * kInvSqrtD);   // in raw q.k units

// LDS map (bytes) of sweep 2: two K tiles, then two V tiles.  Sweep 1 uses
// the same 64 KB as a ring of four 8 KB K blocks followed by a ring of four V blocks.
constexpr int kLdsK0 = 0, kLdsK1 = kTileBytes, kLdsV0 = 2 * kTileBytes, kLdsV1 = 3 * kTileBytes;
constexpr int kLdsTiles = 4 * kTileBytes;           // 64 KB

enum Swizzle { kXor16 = 0, kRot4 = 1 };

// LDS tiles hold 64 rows of 256 B.  Row R keeps its 16-byte piece c at slot
//   kXor16: c ^ (R & 15)         -- conflict-free when 16 lanes read the same piece of 16 consecutive rows
//   kRot4 : (c + 4 (R & 3)) & 15 -- conflict-free when 32 lanes read 64 contiguous bytes of 4 consecutive rows
__device__ __forceinline__ int piece_of(int swz, int R, int slot) {
    return swz == kXor16 ? (slot ^ (R & 15)) : ((slot - 4 * (R & 3)) & 15);
}

__device__ __forceinline__ uint32_t lds_offset_of(const void *p) {
    return (uint32_t)(size_t)(const __attribute__((address_space(3))) char *)p;
}

// One direct-to-LDS transfer: every lane supplies the address of 16 bytes in global
// memory; the wave's 1 KB lands contiguously at LDS byte `lds_off` (lane l at +16 l).
// Marked non-temporal: every sweep reads K and V once, and they are far larger than the L2.
// Issued from inline assembly so that the compiler's wait-count bookkeeping does not tie
// later LDS reads of OTHER tiles to these transfers; the kernels wait for them
// explicitly (wait_async_loads + barrier) before the tile is read.
__device__ __forceinline__ void dma16(const void *gptr, uint32_t lds_off) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt" ::"s"(lds_off), "v"(gptr) : "memory");
}
// Same transfer with the address split into a wave-uniform 64-bit base (scalar registers)
// and a per-lane 32-bit byte offset: no vector-ALU address arithmetic per transfer.
__device__ __forceinline__ void dma16_based(const void *sbase, uint32_t voff, uint32_t lds_off) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt" ::"s"(lds_off), "v"(voff), "s"(sbase) : "memory");
}
__device__ __forceinline__ void wait_async_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// Asynchronous copy of one 64-row tile.  Each wave issues four transfers; lane l of
// transfer n lands at row 4 (4 wave + n) + l / 16, slot l % 16, and picks the global piece
// that belongs in that slot.  Rows past `last_row` re-read `last_row` (memory beyond the
// true length is never touched).
// Per-lane byte offsets of the four transfers inside a tile whose 64 rows all exist.
template <int SWZ>
__device__ __forceinline__ void tile_lane_offsets(uint32_t (&doff)[4], int wave, int lane) {
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        const int R = (wave * 4 + n) * 4 + (lane >> 4);
        doff[n] = (uint32_t)(R * kRowBytes + piece_of(SWZ, R, lane & 15) * 16);
    }
}

template <int SWZ>
__device__ __forceinline__ void tile_load_async(const char *__restrict__ head_base, int t0, int last_row,
                                                uint32_t lds_tile, int wave, int lane, const uint32_t (&doff)[4]) {
    if (t0 + kTileTok - 1 <= last_row) {            // uniform: the common case, every row of the tile exists
        const char *sbase = head_base + (size_t)t0 * kRowBytes;
#pragma unroll
        for (int n = 0; n < 4; ++n) dma16_based(sbase, doff[n], lds_tile + (wave * 4 + n) * 1024);
        return;
    }
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        const int R = (wave * 4 + n) * 4 + (lane >> 4);
        const int c = piece_of(SWZ, R, lane & 15);
        int row = t0 + R;
        row = row > last_row ? last_row : row;
        dma16(head_base + (size_t)row * kRowBytes + c * 16, lds_tile + (wave * 4 + n) * 1024);
    }
}

// The same for one 32-row block (8 KB): two transfers per wave, wave w brings rows 8w .. 8w+7.
constexpr int kBlkBytes = 32 * kRowBytes;
template <int SWZ>
__device__ __forceinline__ void block_lane_offsets(uint32_t (&doff)[2], int wave, int lane) {
#pragma unroll
    for (int n = 0; n < 2; ++n) {
        const int R = (wave * 2 + n) * 4 + (lane >> 4);
        doff[n] = (uint32_t)(R * kRowBytes + piece_of(SWZ, R, lane & 15) * 16);
    }
}
template <int SWZ>
__device__ __forceinline__ void block_load_async(const char *__restrict__ head_base, int t0, int last_row,
                                                 uint32_t lds_block, int wave, int lane, const uint32_t (&doff)[2]) {
    if (t0 + 31 <= last_row) {                      // uniform: every row of the block exists
        const char *sbase = head_base + (size_t)t0 * kRowBytes;
#pragma unroll
        for (int n = 0; n < 2; ++n) dma16_based(sbase, doff[n], lds_block + (wave * 2 + n) * 1024);
        return;
    }
#pragma unroll
    for (int n = 0; n < 2; ++n) {                   // rows past the end re-read the last row
        const int R = (wave * 2 + n) * 4 + (lane >> 4);
        const int c = piece_of(SWZ, R, lane & 15);
        int row = t0 + R;
        row = row > last_row ? last_row : row;
        dma16(head_base + (size_t)row * kRowBytes + c * 16, lds_block + (wave * 2 + n) * 1024);
    }
}
// Waits until at most kKeep of this wave's most recent transfers are still in flight
// (transfers complete in issue order; other memory operations in flight only make the wait stricter).
template <int kKeep>
__device__ __forceinline__ void wait_async_loads_keep() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kKeep) : "memory"); }

// Per-lane byte offset, inside a kXor16 tile, of piece 2 kk + half of row (lane % 32) of a
// 32-row block; add 32 * 256 for the tile's second block.  16-byte matrix-core operand:
// K as the A operand of K Q^T, K and V as B operands of Q K^T and O V^T.
__device__ __forceinline__ int row_piece_offset(int lane, int kk) {
    const int R = lane & 31, c = 2 * kk + (lane >> 5);
    return R * kRowBytes + ((c ^ (R & 15)) << 4);
}

// Per-lane byte offset, inside a kRot4 tile, of the transposing read that serves the A
// operand of O^T += V^T P^T for head_dim block ddb: 16 lanes fetch a 4-token x 16-element
// block and each lane gets one column of it (4 tokens of one head_dim index).  Add
// (first token of the 4-token group) * 256.
__device__ __forceinline__ int vt_piece_offset(int lane, int ddb) {
    const int i = lane & 15, sub = (lane >> 4) & 1, half = lane >> 5;
    const int rq = i >> 2;                              // token inside the group == (row & 3)
    const int c = ddb * 4 + sub * 2 + ((i & 3) >> 1);
    const int slot = (c + 4 * rq) & 15;
    return (4 * half + rq) * kRowBytes + (slot << 4) + ((i & 1) << 3);
}

__device__ __forceinline__ bf16x8 lds_read16(const char *p) { return *(const bf16x8 *)p; }

// The 8 tokens of a k-step in the order in which the accumulator of K Q^T holds them:
// rows r0 + 4 half + {0..3} and r0 + 8 + 4 half + {0..3}.
__device__ __forceinline__ bf16x8 lds_read_vt(const char *p) {
    union { bf16x8 v; i16x4 h[2]; } u;
    u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)(p));
    u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)(p + 8 * kRowBytes));
    return u.v;
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    const f32_2 f = {lo, hi};
    const bf16_2 r = __builtin_convertvector(f, bf16_2);   // v_cvt_pk_bf16_f32, round to nearest even
    return *(const uint32_t *)&r;
}
__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }
// Lanes l and l + 32 of a wave hold the two halves of one row (sweep 1) or token (sweep 2).  One
// register-to-register swap of the wave's halves gives every lane both values: no trip through the LDS crossbar.
__device__ __forceinline__ void both_halves(float x, float &lower, float &upper) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    lower = __uint_as_float(r[0]);      // the value of lane l % 32
    upper = __uint_as_float(r[1]);      // the value of lane l % 32 + 32
}
__device__ __forceinline__ float halves_sum(float x) { float a, b; both_halves(x, a, b); return a + b; }
__device__ __forceinline__ float halves_max(float x) { float a, b; both_halves(x, a, b); return fmaxf(a, b); }
// Sum over the 32 lanes of each half of a wave, the same bits in each of them.  Lane pairings inside a row of
// 16 through the data-parallel-primitive lane controls (neighbours, neighbouring pairs, mirror image inside 8
// and inside 16: register to register), then the row next door.  Call with every lane active.
template <int kCtrl>
__device__ __forceinline__ float dpp_pair_sum(float x) {
    return x + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), kCtrl, 0xf, 0xf, false));
}
__device__ __forceinline__ float row_sum32(float x) {      // over each half of the wave (32 lanes)
    x = dpp_pair_sum<0xB1>(x);
    x = dpp_pair_sum<0x4E>(x);
    x = dpp_pair_sum<0x141>(x);
    x = dpp_pair_sum<0x140>(x);
    return x + __shfl_xor(x, 16);
}
__device__ __forceinline__ f32x16 zero16() {
    f32x16 z;
#pragma unroll
    for (int r = 0; r < 16; ++r) z[r] = 0.f;
    return z;
}

union PiecePair { bf16x8 v; uint32_t u[4]; };

// The second sweep needs, per (row i, token p) pair, w = ||v_p - o^_i||^2 = ||v_p||^2 + ||o^_i||^2 - 2 v_p.o^_i and
// the logit Z = z / sqrt(128) with z the raw dot product off the matrix cores.  Everywhere Z^2 w is formed as
// z^2 (w / 128): 1/128 = (1/sqrt(128))^2 is a power of two, so it can ride, exactly, on the stationary operand and on the
// row constant, and the vector ALUs never form Z itself.  The stationary o_i pieces are stored as bf16 bits of
// -2/128 x (this function), the row constant as ||o^_i||^2 / 128: the cross-term accumulator then holds -2 v_p.o^_i / 128.
// A (row, key) pair that must not count gets this raw dot product in place of its own: its weight is exactly 0 and
// every product the scores form from it stays finite (its square times a squared distance of up to 1e14).
constexpr float kHiddenLogit = -1e12f;
constexpr float kCrossScale = 0.0078125f;          // 1/128
constexpr float kSqrtD = 11.313708498984761f;      // sqrt(128) = 128 / sqrt(128): turns the scaled cross term into Z-units
__device__ __forceinline__ uint16_t cross_operand_bf16(uint16_t bits) {
    return (uint16_t)(__float_as_uint(-2.0f * kCrossScale * __uint_as_float((uint32_t)bits << 16)) >> 16);
}

// Pins a value loaded from global memory as "consumed here", so that the wait for its load
// is placed here (before the pipelined loops) and not inside them, where it would also
// wait for the direct-to-LDS tile loads in flight.
__device__ __forceinline__ void settle(const bf16x8 &x) { asm volatile("" ::"v"(x)); }
__device__ __forceinline__ void settle(const float &x) { asm volatile("" ::"v"(x)); }

// Interleaving recipe for one pipeline step, applied to the step's basic block: after two
// LDS reads, repeat {1 matrix-core op, `valu` vector-ALU ops, `ds` LDS reads}.
template <int kSlots, int kValu, int kDs>
__device__ __forceinline__ void interleave_hint() {
    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
    for (int i = 0; i < kSlots; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, kValu, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, kDs, 0);
    }
}

// Sum of squares of the 8 bf16 values in a 16-byte operand piece.
__device__ __forceinline__ float sumsq8(const bf16x8 x, float acc) {
    union { bf16x8 v; bf16x2 h[4]; } u;
    u.v = x;
#pragma unroll
    for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_fdot2_f32_bf16(u.h[e], u.h[e], acc, false);
    return acc;
}

// Sum of the absolute values of the 8 bf16 values in a 16-byte operand piece: each pair is
// dotted with (+-1, +-1) carrying the pair's own signs.
__device__ __forceinline__ float sumabs8(const bf16x8 x, float acc) {
    union { bf16x8 v; uint32_t u[4]; bf16x2 h[4]; } in, sg;
    in.v = x;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        sg.u[e] = (in.u[e] & 0x80008000u) | 0x3f803f80u;
        acc = __builtin_amdgcn_fdot2_f32_bf16(in.h[e], sg.h[e], acc, false);
    }
    return acc;
}

}  // namespace mfma
}  // namespace obc

// K/V compaction (Appendix E, Algorithm 2: gather of the kept rows).  Pure byte moves:
// each thread copies one 16-byte piece of one kept row with a 128-bit load and store.
#include "internal.h"

namespace obc {
namespace {

__global__ __launch_bounds__(256) void gather_rows(const uint4 *__restrict__ k, const uint4 *__restrict__ v,
                                                   const int32_t *__restrict__ keep_idx, uint4 *__restrict__ k_out,
                                                   uint4 *__restrict__ v_out, int N, int budget, int row_vec,
                                                   size_t total_vec) {
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= total_vec) return;
    const size_t out_row = t / row_vec;             // (b*Hkv + g) * budget + j
    const int c = (int)(t % row_vec);
    const size_t bg = out_row / budget;
    int p = keep_idx[out_row];
    uint4 *out = blockIdx.y == 0 ? k_out : v_out;
    if (p < 0) {                                    // padding of a ragged index list: an all-zero row
        out[t] = make_uint4(0, 0, 0, 0);
        return;
    }
    p = p >= N ? N - 1 : p;
    const size_t src = (bg * N + p) * row_vec + c;
    const uint4 *in = blockIdx.y == 0 ? k : v;
    // (streaming store: the compacted rows are not read again by this path, and kept dirty in the L2 they would be
    // written back in one burst when the kernel ends)
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 x = *(const u32x4 *)(in + src);
    __builtin_nontemporal_store(x, (u32x4 *)(out + t));
}

// Running scores follow their tokens through an eviction: out[bg, j] = in[bg, keep[bg, j]] for
// j < budget, 0 for budget <= j < n_out (slots of tokens still to come).
__global__ __launch_bounds__(256) void gather_scores(const float *__restrict__ in, const int32_t *__restrict__ keep_idx,
                                                     float *__restrict__ out, int N, int budget, int n_out,
                                                     size_t total) {
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= total) return;
    const size_t bg = t / n_out;
    const int j = (int)(t % n_out);
    float x = 0.f;
    if (j < budget) {
        int p = keep_idx[bg * budget + j];
        p = p < 0 ? 0 : (p >= N ? N - 1 : p);
        x = in[bg * N + p];
    }
    out[t] = x;
}

// In-place compaction of one KV head's rows: row j takes the place of row keep_idx[j] >= j.
// A workgroup owns a 64-byte column slice of all rows of one head of K (blockIdx.y == 0) or V
// (1) and walks the index list in chunks of kMoveChunk rows: every thread loads its pieces of
// its source rows, the workgroup meets at a barrier, then every thread stores.  Sources of a
// chunk lie at or above the chunk's first row, so they are untouched by the stores of earlier
// chunks and are all read before this chunk's stores; later chunks read above everything
// stored so far.  The walk starts near the first row that moves at all (the list is ascending,
// so the rows before it are a prefix that stays where it is).
// blockIdx.y == 2 moves the running scores the same way and clears their tail.
constexpr int kMoveThreads = 1024;
constexpr int kMoveRows = 8;                                 // rows per thread and chunk
constexpr int kMoveChunk = kMoveThreads / 4 * kMoveRows;     // rows per chunk (four 16-byte pieces per row slice)

__global__ __launch_bounds__(kMoveThreads) void move_rows_in_place(uint4 *__restrict__ k, uint4 *__restrict__ v,
                                                                   float *__restrict__ scores,
                                                                   const int32_t *__restrict__ keep_idx, int N,
                                                                   int budget, int row_vec) {
    __shared__ int first_probe;
    const size_t bg = blockIdx.z;
    const int32_t *keep = keep_idx + bg * budget;
    if (blockIdx.y == 2 && blockIdx.x != 0) return;

    // Probe kMoveThreads evenly spaced positions; everything up to the last probe before the
    // first one that moves is known to stay.
    int begin = 0;
    if (budget > kMoveChunk) {                      // (a list of one chunk is walked from its start: nothing to save)
        const int stride = (budget + kMoveThreads - 1) / kMoveThreads;
        if (threadIdx.x == 0) first_probe = kMoveThreads;
        __syncthreads();
        const long long pos = (long long)threadIdx.x * stride;
        if (pos >= budget || keep[pos] != (int)pos) atomicMin(&first_probe, (int)threadIdx.x);
        __syncthreads();
        begin = first_probe == 0 ? 0 : (first_probe - 1) * stride;
    }

    if (blockIdx.y == 2) {
        float *s = scores + bg * N;
        for (int j0 = begin; j0 < budget; j0 += kMoveThreads * kMoveRows) {
            float x[kMoveRows];
            int p[kMoveRows];
#pragma unroll
            for (int u = 0; u < kMoveRows; ++u) {
                const int j = j0 + u * kMoveThreads + threadIdx.x;
                x[u] = 0.f;
                p[u] = -1;
                if (j < budget) {
                    p[u] = keep[j];
                    p[u] = p[u] >= N ? N - 1 : p[u];
                    if (p[u] >= 0) x[u] = s[p[u]];
                }
            }
            __syncthreads();
#pragma unroll
            for (int u = 0; u < kMoveRows; ++u) {
                const int j = j0 + u * kMoveThreads + threadIdx.x;
                if (j < budget && p[u] != j) s[j] = x[u];
            }
        }
        for (int j = budget + threadIdx.x; j < N; j += kMoveThreads) s[j] = 0.f;
        return;
    }
    uint4 *rows = (blockIdx.y == 0 ? k : v) + bg * N * row_vec;
    const int c = blockIdx.x * 4 + (threadIdx.x & 3);
    const int r = threadIdx.x >> 2;
    for (int j0 = begin; j0 < budget; j0 += kMoveChunk) {
        uint4 x[kMoveRows];
        int p[kMoveRows];
#pragma unroll
        for (int u = 0; u < kMoveRows; ++u) {
            const int j = j0 + u * (kMoveThreads / 4) + r;
            x[u] = make_uint4(0, 0, 0, 0);
            p[u] = -1;
            if (j < budget && c < row_vec) {
                p[u] = keep[j];
                p[u] = p[u] >= N ? N - 1 : p[u];
                if (p[u] >= 0) x[u] = rows[(size_t)p[u] * row_vec + c];
            }
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < kMoveRows; ++u) {
            const int j = j0 + u * (kMoveThreads / 4) + r;
            if (j < budget && c < row_vec && p[u] != j) rows[(size_t)j * row_vec + c] = x[u];
        }
    }
}

// ------------------------------------------------------------------------------------
// Evict-one (the decoding setup of Appendix C: an eviction decision at every step, the first tokens kept as
// attention sinks, the most recent ones kept as well).
// ------------------------------------------------------------------------------------
// Same order as the selection kernels use: larger score <=> larger key, -0 folded onto +0, NaN lowest.
__device__ __forceinline__ uint32_t evict_order_key(float f) {
    uint32_t u = __float_as_uint(f);
    if (f != f) return 0u;
    if (u == 0x80000000u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// One workgroup per (sequence, KV head): the token a protected selection of all but one competing token would drop,
// i.e. the lowest score among first <= p < len - tail, the highest index among equal scores (the kept ones win ties
// by the lower index).  Packed as (key, ~index) so that one unsigned minimum decides both.
__global__ __launch_bounds__(256) void evict_pick(const float *__restrict__ scores, int N, int Hkv, int ragged,
                                                  SeqLens lens, int first, int tail, int32_t *__restrict__ evicted) {
    __shared__ unsigned long long best_w[4];
    const int bg = blockIdx.x;
    const int len = seq_len_of(lens, ragged, bg / Hkv, N);
    const float *s = scores + (size_t)bg * N;
    unsigned long long best = ~0ull;
    for (int p = first + threadIdx.x; p < len - tail; p += 256) {
        const unsigned long long cand = ((unsigned long long)evict_order_key(s[p]) << 32) | (uint32_t)~p;
        best = cand < best ? cand : best;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const unsigned long long o = __shfl_xor(best, off);
        best = o < best ? o : best;
    }
    if ((threadIdx.x & 63) == 0) best_w[threadIdx.x >> 6] = best;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < 4; ++w) best = best_w[w] < best ? best_w[w] : best;
        evicted[bg] = (int32_t)~(uint32_t)best;         // (the host guarantees at least one competing token)
    }
}

// Closes the gap the evicted token leaves: row j >= e takes row j + 1, for K, V (blockIdx.y = 0, 1; one 64-byte column
// slice per workgroup, rows read chunk by chunk before they are overwritten, as in move_rows_in_place) and for the
// running scores (blockIdx.y = 2), whose slots from len - 1 on are cleared.
__global__ __launch_bounds__(kMoveThreads) void evict_shift(uint4 *__restrict__ k, uint4 *__restrict__ v,
                                                            float *__restrict__ scores,
                                                            const int32_t *__restrict__ evicted, int N, int Hkv,
                                                            int ragged, SeqLens lens, int row_vec) {
    const size_t bg = blockIdx.z;
    const int len = seq_len_of(lens, ragged, (int)(bg / Hkv), N);
    const int e = evicted[bg];
    const int budget = len - 1;                      // rows that remain
    if (e < 0 || e >= len) return;                   // (cannot happen: evict_pick chose among the live tokens)
    if (blockIdx.y == 2) {
        if (blockIdx.x != 0) return;
        float *s = scores + bg * N;
        for (int j0 = e; j0 < budget; j0 += kMoveThreads * kMoveRows) {
            float x[kMoveRows];
#pragma unroll
            for (int u = 0; u < kMoveRows; ++u) {
                const int j = j0 + u * kMoveThreads + threadIdx.x;
                x[u] = j < budget ? s[j + 1] : 0.f;
            }
            __syncthreads();
#pragma unroll
            for (int u = 0; u < kMoveRows; ++u) {
                const int j = j0 + u * kMoveThreads + threadIdx.x;
                if (j < budget) s[j] = x[u];
            }
        }
        for (int j = budget + threadIdx.x; j < N; j += kMoveThreads) s[j] = 0.f;
        return;
    }
    uint4 *rows = (blockIdx.y == 0 ? k : v) + bg * N * row_vec;
    const int c = blockIdx.x * 4 + (threadIdx.x & 3);
    const int r = threadIdx.x >> 2;
    for (int j0 = e; j0 < budget; j0 += kMoveChunk) {
        uint4 x[kMoveRows];
#pragma unroll
        for (int u = 0; u < kMoveRows; ++u) {
            const int j = j0 + u * (kMoveThreads / 4) + r;
            x[u] = make_uint4(0, 0, 0, 0);
            if (j < budget && c < row_vec) x[u] = rows[(size_t)(j + 1) * row_vec + c];
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < kMoveRows; ++u) {
            const int j = j0 + u * (kMoveThreads / 4) + r;
            if (j < budget && c < row_vec) rows[(size_t)j * row_vec + c] = x[u];
        }
    }
}

// Measurement hook: reads `n_vec` 16-byte words once with 128-bit loads and folds them
// into one word per thread (so the loads cannot be dropped).  Its duration gives the box's
// own streaming-read ceiling, the practical denominator next to the nominal HBM peak.
__global__ __launch_bounds__(256) void stream_read(const uint4 *__restrict__ src, size_t n_vec,
                                                   uint32_t *__restrict__ sink) {
    const size_t stride = (size_t)gridDim.x * 256;
    uint4 acc = make_uint4(0, 0, 0, 0);
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n_vec; i += stride) {
        const uint4 x = src[i];
        acc.x ^= x.x; acc.y ^= x.y; acc.z ^= x.z; acc.w ^= x.w;
    }
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = acc.x ^ acc.y ^ acc.z ^ acc.w;
}

}  // namespace

hipError_t launch_gather_scores(const float *in, const int32_t *keep_idx, float *out, int BH, int N, int budget,
                                 int n_out, hipStream_t stream) {
    const size_t total = (size_t)BH * n_out;
    gather_scores<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream>>>(in, keep_idx, out, N, budget, n_out,
                                                                                   total);
    return hipGetLastError();
}

hipError_t launch_stream_read(const void *src, size_t bytes, uint32_t *sink, int blocks, hipStream_t stream) {
    stream_read<<<dim3(blocks), dim3(256), 0, stream>>>((const uint4 *)src, bytes / 16, sink);
    return hipGetLastError();
}

hipError_t launch_compact_in_place(void *k, void *v, float *scores, const int32_t *keep_idx, int B, int Hkv, int N,
                                   int budget, int row_bytes, hipStream_t stream) {
    const int row_vec = row_bytes / 16;
    const dim3 grid((unsigned)((row_vec + 3) / 4), scores ? 3 : 2, (unsigned)(B * Hkv));
    move_rows_in_place<<<grid, dim3(kMoveThreads), 0, stream>>>((uint4 *)k, (uint4 *)v, scores, keep_idx, N, budget, row_vec);
    return hipGetLastError();
}

hipError_t launch_evict_one(void *k, void *v, float *scores, int32_t *evicted, int B, int Hkv, int N, int ragged,
                            const SeqLens &lens, int first, int tail, int row_bytes, hipStream_t stream) {
    evict_pick<<<dim3(B * Hkv), dim3(256), 0, stream>>>(scores, N, Hkv, ragged, lens, first, tail, evicted);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int row_vec = row_bytes / 16;
    const dim3 grid((row_vec + 3) / 4, 3, B * Hkv);
    evict_shift<<<grid, dim3(kMoveThreads), 0, stream>>>((uint4 *)k, (uint4 *)v, scores, evicted, N, Hkv, ragged, lens, row_vec);
    return hipGetLastError();
}

hipError_t launch_compact(const void *k, const void *v, const int32_t *keep_idx, void *k_out, void *v_out, int B,
                          int Hkv, int N, int budget, int row_bytes, hipStream_t stream) {
    const int row_vec = row_bytes / 16;
    const size_t total = (size_t)B * Hkv * budget * row_vec;
    const dim3 grid((unsigned)((total + 255) / 256), 2);
    gather_rows<<<grid, dim3(256), 0, stream>>>((const uint4 *)k, (const uint4 *)v, keep_idx, (uint4 *)k_out,
                                                (uint4 *)v_out, N, budget, row_vec, total);
    return hipGetLastError();
}

}  // namespace obc

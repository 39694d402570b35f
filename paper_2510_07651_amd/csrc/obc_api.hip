// Host side of the C ABI declared in include/obcache.h: argument validation, workspace
// carve-up and kernel dispatch.  Nothing here allocates or synchronises.
#include <atomic>
#include <cstring>
#include <mutex>

#include "internal.h"

// Scratch of obc_score_static: one copy per GPU the library is loaded on, held until the process ends.
// Host code never uses this name as an address; it asks the runtime for the device address once per device.
static __device__ __align__(256) unsigned char scratch[OBC_STATIC_SCRATCH_BYTES];

namespace obc {

// Process-wide routing and tuning set through obc_set_score_path / obc_set_score_tuning.  The size query and
// the scoring call read the same state, so a plan never depends on anything but its arguments and these.
static std::atomic<int> g_score_path{OBC_PATH_AUTO};
static std::atomic<int> g_tuned_splits{0}, g_tuned_range{0}, g_tuned_form{0};
int tuned_splits() { return g_tuned_splits.load(std::memory_order_relaxed); }
int tuned_range() { return g_tuned_range.load(std::memory_order_relaxed); }
int tuned_sweep2_form() { return g_tuned_form.load(std::memory_order_relaxed); }

// Device address of `scratch` on the current device, looked up once per device.
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[kMaxDevices];
static hipError_t static_scratch(void **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p || ((uintptr_t)p & 255) != 0) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static int check_score_shape(int B, int N, int W, int Hq, int Hkv, int d, int dtype, int variant) {
    if (B < 1 || N < 1 || W < 1 || Hq < 1 || Hkv < 1 || d < 1) return OBC_EINVAL;
    if (Hq % Hkv != 0 || W > N) return OBC_EINVAL;
    if (variant < OBC_VALUE || variant > OBC_VATP) return OBC_EINVAL;
    if (dtype != OBC_F32 && dtype != OBC_BF16) return OBC_EUNSUPPORTED;
    if (d != 64 && d != 128) return OBC_EUNSUPPORTED;
    if (W > OBC_MAX_WINDOW || (Hq / Hkv) * W > OBC_MAX_GROUP_ROWS) return OBC_EUNSUPPORTED;
    if ((long long)B * Hq > 65535 * 16LL || (long long)B * Hkv > 65535) return OBC_EUNSUPPORTED;
    if ((long long)N > (1LL << 30)) return OBC_EUNSUPPORTED;
    return OBC_OK;
}

// obc_set_score_path pins the scoring path for comparisons: OBC_PATH_PLAIN routes everything through the
// general vector-ALU kernels, OBC_PATH_MFMA keeps one-row windows on the matrix-core path, OBC_PATH_DECODE
// sends them to the decode kernels whatever the cache size.
static bool score_path_is(int path) { return g_score_path.load(std::memory_order_relaxed) == path; }

int plan_score_workspace(int B, int N, int W, int Hq, int Hkv, int d, int dtype, int variant, ScoreWorkspace *ws) {
    const int rc = check_score_shape(B, N, W, Hq, Hkv, d, dtype, variant);
    if (rc != OBC_OK) return rc;
    std::memset(ws, 0, sizeof(*ws));
    const int G = Hq / Hkv;
    const size_t rows = (size_t)B * Hq * W;
    const bool pinned = score_path_is(OBC_PATH_PLAIN) || score_path_is(OBC_PATH_MFMA);
    ws->use_decode = (decode_path_covers(B, N, W, Hq, Hkv, d, dtype, variant, score_path_is(OBC_PATH_DECODE)) && !pinned) ? 1 : 0;
    ws->use_mfma = (!ws->use_decode && dtype == OBC_BF16 && d == 128 && !score_path_is(OBC_PATH_PLAIN)) ? 1 : 0;
    ws->m_pad = (G * W + 31) / 32 * 32;
    size_t off = 0;
    if (ws->use_decode) {
        decode_plan(B, N, Hq, Hkv, d, ws, &off);
    } else if (ws->use_mfma) {
        mfma_plan(B, N, W, Hq, Hkv, d, variant, ws, &off);
    } else {                                     // the plain path's per-row statistics and outputs
        ws->row_max = off;  off = align_up(off + rows * sizeof(float), 256);
        ws->row_sum = off;  off = align_up(off + rows * sizeof(float), 256);
        ws->out_f32 = off;  off = align_up(off + rows * d * sizeof(float), 256);
        ws->out_rest_f32 = off;  off = align_up(off + rows * d * sizeof(float), 256);
        ws->rest_frac = off;  off = align_up(off + rows * sizeof(float), 256);
        ws->top_token = off;  off = align_up(off + rows * sizeof(int32_t), 256);
    }
    ws->total = align_up(off, 256);
    return OBC_OK;
}

static int fill_lens(const int32_t *seq_lens_host, int B, int N, int min_len, int *ragged, SeqLens *lens) {
    *ragged = 0;
    if (!seq_lens_host) return N >= min_len ? OBC_OK : OBC_EINVAL;
    if (B > OBC_MAX_RAGGED_BATCH) return OBC_EUNSUPPORTED;
    for (int b = 0; b < B; ++b) {
        const int L = seq_lens_host[b];
        if (L > N || L < min_len) return OBC_EINVAL;
        lens->len[b] = L;
    }
    *ragged = 1;
    return OBC_OK;
}

}  // namespace obc

using namespace obc;

extern "C" {

int obc_version(void) { return 104; }

int obc_init(void) {
    void *p = nullptr;
    return static_scratch(&p) == hipSuccess ? OBC_OK : OBC_ELAUNCH;
}

int obc_set_score_path(int path) {
    if (path < OBC_PATH_AUTO || path > OBC_PATH_DECODE) return OBC_EINVAL;
    g_score_path.store(path, std::memory_order_relaxed);
    return OBC_OK;
}

int obc_set_sweep2_form(int form) {
    if (form < 0 || form > 2) return OBC_EINVAL;
    g_tuned_form.store(form, std::memory_order_relaxed);
    return OBC_OK;
}

int obc_set_score_tuning(int splits, int range_len) {
    if (splits < 0 || range_len < 0 || (range_len != 0 && (range_len < 64 || range_len > 65536 || range_len % 64 != 0)))
        return OBC_EINVAL;
    g_tuned_splits.store(splits, std::memory_order_relaxed);
    g_tuned_range.store(range_len, std::memory_order_relaxed);
    return OBC_OK;
}

const char *obc_status_string(int status) {
    switch (status) {
        case OBC_OK: return "OBC_OK";
        case OBC_EINVAL: return "OBC_EINVAL: invalid argument";
        case OBC_EUNSUPPORTED: return "OBC_EUNSUPPORTED: shape or dtype not supported by the gfx950 kernels";
        case OBC_EWORKSPACE: return "OBC_EWORKSPACE: workspace missing, misaligned or too small (obc_score_static: the shape needs more than OBC_STATIC_SCRATCH_BYTES)";
        case OBC_ELAUNCH: return "OBC_ELAUNCH: HIP launch error";
        default: return "unknown obcache status";
    }
}

int obc_score_workspace_bytes(int B, int N, int W, int Hq, int Hkv, int d, int dtype, int variant,
                              size_t *bytes_out) {
    if (!bytes_out) return OBC_EINVAL;
    ScoreWorkspace ws;
    const int rc = plan_score_workspace(B, N, W, Hq, Hkv, d, dtype, variant, &ws);
    if (rc != OBC_OK) return rc;
    *bytes_out = ws.total;
    return OBC_OK;
}

int obc_score(const void *q, const void *k, const void *v, int N, int W, int Hq, int Hkv, int d, int variant,
              float *scores, int B, int dtype, const int32_t *seq_lens_host, void *workspace,
              size_t workspace_bytes, void *hip_stream) {
    return obc_score_stages(q, k, v, N, W, Hq, Hkv, d, variant, scores, B, dtype, seq_lens_host, workspace,
                            workspace_bytes, hip_stream, OBC_STAGE_ALL);
}

static int score_impl(const void *q, const void *k, const void *v, int N, int W, int Hq, int Hkv, int d, int variant,
                      float *scores, int B, int dtype, const int32_t *seq_lens_host, void *workspace,
                      size_t workspace_bytes, void *hip_stream, int stage_mask, int accumulate);

int obc_score_stages(const void *q, const void *k, const void *v, int N, int W, int Hq, int Hkv, int d, int variant,
                     float *scores, int B, int dtype, const int32_t *seq_lens_host, void *workspace,
                     size_t workspace_bytes, void *hip_stream, int stage_mask) {
    return score_impl(q, k, v, N, W, Hq, Hkv, d, variant, scores, B, dtype, seq_lens_host, workspace, workspace_bytes,
                      hip_stream, stage_mask, 0);
}

int obc_score_accumulate(const void *q, const void *k, const void *v, int N, int W, int Hq, int Hkv, int d,
                         int variant, float *scores, int B, int dtype, const int32_t *seq_lens_host,
                         void *workspace, size_t workspace_bytes, void *hip_stream) {
    return score_impl(q, k, v, N, W, Hq, Hkv, d, variant, scores, B, dtype, seq_lens_host, workspace, workspace_bytes,
                      hip_stream, OBC_STAGE_ALL, 1);
}

int obc_score_static(const void *q, const void *k, const void *v, int N, int W, int Hq, int Hkv, int d, int variant,
                     float *scores, int B, int dtype, const int32_t *seq_lens_host, int accumulate, void *hip_stream) {
    if (accumulate != 0 && accumulate != 1) return OBC_EINVAL;
    // (workspace == NULL with the largest size: score_impl takes the library's own scratch and checks the plan against it)
    return score_impl(q, k, v, N, W, Hq, Hkv, d, variant, scores, B, dtype, seq_lens_host, nullptr,
                      OBC_STATIC_SCRATCH_BYTES, hip_stream, OBC_STAGE_ALL, accumulate | 2);
}

// `accumulate` bit 0: add to the scores; bit 1: use the library's static scratch (workspace must be NULL).
static int score_impl(const void *q, const void *k, const void *v, int N, int W, int Hq, int Hkv, int d, int variant,
                      float *scores, int B, int dtype, const int32_t *seq_lens_host, void *workspace,
                      size_t workspace_bytes, void *hip_stream, int stage_mask, int accumulate) {
    const bool own_scratch = (accumulate & 2) != 0;
    accumulate &= 1;
    if (!q || !k || !v || !scores) return OBC_EINVAL;
    if ((((uintptr_t)q | (uintptr_t)k | (uintptr_t)v) & 15) != 0 || ((uintptr_t)scores & 3) != 0) return OBC_EINVAL;
    if (stage_mask < 1 || stage_mask > OBC_STAGE_ALL) return OBC_EINVAL;
    ScoreWorkspace ws;
    int rc = plan_score_workspace(B, N, W, Hq, Hkv, d, dtype, variant, &ws);
    if (rc != OBC_OK) return rc;
    ScoreArgs a;
    std::memset(&a, 0, sizeof(a));
    rc = fill_lens(seq_lens_host, B, N, W, &a.ragged, &a.lens);
    if (rc != OBC_OK) return rc;
    if (own_scratch) {
        if (ws.total > workspace_bytes) return OBC_EWORKSPACE;           // the shape does not fit the static scratch
        if (static_scratch(&workspace) != hipSuccess) return OBC_ELAUNCH;
    }
    if (!workspace || ((uintptr_t)workspace & 255) != 0 || workspace_bytes < ws.total) return OBC_EWORKSPACE;
    a.q = q; a.k = k; a.v = v; a.scores = scores;
    a.B = B; a.N = N; a.W = W; a.Hq = Hq; a.Hkv = Hkv; a.d = d; a.G = Hq / Hkv;
    a.variant = variant; a.dtype = dtype;
    hipStream_t stream = (hipStream_t)hip_stream;
    a.stage_mask = stage_mask;
    a.accumulate = accumulate;
    const hipError_t e = ws.use_decode ? launch_score_decode(a, ws, (char *)workspace, stream)
                         : ws.use_mfma ? launch_score_mfma(a, ws, (char *)workspace, stream)
                                       : launch_score_plain(a, ws, (char *)workspace, stream);
    return e == hipSuccess ? OBC_OK : OBC_ELAUNCH;
}

int obc_select_workspace_bytes(int B, int Hkv, int N, size_t *bytes_out) {
    if (!bytes_out || B < 1 || Hkv < 1 || N < 1) return OBC_EINVAL;
    if ((long long)B * Hkv > 0x7fffffffLL / 2 || (long long)N > (1LL << 30)) return OBC_EUNSUPPORTED;
    *bytes_out = select_prefers_slices(B, Hkv, N) ? select_workspace_bytes(B, Hkv, N) : 0;
    return OBC_OK;
}

int obc_select_pooled(const float *scores, int num_hh, int num_sinks, int num_recent, int num_coming, int pool,
                      int32_t *keep_idx, int B, int Hkv, int N, const int32_t *seq_lens_host, void *workspace,
                      size_t workspace_bytes, void *hip_stream) {
    if (!scores || !keep_idx) return OBC_EINVAL;
    if (B < 1 || Hkv < 1 || N < 1) return OBC_EINVAL;
    if (num_hh < 0 || num_sinks < 0 || num_coming < 0 || num_recent < num_coming) return OBC_EINVAL;
    if (pool < 1 || pool % 2 == 0) return OBC_EINVAL;
    if (pool > OBC_MAX_POOL) return OBC_EUNSUPPORTED;
    if ((long long)B * Hkv > 0x7fffffffLL / 2 || (long long)N > (1LL << 30)) return OBC_EUNSUPPORTED;
    if (workspace && ((uintptr_t)workspace & 255) != 0) return OBC_EWORKSPACE;
    const long long tail = (long long)num_recent - num_coming;
    const long long budget = (long long)num_sinks + num_hh + tail;     // every sequence must hold this many tokens
    if (budget < 1 || budget > N) return OBC_EINVAL;
    int ragged = 0;
    SeqLens lens;
    std::memset(&lens, 0, sizeof(lens));
    const int rc = fill_lens(seq_lens_host, B, N, (int)budget, &ragged, &lens);
    if (rc != OBC_OK) return rc;
    const hipError_t e = launch_select(scores, (int)budget, keep_idx, B, Hkv, N, ragged, lens, num_sinks, (int)tail,
                                       (pool - 1) / 2, workspace, workspace_bytes, (hipStream_t)hip_stream);
    return e == hipSuccess ? OBC_OK : OBC_ELAUNCH;
}

int obc_select_protected(const float *scores, int num_hh, int num_sinks, int num_recent, int num_coming,
                         int32_t *keep_idx, int B, int Hkv, int N, const int32_t *seq_lens_host, void *workspace,
                         size_t workspace_bytes, void *hip_stream) {
    return obc_select_pooled(scores, num_hh, num_sinks, num_recent, num_coming, 1, keep_idx, B, Hkv, N, seq_lens_host,
                             workspace, workspace_bytes, hip_stream);
}

int obc_select(const float *scores, int budget, int32_t *keep_idx, int B, int Hkv, int N,
               const int32_t *seq_lens_host, void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (budget < 1) return OBC_EINVAL;
    return obc_select_pooled(scores, budget, 0, 0, 0, 1, keep_idx, B, Hkv, N, seq_lens_host, workspace,
                             workspace_bytes, hip_stream);
}

static int adaptive_checks(int budget, int n_safe, int cap, int B, int Hkv, int N, const int32_t *seq_lens_host,
                           int *ragged, SeqLens *lens) {
    if (B < 1 || Hkv < 1 || N < 1 || budget < 1 || n_safe < 0 || n_safe > budget || budget > N) return OBC_EINVAL;
    if ((long long)B * Hkv > 0x7fffffffLL / 2 || (long long)Hkv * N > (1LL << 30)) return OBC_EUNSUPPORTED;
    const int rc = fill_lens(seq_lens_host, B, N, budget, ragged, lens);
    if (rc != OBC_OK) return rc;
    for (int b = 0; b < B; ++b) {          // the most one head can receive must fit its index list
        const long long len = *ragged ? lens->len[b] : N;
        long long most = (long long)Hkv * budget - (long long)(Hkv - 1) * n_safe;
        if (most > len) most = len;
        if (cap < most) return OBC_EINVAL;
    }
    return OBC_OK;
}

int obc_select_adaptive_workspace_bytes(int B, int Hkv, int N, int budget, int n_safe, size_t *bytes_out) {
    if (!bytes_out || B < 1 || Hkv < 1 || N < 1 || budget < 1 || n_safe < 0 || n_safe > budget || budget > N) return OBC_EINVAL;
    if ((long long)B * Hkv > 0x7fffffffLL / 2 || (long long)Hkv * N > (1LL << 30)) return OBC_EUNSUPPORTED;
    *bytes_out = select_adaptive_workspace_bytes(B, Hkv, N, budget, n_safe);
    return OBC_OK;
}

int obc_select_adaptive(const float *scores, int budget, int n_safe, int32_t *keep_idx, int32_t *counts, int cap,
                        int B, int Hkv, int N, const int32_t *seq_lens_host, void *workspace, size_t workspace_bytes,
                        void *hip_stream) {
    if (!scores || !keep_idx || !counts) return OBC_EINVAL;
    int ragged = 0;
    SeqLens lens;
    std::memset(&lens, 0, sizeof(lens));
    const int rc = adaptive_checks(budget, n_safe, cap, B, Hkv, N, seq_lens_host, &ragged, &lens);
    if (rc != OBC_OK) return rc;
    if (!workspace || ((uintptr_t)workspace & 255) != 0 ||
        workspace_bytes < select_adaptive_workspace_bytes(B, Hkv, N, budget, n_safe))
        return OBC_EWORKSPACE;
    const hipError_t e = launch_select_adaptive(scores, budget, n_safe, cap, keep_idx, counts, B, Hkv, N, ragged, lens,
                                                workspace, (hipStream_t)hip_stream);
    return e == hipSuccess ? OBC_OK : OBC_ELAUNCH;
}

int obc_compact(const void *k, const void *v, const int32_t *keep_idx, void *k_out, void *v_out, int B, int Hkv,
                int N, int budget, int d, int dtype, void *hip_stream) {
    if (!k || !v || !keep_idx || !k_out || !v_out) return OBC_EINVAL;
    if ((((uintptr_t)k | (uintptr_t)v | (uintptr_t)k_out | (uintptr_t)v_out) & 15) != 0) return OBC_EINVAL;
    if (B < 1 || Hkv < 1 || N < 1 || budget < 1 || d < 1) return OBC_EINVAL;
    if (dtype != OBC_F32 && dtype != OBC_BF16) return OBC_EUNSUPPORTED;
    const long long row_bytes = (long long)d * (dtype == OBC_F32 ? 4 : 2);
    if (row_bytes % 16 != 0 || row_bytes > (1 << 20)) return OBC_EUNSUPPORTED;
    if ((long long)B * Hkv * budget * (row_bytes / 16) > (1LL << 38)) return OBC_EUNSUPPORTED;
    const hipError_t e = launch_compact(k, v, keep_idx, k_out, v_out, B, Hkv, N, budget, (int)row_bytes,
                                        (hipStream_t)hip_stream);
    return e == hipSuccess ? OBC_OK : OBC_ELAUNCH;
}

int obc_compact_inplace(void *k, void *v, float *scores, const int32_t *keep_idx, int B, int Hkv, int N, int budget,
                        int d, int dtype, void *hip_stream) {
    if (!k || !v || !keep_idx) return OBC_EINVAL;
    if ((((uintptr_t)k | (uintptr_t)v) & 15) != 0 || ((uintptr_t)scores & 3) != 0) return OBC_EINVAL;
    if (B < 1 || Hkv < 1 || N < 1 || budget < 1 || budget > N || d < 1) return OBC_EINVAL;
    if (dtype != OBC_F32 && dtype != OBC_BF16) return OBC_EUNSUPPORTED;
    const long long row_bytes = (long long)d * (dtype == OBC_F32 ? 4 : 2);
    if (row_bytes % 16 != 0 || row_bytes > (1 << 20)) return OBC_EUNSUPPORTED;
    if ((long long)B * Hkv > 65535 || (long long)N > (1LL << 30)) return OBC_EUNSUPPORTED;
    const hipError_t e = launch_compact_in_place(k, v, scores, keep_idx, B, Hkv, N, budget, (int)row_bytes,
                                                 (hipStream_t)hip_stream);
    return e == hipSuccess ? OBC_OK : OBC_ELAUNCH;
}

int obc_decode_step_workspace_bytes(int B, int N, int Hq, int Hkv, int d, int dtype, int variant, size_t *bytes_out) {
    if (!bytes_out) return OBC_EINVAL;
    if (variant == OBC_ALL) return OBC_EINVAL;          // one running score per token
    ScoreWorkspace ws;
    const int rc = plan_score_workspace(B, N, 1, Hq, Hkv, d, dtype, variant, &ws);
    if (rc != OBC_OK) return rc;
    *bytes_out = ws.total + align_up((size_t)B * Hkv * sizeof(int32_t), 256);
    return OBC_OK;
}

int obc_decode_step(const void *q, void *k, void *v, float *scores, int32_t *evicted, int N, int Hq, int Hkv, int d,
                    int variant, int B, int dtype, const int32_t *seq_lens_host, int num_sinks, int num_recent,
                    void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (variant == OBC_ALL || num_sinks < 0 || num_recent < 0) return OBC_EINVAL;
    if (((uintptr_t)evicted & 3) != 0) return OBC_EINVAL;
    size_t need = 0;
    int rc = obc_decode_step_workspace_bytes(B, N, Hq, Hkv, d, dtype, variant, &need);
    if (rc != OBC_OK) return rc;
    // every sequence must hold a token that competes: num_sinks + num_recent < len_b (checked before anything runs)
    int ragged = 0;
    SeqLens lens;
    std::memset(&lens, 0, sizeof(lens));
    const long long protect = (long long)num_sinks + num_recent;
    if (protect + 1 > N) return OBC_EINVAL;
    rc = fill_lens(seq_lens_host, B, N, (int)protect + 1, &ragged, &lens);
    if (rc != OBC_OK) return rc;
    if (!workspace || ((uintptr_t)workspace & 255) != 0 || workspace_bytes < need) return OBC_EWORKSPACE;
    const size_t score_bytes = need - align_up((size_t)B * Hkv * sizeof(int32_t), 256);
    rc = score_impl(q, k, v, N, 1, Hq, Hkv, d, variant, scores, B, dtype, seq_lens_host, workspace, score_bytes, hip_stream,
                    OBC_STAGE_ALL, 1);
    if (rc != OBC_OK) return rc;
    int32_t *pick = evicted ? evicted : (int32_t *)((char *)workspace + score_bytes);
    const long long row_bytes = (long long)d * (dtype == OBC_F32 ? 4 : 2);
    const hipError_t e = launch_evict_one(k, v, scores, pick, B, Hkv, N, ragged, lens, num_sinks, num_recent, (int)row_bytes,
                                          (hipStream_t)hip_stream);
    return e == hipSuccess ? OBC_OK : OBC_ELAUNCH;
}

int obc_compact_scores(const float *scores, const int32_t *keep_idx, float *scores_out, int B, int Hkv, int N,
                       int budget, int N_out, void *hip_stream) {
    if (!scores || !keep_idx || !scores_out) return OBC_EINVAL;
    if (B < 1 || Hkv < 1 || N < 1 || budget < 1 || N_out < budget) return OBC_EINVAL;
    if ((long long)B * Hkv * N_out > (1LL << 40)) return OBC_EUNSUPPORTED;
    const hipError_t e = launch_gather_scores(scores, keep_idx, scores_out, B * Hkv, N, budget, N_out,
                                              (hipStream_t)hip_stream);
    return e == hipSuccess ? OBC_OK : OBC_ELAUNCH;
}

int obc_probe_read_bandwidth(const void *buf, size_t bytes, uint32_t *sink, void *hip_stream) {
    if (!buf || !sink || bytes < 16 || bytes % 16 != 0) return OBC_EINVAL;
    if (((uintptr_t)buf & 15) != 0) return OBC_EINVAL;
    const hipError_t e = launch_stream_read(buf, bytes, sink, OBC_PROBE_BLOCKS, (hipStream_t)hip_stream);
    return e == hipSuccess ? OBC_OK : OBC_ELAUNCH;
}

}  // extern "C"

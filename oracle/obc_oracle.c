/*
 * OBCache CPU oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, fp64 implementation of what the GPU hot path must compute,
 * written from the paper (arxiv 2510.07651) and sharing no code with the HIP
 * kernels.  Only tests, the smoke check and the benchmark's cpu_baseline leg
 * may call it.
 *
 * What it follows:
 *   - Section 3 (Prefill / Decoding):  Z = Q K^T / sqrt(d),  A = softmax_row(Z),  O = A V.
 *   - Section 4.3, windowed objective (Eq. 9 / Appendix A.1): only the last W
 *     query rows ("perturbation window") enter the sums.
 *   - Proposition 1 (Eq. 4):  S^value_p = sum_i A_ip^2 ||v_p||^2
 *   - Proposition 2 (Eq. 5):  S^key_p   = sum_i A_ip^2 Z_ip^2 ||v_p - o_i||^2
 *   - Proposition 3 (Eq. 6):  S^joint_p = S^value_p + S^key_p
 *                                       + 2 sum_i A_ip^2 Z_ip (||v_p||^2 - v_p . o_i)
 *   - Appendix A.5 (GQA): the score of KV head g is the sum of the per-query-head
 *     scores over the heads h in H(g), each with its own A^h, Z^h, o^h and the
 *     shared v^g.
 *   - Appendix E, Algorithm 2: top-k by score, kept indices sorted ascending,
 *     rows of K and V gathered.
 *
 * Readings taken where the paper is silent (listed in the design notes too):
 *   - Query row r (0-based, r < W) of a sequence of true length len sits at
 *     absolute position len - W + r and sees keys p <= len - W + r (causal,
 *     window rows causal among themselves).  Invisible (r, p) pairs are absent:
 *     they are not part of the softmax and contribute exactly 0 to every score.
 *   - Z in Eq. 5-6 is the raw scaled logit q.k/sqrt(d), not a max-shifted one.
 *   - Query head h reads KV head g = h / (Hq/Hkv)  (consecutive grouping).
 *   - Top-k ties go to the lowest token index; positions p >= len are never kept
 *     and their scores are 0.
 *
 * Pins (tests/test_oracle_pins.py): softmax rows sum to 1; value score equals
 * the exact output change when v_p is zeroed (brute force); key and joint scores
 * equal the squared directional derivative of the window output (central
 * differences, brute force); q = 0 closed form; library attention
 * (torch scaled_dot_product_attention, fp64); token permutation equivariance;
 * GQA = sum of MHA heads; Eq. 6 literal form == completed-square form;
 * select vs a library stable sort; compaction vs fancy indexing; Eq. 4-6 in
 * 50-digit arithmetic for a key that holds up to 1 - 1e-16 of a row's weight.
 * No function here is "parity unpinned".
 *
 * Arithmetic: fp64 throughout, every formula as printed, with one exception
 * forced by fp64 itself: v_p - o_i for the row's largest-weight key is summed
 * as sum_q A_iq (v_p - v_q) (equal because a softmax row sums to one), since
 * the plain difference cancels as that weight tends to 1 (see obc_oracle_score).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define OBC_ORACLE_OK 0
#define OBC_ORACLE_EINVAL -1

int obc_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int seq_len_of(const int32_t *seq_lens, int b, int N)
{
    return seq_lens ? (int)seq_lens[b] : N;
}

static int check_shapes(int B, int Hq, int Hkv, int N, int W, int d, const int32_t *seq_lens)
{
    if (B < 1 || Hq < 1 || Hkv < 1 || N < 1 || W < 1 || d < 1) return OBC_ORACLE_EINVAL;
    if (Hq % Hkv != 0) return OBC_ORACLE_EINVAL;
    for (int b = 0; b < B; ++b) {
        int len = seq_len_of(seq_lens, b, N);
        if (len > N || len < W) return OBC_ORACLE_EINVAL;
    }
    return OBC_ORACLE_OK;
}

/*
 * One window row of attention (Section 3): logits over the visible keys,
 * softmax, output.  z, a have room for n_vis entries; o has d entries.
 */
static void attention_row(const double *q_row, const double *K, const double *V, int n_vis, int d,
                          double *z, double *a, double *o)
{
    const double inv_sqrt_d = 1.0 / sqrt((double)d);
    double zmax = -INFINITY;
    for (int p = 0; p < n_vis; ++p) {
        double dot = 0.0;
        for (int j = 0; j < d; ++j) dot += q_row[j] * K[(size_t)p * d + j];
        z[p] = dot * inv_sqrt_d;
        if (z[p] > zmax) zmax = z[p];
    }
    double denom = 0.0;
    for (int p = 0; p < n_vis; ++p) {
        a[p] = exp(z[p] - zmax);
        denom += a[p];
    }
    for (int p = 0; p < n_vis; ++p) a[p] /= denom;
    for (int j = 0; j < d; ++j) o[j] = 0.0;
    for (int p = 0; p < n_vis; ++p)
        for (int j = 0; j < d; ++j) o[j] += a[p] * V[(size_t)p * d + j];
}

/*
 * Window attention internals for small cases (tests only):
 *   Z, A : [B, Hq, W, N]  (entries for invisible pairs are set to NaN / 0)
 *   O    : [B, Hq, W, d]
 */
int obc_oracle_window_attention(const double *q, const double *k, const double *v,
                                int B, int Hq, int Hkv, int N, int W, int d,
                                const int32_t *seq_lens, double *Z, double *A, double *O)
{
    int rc = check_shapes(B, Hq, Hkv, N, W, d, seq_lens);
    if (rc) return rc;
    const int G = Hq / Hkv;
    double *z = (double *)malloc(sizeof(double) * (size_t)N);
    double *a = (double *)malloc(sizeof(double) * (size_t)N);
    for (int b = 0; b < B; ++b) {
        int len = seq_len_of(seq_lens, b, N);
        for (int h = 0; h < Hq; ++h) {
            int g = h / G;
            const double *Kg = k + ((size_t)b * Hkv + g) * (size_t)N * d;
            const double *Vg = v + ((size_t)b * Hkv + g) * (size_t)N * d;
            for (int r = 0; r < W; ++r) {
                size_t row = ((size_t)b * Hq + h) * W + r;
                int n_vis = len - W + r + 1;
                attention_row(q + row * d, Kg, Vg, n_vis, d, z, a, O + row * d);
                for (int p = 0; p < N; ++p) {
                    Z[row * N + p] = p < n_vis ? z[p] : NAN;
                    A[row * N + p] = p < n_vis ? a[p] : 0.0;
                }
            }
        }
    }
    free(z);
    free(a);
    return OBC_ORACLE_OK;
}

/*
 * Scores for every (b, kv head g, token p).  Any of s_value, s_key, s_joint may
 * be NULL.  Layouts: q [B,Hq,W,d], k,v [B,Hkv,N,d], outputs [B,Hkv,N], all fp64,
 * contiguous.  seq_lens: NULL or B true lengths (W <= len <= N).
 *
 * joint_form = 0: per visible (i,p) the joint term is A^2 ||(1+Z) v_p - Z o_i||^2,
 *                 the completed square of Eq. 6 (expanding it gives
 *                 ||v||^2 + Z^2 ||v-o||^2 + 2 Z (||v||^2 - v.o)).
 * joint_form = 1: Eq. 6 literally: S^value + S^key + 2 sum A^2 Z (||v||^2 - v.o).
 * joint_form + 2 (test only): every key, the row's largest-weight one included, takes the plain differences
 *                 v_p - o_i; the tests compare this with the default where fp64 resolves both.
 */
int obc_oracle_score(const double *q, const double *k, const double *v,
                     int B, int Hq, int Hkv, int N, int W, int d,
                     const int32_t *seq_lens, int joint_form,
                     double *s_value, double *s_key, double *s_joint)
{
    int rc = check_shapes(B, Hq, Hkv, N, W, d, seq_lens);
    if (rc) return rc;
    const int G = Hq / Hkv;
    const int n_qheads = B * Hq;

    /* Per-query-head scores S_{p,h} (Appendix A.5, first display), one slab per (b, h). */
    double *hv = (double *)calloc((size_t)n_qheads * N, sizeof(double));
    double *hk = (double *)calloc((size_t)n_qheads * N, sizeof(double));
    double *hj = (double *)calloc((size_t)n_qheads * N, sizeof(double));
    double *hx = (double *)calloc((size_t)n_qheads * N, sizeof(double)); /* cross term of Eq. 6 */
    if (!hv || !hk || !hj || !hx) { free(hv); free(hk); free(hj); free(hx); return OBC_ORACLE_EINVAL; }

#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < n_qheads; ++bh) {
        const int b = bh / Hq, h = bh % Hq, g = h / G;
        const int len = seq_len_of(seq_lens, b, N);
        const double *Kg = k + ((size_t)b * Hkv + g) * (size_t)N * d;
        const double *Vg = v + ((size_t)b * Hkv + g) * (size_t)N * d;
        double *z = (double *)malloc(sizeof(double) * (size_t)N);
        double *a = (double *)malloc(sizeof(double) * (size_t)N);
        double *o = (double *)malloc(sizeof(double) * (size_t)d);
        double *dtop = (double *)malloc(sizeof(double) * (size_t)d);
        double *acc_v = hv + (size_t)bh * N, *acc_k = hk + (size_t)bh * N;
        double *acc_j = hj + (size_t)bh * N, *acc_x = hx + (size_t)bh * N;
        for (int r = 0; r < W; ++r) {               /* i = w..s, Eq. 9 */
            const int n_vis = len - W + r + 1;
            const double *q_row = q + ((size_t)bh * W + r) * d;
            attention_row(q_row, Kg, Vg, n_vis, d, z, a, o);
            /*
             * The key with the largest weight of the row.  As that weight tends to 1, o_i tends to
             * v_p and the plain difference v_p - o_i loses eps / (1 - A_ip) of its relative
             * accuracy, all of it once 1 - A_ip reaches 1e-16.  The weights of a row sum to one
             * (Section 3), so v_p - o_i = sum_q A_iq (v_p - v_q) exactly: a sum of small terms
             * whose q = p term is zero.  For this one key of the row the difference is formed
             * that way, (1+Z) v - Z o as v + Z (v - o), and ||v||^2 - v.o as v.(v - o).
             */
            int p_top = 0;
            for (int p = 1; p < n_vis; ++p) if (a[p] > a[p_top]) p_top = p;
            for (int j = 0; j < d; ++j) dtop[j] = 0.0;
            for (int qq = 0; qq < n_vis; ++qq) {
                if (qq == p_top) continue;
                for (int j = 0; j < d; ++j) dtop[j] += a[qq] * (Vg[(size_t)p_top * d + j] - Vg[(size_t)qq * d + j]);
            }
            for (int p = 0; p < n_vis; ++p) {
                const double *vp = Vg + (size_t)p * d;
                const double A2 = a[p] * a[p];
                const int top = p == p_top && !(joint_form & 2);
                double vv = 0.0, vmo2 = 0.0, vvmvo = 0.0, sq = 0.0;
                for (int j = 0; j < d; ++j) {
                    const double diff = top ? dtop[j] : vp[j] - o[j];
                    const double comb = top ? vp[j] + z[p] * dtop[j] : (1.0 + z[p]) * vp[j] - z[p] * o[j];
                    vv += vp[j] * vp[j];
                    vmo2 += diff * diff;
                    vvmvo += top ? vp[j] * dtop[j] : vp[j] * vp[j] - vp[j] * o[j];
                    sq += comb * comb;
                }
                acc_v[p] += A2 * vv;                       /* Eq. 4 */
                acc_k[p] += A2 * z[p] * z[p] * vmo2;       /* Eq. 5 */
                acc_j[p] += A2 * sq;                       /* Eq. 6, completed square */
                acc_x[p] += 2.0 * A2 * z[p] * vvmvo;       /* Eq. 6, cross term */
            }
        }
        free(z); free(a); free(o); free(dtop);
    }

    /* Score of KV head g = sum over its query heads h in H(g) (Appendix A.5, second display). */
    for (int bg = 0; bg < B * Hkv; ++bg) {
        const int b = bg / Hkv, g = bg % Hkv;
        const int len = seq_len_of(seq_lens, b, N);
        for (int p = 0; p < N; ++p) {
            double sv = 0.0, sk = 0.0, sj = 0.0, sx = 0.0;
            for (int hh = 0; hh < G; ++hh) {
                const size_t src = ((size_t)b * Hq + g * G + hh) * N + p;
                sv += hv[src]; sk += hk[src]; sj += hj[src]; sx += hx[src];
            }
            const size_t idx = (size_t)bg * N + p;
            const int live = p < len;
            if (s_value) s_value[idx] = live ? sv : 0.0;
            if (s_key) s_key[idx] = live ? sk : 0.0;
            if (s_joint) s_joint[idx] = live ? ((joint_form & 1) ? sv + sk + sx : sj) : 0.0;
        }
    }
    free(hv); free(hk); free(hj); free(hx);
    return OBC_ORACLE_OK;
}

/*
 * Attention-only score of Section 4.3 (Eq. 8): S^attn_p = sum_i |A_ip| over the
 * window, summed over the query heads of the group.  Used by tests of the
 * special cases (w = s gives the single-row case).
 */
int obc_oracle_attn_score(const double *q, const double *k, const double *v,
                          int B, int Hq, int Hkv, int N, int W, int d,
                          const int32_t *seq_lens, double *s_attn)
{
    int rc = check_shapes(B, Hq, Hkv, N, W, d, seq_lens);
    if (rc) return rc;
    const int G = Hq / Hkv;
    double *z = (double *)malloc(sizeof(double) * (size_t)N);
    double *a = (double *)malloc(sizeof(double) * (size_t)N);
    double *o = (double *)malloc(sizeof(double) * (size_t)d);
    for (int bg = 0; bg < B * Hkv; ++bg) {
        const int b = bg / Hkv, g = bg % Hkv;
        const int len = seq_len_of(seq_lens, b, N);
        for (int p = 0; p < N; ++p) s_attn[(size_t)bg * N + p] = 0.0;
        for (int hh = 0; hh < G; ++hh)
            for (int r = 0; r < W; ++r) {
                const int n_vis = len - W + r + 1;
                const double *q_row = q + (((size_t)b * Hq + g * G + hh) * W + r) * d;
                attention_row(q_row, k + (size_t)bg * N * d, v + (size_t)bg * N * d, n_vis, d, z, a, o);
                for (int p = 0; p < n_vis; ++p) s_attn[(size_t)bg * N + p] += fabs(a[p]);
            }
    }
    free(z); free(a); free(o);
    return OBC_ORACLE_OK;
}

/*
 * VATP score as the paper reproduces it (Appendix C, "VATP and CriticalKV": the value
 * score with the l2 norm replaced by the l1 norm): S_p = sum_i |A_ip| * ||v_p||_1,
 * summed over the window and the query heads of the group; v_p is the group's shared
 * value row, so the norm factors out of the sums.
 */
int obc_oracle_vatp_score(const double *q, const double *k, const double *v,
                          int B, int Hq, int Hkv, int N, int W, int d,
                          const int32_t *seq_lens, double *s_vatp)
{
    int rc = obc_oracle_attn_score(q, k, v, B, Hq, Hkv, N, W, d, seq_lens, s_vatp);
    if (rc) return rc;
    for (size_t t = 0; t < (size_t)B * Hkv * N; ++t) {
        double l1 = 0.0;
        for (int j = 0; j < d; ++j) l1 += fabs(v[t * d + j]);
        s_vatp[t] = s_vatp[t] == 0.0 ? 0.0 : s_vatp[t] * l1;   /* padded rows may hold NaN: never multiplied in */
    }
    return OBC_ORACLE_OK;
}

/* ---- selection (Section 3 "Cache Eviction"; Algorithm 2: topk -> sort) ---- */

typedef struct { float s; int32_t p; } scored_t;

/* NaN ranks below every number; -0.0 equals +0.0. */
static int better(const scored_t *x, const scored_t *y)
{
    const int xn = isnan(x->s), yn = isnan(y->s);
    if (xn != yn) return yn;            /* the non-NaN one is better */
    if (!xn && x->s != y->s) return x->s > y->s;
    return x->p < y->p;                 /* tie: lowest index first */
}
static int cmp_scored(const void *a, const void *b)
{
    const scored_t *x = (const scored_t *)a, *y = (const scored_t *)b;
    if (better(x, y)) return -1;
    if (better(y, x)) return 1;
    return 0;
}
static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * scores [B,Hkv,N] fp32 -> keep_idx [B,Hkv,budget] int32, ascending.
 * Per (b,g): the budget best tokens among p < len_b, by (score descending,
 * index ascending).  Requires 1 <= budget <= len_b.
 */
int obc_oracle_select(const float *scores, int B, int Hkv, int N, int budget,
                      const int32_t *seq_lens, int32_t *keep_idx)
{
    if (B < 1 || Hkv < 1 || N < 1 || budget < 1) return OBC_ORACLE_EINVAL;
    for (int b = 0; b < B; ++b) {
        int len = seq_len_of(seq_lens, b, N);
        if (len > N || budget > len) return OBC_ORACLE_EINVAL;
    }
    scored_t *tmp = (scored_t *)malloc(sizeof(scored_t) * (size_t)N);
    for (int bg = 0; bg < B * Hkv; ++bg) {
        const int len = seq_len_of(seq_lens, bg / Hkv, N);
        for (int p = 0; p < len; ++p) {
            tmp[p].s = scores[(size_t)bg * N + p];
            tmp[p].p = p;
        }
        qsort(tmp, (size_t)len, sizeof(scored_t), cmp_scored);   /* total order: no ties left */
        int32_t *out = keep_idx + (size_t)bg * budget;
        for (int j = 0; j < budget; ++j) out[j] = tmp[j].p;
        qsort(out, (size_t)budget, sizeof(int32_t), cmp_i32);
    }
    free(tmp);
    return OBC_ORACLE_OK;
}

/*
 * Selection with protected regions (Appendix E, Algorithm 2; Appendix C, decoding setup).
 * Algorithm 2 lets only positions below cutoff = len - num_recent + num_coming compete
 * for the num_hh heavy-hitter slots and always keeps the tail [cutoff, len); the
 * decoding experiments additionally always keep the first few tokens as attention
 * sinks.  Per (b, g):
 *   kept = {0 .. num_sinks-1}
 *        + the num_hh highest scores among p in [num_sinks, cutoff)  (ties: lowest index)
 *        + {cutoff .. len-1},
 * written in ascending order; keep_idx is [B, Hkv, num_sinks + num_hh + num_recent - num_coming].
 * With num_sinks = 0 this is Algorithm 2 literally (topk over S[..., :cutoff], sort, then
 * the recent rows appended); with num_recent = num_coming as well it is obc_oracle_select.
 */
int obc_oracle_select_protected(const float *scores, int B, int Hkv, int N, int num_hh, int num_sinks,
                                int num_recent, int num_coming, const int32_t *seq_lens, int32_t *keep_idx)
{
    if (B < 1 || Hkv < 1 || N < 1 || num_hh < 0 || num_sinks < 0 || num_coming < 0 || num_recent < num_coming)
        return OBC_ORACLE_EINVAL;
    const int tail = num_recent - num_coming, total = num_sinks + num_hh + tail;
    if (total < 1) return OBC_ORACLE_EINVAL;
    for (int b = 0; b < B; ++b) {
        int len = seq_len_of(seq_lens, b, N);
        if (len > N || len - tail < num_sinks + num_hh) return OBC_ORACLE_EINVAL;
    }
    scored_t *tmp = (scored_t *)malloc(sizeof(scored_t) * (size_t)N);
    for (int bg = 0; bg < B * Hkv; ++bg) {
        const int len = seq_len_of(seq_lens, bg / Hkv, N);
        const int cutoff = len - tail;
        int32_t *out = keep_idx + (size_t)bg * total;
        int n = 0;
        for (int p = 0; p < num_sinks; ++p) out[n++] = p;
        int m = 0;
        for (int p = num_sinks; p < cutoff; ++p) {
            tmp[m].s = scores[(size_t)bg * N + p];
            tmp[m].p = p;
            ++m;
        }
        qsort(tmp, (size_t)m, sizeof(scored_t), cmp_scored);
        for (int j = 0; j < num_hh; ++j) out[n++] = tmp[j].p;
        qsort(out + num_sinks, (size_t)num_hh, sizeof(int32_t), cmp_i32);
        for (int p = cutoff; p < len; ++p) out[n++] = p;
    }
    free(tmp);
    return OBC_ORACLE_OK;
}

/*
 * Pooled selection (Appendix C, "SnapKV": a one-dimensional average-pooling filter of
 * kernel size 5 smooths the scores before eviction; used for every OBCache-enhanced
 * prefill experiment).  Same kept set as obc_oracle_select_protected, but the candidates
 * p in [num_sinks, cutoff) are ranked by the window sum
 *   P_p = sum_{j = p-r .. p+r, num_sinks <= j < cutoff} S_j ,   r = (pool - 1) / 2,
 * i.e. a centred stride-1 window with zeros beyond the candidate range.  The average is
 * P_p / pool; ranking by the sum avoids a division whose rounding could merge distinct
 * sums.  The sum runs in fp32 in ascending j starting from 0 (out-of-range terms add
 * +0), because this rounding decides which indices are kept and both sides must take
 * the decision in the same precision.  pool = 1 is obc_oracle_select_protected.
 */
int obc_oracle_select_pooled(const float *scores, int B, int Hkv, int N, int num_hh, int num_sinks,
                             int num_recent, int num_coming, int pool, const int32_t *seq_lens,
                             int32_t *keep_idx)
{
    if (pool < 1 || pool % 2 == 0 || N < 1 || B < 1 || Hkv < 1) return OBC_ORACLE_EINVAL;
    if (num_recent < num_coming || num_coming < 0 || num_sinks < 0) return OBC_ORACLE_EINVAL;
    const int r = (pool - 1) / 2, tail = num_recent - num_coming;
    float *pooled = (float *)malloc(sizeof(float) * (size_t)B * Hkv * N);
    for (int bg = 0; bg < B * Hkv; ++bg) {
        const int len = seq_len_of(seq_lens, bg / Hkv, N);
        const int cutoff = len - tail;
        const float *s = scores + (size_t)bg * N;
        float *o = pooled + (size_t)bg * N;
        for (int p = 0; p < N; ++p) {
            volatile float sum = 0.0f;          /* volatile: every partial sum is rounded to fp32 */
            if (p >= num_sinks && p < cutoff)
                for (int j = p - r; j <= p + r; ++j) sum = sum + ((j >= num_sinks && j < cutoff) ? s[j] : 0.0f);
            o[p] = sum;
        }
    }
    const int rc = obc_oracle_select_protected(pooled, B, Hkv, N, num_hh, num_sinks, num_recent, num_coming,
                                               seq_lens, keep_idx);
    free(pooled);
    return rc;
}

/*
 * Head-adaptive selection (Appendix C, "AdaKV": the head-wise budgets follow from ranking
 * the eviction scores globally across all heads of the layer, with a safeguard that is
 * 0.2 in the paper's experiments).  Reading taken here, per sequence b:
 *   - the layer keeps Hkv * budget tokens in total;
 *   - every KV head first keeps its own n_safe highest-scoring tokens (the safeguard:
 *     n_safe = floor(0.2 * budget) in the paper's setting), ties to the lowest index;
 *   - the remaining Hkv * (budget - n_safe) slots go to the highest scores among all other
 *     live (head, token) pairs of the sequence, ties to the lower head, then the lower index.
 * Output per (b, g): counts[b,g] kept tokens, their indices ascending in
 * keep_idx[b,g,0..count), then -1 up to `cap` entries.  n_safe = budget is the per-head
 * selection of obc_oracle_select; n_safe = 0 is a plain global top-k.
 */
typedef struct { float s; int32_t g; int32_t p; } scored3_t;
static int cmp_scored3(const void *a, const void *b)
{
    const scored3_t *x = (const scored3_t *)a, *y = (const scored3_t *)b;
    scored_t sx = { x->s, 0 }, sy = { y->s, 0 };
    int c = cmp_scored(&sx, &sy);              /* score order incl. NaN lowest, -0 == +0; 0 on equal scores */
    if (c) return c;
    if (x->g != y->g) return x->g < y->g ? -1 : 1;
    return x->p < y->p ? -1 : (x->p > y->p ? 1 : 0);
}

int obc_oracle_select_adaptive(const float *scores, int B, int Hkv, int N, int budget, int n_safe, int cap,
                               const int32_t *seq_lens, int32_t *keep_idx, int32_t *counts)
{
    if (B < 1 || Hkv < 1 || N < 1 || budget < 1 || n_safe < 0 || n_safe > budget || cap < 1) return OBC_ORACLE_EINVAL;
    for (int b = 0; b < B; ++b) {
        int len = seq_len_of(seq_lens, b, N);
        if (len > N || budget > len) return OBC_ORACLE_EINVAL;
        long long most = (long long)Hkv * budget - (long long)(Hkv - 1) * n_safe;   /* the most one head can get */
        if (most > len) most = len;
        if (cap < most) return OBC_ORACLE_EINVAL;
    }
    scored_t *tmp = (scored_t *)malloc(sizeof(scored_t) * (size_t)N);
    scored3_t *rest = (scored3_t *)malloc(sizeof(scored3_t) * (size_t)Hkv * N);
    unsigned char *kept = (unsigned char *)malloc((size_t)Hkv * N);
    for (int b = 0; b < B; ++b) {
        const int len = seq_len_of(seq_lens, b, N);
        memset(kept, 0, (size_t)Hkv * N);
        for (int g = 0; g < Hkv; ++g) {                       /* the safeguard: each head's own top n_safe */
            const float *s = scores + ((size_t)b * Hkv + g) * N;
            for (int p = 0; p < len; ++p) { tmp[p].s = s[p]; tmp[p].p = p; }
            qsort(tmp, (size_t)len, sizeof(scored_t), cmp_scored);
            for (int j = 0; j < n_safe; ++j) kept[(size_t)g * N + tmp[j].p] = 1;
        }
        size_t m = 0;                                          /* everything else competes globally */
        for (int g = 0; g < Hkv; ++g)
            for (int p = 0; p < len; ++p)
                if (!kept[(size_t)g * N + p]) {
                    rest[m].s = scores[((size_t)b * Hkv + g) * N + p];
                    rest[m].g = g;
                    rest[m].p = p;
                    ++m;
                }
        qsort(rest, m, sizeof(scored3_t), cmp_scored3);
        const size_t extra = (size_t)Hkv * (size_t)(budget - n_safe);
        for (size_t j = 0; j < extra; ++j) kept[(size_t)rest[j].g * N + rest[j].p] = 1;
        for (int g = 0; g < Hkv; ++g) {
            int32_t *out = keep_idx + ((size_t)b * Hkv + g) * cap;
            int n = 0;
            for (int p = 0; p < len; ++p)
                if (kept[(size_t)g * N + p]) out[n++] = p;
            counts[(size_t)b * Hkv + g] = n;
            for (int j = n; j < cap; ++j) out[j] = -1;
        }
    }
    free(tmp); free(rest); free(kept);
    return OBC_ORACLE_OK;
}

/*
 * Row gather (Algorithm 2 without the recent-window tail):
 *   k_out[b,g,j,:] = k[b,g,keep_idx[b,g,j],:], same for v.  Rows are
 *   row_bytes = d * element size bytes long.  An index of -1 (the padding of the
 *   ragged lists of obc_oracle_select_adaptive) gives an all-zero row.
 */
int obc_oracle_compact(const void *k, const void *v, const int32_t *keep_idx,
                       int B, int Hkv, int N, int budget, size_t row_bytes,
                       void *k_out, void *v_out)
{
    if (B < 1 || Hkv < 1 || N < 1 || budget < 1 || row_bytes < 1) return OBC_ORACLE_EINVAL;
    for (int bg = 0; bg < B * Hkv; ++bg)
        for (int j = 0; j < budget; ++j) {
            int32_t p = keep_idx[(size_t)bg * budget + j];
            if (p >= N) return OBC_ORACLE_EINVAL;
            size_t dst = ((size_t)bg * budget + j) * row_bytes;
            if (p < 0) {                                   /* padding of a ragged index list: an all-zero row */
                memset((char *)k_out + dst, 0, row_bytes);
                memset((char *)v_out + dst, 0, row_bytes);
                continue;
            }
            size_t src = ((size_t)bg * N + p) * row_bytes;
            memcpy((char *)k_out + dst, (const char *)k + src, row_bytes);
            memcpy((char *)v_out + dst, (const char *)v + src, row_bytes);
        }
    return OBC_ORACLE_OK;
}

/*
 * fp64 CPU oracle for causal self-attention over packed variable-length
 * sequences, forward and analytic backward.
 *
 * THIS IS TEST INFRASTRUCTURE.  It defines what the GPU library must compute
 * and is called only by the tests, by the smoke check and by the benchmark's
 * cpu_baseline leg.  It shares no code with the GPU path and the product never
 * falls back to it.
 *
 * What it follows.  The paper names the operators AttentionFwd / AttentionBwd
 * (Appendix "Implementation Details", subsection "Execution": forward and
 * backward executable subgraphs) and refers to the standard attention of
 * Vaswani et al. (Section 2.1, "Sharding and Communication in Training");
 * it never writes the formula.  The model is a causal Llama LM without
 * dropout (Appendix "Training Convergence", model configuration table), the
 * inputs are packed mixed-length sequences whose shapes are only known at run
 * time (Section 6.3 "Execution"; Evaluations, scenario (c)).  So the oracle is
 * the textbook definition, written out row by row, no tiling, no online
 * softmax, no reordering:
 *
 *   for each sequence i (tokens t0 .. t0+L-1), local query head h, kv head
 *   g = h / (Hq/Hkv), query row r and key j <= r (j > r has weight exactly 0):
 *
 *     S_rj  = scale * <q_r, k_j>
 *     m_r   = max_j S_rj            Z_r = sum_j exp(S_rj - m_r)
 *     P_rj  = exp(S_rj - m_r) / Z_r
 *     O_r   = sum_j P_rj v_j        LSE_r = m_r + ln Z_r
 *
 *     dP_rj = <dO_r, v_j>           D_r = sum_j P_rj dP_rj
 *     dS_rj = P_rj (dP_rj - D_r)
 *     dQ_r  = scale * sum_{j<=r} dS_rj k_j
 *     dK_j  = scale * sum_{h in group g} sum_{r>=j} dS_rj q_r
 *     dV_j  =         sum_{h in group g} sum_{r>=j} P_rj  dO_r
 *
 * Readings where the paper is silent: scale is an argument (callers pass
 * 1/sqrt(d)); sequences in a pack never attend to each other; the diagonal
 * j == r is visible; grouped KV heads are contiguous groups of query heads.
 *
 * Layout: q, o, d_o, dq are [T, Hq, d]; k, v, dk, dv are [T, Hkv, d]; all
 * contiguous doubles, token-major.  lse is [Hq, T].  cu[B+1] are the packed
 * sequence offsets (cu[0] = 0, cu[B] = T).
 *
 * oracle_attn_rows / oracle_attn_keys evaluate the same per-row and per-key
 * routines for sampled (token, head) pairs only, so that single outputs of packs
 * too large for a full evaluation can be checked; they are pinned by equality
 * with the full functions.
 *
 * Pins (tests/test_oracle_pins.py): closed forms for Q = 0, length-1
 * sequences, softmax row sums, shift invariance, packed == unpacked,
 * permutation of sequences, GQA == repeated-KV MHA, central finite
 * differences, and an independent dense-matrix evaluation with a library
 * softmax and reverse-mode autodiff.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_BAD_ARG 1
#define ORACLE_NO_MEM 2

static int check_args(const int32_t *cu, int32_t B, int32_t Hq, int32_t Hkv, int32_t d) {
    if (!cu || B < 0 || Hq <= 0 || Hkv <= 0 || d <= 0) return ORACLE_BAD_ARG;
    if (Hq % Hkv != 0) return ORACLE_BAD_ARG;
    if (cu[0] != 0) return ORACLE_BAD_ARG;
    for (int32_t i = 0; i < B; ++i)
        if (cu[i + 1] < cu[i]) return ORACLE_BAD_ARG;
    return ORACLE_OK;
}

static double dot(const double *a, const double *b, int32_t d) {
    double s = 0.0;
    for (int32_t c = 0; c < d; ++c) s += a[c] * b[c];
    return s;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int thread_index(void) {
#ifdef _OPENMP
    return omp_get_thread_num();
#else
    return 0;
#endif
}

/* Scores of one query row against its visible keys: s[j] = scale <q_r, k_j>, j = 0..r.
 * Returns the row maximum. */
static double score_row(const double *q_row, const double *k, int64_t k_tok_stride,
                        int64_t t0, int32_t r, int32_t d, double scale, double *s) {
    double m = -INFINITY;
    for (int32_t j = 0; j <= r; ++j) {
        s[j] = scale * dot(q_row, k + (t0 + j) * k_tok_stride, d);
        if (s[j] > m) m = s[j];
    }
    return m;
}

/* One query row, forward: p[0..r] receives P_rj, o_row (may be NULL) receives O_r.
 * kh / vh point at the row's kv head in token 0.  Returns LSE_r. */
static double row_forward(const double *q_row, const double *kh, const double *vh, int64_t ks,
                          int64_t t0, int32_t r, int32_t d, double scale, double *p, double *o_row) {
    const double m = score_row(q_row, kh, ks, t0, r, d, scale, p);
    double Z = 0.0;
    for (int32_t j = 0; j <= r; ++j) {
        p[j] = exp(p[j] - m);
        Z += p[j];
    }
    for (int32_t j = 0; j <= r; ++j) p[j] /= Z;
    if (o_row) {
        for (int32_t c = 0; c < d; ++c) o_row[c] = 0.0;
        for (int32_t j = 0; j <= r; ++j) {
            const double *v_row = vh + (t0 + j) * ks;
            for (int32_t c = 0; c < d; ++c) o_row[c] += p[j] * v_row[c];
        }
    }
    return m + log(Z);
}

/* One query row, backward, given its P row: dp[0..r] is scratch; dq_row (may be NULL)
 * receives dQ_r.  Returns D_r = sum_j P_rj dP_rj. */
static double row_backward(const double *do_row, const double *kh, const double *vh, int64_t ks,
                           int64_t t0, int32_t r, int32_t d, double scale, const double *p,
                           double *dp, double *dq_row) {
    double Dsum = 0.0;
    for (int32_t j = 0; j <= r; ++j) {
        dp[j] = dot(do_row, vh + (t0 + j) * ks, d);
        Dsum += p[j] * dp[j];
    }
    if (dq_row) {
        for (int32_t c = 0; c < d; ++c) dq_row[c] = 0.0;
        for (int32_t j = 0; j <= r; ++j) {
            const double ds = p[j] * (dp[j] - Dsum);
            const double *k_row = kh + (t0 + j) * ks;
            for (int32_t c = 0; c < d; ++c) dq_row[c] += ds * k_row[c];
        }
        for (int32_t c = 0; c < d; ++c) dq_row[c] *= scale;
    }
    return Dsum;
}

/* One key j of kv head g, backward: sums over the group's query heads and the rows r >= j.
 * lse / Dr are indexed [head_in_group * stat_stride + (r - stat_row0)]. */
static void key_backward(const double *q, const double *d_o, const double *k_row, const double *v_row,
                         int64_t qs, int64_t t0, int32_t L, int32_t j, int32_t g, int32_t G, int32_t d,
                         double scale, const double *lse, const double *Dr, int64_t stat_stride,
                         int32_t stat_row0, double *dk_row, double *dv_row) {
    for (int32_t c = 0; c < d; ++c) { dk_row[c] = 0.0; dv_row[c] = 0.0; }
    for (int32_t hg = 0; hg < G; ++hg) {
        const int32_t h = g * G + hg;
        for (int32_t r = j; r < L; ++r) {
            const double *q_row = q + (t0 + r) * qs + (int64_t)h * d;
            const double *do_row = d_o + (t0 + r) * qs + (int64_t)h * d;
            const int64_t st = (int64_t)hg * stat_stride + (r - stat_row0);
            const double p = exp(scale * dot(q_row, k_row, d) - lse[st]);
            const double ds = p * (dot(do_row, v_row, d) - Dr[st]);
            for (int32_t c = 0; c < d; ++c) {
                dv_row[c] += p * do_row[c];
                dk_row[c] += ds * q_row[c];
            }
        }
    }
    for (int32_t c = 0; c < d; ++c) dk_row[c] *= scale;
}

static int32_t longest(const int32_t *cu, int32_t B) {
    int32_t max_len = 0;
    for (int32_t i = 0; i < B; ++i)
        if (cu[i + 1] - cu[i] > max_len) max_len = cu[i + 1] - cu[i];
    return max_len > 0 ? max_len : 1;
}

/* Forward.  o [T,Hq,d], lse [Hq,T].  probs (may be NULL): only legal with B == 1;
 * receives P for every head as [Hq, L, L] (entries above the diagonal are 0). */
int oracle_attn_fwd(const double *q, const double *k, const double *v, const int32_t *cu,
                    int32_t B, int32_t Hq, int32_t Hkv, int32_t d, double scale,
                    double *o, double *lse, double *probs) {
    int rc = check_args(cu, B, Hq, Hkv, d);
    if (rc) return rc;
    if (!q || !k || !v || !o || !lse) return ORACLE_BAD_ARG;
    if (probs && B != 1) return ORACLE_BAD_ARG;
    const int64_t T = cu[B];
    const int32_t G = Hq / Hkv;
    const int64_t qs = (int64_t)Hq * d, ks = (int64_t)Hkv * d;
    const size_t row_len = (size_t)longest(cu, B);
    double *scratch = (double *)malloc(sizeof(double) * row_len * (size_t)oracle_num_threads());
    if (!scratch) return ORACLE_NO_MEM;
#pragma omp parallel
    {
        double *p = scratch + row_len * (size_t)thread_index();
        for (int32_t i = 0; i < B; ++i) {
            const int64_t t0 = cu[i];
            const int32_t L = cu[i + 1] - cu[i];
            for (int32_t h = 0; h < Hq; ++h) {
                const double *kh = k + (int64_t)(h / G) * d;
                const double *vh = v + (int64_t)(h / G) * d;
#pragma omp for schedule(dynamic, 4) nowait
                for (int32_t r = 0; r < L; ++r) {
                    const double *q_row = q + (t0 + r) * qs + (int64_t)h * d;
                    double *o_row = o + (t0 + r) * qs + (int64_t)h * d;
                    lse[(int64_t)h * T + t0 + r] = row_forward(q_row, kh, vh, ks, t0, r, d, scale, p, o_row);
                    if (probs) {
                        double *dst = probs + ((int64_t)h * L + r) * L;
                        for (int32_t j = 0; j < L; ++j) dst[j] = j <= r ? p[j] : 0.0;
                    }
                }
            }
        }
    }
    free(scratch);
    return ORACLE_OK;
}

/* Backward.  Recomputes the forward quantities it needs from q, k, v (it does not
 * take O or LSE from the caller).  dq [T,Hq,d]; dk, dv [T,Hkv,d]. */
int oracle_attn_bwd(const double *q, const double *k, const double *v, const double *d_o,
                    const int32_t *cu, int32_t B, int32_t Hq, int32_t Hkv, int32_t d,
                    double scale, double *dq, double *dk, double *dv) {
    int rc = check_args(cu, B, Hq, Hkv, d);
    if (rc) return rc;
    if (!q || !k || !v || !d_o || !dq || !dk || !dv) return ORACLE_BAD_ARG;
    const int64_t T = cu[B];
    const int32_t G = Hq / Hkv;
    const int64_t qs = (int64_t)Hq * d, ks = (int64_t)Hkv * d;
    if (T == 0) return ORACLE_OK;
    /* per (head, token): LSE_r and D_r, kept for the key-major pass */
    double *lse = (double *)malloc(sizeof(double) * (size_t)Hq * (size_t)T);
    double *Dr = (double *)malloc(sizeof(double) * (size_t)Hq * (size_t)T);
    const size_t row_len = (size_t)longest(cu, B);
    double *scratch = (double *)malloc(sizeof(double) * 2 * row_len * (size_t)oracle_num_threads());
    if (!lse || !Dr || !scratch) { free(lse); free(Dr); free(scratch); return ORACLE_NO_MEM; }
#pragma omp parallel
    {
        double *p = scratch + 2 * row_len * (size_t)thread_index();
        double *dp = p + row_len;
        /* pass 1, query-major: P row, dP row, D, dS row, dQ row */
        for (int32_t i = 0; i < B; ++i) {
            const int64_t t0 = cu[i];
            const int32_t L = cu[i + 1] - cu[i];
            for (int32_t h = 0; h < Hq; ++h) {
                const double *kh = k + (int64_t)(h / G) * d;
                const double *vh = v + (int64_t)(h / G) * d;
#pragma omp for schedule(dynamic, 4) nowait
                for (int32_t r = 0; r < L; ++r) {
                    const double *q_row = q + (t0 + r) * qs + (int64_t)h * d;
                    const double *do_row = d_o + (t0 + r) * qs + (int64_t)h * d;
                    double *dq_row = dq + (t0 + r) * qs + (int64_t)h * d;
                    lse[(int64_t)h * T + t0 + r] = row_forward(q_row, kh, vh, ks, t0, r, d, scale, p, NULL);
                    Dr[(int64_t)h * T + t0 + r] = row_backward(do_row, kh, vh, ks, t0, r, d, scale, p, dp, dq_row);
                }
            }
        }
#pragma omp barrier
        /* pass 2, key-major: dK_j, dV_j summed over the rows r >= j and the group's heads */
        for (int32_t i = 0; i < B; ++i) {
            const int64_t t0 = cu[i];
            const int32_t L = cu[i + 1] - cu[i];
            for (int32_t g = 0; g < Hkv; ++g) {
#pragma omp for schedule(dynamic, 4) nowait
                for (int32_t j = 0; j < L; ++j) {
                    const int64_t kv = (t0 + j) * ks + (int64_t)g * d;
                    key_backward(q, d_o, k + kv, v + kv, qs, t0, L, j, g, G, d, scale,
                                 lse + (int64_t)g * G * T + t0, Dr + (int64_t)g * G * T + t0, T, 0,
                                 dk + kv, dv + kv);
                }
            }
        }
    }
    free(scratch);
    free(lse);
    free(Dr);
    return ORACLE_OK;
}

/* Sampled rows: for n (token, q head) pairs, O_r [n,d], LSE_r [n] and dQ_r [n,d].
 * Same per-row routines as the full functions; cost O(r d) per sample. */
int oracle_attn_rows(const double *q, const double *k, const double *v, const double *d_o,
                     const int32_t *cu, int32_t B, int32_t Hq, int32_t Hkv, int32_t d, double scale,
                     int32_t n, const int32_t *tokens, const int32_t *heads,
                     double *o_rows, double *lse_rows, double *dq_rows) {
    int rc = check_args(cu, B, Hq, Hkv, d);
    if (rc) return rc;
    if (!q || !k || !v || !d_o || n < 0 || (n > 0 && (!tokens || !heads || !o_rows || !lse_rows || !dq_rows)))
        return ORACLE_BAD_ARG;
    const int32_t G = Hq / Hkv;
    const int64_t qs = (int64_t)Hq * d, ks = (int64_t)Hkv * d;
    for (int32_t x = 0; x < n; ++x)
        if (tokens[x] < 0 || tokens[x] >= cu[B] || heads[x] < 0 || heads[x] >= Hq) return ORACLE_BAD_ARG;
    const size_t row_len = (size_t)longest(cu, B);
    double *scratch = (double *)malloc(sizeof(double) * 2 * row_len * (size_t)oracle_num_threads());
    if (!scratch) return ORACLE_NO_MEM;
#pragma omp parallel
    {
        double *p = scratch + 2 * row_len * (size_t)thread_index();
        double *dp = p + row_len;
#pragma omp for schedule(dynamic, 1)
        for (int32_t x = 0; x < n; ++x) {
            int32_t i = 0;
            while (cu[i + 1] <= tokens[x]) ++i;   /* the sequence that holds this token */
            const int64_t t0 = cu[i];
            const int32_t r = tokens[x] - cu[i], h = heads[x];
            const double *kh = k + (int64_t)(h / G) * d;
            const double *vh = v + (int64_t)(h / G) * d;
            const double *q_row = q + (t0 + r) * qs + (int64_t)h * d;
            const double *do_row = d_o + (t0 + r) * qs + (int64_t)h * d;
            lse_rows[x] = row_forward(q_row, kh, vh, ks, t0, r, d, scale, p, o_rows + (int64_t)x * d);
            row_backward(do_row, kh, vh, ks, t0, r, d, scale, p, dp, dq_rows + (int64_t)x * d);
        }
    }
    free(scratch);
    return ORACLE_OK;
}

/* Sampled keys: for n (token, kv head) pairs, dK_j [n,d] and dV_j [n,d].  LSE_r and D_r of
 * the rows r >= j are evaluated row by row first; samples that share a (sequence, kv head) share
 * that evaluation (from the smallest sampled j on): cost O((L - j_min) L d G) per such group
 * plus O((L - j) d G) per sample. */
int oracle_attn_keys(const double *q, const double *k, const double *v, const double *d_o,
                     const int32_t *cu, int32_t B, int32_t Hq, int32_t Hkv, int32_t d, double scale,
                     int32_t n, const int32_t *tokens, const int32_t *kv_heads,
                     double *dk_rows, double *dv_rows) {
    int rc = check_args(cu, B, Hq, Hkv, d);
    if (rc) return rc;
    if (!q || !k || !v || !d_o || n < 0 || (n > 0 && (!tokens || !kv_heads || !dk_rows || !dv_rows)))
        return ORACLE_BAD_ARG;
    const int32_t G = Hq / Hkv;
    const int64_t qs = (int64_t)Hq * d, ks = (int64_t)Hkv * d;
    for (int32_t x = 0; x < n; ++x)
        if (tokens[x] < 0 || tokens[x] >= cu[B] || kv_heads[x] < 0 || kv_heads[x] >= Hkv) return ORACLE_BAD_ARG;
    const size_t row_len = (size_t)longest(cu, B);
    double *scratch = (double *)malloc(sizeof(double) * 2 * row_len * (size_t)oracle_num_threads());
    double *lse = (double *)malloc(sizeof(double) * row_len * (size_t)G);
    double *Dr = (double *)malloc(sizeof(double) * row_len * (size_t)G);
    int32_t *seq_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    char *done = (char *)calloc((size_t)(n > 0 ? n : 1), 1);
    if (!scratch || !lse || !Dr || !seq_of || !done) {
        free(scratch); free(lse); free(Dr); free(seq_of); free(done);
        return ORACLE_NO_MEM;
    }
    for (int32_t x = 0; x < n; ++x) {
        int32_t i = 0;
        while (cu[i + 1] <= tokens[x]) ++i;   /* the sequence that holds this token */
        seq_of[x] = i;
    }
    for (int32_t x = 0; x < n; ++x) {
        if (done[x]) continue;
        /* the group of samples with this sample's sequence and kv head, and its first key */
        const int32_t i = seq_of[x], g = kv_heads[x];
        const int64_t t0 = cu[i];
        const int32_t L = cu[i + 1] - cu[i];
        int32_t j_min = tokens[x] - cu[i];
        for (int32_t y = x + 1; y < n; ++y)
            if (seq_of[y] == i && kv_heads[y] == g && tokens[y] - cu[i] < j_min) j_min = tokens[y] - cu[i];
        const double *kh = k + (int64_t)g * d;
        const double *vh = v + (int64_t)g * d;
#pragma omp parallel
        {
            double *p = scratch + 2 * row_len * (size_t)thread_index();
            double *dp = p + row_len;
            for (int32_t hg = 0; hg < G; ++hg) {
                const int32_t h = g * G + hg;
#pragma omp for schedule(dynamic, 4) nowait
                for (int32_t r = j_min; r < L; ++r) {
                    const double *q_row = q + (t0 + r) * qs + (int64_t)h * d;
                    const double *do_row = d_o + (t0 + r) * qs + (int64_t)h * d;
                    lse[(int64_t)hg * row_len + (r - j_min)] = row_forward(q_row, kh, vh, ks, t0, r, d, scale, p, NULL);
                    Dr[(int64_t)hg * row_len + (r - j_min)] = row_backward(do_row, kh, vh, ks, t0, r, d, scale, p, dp, NULL);
                }
            }
        }
#pragma omp parallel for schedule(dynamic, 1)
        for (int32_t y = x; y < n; ++y) {
            if (seq_of[y] != i || kv_heads[y] != g) continue;
            const int32_t j = tokens[y] - cu[i];
            const int64_t kv = (t0 + j) * ks + (int64_t)g * d;
            key_backward(q, d_o, k + kv, v + kv, qs, t0, L, j, g, G, d, scale, lse, Dr, (int64_t)row_len, j_min,
                         dk_rows + (int64_t)y * d, dv_rows + (int64_t)y * d);
            done[y] = 1;
        }
    }
    free(scratch);
    free(lse);
    free(Dr);
    free(seq_of);
    free(done);
    return ORACLE_OK;
}

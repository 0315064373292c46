/*
 * vs_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow CPU implementation in fp64 of what the VideoScan streaming
 * attention path computes.  Only tests, the smoke check and the CPU-baseline
 * leg of the benchmark may call it; the GPU library never does and the two
 * share no code, headers, tables or helpers.
 *
 * What it follows (VideoScan paper):
 *   - Section 3.1, Eq. 1: Y = Softmax(Q K^T / sqrt(d_k)) V, evaluated here as
 *     the textbook two-pass softmax, one (head, query row) at a time.
 *   - Section 3.2: the semantic carrier is the LAST token of its frame's run
 *     and its K/V is what stays in the cache.
 *   - Section 3.3, prefilling phase: C^t = (1/N) sum_i E^t_i (mean pool);
 *     the frame's tokens are run through the decoder once.
 *   - Section 3.3, decoding phase: visual tokens are discarded afterwards;
 *     decoding reads the retained carrier K/V only.
 *   - Section 3.3, memory mechanism: a bank of at most M carriers; at
 *     capacity the older carrier of the most similar adjacent pair is dropped.
 *   - Section 3.4, semantic-aware mask: in a run of several frames a token
 *     reaches earlier frames only through their carriers.
 *
 * Readings where the paper is silent (all listed in the design notes):
 *   - every token of the frame run sees all retained cache rows; inside the
 *     run the mask is ordinary causal, diagonal included;
 *   - grouped-query attention: query head h reads KV head h / (Hq / Hkv);
 *   - decode appends the new token's K/V first, then attends over all rows
 *     including the new one;
 *   - cache rows are [prefix | carriers in arrival order], append-only.
 *
 * No tiling, no online softmax, no split along keys, no reordering: loops are
 * written in the order of the definition so they can be checked by eye.
 * All tensors are row-major doubles: Q [Tq][Hq][D], K/V [rows][Hkv][D].
 *
 * Every function here is pinned by tests/test_oracle_pins.py (closed forms,
 * invariants, hand-derived fixtures, brute force); none is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define VSO_OK 0
#define VSO_ERR_ARG 1
#define VSO_ERR_CAPACITY 2
#define VSO_ERR_NOMEM 3

int vs_oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Eq. 1 with a per-row visible prefix: query row i of every head sees key rows
 * 0 .. vis[i]-1 of Kall/Vall (1 <= vis[i] <= R).  If P is not NULL it receives
 * the probabilities, [Hq][Tq][R], zero outside the visible prefix.
 */
int vs_oracle_attention(const double *Q, int64_t Tq, int32_t Hq, int32_t Hkv, int32_t D,
                        const double *Kall, const double *Vall, int64_t R,
                        const int64_t *vis, double scale, double *O, double *P) {
    if (!Q || !Kall || !Vall || !vis || !O) return VSO_ERR_ARG;
    if (Tq < 0 || Hq < 1 || Hkv < 1 || D < 1 || R < 1 || Hq % Hkv != 0) return VSO_ERR_ARG;
    for (int64_t i = 0; i < Tq; ++i)
        if (vis[i] < 1 || vis[i] > R) return VSO_ERR_ARG;
    const int32_t G = Hq / Hkv;
    int failed = 0;

#pragma omp parallel
    {
        double *z = (double *)malloc((size_t)R * sizeof(double));
        if (!z) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for collapse(2) schedule(dynamic, 4)
            for (int32_t h = 0; h < Hq; ++h) {
                for (int64_t i = 0; i < Tq; ++i) {
                    const int32_t g = h / G;
                    const int64_t n = vis[i];
                    const double *q = Q + ((size_t)i * Hq + h) * D;
                    /* scores z_j = scale * <q, k_j> */
                    for (int64_t j = 0; j < n; ++j) {
                        const double *k = Kall + ((size_t)j * Hkv + g) * D;
                        double dot = 0.0;
                        for (int32_t d = 0; d < D; ++d) dot += q[d] * k[d];
                        z[j] = scale * dot;
                    }
                    /* softmax over the visible prefix, two passes */
                    double m = z[0];
                    for (int64_t j = 1; j < n; ++j)
                        if (z[j] > m) m = z[j];
                    double Z = 0.0;
                    for (int64_t j = 0; j < n; ++j) {
                        z[j] = exp(z[j] - m);
                        Z += z[j];
                    }
                    for (int64_t j = 0; j < n; ++j) z[j] /= Z;
                    /* weighted sum of value rows */
                    double *o = O + ((size_t)i * Hq + h) * D;
                    for (int32_t d = 0; d < D; ++d) o[d] = 0.0;
                    for (int64_t j = 0; j < n; ++j) {
                        const double *v = Vall + ((size_t)j * Hkv + g) * D;
                        const double p = z[j];
                        for (int32_t d = 0; d < D; ++d) o[d] += p * v[d];
                    }
                    if (P) {
                        double *prow = P + ((size_t)h * Tq + i) * R;
                        for (int64_t j = 0; j < n; ++j) prow[j] = z[j];
                        for (int64_t j = n; j < R; ++j) prow[j] = 0.0;
                    }
                }
            }
        }
        free(z);
    }
    return failed ? VSO_ERR_NOMEM : VSO_OK;
}

/*
 * Frame prefill (Section 3.3, prefilling phase; carrier last, Section 3.2).
 * Keys/values are the L retained cache rows followed by the T rows of the
 * frame run; frame row i sees the L cache rows and frame rows 0..i.
 */
int vs_oracle_frame_prefill(const double *Q, const double *Kc, const double *Vc, int64_t L,
                            const double *Kf, const double *Vf, int64_t T,
                            int32_t Hq, int32_t Hkv, int32_t D, double scale,
                            double *O, double *P) {
    if (L < 0 || T < 1 || !Kf || !Vf || (L > 0 && (!Kc || !Vc))) return VSO_ERR_ARG;
    if (Hkv < 1 || D < 1) return VSO_ERR_ARG;
    const size_t row = (size_t)Hkv * D;
    const int64_t R = L + T;
    double *Kall = (double *)malloc((size_t)R * row * sizeof(double));
    double *Vall = (double *)malloc((size_t)R * row * sizeof(double));
    int64_t *vis = (int64_t *)malloc((size_t)T * sizeof(int64_t));
    int rc = VSO_ERR_NOMEM;
    if (Kall && Vall && vis) {
        if (L > 0) {
            memcpy(Kall, Kc, (size_t)L * row * sizeof(double));
            memcpy(Vall, Vc, (size_t)L * row * sizeof(double));
        }
        memcpy(Kall + (size_t)L * row, Kf, (size_t)T * row * sizeof(double));
        memcpy(Vall + (size_t)L * row, Vf, (size_t)T * row * sizeof(double));
        for (int64_t i = 0; i < T; ++i) vis[i] = L + i + 1;
        rc = vs_oracle_attention(Q, T, Hq, Hkv, D, Kall, Vall, R, vis, scale, O, P);
    }
    free(Kall);
    free(Vall);
    free(vis);
    return rc;
}

/*
 * Carrier compaction (Sections 3.2 and 3.3): of the frame's T K/V rows only
 * row `carrier` (the last one in the method) is kept, written at cache row
 * *len; rows 0..*len-1 are untouched; *len grows by one.
 */
int vs_oracle_compact_append(double *Kc, double *Vc, int64_t capacity, int64_t *len,
                             const double *Kf, const double *Vf, int64_t T, int64_t carrier,
                             int32_t Hkv, int32_t D, int64_t *row_written) {
    if (!Kc || !Vc || !len || !Kf || !Vf) return VSO_ERR_ARG;
    if (T < 1 || carrier < 0 || carrier >= T || *len < 0 || *len > capacity) return VSO_ERR_ARG;
    if (*len == capacity) return VSO_ERR_CAPACITY;
    const size_t row = (size_t)Hkv * D;
    const int64_t at = *len;
    for (size_t e = 0; e < row; ++e) {
        Kc[(size_t)at * row + e] = Kf[(size_t)carrier * row + e];
        Vc[(size_t)at * row + e] = Vf[(size_t)carrier * row + e];
    }
    if (row_written) *row_written = at;
    *len = at + 1;
    return VSO_OK;
}

/*
 * Decode step for one stream (Section 3.3, decoding phase): the new token's
 * K/V (if given) is appended at row *len, then the single query attends over
 * every valid row, the new one included.
 */
int vs_oracle_decode(const double *q, double *Kc, double *Vc, int64_t capacity, int64_t *len,
                     const double *k_new, const double *v_new,
                     int32_t Hq, int32_t Hkv, int32_t D, double scale, double *o) {
    if (!q || !Kc || !Vc || !len || !o) return VSO_ERR_ARG;
    if ((k_new == NULL) != (v_new == NULL)) return VSO_ERR_ARG;
    if (*len < 0 || *len > capacity) return VSO_ERR_ARG;
    if (k_new) {
        if (*len == capacity) return VSO_ERR_CAPACITY;
        const size_t row = (size_t)Hkv * D;
        for (size_t e = 0; e < row; ++e) {
            Kc[(size_t)(*len) * row + e] = k_new[e];
            Vc[(size_t)(*len) * row + e] = v_new[e];
        }
        *len += 1;
    }
    if (*len < 1) return VSO_ERR_ARG;
    int64_t vis = *len;
    return vs_oracle_attention(q, 1, Hq, Hkv, D, Kc, Vc, *len, &vis, scale, o, NULL);
}

/*
 * Carrier embedding (Section 3.3): c[j] = (1/N) sum_{i<N} E[i][j], summed in
 * index order.
 */
int vs_oracle_mean_pool(const double *E, int64_t N, int64_t d, double *c) {
    if (!E || !c || N < 1 || d < 1) return VSO_ERR_ARG;
    for (int64_t j = 0; j < d; ++j) {
        double s = 0.0;
        for (int64_t i = 0; i < N; ++i) s += E[(size_t)i * d + j];
        c[j] = s / (double)N;
    }
    return VSO_OK;
}

/*
 * Memory bank with capacity M (Section 3.3, memory mechanism): the bank keeps
 * the embeddings of at most M semantic carriers, oldest first, together with
 * their K/V rows.  When a carrier arrives at a full bank, embeddings of
 * adjacent carriers are compared and the older one of the most similar pair
 * is dropped.  Reading taken here (the passage is ambiguous, see the design
 * notes): the sequence s_0 .. s_{M-1} (bank, oldest first), s_M (incoming) has
 * M adjacent pairs (i, i+1); the victim is the i with the largest cosine
 * cos(s_i, s_{i+1}); of equal cosines the smallest i.  policy 1 is the other
 * reading: the i < M with the largest cos(s_i, s_M).  A vector of norm 0 has
 * cosine 0 with everything.
 *
 * E [M][d] bank embeddings, e_new [d].  Writes the M cosines to cosines (may
 * be NULL) and the victim's index to *victim.
 */
int vs_oracle_bank_victim(const double *E, int64_t M, int64_t d, const double *e_new, int32_t policy,
                          double *cosines, int64_t *victim) {
    if (!E || !e_new || !victim || M < 1 || d < 1 || (policy != 0 && policy != 1)) return VSO_ERR_ARG;
    int64_t best = 0;
    double best_cos = 0.0;
    for (int64_t i = 0; i < M; ++i) {
        const double *a = E + (size_t)i * d;
        const double *b = (policy == 1 || i + 1 == M) ? e_new : E + (size_t)(i + 1) * d;
        double ab = 0.0, aa = 0.0, bb = 0.0;
        for (int64_t j = 0; j < d; ++j) {
            ab += a[j] * b[j];
            aa += a[j] * a[j];
            bb += b[j] * b[j];
        }
        const double c = (aa > 0.0 && bb > 0.0) ? ab / (sqrt(aa) * sqrt(bb)) : 0.0;
        if (cosines) cosines[i] = c;
        if (i == 0 || c > best_cos) {
            best = i;
            best_cos = c;
        }
    }
    *victim = best;
    return VSO_OK;
}

/*
 * One carrier arrives at the bank.  rows [capacity][width] is any of the
 * per-carrier tables kept in step with the bank (the embeddings, or one
 * layer's K or V rows behind `first` rows that are not carriers, e.g. a text
 * prefix); n = carriers held before the call (n <= M, first + M <= capacity).
 * With room left the new row is appended at first + n; with the bank full
 * (n == M) row first + victim is removed, the rows behind it move up by one
 * and the new row becomes the last.  Returns the count after the call in *n_out.
 */
int vs_oracle_bank_apply(double *rows, int64_t capacity, int64_t width, int64_t first, int64_t M, int64_t n,
                         int64_t victim, const double *row_new, int64_t *n_out) {
    if (!rows || !row_new || !n_out || width < 1 || first < 0 || M < 1 || n < 0 || n > M) return VSO_ERR_ARG;
    if (first + M > capacity) return VSO_ERR_CAPACITY;
    if (n < M) {
        memcpy(rows + (size_t)(first + n) * width, row_new, (size_t)width * sizeof(double));
        *n_out = n + 1;
        return VSO_OK;
    }
    if (victim < 0 || victim >= M) return VSO_ERR_ARG;
    for (int64_t r = victim; r + 1 < M; ++r)
        memcpy(rows + (size_t)(first + r) * width, rows + (size_t)(first + r + 1) * width, (size_t)width * sizeof(double));
    memcpy(rows + (size_t)(first + M - 1) * width, row_new, (size_t)width * sizeof(double));
    *n_out = M;
    return VSO_OK;
}

/*
 * Several frames in one run with the semantic-aware mask (Section 3.4: later
 * tokens reach earlier frames only through those frames' semantic carriers;
 * Section 3.2: the carrier is the last token of its frame).  The run holds F
 * frames of T tokens each.  Token i of frame a sees
 *   - the L retained cache rows,
 *   - the carriers (token T-1) of frames a' < a of this run,
 *   - tokens 0..i of its own frame,
 * and nothing else.  Q, O [F][T][Hq][D]; Kf, Vf [F][T][Hkv][D].  Written out as
 * the definition: for every (head, query) the visible keys are listed, scored,
 * soft-maxed in two passes and summed.
 */
int vs_oracle_frames_prefill(const double *Q, const double *Kc, const double *Vc, int64_t L,
                             const double *Kf, const double *Vf, int64_t F, int64_t T,
                             int32_t Hq, int32_t Hkv, int32_t D, double scale, double *O) {
    if (L < 0 || F < 1 || T < 1 || !Q || !Kf || !Vf || !O || (L > 0 && (!Kc || !Vc))) return VSO_ERR_ARG;
    if (Hq < 1 || Hkv < 1 || D < 1 || Hq % Hkv != 0) return VSO_ERR_ARG;
    const int32_t G = Hq / Hkv;
    const size_t row = (size_t)Hkv * D;
    const int64_t max_keys = L + F + T;
    int failed = 0;
#ifdef _OPENMP
#pragma omp parallel for collapse(2) schedule(dynamic)
#endif
    for (int64_t a = 0; a < F; ++a) {
        for (int32_t h = 0; h < Hq; ++h) {
            const int32_t g = h / G;
            const double **kp = (const double **)malloc((size_t)max_keys * sizeof(double *));
            const double **vp = (const double **)malloc((size_t)max_keys * sizeof(double *));
            double *z = (double *)malloc((size_t)max_keys * sizeof(double));
            if (!kp || !vp || !z) {
                failed = 1;
                free(kp); free(vp); free(z);
                continue;
            }
            for (int64_t i = 0; i < T; ++i) {
                int64_t n = 0;
                for (int64_t j = 0; j < L; ++j) {            /* retained rows */
                    kp[n] = Kc + (size_t)j * row + (size_t)g * D;
                    vp[n++] = Vc + (size_t)j * row + (size_t)g * D;
                }
                for (int64_t b = 0; b < a; ++b) {            /* carriers of earlier frames of the run */
                    kp[n] = Kf + ((size_t)b * T + (size_t)(T - 1)) * row + (size_t)g * D;
                    vp[n++] = Vf + ((size_t)b * T + (size_t)(T - 1)) * row + (size_t)g * D;
                }
                for (int64_t j = 0; j <= i; ++j) {           /* own frame, causal */
                    kp[n] = Kf + ((size_t)a * T + (size_t)j) * row + (size_t)g * D;
                    vp[n++] = Vf + ((size_t)a * T + (size_t)j) * row + (size_t)g * D;
                }
                const double *q = Q + (((size_t)a * T + (size_t)i) * Hq + (size_t)h) * D;
                double m = -INFINITY;
                for (int64_t k = 0; k < n; ++k) {
                    double s = 0.0;
                    for (int32_t d = 0; d < D; ++d) s += q[d] * kp[k][d];
                    z[k] = s * scale;
                    if (z[k] > m) m = z[k];
                }
                double Z = 0.0;
                for (int64_t k = 0; k < n; ++k) {
                    z[k] = exp(z[k] - m);
                    Z += z[k];
                }
                double *o = O + (((size_t)a * T + (size_t)i) * Hq + (size_t)h) * D;
                for (int32_t d = 0; d < D; ++d) o[d] = 0.0;
                for (int64_t k = 0; k < n; ++k) {
                    const double p = z[k] / Z;
                    for (int32_t d = 0; d < D; ++d) o[d] += p * vp[k][d];
                }
            }
            free(kp); free(vp); free(z);
        }
    }
    return failed ? VSO_ERR_NOMEM : VSO_OK;
}

/*
 * The question after the video (Section 3.3, decoding phase; mask of Section 3.4:
 * text reaches the frames only through the retained carrier rows).  The Tq
 * question tokens arrive in order; token j's K/V row is appended to the cache
 * at row *len + j, then its query attends over every row present, its own
 * included, and over nothing that comes later.  All Tq rows stay in the cache:
 * the answer is decoded on top of them.  Written out token by token, as the
 * sequence of events it is.  Q, O [Tq][Hq][D]; Kt, Vt [Tq][Hkv][D]; Kc, Vc
 * [capacity][Hkv][D] modified in place; *len grows by Tq.
 */
int vs_oracle_query_prefill(const double *Q, double *Kc, double *Vc, int64_t capacity, int64_t *len,
                            const double *Kt, const double *Vt, int64_t Tq,
                            int32_t Hq, int32_t Hkv, int32_t D, double scale, double *O) {
    if (!Q || !Kc || !Vc || !len || !Kt || !Vt || !O) return VSO_ERR_ARG;
    if (Tq < 1 || *len < 0 || *len > capacity) return VSO_ERR_ARG;
    if (*len + Tq > capacity) return VSO_ERR_CAPACITY;
    const size_t row = (size_t)Hkv * D;
    for (int64_t j = 0; j < Tq; ++j) {
        const int64_t at = *len;
        for (size_t e = 0; e < row; ++e) {
            Kc[(size_t)at * row + e] = Kt[(size_t)j * row + e];
            Vc[(size_t)at * row + e] = Vt[(size_t)j * row + e];
        }
        *len = at + 1;
        int64_t vis = *len;
        int rc = vs_oracle_attention(Q + (size_t)j * Hq * D, 1, Hq, Hkv, D, Kc, Vc, *len, &vis, scale,
                                     O + (size_t)j * Hq * D, NULL);
        if (rc != VSO_OK) return rc;
    }
    return VSO_OK;
}

/*
 * The frame's rows and their projections (Section 3.1: Q = X W_Q, K = X W_K,
 * V = X W_V; Section 3.3: the carrier's input embedding is the mean of the
 * frame's N token embeddings; Section 3.2: it is the frame's last token).
 * X has N + 1 rows: E[0..N-1], then C = (1/N) sum_i E[i].  W holds one row of d
 * weights per output feature (n_out of them: the caller stacks W_Q, W_K, W_V),
 * so Y[t][n] = sum_k X[t][k] W[n][k], summed in index order.  Y [N+1][n_out].
 */
int vs_oracle_frame_qkv(const double *E, int64_t N, int64_t d, const double *W, int64_t n_out, double *Y) {
    if (!E || !W || !Y || N < 1 || d < 1 || n_out < 1) return VSO_ERR_ARG;
    double *c = (double *)malloc((size_t)d * sizeof(double));
    if (!c) return VSO_ERR_NOMEM;
    int rc = vs_oracle_mean_pool(E, N, d, c);
    if (rc == VSO_OK) {
#ifdef _OPENMP
#pragma omp parallel for collapse(2) schedule(static)
#endif
        for (int64_t t = 0; t <= N; ++t) {
            for (int64_t n = 0; n < n_out; ++n) {
                const double *x = t < N ? E + (size_t)t * d : c;
                const double *w = W + (size_t)n * d;
                double s = 0.0;
                for (int64_t k = 0; k < d; ++k) s += x[k] * w[k];
                Y[(size_t)t * n_out + n] = s;
            }
        }
    }
    free(c);
    return rc;
}

/*
 * The decoder layer around the attention.  The paper fixes only the attention (Eq. 1) and the
 * projections Q = X W_Q, K = X W_K, V = X W_V (Section 3.1); for the rest it names the model it is
 * built on (Section 4.1), whose layer is the usual pre-norm one.  Readings taken (listed in the
 * design notes): RMS norm y_j = x_j g_j / sqrt(mean_k x_k^2 + eps); projections without bias; no
 * position encoding; a feed-forward gated by SiLU, silu(a) = a / (1 + exp(-a)); residual sums
 * around the attention block and around the feed-forward block.
 */

/* y[t][j] = x[t][j] * g[j] / sqrt((1/d) sum_k x[t][k]^2 + eps) */
int vs_oracle_rmsnorm(const double *X, int64_t T, int64_t d, const double *g, double eps, double *Y) {
    if (!X || !g || !Y || T < 1 || d < 1 || !(eps >= 0.0)) return VSO_ERR_ARG;
    for (int64_t t = 0; t < T; ++t) {
        double ss = 0.0;
        for (int64_t k = 0; k < d; ++k) ss += X[(size_t)t * d + k] * X[(size_t)t * d + k];
        const double r = sqrt(ss / (double)d + eps);
        for (int64_t j = 0; j < d; ++j) Y[(size_t)t * d + j] = X[(size_t)t * d + j] * g[j] / r;
    }
    return VSO_OK;
}

/* Y[t][n] = sum_k X[t][k] W[n][k]: one row of K weights per output feature, summed in index order */
int vs_oracle_linear(const double *X, int64_t T, int64_t K, const double *W, int64_t N, double *Y) {
    if (!X || !W || !Y || T < 1 || K < 1 || N < 1) return VSO_ERR_ARG;
#ifdef _OPENMP
#pragma omp parallel for collapse(2) schedule(static)
#endif
    for (int64_t t = 0; t < T; ++t) {
        for (int64_t n = 0; n < N; ++n) {
            double s = 0.0;
            for (int64_t k = 0; k < K; ++k) s += X[(size_t)t * K + k] * W[(size_t)n * K + k];
            Y[(size_t)t * N + n] = s;
        }
    }
    return VSO_OK;
}

/* Y[t][j] = silu(G[t][j]) * U[t][j] */
int vs_oracle_gated_unit(const double *G, const double *U, int64_t T, int64_t F, double *Y) {
    if (!G || !U || !Y || T < 1 || F < 1) return VSO_ERR_ARG;
    for (int64_t i = 0; i < T * F; ++i) Y[i] = G[i] / (1.0 + exp(-G[i])) * U[i];
    return VSO_OK;
}

/*
 * One layer for one frame run H [T][d] (the frame's N visual tokens, then its carrier):
 *   X1 = rmsnorm(H, g1);  Q = X1 Wq^T, K = X1 Wk^T, V = X1 Wv^T;
 *   A  = frame prefill attention of (Q, K, V) over the L retained rows (vs_oracle_frame_prefill);
 *   H1 = H + A Wo^T;  X2 = rmsnorm(H1, g2);  Hout = H1 + (silu(X2 Wg^T) * (X2 Wu^T)) Wd^T.
 * Wq [Hq D][d], Wk, Wv [Hkv D][d], Wo [d][Hq D], Wg, Wu [F][d], Wd [d][F].  Kf, Vf [T][Hkv][D]
 * receive the run's K and V rows (the caller keeps the last one, the carrier's, with
 * vs_oracle_compact_append).
 */
int vs_oracle_decoder_layer(const double *H, int64_t T, int64_t d, int32_t Hq, int32_t Hkv, int32_t D, int64_t F,
                            const double *g1, const double *Wq, const double *Wk, const double *Wv,
                            const double *Wo, const double *g2, const double *Wg, const double *Wu,
                            const double *Wd, double eps, const double *Kc, const double *Vc, int64_t L,
                            double scale, double *Kf, double *Vf, double *Hout) {
    if (!H || !g1 || !Wq || !Wk || !Wv || !Wo || !g2 || !Wg || !Wu || !Wd || !Kf || !Vf || !Hout) return VSO_ERR_ARG;
    if (T < 1 || d < 1 || Hq < 1 || Hkv < 1 || D < 1 || F < 1 || L < 0) return VSO_ERR_ARG;
    if (Hq % Hkv != 0 || (L > 0 && (!Kc || !Vc))) return VSO_ERR_ARG;  /* (before any weight is read) */
    const int64_t nq = (int64_t)Hq * D, nk = (int64_t)Hkv * D;
    double *x = (double *)malloc((size_t)T * d * sizeof(double));
    double *q = (double *)malloc((size_t)T * nq * sizeof(double));
    double *a = (double *)malloc((size_t)T * nq * sizeof(double));
    double *h1 = (double *)malloc((size_t)T * d * sizeof(double));
    double *gg = (double *)malloc((size_t)T * F * sizeof(double));
    double *uu = (double *)malloc((size_t)T * F * sizeof(double));
    double *o = (double *)malloc((size_t)T * d * sizeof(double));
    int rc = (x && q && a && h1 && gg && uu && o) ? VSO_OK : VSO_ERR_NOMEM;
    if (rc == VSO_OK) rc = vs_oracle_rmsnorm(H, T, d, g1, eps, x);
    if (rc == VSO_OK) rc = vs_oracle_linear(x, T, d, Wq, nq, q);
    if (rc == VSO_OK) rc = vs_oracle_linear(x, T, d, Wk, nk, Kf);
    if (rc == VSO_OK) rc = vs_oracle_linear(x, T, d, Wv, nk, Vf);
    if (rc == VSO_OK) rc = vs_oracle_frame_prefill(q, Kc, Vc, L, Kf, Vf, T, Hq, Hkv, D, scale, a, NULL);
    if (rc == VSO_OK) rc = vs_oracle_linear(a, T, nq, Wo, d, o);
    if (rc == VSO_OK) {
        for (int64_t i = 0; i < T * d; ++i) h1[i] = H[i] + o[i];
        rc = vs_oracle_rmsnorm(h1, T, d, g2, eps, x);
    }
    if (rc == VSO_OK) rc = vs_oracle_linear(x, T, d, Wg, F, gg);
    if (rc == VSO_OK) rc = vs_oracle_linear(x, T, d, Wu, F, uu);
    if (rc == VSO_OK) rc = vs_oracle_gated_unit(gg, uu, T, F, gg);
    if (rc == VSO_OK) rc = vs_oracle_linear(gg, T, F, Wd, d, o);
    if (rc == VSO_OK)
        for (int64_t i = 0; i < T * d; ++i) Hout[i] = h1[i] + o[i];
    free(x); free(q); free(a); free(h1); free(gg); free(uu); free(o);
    return rc;
}

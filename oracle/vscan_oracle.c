/*
 * CPU oracle for the two-stage visual token reduction of VScan.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU
 * library is checked against.  It shares no code, header, table or helper with
 * the HIP path, and nothing in the product path may call it.
 *
 * Everything is evaluated in fp64 on fp32 inputs (bf16 workloads pass values
 * that are already bf16-representable).  Each function follows one passage of
 * the paper, in the paper's order, with no blocking, fusion or reordering:
 *
 *   vso_encoder_scores  Sec. 4.1 "Global Scan", Eq. 1-2; last sentence of that
 *                       paragraph for encoders without a [CLS] token
 *   vso_select          Sec. 4.1 Eq. 2 (global), Eq. 3 (local windows) and the
 *                       footnote on local-before-global priority
 *   vso_assign          Sec. 4.1 "Token Merging": highest cosine similarity
 *   vso_merge           Sec. 4.1 Eq. 4
 *   vso_llm_scores      Sec. 4.2 Eq. 5
 *   vso_topk            Sec. 4.2 (keep the R2 % highest average text attention)
 *   vso_compact         Sec. 4.2 "Remarks on KV Cache": pruned tokens never
 *                       enter the cache, layout otherwise unchanged
 *
 * Readings taken where the paper is silent (all stated again next to the code):
 *   - scale is a parameter (callers pass 1/sqrt(head_dim));
 *   - softmax domain: visual keys only (as Eq. 1 / Eq. 5 are written), or all
 *     keys of the row with the visual slice taken afterwards;
 *   - thresholds tau / tau_w are realised as exact top-k counts;
 *   - ties go to the lowest index; outputs are in ascending index order;
 *   - a local budget that does not divide by the window count gives
 *     floor(kl / W) per window and the remainder to the global scan.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_pins.py
 * (closed forms, invariants, brute force on tiny inputs, an independent numpy
 * evaluation).  The paper prints no selected index, score or merged value, so
 * on realistic inputs the selected indices and merged values are "parity
 * unpinned" by the paper itself; only definitions and invariants pin them.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define VSO_OK 0
#define VSO_ERR_ARG (-1)
#define VSO_ERR_MEM (-2)

int vso_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* softmax of z[0..n) into p[0..n): p_j = exp(z_j - max z) / sum_j exp(z_j - max z) */
static void softmax_row(const double *z, int64_t n, double *p) {
    double m = z[0];
    for (int64_t j = 1; j < n; ++j)
        if (z[j] > m) m = z[j];
    double sum = 0.0;
    for (int64_t j = 0; j < n; ++j) {
        p[j] = exp(z[j] - m);
        sum += p[j];
    }
    for (int64_t j = 0; j < n; ++j) p[j] /= sum;
}

static double dot_f32(const float *a, const float *b, int64_t n) {
    double acc = 0.0;
    for (int64_t e = 0; e < n; ++e) acc += (double)a[e] * (double)b[e];
    return acc;
}

/*
 * Sec. 4.1, Eq. 1-2 and the no-[CLS] sentence after them.
 *
 * q, k: [B, C, H, S, dh] with S = N + has_cls; where has_cls the [CLS] token is
 * row 0.  scores: [B, C, N], one value per patch token.
 *
 * mode 0 ([CLS] row, Eq. 1):  per head h, z_j = scale * q_CLS . k_j over the key
 *   domain, p^h = softmax(z), score_j = (1/H) sum_h p^h_j   (Eq. 2's S^avg).
 * mode 1 (mean attention received): per head h and per patch query row i,
 *   A^h_i = softmax_j(scale * q_i . k_j) over the key domain,
 *   score_j = (1/(H N)) sum_h sum_i A^h_ij   (diagonal included, divisor N).
 * domain 0: keys are the patch tokens only (K_V in Eq. 1).
 * domain 1: keys are all S rows; the [CLS] column is dropped after the softmax.
 */
int vso_encoder_scores(const float *q, const float *k, int B, int C, int H, int S, int dh,
                       int has_cls, int mode, int domain, double scale, double *scores) {
    if (!q || !k || !scores) return VSO_ERR_ARG;
    if (B < 0 || C < 1 || H < 1 || S < 1 || dh < 1) return VSO_ERR_ARG;
    if (has_cls != 0 && has_cls != 1) return VSO_ERR_ARG;
    const int N = S - has_cls;
    if (N < 1) return VSO_ERR_ARG;
    if (mode == 0 && !has_cls) return VSO_ERR_ARG;
    if (mode != 0 && mode != 1) return VSO_ERR_ARG;
    if (domain != 0 && domain != 1) return VSO_ERR_ARG;
    const int first_key = (domain == 1) ? 0 : has_cls; /* first row of the key domain */
    const int n_keys = S - first_key;
    const int col0 = has_cls - first_key;              /* position of patch 0 in the domain */
    int status = VSO_OK;

    for (int64_t bc = 0; bc < (int64_t)B * C; ++bc) {
        double *out = scores + bc * N;
        for (int j = 0; j < N; ++j) out[j] = 0.0;
        for (int h = 0; h < H; ++h) {
            const float *qh = q + (bc * H + h) * (int64_t)S * dh;
            const float *kh = k + (bc * H + h) * (int64_t)S * dh;
            if (mode == 0) {
                double *z = (double *)malloc(sizeof(double) * 2 * n_keys);
                if (!z) return VSO_ERR_MEM;
                double *p = z + n_keys;
                for (int j = 0; j < n_keys; ++j)
                    z[j] = scale * dot_f32(qh, kh + (int64_t)(first_key + j) * dh, dh);
                softmax_row(z, n_keys, p);
                for (int j = 0; j < N; ++j) out[j] += p[col0 + j] / H;
                free(z);
            } else {
                const int nt = vso_threads();
                double *acc = (double *)calloc((size_t)nt * N, sizeof(double));
                double *zbuf = (double *)malloc(sizeof(double) * 2 * n_keys * (size_t)nt);
                if (!acc || !zbuf) {
                    free(acc);
                    free(zbuf);
                    return VSO_ERR_MEM;
                }
#pragma omp parallel num_threads(nt)
                {
#ifdef _OPENMP
                    const int tid = omp_get_thread_num();
#else
                    const int tid = 0;
#endif
                    double *z = zbuf + (size_t)tid * 2 * n_keys;
                    double *p = z + n_keys;
                    double *mine = acc + (size_t)tid * N;
#pragma omp for schedule(static)
                    for (int i = 0; i < N; ++i) {
                        const float *qi = qh + (int64_t)(has_cls + i) * dh;
                        for (int j = 0; j < n_keys; ++j)
                            z[j] = scale * dot_f32(qi, kh + (int64_t)(first_key + j) * dh, dh);
                        softmax_row(z, n_keys, p);
                        for (int j = 0; j < N; ++j) mine[j] += p[col0 + j];
                    }
                }
                free(zbuf);
                for (int t = 0; t < nt; ++t)
                    for (int j = 0; j < N; ++j) out[j] += acc[(size_t)t * N + j] / ((double)H * N);
                free(acc);
            }
        }
    }
    return status;
}

typedef struct {
    double score;
    int32_t idx;
} cand_t;

/* order: higher score first; equal scores: lower index first */
static int cand_cmp(const void *a, const void *b) {
    const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
    if (x->score > y->score) return -1;
    if (x->score < y->score) return 1;
    return (x->idx > y->idx) - (x->idx < y->idx);
}

/*
 * Sec. 4.1, Eq. 3 (local scan), Eq. 2 (global scan) and the footnote: local
 * tokens are chosen first and are excluded from the global selection.
 *
 * s_local, s_global: [B, C, N] scores (N = gh*gw, row-major grid); they may be
 * the same array.  Windows: wr x wc per segment; token (r, c) lies in window
 * (floor(r*wr/gh), floor(c*wc/gw)); each window keeps its kw = floor(kl / W)
 * best tokens by (score desc, index asc); then the kg + (kl - W*kw) best of the
 * remaining tokens of the segment are kept by the same order on s_global.
 * kept: [B, C*(kl+kg)], per image ascending, index = c*N + r*gw + col.
 */
int vso_select(const double *s_local, const double *s_global, int B, int C, int gh, int gw,
               int wr, int wc, int kl, int kg, int32_t *kept) {
    if (!s_local || !s_global || !kept) return VSO_ERR_ARG;
    if (B < 0 || C < 1 || gh < 1 || gw < 1 || wr < 1 || wc < 1 || kl < 0 || kg < 0)
        return VSO_ERR_ARG;
    if (wr > gh || wc > gw) return VSO_ERR_ARG;
    const int N = gh * gw, W = wr * wc;
    if (kl + kg > N) return VSO_ERR_ARG;
    const int kw = kl / W;
    const int kg_eff = kg + (kl - kw * W);
    cand_t *cand = (cand_t *)malloc(sizeof(cand_t) * N);
    char *taken = (char *)malloc(N);
    if (!cand || !taken) {
        free(cand);
        free(taken);
        return VSO_ERR_MEM;
    }
    int status = VSO_OK;
    for (int64_t bc = 0; bc < (int64_t)B * C && status == VSO_OK; ++bc) {
        const double *sl = s_local + bc * N, *sg = s_global + bc * N;
        memset(taken, 0, N);
        for (int w = 0; w < W; ++w) {
            const int wy = w / wc, wx = w % wc;
            int n = 0;
            for (int r = 0; r < gh; ++r)
                for (int c = 0; c < gw; ++c)
                    if ((int)(((int64_t)r * wr) / gh) == wy && (int)(((int64_t)c * wc) / gw) == wx) {
                        cand[n].score = sl[r * gw + c];
                        cand[n].idx = r * gw + c;
                        ++n;
                    }
            if (kw > n) {
                status = VSO_ERR_ARG;
                break;
            }
            qsort(cand, n, sizeof(cand_t), cand_cmp);
            for (int t = 0; t < kw; ++t) taken[cand[t].idx] = 1;
        }
        if (status != VSO_OK) break;
        int n = 0;
        for (int i = 0; i < N; ++i)
            if (!taken[i]) {
                cand[n].score = sg[i];
                cand[n].idx = i;
                ++n;
            }
        qsort(cand, n, sizeof(cand_t), cand_cmp);
        for (int t = 0; t < kg_eff; ++t) taken[cand[t].idx] = 1;
        const int b = (int)(bc / C), c = (int)(bc % C);
        int32_t *out = kept + (int64_t)b * C * (kl + kg) + (int64_t)c * (kl + kg);
        int m = 0;
        for (int i = 0; i < N; ++i)
            if (taken[i]) out[m++] = c * N + i;
        if (m != kl + kg) status = VSO_ERR_ARG;
    }
    free(cand);
    free(taken);
    return status;
}

#define VSO_NORM_EPS 1e-12

static double cosine_rows(const float *a, const float *b, int D) {
    double na = sqrt(dot_f32(a, a, D)), nb = sqrt(dot_f32(b, b, D));
    if (na < VSO_NORM_EPS) na = VSO_NORM_EPS;
    if (nb < VSO_NORM_EPS) nb = VSO_NORM_EPS;
    return dot_f32(a, b, D) / (na * nb);
}

/* cosine similarity of row u[i] and row s[i] of x (flat row indices), for tests
 * that need the oracle's value for one particular pair */
int vso_cos_pairs(const float *x, int D, int64_t n, const int64_t *u, const int64_t *s,
                  double *out) {
    if (!x || !u || !s || !out || D < 1) return VSO_ERR_ARG;
    for (int64_t i = 0; i < n; ++i) out[i] = cosine_rows(x + u[i] * D, x + s[i] * D, D);
    return VSO_OK;
}

/*
 * Sec. 4.1 "Token Merging", assignment step: every unselected token goes to the
 * selected token with the highest cosine similarity (first slot on equality).
 *
 * x: [B, T, D] token features (T tokens per image), kept: [B, K] ascending.
 * assign: [B, T] slot in 0..K-1; a selected token is given its own slot.
 */
int vso_assign(const float *x, const int32_t *kept, int B, int T, int D, int K, int32_t *assign) {
    if (!x || !kept || !assign) return VSO_ERR_ARG;
    if (B < 0 || T < 1 || D < 1 || K < 1 || K > T) return VSO_ERR_ARG;
    int status = VSO_OK;
#pragma omp parallel for schedule(dynamic, 16) collapse(2)
    for (int b = 0; b < B; ++b)
        for (int u = 0; u < T; ++u) {
            const float *xb = x + (int64_t)b * T * D;
            const int32_t *kb = kept + (int64_t)b * K;
            int own = -1;
            for (int s = 0; s < K; ++s)
                if (kb[s] == u) own = s;
            if (own >= 0) {
                assign[(int64_t)b * T + u] = own;
                continue;
            }
            int best = 0;
            double best_cos = 0.0;
            for (int s = 0; s < K; ++s) {
                if (kb[s] < 0 || kb[s] >= T) {
#pragma omp atomic write
                    status = VSO_ERR_ARG;
                    continue;
                }
                const double c = cosine_rows(xb + (int64_t)u * D, xb + (int64_t)kb[s] * D, D);
                if (s == 0 || c > best_cos) {
                    best = s;
                    best_cos = c;
                }
            }
            assign[(int64_t)b * T + u] = best;
        }
    return status;
}

/*
 * Sec. 4.1, Eq. 4: merged_s = (x_s + sum_{u in U_s} x_u) / (|U_s| + 1), where U_s
 * is the set of unselected tokens assigned to slot s.
 *
 * merged: [B, K, D] fp64; counts (optional): [B, K] = |U_s| + 1.
 */
int vso_merge(const float *x, const int32_t *kept, const int32_t *assign, int B, int T, int D,
              int K, double *merged, int32_t *counts) {
    if (!x || !kept || !assign || !merged) return VSO_ERR_ARG;
    if (B < 0 || T < 1 || D < 1 || K < 1 || K > T) return VSO_ERR_ARG;
    char *is_kept = (char *)malloc(T);
    if (!is_kept) return VSO_ERR_MEM;
    int status = VSO_OK;
    for (int b = 0; b < B && status == VSO_OK; ++b) {
        const float *xb = x + (int64_t)b * T * D;
        memset(is_kept, 0, T);
        for (int s = 0; s < K; ++s) {
            const int32_t t = kept[(int64_t)b * K + s];
            if (t < 0 || t >= T) {
                status = VSO_ERR_ARG;
                break;
            }
            is_kept[t] = 1;
        }
        if (status != VSO_OK) break;
        for (int s = 0; s < K; ++s) {
            double *m = merged + ((int64_t)b * K + s) * D;
            const float *xs = xb + (int64_t)kept[(int64_t)b * K + s] * D;
            for (int e = 0; e < D; ++e) m[e] = xs[e];
            int card = 0; /* |U_s| */
            for (int u = 0; u < T; ++u) {
                if (is_kept[u] || assign[(int64_t)b * T + u] != s) continue;
                const float *xu = xb + (int64_t)u * D;
                for (int e = 0; e < D; ++e) m[e] += xu[e];
                ++card;
            }
            for (int e = 0; e < D; ++e) m[e] /= (double)(card + 1);
            if (counts) counts[(int64_t)b * K + s] = card + 1;
        }
    }
    free(is_kept);
    return status;
}

/*
 * Sec. 4.2, Eq. 5, averaged over heads as the sentence after it says.
 *
 * q: [B, Hq, Tq, dh] queries of the last Tq positions of the sequence (the
 * paper uses the last instruction token only, Tq = 1); k: [B, Hkv, S, dh];
 * query head h reads kv head floor(h * Hkv / Hq).  scores: [B, V] over the
 * visual span [vis_start, vis_start + V).
 * domain 0: softmax over the visual keys only (K_V in Eq. 5).
 * domain 1: softmax over the causal row of query t, keys 0 .. S - Tq + t, with
 *           the visual slice taken afterwards.
 * score_j = (1 / (Tq Hq)) sum_t sum_h softmax(...)_j.
 */
int vso_llm_scores(const float *q, const float *k, int B, int Hq, int Hkv, int Tq, int S, int dh,
                   int vis_start, int V, int domain, double scale, double *scores) {
    if (!q || !k || !scores) return VSO_ERR_ARG;
    if (B < 0 || Hq < 1 || Hkv < 1 || Hq % Hkv || Tq < 1 || S < 1 || dh < 1) return VSO_ERR_ARG;
    if (vis_start < 0 || V < 1 || vis_start + V + Tq > S) return VSO_ERR_ARG;
    if (domain != 0 && domain != 1) return VSO_ERR_ARG;
    int status = VSO_OK;
#pragma omp parallel for schedule(static)
    for (int b = 0; b < B; ++b) {
        double *z = (double *)malloc(sizeof(double) * 2 * S);
        if (!z) {
#pragma omp atomic write
            status = VSO_ERR_MEM;
            continue;
        }
        double *p = z + S;
        double *out = scores + (int64_t)b * V;
        for (int j = 0; j < V; ++j) out[j] = 0.0;
        for (int t = 0; t < Tq; ++t)
            for (int h = 0; h < Hq; ++h) {
                const int g = (int)(((int64_t)h * Hkv) / Hq);
                const float *qv = q + (((int64_t)b * Hq + h) * Tq + t) * dh;
                const float *kg = k + ((int64_t)b * Hkv + g) * (int64_t)S * dh;
                const int first = domain ? 0 : vis_start;
                const int n = domain ? (S - Tq + t + 1) : V;
                for (int j = 0; j < n; ++j)
                    z[j] = scale * dot_f32(qv, kg + (int64_t)(first + j) * dh, dh);
                softmax_row(z, n, p);
                for (int j = 0; j < V; ++j) out[j] += p[vis_start - first + j] / ((double)Tq * Hq);
            }
        free(z);
    }
    return status;
}

/* Sec. 4.2: keep the `keep` highest-scoring of V tokens per row, (score desc,
 * index asc); kept: [B, keep] ascending, relative to the start of the span. */
int vso_topk(const double *scores, int B, int V, int keep, int32_t *kept) {
    if (!scores || !kept || B < 0 || V < 1 || keep < 0 || keep > V) return VSO_ERR_ARG;
    cand_t *cand = (cand_t *)malloc(sizeof(cand_t) * V);
    char *taken = (char *)malloc(V);
    if (!cand || !taken) {
        free(cand);
        free(taken);
        return VSO_ERR_MEM;
    }
    for (int b = 0; b < B; ++b) {
        for (int j = 0; j < V; ++j) {
            cand[j].score = scores[(int64_t)b * V + j];
            cand[j].idx = j;
        }
        qsort(cand, V, sizeof(cand_t), cand_cmp);
        memset(taken, 0, V);
        for (int t = 0; t < keep; ++t) taken[cand[t].idx] = 1;
        int m = 0;
        for (int j = 0; j < V; ++j)
            if (taken[j]) kept[(int64_t)b * keep + m++] = j;
    }
    free(cand);
    free(taken);
    return VSO_OK;
}

/*
 * Sec. 4.2 "Remarks on KV Cache": the pruned sequence is
 *   prefix rows [0, vis_start) ++ kept visual rows (original order) ++ rows after
 *   the visual span [vis_start + V, S),
 * applied to a tensor viewed as [B, G, S, Wd] (hidden states: G = 1; K or V:
 * G = kv heads).  out: [B, G, S_out, Wd], S_out = S - V + keep.  Pure copy.
 */
int vso_compact(const float *in, const int32_t *kept, int B, int G, int S, int Wd, int vis_start,
                int V, int keep, float *out) {
    if (!in || !kept || !out) return VSO_ERR_ARG;
    if (B < 0 || G < 1 || S < 1 || Wd < 1 || vis_start < 0 || V < 0 || vis_start + V > S)
        return VSO_ERR_ARG;
    if (keep < 0 || keep > V) return VSO_ERR_ARG;
    const int S_out = S - V + keep;
    for (int b = 0; b < B; ++b)
        for (int g = 0; g < G; ++g) {
            const float *src = in + ((int64_t)b * G + g) * (int64_t)S * Wd;
            float *dst = out + ((int64_t)b * G + g) * (int64_t)S_out * Wd;
            int p = 0;
            for (int r = 0; r < vis_start; ++r, ++p)
                memcpy(dst + (int64_t)p * Wd, src + (int64_t)r * Wd, sizeof(float) * Wd);
            for (int t = 0; t < keep; ++t, ++p) {
                const int32_t j = kept[(int64_t)b * keep + t];
                if (j < 0 || j >= V) return VSO_ERR_ARG;
                memcpy(dst + (int64_t)p * Wd, src + (int64_t)(vis_start + j) * Wd,
                       sizeof(float) * Wd);
            }
            for (int r = vis_start + V; r < S; ++r, ++p)
                memcpy(dst + (int64_t)p * Wd, src + (int64_t)r * Wd, sizeof(float) * Wd);
        }
    return VSO_OK;
}

/*
 * TRIM filter-then-refine scan: plain CPU oracle.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, obviously-correct statement of what the GPU library
 * must compute.  It shares no code with the HIP path and must never be linked
 * into, imported by, or called from the product; only the tests, the smoke
 * check and the benchmark's reported CPU baseline may run it.
 *
 * What it follows (paper: "TRIM", arXiv 2508.17828):
 *   - PQ codes and the distance table T          : Section 2.2 (PQ-based methods)
 *   - landmark = PQ reconstruction, Gamma(l,q)^2
 *     = sum_j T[j][code_j]                        : Section 3.1
 *   - strict bound f and p-relaxed bound g        : Definitions 1-2, Equation 3
 *   - preprocessing (store code and Gamma(l,x))   : Section 3.3
 *   - kNN / range scan with pruning               : Section 4.2
 *   - kNN and range problem statements            : Section 2.1
 *
 * Arithmetic.  The paper does not fix a precision.  Survivor decisions are
 * integers decided by floating point, so they are taken in the kernel's
 * precision, binary32, with every rounding written out (compile with
 * -ffp-contract=off; each fused multiply-add is an explicit fmaf):
 *   sub-vector distance : acc = fmaf(x_t - c_t, x_t - c_t, acc), t ascending, acc0 = 0
 *   table sum           : s = ((T[0][c0] + T[1][c1]) + T[2][c2]) + ...   (j ascending)
 *   bound (Equation 3)  : a = sqrtf(s); e = a - b; g = fmaf((2*gamma)*a, b, e*e)
 *   exact distance      : 32 partial sums; the group of 4 consecutive coordinates
 *                         number G goes, in order, into partial sum G mod 32 with
 *                         fmaf; then p[l] += p[l+h] for h = 16, 8, 4, 2, 1.
 * Pins for each function live in tests/ (float64 closed forms, brute force).
 *
 * Parity unpinned: none of the functions below.  (Recall / pruning *values* at
 * gamma > 0 on the paper's datasets cannot be pinned here: the datasets are absent.)
 */
#include <math.h>
#include <omp.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define TRIM_C 256 /* centroids per subspace; the paper's C (Section 6.1 parameter setting) */

/* ---- elementary pieces ---------------------------------------------------------- */

/* Squared distance of two short sub-vectors (Section 2.2: table entries; also the
 * assignment rule of PQ encoding). */
static float subvec_sqdist(const float *x, const float *c, int len) {
    float acc = 0.0f;
    for (int t = 0; t < len; ++t) {
        float diff = x[t] - c[t];
        acc = fmaf(diff, diff, acc);
    }
    return acc;
}

/* Exact squared Euclidean distance Gamma(q,x)^2 (Section 2.1), d % 4 == 0. */
float trim_oracle_exact_d2(const float *q, const float *x, int d) {
    float p[32];
    for (int l = 0; l < 32; ++l) p[l] = 0.0f;
    for (int g = 0; g < d / 4; ++g) {
        int l = g % 32;
        for (int c = 0; c < 4; ++c) {
            float diff = q[4 * g + c] - x[4 * g + c];
            p[l] = fmaf(diff, diff, p[l]);
        }
    }
    for (int h = 16; h >= 1; h >>= 1)
        for (int l = 0; l < h; ++l) p[l] = p[l] + p[l + h];
    return p[0];
}

/* Gamma(l,q)^2 = sum over subspaces of the table entry the code selects (Section 3.1). */
static float table_sum(const float *T, const uint8_t *code, int M) {
    float s = 0.0f;
    for (int j = 0; j < M; ++j) s = s + T[(size_t)j * TRIM_C + code[j]];
    return s;
}

/* p-relaxed lower bound g(x,q,l) of Equation 3 from s = Gamma(l,q)^2 and b = Gamma(l,x). */
float trim_oracle_plb_from_s(float s, float b, float gamma) {
    float two_gamma = 2.0f * gamma;
    float a = sqrtf(s);
    float e = a - b;
    float t = two_gamma * a;
    return fmaf(t, b, e * e);
}

float trim_oracle_plb(const float *T, const uint8_t *code, int M, float b, float gamma) {
    return trim_oracle_plb_from_s(table_sum(T, code, M), b, gamma);
}

/* ---- preprocessing (Section 3.3, step 1) ------------------------------------------ */

/* codes[x][j] = nearest centroid of subspace j (smallest index on ties);
 * dlx[x] = Gamma(l,x) = sqrt(sum_j of the winning squared distances), j ascending. */
void trim_oracle_encode(const float *base, int64_t n, int d, const float *codebooks,
                            int M, uint8_t *codes, float *dlx) {
    int dsub = d / M;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        float tot = 0.0f;
        for (int j = 0; j < M; ++j) {
            const float *xj = base + (size_t)i * d + (size_t)j * dsub;
            const float *cb = codebooks + (size_t)j * TRIM_C * dsub;
            float best = INFINITY;
            int arg = 0;
            for (int c = 0; c < TRIM_C; ++c) {
                float v = subvec_sqdist(xj, cb + (size_t)c * dsub, dsub);
                if (v < best) { best = v; arg = c; }
            }
            codes[(size_t)i * M + j] = (uint8_t)arg;
            tot = tot + best;
        }
        dlx[i] = sqrtf(tot);
    }
}

/* ---- query processing, operation 1: the distance table (Section 3.3; Section 2.2) -- */

/* lut[q][j][c] = || q_j - centroid_{j,c} ||^2 */
void trim_oracle_build_lut(const float *queries, int64_t nq, int d,
                               const float *codebooks, int M, float *lut) {
    int dsub = d / M;
#pragma omp parallel for schedule(static)
    for (int64_t q = 0; q < nq; ++q)
        for (int j = 0; j < M; ++j)
            for (int c = 0; c < TRIM_C; ++c)
                lut[((size_t)q * M + j) * TRIM_C + c] =
                    subvec_sqdist(queries + (size_t)q * d + (size_t)j * dsub,
                                  codebooks + ((size_t)j * TRIM_C + c) * dsub, dsub);
}

/* ---- candidate order ---------------------------------------------------------------- */

/* Candidates of one query, in scan order: the probed lists in the given order, storage
 * positions ascending inside a list; with no candidate structure, all n positions. */
typedef struct {
    int64_t *pos; /* storage position of the candidate with scan-order number idx */
    int64_t total;
} cand_t;

static cand_t cand_make(int64_t n, int nprobe, const int64_t *list_offsets,
                        const int32_t *probes_q) {
    cand_t c;
    c.total = 0;
    if (!list_offsets) {
        c.total = n;
    } else {
        for (int p = 0; p < nprobe; ++p)
            c.total += list_offsets[probes_q[p] + 1] - list_offsets[probes_q[p]];
    }
    c.pos = malloc(sizeof(int64_t) * (size_t)(c.total > 0 ? c.total : 1));
    int64_t w = 0;
    if (!list_offsets) {
        for (int64_t i = 0; i < n; ++i) c.pos[w++] = i;
    } else {
        for (int p = 0; p < nprobe; ++p)
            for (int64_t i = list_offsets[probes_q[p]]; i < list_offsets[probes_q[p] + 1]; ++i)
                c.pos[w++] = i;
    }
    return c;
}
static void cand_free(cand_t *c) { free(c->pos); }

/* ---- result set R: k smallest (d2, id), ascending (Section 4.2) ---------------------- */

typedef struct { float d2; int32_t id; } hit_t;

static int hit_less(hit_t a, hit_t b) { return a.d2 < b.d2 || (a.d2 == b.d2 && a.id < b.id); }

static void result_insert(hit_t *R, int *size, int k, hit_t h) {
    if (*size == k) {
        if (!hit_less(h, R[k - 1])) return;
        *size = k - 1;
    }
    int i = *size;
    while (i > 0 && hit_less(h, R[i - 1])) { R[i] = R[i - 1]; --i; }
    R[i] = h;
    *size += 1;
}

/* ---- kNN scan (Section 4.2, kNN) ----------------------------------------------------- */
/*
 * Per query: R (size k) is filled with the first k candidates, all with exact distances;
 * afterwards candidates are taken in batches; inside a batch the threshold tau (the k-th
 * squared distance in R, +inf while R is short) is frozen; a candidate survives iff
 * g <= tau; survivors get exact distances and are merged into R.  Every batch holds `batch`
 * candidates (the last one what is left); batch = 1 is the paper's vector-at-a-time rule.
 * Everything is in squared distances.
 *
 * lut may be NULL (the table is then built here).  ids may be NULL (id = position).
 * list_offsets NULL => every query scans positions 0..n-1.
 * mask (nullable): bit (idx % 32) of word mask[q*mask_words + idx/32] set iff the
 * candidate with scan-order number idx had its exact distance computed.
 * Rows short of k results are padded with id -1, d2 +inf.
 */
void trim_oracle_search_knn(const float *base, const uint8_t *codes, const float *dlx,
                            const int32_t *ids, const float *codebooks, int64_t n, int d,
                            int M, const float *queries, int64_t nq, const float *lut,
                            int nprobe, const int64_t *list_offsets, const int32_t *probes,
                            int k, float gamma, int batch, int32_t *out_ids,
                            float *out_d2, int32_t *n_scanned, int32_t *n_exact, uint32_t *mask,
                            int64_t mask_words) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < nq; ++q) {
        const float *qv = queries + (size_t)q * d;
        float *Tq = NULL;
        const float *T;
        if (lut) {
            T = lut + (size_t)q * M * TRIM_C;
        } else {
            Tq = malloc(sizeof(float) * (size_t)M * TRIM_C);
            trim_oracle_build_lut(qv, 1, d, codebooks, M, Tq);
            T = Tq;
        }
        cand_t cs = cand_make(n, nprobe, list_offsets, probes ? probes + (size_t)q * nprobe : NULL);
        hit_t *R = malloc(sizeof(hit_t) * (size_t)k);
        int size = 0;
        int32_t exact = 0;
        uint32_t *mq = mask ? mask + (size_t)q * mask_words : NULL;

        int64_t idx = 0;
        /* seed: the first k candidates populate R */
        for (; idx < cs.total && idx < k; ++idx) {
            int64_t pos = cs.pos[idx];
            hit_t h = { trim_oracle_exact_d2(qv, base + (size_t)pos * d, d),
                        ids ? ids[pos] : (int32_t)pos };
            result_insert(R, &size, k, h);
            ++exact;
            if (mq) mq[idx / 32] |= 1u << (idx % 32);
        }
        hit_t *surv = malloc(sizeof(hit_t) * (size_t)(batch > 0 ? batch : 1));
        while (idx < cs.total) {
            float tau = size >= k ? R[k - 1].d2 : INFINITY;
            int64_t end = idx + batch < cs.total ? idx + batch : cs.total;
            int ns = 0;
            for (; idx < end; ++idx) {
                int64_t pos = cs.pos[idx];
                float g = trim_oracle_plb(T, codes + (size_t)pos * M, M, dlx[pos], gamma);
                if (g <= tau) {
                    surv[ns].d2 = trim_oracle_exact_d2(qv, base + (size_t)pos * d, d);
                    surv[ns].id = ids ? ids[pos] : (int32_t)pos;
                    ++ns;
                    if (mq) mq[idx / 32] |= 1u << (idx % 32);
                }
            }
            for (int i = 0; i < ns; ++i) result_insert(R, &size, k, surv[i]);
            exact += ns;
        }
        for (int i = 0; i < k; ++i) {
            out_ids[(size_t)q * k + i] = i < size ? R[i].id : -1;
            out_d2[(size_t)q * k + i] = i < size ? R[i].d2 : INFINITY;
        }
        if (n_scanned) n_scanned[q] = (int32_t)cs.total;
        if (n_exact) n_exact[q] = exact;
        free(surv); free(R); cand_free(&cs); free(Tq);
    }
}

/* ---- range scan (Section 4.2, range) -------------------------------------------------- */
/*
 * tau = radius2 for every candidate; survive iff g <= tau; a survivor is a result iff its
 * exact squared distance <= radius2.  Results are emitted in scan order.
 * Pass 1 (out_ids == NULL): fills counts[q] only.  Pass 2: offsets[] (nq+1, exclusive prefix
 * of counts, supplied by the caller) says where each query's results go.
 */
void trim_oracle_search_range(const float *base, const uint8_t *codes, const float *dlx,
                              const int32_t *ids, const float *codebooks, int64_t n, int d,
                              int M, const float *queries, int64_t nq, const float *lut,
                              int nprobe, const int64_t *list_offsets, const int32_t *probes,
                              float radius2, float gamma, int64_t *counts,
                              const int64_t *offsets, int32_t *out_ids, float *out_d2,
                              int32_t *n_scanned, int32_t *n_exact, uint32_t *mask,
                              int64_t mask_words) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < nq; ++q) {
        const float *qv = queries + (size_t)q * d;
        float *Tq = NULL;
        const float *T;
        if (lut) {
            T = lut + (size_t)q * M * TRIM_C;
        } else {
            Tq = malloc(sizeof(float) * (size_t)M * TRIM_C);
            trim_oracle_build_lut(qv, 1, d, codebooks, M, Tq);
            T = Tq;
        }
        cand_t cs = cand_make(n, nprobe, list_offsets, probes ? probes + (size_t)q * nprobe : NULL);
        uint32_t *mq = mask ? mask + (size_t)q * mask_words : NULL;
        int64_t cnt = 0;
        int32_t exact = 0;
        for (int64_t idx = 0; idx < cs.total; ++idx) {
            int64_t pos = cs.pos[idx];
            float g = trim_oracle_plb(T, codes + (size_t)pos * M, M, dlx[pos], gamma);
            if (!(g <= radius2)) continue;
            ++exact;
            if (mq) mq[idx / 32] |= 1u << (idx % 32);
            float d2 = trim_oracle_exact_d2(qv, base + (size_t)pos * d, d);
            if (d2 <= radius2) {
                if (out_ids) {
                    out_ids[offsets[q] + cnt] = ids ? ids[pos] : (int32_t)pos;
                    out_d2[offsets[q] + cnt] = d2;
                }
                ++cnt;
            }
        }
        if (counts) counts[q] = cnt;
        if (n_scanned) n_scanned[q] = (int32_t)cs.total;
        if (n_exact) n_exact[q] = exact;
        cand_free(&cs); free(Tq);
    }
}

/* ---- definitions used as anchors: brute force (Section 2.1) --------------------------- */

/* kNN by definition over one query's candidate set, binary32 distances in the order above,
 * ties by id.  Same candidate arguments as the scans. */
void trim_oracle_brute_knn(const float *base, const int32_t *ids, int64_t n, int d,
                           const float *queries, int64_t nq, int nprobe,
                           const int64_t *list_offsets, const int32_t *probes, int k,
                           int32_t *out_ids, float *out_d2) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < nq; ++q) {
        const float *qv = queries + (size_t)q * d;
        cand_t cs = cand_make(n, nprobe, list_offsets, probes ? probes + (size_t)q * nprobe : NULL);
        hit_t *R = malloc(sizeof(hit_t) * (size_t)k);
        int size = 0;
        for (int64_t idx = 0; idx < cs.total; ++idx) {
            int64_t pos = cs.pos[idx];
            hit_t h = { trim_oracle_exact_d2(qv, base + (size_t)pos * d, d),
                        ids ? ids[pos] : (int32_t)pos };
            result_insert(R, &size, k, h);
        }
        for (int i = 0; i < k; ++i) {
            out_ids[(size_t)q * k + i] = i < size ? R[i].id : -1;
            out_d2[(size_t)q * k + i] = i < size ? R[i].d2 : INFINITY;
        }
        free(R); cand_free(&cs);
    }
}

/* Ground truth for recall: kNN over ALL n vectors in binary64, plain sum of squares. */
typedef struct { double d2; int32_t id; } hit64_t;
void trim_oracle_brute_knn_f64(const float *base, const int32_t *ids, int64_t n, int d,
                                   const float *queries, int64_t nq, int k, int32_t *out_ids,
                                   double *out_d2) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < nq; ++q) {
        const float *qv = queries + (size_t)q * d;
        hit64_t *R = malloc(sizeof(hit64_t) * (size_t)k);
        int size = 0;
        for (int64_t pos = 0; pos < n; ++pos) {
            const float *x = base + (size_t)pos * d;
            double acc = 0.0;
            for (int t = 0; t < d; ++t) {
                double diff = (double)qv[t] - (double)x[t];
                acc += diff * diff;
            }
            int32_t id = ids ? ids[pos] : (int32_t)pos;
            if (size == k) {
                hit64_t w = R[k - 1];
                if (!(acc < w.d2 || (acc == w.d2 && id < w.id))) continue;
                size = k - 1;
            }
            int i = size;
            while (i > 0 && (acc < R[i - 1].d2 || (acc == R[i - 1].d2 && id < R[i - 1].id))) {
                R[i] = R[i - 1]; --i;
            }
            R[i].d2 = acc; R[i].id = id;
            ++size;
        }
        for (int i = 0; i < k; ++i) {
            out_ids[(size_t)q * k + i] = i < size ? R[i].id : -1;
            out_d2[(size_t)q * k + i] = i < size ? R[i].d2 : INFINITY;
        }
        free(R);
    }
}

/* Batched exact distances between given (query row, base position) pairs. */
void trim_oracle_exact_pairs(const float *base, int d, const float *queries,
                             const int64_t *qrow, const int64_t *pos, int64_t npairs,
                             float *out_d2) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < npairs; ++i)
        out_d2[i] = trim_oracle_exact_d2(queries + (size_t)qrow[i] * d,
                                         base + (size_t)pos[i] * d, d);
}

/* Bounds for given (query row, base position) pairs: s = Gamma(l,q)^2 and g. */
void trim_oracle_plb_pairs(const float *lut, int M, const uint8_t *codes, const float *dlx,
                           const int64_t *qrow, const int64_t *pos, int64_t npairs,
                           float gamma, float *out_s, float *out_g) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < npairs; ++i) {
        const float *T = lut + (size_t)qrow[i] * M * TRIM_C;
        float s = table_sum(T, codes + (size_t)pos[i] * M, M);
        if (out_s) out_s[i] = s;
        if (out_g) out_g[i] = trim_oracle_plb_from_s(s, dlx[pos[i]], gamma);
    }
}

/* ---- candidate generation: the nprobe nearest coarse centroids (Section 6.1: IVFPQ with
 * C' lists and a tuned nprobe), nearest first, ties by smaller list id ------------------- */
void trim_oracle_ivf_probe(const float *queries, int64_t nq, int d, const float *centroids,
                           int nlist, int nprobe, int32_t *probes) {
#pragma omp parallel for schedule(static)
    for (int64_t q = 0; q < nq; ++q) {
        hit_t *R = malloc(sizeof(hit_t) * (size_t)nprobe);
        int size = 0;
        for (int l = 0; l < nlist; ++l) {
            hit_t h = { trim_oracle_exact_d2(queries + (size_t)q * d,
                                             centroids + (size_t)l * d, d), l };
            result_insert(R, &size, nprobe, h);
        }
        for (int p = 0; p < nprobe; ++p) probes[(size_t)q * nprobe + p] = p < size ? R[p].id : -1;
        free(R);
    }
}

/* Threads the parallel loops above use (reported next to the CPU-baseline timing). */
int trim_oracle_num_threads(void) { return omp_get_max_threads(); }

/*
 * TRIM with 4-bit landmark codes (the paper's FastScan-compatible variant "tIVFPQfs"):
 * plain CPU oracle.  TEST INFRASTRUCTURE ONLY -- same rules as trim_oracle.c: never linked
 * into, imported by, or called from the product.
 *
 * What it follows (paper: "TRIM", arXiv 2508.17828):
 *   - Section 6.1, parameter setting: the FastScan variants use 4-bit codes with m = d/2
 *     subspaces, i.e. 16 centroids per subspace instead of 256;
 *   - everything else is the method as it stands: landmark = PQ reconstruction and
 *     Gamma(l,q)^2 = sum_j T[j][code_j] (Section 3.1), the bounds of Definitions 1-2 /
 *     Equation 3, the stored code and Gamma(l,x) (Section 3.3), the scan of Section 4.2.
 *
 * Readings (the paper says no more about this variant than the two parameters above):
 *   - the table keeps binary32 entries, as in the 8-bit variant: Section 3.1 computes
 *     Gamma(l,q) "exactly" from the table, and Equation 3 needs Gamma(l,q) itself, not an
 *     8-bit approximation of it (the CPU library the paper builds on quantises its table to
 *     fit SIMD registers; nothing in the method asks for that);
 *   - storage: two codes per byte, subspace 2i in the low half of byte i, subspace 2i+1 in
 *     the high half (m must be even);
 *   - the seed / batch rule, the comparisons (g <= tau, d2 <= radius^2), tie rules and the
 *     rounding order are those of trim_oracle.c:
 *       sub-vector distance : acc = fmaf(x_t - c_t, x_t - c_t, acc), t ascending
 *       table sum           : s = ((T[0][c0] + T[1][c1]) + T[2][c2]) + ...   (j ascending)
 *       bound, exact distance: trim_oracle_plb_from_s, trim_oracle_exact_d2 (called, not copied).
 * Pins live in tests/test_oracle_fs_pins.py.  Parity unpinned: none of the functions below.
 */
#include <math.h>
#include <omp.h>
#include <stdint.h>
#include <stdlib.h>

#define FS_C 16 /* centroids per subspace: 4-bit codes (Section 6.1) */

/* defined in trim_oracle.c (same library) */
float trim_oracle_exact_d2(const float *q, const float *x, int d);
float trim_oracle_plb_from_s(float s, float b, float gamma);

static float subvec_sqdist(const float *x, const float *c, int len) {
    float acc = 0.0f;
    for (int t = 0; t < len; ++t) {
        float diff = x[t] - c[t];
        acc = fmaf(diff, diff, acc);
    }
    return acc;
}

/* The 4-bit code of subspace j inside a packed code. */
static int code_at(const uint8_t *code, int j) {
    return (j & 1) ? (code[j >> 1] >> 4) : (code[j >> 1] & 15);
}

/* Gamma(l,q)^2 = sum over the m subspaces of the table entry the code selects (Section 3.1). */
float trim_oracle_fs_table_sum(const float *T, const uint8_t *code, int m) {
    float s = 0.0f;
    for (int j = 0; j < m; ++j) s = s + T[(size_t)j * FS_C + code_at(code, j)];
    return s;
}

/* Preprocessing (Section 3.3, step 1) with 16 centroids per subspace: codes[x] holds m/2 bytes;
 * nearest centroid per subspace, smallest index on ties; dlx[x] = Gamma(l,x). */
void trim_oracle_fs_encode(const float *base, int64_t n, int d, const float *codebooks, int m,
                           uint8_t *codes, float *dlx) {
    int dsub = d / m;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        float tot = 0.0f;
        for (int j = 0; j < m; ++j) {
            const float *xj = base + (size_t)i * d + (size_t)j * dsub;
            const float *cb = codebooks + (size_t)j * FS_C * dsub;
            float best = INFINITY;
            int arg = 0;
            for (int c = 0; c < FS_C; ++c) {
                float v = subvec_sqdist(xj, cb + (size_t)c * dsub, dsub);
                if (v < best) { best = v; arg = c; }
            }
            uint8_t *byte = codes + (size_t)i * (m / 2) + j / 2;
            if (j & 1) *byte = (uint8_t)(*byte | (arg << 4));
            else *byte = (uint8_t)arg;
            tot = tot + best;
        }
        dlx[i] = sqrtf(tot);
    }
}

/* Distance table (Section 3.3, query processing, operation 1): lut[q][j][c], c < 16. */
void trim_oracle_fs_build_lut(const float *queries, int64_t nq, int d, const float *codebooks,
                              int m, float *lut) {
    int dsub = d / m;
#pragma omp parallel for schedule(static)
    for (int64_t q = 0; q < nq; ++q)
        for (int j = 0; j < m; ++j)
            for (int c = 0; c < FS_C; ++c)
                lut[((size_t)q * m + j) * FS_C + c] =
                    subvec_sqdist(queries + (size_t)q * d + (size_t)j * dsub,
                                  codebooks + ((size_t)j * FS_C + c) * dsub, dsub);
}

/* ---- candidate order and result set: as in Section 4.2 (see trim_oracle.c) ---------------- */

typedef struct { int64_t *pos; int64_t total; } cand_t;

static cand_t cand_make(int64_t n, int nprobe, const int64_t *list_offsets, const int32_t *probes_q) {
    cand_t c;
    c.total = 0;
    if (!list_offsets) c.total = n;
    else
        for (int p = 0; p < nprobe; ++p)
            c.total += list_offsets[probes_q[p] + 1] - list_offsets[probes_q[p]];
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

static const float *table_of(const float *lut, float **own, const float *qv, int64_t q, int d,
                             const float *codebooks, int m) {
    if (lut) return lut + (size_t)q * m * FS_C;
    *own = malloc(sizeof(float) * (size_t)m * FS_C);
    trim_oracle_fs_build_lut(qv, 1, d, codebooks, m, *own);
    return *own;
}

/* kNN scan of Section 4.2 over 4-bit codes: seed of k, then batches of `batch` with tau frozen
 * inside a batch; survive iff g <= tau.  Arguments as trim_oracle_search_knn, with m subspaces
 * of 16 centroids and codes [n][m/2]. */
void trim_oracle_fs_search_knn(const float *base, const uint8_t *codes, const float *dlx,
                               const int32_t *ids, const float *codebooks, int64_t n, int d, int m,
                               const float *queries, int64_t nq, const float *lut, int nprobe,
                               const int64_t *list_offsets, const int32_t *probes, int k,
                               float gamma, int batch, int32_t *out_ids, float *out_d2,
                               int32_t *n_scanned, int32_t *n_exact, uint32_t *mask,
                               int64_t mask_words) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < nq; ++q) {
        const float *qv = queries + (size_t)q * d;
        float *Tq = NULL;
        const float *T = table_of(lut, &Tq, qv, q, d, codebooks, m);
        cand_t cs = cand_make(n, nprobe, list_offsets, probes ? probes + (size_t)q * nprobe : NULL);
        hit_t *R = malloc(sizeof(hit_t) * (size_t)k);
        hit_t *surv = malloc(sizeof(hit_t) * (size_t)(batch > 0 ? batch : 1));
        int size = 0;
        int32_t exact = 0;
        uint32_t *mq = mask ? mask + (size_t)q * mask_words : NULL;
        int64_t idx = 0;
        for (; idx < cs.total && idx < k; ++idx) { /* seed */
            int64_t pos = cs.pos[idx];
            hit_t h = { trim_oracle_exact_d2(qv, base + (size_t)pos * d, d), ids ? ids[pos] : (int32_t)pos };
            result_insert(R, &size, k, h);
            ++exact;
            if (mq) mq[idx / 32] |= 1u << (idx % 32);
        }
        while (idx < cs.total) {
            float tau = size >= k ? R[k - 1].d2 : INFINITY;
            int64_t end = idx + batch < cs.total ? idx + batch : cs.total;
            int ns = 0;
            for (; idx < end; ++idx) {
                int64_t pos = cs.pos[idx];
                float s = trim_oracle_fs_table_sum(T, codes + (size_t)pos * (m / 2), m);
                float g = trim_oracle_plb_from_s(s, dlx[pos], gamma);
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
        free(surv); free(R); free(cs.pos); free(Tq);
    }
}

/* Range scan of Section 4.2 over 4-bit codes: tau = radius2 throughout; results in scan order.
 * Two passes as trim_oracle_search_range (out_ids == NULL: counts only). */
void trim_oracle_fs_search_range(const float *base, const uint8_t *codes, const float *dlx,
                                 const int32_t *ids, const float *codebooks, int64_t n, int d, int m,
                                 const float *queries, int64_t nq, const float *lut, int nprobe,
                                 const int64_t *list_offsets, const int32_t *probes, float radius2,
                                 float gamma, int64_t *counts, const int64_t *offsets,
                                 int32_t *out_ids, float *out_d2, int32_t *n_scanned,
                                 int32_t *n_exact, uint32_t *mask, int64_t mask_words) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < nq; ++q) {
        const float *qv = queries + (size_t)q * d;
        float *Tq = NULL;
        const float *T = table_of(lut, &Tq, qv, q, d, codebooks, m);
        cand_t cs = cand_make(n, nprobe, list_offsets, probes ? probes + (size_t)q * nprobe : NULL);
        uint32_t *mq = mask ? mask + (size_t)q * mask_words : NULL;
        int64_t cnt = 0;
        int32_t exact = 0;
        for (int64_t idx = 0; idx < cs.total; ++idx) {
            int64_t pos = cs.pos[idx];
            float s = trim_oracle_fs_table_sum(T, codes + (size_t)pos * (m / 2), m);
            float g = trim_oracle_plb_from_s(s, dlx[pos], gamma);
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
        free(cs.pos); free(Tq);
    }
}

/* Bounds for given (query row, base position) pairs: s = Gamma(l,q)^2 and g. */
void trim_oracle_fs_plb_pairs(const float *lut, int m, const uint8_t *codes, const float *dlx,
                              const int64_t *qrow, const int64_t *pos, int64_t npairs, float gamma,
                              float *out_s, float *out_g) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < npairs; ++i) {
        const float *T = lut + (size_t)qrow[i] * m * FS_C;
        float s = trim_oracle_fs_table_sum(T, codes + (size_t)pos[i] * (m / 2), m);
        if (out_s) out_s[i] = s;
        if (out_g) out_g[i] = trim_oracle_plb_from_s(s, dlx[pos[i]], gamma);
    }
}

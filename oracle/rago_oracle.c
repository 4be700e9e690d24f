/*
 * CPU oracle for IVF-PQ search and exact flat search.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, step-by-step statement of what the retrieval stage computes, used to
 * check the HIP library and as the timed CPU baseline.  Nothing in the product path may
 * call it, and it shares no code, header, table or helper with the HIP path.
 *
 * What the paper fixes: vector search returns the K most similar vectors to a D-dim query
 * from a database (Section 2, "Vector search for retrieval"); IVF-PQ = inverted-file index
 * + product quantisation, one byte per 4-16 dimensions (Section 2); a query scans only a
 * P_scan fraction of the database, cost = bytes of PQ codes scanned (Section 3.3,
 * "Retrieval component"); small per-request corpora are searched by brute-force kNN
 * (Section 5.2).  The paper gives no listing for IVF-PQ, so the steps below are the standard
 * algorithm with every unspecified choice (metric, residual PQ, table quantisation,
 * tie-breaks, padding) fixed as documented at each function.
 *
 * Metric: inner product, larger = better (metric 0), or the Euclidean distance the paper names
 * first among its similarity notions (Section 2), as similarity = MINUS the squared distance, so
 * that larger = better there too and every later step is shared (metric 1).  All pointers are
 * host memory.  Floating point: fp64 accumulation rounded once to fp32 where stated; compile
 * with -ffp-contract=off so no multiply-add is fused.
 *
 * Pins (tests/, CPU-only): exhaustive reconstruct-and-matmul ADC at nprobe = nlist, the
 * look-up-table sum identity, an integer-exact worked case, quantisation error bound and
 * end points, brute-force sorts with forced ties, numpy matmul for coarse and flat scores;
 * the rounding conventions of steps 3-4 (ties to even in the 8-bit entries and the bias, the
 * fp32 subtract and IEEE divide, fp64 accumulation with one rounding in both kinds of table,
 * the fp64 sum and quotient of the bias) by hand-derived worked cases and half-ulp bounds;
 * Euclidean metric: numpy distances for the coarse scores, the table sum identity against an
 * independent reconstruction, zero entries at exact matches, its relation to the inner-product
 * tables through the norms, exhaustive search at nprobe = nlist, agreement with the inner-product
 * ranking on lossless codes of unit vectors.
 * Parity unpinned: absolute recall values on synthetic data (data-dependent; reported only).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define KSUB 256

enum { ORACLE_OK = 0, ORACLE_EINVAL = -1, ORACLE_ENOMEM = -2 };

/* ---- ordered selection: the best `k` of a stream under (key descending, id ascending) ---- */
typedef struct { double key; int64_t id; } cand_t;

static int better(cand_t a, cand_t b) { return a.key > b.key || (a.key == b.key && a.id < b.id); }

/* best[0..*cnt) is kept sorted best-first; equivalent to sorting everything and taking k. */
static void offer(cand_t* best, int64_t* cnt, int64_t k, cand_t c) {
    if (k <= 0) return;
    if (*cnt == k && !better(c, best[k - 1])) return;
    int64_t i = (*cnt < k) ? (*cnt)++ : k - 1;
    while (i > 0 && better(c, best[i - 1])) { best[i] = best[i - 1]; --i; }
    best[i] = c;
}

/* ---- step 1: coarse scores S[q][l] = <Q[q], C[l]>, fp64 accumulate -> fp32 (IVF level, Section 2) ---- */
int oracle_coarse(const float* Q, const float* C, int64_t nq, int64_t nlist, int64_t d, float* S) {
    if (!Q || !C || !S || nq < 0 || nlist <= 0 || d <= 0) return ORACLE_EINVAL;
    for (int64_t q = 0; q < nq; ++q)
        for (int64_t l = 0; l < nlist; ++l) {
            double acc = 0.0;
            for (int64_t t = 0; t < d; ++t) acc += (double)Q[q * d + t] * (double)C[l * d + t];
            S[q * nlist + l] = (float)acc;
        }
    return ORACLE_OK;
}

/* ---- step 1, Euclidean metric: S[q][l] = -|Q[q] - C[l]|^2, fp64 accumulate -> fp32 ---- */
int oracle_coarse_l2(const float* Q, const float* C, int64_t nq, int64_t nlist, int64_t d, float* S) {
    if (!Q || !C || !S || nq < 0 || nlist <= 0 || d <= 0) return ORACLE_EINVAL;
    for (int64_t q = 0; q < nq; ++q)
        for (int64_t l = 0; l < nlist; ++l) {
            double acc = 0.0;
            for (int64_t t = 0; t < d; ++t) {
                const double diff = (double)Q[q * d + t] - (double)C[l * d + t];
                acc += diff * diff;
            }
            S[q * nlist + l] = (float)(-acc);
        }
    return ORACLE_OK;
}

/* ---- step 2: the nprobe lists with the largest S, ties -> lower list number, in rank order
 *      (the scanned subset of Section 3.3) ---- */
int oracle_select(const float* S, int64_t nq, int64_t nlist, int64_t nprobe, int32_t* probes) {
    if (!S || !probes || nq < 0 || nprobe <= 0 || nprobe > nlist) return ORACLE_EINVAL;
    cand_t* best = (cand_t*)malloc(sizeof(cand_t) * (size_t)nprobe);
    if (!best) return ORACLE_ENOMEM;
    for (int64_t q = 0; q < nq; ++q) {
        int64_t cnt = 0;
        for (int64_t l = 0; l < nlist; ++l) {
            cand_t c = { (double)S[q * nlist + l], l };
            offer(best, &cnt, nprobe, c);
        }
        for (int64_t p = 0; p < nprobe; ++p) probes[q * nprobe + p] = (int32_t)best[p].id;
    }
    free(best);
    return ORACLE_OK;
}

/* ---- steps 1-2 with an upper level over the lists (the multi-level tree of Section 4, "Models
 *      and database"; searching an upper level is itself a vector scan, Section 4 "Retrieval
 *      performance modeling").  The lists are partitioned into nsuper groups: group s holds the
 *      lists super_lists[super_offsets[s] .. super_offsets[s+1]) and has a centroid SC[s].  A query
 *      scores the nsuper group centroids, keeps the nsp best groups (ties -> lower group), scores
 *      only the lists of those groups, and takes the nprobe best of them (ties -> lower list).
 *      Lists outside the kept groups count as -inf: when the kept groups hold fewer than nprobe
 *      lists, the lowest-numbered other lists fill up.  Scores as in step 1 for the metric. ---- */
int oracle_select_tree(const float* Q, const float* SC, const int64_t* super_offsets, const int32_t* super_lists,
                       const float* C, int64_t nq, int64_t nsuper, int64_t nlist, int64_t d, int64_t nsp,
                       int64_t nprobe, int metric, int32_t* probes, int32_t* out_supers) {
    if (!Q || !SC || !super_offsets || !super_lists || !C || !probes) return ORACLE_EINVAL;
    if (nsuper <= 0 || nsp <= 0 || nsp > nsuper || nprobe <= 0 || nprobe > nlist || (metric != 0 && metric != 1)) return ORACLE_EINVAL;
    float* Ssup = (float*)malloc(sizeof(float) * (size_t)nsuper);
    int32_t* sup = (int32_t*)malloc(sizeof(int32_t) * (size_t)nsp);
    float* S = (float*)malloc(sizeof(float) * (size_t)nlist);
    int rc = (Ssup && sup && S) ? ORACLE_OK : ORACLE_ENOMEM;
    for (int64_t q = 0; q < nq && !rc; ++q) {
        const float* qv = Q + q * d;
        rc = metric ? oracle_coarse_l2(qv, SC, 1, nsuper, d, Ssup) : oracle_coarse(qv, SC, 1, nsuper, d, Ssup);
        if (!rc) rc = oracle_select(Ssup, 1, nsuper, nsp, sup);
        if (rc) break;
        for (int64_t l = 0; l < nlist; ++l) S[l] = -INFINITY;
        for (int64_t i = 0; i < nsp; ++i)
            for (int64_t e = super_offsets[sup[i]]; e < super_offsets[sup[i] + 1]; ++e) {
                const int64_t l = super_lists[e];
                if (l < 0 || l >= nlist) { rc = ORACLE_EINVAL; break; }
                rc = metric ? oracle_coarse_l2(qv, C + l * d, 1, 1, d, S + l) : oracle_coarse(qv, C + l * d, 1, 1, d, S + l);
            }
        if (!rc) rc = oracle_select(S, 1, nlist, nprobe, probes + q * nprobe);
        if (!rc && out_supers) memcpy(out_supers + q * nsp, sup, sizeof(int32_t) * (size_t)nsp);
    }
    free(Ssup); free(sup); free(S);
    return rc;
}

/* ---- step 3: fp32 look-up tables of the residual PQ, one per (query, probed list).
 *      A database vector in list l with code (c_0..c_{m-1}) is reconstructed as
 *      C[l] + concat_j CB[j][c_j]; its score with q splits over the m sub-spaces, so
 *      L[q,p][j][c] = < q_j , C[l]_j + CB[j][c] >  (fp64 accumulate -> fp32). ---- */
int oracle_lut_f32(const float* Q, const float* C, const float* CB, const int32_t* probes,
                   int64_t nq, int64_t nprobe, int64_t d, int64_t m, float* L) {
    if (!Q || !C || !CB || !probes || !L || m <= 0 || d % m) return ORACLE_EINVAL;
    const int64_t dsub = d / m;
    for (int64_t q = 0; q < nq; ++q)
        for (int64_t p = 0; p < nprobe; ++p) {
            const int64_t l = probes[q * nprobe + p];
            for (int64_t j = 0; j < m; ++j)
                for (int64_t c = 0; c < KSUB; ++c) {
                    double acc = 0.0;
                    for (int64_t t = 0; t < dsub; ++t)
                        acc += (double)Q[q * d + j * dsub + t] *
                               ((double)C[l * d + j * dsub + t] + (double)CB[(j * KSUB + c) * dsub + t]);
                    L[(((q * nprobe + p) * m + j) * KSUB) + c] = (float)acc;
                }
        }
    return ORACLE_OK;
}

/* ---- step 3, Euclidean metric: the squared distance to the reconstruction splits over the m
 *      sub-spaces as well, but not into a per-query and a per-list part:
 *      L[q,p][j][c] = - | q_j - (C[l]_j + CB[j][c]) |^2  (fp64 accumulate -> fp32). ---- */
int oracle_lut_f32_l2(const float* Q, const float* C, const float* CB, const int32_t* probes,
                      int64_t nq, int64_t nprobe, int64_t d, int64_t m, float* L) {
    if (!Q || !C || !CB || !probes || !L || m <= 0 || d % m) return ORACLE_EINVAL;
    const int64_t dsub = d / m;
    for (int64_t q = 0; q < nq; ++q)
        for (int64_t p = 0; p < nprobe; ++p) {
            const int64_t l = probes[q * nprobe + p];
            for (int64_t j = 0; j < m; ++j)
                for (int64_t c = 0; c < KSUB; ++c) {
                    double acc = 0.0;
                    for (int64_t t = 0; t < dsub; ++t) {
                        const double diff = (double)Q[q * d + j * dsub + t] -
                                            ((double)C[l * d + j * dsub + t] + (double)CB[(j * KSUB + c) * dsub + t]);
                        acc += diff * diff;
                    }
                    L[(((q * nprobe + p) * m + j) * KSUB) + c] = (float)(-acc);
                }
        }
    return ORACLE_OK;
}

/* ---- step 4: 8-bit tables (the lower-precision, memory-bound PQ variant of Section 2).
 *      lo/hi = min/max over c of one sub-table; one step per QUERY,
 *      delta_q = max_{p,j}(hi - lo) / 255 (fp32; 1 if zero), so integer scores of different
 *      lists of a query are comparable; LUT8 = clamp(rne((L - lo) / delta_q), 0, 255) in
 *      fp32; the dropped offsets go into one integer bias per (query, probe):
 *      B = rne( (sum_j lo_j in fp64) / delta_q ). ---- */
int oracle_quantise(const float* L, int64_t nq, int64_t nprobe, int64_t m,
                    uint8_t* LUT8, int32_t* B, float* delta) {
    if (!L || !LUT8 || !B || !delta) return ORACLE_EINVAL;
    for (int64_t q = 0; q < nq; ++q) {
        float range = 0.0f;
        for (int64_t pj = 0; pj < nprobe * m; ++pj) {
            const float* row = L + (q * nprobe * m + pj) * KSUB;
            float lo = row[0], hi = row[0];
            for (int c = 1; c < KSUB; ++c) { if (row[c] < lo) lo = row[c]; if (row[c] > hi) hi = row[c]; }
            if (hi - lo > range) range = hi - lo;
        }
        float dq = range / 255.0f;
        if (!(dq > 0.0f)) dq = 1.0f;
        delta[q] = dq;
        for (int64_t p = 0; p < nprobe; ++p) {
            double losum = 0.0;
            for (int64_t j = 0; j < m; ++j) {
                const float* row = L + ((q * nprobe + p) * m + j) * KSUB;
                uint8_t* out = LUT8 + ((q * nprobe + p) * m + j) * KSUB;
                float lo = row[0];
                for (int c = 1; c < KSUB; ++c) if (row[c] < lo) lo = row[c];
                for (int c = 0; c < KSUB; ++c) {
                    float r = nearbyintf((row[c] - lo) / dq);
                    out[c] = (uint8_t)(r < 0.0f ? 0.0f : (r > 255.0f ? 255.0f : r));
                }
                losum += (double)lo;
            }
            B[q * nprobe + p] = (int32_t)nearbyint(losum / (double)dq);
        }
    }
    return ORACLE_OK;
}

/* ---- steps 5-6: integer ADC scan of every vector of every probed list,
 *      I = B[q,p] + sum_j LUT8[q,p][j][code_j]; best k by (I descending, id ascending);
 *      scores = (float)I * delta_q; short results padded with (-1, INT32_MIN, -inf). ---- */
int oracle_scan_topk(const int32_t* probes, const uint8_t* LUT8, const int32_t* B, const float* delta,
                     const int64_t* list_offsets, const uint8_t* codes, const int64_t* ids,
                     int64_t nq, int64_t nprobe, int64_t m, int64_t k,
                     int64_t* out_ids, int32_t* out_iscores, float* out_scores) {
    if (!probes || !LUT8 || !B || !list_offsets || !codes || !ids || !out_ids || k <= 0) return ORACLE_EINVAL;
    int rc = ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < nq; ++q) {
        cand_t* best = (cand_t*)malloc(sizeof(cand_t) * (size_t)k);
        if (!best) { rc = ORACLE_ENOMEM; continue; }
        int64_t cnt = 0;
        for (int64_t p = 0; p < nprobe; ++p) {
            const int64_t l = probes[q * nprobe + p];
            const uint8_t* lut = LUT8 + (q * nprobe + p) * m * KSUB;
            for (int64_t i = list_offsets[l]; i < list_offsets[l + 1]; ++i) {
                int32_t I = B[q * nprobe + p];
                for (int64_t j = 0; j < m; ++j) I += lut[j * KSUB + codes[i * m + j]];
                cand_t c = { (double)I, ids[i] };
                offer(best, &cnt, k, c);
            }
        }
        for (int64_t r = 0; r < k; ++r) {
            const int have = r < cnt;
            out_ids[q * k + r] = have ? best[r].id : -1;
            const int32_t I = have ? (int32_t)best[r].key : INT32_MIN;
            if (out_iscores) out_iscores[q * k + r] = I;
            if (out_scores) out_scores[q * k + r] = have ? (float)I * (delta ? delta[q] : 1.0f) : -INFINITY;
        }
        free(best);
    }
    return rc;
}

/* ---- step 7 (checking mode, never compared with the HIP path): ADC without table
 *      quantisation, F = fp32( sum_j L[q,p][j][code_j] in fp64 ), best k by (F desc, id asc). ---- */
int oracle_adc_f32_topk(const int32_t* probes, const float* L, const int64_t* list_offsets,
                        const uint8_t* codes, const int64_t* ids, int64_t nq, int64_t nprobe,
                        int64_t m, int64_t k, int64_t* out_ids, float* out_scores) {
    if (!probes || !L || !list_offsets || !codes || !ids || !out_ids || !out_scores || k <= 0) return ORACLE_EINVAL;
    cand_t* best = (cand_t*)malloc(sizeof(cand_t) * (size_t)k);
    if (!best) return ORACLE_ENOMEM;
    for (int64_t q = 0; q < nq; ++q) {
        int64_t cnt = 0;
        for (int64_t p = 0; p < nprobe; ++p) {
            const int64_t l = probes[q * nprobe + p];
            const float* lut = L + (q * nprobe + p) * m * KSUB;
            for (int64_t i = list_offsets[l]; i < list_offsets[l + 1]; ++i) {
                double acc = 0.0;
                for (int64_t j = 0; j < m; ++j) acc += (double)lut[j * KSUB + codes[i * m + j]];
                cand_t c = { (double)(float)acc, ids[i] };
                offer(best, &cnt, k, c);
            }
        }
        for (int64_t r = 0; r < k; ++r) {
            out_ids[q * k + r] = r < cnt ? best[r].id : -1;
            out_scores[q * k + r] = r < cnt ? (float)best[r].key : -INFINITY;
        }
    }
    free(best);
    return ORACLE_OK;
}

/* ---- 4-bit product quantisation (Section 2: a byte of code covers 4 to 16 dimensions).  Two
 *      consecutive sub-quantisers of 16 codewords share a code byte, the even one in the low
 *      nibble.  A byte b of sub-quantisers (2j, 2j+1) therefore is one symbol of a 256-word
 *      codebook over their joint sub-space, word b = CB16[2j][b & 15] followed by
 *      CB16[2j+1][b >> 4]; every other step of the search takes that codebook, with m/2
 *      sub-quantisers of twice the width, unchanged (the table of a byte is the table of its joint
 *      word, so quantisation to 8 bits is per byte, like the scan that consumes it).
 *      CB16 [m][16][dsub] -> CB256 [m/2][256][2*dsub]. ---- */
int oracle_expand_pq4(const float* CB16, int64_t m, int64_t dsub, float* CB256) {
    if (!CB16 || !CB256 || m <= 0 || (m & 1) || dsub <= 0) return ORACLE_EINVAL;
    for (int64_t j = 0; j < m / 2; ++j)
        for (int64_t b = 0; b < KSUB; ++b)
            for (int64_t t = 0; t < 2 * dsub; ++t)
                CB256[(j * KSUB + b) * 2 * dsub + t] = t < dsub ? CB16[((2 * j) * 16 + (b & 15)) * dsub + t]
                                                                 : CB16[((2 * j + 1) * 16 + (b >> 4)) * dsub + (t - dsub)];
    return ORACLE_OK;
}

/* ---- whole search, steps 1-6 chained query by query (so the fp32 tables of only one query
 *      are alive at a time).  metric 0 = inner product, 1 = minus squared Euclidean distance.
 *      Optional outputs may be NULL. ---- */
int oracle_ivfpq_search(const float* Q, int64_t nq, int64_t d, const float* C, int64_t nlist,
                        const float* CB, int64_t m, const int64_t* list_offsets, const uint8_t* codes,
                        const int64_t* ids, int64_t nprobe, int64_t k, int metric,
                        int64_t* out_ids, float* out_scores, int32_t* out_iscores,
                        int32_t* out_probes, float* out_delta) {
    if (!Q || !C || !CB || !out_ids || nprobe <= 0 || nprobe > nlist || k <= 0 || m <= 0 || d % m) return ORACLE_EINVAL;
    if (metric != 0 && metric != 1) return ORACLE_EINVAL;
    int rc = ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < nq; ++q) {
        float* S = (float*)malloc(sizeof(float) * (size_t)nlist);
        int32_t* pr = (int32_t*)malloc(sizeof(int32_t) * (size_t)nprobe);
        float* L = (float*)malloc(sizeof(float) * (size_t)(nprobe * m * KSUB));
        uint8_t* L8 = (uint8_t*)malloc((size_t)(nprobe * m * KSUB));
        int32_t* B = (int32_t*)malloc(sizeof(int32_t) * (size_t)nprobe);
        float dq = 1.0f;
        int r = (S && pr && L && L8 && B) ? ORACLE_OK : ORACLE_ENOMEM;
        if (!r) r = metric ? oracle_coarse_l2(Q + q * d, C, 1, nlist, d, S) : oracle_coarse(Q + q * d, C, 1, nlist, d, S);
        if (!r) r = oracle_select(S, 1, nlist, nprobe, pr);
        if (!r) r = metric ? oracle_lut_f32_l2(Q + q * d, C, CB, pr, 1, nprobe, d, m, L)
                           : oracle_lut_f32(Q + q * d, C, CB, pr, 1, nprobe, d, m, L);
        if (!r) r = oracle_quantise(L, 1, nprobe, m, L8, B, &dq);
        if (!r) r = oracle_scan_topk(pr, L8, B, &dq, list_offsets, codes, ids, 1, nprobe, m, k,
                                     out_ids + q * k, out_iscores ? out_iscores + q * k : NULL,
                                     out_scores ? out_scores + q * k : NULL);
        if (!r && out_probes) memcpy(out_probes + q * nprobe, pr, sizeof(int32_t) * (size_t)nprobe);
        if (!r && out_delta) out_delta[q] = dq;
        if (r) rc = r;
        free(S); free(pr); free(L); free(L8); free(B);
    }
    return rc;
}

/* ---- exact flat search over small per-request corpora (brute-force kNN, Section 5.2):
 *      s[r][q][i] = fp32( sum_t bf16(Q) * bf16(X) in fp64 ), best k by (s desc, i asc).
 *      bf16 = upper 16 bits of an IEEE fp32. ---- */
static float bf16_to_f32(uint16_t h) { uint32_t u = (uint32_t)h << 16; float f; memcpy(&f, &u, 4); return f; }

/* IEEE 754 binary16 (1 sign, 5 exponent, 10 fraction bits; the format the paper caches freshly
 * encoded chunks in, Section 5.2): value = (-1)^s 2^(e-15) (1 + f/1024), e = 0: (-1)^s 2^-14 f/1024,
 * e = 31: infinity (f = 0) or NaN. */
static double f16_to_f64(uint16_t h) {
    const int s = h >> 15, e = (h >> 10) & 31, f = h & 1023;
    double v;
    if (e == 0) v = ldexp((double)f, -24);
    else if (e == 31) v = f ? NAN : INFINITY;
    else v = ldexp(1.0 + (double)f / 1024.0, e - 15);
    return s ? -v : v;
}

static int flat_search(const uint16_t* X, const uint16_t* Qb, int64_t R, int64_t n, int64_t nqr,
                       int64_t d, int64_t k, int half, int64_t* out_ids, float* out_scores) {
    if (!X || !Qb || !out_ids || !out_scores || R < 0 || n < 0 || nqr < 0 || d <= 0 || k <= 0) return ORACLE_EINVAL;
    int rc = ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t rq = 0; rq < R * nqr; ++rq) {
        const int64_t r = rq / nqr;
        cand_t* best = (cand_t*)malloc(sizeof(cand_t) * (size_t)k);
        if (!best) { rc = ORACLE_ENOMEM; continue; }
        int64_t cnt = 0;
        for (int64_t i = 0; i < n; ++i) {
            double acc = 0.0;
            for (int64_t t = 0; t < d; ++t) {
                const uint16_t a = Qb[rq * d + t], b = X[(r * n + i) * d + t];
                acc += half ? f16_to_f64(a) * f16_to_f64(b) : (double)bf16_to_f32(a) * (double)bf16_to_f32(b);
            }
            cand_t c = { (double)(float)acc, i };
            offer(best, &cnt, k, c);
        }
        for (int64_t j = 0; j < k; ++j) {
            out_ids[rq * k + j] = j < cnt ? best[j].id : -1;
            out_scores[rq * k + j] = j < cnt ? (float)best[j].key : -INFINITY;
        }
        free(best);
    }
    return rc;
}

int oracle_flat_search(const uint16_t* X, const uint16_t* Qb, int64_t R, int64_t n, int64_t nqr,
                       int64_t d, int64_t k, int64_t* out_ids, float* out_scores) {
    return flat_search(X, Qb, R, n, nqr, d, k, 0, out_ids, out_scores);
}

/* The same search over binary16 bit patterns (finite values). */
int oracle_flat_search_f16(const uint16_t* X, const uint16_t* Qb, int64_t R, int64_t n, int64_t nqr,
                           int64_t d, int64_t k, int64_t* out_ids, float* out_scores) {
    return flat_search(X, Qb, R, n, nqr, d, k, 1, out_ids, out_scores);
}

int oracle_num_threads(void) {
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Runs every function of the CPU oracle on small inputs with edge cases (an empty list, k larger than
 * the number of candidates, one query, zero queries) so that a build with -fsanitize=address,undefined
 * can flag out-of-bounds accesses and undefined behaviour in it.  Test infrastructure: built and run by
 * tests/test_sanitizers.py only. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_coarse(const float*, const float*, int64_t, int64_t, int64_t, float*);
int oracle_coarse_l2(const float*, const float*, int64_t, int64_t, int64_t, float*);
int oracle_select(const float*, int64_t, int64_t, int64_t, int32_t*);
int oracle_select_tree(const float*, const float*, const int64_t*, const int32_t*, const float*, int64_t, int64_t, int64_t, int64_t,
                       int64_t, int64_t, int, int32_t*, int32_t*);
int oracle_lut_f32(const float*, const float*, const float*, const int32_t*, int64_t, int64_t, int64_t, int64_t, float*);
int oracle_lut_f32_l2(const float*, const float*, const float*, const int32_t*, int64_t, int64_t, int64_t, int64_t, float*);
int oracle_quantise(const float*, int64_t, int64_t, int64_t, uint8_t*, int32_t*, float*);
int oracle_scan_topk(const int32_t*, const uint8_t*, const int32_t*, const float*, const int64_t*, const uint8_t*, const int64_t*,
                     int64_t, int64_t, int64_t, int64_t, int64_t*, int32_t*, float*);
int oracle_adc_f32_topk(const int32_t*, const float*, const int64_t*, const uint8_t*, const int64_t*, int64_t, int64_t, int64_t,
                        int64_t, int64_t*, float*);
int oracle_expand_pq4(const float*, int64_t, int64_t, float*);
int oracle_ivfpq_search(const float*, int64_t, int64_t, const float*, int64_t, const float*, int64_t, const int64_t*,
                        const uint8_t*, const int64_t*, int64_t, int64_t, int, int64_t*, float*, int32_t*, int32_t*, float*);
int oracle_flat_search(const uint16_t*, const uint16_t*, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t*, float*);
int oracle_flat_search_f16(const uint16_t*, const uint16_t*, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t*, float*);

static uint32_t rng_state = 12345u;
static float frand(void) { rng_state = rng_state * 1664525u + 1013904223u; return (float)(rng_state >> 8) / 8388608.0f - 1.0f; }
#define CHECK(x) do { if (!(x)) { fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #x); return 1; } } while (0)

int main(void) {
    enum { D = 16, M = 4, DSUB = 4, NLIST = 8, N = 500, NQ = 3, NPROBE = 5, K = 40 };
    float* Q = malloc(sizeof(float) * NQ * D);
    float* C = malloc(sizeof(float) * NLIST * D);
    float* CB = malloc(sizeof(float) * M * 256 * DSUB);
    for (int i = 0; i < NQ * D; ++i) Q[i] = frand();
    for (int i = 0; i < NLIST * D; ++i) C[i] = frand();
    for (int i = 0; i < M * 256 * DSUB; ++i) CB[i] = 0.3f * frand();
    int64_t off[NLIST + 1];
    off[0] = 0;
    for (int l = 0; l < NLIST; ++l) off[l + 1] = off[l] + (l == 2 ? 0 : (l == 5 ? 3 : (N - 3) / (NLIST - 2) + (l == 7 ? (N - 3) % (NLIST - 2) : 0)));
    const int64_t n = off[NLIST];
    uint8_t* codes = malloc((size_t)n * M);
    int64_t* ids = malloc(sizeof(int64_t) * (size_t)n);
    for (int64_t i = 0; i < n * M; ++i) { rng_state = rng_state * 1664525u + 1013904223u; codes[i] = (uint8_t)(rng_state >> 24); }
    for (int64_t i = 0; i < n; ++i) ids[i] = 1000 + i;

    float* S = malloc(sizeof(float) * NQ * NLIST);
    int32_t* probes = malloc(sizeof(int32_t) * NQ * NLIST);
    float* L = malloc(sizeof(float) * NQ * NPROBE * M * 256);
    uint8_t* L8 = malloc((size_t)NQ * NPROBE * M * 256);
    int32_t* B = malloc(sizeof(int32_t) * NQ * NPROBE);
    float delta[NQ];
    int64_t* oi = malloc(sizeof(int64_t) * NQ * 600);
    int32_t* ois = malloc(sizeof(int32_t) * NQ * 600);
    float* osc = malloc(sizeof(float) * NQ * 600);
    for (int metric = 0; metric < 2; ++metric) {
        CHECK((metric ? oracle_coarse_l2 : oracle_coarse)(Q, C, NQ, NLIST, D, S) == 0);
        CHECK(oracle_select(S, NQ, NLIST, NPROBE, probes) == 0);
        CHECK(oracle_select(S, NQ, NLIST, NLIST, probes) == 0 && oracle_select(S, NQ, NLIST, NPROBE, probes) == 0);
        CHECK(oracle_select(S, NQ, NLIST, NLIST + 1, probes) != 0);
        CHECK((metric ? oracle_lut_f32_l2 : oracle_lut_f32)(Q, C, CB, probes, NQ, NPROBE, D, M, L) == 0);
        CHECK(oracle_quantise(L, NQ, NPROBE, M, L8, B, delta) == 0);
        CHECK(oracle_scan_topk(probes, L8, B, delta, off, codes, ids, NQ, NPROBE, M, K, oi, ois, osc) == 0);
        CHECK(oracle_scan_topk(probes, L8, B, NULL, off, codes, ids, NQ, NPROBE, M, 600, oi, ois, osc) == 0);   /* k > candidates */
        CHECK(oi[599] == -1 && ois[599] == INT32_MIN);
        CHECK(oracle_adc_f32_topk(probes, L, off, codes, ids, NQ, NPROBE, M, K, oi, osc) == 0);
        CHECK(oracle_ivfpq_search(Q, NQ, D, C, NLIST, CB, M, off, codes, ids, NPROBE, K, metric, oi, osc, ois, probes, delta) == 0);
        CHECK(oracle_ivfpq_search(Q, 1, D, C, NLIST, CB, M, off, codes, ids, 1, 1, metric, oi, osc, NULL, NULL, NULL) == 0);
        CHECK(oracle_ivfpq_search(Q, 0, D, C, NLIST, CB, M, off, codes, ids, NPROBE, K, metric, oi, osc, ois, probes, delta) == 0);
        /* an upper level: 3 groups of lists */
        const int64_t soff[4] = {0, 3, 4, 8};
        const int32_t slists[8] = {0, 3, 6, 2, 1, 4, 5, 7};
        float SC[3 * D];
        for (int i = 0; i < 3 * D; ++i) SC[i] = frand();
        int32_t sup[NQ * 2];
        CHECK(oracle_select_tree(Q, SC, soff, slists, C, NQ, 3, NLIST, D, 2, NPROBE, metric, probes, sup) == 0);
        CHECK(oracle_select_tree(Q, SC, soff, slists, C, NQ, 3, NLIST, D, 1, NLIST, metric, probes, NULL) == 0);   /* fills up */
    }
    /* 4-bit codebooks -> 256-word codebooks */
    float* cb16 = malloc(sizeof(float) * 8 * 16 * 2);
    float* cb256 = malloc(sizeof(float) * 4 * 256 * 4);
    for (int i = 0; i < 8 * 16 * 2; ++i) cb16[i] = frand();
    CHECK(oracle_expand_pq4(cb16, 8, 2, cb256) == 0);
    CHECK(oracle_expand_pq4(cb16, 7, 2, cb256) != 0);
    /* flat search, both formats, k beyond the corpus */
    enum { R = 2, FN = 37, FQ = 3, FD = 64, FK = 50 };
    uint16_t* X = malloc(sizeof(uint16_t) * R * FN * FD);
    uint16_t* Xq = malloc(sizeof(uint16_t) * R * FQ * FD);
    for (int i = 0; i < R * FN * FD; ++i) { float f = frand(); uint32_t u; memcpy(&u, &f, 4); X[i] = (uint16_t)(u >> 16); }
    for (int i = 0; i < R * FQ * FD; ++i) { float f = frand(); uint32_t u; memcpy(&u, &f, 4); Xq[i] = (uint16_t)(u >> 16); }
    CHECK(oracle_flat_search(X, Xq, R, FN, FQ, FD, FK, oi, osc) == 0);
    CHECK(oi[FK - 1] == -1 && oi[FN - 1] >= 0);
    for (int i = 0; i < R * FN * FD; ++i) X[i] = (uint16_t)((X[i] & 0x8000u) | ((i * 37u) & 0x7bffu));   /* finite binary16 patterns incl. subnormals */
    for (int i = 0; i < R * FQ * FD; ++i) Xq[i] = (uint16_t)((i * 91u) & 0x3fffu);
    CHECK(oracle_flat_search_f16(X, Xq, R, FN, FQ, FD, FK, oi, osc) == 0);
    CHECK(oracle_flat_search(X, Xq, 0, FN, FQ, FD, FK, oi, osc) == 0);
    free(Q); free(C); free(CB); free(codes); free(ids); free(S); free(probes); free(L); free(L8); free(B);
    free(oi); free(ois); free(osc); free(cb16); free(cb256); free(X); free(Xq);
    printf("oracle sanitize check ok\n");
    return 0;
}

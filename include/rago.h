/*
 * rago.h - C ABI of the MI355X (gfx950) retrieval library.
 *
 * The retrieval stage of a RAG pipeline: batched approximate nearest-neighbour search over a
 * product-quantised inverted-file (IVF-PQ) vector database, plus exact brute-force search over
 * small per-request corpora.  Problem statement: return the K most similar database vectors to
 * a D-dimensional query (paper Section 2, "Vector search for retrieval"); IVF-PQ and its
 * byte-per-8-dimensions codes (Section 2; Section 4, "Models and database"); a query scans a
 * P_scan fraction of the database and costs the bytes of PQ codes scanned (Section 3.3,
 * "Retrieval component"); brute-force kNN for 1K-100K vector corpora (Section 5.2).
 * Similarity = inner product (larger is better); on L2-normalised vectors this is cosine.
 *
 * Conventions
 *  - Every function returns RAGO_OK (0) or a negative rago_status.  rago_last_error() gives a
 *    thread-local message for the last failing call on this thread.
 *  - "DEVICE" pointers are HIP device memory on the index's GPU; "HOST" pointers are ordinary
 *    host memory.  The caller owns every buffer it passes and must keep DEVICE buffers alive
 *    until `stream` has passed the call.  The library owns the index and its workspace.
 *  - Search calls only enqueue work on `stream` (a hipStream_t, NULL = default stream).  Argument
 *    errors are detected synchronously and leave the outputs untouched.  Calls on the same index
 *    must be serialised on one stream (they share the index's workspace); so must the flat
 *    searches on one device (they share a per-device workspace: two of them in flight at once,
 *    from different streams or threads, overwrite each other's candidates).
 *  - Workspace: after rago_index_reserve a search within the reserved maxima allocates nothing and
 *    does not synchronise with the host.  Without it the workspace grows on demand: the first call
 *    at a larger size frees and allocates device memory (which synchronises the device and cannot
 *    be captured into a HIP graph); later calls at that size or below do not.
 *  - Nothing here allocates through, links against, or knows about PyTorch.
 */
#ifndef RAGO_H
#define RAGO_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum rago_status {
    RAGO_OK = 0,
    RAGO_INVALID_ARG = -1,   /* null/misaligned pointer, size out of range, nprobe > nlist, ...   */
    RAGO_IO = -2,            /* file cannot be opened / read                                      */
    RAGO_FORMAT = -3,        /* bad magic, truncated file, inconsistent offsets, unsorted ids     */
    RAGO_OOM = -4,           /* host or device allocation failed                                  */
    RAGO_DEVICE = -5,        /* a HIP call failed                                                 */
    RAGO_UNSUPPORTED = -6    /* legal request outside what the kernels are built for              */
} rago_status;

typedef struct rago_index rago_index; /* opaque */

typedef struct rago_index_desc {
    int32_t d;        /* vector dimension                                   */
    int32_t m;        /* PQ sub-quantisers (code bytes per vector = m for ksub 256, m/2 for ksub 16) */
    int32_t ksub;     /* codewords per sub-quantiser: 256 or 16             */
    int32_t nlist;    /* inverted lists / coarse centroids                  */
    int64_t n;        /* database vectors                                   */
    int32_t metric;   /* 0 = inner product, 1 = Euclidean (see rago_index_arrays) */
    int32_t device;   /* HIP device ordinal holding the index               */
    int64_t max_list_len;
    int64_t code_bytes_resident;  /* bytes of the re-laid-out code array in HBM (incl. padding) */
} rago_index_desc;

/* Plain (un-laid-out) IVF-PQ index handed over as arrays; see rago_index_wrap. */
typedef struct rago_index_arrays {
    int32_t d, m, nlist;
    int32_t metric;               /* 0 = inner product (larger is better); 1 = Euclidean: similarity is MINUS the
                                     squared distance to the reconstruction, so larger is better there too and
                                     scores come back <= 0 (Section 2 names both notions)                        */
    int64_t n;
    int32_t ksub;                 /* codewords per sub-quantiser: 256 (0 means 256) = one code byte each, the
                                     paper's configuration (Section 4); 16 = 4-bit codes, two sub-quantisers per
                                     byte, sub-quantiser 2i in the low nibble of byte i and 2i+1 in the high one */
    int32_t reserved;             /* set to 0                                                      */
    const float*   centroids;     /* [nlist][d] fp32                                              */
    const float*   codebooks;     /* [m][ksub][d/m] fp32                                          */
    const int64_t* list_offsets;  /* [nlist+1], list l = rows list_offsets[l] .. list_offsets[l+1] */
    const uint8_t* codes;         /* [n][m] (ksub 256) or [n][m/2] (ksub 16), one row per vector, list-major */
    const int64_t* ids;           /* [n] list-major; unique; ascending inside every list          */
} rago_index_arrays;

/*
 * rago_index_load: read an index file (HOST path) and place it on GPU `device`.
 * File, little-endian: 64-byte header {char magic[8]="RAGOIVPQ", u32 version=1, u32 metric (0 or 1),
 * u32 d, u32 m, u32 ksub (256 or 16), u32 nlist, u64 n, zero pad}, then centroids f32[nlist][d],
 * codebooks f32[m][ksub][d/m], list_offsets i64[nlist+1], codes u8[n][m] (u8[n][m/2] for ksub 16,
 * nibble order as in rago_index_arrays), ids i64[n].  A 4-bit index is searched as the 8-bit index
 * it is equivalent to: a code byte is one symbol of the 256 concatenations of its two sub-quantisers'
 * codewords, so tables, scores and results are those of an index with m/2 sub-quantisers over d/(m/2)
 * dimensions each.
 * The codes are re-laid-out once for the scan (paper Section 4: 96-byte codes, 1 byte per 8
 * dimensions, are what the scan streams).  On success *out owns all device memory.
 * Errors: RAGO_IO, RAGO_FORMAT (incl. truncated), RAGO_UNSUPPORTED (code bytes per vector not in
 * {16,32,64,96,128}, ksub not 256 or 16, d % m != 0, a list longer than 2^31-65 vectors), RAGO_OOM,
 * RAGO_DEVICE.
 */
int rago_index_load(const char* path, int device, rago_index** out);

/*
 * rago_index_wrap: same as rago_index_load but from arrays instead of a file.
 * `arrays_on_device` != 0: all five arrays are DEVICE pointers on `device`; else HOST pointers.
 * The arrays are copied / re-laid-out; the caller may free them when the call returns
 * (the call synchronises the device).  Same errors as rago_index_load minus RAGO_IO.
 */
int rago_index_wrap(const rago_index_arrays* arrays, int arrays_on_device, int device, rago_index** out);

/*
 * rago_index_set_upper_level: give the index an upper level over its lists (the paper's database is
 * a multi-level tree, Section 4): nsuper groups of lists, group s = the lists
 * super_lists[super_offsets[s] .. super_offsets[s+1]) with centroid super_centroids[s].
 *   super_centroids [nsuper][d] fp32, super_offsets [nsuper+1] int64 (0 .. nlist, non-decreasing),
 *   super_lists [nlist] int32: every list exactly once, ascending inside a group;
 *   arrays_on_device as in rago_index_wrap.  The arrays are copied.  nsuper = 0 removes the level.
 * rago_index_set_upper_probe: number of groups a query keeps (nsp).  0 (the default) = score every
 * list centroid as before.  With nsp >= 1 a search scores the nsuper group centroids, keeps the nsp
 * best groups (ties -> lower group), scores only their lists and probes the nprobe best of them
 * (ties -> lower list); lists of other groups count as -inf, so if the kept groups hold fewer than
 * nprobe lists the lowest-numbered other lists fill up.  Errors: RAGO_INVALID_ARG (no upper level,
 * nsp > nsuper, malformed arrays), RAGO_UNSUPPORTED (nsuper > 8192 or nsp * largest group > 8192).
 */
int rago_index_set_upper_level(rago_index* idx, int32_t nsuper, const float* super_centroids, const int64_t* super_offsets,
                               const int32_t* super_lists, int arrays_on_device);
int rago_index_set_upper_probe(rago_index* idx, int32_t nsp);

/*
 * rago_index_reserve: size the index's workspace once for every search with nq <= max_nq,
 * nprobe <= max_nprobe and k <= max_k (either metric's tables, either scan kernel, and the stage
 * through the upper level if the index has one at this point).  Afterwards rago_ivfpq_search within
 * those maxima performs no allocation, free or host synchronisation, and a search beyond them fails
 * with RAGO_UNSUPPORTED and leaves the workspace as it is (reserve again for larger maxima).  The
 * call synchronises the device.  Limits and errors as for rago_ivfpq_search, plus RAGO_OOM.
 */
int rago_index_reserve(rago_index* idx, int64_t max_nq, int32_t max_nprobe, int32_t max_k);

/* Release the index and its workspace (synchronises the device).  NULL is accepted. */
int rago_index_free(rago_index* idx);

/* Fill *out with the index's shape.  HOST pointers. */
int rago_index_info(const rago_index* idx, rago_index_desc* out);

/*
 * rago_ivfpq_search: batched IVF-PQ search (Sections 2 and 3.3): coarse scores of every query
 * against every centroid, the nprobe best lists per query, an 8-bit look-up table per
 * (query, list), an integer asymmetric-distance scan of the lists' codes, best k per query by
 * (integer score descending, id ascending).  Under the Euclidean metric the coarse scores are
 * -|q - c|^2 and the tables -|q_j - (c_j + codeword)|^2; they then no longer split into a
 * per-query and a per-list part, so a full table is computed for every (query, list) pair.
 *   queries     DEVICE [nq][d] fp32 row-major, 16-byte aligned
 *   nq >= 0, 1 <= nprobe <= min(nlist, 2016) (up to 2048 when nprobe = nlist), nq * nprobe <= 2^30, 1 <= k <= 128
 *   (RAGO_INVALID_ARG for nprobe > nlist or k < 1, RAGO_UNSUPPORTED beyond the other limits)
 *   out_ids     DEVICE [nq][k] int64, best first, padded with -1
 *   out_scores  DEVICE [nq][k] fp32 = integer score * the query's table step; pad = -inf
 *   out_iscores DEVICE [nq][k] int32 or NULL; pad = INT32_MIN
 * Workspace: see rago_index_reserve and the conventions at the top.
 * The scan runs one of three kernels, chosen from the batch and list sizes (long tasks with lists
 * shared by several queries: four (query, list) pairs per pass of a list; short lists: one wavefront
 * per (pair, chunk of a list), pairs grouped by query; otherwise two pairs per pass); results are
 * identical (rago_debug_force_scan_kernel pins one of them for tests).
 * ids must ascend inside every list (RAGO_FORMAT at load otherwise): the scan orders equal scores by
 * position in the list, which is the order by id only then; an index writer sorts each list once,
 * where it has the vectors at hand, rather than every load permuting ~100 GB of codes.
 */
int rago_ivfpq_search(rago_index* idx, const float* queries, int64_t nq, int32_t nprobe, int32_t k,
                      int64_t* out_ids, float* out_scores, int32_t* out_iscores, void* stream);

/*
 * rago_flat_search: exact inner-product search of R independent requests, each with its own
 * corpus (brute-force kNN over freshly embedded long-context chunks, Section 5.2).
 *   corpus_bf16  DEVICE [R][n][d] bf16 row-major, 16-byte aligned;  d in {64,128,256,384,512,768,1024}
 *   queries_bf16 DEVICE [R][nqr][d] bf16;  1 <= nqr <= 16
 *   1 <= k <= 128
 *   out_ids      DEVICE [R][nqr][k] int64 row index inside the request's corpus, pad -1
 *   out_scores   DEVICE [R][nqr][k] fp32 (bf16 products, fp32 accumulation), pad -inf
 * Order: score descending, ties by lower index.  `device` = GPU of the buffers.
 * Uses a per-device workspace owned by the library, grown on demand (the first call at a larger
 * R * n allocates, which synchronises the device); flat searches on one device must therefore be
 * serialised on one stream.
 */
int rago_flat_search(const void* corpus_bf16, const void* queries_bf16, int32_t R, int64_t n, int32_t nqr,
                     int32_t d, int32_t k, int64_t* out_ids, float* out_scores, int device, void* stream);

/*
 * rago_flat_search_f16: the same search over IEEE binary16 ("FP16") embeddings, the format in which
 * Section 5.2 caches the vectors of an encoded context for reuse.  corpus_f16 DEVICE [R][n][d] and
 * queries_f16 DEVICE [R][nqr][d] hold binary16 numbers (finite; subnormals keep their value); scores
 * are sums of exact fp16 products accumulated in fp32.  Every other argument, limit, the order of
 * the results and the errors are those of rago_flat_search.
 */
int rago_flat_search_f16(const void* corpus_f16, const void* queries_f16, int32_t R, int64_t n, int32_t nqr,
                         int32_t d, int32_t k, int64_t* out_ids, float* out_scores, int device, void* stream);

/*
 * rago_flat_search_static: rago_flat_search / rago_flat_search_f16 for callers that cannot allocate
 * device memory: code running under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  It performs no allocation, free or host synchronisation on any call, the first
 * included: its scratch memory (candidate keys, counts, threshold bins: 32 MiB + 32 KiB) is a static
 * device array inside the library, which every GPU the library runs on holds until the process ends.
 *   format 0 = bf16, 1 = IEEE binary16; every other argument, the results and their order as in
 *   rago_flat_search.  Limit: R <= 256 requests per call (RAGO_UNSUPPORTED beyond; split the batch).
 *   The corpus is cut into at most 256 / R slabs per request (512 / R in rago_flat_search), so large
 *   calls run on half as many workgroups.
 * All calls on one GPU share that array: calls that overlap on one GPU (different streams or
 * threads) race; serialise them on one stream.  Nothing needs clearing between calls (the call
 * zeroes the threshold bins itself, with a kernel, so it can be captured into a HIP graph).
 */
int rago_flat_search_static(const void* corpus, const void* queries, int32_t R, int64_t n, int32_t nqr, int32_t d,
                            int32_t k, int32_t format, int64_t* out_ids, float* out_scores, int device, void* stream);

/* Thread-local message of the last error on this thread ("" if none). */
const char* rago_last_error(void);

/* ---- stage-isolated entry points (same kernels as rago_ivfpq_search, one stage each) ---- */

/* Coarse scores S[q][l] = <Q[q], C[l]> (fp32 MFMA; from 128 queries up bf16 MFMA on operands split
 * into two bf16 terms; either way within 1e-4 |q||c| of the exact product).  out_S DEVICE [nq][nlist] fp32. */
int rago_debug_coarse(rago_index* idx, const float* queries, int64_t nq, float* out_S, void* stream);

/* Probes through the upper level (rago_index_set_upper_probe >= 1), the stage the search then runs
 * instead of the two above.  out_probes DEVICE [nq][nprobe] int32; out_groups DEVICE [nq][nsp] int32 or NULL. */
int rago_debug_select_tree(rago_index* idx, const float* queries, int64_t nq, int32_t nprobe, int32_t* out_probes,
                           int32_t* out_groups, void* stream);

/* The nprobe best lists per query, best first, ties by lower list number.  Scores of the lists
 * near the cut are recomputed in fp64 from `queries`, and a query whose scores are packed more
 * closely around the cut than the rounding error of S is selected again on exact scores of all
 * lists, so the choice never depends on the rounding of S.
 * S DEVICE [nq][nlist] (not modified); out_probes DEVICE [nq][nprobe] int32. */
int rago_debug_select(rago_index* idx, const float* queries, const float* S, int64_t nq, int32_t nprobe,
                      int32_t* out_probes, void* stream);

/* Look-up tables for given probes.  probes DEVICE [nq][nprobe] int32 (valid list numbers).
 * Here and in rago_debug_scan, m counts CODE BYTES per vector (half the sub-quantisers of a 4-bit index).
 * out_L_f32 DEVICE [nq][nprobe][m][256] fp32 or NULL; out_LUT8 DEVICE [nq][nprobe][m][256] u8 or
 * NULL; out_B DEVICE [nq][nprobe] int32 or NULL; out_delta DEVICE [nq] fp32 or NULL. */
int rago_debug_build_lut(rago_index* idx, const float* queries, const int32_t* probes, int64_t nq,
                         int32_t nprobe, float* out_L_f32, uint8_t* out_LUT8, int32_t* out_B,
                         float* out_delta, void* stream);

/* Integer scan + top-k with caller-supplied tables: LUT8 DEVICE [nq][nprobe][m][256] u8,
 * B DEVICE [nq][nprobe] int32.  Outputs as rago_ivfpq_search (scores omitted). */
int rago_debug_scan(rago_index* idx, const int32_t* probes, const uint8_t* LUT8, const int32_t* B,
                    int64_t nq, int32_t nprobe, int32_t k, int64_t* out_ids, int32_t* out_iscores,
                    void* stream);

/* Counters of the last search on this index, HOST out[8] (synchronises `stream`):
 * [0] scan tasks (the wavefront-per-item kernel: items), [1] code bytes streamed by the scan (a pass
 * over a list serves up to four, two or one of its pairs, by kernel), [2] algorithmic code bytes
 * (sum over (query, probe) of list length * m), [3] queries whose probe choice had to be made on
 * exact scores of all lists (it could not be shown independent of fp32 rounding otherwise), [4] table entries whose rounding had to be evaluated per
 * (query, list) pair (summed over queries), [5] queries whose tables were evaluated entry by entry
 * for every pair (Euclidean metric: [4] entries re-evaluated in fp64 over both table passes, [5]
 * workgroups that re-evaluated all their entries, counted once per pass), [6] the scan kernel that ran, numbered
 * as in rago_debug_force_scan_kernel (1, 2 or 3), [7] reserved. */
int rago_debug_counters(rago_index* idx, int64_t* out, void* stream);

/* Pin the scan kernel of every following search in this process: 0 = chosen from the sizes (default),
 * 1 = the four-pairs-per-pass kernel, 2 = the two-pairs-per-pass kernel, 3 = the kernel with one
 * wavefront per (pair, chunk) (chosen by itself only for short lists with per-query base tables;
 * when pinned with full tables per pair - Euclidean metric, rago_debug_scan - a workgroup installs
 * each pair's table in turn).  RAGO_INVALID_ARG for other values.  For tests. */
int rago_debug_force_scan_kernel(int which);

/* Number of device allocations the library's workspaces have made in this process so far (a test
 * reads it before and after searches that must not allocate). */
int64_t rago_debug_allocations(void);

/* Plain copy kernel (rago_calib_copy_kernel) of `bytes` bytes, DEVICE src -> DEVICE dst, both
 * 16-byte aligned, bytes % 16 == 0, on the current device: a transfer of known size against which
 * hardware HBM byte counters are calibrated when the scan is profiled. */
int rago_debug_copy(const void* src, void* dst, int64_t bytes, void* stream);

/* Plain read stream (rago_calib_read_kernel) over `bytes` bytes of DEVICE src (16-byte aligned,
 * bytes % 16 == 0) on the current device: the rate a kernel that only reads HBM reaches, i.e. the
 * practical ceiling the scans are measured against besides the 8 TB/s peak (Section 4, "Retrieval
 * performance modeling": a good code scan reaches ~80 % of the memory bandwidth).  sink DEVICE
 * [4096] uint32 receives the XOR of what each workgroup read (so the loads are not dropped). */
int rago_debug_read_stream(const void* src, int64_t bytes, uint32_t* sink, void* stream);

/* Per-stage timing of rago_ivfpq_search with HIP events recorded on the caller's stream.
 * rago_debug_profile(idx, 1) starts (and resets) recording for up to 64 following search calls,
 * (idx, 0) stops it.  rago_debug_stage_ms waits for the recorded calls and returns, averaged over
 * them, HOST out_ms[8] = {coarse GEMM, selection, table build, scan bookkeeping, scan kernel,
 * merge, whole call, 0} in milliseconds and *out_calls = number of calls averaged. */
int rago_debug_profile(rago_index* idx, int enable);
int rago_debug_stage_ms(rago_index* idx, float* out_ms, int32_t* out_calls);

/* The same for the flat searches on `device`: rago_debug_flat_profile(device, 1) starts (and resets)
 * recording for up to 128 following rago_flat_search / rago_flat_search_f16 calls, (device, 0) stops
 * it; rago_debug_flat_stage_ms waits for them and returns HOST out_ms[2] = {scan kernel, merge
 * kernel} in milliseconds averaged over *out_calls calls. */
int rago_debug_flat_profile(int device, int enable);
int rago_debug_flat_stage_ms(int device, float* out_ms, int32_t* out_calls);

#ifdef __cplusplus
}
#endif
#endif /* RAGO_H */

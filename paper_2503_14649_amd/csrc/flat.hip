// Exact inner-product search over small per-request corpora: brute-force kNN on freshly embedded
// long-context chunks (Section 5.2: 1K-100K 768-d vectors per request, no index because the
// embeddings are new).  s[r][q][i] = <Q_r[q], X_r[i]>, bf16 inputs, fp32 accumulation, best k per
// (request, query) by (score descending, row ascending).
//
// The work is one pass over the corpus, 2*d bytes per row for up to 16 queries, i.e. 16 flop/byte:
// HBM-bound, the MFMA only keeps the arithmetic off the vector ALUs.
//  * v_mfma_f32_16x16x32_bf16: M = 16 corpus rows, N = 16 queries of the request, K = 32.
//    Lane (i = lane%16, g = lane/16) supplies 8 bf16 of row i; both operands use the same
//    lane -> k mapping, and k may be permuted freely inside the sum, so every lane loads 32
//    contiguous bytes per 128-byte row segment (two dwordx4, two MFMA steps): each cache line is
//    consumed whole by four lanes in back-to-back instructions.
//  * queries sit in LDS (row stride padded by 16 B so the 16 query rows fall in different banks).
//  * a workgroup (4 waves) streams one slab of one request; a wave takes 16-row blocks, the next
//    block's 24 loads are in flight while the current block is multiplied.
//  * selection: 64-bit keys (ordered score bits << 32 | ~row) appended to per-query LDS buffers
//    when they reach the query's running threshold; every 256 rows the workgroup synchronises and
//    prunes buffers that grew beyond k with a wave-level radix select, which also raises the
//    threshold.  Each slab writes <= k keys per query; a second kernel merges the slabs.
#include "rago_internal.h"

namespace rago {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;

constexpr int FLAT_THREADS = 256;
constexpr int FLAT_WAVES = 4;
constexpr int FLAT_RB = 4;                                  // 16-row blocks per wave between barriers
constexpr int FLAT_ROUND_ROWS = FLAT_WAVES * FLAT_RB * 16;  // 256 rows per workgroup round
constexpr int FLAT_MAXD = 1024;

__device__ __forceinline__ uint32_t fkey(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float fkey_inv(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}
__device__ __forceinline__ int lane_rank64(uint64_t mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

// k-th largest of up to NR*64 non-zero 64-bit keys held NR per lane (wave-uniform result).
template <int NR>
__device__ __forceinline__ uint64_t select_kth64(const uint64_t (&r)[NR], int k) {
    uint64_t prefix = 0;
    int rem = k;
    for (int bit = 63; bit >= 0; --bit) {
        const uint64_t test = prefix | (1ull << bit);
        const uint64_t hm = ~((1ull << bit) - 1ull);
        int c1 = 0;
#pragma unroll
        for (int i = 0; i < NR; ++i) c1 += __popcll(__ballot((r[i] & hm) == test));
        if (c1 >= rem) prefix = test; else rem -= c1;
    }
    return prefix;
}

constexpr int FLAT_NR = (KMAX + FLAT_ROUND_ROWS + 63) / 64;   // registers per lane to hold a full buffer

// Keep the best k of buf[0..cnt) (cnt > k); returns the k-th key.
__device__ __forceinline__ uint64_t prune64(uint64_t* buf, int cnt, int k, int lane) {
    uint64_t r[FLAT_NR];
#pragma unroll
    for (int i = 0; i < FLAT_NR; ++i) r[i] = (lane + 64 * i < cnt) ? buf[lane + 64 * i] : 0ull;
    const uint64_t kth = select_kth64<FLAT_NR>(r, k);
    int base = 0;
#pragma unroll
    for (int i = 0; i < FLAT_NR; ++i) {
        const bool keep = r[i] >= kth && r[i] != 0ull;
        const uint64_t mask = __ballot(keep);
        if (keep) buf[base + lane_rank64(mask)] = r[i];
        base += __popcll(mask);
    }
    return kth;
}

struct FlatParams {
    const uint16_t* corpus;   // [R][n][d] bf16
    const uint16_t* queries;  // [R][nqr][d] bf16
    int64_t n;
    int R, nqr, d, k, nslab;
    int64_t slab_rows;        // rows per slab (multiple of 16)
    uint64_t* part_keys;      // [R][nslab][16][k]
    int32_t* part_cnt;        // [R][nslab][16]
};

template <int D>
__global__ void __launch_bounds__(FLAT_THREADS, 2) flat_scan_kernel(const FlatParams P) {
    constexpr int NP = D / 64;              // 128-byte segments per row
    constexpr int QS = D * 2 + 16;          // padded query row stride in LDS (bytes)
    extern __shared__ __align__(16) uint8_t smem[];
    uint8_t* qs = smem;                                               // 16 * QS
    const int capq = P.k + FLAT_ROUND_ROWS;
    uint64_t* bufs = reinterpret_cast<uint64_t*>(smem + 16 * QS);     // [16][capq]
    int32_t* cnt = reinterpret_cast<int32_t*>(bufs + 16 * capq);      // [16]
    uint32_t* thr = reinterpret_cast<uint32_t*>(cnt + 16);            // [16] ordered score bits
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i16 = lane & 15, g = lane >> 4;
    const int r = blockIdx.x / P.nslab, slab = blockIdx.x % P.nslab;
    const int64_t row0 = (int64_t)slab * P.slab_rows;
    const int64_t row1 = min(P.n, row0 + P.slab_rows);

    // queries of this request into LDS (zero rows beyond nqr)
    for (int idx = tid; idx < 16 * (D / 8); idx += FLAT_THREADS) {
        const int qrow = idx / (D / 8), c = idx % (D / 8);
        uint4 v = make_uint4(0, 0, 0, 0);
        if (qrow < P.nqr) v = *reinterpret_cast<const uint4*>(P.queries + ((int64_t)r * P.nqr + qrow) * D + c * 8);
        *reinterpret_cast<uint4*>(qs + qrow * QS + c * 16) = v;
    }
    if (tid < 16) { cnt[tid] = 0; thr[tid] = 0u; }
    __syncthreads();

    const uint16_t* X = P.corpus + (int64_t)r * P.n * D;
    uint4 a[2 * NP], an[2 * NP];
    auto load_rows = [&](uint4 (&dst)[2 * NP], int64_t rb) {   // rb = first row of a 16-row block
        const int64_t row = min(rb + i16, P.n - 1);
        const uint4* p = reinterpret_cast<const uint4*>(X + row * D + g * 16);
#pragma unroll
        for (int sp = 0; sp < NP; ++sp) { dst[2 * sp] = p[sp * 8]; dst[2 * sp + 1] = p[sp * 8 + 1]; }
    };
    auto multiply = [&](const uint4 (&src)[2 * NP], int64_t rb) {
        v4f acc = {0.f, 0.f, 0.f, 0.f};
        const uint8_t* qrow = qs + i16 * QS + g * 32;
#pragma unroll
        for (int sp = 0; sp < NP; ++sp) {
            const uint4 b0 = *reinterpret_cast<const uint4*>(qrow + sp * 128);
            const uint4 b1 = *reinterpret_cast<const uint4*>(qrow + sp * 128 + 16);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, src[2 * sp]), __builtin_bit_cast(bf16x8, b0), acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, src[2 * sp + 1]), __builtin_bit_cast(bf16x8, b1), acc, 0, 0, 0);
        }
        // acc[e] = score of row rb + 4*g + e with query i16
        const uint32_t t = thr[i16];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int64_t row = rb + 4 * g + e;
            const uint32_t key = fkey(acc[e]);
            if (row < row1 && i16 < P.nqr && key >= t) {
                const int pos = atomicAdd(&cnt[i16], 1);
                bufs[i16 * capq + pos] = ((uint64_t)key << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)row);
            }
        }
    };

    // rounds of 256 rows: wave w owns blocks w*FLAT_RB .. +FLAT_RB of the round
    int64_t rb = row0 + (int64_t)wave * FLAT_RB * 16;
    if (rb < row1) load_rows(a, rb);
    for (int64_t round0 = row0; round0 < row1; round0 += FLAT_ROUND_ROWS) {
#pragma unroll 1
        for (int bb = 0; bb < FLAT_RB; bb += 2) {
            const int64_t r0 = round0 + ((int64_t)wave * FLAT_RB + bb) * 16, r1 = r0 + 16;
            int64_t r2 = r0 + 32;
            if (bb + 2 >= FLAT_RB) r2 = round0 + FLAT_ROUND_ROWS + (int64_t)wave * FLAT_RB * 16;   // first block of next round
            if (r1 < row1) load_rows(an, r1);
            if (r0 < row1) multiply(a, r0);
            if (r2 < row1) load_rows(a, r2);
            if (r1 < row1) multiply(an, r1);
        }
        __syncthreads();
        // buffers that can no longer absorb a full round are cut back to the best k
        for (int qj = wave; qj < P.nqr; qj += FLAT_WAVES) {
            const int c = cnt[qj];
            if (c > P.k) {
                const uint64_t kth = prune64(bufs + qj * capq, c, P.k, lane);
                if (lane == 0) { cnt[qj] = P.k; thr[qj] = (uint32_t)(kth >> 32); }
            }
        }
        __syncthreads();
    }
    // slab result
    const int64_t pbase = ((int64_t)r * P.nslab + slab) * 16;
    for (int qj = wave; qj < P.nqr; qj += FLAT_WAVES) {
        const int c = cnt[qj];
        for (int e = lane; e < c; e += 64) P.part_keys[(pbase + qj) * P.k + e] = bufs[qj * capq + e];
        if (lane == 0) P.part_cnt[pbase + qj] = c;
    }
}

// One workgroup per (request, query): sort the slabs' keys descending, write the best k.
constexpr int FM_THREADS = 256;
__global__ void __launch_bounds__(FM_THREADS) flat_merge_kernel(const FlatParams P, int n2, int64_t* __restrict__ out_ids,
                                                                float* __restrict__ out_scores) {
    extern __shared__ __align__(16) uint8_t smem[];
    uint64_t* keys = reinterpret_cast<uint64_t*>(smem);   // [n2]
    __shared__ int s_cnt;
    const int r = blockIdx.x / P.nqr, q = blockIdx.x % P.nqr;
    if (threadIdx.x == 0) s_cnt = 0;
    for (int i = threadIdx.x; i < n2; i += FM_THREADS) keys[i] = 0ull;
    __syncthreads();
    for (int e = threadIdx.x; e < P.nslab * P.k; e += FM_THREADS) {
        const int slab = e / P.k, j = e % P.k;
        const int64_t pb = ((int64_t)r * P.nslab + slab) * 16 + q;
        if (j < P.part_cnt[pb]) keys[atomicAdd(&s_cnt, 1)] = P.part_keys[pb * P.k + j];
    }
    for (int size = 2; size <= n2; size <<= 1)
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            for (int t = threadIdx.x; t < n2 / 2; t += FM_THREADS) {
                const int i = 2 * t - (t & (stride - 1)), j = i + stride;
                const bool desc = (i & size) == 0;
                const uint64_t a = keys[i], b = keys[j];
                if (desc ? (b > a) : (a > b)) { keys[i] = b; keys[j] = a; }
            }
        }
    __syncthreads();
    const int have = min(s_cnt, P.k);
    for (int j = threadIdx.x; j < P.k; j += FM_THREADS) {
        const int64_t o = ((int64_t)r * P.nqr + q) * P.k + j;
        if (j < have) {
            out_ids[o] = (int64_t)(0xFFFFFFFFu - (uint32_t)keys[j]);
            out_scores[o] = fkey_inv((uint32_t)(keys[j] >> 32));
        } else {
            out_ids[o] = -1;
            out_scores[o] = -INFINITY;
        }
    }
}

static DevBuf g_flat_keys[16], g_flat_cnt[16];

template <int D>
static int launch_flat_d(const FlatParams& P, int grid, size_t lds, hipStream_t st) {
    static bool attr_done = false;
    if (!attr_done) {
        RAGO_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(flat_scan_kernel<D>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, 16 * (D * 2 + 16) + 16 * (KMAX + FLAT_ROUND_ROWS) * 8 + 128));
        attr_done = true;
    }
    flat_scan_kernel<D><<<grid, FLAT_THREADS, lds, st>>>(P);
    RAGO_HIP(hipGetLastError());
    return RAGO_OK;
}

int launch_flat(const void* corpus, const void* queries, int R, int64_t n, int nqr, int d, int k, int64_t* out_ids,
                float* out_scores, int device, hipStream_t st) {
    if (device < 0 || device >= 16) return fail(RAGO_INVALID_ARG, "device ordinal out of range");
    if (d % 64 || d > FLAT_MAXD) return fail(RAGO_UNSUPPORTED, "d must be a multiple of 64, at most 1024");
    FlatParams P;
    P.corpus = static_cast<const uint16_t*>(corpus);
    P.queries = static_cast<const uint16_t*>(queries);
    P.n = n; P.R = R; P.nqr = nqr; P.d = d; P.k = k;
    // slabs: ~1024 workgroups in total, at least one round each, merge fits 4096 keys
    int nslab = (int)std::min<int64_t>((1024 + R - 1) / R, (n + FLAT_ROUND_ROWS - 1) / FLAT_ROUND_ROWS);
    nslab = std::max(1, std::min(nslab, 4096 / k));
    int64_t slab_rows = (n + nslab - 1) / nslab;
    slab_rows = (slab_rows + FLAT_ROUND_ROWS - 1) / FLAT_ROUND_ROWS * FLAT_ROUND_ROWS;
    if (slab_rows == 0) slab_rows = FLAT_ROUND_ROWS;
    nslab = (int)std::max<int64_t>(1, (n + slab_rows - 1) / slab_rows);
    P.nslab = nslab; P.slab_rows = slab_rows;
    int rc;
    if ((rc = g_flat_keys[device].reserve((size_t)R * nslab * 16 * k * 8))) return rc;
    if ((rc = g_flat_cnt[device].reserve((size_t)R * nslab * 16 * 4))) return rc;
    P.part_keys = g_flat_keys[device].as<uint64_t>();
    P.part_cnt = g_flat_cnt[device].as<int32_t>();
    const size_t lds = 16 * (size_t)(d * 2 + 16) + 16 * (size_t)(k + FLAT_ROUND_ROWS) * 8 + 128;
    const int grid = R * nslab;
    switch (d) {
        case 64: rc = launch_flat_d<64>(P, grid, lds, st); break;
        case 128: rc = launch_flat_d<128>(P, grid, lds, st); break;
        case 256: rc = launch_flat_d<256>(P, grid, lds, st); break;
        case 384: rc = launch_flat_d<384>(P, grid, lds, st); break;
        case 512: rc = launch_flat_d<512>(P, grid, lds, st); break;
        case 768: rc = launch_flat_d<768>(P, grid, lds, st); break;
        case 1024: rc = launch_flat_d<1024>(P, grid, lds, st); break;
        default: return fail(RAGO_UNSUPPORTED, "d must be one of 64, 128, 256, 384, 512, 768, 1024");
    }
    if (rc) return rc;
    int n2 = 2;
    while (n2 < nslab * k) n2 <<= 1;
    flat_merge_kernel<<<R * nqr, FM_THREADS, (size_t)n2 * 8, st>>>(P, n2, out_ids, out_scores);
    RAGO_HIP(hipGetLastError());
    return RAGO_OK;
}

}  // namespace rago

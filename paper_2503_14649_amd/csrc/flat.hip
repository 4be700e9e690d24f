// Exact inner-product search over small per-request corpora: brute-force kNN on freshly embedded
// long-context chunks (Section 5.2: 1K-100K 768-d vectors per request, no index because the
// embeddings are new).  s[r][q][i] = <Q_r[q], X_r[i]>, bf16 inputs, fp32 accumulation, best k per
// (request, query) by (score descending, row ascending).
//
// The work is one pass over the corpus, 2*d bytes per row for up to 16 queries, i.e. 16 flop/byte:
// HBM-bound, the MFMA only keeps the arithmetic off the vector ALUs.
//  * v_mfma_f32_16x16x32_bf16: M = 16 corpus rows, N = 16 queries of the request, K = 32.
//    Lane (i = lane%16, g = lane/16) supplies 8 bf16 of row i; both operands use the same
//    lane -> k mapping, and k may be permuted freely inside the sum, so the four lanes of a row
//    load 64 contiguous bytes per instruction and the two halves of each 128-byte row segment are
//    consumed by back-to-back instructions (two dwordx4 per lane, two MFMA steps).
//  * queries sit in LDS (row stride padded by 16 B so the 16 query rows fall in different banks).
//  * a workgroup (4 waves) streams one slab of one request; a wave takes 16-row blocks, one in
//    registers at a time (its 24 loads are issued right after the previous block's multiply).
//  * selection: a score is a candidate when its histogram bin (width 1/128) is not below the
//    query's threshold bin; in the stream that is four compares and one wave-uniform branch per
//    block.  A candidate first goes to the wave's staging area in LDS (positions from ballots, so
//    nothing is waited for); at the end of a round the wave appends its staged candidates as 64-bit
//    keys (ordered score bits << 32 | ~row) to a per-(slab, query) area in HBM and counts them in
//    a per-query LDS histogram (atomics and stores with all lanes busy instead of one or two).  Every 256
//    rows the workgroup synchronises and 16 lanes move each query's threshold to the highest bin
//    that still has k candidates at or above it, so after the first round only ~k/round new keys
//    appear.  An area that could overflow is cut back to its best k with a wave-level radix select
//    (rare).  Each slab leaves <= k keys per query; a second kernel merges the slabs.
#include <mutex>

#include "rago_internal.h"

namespace rago {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// One 16x16x32 product-accumulate on eight 16-bit numbers per lane and operand: bf16, or IEEE
// binary16 (the format of the embedding cache of Section 5.2) when HALF.
template <bool HALF>
__device__ __forceinline__ v4f mma16(const uint4& a, const uint4& b, v4f acc) {
    if constexpr (HALF) return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), acc, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}

constexpr int FLAT_THREADS = 256;
constexpr int FLAT_WAVES = 4;
constexpr int FLAT_RB = 4;                                  // 16-row blocks per wave between barriers
constexpr int FLAT_ROUND_ROWS = FLAT_WAVES * FLAT_RB * 16;  // 256 rows per workgroup round
constexpr int FLAT_MAXD = 1024;
constexpr int FLAT_CAP = 1024;                              // candidate keys per (slab, query) in the HBM scratch
constexpr int FLAT_BINS = 256;                              // score histogram bins per query
constexpr int FLAT_CHUNKS = 2;                              // a block is multiplied and re-requested in this many pieces
constexpr int FLAT_STAGE = 1024;                            // staged candidates per wave (LDS), flushed past 768 or at a round's end
constexpr size_t flat_lds_bytes(int d) { return 16 * (size_t)(d * 2 + 16) + 16 * FLAT_BINS * 2 + 256 + (size_t)FLAT_WAVES * FLAT_STAGE * 8; }

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
// Monotone map of a score to a histogram bin (bins of width 1/128 over [-1, 1], clamped: for
// unit-norm embeddings every score falls inside; outside it the filter only gets coarser).
__device__ __forceinline__ int score_bin(float s) {
    const float x = (s + 1.0f) * 128.0f;
    return x <= 0.0f ? 0 : (x >= 255.0f ? 255 : (int)x);
}

// k-th largest of up to NR*64 non-zero 64-bit keys held NR per lane (wave-uniform result).
// Two 32-bit radix selects: first on the score half; the row half only among keys that tie on
// the k-th score, and only if not all of them are wanted.
template <int NR>
__device__ __forceinline__ uint64_t select_kth64(const uint64_t (&r)[NR], int k) {
    uint32_t prefix = 0;
    int rem = k;
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t test = prefix | (1u << bit);
        const uint32_t hm = ~((1u << bit) - 1u);
        int c1 = 0;
#pragma unroll
        for (int i = 0; i < NR; ++i) c1 += __popcll(__ballot(r[i] != 0ull && ((uint32_t)(r[i] >> 32) & hm) == test));
        if (c1 >= rem) prefix = test; else rem -= c1;
    }
    // rem of the keys whose score half equals prefix are wanted (those with the lowest rows)
    int ties = 0;
#pragma unroll
    for (int i = 0; i < NR; ++i) ties += __popcll(__ballot(r[i] != 0ull && (uint32_t)(r[i] >> 32) == prefix));
    uint32_t low = 0;
    if (ties > rem) {
        for (int bit = 31; bit >= 0; --bit) {
            const uint32_t test = low | (1u << bit);
            const uint32_t hm = ~((1u << bit) - 1u);
            int c1 = 0;
#pragma unroll
            for (int i = 0; i < NR; ++i) c1 += __popcll(__ballot(r[i] != 0ull && (uint32_t)(r[i] >> 32) == prefix && ((uint32_t)r[i] & hm) == test));
            if (c1 >= rem) low = test; else rem -= c1;
        }
    }
    return ((uint64_t)prefix << 32) | low;
}

// Keep the best k of buf[0..cnt) (k < cnt <= NR*64), compacted to buf[0..k).
template <int NR>
__device__ __forceinline__ void prune64_n(uint64_t* buf, int cnt, int k, int lane) {
    uint64_t r[NR];
#pragma unroll
    for (int i = 0; i < NR; ++i)   // read at device scope: other waves of the workgroup wrote these keys
        r[i] = (lane + 64 * i < cnt) ? __hip_atomic_load(buf + lane + 64 * i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0ull;
    const uint64_t kth = select_kth64<NR>(r, k);
    int base = 0;
#pragma unroll
    for (int i = 0; i < NR; ++i) {
        const bool keep = r[i] >= kth && r[i] != 0ull;
        const uint64_t mask = __ballot(keep);
        if (keep) buf[base + lane_rank64(mask)] = r[i];
        base += __popcll(mask);
    }
}

__device__ __forceinline__ void prune64(uint64_t* buf, int cnt, int k, int lane) {
    if (cnt <= 5 * 64) prune64_n<5>(buf, cnt, k, lane);
    else prune64_n<FLAT_CAP / 64>(buf, cnt, k, lane);
}

struct FlatParams {
    const uint16_t* corpus;   // [R][n][d] bf16
    const uint16_t* queries;  // [R][nqr][d] bf16
    int64_t n;
    int R, nqr, d, k, nslab;
    int64_t slab_rows;        // rows per slab (multiple of 16)
    uint64_t* cand;           // [R][nslab][16][FLAT_CAP] candidate keys of each slab (its first k = the slab's result)
    int32_t* part_cnt;        // [R][nslab][16]
    int32_t* shared_tbin;     // [R][16] threshold bin reached by any slab of the request (zeroed at the start of every call)
};

typedef uint32_t f_u32x4 __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(1))) f_u32x4* f_global_ptr;

template <int D, bool HALF>
__global__ void __launch_bounds__(FLAT_THREADS, 2) flat_scan_kernel(const FlatParams P) {
    constexpr int NP = D / 64;              // 128-byte segments per row
    constexpr int QS = D * 2 + 16;          // padded query row stride in LDS (bytes)
    extern __shared__ __align__(16) uint8_t smem[];
    uint8_t* qs = smem;                                                       // 16 * QS
    uint16_t* hist = reinterpret_cast<uint16_t*>(smem + 16 * QS);             // [16][FLAT_BINS] candidates per score bin
    int32_t* cnt = reinterpret_cast<int32_t*>(hist + 16 * FLAT_BINS);         // [16]
    int32_t* tbin = cnt + 16;                                                 // [16] lowest bin that can still hold a top-k score
    uint64_t* stage = reinterpret_cast<uint64_t*>(smem + 16 * QS + 16 * FLAT_BINS * 2 + 256) + (threadIdx.x >> 6) * FLAT_STAGE;   // this wave's
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i16 = lane & 15, g = lane >> 4;
    const int r = blockIdx.x / P.nslab, slab = blockIdx.x % P.nslab;
    const int64_t row0 = (int64_t)slab * P.slab_rows;
    const int64_t row1 = min(P.n, row0 + P.slab_rows);
    const int64_t pbase = ((int64_t)r * P.nslab + slab) * 16;
    uint64_t* mycand = P.cand + pbase * FLAT_CAP;

    // queries of this request into LDS (zero rows beyond nqr)
    for (int idx = tid; idx < 16 * (D / 8); idx += FLAT_THREADS) {
        const int qrow = idx / (D / 8), c = idx % (D / 8);
        uint4 v = make_uint4(0, 0, 0, 0);
        if (qrow < P.nqr) v = *reinterpret_cast<const uint4*>(P.queries + ((int64_t)r * P.nqr + qrow) * D + c * 8);
        *reinterpret_cast<uint4*>(qs + qrow * QS + c * 16) = v;
    }
    for (int idx = tid; idx < 16 * FLAT_BINS; idx += FLAT_THREADS) hist[idx] = 0;
    // A slab that starts after others of its request have made progress takes over the bin they have reached.
    if (tid < 16) {
        cnt[tid] = 0;
        tbin[tid] = tid < P.nqr ? __hip_atomic_load(P.shared_tbin + r * 16 + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0;
    }
    __syncthreads();

    const uint16_t* X = P.corpus + (int64_t)r * P.n * D;
    const float never = __builtin_huge_valf();
    float thrx = i16 < P.nqr ? (tbin[i16] > 0 ? (float)tbin[i16] : -never) : never;   // this lane's query: threshold bin as a float, -inf while it is bin 0
    int nstage = 0;                              // candidates in this wave's staging area (wave-uniform)
    int64_t round_base = row0;                   // first row of the current round
    uint4 a[2 * NP];
    // loads are unconditional (row clamped into the corpus): a conditional prefetch would make the
    // compiler wait for every outstanding load before each use
    // Load layout: lane l fetches 16 bytes of row l / 8 at byte (l % 8) * 16 of a 128-byte segment, so one load
    // instruction asks for whole 128-byte lines of 8 rows, and two instructions (rows 0..7 -> A, rows 8..15 -> B) cover
    // a segment of the block.  Whole lines in one instruction let the loads be non-temporal (a line is used once and
    // not kept), which is what a plain read stream needs to reach its best rate; and the address unit looks up 8
    // cache tags per instruction.  (In the matrix unit's own operand layout, row = lane % 16, the four lanes the
    // address unit handles together belong to four different rows and every instruction costs 64 tag lookups:
    // counters showed the address unit stalled behind the cache for 80 % of the kernel, and non-temporal loads,
    // each touching half a line, measured 8 % slower than ordinary ones.)
    // The matrix unit wants lane (i16, g) to hold bytes g * 16 .. + 16 of one 64-byte half of row i16's segment.
    // For the first half these sit in A's lanes with l % 8 < 4 (rows 0..7) and in B's (rows 8..15).  One DPP move
    // folds both into one register: A's value stays in the lanes that loaded the first half, B's first-half values
    // shift by four lanes into the lanes that loaded the second half; one lane permutation through the LDS crossbar
    // (no LDS memory) then puts every value into its operand lane.  The second half mirrors this.
    const int lrow = lane >> 3, lc = lane & 7;
    const bool upper = i16 >= 8;
    const int take0 = ((i16 & 7) * 8 + g + (upper ? 4 : 0)) << 2, take1 = ((i16 & 7) * 8 + g + (upper ? 0 : 4)) << 2;
    // loads are unconditional (rows clamped into the corpus): a conditional prefetch would make the
    // compiler wait for every outstanding load before each use
    auto load_rows = [&](uint4 (&dst)[2 * NP], int64_t rb, int sp0, int sp1) {   // rb = first row of a 16-row block
        const int64_t rowa = max((int64_t)0, min(rb + lrow, P.n - 1));
        const int64_t rowb = max((int64_t)0, min(rb + 8 + lrow, P.n - 1));
        f_global_ptr pa = (f_global_ptr)(reinterpret_cast<const f_u32x4*>(X + rowa * D + lc * 8));
        f_global_ptr pb = (f_global_ptr)(reinterpret_cast<const f_u32x4*>(X + rowb * D + lc * 8));
#pragma unroll
        for (int sp = 0; sp < NP; ++sp) {
            if (sp < sp0 || sp >= sp1) continue;
            const f_u32x4 v0 = __builtin_nontemporal_load(pa + sp * 8), v1 = __builtin_nontemporal_load(pb + sp * 8);
            dst[2 * sp] = make_uint4(v0.x, v0.y, v0.z, v0.w);
            dst[2 * sp + 1] = make_uint4(v1.x, v1.y, v1.z, v1.w);
        }
    };
    auto first_half = [&](uint32_t a, uint32_t b) {      // row_shr:4 into lanes 4..7 and 12..15 of every 16
        return (uint32_t)__builtin_amdgcn_ds_bpermute(take0, __builtin_amdgcn_update_dpp((int)a, (int)b, 0x114, 0xF, 0xA, false));
    };
    auto second_half = [&](uint32_t a, uint32_t b) {     // row_shl:4 into lanes 0..3 and 8..11 of every 16
        return (uint32_t)__builtin_amdgcn_ds_bpermute(take1, __builtin_amdgcn_update_dpp((int)a, (int)b, 0x104, 0xF, 0x5, false));
    };
    auto multiply = [&](const uint4 (&src)[2 * NP], v4f acc, int sp0, int sp1) {
        const uint8_t* qrow = qs + i16 * QS + g * 16;
#pragma unroll
        for (int sp = 0; sp < NP; ++sp) {
            if (sp < sp0 || sp >= sp1) continue;
            const uint4 b0 = *reinterpret_cast<const uint4*>(qrow + sp * 128);
            const uint4 b1 = *reinterpret_cast<const uint4*>(qrow + sp * 128 + 64);
            const uint4 &A = src[2 * sp], &B = src[2 * sp + 1];
            acc = mma16<HALF>(make_uint4(first_half(A.x, B.x), first_half(A.y, B.y), first_half(A.z, B.z), first_half(A.w, B.w)), b0, acc);
            acc = mma16<HALF>(make_uint4(second_half(A.x, B.x), second_half(A.y, B.y), second_half(A.z, B.z), second_half(A.w, B.w)), b1, acc);
        }
        return acc;
    };
    auto select = [&](const v4f acc, int64_t rb) {
        // acc[e] = score of row rb + 4*g + e with query i16.  A score is a candidate when its bin is not
        // below the query's threshold bin, i.e. (for a threshold >= 1) when x = (s + 1) * 128 >= threshold:
        // the same x the bin is the integer part of.  Candidates are rare once the thresholds have risen,
        // so the common path is four compares and one wave-uniform branch; a candidate goes to the wave's
        // staging area in LDS (positions from ballots: no atomics, nothing to wait for).
        bool pass[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) pass[e] = (acc[e] + 1.0f) * 128.0f >= thrx;
        if (__ballot(pass[0] | pass[1] | pass[2] | pass[3])) {
            const bool partial = rb + 16 > row1;                    // only a slab's last block: rows past its end are repeats
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool pe = pass[e] && (!partial || rb + 4 * g + e < row1);
                const uint64_t mask = __ballot(pe);
                if (pe) stage[nstage + lane_rank64(mask)] =
                    ((uint64_t)fkey(acc[e]) << 32) | (uint32_t)(i16 << 16) | (uint32_t)(rb - round_base + 4 * g + e);
                nstage += __popcll(mask);
            }
        }
    };
    // Move the wave's staged candidates into the per-query areas in HBM and count them in the histograms.
    auto flush = [&]() {
        for (int e = lane; e < nstage; e += 64) {
            const uint64_t s = stage[e];
            const int q = (int)((uint32_t)s >> 16), bin = score_bin(fkey_inv((uint32_t)(s >> 32)));
            const int pos = atomicAdd(&cnt[q], 1);                  // < FLAT_CAP: see the round-end check
            atomicAdd(reinterpret_cast<unsigned int*>(hist) + ((q * FLAT_BINS + bin) >> 1), (bin & 1) ? 0x10000u : 1u);
            mycand[(int64_t)q * FLAT_CAP + pos] = (s & 0xFFFFFFFF00000000ull) | (uint32_t)(0xFFFFFFFFu - (uint32_t)(round_base + (int64_t)(s & 0xFFFFu)));
        }
        nstage = 0;
    };

    int shared_seen = 0;   // what the request-wide threshold word held one round ago (threads < nqr)
    // rounds of 256 rows: wave w owns blocks w*FLAT_RB .. +FLAT_RB of the round
    if (row0 < row1) load_rows(a, row0 + (int64_t)wave * FLAT_RB * 16, 0, NP);
    for (int64_t round0 = row0; round0 < row1; round0 += FLAT_ROUND_ROWS) {
        // One block per wave in registers: the next block is requested as soon as the current one has gone through
        // the matrix unit, and the other seven waves of the CU cover the wait.  (Two blocks per wave, the second
        // in flight during the multiply, measured the same at d = 768 and does not fit the registers at d = 1024.)
#pragma unroll 1
        for (int bb = 0; bb < FLAT_RB; ++bb) {
            const int64_t r0 = round0 + ((int64_t)wave * FLAT_RB + bb) * 16;
            const int64_t rn = bb + 1 < FLAT_RB ? r0 + 16 : round0 + FLAT_ROUND_ROWS + (int64_t)wave * FLAT_RB * 16;   // or the first of the next round
            if (nstage > FLAT_STAGE - 256) flush();      // a block adds up to 256 candidates while nothing is filtered
            // As soon as half a block has gone through the matrix unit its registers are requested again for the next
            // block, so those loads are in flight during the other half's multiply (0.821 -> 0.813 ms; thirds to
            // twelfths measured the same).  The empty asm statements keep the compiler from moving the loads back.
            v4f acc = {0.f, 0.f, 0.f, 0.f};
            constexpr int NCH = NP < FLAT_CHUNKS ? NP : FLAT_CHUNKS;
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                acc = multiply(a, acc, c * NP / NCH, (c + 1) * NP / NCH);
                asm volatile("" ::: "memory");
                load_rows(a, rn, c * NP / NCH, (c + 1) * NP / NCH);
                asm volatile("" ::: "memory");
            }
            if (r0 < row1) select(acc, r0);
        }
        if (nstage) flush();
        __syncthreads();
        // Per query (one wave each, four queries per wave): first cut an area back to its best k if it
        // could overflow in the next round (256 more keys at worst) and rebuild its histogram from the
        // survivors; then move the threshold to the highest bin b that has at least k candidates in
        // bins >= b.  Every candidate counted is a real row, so the k-th best score is not below bin b.
        for (int qj = wave; qj < P.nqr; qj += FLAT_WAVES) {
            uint32_t* hq = reinterpret_cast<uint32_t*>(hist + qj * FLAT_BINS);    // two 16-bit bins per word
            const int c = cnt[qj];
            if (c + FLAT_ROUND_ROWS > FLAT_CAP) {
                uint64_t* buf = mycand + (int64_t)qj * FLAT_CAP;
                prune64(buf, c, P.k, lane);
                for (int w = lane; w < FLAT_BINS / 2; w += 64) hq[w] = 0;
                if (lane == 0) cnt[qj] = P.k;
                for (int e = lane; e < P.k; e += 64) {
                    const int bin = score_bin(fkey_inv((uint32_t)(__hip_atomic_load(buf + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >> 32)));
                    atomicAdd(hq + (bin >> 1), (bin & 1) ? 0x10000u : 1u);
                }
            }
            // lane L sums bins 4L..4L+3; suffix sums over lanes; the highest lane reaching k holds the bin
            const uint32_t w0 = hq[2 * lane], w1 = hq[2 * lane + 1];
            const int h0 = w0 & 0xffff, h1 = w0 >> 16, h2 = w1 & 0xffff, h3 = w1 >> 16;
            int suf = h0 + h1 + h2 + h3;
            for (int o = 1; o < 64; o <<= 1) {
                const int v = __shfl_down(suf, o);
                if (lane + o < 64) suf += v;
            }
            const uint64_t reach = __ballot(suf >= P.k);
            if (reach) {
                const int L = 63 - __builtin_clzll(reach);
                if (lane == L) {
                    int cum = suf - (h0 + h1 + h2 + h3), b = 4 * L + 3;
                    const int hh[4] = {h0, h1, h2, h3};
                    for (; b > 4 * L; --b) {
                        cum += hh[b - 4 * L];
                        if (cum >= P.k) break;
                    }
                    if (b > tbin[qj]) tbin[qj] = b;
                }
            }
        }
        __syncthreads();
        // k rows of this request at or above a bin, seen by ANY slab, bound the request's k-th best: the
        // bins are exchanged through one word per (request, query).  The reply of this round's atomic is
        // only looked at after the next round, so its latency is never waited for.
        if (tid < P.nqr) {
            if (shared_seen > tbin[tid]) tbin[tid] = shared_seen;
            shared_seen = atomicMax(P.shared_tbin + r * 16 + tid, tbin[tid]);
        }
        __syncthreads();
        if (i16 < P.nqr) {
            const int tb = tbin[i16];
            thrx = tb > 0 ? (float)tb : -never;
        }
        round_base = round0 + FLAT_ROUND_ROWS;
    }
    // slab result: everything collected (the merge filters it with the request's final threshold bin)
    if (tid < P.nqr) {
        P.part_cnt[pbase + tid] = cnt[tid];
        atomicMax(P.shared_tbin + r * 16 + tid, tbin[tid]);
    }
}

// One workgroup per (request, query): keep the slabs' keys whose score bin reaches the request's
// final threshold bin (at least k rows do, and nothing below it can be in the result), sort them
// descending, write the best k.  If more than FM_CAP keys pass (many equal scores), slabs are
// folded in one at a time, keeping the best k after each.
constexpr int FM_THREADS = 256;
constexpr int FM_CAP = 4096;
__device__ void fm_sort_desc(uint64_t* keys, int n2) {
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
}

__global__ void __launch_bounds__(FM_THREADS) flat_merge_kernel(const FlatParams P, int64_t* __restrict__ out_ids,
                                                                float* __restrict__ out_scores) {
    __shared__ uint64_t keys[FM_CAP];
    __shared__ int s_cnt;
    const int r = blockIdx.x / P.nqr, q = blockIdx.x % P.nqr;
    const int tb = P.shared_tbin[r * 16 + q];
    auto gather = [&](int slab0, int slab1, int base) {   // append passing keys of slabs [slab0, slab1) after keys[0..base)
        if (threadIdx.x == 0) s_cnt = base;
        __syncthreads();
        for (int slab = slab0; slab < slab1; ++slab) {
            const int64_t pb = ((int64_t)r * P.nslab + slab) * 16 + q;
            const int c = P.part_cnt[pb];
            for (int j = threadIdx.x; j < c; j += FM_THREADS) {
                const uint64_t key = P.cand[pb * FLAT_CAP + j];
                if (score_bin(fkey_inv((uint32_t)(key >> 32))) >= tb) {
                    const int o = atomicAdd(&s_cnt, 1);
                    if (o < FM_CAP) keys[o] = key;
                }
            }
        }
        __syncthreads();
        return s_cnt;
    };
    auto sort_keep = [&](int have) {
        int n2 = 2;
        while (n2 < have) n2 <<= 1;
        for (int i = have + threadIdx.x; i < n2; i += FM_THREADS) keys[i] = 0ull;
        fm_sort_desc(keys, n2);
        return min(have, P.k);
    };
    int have = gather(0, P.nslab, 0);
    int fill;
    if (have <= FM_CAP) {
        fill = sort_keep(have);
    } else {
        fill = 0;
        const int per = (FM_CAP - P.k) / FLAT_CAP;   // slabs per pass that always fit (>= 3)
        for (int s0 = 0; s0 < P.nslab; s0 += per) {
            __syncthreads();
            have = gather(s0, min(P.nslab, s0 + per), fill);
            fill = sort_keep(have);
        }
    }
    __syncthreads();
    for (int j = threadIdx.x; j < P.k; j += FM_THREADS) {
        const int64_t o = ((int64_t)r * P.nqr + q) * P.k + j;
        if (j < fill) {
            out_ids[o] = (int64_t)(0xFFFFFFFFu - (uint32_t)keys[j]);
            out_scores[o] = fkey_inv((uint32_t)(keys[j] >> 32));
        } else {
            out_ids[o] = -1;
            out_scores[o] = -INFINITY;
        }
    }
}

static DevBuf g_flat_keys[16], g_flat_cnt[16], g_flat_tbin[16];

// Optional per-kernel timing of the flat search (HIP events on the caller's stream), per device.
constexpr int FLAT_PROF_CALLS = 128;
struct FlatProfiler {
    bool on = false, created = false;
    int ncalls = 0;
    hipEvent_t ev[FLAT_PROF_CALLS][3];
};
static FlatProfiler g_flat_prof[16];

int flat_profile(int device, int enable) {
    if (device < 0 || device >= 16) return fail(RAGO_INVALID_ARG, "device ordinal out of range");
    FlatProfiler& pr = g_flat_prof[device];
    if (enable && !pr.created) {
        for (auto& c : pr.ev)
            for (auto& e : c) RAGO_HIP(hipEventCreate(&e));
        pr.created = true;
    }
    pr.on = enable != 0;
    if (enable) pr.ncalls = 0;
    return RAGO_OK;
}

int flat_stage_ms(int device, float* out_ms, int32_t* out_calls) {
    if (device < 0 || device >= 16) return fail(RAGO_INVALID_ARG, "device ordinal out of range");
    FlatProfiler& pr = g_flat_prof[device];
    out_ms[0] = out_ms[1] = 0.f;
    *out_calls = pr.ncalls;
    for (int c = 0; c < pr.ncalls; ++c) {
        RAGO_HIP(hipEventSynchronize(pr.ev[c][2]));
        for (int i = 0; i < 2; ++i) {
            float ms = 0.f;
            RAGO_HIP(hipEventElapsedTime(&ms, pr.ev[c][i], pr.ev[c][i + 1]));
            out_ms[i] += ms / pr.ncalls;
        }
    }
    return RAGO_OK;
}

// (a kernel rather than a memset node: the call may be recorded into a HIP graph by the caller)
__global__ void flat_zero_kernel(int32_t* p, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0;
}

template <int D, bool HALF>
static int launch_flat_dh(const FlatParams& P, int grid, size_t lds, hipStream_t st) {
    static OncePerDevice attr;
    if (attr.first()) {
        RAGO_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(flat_scan_kernel<D, HALF>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)flat_lds_bytes(D)));
    }
    flat_scan_kernel<D, HALF><<<grid, FLAT_THREADS, lds, st>>>(P);
    RAGO_HIP(hipGetLastError());
    return RAGO_OK;
}

template <int D>
static int launch_flat_d(const FlatParams& P, int grid, size_t lds, bool half, hipStream_t st) {
    return half ? launch_flat_dh<D, true>(P, grid, lds, st) : launch_flat_dh<D, false>(P, grid, lds, st);
}

// Slabs of whole rounds, about `target` workgroups in all (never more when `exact`).
static void flat_slabs(int R, int64_t n, int target, bool exact, int* nslab_out, int64_t* slab_rows_out) {
    const int per_request = exact ? std::max(1, target / R) : (target + R - 1) / R;
    int nslab = (int)std::min<int64_t>(per_request, (n + FLAT_ROUND_ROWS - 1) / FLAT_ROUND_ROWS);
    nslab = std::max(1, nslab);
    int64_t slab_rows = (n + nslab - 1) / nslab;
    slab_rows = (slab_rows + FLAT_ROUND_ROWS - 1) / FLAT_ROUND_ROWS * FLAT_ROUND_ROWS;
    if (slab_rows == 0) slab_rows = FLAT_ROUND_ROWS;
    *nslab_out = (int)std::max<int64_t>(1, (n + slab_rows - 1) / slab_rows);
    *slab_rows_out = slab_rows;
}

// Both kernels of a flat search on given scratch memory: cand [R * nslab][16][FLAT_CAP] keys,
// part_cnt [R * nslab][16], tbin [R][16].
static int run_flat(const void* corpus, const void* queries, int R, int64_t n, int nqr, int d, int k, int64_t* out_ids,
                    float* out_scores, int device, bool half, hipStream_t st, int nslab, int64_t slab_rows, uint64_t* cand,
                    int32_t* part_cnt, int32_t* tbin) {
    FlatParams P;
    P.corpus = static_cast<const uint16_t*>(corpus);
    P.queries = static_cast<const uint16_t*>(queries);
    P.n = n; P.R = R; P.nqr = nqr; P.d = d; P.k = k;
    P.nslab = nslab; P.slab_rows = slab_rows;
    P.cand = cand; P.part_cnt = part_cnt; P.shared_tbin = tbin;
    // the request-wide threshold bins start at zero (a kernel, not a memset node: the call may be
    // recorded into a HIP graph by the caller)
    flat_zero_kernel<<<(R * 16 + 255) / 256, 256, 0, st>>>(tbin, (int64_t)R * 16);
    RAGO_HIP(hipGetLastError());
    const size_t lds = flat_lds_bytes(d);
    const int grid = R * nslab;
    FlatProfiler& prof = g_flat_prof[device];
    hipEvent_t* ev = prof.on && prof.ncalls < FLAT_PROF_CALLS ? prof.ev[prof.ncalls] : nullptr;
    if (ev) RAGO_HIP(hipEventRecord(ev[0], st));
    int rc;
    switch (d) {
        case 64: rc = launch_flat_d<64>(P, grid, lds, half, st); break;
        case 128: rc = launch_flat_d<128>(P, grid, lds, half, st); break;
        case 256: rc = launch_flat_d<256>(P, grid, lds, half, st); break;
        case 384: rc = launch_flat_d<384>(P, grid, lds, half, st); break;
        case 512: rc = launch_flat_d<512>(P, grid, lds, half, st); break;
        case 768: rc = launch_flat_d<768>(P, grid, lds, half, st); break;
        case 1024: rc = launch_flat_d<1024>(P, grid, lds, half, st); break;
        default: return fail(RAGO_UNSUPPORTED, "d must be one of 64, 128, 256, 384, 512, 768, 1024");
    }
    if (rc) return rc;
    if (ev) RAGO_HIP(hipEventRecord(ev[1], st));
    flat_merge_kernel<<<R * nqr, FM_THREADS, 0, st>>>(P, out_ids, out_scores);
    RAGO_HIP(hipGetLastError());
    if (ev) { RAGO_HIP(hipEventRecord(ev[2], st)); ++prof.ncalls; }
    return RAGO_OK;
}

int launch_flat(const void* corpus, const void* queries, int R, int64_t n, int nqr, int d, int k, int64_t* out_ids,
                float* out_scores, int device, bool half, hipStream_t st) {
    if (device < 0 || device >= 16) return fail(RAGO_INVALID_ARG, "device ordinal out of range");
    if (d % 64 || d > FLAT_MAXD) return fail(RAGO_UNSUPPORTED, "d must be a multiple of 64, at most 1024");
    // one resident wave of workgroups (2 per CU): per-slab start-up (unfiltered first round) is paid once per slot
    int nslab;
    int64_t slab_rows;
    flat_slabs(R, n, 512, false, &nslab, &slab_rows);
    int rc;
    if ((rc = g_flat_keys[device].reserve((size_t)R * nslab * 16 * FLAT_CAP * 8))) return rc;
    if ((rc = g_flat_cnt[device].reserve((size_t)R * nslab * 16 * 4))) return rc;
    if ((rc = g_flat_tbin[device].reserve((size_t)R * 16 * 4))) return rc;
    return run_flat(corpus, queries, R, n, nqr, d, k, out_ids, out_scores, device, half, st, nslab, slab_rows,
                    g_flat_keys[device].as<uint64_t>(), g_flat_cnt[device].as<int32_t>(), g_flat_tbin[device].as<int32_t>());
}

// ------------------------------------------------------------------ the flat search that allocates nothing
// Its scratch memory (candidate keys, per-slab counts, threshold bins) is a device array of the code object
// instead of a grown workspace.  Every GPU the library runs on holds its own copy of the array at its own
// address, looked up once per device (with that device current) and kept; host code only ever uses that looked-up
// address, never the array's name, which on the host is a stand-in and not a device address.
constexpr int FLAT_STATIC_SLABS = 256;                                           // workgroups (requests x slabs) per call
constexpr size_t FLAT_STATIC_KEYS = (size_t)FLAT_STATIC_SLABS * 16 * FLAT_CAP * 8;   // 32 MiB of candidate keys
constexpr size_t FLAT_STATIC_CNT = (size_t)FLAT_STATIC_SLABS * 16 * 4;
constexpr size_t FLAT_STATIC_TBIN = (size_t)FLAT_STATIC_SLABS * 16 * 4;              // (requests <= slabs)
constexpr size_t FLAT_STATIC_BYTES = FLAT_STATIC_KEYS + FLAT_STATIC_CNT + FLAT_STATIC_TBIN;
static __device__ __align__(256) unsigned char scratch[FLAT_STATIC_BYTES];

static std::mutex g_scratch_mutex;
static unsigned char* g_scratch_ptr[16] = {};

int flat_static_max_requests() { return FLAT_STATIC_SLABS; }

int launch_flat_static(const void* corpus, const void* queries, int R, int64_t n, int nqr, int d, int k, int64_t* out_ids,
                       float* out_scores, int device, bool half, hipStream_t st) {
    if (device < 0 || device >= 16) return fail(RAGO_INVALID_ARG, "device ordinal out of range");
    if (d % 64 || d > FLAT_MAXD) return fail(RAGO_UNSUPPORTED, "d must be a multiple of 64, at most 1024");
    if (R > FLAT_STATIC_SLABS)
        return fail(RAGO_UNSUPPORTED, "more than " + std::to_string(FLAT_STATIC_SLABS) + " requests in one call: beyond the static scratch memory");
    unsigned char* base;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[device]) {          // (the caller has made `device` current)
            void* p = nullptr;
            RAGO_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
            g_scratch_ptr[device] = static_cast<unsigned char*>(p);
        }
        base = g_scratch_ptr[device];
    }
    int nslab;
    int64_t slab_rows;
    flat_slabs(R, n, FLAT_STATIC_SLABS, true, &nslab, &slab_rows);
    if ((int64_t)R * nslab > FLAT_STATIC_SLABS) return fail(RAGO_UNSUPPORTED, "internal: slab count beyond the static scratch memory");
    // nothing in the scratch memory needs clearing beyond the threshold bins, which run_flat zeroes with a kernel:
    // the counts are written by every workgroup before the merge reads them, and keys are only read below a count
    return run_flat(corpus, queries, R, n, nqr, d, k, out_ids, out_scores, device, half, st, nslab, slab_rows,
                    reinterpret_cast<uint64_t*>(base), reinterpret_cast<int32_t*>(base + FLAT_STATIC_KEYS),
                    reinterpret_cast<int32_t*>(base + FLAT_STATIC_KEYS + FLAT_STATIC_CNT));
}

}  // namespace rago

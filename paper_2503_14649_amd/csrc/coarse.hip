// Coarse quantiser: scores of every query against every list centroid (the IVF level of the
// index, Section 2; an upper tree level is itself a vector scan, Section 4 "Retrieval performance
// modeling") and the choice of the nprobe best lists per query (the scanned subset, Section 3.3).
//
//  * coarse_gemm: S = Q * C^T with fp32 MFMA (v_mfma_f32_32x32x2_f32), both operands K-contiguous,
//    LDS-staged 128x128 (or 32x128 for small batches) tiles, next tile prefetched into registers;
//    from 128 queries up the product runs on the bf16 matrix cores with every operand split into
//    two bf16 terms (three products per term pair).
//  * select: per query, radix-select the nprobe+32 largest fp32 scores, recompute exactly those
//    in fp64 straight from the query and the centroids, round to fp32, sort by (score descending,
//    list ascending) and keep nprobe.  The extra candidates make the result independent of the
//    rounding of the MFMA accumulation: a list outside the candidate set has an fp32 score below
//    every candidate's, so its exact score is at most (smallest candidate score + E) with
//    E = (d * 2^-22 + 2^-16) * |q| * max|c| bounding the accumulation error and that of the split
//    product; when the nprobe-th exact score
//    exceeds that, no outside list can belong to the result.  Queries where this cannot be shown
//    (scores packed closer than E around the cut) are queued; a second launch of the same kernel
//    replaces their rows by exact scores and selects again, so the result is always the one exact
//    scores give.  (Never needed on the workloads here; the counter says how often it was.)
#include "rago_internal.h"

namespace rago {

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int G_TN = 128, G_KT = 32, G_LS = 36;  // LDS row stride in floats (144 B: b128 reads conflict-free)

// qn2 / cn2 null: S = <q, c>.  Else (Euclidean metric) S = 2 <q, c> - |c|^2 - |q|^2 = -|q - c|^2.
__device__ __forceinline__ float coarse_score(float ip, int row, int col, const float* __restrict__ qn2, const float* __restrict__ cn2) {
    return qn2 ? 2.0f * ip - cn2[col] - qn2[row] : ip;
}

__global__ void __launch_bounds__(256) coarse_gemm_kernel(const float* __restrict__ Q, const float* __restrict__ C, int nq,
                                                          int nlist, int d, const float* __restrict__ qn2,
                                                          const float* __restrict__ cn2, float* __restrict__ S, int64_t* zero_me) {
    if (zero_me && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *zero_me = 0;   // (the selection's counter of queued queries)
    constexpr int TM = 32;                 // query rows per workgroup: one 32x32 MFMA tile per wave, the four waves side by side
    constexpr int MT = 1, NT = 1;
    constexpr int AF = TM * 8 / 256;       // float4 loads per thread for the A tile
    constexpr int BF = G_TN * 8 / 256;
    __shared__ __align__(16) float As[TM * G_LS];
    __shared__ __align__(16) float Bs[G_TN * G_LS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i32 = lane & 31, h = lane >> 5;
    const int n0 = blockIdx.x * G_TN, m0 = blockIdx.y * TM;
    const int wm = 0, wn = wave * 32;

    v16f acc[MT][NT];
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int b = 0; b < NT; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    // Two K tiles are on their way at any time, in two sets of registers.  (Neither that nor 16-row tiles on the
    // 16x16x4 instruction - half the matrix cycles - changed the 40 us this kernel takes for 65536 x 768, where the
    // streaming kernel for one or two queries takes 33: what it pays for is the trip of every tile through LDS, two
    // barriers per 20 KB.)
    constexpr int AHEAD = 2;
    float4 pa0[AF], pb0[BF], pa1[AF], pb1[BF];
    auto gload = [&](float4 (&pa)[AF], float4 (&pb)[BF], int k0) {
#pragma unroll
        for (int r = 0; r < AF; ++r) {
            const int f = tid + 256 * r, row = f >> 3, c4 = f & 7;
            const int gr = min(m0 + row, nq - 1), gk = k0 + c4 * 4;
            pa[r] = gk < d ? *reinterpret_cast<const float4*>(Q + (int64_t)gr * d + gk) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int r = 0; r < BF; ++r) {
            const int f = tid + 256 * r, row = f >> 3, c4 = f & 7;
            const int gr = min(n0 + row, nlist - 1), gk = k0 + c4 * 4;
            pb[r] = gk < d ? *reinterpret_cast<const float4*>(C + (int64_t)gr * d + gk) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    // one K tile: the registers that hold it go to LDS and are sent for the tile after the next; then the products
    auto step = [&](float4 (&pa)[AF], float4 (&pb)[BF], int k0) {
        __syncthreads();  // previous tile fully consumed
#pragma unroll
        for (int r = 0; r < AF; ++r) {
            const int f = tid + 256 * r;
            *reinterpret_cast<float4*>(As + (f >> 3) * G_LS + (f & 7) * 4) = pa[r];
        }
#pragma unroll
        for (int r = 0; r < BF; ++r) {
            const int f = tid + 256 * r;
            *reinterpret_cast<float4*>(Bs + (f >> 3) * G_LS + (f & 7) * 4) = pb[r];
        }
        if (k0 + AHEAD * G_KT < d) gload(pa, pb, k0 + AHEAD * G_KT);
        __syncthreads();
        // lane (i32, h) owns k = h*16 .. h*16+15 of this tile for both operands
        float af[MT][16], bf[NT][16];
#pragma unroll
        for (int a = 0; a < MT; ++a)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float4 x = *reinterpret_cast<const float4*>(As + (wm + a * 32 + i32) * G_LS + h * 16 + v * 4);
                af[a][4 * v] = x.x; af[a][4 * v + 1] = x.y; af[a][4 * v + 2] = x.z; af[a][4 * v + 3] = x.w;
            }
#pragma unroll
        for (int b = 0; b < NT; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float4 x = *reinterpret_cast<const float4*>(Bs + (wn + b * 32 + i32) * G_LS + h * 16 + v * 4);
                bf[b][4 * v] = x.x; bf[b][4 * v + 1] = x.y; bf[b][4 * v + 2] = x.z; bf[b][4 * v + 3] = x.w;
            }
#pragma unroll
        for (int s = 0; s < 16; ++s)
#pragma unroll
            for (int a = 0; a < MT; ++a)
#pragma unroll
                for (int b = 0; b < NT; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[a][s], bf[b][s], acc[a][b], 0, 0, 0);
    };
    gload(pa0, pb0, 0);
    gload(pa1, pb1, G_KT);                // (beyond d: zeros, no loads)
    for (int k0 = 0; k0 < d; k0 += 2 * G_KT) {
        step(pa0, pb0, k0);
        if (k0 + G_KT < d) step(pa1, pb1, k0 + G_KT);
    }
    // D layout of the 32x32 tile: register r, lane (i32, h) -> row 8*(r/4) + 4*h + r%4, column i32
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int b = 0; b < NT; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm + a * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                const int col = n0 + wn + b * 32 + i32;
                if (row < nq && col < nlist) S[(int64_t)row * nlist + col] = coarse_score(acc[a][b][r], row, col, qn2, cn2);
            }
}

// ---- large batches: the same product on the bf16 matrix cores, each fp32 operand split into two
// bf16 terms x = hi + lo (hi = bf16(x), lo = bf16(x - hi), |x - hi - lo| <= 2^-18 |x|) and
//     <q, c> ~ sum q_hi c_hi + q_hi c_lo + q_lo c_hi           (fp32 accumulation)
// whose error, lo * lo dropped and the two roundings of lo, is at most 3 * 2^-18 * |q| |c|: an
// order of magnitude inside the 1e-4 the scores are held to, at 16x the fp32 MFMA rate per
// instruction.  The centroids are split once when the index is loaded, the queries on their way
// into LDS.  v_mfma_f32_32x32x16_bf16: lane (i32, h) supplies k = 8h .. 8h+7 of row i32 of both
// operands; 128x128 tile per workgroup, 64x64 per wave.
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
constexpr int X_T = 128;
// LDS row stride in bf16 for a K tile of KT: 8 more (144 or 80 B: the b128 reads of 8 consecutive rows cover all banks once)
constexpr int x_ls(int KT) { return KT + 8; }
// bytes: hi and lo tiles of both operands (TM query rows, X_T centroid rows)
constexpr int x_lds(int TM, int KT) { return (TM * 2 + X_T * 2) * x_ls(KT) * 2; }

__device__ __forceinline__ uint32_t bf16_rne(float x) {
    const uint32_t u = __float_as_uint(x);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Two floats -> their bf16 parts, packed (first in the low half): hi = bf16(x), lo = bf16(x - hi), both rounded to
// nearest even by the chip's packed conversion (v_cvt_pk_bf16_f32: one instruction per pair, where the bit arithmetic of
// bf16_rne takes four per number).  The split of the query tile was two thirds of the tile kernel's vector instructions
// (384 of 422 per wave and K tile of 64, 104 now); the kernel gained 4 % (0.41 -> 0.39 ms per 1024 x 65536 x 768): what
// it waits for is the next tile's loads from L2, with two workgroups per compute unit then.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void split_bf16_pair(float a, float b, uint32_t& hi, uint32_t& lo) {
    const f32x2_t v = {a, b};
    const uint32_t h = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
    const f32x2_t r = {a - __uint_as_float(h << 16), b - __uint_as_float(h & 0xffff0000u)};
    hi = h;
    lo = __builtin_bit_cast(uint32_t, __builtin_convertvector(r, bf16x2_t));
}

__global__ void __launch_bounds__(256) split_bf16_kernel(const float* __restrict__ x, int64_t n, uint16_t* __restrict__ hi,
                                                         uint16_t* __restrict__ lo) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const float v = x[i];
        const uint32_t h = bf16_rne(v);
        hi[i] = (uint16_t)h;
        lo[i] = (uint16_t)bf16_rne(v - __uint_as_float(h << 16));
    }
}

int launch_split_centroids(rago_index* idx, hipStream_t st) {
    split_bf16_kernel<<<2048, 256, 0, st>>>(idx->centroids, (int64_t)idx->nlist * idx->d, idx->cen_hi, idx->cen_lo);
    RAGO_HIP(hipGetLastError());
    return RAGO_OK;
}

// Workgroup b works on centroid tile (b / 8 / nqt) * 8 + b % 8 and query tile (b / 8) % nqt: the
// nqt workgroups that share a centroid tile are dispatched back to back onto the same XCD
// (workgroups go round-robin over the 8 XCDs), so the tile is fetched from HBM once and then
// served by that XCD's L2.
// TM = query rows per workgroup: 128 (a wave takes 64 x 64), or 64 (a wave takes 64 x 32) for batches that would
// otherwise leave a workgroup alone on its compute unit with nothing to hide its loads behind.
// KT = dimensions per K tile: 64, or 32 for the 128-row tile, whose registers then allow a third workgroup per compute unit
// (1024 x 65536 x 768: 0.39 -> 0.35 ms; the 64-row tile on 256 queries loses 10 % with it).
template <int TM, int KT>
__global__ void __launch_bounds__(256, KT == 32 ? 3 : 1) coarse_gemm_split_kernel(const float* __restrict__ Q, const uint16_t* __restrict__ Chi,
                                                                const uint16_t* __restrict__ Clo, int nq, int nlist, int d, int nqt,
                                                                int nct, const float* __restrict__ qn2,
                                                                const float* __restrict__ cn2, float* __restrict__ S, int64_t* zero_me) {
    if (zero_me && blockIdx.x == 0 && threadIdx.x == 0) *zero_me = 0;   // (the selection's counter of queued queries)
    constexpr int LS = x_ls(KT);
    extern __shared__ __align__(16) uint16_t x_smem[];
    uint16_t *Ah = x_smem, *Al = Ah + TM * LS, *Bh = Al + TM * LS, *Bl = Bh + X_T * LS;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i32 = lane & 31, h = lane >> 5;
    const int r8 = blockIdx.x >> 3;
    const int ct = (r8 / nqt) * 8 + (blockIdx.x & 7), qt = r8 % nqt;
    if (ct >= nct) return;
    constexpr int NBT = TM == 128 ? 2 : 1;          // 32-column tiles per wave
    const int n0 = ct * X_T, m0 = qt * TM;
    const int wm = TM == 128 ? (wave >> 1) * 64 : 0, wn = TM == 128 ? (wave & 1) * 64 : wave * 32;

    v16f acc[2][NBT];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < NBT; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    constexpr int NA = TM * (KT / 4) / 256, NB = KT / 16;       // 16-byte loads per thread and K tile: A (fp32), B (bf16, hi and lo)
    float4 pa[NA];
    uint4 pbh[NB], pbl[NB];
    auto gload = [&](int k0) {
#pragma unroll
        for (int r = 0; r < NA; ++r) {         // A: TM rows x (KT / 4) float4
            const int f = tid + 256 * r, row = f / (KT / 4), c4 = f % (KT / 4);
            const int gr = min(m0 + row, nq - 1), gk = k0 + c4 * 4;
            pa[r] = gk < d ? *reinterpret_cast<const float4*>(Q + (int64_t)gr * d + gk) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int r = 0; r < NB; ++r) {         // B: 128 rows x (KT / 8) x (8 bf16), twice
            const int f = tid + 256 * r, row = f / (KT / 8), c8 = f % (KT / 8);
            const int gr = min(n0 + row, nlist - 1), gk = k0 + c8 * 8;
            const bool in = gk < d;
            pbh[r] = in ? *reinterpret_cast<const uint4*>(Chi + (int64_t)gr * d + gk) : make_uint4(0u, 0u, 0u, 0u);
            pbl[r] = in ? *reinterpret_cast<const uint4*>(Clo + (int64_t)gr * d + gk) : make_uint4(0u, 0u, 0u, 0u);
        }
    };
    gload(0);
    for (int k0 = 0; k0 < d; k0 += KT) {
        __syncthreads();  // previous tile fully consumed
#pragma unroll
        for (int r = 0; r < NA; ++r) {
            const int f = tid + 256 * r, row = f / (KT / 4), c4 = f % (KT / 4);
            uint32_t h01, l01, h23, l23;
            split_bf16_pair(pa[r].x, pa[r].y, h01, l01);
            split_bf16_pair(pa[r].z, pa[r].w, h23, l23);
            *reinterpret_cast<uint2*>(Ah + row * LS + c4 * 4) = make_uint2(h01, h23);
            *reinterpret_cast<uint2*>(Al + row * LS + c4 * 4) = make_uint2(l01, l23);
        }
#pragma unroll
        for (int r = 0; r < NB; ++r) {
            const int f = tid + 256 * r, row = f / (KT / 8), c8 = f % (KT / 8);
            *reinterpret_cast<uint4*>(Bh + row * LS + c8 * 8) = pbh[r];
            *reinterpret_cast<uint4*>(Bl + row * LS + c8 * 8) = pbl[r];
        }
        if (k0 + KT < d) gload(k0 + KT);     // (the registers are free again: the next tile's loads go out ahead of the barrier)
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < KT / 16; ++ks) {
            bf16x8 ah[2], al[2], bh[NBT], bl[NBT];
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                const int o = (wm + a * 32 + i32) * LS + ks * 16 + h * 8;
                ah[a] = *reinterpret_cast<const bf16x8*>(Ah + o);
                al[a] = *reinterpret_cast<const bf16x8*>(Al + o);
            }
#pragma unroll
            for (int b = 0; b < NBT; ++b) {
                const int o = (wn + b * 32 + i32) * LS + ks * 16 + h * 8;
                bh[b] = *reinterpret_cast<const bf16x8*>(Bh + o);
                bl[b] = *reinterpret_cast<const bf16x8*>(Bl + o);
            }
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < NBT; ++b) {
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[a], bh[b], acc[a][b], 0, 0, 0);
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[a], bl[b], acc[a][b], 0, 0, 0);
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[a], bh[b], acc[a][b], 0, 0, 0);
                }
        }
    }
    // D layout of the 32x32 tile: register r, lane (i32, h) -> row 8*(r/4) + 4*h + r%4, column i32
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < NBT; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm + a * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                const int col = n0 + wn + b * 32 + i32;
                if (row < nq && col < nlist) S[(int64_t)row * nlist + col] = coarse_score(acc[a][b][r], row, col, qn2, cn2);
            }
}

// ---- one or two queries: the product is a stream over C (a round of iterative retrieval, Section 5.3, reads all
// of C for a handful of queries), so the only thing that matters is how many bytes are in flight.  A wave takes
// GV_R rows of C at a time, its lanes 16 bytes each of every 1 KiB of a row; the queries sit in LDS; partial
// sums are added up across the lanes at the end of the rows.  Plain fp32: the selection only needs the scores to
// within its bound (d * 2^-22 |q||c|), which any order of fp32 products and sums stays inside.
constexpr int GV_R = 8, GV_THREADS = 256;
template <int NQ>
__global__ void __launch_bounds__(GV_THREADS) coarse_gemv_kernel(const float* __restrict__ Q, const float* __restrict__ C, int nq,
                                                                 int nlist, int d, const float* __restrict__ qn2,
                                                                 const float* __restrict__ cn2, float* __restrict__ S, int64_t* zero_me) {
    extern __shared__ __align__(16) float gv_q[];          // [NQ][d]
    if (zero_me && blockIdx.x == 0 && threadIdx.x == 0) *zero_me = 0;
    const int tid = threadIdx.x, lane = tid & 63;
    for (int i = tid; i < NQ * d; i += GV_THREADS) gv_q[i] = i / d < nq ? Q[i] : 0.f;
    __syncthreads();
    const int wave_id = blockIdx.x * (GV_THREADS / 64) + (tid >> 6), nwaves = gridDim.x * (GV_THREADS / 64);
    for (int r0 = wave_id * GV_R; r0 < nlist; r0 += nwaves * GV_R) {
        float acc[GV_R][NQ];
#pragma unroll
        for (int r = 0; r < GV_R; ++r)
#pragma unroll
            for (int qi = 0; qi < NQ; ++qi) acc[r][qi] = 0.f;
        const float* rows[GV_R];
#pragma unroll
        for (int r = 0; r < GV_R; ++r) rows[r] = C + (int64_t)min(r0 + r, nlist - 1) * d;
        for (int t = lane * 4; t < d; t += 256) {
            typedef float gv_f4 __attribute__((ext_vector_type(4)));
            gv_f4 c4[GV_R];
#pragma unroll
            for (int r = 0; r < GV_R; ++r) c4[r] = __builtin_nontemporal_load(reinterpret_cast<const gv_f4*>(rows[r] + t));
#pragma unroll
            for (int qi = 0; qi < NQ; ++qi) {
                const float4 q4 = *reinterpret_cast<const float4*>(gv_q + qi * d + t);
#pragma unroll
                for (int r = 0; r < GV_R; ++r)
                    acc[r][qi] += c4[r].x * q4.x + c4[r].y * q4.y + c4[r].z * q4.z + c4[r].w * q4.w;
            }
        }
#pragma unroll
        for (int qi = 0; qi < NQ; ++qi) {
            float mine = 0.f;                               // lane r keeps row r0 + r
#pragma unroll
            for (int r = 0; r < GV_R; ++r) {
                float v = acc[r][qi];
                for (int o = 32; o; o >>= 1) v += __shfl_xor(v, o);
                mine = lane == r ? v : mine;
            }
            if (lane < GV_R && r0 + lane < nlist && qi < nq)
                S[(int64_t)qi * nlist + r0 + lane] = coarse_score(mine, qi, r0 + lane, qn2, cn2);
        }
    }
}

// |q|^2 per query (fp64 accumulation, one rounding): one wave per query
__global__ void __launch_bounds__(256) qnorm2_kernel(const float* __restrict__ Q, int64_t nq, int d, float* __restrict__ out) {
    const int64_t q = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (q >= nq) return;
    double acc = 0.0;
    for (int t = threadIdx.x & 63; t < d; t += 64) acc = acc + (double)Q[q * d + t] * (double)Q[q * d + t];
    for (int o = 32; o; o >>= 1) acc = acc + __shfl_xor(acc, o);
    if ((threadIdx.x & 63) == 0) out[q] = (float)acc;
}

int launch_coarse(rago_index* idx, const float* q, int64_t nq, float* S, hipStream_t st, bool zero_select_counter) {
    const int nlist = idx->nlist, d = idx->d;
    if (nq > 0x7fffffff) return fail(RAGO_UNSUPPORTED, "nq too large");
    const float *qn2 = nullptr, *cn2 = nullptr;
    if (idx->metric == 1) {
        int rc = idx->ws.qn2.reserve((size_t)nq * 4);
        if (rc) return rc;
        if (idx->reserving) return RAGO_OK;
        qnorm2_kernel<<<(unsigned)((nq + 3) / 4), 256, 0, st>>>(q, nq, d, idx->ws.qn2.as<float>());
        qn2 = idx->ws.qn2.as<float>();
        cn2 = idx->cn2;
    }
    if (idx->reserving) return RAGO_OK;
    int64_t* zero_me = nullptr;
    if (zero_select_counter) {
        int rc = idx->ws.counters.reserve(64);
        if (rc) return rc;
        zero_me = idx->ws.counters.as<int64_t>() + 3;
    }
    const unsigned gx = (unsigned)((nlist + G_TN - 1) / G_TN);
    if (nq <= 2 && d % 4 == 0 && (size_t)2 * d * 4 <= 48 * 1024) {
        // (measured on 65536 x 768: 38 us against the tile kernel's 45 for one query; four queries are level)
        const unsigned grid = (unsigned)std::min<int64_t>((nlist + GV_R * 4 - 1) / (GV_R * 4), (int64_t)idx->n_cu * 8);
        const size_t lds = (size_t)nq * d * 4;
        if (nq == 1) coarse_gemv_kernel<1><<<grid, GV_THREADS, lds, st>>>(q, idx->centroids, (int)nq, nlist, d, qn2, cn2, S, zero_me);
        else coarse_gemv_kernel<2><<<grid, GV_THREADS, lds, st>>>(q, idx->centroids, (int)nq, nlist, d, qn2, cn2, S, zero_me);
    } else if (nq <= 32) {
        // (up to 32 queries the fp32 products of one 32-row tile keep pace with the centroids' stream: 46 us for
        // 65536 x 768 against 55 with the split kernel's 64-row tile; from 33 on they do not: 48 queries 122 us against 58)
        coarse_gemm_kernel<<<dim3(gx, 1), 256, 0, st>>>(q, idx->centroids, (int)nq, nlist, d, qn2, cn2, S, zero_me);
    } else {
        // (the split kernel reads the centroids 8 bf16 at a time: d is a multiple of 16, since m is one and d one of m)
        // query rows per workgroup: 64 while 128 would give the chip fewer than two workgroups per compute unit
        const int nct = (nlist + X_T - 1) / X_T;
        const bool half_tile = (int64_t)((nq + X_T - 1) / X_T) * nct < 2 * (int64_t)idx->n_cu;
        const int tm = half_tile ? 64 : X_T;
        const int nqt = (int)((nq + tm - 1) / tm);
        const int64_t grid = (int64_t)((nct + 7) / 8) * 8 * nqt;
        if (grid > 0x7fffffff) return fail(RAGO_UNSUPPORTED, "nq * nlist too large");
        static OncePerDevice attr;
        if (attr.first()) {
            RAGO_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(coarse_gemm_split_kernel<128, 32>), hipFuncAttributeMaxDynamicSharedMemorySize, x_lds(128, 32)));
            RAGO_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(coarse_gemm_split_kernel<64, 64>), hipFuncAttributeMaxDynamicSharedMemorySize, x_lds(64, 64)));
        }
        if (half_tile)
            coarse_gemm_split_kernel<64, 64><<<(unsigned)grid, 256, x_lds(64, 64), st>>>(q, idx->cen_hi, idx->cen_lo, (int)nq, nlist, d, nqt, nct, qn2, cn2, S, zero_me);
        else
            coarse_gemm_split_kernel<128, 32><<<(unsigned)grid, 256, x_lds(128, 32), st>>>(q, idx->cen_hi, idx->cen_lo, (int)nq, nlist, d, nqt, nct, qn2, cn2, S, zero_me);
    }
    RAGO_HIP(hipGetLastError());
    return RAGO_OK;
}

// ------------------------------------------------------------------ selection
constexpr int SEL_THREADS = 1024;
constexpr int SEL_WAVES = SEL_THREADS / 64;
constexpr int SEL_EXTRA = 32;
constexpr int SEL_CAP = 2048;   // candidate capacity (power of two): nprobe + SEL_EXTRA <= SEL_CAP

__device__ __forceinline__ uint32_t float_key(float f) {  // ascending uint order == ascending float order
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// REG = fp32 scores held per thread (nlist <= REG * 1024: the row is read from memory once).
// REG = 0: rows of any length, re-read from L2 in every pass.
template <int REG>
__global__ void __launch_bounds__(SEL_THREADS) select_kernel(const float* __restrict__ Q, const float* __restrict__ C,
                                                             float* S, int nlist, int d, int nprobe,
                                                             float max_cnorm, int metric, int32_t* __restrict__ probes,
                                                             int64_t* counters, int32_t* redo_q, int redo) {
    // 32 copies of every bin, copy = lane % 32: the lanes of a half-wave never share an LDS word,
    // so the atomics run at full rate even when all scores fall into one bin (pass 0: same exponent)
    __shared__ int hist32[256 * 32];
    __shared__ int hist[256];
    __shared__ uint32_t s_prefix;
    __shared__ int s_rem, s_rem_next, s_ngt, s_neq;
    __shared__ int s_sfx[256];
    __shared__ int s_weq[SEL_WAVES];
    __shared__ int c_idx[SEL_CAP];
    __shared__ float c_val[SEL_CAP];
    // Second launch (`redo`): only the queries whose choice the first launch could not show independent of the
    // rounding of S.  Their rows are replaced by exact scores (fp64 accumulation, one rounding) and selected again.
    if (redo && (int64_t)blockIdx.x >= counters[3]) return;
    const int64_t q = redo ? redo_q[blockIdx.x] : blockIdx.x;
    float* row = S + q * nlist;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (redo) {
        const float* qx = Q + q * d;
        for (int l = wave; l < nlist; l += SEL_WAVES) {
            const float* cx = C + (int64_t)l * d;
            double acc = 0.0;
            for (int t = lane; t < d; t += 64) {
                if (metric == 1) { const double diff = (double)qx[t] - (double)cx[t]; acc = acc + diff * diff; }
                else acc = acc + (double)qx[t] * (double)cx[t];
            }
            for (int o = 32; o; o >>= 1) acc = acc + __shfl_xor(acc, o);
            if (lane == 0) row[l] = metric == 1 ? (float)(-acc) : (float)acc;
        }
        __threadfence();
        __syncthreads();
    }
    const int want = min(nprobe + SEL_EXTRA, nlist);
    constexpr int NR = REG > 0 ? REG : 1;
    // Exact scores (fp64 accumulation, one rounding to fp32) of n rows of C, RU per wave at a time: the rows come
    // from HBM at random, and the time of this step is the number of such rounds times the latency of a loaded
    // memory system; with 16-byte loads a lane has d / 256 loads per row, so a whole round is in flight at once.
    const float* qv = Q + q * d;
    constexpr int RU = 8;
    const bool vec4 = (d & 3) == 0;
    auto exact_scores = [&](int n, auto row_of, auto store) {
        for (int c0 = wave * RU; c0 < n; c0 += SEL_WAVES * RU) {
            double acc[RU];
            const float* cv[RU];
#pragma unroll
            for (int u = 0; u < RU; ++u) { acc[u] = 0.0; cv[u] = C + (int64_t)row_of(min(c0 + u, n - 1)) * d; }
            if (vec4) {
                for (int t = lane * 4; t < d; t += 256) {
                    const float4 q4 = *reinterpret_cast<const float4*>(qv + t);
                    float4 c4[RU];
#pragma unroll
                    for (int u = 0; u < RU; ++u) c4[u] = *reinterpret_cast<const float4*>(cv[u] + t);
                    const double qa[4] = {(double)q4.x, (double)q4.y, (double)q4.z, (double)q4.w};
#pragma unroll
                    for (int u = 0; u < RU; ++u) {
                        const double ca[4] = {(double)c4[u].x, (double)c4[u].y, (double)c4[u].z, (double)c4[u].w};
#pragma unroll
                        for (int x = 0; x < 4; ++x) {
                            if (metric == 1) { const double diff = qa[x] - ca[x]; acc[u] = acc[u] + diff * diff; }
                            else acc[u] = acc[u] + qa[x] * ca[x];
                        }
                    }
                }
            } else if (metric == 1) {
                for (int t = lane; t < d; t += 64) {
                    const double qt = (double)qv[t];
#pragma unroll
                    for (int u = 0; u < RU; ++u) {
                        const double diff = qt - (double)cv[u][t];
                        acc[u] = acc[u] + diff * diff;
                    }
                }
            } else {
                for (int t = lane; t < d; t += 64) {
                    const double qt = (double)qv[t];
#pragma unroll
                    for (int u = 0; u < RU; ++u) acc[u] = acc[u] + qt * (double)cv[u][t];
                }
            }
#pragma unroll
            for (int u = 0; u < RU; ++u) {
                for (int o = 32; o; o >>= 1) acc[u] = acc[u] + __shfl_xor(acc[u], o);
                if (lane == 0 && c0 + u < n) store(c0 + u, metric == 1 ? (float)(-acc[u]) : (float)acc[u]);
            }
        }
    };
    uint32_t key[NR];
    if (REG > 0) {
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            const int i = r * SEL_THREADS + tid;
            key[r] = i < nlist ? float_key(row[i]) : 0u;      // 0 sorts below every real score
        }
    }
    const int nrounds = REG > 0 ? REG : (nlist + SEL_THREADS - 1) / SEL_THREADS;
    auto key_at = [&](int r) -> uint32_t {
        if (REG > 0) return key[r];
        const int i = r * SEL_THREADS + tid;
        return i < nlist ? float_key(row[i]) : 0u;
    };

    // ---- radix select: key of the want-th largest score
    if (tid == 0) { s_prefix = 0; s_rem = want; s_ngt = 0; s_neq = 0; }
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        for (int i = tid; i < 256 * 32; i += SEL_THREADS) hist32[i] = 0;
        __syncthreads();
        const uint32_t prefix = s_prefix;
        const uint32_t himask = pass == 0 ? 0u : (0xFFFFFFFFu << (shift + 8));
        auto count = [&](uint32_t kk, int i) {
            if (i < nlist && (kk & himask) == prefix) atomicAdd(&hist32[(((kk >> shift) & 255u) << 5) | (lane & 31)], 1);
        };
        if (REG > 0) {
#pragma unroll
            for (int r = 0; r < NR; ++r) count(key[r], r * SEL_THREADS + tid);
        } else {
            for (int r = 0; r < nrounds; ++r) count(key_at(r), r * SEL_THREADS + tid);
        }
        __syncthreads();
        // digit = the highest bin whose count, together with all higher bins, reaches `rem`:
        // thread t < 256 owns bin t; suffix sums inside each of the four waves, then across them
        if (tid < 256) {
            int tot = 0;
#pragma unroll
            for (int c = 0; c < 32; ++c) tot += hist32[(tid << 5) | ((c + tid) & 31)];   // rotated: no bank conflicts
            hist[tid] = tot;
            int sfx = tot;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int t = __shfl_down(sfx, o);
                if (lane + o < 64) sfx += t;
            }
            if (lane == 0) s_weq[wave] = sfx;        // total of this wave's 64 bins
            s_sfx[tid] = sfx;
        }
        __syncthreads();
        if (tid < 256) {
            int above = 0;                           // keys in the bins of the higher waves
            for (int w = wave + 1; w < 4; ++w) above += s_weq[w];
            const int rem = s_rem;
            const int mine = s_sfx[tid] + above;     // keys in bins >= tid
            const int next = mine - hist[tid];       // keys in bins > tid
            if (mine >= rem && next < rem) {         // exactly one bin (counts are >= 0, the total is >= rem)
                s_prefix = prefix | ((uint32_t)tid << shift);
                s_rem_next = rem - next;
            }
        }
        __syncthreads();
        if (tid == 0) s_rem = s_rem_next;
    }
    __syncthreads();
    const uint32_t kth = s_prefix;   // exact key of the want-th largest
    const int need_eq = s_rem;       // how many of the entries equal to it are taken (lowest lists first)
    const int total_eq = hist[(kth)&255];
    const int gt_total = want - need_eq;

    // ---- collection: entries above the cut in any order; entries AT the cut by ascending list
    auto collect_gt = [&](uint32_t kk, int i) {
        const bool g = i < nlist && kk > kth;
        const uint64_t mg = __ballot(g);
        if (mg) {
            int base = 0;
            if (lane == 0) base = atomicAdd(&s_ngt, __popcll(mg));
            base = __builtin_amdgcn_readfirstlane(base);
            if (g) c_idx[base + __popcll(mg & ((1ull << lane) - 1ull))] = i;
        }
    };
    if (REG > 0) {
#pragma unroll
        for (int r = 0; r < NR; ++r) collect_gt(key[r], r * SEL_THREADS + tid);
    } else {
        for (int r = 0; r < nrounds; ++r) collect_gt(key_at(r), r * SEL_THREADS + tid);
    }
    if (total_eq == need_eq) {       // every tie is taken: order is irrelevant here (sorted later)
        auto collect_eq = [&](uint32_t kk, int i) {
            const bool e = i < nlist && kk == kth;
            const uint64_t me = __ballot(e);
            if (me) {
                int base = 0;
                if (lane == 0) base = atomicAdd(&s_neq, __popcll(me));
                base = __builtin_amdgcn_readfirstlane(base);
                if (e) c_idx[gt_total + base + __popcll(me & ((1ull << lane) - 1ull))] = i;
            }
        };
        if (REG > 0) {
#pragma unroll
            for (int r = 0; r < NR; ++r) collect_eq(key[r], r * SEL_THREADS + tid);
        } else {
            for (int r = 0; r < nrounds; ++r) collect_eq(key_at(r), r * SEL_THREADS + tid);
        }
    } else {
        // ties straddle the cut (rare): walk the row in list order, round by round
        int eq_base = 0;
        for (int r = 0; r < nrounds && eq_base < need_eq; ++r) {
            const int i = r * SEL_THREADS + tid;
            uint32_t kk = 0;
            if (REG > 0) {
#pragma unroll
                for (int rr = 0; rr < NR; ++rr) if (rr == r) kk = key[rr];
            } else kk = key_at(r);
            const bool e = i < nlist && kk == kth;
            const uint64_t me = __ballot(e);
            __syncthreads();
            if (lane == 0) s_weq[wave] = __popcll(me);
            __syncthreads();
            int before = 0, tot = 0;
            for (int w = 0; w < SEL_WAVES; ++w) { if (w < wave) before += s_weq[w]; tot += s_weq[w]; }
            const int o = eq_base + before + __popcll(me & ((1ull << lane) - 1ull));
            if (e && o < need_eq) c_idx[gt_total + o] = i;
            eq_base += tot;
        }
    }
    __syncthreads();

    // ---- exact scores of the candidates: fp64 accumulation, one rounding to fp32
    float qn = 0.f;
    for (int t = lane; t < d; t += 64) qn += qv[t] * qv[t];
    for (int o = 32; o; o >>= 1) qn += __shfl_xor(qn, o);
    exact_scores(want, [&](int c) { return c_idx[c]; }, [&](int c, float v) { c_val[c] = v; });
    __syncthreads();
    if (want <= SEL_THREADS) {
        // ---- order by (score desc, list asc): one 64-bit key per candidate (ordered score bits, then the complement
        // of the list number), and every candidate counts the keys above its own: that count is its rank (lists are
        // distinct, so the ranks are a permutation).  The G = 1024 / want thread groups each count a residue class
        // of j; the lanes of a wave read the same key at a time (a broadcast).
        uint64_t* key64 = reinterpret_cast<uint64_t*>(hist32);              // [want]   (the histograms are no longer needed)
        int* rank = hist32 + 2 * SEL_CAP;                                  // [want]
        if (tid < want) {
            key64[tid] = ((uint64_t)float_key(c_val[tid] + 0.0f) << 32)   /* (-0 counts as +0) */
                         | (uint32_t)(0xFFFFFFFFu - (uint32_t)c_idx[tid]);
            rank[tid] = 0;
        }
        __syncthreads();
        const int G = SEL_THREADS / want, c = tid % want, g = tid / want;
        if (g < G) {
            const uint64_t mine = key64[c];
            int above = 0;
            for (int j = g; j < want; j += G) above += key64[j] > mine ? 1 : 0;
            if (above) atomicAdd(&rank[c], above);
        }
        __syncthreads();
        int mine_i = 0, r = 0;
        float mine_v = 0.f;
        if (tid < want) { mine_i = c_idx[tid]; mine_v = c_val[tid]; r = rank[tid]; }
        __syncthreads();                             // every c_idx / c_val read is done
        if (tid < want) { c_idx[r] = mine_i; c_val[r] = mine_v; }
        __syncthreads();
    } else {
        int n2 = 1;
        while (n2 < want) n2 <<= 1;
        for (int i = want + tid; i < n2; i += SEL_THREADS) { c_idx[i] = 0x7fffffff; c_val[i] = -INFINITY; }
        // ---- bitonic sort by (score desc, list asc)
        for (int size = 2; size <= n2; size <<= 1)
            for (int stride = size >> 1; stride > 0; stride >>= 1) {
                __syncthreads();
                for (int t = tid; t < n2 / 2; t += SEL_THREADS) {
                    const int i = 2 * t - (t & (stride - 1)), j = i + stride;
                    const bool up = (i & size) == 0;
                    const float va = c_val[i], vb = c_val[j];
                    const int ia = c_idx[i], ib = c_idx[j];
                    const bool b_first = vb > va || (vb == va && ib < ia);
                    const bool a_first = va > vb || (va == vb && ia < ib);
                    if (up ? b_first : a_first) { c_val[i] = vb; c_val[j] = va; c_idx[i] = ib; c_idx[j] = ia; }
                }
            }
        __syncthreads();
    }
    for (int p = tid; p < nprobe; p += SEL_THREADS) probes[q * nprobe + p] = c_idx[p];
    if (tid == 0 && !redo && want < nlist) {
        // smallest fp32 score among the candidates = score with key `kth`
        const uint32_t u = (kth & 0x80000000u) ? (kth & 0x7fffffffu) : ~kth;
        const float s_cut = __uint_as_float(u);
        // (Euclidean: twice the product's error, plus the roundings of the two squared norms and of the sum)
        float E = ((float)d * 2.384185791015625e-07f + 1.52587890625e-05f) * sqrtf(qn) * max_cnorm;
        if (metric == 1) E = 2.0f * E + 4.76837158203125e-07f * (qn + max_cnorm * max_cnorm);
        E += (float)d * 2.4e-38f;        // products that underflow (the matrix cores may flush subnormal numbers)
        // A list outside the candidates has an exact score <= s_cut + E.  If the nprobe-th exact score is above
        // that, the choice is the one exact scores give.  Otherwise (scores packed closer than the product's
        // error around the cut) the query is queued for the second launch; counters[3] counts them.
        if (!(c_val[nprobe - 1] > s_cut + E))
            redo_q[atomicAdd(reinterpret_cast<unsigned long long*>(counters + 3), 1ull)] = (int32_t)q;
    }
}

// ------------------------------------------------------------------ selection, rows of up to 65536 scores
// One workgroup per query leaves the chip idle when a batch has a handful of queries, and its time is then the
// latency of a request (iterative retrieval, Section 5.3: batches of 1 to 16).  Here up to SS_G workgroups share a
// query (one per query once the batch fills the chip: the single histogram pass still beats four radix passes).
// Each of them finds the same candidate set by itself (the row of scores comes from L2; a histogram over a linear
// map of the row's range finds the cut in one pass; the scores in and above the cut's bin are ordered exactly by
// their fp32 keys), then the exact scores of the candidates - random rows of C from HBM, the expensive step on one
// compute unit - are divided among the workgroups, and the one that finishes last orders the exact scores and
// writes the probes.  A row this scheme cannot handle (not-a-number or infinite scores, no spread, more than
// SS_CAP scores in and above the cut's bin) is queued for the exact second launch of select_kernel.
constexpr int SS_G = 16;            // workgroups per query at most (fewer when the batch fills the chip anyway)
constexpr int SS_BINS = 4096;
constexpr int SS_CAP = 1024;        // scores in and above the cut's bin that are ordered in LDS
constexpr int SS_REG = 64;          // scores per thread at most: nlist <= 65536
constexpr int SS_MAX_WANT = 512;    // nprobe + SEL_EXTRA

// scratch in HBM, per index: exact scores [nq][SS_MAX_WANT], then a count per query of the workgroups that are done
// (zero between launches: the last workgroup resets it)

// rank[c] = number of keys above key[c] (keys distinct), counted by n threads or by several groups of n threads
__device__ __forceinline__ void rank_keys(const uint64_t* key, int n, int* rank, int tid) {
    for (int i = tid; i < n; i += SEL_THREADS) rank[i] = 0;
    __syncthreads();
    const int G = SEL_THREADS / n;              // n <= SEL_THREADS
    const int c = tid % n, gg = tid / n;
    if (gg < G) {
        const uint64_t mine = key[c];
        int above = 0;
#pragma unroll 8
        for (int j = gg; j < n; j += G) above += key[j] > mine ? 1 : 0;      // (independent LDS reads, several in flight)
        if (above) atomicAdd(&rank[c], above);
    }
    __syncthreads();
}

// REG = scores per thread (nlist <= REG * SEL_THREADS: a short row should not pay for 64 loads, clamped or not);
// RU = rows of C a wave scores at a time (random rows from HBM, one round trip per round of the workgroup's waves:
// a workgroup that has a query to itself takes its ~100 rows in one round, one of sixteen has only a few).
// ALONE: gridDim.y == 1, the workgroup has the query to itself: the exact scores stay in LDS, and the two round trips
// to memory that pass them between workgroups (store and acknowledge, count and read back) fall away.
template <int REG, int RU, bool ALONE>
__global__ void __launch_bounds__(SEL_THREADS) select_small_kernel(const float* __restrict__ Q, const float* __restrict__ C,
                                                                   const float* __restrict__ S, int nlist, int d, int nprobe,
                                                                   float max_cnorm, int metric, int32_t* __restrict__ probes,
                                                                   int64_t* counters, int32_t* redo_q, float* exact, int* done) {
    __shared__ int hist[SS_BINS];
    __shared__ uint64_t c_key[SS_CAP];          // (ordered score bits << 32) | ~list: descending = (score desc, list asc)
    __shared__ int rank[SS_CAP];
    __shared__ uint64_t sel_key[SS_MAX_WANT];   // the chosen candidates in descending key order
    __shared__ float s_red[2 * SEL_WAVES];
    __shared__ int s_wtot[SEL_WAVES];
    __shared__ int s_bin, s_ncand, s_cnt, s_last;
    const int q = blockIdx.x, g = blockIdx.y, G = gridDim.y;     // (queries along x: any batch size fits the grid)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* row = S + (int64_t)q * nlist;
    exact += (int64_t)q * SS_MAX_WANT;
    const int want = nprobe + SEL_EXTRA;        // < nlist and <= SS_MAX_WANT (the launcher's conditions)
    if (tid == 0) s_cnt = 0;

    // ---- the row, its range
    // (unconditional loads from a clamped index: a branch per element would make every load wait for the one before)
    float v[REG];
    float lo = INFINITY, hi = -INFINITY;
    bool odd = false;
#pragma unroll
    for (int r = 0; r < REG; ++r) v[r] = row[min(r * SEL_THREADS + tid, nlist - 1)];
#pragma unroll
    for (int r = 0; r < REG; ++r) {          // (a repeated last element changes neither the range nor `odd`)
        lo = fminf(lo, v[r]); hi = fmaxf(hi, v[r]);
        odd |= !(fabsf(v[r]) <= 3.0e38f);       // not a number, or infinite
    }
    for (int o = 32; o; o >>= 1) { lo = fminf(lo, __shfl_xor(lo, o)); hi = fmaxf(hi, __shfl_xor(hi, o)); }
    if (lane == 0) { s_red[wave] = lo; s_red[SEL_WAVES + wave] = hi; }
    for (int i = tid; i < SS_BINS; i += SEL_THREADS) hist[i] = 0;
    const int any_odd = __syncthreads_or(odd ? 1 : 0);
    for (int w = 0; w < SEL_WAVES; ++w) { lo = fminf(lo, s_red[w]); hi = fmaxf(hi, s_red[SEL_WAVES + w]); }
    const float scale = (float)SS_BINS / (hi - lo);
    // (every workgroup of the query takes the same decisions: they depend on the row only)
    // (a row whose scores all lie within 2^-9 of their magnitude goes to the exact launch: the bins would be as
    // narrow as the rounding errors of the map)
    bool give_up = any_odd || !(hi > lo) || !(scale <= 3.0e38f) || !((hi - lo) * 512.f > fmaxf(fabsf(lo), fabsf(hi)));
    // monotone in the score: subtraction, multiplication by a positive number and truncation all are
    auto bin_of = [&](float x) { return (int)fminf(fmaxf((x - lo) * scale, 0.f), (float)(SS_BINS - 1)); };
    if (!give_up) {
#pragma unroll
        for (int r = 0; r < REG; ++r)
            if (r * SEL_THREADS + tid < nlist) atomicAdd(&hist[bin_of(v[r])], 1);
    }
    __syncthreads();
    // ---- the highest bin b with at least `want` scores in bins >= b: thread t owns bins 4t .. 4t+3
    {
        const int h0 = hist[4 * tid], h1 = hist[4 * tid + 1], h2 = hist[4 * tid + 2], h3 = hist[4 * tid + 3];
        const int own = h0 + h1 + h2 + h3;
        int sfx = own;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_down(sfx, o);
            if (lane + o < 64) sfx += t;
        }
        if (lane == 0) s_wtot[wave] = sfx;
        __syncthreads();
        int above = 0;
        for (int w = wave + 1; w < SEL_WAVES; ++w) above += s_wtot[w];
        const int incl = sfx + above, excl = incl - own;          // scores in bins >= 4t, in bins > 4t+3
        if (!give_up && incl >= want && excl < want) {            // exactly one thread (nlist > want)
            int cum = excl, b = 4 * tid + 3;
            const int hh[4] = {h0, h1, h2, h3};
            for (;; --b) {
                cum += hh[b - 4 * tid];
                if (cum >= want || b == 4 * tid) break;
            }
            s_bin = b; s_ncand = cum;
        }
        __syncthreads();
    }
    if (give_up || s_ncand > SS_CAP - 64) {
        if (g == 0 && tid == 0) redo_q[atomicAdd(reinterpret_cast<unsigned long long*>(counters + 3), 1ull)] = q;
        return;
    }
    // ---- the candidates: every score whose bin is at least the cut's lies above `floor_v`, one bin width below the
    // cut's lower edge (a bin width is at least 8 times the rounding errors of the map and of `floor_v`: the range is
    // more than 2^-9 of the magnitudes, a bin 2^-12 of the range, an error 2^-24 of the magnitudes), and one
    // comparison per score is cheaper than the map; the few extra scores between the two are ordered like the rest.  They are ordered
    // by their exact 64-bit keys, the first `want` are chosen.
    const float floor_v = lo + (float)(s_bin - 1) / scale;
#pragma unroll
    for (int r = 0; r < REG; ++r) {
        const int i = r * SEL_THREADS + tid;
        const bool in = i < nlist && v[r] >= floor_v;
        const uint64_t m = __ballot(in);
        if (m) {
            int base = 0;
            if (lane == 0) base = atomicAdd(&s_cnt, __popcll(m));
            base = __builtin_amdgcn_readfirstlane(base);
            const int pos = base + __popcll(m & ((1ull << lane) - 1ull));
            if (in && pos < SS_CAP) c_key[pos] = ((uint64_t)float_key(v[r]) << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)i);
        }
    }
    __syncthreads();
    const int ncand = s_cnt;
    if (ncand > SS_CAP) {                       // (the same in every workgroup of the query)
        if (g == 0 && tid == 0) redo_q[atomicAdd(reinterpret_cast<unsigned long long*>(counters + 3), 1ull)] = q;
        return;
    }
    rank_keys(c_key, ncand, rank, tid);
    if (tid < ncand && rank[tid] < want) sel_key[rank[tid]] = c_key[tid];
    __syncthreads();

    // ---- exact scores (fp64 accumulation, one rounding to fp32) of this workgroup's share: ranks g, g + G, ...
    const float* qv = Q + (int64_t)q * d;
    const bool vec4 = (d & 3) == 0;
    const int nmine = (want - g + G - 1) / G;
    for (int c0 = wave * RU; c0 < nmine; c0 += SEL_WAVES * RU) {
        double acc[RU];
        const float* cv[RU];
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            acc[u] = 0.0;
            const int pos = g + min(c0 + u, nmine - 1) * G;
            cv[u] = C + (int64_t)(0xFFFFFFFFu - (uint32_t)sel_key[pos]) * d;
        }
        if (vec4) {
            // (the loads of the next trip round the loop go out ahead of this trip's arithmetic: one round trip to the
            // rows in all instead of one per 256 dimensions)
            float4 q4n = make_float4(0.f, 0.f, 0.f, 0.f), c4n[RU];
#pragma unroll
            for (int u = 0; u < RU; ++u) c4n[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (lane * 4 < d) {
                q4n = *reinterpret_cast<const float4*>(qv + lane * 4);
#pragma unroll
                for (int u = 0; u < RU; ++u) c4n[u] = *reinterpret_cast<const float4*>(cv[u] + lane * 4);
            }
            for (int t = lane * 4; t < d; t += 256) {
                const float4 q4 = q4n;
                float4 c4[RU];
#pragma unroll
                for (int u = 0; u < RU; ++u) c4[u] = c4n[u];
                if (t + 256 < d) {
                    q4n = *reinterpret_cast<const float4*>(qv + t + 256);
#pragma unroll
                    for (int u = 0; u < RU; ++u) c4n[u] = *reinterpret_cast<const float4*>(cv[u] + t + 256);
                }
                const double qa[4] = {(double)q4.x, (double)q4.y, (double)q4.z, (double)q4.w};
#pragma unroll
                for (int u = 0; u < RU; ++u) {
                    const double ca[4] = {(double)c4[u].x, (double)c4[u].y, (double)c4[u].z, (double)c4[u].w};
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        if (metric == 1) { const double diff = qa[x] - ca[x]; acc[u] = acc[u] + diff * diff; }
                        else acc[u] = acc[u] + qa[x] * ca[x];
                    }
                }
            }
        } else {
            for (int t = lane; t < d; t += 64) {
                const double qt = (double)qv[t];
#pragma unroll
                for (int u = 0; u < RU; ++u) {
                    if (metric == 1) { const double diff = qt - (double)cv[u][t]; acc[u] = acc[u] + diff * diff; }
                    else acc[u] = acc[u] + qt * (double)cv[u][t];
                }
            }
        }
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            for (int o = 32; o; o >>= 1) acc[u] = acc[u] + __shfl_xor(acc[u], o);
            if (lane == 0 && c0 + u < nmine) {
                const float ex = metric == 1 ? (float)(-acc[u]) : (float)acc[u];
                if constexpr (ALONE) reinterpret_cast<float*>(hist)[c0 + u] = ex;      // (the histogram has served; G = 1: position c0 + u)
                else __hip_atomic_store(&exact[g + (c0 + u) * G], ex, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
    // ---- the workgroup that finishes last goes on.  The exact scores were written by device-scope atomic stores, which
    // go through to where every compute unit's device-scope loads read them; once they are acknowledged (the wait)
    // the count may be raised.  (A release fence would also write back every dirty line of this chiplet's L2 -
    // here the whole score matrix the kernel before has just written - and was measured at 4 to 55 us.)
    if constexpr (ALONE) {
        __syncthreads();
    } else {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) s_last = atomicAdd(&done[q], 1) == G - 1;
        __syncthreads();
        if (!s_last) return;
    }
    // ---- order by (exact score desc, list asc); c_key and rank are free again
    if (tid < want) {
        const float ex = ALONE ? reinterpret_cast<const float*>(hist)[tid] : __hip_atomic_load(&exact[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        c_key[tid] = ((uint64_t)float_key(ex + 0.0f) << 32) /* (-0 counts as +0) */ | (uint32_t)sel_key[tid];
    }
    __syncthreads();
    rank_keys(c_key, want, rank, tid);
    if (tid < want && rank[tid] < nprobe) probes[(int64_t)q * nprobe + rank[tid]] = (int32_t)(0xFFFFFFFFu - (uint32_t)c_key[tid]);
    if (tid < want && rank[tid] == nprobe - 1) hist[0] = (int)(c_key[tid] >> 32);     // key of the nprobe-th exact score
    float qn = 0.f;
    if (wave == 0) {
        for (int t = lane; t < d; t += 64) qn += qv[t] * qv[t];
        for (int o = 32; o; o >>= 1) qn += __shfl_xor(qn, o);
    }
    __syncthreads();
    if (tid == 0) {
        if (!ALONE) done[q] = 0;
        auto unkey = [](uint32_t kk) { return __uint_as_float((kk & 0x80000000u) ? (kk & 0x7fffffffu) : ~kk); };
        const float s_cut = unkey((uint32_t)(sel_key[want - 1] >> 32));   // smallest fp32 score among the candidates
        const float nth = unkey((uint32_t)hist[0]);
        // (the same bound and the same rule as in select_kernel)
        float E = ((float)d * 2.384185791015625e-07f + 1.52587890625e-05f) * sqrtf(qn) * max_cnorm;
        if (metric == 1) E = 2.0f * E + 4.76837158203125e-07f * (qn + max_cnorm * max_cnorm);
        E += (float)d * 2.4e-38f;
        if (!(nth > s_cut + E))
            redo_q[atomicAdd(reinterpret_cast<unsigned long long*>(counters + 3), 1ull)] = q;
    }
}

__global__ void zero_counter_kernel(int64_t* counters) { counters[3] = 0; }

int launch_select(rago_index* idx, const float* q, float* S, int64_t nq, int nprobe, int32_t* probes, hipStream_t st, bool counter_is_zero) {
    if (nprobe + SEL_EXTRA > SEL_CAP && nprobe < idx->nlist && idx->nlist > SEL_CAP)
        return fail(RAGO_UNSUPPORTED, "nprobe > 2016 on an index with more than 2048 lists");
    if (std::min(nprobe + SEL_EXTRA, idx->nlist) > SEL_CAP) return fail(RAGO_UNSUPPORTED, "nprobe > 2016");
    int rc;
    if ((rc = idx->ws.counters.reserve(64))) return rc;
    if ((rc = idx->ws.sel_redo.reserve((size_t)nq * 4))) return rc;
    {   // scratch of the kernel for short rows (whatever this batch takes: a later one must not have to allocate)
        if ((rc = idx->ws.sel_small.reserve((size_t)nq * SS_MAX_WANT * 4))) return rc;
        const void* before = idx->ws.sel_done.p;
        if ((rc = idx->ws.sel_done.reserve((size_t)nq * 4))) return rc;
        if (idx->ws.sel_done.p != before) RAGO_HIP(hipMemset(idx->ws.sel_done.p, 0, idx->ws.sel_done.cap));   // the counts start at zero
    }
    if (idx->reserving) return RAGO_OK;
    if (!counter_is_zero) zero_counter_kernel<<<1, 1, 0, st>>>(idx->ws.counters.as<int64_t>());
    int64_t* cnt = idx->ws.counters.as<int64_t>();
    int32_t* rq = idx->ws.sel_redo.as<int32_t>();
    const int nl = idx->nlist;
    // first the whole batch on the approximate scores, then (second launch, whose workgroups leave at once when
    // the first queued nothing) the queued queries on exact ones
    // rows of at most 65536 scores: one histogram pass instead of four, and the exact rescoring shared among a query's
    // workgroups while the batch leaves compute units idle
    // As many workgroups per query as leave every workgroup a compute unit of its own (each repeats the histogram;
    // measured with 256 queries x 16384 lists: two per query 59 us, one 40, the kernel that passes over its
    // registers four times 44; with 1024 queries x 65536 lists: one per query 0.21 ms against 0.34).
    const bool small = nl <= SS_REG * SEL_THREADS && nprobe + SEL_EXTRA < nl && nprobe + SEL_EXTRA <= SS_MAX_WANT;
    const unsigned ss_g = (unsigned)std::max<int64_t>(1, std::min<int64_t>(SS_G, idx->n_cu / nq));
    float* ss_exact = idx->ws.sel_small.as<float>();
    int* ss_done = idx->ws.sel_done.as<int>();      // (nothing else ever writes here: zero between launches)
    for (int redo = 0; redo < 2; ++redo) {
        if (small && !redo) {
            auto go = [&](auto kern) {
                kern<<<dim3((unsigned)nq, ss_g), SEL_THREADS, 0, st>>>(q, idx->centroids, S, nl, idx->d, nprobe, idx->max_cnorm, idx->metric, probes, cnt,
                                                                       rq, ss_exact, ss_done);
            };
            const bool alone = ss_g == 1;
            if (nl <= 16 * SEL_THREADS) { if (alone) go(select_small_kernel<16, 6, true>); else go(select_small_kernel<16, 2, false>); }
            else if (nl <= 32 * SEL_THREADS) { if (alone) go(select_small_kernel<32, 6, true>); else go(select_small_kernel<32, 2, false>); }
            else { if (alone) go(select_small_kernel<64, 6, true>); else go(select_small_kernel<64, 2, false>); }
        }
        else if (nl <= 8 * SEL_THREADS)
            select_kernel<8><<<(unsigned)nq, SEL_THREADS, 0, st>>>(q, idx->centroids, S, nl, idx->d, nprobe, idx->max_cnorm, idx->metric, probes, cnt, rq, redo);
        else if (nl <= 32 * SEL_THREADS)
            select_kernel<32><<<(unsigned)nq, SEL_THREADS, 0, st>>>(q, idx->centroids, S, nl, idx->d, nprobe, idx->max_cnorm, idx->metric, probes, cnt, rq, redo);
        else if (nl <= 64 * SEL_THREADS)
            select_kernel<64><<<(unsigned)nq, SEL_THREADS, 0, st>>>(q, idx->centroids, S, nl, idx->d, nprobe, idx->max_cnorm, idx->metric, probes, cnt, rq, redo);
        else
            select_kernel<0><<<(unsigned)nq, SEL_THREADS, 0, st>>>(q, idx->centroids, S, nl, idx->d, nprobe, idx->max_cnorm, idx->metric, probes, cnt, rq, redo);
    }
    RAGO_HIP(hipGetLastError());
    return RAGO_OK;
}

}  // namespace rago

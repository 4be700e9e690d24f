// Euclidean-metric tables, fast path: L[q,p][j][c] = -|q_j - (C[l]_j + CB[j][c])|^2 for every
// (query, list) pair (the metric of Section 2 under which the tables no longer factorise).
//
// The entry is DEFINED by an fp64 accumulation rounded once to fp32, and everything derived from it
// (sub-table minima, the query's step, the 8-bit codes) must come out as from that definition.
// Evaluating all m*256 entries of all pairs twice in fp64 costs ~5 fp64-rate operations per term.
// Here both passes evaluate in fp32 with a proven error bound and go back to the fp64 definition
// only for the entries whose outcome the bound cannot decide:
//
//   fp32 evaluation  r_t = fl(q_t - c_t), e_t = fl(r_t - cb_t), acc = fma(e_t, e_t, acc):
//   |L~ - L64| <= (dsub + 4) u M,  M = sum_t (|q_t| + |c_t| + max_c |cb_t|)^2,  u = 2^-24;
//   E = 2 (dsub + 6) u M is used (twice the bound, which also covers the rounding of E itself).
//
//   pass 1 (minima, range): the entry attaining the exact minimum of a sub-table has
//   L~ <= min L~ + 2E, so the exact minimum is the least fp32(fp64) value among those candidates;
//   same for the maximum.  Typically 2-4 candidates per sub-table.
//   pass 2 (codes): b~ = (L~ - lo) * (1/dq) differs from the defining fp32 value
//   b = fl(fl(L - lo) / dq) by at most eta = (E + u M)/dq + 2^-13; if b~ is farther than eta from
//   every half-integer, rint(b~) = rint(b).  Otherwise (about one entry in a thousand) the entry
//   is put on a list and evaluated by the definition.
//
// Candidates and undecided entries are collected in LDS and evaluated afterwards with all lanes
// busy.  If a list overflows (tables that are flat relative to their magnitude make every entry
// undecidable) the workgroup evaluates all its entries by the definition.
//
// A workgroup handles P consecutive pairs so that one load of a codeword serves P tables (the
// codebooks are the same for every pair; one pair per workgroup re-reads m*256*dsub*4 bytes from
// L2 per pair and pass).  Pass 1: wave = sub-quantiser, lane = codewords lane + 64 i (min/max are
// lane-local over i, then one wave reduction).  Pass 2: wave = (plane, 64 codewords), lane =
// codeword, loop over the 32 slots of the plane, the 32 code bytes of (codeword, plane) packed in
// registers and written with two 16-byte stores per lane: the plane-major table
// [plane][codeword][slot] goes to HBM coalesced without a copy in LDS.
#include "rago_internal.h"
#include "lut_common.h"

namespace rago {

namespace {

constexpr int L2F_THREADS = 256;
constexpr int L2F_LIST = 4096;          // list entries (4 bytes each) per workgroup

__device__ __forceinline__ uint32_t okey(float f) {            // order-preserving map float -> uint32
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float okey_inv(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

template <int DSUB>
__device__ __forceinline__ void load_vec(const float* __restrict__ p, float (&v)[DSUB]) {
    static_assert(DSUB % 4 == 0, "16-byte loads");
#pragma unroll
    for (int t = 0; t < DSUB; t += 4) {
        const float4 x = *reinterpret_cast<const float4*>(p + t);
        v[t] = x.x; v[t + 1] = x.y; v[t + 2] = x.z; v[t + 3] = x.w;
    }
}

template <int DSUB>
__device__ __forceinline__ float l2_approx(const float* __restrict__ r, const float (&cb)[DSUB]) {
    float acc = 0.0f;
#pragma unroll
    for (int t = 0; t < DSUB; ++t) {
        const float e = r[t] - cb[t];
        acc = __fmaf_rn(e, e, acc);
    }
    return -acc;
}

// r[p][t] = fl(q_t - c_t), E[p][j] for the workgroup's pairs.
template <int DSUB>
__device__ __forceinline__ void prepare_pairs(const float* __restrict__ Q, const float* __restrict__ C, const float* __restrict__ cbmax,
                                              const int32_t* __restrict__ probes, int64_t pair0, int np, int nprobe, int d, int m,
                                              float* __restrict__ r, float* __restrict__ E, float* __restrict__ Mj) {
    for (int idx = threadIdx.x; idx < np * d; idx += L2F_THREADS) {
        const int p = idx / d, t = idx - p * d;
        const int64_t q = (pair0 + p) / nprobe;
        const int l = probes[pair0 + p];
        r[p * d + t] = Q[q * d + t] - C[(int64_t)l * d + t];
    }
    for (int idx = threadIdx.x; idx < np * m; idx += L2F_THREADS) {
        const int p = idx / m, j = idx - p * m;
        const int64_t q = (pair0 + p) / nprobe;
        const int l = probes[pair0 + p];
        float M = 0.0f;
        for (int t = 0; t < DSUB; ++t) {
            const int x = j * DSUB + t;
            const float a = fabsf(Q[q * d + x]) + fabsf(C[(int64_t)l * d + x]) + cbmax[x];
            M = __fmaf_rn(a, a, M);
        }
        Mj[p * m + j] = M;
        E[p * m + j] = 2.0f * (float)(DSUB + 6) * 5.9604644775390625e-08f * M;
    }
}

// ---- pass 1
template <int DSUB, int P>
__global__ void __launch_bounds__(L2F_THREADS) l2f_range_kernel(const float* __restrict__ Q, const float* __restrict__ C,
                                                                const float* __restrict__ CB, const float* __restrict__ cbmax,
                                                                const int32_t* __restrict__ probes, int64_t npairs, int nprobe, int d,
                                                                int m, float* __restrict__ lo_out, uint32_t* __restrict__ range_bits,
                                                                int64_t* __restrict__ counters) {
    extern __shared__ __align__(16) uint8_t smem[];
    float* r = reinterpret_cast<float*>(smem);                       // [P][d]
    float* E = r + P * d;                                            // [P][m]
    float* Mj = E + P * m;                                           // [P][m]
    uint32_t* lo_key = reinterpret_cast<uint32_t*>(Mj + P * m);      // [P][m]
    uint32_t* hi_key = lo_key + P * m;                               // [P][m]
    uint32_t* list = hi_key + P * m;                                 // [L2F_LIST]  p << 16 | j << 8 | c
    __shared__ int nlist;
    __shared__ float s_rng[P];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t pair0 = (int64_t)blockIdx.x * P;
    const int np = (int)min((int64_t)P, npairs - pair0);
    prepare_pairs<DSUB>(Q, C, cbmax, probes, pair0, np, nprobe, d, m, r, E, Mj);
    for (int idx = threadIdx.x; idx < P * m; idx += L2F_THREADS) { lo_key[idx] = 0xFFFFFFFFu; hi_key[idx] = 0u; }
    if (threadIdx.x == 0) nlist = 0;
    if (threadIdx.x < P) s_rng[threadIdx.x] = 0.0f;
    __syncthreads();

    for (int j = wave; j < m; j += 4) {
        float cb[4][DSUB];
#pragma unroll
        for (int i = 0; i < 4; ++i) load_vec<DSUB>(CB + ((int64_t)j * KSUB + lane + 64 * i) * DSUB, cb[i]);
#pragma unroll
        for (int p = 0; p < P; ++p) {
            if (p < np) {
                const float* rp = r + p * d + j * DSUB;
                float v[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = l2_approx<DSUB>(rp, cb[i]);
                float mn = fminf(fminf(v[0], v[1]), fminf(v[2], v[3]));
                float mx = fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3]));
                for (int o = 32; o; o >>= 1) { mn = fminf(mn, __shfl_xor(mn, o)); mx = fmaxf(mx, __shfl_xor(mx, o)); }
                const float marg = 2.0f * E[p * m + j];
                const float lo_cut = mn + marg, hi_cut = mx - marg;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (v[i] <= lo_cut || v[i] >= hi_cut) {
                        const int pos = atomicAdd(&nlist, 1);
                        if (pos < L2F_LIST) list[pos] = (uint32_t)(p << 16 | j << 8 | (lane + 64 * i));
                    }
                }
            }
        }
    }
    __syncthreads();
    const int n = nlist;
    const bool all = n > L2F_LIST;                 // undecidable almost everywhere: evaluate every entry by the definition
    const int total = all ? np * m * KSUB : n;
    for (int e = threadIdx.x; e < total; e += L2F_THREADS) {
        const uint32_t w = all ? (uint32_t)((e / (m * KSUB)) << 16 | ((e / KSUB) % m) << 8 | (e % KSUB)) : list[e];
        const int p = w >> 16, j = (w >> 8) & 255, c = w & 255;
        const int64_t q = (pair0 + p) / nprobe;
        const int l = probes[pair0 + p];
        const float L = l2_entry<DSUB>(Q + q * d + j * DSUB, C + (int64_t)l * d + j * DSUB, CB + ((int64_t)j * KSUB + c) * DSUB, DSUB);
        const uint32_t k = okey(L);
        atomicMin(&lo_key[p * m + j], k);
        atomicMax(&hi_key[p * m + j], k);
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < np * m; idx += L2F_THREADS) {
        const int p = idx / m;
        const float lo = okey_inv(lo_key[idx]), hi = okey_inv(hi_key[idx]);
        lo_out[(pair0 + p) * m + (idx - p * m)] = lo;
        const float rng = hi - lo;
        if (rng > 0.0f) atomicMax(reinterpret_cast<uint32_t*>(&s_rng[p]), __float_as_uint(rng));
    }
    __syncthreads();
    if (threadIdx.x < np) {
        const float rng = s_rng[threadIdx.x];
        if (rng > 0.0f) atomicMax(range_bits + (pair0 + threadIdx.x) / nprobe, __float_as_uint(rng));
    }
    if (threadIdx.x == 0) {
        atomicAdd(reinterpret_cast<unsigned long long*>(counters + 4), (unsigned long long)total);
        if (all) atomicAdd(reinterpret_cast<unsigned long long*>(counters + 5), 1ull);
    }
}

// ---- pass 2
template <int DSUB, int P>
__global__ void __launch_bounds__(L2F_THREADS) l2f_quant_kernel(const float* __restrict__ Q, const float* __restrict__ C,
                                                                const float* __restrict__ CB, const float* __restrict__ cbmax,
                                                                const int32_t* __restrict__ probes, int64_t npairs, int nprobe, int d,
                                                                int m, const float* __restrict__ lo_in, const uint32_t* __restrict__ range_bits,
                                                                uint8_t* __restrict__ tables, int32_t* __restrict__ bias,
                                                                float* __restrict__ delta, uint8_t* __restrict__ out_LUT8,
                                                                int64_t* __restrict__ counters) {
    extern __shared__ __align__(16) uint8_t smem[];
    float* r = reinterpret_cast<float*>(smem);                       // [P][d]
    float* E = r + P * d;                                            // [P][m]   here: eta, the undecided zone of b~
    float* Mj = E + P * m;                                           // [P][m]
    float* lo = Mj + P * m;                                          // [P][m]
    uint32_t* list = reinterpret_cast<uint32_t*>(lo + P * m);        // [L2F_LIST]
    __shared__ int nlist;
    __shared__ float s_dq[P], s_inv[P];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t pair0 = (int64_t)blockIdx.x * P;
    const int np = (int)min((int64_t)P, npairs - pair0);
    const int S = rago_steps(m), planes = rago_planes(m);
    prepare_pairs<DSUB>(Q, C, cbmax, probes, pair0, np, nprobe, d, m, r, E, Mj);
    if (threadIdx.x == 0) nlist = 0;
    if (threadIdx.x < np) {
        const float dq = lut_step(__uint_as_float(range_bits[(pair0 + threadIdx.x) / nprobe]));
        s_dq[threadIdx.x] = dq;
        s_inv[threadIdx.x] = 1.0f / dq;
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < np * m; idx += L2F_THREADS) {
        const int p = idx / m;
        lo[idx] = lo_in[(pair0 + p) * m + (idx - p * m)];
        E[idx] = (E[idx] + 5.9604644775390625e-08f * Mj[idx]) * s_inv[p] * 1.001f + 1.220703125e-4f;
    }
    __syncthreads();

    for (int u = wave; u < planes * 4; u += 4) {
        const int plane = u >> 2, c = (u & 3) * 64 + lane;
        // pk[p][0..7]: the 32 code bytes of (codeword c, this plane) for pair p.  The words are produced in
        // order and shifted in at the top, so that no register is indexed by a loop variable.
        uint32_t pk[P][8];
#pragma unroll
        for (int p = 0; p < P; ++p)
#pragma unroll
            for (int w = 0; w < 8; ++w) pk[p][w] = 0u;
#pragma unroll 1
        for (int w = 0; w < S / 4; ++w) {
            uint32_t word[P];
#pragma unroll
            for (int p = 0; p < P; ++p) word[p] = 0u;
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
                const int j = plane * 32 + w * 4 + s4;
                float cb[DSUB];
                load_vec<DSUB>(CB + ((int64_t)j * KSUB + c) * DSUB, cb);
#pragma unroll
                for (int p = 0; p < P; ++p) {
                    if (p < np) {
                        const float Lt = l2_approx<DSUB>(r + p * d + j * DSUB, cb);
                        const float b = (Lt - lo[p * m + j]) * s_inv[p];
                        float rr = rintf(b);
                        rr = rr < 0.0f ? 0.0f : (rr > 255.0f ? 255.0f : rr);
                        const uint32_t v = (uint32_t)rr;
                        const float fr = b - floorf(b);
                        if (fabsf(fr - 0.5f) <= E[p * m + j]) {
                            const int pos = atomicAdd(&nlist, 1);
                            if (pos < L2F_LIST) list[pos] = (uint32_t)(p << 16 | j << 8 | c);
                        }
                        word[p] |= v << (8 * s4);
                        if (out_LUT8) out_LUT8[((pair0 + p) * m + j) * KSUB + c] = (uint8_t)v;
                    }
                }
            }
#pragma unroll
            for (int p = 0; p < P; ++p) {
#pragma unroll
                for (int x = 0; x < 7; ++x) pk[p][x] = pk[p][x + 1];
                pk[p][7] = word[p];
            }
        }
        if (S == 16) {                  // fewer than 32 sub-quantisers: slots 16..31 repeat slots 0..15
#pragma unroll
            for (int p = 0; p < P; ++p)
#pragma unroll
                for (int x = 0; x < 4; ++x) pk[p][x] = pk[p][x + 4];
        }
#pragma unroll
        for (int p = 0; p < P; ++p) {
            if (p < np) {
                uint4* dst = reinterpret_cast<uint4*>(tables + (pair0 + p) * LUT_BYTES + (int64_t)plane * LUT_PLANE + c * 32);
                dst[0] = make_uint4(pk[p][0], pk[p][1], pk[p][2], pk[p][3]);
                dst[1] = make_uint4(pk[p][4], pk[p][5], pk[p][6], pk[p][7]);
            }
        }
    }
    __threadfence();
    __syncthreads();                                 // the packed stores are complete before single bytes are corrected
    const int n = nlist;
    const bool all = n > L2F_LIST;
    const int total = all ? np * m * KSUB : n;
    for (int e = threadIdx.x; e < total; e += L2F_THREADS) {
        const uint32_t w = all ? (uint32_t)((e / (m * KSUB)) << 16 | ((e / KSUB) % m) << 8 | (e % KSUB)) : list[e];
        const int p = w >> 16, j = (w >> 8) & 255, c = w & 255;
        const int64_t q = (pair0 + p) / nprobe;
        const int l = probes[pair0 + p];
        const float L = l2_entry<DSUB>(Q + q * d + j * DSUB, C + (int64_t)l * d + j * DSUB, CB + ((int64_t)j * KSUB + c) * DSUB, DSUB);
        float rr = rintf(__fdiv_rn(L - lo[p * m + j], s_dq[p]));
        rr = rr < 0.0f ? 0.0f : (rr > 255.0f ? 255.0f : rr);
        const uint8_t v = (uint8_t)rr;
        uint8_t* tab = tables + (pair0 + p) * LUT_BYTES + (int64_t)(j >> 5) * LUT_PLANE + c * 32;
        for (int rep = j & (S - 1); rep < 32; rep += S) tab[rep] = v;
        if (out_LUT8) out_LUT8[((pair0 + p) * m + j) * KSUB + c] = v;
    }
    if (threadIdx.x < np) {
        const int p = threadIdx.x;
        double losum = 0.0;
        for (int j = 0; j < m; ++j) losum = losum + (double)lo[p * m + j];
        bias[pair0 + p] = (int32_t)rint(losum / (double)s_dq[p]);
        if ((pair0 + p) % nprobe == 0) delta[(pair0 + p) / nprobe] = s_dq[p];
    }
    if (threadIdx.x == 0) {
        atomicAdd(reinterpret_cast<unsigned long long*>(counters + 4), (unsigned long long)total);
        if (all) atomicAdd(reinterpret_cast<unsigned long long*>(counters + 5), 1ull);
    }
}

// max over codewords of |CB[j][c][t]| for every dimension (j, t)
__global__ void __launch_bounds__(256) cb_absmax_kernel(const float* __restrict__ CB, int d, int dsub, float* __restrict__ out) {
    const int x = blockIdx.x * 256 + threadIdx.x;
    if (x >= d) return;
    const int j = x / dsub, t = x - j * dsub;
    float mx = 0.0f;
    for (int c = 0; c < KSUB; ++c) mx = fmaxf(mx, fabsf(CB[((int64_t)j * KSUB + c) * dsub + t]));
    out[x] = mx;
}

template <int DSUB, int P>
int launch_l2f(rago_index* idx, const float* q, const int32_t* probes, int64_t npairs, int nprobe, float* lo, uint32_t* range_bits,
               uint8_t* out_LUT8, hipStream_t st) {
    Workspace& ws = idx->ws;
    const int d = idx->d, m = idx->m;
    const size_t lds1 = (size_t)P * d * 4 + (size_t)P * m * 16 + (size_t)L2F_LIST * 4;
    const size_t lds2 = (size_t)P * d * 4 + (size_t)P * m * 12 + (size_t)L2F_LIST * 4;
    static bool attr_done = false;
    if (!attr_done) {
        RAGO_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(l2f_range_kernel<DSUB, P>), hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024));
        RAGO_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(l2f_quant_kernel<DSUB, P>), hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024));
        attr_done = true;
    }
    const unsigned grid = (unsigned)((npairs + P - 1) / P);
    l2f_range_kernel<DSUB, P><<<grid, L2F_THREADS, lds1, st>>>(q, idx->centroids, idx->codebooks, idx->cb_absmax, probes, npairs, nprobe, d, m,
                                                               lo, range_bits, ws.counters.as<int64_t>());
    l2f_quant_kernel<DSUB, P><<<grid, L2F_THREADS, lds2, st>>>(q, idx->centroids, idx->codebooks, idx->cb_absmax, probes, npairs, nprobe, d, m,
                                                               lo, range_bits, ws.tmp_lut8sw.as<uint8_t>(), ws.bias.as<int32_t>(),
                                                               ws.delta.as<float>(), out_LUT8, ws.counters.as<int64_t>());
    RAGO_HIP(hipGetLastError());
    return RAGO_OK;
}

}  // namespace

int launch_cb_absmax(rago_index* idx, hipStream_t st) {
    cb_absmax_kernel<<<(idx->d + 255) / 256, 256, 0, st>>>(idx->codebooks, idx->d, idx->dsub, idx->cb_absmax);
    RAGO_HIP(hipGetLastError());
    return RAGO_OK;
}

bool lut_l2_fast_supported(const rago_index* idx) {
    const int dsub = idx->dsub;
    return (dsub == 4 || dsub == 8 || dsub == 16) && idx->d <= 4096;
}

// Both passes for all pairs.  `lo` [npairs][m] fp32 and `range_bits` [nq] (zeroed) are workspace; the
// tables, bias and step land in the workspace members the scan reads.
int launch_lut_l2_fast(rago_index* idx, const float* q, const int32_t* probes, int64_t npairs, int nprobe, float* lo, uint32_t* range_bits,
                       uint8_t* out_LUT8, hipStream_t st) {
    const bool wide = idx->d <= 1024;              // eight pairs per workgroup fit the LDS; else two
    switch (idx->dsub) {
        case 4: return wide ? launch_l2f<4, 8>(idx, q, probes, npairs, nprobe, lo, range_bits, out_LUT8, st)
                            : launch_l2f<4, 2>(idx, q, probes, npairs, nprobe, lo, range_bits, out_LUT8, st);
        case 8: return wide ? launch_l2f<8, 8>(idx, q, probes, npairs, nprobe, lo, range_bits, out_LUT8, st)
                            : launch_l2f<8, 2>(idx, q, probes, npairs, nprobe, lo, range_bits, out_LUT8, st);
        case 16: return wide ? launch_l2f<16, 8>(idx, q, probes, npairs, nprobe, lo, range_bits, out_LUT8, st)
                             : launch_l2f<16, 2>(idx, q, probes, npairs, nprobe, lo, range_bits, out_LUT8, st);
    }
    return fail(RAGO_UNSUPPORTED, "sub-vector length without a fast Euclidean table path");
}

}  // namespace rago

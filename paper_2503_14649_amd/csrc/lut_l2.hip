// Euclidean-metric tables, fast path: L[q,p][j][c] = -|q_j - (C[l]_j + CB[j][c])|^2 for every
// (query, list) pair (the metric of Section 2 under which the tables no longer factorise).
//
// The entry is DEFINED by an fp64 accumulation rounded once to fp32, and everything derived from it
// (sub-table minima, the query's step, the 8-bit codes) must come out as from that definition.
// Evaluating all m*256 entries of all pairs twice in fp64 costs ~5 fp64-rate operations per term.
// Here both passes evaluate in fp32 with a proven error bound and go back to the fp64 definition
// only for the entries whose outcome the bound cannot decide:
//
//   fp32 evaluation  r_t = fl(q_t - c_t), L~ = fl(fma(2, dot, -rr) - cc) with dot = <r, cb> and
//   rr = |r|^2 by fma chains and cc = fl(|cb|^2): the chains err by at most dsub u times the sum of
//   the absolute terms, the two last roundings and cc by u each, the rounding of r_t by 2 u:
//   |L~ - L64| <= (dsub + 4) u M,  M = sum_t (|q_t| + |c_t| + max_c |cb_t|)^2,  u = 2^-24;
//   E = 2 (dsub + 6) (u M + 2^-126) is used: twice the bound, which also covers the rounding of E itself, plus
//   the smallest normal number per operation, which covers results that underflow.
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
// L2 per pair and pass).  What is the same for all lanes (r_j, |r_j|^2, E, the minimum) is written
// per pair by a small kernel first and read with uniform addresses, so it arrives in scalar
// registers and costs neither LDS reads nor vector instructions; wave reductions use DPP moves.
// Pass 1: wave = sub-quantiser, lane = codewords lane + 64 i (min/max are
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
constexpr float L2F_U = 5.9604644775390625e-08f;   // 2^-24

__device__ __forceinline__ uint32_t okey(float f) {            // order-preserving map float -> uint32
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float okey_inv(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// One entry of the packed codebook: DSUB coordinates, then the squared norm (and three unused floats, so that an
// entry is a whole number of 16-byte loads from one address).
template <int DSUB>
__device__ __forceinline__ void load_codeword(const float* __restrict__ cbx, uint32_t entry, float (&v)[DSUB], float& cc) {
    static_assert(DSUB % 4 == 0, "16-byte loads");
    const float4* p = reinterpret_cast<const float4*>(cbx + entry * (uint32_t)(DSUB + 4));
#pragma unroll
    for (int t = 0; t < DSUB; t += 4) {
        const float4 x = p[t / 4];
        v[t] = x.x; v[t + 1] = x.y; v[t + 2] = x.z; v[t + 3] = x.w;
    }
    cc = p[DSUB / 4].x;
}

// -|r - cb|^2 = 2 <r, cb> - |r|^2 - |cb|^2 with the two norms precomputed: dsub + 2 operations.  `r` and `rr`
// are the same for all lanes (they sit in scalar registers).
template <int DSUB>
__device__ __forceinline__ float l2_approx(const float* __restrict__ r, float rr, const float (&cb)[DSUB], float cc) {
    float dot = 0.0f;
#pragma unroll
    for (int t = 0; t < DSUB; ++t) dot = __fmaf_rn(r[t], cb[t], dot);
    return __fmaf_rn(2.0f, dot, -rr) - cc;
}

// Cross-lane moves inside the vector ALU (no LDS traffic): value of another lane of the same row of 16,
// or of the last lane of the previous row(s); lanes the pattern does not reach keep their own value.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_mov(float v) {
    const int x = __builtin_bit_cast(int, v);
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(x, x, CTRL, ROW_MASK, 0xF, false));
}
// Minimum and maximum over the 64 lanes, returned in every lane.
__device__ __forceinline__ void wave_min_max(float& mn, float& mx) {
    mn = fminf(mn, dpp_mov<0xB1, 0xF>(mn));  mx = fmaxf(mx, dpp_mov<0xB1, 0xF>(mx));     // lane ^ 1
    mn = fminf(mn, dpp_mov<0x4E, 0xF>(mn));  mx = fmaxf(mx, dpp_mov<0x4E, 0xF>(mx));     // lane ^ 2
    mn = fminf(mn, dpp_mov<0x141, 0xF>(mn)); mx = fmaxf(mx, dpp_mov<0x141, 0xF>(mx));    // mirror inside each 8
    mn = fminf(mn, dpp_mov<0x140, 0xF>(mn)); mx = fmaxf(mx, dpp_mov<0x140, 0xF>(mx));    // mirror inside each 16: rows done
    mn = fminf(mn, dpp_mov<0x142, 0xA>(mn)); mx = fmaxf(mx, dpp_mov<0x142, 0xA>(mx));    // rows 1, 3 <- last lane of rows 0, 2
    mn = fminf(mn, dpp_mov<0x143, 0xC>(mn)); mx = fmaxf(mx, dpp_mov<0x143, 0xC>(mx));    // rows 2, 3 <- lane 31: lane 63 holds all
    mn = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mn), 63));
    mx = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mx), 63));
}

// Per (pair, sub-quantiser) one record of DSUB + 4 floats: r[t] = fl(q_t - c_t), |r|^2 (fp32), the bound E,
// and two fields that pass 2 fills in while it copies its records to LDS.
template <int DSUB>
__global__ void __launch_bounds__(256) l2f_prepare_kernel(const float* __restrict__ Q, const float* __restrict__ C,
                                                          const float* __restrict__ cbmax, const int32_t* __restrict__ probes,
                                                          int64_t npairs, int nprobe, int d, int m, float* __restrict__ rec) {
    constexpr int RS = DSUB + 4;
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;       // one thread per (pair, sub-quantiser)
    if (g >= npairs * m) return;
    const int64_t pair = g / m;
    const int j = (int)(g - pair * m);
    const float* qv = Q + (pair / nprobe) * d + j * DSUB;
    const float* cv = C + (int64_t)probes[pair] * d + j * DSUB;
    float q[DSUB], c[DSUB];
#pragma unroll
    for (int t = 0; t < DSUB; t += 4) {
        const float4 a = *reinterpret_cast<const float4*>(qv + t), b = *reinterpret_cast<const float4*>(cv + t);
        q[t] = a.x; q[t + 1] = a.y; q[t + 2] = a.z; q[t + 3] = a.w;
        c[t] = b.x; c[t + 1] = b.y; c[t + 2] = b.z; c[t + 3] = b.w;
    }
    float out[RS];
    float rr = 0.0f, M = 0.0f;
#pragma unroll
    for (int t = 0; t < DSUB; ++t) {
        const float r = q[t] - c[t];
        out[t] = r;
        rr = __fmaf_rn(r, r, rr);
        const float a = fabsf(q[t]) + fabsf(c[t]) + cbmax[j * DSUB + t];
        M = __fmaf_rn(a, a, M);
    }
    out[DSUB] = rr;
    out[DSUB + 1] = 2.0f * (float)(DSUB + 6) * (L2F_U * M + 1.17549435e-38f);   // (+ one smallest normal number per operation: underflow)
    out[DSUB + 2] = 0.0f;
    out[DSUB + 3] = 0.0f;
    float4* e = reinterpret_cast<float4*>(rec + g * RS);
#pragma unroll
    for (int t = 0; t < RS; t += 4) e[t / 4] = make_float4(out[t], out[t + 1], out[t + 2], out[t + 3]);
}

// ---- pass 1
template <int DSUB, int P>
__global__ void __launch_bounds__(L2F_THREADS) l2f_range_kernel(const float* __restrict__ Q, const float* __restrict__ C,
                                                                const float* __restrict__ CB, const float* __restrict__ cbx,
                                                                const float* __restrict__ rec,
                                                                const int32_t* __restrict__ probes, int64_t npairs, int nprobe, int d,
                                                                int m, float* __restrict__ lo_out, uint32_t* __restrict__ range_bits,
                                                                int64_t* __restrict__ counters) {
    extern __shared__ __align__(16) uint8_t smem[];
    uint32_t* lo_key = reinterpret_cast<uint32_t*>(smem);            // [P][m]
    uint32_t* hi_key = lo_key + P * m;                               // [P][m]
    uint32_t* list = hi_key + P * m;                                 // [L2F_LIST]  p << 16 | j << 8 | c
    __shared__ int nlist;
    __shared__ float s_rng[P];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t pair0 = (int64_t)blockIdx.x * P;
    const int np = (int)min((int64_t)P, npairs - pair0);
    for (int idx = threadIdx.x; idx < P * m; idx += L2F_THREADS) { lo_key[idx] = 0xFFFFFFFFu; hi_key[idx] = 0u; }
    if (threadIdx.x == 0) nlist = 0;
    if (threadIdx.x < P) s_rng[threadIdx.x] = 0.0f;
    __syncthreads();
    constexpr int RS = DSUB + 4;
    const float* rec0 = rec + pair0 * m * RS;

    for (int j = wave; j < m; j += 4) {
        float cb[4][DSUB], cc[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) load_codeword<DSUB>(cbx, (uint32_t)(j * KSUB + lane + 64 * i), cb[i], cc[i]);
#pragma unroll
        for (int p = 0; p < P; ++p) {
            if (p < np) {
                const float* e = rec0 + (uint32_t)((p * m + j) * RS);       // same address in all lanes: scalar loads
                float v[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = l2_approx<DSUB>(e, e[DSUB], cb[i], cc[i]);
                float mn = fminf(fminf(v[0], v[1]), fminf(v[2], v[3]));
                float mx = fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3]));
                wave_min_max(mn, mx);
                const float marg = 2.0f * e[DSUB + 1];
                const float lo_cut = mn + marg, hi_cut = mx - marg;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (!(v[i] > lo_cut && v[i] < hi_cut)) {          // (written so that a NaN anywhere means "candidate")
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
constexpr int L2Q_THREADS = 128;        // two waves: a plane splits into two units of 128 codewords, two per lane
constexpr int L2Q_PAIRS = 4;
constexpr int L2Q_LIST = 2048;

// One (plane, 128 codewords) unit of a workgroup's pairs: lane = codewords c and c + 64; per (lane, pair, codeword)
// 32 code bytes in registers, written with two 16-byte stores.  One read of a record (LDS, the same address in all
// lanes) serves two entries per lane.  FULL: all P pairs exist (no guards in the loop).
template <int DSUB, int P, bool FULL, bool DBG>
__device__ __forceinline__ void l2f_quant_unit(const float* __restrict__ cbx, const float* __restrict__ rec0,
                                               int np, int m, int S, int plane, int c, const float (&inv)[P],
                                               uint8_t* __restrict__ tab0, uint8_t* __restrict__ dbg0, uint32_t* __restrict__ list,
                                               int* __restrict__ nlist) {
    constexpr int RS = DSUB + 4;
    // pk[p][i][0..7]: the 32 code bytes of (codeword c + 64 i, this plane) for pair p.  The words are produced in
    // order and shifted in at the top, so that no register is indexed by a loop variable.
    uint32_t pk[P][2][8];
#pragma unroll
    for (int p = 0; p < P; ++p)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int w = 0; w < 8; ++w) pk[p][i][w] = 0u;
    // Steps (sub-quantiser j, pair p) run j-major; the codewords of sub-quantiser j + 2 are requested while the P
    // steps of j run (past the end of the plane: its last sub-quantiser again): a load from L2 takes longer than
    // the steps of one sub-quantiser.
    const int jfirst = plane * 32, jlast = plane * 32 + S - 1;
    float cbc[2][DSUB], ccc[2], cbm[2][DSUB], ccm[2];          // codewords of sub-quantisers j and j + 1 (j + 2 is on its way)
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        load_codeword<DSUB>(cbx, (uint32_t)(jfirst * KSUB + c + 64 * i), cbc[i], ccc[i]);
        load_codeword<DSUB>(cbx, (uint32_t)(min(jfirst + 1, jlast) * KSUB + c + 64 * i), cbm[i], ccm[i]);
    }
#pragma unroll 1
    for (int w = 0; w < S / 4; ++w) {
        uint32_t word[P][2];
#pragma unroll
        for (int p = 0; p < P; ++p) { word[p][0] = 0u; word[p][1] = 0u; }
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
            const int j = jfirst + w * 4 + s4, jn = min(j + 2, jlast);
            float cbn[2][DSUB], ccn[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) load_codeword<DSUB>(cbx, (uint32_t)(jn * KSUB + c + 64 * i), cbn[i], ccn[i]);
#pragma unroll
            for (int p = 0; p < P; ++p) {
                if (FULL || p < np) {
                    const float* e = rec0 + (p * m + j) * RS;
                    float r[DSUB];
#pragma unroll
                    for (int t = 0; t < DSUB; t += 4) {
                        const float4 x = *reinterpret_cast<const float4*>(e + t);
                        r[t] = x.x; r[t + 1] = x.y; r[t + 2] = x.z; r[t + 3] = x.w;
                    }
                    const float4 a = *reinterpret_cast<const float4*>(e + DSUB);     // |r|^2, E, minimum, eta
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        const float Lt = l2_approx<DSUB>(r, a.x, cbc[i], ccc[i]);
                        const float b = (Lt - a.z) * inv[p];
                        const float rr = fminf(fmaxf(rintf(b), 0.0f), 255.0f);
                        word[p][i] |= (uint32_t)rr << (8 * s4);
                        // undecided (about one entry in a thousand): on the list
                        if (!(fabsf(__builtin_amdgcn_fractf(b) - 0.5f) > a.w)) {      // (a NaN or infinite b~ or eta means "undecided")
                            const int pos = atomicAdd(nlist, 1);
                            if (pos < L2Q_LIST) list[pos] = (uint32_t)(p << 16 | j << 8 | (c + 64 * i));
                        }
                        if (DBG) dbg0[((int64_t)p * m + j) * KSUB + c + 64 * i] = (uint8_t)rr;
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < 2; ++i) {
#pragma unroll
                for (int t = 0; t < DSUB; ++t) { cbc[i][t] = cbm[i][t]; cbm[i][t] = cbn[i][t]; }
                ccc[i] = ccm[i]; ccm[i] = ccn[i];
            }
        }
#pragma unroll
        for (int p = 0; p < P; ++p)
#pragma unroll
            for (int i = 0; i < 2; ++i) {
#pragma unroll
                for (int x = 0; x < 7; ++x) pk[p][i][x] = pk[p][i][x + 1];
                pk[p][i][7] = word[p][i];
            }
    }
    if (S == 16) {                  // fewer than 32 sub-quantisers: slots 16..31 repeat slots 0..15
#pragma unroll
        for (int p = 0; p < P; ++p)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int x = 0; x < 4; ++x) pk[p][i][x] = pk[p][i][x + 4];
    }
#pragma unroll
    for (int p = 0; p < P; ++p) {
        if (FULL || p < np) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                uint4* dst = reinterpret_cast<uint4*>(tab0 + (int64_t)p * LUT_BYTES + (int64_t)plane * LUT_PLANE + (c + 64 * i) * 32);
                dst[0] = make_uint4(pk[p][i][0], pk[p][i][1], pk[p][i][2], pk[p][i][3]);
                dst[1] = make_uint4(pk[p][i][4], pk[p][i][5], pk[p][i][6], pk[p][i][7]);
            }
        }
    }
}

template <int DSUB, bool DBG>
__global__ void __launch_bounds__(L2Q_THREADS) l2f_quant_kernel(const float* __restrict__ Q, const float* __restrict__ C,
                                                                const float* __restrict__ CB, const float* __restrict__ cbx,
                                                                const float* __restrict__ rec,
                                                                const int32_t* __restrict__ probes, int64_t npairs, int nprobe, int d,
                                                                int m, const float* __restrict__ lo_in, const uint32_t* __restrict__ range_bits,
                                                                uint8_t* __restrict__ tables, int32_t* __restrict__ bias,
                                                                float* __restrict__ delta, uint8_t* __restrict__ out_LUT8,
                                                                int64_t* __restrict__ counters) {
    constexpr int P = L2Q_PAIRS;
    extern __shared__ __align__(16) uint8_t smem[];
    uint32_t* list = reinterpret_cast<uint32_t*>(smem);                        // [L2Q_LIST]
    float* rec_s = reinterpret_cast<float*>(smem + L2Q_LIST * 4);              // [P][m][DSUB + 4] this workgroup's records
    __shared__ int nlist;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t pair0 = (int64_t)blockIdx.x * P;
    const int np = (int)min((int64_t)P, npairs - pair0);
    const int S = rago_steps(m), planes = rago_planes(m);
    if (threadIdx.x == 0) nlist = 0;
    float inv[P];                          // per pair: the reciprocal of the query's step
#pragma unroll
    for (int p = 0; p < P; ++p) inv[p] = 1.0f / lut_step(__uint_as_float(range_bits[(pair0 + min(p, np - 1)) / nprobe]));
    {
        // Records into LDS.  Their last two fields are filled in here: the sub-table's exact minimum (pass 1) and, now
        // that the query's step dq is known, the half-width eta of the zone around a half-integer inside which b~ is
        // not trusted: (E + u M) / dq + 2^-13 with M = E / (2 (dsub + 6) u).
        const float4* src = reinterpret_cast<const float4*>(rec + pair0 * m * (DSUB + 4));
        float4* dst = reinterpret_cast<float4*>(rec_s);
        constexpr int Q4 = (DSUB + 4) / 4;                 // 16-byte pieces per record
        for (int i = threadIdx.x; i < np * m * Q4; i += L2Q_THREADS) {
            float4 v = src[i];
            if (i % Q4 == Q4 - 1) {
                const int pj = i / Q4, p = pj / m;
                float ip = inv[0];
#pragma unroll
                for (int x = 1; x < P; ++x) ip = p == x ? inv[x] : ip;
                v.z = lo_in[pair0 * m + pj];
                v.w = __fmaf_rn(v.y, (1.0f + 1.0f / (2.0f * (float)(DSUB + 6))) * ip * 1.001f, 1.220703125e-4f);
            }
            dst[i] = v;
        }
    }
    __syncthreads();
    const float* rec0 = rec_s;
    uint8_t* tab0 = tables + pair0 * LUT_BYTES;
    uint8_t* dbg0 = DBG ? out_LUT8 + pair0 * m * KSUB : nullptr;
    for (int u = wave; u < planes * 2; u += 2) {
        const int plane = u >> 1, c = (u & 1) * 128 + lane;
        if (np == P) l2f_quant_unit<DSUB, P, true, DBG>(cbx, rec0, np, m, S, plane, c, inv, tab0, dbg0, list, &nlist);
        else l2f_quant_unit<DSUB, P, false, DBG>(cbx, rec0, np, m, S, plane, c, inv, tab0, dbg0, list, &nlist);
    }
    // The packed stores are ordered before the single-byte corrections by the barrier's workgroup-scope release:
    // both come from this workgroup and go through the same L2.  (A device-scope fence here makes every
    // workgroup write back its XCD's L2 and costs more than the whole computation.)
    __syncthreads();
    const int n = nlist;
    const bool all = n > L2Q_LIST;
    const int total = all ? np * m * KSUB : n;
    for (int e = threadIdx.x; e < total; e += L2Q_THREADS) {
        const uint32_t w = all ? (uint32_t)((e / (m * KSUB)) << 16 | ((e / KSUB) % m) << 8 | (e % KSUB)) : list[e];
        const int p = w >> 16, j = (w >> 8) & 255, c = w & 255;
        const int64_t q = (pair0 + p) / nprobe;
        const int l = probes[pair0 + p];
        const float L = l2_entry<DSUB>(Q + q * d + j * DSUB, C + (int64_t)l * d + j * DSUB, CB + ((int64_t)j * KSUB + c) * DSUB, DSUB);
        const float step = lut_step(__uint_as_float(range_bits[q]));
        float rr = rintf(__fdiv_rn(L - rec_s[(p * m + j) * (DSUB + 4) + DSUB + 2], step));
        rr = rr < 0.0f ? 0.0f : (rr > 255.0f ? 255.0f : rr);
        const uint8_t v = (uint8_t)rr;
        uint8_t* tab = tables + (pair0 + p) * LUT_BYTES + (int64_t)(j >> 5) * LUT_PLANE + c * 32;
        for (int rep = j & (S - 1); rep < 32; rep += S) tab[rep] = v;
        if (DBG) out_LUT8[((pair0 + p) * m + j) * KSUB + c] = v;
    }
    if (threadIdx.x < np) {
        const int p = threadIdx.x;
        const float step = lut_step(__uint_as_float(range_bits[(pair0 + p) / nprobe]));
        double losum = 0.0;                      // in index order (the order that defines the bias), minima from the records in LDS
        for (int j = 0; j < m; ++j) losum = losum + (double)rec_s[(p * m + j) * (DSUB + 4) + DSUB + 2];
        bias[pair0 + p] = (int32_t)rint(losum / (double)step);
        if ((pair0 + p) % nprobe == 0) delta[(pair0 + p) / nprobe] = step;
    }
    if (threadIdx.x == 0) {
        atomicAdd(reinterpret_cast<unsigned long long*>(counters + 4), (unsigned long long)total);
        if (all) atomicAdd(reinterpret_cast<unsigned long long*>(counters + 5), 1ull);
    }
}

// Per dimension the largest |codeword coordinate|; the packed codebook [m][256][dsub + 4]: coordinates, squared
// norm (fp64 sum, one rounding), three zeros.
__global__ void __launch_bounds__(256) cb_stats_kernel(const float* __restrict__ CB, int d, int m, int dsub, float* __restrict__ absmax,
                                                       float* __restrict__ cbx) {
    const int x = blockIdx.x * 256 + threadIdx.x;
    if (x < d) {
        const int j = x / dsub, t = x - j * dsub;
        float mx = 0.0f;
        for (int c = 0; c < KSUB; ++c) mx = fmaxf(mx, fabsf(CB[((int64_t)j * KSUB + c) * dsub + t]));
        absmax[x] = mx;
    }
    if (x < m * KSUB) {
        double acc = 0.0;
        float* o = cbx + (int64_t)x * (dsub + 4);
        for (int t = 0; t < dsub; ++t) { const float f = CB[(int64_t)x * dsub + t]; o[t] = f; acc = acc + (double)f * (double)f; }
        o[dsub] = (float)acc;
        o[dsub + 1] = 0.0f; o[dsub + 2] = 0.0f; o[dsub + 3] = 0.0f;
    }
}

template <int DSUB, int P>
int launch_l2f(rago_index* idx, const float* q, const int32_t* probes, int64_t npairs, int nprobe, float* lo, uint32_t* range_bits,
               uint8_t* out_LUT8, hipStream_t st) {
    Workspace& ws = idx->ws;
    const int d = idx->d, m = idx->m;
    int rc;
    if ((rc = ws.l2_r.reserve((size_t)npairs * m * (DSUB + 4) * 4))) return rc;
    float* rec = ws.l2_r.as<float>();
    const size_t lds1 = (size_t)P * m * 8 + (size_t)L2F_LIST * 4;
    const size_t lds2 = (size_t)L2Q_LIST * 4 + (size_t)L2Q_PAIRS * m * (DSUB + 4) * 4;     // <= 42 KB
    const unsigned grid = (unsigned)((npairs + P - 1) / P), grid2 = (unsigned)((npairs + L2Q_PAIRS - 1) / L2Q_PAIRS);
    l2f_prepare_kernel<DSUB><<<(unsigned)((npairs * m + 255) / 256), 256, 0, st>>>(q, idx->centroids, idx->cb_absmax, probes, npairs, nprobe, d, m, rec);
    l2f_range_kernel<DSUB, P><<<grid, L2F_THREADS, lds1, st>>>(q, idx->centroids, idx->codebooks, idx->cbx, rec, probes, npairs, nprobe,
                                                               d, m, lo, range_bits, ws.counters.as<int64_t>());
    if (out_LUT8)
        l2f_quant_kernel<DSUB, true><<<grid2, L2Q_THREADS, lds2, st>>>(q, idx->centroids, idx->codebooks, idx->cbx, rec, probes, npairs, nprobe, d,
                                                                       m, lo, range_bits, ws.tmp_lut8sw.as<uint8_t>(), ws.bias.as<int32_t>(),
                                                                       ws.delta.as<float>(), out_LUT8, ws.counters.as<int64_t>());
    else
        l2f_quant_kernel<DSUB, false><<<grid2, L2Q_THREADS, lds2, st>>>(q, idx->centroids, idx->codebooks, idx->cbx, rec, probes, npairs, nprobe, d,
                                                                        m, lo, range_bits, ws.tmp_lut8sw.as<uint8_t>(), ws.bias.as<int32_t>(),
                                                                        ws.delta.as<float>(), nullptr, ws.counters.as<int64_t>());
    RAGO_HIP(hipGetLastError());
    return RAGO_OK;
}

}  // namespace

int launch_cb_stats(rago_index* idx, hipStream_t st) {
    const int n = std::max(idx->d, idx->m * KSUB);
    cb_stats_kernel<<<(n + 255) / 256, 256, 0, st>>>(idx->codebooks, idx->d, idx->m, idx->dsub, idx->cb_absmax, idx->cbx);
    RAGO_HIP(hipGetLastError());
    return RAGO_OK;
}

bool lut_l2_fast_supported(const rago_index* idx) {
    const int dsub = idx->dsub;
    return dsub == 4 || dsub == 8 || dsub == 16;
}

// Both passes for all pairs.  `lo` [npairs][m] fp32 and `range_bits` [nq] (zeroed) are workspace; the
// tables, bias and step land in the workspace members the scan reads.
int launch_lut_l2_fast(rago_index* idx, const float* q, const int32_t* probes, int64_t npairs, int nprobe, float* lo, uint32_t* range_bits,
                       uint8_t* out_LUT8, hipStream_t st) {
    switch (idx->dsub) {
        case 4: return launch_l2f<4, 8>(idx, q, probes, npairs, nprobe, lo, range_bits, out_LUT8, st);
        case 8: return launch_l2f<8, 8>(idx, q, probes, npairs, nprobe, lo, range_bits, out_LUT8, st);
        case 16: return launch_l2f<16, 8>(idx, q, probes, npairs, nprobe, lo, range_bits, out_LUT8, st);
    }
    return fail(RAGO_UNSUPPORTED, "sub-vector length without a fast Euclidean table path");
}

}  // namespace rago

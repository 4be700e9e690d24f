// Look-up tables of the residual PQ under the inner-product metric, one per (query, probed list),
// and their 8-bit quantisation (the lower-precision, memory-bound PQ variant of Section 2).
//
//   L[q,p][j][c] = < q_j , C[l_p]_j + CB[j][c] >                     (fp64 accumulate -> fp32)
//   lo/hi        = min/max over c;  delta_q = max_{p,j}(hi - lo) / 255  (fp32; 1 if zero)
//   LUT8         = clamp(rne((L - lo) / delta_q), 0, 255)            (fp32, IEEE divide)
//   B[q,p]       = rne( (sum_j lo_j in fp64) / delta_q )
//
// The inner product splits into a per-query part T[q][j][c] = <q_j, CB[j][c]> and a per-pair
// scalar t[q,p][j] = <q_j, C[l]_j>; both are accumulated in fp64 (left to right, no fused
// multiply-add) and added in fp64 before the single rounding to fp32, so L equals the directly
// accumulated value except where two fp64 roundings straddle an fp32 rounding boundary
// (probability ~1e-9 per entry).  min/max commute with the monotone rounding, so lo/hi come from
// the per-query extrema of T.
//
// In exact arithmetic (L - lo) / delta does not depend on the probed list: it is
// u = (T - Tmin) / delta.  The fp32 evaluation prescribed above differs from u by at most
//   eta_0 = 2^-24 * ((2 M + range) / delta + 256),   M = max |lo|,|hi| over the query's pairs,
// (two roundings of magnitude <= M, one of the difference <= range, one of the quotient <= 256).
// So one BASE table per query, rne(u), is the exact per-pair table wherever u is farther than
// eta = 2 eta_0 from every half-integer; the few entries closer than that ("ambiguous", ~1e-3 of
// a table) are evaluated per pair with the prescribed fp32 expression and stored as PATCHES.
// The scan loads the base table of the query and overwrites the patched bytes.  If a query has
// more ambiguous entries than AMB_MAX (nearly constant tables), its pairs are flagged and every
// consumer evaluates the full per-pair table with the same expression instead.
//
// Table layout in HBM ("plane-major", what the scan interleaves into LDS): [plane][c][slot], one
// byte each = entry c of sub-quantiser plane*32 + slot; for m < 32 the m sub-tables are
// replicated 32/m times over the 32 slots.  A table occupies planes * 8192 bytes of its
// LUT_BYTES stride.
#include <algorithm>

#include "lut_common.h"
#include "scan_setup.h"
#include "scan_plan.h"
#include "rago_internal.h"

namespace rago {

// <a, b> over one sub-vector, accumulated left to right in fp64 without fused multiply-add.
// DSUB = 0: any length (`dsub`), else the compile-time length (vector loads, unrolled).
template <int DSUB>
__device__ __forceinline__ double subdot(const float* __restrict__ a, const float* __restrict__ b, int dsub) {
    double acc = 0.0;
    if constexpr (DSUB == 8) {
        const float4 a0 = *reinterpret_cast<const float4*>(a), a1 = *reinterpret_cast<const float4*>(a + 4);
        const float4 b0 = *reinterpret_cast<const float4*>(b), b1 = *reinterpret_cast<const float4*>(b + 4);
        acc = acc + (double)a0.x * (double)b0.x; acc = acc + (double)a0.y * (double)b0.y;
        acc = acc + (double)a0.z * (double)b0.z; acc = acc + (double)a0.w * (double)b0.w;
        acc = acc + (double)a1.x * (double)b1.x; acc = acc + (double)a1.y * (double)b1.y;
        acc = acc + (double)a1.z * (double)b1.z; acc = acc + (double)a1.w * (double)b1.w;
    } else {
        for (int t = 0; t < dsub; ++t) acc = acc + (double)a[t] * (double)b[t];
    }
    return acc;
}

// T64[q][j][c] = <q_j, CB[j][c]> with Tmin/Tmax[q][j] (one wave per (query, sub-quantiser): a lane handles codewords
// lane, lane + 64, lane + 128, lane + 192), and the per-pair scalars t64[pair][j] = <q_j, C[l]_j> (one wave per pair,
// lanes = sub-quantisers, `ppw` consecutive pairs per wave), in ONE launch, since neither depends on the other:
// after `first` workgroups, `tg` do T, the others the pairs.  The first `first` plan the wave-per-item scan, a query
// each (scan_plan.h), when that rides along: it needs only the probes (first: they are chains of dependent steps, short
// on work, and at the end of the grid they would run on after everything else is done).
template <int DSUB>
__global__ void __launch_bounds__(256) lut_Tt_kernel(const float* __restrict__ Q, const float* __restrict__ C, const float* __restrict__ CB,
                                                     const int32_t* __restrict__ probes, int64_t nq, int64_t npairs, int ppw, int d, int m,
                                                     unsigned first, unsigned tg, int qb, double* __restrict__ T64, double* __restrict__ Tmin,
                                                     double* __restrict__ Tmax, double* __restrict__ t64, int64_t* __restrict__ counters,
                                                     const WavePlanArgs plan) {
    const int lane = threadIdx.x & 63;
    const int dsub = DSUB ? DSUB : d / m;
    if (blockIdx.x < first) {
        wave_plan_body(plan, (int)blockIdx.x);
        return;
    }
    const unsigned bx = blockIdx.x - first;
    if (bx < tg) {
        // a wave takes sub-quantiser j for `qb` consecutive queries: its codewords come from L2 once, not once per query
        const int64_t w = (int64_t)bx * 4 + (threadIdx.x >> 6);
        const int64_t nqb = (nq + qb - 1) / qb;
        if (w >= nqb * m) return;
        const int64_t q0 = (w / m) * qb, q1 = q0 + qb < nq ? q0 + qb : nq;
        const int j = (int)(w % m);
        if (w == 0 && lane == 0) { counters[4] = 0; counters[5] = 0; }
        __attribute__((aligned(16))) float cw[4][DSUB ? DSUB : 4];
        if constexpr (DSUB != 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int t = 0; t < DSUB; t += 4) {
                    const float4 x = *reinterpret_cast<const float4*>(CB + ((int64_t)j * KSUB + lane + 64 * i) * DSUB + t);
                    cw[i][t] = x.x; cw[i][t + 1] = x.y; cw[i][t + 2] = x.z; cw[i][t + 3] = x.w;
                }
        }
        for (int64_t q = q0; q < q1; ++q) {
            const float* qv = Q + q * d + j * dsub;
            double mn = 0.0, mx = 0.0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int c = lane + 64 * i;
                double acc;
                if constexpr (DSUB != 0) acc = subdot<DSUB>(qv, cw[i], dsub);
                else acc = subdot<DSUB>(qv, CB + ((int64_t)j * KSUB + c) * dsub, dsub);
                T64[(q * m + j) * KSUB + c] = acc;
                mn = i ? fmin(mn, acc) : acc;
                mx = i ? fmax(mx, acc) : acc;
            }
            for (int o = 32; o; o >>= 1) {
                mn = fmin(mn, __shfl_xor(mn, o));
                mx = fmax(mx, __shfl_xor(mx, o));
            }
            if (lane == 0) { Tmin[q * m + j] = mn; Tmax[q * m + j] = mx; }
        }
        return;
    }
    const int64_t w = (int64_t)(bx - tg) * 4 + (threadIdx.x >> 6);
    for (int pp = 0; pp < ppw; ++pp) {
        const int64_t pair = w * ppw + pp;
        if (pair >= npairs) return;
        const int64_t q = pair / (npairs / nq);
        const int l = probes[pair];
        for (int j = lane; j < m; j += 64) t64[pair * m + j] = subdot<DSUB>(Q + q * d + j * dsub, C + (int64_t)l * d + j * dsub, dsub);
    }
}

// Everything of one query that follows from T and the pairs' scalars, in workgroups of 16 waves: the query's range
// and step (maxima over its pairs of the fp32 expressions the definition prescribes), its base table and ambiguous
// entries, then bias and patches of its pairs (a wave per pair at a time).  gridDim.y workgroups share a query's
// pairs (small batches: one workgroup per query would leave the chip idle); each of them derives the range and the
// list of ambiguous entries for itself, in the same order (positions from a prefix sum over the threads, not from
// an atomic counter), and the first one writes the per-query outputs.
constexpr int LQ_THREADS = 1024;
__global__ void __launch_bounds__(LQ_THREADS, 8) lut_query_kernel(const double* __restrict__ T64, const double* __restrict__ Tmin,
                                                               const double* __restrict__ Tmax, const double* __restrict__ t64, int nprobe,
                                                               int m, uint32_t* __restrict__ range_bits, uint32_t* __restrict__ mag_bits,
                                                               uint8_t* __restrict__ lut_base, uint16_t* __restrict__ amb_addr,
                                                               int32_t* __restrict__ namb, float* __restrict__ delta,
                                                               int32_t* __restrict__ bias, uint8_t* __restrict__ patch_val,
                                                               int64_t* __restrict__ counters, int lq_y, const SmallSetupArgs setup,
                                                               const WaveFixArgs fix) {
    // One extra row of workgroups, the first to be dispatched, when the scan's bookkeeping rides along: its first
    // workgroup does that work, which needs nothing from the tables, the others leave.
    const int ty = (int)blockIdx.y - (setup.enable ? 1 : 0);       // this workgroup's row among the query's lq_y
    if (ty < 0) {
        extern __shared__ __align__(16) int32_t ssu[];
        if (blockIdx.x == 0) small_setup_body(setup, ssu);
        return;
    }
    __shared__ uint32_t s_rng, s_mag;
    __shared__ int s_n;
    __shared__ int s_wcnt[LQ_THREADS / 64];
    __shared__ uint16_t s_amb[AMB_MAX];
    __shared__ double s_t16[LQ_THREADS / 64][128];
    __shared__ float s_lo16[LQ_THREADS / 64][128];
    __shared__ double s_Tmin[128], s_Tmax[128];
    const int64_t q = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) { s_rng = 0u; s_mag = 0u; s_n = 0; }
    for (int j = tid; j < m; j += LQ_THREADS) { s_Tmin[j] = Tmin[q * m + j]; s_Tmax[j] = Tmax[q * m + j]; }
    __syncthreads();
    // ---- range and magnitude over the query's (pair, sub-quantiser) entries
    {
        float rng = 0.f, mag = 0.f;
        const double* tq = t64 + q * nprobe * m;
        // (eight loads at a time while eight are left: one load per trip round the loop is a trip to memory each)
        const int total = nprobe * m;
        auto look = [&](int i, double t) {
            const int j = i % m;
            const float lo = (float)(s_Tmin[j] + t), hi = (float)(s_Tmax[j] + t);
            rng = fmaxf(rng, hi - lo);
            mag = fmaxf(mag, fmaxf(fabsf(lo), fabsf(hi)));
        };
        int i0 = tid;
        for (; i0 + 7 * LQ_THREADS < total; i0 += 8 * LQ_THREADS) {
            double t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = tq[i0 + u * LQ_THREADS];
#pragma unroll
            for (int u = 0; u < 8; ++u) look(i0 + u * LQ_THREADS, t[u]);
        }
        for (; i0 < total; i0 += LQ_THREADS) look(i0, tq[i0]);
        for (int o = 32; o; o >>= 1) { rng = fmaxf(rng, __shfl_xor(rng, o)); mag = fmaxf(mag, __shfl_xor(mag, o)); }
        if (lane == 0) {     // (non-negative floats order like their bit patterns)
            if (rng > 0.f) atomicMax(&s_rng, __float_as_uint(rng));
            if (mag > 0.f) atomicMax(&s_mag, __float_as_uint(mag));
        }
    }
    __syncthreads();
    const float range = __uint_as_float(s_rng);
    const float dq = lut_step(range);
    const bool writer = ty == 0;
    if (tid == 0 && writer) { range_bits[q] = s_rng; mag_bits[q] = s_mag; delta[q] = dq; }
    // ---- base table and ambiguous entries: thread = (plane, codeword)
    {
        const double eta = lut_eta(range, __uint_as_float(s_mag), dq);
        const double inv_dq = 1.0 / (double)dq;
        const int S = rago_steps(m), planes = rago_planes(m);
        const int plane = tid >> 8, c = tid & 255;
        uint32_t row[8];                      // 32 slots of this plane, one byte each
#pragma unroll
        for (int i = 0; i < 8; ++i) row[i] = 0;
        uint32_t flagged = 0;                 // slots of (plane, c) whose rounding depends on the pair
        if (plane < planes) {
            const double* Tq = T64 + q * m * KSUB + c;
#pragma unroll
            for (int slot = 0; slot < 32; ++slot) {
                if (slot >= S) continue;
                const int j = plane * 32 + slot;
                const double u = (Tq[(int64_t)j * KSUB] - s_Tmin[j]) * inv_dq;   // (2^-52 relative off the quotient: far inside eta)
                double r = rint(u);
                r = r < 0.0 ? 0.0 : (r > 255.0 ? 255.0 : r);
                row[slot >> 2] |= (uint32_t)r << (8 * (slot & 3));
                if (fabs((u - floor(u)) - 0.5) <= eta) flagged |= 1u << slot;
            }
            if (S < 32) {
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (i * 4 >= S) row[i] = row[i & (S / 4 - 1)];
            }
            if (writer) {
                uint4* dst = reinterpret_cast<uint4*>(lut_base + q * LUT_BYTES + (int64_t)plane * LUT_PLANE + c * 32);
                dst[0] = make_uint4(row[0], row[1], row[2], row[3]);
                dst[1] = make_uint4(row[4], row[5], row[6], row[7]);
            }
        }
        // positions of the flagged entries in the query's list: exclusive prefix sum over the threads (every replica
        // of a sub-table counts, m < 32), so that every workgroup of the query builds the same list
        const int mine = __popc(flagged) * (32 / S);
        int inc = mine;
        for (int o = 1; o < 64; o <<= 1) {
            const int v = __shfl_up(inc, o);
            if (lane >= o) inc += v;
        }
        if (lane == 63) s_wcnt[wave] = inc;
        __syncthreads();
        int at = inc - mine;
        for (int w = 0; w < wave; ++w) at += s_wcnt[w];
        if (tid == LQ_THREADS - 1) s_n = at + mine;
        for (uint32_t f = flagged; f; f &= f - 1) {
            const int slot = __ffs(f) - 1;
            for (int rep = slot; rep < 32; rep += S) {
                if (at < AMB_MAX) {
                    const uint16_t a = (uint16_t)(plane * LUT_PLANE + c * 32 + rep);
                    s_amb[at] = a;
                    if (writer) amb_addr[q * AMB_MAX + at] = a;
                }
                ++at;
            }
        }
    }
    __syncthreads();
    const int n = s_n;
    if (tid == 0 && writer) {
        namb[q] = n > AMB_MAX ? AMB_MAX + 1 : n;   // AMB_MAX + 1 = "evaluate per pair"
        if (fix.enable && n > AMB_MAX) wave_fix_per_pair(fix, (int)q);      // (the plan took the query's tables to be shared)
        if (n > AMB_MAX) atomicAdd(reinterpret_cast<unsigned long long*>(counters + 5), 1ull);
        else atomicAdd(reinterpret_cast<unsigned long long*>(counters + 4), (unsigned long long)n);
    }
    // ---- bias and patches: a wave per pair
    {
        double* s_t = s_t16[wave];
        float* s_lo = s_lo16[wave];
        const int S = rago_steps(m);
        for (int p = ty * (LQ_THREADS / 64) + wave; p < nprobe; p += lq_y * (LQ_THREADS / 64)) {
            const int64_t pair = q * nprobe + p;
            float lo_reg[2] = {0.f, 0.f};                  // lane holds sub-quantisers lane and lane + 64 (m <= 128)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int j = lane + 64 * h;
                if (j < m) {
                    const double t = t64[pair * m + j];
                    s_t[j] = t;
                    lo_reg[h] = (float)(s_Tmin[j] + t);
                    s_lo[j] = lo_reg[h];
                }
            }
            // (the wave's own LDS writes are visible to its later reads: LDS operations of a wave complete in order;
            // the wave barrier only keeps the compiler from moving the reads up)
            __builtin_amdgcn_wave_barrier();
            {
                // The definition sums the minima over the sub-quantisers in order, in fp64.  When every partial sum
                // of any order is exactly representable - all terms multiples of 2^(emin - 23), all sums below
                // 2^(emax + 8), and emax - emin <= 22 leaves them 53 bits - the order does not matter and a
                // tree over the lanes gives that sum; otherwise one lane adds them in order.
                const uint32_t e0 = (__float_as_uint(lo_reg[0]) >> 23) & 255u, e1 = (__float_as_uint(lo_reg[1]) >> 23) & 255u;
                int emax = (int)max(e0, e1);
                int emin = (int)min(lo_reg[0] != 0.f ? e0 : 255u, lo_reg[1] != 0.f ? e1 : 255u);
                double losum = (double)lo_reg[0] + (double)lo_reg[1];
                for (int o = 32; o; o >>= 1) {
                    losum = losum + __shfl_xor(losum, o);
                    emax = max(emax, __shfl_xor(emax, o));
                    emin = min(emin, __shfl_xor(emin, o));
                }
                // (exponent field 0: subnormal terms, multiples of 2^-149 like those of field 1; 255: infinities and
                // not-a-numbers go the ordered way)
                if (emax == 255 || emax - max(emin, 1) > 22) {
                    losum = 0.0;
                    if (lane == 0)
                        for (int j = 0; j < m; ++j) losum = losum + (double)s_lo[j];
                }
                if (lane == 0) bias[pair] = (int32_t)rint(losum / (double)dq);
            }
            if (n <= AMB_MAX) {
                for (int i = lane; i < n; i += 64) {
                    const int addr = s_amb[i];
                    const int plane = addr / LUT_PLANE, c = (addr >> 5) & 255, slot = addr & 31;
                    const int j = plane * 32 + (slot & (S - 1));
                    patch_val[pair * AMB_MAX + i] = lut_entry(T64[(q * m + j) * KSUB + c], s_t[j], s_lo[j], dq);
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
}

// Plain per-pair tables [pair][m][256] (u8 and/or fp32) for inspection: base + patches, or the
// full evaluation for flagged queries.
__global__ void __launch_bounds__(256) lut_expand_kernel(const double* __restrict__ T64, const double* __restrict__ Tmin,
                                                         const double* __restrict__ t64, const uint32_t* __restrict__ range_bits,
                                                         const uint8_t* __restrict__ lut_base, const uint16_t* __restrict__ amb_addr,
                                                         const int32_t* __restrict__ namb, const uint8_t* __restrict__ patch_val,
                                                         int nprobe, int m, float* __restrict__ out_L, uint8_t* __restrict__ out_LUT8) {
    const int64_t pair = blockIdx.x;
    const int64_t q = pair / nprobe;
    const int c = threadIdx.x;
    const float dq = lut_step(__uint_as_float(range_bits[q]));
    const int n = namb[q];
    const int S = rago_steps(m);
    for (int j = 0; j < m; ++j) {
        const double t = t64[pair * m + j];
        const double Tv = T64[(q * m + j) * KSUB + c];
        if (out_L) out_L[(pair * m + j) * KSUB + c] = (float)(Tv + t);
        if (out_LUT8) {
            uint8_t v;
            if (n > AMB_MAX) v = lut_entry(Tv, t, (float)(Tmin[q * m + j] + t), dq);
            else v = lut_base[q * LUT_BYTES + (int64_t)(j >> 5) * LUT_PLANE + c * 32 + (j & (S - 1))];
            out_LUT8[(pair * m + j) * KSUB + c] = v;
        }
    }
    if (!out_LUT8 || n > AMB_MAX) return;
    __syncthreads();
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
        const int addr = amb_addr[q * AMB_MAX + i];
        const int plane = addr / LUT_PLANE, cc = (addr >> 5) & 255, slot = addr & 31;
        const int j = plane * 32 + (slot & (S - 1));
        out_LUT8[(pair * m + j) * KSUB + cc] = patch_val[pair * AMB_MAX + i];
    }
}

// plain [pair][m][256] u8 -> plane-major [pair][plane][256][32]
__global__ void __launch_bounds__(256) lut_swizzle_kernel(const uint8_t* __restrict__ plain, int m, uint8_t* __restrict__ lut8sw) {
    const int64_t pair = blockIdx.x;
    const int c = threadIdx.x;
    const int S = rago_steps(m), planes = rago_planes(m);
    for (int plane = 0; plane < planes; ++plane) {
        uint32_t row[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) row[i] = 0;
#pragma unroll
        for (int slot = 0; slot < 32; ++slot) {
            const uint32_t v = plain[(pair * m + plane * 32 + (slot & (S - 1))) * KSUB + c];
            row[slot >> 2] |= v << (8 * (slot & 3));
        }
        uint4* dst = reinterpret_cast<uint4*>(lut8sw + pair * LUT_BYTES + (int64_t)plane * LUT_PLANE + c * 32);
        dst[0] = make_uint4(row[0], row[1], row[2], row[3]);
        dst[1] = make_uint4(row[4], row[5], row[6], row[7]);
    }
}

// ------------------------------------------------------------------ Euclidean metric
// L[q,p][j][c] = -|q_j - (C[l]_j + CB[j][c])|^2 does not split into a per-query and a per-list part,
// so every (query, list) pair gets a full table, in two passes because the step is per query:
// pass 1 finds each sub-table's minimum and the query's largest range, pass 2 evaluates the entries
// again, quantises them and writes the pair's plane-major table (staged in LDS so that the store to
// HBM is contiguous), bias and, for inspection, plain copies.  One workgroup per pair, one wave per
// sub-quantiser at a time, lane = codewords lane, lane + 64, lane + 128, lane + 192.
// These two kernels evaluate EVERY entry by the fp64 definition.  They serve sub-vector lengths that the
// fp32 path with exact re-evaluation (lut_l2.hip) does not cover, and the plain fp32 tables of the inspection call.
template <int DSUB>
__global__ void __launch_bounds__(256) lut_l2_range_kernel(const float* __restrict__ Q, const float* __restrict__ C,
                                                           const float* __restrict__ CB, const int32_t* __restrict__ probes,
                                                           int nprobe, int d, int m, float* __restrict__ lo_out,
                                                           uint32_t* __restrict__ range_bits) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t pair = blockIdx.x;
    const int64_t q = pair / nprobe;
    const int l = probes[pair];
    const int dsub = DSUB ? DSUB : d / m;
    float rng = 0.f;
    for (int j = wave; j < m; j += 4) {
        const float* qv = Q + q * d + j * dsub;
        const float* cv = C + (int64_t)l * d + j * dsub;
        float mn = 0.f, mx = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = lane + 64 * i;
            const float v = l2_entry<DSUB>(qv, cv, CB + ((int64_t)j * KSUB + c) * dsub, dsub);
            mn = i ? fminf(mn, v) : v;
            mx = i ? fmaxf(mx, v) : v;
        }
        for (int o = 32; o; o >>= 1) { mn = fminf(mn, __shfl_xor(mn, o)); mx = fmaxf(mx, __shfl_xor(mx, o)); }
        if (lane == 0) lo_out[pair * m + j] = mn;
        rng = fmaxf(rng, mx - mn);
    }
    if (lane == 0 && rng > 0.f) atomicMax(range_bits + q, __float_as_uint(rng));
}

template <int DSUB>
__global__ void __launch_bounds__(256) lut_l2_quant_kernel(const float* __restrict__ Q, const float* __restrict__ C,
                                                           const float* __restrict__ CB, const int32_t* __restrict__ probes,
                                                           int nprobe, int d, int m, const float* __restrict__ lo_in,
                                                           const uint32_t* __restrict__ range_bits, uint8_t* __restrict__ tables,
                                                           int32_t* __restrict__ bias, float* __restrict__ delta,
                                                           float* __restrict__ out_L, uint8_t* __restrict__ out_LUT8) {
    __shared__ __align__(16) uint8_t tab[LUT_BYTES];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t pair = blockIdx.x;
    const int64_t q = pair / nprobe;
    const int l = probes[pair];
    const int dsub = DSUB ? DSUB : d / m;
    const int S = rago_steps(m), planes = rago_planes(m);
    const float dq = lut_step(__uint_as_float(range_bits[q]));
    for (int j = wave; j < m; j += 4) {
        const float* qv = Q + q * d + j * dsub;
        const float* cv = C + (int64_t)l * d + j * dsub;
        const float lo = lo_in[pair * m + j];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = lane + 64 * i;
            const float L = l2_entry<DSUB>(qv, cv, CB + ((int64_t)j * KSUB + c) * dsub, dsub);
            float r = rintf(__fdiv_rn(L - lo, dq));
            r = r < 0.0f ? 0.0f : (r > 255.0f ? 255.0f : r);
            const uint8_t v = (uint8_t)r;
            for (int rep = j & (S - 1); rep < 32; rep += S) tab[(j >> 5) * LUT_PLANE + c * 32 + rep] = v;
            if (out_L) out_L[(pair * m + j) * KSUB + c] = L;
            if (out_LUT8) out_LUT8[(pair * m + j) * KSUB + c] = v;
        }
    }
    __syncthreads();
    uint4* dst = reinterpret_cast<uint4*>(tables + pair * LUT_BYTES);
    const uint4* src = reinterpret_cast<const uint4*>(tab);
    for (int i = threadIdx.x; i < planes * LUT_PLANE / 16; i += 256) dst[i] = src[i];
    if (threadIdx.x == 0) {
        double losum = 0.0;
        for (int j = 0; j < m; ++j) losum = losum + (double)lo_in[pair * m + j];
        bias[pair] = (int32_t)rint(losum / (double)dq);
        if (pair % nprobe == 0) delta[q] = dq;
    }
}

__global__ void fill_u32_kernel(uint32_t* p, uint32_t v, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
}

int launch_swizzle_lut(rago_index* idx, const uint8_t* lut8_plain, int64_t npairs, uint8_t* lut8sw, hipStream_t st) {
    lut_swizzle_kernel<<<(unsigned)npairs, 256, 0, st>>>(lut8_plain, idx->m, lut8sw);
    RAGO_HIP(hipGetLastError());
    return RAGO_OK;
}

int launch_build_lut(rago_index* idx, const float* q, const int32_t* probes, int64_t nq, int nprobe, LutTables* out,
                     float* out_L_f32, uint8_t* out_LUT8, hipStream_t st, const SmallSetupArgs* setup, const WavePlanArgs* wave_plan) {
    Workspace& ws = idx->ws;
    const int m = idx->m, d = idx->d;
    const int64_t npairs = nq * nprobe;
    int rc;
    if ((rc = ws.T64.reserve((size_t)nq * m * KSUB * 8))) return rc;
    if ((rc = ws.Tmin.reserve((size_t)nq * m * 8))) return rc;
    if ((rc = ws.Tmax.reserve((size_t)nq * m * 8 + (size_t)nq * 8))) return rc;   // + range and magnitude bits per query
    if ((rc = ws.pair_lo.reserve((size_t)npairs * m * 8))) return rc;
    if ((rc = ws.lut8.reserve((size_t)nq * LUT_BYTES))) return rc;
    if ((rc = ws.amb.reserve((size_t)nq * AMB_MAX * 2 + (size_t)nq * 4))) return rc;
    if ((rc = ws.patch.reserve((size_t)npairs * AMB_MAX))) return rc;
    if ((rc = ws.bias.reserve((size_t)npairs * 4))) return rc;
    if ((rc = ws.delta.reserve((size_t)nq * 4))) return rc;
    double* Tmax = ws.Tmax.as<double>();
    uint32_t* range_bits = reinterpret_cast<uint32_t*>(Tmax + nq * m);
    uint32_t* mag_bits = range_bits + nq;
    uint16_t* amb_addr = ws.amb.as<uint16_t>();
    int32_t* namb = reinterpret_cast<int32_t*>(amb_addr + nq * AMB_MAX);
    if ((rc = ws.counters.reserve(64))) return rc;
    if (idx->reserving) return RAGO_OK;
    const int ppw = npairs >= 32768 ? 8 : 1;
    // queries per wave of the T part: eight once that still leaves every compute unit eight waves (256 queries x 96
    // sub-quantisers: both kernels of this file 66 -> 57 us; 4 per wave the same, 16 per wave 64)
    const int qb = nq * m >= (int64_t)64 * idx->n_cu ? 8 : 1;
    const unsigned tg = (unsigned)(((nq + qb - 1) / qb * m + 3) / 4), pgrid = (unsigned)((npairs + 4 * ppw - 1) / (4 * ppw));
    // two launches: the per-query tables together with the per-pair scalars, then everything else of a query
    WavePlanArgs wp{};
    WaveFixArgs fix{};
    if (wave_plan && wave_plan->enable) {
        wp = *wave_plan;
        fix.enable = 1; fix.qinfo = wp.qinfo; fix.qnext = wp.qnext; fix.nq = wp.nq; fix.nwg = wp.nwg; fix.nprobe = wp.nprobe;
    }
    const unsigned plan_wgs = wp.enable ? (unsigned)nq : 0u;
    if (d / m == 8 && d % 4 == 0)        // (16-byte loads of the sub-vectors)
        lut_Tt_kernel<8><<<tg + pgrid + plan_wgs, 256, 0, st>>>(q, idx->centroids, idx->codebooks, probes, nq, npairs, ppw, d, m, plan_wgs, tg, qb,
                                                                ws.T64.as<double>(), ws.Tmin.as<double>(), Tmax, ws.pair_lo.as<double>(),
                                                                ws.counters.as<int64_t>(), wp);
    else
        lut_Tt_kernel<0><<<tg + pgrid + plan_wgs, 256, 0, st>>>(q, idx->centroids, idx->codebooks, probes, nq, npairs, ppw, d, m, plan_wgs, tg, qb,
                                                                ws.T64.as<double>(), ws.Tmin.as<double>(), Tmax, ws.pair_lo.as<double>(),
                                                                ws.counters.as<int64_t>(), wp);
    // (workgroups per query: enough to fill the chip on a small batch, at most one per 32 pairs)
    // workgroups per query: a wave per pair at a time; one round of pairs per workgroup while the batch leaves room
    const unsigned lq_y = (unsigned)std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(512 / nq, (nprobe + 15) / 16), 32));
    SmallSetupArgs su{};
    if (setup && setup->enable) {
        static_assert(SSU_THREADS == LQ_THREADS, "the bookkeeping rides in a workgroup of the table kernel");
        su = *setup;
        static OncePerDevice once;
        if (once.first())
            RAGO_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(lut_query_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)SSU_LDS));
    }
    lut_query_kernel<<<dim3((unsigned)nq, lq_y + (su.enable ? 1u : 0u)), LQ_THREADS, su.enable ? SSU_LDS : 0, st>>>(
        ws.T64.as<double>(), ws.Tmin.as<double>(), Tmax, ws.pair_lo.as<double>(), nprobe, m, range_bits, mag_bits, ws.lut8.as<uint8_t>(), amb_addr,
        namb, ws.delta.as<float>(), ws.bias.as<int32_t>(), ws.patch.as<uint8_t>(), ws.counters.as<int64_t>(), (int)lq_y, su, fix);
    if (out_L_f32 || out_LUT8)
        lut_expand_kernel<<<(unsigned)npairs, 256, 0, st>>>(ws.T64.as<double>(), ws.Tmin.as<double>(), ws.pair_lo.as<double>(), range_bits,
                                                            ws.lut8.as<uint8_t>(), amb_addr, namb, ws.patch.as<uint8_t>(), nprobe, m,
                                                            out_L_f32, out_LUT8);
    RAGO_HIP(hipGetLastError());
    out->lut_base = ws.lut8.as<uint8_t>();
    out->amb_addr = amb_addr;
    out->namb = namb;
    out->patch_val = ws.patch.as<uint8_t>();
    out->T64 = ws.T64.as<double>();
    out->Tmin = ws.Tmin.as<double>();
    out->t64 = ws.pair_lo.as<double>();
    out->range_bits = range_bits;
    out->bias = ws.bias.as<int32_t>();
    out->delta = ws.delta.as<float>();
    return RAGO_OK;
}

int launch_build_lut_l2(rago_index* idx, const float* q, const int32_t* probes, int64_t nq, int nprobe, float* out_L_f32,
                        uint8_t* out_LUT8, hipStream_t st) {
    Workspace& ws = idx->ws;
    const int m = idx->m, d = idx->d;
    const int64_t npairs = nq * nprobe;
    int rc;
    if ((rc = ws.tmp_lut8sw.reserve((size_t)npairs * LUT_BYTES))) return rc;
    if ((rc = ws.pair_lo.reserve((size_t)(npairs + 32) * m * 8))) return rc;  // per-(pair, sub-quantiser) minima (fp32; the fast path rounds the pairs up to 32)
    if ((rc = ws.Tmax.reserve((size_t)nq * m * 8 + (size_t)nq * 8))) return rc;   // the range words live behind the fp64 maxima
    if ((rc = ws.bias.reserve((size_t)npairs * 4))) return rc;
    if ((rc = ws.delta.reserve((size_t)nq * 4))) return rc;
    if ((rc = ws.counters.reserve(64))) return rc;
    if (idx->reserving) return lut_l2_fast_supported(idx) ? launch_lut_l2_fast(idx, q, probes, npairs, nprobe, nullptr, nullptr, nullptr, st) : RAGO_OK;
    uint32_t* range_bits = reinterpret_cast<uint32_t*>(ws.Tmax.as<double>() + nq * m);
    float* lo = ws.pair_lo.as<float>();
    fill_u32_kernel<<<(unsigned)std::min<int64_t>(1024, (nq + 255) / 256), 256, 0, st>>>(range_bits, 0u, nq);
    fill_u32_kernel<<<1, 64, 0, st>>>(reinterpret_cast<uint32_t*>(ws.counters.as<int64_t>() + 4), 0u, 4);   // counters [4], [5]
    // The fp32 path with exact fix-ups produces the tables, bias and step; the plain fp32 tables (an inspection
    // output) and sub-vector lengths without a fast path come from the kernels that evaluate every entry in fp64.
    const bool fast = lut_l2_fast_supported(idx);
    if (!fast || out_L_f32) {
        if (d / m == 8 && d % 4 == 0) {
            lut_l2_range_kernel<8><<<(unsigned)npairs, 256, 0, st>>>(q, idx->centroids, idx->codebooks, probes, nprobe, d, m, lo, range_bits);
            lut_l2_quant_kernel<8><<<(unsigned)npairs, 256, 0, st>>>(q, idx->centroids, idx->codebooks, probes, nprobe, d, m, lo, range_bits,
                                                                    ws.tmp_lut8sw.as<uint8_t>(), ws.bias.as<int32_t>(), ws.delta.as<float>(),
                                                                    out_L_f32, fast ? nullptr : out_LUT8);
        } else {
            lut_l2_range_kernel<0><<<(unsigned)npairs, 256, 0, st>>>(q, idx->centroids, idx->codebooks, probes, nprobe, d, m, lo, range_bits);
            lut_l2_quant_kernel<0><<<(unsigned)npairs, 256, 0, st>>>(q, idx->centroids, idx->codebooks, probes, nprobe, d, m, lo, range_bits,
                                                                    ws.tmp_lut8sw.as<uint8_t>(), ws.bias.as<int32_t>(), ws.delta.as<float>(),
                                                                    out_L_f32, fast ? nullptr : out_LUT8);
        }
    }
    if (fast) {
        if (out_L_f32) {           // start the fast path from scratch, so that it is what the caller's tables come from
            fill_u32_kernel<<<(unsigned)std::min<int64_t>(1024, (nq + 255) / 256), 256, 0, st>>>(range_bits, 0u, nq);
            fill_u32_kernel<<<(unsigned)std::min<int64_t>(4096, ((npairs + 32) * m + 255) / 256), 256, 0, st>>>(reinterpret_cast<uint32_t*>(lo), 0x7fc00000u, (npairs + 32) * m);
        }
        if ((rc = launch_lut_l2_fast(idx, q, probes, npairs, nprobe, lo, range_bits, out_LUT8, st))) return rc;
    }
    RAGO_HIP(hipGetLastError());
    return RAGO_OK;
}

}  // namespace rago

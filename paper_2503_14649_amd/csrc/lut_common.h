// The one fp32 expression that defines an 8-bit table entry, shared by every kernel that may
// have to evaluate it (patch builder, table expansion, the scan's per-pair path).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rago {

constexpr int AMB_MAX = 512;   // ambiguous entries kept per query; more -> per-pair evaluation

__device__ __forceinline__ float lut_step(float range) {
    const float dq = range / 255.0f;
    return dq > 0.0f ? dq : 1.0f;
}

// Half-width of the zone around a half-integer in which the per-pair fp32 result may differ from
// rne((T - Tmin) / delta): twice the bound 2^-24 * ((2 M + range) / delta + 256), plus, for tables so small that
// their entries are subnormal fp32 numbers (absolute rounding error 2^-150 instead of a relative one), four
// smallest subnormals over delta.
__device__ __forceinline__ double lut_eta(float range, float mag, float dq) {
    return 2.0 * 5.9604644775390625e-08 * ((2.0 * (double)mag + (double)range) / (double)dq + 256.0) +
           4.0 * 1.401298464324817e-45 / (double)dq;
}

// LUT8 entry from the fp64 per-query part Tv, the fp64 per-pair part t and the pair's fp32 minimum.
__device__ __forceinline__ uint8_t lut_entry(double Tv, double t, float lo, float dq) {
    const float L = (float)(Tv + t);
    float r = rintf(__fdiv_rn(L - lo, dq));
    r = r < 0.0f ? 0.0f : (r > 255.0f ? 255.0f : r);
    return (uint8_t)r;
}

// Euclidean metric: table entry -|q_j - (c_j + codeword)|^2 accumulated in fp64 in index order, one rounding to fp32
// (the expression and order that define the entry).  DSUB = 0: any length (`dsub`).
template <int DSUB>
__device__ __forceinline__ float l2_entry(const float* __restrict__ qv, const float* __restrict__ cv, const float* __restrict__ cb,
                                          int dsub) {
    double acc = 0.0;
    if constexpr (DSUB == 8) {
        const float4 q0 = *reinterpret_cast<const float4*>(qv), q1 = *reinterpret_cast<const float4*>(qv + 4);
        const float4 c0 = *reinterpret_cast<const float4*>(cv), c1 = *reinterpret_cast<const float4*>(cv + 4);
        const float4 b0 = *reinterpret_cast<const float4*>(cb), b1 = *reinterpret_cast<const float4*>(cb + 4);
        const float qa[8] = {q0.x, q0.y, q0.z, q0.w, q1.x, q1.y, q1.z, q1.w};
        const float ca[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
        const float ba[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const double diff = (double)qa[t] - ((double)ca[t] + (double)ba[t]);
            acc = acc + diff * diff;
        }
    } else {
        for (int t = 0; t < dsub; ++t) {
            const double diff = (double)qv[t] - ((double)cv[t] + (double)cb[t]);
            acc = acc + diff * diff;
        }
    }
    return (float)(-acc);
}

// Everything a consumer needs to obtain the table of one (query, list) pair.
struct LutTables {
    const uint8_t* lut_base;    // [nq][plane][256][32] base tables
    const uint16_t* amb_addr;   // [nq][AMB_MAX] positions (plane*8192 + code*32 + slot) of ambiguous entries
    const int32_t* namb;        // [nq] number of ambiguous entries, AMB_MAX + 1 = evaluate per pair
    const uint8_t* patch_val;   // [npairs][AMB_MAX] exact values of those entries
    const double* T64;          // [nq][m][256]
    const double* Tmin;         // [nq][m]
    const double* t64;          // [npairs][m]
    const uint32_t* range_bits; // [nq] float bits of max (hi - lo)
    const int32_t* bias;        // [npairs]
    const float* delta;         // [nq]
};

}  // namespace rago

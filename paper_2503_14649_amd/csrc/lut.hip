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
// Output table layout ("swizzled", what the scan copies into LDS): [pair][c][128] with byte
// slot*4 + plane = entry c of sub-quantiser plane*32 + slot; for m < 32 the m sub-tables are
// replicated 32/m times over the 32 slots.
#include "rago_internal.h"

namespace rago {

// T64[q][j][c], Tmin/Tmax[q][j].  grid (nq, m), 256 threads = one per codeword.
__global__ void __launch_bounds__(256) lut_T_kernel(const float* __restrict__ Q, const float* __restrict__ CB, int d, int m,
                                                    double* __restrict__ T64, double* __restrict__ Tmin, double* __restrict__ Tmax) {
    const int j = blockIdx.y, c = threadIdx.x;
    const int64_t q = blockIdx.x;
    const int dsub = d / m;
    const float* qv = Q + q * d + j * dsub;
    const float* cb = CB + ((int64_t)j * KSUB + c) * dsub;
    double acc = 0.0;
    for (int t = 0; t < dsub; ++t) acc = acc + (double)qv[t] * (double)cb[t];
    T64[(q * m + j) * KSUB + c] = acc;
    double mn = acc, mx = acc;
    for (int o = 32; o; o >>= 1) {
        mn = fmin(mn, __shfl_xor(mn, o));
        mx = fmax(mx, __shfl_xor(mx, o));
    }
    __shared__ double s_mn[4], s_mx[4];
    if ((c & 63) == 0) { s_mn[c >> 6] = mn; s_mx[c >> 6] = mx; }
    __syncthreads();
    if (c == 0) {
        Tmin[q * m + j] = fmin(fmin(s_mn[0], s_mn[1]), fmin(s_mn[2], s_mn[3]));
        Tmax[q * m + j] = fmax(fmax(s_mx[0], s_mx[1]), fmax(s_mx[2], s_mx[3]));
    }
}

// Per pair: t64[pair][j]; per query: running max of (hi - lo) as float bits (values are >= 0).
__global__ void __launch_bounds__(128) lut_pair_kernel(const float* __restrict__ Q, const float* __restrict__ C,
                                                       const int32_t* __restrict__ probes, int nprobe, int d, int m,
                                                       const double* __restrict__ Tmin, const double* __restrict__ Tmax,
                                                       double* __restrict__ t64, uint32_t* __restrict__ range_bits) {
    const int64_t pair = blockIdx.x;
    const int64_t q = pair / nprobe;
    const int l = probes[pair];
    const int dsub = d / m;
    float rng = 0.f;
    for (int j = threadIdx.x; j < m; j += blockDim.x) {
        const float* qv = Q + q * d + j * dsub;
        const float* cv = C + (int64_t)l * d + j * dsub;
        double acc = 0.0;
        for (int t = 0; t < dsub; ++t) acc = acc + (double)qv[t] * (double)cv[t];
        t64[pair * m + j] = acc;
        const float lo = (float)(Tmin[q * m + j] + acc), hi = (float)(Tmax[q * m + j] + acc);
        rng = fmaxf(rng, hi - lo);
    }
    for (int o = 32; o; o >>= 1) rng = fmaxf(rng, __shfl_xor(rng, o));
    if ((threadIdx.x & 63) == 0 && rng > 0.f) atomicMax(range_bits + q, __float_as_uint(rng));
}

// Per pair: quantise.  256 threads = one per codeword c (one table row each).
template <bool PLAIN>
__global__ void __launch_bounds__(256) lut_quant_kernel(const double* __restrict__ T64, const double* __restrict__ Tmin,
                                                        const double* __restrict__ t64, const uint32_t* __restrict__ range_bits,
                                                        int nprobe, int m, uint8_t* __restrict__ lut8sw, int32_t* __restrict__ bias,
                                                        float* __restrict__ delta, float* __restrict__ out_L,
                                                        uint8_t* __restrict__ out_LUT8) {
    __shared__ double s_t[128];
    __shared__ float s_lo[128];
    const int64_t pair = blockIdx.x;
    const int64_t q = pair / nprobe;
    const int c = threadIdx.x;
    float dq = __uint_as_float(range_bits[q]) / 255.0f;
    if (!(dq > 0.0f)) dq = 1.0f;
    if (c < m) {
        const double t = t64[pair * m + c];
        s_t[c] = t;
        s_lo[c] = (float)(Tmin[q * m + c] + t);
    }
    __syncthreads();
    if (c == 0) {
        double losum = 0.0;
        for (int j = 0; j < m; ++j) losum = losum + (double)s_lo[j];
        bias[pair] = (int32_t)rint(losum / (double)dq);
        if (pair % nprobe == 0) delta[q] = dq;
    }
    uint32_t row[LUT_ROW / 4];
#pragma unroll
    for (int i = 0; i < LUT_ROW / 4; ++i) row[i] = 0;
    const double* Tq = T64 + q * m * KSUB + c;
    const int S = rago_steps(m);
    for (int j = 0; j < m; ++j) {
        const float L = (float)(Tq[(int64_t)j * KSUB] + s_t[j]);
        float r = rintf(__fdiv_rn(L - s_lo[j], dq));
        r = r < 0.0f ? 0.0f : (r > 255.0f ? 255.0f : r);
        const uint32_t v = (uint32_t)r;
        if (PLAIN) {
            if (out_L) out_L[(pair * m + j) * KSUB + c] = L;
            if (out_LUT8) out_LUT8[(pair * m + j) * KSUB + c] = (uint8_t)v;
        }
        const int slot = j & (S - 1), plane = j >> 5;
        row[slot] |= v << (8 * plane);   // slot*4 + plane = byte `plane` of dword `slot`
    }
    if (S < 32) {                        // replicate the m sub-tables over all 32 slots
        for (int s = S; s < 32; ++s) row[s] = row[s & (S - 1)];
    }
    uint4* dst = reinterpret_cast<uint4*>(lut8sw + pair * LUT_BYTES + (int64_t)c * LUT_ROW);
#pragma unroll
    for (int i = 0; i < LUT_ROW / 16; ++i) dst[i] = make_uint4(row[4 * i], row[4 * i + 1], row[4 * i + 2], row[4 * i + 3]);
}

// plain [pair][m][256] u8 -> swizzled [pair][256][128]
__global__ void __launch_bounds__(256) lut_swizzle_kernel(const uint8_t* __restrict__ plain, int m, uint8_t* __restrict__ lut8sw) {
    const int64_t pair = blockIdx.x;
    const int c = threadIdx.x;
    uint32_t row[LUT_ROW / 4];
#pragma unroll
    for (int i = 0; i < LUT_ROW / 4; ++i) row[i] = 0;
    const int S = rago_steps(m);
    for (int j = 0; j < m; ++j) {
        const uint32_t v = plain[(pair * m + j) * KSUB + c];
        row[j & (S - 1)] |= v << (8 * (j >> 5));
    }
    if (S < 32) {
        for (int s = S; s < 32; ++s) row[s] = row[s & (S - 1)];
    }
    uint4* dst = reinterpret_cast<uint4*>(lut8sw + pair * LUT_BYTES + (int64_t)c * LUT_ROW);
#pragma unroll
    for (int i = 0; i < LUT_ROW / 16; ++i) dst[i] = make_uint4(row[4 * i], row[4 * i + 1], row[4 * i + 2], row[4 * i + 3]);
}

__global__ void fill_u32_kernel(uint32_t* p, uint32_t v, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
}

int launch_swizzle_lut(rago_index* idx, const uint8_t* lut8_plain, int64_t npairs, uint8_t* lut8sw, hipStream_t st) {
    lut_swizzle_kernel<<<(unsigned)npairs, 256, 0, st>>>(lut8_plain, idx->m, lut8sw);
    RAGO_HIP(hipGetLastError());
    return RAGO_OK;
}

int launch_build_lut(rago_index* idx, const float* q, const int32_t* probes, int64_t nq, int nprobe, uint8_t* lut8sw,
                     int32_t* bias, float* delta, float* out_L_f32, uint8_t* out_LUT8, hipStream_t st) {
    Workspace& ws = idx->ws;
    const int m = idx->m, d = idx->d;
    const int64_t npairs = nq * nprobe;
    int rc;
    if ((rc = ws.T64.reserve((size_t)nq * m * KSUB * 8))) return rc;
    if ((rc = ws.Tmin.reserve((size_t)nq * m * 8))) return rc;
    if ((rc = ws.Tmax.reserve((size_t)nq * m * 8 + (size_t)nq * 4))) return rc;   // + range bits per query
    if ((rc = ws.pair_lo.reserve((size_t)npairs * m * 8))) return rc;
    double* Tmax = ws.Tmax.as<double>();
    uint32_t* range_bits = reinterpret_cast<uint32_t*>(Tmax + nq * m);
    fill_u32_kernel<<<64, 256, 0, st>>>(range_bits, 0u, nq);
    lut_T_kernel<<<dim3((unsigned)nq, m), 256, 0, st>>>(q, idx->codebooks, d, m, ws.T64.as<double>(), ws.Tmin.as<double>(), Tmax);
    lut_pair_kernel<<<(unsigned)npairs, 128, 0, st>>>(q, idx->centroids, probes, nprobe, d, m, ws.Tmin.as<double>(), Tmax,
                                                      ws.pair_lo.as<double>(), range_bits);
    if (out_L_f32 || out_LUT8)
        lut_quant_kernel<true><<<(unsigned)npairs, 256, 0, st>>>(ws.T64.as<double>(), ws.Tmin.as<double>(), ws.pair_lo.as<double>(),
                                                                 range_bits, nprobe, m, lut8sw, bias, delta, out_L_f32, out_LUT8);
    else
        lut_quant_kernel<false><<<(unsigned)npairs, 256, 0, st>>>(ws.T64.as<double>(), ws.Tmin.as<double>(), ws.pair_lo.as<double>(),
                                                                  range_bits, nprobe, m, lut8sw, bias, delta, nullptr, nullptr);
    RAGO_HIP(hipGetLastError());
    return RAGO_OK;
}

}  // namespace rago

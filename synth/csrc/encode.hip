// Input-generator helper (not part of the retrieval library, not used by the oracle):
// product-quantiser ENCODING of freshly sampled vectors at billion-vector scale.
// codes[v][j] = argmin_c | (x[v]_j - C[list[v]]_j) - CB[j][c] |^2, ties -> lower c.
#include <hip/hip_runtime.h>
#include <stdint.h>

template <int DSUB>
__global__ void __launch_bounds__(256) encode_kernel(const float* __restrict__ x, const float* __restrict__ centroids,
                                                     const int64_t* __restrict__ list, const float* __restrict__ cb,
                                                     int64_t n, int d, int m, uint8_t* __restrict__ codes) {
    __shared__ float s_cb[256 * DSUB];
    const int j = blockIdx.y;
    for (int i = threadIdx.x; i < 256 * DSUB; i += 256) s_cb[i] = cb[(int64_t)j * 256 * DSUB + i];
    __syncthreads();
    for (int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x; v < n; v += (int64_t)gridDim.x * 256) {
        float r[DSUB];
        const float* xv = x + v * d + j * DSUB;
        const float* cv = centroids + list[v] * d + j * DSUB;
#pragma unroll
        for (int t = 0; t < DSUB; ++t) r[t] = xv[t] - cv[t];
        float best = 3.4e38f;
        int bc = 0;
        for (int c = 0; c < 256; ++c) {
            float dist = 0.f;
#pragma unroll
            for (int t = 0; t < DSUB; ++t) {
                const float e = r[t] - s_cb[c * DSUB + t];
                dist += e * e;
            }
            if (dist < best) { best = dist; bc = c; }
        }
        codes[v * m + j] = (uint8_t)bc;
    }
}

extern "C" int synth_pq_encode(const float* x, const float* centroids, const int64_t* list, const float* cb, int64_t n,
                               int d, int m, uint8_t* codes, void* stream) {
    if (n <= 0) return 0;
    const int dsub = d / m;
    unsigned gx = (unsigned)((n + 255) / 256);
    if (gx > 16384) gx = 16384;
    dim3 grid(gx, m);
    hipStream_t st = (hipStream_t)stream;
    switch (dsub) {
        case 1: encode_kernel<1><<<grid, 256, 0, st>>>(x, centroids, list, cb, n, d, m, codes); break;
        case 2: encode_kernel<2><<<grid, 256, 0, st>>>(x, centroids, list, cb, n, d, m, codes); break;
        case 4: encode_kernel<4><<<grid, 256, 0, st>>>(x, centroids, list, cb, n, d, m, codes); break;
        case 8: encode_kernel<8><<<grid, 256, 0, st>>>(x, centroids, list, cb, n, d, m, codes); break;
        case 16: encode_kernel<16><<<grid, 256, 0, st>>>(x, centroids, list, cb, n, d, m, codes); break;
        case 3: encode_kernel<3><<<grid, 256, 0, st>>>(x, centroids, list, cb, n, d, m, codes); break;
        case 6: encode_kernel<6><<<grid, 256, 0, st>>>(x, centroids, list, cb, n, d, m, codes); break;
        case 12: encode_kernel<12><<<grid, 256, 0, st>>>(x, centroids, list, cb, n, d, m, codes); break;
        case 24: encode_kernel<24><<<grid, 256, 0, st>>>(x, centroids, list, cb, n, d, m, codes); break;
        default: return -1;
    }
    return hipGetLastError() == hipSuccess ? 0 : -2;
}

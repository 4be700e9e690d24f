// One-time re-layout of the PQ codes for the scan (index load / wrap time).
//
// The scan keeps 8-bit look-up tables in LDS with every sub-table confined to one LDS bank
// (32 banks x 4 bytes on gfx950: a half-wavefront of 32 lanes is served per clock when all
// lanes hit different banks).  One lane scans one vector.  For the 32 lanes of a half-wave to
// hit 32 different banks in the same instruction they must be working on 32 different
// sub-quantisers, so lane l at step s handles sub-quantiser (s + l) mod 32 (per plane of 32
// sub-quantisers).  To keep the byte extraction identical in all lanes, this rotation is baked
// into the stored bytes: position t of lane l's byte string holds the code of sub-quantiser
//   j(t, l) = plane(t) * 32 + slot(step(t), l),   plane = t / S, step = t % S,
//   slot(s, l) = ((s + l) & (S-1)) | (l & 31 & ~(S-1)),   S = min(m, 32)
// (for m < 32 the 32 lanes cover 32/m replicas of the tables, one replica per group of m banks).
//
// A block = 64 consecutive vectors of one list (last block zero-padded) = 64*m bytes laid out
// [t / 16][lane][t % 16], so one dwordx4 load per lane reads 1 KiB contiguous per wavefront.
#include <algorithm>
#include "rago_internal.h"

namespace rago {

__global__ void __launch_bounds__(256) relayout_kernel(const uint8_t* __restrict__ plain, const int64_t* __restrict__ list_off,
                                                       const int64_t* __restrict__ blk_off, int nlist, int m,
                                                       uint8_t* __restrict__ out) {
    __shared__ int s_list;
    const int64_t b = blockIdx.x;
    if (threadIdx.x == 0) {
        int lo = 0, hi = nlist;  // largest l with blk_off[l] <= b
        while (hi - lo > 1) {
            int mid = (lo + hi) >> 1;
            if (blk_off[mid] <= b) lo = mid; else hi = mid;
        }
        s_list = lo;
    }
    __syncthreads();
    const int l = s_list;
    const int64_t v0 = list_off[l] + (b - blk_off[l]) * BLOCK_VECS;  // first vector row of the block
    const int64_t vend = list_off[l + 1];
    const int S = rago_steps(m);
    const int npieces = BLOCK_VECS * m / 16;
    uint8_t* dst = out + b * (int64_t)(BLOCK_VECS * m);
    for (int piece = threadIdx.x; piece < npieces; piece += blockDim.x) {
        const int chunk = piece / BLOCK_VECS, lane = piece % BLOCK_VECS;
        const int64_t v = v0 + lane;
        uint32_t w[4] = {0, 0, 0, 0};
        if (v < vend) {
            const uint8_t* row = plain + v * m;
            const int l32 = lane & 31;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int t = chunk * 16 + e;
                const int plane = t / S, step = t % S;
                const int slot = ((step + l32) & (S - 1)) | (l32 & ~(S - 1));
                const int j = plane * 32 + (slot & (S - 1));
                w[e >> 2] |= (uint32_t)row[j] << (8 * (e & 3));
            }
        }
        *reinterpret_cast<uint4*>(dst + (int64_t)piece * 16) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// flag[0] != 0 if ids are not strictly ascending inside some list
__global__ void __launch_bounds__(256) check_ids_kernel(const int64_t* __restrict__ ids, const int64_t* __restrict__ list_off,
                                                        int* flag) {
    const int l = blockIdx.x;
    const int64_t a = list_off[l], e = list_off[l + 1];
    for (int64_t i = a + 1 + threadIdx.x; i < e; i += blockDim.x)
        if (ids[i] <= ids[i - 1]) *flag = 1;
}

__global__ void __launch_bounds__(256) cnorm_kernel(const float* __restrict__ C, int nlist, int d, float* __restrict__ out,
                                                    float* __restrict__ out2) {
    const int l = blockIdx.x * (blockDim.x / 64) + threadIdx.x / 64;
    if (l >= nlist) return;
    float acc = 0.f;
    double acc2 = 0.0;
    for (int t = threadIdx.x & 63; t < d; t += 64) {
        const float v = C[(int64_t)l * d + t];
        acc += v * v;
        acc2 = acc2 + (double)v * (double)v;
    }
    for (int o = 32; o; o >>= 1) { acc += __shfl_xor(acc, o); acc2 = acc2 + __shfl_xor(acc2, o); }
    if ((threadIdx.x & 63) == 0) {
        out[l] = sqrtf(acc) * 1.0001f;  // slight over-estimate: used as a bound
        out2[l] = (float)acc2;          // |c|^2 for the Euclidean coarse scores
    }
}

// Plain device-to-device copy of known size: the yardstick that hardware byte counters are
// scaled by when a profile of the scan is taken.
__global__ void __launch_bounds__(256) rago_calib_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t n16) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (int64_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

int launch_calib_copy(const void* src, void* dst, int64_t bytes, hipStream_t st) {
    rago_calib_copy_kernel<<<8192, 256, 0, st>>>(static_cast<const uint4*>(src), static_cast<uint4*>(dst), bytes / 16);
    RAGO_HIP(hipGetLastError());
    return RAGO_OK;
}

// Plain read stream of known size: what a kernel that only reads HBM reaches on this device, the
// practical ceiling the scans are also held against (Section 4, "Retrieval performance modeling",
// takes ~80 % of the memory bandwidth as what a good code scan reaches).  Every workgroup leaves the XOR
// of what it read in sink[blockIdx.x] so the loads cannot be dropped.
constexpr int READ_STREAM_BLOCKS = 4096;
typedef uint32_t rs_u32x4 __attribute__((ext_vector_type(4)));
__global__ void __launch_bounds__(256) rago_calib_read_kernel(const rs_u32x4* __restrict__ src, int64_t n16, uint32_t* __restrict__ sink) {
    // every workgroup reads one contiguous run; eight independent non-temporal 16-byte loads per lane in flight
    const int64_t per = (n16 + gridDim.x - 1) / gridDim.x;
    const int64_t first = blockIdx.x * per, end = first + per < n16 ? first + per : n16;
    rs_u32x4 acc = {0u, 0u, 0u, 0u};
    int64_t i = first + threadIdx.x;
    for (; i + 7 * 256 < end; i += 8 * 256) {
        rs_u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + i + u * 256);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u];
    }
    for (; i < end; i += 256) acc ^= __builtin_nontemporal_load(src + i);
    uint32_t v = acc.x ^ acc.y ^ acc.z ^ acc.w;
    for (int o = 32; o; o >>= 1) v ^= __shfl_xor(v, o);
    if ((threadIdx.x & 63) == 0) atomicXor(&sink[blockIdx.x], v);
}

int read_stream_sink_words() { return READ_STREAM_BLOCKS; }

int launch_calib_read(const void* src, int64_t bytes, uint32_t* sink, hipStream_t st) {
    rago_calib_read_kernel<<<READ_STREAM_BLOCKS, 256, 0, st>>>(static_cast<const rs_u32x4*>(src), bytes / 16, sink);
    RAGO_HIP(hipGetLastError());
    return RAGO_OK;
}

// 4-bit product quantisation (a finer-grained trade of code size against accuracy than Section 4's
// one byte per 8 dimensions): a code byte holds two sub-quantisers of 16 codewords, the even one in
// its low nibble.  Read as ONE symbol, that byte indexes the 256 concatenations of the two sets of
// codewords over the joint sub-space; this kernel writes that 256-word codebook ([m/2][256][2 dsub],
// pure copies), after which the index is an ordinary 8-bit one with m/2 code bytes.
__global__ void __launch_bounds__(256) expand_pq4_kernel(const float* __restrict__ cb16, int m, int dsub, float* __restrict__ cb256) {
    const int64_t total = (int64_t)(m / 2) * 256 * 2 * dsub;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int t = (int)(i % (2 * dsub));
        const int b = (int)((i / (2 * dsub)) % 256);
        const int j = (int)(i / ((int64_t)2 * dsub * 256));
        const int sub = t < dsub ? 2 * j : 2 * j + 1;
        const int nib = t < dsub ? (b & 15) : (b >> 4);
        cb256[i] = cb16[((int64_t)sub * 16 + nib) * dsub + (t < dsub ? t : t - dsub)];
    }
}

int launch_expand_pq4(const float* d_cb16, int m, int dsub, float* d_cb256, hipStream_t st) {
    const int64_t total = (int64_t)(m / 2) * 256 * 2 * dsub;
    const int blocks = (int)std::min<int64_t>((total + 255) / 256, 4096);
    expand_pq4_kernel<<<blocks, 256, 0, st>>>(d_cb16, m, dsub, d_cb256);
    RAGO_HIP(hipGetLastError());
    RAGO_HIP(hipStreamSynchronize(st));
    return RAGO_OK;
}

int build_layout(rago_index* idx, const uint8_t* d_codes_plain, hipStream_t st) {
    if (idx->total_blocks > 0) {
        if (idx->total_blocks > 0x7fffffffLL) return fail(RAGO_UNSUPPORTED, "more than 2^31 code blocks");
        relayout_kernel<<<dim3((unsigned)idx->total_blocks), 256, 0, st>>>(d_codes_plain, idx->list_off, idx->blk_off,
                                                                          idx->nlist, idx->m, idx->codes_blk);
        RAGO_HIP(hipGetLastError());
    }
    int* flag = nullptr;
    RAGO_HIP(hipMalloc(&flag, sizeof(int)));
    RAGO_HIP(hipMemsetAsync(flag, 0, sizeof(int), st));
    check_ids_kernel<<<idx->nlist, 256, 0, st>>>(idx->ids, idx->list_off, flag);
    cnorm_kernel<<<(idx->nlist + 3) / 4, 256, 0, st>>>(idx->centroids, idx->nlist, idx->d, idx->cnorm, idx->cn2);
    int h = 0;
    hipError_t e = hipMemcpyAsync(&h, flag, sizeof(int), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    hipFree(flag);
    if (e != hipSuccess) return fail(RAGO_DEVICE, std::string("layout: ") + hipGetErrorString(e));
    if (h) return fail(RAGO_FORMAT, "ids must be strictly ascending inside every list");
    return RAGO_OK;
}

}  // namespace rago

// Planning of the wave-per-item scan (scan_wave.hip): one workgroup of 256 threads per query.  A header because two
// kernels run it: plan_kernel by itself, and the first table kernel of the inner-product path as the work of nq extra
// workgroups (the plan needs only the probes, so it runs beside the tables instead of in a launch of its own between
// them and the scan).  There it cannot know yet whether a query's tables will come per pair - that follows from the
// tables - so the second table kernel, which finds out, corrects the three words that depend on it (WaveFixArgs).
#pragma once
#include "rago_internal.h"
#include "scan_common.h"

namespace rago {

// One probed list of one query: where its codes and rows start, how long it is, and the query-local number of its
// first item.  32 bytes.  The descriptors of a query stand in the order its items are handed out, `pair` says whose
// they are: probe number `pair` of the query.
struct WavePairDesc { int64_t blk0, row0; int32_t nblk, len, pre, pair; };

constexpr int WAVE_BATCH = 16;      // items a workgroup of the scan claims at a time (two per wave)

struct WavePlanArgs {
    int enable;                     // 0: nothing to do (the scan launches plan_kernel itself)
    const int32_t* probes;          // [nq][nprobe]
    const int64_t* blk_off;         // [nlist + 1]
    const int64_t* list_off;        // [nlist + 1]
    int nprobe, CH, m, nq, nwg;     // nwg = workgroups of the scan kernel
    const int32_t* namb;            // [nq] ambiguous entries per query, or null: not known yet (see WaveFixArgs)
    int all_per_pair;               // every query's tables come per pair (caller's tables, Euclidean metric)
    WavePairDesc* pdesc;            // out [npairs]
    int32_t* pair_pre;              // out [npairs]
    int4* qinfo;                    // out [nq] {units (items, or pairs when tables come per pair), items, per-pair tables?, 0}
    int32_t* qnext;                 // out [nq] next unclaimed unit
    int32_t* qatt;                  // out [nq] 0
    int64_t* qbytes;                // out [nq][2] code bytes streamed / algorithmic code bytes of the query
    int32_t* tauq;                  // out [nq] INT32_MIN
    int64_t* counters;              // out [0..2] = 0 (the scan kernel adds the batch's totals)
};

// What a query whose tables turn out to come per pair changes in its plan (its units are then pairs, not items).
struct WaveFixArgs {
    int enable;
    int4* qinfo;
    int32_t* qnext;
    int nq, nwg, nprobe;
};

// workgroups of the scan that first attach to query q (workgroup b takes query b mod nq)
__device__ __forceinline__ int wave_attached(int q, int nq, int nwg) { return q < nwg ? (nwg - 1 - q) / nq + 1 : 0; }

__device__ __forceinline__ void wave_fix_per_pair(const WaveFixArgs& F, int q) {
    F.qinfo[q].x = F.nprobe;
    F.qinfo[q].z = 1;
    F.qnext[q] = wave_attached(q, F.nq, F.nwg);
}

// The descriptor of every pair of query q, the query-local number of each pair's first item, the query's totals, its
// counters and its bound.  The r-th workgroup that first attaches to the query takes items r * WAVE_BATCH .. without
// asking, so the query's counter starts behind those.  256 threads.
__device__ __forceinline__ void wave_plan_body(const WavePlanArgs& A, int q) {
    __shared__ int s_w[4];
    __shared__ int s_carry;
    __shared__ unsigned long long s_bytes[2];
    __shared__ int s_key[256];
    __shared__ WavePairDesc s_pd[256];
    const int nprobe = A.nprobe, CH = A.CH, m = A.m;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) { s_carry = 0; s_bytes[0] = 0; s_bytes[1] = 0; }
    if (q == 0 && tid < 3) A.counters[tid] = 0;
    __syncthreads();
    unsigned long long streamed = 0, algo = 0;
    for (int p0 = 0; p0 < nprobe; p0 += 256) {
        const int p = p0 + tid, np = min(256, nprobe - p0);
        WavePairDesc pd = {0, 0, 0, 0, 0, 0};
        if (p < nprobe) {
            const int l = A.probes[(int64_t)q * nprobe + p];
            pd.blk0 = A.blk_off[l];
            pd.row0 = A.list_off[l];
            pd.nblk = (int)(A.blk_off[l + 1] - pd.blk0);
            pd.len = (int)(A.list_off[l + 1] - pd.row0);
            pd.pair = p;
            streamed += (unsigned long long)pd.nblk * (BLOCK_VECS * m);
            algo += (unsigned long long)pd.len * m;
        }
        // Longest first among these (up to) 256 pairs: a query's items are handed out in this order, and what its
        // waves wait for at the end - the last items still running - are then the short ones.
        s_key[tid] = pd.nblk;
        __syncthreads();
        if (p < nprobe) {
            int pos = 0;
#pragma unroll 8
            for (int j = 0; j < np; ++j) {
                const int o = s_key[j];
                pos += o > pd.nblk || (o == pd.nblk && j < tid) ? 1 : 0;
            }
            s_pd[pos] = pd;
        }
        __syncthreads();
        if (p < nprobe) pd = s_pd[tid];
        const int n = p < nprobe ? (pd.nblk + CH - 1) / CH : 0;
        int inc = n;
        for (int o = 1; o < 64; o <<= 1) {
            const int v = __shfl_up(inc, o);
            if (lane >= o) inc += v;
        }
        if (lane == 63) s_w[wave] = inc;
        __syncthreads();
        int before = s_carry;
        for (int w = 0; w < wave; ++w) before += s_w[w];
        if (p < nprobe) {
            pd.pre = before + inc - n;
            A.pdesc[(int64_t)q * nprobe + p] = pd;
            A.pair_pre[(int64_t)q * nprobe + p] = pd.pre;
        }
        __syncthreads();
        if (tid == 255) s_carry = before + inc;
        __syncthreads();
    }
    for (int o = 32; o; o >>= 1) { streamed += __shfl_xor(streamed, o); algo += __shfl_xor(algo, o); }
    if (lane == 0) { atomicAdd(&s_bytes[0], streamed); atomicAdd(&s_bytes[1], algo); }
    __syncthreads();
    if (tid == 0) {
        const int items = s_carry;
        const int per_pair = A.all_per_pair || (A.namb && A.namb[q] > AMB_MAX);
        A.qinfo[q] = make_int4(per_pair ? nprobe : items, items, per_pair, 0);
        A.qnext[q] = wave_attached(q, A.nq, A.nwg) * (per_pair ? 1 : WAVE_BATCH);
        A.qatt[q] = 0;
        A.tauq[q] = INT32_MIN;
        A.qbytes[2 * q] = (int64_t)s_bytes[0];
        A.qbytes[2 * q + 1] = (int64_t)s_bytes[1];
    }
}

}  // namespace rago

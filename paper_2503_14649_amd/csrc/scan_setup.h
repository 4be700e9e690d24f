// Bookkeeping of a small batch in one workgroup: (query, list) pairs grouped by list and the table of scan tasks.
// A header because two kernels run it: small_setup_kernel by itself, and the table kernel of the inner-product path as
// the work of one extra workgroup (the bookkeeping needs only the probes, so it runs beside the tables instead of
// after them: one dependent launch less on the path of a latency-bound round, Section 5.3).
#pragma once
#include "rago_internal.h"

namespace rago {

// For batches of at most SSU_PAIRS pairs (iterative retrieval, Section 5.3: a few queries per round, where six
// dependent launches cost more than the work in them).  The lists are found through a hash table in LDS instead of
// arrays over all nlist lists, so nothing of size nlist is cleared or read.  Touched lists are numbered in
// hash-table order; the order of a list's pairs is whatever order their atomics arrive in.
constexpr int SSU_PAIRS = 4096, SSU_HASH = 8192, SSU_THREADS = 1024;
constexpr size_t SSU_LDS = (size_t)(2 * SSU_HASH + 3 * (SSU_PAIRS + 2)) * 4 + 1024;

struct SmallSetupArgs {
    int enable;                 // 0: nothing to do (the caller launches the bookkeeping kernels itself)
    const int32_t* probes;      // [npairs]
    int npairs, nq;
    const int2* list_meta;      // [nlist] {blocks, vectors} of each list
    int CH, group, m;
    int32_t* pair_sorted;       // out [npairs]
    int4* table;                // out: one record per task
    int32_t* ctrl;              // out [4]: task counter, tasks, touched lists, 0
    int32_t* tauq;              // out [nq]: INT32_MIN
    int64_t* counters;          // out [0..2]: tasks, code bytes streamed, algorithmic code bytes
};

// The work of one workgroup of SSU_THREADS threads on SSU_LDS bytes of LDS at `ssu` (16-byte aligned).
__device__ __forceinline__ void small_setup_body(const SmallSetupArgs& A, int32_t* ssu) {
    const int32_t* __restrict__ probes = A.probes;
    const int npairs = A.npairs, nq = A.nq, CH = A.CH, group = A.group, m = A.m;
    const int2* __restrict__ list_meta = A.list_meta;
    int32_t* __restrict__ pair_sorted = A.pair_sorted;
    int4* __restrict__ table = A.table;
    int32_t* __restrict__ ctrl = A.ctrl;
    int32_t* __restrict__ tauq = A.tauq;
    int64_t* __restrict__ counters = A.counters;
    int32_t* keys = ssu;                          // [SSU_HASH] list number or -1
    int32_t* cnt = keys + SSU_HASH;               // [SSU_HASH] pairs of that list; later: where its pairs start
    int32_t* t_list = cnt + SSU_HASH;             // by touched slot: list, first pair, first task (one more: the totals)
    int32_t* t_po = t_list + SSU_PAIRS + 2;       // (an even number of words each: s_acc below stays 8-byte aligned)
    int32_t* t_to = t_po + SSU_PAIRS + 2;
    int32_t* s_w = t_to + SSU_PAIRS + 2;          // [3][16] wave totals of the scans, [48..50] their grand totals
    unsigned long long* s_acc = reinterpret_cast<unsigned long long*>(s_w + 52);   // streamed, algorithmic bytes (8-byte aligned)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // (the probes are requested before LDS is cleared, and unconditionally: the trip to memory overlaps the clearing)
    constexpr int PER = SSU_PAIRS / SSU_THREADS;
    int pl[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) pl[e] = probes[min(e * SSU_THREADS + tid, npairs - 1)];
    for (int i = tid; i < SSU_HASH; i += SSU_THREADS) { keys[i] = -1; cnt[i] = 0; }
    for (int i = tid; i < nq; i += SSU_THREADS) tauq[i] = INT32_MIN;
    if (tid < 2) s_acc[tid] = 0ull;
    __syncthreads();
    // ---- every pair finds or claims its list's cell and takes a position among the list's pairs
    int cell[PER], ppos[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        const int i = e * SSU_THREADS + tid;
        cell[e] = -1; ppos[e] = 0;
        if (i < npairs) {
            const int l = pl[e];
            unsigned h = ((unsigned)l * 2654435761u) >> 19;       // 13 bits
            for (;;) {                                            // (at most SSU_PAIRS of the SSU_HASH cells are ever taken)
                const int old = atomicCAS(&keys[h], -1, l);
                if (old == -1 || old == l) break;
                h = (h + 1) & (SSU_HASH - 1);
            }
            cell[e] = (int)h;
            ppos[e] = atomicAdd(&cnt[h], 1);
        }
    }
    __syncthreads();
    // Exclusive sums over the workgroup of up to three values per thread: inside each wave by shuffles, across the
    // waves by the first wave (a loop over the 16 wave totals in every thread costs 48 dependent LDS reads).
    auto scan3 = [&](int& a, int& b, int& c, int& ta, int& tb, int& tc) {
        int ia = a, ib = b, ic = c;
        for (int o = 1; o < 64; o <<= 1) {
            const int x = __shfl_up(ia, o), y = __shfl_up(ib, o), z = __shfl_up(ic, o);
            if (lane >= o) { ia += x; ib += y; ic += z; }
        }
        __syncthreads();
        if (lane == 63) { s_w[wave] = ia; s_w[16 + wave] = ib; s_w[32 + wave] = ic; }
        __syncthreads();
        if (wave == 0) {
            const int n = SSU_THREADS / 64;
            int wa = lane < n ? s_w[lane] : 0, wb = lane < n ? s_w[16 + lane] : 0, wc = lane < n ? s_w[32 + lane] : 0;
            const int oa = wa, ob = wb, oc = wc;
            for (int o = 1; o < 16; o <<= 1) {
                const int x = __shfl_up(wa, o), y = __shfl_up(wb, o), z = __shfl_up(wc, o);
                if (lane >= o) { wa += x; wb += y; wc += z; }
            }
            if (lane < n) { s_w[lane] = wa - oa; s_w[16 + lane] = wb - ob; s_w[32 + lane] = wc - oc; }
            if (lane == n - 1) { s_w[48] = wa; s_w[49] = wb; s_w[50] = wc; }
        }
        __syncthreads();
        a = ia - a + s_w[wave]; b = ib - b + s_w[16 + wave]; c = ic - c + s_w[32 + wave];
        ta = s_w[48]; tb = s_w[49]; tc = s_w[50];
    };
    // ---- per cell (eight per thread): is it taken, how many pairs; exclusive sums give every touched list its slot
    // number and its first pair
    constexpr int CPT = SSU_HASH / SSU_THREADS;
    int cl[CPT], cc[CPT];
    int bo = 0, bc = 0, unused = 0, tot_o, tot_c, tot_t;
#pragma unroll
    for (int e = 0; e < CPT; ++e) {
        cl[e] = keys[tid * CPT + e]; cc[e] = cnt[tid * CPT + e];
        bo += cl[e] >= 0 ? 1 : 0; bc += cl[e] >= 0 ? cc[e] : 0;
    }
    scan3(bo, bc, unused, tot_o, tot_c, tot_t);
#pragma unroll
    for (int e = 0; e < CPT; ++e) {
        if (cl[e] >= 0) {
            t_list[bo] = cl[e]; t_po[bo] = bc;
            cnt[tid * CPT + e] = bc;
            bo += 1; bc += cc[e];
        }
    }
    if (tid == 0) t_po[tot_o] = tot_c;
    __syncthreads();
    // ---- per touched list (four consecutive slots per thread): its tasks; their exclusive sums.  The loads are
    // unconditional, from a clamped slot: one trip to memory for all of them.
    constexpr int SPT = SSU_PAIRS / SSU_THREADS;
    int st[SPT], pc[SPT], bt = 0, u1 = 0, u2 = 0, x1, x2;
    unsigned long long streamed = 0, algo = 0;
    {
        int2 meta[SPT];
#pragma unroll
        for (int e = 0; e < SPT; ++e) {
            const int sl = min(tid * SPT + e, max(tot_o - 1, 0));
            pc[e] = t_po[sl + 1] - t_po[sl];
            meta[e] = list_meta[t_list[sl]];
        }
#pragma unroll
        for (int e = 0; e < SPT; ++e) {
            const bool live = tid * SPT + e < tot_o;
            const int c = pc[e], nblk = meta[e].x;
            st[e] = live ? ((c + group - 1) / group) * ((nblk + CH - 1) / CH) : 0;
            streamed += live ? (unsigned long long)((c + group - 1) / group) * nblk * (BLOCK_VECS * m) : 0ull;
            algo += live ? (unsigned long long)c * (unsigned long long)meta[e].y * m : 0ull;
            bt += st[e];
        }
    }
    for (int o = 32; o; o >>= 1) { streamed += __shfl_xor(streamed, o); algo += __shfl_xor(algo, o); }
    if (lane == 0 && (streamed | algo)) { atomicAdd(&s_acc[0], streamed); atomicAdd(&s_acc[1], algo); }
    scan3(bt, u1, u2, tot_t, x1, x2);
    // ---- pairs grouped by list
#pragma unroll
    for (int e = 0; e < PER; ++e)
        if (cell[e] >= 0) pair_sorted[cnt[cell[e]] + ppos[e]] = e * SSU_THREADS + tid;
#pragma unroll
    for (int e = 0; e < SPT; ++e) {
        if (tid * SPT + e < tot_o) t_to[tid * SPT + e] = bt;
        bt += st[e];
    }
    if (tid == 0) t_to[tot_o] = tot_t;
    __syncthreads();
    // ---- one record per task (as task_table_kernel)
    for (int t = tid; t < tot_t; t += SSU_THREADS) {
        int lo = 0, hi = tot_o;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (t_to[mid] <= t) lo = mid; else hi = mid;
        }
        const int rem = t - t_to[lo];
        const int npl = t_po[lo + 1] - t_po[lo];
        const int ngroups = (npl + group - 1) / group;
        const int chunk = rem / ngroups, grp = rem - chunk * ngroups;
        const int per = npl / ngroups, extra = npl - per * ngroups;
        const int first = grp * per + min(grp, extra);
        table[t] = make_int4(t_list[lo], chunk, t_po[lo] + first, per + (grp < extra ? 1 : 0));
    }
    __syncthreads();
    if (tid == 0) {
        ctrl[0] = 0; ctrl[1] = tot_t; ctrl[2] = tot_o; ctrl[3] = 0;
        counters[0] = tot_t; counters[1] = (int64_t)s_acc[0]; counters[2] = (int64_t)s_acc[1];
    }
}


}  // namespace rago

// Declarations shared by the two scan kernels (scan.hip: four pairs per pass, one workgroup per
// CU, for long tasks; scan_narrow.hip: two pairs per pass, two workgroups per CU, for short ones)
// and the bookkeeping / merge kernels around them.
#pragma once
#include "rago_internal.h"

namespace rago {

constexpr int CAPW = 192;       // keys per (wave, pair) buffer: k <= 128 survivors + one block of 64

struct ScanParams {
    const uint8_t* codes;
    const int64_t* blk_off;
    const int64_t* list_off;
    const int64_t* ids;
    const int32_t* probes;       // [npairs] list of each pair
    const uint8_t* lut8sw;       // [npairs] plane-major per-pair tables (stride LUT_BYTES), or null: use `T`
    LutTables T;                 // per-query base tables + per-pair patches
    const int32_t* bias;         // [npairs]
    int m;
    const int32_t* pair_sorted;  // pairs grouped by list
    const int4* task_table;      // [ntasks] {list, chunk, first position in pair_sorted, number of pairs}
    int32_t* ctrl;               // [0] task counter, [1] number of tasks
    int32_t* tauq;               // [nq] lower bound of the k-th best integer score
    int32_t* part_I;             // [npairs][maxchunks][k]
    int64_t* part_row;           // same shape: row of the entry in the list-major arrays
    int32_t* part_cnt;           // [npairs][maxchunks]
    int nlist, nprobe, k, CH, maxchunks;
};

// ------------------------------------------------------------------ small helpers
// Publish a bound on a query's k-th best score.  Any value ever published is a valid bound, so a plain store is
// enough (a late smaller store only weakens the word until the next one): read-modify-write operations on ONE address
// in HBM run at a few tens of millions per second and, on this hardware, hold up every later load of the wave that
// issued them, which costs tens of microseconds when hundreds of workgroups work on a handful of queries.
__device__ __forceinline__ void publish_bound(int32_t* tauq, int32_t value) {
    if (value > __hip_atomic_load(tauq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
        __hip_atomic_store(tauq, value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ int lane_rank(uint64_t mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

// k-th largest of the non-zero keys held NR per lane by one wave (wave-uniform result).
template <int NR>
__device__ __forceinline__ uint32_t select_kth(const uint32_t (&r)[NR], int k) {
    uint32_t prefix = 0;
    int rem = k;
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t test = prefix | (1u << bit);
        const uint32_t hm = ~((1u << bit) - 1u);
        int c1 = 0;
#pragma unroll
        for (int i = 0; i < NR; ++i) c1 += __popcll(__ballot((r[i] & hm) == test));
        if (c1 >= rem) prefix = test; else rem -= c1;
    }
    return prefix;
}

// Keep the best k keys of buf[0..cnt) (cnt > k), compacted to buf[0..k); returns the k-th key.
__device__ __forceinline__ uint32_t wave_prune(uint32_t* buf, int& cnt, int k, int lane) {
    uint32_t r[CAPW / 64];
#pragma unroll
    for (int i = 0; i < CAPW / 64; ++i) r[i] = (lane + 64 * i < cnt) ? buf[lane + 64 * i] : 0u;
    const uint32_t kth = select_kth<CAPW / 64>(r, k);
    int base = 0;
#pragma unroll
    for (int i = 0; i < CAPW / 64; ++i) {
        const bool keep = r[i] >= kth && r[i] != 0u;
        const uint64_t mask = __ballot(keep);
        if (keep) buf[base + lane_rank(mask)] = r[i];
        base += __popcll(mask);
    }
    cnt = base;
    return kth;
}

// Append the lanes whose sum reaches the threshold to the wave's key buffer (prune when full).
__device__ __forceinline__ void offer(bool valid, uint32_t sum, uint32_t pos, uint32_t* buf, int& cnt, uint32_t& thr,
                                      int32_t* sh_tau, int k, int lane) {
    const bool c = valid && sum >= thr;
    const uint64_t mask = __ballot(c);
    if (mask == 0) return;
    const int add = __popcll(mask);
    if (cnt + add > CAPW) {
        const uint32_t kth = wave_prune(buf, cnt, k, lane);
        const uint32_t t = kth >> 16;
        if (t > thr) thr = t;
        if (lane == 0) atomicMax(sh_tau, (int32_t)thr);
    }
    if (c) buf[cnt + lane_rank(mask)] = (sum << 16) | (0xFFFFu - pos);
    cnt += add;
}

// The code stream and the tables are read through pointers explicitly in the global address
// space: a generic (flat) load would also count on the LDS/scalar wait counter and every
// hand-placed s_waitcnt lgkmcnt in the look-up code would then wait for HBM.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef const __attribute__((address_space(1))) u32x4* global_u32x4_ptr;
typedef const __attribute__((address_space(1))) u32x2* global_u32x2_ptr;

// NT: non-temporal loads, for streams that are read once by one workgroup and far larger than the caches (the
// billion-vector batch: 14.2 ms against 14.6 ms per scan with ordinary loads; a plain read stream of 8 GiB reaches
// 6.9 TB/s against 6.1 TB/s).  Where lists are probed again soon afterwards by other tasks (batches over a database
// of about the size of the 256 MiB last-level cache) ordinary loads are the faster ones, by 6 %.
template <int MPAD, bool NT = false>
__device__ __forceinline__ void load_block(uint4 (&w)[MPAD / 16], const uint8_t* blk, int lane) {
    global_u32x4_ptr p = (global_u32x4_ptr)(reinterpret_cast<const u32x4*>(blk) + lane);
#pragma unroll
    for (int i = 0; i < MPAD / 16; ++i) {
        const u32x4 v = NT ? __builtin_nontemporal_load(p + i * 64) : p[i * 64];
        w[i] = make_uint4(v.x, v.y, v.z, v.w);
    }
}

// ------------------------------------------------------------------ final per-query merge: shared pieces
constexpr int MERGE_THREADS = 256;
constexpr int MERGE_CAP = 2048;

__device__ __forceinline__ bool entry_before(int32_t ia, int64_t da, int32_t ib, int64_t db) {
    return ia > ib || (ia == ib && da < db);
}

// Sort sI/sId[0..n2) (n2 a power of two) by (I desc, id asc).
__device__ inline void bitonic_sort(int32_t* sI, int64_t* sId, int n2) {
    for (int size = 2; size <= n2; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            for (int t = threadIdx.x; t < n2 / 2; t += blockDim.x) {
                const int i = 2 * t - (t & (stride - 1));
                const int j = i + stride;
                const bool up = (i & size) == 0;  // this sub-sequence ends best-first
                const int32_t ia = sI[i], ib = sI[j];
                const int64_t da = sId[i], db = sId[j];
                const bool swap = up ? entry_before(ib, db, ia, da) : entry_before(ia, da, ib, db);
                if (swap) { sI[i] = ib; sI[j] = ia; sId[i] = db; sId[j] = da; }
            }
        }
    }
    __syncthreads();
}

// The best k of sI/sId[0..have), have <= blockDim.x, into sI/sId[0..min(have, k)) in order, one entry per thread and
// without a sorting network.  First by score alone: an entry with k or more strictly better scores above it cannot be
// in the result; the others (k plus ties at the k-th score) move to a side buffer.  Then a full rank among those:
// every entry of the result has only entries of the result before it, so its rank there is its place.  (Equal entries
// - an id the caller stored twice - rank by position, so every place is taken once.)  Returns false, with the first
// `have` entries untouched, when more than RANK_CAND entries reach the side buffer (massive ties).
// sI: 16-byte aligned, room for have + 4 entries; tmp: 3 * RANK_CAND + 1 words of LDS, 8-byte aligned.
constexpr int RANK_CAND = 256;
__device__ inline bool rank_top_k(int32_t* sI, int64_t* sId, int have, int k, int32_t* tmp) {
    int32_t* cI = tmp;
    int64_t* cId = reinterpret_cast<int64_t*>(tmp + RANK_CAND);
    int* nc = tmp + 3 * RANK_CAND;
    const int t = threadIdx.x;
    if (t == 0) *nc = 0;
    if (t < 4) sI[have + t] = INT32_MIN;             // the scores are read four at a time
    __syncthreads();
    int32_t mi = 0;
    int64_t md = 0;
    bool cand = false;
    if (t < have) {
        mi = sI[t]; md = sId[t];
        int gt = 0;
#pragma unroll 4
        for (int j = 0; j < have; j += 4) {
            const int4 v = *reinterpret_cast<const int4*>(sI + j);
            gt += (v.x > mi ? 1 : 0) + (v.y > mi ? 1 : 0) + (v.z > mi ? 1 : 0) + (v.w > mi ? 1 : 0);
        }
        cand = gt < k;
    }
    if (cand) {
        const int o = atomicAdd(nc, 1);
        if (o < RANK_CAND) { cI[o] = mi; cId[o] = md; }
    }
    __syncthreads();
    const int n = *nc;
    if (n > RANK_CAND) return false;
    if (t < n) {
        mi = cI[t]; md = cId[t];
        int before = 0;
#pragma unroll 8
        for (int j = 0; j < n; ++j) {
            const int32_t oi = cI[j];
            const int64_t od = cId[j];
            before += entry_before(oi, od, mi, md) || (oi == mi && od == md && j < t) ? 1 : 0;
        }
        if (before < k) { sI[before] = mi; sId[before] = md; }
    }
    __syncthreads();
    return true;
}

// scan_narrow.hip: the two-pairs-per-pass kernel on 2 * n_cu workgroups (task records with 1 or 2 pairs)
int launch_scan_narrow(const ScanParams& P, int n_cu, hipStream_t st);

// scan_wave.hip: one wave per (pair, chunk) item, pairs grouped by query.  Plans, scans and sorts the results itself.
int wave_chunk_len(double total_blocks, int n_cu);
size_t wave_pair_bytes();
size_t wave_stage_bytes(int64_t nq, int k);
struct WavePlanArgs;        // scan_plan.h
void fill_wave_plan(const ScanParams& P, int64_t nq, int n_cu, void* pdesc, int32_t* pair_pre, int32_t* qwork, int64_t* counters,
                    WavePlanArgs* A);
int launch_scan_wave(const ScanParams& P, int64_t nq, int n_cu, double avgblk, void* pdesc, int32_t* pair_pre, int32_t* qwork,
                     void* stage, int64_t* counters, const float* delta, int64_t* out_ids, float* out_scores, int32_t* out_iscores,
                     hipEvent_t* ev, hipStream_t st, bool plan_done);

}  // namespace rago

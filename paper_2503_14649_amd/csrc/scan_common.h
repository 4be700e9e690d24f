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

// scan_narrow.hip: the two-pairs-per-pass kernel on 2 * n_cu workgroups (task records with 1 or 2 pairs)
int launch_scan_narrow(const ScanParams& P, int n_cu, hipStream_t st);

// scan_wave.hip: one wave per (pair, chunk) item, pairs grouped by query.  Plans its items and tasks itself.
int wave_chunk_len(double total_blocks, int n_cu);
size_t wave_item_bytes();
int launch_scan_wave(const ScanParams& P, int64_t nq, int n_cu, double avgblk, void* items, int4* tasks, int32_t* pair_items,
                     int4* qinfo, int64_t* qbytes, int64_t* counters, hipEvent_t ev_scan, hipStream_t st);

}  // namespace rago

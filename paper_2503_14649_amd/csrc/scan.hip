// Integer asymmetric-distance scan of the probed lists + per-query top-k (the retrieval cost the
// paper measures in bytes of PQ codes scanned per query, Section 3.3; low-precision tables make
// the scan memory-bound, Section 2).
//
// For every (query, probed list) pair and every vector i of the list:
//     I = B[pair] + sum_j LUT8[pair][j][code[i][j]]
// and per query the best k of all its pairs by (I descending, id ascending).
//
// Work organisation
//  * pairs are grouped by list; a task = (list, chunk of <= CH 64-vector blocks, up to two pairs
//    of that list).  Both pairs' tables sit in LDS at once, so a code byte fetched once serves
//    two queries.  Persistent workgroups pull task numbers from one atomic counter; consecutive
//    task numbers share list and chunk, so repeats of a chunk hit in cache.
//  * LDS table layout (64 KiB): byte address = code * 256 + slot * 4 + plane (+128 for the
//    second pair).  `slot` selects the bank, so a sub-table lives in ONE bank; the 32 lanes of a
//    half-wave always work on 32 different slots (see layout.hip), which makes every ds_read_u8
//    conflict-free whatever the code values are.  The address is built with a single v_perm_b32
//    from the code dword and a per-lane register holding slot*4 for four consecutive steps;
//    plane and pair select ride in the instruction's immediate offset.
//  * one lane = one vector: 6 x dwordx4 loads (m = 96) per lane per block, 1 KiB contiguous per
//    wave and load, next block's loads issued before the current block is processed.
//  * selection: scores are <= 24480 so (score << 16 | 0xFFFF - position in chunk) is a 32-bit
//    key whose order is (score desc, position asc) = (score desc, id asc) inside one list.
//    Each wave keeps a private LDS buffer of keys above a running threshold and prunes it to the
//    best k with a radix select on ballots (no barriers, no atomics in the streaming loop).
//    Thresholds are shared through LDS (per task) and through a per-query word in HBM
//    (atomicMax of each finished task's k-th best score): a candidate below a score that k other
//    candidates of the same query already reach can never be in the result.
//  * each task writes <= k (I, id) entries; a final kernel per query merges them, sorts by
//    (I desc, id asc) and writes ids / scores.
#include "rago_internal.h"

namespace rago {

constexpr int SCAN_WAVES = 8;
constexpr int SCAN_THREADS = SCAN_WAVES * 64;
constexpr int CAPW = 192;  // keys per (wave, pair) buffer: k <= 128 survivors + one block of 64
constexpr int LUT_LDS = 65536;
constexpr int SCAN_LDS = LUT_LDS + SCAN_WAVES * 2 * CAPW * 4 + 512;
constexpr int DESC_INTS = 20;   // task descriptor in LDS (see fetch_task)

struct ScanParams {
    const uint8_t* codes;
    const int64_t* blk_off;
    const int64_t* list_off;
    const int64_t* ids;
    const int32_t* probes;       // [npairs] list of each pair
    const uint8_t* lut8sw;       // [npairs][256][128] swizzled per-pair tables, or null: use `T`
    LutTables T;                 // per-query base tables + per-pair patches
    const int32_t* bias;         // [npairs]
    int m;
    const int32_t* pair_sorted;  // pairs grouped by list
    const int4* task_table;      // [ntasks] {list, chunk, pairA, pairB (-1: none)}
    int32_t* ctrl;               // [0] task counter, [1] number of tasks
    int32_t* tauq;               // [nq] lower bound of the k-th best integer score
    int32_t* part_I;             // [npairs][maxchunks][k]
    int64_t* part_id;
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

// All lookups of one 64-vector block: lane = vector.  Hand-scheduled: the compiler serialises
// the byte loads behind full LDS waits and spills when given the plain C++ form.
//
// One code dword `w` holds 4 consecutive steps of one plane; `o` holds slot*4 of those 4 steps.
// v_perm_b32 puts code byte kb into byte 1 and o's byte kb into byte 0: address = code*256 + slot*4.
// Selector kb = 0x0c0c0000 | (4+kb) << 8 | kb.  The table region starts at LDS address 0.
// Each asm statement drains its own LDS reads (lgkmcnt(0)) before it ends, so the compiler's
// own wait counts around it stay valid.
#define RAGO_SEL0 0x0c0c0400u
#define RAGO_SEL1 0x0c0c0501u
#define RAGO_SEL2 0x0c0c0602u
#define RAGO_SEL3 0x0c0c0703u

// 16 lookups of one table (one dwordx4 = 4 code dwords, all in plane PL), added into `sum`.
template <int PL>
__device__ __forceinline__ void lookup16(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t w3, uint32_t o0, uint32_t o1,
                                         uint32_t o2, uint32_t o3, uint32_t s0, uint32_t s1, uint32_t s2, uint32_t s3,
                                         uint32_t& sum) {
    uint32_t t0, t1, t2, t3, t4, t5, t6, t7, t8, t9, t10, t11, t12, t13, t14, t15;
    asm volatile(
        "v_perm_b32 %[t0], %[w0], %[o0], %[s0]\n v_perm_b32 %[t1], %[w0], %[o0], %[s1]\n"
        "v_perm_b32 %[t2], %[w0], %[o0], %[s2]\n v_perm_b32 %[t3], %[w0], %[o0], %[s3]\n"
        "ds_read_u8 %[t0], %[t0] offset:%[pl]\n ds_read_u8 %[t1], %[t1] offset:%[pl]\n"
        "ds_read_u8 %[t2], %[t2] offset:%[pl]\n ds_read_u8 %[t3], %[t3] offset:%[pl]\n"
        "v_perm_b32 %[t4], %[w1], %[o1], %[s0]\n v_perm_b32 %[t5], %[w1], %[o1], %[s1]\n"
        "v_perm_b32 %[t6], %[w1], %[o1], %[s2]\n v_perm_b32 %[t7], %[w1], %[o1], %[s3]\n"
        "ds_read_u8 %[t4], %[t4] offset:%[pl]\n ds_read_u8 %[t5], %[t5] offset:%[pl]\n"
        "ds_read_u8 %[t6], %[t6] offset:%[pl]\n ds_read_u8 %[t7], %[t7] offset:%[pl]\n"
        "v_perm_b32 %[t8], %[w2], %[o2], %[s0]\n v_perm_b32 %[t9], %[w2], %[o2], %[s1]\n"
        "v_perm_b32 %[t10], %[w2], %[o2], %[s2]\n v_perm_b32 %[t11], %[w2], %[o2], %[s3]\n"
        "ds_read_u8 %[t8], %[t8] offset:%[pl]\n ds_read_u8 %[t9], %[t9] offset:%[pl]\n"
        "ds_read_u8 %[t10], %[t10] offset:%[pl]\n ds_read_u8 %[t11], %[t11] offset:%[pl]\n"
        "v_perm_b32 %[t12], %[w3], %[o3], %[s0]\n v_perm_b32 %[t13], %[w3], %[o3], %[s1]\n"
        "v_perm_b32 %[t14], %[w3], %[o3], %[s2]\n v_perm_b32 %[t15], %[w3], %[o3], %[s3]\n"
        "ds_read_u8 %[t12], %[t12] offset:%[pl]\n ds_read_u8 %[t13], %[t13] offset:%[pl]\n"
        "ds_read_u8 %[t14], %[t14] offset:%[pl]\n ds_read_u8 %[t15], %[t15] offset:%[pl]\n"
        "s_waitcnt lgkmcnt(10)\n"
        "v_add3_u32 %[t0], %[t0], %[t1], %[t2]\n v_add3_u32 %[t3], %[t3], %[t4], %[t5]\n"
        "s_waitcnt lgkmcnt(4)\n"
        "v_add3_u32 %[t6], %[t6], %[t7], %[t8]\n v_add3_u32 %[t9], %[t9], %[t10], %[t11]\n"
        "v_add3_u32 %[sum], %[sum], %[t0], %[t3]\n"
        "s_waitcnt lgkmcnt(0)\n"
        "v_add3_u32 %[t12], %[t12], %[t13], %[t14]\n v_add3_u32 %[t6], %[t6], %[t9], %[t15]\n"
        "v_add3_u32 %[sum], %[sum], %[t6], %[t12]\n"
        : [sum] "+v"(sum), [t0] "=&v"(t0), [t1] "=&v"(t1), [t2] "=&v"(t2), [t3] "=&v"(t3), [t4] "=&v"(t4), [t5] "=&v"(t5),
          [t6] "=&v"(t6), [t7] "=&v"(t7), [t8] "=&v"(t8), [t9] "=&v"(t9), [t10] "=&v"(t10), [t11] "=&v"(t11),
          [t12] "=&v"(t12), [t13] "=&v"(t13), [t14] "=&v"(t14), [t15] "=&v"(t15)
        : [w0] "v"(w0), [w1] "v"(w1), [w2] "v"(w2), [w3] "v"(w3), [o0] "v"(o0), [o1] "v"(o1), [o2] "v"(o2), [o3] "v"(o3),
          [s0] "s"(s0), [s1] "s"(s1), [s2] "s"(s2), [s3] "s"(s3), [pl] "n"(PL)
        : "memory");
}

// 8 lookups (2 code dwords) in each of the two resident tables (second table at +128).
template <int PL>
__device__ __forceinline__ void lookup8x2(uint32_t w0, uint32_t w1, uint32_t o0, uint32_t o1, uint32_t s0, uint32_t s1,
                                          uint32_t s2, uint32_t s3, uint32_t& suma, uint32_t& sumb) {
    uint32_t t0, t1, t2, t3, t4, t5, t6, t7, u0, u1, u2, u3, u4, u5, u6, u7;
    asm volatile(
        "v_perm_b32 %[t0], %[w0], %[o0], %[s0]\n v_perm_b32 %[t1], %[w0], %[o0], %[s1]\n"
        "v_perm_b32 %[t2], %[w0], %[o0], %[s2]\n v_perm_b32 %[t3], %[w0], %[o0], %[s3]\n"
        "ds_read_u8 %[u0], %[t0] offset:%[pb]\n ds_read_u8 %[u1], %[t1] offset:%[pb]\n"
        "ds_read_u8 %[u2], %[t2] offset:%[pb]\n ds_read_u8 %[u3], %[t3] offset:%[pb]\n"
        "ds_read_u8 %[t0], %[t0] offset:%[pa]\n ds_read_u8 %[t1], %[t1] offset:%[pa]\n"
        "ds_read_u8 %[t2], %[t2] offset:%[pa]\n ds_read_u8 %[t3], %[t3] offset:%[pa]\n"
        "v_perm_b32 %[t4], %[w1], %[o1], %[s0]\n v_perm_b32 %[t5], %[w1], %[o1], %[s1]\n"
        "v_perm_b32 %[t6], %[w1], %[o1], %[s2]\n v_perm_b32 %[t7], %[w1], %[o1], %[s3]\n"
        "ds_read_u8 %[u4], %[t4] offset:%[pb]\n ds_read_u8 %[u5], %[t5] offset:%[pb]\n"
        "ds_read_u8 %[u6], %[t6] offset:%[pb]\n ds_read_u8 %[u7], %[t7] offset:%[pb]\n"
        "ds_read_u8 %[t4], %[t4] offset:%[pa]\n ds_read_u8 %[t5], %[t5] offset:%[pa]\n"
        "ds_read_u8 %[t6], %[t6] offset:%[pa]\n ds_read_u8 %[t7], %[t7] offset:%[pa]\n"
        "s_waitcnt lgkmcnt(12)\n"
        "v_add3_u32 %[sumb], %[sumb], %[u0], %[u1]\n v_add_u32 %[u2], %[u2], %[u3]\n"
        "s_waitcnt lgkmcnt(8)\n"
        "v_add3_u32 %[suma], %[suma], %[t0], %[t1]\n v_add_u32 %[t2], %[t2], %[t3]\n"
        "s_waitcnt lgkmcnt(4)\n"
        "v_add3_u32 %[u4], %[u4], %[u5], %[u6]\n v_add3_u32 %[sumb], %[sumb], %[u2], %[u7]\n"
        "s_waitcnt lgkmcnt(0)\n"
        "v_add3_u32 %[t4], %[t4], %[t5], %[t6]\n v_add3_u32 %[suma], %[suma], %[t2], %[t7]\n"
        "v_add_u32 %[sumb], %[sumb], %[u4]\n v_add_u32 %[suma], %[suma], %[t4]\n"
        : [suma] "+v"(suma), [sumb] "+v"(sumb), [t0] "=&v"(t0), [t1] "=&v"(t1), [t2] "=&v"(t2), [t3] "=&v"(t3),
          [t4] "=&v"(t4), [t5] "=&v"(t5), [t6] "=&v"(t6), [t7] "=&v"(t7), [u0] "=&v"(u0), [u1] "=&v"(u1), [u2] "=&v"(u2),
          [u3] "=&v"(u3), [u4] "=&v"(u4), [u5] "=&v"(u5), [u6] "=&v"(u6), [u7] "=&v"(u7)
        : [w0] "v"(w0), [w1] "v"(w1), [o0] "v"(o0), [o1] "v"(o1), [s0] "s"(s0), [s1] "s"(s1), [s2] "s"(s2), [s3] "s"(s3),
          [pa] "n"(PL), [pb] "n"(PL + 128)
        : "memory");
}

template <int MPAD, int Q, int I>
__device__ __forceinline__ void block_sums_chunk(const uint4 (&w)[MPAD / 16], const uint32_t (&off)[(MPAD < 32 ? MPAD : 32) / 4],
                                                 uint32_t s0, uint32_t s1, uint32_t s2, uint32_t s3, uint32_t& sa, uint32_t& sb) {
    constexpr int S = MPAD < 32 ? MPAD : 32;
    constexpr int PL = (I * 16) / S;               // plane of this dwordx4
    constexpr int G = ((I * 16) % S) / 4;          // first of its four step groups
    if (Q == 1) {
        lookup16<PL>(w[I].x, w[I].y, w[I].z, w[I].w, off[G], off[G + 1], off[G + 2], off[G + 3], s0, s1, s2, s3, sa);
    } else {
        lookup8x2<PL>(w[I].x, w[I].y, off[G], off[G + 1], s0, s1, s2, s3, sa, sb);
        lookup8x2<PL>(w[I].z, w[I].w, off[G + 2], off[G + 3], s0, s1, s2, s3, sa, sb);
    }
    if constexpr (I + 1 < MPAD / 16) block_sums_chunk<MPAD, Q, I + 1>(w, off, s0, s1, s2, s3, sa, sb);
}

template <int MPAD, int Q>
__device__ __forceinline__ void block_sums(const uint4 (&w)[MPAD / 16], const uint32_t (&off)[(MPAD < 32 ? MPAD : 32) / 4],
                                           uint32_t s0, uint32_t s1, uint32_t s2, uint32_t s3, uint32_t& sa, uint32_t& sb) {
    sa = 0;
    sb = 0;
    block_sums_chunk<MPAD, Q, 0>(w, off, s0, s1, s2, s3, sa, sb);
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

// Copy swizzled tables (256 rows of 128 B) into the two halves of the 256-byte LDS rows; a null
// source leaves that half untouched.  `between` runs after the loads are issued and before their
// data is needed (the caller puts the first code-block loads there, so they queue behind the
// table loads instead of in front of them: the load counter retires in order).
template <class F>
__device__ __forceinline__ void copy_table(const uint4* srcA, const uint4* srcB, uint8_t* lut, F between) {
    // (named scalars, not arrays: conditionally filled arrays end up in scratch memory)
    const uint4 z = make_uint4(0, 0, 0, 0);
    uint4 a0 = z, a1 = z, a2 = z, a3 = z, b0 = z, b1 = z, b2 = z, b3 = z;
    const int t = threadIdx.x;
    if (srcA) { a0 = srcA[t]; a1 = srcA[t + SCAN_THREADS]; a2 = srcA[t + 2 * SCAN_THREADS]; a3 = srcA[t + 3 * SCAN_THREADS]; }
    if (srcB) { b0 = srcB[t]; b1 = srcB[t + SCAN_THREADS]; b2 = srcB[t + 2 * SCAN_THREADS]; b3 = srcB[t + 3 * SCAN_THREADS]; }
    between();
    // piece p = 16 bytes: row p >> 3, column (p & 7) * 16 of the 128-byte table row
    uint8_t* d0 = lut + (t >> 3) * 256 + (t & 7) * 16;
    constexpr int STEP = (SCAN_THREADS >> 3) * 256;   // rows advanced by SCAN_THREADS pieces
    if (srcA) {
        *reinterpret_cast<uint4*>(d0) = a0;
        *reinterpret_cast<uint4*>(d0 + STEP) = a1;
        *reinterpret_cast<uint4*>(d0 + 2 * STEP) = a2;
        *reinterpret_cast<uint4*>(d0 + 3 * STEP) = a3;
    }
    if (srcB) {
        *reinterpret_cast<uint4*>(d0 + 128) = b0;
        *reinterpret_cast<uint4*>(d0 + 128 + STEP) = b1;
        *reinterpret_cast<uint4*>(d0 + 128 + 2 * STEP) = b2;
        *reinterpret_cast<uint4*>(d0 + 128 + 3 * STEP) = b3;
    }
}

struct ScanParams;
__device__ void eval_table(const ScanParams& P, int pair, int q, uint8_t* slot);

// The code stream is read through pointers explicitly in the global address space: a generic
// (flat) load would also count on the LDS/scalar wait counter and every hand-placed
// s_waitcnt lgkmcnt in the look-up code would then wait for HBM.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(1))) u32x4* global_u32x4_ptr;

template <int MPAD>
__device__ __forceinline__ void load_block(uint4 (&w)[MPAD / 16], const uint8_t* blk, int lane) {
    global_u32x4_ptr p = (global_u32x4_ptr)(reinterpret_cast<const u32x4*>(blk) + lane);
#pragma unroll
    for (int i = 0; i < MPAD / 16; ++i) {
        const u32x4 v = p[i * 64];
        w[i] = make_uint4(v.x, v.y, v.z, v.w);
    }
}

// Full per-pair evaluation of a table straight into an LDS slot (queries whose tables are too
// flat for the base + patch form).
__device__ __forceinline__ void eval_table(const ScanParams& P, int pair, int q, uint8_t* slot) {
    const int m = P.m, S = rago_steps(m);
    const float dq = lut_step(__uint_as_float(P.T.range_bits[q]));
    for (int e = threadIdx.x; e < m * KSUB; e += SCAN_THREADS) {
        const int j = e >> 8, c = e & 255;
        const double t = P.T.t64[(int64_t)pair * m + j];
        const uint8_t v = lut_entry(P.T.T64[((int64_t)q * m + j) * KSUB + c], t, (float)(P.T.Tmin[(int64_t)q * m + j] + t), dq);
        for (int rep = j & (S - 1); rep < 32; rep += S) slot[c * 256 + rep * 4 + (j >> 5)] = v;
    }
}

// Claim the next task and put everything its prologue needs into LDS (run by ONE wave; all
// values are wave-uniform so the loads are scalar).  d[0] = task number or -1 when none is left.
__device__ __forceinline__ void fetch_task(const ScanParams& P, int ntasks, int32_t* d, int lane) {
    int t = 0;
    if (lane == 0) t = atomicAdd(P.ctrl, 1);
    t = __builtin_amdgcn_readfirstlane(t);
    if (t >= ntasks) {
        if (lane == 0) d[0] = -1;
        return;
    }
    const int4 rec = P.task_table[t];
    const int l = rec.x, pairA = rec.z, pairB = rec.w;
    const int64_t b0 = P.blk_off[l], v0 = P.list_off[l];
    const int nblk = (int)(P.blk_off[l + 1] - b0), len = (int)(P.list_off[l + 1] - v0);
    const int qA = pairA / P.nprobe, qB = pairB >= 0 ? pairB / P.nprobe : 0;
    const int biasA = P.bias[pairA], biasB = pairB >= 0 ? P.bias[pairB] : 0;
    int nA = 0, nB = 0;
    if (!P.lut8sw) { nA = P.T.namb[qA]; nB = pairB >= 0 ? P.T.namb[qB] : 0; }
    if (lane == 0) {
        d[0] = t; d[1] = l; d[2] = rec.y; d[3] = pairA; d[4] = pairB; d[5] = biasA; d[6] = biasB; d[7] = qA; d[8] = qB;
        d[9] = (int32_t)(uint32_t)b0; d[10] = (int32_t)(b0 >> 32); d[11] = nblk;
        d[12] = (int32_t)(uint32_t)v0; d[13] = (int32_t)(v0 >> 32); d[14] = len; d[15] = nA; d[16] = nB;
    }
}

// ------------------------------------------------------------------ the scan kernel
template <int MPAD>
__global__ void __launch_bounds__(SCAN_THREADS, 4) scan_kernel(const ScanParams P) {
    constexpr int S = MPAD < 32 ? MPAD : 32;
    extern __shared__ __align__(16) uint8_t smem[];
    uint8_t* lut = smem;
    uint32_t* cand = reinterpret_cast<uint32_t*>(smem + LUT_LDS);                         // [wave][pair][CAPW]
    int32_t* sh = reinterpret_cast<int32_t*>(smem + LUT_LDS + SCAN_WAVES * 2 * CAPW * 4);  // scalars
    // sh[2..3] tau per pair (sum units), sh[4] block counter, sh[5] finisher ticket, sh[8 + wave*2 + pair] wave counts, sh[32..] descriptors
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    uint32_t off[S / 4];
#pragma unroll
    for (int g = 0; g < S / 4; ++g) {
        uint32_t v = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int step = g * 4 + b, l32 = lane & 31;
            const int slot = ((step + l32) & (S - 1)) | (l32 & ~(S - 1));
            v |= (uint32_t)(slot * 4) << (8 * b);
        }
        off[g] = v;
    }
    const int ntasks = P.ctrl[1];
    int loadedA = -1, loadedB = -1;   // query whose base table currently sits in each LDS slot
    // selectors live in SGPRs (VOP3 takes no literal on gfx9); the asm fence keeps them out of constant folding
    uint32_t sel0 = RAGO_SEL0, sel1 = RAGO_SEL1, sel2 = RAGO_SEL2, sel3 = RAGO_SEL3;
    const int k = P.k;
    int32_t* desc = sh + 32;          // two task descriptors: the running task and the prefetched next one

    if (wave == SCAN_WAVES - 1) fetch_task(P, ntasks, desc, lane);
    __syncthreads();
    for (int cur = 0;; cur ^= 1) {
        const int32_t* D = desc + cur * DESC_INTS;
        const int tid = __builtin_amdgcn_readfirstlane(D[0]);
        if (tid < 0) break;           // every wave reads the same descriptor: all leave together
        const int chunk = __builtin_amdgcn_readfirstlane(D[2]);
        const int pairA = __builtin_amdgcn_readfirstlane(D[3]), pairB = __builtin_amdgcn_readfirstlane(D[4]);
        const int biasA = __builtin_amdgcn_readfirstlane(D[5]), biasB = __builtin_amdgcn_readfirstlane(D[6]);
        const int qA = __builtin_amdgcn_readfirstlane(D[7]), qB = __builtin_amdgcn_readfirstlane(D[8]);
        const int64_t b0 = ((int64_t)__builtin_amdgcn_readfirstlane(D[10]) << 32) | (uint32_t)__builtin_amdgcn_readfirstlane(D[9]);
        const int nblk_list = __builtin_amdgcn_readfirstlane(D[11]);
        const int64_t v0 = ((int64_t)__builtin_amdgcn_readfirstlane(D[13]) << 32) | (uint32_t)__builtin_amdgcn_readfirstlane(D[12]);
        const int len = __builtin_amdgcn_readfirstlane(D[14]);
        const int nA = __builtin_amdgcn_readfirstlane(D[15]), nB = __builtin_amdgcn_readfirstlane(D[16]);
        const int cb0 = chunk * P.CH;
        const int nb = min(P.CH, nblk_list - cb0);
        const int cvec0 = cb0 * BLOCK_VECS;          // first vector of the chunk inside the list
        const int cvecs = min(len - cvec0, nb * BLOCK_VECS);
        // the wave's first block is requested before the tables are touched
        constexpr int64_t BLK_BYTES = BLOCK_VECS * MPAD;
        const uint8_t* base = P.codes + (b0 + cb0) * BLK_BYTES;
        uint4 cur_w[MPAD / 16], nxt_w[MPAD / 16];
        int b = wave;
        // (every load of the stream is unconditional, with the block number clamped into the chunk: a
        // conditional prefetch makes the compiler wait for ALL outstanding loads before each use)
        auto first_load = [&]() { load_block<MPAD>(cur_w, base + (int64_t)min(b, nb - 1) * BLK_BYTES, lane); };

        // ---- tables into LDS (rows of 128 B into rows of 256 B), thresholds
        if (P.lut8sw) {
            const uint4* srcA = reinterpret_cast<const uint4*>(P.lut8sw + (int64_t)pairA * LUT_BYTES);
            const uint4* srcB = reinterpret_cast<const uint4*>(P.lut8sw + (int64_t)(pairB >= 0 ? pairB : pairA) * LUT_BYTES);
            copy_table(srcA, pairB >= 0 ? srcB : nullptr, lut, first_load);
            loadedA = loadedB = -1;
        } else {
            // base table of the query (kept while consecutive tasks use the same query in this slot),
            // then the pair's patches; flagged queries are evaluated entry by entry
            const bool baseA = nA <= AMB_MAX && loadedA != qA;
            const bool baseB = pairB >= 0 && nB <= AMB_MAX && loadedB != qB;
            // Patches are written by the wave that copies the 16-byte piece they fall into, so program
            // order inside the wave puts them after the copy and no workgroup barrier is needed in between.
            // Piece of LDS offset a: row a >> 8, column (a & 127) >> 4; copied by thread (piece & 511).
            // (the arrays always hold AMB_MAX entries, so the first 64 can be read unconditionally)
            const bool useA = nA <= AMB_MAX, useB = pairB >= 0 && nB <= AMB_MAX;
            const uint32_t a0 = P.T.amb_addr[(int64_t)qA * AMB_MAX + lane];
            const uint32_t v0 = P.T.patch_val[(int64_t)pairA * AMB_MAX + lane];
            const uint32_t a1 = P.T.amb_addr[(int64_t)(pairB >= 0 ? qB : qA) * AMB_MAX + lane];
            const uint32_t v1 = P.T.patch_val[(int64_t)(pairB >= 0 ? pairB : pairA) * AMB_MAX + lane];
            copy_table(baseA ? reinterpret_cast<const uint4*>(P.T.lut_base + (int64_t)qA * LUT_BYTES) : nullptr,
                       baseB ? reinterpret_cast<const uint4*>(P.T.lut_base + (int64_t)qB * LUT_BYTES) : nullptr, lut, first_load);
            if (nA > AMB_MAX) eval_table(P, pairA, qA, lut);
            if (pairB >= 0 && nB > AMB_MAX) eval_table(P, pairB, qB, lut + 128);
            auto owner = [](uint32_t a) { return ((((a >> 8) << 3) | ((a & 127u) >> 4)) & 511u) >> 6; };
            if (useA && lane < nA && owner(a0) == (uint32_t)wave) lut[a0] = (uint8_t)v0;
            if (useB && lane < nB && owner(a1) == (uint32_t)wave) lut[128 + a1] = (uint8_t)v1;
            if (useA)
                for (int i = 64 + lane; i < nA; i += 64) {
                    const uint32_t a = P.T.amb_addr[(int64_t)qA * AMB_MAX + i];
                    if (owner(a) == (uint32_t)wave) lut[a] = P.T.patch_val[(int64_t)pairA * AMB_MAX + i];
                }
            if (useB)
                for (int i = 64 + lane; i < nB; i += 64) {
                    const uint32_t a = P.T.amb_addr[(int64_t)qB * AMB_MAX + i];
                    if (owner(a) == (uint32_t)wave) lut[128 + a] = P.T.patch_val[(int64_t)pairB * AMB_MAX + i];
                }
            loadedA = nA <= AMB_MAX ? qA : -1;
            if (pairB >= 0) loadedB = nB <= AMB_MAX ? qB : -1;
        }
        if (threadIdx.x < 2) {
            const int pr = threadIdx.x == 0 ? pairA : pairB;
            int32_t t0 = 0;
            if (pr >= 0) {
                const int32_t g = __hip_atomic_load(P.tauq + (threadIdx.x == 0 ? qA : qB), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const int64_t t = (int64_t)g - (threadIdx.x == 0 ? biasA : biasB);
                t0 = t <= 0 ? 0 : (t > 0x7fffffff ? 0x7fffffff : (int32_t)t);
            }
            sh[2 + threadIdx.x] = t0;
            if (threadIdx.x == 0) { sh[4] = SCAN_WAVES; sh[5] = 0; }   // next unclaimed block of the chunk; finisher ticket
        }
        __syncthreads();

        // ---- stream the chunk: wave w takes blocks w, w+8, ...
        uint32_t* bufA = cand + (wave * 2 + 0) * CAPW;
        uint32_t* bufB = cand + (wave * 2 + 1) * CAPW;
        int cntA = 0, cntB = 0;
        uint32_t thrA = (uint32_t)sh[2], thrB = (uint32_t)sh[3];
        // one wave claims and decodes the next task while its first loads are in flight
        auto process = [&](const uint4 (&w)[MPAD / 16], int blk) {
            const uint32_t pos = (uint32_t)(blk * BLOCK_VECS + lane);
            const bool valid = (int)pos < cvecs;
            uint32_t sa, sb;
            if (pairB >= 0) {
                block_sums<MPAD, 2>(w, off, sel0, sel1, sel2, sel3, sa, sb);
                const uint32_t ta = (uint32_t)sh[2], tb = (uint32_t)sh[3];
                if (ta > thrA) thrA = ta;
                if (tb > thrB) thrB = tb;
                offer(valid, sa, pos, bufA, cntA, thrA, sh + 2, k, lane);
                offer(valid, sb, pos, bufB, cntB, thrB, sh + 3, k, lane);
            } else {
                block_sums<MPAD, 1>(w, off, sel0, sel1, sel2, sel3, sa, sb);
                const uint32_t ta = (uint32_t)sh[2];
                if (ta > thrA) thrA = ta;
                offer(valid, sa, pos, bufA, cntA, thrA, sh + 2, k, lane);
            }
        };
        // blocks beyond each wave's first are claimed from an LDS counter: a wave that was held up
        // (the one that fetched the next task, one that pruned) simply takes fewer
        auto claim = [&]() {
            int v = 0;
            if (lane == 0) v = atomicAdd(&sh[4], 1);
            return __builtin_amdgcn_readfirstlane(v);
        };
        int bn = claim();
        load_block<MPAD>(nxt_w, base + (int64_t)min(bn, nb - 1) * BLK_BYTES, lane);
        while (b < nb) {                       // ping-pong between the two register sets
            process(cur_w, b);
            b = claim();
            load_block<MPAD>(cur_w, base + (int64_t)min(b, nb - 1) * BLK_BYTES, lane);
            if (bn >= nb) break;               // claims are monotonic: nothing newer can be valid either
            process(nxt_w, bn);
            bn = claim();
            load_block<MPAD>(nxt_w, base + (int64_t)min(bn, nb - 1) * BLK_BYTES, lane);
        }
        // The first wave to run out of blocks claims and decodes the next task while the others finish
        // (claiming it at the start of the chunk instead costs ~5 % of the kernel: the claiming wave's
        // scalar-load chain then delays its share of the stream).
        {
            int ticket = 0;
            if (lane == 0) ticket = atomicAdd(&sh[5], 1);
            if (__builtin_amdgcn_readfirstlane(ticket) == 0) fetch_task(P, ntasks, desc + (cur ^ 1) * DESC_INTS, lane);
        }
        // ---- task result: every wave trims its buffers to k, then one wave per pair merges
        if (cntA > k) wave_prune(bufA, cntA, k, lane);
        if (cntB > k) wave_prune(bufB, cntB, k, lane);
        if (lane == 0) { sh[8 + wave * 2] = cntA; sh[8 + wave * 2 + 1] = cntB; }
        __syncthreads();
        if (wave < 2 && (wave == 0 || pairB >= 0)) {
            const int pr = wave == 0 ? pairA : pairB;
            const int bias = wave == 0 ? biasA : biasB;
            uint32_t r[2 * SCAN_WAVES];
            int total = 0;
#pragma unroll
            for (int w = 0; w < SCAN_WAVES; ++w) {
                const int c = sh[8 + w * 2 + wave];
                const uint32_t* bw = cand + (w * 2 + wave) * CAPW;
                r[2 * w] = lane < c ? bw[lane] : 0u;
                r[2 * w + 1] = lane + 64 < c ? bw[lane + 64] : 0u;
                total += c;
            }
            uint32_t kth = 1u;
            if (total >= k) kth = select_kth<2 * SCAN_WAVES>(r, k);
            const int64_t slot = (int64_t)pr * P.maxchunks + chunk;
            int32_t* oI = P.part_I + slot * k;
            int64_t* oid = P.part_id + slot * k;
            const int64_t* idp = P.ids + v0 + cvec0;
            int base_o = 0;
#pragma unroll
            for (int i = 0; i < 2 * SCAN_WAVES; ++i) {
                const bool keep = r[i] >= kth && r[i] != 0u;
                const uint64_t mask = __ballot(keep);
                if (keep) {
                    const int o = base_o + lane_rank(mask);
                    oI[o] = bias + (int32_t)(r[i] >> 16);
                    oid[o] = idp[0xFFFFu - (r[i] & 0xFFFFu)];
                }
                base_o += __popcll(mask);
            }
            if (lane == 0) {
                P.part_cnt[slot] = base_o;
                // k entries reach the k-th key's score: a valid lower bound of the query's k-th best
                if (total >= k) atomicMax(P.tauq + (wave == 0 ? qA : qB), bias + (int32_t)(kth >> 16));
            }
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------ task bookkeeping kernels
// The (query, list) pairs are grouped by list without ever touching all nlist lists: the first
// pair that reaches a list registers it in `touched`; prefix sums run over the touched lists only
// (at most one per pair), so a single query costs a few hundred entries, not nlist.
// ctrl[0] task counter, ctrl[1] number of tasks, ctrl[2] number of touched lists.
__global__ void scan_init_kernel(int32_t* __restrict__ list_cnt2, int64_t n2, int32_t* __restrict__ tauq, int64_t nq,
                                 int32_t* __restrict__ ctrl, int64_t* __restrict__ counters) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t j = i; j < n2; j += stride) list_cnt2[j] = 0;     // list_cnt and cursor
    for (int64_t j = i; j < nq; j += stride) tauq[j] = INT32_MIN;
    if (i < 4) ctrl[i] = 0;
    if (i == 0) { counters[1] = 0; counters[2] = 0; }
}

__global__ void __launch_bounds__(256) count_pairs_kernel(const int32_t* __restrict__ probes, int64_t npairs, int32_t* __restrict__ list_cnt,
                                                          int32_t* __restrict__ touched, int32_t* __restrict__ ctrl) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int lane = threadIdx.x & 63;
    int l = -1;
    bool first = false;
    if (i < npairs) {
        l = probes[i];
        first = atomicAdd(&list_cnt[l], 1) == 0;
    }
    const uint64_t m = __ballot(first);         // one slot reservation per wave, not per list
    if (m) {
        int base = 0;
        if (lane == __builtin_ctzll(m)) base = atomicAdd(&ctrl[2], __popcll(m));
        base = __builtin_amdgcn_readlane(base, __builtin_ctzll(m));
        if (first) touched[base + __popcll(m & ((1ull << lane) - 1ull))] = l;
    }
}

// Per touched list: its pair count and task count (any number of workgroups), and where it sits.
__global__ void __launch_bounds__(256) touched_values_kernel(const int32_t* __restrict__ touched, const int32_t* __restrict__ list_cnt,
                                                             const int64_t* __restrict__ blk_off, const int64_t* __restrict__ list_off,
                                                             int CH, int m, int64_t max_n, const int32_t* __restrict__ ctrl,
                                                             int32_t* __restrict__ list_slot, int32_t* __restrict__ vp,
                                                             int32_t* __restrict__ vt, int64_t* __restrict__ counters) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    unsigned long long streamed = 0, algo = 0;
    if (i < max_n && i < ctrl[2]) {
        const int l = touched[i];
        const int c = list_cnt[l];
        const int nblk = (int)(blk_off[l + 1] - blk_off[l]);
        list_slot[l] = (int)i;
        vp[i] = c;
        vt[i] = ((c + 1) >> 1) * ((nblk + CH - 1) / CH);
        streamed = (unsigned long long)((c + 1) >> 1) * nblk * (BLOCK_VECS * m);
        algo = (unsigned long long)c * (unsigned long long)(list_off[l + 1] - list_off[l]) * m;
    }
    for (int o = 32; o; o >>= 1) { streamed += __shfl_xor(streamed, o); algo += __shfl_xor(algo, o); }
    if ((threadIdx.x & 63) == 0 && (streamed | algo)) {
        atomicAdd(reinterpret_cast<unsigned long long*>(counters + 1), streamed);
        atomicAdd(reinterpret_cast<unsigned long long*>(counters + 2), algo);
    }
}

// Exclusive prefix sums (in place) of the per-list pair and task counts: one workgroup, coalesced.
__global__ void __launch_bounds__(1024) touched_scan_kernel(int32_t* __restrict__ vp, int32_t* __restrict__ vt,
                                                            int32_t* __restrict__ ctrl, int64_t* __restrict__ counters) {
    __shared__ int s_wp[16], s_wt[16];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int n = ctrl[2];
    int carry_p = 0, carry_t = 0;
    for (int base = 0; base < n; base += 1024) {
        const int i = base + t;
        const int p = i < n ? vp[i] : 0, q = i < n ? vt[i] : 0;
        int ip = p, it = q;                        // inclusive scan across the wave
        for (int o = 1; o < 64; o <<= 1) {
            const int a = __shfl_up(ip, o), b = __shfl_up(it, o);
            if (lane >= o) { ip += a; it += b; }
        }
        __syncthreads();                           // previous tile's wave totals consumed
        if (lane == 63) { s_wp[wave] = ip; s_wt[wave] = it; }
        __syncthreads();
        int wp = 0, wt = 0, tot_p = 0, tot_t = 0;
        for (int w = 0; w < 16; ++w) {
            if (w < wave) { wp += s_wp[w]; wt += s_wt[w]; }
            tot_p += s_wp[w]; tot_t += s_wt[w];
        }
        if (i < n) { vp[i] = carry_p + wp + ip - p; vt[i] = carry_t + wt + it - q; }
        carry_p += tot_p; carry_t += tot_t;
    }
    if (t == 0) {
        vp[n] = carry_p; vt[n] = carry_t;
        ctrl[0] = 0; ctrl[1] = carry_t;
        counters[0] = carry_t;
    }
}

__global__ void scatter_pairs_kernel(const int32_t* __restrict__ probes, int64_t npairs, const int32_t* __restrict__ list_slot,
                                     const int32_t* __restrict__ pair_off, int32_t* __restrict__ cursor,
                                     int32_t* __restrict__ pair_sorted) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= npairs) return;
    const int l = probes[i];
    pair_sorted[pair_off[list_slot[l]] + atomicAdd(&cursor[l], 1)] = (int32_t)i;
}

// One record per task: binary search of the touched list, then chunk / pair group.
__global__ void __launch_bounds__(256) task_table_kernel(const int32_t* __restrict__ task_off, const int32_t* __restrict__ pair_off,
                                                         const int32_t* __restrict__ pair_sorted, const int32_t* __restrict__ touched,
                                                         const int32_t* __restrict__ ctrl, int64_t max_tasks, int4* __restrict__ table) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= max_tasks || t >= ctrl[1]) return;
    int lo = 0, hi = ctrl[2];   // largest slot with task_off[slot] <= t
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (task_off[mid] <= (int)t) lo = mid; else hi = mid;
    }
    const int rem = (int)t - task_off[lo];
    const int npl = pair_off[lo + 1] - pair_off[lo];
    const int ngroups = (npl + 1) >> 1;
    const int chunk = rem / ngroups, grp = rem - chunk * ngroups;   // groups of one chunk are consecutive tasks
    const int pa = pair_sorted[pair_off[lo] + 2 * grp];
    const int pb = (2 * grp + 1 < npl) ? pair_sorted[pair_off[lo] + 2 * grp + 1] : -1;
    table[t] = make_int4(touched[lo], chunk, pa, pb);
}

// ------------------------------------------------------------------ per-query merge of the task results
constexpr int MERGE_THREADS = 256;
constexpr int MERGE_CAP = 2048;

__device__ __forceinline__ bool entry_before(int32_t ia, int64_t da, int32_t ib, int64_t db) {
    return ia > ib || (ia == ib && da < db);
}

// Sort sI/sId[0..n2) (n2 a power of two) by (I desc, id asc).
__device__ void bitonic_sort(int32_t* sI, int64_t* sId, int n2) {
    for (int size = 2; size <= n2; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            for (int t = threadIdx.x; t < n2 / 2; t += MERGE_THREADS) {
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

__global__ void __launch_bounds__(MERGE_THREADS) merge_kernel(const ScanParams P, const float* __restrict__ delta,
                                                              int64_t* __restrict__ out_ids, float* __restrict__ out_scores,
                                                              int32_t* __restrict__ out_iscores) {
    __shared__ int32_t sI[MERGE_CAP];
    __shared__ int64_t sId[MERGE_CAP];
    __shared__ int s_cnt;
    const int q = blockIdx.x, k = P.k;
    int32_t tau = P.tauq[q];   // k candidates of this query reach tau: nothing below can be in the result
    // Slots = (probe, chunk) pairs that exist: chunk counts per probe are prefix-summed in LDS
    // (s_pre), then one thread per slot reads the slot's count and its few surviving entries.
    __shared__ int s_pre[2049];            // nprobe <= 2048 (enforced by the selection stage / argument check)
    for (int p = threadIdx.x; p < P.nprobe; p += MERGE_THREADS) {
        const int l = P.probes[q * P.nprobe + p];
        const int nblk = (int)(P.blk_off[l + 1] - P.blk_off[l]);
        s_pre[p + 1] = (nblk + P.CH - 1) / P.CH;
    }
    if (threadIdx.x == 0) s_pre[0] = 0;
    __syncthreads();
    if (threadIdx.x == 0)
        for (int p = 0; p < P.nprobe; ++p) s_pre[p + 1] += s_pre[p];
    __syncthreads();
    const int nslots = s_pre[P.nprobe];
    auto gather = [&](int s0, int s1, int base_fill) {
        if (threadIdx.x == 0) s_cnt = base_fill;
        __syncthreads();
        for (int s = s0 + threadIdx.x; s < s1; s += MERGE_THREADS) {
            int lo = 0, hi = P.nprobe;     // probe p with s_pre[p] <= s < s_pre[p + 1]
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (s_pre[mid] <= s) lo = mid; else hi = mid;
            }
            const int64_t gs = ((int64_t)q * P.nprobe + lo) * P.maxchunks + (s - s_pre[lo]);
            const int n = P.part_cnt[gs];
            for (int r = 0; r < n; ++r) {
                const int32_t I = P.part_I[gs * k + r];
                if (I >= tau) {
                    const int o = atomicAdd(&s_cnt, 1);
                    if (o < MERGE_CAP) { sI[o] = I; sId[o] = P.part_id[gs * k + r]; }
                }
            }
        }
        __syncthreads();
        return s_cnt;
    };
    auto sort_keep_k = [&](int have) {
        int n2 = 1;
        while (n2 < have) n2 <<= 1;
        for (int i = have + threadIdx.x; i < n2; i += MERGE_THREADS) { sI[i] = INT32_MIN; sId[i] = INT64_MAX; }
        if (n2 > 1) bitonic_sort(sI, sId, n2); else __syncthreads();
        return min(have, k);
    };
    // optimistic: everything that passes tau fits the buffer (the usual case by far)
    int have = gather(0, nslots, 0);
    int fill;
    if (have <= MERGE_CAP) {
        fill = sort_keep_k(have);
    } else {
        // rounds small enough that even if every entry passes the buffer cannot overflow
        const int per_round = (MERGE_CAP - k) / k;
        fill = 0;
        for (int s0 = 0; s0 < nslots; s0 += per_round) {
            __syncthreads();
            have = gather(s0, min(nslots, s0 + per_round), fill);
            fill = sort_keep_k(have);
            if (fill == k && sI[k - 1] > tau) tau = sI[k - 1];
        }
    }
    __syncthreads();
    for (int r = threadIdx.x; r < k; r += MERGE_THREADS) {
        const bool ok = r < fill;
        const int32_t I = ok ? sI[r] : INT32_MIN;
        out_ids[(int64_t)q * k + r] = ok ? sId[r] : -1;
        if (out_iscores) out_iscores[(int64_t)q * k + r] = I;
        if (out_scores) out_scores[(int64_t)q * k + r] = ok ? (float)I * (delta ? delta[q] : 1.0f) : -INFINITY;
    }
}

// ------------------------------------------------------------------ host side
template <int MPAD>
static int launch_scan_kernel(const ScanParams& P, int grid, hipStream_t st) {
    static bool attr_done = false;
    if (!attr_done) {
        RAGO_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(scan_kernel<MPAD>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, SCAN_LDS));
        attr_done = true;
    }
    scan_kernel<MPAD><<<grid, SCAN_THREADS, SCAN_LDS, st>>>(P);
    RAGO_HIP(hipGetLastError());
    return RAGO_OK;
}

int launch_scan(rago_index* idx, const int32_t* probes, const uint8_t* lut8sw, const int32_t* bias, const LutTables* tables,
                const float* delta, int64_t nq, int nprobe, int k, int64_t* out_ids, float* out_scores, int32_t* out_iscores,
                hipStream_t st, hipEvent_t* ev) {
    Workspace& ws = idx->ws;
    const int64_t npairs = nq * nprobe;
    const int nlist = idx->nlist;
    // chunk length: aim at ~2048 tasks, between 16 and 256 blocks
    const double avgblk = (double)idx->total_blocks / nlist;
    // (pairs of one list share a pass when several queries are in the batch: ~1.5 pairs per task)
    const double share = nq > 1 ? 1.5 : 1.0;
    int CH = 16;
    while (CH < 256 && (double)npairs * avgblk / (share * CH) > 2048.0) CH <<= 1;
    const int64_t maxblk = (idx->max_list_len + BLOCK_VECS - 1) / BLOCK_VECS;
    const int maxchunks = (int)std::max<int64_t>(1, (maxblk + CH - 1) / CH);
    if ((double)npairs * maxchunks * k > 4.0e9) return fail(RAGO_UNSUPPORTED, "nq * nprobe * chunks * k too large for the workspace");
    int rc;
    if ((rc = ws.list_cnt.reserve((size_t)(3 * nlist + 8) * 4))) return rc;   // list_cnt, cursor, list_slot, ctrl
    if ((rc = ws.pair_off.reserve((size_t)(npairs + 2) * 4))) return rc;      // per touched list
    if ((rc = ws.task_off.reserve((size_t)(npairs + 2) * 4))) return rc;
    if ((rc = ws.touched.reserve((size_t)(npairs + 2) * 4))) return rc;
    if ((rc = ws.pair_sorted.reserve((size_t)npairs * 4))) return rc;
    if ((rc = ws.tauq.reserve((size_t)nq * 4))) return rc;
    if ((rc = ws.part_I.reserve((size_t)npairs * maxchunks * k * 4))) return rc;
    if ((rc = ws.part_id.reserve((size_t)npairs * maxchunks * k * 8))) return rc;
    if ((rc = ws.part_cnt.reserve((size_t)npairs * maxchunks * 4))) return rc;
    if ((rc = ws.counters.reserve(64))) return rc;
    const int64_t max_tasks = npairs * maxchunks;
    if ((rc = ws.task_table.reserve((size_t)max_tasks * 16))) return rc;

    int32_t* list_cnt = ws.list_cnt.as<int32_t>();
    int32_t* cursor = list_cnt + nlist;
    int32_t* list_slot = list_cnt + 2 * nlist;
    int32_t* ctrl = list_cnt + 3 * nlist;
    ScanParams P;
    P.codes = idx->codes_blk; P.blk_off = idx->blk_off; P.list_off = idx->list_off; P.ids = idx->ids;
    P.probes = probes; P.lut8sw = lut8sw; P.bias = bias; P.m = idx->m;
    if (tables) P.T = *tables; else P.T = LutTables{};
    P.pair_sorted = ws.pair_sorted.as<int32_t>();
    P.task_table = ws.task_table.as<int4>();
    P.ctrl = ctrl;
    P.tauq = ws.tauq.as<int32_t>(); P.part_I = ws.part_I.as<int32_t>(); P.part_id = ws.part_id.as<int64_t>();
    P.part_cnt = ws.part_cnt.as<int32_t>();
    P.nlist = nlist; P.nprobe = nprobe; P.k = k; P.CH = CH; P.maxchunks = maxchunks;

    const unsigned pg = (unsigned)((npairs + 255) / 256);
    scan_init_kernel<<<(unsigned)std::min<int64_t>(256, (2 * nlist + nq + 255) / 256 + 1), 256, 0, st>>>(list_cnt, 2 * (int64_t)nlist, P.tauq, nq, ctrl, ws.counters.as<int64_t>());
    count_pairs_kernel<<<pg, 256, 0, st>>>(probes, npairs, list_cnt, ws.touched.as<int32_t>(), ctrl);
    touched_values_kernel<<<pg, 256, 0, st>>>(ws.touched.as<int32_t>(), list_cnt, idx->blk_off, idx->list_off, CH, idx->m, npairs, ctrl,
                                              list_slot, ws.pair_off.as<int32_t>(), ws.task_off.as<int32_t>(), ws.counters.as<int64_t>());
    touched_scan_kernel<<<1, 1024, 0, st>>>(ws.pair_off.as<int32_t>(), ws.task_off.as<int32_t>(), ctrl, ws.counters.as<int64_t>());
    scatter_pairs_kernel<<<pg, 256, 0, st>>>(probes, npairs, list_slot, ws.pair_off.as<int32_t>(), cursor, ws.pair_sorted.as<int32_t>());
    task_table_kernel<<<(unsigned)((max_tasks + 255) / 256), 256, 0, st>>>(ws.task_off.as<int32_t>(), ws.pair_off.as<int32_t>(),
                                                                           P.pair_sorted, ws.touched.as<int32_t>(), ctrl, max_tasks,
                                                                           ws.task_table.as<int4>());
    RAGO_HIP(hipGetLastError());

    static int n_cu = 0;
    if (!n_cu) {
        hipDeviceProp_t pr;
        RAGO_HIP(hipGetDeviceProperties(&pr, idx->device));
        n_cu = pr.multiProcessorCount;
    }
    const int grid = 2 * n_cu;
    if (ev) RAGO_HIP(hipEventRecord(ev[4], st));
    switch (idx->m) {
        case 16: rc = launch_scan_kernel<16>(P, grid, st); break;
        case 32: rc = launch_scan_kernel<32>(P, grid, st); break;
        case 64: rc = launch_scan_kernel<64>(P, grid, st); break;
        case 96: rc = launch_scan_kernel<96>(P, grid, st); break;
        case 128: rc = launch_scan_kernel<128>(P, grid, st); break;
        default: return fail(RAGO_UNSUPPORTED, "code width");
    }
    if (rc) return rc;
    if (ev) RAGO_HIP(hipEventRecord(ev[5], st));
    merge_kernel<<<(unsigned)nq, MERGE_THREADS, 0, st>>>(P, delta, out_ids, out_scores, out_iscores);
    RAGO_HIP(hipGetLastError());
    if (ev) RAGO_HIP(hipEventRecord(ev[6], st));
    return RAGO_OK;
}

}  // namespace rago

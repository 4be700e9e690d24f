// The scan kernel for short lists and small batches: one WAVE scans one (query, list, chunk) item
// from start to end, so the streaming loop has no workgroup barrier, no merge across waves and no
// per-task fixed work.  Same results as the kernels of scan.hip and scan_narrow.hip, which group
// the pairs by list; this one groups them by QUERY:
//
//  * a workgroup (8 waves, two workgroups per CU) attaches to a query: it brings that query's
//    8-bit base table into LDS once, then its waves claim items of the query (in batches, from a
//    per-query counter in HBM) and work through them independently (the item after the current one
//    is claimed and resolved while the current one streams).  Any number of workgroups may be
//    attached to one query; a workgroup whose query has run out of items attaches to the query
//    with the most items left per attached workgroup, and leaves when no query has any.  With one
//    query all workgroups share it; with thousands each workgroup takes whole queries.
//  * under the inner product the tables of a query's pairs differ from its base table only in the
//    few entries whose rounding depends on the pair (lut.hip).  Those entries are not patched into
//    the shared table: a wave turns the pair's patches into corrections (sub-quantiser, code,
//    +-difference), sums with the base table, and applies the corrections, from the code bytes it
//    holds in registers, only to blocks in which some vector comes within the corrections' reach
//    of the threshold.
//  * per-pair tables (Euclidean metric, caller-supplied tables, queries whose tables are too flat
//    for the base + patch form): the workgroup claims whole pairs, installs the pair's table
//    between two barriers, and its waves share out that pair's items.
//  * LDS table layout (32 KiB): byte address = code * 128 + slot * 4 + plane.  `slot` selects the
//    bank, so a sub-table lives in ONE bank; the 32 lanes of a half-wave always work on 32
//    different slots (layout.hip), so every ds_read_u8 is conflict-free whatever the codes are.
//    One v_perm_b32 places two code bytes next to the lane's slot * 8 bytes; a bit-field extract
//    and a shift by one bit turn the halves into addresses; the plane rides in the immediate.
//  * an item leaves its best <= k entries that still reach the query's bound in its own slot of
//    the result arrays (slot = number of the item inside its query: nothing to synchronise); the
//    bound on the k-th best score is shared through LDS and a word in HBM; the final merge runs
//    in two stages when a query has thousands of items (slices of the slots, then the slices'
//    results).
//  * the k-th best score of a single item is a weak bound when lists are short and k is large (the
//    100th of 600 vectors, where the query's answer is the 100th of 40 000).  Every workgroup
//    therefore counts the candidates of all its items of the query in a histogram of their
//    scores above its first bound (LDS): k candidates at or above a bin edge make that edge a
//    bound.  With it an item leaves a handful of entries instead of k.
//  * a single address in HBM takes only a few tens of millions of atomic operations per second,
//    so nothing here issues one per item: a workgroup claims items of its query sixteen at a time
//    (its waves share them out through LDS), the first sixteen come with the attachment, and the
//    bound goes to HBM only when the workgroup's own copy improved.
#include <algorithm>

#include "scan_common.h"
#include "scan_plan.h"

namespace rago {
namespace wavescan {

constexpr int WAVES = 8;
constexpr int THREADS = WAVES * 64;
constexpr int LUT_LDS = 32768;
constexpr int CORR_CAP = AMB_MAX;
constexpr int BATCH = WAVE_BATCH;               // items a workgroup claims at a time (two per wave)
static_assert(WAVE_BATCH == 2 * WAVES, "two items per wave");
constexpr int PRE_CAP = 2048 + 1;               // first item of every pair of the query (nprobe <= 2048) and the total
// LDS: table | key buffers [wave][CAPW] | corrections [wave][CORR_CAP] | ambiguous entries of the query: address u16,
// base value u8 | first item of each pair | scalars | histogram of candidate scores
constexpr int OFF_CAND = LUT_LDS;
constexpr int OFF_CORR = OFF_CAND + WAVES * CAPW * 4;
constexpr int OFF_AMB = OFF_CORR + WAVES * CORR_CAP * 4;
constexpr int OFF_AMBV = OFF_AMB + AMB_MAX * 2;
constexpr int OFF_PRE = OFF_AMBV + AMB_MAX;
constexpr int OFF_SH = OFF_PRE + ((PRE_CAP * 4 + 15) & ~15);
constexpr int HIST_BINS = 1024, HIST_SHIFT = 2;  // scores of the workgroup's candidates above its first bound, 4 to a bin
constexpr int OFF_HIST = OFF_SH + 64 * 4;
constexpr int SCAN_LDS = OFF_HIST + HIST_BINS * 4;

#define RAGO_WSEL_A 0x05010400u   // {code1, slot1*8, code0, slot0*8}
#define RAGO_WSEL_B 0x07030602u   // {code3, slot3*8, code2, slot2*8}

// 16 look-ups (one dwordx4 of codes, all in plane PL) added into `sum`.  Hand-scheduled like the
// other scan kernels: the asm statement drains its own LDS reads before it ends.
template <int PL>
__device__ __forceinline__ void lookup16(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t w3, uint32_t o0, uint32_t o1,
                                         uint32_t o2, uint32_t o3, uint32_t sa, uint32_t sb, uint32_t& sum) {
    uint32_t t0, t1, t2, t3, t4, t5, t6, t7, t8, t9, t10, t11, t12, t13, t14, t15;
    asm volatile(
        "v_perm_b32 %[t1], %[w0], %[o0], %[sa]\n v_perm_b32 %[t3], %[w0], %[o0], %[sb]\n"
        "v_bfe_u32 %[t0], %[t1], 1, 15\n v_lshrrev_b32 %[t1], 17, %[t1]\n"
        "v_bfe_u32 %[t2], %[t3], 1, 15\n v_lshrrev_b32 %[t3], 17, %[t3]\n"
        "ds_read_u8 %[t0], %[t0] offset:%[pl]\n ds_read_u8 %[t1], %[t1] offset:%[pl]\n"
        "ds_read_u8 %[t2], %[t2] offset:%[pl]\n ds_read_u8 %[t3], %[t3] offset:%[pl]\n"
        "v_perm_b32 %[t5], %[w1], %[o1], %[sa]\n v_perm_b32 %[t7], %[w1], %[o1], %[sb]\n"
        "v_bfe_u32 %[t4], %[t5], 1, 15\n v_lshrrev_b32 %[t5], 17, %[t5]\n"
        "v_bfe_u32 %[t6], %[t7], 1, 15\n v_lshrrev_b32 %[t7], 17, %[t7]\n"
        "ds_read_u8 %[t4], %[t4] offset:%[pl]\n ds_read_u8 %[t5], %[t5] offset:%[pl]\n"
        "ds_read_u8 %[t6], %[t6] offset:%[pl]\n ds_read_u8 %[t7], %[t7] offset:%[pl]\n"
        "v_perm_b32 %[t9], %[w2], %[o2], %[sa]\n v_perm_b32 %[t11], %[w2], %[o2], %[sb]\n"
        "v_bfe_u32 %[t8], %[t9], 1, 15\n v_lshrrev_b32 %[t9], 17, %[t9]\n"
        "v_bfe_u32 %[t10], %[t11], 1, 15\n v_lshrrev_b32 %[t11], 17, %[t11]\n"
        "ds_read_u8 %[t8], %[t8] offset:%[pl]\n ds_read_u8 %[t9], %[t9] offset:%[pl]\n"
        "ds_read_u8 %[t10], %[t10] offset:%[pl]\n ds_read_u8 %[t11], %[t11] offset:%[pl]\n"
        "v_perm_b32 %[t13], %[w3], %[o3], %[sa]\n v_perm_b32 %[t15], %[w3], %[o3], %[sb]\n"
        "v_bfe_u32 %[t12], %[t13], 1, 15\n v_lshrrev_b32 %[t13], 17, %[t13]\n"
        "v_bfe_u32 %[t14], %[t15], 1, 15\n v_lshrrev_b32 %[t15], 17, %[t15]\n"
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
          [sa] "s"(sa), [sb] "s"(sb), [pl] "n"(PL)
        : "memory");
}

template <int MPAD, int I>
__device__ __forceinline__ void block_sum_chunk(const uint4 (&w)[MPAD / 16], const uint32_t (&off)[(MPAD < 32 ? MPAD : 32) / 4],
                                                uint32_t sa, uint32_t sb, uint32_t& sum) {
    constexpr int S = MPAD < 32 ? MPAD : 32;
    constexpr int PL = (I * 16) / S;               // plane of this dwordx4
    constexpr int G = ((I * 16) % S) / 4;          // first of its four step groups
    lookup16<PL>(w[I].x, w[I].y, w[I].z, w[I].w, off[G], off[G + 1], off[G + 2], off[G + 3], sa, sb, sum);
    if constexpr (I + 1 < MPAD / 16) block_sum_chunk<MPAD, I + 1>(w, off, sa, sb, sum);
}

// The code byte of sub-quantiser j (wave-uniform) in the lane's block registers.  Position t of a lane's
// byte string holds sub-quantiser plane(t) * 32 + ((step(t) + lane) mod S), so j sits at step (j - lane) mod S
// of plane j / 32: a lane-dependent dword of that plane's S / 4, picked with a binary tree of selects.
template <int MPAD>
__device__ __forceinline__ uint32_t code_of(const uint4 (&w)[MPAD / 16], int j, int lane) {
    constexpr int S = MPAD < 32 ? MPAD : 32;
    const int step = ((j & (S - 1)) - lane) & (S - 1);
    const int D = step >> 2;
    // (plain scalars picked by value: references to the elements of `w` would force the block registers into
    // scratch memory)
    uint32_t a0 = w[0].x, a1 = w[0].y, a2 = w[0].z, a3 = w[0].w, a4 = 0, a5 = 0, a6 = 0, a7 = 0;
    if constexpr (S == 32) {
        a4 = w[1].x; a5 = w[1].y; a6 = w[1].z; a7 = w[1].w;
        const int plane = j >> 5;          // wave-uniform; selects, not branches (branches get merged into an indexed access)
        if constexpr (MPAD >= 64) {
            const bool p = plane == 1;
            a0 = p ? w[2].x : a0; a1 = p ? w[2].y : a1; a2 = p ? w[2].z : a2; a3 = p ? w[2].w : a3;
            a4 = p ? w[3].x : a4; a5 = p ? w[3].y : a5; a6 = p ? w[3].z : a6; a7 = p ? w[3].w : a7;
        }
        if constexpr (MPAD >= 96) {
            const bool p = plane == 2;
            a0 = p ? w[4].x : a0; a1 = p ? w[4].y : a1; a2 = p ? w[4].z : a2; a3 = p ? w[4].w : a3;
            a4 = p ? w[5].x : a4; a5 = p ? w[5].y : a5; a6 = p ? w[5].z : a6; a7 = p ? w[5].w : a7;
        }
        if constexpr (MPAD >= 128) {
            const bool p = plane == 3;
            a0 = p ? w[6].x : a0; a1 = p ? w[6].y : a1; a2 = p ? w[6].z : a2; a3 = p ? w[6].w : a3;
            a4 = p ? w[7].x : a4; a5 = p ? w[7].y : a5; a6 = p ? w[7].z : a6; a7 = p ? w[7].w : a7;
        }
    }
    const uint32_t b0 = (D & 1) ? a1 : a0, b1 = (D & 1) ? a3 : a2, b2 = (D & 1) ? a5 : a4, b3 = (D & 1) ? a7 : a6;
    const uint32_t c0 = (D & 2) ? b1 : b0, c1 = (D & 2) ? b3 : b2;
    const uint32_t dw = (D & 4) ? c1 : c0;
    return (dw >> (8 * (step & 3))) & 255u;
}

using PairDesc = WavePairDesc;      // scan_plan.h

struct WaveParams {
    ScanParams S;              // codes, tables, nprobe, k, CH (= blocks per item), maxchunks; part_* = per-item result slots
    const PairDesc* pdesc;     // [npairs]
    const int32_t* pair_pre;   // [npairs] first item of the pair inside its query
    const int4* qinfo;         // [nq] {units (items, or pairs when tables come per pair), items, per-pair tables?, 0}
    int32_t* qnext;            // [nq] next unclaimed unit
    int32_t* qatt;             // [nq] workgroups attached
    const int64_t* qbytes;     // [nq][2] code bytes streamed / algorithmic code bytes of the query
    int64_t* counters;
    int nq;
    int64_t qslots;            // result slots per query (= nprobe * maxchunks >= its items)
    int nslice;                // slices of a query's slots in the first stage of the merge (1: the only stage)
    int32_t* stage_I;          // [nq][nslice][k] first-stage results (score, id), INT32_MIN = none
    int64_t* stage_id;
};

// Interleave one plane-major table (HBM, [plane][c][slot] bytes) into the LDS table: the planes of a (code, slot)
// entry become the bytes of one dword.  Unit u = 8 consecutive slots of one code, thread u mod THREADS.
template <int planes>
__device__ __forceinline__ void install_table(const uint8_t* src, uint8_t* lut) {
    const int t = threadIdx.x;
    u32x2 a[2][4];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int u = t + r * THREADS;
#pragma unroll
        for (int p = 0; p < 4; ++p) a[r][p] = ((global_u32x2_ptr)(src + (p < planes ? p : 0) * LUT_PLANE))[u];
    }
    const uint32_t m1 = planes > 1 ? ~0u : 0u, m2 = planes > 2 ? ~0u : 0u, m3 = planes > 3 ? ~0u : 0u;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int u = t + r * THREADS;
        uint4 out[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t p0 = h ? a[r][0].y : a[r][0].x, p1 = (h ? a[r][1].y : a[r][1].x) & m1;
            const uint32_t p2 = (h ? a[r][2].y : a[r][2].x) & m2, p3 = (h ? a[r][3].y : a[r][3].x) & m3;
            const uint32_t lo01 = __builtin_amdgcn_perm(p1, p0, 0x05010400u), lo23 = __builtin_amdgcn_perm(p1, p0, 0x07030602u);
            const uint32_t hi01 = __builtin_amdgcn_perm(p3, p2, 0x05010400u), hi23 = __builtin_amdgcn_perm(p3, p2, 0x07030602u);
            out[h] = make_uint4(__builtin_amdgcn_perm(hi01, lo01, 0x05040100u), __builtin_amdgcn_perm(hi01, lo01, 0x07060302u),
                                __builtin_amdgcn_perm(hi23, lo23, 0x05040100u), __builtin_amdgcn_perm(hi23, lo23, 0x07060302u));
        }
        uint4* d = reinterpret_cast<uint4*>(lut + u * 32);
        d[0] = out[0];
        d[1] = out[1];
    }
}

// LDS offset of table entry e = plane * 8192 + code * 32 + slot
__device__ __forceinline__ uint32_t entry_lds(uint32_t e) { return ((e >> 5) & 255u) * 128u + (e & 31u) * 4u + (e >> 13); }

// Full per-pair evaluation of a table straight into LDS (queries whose tables are too flat for the base + patch form).
__device__ __forceinline__ void eval_table(const ScanParams& P, int pair, int q, uint8_t* lut) {
    const int m = P.m, S = rago_steps(m);
    const float dq = lut_step(__uint_as_float(P.T.range_bits[q]));
    for (int e = threadIdx.x; e < m * KSUB; e += THREADS) {
        const int j = e >> 8, c = e & 255;
        const double t = P.T.t64[(int64_t)pair * m + j];
        const uint8_t v = lut_entry(P.T.T64[((int64_t)q * m + j) * KSUB + c], t, (float)(P.T.Tmin[(int64_t)q * m + j] + t), dq);
        for (int rep = j & (S - 1); rep < 32; rep += S) lut[c * 128 + rep * 4 + (j >> 5)] = v;
    }
}

struct ItemDesc { int64_t blk0, row0; int nb, cvecs, pair, valid, item; };   // item = its number inside the query

template <int MPAD>
__global__ void __launch_bounds__(THREADS, 4) scan_kernel(const WaveParams W) {
    constexpr int S = MPAD < 32 ? MPAD : 32;
    constexpr int planes = MPAD < 32 ? 1 : MPAD / 32;
    constexpr int64_t BLK_BYTES = BLOCK_VECS * MPAD;
    const ScanParams& P = W.S;
    extern __shared__ __align__(16) uint8_t smem[];
    uint8_t* lut = smem;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t* buf = reinterpret_cast<uint32_t*>(smem + OFF_CAND) + wave * CAPW;
    uint32_t* corr = reinterpret_cast<uint32_t*>(smem + OFF_CORR) + wave * CORR_CAP;
    uint16_t* s_amb = reinterpret_cast<uint16_t*>(smem + OFF_AMB);
    uint8_t* s_ambv = smem + OFF_AMBV;
    int32_t* s_pre = reinterpret_cast<int32_t*>(smem + OFF_PRE);
    int32_t* sh = reinterpret_cast<int32_t*>(smem + OFF_SH);
    int32_t* hist = reinterpret_cast<int32_t*>(smem + OFF_HIST);
    // sh[0] query, sh[1] unit / chunk counter, sh[2] bound on the query's k-th best score (absolute integer score),
    // sh[3] the first bound the workgroup had for this query = origin of its score histogram (INT32_MIN: none yet),
    // sh[4..5] best (work left per attached workgroup, query) of the search for a query, sh[8..9] the workgroup's
    // batch of items as one 64-bit word (end << 32 | next), sh[10] lock of the wave that fetches a new batch,
    // sh[11] the query's counter may still have items

    uint32_t off[S / 4];
#pragma unroll
    for (int g = 0; g < S / 4; ++g) {
        uint32_t v = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int step = g * 4 + b, l32 = lane & 31;
            const int slot = ((step + l32) & (S - 1)) | (l32 & ~(S - 1));
            v |= (uint32_t)(slot * 8) << (8 * b);
        }
        off[g] = v;
    }
    uint32_t sa = RAGO_WSEL_A, sb = RAGO_WSEL_B;
    const int k = P.k, nq = W.nq, nprobe = P.nprobe, CH = P.CH;
    int loaded_q = -1;                         // query whose base table (and ambiguous entries) sit in LDS

    if (blockIdx.x == 0) {                     // the batch's byte counts (sums of the planning kernel's per-query figures)
        unsigned long long st = 0, al = 0, it = 0;
        for (int i = threadIdx.x; i < nq; i += THREADS) {
            st += (unsigned long long)W.qbytes[2 * i]; al += (unsigned long long)W.qbytes[2 * i + 1]; it += (unsigned long long)W.qinfo[i].y;
        }
        for (int o = 32; o; o >>= 1) { st += __shfl_xor(st, o); al += __shfl_xor(al, o); it += __shfl_xor(it, o); }
        if (lane == 0) {
            atomicAdd(reinterpret_cast<unsigned long long*>(W.counters + 1), st);
            atomicAdd(reinterpret_cast<unsigned long long*>(W.counters + 2), al);
            atomicAdd(reinterpret_cast<unsigned long long*>(W.counters + 0), it);
        }
    }

    // ---- one item: stream its blocks, keep its best k, append what still matters to the query's candidate list.
    // `wa` holds the item's first block when `first_loaded`; on return it holds the first block at `after` (the
    // wave's next item, if it has one).
    uint4 wa[MPAD / 16], wb[MPAD / 16];
    auto run_item = [&](const ItemDesc& d, int q, bool shared_base, int namb, const uint8_t* after_or_null, bool first_loaded) {
        if (lane == 0) {                       // bounds found by other workgroups meanwhile (a plain load: cheap)
            const int32_t g = __hip_atomic_load(P.tauq + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (g > sh[2]) atomicMax(&sh[2], g);
        }
        const int pair = d.pair, nb = d.nb, cvecs = d.cvecs;
        const uint8_t* base = P.codes + d.blk0 * BLK_BYTES;
        const uint8_t* after = after_or_null ? after_or_null : base;
        if (!first_loaded) load_block<MPAD>(wa, base, lane);
        const int bias = __builtin_amdgcn_readfirstlane(P.bias[pair]);
        // ---- corrections of this pair: entries whose exact value differs from the base table's
        int ncorr = 0, maxpos = 0;
        if (shared_base) {
            for (int i0c = 0; i0c < namb; i0c += 64) {
                const int i = i0c + lane;
                int dlt = 0;
                uint32_t e = 0;
                if (i < namb) {
                    e = s_amb[i];
                    dlt = (int)P.T.patch_val[(int64_t)pair * AMB_MAX + i] - (int)s_ambv[i];
                    if ((int)(e & 31u) >= S) dlt = 0;        // a replica of a sub-table (m < 32): counted once
                }
                const uint64_t mask = __ballot(dlt != 0);
                if (dlt != 0) {
                    const uint32_t j = (e >> 13) * 32u + (e & 31u), c = (e >> 5) & 255u;
                    corr[ncorr + lane_rank(mask)] = (j << 16) | (c << 8) | ((uint32_t)dlt & 255u);
                }
                ncorr += __popcll(mask);
                int pos = dlt > 0 ? dlt : 0;
                for (int o = 32; o; o >>= 1) pos += __shfl_xor(pos, o);
                maxpos += pos;
            }
            maxpos = __builtin_amdgcn_readfirstlane(maxpos);
        }
        int cnt = 0;
        auto bound = [&]() {            // the query's bound in units of this pair's sums
            const int64_t dd = (int64_t)sh[2] - bias;
            return (uint32_t)(dd <= 0 ? 0 : (dd > 0x7fffffff ? 0x7fffffff : dd));
        };
        uint32_t thr = bound();
        auto process = [&](const uint4 (&w)[MPAD / 16], int blk) {
            const uint32_t pos = (uint32_t)(blk * BLOCK_VECS + lane);
            const bool valid = (int)pos < cvecs;
            uint32_t sum = 0;
            block_sum_chunk<MPAD, 0>(w, off, sa, sb, sum);
            const uint32_t tb = bound();
            if (tb > thr) thr = tb;
            if (ncorr && __ballot(valid && sum + (uint32_t)maxpos >= thr)) {
                for (int ci = 0; ci < ncorr; ++ci) {
                    const uint32_t e = __builtin_amdgcn_readfirstlane(corr[ci]);
                    const uint32_t code = code_of<MPAD>(w, (int)(e >> 16), lane);
                    if (code == ((e >> 8) & 255u)) sum += (uint32_t)(int)(int8_t)(e & 255u);
                }
            }
            const bool c = valid && sum >= thr;
            const uint64_t mask = __ballot(c);
            if (mask) {
                const int32_t origin = sh[3];
                if (c && origin != INT32_MIN) {
                    const int64_t dd = (int64_t)bias + (int64_t)sum - origin;
                    if (dd >= 0) atomicAdd(&hist[(int)min(dd >> HIST_SHIFT, (int64_t)(HIST_BINS - 1))], 1);
                }
                const int add = __popcll(mask);
                if (cnt + add > CAPW) {
                    const uint32_t kth = wave_prune(buf, cnt, k, lane);
                    if ((kth >> 16) > thr) thr = kth >> 16;
                    if (lane == 0) atomicMax(&sh[2], bias + (int32_t)thr);
                }
                if (c) buf[cnt + lane_rank(mask)] = (sum << 16) | (0xFFFFu - pos);
                cnt += add;
            }
        };
        // ---- stream the item's blocks: the block after the current one is always in flight (the first block of
        // the wave's next item after the last); unconditional loads from addresses that are always legal
        int b = 0;
        for (;;) {
            load_block<MPAD>(wb, b + 1 < nb ? base + (int64_t)(b + 1) * BLK_BYTES : after, lane);
            process(wa, b);
            if (++b == nb) {                       // the next item's first block sits in wb: move it over
#pragma unroll
                for (int i = 0; i < MPAD / 16; ++i) wa[i] = wb[i];
                break;
            }
            load_block<MPAD>(wa, b + 1 < nb ? base + (int64_t)(b + 1) * BLK_BYTES : after, lane);
            process(wb, b);
            if (++b == nb) break;
        }
        // ---- the item's result: its best k by (sum desc, position asc), and what they say about the query
        uint32_t kth = 0;
        if (cnt > k) kth = wave_prune(buf, cnt, k, lane);
        else if (cnt == k) {
            uint32_t r[CAPW / 64];
#pragma unroll
            for (int i = 0; i < CAPW / 64; ++i) r[i] = (lane + 64 * i < cnt) ? buf[lane + 64 * i] : 0u;
            kth = select_kth<CAPW / 64>(r, k);
        }
        if (cnt >= k && lane == 0) {          // k entries reach the k-th key's score: a bound on the query's k-th best
            const int32_t tq = bias + (int32_t)(kth >> 16);
            if (atomicMax(&sh[2], tq) < tq) publish_bound(P.tauq + q, tq);  // (to HBM only when it is news to this workgroup)
        }
        // ---- the bound from the histogram of all the workgroup's candidates of this query: the highest bin edge with
        // k candidates at or above it (lane L owns bins 16 L .. 16 L + 15)
        {
            const int32_t origin = sh[3];
            if (origin != INT32_MIN) {
                int tot = 0;
                for (int i = 0; i < HIST_BINS / 64; ++i) tot += hist[lane * (HIST_BINS / 64) + i];
                int sfx = tot;
                for (int o = 1; o < 64; o <<= 1) {
                    const int v = __shfl_down(sfx, o);
                    if (lane + o < 64) sfx += v;
                }
                const uint64_t reach = __ballot(sfx >= k);
                if (reach) {
                    const int L = 63 - __builtin_clzll(reach);
                    if (lane == L) {
                        // (counts may have grown since the first look: more candidates only make the edge more valid)
                        int cum = sfx - tot, b = L * (HIST_BINS / 64);
                        for (int i = HIST_BINS / 64 - 1; i >= 0; --i) {
                            cum += hist[L * (HIST_BINS / 64) + i];
                            if (cum >= k) { b = L * (HIST_BINS / 64) + i; break; }
                        }
                        const int64_t edge = (int64_t)origin + ((int64_t)b << HIST_SHIFT);
                        const int32_t tq = (int32_t)min(edge, (int64_t)0x7fffffff);
                        if (atomicMax(&sh[2], tq) < tq) publish_bound(P.tauq + q, tq);
                    }
                }
            } else if (lane == 0 && sh[2] != INT32_MIN) {
                atomicCAS(&sh[3], INT32_MIN, sh[2]);       // the histogram starts here
            }
        }
        // entries below the bound can never be in the query's result: only the others go to the item's slot
        const int32_t tau_now = sh[2];
        uint32_t k0 = 0, k1 = 0;               // (cnt <= k <= 128: two keys per lane)
        if (lane < cnt) k0 = buf[lane];
        if (lane + 64 < cnt) k1 = buf[lane + 64];
        const bool w0 = lane < cnt && bias + (int32_t)(k0 >> 16) >= tau_now, w1 = lane + 64 < cnt && bias + (int32_t)(k1 >> 16) >= tau_now;
        const uint64_t m0 = __ballot(w0), m1 = __ballot(w1);
        const int n0 = __popcll(m0), n1 = __popcll(m1);
        const int64_t slot = (int64_t)q * W.qslots + d.item;
        int32_t* oI = P.part_I + slot * k;
        int64_t* orow = P.part_row + slot * k;
        if (w0) { const int o = lane_rank(m0); oI[o] = bias + (int32_t)(k0 >> 16); orow[o] = d.row0 + (int64_t)(0xFFFFu - (k0 & 0xFFFFu)); }
        if (w1) { const int o = n0 + lane_rank(m1); oI[o] = bias + (int32_t)(k1 >> 16); orow[o] = d.row0 + (int64_t)(0xFFFFu - (k1 & 0xFFFFu)); }
        if (lane == 0) P.part_cnt[slot] = n0 + n1;
    };

    // chunk c of a pair as an item
    auto item_of = [&](const PairDesc& pd, int pair, int c, bool valid) {
        ItemDesc d;
        d.blk0 = pd.blk0 + (int64_t)c * CH;
        d.row0 = pd.row0 + (int64_t)c * CH * BLOCK_VECS;
        d.nb = min(CH, pd.nblk - c * CH);
        d.cvecs = min(pd.len - c * CH * BLOCK_VECS, d.nb * BLOCK_VECS);
        d.pair = pair;
        d.valid = valid;
        d.item = pd.pre + c;
        return d;
    };
    auto load_pdesc = [&](int64_t pair) {       // (every lane loads the same 32 bytes: one request)
        const int4* p = reinterpret_cast<const int4*>(W.pdesc + pair);
        const int4 a = p[0], b = p[1];
        PairDesc pd;
        pd.blk0 = ((int64_t)__builtin_amdgcn_readfirstlane(a.y) << 32) | (uint32_t)__builtin_amdgcn_readfirstlane(a.x);
        pd.row0 = ((int64_t)__builtin_amdgcn_readfirstlane(a.w) << 32) | (uint32_t)__builtin_amdgcn_readfirstlane(a.z);
        pd.nblk = __builtin_amdgcn_readfirstlane(b.x); pd.len = __builtin_amdgcn_readfirstlane(b.y);
        pd.pre = __builtin_amdgcn_readfirstlane(b.z); pd.pair = __builtin_amdgcn_readfirstlane(b.w);
        return pd;
    };

    // first attachment: workgroup b takes query b mod nq, as number b / nq of those that do
    int q = blockIdx.x % nq;
    int rank = blockIdx.x / nq;
    bool first_round = true;
    for (;;) {
        __syncthreads();                       // every wave is done with the previous query's table and scalars
        if (!first_round) {
            // ---- look for the query with the most work left per attached workgroup
            if (threadIdx.x == 0) { sh[4] = 0; sh[5] = 0; }     // one 64-bit word: (work left per workgroup + 1) << 32 | query; 0 = none
            __syncthreads();
            int best = 0, bq = -1;
            for (int i = threadIdx.x; i < nq; i += THREADS) {
                const int left = W.qinfo[i].x - __hip_atomic_load(W.qnext + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (left > 0) {
                    const int att = __hip_atomic_load(W.qatt + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    const int score = left / (att + 1) + 1;
                    if (score > best) { best = score; bq = i; }
                }
            }
            for (int o = 32; o; o >>= 1) {
                const int ob = __shfl_xor(best, o), oq = __shfl_xor(bq, o);
                if (ob > best || (ob == best && oq > bq)) { best = ob; bq = oq; }
            }
            if (lane == 0 && bq >= 0) atomicMax(reinterpret_cast<unsigned long long*>(sh + 4), ((unsigned long long)(uint32_t)best << 32) | (uint32_t)bq);
            __syncthreads();
            const unsigned long long pick = *reinterpret_cast<const unsigned long long*>(sh + 4);
            if ((pick >> 32) == 0) break;      // no query has anything left: every wave reads the same word, all leave together
            q = (int)(uint32_t)pick;
            rank = -1;
            __syncthreads();
        }
        first_round = false;
        const int4 qi = W.qinfo[q];
        const int nunits = __builtin_amdgcn_readfirstlane(qi.x);
        const bool per_pair = __builtin_amdgcn_readfirstlane(qi.z) != 0;
        const int namb = per_pair ? 0 : __builtin_amdgcn_readfirstlane(P.T.namb[q]);
        if (threadIdx.x == 0) {
            sh[2] = __hip_atomic_load(P.tauq + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            atomicAdd(W.qatt + q, 1);
            // the first batch comes with the first attachment (the query's counter starts behind those batches)
            const int b0 = rank >= 0 ? rank * BATCH : 0, b1 = rank >= 0 ? min(b0 + BATCH, nunits) : 0;
            sh[8] = b0; sh[9] = max(b0, b1);
            sh[10] = 0; sh[11] = 1;
            sh[3] = sh[2];                     // (a bound found by others already: the histogram can start at once)
        }
        for (int i = threadIdx.x; i < HIST_BINS; i += THREADS) hist[i] = 0;
        if (!per_pair) {
            if (loaded_q != q) {               // (a batch of one query, or the same query again: nothing to install)
                install_table<planes>(P.T.lut_base + (int64_t)q * LUT_BYTES, lut);
                for (int i = threadIdx.x; i < namb; i += THREADS) s_amb[i] = P.T.amb_addr[(int64_t)q * AMB_MAX + i];
                for (int i = threadIdx.x; i < nprobe; i += THREADS) s_pre[i] = W.pair_pre[(int64_t)q * nprobe + i];
                if (threadIdx.x == 0) s_pre[nprobe] = qi.y;
                __syncthreads();
                for (int i = threadIdx.x; i < namb; i += THREADS) s_ambv[i] = lut[entry_lds(s_amb[i])];
            }
            loaded_q = q;
            __syncthreads();
            // ---- the waves' items: the first by rank (first attachment), the others from the query's counter
            // An item from the workgroup's batch; when the batch is used up, one wave fetches the next from the
            // query's counter while the others back off (a wave only ever waits for a wave that holds the lock, and
            // that wave waits for nobody).  INT_MAX = the query has no items left.
            unsigned long long* s_batch = reinterpret_cast<unsigned long long*>(sh + 8);
            auto claim = [&]() {
                for (;;) {
                    unsigned long long old = 0;
                    if (lane == 0) old = atomicAdd(s_batch, 1ull);
                    const uint32_t cur = __builtin_amdgcn_readfirstlane((uint32_t)old), end = __builtin_amdgcn_readfirstlane((uint32_t)(old >> 32));
                    if (cur < end) return (int)cur;
                    int state = 0;             // 0: go round again, 1: nothing left
                    if (lane == 0) {
                        if (__hip_atomic_load(&sh[11], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) == 0) state = 1;
                        else if (atomicCAS(&sh[10], 0, 1) == 0) {
                            const unsigned long long now = __hip_atomic_load(s_batch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                            if ((uint32_t)now >= (uint32_t)(now >> 32)) {          // still used up: nobody refilled it meanwhile
                                const int base = atomicAdd(W.qnext + q, BATCH);
                                if (base >= nunits) __hip_atomic_store(&sh[11], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                                else atomicExch(s_batch, ((unsigned long long)(uint32_t)min(base + BATCH, nunits) << 32) | (uint32_t)base);
                            }
                            __hip_atomic_store(&sh[10], 0, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
                        } else {
                            __builtin_amdgcn_s_sleep(8);
                        }
                    }
                    if (__builtin_amdgcn_readfirstlane(state)) return 0x7fffffff;
                }
            };
            auto resolve = [&](int i) {
                const bool valid = i < nunits;
                const int ii = valid ? i : nunits - 1;
                int lo = 0, hi = nprobe;       // pair p with s_pre[p] <= ii < s_pre[p + 1] (pairs without items share a value with their successor)
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    if (s_pre[mid] <= ii) lo = mid; else hi = mid;
                }
                const PairDesc pd = load_pdesc((int64_t)q * nprobe + lo);
                return item_of(pd, q * nprobe + pd.pair, ii - pd.pre, valid);
            };
            if (nunits > 0) {
                int i_cur = claim();
                int i_nxt = claim();
                ItemDesc cur = resolve(i_cur);
                bool first_loaded = false;
                while (cur.valid) {
                    const ItemDesc nxt = resolve(i_nxt);
                    const int i_nn = claim();
                    run_item(cur, q, true, namb, nxt.valid ? P.codes + nxt.blk0 * BLK_BYTES : nullptr, first_loaded);
                    first_loaded = true;
                    cur = nxt;
                    i_nxt = i_nn;
                }
            }
        } else {
            // ---- per-pair tables: the workgroup takes whole pairs, its waves share out the pair's items
            loaded_q = -1;
            for (bool first_pair = true;; first_pair = false) {
                __syncthreads();               // the previous pair's table is no longer read
                if (threadIdx.x == 0) {
                    sh[0] = first_pair && rank >= 0 ? rank : atomicAdd(W.qnext + q, 1);
                    sh[1] = 0;
                }
                __syncthreads();
                const int p = __builtin_amdgcn_readfirstlane(sh[0]);
                if (p >= nunits) break;
                const PairDesc pd = load_pdesc((int64_t)q * nprobe + p);
                const int64_t pair = (int64_t)q * nprobe + pd.pair;
                if (P.lut8sw) install_table<planes>(P.lut8sw + pair * LUT_BYTES, lut);
                else eval_table(P, (int)pair, q, lut);
                const int nchunks = (pd.nblk + CH - 1) / CH;
                __syncthreads();
                for (;;) {
                    int c = 0;
                    if (lane == 0) c = atomicAdd(&sh[1], 1);
                    c = __builtin_amdgcn_readfirstlane(c);
                    if (c >= nchunks) break;
                    run_item(item_of(pd, (int)pair, c, true), q, false, 0, nullptr, false);
                }
            }
        }
        __syncthreads();
        if (threadIdx.x == 0) atomicSub(W.qatt + q, 1);
    }
}

// ------------------------------------------------------------------ planning kernel
// (the work itself: scan_plan.h)
__global__ void __launch_bounds__(256) plan_kernel(const WavePlanArgs A) { wave_plan_body(A, (int)blockIdx.x); }

// ------------------------------------------------------------------ per-query merge of the items' results
// Stage 1: workgroup (query, slice) takes the slots of its slice of the query's items, keeps the entries that reach
// the query's final bound, looks up their ids, sorts by (score desc, id asc) and keeps k.  With one slice per query
// that is the result; else it goes to the stage arrays and stage 2 (one workgroup per query) merges the slices'.
struct TopK {
    int32_t* sI;
    int64_t* sId;
    int* s_cnt;
    int k;
    int32_t* tmp;        // LDS for rank_top_k, the one-entry-per-thread path (may be null)
    // sort the first `have` entries of the buffer, keep k
    __device__ int sort_keep_k(int have) {
        if (tmp && have <= (int)blockDim.x && have > 1 && rank_top_k(sI, sId, have, k, tmp)) return min(have, k);
        int n2 = 1;
        while (n2 < have) n2 <<= 1;
        for (int i = have + threadIdx.x; i < n2; i += blockDim.x) { sI[i] = INT32_MIN; sId[i] = INT64_MAX; }
        if (n2 > 1) bitonic_sort(sI, sId, n2); else __syncthreads();
        return min(have, k);
    }
};

// NT threads: 256, or 1024 while the batch has no more workgroups than the chip has room for (the walks over the slots are
// chains of dependent round trips, four times shorter then).
template <int NT>
__global__ void __launch_bounds__(NT) merge_slots_kernel(const WaveParams W, const float* __restrict__ delta,
                                                         int64_t* __restrict__ out_ids, float* __restrict__ out_scores,
                                                         int32_t* __restrict__ out_iscores) {
    __shared__ __align__(16) int32_t sI[MERGE_CAP];
    __shared__ int64_t sId[MERGE_CAP];
    __shared__ int s_cnt;
    const ScanParams& P = W.S;
    const int q = blockIdx.x / W.nslice, slice = blockIdx.x % W.nslice, k = P.k;
    int32_t tau = P.tauq[q];   // k candidates of this query reach tau: nothing below can be in the result
    const int nitems = W.qinfo[q].y;
    const int per = (nitems + W.nslice - 1) / W.nslice;
    const int i0 = slice * per, i1 = min(nitems, i0 + per);
    const int64_t slot0 = (int64_t)q * W.qslots;
    TopK T{sI, sId, &s_cnt, k, nullptr};
    // Every entry of the slots [a, b), in tiles of MS_TILE slots: a thread per slot reads the slot's count into LDS, then the
    // tile's entries are walked as ONE flat array (entry f = slot f / k, position f % k; positions beyond a slot's count
    // are stale and skipped): neighbouring lanes read neighbouring words, four loads per lane in flight.  (Sharing out
    // only the live entries needs a search per entry and left one dependent load per trip round the loop: the three
    // passes of a query's ~190 slots x 100 entries took 53 us.)  f(score, position in the result arrays).
    constexpr int MS_TILE = 1024;
    __shared__ __align__(8) int s_n[MS_TILE];
    __shared__ int s_max;
    static_assert(MS_TILE >= 3 * RANK_CAND + 1, "the slot counts' words double as the ranking path's side buffer");
    if (NT >= 1024) T.tmp = s_n;          // (with fewer threads the buffer seldom fits one entry per thread)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    auto each_entry = [&](int a, int b, auto f) {
        for (int t0 = a; t0 < b; t0 += MS_TILE) {
            const int ts = min(MS_TILE, b - t0);
            __syncthreads();
            for (int j = threadIdx.x; j < ts; j += NT) s_n[j] = P.part_cnt[slot0 + t0 + j];
            __syncthreads();
            const int total = ts * k;
            const int64_t base = (slot0 + t0) * k;
            constexpr int U = 4;
            for (int f0 = threadIdx.x; f0 < total; f0 += NT * U) {
                int32_t I[U];
                bool live[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int fi = min(f0 + u * NT, total - 1);
                    const int j = fi / k;
                    live[u] = f0 + u * NT < total && fi - j * k < s_n[j];
                    I[u] = P.part_I[base + fi];
                }
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (live[u]) f(I[u], base + f0 + u * NT);
            }
        }
    };
    // entries that reach tau, appended behind the first base_fill entries of the buffer; returns how many reach it (those
    // beyond the buffer's capacity are counted, not kept) and leaves the largest margin over tau in s_max
    auto gather = [&](int a, int b, int base_fill) {
        if (threadIdx.x == 0) { s_cnt = base_fill; s_max = 0; }
        __syncthreads();
        int mx = 0;
        each_entry(a, b, [&](int32_t I, int64_t at) {
            if (I >= tau) {
                mx = max(mx, (int)min((int64_t)I - tau, (int64_t)0x7fffffff));
                const int o = atomicAdd(&s_cnt, 1);
                if (o < MERGE_CAP) { sI[o] = I; sId[o] = P.ids[P.part_row[at]]; }
            }
        });
        for (int o = 32; o; o >>= 1) mx = max(mx, __shfl_xor(mx, o));
        if (lane == 0 && mx > 0) atomicMax(&s_max, mx);
        __syncthreads();
        return s_cnt;
    };
    // Optimistic: everything that passes tau fits the buffer (the usual case by far).  The bound the scan leaves is the
    // best k-th score of a single item, which is weak when lists are short and k is large: if more entries pass it than
    // the buffer holds, a histogram of their scores gives a bound with at least k entries at or above it that is within
    // one bin of the slice's true k-th score, and the entries are gathered again.
    int have = gather(i0, i1, 0);
    if (have > MERGE_CAP) {
        const int maxd = s_max;
        __syncthreads();
        constexpr int BINS = 1024;
        int* hist = reinterpret_cast<int*>(sI);                  // (what the buffer holds is gathered again below)
        int shift = 0;
        while ((maxd >> shift) >= BINS) ++shift;
        for (int i = threadIdx.x; i < BINS; i += NT) hist[i] = 0;
        __syncthreads();
        each_entry(i0, i1, [&](int32_t I, int64_t) {
            if (I >= tau) atomicAdd(&hist[(int)(((int64_t)I - tau) >> shift)], 1);
        });
        __syncthreads();
        // the highest bin with at least k entries in it and above: thread t < 256 owns bins 4t .. 4t + 3
        __shared__ int s_wsum[NT / 64];
        __shared__ int s_bin;
        const int t = threadIdx.x;
        const bool own = t < BINS / 4;
        const int h0 = own ? hist[4 * t] : 0, h1 = own ? hist[4 * t + 1] : 0, h2 = own ? hist[4 * t + 2] : 0, h3 = own ? hist[4 * t + 3] : 0;
        int sfx = h0 + h1 + h2 + h3;
        for (int o = 1; o < 64; o <<= 1) {
            const int v = __shfl_down(sfx, o);
            if (lane + o < 64) sfx += v;
        }
        if (lane == 0) s_wsum[wave] = sfx;
        if (t == 0) s_bin = 0;
        __syncthreads();
        int above = 0;
        for (int w = wave + 1; w < NT / 64; ++w) above += s_wsum[w];
        const int mine = sfx + above;                            // entries in bins >= 4t
        const int next = mine - (h0 + h1 + h2 + h3);             // entries in bins >= 4t + 4
        if (mine >= k && next < k) {                             // exactly one thread
            int cum = next, bsel = 4 * t;
            const int hh[4] = {h0, h1, h2, h3};
            for (int i = 3; i >= 0; --i) {
                cum += hh[i];
                if (cum >= k) { bsel = 4 * t + i; break; }
            }
            s_bin = bsel;
        }
        __syncthreads();
        tau += (int32_t)((int64_t)s_bin << shift);
        __syncthreads();
        have = gather(i0, i1, 0);
    }
    int fill;
    if (have <= MERGE_CAP) {
        fill = T.sort_keep_k(have);
    } else {
        const int per_round = max(1, (MERGE_CAP - k) / k);      // slots per round that cannot overflow the buffer
        fill = 0;
        for (int a = i0; a < i1; a += per_round) {
            __syncthreads();
            have = gather(a, min(i1, a + per_round), fill);
            fill = T.sort_keep_k(have);
            if (fill == k && sI[k - 1] > tau) tau = sI[k - 1];
        }
    }
    __syncthreads();
    if (W.nslice > 1) {
        const int64_t o = ((int64_t)q * W.nslice + slice) * k;
        for (int r = threadIdx.x; r < k; r += NT) {
            W.stage_I[o + r] = r < fill ? sI[r] : INT32_MIN;
            W.stage_id[o + r] = r < fill ? sId[r] : -1;
        }
        return;
    }
    for (int r = threadIdx.x; r < k; r += NT) {
        const bool ok = r < fill;
        const int32_t I = ok ? sI[r] : INT32_MIN;
        out_ids[(int64_t)q * k + r] = ok ? sId[r] : -1;
        if (out_iscores) out_iscores[(int64_t)q * k + r] = I;
        if (out_scores) out_scores[(int64_t)q * k + r] = ok ? (float)I * (delta ? delta[q] : 1.0f) : -INFINITY;
    }
}

// Stage 2: the slices' results of one query (nslice * k entries, ids already looked up).
__global__ void __launch_bounds__(MERGE_THREADS) merge_stage2_kernel(const WaveParams W, const float* __restrict__ delta,
                                                                     int64_t* __restrict__ out_ids, float* __restrict__ out_scores,
                                                                     int32_t* __restrict__ out_iscores) {
    __shared__ int32_t sI[MERGE_CAP];
    __shared__ int64_t sId[MERGE_CAP];
    __shared__ int s_cnt;
    const int q = blockIdx.x, k = W.S.k;
    const int64_t o = (int64_t)q * W.nslice * k;
    const int n = W.nslice * k;
    TopK T{sI, sId, &s_cnt, k, nullptr};
    int fill = 0;
    const int per_round = MERGE_CAP - k;                         // entries per round that cannot overflow the buffer
    for (int a = 0; a < n; a += per_round) {
        __syncthreads();
        if (threadIdx.x == 0) s_cnt = fill;
        __syncthreads();
        for (int e = a + (int)threadIdx.x; e < min(n, a + per_round); e += MERGE_THREADS) {
            const int32_t I = W.stage_I[o + e];
            if (I != INT32_MIN) {
                const int at = atomicAdd(&s_cnt, 1);
                sI[at] = I; sId[at] = W.stage_id[o + e];
            }
        }
        __syncthreads();
        fill = T.sort_keep_k(s_cnt);
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

template <int MPAD>
static int launch_one(const WaveParams& W, int grid, hipStream_t st) {
    static OncePerDevice attr;
    if (attr.first()) {
        RAGO_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(scan_kernel<MPAD>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     SCAN_LDS));
    }
    scan_kernel<MPAD><<<grid, THREADS, SCAN_LDS, st>>>(W);
    RAGO_HIP(hipGetLastError());
    return RAGO_OK;
}

}  // namespace wavescan

// Blocks per item: enough items for every resident wave to take many (a wave works through an item alone, so what
// is left at the end of the kernel is the longest item still running), at most 512 blocks (position field).
constexpr double WV_ITEMS_PER_WAVE = 4.0;   // items aimed at per resident wave
constexpr int WV_MIN_CHUNK = 8;
int wave_chunk_len(double total_blocks, int n_cu) {
    const double want = WV_ITEMS_PER_WAVE * 2 * wavescan::WAVES * n_cu;
    int c = WV_MIN_CHUNK;
    while (c < 512 && total_blocks / c > want) c <<= 1;
    return c;
}

size_t wave_pair_bytes() { return sizeof(wavescan::PairDesc); }

// Slices of a query's item slots in the first merge stage: one per ~256 items (one round of its workgroup), at most 32.
constexpr int MAX_SLICES = 32;
int wave_merge_slices(double items_per_query) {
    int r = 1;
    while (r < MAX_SLICES && items_per_query / r > 256.0) r <<= 1;
    return r;
}
size_t wave_stage_bytes(int64_t nq, int k) { return (size_t)nq * MAX_SLICES * k * 12; }

// Where the plan's outputs live in the workspace arrays (pdesc [npairs], pair_pre [npairs], qwork [nq * 12 ints]).
void fill_wave_plan(const ScanParams& P, int64_t nq, int n_cu, void* pdesc, int32_t* pair_pre, int32_t* qwork, int64_t* counters,
                    WavePlanArgs* A) {
    A->enable = 1;
    A->probes = P.probes; A->blk_off = P.blk_off; A->list_off = P.list_off;
    A->nprobe = P.nprobe; A->CH = P.CH; A->m = P.m; A->nq = (int)nq; A->nwg = 2 * n_cu;
    A->namb = P.T.namb; A->all_per_pair = P.lut8sw != nullptr;
    A->pdesc = static_cast<WavePairDesc*>(pdesc);
    A->pair_pre = pair_pre;
    A->qinfo = reinterpret_cast<int4*>(qwork);
    A->qnext = qwork + 4 * nq;
    A->qatt = qwork + 5 * nq;
    A->qbytes = reinterpret_cast<int64_t*>(qwork + 8 * nq);
    A->tauq = P.tauq;
    A->counters = counters;
}

// Plans on the device (one small kernel, unless `plan_done`), scans, merges the items' results.  P.CH / P.maxchunks
// are the blocks per item and the most items any pair can have; pdesc [npairs], pair_pre [npairs], qwork [nq * 12
// ints], stage [wave_stage_bytes] are workspace; P.part_* hold the items' results (nprobe * maxchunks slots per query).
int launch_scan_wave(const ScanParams& P, int64_t nq, int n_cu, double avgblk, void* pdesc, int32_t* pair_pre, int32_t* qwork,
                     void* stage, int64_t* counters, const float* delta, int64_t* out_ids, float* out_scores, int32_t* out_iscores,
                     hipEvent_t* ev, hipStream_t st, bool plan_done) {
    using namespace wavescan;
    WavePlanArgs A;
    fill_wave_plan(P, nq, n_cu, pdesc, pair_pre, qwork, counters, &A);
    const int grid = A.nwg;
    WaveParams W;
    W.S = P;
    W.pdesc = A.pdesc;
    W.pair_pre = pair_pre;
    W.qinfo = A.qinfo;
    W.qnext = A.qnext;
    W.qatt = A.qatt;
    W.qbytes = A.qbytes;
    W.counters = counters;
    W.nq = (int)nq;
    W.qslots = (int64_t)P.nprobe * P.maxchunks;
    W.nslice = wave_merge_slices((double)P.nprobe * std::max(1.0, avgblk / P.CH));
    W.stage_id = static_cast<int64_t*>(stage);
    W.stage_I = reinterpret_cast<int32_t*>(W.stage_id + nq * MAX_SLICES * P.k);
    if (!plan_done) plan_kernel<<<(unsigned)nq, 256, 0, st>>>(A);      // (else a kernel of the caller's has done it)
    RAGO_HIP(hipGetLastError());
    if (ev) RAGO_HIP(hipEventRecord(ev[4], st));
    int rc;
    switch (P.m) {
        case 16: rc = launch_one<16>(W, grid, st); break;
        case 32: rc = launch_one<32>(W, grid, st); break;
        case 64: rc = launch_one<64>(W, grid, st); break;
        case 96: rc = launch_one<96>(W, grid, st); break;
        case 128: rc = launch_one<128>(W, grid, st); break;
        default: return fail(RAGO_UNSUPPORTED, "code width");
    }
    if (rc) return rc;
    if (ev) RAGO_HIP(hipEventRecord(ev[5], st));
    if (nq * W.nslice <= 2 * n_cu) merge_slots_kernel<1024><<<(unsigned)(nq * W.nslice), 1024, 0, st>>>(W, delta, out_ids, out_scores, out_iscores);
    else merge_slots_kernel<MERGE_THREADS><<<(unsigned)(nq * W.nslice), MERGE_THREADS, 0, st>>>(W, delta, out_ids, out_scores, out_iscores);
    if (W.nslice > 1) merge_stage2_kernel<<<(unsigned)nq, MERGE_THREADS, 0, st>>>(W, delta, out_ids, out_scores, out_iscores);
    RAGO_HIP(hipGetLastError());
    if (ev) RAGO_HIP(hipEventRecord(ev[6], st));
    return RAGO_OK;
}

}  // namespace rago

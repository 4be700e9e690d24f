// Integer asymmetric-distance scan of the probed lists + per-query top-k (the retrieval cost the
// paper measures in bytes of PQ codes scanned per query, Section 3.3; low-precision tables make
// the scan memory-bound, Section 2).
//
// For every (query, probed list) pair and every vector i of the list:
//     I = B[pair] + sum_j LUT8[pair][j][code[i][j]]
// and per query the best k of all its pairs by (I descending, id ascending).
//
// Work organisation
//  * pairs are grouped by list; a task = (list, chunk of <= CH 64-vector blocks, up to FOUR pairs
//    of that list).  The four pairs' tables sit in LDS interleaved byte by byte, so a code byte
//    fetched once from HBM serves four queries with ONE 32-bit LDS read.  Persistent workgroups
//    (one per CU) pull task numbers from one atomic counter.
//  * LDS table layout: byte address = plane * 32768 + code * 128 + slot * 4 + cell, where the
//    four cells of a dword belong to the four pairs (pair 0..3 in bytes 0, 2, 1, 3).  `slot`
//    selects the bank, so a sub-table lives in ONE bank; the 32 lanes of a half-wave always work
//    on 32 different slots (see layout.hip), which makes every ds_read_b32 conflict-free whatever
//    the code values are.  One v_perm_b32 places two code bytes next to the lane's slot bytes
//    (slot * 8), a bit-field extract / funnel shift by one bit turns each half into
//    code * 128 + slot * 4; planes ride in the immediate offset (and, beyond its 64 KiB reach, in
//    a flag bit of the slot byte and the funnel shift's upper operand).
//  * accumulation is packed: with at most two pairs the cells in bytes 1 and 3 are zero and a plain
//    32-bit add accumulates two 16-bit sums at once (sums are <= 128 * 255 < 2^16); with three or
//    four pairs the odd bytes of two look-ups are gathered by one v_perm_b32 into 16-bit lanes of
//    their own accumulators and subtracted from the running 32-bit sum at the end of the block.
//  * one lane = one vector: 6 x dwordx4 loads (m = 96) per lane per block, 1 KiB contiguous per
//    wave and load, next block's loads issued before the current block is processed.
//  * selection: scores are <= 32640 so (score << 16 | 0xFFFF - position in chunk) is a 32-bit
//    key whose order is (score desc, position asc) = (score desc, id asc) inside one list.
//    Each wave keeps a private LDS buffer of keys per pair above a running threshold and prunes it
//    to the best k with a radix select on ballots (no barriers, no atomics in the streaming loop).
//    Thresholds are shared through LDS (per task) and through a per-query word in HBM
//    (atomicMax of each finished task's k-th best score): a candidate below a score that k other
//    candidates of the same query already reach can never be in the result.
//  * each task writes <= k (I, id) entries per pair; the waves that merge a finished task's
//    buffers do so while the other waves already load the next task's tables; a final kernel per
//    query merges the task results, sorts by (I desc, id asc) and writes ids / scores.
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <type_traits>

#include "scan_common.h"
#include "scan_setup.h"
#include "scan_plan.h"

namespace rago {

constexpr int NPMAX = 4;        // pairs (tables) per pass
constexpr int DESC_INTS = 28;   // task descriptor in LDS (see fetch_task)
constexpr int SH_INTS = 256;    // scalars + two descriptors

template <int MPAD>
struct ScanShape {
    static constexpr int S = MPAD < 32 ? MPAD : 32;            // steps per plane
    static constexpr int PLANES = MPAD < 32 ? 1 : MPAD / 32;
    static constexpr int NW = MPAD > 96 ? 8 : 16;              // waves per workgroup (LDS-limited)
    static constexpr int NT = NW * 64;
    static constexpr int LUT_LDS = PLANES * 4 * LUT_PLANE;     // four interleaved tables
    static constexpr int LDS = LUT_LDS + NW * NPMAX * CAPW * 4 + SH_INTS * 4 + NPMAX * 256 * 4;   // + merge histograms
};

// Eight look-ups (two code dwords of one plane) in all resident tables at once.  Hand-scheduled:
// the compiler serialises LDS reads behind full waits and spills when given the plain C++ form.
//
// A code dword `w` holds 4 consecutive steps of one plane; `o` holds slot*8 of those 4 steps.
// v_perm_b32 with selector SEL_A (SEL_B) builds {code1, slot1*8, code0, slot0*8} (codes 3, 2);
// bits [16:1] of that are code0*128 + slot0*4 (+32768 when bit 0 of the next slot byte is set: the
// flagged copies of `o` used for planes 2 and 3), and a funnel shift by 17 gives code1*128 +
// slot1*4 with `HI` shifted in above (HI * 32768).  The table region starts at LDS address 0.
// Each asm statement drains its own LDS reads (lgkmcnt(0)) before it ends, so the compiler's
// own wait counts around it stay valid.
#define RAGO_SEL_A 0x05010400u
#define RAGO_SEL_B 0x07030602u
#define RAGO_SEL_O1 0x0c050c01u   // {0, hi.byte1, 0, lo.byte1}
#define RAGO_SEL_O3 0x0c070c03u   // {0, hi.byte3, 0, lo.byte3}

#define RAGO_LK_ADDR(W, O, A, B, C, D)                         \
    "v_perm_b32 %[" #B "], %[" #W "], %[" #O "], %[sa]\n"      \
    "v_perm_b32 %[" #D "], %[" #W "], %[" #O "], %[sb]\n"      \
    "v_bfe_u32 %[" #A "], %[" #B "], 1, 16\n"                  \
    "v_alignbit_b32 %[" #B "], %[hi], %[" #B "], 17\n"         \
    "v_bfe_u32 %[" #C "], %[" #D "], 1, 16\n"                  \
    "v_alignbit_b32 %[" #D "], %[hi], %[" #D "], 17\n"
#define RAGO_LK_EXTRA(A, C) "v_add_u32 %[" #A "], 0x8000, %[" #A "]\n v_add_u32 %[" #C "], 0x8000, %[" #C "]\n"
#define RAGO_LK_READ(A, B, C, D)                                                                   \
    "ds_read_b32 %[" #A "], %[" #A "] offset:%[imm]\n ds_read_b32 %[" #B "], %[" #B "] offset:%[imm]\n" \
    "ds_read_b32 %[" #C "], %[" #C "] offset:%[imm]\n ds_read_b32 %[" #D "], %[" #D "] offset:%[imm]\n"
#define RAGO_LK_ALL(A, B, C, D) \
    "v_add3_u32 %[all], %[all], %[" #A "], %[" #B "]\n v_add3_u32 %[all], %[all], %[" #C "], %[" #D "]\n"
#define RAGO_LK_ODD(A, B, C, D, SEL, ACC)                                                          \
    "v_perm_b32 %[p0], %[" #B "], %[" #A "], %[" #SEL "]\n v_perm_b32 %[p1], %[" #D "], %[" #C "], %[" #SEL "]\n" \
    "v_add3_u32 %[" #ACC "], %[" #ACC "], %[p0], %[p1]\n"
#define RAGO_LK_OPERANDS                                                                                       \
    : [all] "+v"(all), [o1] "+v"(o1), [o3] "+v"(o3), [t0] "=&v"(t0), [t1] "=&v"(t1), [t2] "=&v"(t2), [t3] "=&v"(t3), \
      [t4] "=&v"(t4), [t5] "=&v"(t5), [t6] "=&v"(t6), [t7] "=&v"(t7), [p0] "=&v"(p0), [p1] "=&v"(p1)            \
    : [w0] "v"(w0), [w1] "v"(w1), [oa] "v"(oa), [ob] "v"(ob), [sa] "s"(sa), [sb] "s"(sb), [so1] "s"(so1),      \
      [so3] "s"(so3), [imm] "n"(IMM), [hi] "n"(HI)                                                             \
    : "memory"

// NPV = 2: cells 0 and 2 only (the others hold zeros); 3: + cell 1; 4: all four.
template <int NPV, int IMM, int HI, bool EXTRA>
__device__ __forceinline__ void lookup8(uint32_t w0, uint32_t w1, uint32_t oa, uint32_t ob, uint32_t sa, uint32_t sb,
                                        uint32_t so1, uint32_t so3, uint32_t& all, uint32_t& o1, uint32_t& o3) {
    uint32_t t0, t1, t2, t3, t4, t5, t6, t7, p0, p1;
    if constexpr (!EXTRA && NPV == 2) {
        asm volatile(RAGO_LK_ADDR(w0, oa, t0, t1, t2, t3) RAGO_LK_READ(t0, t1, t2, t3)
                     RAGO_LK_ADDR(w1, ob, t4, t5, t6, t7) RAGO_LK_READ(t4, t5, t6, t7)
                     "s_waitcnt lgkmcnt(4)\n" RAGO_LK_ALL(t0, t1, t2, t3)
                     "s_waitcnt lgkmcnt(0)\n" RAGO_LK_ALL(t4, t5, t6, t7) RAGO_LK_OPERANDS);
    } else if constexpr (!EXTRA && NPV == 3) {
        asm volatile(RAGO_LK_ADDR(w0, oa, t0, t1, t2, t3) RAGO_LK_READ(t0, t1, t2, t3)
                     RAGO_LK_ADDR(w1, ob, t4, t5, t6, t7) RAGO_LK_READ(t4, t5, t6, t7)
                     "s_waitcnt lgkmcnt(4)\n" RAGO_LK_ODD(t0, t1, t2, t3, so1, o1) RAGO_LK_ALL(t0, t1, t2, t3)
                     "s_waitcnt lgkmcnt(0)\n" RAGO_LK_ODD(t4, t5, t6, t7, so1, o1) RAGO_LK_ALL(t4, t5, t6, t7)
                     RAGO_LK_OPERANDS);
    } else if constexpr (!EXTRA && NPV == 4) {
        asm volatile(RAGO_LK_ADDR(w0, oa, t0, t1, t2, t3) RAGO_LK_READ(t0, t1, t2, t3)
                     RAGO_LK_ADDR(w1, ob, t4, t5, t6, t7) RAGO_LK_READ(t4, t5, t6, t7)
                     "s_waitcnt lgkmcnt(4)\n" RAGO_LK_ODD(t0, t1, t2, t3, so1, o1) RAGO_LK_ODD(t0, t1, t2, t3, so3, o3)
                     RAGO_LK_ALL(t0, t1, t2, t3)
                     "s_waitcnt lgkmcnt(0)\n" RAGO_LK_ODD(t4, t5, t6, t7, so1, o1) RAGO_LK_ODD(t4, t5, t6, t7, so3, o3)
                     RAGO_LK_ALL(t4, t5, t6, t7) RAGO_LK_OPERANDS);
    } else if constexpr (EXTRA && NPV == 2) {
        asm volatile(RAGO_LK_ADDR(w0, oa, t0, t1, t2, t3) RAGO_LK_EXTRA(t0, t2) RAGO_LK_READ(t0, t1, t2, t3)
                     RAGO_LK_ADDR(w1, ob, t4, t5, t6, t7) RAGO_LK_EXTRA(t4, t6) RAGO_LK_READ(t4, t5, t6, t7)
                     "s_waitcnt lgkmcnt(4)\n" RAGO_LK_ALL(t0, t1, t2, t3)
                     "s_waitcnt lgkmcnt(0)\n" RAGO_LK_ALL(t4, t5, t6, t7) RAGO_LK_OPERANDS);
    } else if constexpr (EXTRA && NPV == 3) {
        asm volatile(RAGO_LK_ADDR(w0, oa, t0, t1, t2, t3) RAGO_LK_EXTRA(t0, t2) RAGO_LK_READ(t0, t1, t2, t3)
                     RAGO_LK_ADDR(w1, ob, t4, t5, t6, t7) RAGO_LK_EXTRA(t4, t6) RAGO_LK_READ(t4, t5, t6, t7)
                     "s_waitcnt lgkmcnt(4)\n" RAGO_LK_ODD(t0, t1, t2, t3, so1, o1) RAGO_LK_ALL(t0, t1, t2, t3)
                     "s_waitcnt lgkmcnt(0)\n" RAGO_LK_ODD(t4, t5, t6, t7, so1, o1) RAGO_LK_ALL(t4, t5, t6, t7)
                     RAGO_LK_OPERANDS);
    } else {
        asm volatile(RAGO_LK_ADDR(w0, oa, t0, t1, t2, t3) RAGO_LK_EXTRA(t0, t2) RAGO_LK_READ(t0, t1, t2, t3)
                     RAGO_LK_ADDR(w1, ob, t4, t5, t6, t7) RAGO_LK_EXTRA(t4, t6) RAGO_LK_READ(t4, t5, t6, t7)
                     "s_waitcnt lgkmcnt(4)\n" RAGO_LK_ODD(t0, t1, t2, t3, so1, o1) RAGO_LK_ODD(t0, t1, t2, t3, so3, o3)
                     RAGO_LK_ALL(t0, t1, t2, t3)
                     "s_waitcnt lgkmcnt(0)\n" RAGO_LK_ODD(t4, t5, t6, t7, so1, o1) RAGO_LK_ODD(t4, t5, t6, t7, so3, o3)
                     RAGO_LK_ALL(t4, t5, t6, t7) RAGO_LK_OPERANDS);
    }
}

struct Sel { uint32_t a, b, o1, o3; };

template <int MPAD, int NPV, int I>
__device__ __forceinline__ void block_sums_chunk(const uint4 (&w)[MPAD / 16], const uint32_t (&off)[ScanShape<MPAD>::S / 4],
                                                 const Sel& sel, uint32_t& all, uint32_t& o1, uint32_t& o3) {
    constexpr int S = ScanShape<MPAD>::S;
    constexpr int PL = (I * 16) / S;               // plane of this dwordx4
    constexpr int G = ((I * 16) % S) / 4;          // first of its four step groups
    constexpr int IMM = PL >= 1 ? 32768 : 0;
    constexpr int HI = PL == 2 ? 1 : (PL == 3 ? 2 : 0);
    if constexpr (PL < 2) {
        lookup8<NPV, IMM, HI, false>(w[I].x, w[I].y, off[G], off[G + 1], sel.a, sel.b, sel.o1, sel.o3, all, o1, o3);
        lookup8<NPV, IMM, HI, false>(w[I].z, w[I].w, off[G + 2], off[G + 3], sel.a, sel.b, sel.o1, sel.o3, all, o1, o3);
    } else {
        // (+32768 for the even look-ups of planes 2 and 3: bit 0 of the following slot byte)
        constexpr uint32_t F = 0x01000100u;
        lookup8<NPV, IMM, HI, PL == 3>(w[I].x, w[I].y, off[G] | F, off[G + 1] | F, sel.a, sel.b, sel.o1, sel.o3, all, o1, o3);
        lookup8<NPV, IMM, HI, PL == 3>(w[I].z, w[I].w, off[G + 2] | F, off[G + 3] | F, sel.a, sel.b, sel.o1, sel.o3, all, o1, o3);
    }
    if constexpr (I + 1 < MPAD / 16) block_sums_chunk<MPAD, NPV, I + 1>(w, off, sel, all, o1, o3);
}

// Sums of one 64-vector block (lane = vector) for the pairs in cells 0..NPV-1: sum[pair].
template <int MPAD, int NPV>
__device__ __forceinline__ void block_sums(const uint4 (&w)[MPAD / 16], const uint32_t (&off)[ScanShape<MPAD>::S / 4],
                                           const Sel& sel, uint32_t (&sum)[NPMAX]) {
    uint32_t all = 0, o1 = 0, o3 = 0;
    block_sums_chunk<MPAD, NPV, 0>(w, off, sel, all, o1, o3);
    // cells: pair 0 = byte 0, pair 1 = byte 2, pair 2 = byte 1, pair 3 = byte 3
    const uint32_t s2 = (o1 & 0xFFFFu) + (o1 >> 16), s3 = (o3 & 0xFFFFu) + (o3 >> 16);
    uint32_t even = all;
    if (NPV >= 3) even -= s2 << 8;
    if (NPV >= 4) even -= s3 << 24;
    sum[0] = even & 0xFFFFu;
    sum[1] = even >> 16;
    sum[2] = s2;
    sum[3] = s3;
}

__device__ __forceinline__ int cell_byte(int pair_slot) { return pair_slot == 0 ? 0 : (pair_slot == 1 ? 2 : (pair_slot == 2 ? 1 : 3)); }

// Everything a wave holds of a task before the task's tables are in LDS: the scalars of its
// descriptor and, in flight from HBM, its share of the tables, the first 64 patches of each
// pair and the query's current bound.
struct Task {
    int tid, chunk, np, nb, cvecs;
    int pair[NPMAX], bias[NPMAX], qq[NPMAX], namb[NPMAX];
    const uint8_t* base;     // first code block of the chunk
    unsigned use, evalm;     // cells with a base table / cells evaluated entry by entry
    bool same;               // the cells already hold these queries' base tables
};

template <int MPAD>
struct TableRegs {
    static constexpr int PER = ScanShape<MPAD>::PLANES * 1024 / ScanShape<MPAD>::NT;
    static_assert(ScanShape<MPAD>::PLANES * 1024 % ScanShape<MPAD>::NT == 0, "pieces must divide over the threads");
    u32x2 a[PER], b[PER], c[PER], d[PER];
    uint32_t pa[NPMAX], pv[NPMAX];
    int32_t tau;
};

// Interleave up to four plane-major tables (HBM, [plane][c][slot] bytes) into the LDS table
// region: dword (plane, c, slot) = {src0, src2, src1, src3} bytes; `use` bit s clear = zeros in
// that cell.  Piece p = 8 consecutive entries (8 source bytes per table, 32 bytes of LDS),
// handled by thread p mod NT.  Loading and storing are separate so that the round trip to HBM
// overlaps the end of the previous task.
template <int MPAD>
__device__ __forceinline__ void load_tables(TableRegs<MPAD>& R, const uint8_t* s0, const uint8_t* s1, const uint8_t* s2,
                                            const uint8_t* s3) {
    // every source pointer must be readable (absent tables alias a present one)
#pragma unroll
    for (int r = 0; r < TableRegs<MPAD>::PER; ++r) {
        const int p = threadIdx.x + r * ScanShape<MPAD>::NT;
        R.a[r] = ((global_u32x2_ptr)s0)[p];
        R.b[r] = ((global_u32x2_ptr)s1)[p];
        R.c[r] = ((global_u32x2_ptr)s2)[p];
        R.d[r] = ((global_u32x2_ptr)s3)[p];
    }
}

template <int MPAD>
__device__ __forceinline__ void store_tables(const TableRegs<MPAD>& R, unsigned use, uint8_t* lut) {
    const uint32_t m0 = (use & 1u) ? ~0u : 0u, m1 = (use & 2u) ? ~0u : 0u, m2 = (use & 4u) ? ~0u : 0u, m3 = (use & 8u) ? ~0u : 0u;
#pragma unroll
    for (int r = 0; r < TableRegs<MPAD>::PER; ++r) {
        const int p = threadIdx.x + r * ScanShape<MPAD>::NT;
        uint4 out[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t aw = (h ? R.a[r].y : R.a[r].x) & m0, bw = (h ? R.b[r].y : R.b[r].x) & m1;
            const uint32_t cw = (h ? R.c[r].y : R.c[r].x) & m2, dw = (h ? R.d[r].y : R.d[r].x) & m3;
            // bytes 0 and 1 of a dword come from tables 0 and 2, bytes 2 and 3 from tables 1 and 3
            const uint32_t lo01 = __builtin_amdgcn_perm(cw, aw, 0x05010400u), lo23 = __builtin_amdgcn_perm(cw, aw, 0x07030602u);
            const uint32_t hi01 = __builtin_amdgcn_perm(dw, bw, 0x05010400u), hi23 = __builtin_amdgcn_perm(dw, bw, 0x07030602u);
            out[h] = make_uint4(__builtin_amdgcn_perm(hi01, lo01, 0x05040100u), __builtin_amdgcn_perm(hi01, lo01, 0x07060302u),
                                __builtin_amdgcn_perm(hi23, lo23, 0x05040100u), __builtin_amdgcn_perm(hi23, lo23, 0x07060302u));
        }
        uint4* dst = reinterpret_cast<uint4*>(lut + (int64_t)p * 32);
        dst[0] = out[0];
        dst[1] = out[1];
    }
}

// Full per-pair evaluation of a table straight into its LDS cells (queries whose tables are too
// flat for the base + patch form).
template <int NT>
__device__ __forceinline__ void eval_table(const ScanParams& P, int pair, int q, uint8_t* cell) {
    const int m = P.m, S = rago_steps(m);
    const float dq = lut_step(__uint_as_float(P.T.range_bits[q]));
    for (int e = threadIdx.x; e < m * KSUB; e += NT) {
        const int j = e >> 8, c = e & 255;
        const double t = P.T.t64[(int64_t)pair * m + j];
        const uint8_t v = lut_entry(P.T.T64[((int64_t)q * m + j) * KSUB + c], t, (float)(P.T.Tmin[(int64_t)q * m + j] + t), dq);
        for (int rep = j & (S - 1); rep < 32; rep += S) cell[((j >> 5) * LUT_PLANE + c * 32 + rep) * 4] = v;
    }
}

// Claim the next task and put everything its prologue needs into LDS (run by ONE wave; all
// values are wave-uniform so the loads are scalar).  d[0] = task number or -1 when none is left.
// d[1] list, d[2] chunk, d[3] pairs in the task, d[4..7] pair, d[8..11] bias, d[12..15] query,
// d[16..19] ambiguous entries of the query, d[20..21] first block, d[22] blocks of the list,
// d[23..24] first vector, d[25] vectors of the list.
__device__ __forceinline__ void fetch_task(const ScanParams& P, int ntasks, int32_t* d, int lane) {
    int t = 0;
    if (lane == 0) t = atomicAdd(P.ctrl, 1);
    t = __builtin_amdgcn_readfirstlane(t);
    if (t >= ntasks) {
        if (lane == 0) d[0] = -1;
        return;
    }
    const int4 rec = P.task_table[t];
    const int l = rec.x, np = rec.w;
    const int64_t b0 = P.blk_off[l], v0 = P.list_off[l];
    const int nblk = (int)(P.blk_off[l + 1] - b0), len = (int)(P.list_off[l + 1] - v0);
    int pr[NPMAX], q[NPMAX], bias[NPMAX], na[NPMAX];
#pragma unroll
    for (int s = 0; s < NPMAX; ++s) {
        pr[s] = P.pair_sorted[rec.z + (s < np ? s : 0)];
        q[s] = pr[s] / P.nprobe;
        bias[s] = P.bias[pr[s]];
        na[s] = P.lut8sw ? 0 : P.T.namb[q[s]];
    }
    if (lane == 0) {
        d[0] = t; d[1] = l; d[2] = rec.y; d[3] = np;
#pragma unroll
        for (int s = 0; s < NPMAX; ++s) { d[4 + s] = pr[s]; d[8 + s] = bias[s]; d[12 + s] = q[s]; d[16 + s] = na[s]; }
        d[20] = (int32_t)(uint32_t)b0; d[21] = (int32_t)(b0 >> 32); d[22] = nblk;
        d[23] = (int32_t)(uint32_t)v0; d[24] = (int32_t)(v0 >> 32); d[25] = len;
    }
}

// A finished task's result (<= k entries per pair) is produced by one wave per pair cell from the
// keys of all the workgroup's buffers of that cell, between the barrier that ends the task's
// stream and the one that starts the next task's.  The keys stay in the LDS buffers and are
// re-read on every pass (a register copy of up to 2 x NW keys per lane would have to live
// alongside the next task's table data, which is in flight at this point).
//
// When the buffers hold k keys or more, the k-th largest is found by 8-bit radix passes over a
// 256-bin LDS histogram owned by the wave (a ballot radix select costs 32 wave-wide votes per
// key register, far too many here).  The passes start at the highest bit on which the keys
// differ: the bits above it are common to all keys, and a histogram of them would pile every key
// onto one LDS address.
template <int NW, class F>
__device__ __forceinline__ void for_each_key(const uint32_t* cand, int s, int myn, int lane, F f) {
#pragma unroll 4
    for (int w = 0; w < NW; ++w) {
        const int n = __builtin_amdgcn_readlane(myn, w);
        const uint32_t* bw = cand + (w * NPMAX + s) * CAPW;
        const uint32_t k0 = bw[lane], k1 = bw[lane + 64];       // (inside the buffer's CAPW entries whatever its fill)
        f(lane < n ? k0 : 0u);
        f(lane + 64 < n ? k1 : 0u);
    }
}

template <int NW>
__device__ __forceinline__ uint32_t select_kth_lds(const uint32_t* cand, int s, int myn, int k, uint32_t* hist, int lane) {
    uint32_t orv = 0u, andv = ~0u;
    for_each_key<NW>(cand, s, myn, lane, [&](uint32_t key) {
        orv |= key;
        andv &= key ? key : ~0u;
    });
#pragma unroll
    for (int o = 32; o; o >>= 1) {
        orv |= __shfl_xor(orv, o);
        andv &= __shfl_xor(andv, o);
    }
    orv = __builtin_amdgcn_readfirstlane(orv);
    andv = __builtin_amdgcn_readfirstlane(andv);
    const uint32_t vary = orv & ~andv;
    if (vary == 0u) return orv;                    // one distinct key
    const int hb = 31 - __builtin_clz(vary);
    uint32_t mask = hb == 31 ? 0u : ~((2u << hb) - 1u);   // bits decided so far
    uint32_t prefix = orv & mask;
    int rem = k;
    for (int shift = hb > 7 ? hb - 7 : 0;; shift = shift > 8 ? shift - 8 : 0) {
        reinterpret_cast<uint4*>(hist)[lane] = make_uint4(0u, 0u, 0u, 0u);   // (LDS operations of one wave execute in order)
        for_each_key<NW>(cand, s, myn, lane, [&](uint32_t key) {
            if (key != 0u && (key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
        });
        const uint4 h = reinterpret_cast<const uint4*>(hist)[lane];          // bins 4*lane .. 4*lane + 3
        const int c = (int)(h.x + h.y + h.z + h.w);
        int sfx = c;                                                           // keys in this lane's bins and all higher ones
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_down(sfx, o);
            if (lane + o < 64) sfx += t;
        }
        const uint64_t reach = __ballot(sfx >= rem);                           // never empty: at least `rem` keys match the prefix
        const int L = 63 - __builtin_clzll(reach);
        int need = rem - (__builtin_amdgcn_readlane(sfx, L) - __builtin_amdgcn_readlane(c, L));
        const int hw = __builtin_amdgcn_readlane((int)h.w, L), hz = __builtin_amdgcn_readlane((int)h.z, L);
        const int hy = __builtin_amdgcn_readlane((int)h.y, L);
        int dgt;
        if (hw >= need) dgt = 3;
        else if (hw + hz >= need) { dgt = 2; need -= hw; }
        else if (hw + hz + hy >= need) { dgt = 1; need -= hw + hz; }
        else { dgt = 0; need -= hw + hz + hy; }
        rem = need;
        // (a window may overlap bits decided before: the keys still in play agree on them)
        prefix = (prefix & ~(255u << shift)) | ((uint32_t)(4 * L + dgt) << shift);
        mask |= 255u << shift;
        if (shift == 0) break;
    }
    return prefix;
}

template <int NW>
__device__ __forceinline__ void merge_task(const ScanParams& P, const int32_t* D, int s, const uint32_t* cand, const int32_t* sh,
                                           uint32_t* hist, int lane) {
    const int k = P.k;
    const int chunk = __builtin_amdgcn_readfirstlane(D[2]);
    const int pr = __builtin_amdgcn_readfirstlane(D[4 + s]), bias = __builtin_amdgcn_readfirstlane(D[8 + s]);
    const int q = __builtin_amdgcn_readfirstlane(D[12 + s]);
    const int64_t v0 = ((int64_t)__builtin_amdgcn_readfirstlane(D[24]) << 32) | (uint32_t)__builtin_amdgcn_readfirstlane(D[23]);
    const int myn = lane < NW ? sh[8 + lane * NPMAX + s] : 0;     // lane w: fill of wave w's buffer
    int total = myn;
#pragma unroll
    for (int o = 32; o; o >>= 1) total += __shfl_xor(total, o);
    total = __builtin_amdgcn_readfirstlane(total);
    uint32_t kth = 1u;
    if (total >= k) kth = select_kth_lds<NW>(cand, s, myn, k, hist, lane);
    const int64_t slot = (int64_t)pr * P.maxchunks + chunk;
    int32_t* oI = P.part_I + slot * k;
    int64_t* orow = P.part_row + slot * k;
    // (rows, not ids: translating them here would put a dependent HBM round trip into every step
    // of this loop; the final merge looks up the ids of the few entries that survive)
    const int64_t row0 = v0 + (int64_t)chunk * P.CH * BLOCK_VECS;
    int base_o = 0;
    for_each_key<NW>(cand, s, myn, lane, [&](uint32_t key) {
        const bool keep = key >= kth && key != 0u;
        const uint64_t mask = __ballot(keep);
        if (mask != 0) {
            if (keep) {
                const int o = base_o + lane_rank(mask);
                oI[o] = bias + (int32_t)(key >> 16);
                orow[o] = row0 + (int64_t)(0xFFFFu - (key & 0xFFFFu));
            }
            base_o += __popcll(mask);
        }
    });
    if (lane == 0) {
        P.part_cnt[slot] = base_o;
        // k entries reach the k-th key's score: a valid lower bound of the query's k-th best
        if (total >= k) publish_bound(P.tauq + q, bias + (int32_t)(kth >> 16));
    }
}

// ------------------------------------------------------------------ the scan kernel
// Per task: [install] tables from registers into LDS, patches, thresholds - barrier - [stream] -
// next task's descriptor (first wave to finish) and, as soon as a wave has that descriptor, its
// share of the next task's table loads - trim own buffers - barrier - [merge] (one wave per pair)
// while the table loads are in flight - back to [install].
template <int MPAD>
__global__ void __launch_bounds__(ScanShape<MPAD>::NT) scan_kernel(const ScanParams P) {
    using SH = ScanShape<MPAD>;
    constexpr int S = SH::S, NW = SH::NW, NT = SH::NT;
    extern __shared__ __align__(16) uint8_t smem[];
    uint8_t* lut = smem;
    uint32_t* cand = reinterpret_cast<uint32_t*>(smem + SH::LUT_LDS);                          // [wave][pair][CAPW]
    int32_t* sh = reinterpret_cast<int32_t*>(smem + SH::LUT_LDS + NW * NPMAX * CAPW * 4);      // scalars
    uint32_t* hist = reinterpret_cast<uint32_t*>(sh + SH_INTS);                                // [pair][256] merge histograms
    // sh[0..3] tau per pair (sum units), sh[4] block counter, sh[5] finisher ticket,
    // sh[8 + wave*4 + pair] wave counts, sh[80..] three task descriptors
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

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
    const int ntasks = P.ctrl[1];
    int loaded0 = -3, loaded1 = -3, loaded2 = -3, loaded3 = -3;   // query whose base table sits in each cell (-2: zeros)
    Sel sel{RAGO_SEL_A, RAGO_SEL_B, RAGO_SEL_O1, RAGO_SEL_O3};
    const int k = P.k;
    int32_t* desc = sh + 80;          // ring of three task descriptors: the previous (being merged) / running task, the next, the one after
    constexpr int64_t BLK_BYTES = BLOCK_VECS * MPAD;

    uint4 cur_w[MPAD / 16], nxt_w[MPAD / 16];
    TableRegs<MPAD> R;

    // descriptor -> task scalars (all wave-uniform)
    auto decode = [&](const int32_t* D, Task& T) {
        T.tid = __builtin_amdgcn_readfirstlane(D[0]);
        T.chunk = __builtin_amdgcn_readfirstlane(D[2]);
        T.np = __builtin_amdgcn_readfirstlane(D[3]);
#pragma unroll
        for (int s = 0; s < NPMAX; ++s) {
            T.pair[s] = __builtin_amdgcn_readfirstlane(D[4 + s]);
            T.bias[s] = __builtin_amdgcn_readfirstlane(D[8 + s]);
            T.qq[s] = __builtin_amdgcn_readfirstlane(D[12 + s]);
            T.namb[s] = __builtin_amdgcn_readfirstlane(D[16 + s]);
        }
        const int64_t b0 = ((int64_t)__builtin_amdgcn_readfirstlane(D[21]) << 32) | (uint32_t)__builtin_amdgcn_readfirstlane(D[20]);
        const int nblk_list = __builtin_amdgcn_readfirstlane(D[22]);
        const int len = __builtin_amdgcn_readfirstlane(D[25]);
        const int cb0 = T.chunk * P.CH;
        T.nb = min(P.CH, nblk_list - cb0);
        T.cvecs = min(len - cb0 * BLOCK_VECS, T.nb * BLOCK_VECS);
        T.base = P.codes + (b0 + cb0) * BLK_BYTES;
        T.use = 0; T.evalm = 0;
        if (P.lut8sw) {
            T.use = (1u << T.np) - 1u;
            T.same = false;
        } else {
            int want[NPMAX];
#pragma unroll
            for (int s = 0; s < NPMAX; ++s) {
                want[s] = s < T.np ? (T.namb[s] <= AMB_MAX ? T.qq[s] : -1) : -2;
                if (want[s] >= 0) T.use |= 1u << s;
                if (want[s] == -1) T.evalm |= 1u << s;
            }
            // (the cells hold the running task's tables by the time this one is installed)
            T.same = want[0] == loaded0 && want[1] == loaded1 && want[2] == loaded2 && want[3] == loaded3 && T.evalm == 0;
        }
    };
    // everything of a task that comes from HBM before its stream: requested as early as possible.
    // (every field of R is written on every path, with zeros where nothing is loaded: a field that
    // is only written under a condition keeps its old value alive across the whole task loop, and
    // the table registers then get spilled)
    auto issue_tables = [&](const int32_t* D, const Task& T) {
        const bool live = T.tid >= 0;
        R.tau = INT32_MIN;
        if (live && threadIdx.x < NPMAX && (int)threadIdx.x < T.np)
            R.tau = __hip_atomic_load(P.tauq + D[12 + threadIdx.x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (live && !P.lut8sw) {
            // (the arrays always hold AMB_MAX entries, so the first 64 can be read unconditionally)
#pragma unroll
            for (int s = 0; s < NPMAX; ++s) {
                R.pa[s] = P.T.amb_addr[(int64_t)T.qq[s] * AMB_MAX + lane];
                R.pv[s] = P.T.patch_val[(int64_t)T.pair[s] * AMB_MAX + lane];
            }
        } else {
#pragma unroll
            for (int s = 0; s < NPMAX; ++s) { R.pa[s] = 0u; R.pv[s] = 0u; }
        }
        if (live && !T.same) {
            const uint8_t* tb = P.lut8sw ? P.lut8sw : P.T.lut_base;
            const int* ix = P.lut8sw ? T.pair : T.qq;
            load_tables<MPAD>(R, tb + (int64_t)ix[0] * LUT_BYTES, tb + (int64_t)ix[1] * LUT_BYTES, tb + (int64_t)ix[2] * LUT_BYTES,
                              tb + (int64_t)ix[3] * LUT_BYTES);
        } else {
#pragma unroll
            for (int r = 0; r < TableRegs<MPAD>::PER; ++r) { R.a[r] = 0u; R.b[r] = 0u; R.c[r] = 0u; R.d[r] = 0u; }
        }
    };

    // Descriptors are claimed TWO tasks ahead: the one a wave needs when it finishes its share of the
    // running task (to request the next task's tables) is then always in place, on every wave, at the
    // same point of the program.
    if (wave == NW - 1) {
        fetch_task(P, ntasks, desc, lane);
        fetch_task(P, ntasks, desc + DESC_INTS, lane);
    }
    __syncthreads();
    Task T;
    decode(desc, T);
    if (T.tid < 0) return;            // nothing to do (every wave reads the same descriptor)
    issue_tables(desc, T);
    // The wave's first block.  The stream's loads are issued unconditionally and at fixed places of
    // the program, this one included: the compiler counts outstanding loads statically, and a load
    // that is issued on some paths only makes it wait for ALL outstanding loads before each use.
    load_block<MPAD, true>(cur_w, T.base + (int64_t)min(wave, T.nb - 1) * BLK_BYTES, lane);
    bool have_prev = false;
    for (int cur = 0;; cur = cur == 2 ? 0 : cur + 1) {
        const int32_t* D = desc + cur * DESC_INTS;
        const int nxt = cur == 2 ? 0 : cur + 1, prv = cur == 0 ? 2 : cur - 1;   // ring positions of the next / previous task
        // ---- result of the previous task: one wave per pair
        if (have_prev) {
            const int32_t* Dp = desc + prv * DESC_INTS;
            if (wave < __builtin_amdgcn_readfirstlane(Dp[3])) merge_task<NW>(P, Dp, wave, cand, sh, hist + wave * 256, lane);
        }
        if (T.tid < 0) break;         // every wave reads the same descriptor: all leave together
        const int np = T.np;

        // ---- install: tables into LDS, patches, thresholds
        if (!T.same) store_tables<MPAD>(R, T.use, lut);
        if (T.evalm) {                // rare: the cells' dwords are shared, so the other tables must be in place first
            __syncthreads();
#pragma unroll
            for (int s = 0; s < NPMAX; ++s)
                if (T.evalm & (1u << s)) eval_table<NT>(P, T.pair[s], T.qq[s], lut + cell_byte(s));
        }
        if (!P.lut8sw) {
            // Patches are written by the wave that copies the 32-byte piece they fall into, so program
            // order inside the wave puts them after the copy and no workgroup barrier is needed in between.
            auto owner = [](uint32_t e) { return (int)(((e >> 3) & (uint32_t)(NT - 1)) >> 6); };
#pragma unroll
            for (int s = 0; s < NPMAX; ++s) {
                if (!(T.use & (1u << s))) continue;
                if (lane < T.namb[s] && owner(R.pa[s]) == wave) lut[R.pa[s] * 4 + cell_byte(s)] = (uint8_t)R.pv[s];
                for (int i = 64 + lane; i < T.namb[s]; i += 64) {
                    const uint32_t e = P.T.amb_addr[(int64_t)T.qq[s] * AMB_MAX + i];
                    if (owner(e) == wave) lut[e * 4 + cell_byte(s)] = P.T.patch_val[(int64_t)T.pair[s] * AMB_MAX + i];
                }
            }
#pragma unroll
            for (int s = 0; s < NPMAX; ++s) {
                const int w = s < np ? (T.namb[s] <= AMB_MAX ? T.qq[s] : -1) : -2;
                if (s == 0) loaded0 = w; else if (s == 1) loaded1 = w; else if (s == 2) loaded2 = w; else loaded3 = w;
            }
        }
        if (threadIdx.x < NPMAX) {
            const int s = threadIdx.x;
            int32_t t0 = 0;
            if (s < np) {
                const int64_t t = (int64_t)R.tau - D[8 + s];
                t0 = t <= 0 ? 0 : (t > 0x7fffffff ? 0x7fffffff : (int32_t)t);
            }
            sh[s] = t0;
            if (s == 0) { sh[4] = NW; sh[5] = 0; }   // next unclaimed block; finisher ticket
        }
        __syncthreads();

        // ---- stream the chunk: wave w starts with block w, further blocks are claimed from an LDS counter
        // (a wave that was held up - the one that fetched the next task, one that pruned - simply takes fewer)
        const uint8_t* base = T.base;
        const int nb = T.nb, cvecs = T.cvecs;
        int b = wave;
        int cnt[NPMAX] = {0, 0, 0, 0};
        uint32_t thr[NPMAX];
#pragma unroll
        for (int s = 0; s < NPMAX; ++s) thr[s] = (uint32_t)sh[s];
        auto claim = [&]() {
            int v = 0;
            if (lane == 0) v = atomicAdd(&sh[4], 1);
            return __builtin_amdgcn_readfirstlane(v);
        };
        // (unconditional loads, the block number clamped into the chunk)
        auto stream = [&](auto npv_tag) {
            constexpr int NPV = decltype(npv_tag)::value;
            auto process = [&](const uint4 (&w)[MPAD / 16], int blk) {
                const uint32_t pos = (uint32_t)(blk * BLOCK_VECS + lane);
                const bool valid = (int)pos < cvecs;
                uint32_t sum[NPMAX];
                block_sums<MPAD, NPV>(w, off, sel, sum);
#pragma unroll
                for (int s = 0; s < NPV; ++s) {
                    if (s < np) {
                        const uint32_t ta = (uint32_t)sh[s];
                        if (ta > thr[s]) thr[s] = ta;
                        offer(valid, sum[s], pos, cand + (wave * NPMAX + s) * CAPW, cnt[s], thr[s], sh + s, k, lane);
                    }
                }
            };
            int bn = claim();
            load_block<MPAD, true>(nxt_w, base + (int64_t)min(bn, nb - 1) * BLK_BYTES, lane);
            while (b < nb) {                       // ping-pong between the two register sets
                process(cur_w, b);
                b = claim();
                load_block<MPAD, true>(cur_w, base + (int64_t)min(b, nb - 1) * BLK_BYTES, lane);
                if (bn >= nb) break;               // claims are monotonic: nothing newer can be valid either
                process(nxt_w, bn);
                bn = claim();
                load_block<MPAD, true>(nxt_w, base + (int64_t)min(bn, nb - 1) * BLK_BYTES, lane);
            }
        };
        if (np <= 2) stream(std::integral_constant<int, 2>{});
        else if (np == 3) stream(std::integral_constant<int, 3>{});
        else stream(std::integral_constant<int, 4>{});
        // ---- the next task's tables, patches and bound: requested by every wave as soon as it has run out of blocks
        const int32_t* Dn = desc + nxt * DESC_INTS;
        Task Tn;
        decode(Dn, Tn);
        issue_tables(Dn, Tn);
        // (and the wave's first block of it; after the last task: any readable block)
        load_block<MPAD, true>(cur_w, Tn.tid >= 0 ? Tn.base + (int64_t)min(wave, Tn.nb - 1) * BLK_BYTES : T.base, lane);
        // ---- the first wave to run out of blocks claims the task after the next while the others finish (its
        // descriptor replaces the previous task's, whose merge ended before this task's stream began)
        {
            int ticket = 0;
            if (lane == 0) ticket = atomicAdd(&sh[5], 1);
            if (__builtin_amdgcn_readfirstlane(ticket) == 0) {
                if (Tn.tid >= 0) fetch_task(P, ntasks, desc + prv * DESC_INTS, lane);
                else if (lane == 0) desc[prv * DESC_INTS] = -1;
            }
        }
        // ---- every wave trims its buffers to k
#pragma unroll
        for (int s = 0; s < NPMAX; ++s) {
            if (s < np && cnt[s] > k) wave_prune(cand + (wave * NPMAX + s) * CAPW, cnt[s], k, lane);
            if (lane == 0) sh[8 + wave * NPMAX + s] = cnt[s];
        }
        __syncthreads();
        T = Tn;
        have_prev = true;
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

// `phase` 0: only each query's best list (probe rank 0), 1: only the other ranks, 2: all pairs.  Lists
// are scanned in the order they are registered here; running phase 0 before phase 1 puts every
// query's best list among the first tasks, so its bound on the k-th best score is tight early and
// fewer of its later tasks collect k candidates or more.
__global__ void __launch_bounds__(256) count_pairs_kernel(const int32_t* __restrict__ probes, int64_t npairs, int nprobe, int phase,
                                                          int32_t* __restrict__ list_cnt, int32_t* __restrict__ touched,
                                                          int32_t* __restrict__ ctrl) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int lane = threadIdx.x & 63;
    int l = -1;
    bool first = false;
    const bool mine = i < npairs && (phase == 2 || ((i % nprobe) == 0) == (phase == 0));
    if (mine) {
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
                                                             int CH, int group, int m, int64_t max_n, const int32_t* __restrict__ ctrl,
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
        vt[i] = ((c + group - 1) / group) * ((nblk + CH - 1) / CH);
        streamed = (unsigned long long)((c + group - 1) / group) * nblk * (BLOCK_VECS * m);
        algo = (unsigned long long)c * (unsigned long long)(list_off[l + 1] - list_off[l]) * m;
    }
    for (int o = 32; o; o >>= 1) { streamed += __shfl_xor(streamed, o); algo += __shfl_xor(algo, o); }
    if ((threadIdx.x & 63) == 0 && (streamed | algo)) {
        atomicAdd(reinterpret_cast<unsigned long long*>(counters + 1), streamed);
        atomicAdd(reinterpret_cast<unsigned long long*>(counters + 2), algo);
    }
}

// Exclusive prefix sums (in place) of the per-list pair and task counts: one workgroup; a thread takes eight
// consecutive entries per tile (two 16-byte loads per array), so a tile is 8192 entries and the number of
// load -> wave scan -> barrier rounds, each of which costs a memory latency, is n / 8192.
__global__ void __launch_bounds__(1024) touched_scan_kernel(int32_t* __restrict__ vp, int32_t* __restrict__ vt,
                                                            int32_t* __restrict__ ctrl, int64_t* __restrict__ counters) {
    __shared__ int s_wp[16], s_wt[16];
    constexpr int E = 8;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int n = ctrl[2];
    int carry_p = 0, carry_t = 0;
    for (int base = 0; base < n; base += 1024 * E) {
        const int i0 = base + t * E;
        int p[E], q[E];
        if (i0 + E <= n) {
            const int4 a0 = *reinterpret_cast<const int4*>(vp + i0), a1 = *reinterpret_cast<const int4*>(vp + i0 + 4);
            const int4 b0 = *reinterpret_cast<const int4*>(vt + i0), b1 = *reinterpret_cast<const int4*>(vt + i0 + 4);
            p[0] = a0.x; p[1] = a0.y; p[2] = a0.z; p[3] = a0.w; p[4] = a1.x; p[5] = a1.y; p[6] = a1.z; p[7] = a1.w;
            q[0] = b0.x; q[1] = b0.y; q[2] = b0.z; q[3] = b0.w; q[4] = b1.x; q[5] = b1.y; q[6] = b1.z; q[7] = b1.w;
        } else {
#pragma unroll
            for (int e = 0; e < E; ++e) { p[e] = i0 + e < n ? vp[i0 + e] : 0; q[e] = i0 + e < n ? vt[i0 + e] : 0; }
        }
        int sp = 0, sq = 0;
#pragma unroll
        for (int e = 0; e < E; ++e) { sp += p[e]; sq += q[e]; }
        int ip = sp, it = sq;                      // inclusive scan of the threads' sums across the wave
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
        int ep = carry_p + wp + ip - sp, et = carry_t + wt + it - sq;      // exclusive prefix of this thread's first entry
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int pe = p[e], qe = q[e];
            p[e] = ep; q[e] = et;
            ep += pe; et += qe;
        }
        if (i0 + E <= n) {
            *reinterpret_cast<int4*>(vp + i0) = make_int4(p[0], p[1], p[2], p[3]);
            *reinterpret_cast<int4*>(vp + i0 + 4) = make_int4(p[4], p[5], p[6], p[7]);
            *reinterpret_cast<int4*>(vt + i0) = make_int4(q[0], q[1], q[2], q[3]);
            *reinterpret_cast<int4*>(vt + i0 + 4) = make_int4(q[4], q[5], q[6], q[7]);
        } else {
#pragma unroll
            for (int e = 0; e < E; ++e)
                if (i0 + e < n) { vp[i0 + e] = p[e]; vt[i0 + e] = q[e]; }
        }
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
                                                         const int32_t* __restrict__ touched, int group,
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
    const int ngroups = (npl + group - 1) / group;
    const int chunk = rem / ngroups, grp = rem - chunk * ngroups;   // groups of one chunk are consecutive tasks
    // the list's pairs are spread evenly over its groups (5 pairs = 3 + 2, not 4 + 1: fewer cells per look-up)
    const int per = npl / ngroups, extra = npl - per * ngroups;
    const int first = grp * per + min(grp, extra);
    table[t] = make_int4(touched[lo], chunk, pair_off[lo] + first, per + (grp < extra ? 1 : 0));
}

// All of the above in one workgroup, for batches of at most SSU_PAIRS pairs (scan_setup.h).
__global__ void __launch_bounds__(SSU_THREADS) small_setup_kernel(const SmallSetupArgs A) {
    extern __shared__ __align__(16) int32_t ssu[];
    small_setup_body(A, ssu);
}

// ------------------------------------------------------------------ per-query merge of the task results
// NT threads: 256 when a batch brings a workgroup per compute unit or more, 1024 for the few queries of a latency-bound round.
template <int NT>
__global__ void __launch_bounds__(NT) merge_kernel(const ScanParams P, const float* __restrict__ delta,
                                                              int64_t* __restrict__ out_ids, float* __restrict__ out_scores,
                                                              int32_t* __restrict__ out_iscores) {
    __shared__ __align__(16) int32_t sI[MERGE_CAP];
    __shared__ int64_t sId[MERGE_CAP];
    __shared__ int s_cnt;
    constexpr int MERGE_TILE = 2048;
    __shared__ __align__(8) int s_slot[MERGE_TILE];      // per slot of the current tile: (place in the result arrays << 8) | entries
    static_assert(MERGE_TILE >= 3 * RANK_CAND + 1 && MERGE_CAP >= 1024 + 4, "rank_top_k's side buffer and padding");
    const int q = blockIdx.x, k = P.k;
    int32_t tau = P.tauq[q];   // k candidates of this query reach tau: nothing below can be in the result
    // Slots = (probe, chunk) pairs that exist: chunk counts per probe are prefix-summed in LDS
    // (s_pre), then one thread per slot reads the slot's count and its few surviving entries.
    __shared__ int s_pre[2049];            // nprobe <= 2048 (enforced by the selection stage / argument check)
    for (int p = threadIdx.x; p < P.nprobe; p += NT) {
        const int l = P.probes[q * P.nprobe + p];
        const int nblk = (int)(P.blk_off[l + 1] - P.blk_off[l]);
        s_pre[p + 1] = (nblk + P.CH - 1) / P.CH;
    }
    if (threadIdx.x == 0) s_pre[0] = 0;
    __syncthreads();
    {
        // inclusive prefix sum of s_pre[1 .. nprobe]: every thread sums a run of consecutive entries, the runs'
        // totals are scanned inside each wave (shuffles) and across the waves (LDS), then each run is rewritten
        __shared__ int s_wsum[NT / 64];
        const int per = (P.nprobe + NT - 1) / NT;       // <= 8
        const int a = 1 + threadIdx.x * per, b = min(a + per, P.nprobe + 1);
        int run = 0;
        for (int i = a; i < b; ++i) run += s_pre[i];
        int inc = run;
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        for (int o = 1; o < 64; o <<= 1) {
            const int v = __shfl_up(inc, o);
            if (lane >= o) inc += v;
        }
        if (lane == 63) s_wsum[wave] = inc;
        __syncthreads();
        int before = inc - run;
        for (int w = 0; w < wave; ++w) before += s_wsum[w];
        for (int i = a; i < b; ++i) { before += s_pre[i]; s_pre[i] = before; }
    }
    __syncthreads();
    const int nslots = s_pre[P.nprobe];
    auto gather = [&](int s0, int s1, int base_fill) {
        if (threadIdx.x == 0) s_cnt = base_fill;
        __syncthreads();
        // 256 slots at a time, dealt to the four waves in turn; a lane reads its slot's count, a scan over the wave
        // turns the 64 counts into offsets, and then the wave's lanes share out ALL entries of its 64 slots evenly
        // (entry e belongs to the slot whose offset range holds e).  A thread per slot would walk up to k entries
        // one after the other, each a dependent trip to memory; a wave per slot idles when slots hold few entries.
        __shared__ int s_wpre[NT / 64][64];
        __shared__ int64_t s_wgs[NT / 64][64];
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        if ((int64_t)P.nprobe * P.maxchunks < (1 << 23)) {
            // Tiles of MERGE_TILE slots.  A thread per slot finds the slot's place in the result arrays and reads its
            // count (neighbouring slots are neighbours in memory); both go into one LDS word.  Then the tile's
            // entries are walked as one flat array, entry f = slot f / k, position f % k: neighbouring lanes read
            // neighbouring words, stale positions beyond a slot's count are skipped.  (A thread per slot reading its
            // k entries itself makes every load instruction touch 64 cache lines, and the merge of one query's
            // 2000 slots took 38 us in the address unit.)
            const int64_t qbase = (int64_t)q * P.nprobe * P.maxchunks;
            constexpr int U = 4;
            for (int t0 = s0; t0 < s1; t0 += MERGE_TILE) {
                const int ts = min(MERGE_TILE, s1 - t0);
                __syncthreads();
                for (int j = threadIdx.x; j < ts; j += NT) {
                    const int sl = t0 + j;
                    int lo = 0, hi = P.nprobe;
                    while (hi - lo > 1) {
                        const int mid = (lo + hi) >> 1;
                        if (s_pre[mid] <= sl) lo = mid; else hi = mid;
                    }
                    const int rel = lo * P.maxchunks + (sl - s_pre[lo]);
                    s_slot[j] = (rel << 8) | P.part_cnt[qbase + rel];       // counts are <= k <= 128
                }
                __syncthreads();
                const int total = ts * k;
                for (int f0 = threadIdx.x; f0 < total; f0 += NT * U) {
                    int32_t I[U];
                    int64_t at[U];
                    bool live[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int f = f0 + u * NT;
                        const int j = min(f / k, ts - 1), r = f - j * k;
                        const int word = s_slot[j];
                        live[u] = f < total && r < (word & 255);
                        at[u] = (qbase + (word >> 8)) * k + (live[u] ? r : 0);
                        I[u] = P.part_I[at[u]];
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        if (live[u] && I[u] >= tau) {
                            const int o = atomicAdd(&s_cnt, 1);
                            if (o < MERGE_CAP) { sI[o] = I[u]; sId[o] = P.ids[P.part_row[at[u]]]; }
                        }
                    }
                }
            }
        } else
        for (int b = s0; b < s1; b += NT) {
            const int sl = b + lane * (NT / 64) + wave;
            int n = 0;
            int64_t gs = 0;
            if (sl < s1) {
                int lo = 0, hi = P.nprobe;     // probe p with s_pre[p] <= sl < s_pre[p + 1]
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    if (s_pre[mid] <= sl) lo = mid; else hi = mid;
                }
                gs = ((int64_t)q * P.nprobe + lo) * P.maxchunks + (sl - s_pre[lo]);
                n = P.part_cnt[gs];
            }
            int inc = n;
            for (int o = 1; o < 64; o <<= 1) {
                const int v = __shfl_up(inc, o);
                if (lane >= o) inc += v;
            }
            const int total = __shfl(inc, 63);
            s_wpre[wave][lane] = inc - n;
            s_wgs[wave][lane] = gs;
            __builtin_amdgcn_wave_barrier();       // (a wave's LDS operations complete in order; this only pins the compiler)
            for (int e = lane; e < total; e += 64) {
                int lo = 0, hi = 64;               // the last slot whose offset is <= e (empty slots share an offset with their successor)
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    if (s_wpre[wave][mid] <= e) lo = mid; else hi = mid;
                }
                const int64_t g = s_wgs[wave][lo];
                const int r = e - s_wpre[wave][lo];
                const int32_t I = P.part_I[g * k + r];
                if (I >= tau) {
                    const int o = atomicAdd(&s_cnt, 1);
                    if (o < MERGE_CAP) { sI[o] = I; sId[o] = P.ids[P.part_row[g * k + r]]; }
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
        __syncthreads();
        return s_cnt;
    };
    auto sort_keep_k = [&](int have) {
        // (the tile words are no longer needed)
        if (NT >= 1024 && have <= NT && have > 1 && rank_top_k(sI, sId, have, k, s_slot)) return min(have, k);
        int n2 = 1;
        while (n2 < have) n2 <<= 1;
        for (int i = have + threadIdx.x; i < n2; i += NT) { sI[i] = INT32_MIN; sId[i] = INT64_MAX; }
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
    for (int r = threadIdx.x; r < k; r += NT) {
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
    static OncePerDevice attr;
    if (attr.first()) {
        RAGO_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(scan_kernel<MPAD>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, ScanShape<MPAD>::LDS));
    }
    scan_kernel<MPAD><<<grid, ScanShape<MPAD>::NT, ScanShape<MPAD>::LDS, st>>>(P);
    RAGO_HIP(hipGetLastError());
    return RAGO_OK;
}

// Which kernel and which chunk length.  The wide kernel (four pairs per pass, one workgroup per CU) pays a
// fixed price per task that only long tasks amortise; small batches go to the narrow one (two pairs per pass,
// two workgroups per CU), short lists to the one with a wave per item (scan_wave.hip);
// rago_debug_force_scan_kernel overrides the choice (tests run every case through all three).  Chunk length: aim at ~2048 tasks.  (<= 512 blocks: the position half of a key,
// 0xFFFF - position, then never vanishes, so a key is never 0 = "empty")
enum { SCAN_WIDE = 0, SCAN_NARROW = 1, SCAN_WAVE = 2 };
struct ScanPlan { int kind; int CH, group, maxchunks; };

static int chunk_len(double npairs, double avgblk, double pairs_per_task, int cap, double tasks = 2048.0) {
    int c = 16;
    while (c < cap && npairs * avgblk / (pairs_per_task * c) > tasks) c <<= 1;
    return c;
}

static ScanPlan plan_scan(const rago_index* idx, int64_t nq, int64_t npairs, bool base_tables) {
    const double avgblk = (double)idx->total_blocks / idx->nlist;
    const int CH_wide = chunk_len((double)npairs, avgblk, nq > 1 ? 2.0 : 1.0, 512);
    // (measured on a 1e9 x 96 B index with 65536 lists: the wide kernel wins from about two pairs per list up,
    // where a good share of the lists is probed by three queries or more)
    bool wide = std::min((double)CH_wide, avgblk) >= 64.0 && (double)npairs >= 1.5 * idx->nlist;
    const int force = forced_scan_kernel();
    ScanPlan p;
    p.kind = wide ? SCAN_WIDE : SCAN_NARROW;
    // Short lists under the inner product (a query's pairs share its base table): one wave per item, pairs grouped
    // by query.  Measured on 10M x 96 B with 16384 lists of ~10 blocks, 256 queries x 64 lists: 0.20 ms against
    // 0.25 ms, and 8 us of planning against 40.  On lists of hundreds of blocks the kernels that put eight waves on
    // neighbouring blocks stream 15 % faster (1e9 x 96 B, 1 to 16 queries x 256 lists).
    if (!wide && base_tables && avgblk <= 32.0) p.kind = SCAN_WAVE;
    if (force >= 1 && force <= 3) p.kind = force - 1;
    if (p.kind == SCAN_WIDE) p.CH = CH_wide;
    // (a single query: ~1000 tasks, two per resident workgroup, measured best on 256 lists of ~240 blocks - 0.218 ms a
    // round against 0.232 with 2000 tasks and 0.239 with 250: what a task costs to start outweighs the uneven end)
    else if (p.kind == SCAN_NARROW) p.CH = chunk_len((double)npairs, avgblk, nq > 1 ? 1.5 : 1.0, 256, nq > 1 ? 2048.0 : 1024.0);
    else p.CH = wave_chunk_len((double)npairs * avgblk, idx->n_cu);
    p.group = p.kind == SCAN_WIDE ? NPMAX : 2;          // pairs of one list per task
    const int64_t maxblk = (idx->max_list_len + BLOCK_VECS - 1) / BLOCK_VECS;
    p.maxchunks = (int)std::max<int64_t>(1, (maxblk + p.CH - 1) / p.CH);
    return p;
}

// The largest npairs * maxchunks over all calls with nq <= max_nq and nprobe <= max_nprobe, whichever kernel
// runs them.  Inside a range of npairs with one chunk length the product grows with npairs, so only the
// upper end of every such range (and the maxima themselves) needs looking at.
static int64_t max_result_slots(const rago_index* idx, int64_t max_nq, int max_nprobe) {
    const double avgblk = std::max((double)idx->total_blocks / idx->nlist, 1e-9);
    const int64_t maxblk = (idx->max_list_len + BLOCK_VECS - 1) / BLOCK_VECS;
    int64_t best = 1;
    auto look = [&](int64_t np, int64_t np_max, int ch_of_np) {
        (void)np_max;
        best = std::max(best, np * std::max<int64_t>(1, (maxblk + ch_of_np - 1) / ch_of_np));
    };
    for (int single = 0; single < 2; ++single) {                    // batches of one query use other task sizes
        const int64_t np_max = single ? max_nprobe : max_nq * max_nprobe;
        const double ppts[2] = {single ? 1.0 : 2.0, single ? 1.0 : 1.5};
        const int caps[2] = {512, 256};
        for (int kern = 0; kern < 2; ++kern)
            for (int c = 16; c <= caps[kern]; c <<= 1) {
                const double tasks = kern == 1 && single ? 1024.0 : 2048.0;
                const int64_t edge = (int64_t)(tasks * ppts[kern] * c / avgblk);
                for (int64_t np : {edge - 1, edge, edge + 1, np_max}) {
                    np = std::min(std::max<int64_t>(np, 1), np_max);
                    look(np, np_max, chunk_len((double)np, avgblk, ppts[kern], caps[kern], tasks));
                }
            }
        for (int c = 1; c <= 512; c <<= 1) {                        // the kernel with one wave per item
            const int64_t edge = (int64_t)(4.0 * 2 * 8 * idx->n_cu * c / avgblk);
            for (int64_t np : {edge - 1, edge, edge + 1, np_max}) {
                np = std::min(std::max<int64_t>(np, 1), np_max);
                look(np, np_max, wave_chunk_len((double)np * avgblk, idx->n_cu));
            }
        }
    }
    return best;
}

// The workspace of a scan of this size (for this call, or - when the workspace is being sized - the most any call
// within these maxima can need: smaller batches take shorter chunks, i.e. more chunks per pair).
static int reserve_scan(rago_index* idx, int64_t nq, int nprobe, int k, const ScanPlan& plan) {
    Workspace& ws = idx->ws;
    const int64_t npairs = nq * nprobe;
    const int nlist = idx->nlist;
    const int64_t slots = idx->reserving ? max_result_slots(idx, nq, nprobe) : npairs * plan.maxchunks;
    if ((double)slots * k > 4.0e9) return fail(RAGO_UNSUPPORTED, "nq * nprobe * chunks * k too large for the workspace");
    int rc;
    if ((rc = ws.list_cnt.reserve((size_t)(3 * nlist + 8) * 4))) return rc;   // list_cnt, cursor, list_slot, ctrl
    if ((rc = ws.pair_off.reserve((size_t)(npairs + 2) * 4))) return rc;      // per touched list
    if ((rc = ws.task_off.reserve((size_t)(npairs + 2) * 4))) return rc;
    if ((rc = ws.touched.reserve((size_t)(npairs + 2) * 4))) return rc;
    if ((rc = ws.pair_sorted.reserve((size_t)npairs * 4))) return rc;
    if ((rc = ws.tauq.reserve((size_t)nq * 4))) return rc;
    if ((rc = ws.part_I.reserve((size_t)slots * k * 4))) return rc;
    if ((rc = ws.part_id.reserve((size_t)slots * k * 8))) return rc;
    if ((rc = ws.part_cnt.reserve((size_t)slots * 4))) return rc;
    if ((rc = ws.counters.reserve(64))) return rc;
    if ((rc = ws.task_table.reserve((size_t)slots * 16))) return rc;
    if (idx->reserving || plan.kind == SCAN_WAVE) {
        if ((rc = ws.wave_items.reserve((size_t)npairs * wave_pair_bytes()))) return rc;
        if ((rc = ws.wave_q.reserve((size_t)nq * 48))) return rc;
        if ((rc = ws.wave_stage.reserve(wave_stage_bytes(nq, k)))) return rc;
    }
    return RAGO_OK;
}

static void fill_small_setup(rago_index* idx, const int32_t* probes, int64_t nq, int nprobe, const ScanPlan& plan, SmallSetupArgs* A) {
    Workspace& ws = idx->ws;
    A->enable = 1;
    A->probes = probes; A->npairs = (int)(nq * nprobe); A->nq = (int)nq;
    A->list_meta = idx->list_meta;
    A->CH = plan.CH; A->group = plan.group; A->m = idx->m;
    A->pair_sorted = ws.pair_sorted.as<int32_t>();
    A->table = ws.task_table.as<int4>();
    A->ctrl = ws.list_cnt.as<int32_t>() + 3 * idx->nlist;
    A->tauq = ws.tauq.as<int32_t>();
    A->counters = ws.counters.as<int64_t>();
}

// For a caller that runs the scan's bookkeeping inside kernels of its own (the table kernels of the inner-product
// path): sizes the scan's workspace and says what those workgroups have to do - `small` (may be null) for a small
// batch's pairs-by-list bookkeeping, `wave` (may be null) for the plan of the wave-per-item kernel; `enable` stays 0
// in both when the scan of this call does its bookkeeping itself.  launch_scan is then told that it is done.
int plan_scan_setup(rago_index* idx, const int32_t* probes, int64_t nq, int nprobe, int k, bool base_tables, SmallSetupArgs* small,
                    WavePlanArgs* wave) {
    if (small) small->enable = 0;
    if (wave) wave->enable = 0;
    const ScanPlan plan = plan_scan(idx, nq, nq * nprobe, base_tables);
    int rc = reserve_scan(idx, nq, nprobe, k, plan);
    if (rc || idx->reserving) return rc;
    Workspace& ws = idx->ws;
    if (plan.kind == SCAN_WAVE) {
        if (wave) {
            ScanParams P{};         // (what the plan reads of it; the tables do not exist yet: namb stays null)
            P.probes = probes; P.blk_off = idx->blk_off; P.list_off = idx->list_off;
            P.nprobe = nprobe; P.CH = plan.CH; P.m = idx->m; P.tauq = ws.tauq.as<int32_t>();
            fill_wave_plan(P, nq, idx->n_cu, ws.wave_items.p, ws.pair_sorted.as<int32_t>(), ws.wave_q.as<int32_t>(), ws.counters.as<int64_t>(), wave);
        }
    } else if (small && nq * nprobe <= SSU_PAIRS) {
        fill_small_setup(idx, probes, nq, nprobe, plan, small);
    }
    return RAGO_OK;
}

int launch_scan(rago_index* idx, const int32_t* probes, const uint8_t* lut8sw, const int32_t* bias, const LutTables* tables,
                const float* delta, int64_t nq, int nprobe, int k, int64_t* out_ids, float* out_scores, int32_t* out_iscores,
                hipStream_t st, hipEvent_t* ev, bool setup_done) {
    Workspace& ws = idx->ws;
    const int64_t npairs = nq * nprobe;
    const int nlist = idx->nlist;
    const ScanPlan plan = plan_scan(idx, nq, npairs, tables != nullptr);
    const bool wide = plan.kind == SCAN_WIDE;
    const int CH = plan.CH, group = plan.group, maxchunks = plan.maxchunks;
    int rc;
    if ((rc = reserve_scan(idx, nq, nprobe, k, plan))) return rc;
    const int64_t max_tasks = npairs * maxchunks;
    if (idx->reserving) return RAGO_OK;
    idx->last_scan_kernel = plan.kind + 1;

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
    P.tauq = ws.tauq.as<int32_t>(); P.part_I = ws.part_I.as<int32_t>(); P.part_row = ws.part_id.as<int64_t>();
    P.part_cnt = ws.part_cnt.as<int32_t>();
    P.nlist = nlist; P.nprobe = nprobe; P.k = k; P.CH = CH; P.maxchunks = maxchunks;

    const int n_cu = idx->n_cu;
    if (plan.kind == SCAN_WAVE)
        return launch_scan_wave(P, nq, n_cu, (double)idx->total_blocks / nlist, ws.wave_items.p, ws.pair_sorted.as<int32_t>(),
                                ws.wave_q.as<int32_t>(), ws.wave_stage.p, ws.counters.as<int64_t>(), delta, out_ids, out_scores, out_iscores,
                                ev, st, setup_done);
    const unsigned pg = (unsigned)((npairs + 255) / 256);
    if (setup_done) {
        // (the caller's kernel has done it: plan_scan_setup)
    } else if (npairs <= SSU_PAIRS) {
        static OncePerDevice once;
        if (once.first())
            RAGO_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(small_setup_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)SSU_LDS));
        SmallSetupArgs A;
        fill_small_setup(idx, probes, nq, nprobe, plan, &A);
        small_setup_kernel<<<1, SSU_THREADS, SSU_LDS, st>>>(A);
    } else {
    scan_init_kernel<<<(unsigned)std::min<int64_t>(256, (2 * nlist + nq + 255) / 256 + 1), 256, 0, st>>>(list_cnt, 2 * (int64_t)nlist, P.tauq, nq, ctrl, ws.counters.as<int64_t>());
    if (nq >= 64) {
        count_pairs_kernel<<<pg, 256, 0, st>>>(probes, npairs, nprobe, 0, list_cnt, ws.touched.as<int32_t>(), ctrl);
        count_pairs_kernel<<<pg, 256, 0, st>>>(probes, npairs, nprobe, 1, list_cnt, ws.touched.as<int32_t>(), ctrl);
    } else {
        count_pairs_kernel<<<pg, 256, 0, st>>>(probes, npairs, nprobe, 2, list_cnt, ws.touched.as<int32_t>(), ctrl);
    }
    touched_values_kernel<<<pg, 256, 0, st>>>(ws.touched.as<int32_t>(), list_cnt, idx->blk_off, idx->list_off, CH, group, idx->m, npairs, ctrl,
                                              list_slot, ws.pair_off.as<int32_t>(), ws.task_off.as<int32_t>(), ws.counters.as<int64_t>());
    touched_scan_kernel<<<1, 1024, 0, st>>>(ws.pair_off.as<int32_t>(), ws.task_off.as<int32_t>(), ctrl, ws.counters.as<int64_t>());
    scatter_pairs_kernel<<<pg, 256, 0, st>>>(probes, npairs, list_slot, ws.pair_off.as<int32_t>(), cursor, ws.pair_sorted.as<int32_t>());
    task_table_kernel<<<(unsigned)((max_tasks + 255) / 256), 256, 0, st>>>(ws.task_off.as<int32_t>(), ws.pair_off.as<int32_t>(),
                                                                           ws.touched.as<int32_t>(), group, ctrl, max_tasks,
                                                                           ws.task_table.as<int4>());
    }
    RAGO_HIP(hipGetLastError());

    if (ev) RAGO_HIP(hipEventRecord(ev[4], st));
    if (!wide) {
        rc = launch_scan_narrow(P, n_cu, st);
    } else {
        const int grid = n_cu;       // one workgroup per CU: the four interleaved tables fill most of its LDS
        switch (idx->m) {
            case 16: rc = launch_scan_kernel<16>(P, grid, st); break;
            case 32: rc = launch_scan_kernel<32>(P, grid, st); break;
            case 64: rc = launch_scan_kernel<64>(P, grid, st); break;
            case 96: rc = launch_scan_kernel<96>(P, grid, st); break;
            case 128: rc = launch_scan_kernel<128>(P, grid, st); break;
            default: return fail(RAGO_UNSUPPORTED, "code width");
        }
    }
    if (rc) return rc;
    if (ev) RAGO_HIP(hipEventRecord(ev[5], st));
    if (nq <= 32) merge_kernel<1024><<<(unsigned)nq, 1024, 0, st>>>(P, delta, out_ids, out_scores, out_iscores);
    else merge_kernel<MERGE_THREADS><<<(unsigned)nq, MERGE_THREADS, 0, st>>>(P, delta, out_ids, out_scores, out_iscores);
    RAGO_HIP(hipGetLastError());
    if (ev) RAGO_HIP(hipEventRecord(ev[6], st));
    return RAGO_OK;
}

}  // namespace rago

// The scan kernel for short lists and small batches: one WAVE scans one (query, list, chunk) item
// from start to end, so the streaming loop has no workgroup barrier, no merge across waves and no
// per-task fixed work.  Same results as the kernels of scan.hip and scan_narrow.hip, which group
// the pairs by list; this one groups them by QUERY:
//
//  * a task = a run of consecutive items of one query; the workgroup (8 waves, two workgroups per
//    CU) brings that query's 8-bit base table into LDS once, then its waves claim items from an
//    LDS counter and work through them independently.  Under the inner product the tables of a
//    query's pairs differ from its base table only in the few entries whose rounding depends on
//    the pair (lut.hip).  Those entries are not patched into the shared table: a wave turns the
//    pair's patches into corrections (sub-quantiser, code, +-difference), sums with the base
//    table, and applies the corrections, from the code bytes it holds in registers, only to blocks
//    in which some vector comes within the corrections' reach of the threshold.
//  * per-pair tables (Euclidean metric, caller-supplied tables, queries whose tables are too flat
//    for the base + patch form) are installed pair by pair, with a barrier before and after, and
//    the waves share out that pair's items.
//  * LDS table layout (32 KiB): byte address = code * 128 + slot * 4 + plane.  `slot` selects the
//    bank, so a sub-table lives in ONE bank; the 32 lanes of a half-wave always work on 32
//    different slots (layout.hip), so every ds_read_u8 is conflict-free whatever the codes are.
//    One v_perm_b32 places two code bytes next to the lane's slot * 8 bytes; a bit-field extract
//    and a shift by one bit turn the halves into addresses; the plane rides in the immediate.
//  * an item leaves <= k (score, row) entries in its own slot of the per-task result arrays; the
//    per-query bound on the k-th best score is shared through LDS and a word in HBM; the final
//    merge is the one of scan.hip.
#include <algorithm>

#include "scan_common.h"

namespace rago {
namespace wavescan {

constexpr int WAVES = 8;
constexpr int THREADS = WAVES * 64;
constexpr int LUT_LDS = 32768;
constexpr int CORR_CAP = AMB_MAX;
// LDS: table | key buffers [wave][CAPW] | corrections [wave][CORR_CAP] | ambiguous entries of the query: address u16, base value u8 | scalars
constexpr int OFF_CAND = LUT_LDS;
constexpr int OFF_CORR = OFF_CAND + WAVES * CAPW * 4;
constexpr int OFF_AMB = OFF_CORR + WAVES * CORR_CAP * 4;
constexpr int OFF_AMBV = OFF_AMB + AMB_MAX * 2;
constexpr int OFF_SH = OFF_AMBV + AMB_MAX;
constexpr int SCAN_LDS = OFF_SH + 64 * 4;

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

struct Item { int64_t blk0, row0; int32_t nb, cvecs, pair, chunk; };   // 32 bytes: one (pair, chunk of the list)

struct WaveParams {
    ScanParams S;              // codes, tables, result arrays, nprobe, k, CH (= blocks per item), maxchunks
    const Item* items;         // [nitems] grouped by query, then pair, then chunk
    const int4* tasks;         // [ntasks] {query, first item, end item, 0}
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
    int32_t* sh = reinterpret_cast<int32_t*>(smem + OFF_SH);
    // sh[0] task, sh[1] item counter, sh[2] bound on the query's k-th best score (absolute integer score)

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
    const int ntasks = P.ctrl[1];
    const int k = P.k;
    int loaded_q = -1;                         // query whose base table (and ambiguous entries) sit in LDS

    for (;;) {
        __syncthreads();                       // every wave is done with the previous task's table and scalars
        if (threadIdx.x == 0) sh[0] = atomicAdd(P.ctrl, 1);
        __syncthreads();
        const int t = __builtin_amdgcn_readfirstlane(sh[0]);
        if (t >= ntasks) break;                // every wave reads the same word: all leave together
        const int4 rec = W.tasks[t];
        const int q = __builtin_amdgcn_readfirstlane(rec.x);
        const int i0 = __builtin_amdgcn_readfirstlane(rec.y), i1 = __builtin_amdgcn_readfirstlane(rec.z);
        const int namb = P.lut8sw ? 0 : __builtin_amdgcn_readfirstlane(P.T.namb[q]);
        const bool shared_base = !P.lut8sw && namb <= AMB_MAX;
        if (threadIdx.x == 0) sh[2] = __hip_atomic_load(P.tauq + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (shared_base && loaded_q != q) {        // (consecutive tasks of one query, a batch of one query: nothing to do)
            install_table<planes>(P.T.lut_base + (int64_t)q * LUT_BYTES, lut);
            for (int i = threadIdx.x; i < namb; i += THREADS) s_amb[i] = P.T.amb_addr[(int64_t)q * AMB_MAX + i];
            __syncthreads();
            for (int i = threadIdx.x; i < namb; i += THREADS) s_ambv[i] = lut[entry_lds(s_amb[i])];
        }
        loaded_q = shared_base ? q : -1;
        // Segments: the whole task when the waves share the query's base table; else one segment per pair, whose
        // table is installed between two barriers.
        int seg0 = i0;
        while (seg0 < i1) {
            int seg1 = i1;
            if (!shared_base) {
                const int pr = W.items[seg0].pair;
                seg1 = seg0 + 1;
                while (seg1 < i1 && W.items[seg1].pair == pr) ++seg1;
                __syncthreads();               // the previous pair's table is no longer read
                if (P.lut8sw) install_table<planes>(P.lut8sw + (int64_t)pr * LUT_BYTES, lut);
                else eval_table(P, pr, q, lut);
            }
            if (threadIdx.x == 0) sh[1] = seg0;
            __syncthreads();

            // ---- the wave's items of this segment
            auto claim = [&]() {
                int v = 0;
                if (lane == 0) v = atomicAdd(&sh[1], 1);
                return __builtin_amdgcn_readfirstlane(v);
            };
            auto load_item = [&](int i) {
                // (every lane loads the same 32 bytes: one request; the index is clamped so the load is always legal)
                const int4* p = reinterpret_cast<const int4*>(W.items + min(i, seg1 - 1));
                const int4 a = p[0], b = p[1];
                Item it;
                it.blk0 = ((int64_t)__builtin_amdgcn_readfirstlane(a.y) << 32) | (uint32_t)__builtin_amdgcn_readfirstlane(a.x);
                it.row0 = ((int64_t)__builtin_amdgcn_readfirstlane(a.w) << 32) | (uint32_t)__builtin_amdgcn_readfirstlane(a.z);
                it.nb = __builtin_amdgcn_readfirstlane(b.x); it.cvecs = __builtin_amdgcn_readfirstlane(b.y);
                it.pair = __builtin_amdgcn_readfirstlane(b.z); it.chunk = __builtin_amdgcn_readfirstlane(b.w);
                return it;
            };
            uint4 wa[MPAD / 16], wb[MPAD / 16];
            int cur_i = claim();
            Item cur = load_item(cur_i);
            int nxt_i = claim();
            Item nxt = load_item(nxt_i);
            if (cur_i < seg1) load_block<MPAD>(wa, P.codes + cur.blk0 * BLK_BYTES, lane);
            while (cur_i < seg1) {
                const int pair = cur.pair, nb = cur.nb, cvecs = cur.cvecs;
                const uint8_t* base = P.codes + cur.blk0 * BLK_BYTES;
                const uint8_t* after = nxt_i < seg1 ? P.codes + nxt.blk0 * BLK_BYTES : base;   // what follows this item's last block
                const int bias = __builtin_amdgcn_readfirstlane(P.bias[pair]);
                // ---- corrections of this pair: entries whose exact value differs from the base table's
                int ncorr = 0, maxpos = 0;
#ifdef RAGO_WV_NOCORR
                if (false) {
#else
                if (shared_base) {
#endif
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
                    const int64_t d = (int64_t)sh[2] - bias;
                    return (uint32_t)(d <= 0 ? 0 : (d > 0x7fffffff ? 0x7fffffff : d));
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
                // ---- stream the item's blocks: the block after the current one is always in flight (the first
                // block of the wave's next item after the last); unconditional loads from clamped addresses
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
                const int64_t slot = (int64_t)pair * P.maxchunks + cur.chunk;
                int32_t* oI = P.part_I + slot * k;
                int64_t* orow = P.part_row + slot * k;
                for (int e = lane; e < cnt; e += 64) {
                    const uint32_t key = buf[e];
                    oI[e] = bias + (int32_t)(key >> 16);
                    orow[e] = cur.row0 + (int64_t)(0xFFFFu - (key & 0xFFFFu));
                }
                if (lane == 0) {
                    P.part_cnt[slot] = cnt;
                    if (cnt >= k) {                    // k entries reach the k-th key's score: a bound on the query's k-th best
                        const int32_t tq = bias + (int32_t)(kth >> 16);
                        atomicMax(&sh[2], tq);
                        atomicMax(P.tauq + q, tq);
                    }
                }
                cur_i = nxt_i;
                cur = nxt;
                nxt_i = claim();
                nxt = load_item(nxt_i);
            }
            seg0 = seg1;
        }
    }
}

// ------------------------------------------------------------------ planning kernels
// Items of one query: its pairs in probe order, each cut into chunks of CH blocks.  One workgroup per query:
// counts, an exclusive scan inside the query, and the query's totals for the scan over the queries.
// qinfo[q] = {items, tasks, item base, task base}; qbytes[q] = {code bytes streamed, algorithmic code bytes}.
__global__ void __launch_bounds__(256) count_kernel(const int32_t* __restrict__ probes, const int64_t* __restrict__ blk_off,
                                                    const int64_t* __restrict__ list_off, int nprobe, int CH, int ipt, int m,
                                                    int32_t* __restrict__ pair_items, int4* __restrict__ qinfo,
                                                    int64_t* __restrict__ qbytes, int32_t* __restrict__ tauq) {
    __shared__ int s_w[4];
    __shared__ int s_carry;
    __shared__ unsigned long long s_bytes[2];
    const int q = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) { s_carry = 0; s_bytes[0] = 0; s_bytes[1] = 0; tauq[q] = INT32_MIN; }
    __syncthreads();
    unsigned long long streamed = 0, algo = 0;
    for (int p0 = 0; p0 < nprobe; p0 += 256) {
        const int p = p0 + tid;
        int n = 0;
        if (p < nprobe) {
            const int l = probes[(int64_t)q * nprobe + p];
            const int nblk = (int)(blk_off[l + 1] - blk_off[l]);
            n = (nblk + CH - 1) / CH;
            streamed += (unsigned long long)nblk * (BLOCK_VECS * m);
            algo += (unsigned long long)(list_off[l + 1] - list_off[l]) * m;
        }
        int inc = n;
        for (int o = 1; o < 64; o <<= 1) {
            const int v = __shfl_up(inc, o);
            if (lane >= o) inc += v;
        }
        if (lane == 63) s_w[wave] = inc;
        __syncthreads();
        int before = s_carry;
        for (int w = 0; w < wave; ++w) before += s_w[w];
        if (p < nprobe) pair_items[(int64_t)q * nprobe + p] = before + inc - n;     // first item of the pair inside its query
        __syncthreads();
        if (tid == 255) s_carry = before + inc;
        __syncthreads();
    }
    for (int o = 32; o; o >>= 1) { streamed += __shfl_xor(streamed, o); algo += __shfl_xor(algo, o); }
    if (lane == 0) { atomicAdd(&s_bytes[0], streamed); atomicAdd(&s_bytes[1], algo); }
    __syncthreads();
    if (tid == 0) {
        const int items = s_carry;
        qinfo[q] = make_int4(items, (items + ipt - 1) / ipt, 0, 0);
        qbytes[2 * q] = (int64_t)s_bytes[0];
        qbytes[2 * q + 1] = (int64_t)s_bytes[1];
    }
}

// Exclusive scan over the queries (one workgroup): item and task bases, totals, counters.
__global__ void __launch_bounds__(1024) bases_kernel(int4* __restrict__ qinfo, const int64_t* __restrict__ qbytes, int nq,
                                                     int32_t* __restrict__ ctrl, int64_t* __restrict__ counters) {
    __shared__ int s_wi[16], s_wt[16];
    __shared__ unsigned long long s_b[2];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) { s_b[0] = 0; s_b[1] = 0; }
    int carry_i = 0, carry_t = 0;
    unsigned long long streamed = 0, algo = 0;
    for (int q0 = 0; q0 < nq; q0 += 1024) {
        const int q = q0 + tid;
        int4 r = make_int4(0, 0, 0, 0);
        if (q < nq) { r = qinfo[q]; streamed += (unsigned long long)qbytes[2 * q]; algo += (unsigned long long)qbytes[2 * q + 1]; }
        int ii = r.x, it = r.y;
        for (int o = 1; o < 64; o <<= 1) {
            const int a = __shfl_up(ii, o), b = __shfl_up(it, o);
            if (lane >= o) { ii += a; it += b; }
        }
        __syncthreads();
        if (lane == 63) { s_wi[wave] = ii; s_wt[wave] = it; }
        __syncthreads();
        int bi = carry_i, bt = carry_t, ti = 0, tt = 0;
        for (int w = 0; w < 16; ++w) {
            if (w < wave) { bi += s_wi[w]; bt += s_wt[w]; }
            ti += s_wi[w]; tt += s_wt[w];
        }
        if (q < nq) qinfo[q] = make_int4(r.x, r.y, bi + ii - r.x, bt + it - r.y);
        carry_i += ti; carry_t += tt;
    }
    for (int o = 32; o; o >>= 1) { streamed += __shfl_xor(streamed, o); algo += __shfl_xor(algo, o); }
    if (lane == 0) { atomicAdd(&s_b[0], streamed); atomicAdd(&s_b[1], algo); }
    __syncthreads();
    if (tid == 0) {
        ctrl[0] = 0; ctrl[1] = carry_t;
        counters[0] = carry_t; counters[1] = (int64_t)s_b[0]; counters[2] = (int64_t)s_b[1];
    }
}

// The item and task records of one query (one workgroup per query).
__global__ void __launch_bounds__(256) items_kernel(const int32_t* __restrict__ probes, const int64_t* __restrict__ blk_off,
                                                    const int64_t* __restrict__ list_off, int nprobe, int CH, int ipt,
                                                    const int32_t* __restrict__ pair_items, const int4* __restrict__ qinfo,
                                                    Item* __restrict__ items, int4* __restrict__ tasks) {
    const int q = blockIdx.x;
    const int4 qi = qinfo[q];
    for (int lt = threadIdx.x; lt < qi.y; lt += 256)
        tasks[qi.w + lt] = make_int4(q, qi.z + lt * ipt, qi.z + min(qi.x, (lt + 1) * ipt), 0);
    for (int p = threadIdx.x; p < nprobe; p += 256) {
        const int64_t pair = (int64_t)q * nprobe + p;
        const int l = probes[pair];
        const int64_t b0 = blk_off[l], v0 = list_off[l];
        const int nblk = (int)(blk_off[l + 1] - b0), len = (int)(list_off[l + 1] - v0);
        Item* out = items + qi.z + pair_items[pair];
        for (int c = 0; c * CH < nblk; ++c) {
            Item it;
            it.blk0 = b0 + (int64_t)c * CH;
            it.row0 = v0 + (int64_t)c * CH * BLOCK_VECS;
            it.nb = min(CH, nblk - c * CH);
            it.cvecs = min(len - c * CH * BLOCK_VECS, it.nb * BLOCK_VECS);
            it.pair = (int32_t)pair;
            it.chunk = c;
            out[c] = it;
        }
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

// Blocks per item: about three items per resident wave, at least 8 blocks (a wave keeps one block in flight while
// it works on another, so an item shorter than that is mostly start and end) and at most 512 (position field).
int wave_chunk_len(double total_blocks, int n_cu) {
    const double want = 3.0 * 2 * wavescan::WAVES * n_cu;
    int c = 8;
    while (c < 512 && total_blocks / c > want) c <<= 1;
#ifdef RAGO_WV_CH
    c = RAGO_WV_CH;
#endif
    return c;
}

size_t wave_item_bytes() { return sizeof(wavescan::Item); }

// Plans the items and tasks on the device (three small kernels), then runs the scan.  P.CH / P.maxchunks are the
// blocks per item and the most items any pair can have; items / tasks / pair_items / qinfo / qbytes are workspace.
int launch_scan_wave(const ScanParams& P, int64_t nq, int n_cu, double avgblk, void* items, int4* tasks, int32_t* pair_items,
                     int4* qinfo, int64_t* qbytes, int64_t* counters, hipEvent_t ev_scan, hipStream_t st) {
    using namespace wavescan;
    const int grid = 2 * n_cu;
    // items per task: about two tasks per workgroup, one item per wave at least
    const double est_items = std::max(1.0, (double)nq * P.nprobe * std::max(1.0, avgblk / P.CH));
    int ipt = 8;
    while (ipt < 256 && est_items / ipt > 2.0 * grid) ipt <<= 1;
#ifdef RAGO_WV_IPT
    ipt = RAGO_WV_IPT;
#endif
    count_kernel<<<(unsigned)nq, 256, 0, st>>>(P.probes, P.blk_off, P.list_off, P.nprobe, P.CH, ipt, P.m, pair_items, qinfo, qbytes, P.tauq);
    bases_kernel<<<1, 1024, 0, st>>>(qinfo, qbytes, (int)nq, P.ctrl, counters);
    items_kernel<<<(unsigned)nq, 256, 0, st>>>(P.probes, P.blk_off, P.list_off, P.nprobe, P.CH, ipt, pair_items, qinfo,
                                               static_cast<Item*>(items), tasks);
    RAGO_HIP(hipGetLastError());
    if (ev_scan) RAGO_HIP(hipEventRecord(ev_scan, st));
    WaveParams W;
    W.S = P;
    W.items = static_cast<const Item*>(items);
    W.tasks = tasks;
    switch (P.m) {
        case 16: return launch_one<16>(W, grid, st);
        case 32: return launch_one<32>(W, grid, st);
        case 64: return launch_one<64>(W, grid, st);
        case 96: return launch_one<96>(W, grid, st);
        case 128: return launch_one<128>(W, grid, st);
        default: return fail(RAGO_UNSUPPORTED, "code width");
    }
}

}  // namespace rago

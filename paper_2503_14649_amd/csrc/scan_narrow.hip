// The scan kernel for short tasks (short lists, small batches): two pairs of a list per pass,
// eight waves per workgroup, two workgroups per CU, so that one workgroup streams while the other
// sits in the fixed per-task work (tables into LDS, barriers, merge of the wave buffers).  Same
// results as the wide kernel of scan.hip, which needs long tasks to amortise that work.
//
//  * LDS table layout (64 KiB): byte address = code * 256 + slot * 4 + plane (+128 for the
//    second pair).  `slot` selects the bank, so a sub-table lives in ONE bank; the 32 lanes of a
//    half-wave always work on 32 different slots (see layout.hip), which makes every ds_read_u8
//    conflict-free whatever the code values are.  The address is built with a single v_perm_b32
//    from the code dword and a per-lane register holding slot*4 for four consecutive steps;
//    plane and pair select ride in the instruction's immediate offset.
//  * everything else (one lane = one vector, 32-bit keys, per-wave key buffers pruned by radix
//    select on ballots, thresholds shared through LDS and a per-query word in HBM, the first
//    wave that runs out of blocks fetches the next task) as described in scan.hip.
#include "scan_common.h"

namespace rago {
namespace narrow {

constexpr int SCAN_WAVES = 8;
constexpr int SCAN_THREADS = SCAN_WAVES * 64;
constexpr int LUT_LDS = 65536;
constexpr int SCAN_LDS = LUT_LDS + SCAN_WAVES * 2 * CAPW * 4 + 512;
constexpr int DESC_INTS = 20;   // task descriptor in LDS (see fetch_task)

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

// Bring plane-major tables (HBM, [plane][c][slot] bytes) into the LDS rows: the four planes of a
// (code, slot) entry become the four bytes of one dword.  Unit u = 8 consecutive slots of one code
// (8 source bytes per plane, 32 bytes of LDS), handled by thread u mod SCAN_THREADS; a null source
// leaves that pair's half of the rows untouched.  `between` runs after the loads are issued and
// before their data is needed (the caller puts the first code-block loads there, so they queue
// behind the table loads instead of in front of them: the load counter retires in order).
template <int planes, class F>
__device__ __forceinline__ void copy_table(const uint8_t* srcA, const uint8_t* srcB, uint8_t* lut, F between) {
    // (every field is loaded unconditionally from a readable address and masked afterwards:
    // conditionally filled register arrays end up in scratch memory)
    const uint8_t* sa = srcA ? srcA : srcB;
    const uint8_t* sb = srcB ? srcB : srcA;
    const int t = threadIdx.x;
    u32x2 a[2][4], b[2][4];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int u = t + r * SCAN_THREADS;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int pp = p < planes ? p : 0;
            a[r][p] = ((global_u32x2_ptr)(sa + pp * LUT_PLANE))[u];
            b[r][p] = ((global_u32x2_ptr)(sb + pp * LUT_PLANE))[u];
        }
    }
    between();
    const uint32_t m1 = planes > 1 ? ~0u : 0u, m2 = planes > 2 ? ~0u : 0u, m3 = planes > 3 ? ~0u : 0u;
    auto interleave = [&](const u32x2 (&v)[4], uint8_t* dst) {
        uint4 out[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t p0 = h ? v[0].y : v[0].x, p1 = (h ? v[1].y : v[1].x) & m1;
            const uint32_t p2 = (h ? v[2].y : v[2].x) & m2, p3 = (h ? v[3].y : v[3].x) & m3;
            const uint32_t lo01 = __builtin_amdgcn_perm(p1, p0, 0x05010400u), lo23 = __builtin_amdgcn_perm(p1, p0, 0x07030602u);
            const uint32_t hi01 = __builtin_amdgcn_perm(p3, p2, 0x05010400u), hi23 = __builtin_amdgcn_perm(p3, p2, 0x07030602u);
            out[h] = make_uint4(__builtin_amdgcn_perm(hi01, lo01, 0x05040100u), __builtin_amdgcn_perm(hi01, lo01, 0x07060302u),
                                __builtin_amdgcn_perm(hi23, lo23, 0x05040100u), __builtin_amdgcn_perm(hi23, lo23, 0x07060302u));
        }
        reinterpret_cast<uint4*>(dst)[0] = out[0];
        reinterpret_cast<uint4*>(dst)[1] = out[1];
    };
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int u = t + r * SCAN_THREADS;
        uint8_t* d = lut + (u >> 2) * 256 + (u & 3) * 32;
        if (srcA) interleave(a[r], d);
        if (srcB) interleave(b[r], d + 128);
    }
}

// LDS offset (inside one pair's half of the rows) of entry e = plane*8192 + code*32 + slot, and the
// wave whose thread copies the unit that contains it.
__device__ __forceinline__ uint32_t entry_lds(uint32_t e) { return ((e >> 5) & 255u) * 256u + (e & 31u) * 4u + (e >> 13); }
__device__ __forceinline__ uint32_t entry_owner(uint32_t e) { return (((e & 8191u) >> 3) & (uint32_t)(SCAN_THREADS - 1)) >> 6; }

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
    const int4 rec = P.task_table[t];      // {list, chunk, first position in pair_sorted, pairs (1 or 2)}
    const int l = rec.x;
    const int pairA = P.pair_sorted[rec.z], pairB = rec.w > 1 ? P.pair_sorted[rec.z + 1] : -1;
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
        constexpr int planes = MPAD < 32 ? 1 : MPAD / 32;
        if (P.lut8sw) {
            copy_table<planes>(P.lut8sw + (int64_t)pairA * LUT_BYTES, pairB >= 0 ? P.lut8sw + (int64_t)pairB * LUT_BYTES : nullptr, lut,
                               first_load);
            loadedA = loadedB = -1;
        } else {
            // base table of the query (kept while consecutive tasks use the same query in this slot),
            // then the pair's patches; flagged queries are evaluated entry by entry
            const bool baseA = nA <= AMB_MAX && loadedA != qA;
            const bool baseB = pairB >= 0 && nB <= AMB_MAX && loadedB != qB;
            // Patches are written by the wave that copies the unit they fall into, so program order inside
            // the wave puts them after the copy and no workgroup barrier is needed in between.
            // (the arrays always hold AMB_MAX entries, so the first 64 can be read unconditionally)
            const bool useA = nA <= AMB_MAX, useB = pairB >= 0 && nB <= AMB_MAX;
            const uint32_t a0 = P.T.amb_addr[(int64_t)qA * AMB_MAX + lane];
            const uint32_t v0 = P.T.patch_val[(int64_t)pairA * AMB_MAX + lane];
            const uint32_t a1 = P.T.amb_addr[(int64_t)(pairB >= 0 ? qB : qA) * AMB_MAX + lane];
            const uint32_t v1 = P.T.patch_val[(int64_t)(pairB >= 0 ? pairB : pairA) * AMB_MAX + lane];
            if (baseA || baseB)
                copy_table<planes>(baseA ? P.T.lut_base + (int64_t)qA * LUT_BYTES : nullptr,
                                   baseB ? P.T.lut_base + (int64_t)qB * LUT_BYTES : nullptr, lut, first_load);
            else
                first_load();
            if (nA > AMB_MAX) eval_table(P, pairA, qA, lut);
            if (pairB >= 0 && nB > AMB_MAX) eval_table(P, pairB, qB, lut + 128);
            if (useA && lane < nA && entry_owner(a0) == (uint32_t)wave) lut[entry_lds(a0)] = (uint8_t)v0;
            if (useB && lane < nB && entry_owner(a1) == (uint32_t)wave) lut[128 + entry_lds(a1)] = (uint8_t)v1;
            if (useA)
                for (int i = 64 + lane; i < nA; i += 64) {
                    const uint32_t a = P.T.amb_addr[(int64_t)qA * AMB_MAX + i];
                    if (entry_owner(a) == (uint32_t)wave) lut[entry_lds(a)] = P.T.patch_val[(int64_t)pairA * AMB_MAX + i];
                }
            if (useB)
                for (int i = 64 + lane; i < nB; i += 64) {
                    const uint32_t a = P.T.amb_addr[(int64_t)qB * AMB_MAX + i];
                    if (entry_owner(a) == (uint32_t)wave) lut[128 + entry_lds(a)] = P.T.patch_val[(int64_t)pairB * AMB_MAX + i];
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
            int64_t* orow = P.part_row + slot * k;      // rows; the final merge looks up the ids of the survivors
            const int64_t row0 = v0 + cvec0;
            int base_o = 0;
#pragma unroll
            for (int i = 0; i < 2 * SCAN_WAVES; ++i) {
                const bool keep = r[i] >= kth && r[i] != 0u;
                const uint64_t mask = __ballot(keep);
                if (keep) {
                    const int o = base_o + lane_rank(mask);
                    oI[o] = bias + (int32_t)(r[i] >> 16);
                    orow[o] = row0 + (int64_t)(0xFFFFu - (r[i] & 0xFFFFu));
                }
                base_o += __popcll(mask);
            }
            if (lane == 0) {
                P.part_cnt[slot] = base_o;
                // k entries reach the k-th key's score: a valid lower bound of the query's k-th best
                if (total >= k) publish_bound(P.tauq + (wave == 0 ? qA : qB), bias + (int32_t)(kth >> 16));
            }
        }
        __syncthreads();
    }
}


template <int MPAD>
static int launch_one(const ScanParams& P, int grid, hipStream_t st) {
    static OncePerDevice attr;
    if (attr.first()) {
        RAGO_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(scan_kernel<MPAD>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     SCAN_LDS));
    }
    scan_kernel<MPAD><<<grid, SCAN_THREADS, SCAN_LDS, st>>>(P);
    RAGO_HIP(hipGetLastError());
    return RAGO_OK;
}

}  // namespace narrow

// Two workgroups per CU.
int launch_scan_narrow(const ScanParams& P, int n_cu, hipStream_t st) {
    const int grid = 2 * n_cu;
    switch (P.m) {
        case 16: return narrow::launch_one<16>(P, grid, st);
        case 32: return narrow::launch_one<32>(P, grid, st);
        case 64: return narrow::launch_one<64>(P, grid, st);
        case 96: return narrow::launch_one<96>(P, grid, st);
        case 128: return narrow::launch_one<128>(P, grid, st);
        default: return fail(RAGO_UNSUPPORTED, "code width");
    }
}

}  // namespace rago

// Euclidean-metric tables, fast path: L[q,p][j][c] = -|q_j - (C[l]_j + CB[j][c])|^2 for every
// (query, list) pair (the metric of Section 2 under which the tables no longer factorise).
//
// The entry is DEFINED by an fp64 accumulation rounded once to fp32, and everything derived from it
// (sub-table minima, the query's step, the 8-bit codes) must come out as from that definition.
// Evaluating all m*256 entries of all pairs twice in fp64 costs ~5 fp64-rate operations per term.
// Here both passes evaluate in fp32 on the matrix cores with a proven error bound and go back to the
// fp64 definition only for the entries whose outcome the bound cannot decide.
//
//   The contraction.  Per sub-quantiser j the table of 32 pairs is a product of a [256 x K] and a [K x 32]
//   matrix with K = dsub + 2:
//       codeword side  a = (cb_0 .. cb_{dsub-1}, 1, |cb|^2)          (|cb|^2: fp64 sum, one rounding)
//       pair side      b = (2 r_0 .. 2 r_{dsub-1}, -|r|^2, -1)       (r_t = fl(q_t - c_t), |r|^2 by an fma chain)
//       L~ = sum_k a_k b_k = 2 <r, cb> - |r|^2 - |cb|^2
//   on v_mfma_f32_32x32x2_f32 (rows = codewords, columns = pairs).  That instruction accumulates like a
//   chain of fmaf in k order (checked bit for bit on 4e5 random products including subnormal ones), so with
//   x_t = q_t - c_t exact, y_t = cb_t, u = 2^-24:
//       inputs:  |2 r_t y_t - 2 x_t y_t| <= 2u |x_t||y_t|;  | |r|^2 - sum x_t^2 | <= (dsub + 2) u sum x_t^2;
//                | fl|cb|^2 - sum y_t^2 | <= u sum y_t^2
//       chain:   K roundings, each relative to a partial sum of absolute value <= sum_k |a_k b_k|
//                <= (dsub + 2) u (2 sum |x||y| + sum x^2 + sum y^2)
//       |L~ - L64| <= (2 dsub + 4) u M (1 + 1e-5),   M = sum_t (|q_t| + |c_t| + max_c |cb_t|)^2.
//   E = (3 dsub + 8) (u M + 2^-126) is used: at least 1.5 times the bound (which also covers the rounding of
//   M and E themselves) plus a smallest normal number per operation for results that underflow.  Overflow
//   gives infinities or NaNs, which every comparison below treats as "undecided".
//
//   pass 1 (minima, range): the entry attaining the exact minimum of a sub-table has L~ <= min L~ + 2E, so
//   the exact minimum is the least fp32(fp64) value among those candidates; same for the maximum.  The
//   minimum is taken as a running one over the eight tiles of 32 codewords, which only adds candidates
//   (about 6 per sub-table).
//   pass 2 (codes): b~ = fma(L~, 1/dq, fl(-lo/dq)) differs from the defining fp32 value
//   b = fl(fl(L - lo) / dq) by at most (E + 4 u M)/dq + 3 * 2^-16 (L~ against L64: E; L64 against its fp32
//   rounding L, the rounding of 1/dq applied to L~ <= M, and the two roundings in fl(-lo/dq) with |lo| <= M:
//   u M each; the roundings of b~ and b: 3 u 256); eta = E (1 + 4/(3 dsub + 8)) 1.001/dq + 2^-13 is used.
//   If b~ is farther than eta from every half-integer, rint(b~) = rint(b): v_cvt_pk_u8_f32 (round to nearest
//   even, clamped to 0..255, NaN -> 0) writes it into its byte.  Otherwise (one entry in ~300) the entry goes
//   on a list and is evaluated by the definition afterwards, all lanes busy.
//
// If a list overflows (tables that are flat relative to their magnitude make every entry undecidable) the
// workgroup evaluates all the entries concerned by the definition.
//
// Layout.  Both operand sides are stored per (row, half): a lane of the MFMA supplies, for its row or column
// (lane mod 32), the k values of its half (lane / 32): KH = dsub/2 + 1 of them, in a slot of KS = KH + 1
// floats (8-byte aligned; the spare float of a pair-side slot holds E).  Workgroups take 64 pairs (32 and a
// slice of the sub-quantisers each when the batch is small).  Pass 1: wave
// = sub-quantiser, loop over the 8 tiles of 32 codewords, each codeword load serving both column tiles;
// pass 2: round = (column tile, plane), wave = 8 of the plane's 32 sub-quantisers, loop
// over the 8 codeword tiles; a lane holds column = pair and 16 codewords and packs their 8 code bytes; the four
// waves put the pieces of each 32-byte row [plane][codeword][32 slots] together in LDS (a lane's neighbours
// hold other PAIRS, whose tables lie 32 KiB apart) and store contiguous 256-byte runs per pair.  Pair
// operands and minima are stored per tile of 32 pairs so that the 64 lanes' loads are contiguous (a load
// whose lanes hit 32 different cache lines occupied the CU's memory pipeline longer than the arithmetic).
// Registers decide the rest: 168 per lane keep three workgroups per CU resident; 8 sub-quantisers per wave
// instead of 16 (32 fewer packing registers) bought the third, worth 12 %.
#include "rago_internal.h"
#include "lut_common.h"

namespace rago {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int L2M_THREADS = 256;
constexpr int L2M_LIST1 = 1024;         // pass 1: candidates per wave and round (its sub-quantiser, 64 pairs: ~400)
constexpr int L2M_LIST2 = 2048;         // pass 2: undecided entries per wave (of 393 216 it evaluates at m = 96: ~1300)
constexpr int L2M_AHEAD = 2;          // pass 2: operands are requested this many steps ahead (1, 2 or 4)
constexpr int L2M_TRS = 8 * 32 + 16;    // pass 2: bytes per pair in the transposition buffer (16 bytes of padding)
constexpr float L2M_U = 5.9604644775390625e-08f;   // 2^-24

template <int DSUB>
struct L2M {
    static_assert(DSUB % 2 == 0, "two halves");
    static constexpr int KH = DSUB / 2 + 1;      // k values per half = MFMA steps per tile
    static constexpr int KS = KH + 1;            // floats per (row, half) slot
    static constexpr float CE = (float)(3 * DSUB + 8);
};

__device__ __forceinline__ uint32_t okey(float f) {            // order-preserving map float -> uint32
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float okey_inv(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// Pair-side operands and sub-table minima are stored per tile of 32 consecutive pairs, so that what the 64 lanes of
// a wave load together is contiguous: slot (pair, j, half) and minimum (pair, j).
__device__ __forceinline__ int64_t rec_slot(int64_t pair, int j, int half, int m) { return (((pair >> 5) * m + j) * 2 + half) * 32 + (pair & 31); }
__device__ __forceinline__ int64_t lo_index(int64_t pair, int j, int m) { return ((pair >> 5) * m + j) * 32 + (pair & 31); }

template <int KS>
__device__ __forceinline__ void load_slot(const float* __restrict__ p, float (&v)[KS]) {
    static_assert(KS % 2 == 0, "8-byte loads");
#pragma unroll
    for (int t = 0; t < KS; t += 2) {
        const float2 x = *reinterpret_cast<const float2*>(p + t);
        v[t] = x.x; v[t + 1] = x.y;
    }
}

// One 32 x 32 tile: rows = the codewords of `a`, columns = the pairs of `b`.  Lane l holds column l mod 32 and
// rows tile_row(i, l / 32), i = 0..15.
template <int KH, int KS>
__device__ __forceinline__ f32x16 tile_product(const float (&a)[KS], const float (&b)[KS]) {
    f32x16 acc = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int s = 0; s < KH; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s], b[s], acc, 0, 0, 0);
    return acc;
}
__device__ __forceinline__ int tile_row(int i, int half) { return (i >> 2) * 8 + half * 4 + (i & 3); }

// Per (pair, sub-quantiser) the pair-side operand: two slots of KS floats (see the head of the file).
template <int DSUB>
__global__ void __launch_bounds__(256) l2m_prepare_kernel(const float* __restrict__ Q, const float* __restrict__ C,
                                                          const float* __restrict__ cbmax, const int32_t* __restrict__ probes,
                                                          int64_t npairs, int nprobe, int d, int m, float* __restrict__ rec) {
    constexpr int KH = L2M<DSUB>::KH, KS = L2M<DSUB>::KS, H = DSUB / 2;
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;       // one thread per (tile of 32 pairs, sub-quantiser, pair in the tile)
    const int64_t tj = g >> 5;
    const int64_t pair = (tj / m) * 32 + (g & 31);
    const int j = (int)(tj % m);
    if (pair >= npairs) return;
    const float* qv = Q + (pair / nprobe) * d + j * DSUB;
    const float* cv = C + (int64_t)probes[pair] * d + j * DSUB;
    float out[2 * KS];
    float rr = 0.0f, M = 0.0f;
#pragma unroll
    for (int t = 0; t < DSUB; ++t) {
        const float q = qv[t], c = cv[t];
        const float r = q - c;
        out[(t / H) * KS + (t % H)] = 2.0f * r;
        rr = __fmaf_rn(r, r, rr);
        const float a = fabsf(q) + fabsf(c) + cbmax[j * DSUB + t];
        M = __fmaf_rn(a, a, M);
    }
    const float E = L2M<DSUB>::CE * (L2M_U * M + 1.17549435e-38f);
    out[KH - 1] = -rr;       out[KH] = E;
    out[KS + KH - 1] = -1.0f; out[KS + KH] = E;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        float2* e = reinterpret_cast<float2*>(rec + rec_slot(pair, j, h, m) * KS);
#pragma unroll
        for (int t = 0; t < KS; t += 2) e[t / 2] = make_float2(out[h * KS + t], out[h * KS + t + 1]);
    }
}

// ---- pass 1.  CT column tiles of 32 pairs per workgroup; blockIdx.y picks a slice of the sub-quantisers (small
// batches are split that way so that the launch still fills the chip).
template <int DSUB, int CT>
__global__ void __launch_bounds__(L2M_THREADS, 2) l2m_range_kernel(const float* __restrict__ Q, const float* __restrict__ C,
                                                                const float* __restrict__ CB, const float* __restrict__ cbx,
                                                                const float* __restrict__ rec,
                                                                const int32_t* __restrict__ probes, int64_t npairs, int nprobe, int d,
                                                                int m, float* __restrict__ lo_out, uint32_t* __restrict__ range_bits,
                                                                int64_t* __restrict__ counters) {
    constexpr int KH = L2M<DSUB>::KH, KS = L2M<DSUB>::KS, P = 32 * CT;
    __shared__ uint32_t lo_key[L2M_THREADS], hi_key[L2M_THREADS];        // [pair][4]: this round's four sub-quantisers
    __shared__ uint32_t list[4][L2M_LIST1];                  // per wave: pair << 16 | j << 8 | codeword
    __shared__ int s_cnt[4];
    __shared__ float s_rng[P];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col = lane & 31, half = lane >> 5;
    const int64_t pair0 = (int64_t)blockIdx.x * P;
    const int np = (int)min((int64_t)P, npairs - pair0);
    lo_key[threadIdx.x] = 0xFFFFFFFFu; hi_key[threadIdx.x] = 0u;
    if (threadIdx.x < P) s_rng[threadIdx.x] = 0.0f;
    unsigned long long evaluated = 0, overflows = 0;                   // thread 0's tally
    const float inf = __builtin_inff();

    const int jslice = m / (int)gridDim.y;                            // (a multiple of 4)
    for (int j0 = blockIdx.y * jslice; j0 < (int)(blockIdx.y + 1) * jslice; j0 += 4) {
        __syncthreads();                                               // keys reset, the previous round's list consumed
        const int j = j0 + wave;
        float bv[CT][KS];
        int pl[CT];
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            pl[ct] = ct * 32 + col;
            load_slot<KS>(rec + rec_slot(pair0 + min(pl[ct], np - 1), j, half, m) * KS, bv[ct]);
        }
        float rmn[CT], rmx[CT];
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) { rmn[ct] = inf; rmx[ct] = -inf; }
        int cnt = 0;                                                   // wave-uniform: entries on this wave's list
        float av[KS];
        load_slot<KS>(cbx + (((uint32_t)j * KSUB + col) * 2 + half) * KS, av);
#pragma unroll 1
        for (int t = 0; t < 8; ++t) {
            float an[KS];
            load_slot<KS>(cbx + (((uint32_t)j * KSUB + min(t + 1, 7) * 32 + col) * 2 + half) * KS, an);
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                const f32x16 v = tile_product<KH, KS>(av, bv[ct]);
                float mn = fminf(fminf(fminf(v[0], v[1]), fminf(v[2], v[3])), fminf(fminf(v[4], v[5]), fminf(v[6], v[7])));
                mn = fminf(mn, fminf(fminf(fminf(v[8], v[9]), fminf(v[10], v[11])), fminf(fminf(v[12], v[13]), fminf(v[14], v[15]))));
                float mx = fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])), fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7])));
                mx = fmaxf(mx, fmaxf(fmaxf(fmaxf(v[8], v[9]), fmaxf(v[10], v[11])), fmaxf(fmaxf(v[12], v[13]), fmaxf(v[14], v[15]))));
                mn = fminf(mn, __shfl_xor(mn, 32));                    // the column's other 16 rows
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                rmn[ct] = fminf(rmn[ct], mn);
                rmx[ct] = fmaxf(rmx[ct], mx);
                const float marg = 2.0f * bv[ct][KH];
                const float lo_cut = rmn[ct] + marg, hi_cut = rmx[ct] - marg;
                uint32_t mask = 0;
#pragma unroll
                for (int i = 0; i < 16; ++i) mask |= (!(v[i] > lo_cut && v[i] < hi_cut) ? 1u : 0u) << i;   // (a NaN anywhere: candidate)
                if (pl[ct] >= np) mask = 0;
                // Lanes with candidates append them to the wave's list, one per lane and turn: positions from a
                // ballot, the count in a scalar register, nothing to wait for.
                while (true) {
                    const uint64_t b = __builtin_amdgcn_ballot_w64(mask != 0);
                    if (!b) break;
                    if (mask) {
                        const int i = __builtin_ctz(mask);
                        mask &= mask - 1;
                        const int pos = cnt + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(b >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b, 0));
                        if (pos < L2M_LIST1) list[wave][pos] = (uint32_t)(pl[ct] << 16 | j << 8 | (t * 32 + tile_row(i, half)));
                    }
                    cnt += __builtin_popcountll(b);
                }
            }
#pragma unroll
            for (int x = 0; x < KS; ++x) av[x] = an[x];
        }
        if (lane == 0) s_cnt[wave] = cnt;
        __syncthreads();
        // The candidates by the definition; a wave whose list overflowed makes the round evaluate every entry.
        const int c0 = s_cnt[0], c1 = s_cnt[1], c2 = s_cnt[2], c3 = s_cnt[3];
        const bool all = c0 > L2M_LIST1 || c1 > L2M_LIST1 || c2 > L2M_LIST1 || c3 > L2M_LIST1;
        const int total = all ? np * 4 * KSUB : c0 + c1 + c2 + c3;
        for (int e = threadIdx.x; e < total; e += L2M_THREADS) {
            uint32_t w;
            if (all) w = (uint32_t)((e / (4 * KSUB)) << 16 | (j0 + (e / KSUB) % 4) << 8 | (e % KSUB));
            else w = e < c0 ? list[0][e] : e < c0 + c1 ? list[1][e - c0] : e < c0 + c1 + c2 ? list[2][e - c0 - c1] : list[3][e - c0 - c1 - c2];
            const int p = w >> 16, jj = (w >> 8) & 255, c = w & 255;
            const int64_t q = (pair0 + p) / nprobe;
            const int l = probes[pair0 + p];
            const float L = l2_entry<DSUB>(Q + q * d + jj * DSUB, C + (int64_t)l * d + jj * DSUB, CB + ((int64_t)jj * KSUB + c) * DSUB, DSUB);
            const uint32_t k = okey(L);
            atomicMin(&lo_key[p * 4 + (jj - j0)], k);
            atomicMax(&hi_key[p * 4 + (jj - j0)], k);
        }
        __syncthreads();
        {
            const int p = threadIdx.x >> 2, jj = threadIdx.x & 3;
            if (p < np) {
                const float lo = okey_inv(lo_key[threadIdx.x]), hi = okey_inv(hi_key[threadIdx.x]);
                lo_out[lo_index(pair0 + p, j0 + jj, m)] = lo;
                const float rng = hi - lo;
                if (rng > 0.0f) atomicMax(reinterpret_cast<uint32_t*>(&s_rng[p]), __float_as_uint(rng));
            }
            lo_key[threadIdx.x] = 0xFFFFFFFFu; hi_key[threadIdx.x] = 0u;
        }
        evaluated += (unsigned long long)total;
        overflows += all ? 1ull : 0ull;
    }
    __syncthreads();
    if (threadIdx.x < np) {
        const float rng = s_rng[threadIdx.x];
        if (rng > 0.0f) atomicMax(range_bits + (pair0 + threadIdx.x) / nprobe, __float_as_uint(rng));
    }
    if (threadIdx.x == 0) {
        atomicAdd(reinterpret_cast<unsigned long long*>(counters + 4), evaluated);
        if (overflows) atomicAdd(reinterpret_cast<unsigned long long*>(counters + 5), overflows);
    }
}

// ---- pass 2
// CT column tiles of 32 pairs per workgroup; with gridDim.y > 1, blockIdx.y picks the plane.
template <int DSUB, int CT, bool DBG>
__global__ void __launch_bounds__(L2M_THREADS, 3) l2m_quant_kernel(const float* __restrict__ Q, const float* __restrict__ C,
                                                                const float* __restrict__ CB, const float* __restrict__ cbx,
                                                                const float* __restrict__ rec,
                                                                const int32_t* __restrict__ probes, int64_t npairs, int nprobe, int d,
                                                                int m, const float* __restrict__ lo_in, const uint32_t* __restrict__ range_bits,
                                                                uint8_t* __restrict__ tables, int32_t* __restrict__ bias,
                                                                float* __restrict__ delta, uint8_t* __restrict__ out_LUT8,
                                                                int64_t* __restrict__ counters) {
    constexpr int KH = L2M<DSUB>::KH, KS = L2M<DSUB>::KS, P = 32 * CT;
    extern __shared__ __align__(16) uint8_t smem[];
    uint32_t* list = reinterpret_cast<uint32_t*>(smem);            // [4][L2M_LIST2] per wave: pair << 16 | j << 8 | codeword
    __shared__ int s_cnt[4];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col = lane & 31, half = lane >> 5;
    const int64_t pair0 = (int64_t)blockIdx.x * P;
    const int np = (int)min((int64_t)P, npairs - pair0);
    const int S = rago_steps(m);
    const int planes = rago_planes(m);
    constexpr float ETA_SCALE = (1.0f + 4.0f / L2M<DSUB>::CE) * 1.001f;
    int cnt = 0;                                                    // wave-uniform: entries on this wave's list
    uint32_t* mylist = list + wave * L2M_LIST2;
    uint8_t* tr = smem + 4 * L2M_LIST2 * 4;                         // [32 pairs][8 codewords][32 bytes], rows padded

    // A round = (column tile of 32 pairs, plane); the four waves take a quarter of the plane's 32 slots each (8
    // sub-quantisers) and put their 8-byte pieces of every 32-byte row together in LDS before storing.  With
    // m = 16 the slots 16..31 repeat the slots 0..15: waves 2 and 3 compute what waves 0 and 1 compute.
    const int pb = gridDim.y > 1 ? (int)blockIdx.y : 0, pn = gridDim.y > 1 ? 1 : planes;      // this workgroup's planes
    for (int rd = 0; rd < CT * pn; ++rd) {
        const int ct = rd / pn, plane = pb + rd - ct * pn;
        const int pl = ct * 32 + col;
        const bool valid = pl < np;
        const bool lists = valid && wave * 8 < S;                   // (a repeated slot's undecided entries are listed once)
        const int64_t pair = pair0 + min(pl, np - 1);
        const float inv = 1.0f / lut_step(__uint_as_float(range_bits[pair / nprobe]));
        const float* recp = rec + rec_slot(pair, 0, half, m) * KS;      // + j * 64 KS: the slot of sub-quantiser j
        const float* lop = lo_in + lo_index(pair, 0, m);                // + j * 32
        uint8_t* tab0 = tables + pair0 * LUT_BYTES + (int64_t)plane * LUT_PLANE;      // (of the workgroup's first pair)
        uint8_t* dbg = DBG ? out_LUT8 + pair * m * KSUB : nullptr;
        const int jfirst = plane * 32 + ((wave * 8) & (S - 1));
        // Operands of step (t, jj): codeword slot, pair slot, the sub-table's minimum.  They are requested L2M_AHEAD
        // steps ahead (past the end of the round: steps of its last tile again): a load from L2 or HBM takes several steps.
        auto load_step = [&](int t, int jj, float (&a)[KS], float (&b)[KS], float& lo) {
            const int j = jfirst + jj;
            load_slot<KS>(cbx + (((uint32_t)j * KSUB + t * 32 + col) * 2 + half) * KS, a);
            load_slot<KS>(recp + (uint32_t)j * 64 * KS, b);
            lo = lop[j * 32];
        };
        float an[L2M_AHEAD][KS], bn[L2M_AHEAD][KS], lon[L2M_AHEAD];      // ring: slot s mod L2M_AHEAD holds step s, then is refilled for step s + L2M_AHEAD
#pragma unroll
        for (int s = 0; s < L2M_AHEAD; ++s) load_step(0, s, an[s], bn[s], lon[s]);
#pragma unroll 1
        for (int t = 0; t < 8; ++t) {
            // pk[i][0..1]: the 8 code bytes of (pair, codeword row i).  A word of four bytes is built per group of four
            // sub-quantisers and shifted in at the top, so that no register is indexed by a loop variable.
            uint32_t pk[16][2];
#pragma unroll
            for (int i = 0; i < 16; ++i) { pk[i][0] = 0u; pk[i][1] = 0u; }
#pragma unroll 1
            for (int g = 0; g < 2; ++g) {
                uint32_t word[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) word[i] = 0u;
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const int j = jfirst + g * 4 + s;
                    float av[KS], bv[KS];
                    constexpr int R = L2M_AHEAD;
#pragma unroll
                    for (int x = 0; x < KS; ++x) { av[x] = an[s % R][x]; bv[x] = bn[s % R][x]; }
                    const float lo = lon[s % R];
                    {
                        const int nx = g * 4 + s + R;
                        load_step(min(t + (nx >> 3), 7), nx & 7, an[s % R], bn[s % R], lon[s % R]);
                    }
                    const float nlo = -lo * inv;
                    const float eta = __fmaf_rn(bv[KH], ETA_SCALE * inv, 1.220703125e-4f);
                    const f32x16 v = tile_product<KH, KS>(av, bv);
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const float b = __fmaf_rn(v[i], inv, nlo);
                        word[i] = __builtin_amdgcn_cvt_pk_u8_f32(b, s, word[i]);
                        // undecided (a NaN or infinite b~ or eta included): on the list
                        if (__builtin_expect(__builtin_amdgcn_ballot_w64(!(fabsf(__builtin_amdgcn_fractf(b) - 0.5f) > eta)) != 0, 0)) {
                            const bool amb = lists && !(fabsf(__builtin_amdgcn_fractf(b) - 0.5f) > eta);
                            const uint64_t bal = __builtin_amdgcn_ballot_w64(amb);
                            if (amb) {
                                const int pos = cnt + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0));
                                if (pos < L2M_LIST2) mylist[pos] = (uint32_t)(pl << 16 | j << 8 | (t * 32 + tile_row(i, half)));
                            }
                            cnt += __builtin_popcountll(bal);
                        }
                        if (DBG && lists) dbg[(int64_t)j * KSUB + t * 32 + tile_row(i, half)] = (uint8_t)(word[i] >> (8 * s));
                    }
                }
#pragma unroll
                for (int i = 0; i < 16; ++i) { pk[i][0] = pk[i][1]; pk[i][1] = word[i]; }
            }
            // To HBM through a transposition in LDS: a lane holds one pair and 16 codewords, but lanes that store
            // together should cover consecutive bytes of one pair's table (tables of different pairs lie 32 KiB apart)
            // and whole 32-byte rows should reach memory at once.  Four turns of 8 codewords: every wave writes its
            // 8-byte pieces, then stores a quarter of the 8 KiB.
#pragma unroll
            for (int qt = 0; qt < 4; ++qt) {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<uint2*>(tr + col * L2M_TRS + (half * 4 + q) * 32 + wave * 8) = make_uint2(pk[qt * 4 + q][0], pk[qt * 4 + q][1]);
                __syncthreads();
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                    const int x = (wave * 2 + r) * 64 + lane;              // 16-byte piece of the buffer
                    const int pr = x >> 4, within = x & 15;
                    const uint4 w = *reinterpret_cast<const uint4*>(tr + pr * L2M_TRS + within * 16);
                    if (ct * 32 + pr < np)
                        *reinterpret_cast<uint4*>(tab0 + (int64_t)(ct * 32 + pr) * LUT_BYTES + (t * 32 + qt * 8) * 32 + within * 16) = w;
                }
                __syncthreads();
            }
        }
    }
    if (lane == 0) s_cnt[wave] = cnt;
    // The packed stores are ordered before the single-byte corrections by the barrier's workgroup-scope release:
    // both come from this workgroup and go through the same L2.  (A device-scope fence here makes every
    // workgroup write back its XCD's L2 and costs more than the whole computation.)
    __syncthreads();
    const int c0 = s_cnt[0], c1 = s_cnt[1], c2 = s_cnt[2], c3 = s_cnt[3];
    const bool all = c0 > L2M_LIST2 || c1 > L2M_LIST2 || c2 > L2M_LIST2 || c3 > L2M_LIST2;
    const int jb = pb * 32, jn = gridDim.y > 1 ? S : m;            // this workgroup's sub-quantisers
    const int total = all ? np * jn * KSUB : c0 + c1 + c2 + c3;
    for (int e = threadIdx.x; e < total; e += L2M_THREADS) {
        uint32_t w;
        if (all) w = (uint32_t)((e / (jn * KSUB)) << 16 | (jb + (e / KSUB) % jn) << 8 | (e % KSUB));
        else w = e < c0 ? list[e] : e < c0 + c1 ? list[L2M_LIST2 + e - c0] : e < c0 + c1 + c2 ? list[2 * L2M_LIST2 + e - c0 - c1]
                                                                                               : list[3 * L2M_LIST2 + e - c0 - c1 - c2];
        const int p = w >> 16, j = (w >> 8) & 255, c = w & 255;
        const int64_t q = (pair0 + p) / nprobe;
        const int l = probes[pair0 + p];
        const float L = l2_entry<DSUB>(Q + q * d + j * DSUB, C + (int64_t)l * d + j * DSUB, CB + ((int64_t)j * KSUB + c) * DSUB, DSUB);
        const float step = lut_step(__uint_as_float(range_bits[q]));
        float rr = rintf(__fdiv_rn(L - lo_in[lo_index(pair0 + p, j, m)], step));
        rr = rr < 0.0f ? 0.0f : (rr > 255.0f ? 255.0f : rr);
        const uint8_t v = (uint8_t)rr;
        uint8_t* tab = tables + (pair0 + p) * LUT_BYTES + (int64_t)(j >> 5) * LUT_PLANE + c * 32;
        for (int rep = j & (S - 1); rep < 32; rep += S) tab[rep] = v;
        if (DBG) out_LUT8[((pair0 + p) * m + j) * KSUB + c] = v;
    }
    if (threadIdx.x < np && blockIdx.y == 0) {
        const int p = threadIdx.x;
        const float step = lut_step(__uint_as_float(range_bits[(pair0 + p) / nprobe]));
        double losum = 0.0;                      // in index order (the order that defines the bias)
        for (int j = 0; j < m; ++j) losum = losum + (double)lo_in[lo_index(pair0 + p, j, m)];
        bias[pair0 + p] = (int32_t)rint(losum / (double)step);
        if ((pair0 + p) % nprobe == 0) delta[(pair0 + p) / nprobe] = step;
    }
    if (threadIdx.x == 0) {
        atomicAdd(reinterpret_cast<unsigned long long*>(counters + 4), (unsigned long long)total);
        if (all) atomicAdd(reinterpret_cast<unsigned long long*>(counters + 5), 1ull);
    }
}

// Per dimension the largest |codeword coordinate|; the codeword-side operand [m][256][2][KS] (see the head of
// the file; |cb|^2 is an fp64 sum rounded once).
__global__ void __launch_bounds__(256) cb_stats_kernel(const float* __restrict__ CB, int d, int m, int dsub, float* __restrict__ absmax,
                                                       float* __restrict__ cbx) {
    const int x = blockIdx.x * 256 + threadIdx.x;
    if (x < d) {
        const int j = x / dsub, t = x - j * dsub;
        float mx = 0.0f;
        for (int c = 0; c < KSUB; ++c) mx = fmaxf(mx, fabsf(CB[((int64_t)j * KSUB + c) * dsub + t]));
        absmax[x] = mx;
    }
    if (x < m * KSUB && dsub % 2 == 0) {
        const int H = dsub / 2, KH = H + 1, KS = KH + 1;
        double acc = 0.0;
        float* o = cbx + (int64_t)x * 2 * KS;
        for (int t = 0; t < dsub; ++t) {
            const float f = CB[(int64_t)x * dsub + t];
            o[(t / H) * KS + (t % H)] = f;
            acc = acc + (double)f * (double)f;
        }
        o[KH - 1] = 1.0f;           o[KH] = 0.0f;
        o[KS + KH - 1] = (float)acc; o[KS + KH] = 0.0f;
    }
}

template <int DSUB, int CT>
int launch_l2m_passes(rago_index* idx, const float* q, const int32_t* probes, int64_t npairs, int nprobe, const float* rec, float* lo,
                      uint32_t* range_bits, uint8_t* out_LUT8, int gy, hipStream_t st) {
    Workspace& ws = idx->ws;
    const int d = idx->d, m = idx->m;
    const size_t lds2 = (size_t)4 * L2M_LIST2 * 4 + (size_t)32 * L2M_TRS;      // 41 KB
    const dim3 grid((unsigned)((npairs + 32 * CT - 1) / (32 * CT)), (unsigned)gy);
    l2m_range_kernel<DSUB, CT><<<grid, L2M_THREADS, 0, st>>>(q, idx->centroids, idx->codebooks, idx->cbx, rec, probes, npairs, nprobe,
                                                             d, m, lo, range_bits, ws.counters.as<int64_t>());
    if (out_LUT8)
        l2m_quant_kernel<DSUB, CT, true><<<grid, L2M_THREADS, lds2, st>>>(q, idx->centroids, idx->codebooks, idx->cbx, rec, probes, npairs, nprobe, d,
                                                                          m, lo, range_bits, ws.tmp_lut8sw.as<uint8_t>(), ws.bias.as<int32_t>(),
                                                                          ws.delta.as<float>(), out_LUT8, ws.counters.as<int64_t>());
    else
        l2m_quant_kernel<DSUB, CT, false><<<grid, L2M_THREADS, lds2, st>>>(q, idx->centroids, idx->codebooks, idx->cbx, rec, probes, npairs, nprobe, d,
                                                                           m, lo, range_bits, ws.tmp_lut8sw.as<uint8_t>(), ws.bias.as<int32_t>(),
                                                                           ws.delta.as<float>(), nullptr, ws.counters.as<int64_t>());
    RAGO_HIP(hipGetLastError());
    return RAGO_OK;
}

template <int DSUB>
int launch_l2m(rago_index* idx, const float* q, const int32_t* probes, int64_t npairs, int nprobe, float* lo, uint32_t* range_bits,
               uint8_t* out_LUT8, hipStream_t st) {
    Workspace& ws = idx->ws;
    const int d = idx->d, m = idx->m;
    int rc;
    const int64_t npad = (npairs + 31) / 32 * 32;                     // whole tiles of 32 pairs
    if ((rc = ws.l2_r.reserve((size_t)npad * m * 2 * L2M<DSUB>::KS * 4))) return rc;
    if (idx->reserving) return RAGO_OK;
    float* rec = ws.l2_r.as<float>();
    l2m_prepare_kernel<DSUB><<<(unsigned)((npad * m + 255) / 256), 256, 0, st>>>(q, idx->centroids, idx->cb_absmax, probes, npairs, nprobe, d, m, rec);
    // Large batches: 64 pairs per workgroup (each codeword load serves two column tiles).  Fewer than ~4 such
    // workgroups per CU: 32 pairs per workgroup and one workgroup per plane, so that the launch still fills the chip.
    if ((npairs + 63) / 64 >= 1024) return launch_l2m_passes<DSUB, 2>(idx, q, probes, npairs, nprobe, rec, lo, range_bits, out_LUT8, 1, st);
    return launch_l2m_passes<DSUB, 1>(idx, q, probes, npairs, nprobe, rec, lo, range_bits, out_LUT8, rago_planes(m), st);
}

}  // namespace

int launch_cb_stats(rago_index* idx, hipStream_t st) {
    const int n = std::max(idx->d, idx->m * KSUB);
    cb_stats_kernel<<<(n + 255) / 256, 256, 0, st>>>(idx->codebooks, idx->d, idx->m, idx->dsub, idx->cb_absmax, idx->cbx);
    RAGO_HIP(hipGetLastError());
    return RAGO_OK;
}

bool lut_l2_fast_supported(const rago_index* idx) {
    const int dsub = idx->dsub;
    return (dsub == 4 || dsub == 8 || dsub == 16) && idx->m % 16 == 0;
}

// Both passes for all pairs.  `lo` (fp32, m floats per pair with the number of pairs rounded up to a multiple of 32)
// and `range_bits` [nq] (zeroed) are workspace; the
// tables, bias and step land in the workspace members the scan reads.
int launch_lut_l2_fast(rago_index* idx, const float* q, const int32_t* probes, int64_t npairs, int nprobe, float* lo, uint32_t* range_bits,
                       uint8_t* out_LUT8, hipStream_t st) {
    switch (idx->dsub) {
        case 4: return launch_l2m<4>(idx, q, probes, npairs, nprobe, lo, range_bits, out_LUT8, st);
        case 8: return launch_l2m<8>(idx, q, probes, npairs, nprobe, lo, range_bits, out_LUT8, st);
        case 16: return launch_l2m<16>(idx, q, probes, npairs, nprobe, lo, range_bits, out_LUT8, st);
    }
    return fail(RAGO_UNSUPPORTED, "sub-vector length without a fast Euclidean table path");
}

}  // namespace rago

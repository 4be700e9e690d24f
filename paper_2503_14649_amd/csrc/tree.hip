// Probe selection through an upper level over the lists (the paper's database is a multi-level
// tree, Section 4 "Models and database"; searching an upper level is itself a vector scan,
// Section 4 "Retrieval performance modeling").  The lists are partitioned into groups with a
// centroid each; a query scores the group centroids, keeps the nsp best groups, scores only the
// lists of those groups and takes the nprobe best of them.  For a single query this replaces
// the read of all nlist centroids (201 MB at 65536 x 768) by nsuper + nsp * (lists per group)
// rows, which is what the latency of small batches is made of.
//
// Every score is computed once, exactly as the oracle states it (fp64 accumulation, one rounding
// to fp32), so there is no approximate stage to correct: keys (ordered score << 32 | ~row) are
// sorted in LDS and the best taken; ties go to the lower row number by construction of the key.
#include <algorithm>

#include "rago_internal.h"

namespace rago {

constexpr int TREE_CAP = 8192;     // candidate rows per query at either level (LDS sort: 64 KiB of keys)
constexpr int TREE_ROWS = 32;      // rows per scoring workgroup (4 waves x 8 rows in flight)

__device__ __forceinline__ uint32_t tree_float_key(float f) {  // ascending uint order == ascending float order
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Scores of rows ids[first .. first + count) of `rows` against query vector qv -> keys[first ..].
// One wave per row, eight rows per wave in flight.  (ids null: row number = position)
__device__ __forceinline__ void tree_score_rows(const float* __restrict__ qv, const float* __restrict__ rows, const int32_t* __restrict__ ids,
                                                int first, int count, int d, int metric, uint64_t* __restrict__ keys) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    constexpr int RU = 8;
    for (int r0 = wave * RU; r0 < count; r0 += 4 * RU) {
        double acc[RU];
        const float* rv[RU];
        int id[RU];
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            const int pos = first + min(r0 + u, count - 1);
            id[u] = ids ? ids[pos] : pos;
            rv[u] = rows + (int64_t)id[u] * d;
            acc[u] = 0.0;
        }
        if (metric == 1) {
            for (int t = lane; t < d; t += 64) {
                const double qt = (double)qv[t];
#pragma unroll
                for (int u = 0; u < RU; ++u) {
                    const double diff = qt - (double)rv[u][t];
                    acc[u] = acc[u] + diff * diff;
                }
            }
        } else {
            for (int t = lane; t < d; t += 64) {
                const double qt = (double)qv[t];
#pragma unroll
                for (int u = 0; u < RU; ++u) acc[u] = acc[u] + qt * (double)rv[u][t];
            }
        }
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            for (int o = 32; o; o >>= 1) acc[u] = acc[u] + __shfl_xor(acc[u], o);
            if (lane == 0 && r0 + u < count) {
                const float s = metric == 1 ? (float)(-acc[u]) : (float)acc[u];
                keys[first + r0 + u] = ((uint64_t)tree_float_key(s) << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)id[u]);
            }
        }
    }
}

// Level 1: every group centroid.  grid (nq, ceil(nsuper / TREE_ROWS)).
__global__ void __launch_bounds__(256) tree_score_groups_kernel(const float* __restrict__ Q, const float* __restrict__ SC, int nsuper, int d,
                                                                int metric, uint64_t* __restrict__ keys) {
    const int64_t q = blockIdx.x;
    const int first = blockIdx.y * TREE_ROWS;
    tree_score_rows(Q + q * d, SC, nullptr, first, min(TREE_ROWS, nsuper - first), d, metric, keys + q * TREE_CAP);
}

// Level 2: the lists of the kept groups.  grid (nq, nsp, ceil(largest group / TREE_ROWS)).  The
// candidates of a query are laid out group after group in the order the groups were kept.
__global__ void __launch_bounds__(256) tree_score_members_kernel(const float* __restrict__ Q, const float* __restrict__ C,
                                                                 const int64_t* __restrict__ super_off, const int32_t* __restrict__ super_lists,
                                                                 const int32_t* __restrict__ kept, int nsp, int d, int metric,
                                                                 uint64_t* __restrict__ keys) {
    const int64_t q = blockIdx.x;
    const int i = blockIdx.y;
    const int32_t* kq = kept + q * nsp;
    const int s = kq[i];
    const int size = (int)(super_off[s + 1] - super_off[s]);
    const int first_in_group = blockIdx.z * TREE_ROWS;
    if (first_in_group >= size) return;
    int base = 0;                               // candidates of the groups kept before this one
    for (int j = 0; j < i; ++j) base += (int)(super_off[kq[j] + 1] - super_off[kq[j]]);
    // (keys + base - super_off[s] + position in super_lists = position in the candidate array)
    tree_score_rows(Q + q * d, C, super_lists, (int)super_off[s] + first_in_group, min(TREE_ROWS, size - first_in_group), d, metric,
                    keys + q * TREE_CAP + base - (int)super_off[s]);
}

// The `want` best of a query's candidate keys -> their row numbers, best first.  One workgroup per
// query, bitonic sort in LDS.  `kept` null: the candidates are rows 0 .. ncand_const - 1 (level 1).
// Else (level 2) their number is the total size of the kept groups, and if that is less than `want`
// the lowest-numbered lists of the other groups fill up (they count as -inf, ties to the lower list).
__global__ void __launch_bounds__(1024) tree_pick_kernel(const uint64_t* __restrict__ keys, int ncand_const, const int32_t* __restrict__ kept,
                                                         int nsp, const int64_t* __restrict__ super_off, const int32_t* __restrict__ super_of,
                                                         int nlist, int want, int32_t* __restrict__ out) {
    extern __shared__ __align__(16) uint64_t sk[];      // the keys, padded to a power of two (sized by the host)
    __shared__ int s_ncand;
    const int64_t q = blockIdx.x;
    const int tid = threadIdx.x;
    if (tid == 0) {
        int n = ncand_const;
        if (kept) {
            n = 0;
            for (int j = 0; j < nsp; ++j) n += (int)(super_off[kept[q * nsp + j] + 1] - super_off[kept[q * nsp + j]]);
        }
        s_ncand = n;
    }
    __syncthreads();
    const int ncand = s_ncand;
    int n2 = 1;
    while (n2 < ncand) n2 <<= 1;
    for (int i = tid; i < n2; i += 1024) sk[i] = i < ncand ? keys[q * TREE_CAP + i] : 0ull;   // 0 sorts below every real key
    for (int size = 2; size <= n2; size <<= 1)
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            for (int t = tid; t < n2 / 2; t += 1024) {
                const int i = 2 * t - (t & (stride - 1)), j = i + stride;
                const bool up = (i & size) == 0;      // this sub-sequence ends largest-first
                const uint64_t a = sk[i], b = sk[j];
                if (up ? b > a : a > b) { sk[i] = b; sk[j] = a; }
            }
        }
    __syncthreads();
    const int have = min(want, ncand);
    for (int p = tid; p < have; p += 1024) out[q * want + p] = (int32_t)(0xFFFFFFFFu - (uint32_t)sk[p]);
    if (have < want && tid == 0) {
        int p = have;
        for (int l = 0; l < nlist && p < want; ++l) {
            bool in_kept = false;
            for (int j = 0; j < nsp; ++j) in_kept |= kept[q * nsp + j] == super_of[l];
            if (!in_kept) out[q * want + p++] = l;
        }
    }
}

int launch_select_tree(rago_index* idx, const float* q, int64_t nq, int nprobe, int32_t* probes, hipStream_t st) {
    Workspace& ws = idx->ws;
    const int nsuper = idx->nsuper, nsp = idx->nsp, d = idx->d;
    int rc;
    if ((rc = ws.S.reserve((size_t)nq * TREE_CAP * 8))) return rc;            // candidate keys (the score matrix is not needed)
    if ((rc = ws.cand_idx.reserve((size_t)nq * nsp * 4))) return rc;          // kept groups
    if (nq > 0x7fffffff) return fail(RAGO_UNSUPPORTED, "nq too large");
    if (idx->reserving) return RAGO_OK;
    uint64_t* keys = ws.S.as<uint64_t>();
    int32_t* kept = ws.cand_idx.as<int32_t>();
    tree_score_groups_kernel<<<dim3((unsigned)nq, (unsigned)((nsuper + TREE_ROWS - 1) / TREE_ROWS)), 256, 0, st>>>(q, idx->sup_cen, nsuper, d,
                                                                                                            idx->metric, keys);
    static OncePerDevice attr;
    if (attr.first()) {
        RAGO_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(tree_pick_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, TREE_CAP * 8));
    }
    auto pow2 = [](int n) { int p = 1; while (p < n) p <<= 1; return p; };
    tree_pick_kernel<<<(unsigned)nq, 1024, (size_t)pow2(nsuper) * 8, st>>>(keys, nsuper, nullptr, 0, nullptr, nullptr, 0, nsp, kept);
    tree_score_members_kernel<<<dim3((unsigned)nq, (unsigned)nsp, (unsigned)((idx->max_group + TREE_ROWS - 1) / TREE_ROWS)), 256, 0, st>>>(
        q, idx->centroids, idx->sup_off, idx->sup_lists, kept, nsp, d, idx->metric, keys);
    // (a query's candidates: at most nsp * largest group <= TREE_CAP, checked when nsp is set)
    tree_pick_kernel<<<(unsigned)nq, 1024, (size_t)pow2(std::max(1, std::min(TREE_CAP, nsp * idx->max_group))) * 8, st>>>(
        keys, 0, kept, nsp, idx->sup_off, idx->sup_of, idx->nlist, nprobe, probes);
    RAGO_HIP(hipGetLastError());
    return RAGO_OK;
}

int tree_cap() { return TREE_CAP; }

}  // namespace rago

// Internal declarations shared by the translation units of librago (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>

#include "../../include/rago.h"
#include "lut_common.h"

namespace rago {

constexpr int KSUB = 256;          // codewords per sub-quantiser
constexpr int BLOCK_VECS = 64;     // vectors per code block = one wavefront, one vector per lane
constexpr int KMAX = 128;          // largest k served by the wave-level selection buffers
constexpr int LUT_PLANE = KSUB * 32;       // bytes of one plane of a table: [c][slot], 32 sub-quantisers
constexpr int LUT_BYTES = 4 * LUT_PLANE;   // stride of one 8-bit table in HBM (planes * LUT_PLANE bytes used)

void set_error(const std::string& msg);
int fail(int code, const std::string& msg);

// "Has this been done on the current device yet?"  Kernel attributes (a larger dynamic LDS limit) are per device,
// so a process that drives several GPUs has to set them on each.  Races between threads are harmless: the
// attribute call is idempotent.
struct OncePerDevice {
    bool done[64] = {};
    bool first() {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return true;
        if (done[dev]) return false;
        done[dev] = true;
        return true;
    }
};
#define RAGO_HIP(call)                                                                       \
    do {                                                                                     \
        hipError_t e_ = (call);                                                              \
        if (e_ != hipSuccess)                                                                \
            return ::rago::fail(RAGO_DEVICE, std::string(#call) + ": " + hipGetErrorString(e_)); \
    } while (0)

// Grow-only device buffer.  Growing frees and allocates (which synchronises the device), so a caller
// that must not do either sizes the workspace once with rago_index_reserve; searches on that index then
// run with growth switched off (NoGrowScope) and fail with RAGO_UNSUPPORTED rather than allocate.
struct DevBuf {
    void* p = nullptr;
    size_t cap = 0;
    int reserve(size_t bytes);   // RAGO_OK / RAGO_OOM / RAGO_UNSUPPORTED (growth switched off)
    void release();
    template <class T> T* as() const { return static_cast<T*>(p); }
};

struct NoGrowScope {             // while alive on this thread, DevBuf::reserve refuses to grow
    bool active;
    explicit NoGrowScope(bool on);
    ~NoGrowScope();
};
long long device_allocations();  // number of times any DevBuf grew (process-wide)
int forced_scan_kernel();        // 0 = pick by sizes, 1 = wide, 2 = narrow, 3 = wave per item (rago_debug_force_scan_kernel)

struct Workspace {
    DevBuf S, cand_idx, probes, probe_scores, T64, Tmin, Tmax, lut8, bias, delta, pair_lo, Lf32;
    DevBuf list_cnt, pair_off, task_off, task_table, pair_sorted, tauq, part_I, part_id, part_cnt, counters;
    DevBuf tmp_lut8sw, amb, patch, touched, qn2, l2_r, sel_redo, sel_small, sel_done, wave_items, wave_q, wave_stage;
    void release();
};

}  // namespace rago

// Steps (lanes advance through this many sub-quantisers) and planes of a code width.
__host__ __device__ inline int rago_steps(int m) { return m < 32 ? m : 32; }
__host__ __device__ inline int rago_planes(int m) { return m < 32 ? 1 : m / 32; }

namespace rago {
constexpr int PROF_CALLS = 64, PROF_EVENTS = 7;
struct Profiler {
    bool on = false;
    bool created = false;
    int ncalls = 0;
    hipEvent_t ev[PROF_CALLS][PROF_EVENTS];
};
}  // namespace rago

struct rago_index {
    int device = 0;
    int d = 0, m = 0, dsub = 0, nlist = 0;   // m = code bytes per vector, dsub = dimensions one byte covers
    int user_m = 0, user_ksub = 256;         // as handed over: with 16-word sub-quantisers user_m = 2 m
    int metric = 0;                // 0 inner product, 1 Euclidean (similarity = minus squared distance)
    int64_t n = 0;
    int64_t max_list_len = 0;
    int64_t total_blocks = 0;
    float* centroids = nullptr;    // [nlist][d]
    float* cnorm = nullptr;        // [nlist] Euclidean norm of each centroid
    float* cn2 = nullptr;          // [nlist] squared norm (fp64 accumulation, one rounding)
    uint16_t* cen_hi = nullptr;    // [nlist][d] bf16(centroid)
    uint16_t* cen_lo = nullptr;    // [nlist][d] bf16(centroid - cen_hi): centroid = hi + lo to 2^-18 relative
    float* codebooks = nullptr;    // [m][256][dsub]
    float* cb_absmax = nullptr;    // [d] largest |codeword coordinate| per dimension (error bounds of the fp32 table path)
    float* cbx = nullptr;          // [m][256][dsub + 4] codeword, its squared norm, three zeros (one address per entry)
    int64_t* list_off = nullptr;   // [nlist+1] vector offsets (list-major rows)
    int64_t* blk_off = nullptr;    // [nlist+1] offsets in 64-vector blocks into codes_blk
    int2* list_meta = nullptr;     // [nlist] {blocks, vectors} of each list: one load where the bookkeeping wants both
    uint8_t* codes_blk = nullptr;  // total_blocks * 64 * m bytes, skewed lane-major layout
    int64_t* ids = nullptr;        // [n]
    float max_cnorm = 0.f;
    // optional upper level over the lists (tree.hip): groups of lists with a centroid each
    int nsuper = 0, nsp = 0, max_group = 0;   // groups, groups kept per query (0: exhaustive list level), largest group
    float* sup_cen = nullptr;      // [nsuper][d]
    int64_t* sup_off = nullptr;    // [nsuper+1] into sup_lists
    int32_t* sup_lists = nullptr;  // [nlist] lists grouped by group, ascending inside a group
    int32_t* sup_of = nullptr;     // [nlist] group of each list
    int n_cu = 0;                  // compute units of `device`
    bool reserving = false;        // rago_index_reserve: the stage launchers size their buffers and return
    bool ws_frozen = false;        // the workspace was sized by rago_index_reserve: searches do not grow it
    int64_t res_nq = 0;            // ... for these maxima
    int res_nprobe = 0, res_k = 0;
    rago::Workspace ws;
    rago::Profiler prof;
    // the scan kernel of the last search (for rago_debug_counters): 1 four pairs per pass, 2 two pairs, 3 wave per item
    int last_scan_kernel = 0;
};

namespace rago {

struct SmallSetupArgs;      // scan_setup.h
struct WavePlanArgs;        // scan_plan.h

// layout.hip
int build_layout(rago_index* idx, const uint8_t* d_codes_plain, hipStream_t st);
int launch_calib_copy(const void* src, void* dst, int64_t bytes, hipStream_t st);
int launch_calib_read(const void* src, int64_t bytes, uint32_t* sink, hipStream_t st);
int read_stream_sink_words();
int launch_expand_pq4(const float* d_cb16, int m, int dsub, float* d_cb256, hipStream_t st);

// coarse.hip
// (zero_select_counter: also clear the counter launch_select adds to, which then need not launch a kernel for it)
int launch_coarse(rago_index* idx, const float* q, int64_t nq, float* S, hipStream_t st, bool zero_select_counter = false);
int launch_split_centroids(rago_index* idx, hipStream_t st);
// (S is read and, for a query whose choice cannot be shown independent of its rounding, overwritten with exact scores)
int launch_select(rago_index* idx, const float* q, float* S, int64_t nq, int nprobe, int32_t* probes,
                  hipStream_t st, bool counter_is_zero = false);

// tree.hip
int launch_select_tree(rago_index* idx, const float* q, int64_t nq, int nprobe, int32_t* probes, hipStream_t st);
int tree_cap();

// lut.hip
// (setup / wave_plan: bookkeeping of the scan that rides in the two kernels, see plan_scan_setup)
int launch_build_lut(rago_index* idx, const float* q, const int32_t* probes, int64_t nq, int nprobe,
                     LutTables* out, float* out_L_f32, uint8_t* out_LUT8, hipStream_t st, const SmallSetupArgs* setup = nullptr,
                     const WavePlanArgs* wave_plan = nullptr);
int launch_swizzle_lut(rago_index* idx, const uint8_t* lut8_plain, int64_t npairs, uint8_t* lut8sw, hipStream_t st);
// Euclidean metric: one full table per pair (plane-major, stride LUT_BYTES) into ws.tmp_lut8sw, biases into
// ws.bias, steps into ws.delta; optional plain copies for inspection.
int launch_cb_stats(rago_index* idx, hipStream_t st);
bool lut_l2_fast_supported(const rago_index* idx);
int launch_lut_l2_fast(rago_index* idx, const float* q, const int32_t* probes, int64_t npairs, int nprobe, float* lo, uint32_t* range_bits,
                       uint8_t* out_LUT8, hipStream_t st);
int launch_build_lut_l2(rago_index* idx, const float* q, const int32_t* probes, int64_t nq, int nprobe, float* out_L_f32,
                        uint8_t* out_LUT8, hipStream_t st);

// scan.hip
// Tables come either per pair (`lut8sw` [npairs][plane][256][32] + `bias`, `tables` null) or as per-query
// base tables with per-pair patches (`tables`, `lut8sw` null).
// (setup_done: the scan's bookkeeping has been run by the caller's kernels, see plan_scan_setup)
int launch_scan(rago_index* idx, const int32_t* probes, const uint8_t* lut8sw, const int32_t* bias,
                const LutTables* tables, const float* delta, int64_t nq, int nprobe, int k, int64_t* out_ids,
                float* out_scores, int32_t* out_iscores, hipStream_t st, hipEvent_t* ev = nullptr, bool setup_done = false);
int plan_scan_setup(rago_index* idx, const int32_t* probes, int64_t nq, int nprobe, int k, bool base_tables, SmallSetupArgs* small,
                    WavePlanArgs* wave);

// flat.hip
int launch_flat(const void* corpus, const void* queries, int R, int64_t n, int nqr, int d, int k,
                int64_t* out_ids, float* out_scores, int device, bool half, hipStream_t st);
int launch_flat_static(const void* corpus, const void* queries, int R, int64_t n, int nqr, int d, int k,
                       int64_t* out_ids, float* out_scores, int device, bool half, hipStream_t st);
int flat_profile(int device, int enable);
int flat_stage_ms(int device, float* out_ms, int32_t* out_calls);

}  // namespace rago

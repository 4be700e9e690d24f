// C ABI of librago: index life-cycle, argument checking, stage sequencing.
#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <memory>
#include <vector>

#include "rago_internal.h"
#include "scan_setup.h"
#include "scan_plan.h"

namespace rago {

static thread_local std::string g_err;
void set_error(const std::string& msg) { g_err = msg; }
int fail(int code, const std::string& msg) { g_err = msg; return code; }

static thread_local int tl_no_grow = 0;
static std::atomic<long long> g_allocations{0};
static std::atomic<int> g_forced_scan{0};
NoGrowScope::NoGrowScope(bool on) : active(on) { if (active) ++tl_no_grow; }
NoGrowScope::~NoGrowScope() { if (active) --tl_no_grow; }
long long device_allocations() { return g_allocations.load(); }
int forced_scan_kernel() { return g_forced_scan.load(); }

int DevBuf::reserve(size_t bytes) {
    if (bytes <= cap) return RAGO_OK;
    if (tl_no_grow)
        return fail(RAGO_UNSUPPORTED, "the call needs more workspace than rago_index_reserve sized (" + std::to_string(bytes) +
                                          " > " + std::to_string(cap) + " bytes); reserve again for larger maxima");
    if (p) { hipFree(p); p = nullptr; cap = 0; }
    size_t want = bytes + bytes / 8 + 256;
    if (hipMalloc(&p, want) != hipSuccess) {
        p = nullptr;
        (void)hipGetLastError();
        return fail(RAGO_OOM, "device allocation of " + std::to_string(want) + " bytes failed");
    }
    ++g_allocations;
    cap = want;
    return RAGO_OK;
}
void DevBuf::release() { if (p) hipFree(p); p = nullptr; cap = 0; }
void Workspace::release() {
    DevBuf* all[] = {&S, &cand_idx, &probes, &probe_scores, &T64, &Tmin, &Tmax, &lut8, &bias, &delta, &pair_lo, &Lf32,
                     &list_cnt, &pair_off, &task_off, &task_table, &pair_sorted, &tauq, &part_I, &part_id, &part_cnt,
                     &counters, &tmp_lut8sw, &amb, &patch, &touched, &qn2, &l2_r, &sel_redo, &sel_small, &sel_done, &wave_items, &wave_q, &wave_stage};
    for (DevBuf* b : all) b->release();
}

static bool supported_m(int m) { return m == 16 || m == 32 || m == 64 || m == 96 || m == 128; }

struct DeviceGuard {
    int prev = -1;
    bool ok = true;
    explicit DeviceGuard(int dev) {
        if (hipGetDevice(&prev) != hipSuccess) prev = -1;
        ok = hipSetDevice(dev) == hipSuccess;
    }
    ~DeviceGuard() { if (prev >= 0) (void)hipSetDevice(prev); }
};

static void destroy(rago_index* idx) {
    if (!idx) return;
    hipFree(idx->centroids); hipFree(idx->cnorm); hipFree(idx->cn2); hipFree(idx->cen_hi); hipFree(idx->cen_lo); hipFree(idx->codebooks); hipFree(idx->cb_absmax); hipFree(idx->cbx); hipFree(idx->list_off);
    hipFree(idx->blk_off); hipFree(idx->list_meta); hipFree(idx->codes_blk); hipFree(idx->ids);
    hipFree(idx->sup_cen); hipFree(idx->sup_off); hipFree(idx->sup_lists); hipFree(idx->sup_of);
    idx->ws.release();
    if (idx->prof.created)
        for (auto& c : idx->prof.ev) for (auto& e : c) hipEventDestroy(e);
    delete idx;
}

// Shape checks + small arrays; leaves codes_blk / ids allocated but unfilled.
// `m` and `ksub` are the caller's: with ksub = 16 two sub-quantisers share a code byte and the
// index continues as an 8-bit one over m/2 bytes (the caller's codebooks are expanded by set_codebooks).
static int prepare(rago_index* idx, int d, int m, int ksub, int nlist, int64_t n, const int64_t* h_list_off, int metric) {
    if (metric != 0 && metric != 1) return fail(RAGO_UNSUPPORTED, "metric must be 0 (inner product) or 1 (Euclidean)");
    idx->metric = metric;
    if (d <= 0 || m <= 0 || nlist <= 0 || n < 0) return fail(RAGO_INVALID_ARG, "non-positive index dimension");
    if (ksub != KSUB && ksub != 16) return fail(RAGO_UNSUPPORTED, "ksub must be 256 or 16");
    if (d % m) return fail(RAGO_UNSUPPORTED, "d must be a multiple of m");
    idx->user_m = m; idx->user_ksub = ksub;
    if (ksub == 16) {
        if (m % 2) return fail(RAGO_UNSUPPORTED, "with ksub = 16, m must be even");
        m /= 2;
        if (!supported_m(m)) return fail(RAGO_UNSUPPORTED, "with ksub = 16, m must be one of 32, 64, 128, 192, 256");
    }
    if (!supported_m(m)) return fail(RAGO_UNSUPPORTED, "m must be one of 16, 32, 64, 96, 128");
    if (d > 4096) return fail(RAGO_UNSUPPORTED, "d > 4096");
    if (h_list_off[0] != 0 || h_list_off[nlist] != n) return fail(RAGO_FORMAT, "list_offsets must start at 0 and end at n");
    std::vector<int64_t> blk(nlist + 1);
    blk[0] = 0;
    int64_t maxlen = 0;
    for (int l = 0; l < nlist; ++l) {
        int64_t len = h_list_off[l + 1] - h_list_off[l];
        if (len < 0) return fail(RAGO_FORMAT, "list_offsets must be non-decreasing");
        if (len > 0x7fffffffLL - 64) return fail(RAGO_UNSUPPORTED, "list longer than 2^31-65 vectors");
        if (len > maxlen) maxlen = len;
        blk[l + 1] = blk[l] + (len + BLOCK_VECS - 1) / BLOCK_VECS;
    }
    idx->d = d; idx->m = m; idx->dsub = d / m; idx->nlist = nlist; idx->n = n;
    idx->max_list_len = maxlen; idx->total_blocks = blk[nlist];
    const size_t code_bytes = (size_t)idx->total_blocks * BLOCK_VECS * m;
    if (hipMalloc(&idx->centroids, sizeof(float) * (size_t)nlist * d) != hipSuccess ||
        hipMalloc(&idx->cnorm, sizeof(float) * (size_t)nlist) != hipSuccess ||
        hipMalloc(&idx->cn2, sizeof(float) * (size_t)nlist) != hipSuccess ||
        hipMalloc(&idx->cen_hi, sizeof(uint16_t) * (size_t)nlist * d) != hipSuccess ||
        hipMalloc(&idx->cen_lo, sizeof(uint16_t) * (size_t)nlist * d) != hipSuccess ||
        hipMalloc(&idx->codebooks, sizeof(float) * (size_t)m * KSUB * idx->dsub) != hipSuccess ||
        hipMalloc(&idx->cb_absmax, sizeof(float) * (size_t)d) != hipSuccess ||
        hipMalloc(&idx->cbx, sizeof(float) * (size_t)m * KSUB * (idx->dsub + 4)) != hipSuccess ||
        hipMalloc(&idx->list_off, sizeof(int64_t) * (size_t)(nlist + 1)) != hipSuccess ||
        hipMalloc(&idx->blk_off, sizeof(int64_t) * (size_t)(nlist + 1)) != hipSuccess ||
        hipMalloc(&idx->list_meta, sizeof(int2) * (size_t)nlist) != hipSuccess ||
        hipMalloc(&idx->codes_blk, code_bytes + 16) != hipSuccess ||
        hipMalloc(&idx->ids, sizeof(int64_t) * (size_t)(n + 1)) != hipSuccess) {
        (void)hipGetLastError();
        return fail(RAGO_OOM, "device allocation for the index failed");
    }
    RAGO_HIP(hipMemcpy(idx->list_off, h_list_off, sizeof(int64_t) * (size_t)(nlist + 1), hipMemcpyHostToDevice));
    RAGO_HIP(hipMemcpy(idx->blk_off, blk.data(), sizeof(int64_t) * (size_t)(nlist + 1), hipMemcpyHostToDevice));
    {   // blocks and vectors of every list in one 8-byte word (lists are shorter than 2^31 vectors: checked above)
        std::vector<int2> meta((size_t)nlist);
        for (int l = 0; l < nlist; ++l) meta[l] = make_int2((int)(blk[l + 1] - blk[l]), (int)(h_list_off[l + 1] - h_list_off[l]));
        RAGO_HIP(hipMemcpy(idx->list_meta, meta.data(), sizeof(int2) * (size_t)nlist, hipMemcpyHostToDevice));
    }
    return RAGO_OK;
}

// Codebooks as the caller holds them ([user_m][user_ksub][d / user_m]) -> idx->codebooks.
static int set_codebooks(rago_index* idx, const float* src, hipMemcpyKind kind) {
    const size_t floats = (size_t)idx->user_m * idx->user_ksub * (idx->d / idx->user_m);
    if (idx->user_ksub == KSUB) {
        RAGO_HIP(hipMemcpy(idx->codebooks, src, floats * 4, kind));
        return RAGO_OK;
    }
    float* small = nullptr;
    if (hipMalloc(&small, floats * 4) != hipSuccess) { (void)hipGetLastError(); return fail(RAGO_OOM, "staging buffer for codebooks"); }
    hipError_t e = hipMemcpy(small, src, floats * 4, kind);
    int rc = e == hipSuccess ? launch_expand_pq4(small, idx->user_m, idx->d / idx->user_m, idx->codebooks, nullptr)
                             : fail(RAGO_DEVICE, std::string("copying codebooks: ") + hipGetErrorString(e));
    hipFree(small);
    return rc;
}

static int finish(rago_index* idx, const uint8_t* d_codes_plain) {
    int rc = build_layout(idx, d_codes_plain, nullptr);
    if (rc) return rc;
    if ((rc = launch_split_centroids(idx, nullptr))) return rc;
    if ((rc = launch_cb_stats(idx, nullptr))) return rc;
    std::vector<float> cn(idx->nlist);
    RAGO_HIP(hipMemcpy(cn.data(), idx->cnorm, sizeof(float) * cn.size(), hipMemcpyDeviceToHost));
    float mx = 0.f;
    for (float v : cn) if (v > mx) mx = v;
    idx->max_cnorm = mx;
    hipDeviceProp_t pr;
    RAGO_HIP(hipGetDeviceProperties(&pr, idx->device));
    idx->n_cu = pr.multiProcessorCount;
    return RAGO_OK;
}

}  // namespace rago

using namespace rago;

extern "C" {

const char* rago_last_error(void) { return g_err.c_str(); }

int rago_index_wrap(const rago_index_arrays* a, int on_device, int device, rago_index** out) {
    if (!a || !out) return fail(RAGO_INVALID_ARG, "null argument");
    if (!a->centroids || !a->codebooks || !a->list_offsets || (a->n > 0 && (!a->codes || !a->ids)))
        return fail(RAGO_INVALID_ARG, "null array in rago_index_arrays");
    if (a->nlist <= 0 || a->d <= 0 || a->m <= 0 || a->n < 0) return fail(RAGO_INVALID_ARG, "non-positive index dimension");
    DeviceGuard g(device);
    if (!g.ok) return fail(RAGO_DEVICE, "hipSetDevice failed");
    const hipMemcpyKind kind = on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
    std::vector<int64_t> off(a->nlist + 1);
    if (on_device) RAGO_HIP(hipMemcpy(off.data(), a->list_offsets, sizeof(int64_t) * off.size(), hipMemcpyDeviceToHost));
    else std::memcpy(off.data(), a->list_offsets, sizeof(int64_t) * off.size());
    rago_index* idx = new rago_index();
    idx->device = device;
    int rc = prepare(idx, a->d, a->m, a->ksub ? a->ksub : KSUB, a->nlist, a->n, off.data(), a->metric);
    uint8_t* plain = nullptr;
    if (!rc) {
        hipError_t e = hipMemcpy(idx->centroids, a->centroids, sizeof(float) * (size_t)a->nlist * a->d, kind);
        if (e == hipSuccess && a->n) e = hipMemcpy(idx->ids, a->ids, sizeof(int64_t) * (size_t)a->n, kind);
        if (e != hipSuccess) rc = fail(RAGO_DEVICE, std::string("copying index arrays: ") + hipGetErrorString(e));
    }
    if (!rc) rc = set_codebooks(idx, a->codebooks, kind);
    if (!rc) {
        if (on_device) {
            rc = finish(idx, a->codes);
        } else {
            const size_t bytes = (size_t)a->n * idx->m;
            if (hipMalloc(&plain, bytes + 16) != hipSuccess) { (void)hipGetLastError(); rc = fail(RAGO_OOM, "staging buffer for codes"); }
            if (!rc && bytes && hipMemcpy(plain, a->codes, bytes, hipMemcpyHostToDevice) != hipSuccess) rc = fail(RAGO_DEVICE, "copying codes");
            if (!rc) rc = finish(idx, plain);
        }
    }
    if (plain) hipFree(plain);
    if (rc) { destroy(idx); return rc; }
    *out = idx;
    return RAGO_OK;
}

int rago_index_load(const char* path, int device, rago_index** out) {
    if (!path || !out) return fail(RAGO_INVALID_ARG, "null argument");
    FILE* f = std::fopen(path, "rb");
    if (!f) return fail(RAGO_IO, std::string("cannot open ") + path);
    std::unique_ptr<FILE, int (*)(FILE*)> closer(f, std::fclose);
    unsigned char hdr[64];
    if (std::fread(hdr, 1, 64, f) != 64) return fail(RAGO_FORMAT, "file shorter than its header");
    if (std::memcmp(hdr, "RAGOIVPQ", 8) != 0) return fail(RAGO_FORMAT, "bad magic");
    uint32_t u[6];
    uint64_t n64;
    std::memcpy(u, hdr + 8, 24);
    std::memcpy(&n64, hdr + 32, 8);
    const uint32_t version = u[0], metric = u[1], d = u[2], m = u[3], ksub = u[4], nlist = u[5];
    if (version != 1) return fail(RAGO_FORMAT, "unknown index version");
    if (metric > 1) return fail(RAGO_UNSUPPORTED, "metric must be 0 (inner product) or 1 (Euclidean)");
    if (ksub != KSUB && ksub != 16) return fail(RAGO_UNSUPPORTED, "ksub must be 256 or 16");
    if (ksub == 16 && m % 2) return fail(RAGO_UNSUPPORTED, "with ksub = 16, m must be even");
    const uint64_t cbytes = ksub == 16 ? m / 2 : m;   // code bytes per vector
    if (!d || !m || !nlist || d > (1u << 20) || nlist > (1u << 28) || n64 > (1ull << 40)) return fail(RAGO_FORMAT, "implausible header");
    if (d % m) return fail(RAGO_UNSUPPORTED, "d must be a multiple of m");
    const uint64_t expect = 64 + 4ull * nlist * d + 4ull * m * ksub * (d / m) + 8ull * (nlist + 1) + n64 * cbytes + 8ull * n64;
    if (std::fseek(f, 0, SEEK_END) != 0) return fail(RAGO_IO, "seek failed");
    const uint64_t have = (uint64_t)std::ftell(f);
    if (have != expect) return fail(RAGO_FORMAT, "file size does not match its header (truncated or corrupt)");
    std::fseek(f, 64, SEEK_SET);
    std::vector<float> cen((size_t)nlist * d), cb((size_t)m * ksub * (d / m));
    std::vector<int64_t> off(nlist + 1);
    if (std::fread(cen.data(), 4, cen.size(), f) != cen.size() || std::fread(cb.data(), 4, cb.size(), f) != cb.size() ||
        std::fread(off.data(), 8, off.size(), f) != off.size())
        return fail(RAGO_IO, "read failed");
    DeviceGuard g(device);
    if (!g.ok) return fail(RAGO_DEVICE, "hipSetDevice failed");
    rago_index* idx = new rago_index();
    idx->device = device;
    int rc = prepare(idx, (int)d, (int)m, (int)ksub, (int)nlist, (int64_t)n64, off.data(), (int)metric);
    uint8_t* plain = nullptr;
    void* stage = nullptr;
    const size_t CH = (size_t)64 << 20;
    if (!rc && hipMalloc(&plain, (size_t)n64 * cbytes + 16) != hipSuccess) { (void)hipGetLastError(); rc = fail(RAGO_OOM, "staging buffer for codes"); }
    if (!rc && hipHostMalloc(&stage, CH) != hipSuccess) { (void)hipGetLastError(); rc = fail(RAGO_OOM, "pinned staging buffer"); }
    if (!rc) {
        hipError_t e = hipMemcpy(idx->centroids, cen.data(), cen.size() * 4, hipMemcpyHostToDevice);
        if (e != hipSuccess) rc = fail(RAGO_DEVICE, "copying centroids");
    }
    if (!rc) rc = set_codebooks(idx, cb.data(), hipMemcpyHostToDevice);
    // stream codes then ids through the pinned buffer
    for (int pass = 0; pass < 2 && !rc; ++pass) {
        size_t total = pass == 0 ? (size_t)n64 * cbytes : (size_t)n64 * 8;
        char* dst = pass == 0 ? (char*)plain : (char*)idx->ids;
        for (size_t a = 0; a < total && !rc; a += CH) {
            size_t len = total - a < CH ? total - a : CH;
            if (std::fread(stage, 1, len, f) != len) rc = fail(RAGO_IO, "read failed");
            else if (hipMemcpy(dst + a, stage, len, hipMemcpyHostToDevice) != hipSuccess) rc = fail(RAGO_DEVICE, "copying index data");
        }
    }
    if (!rc) rc = finish(idx, plain);
    if (stage) hipHostFree(stage);
    if (plain) hipFree(plain);
    if (rc) { destroy(idx); return rc; }
    *out = idx;
    return RAGO_OK;
}

int rago_index_set_upper_level(rago_index* idx, int32_t nsuper, const float* super_centroids, const int64_t* super_offsets,
                               const int32_t* super_lists, int on_device) {
    if (!idx) return fail(RAGO_INVALID_ARG, "null index");
    DeviceGuard g(idx->device);
    (void)hipDeviceSynchronize();
    hipFree(idx->sup_cen); hipFree(idx->sup_off); hipFree(idx->sup_lists); hipFree(idx->sup_of);
    idx->sup_cen = nullptr; idx->sup_off = nullptr; idx->sup_lists = nullptr; idx->sup_of = nullptr;
    idx->nsuper = 0; idx->nsp = 0; idx->max_group = 0;
    if (nsuper == 0) return RAGO_OK;
    if (nsuper < 0 || !super_centroids || !super_offsets || !super_lists) return fail(RAGO_INVALID_ARG, "bad upper-level argument");
    if (nsuper > tree_cap()) return fail(RAGO_UNSUPPORTED, "more than 8192 groups");
    const int nlist = idx->nlist;
    std::vector<int64_t> off(nsuper + 1);
    std::vector<int32_t> lists(nlist), of(nlist, -1);
    if (on_device) {
        RAGO_HIP(hipMemcpy(off.data(), super_offsets, off.size() * 8, hipMemcpyDeviceToHost));
        RAGO_HIP(hipMemcpy(lists.data(), super_lists, lists.size() * 4, hipMemcpyDeviceToHost));
    } else {
        std::memcpy(off.data(), super_offsets, off.size() * 8);
        std::memcpy(lists.data(), super_lists, lists.size() * 4);
    }
    if (off[0] != 0 || off[nsuper] != nlist) return fail(RAGO_INVALID_ARG, "super_offsets must run from 0 to nlist");
    int64_t largest = 0;
    for (int s = 0; s < nsuper; ++s) {
        if (off[s + 1] < off[s]) return fail(RAGO_INVALID_ARG, "super_offsets must be non-decreasing");
        largest = std::max(largest, off[s + 1] - off[s]);
        for (int64_t e = off[s]; e < off[s + 1]; ++e) {
            const int32_t l = lists[e];
            if (l < 0 || l >= nlist || of[l] != -1) return fail(RAGO_INVALID_ARG, "super_lists must hold every list exactly once");
            if (e > off[s] && lists[e - 1] >= l) return fail(RAGO_INVALID_ARG, "lists must ascend inside a group");
            of[l] = s;
        }
    }
    if (hipMalloc(&idx->sup_cen, sizeof(float) * (size_t)nsuper * idx->d) != hipSuccess ||
        hipMalloc(&idx->sup_off, sizeof(int64_t) * (size_t)(nsuper + 1)) != hipSuccess ||
        hipMalloc(&idx->sup_lists, sizeof(int32_t) * (size_t)nlist) != hipSuccess ||
        hipMalloc(&idx->sup_of, sizeof(int32_t) * (size_t)nlist) != hipSuccess) {
        (void)hipGetLastError();
        return fail(RAGO_OOM, "device allocation for the upper level failed");
    }
    RAGO_HIP(hipMemcpy(idx->sup_cen, super_centroids, sizeof(float) * (size_t)nsuper * idx->d,
                       on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice));
    RAGO_HIP(hipMemcpy(idx->sup_off, off.data(), off.size() * 8, hipMemcpyHostToDevice));
    RAGO_HIP(hipMemcpy(idx->sup_lists, lists.data(), lists.size() * 4, hipMemcpyHostToDevice));
    RAGO_HIP(hipMemcpy(idx->sup_of, of.data(), of.size() * 4, hipMemcpyHostToDevice));
    idx->nsuper = nsuper;
    idx->max_group = (int)largest;
    return RAGO_OK;
}

int rago_index_set_upper_probe(rago_index* idx, int32_t nsp) {
    if (!idx) return fail(RAGO_INVALID_ARG, "null index");
    if (nsp < 0) return fail(RAGO_INVALID_ARG, "nsp < 0");
    if (nsp > 0 && idx->nsuper == 0) return fail(RAGO_INVALID_ARG, "the index has no upper level");
    if (nsp > idx->nsuper) return fail(RAGO_INVALID_ARG, "nsp > nsuper");
    if ((int64_t)nsp * idx->max_group > tree_cap()) return fail(RAGO_UNSUPPORTED, "nsp * largest group > 8192");
    idx->nsp = nsp;
    return RAGO_OK;
}

int rago_index_free(rago_index* idx) {
    if (!idx) return RAGO_OK;
    DeviceGuard g(idx->device);
    (void)hipDeviceSynchronize();
    destroy(idx);
    return RAGO_OK;
}

int rago_index_info(const rago_index* idx, rago_index_desc* out) {
    if (!idx || !out) return fail(RAGO_INVALID_ARG, "null argument");
    out->d = idx->d; out->m = idx->user_m; out->ksub = idx->user_ksub; out->nlist = idx->nlist; out->n = idx->n;
    out->metric = idx->metric; out->device = idx->device; out->max_list_len = idx->max_list_len;
    out->code_bytes_resident = idx->total_blocks * BLOCK_VECS * idx->m;
    return RAGO_OK;
}

static int check_search_args(const rago_index* idx, const void* a, const void* b, int64_t nq, int nprobe, int k) {
    if (!idx) return fail(RAGO_INVALID_ARG, "null index");
    if (nq < 0) return fail(RAGO_INVALID_ARG, "nq < 0");
    if (nq > 0 && (!a || !b)) return fail(RAGO_INVALID_ARG, "null buffer");
    if (nprobe < 1 || nprobe > idx->nlist) return fail(RAGO_INVALID_ARG, "nprobe must be in [1, nlist]");
    if (k < 1) return fail(RAGO_INVALID_ARG, "k must be >= 1");
    if (k > KMAX) return fail(RAGO_UNSUPPORTED, "k > 128");
    if (nprobe > 2048) return fail(RAGO_UNSUPPORTED, "nprobe > 2048");
    if (nq * (int64_t)nprobe > (1ll << 30)) return fail(RAGO_UNSUPPORTED, "nq * nprobe > 2^30");
    return RAGO_OK;
}

int rago_debug_coarse(rago_index* idx, const float* queries, int64_t nq, float* out_S, void* stream) {
    if (!idx || nq < 0 || (nq > 0 && (!queries || !out_S))) return fail(RAGO_INVALID_ARG, "bad argument");
    if (((uintptr_t)queries & 15) != 0) return fail(RAGO_INVALID_ARG, "queries must be 16-byte aligned");
    if (nq == 0) return RAGO_OK;
    DeviceGuard g(idx->device);
    return launch_coarse(idx, queries, nq, out_S, (hipStream_t)stream);
}

int rago_debug_select(rago_index* idx, const float* queries, const float* S, int64_t nq, int32_t nprobe,
                      int32_t* out_probes, void* stream) {
    int rc = check_search_args(idx, S, out_probes, nq, nprobe, 1);
    if (rc) return rc;
    if (nq > 0 && !queries) return fail(RAGO_INVALID_ARG, "null queries");
    if (nq == 0) return RAGO_OK;
    DeviceGuard g(idx->device);
    // the selection may replace a row by exact scores: it works on a copy, the caller's S stays as it is
    if ((rc = idx->ws.S.reserve((size_t)nq * idx->nlist * 4))) return rc;
    RAGO_HIP(hipMemcpyAsync(idx->ws.S.p, S, (size_t)nq * idx->nlist * 4, hipMemcpyDeviceToDevice, (hipStream_t)stream));
    return launch_select(idx, queries, idx->ws.S.as<float>(), nq, nprobe, out_probes, (hipStream_t)stream);
}

int rago_debug_select_tree(rago_index* idx, const float* queries, int64_t nq, int32_t nprobe, int32_t* out_probes,
                           int32_t* out_groups, void* stream) {
    int rc = check_search_args(idx, queries, out_probes, nq, nprobe, 1);
    if (rc) return rc;
    if (idx->nsp < 1) return fail(RAGO_INVALID_ARG, "no groups are kept (rago_index_set_upper_probe)");
    if (nq == 0) return RAGO_OK;
    DeviceGuard g(idx->device);
    hipStream_t st = (hipStream_t)stream;
    if ((rc = launch_select_tree(idx, queries, nq, nprobe, out_probes, st))) return rc;
    if (out_groups)
        RAGO_HIP(hipMemcpyAsync(out_groups, idx->ws.cand_idx.p, (size_t)nq * idx->nsp * 4, hipMemcpyDeviceToDevice, st));
    return RAGO_OK;
}

int rago_debug_build_lut(rago_index* idx, const float* queries, const int32_t* probes, int64_t nq, int32_t nprobe,
                         float* out_L, uint8_t* out_LUT8, int32_t* out_B, float* out_delta, void* stream) {
    int rc = check_search_args(idx, queries, probes, nq, nprobe, 1);
    if (rc) return rc;
    if (nq == 0) return RAGO_OK;
    DeviceGuard g(idx->device);
    const int64_t npairs = nq * nprobe;
    hipStream_t st = (hipStream_t)stream;
    const int32_t* bias;
    const float* delta;
    if (idx->metric == 1) {
        if ((rc = launch_build_lut_l2(idx, queries, probes, nq, nprobe, out_L, out_LUT8, st))) return rc;
        bias = idx->ws.bias.as<int32_t>();
        delta = idx->ws.delta.as<float>();
    } else {
        LutTables T;
        if ((rc = launch_build_lut(idx, queries, probes, nq, nprobe, &T, out_L, out_LUT8, st))) return rc;
        bias = T.bias;
        delta = T.delta;
    }
    if (out_B) RAGO_HIP(hipMemcpyAsync(out_B, bias, (size_t)npairs * 4, hipMemcpyDeviceToDevice, st));
    if (out_delta) RAGO_HIP(hipMemcpyAsync(out_delta, delta, (size_t)nq * 4, hipMemcpyDeviceToDevice, st));
    return RAGO_OK;
}

int rago_debug_scan(rago_index* idx, const int32_t* probes, const uint8_t* LUT8, const int32_t* B, int64_t nq,
                    int32_t nprobe, int32_t k, int64_t* out_ids, int32_t* out_iscores, void* stream) {
    int rc = check_search_args(idx, probes, out_ids, nq, nprobe, k);
    if (rc) return rc;
    if (nq > 0 && (!LUT8 || !B)) return fail(RAGO_INVALID_ARG, "null tables");
    if (nq == 0) return RAGO_OK;
    DeviceGuard g(idx->device);
    Workspace& ws = idx->ws;
    const int64_t npairs = nq * nprobe;
    if ((rc = ws.tmp_lut8sw.reserve((size_t)npairs * LUT_BYTES))) return rc;
    hipStream_t st = (hipStream_t)stream;
    if ((rc = launch_swizzle_lut(idx, LUT8, npairs, ws.tmp_lut8sw.as<uint8_t>(), st))) return rc;
    return launch_scan(idx, probes, ws.tmp_lut8sw.as<uint8_t>(), B, nullptr, nullptr, nq, nprobe, k, out_ids, nullptr, out_iscores, st);
}

// The stages of a search in order.  With idx->reserving set every stage launcher sizes its buffers and returns
// before launching anything, so the same code that runs a search also sizes the workspace for it.
static int run_search(rago_index* idx, const float* queries, int64_t nq, int32_t nprobe, int32_t k, int64_t* out_ids,
                      float* out_scores, int32_t* out_iscores, hipStream_t st, hipEvent_t* ev, bool tree) {
    Workspace& ws = idx->ws;
    const int64_t npairs = nq * nprobe;
    int rc;
    if ((rc = ws.probes.reserve((size_t)npairs * 4))) return rc;
    if (ev) RAGO_HIP(hipEventRecord(ev[0], st));
    if (tree) {
        // through the upper level: both steps in one (the coarse-score slot of the stage times stays empty)
        if (ev) RAGO_HIP(hipEventRecord(ev[1], st));
        if ((rc = launch_select_tree(idx, queries, nq, nprobe, ws.probes.as<int32_t>(), st))) return rc;
    } else {
        if ((rc = ws.S.reserve((size_t)nq * idx->nlist * 4))) return rc;
        if ((rc = launch_coarse(idx, queries, nq, ws.S.as<float>(), st, true))) return rc;
        if (ev) RAGO_HIP(hipEventRecord(ev[1], st));
        if ((rc = launch_select(idx, queries, ws.S.as<float>(), nq, nprobe, ws.probes.as<int32_t>(), st, true))) return rc;
    }
    if (ev) RAGO_HIP(hipEventRecord(ev[2], st));
    if (idx->metric == 1) {
        // Euclidean metric: one full table per pair, handed to the scan like caller-supplied tables
        if ((rc = launch_build_lut_l2(idx, queries, ws.probes.as<int32_t>(), nq, nprobe, nullptr, nullptr, st))) return rc;
        if (ev) RAGO_HIP(hipEventRecord(ev[3], st));
        rc = launch_scan(idx, ws.probes.as<int32_t>(), ws.tmp_lut8sw.as<uint8_t>(), ws.bias.as<int32_t>(), nullptr,
                         ws.delta.as<float>(), nq, nprobe, k, out_ids, out_scores, out_iscores, st, ev);
    } else {
        LutTables T{};
        // The scan's bookkeeping rides in the table kernels (it needs only the probes): the plan of the wave-per-item
        // kernel always, the pairs-by-list bookkeeping of the other two for up to 16 queries (the latency-bound rounds
        // of Section 5.3: with more, the table kernel fills the chip and the extra workgroup, which needs most of a
        // compute unit's LDS, would wait for one of its workgroups to finish).
        SmallSetupArgs su{};
        WavePlanArgs wp{};
        if ((rc = plan_scan_setup(idx, ws.probes.as<int32_t>(), nq, nprobe, k, true, nq <= 16 ? &su : nullptr, &wp))) return rc;
        if ((rc = launch_build_lut(idx, queries, ws.probes.as<int32_t>(), nq, nprobe, &T, nullptr, nullptr, st, &su, &wp))) return rc;
        if (ev) RAGO_HIP(hipEventRecord(ev[3], st));
        rc = launch_scan(idx, ws.probes.as<int32_t>(), nullptr, T.bias, &T, T.delta, nq, nprobe, k, out_ids, out_scores,
                         out_iscores, st, ev, su.enable != 0 || wp.enable != 0);
    }
    return rc;
}

int rago_ivfpq_search(rago_index* idx, const float* queries, int64_t nq, int32_t nprobe, int32_t k, int64_t* out_ids,
                      float* out_scores, int32_t* out_iscores, void* stream) {
    int rc = check_search_args(idx, queries, out_ids, nq, nprobe, k);
    if (rc) return rc;
    if (nq > 0 && !out_scores) return fail(RAGO_INVALID_ARG, "null out_scores");
    if (((uintptr_t)queries & 15) != 0) return fail(RAGO_INVALID_ARG, "queries must be 16-byte aligned");
    if (nq == 0) return RAGO_OK;
    if (idx->ws_frozen && (nq > idx->res_nq || nprobe > idx->res_nprobe || k > idx->res_k))
        return fail(RAGO_UNSUPPORTED, "the call exceeds the maxima given to rago_index_reserve (nq " + std::to_string(idx->res_nq) +
                                          ", nprobe " + std::to_string(idx->res_nprobe) + ", k " + std::to_string(idx->res_k) + ")");
    DeviceGuard g(idx->device);
    NoGrowScope frozen(idx->ws_frozen);
    hipStream_t st = (hipStream_t)stream;
    hipEvent_t* ev = nullptr;
    if (idx->prof.on && idx->prof.ncalls < PROF_CALLS) ev = idx->prof.ev[idx->prof.ncalls];
    rc = run_search(idx, queries, nq, nprobe, k, out_ids, out_scores, out_iscores, st, ev, idx->nsp > 0);
    if (!rc && ev) ++idx->prof.ncalls;
    return rc;
}

int rago_index_reserve(rago_index* idx, int64_t max_nq, int32_t max_nprobe, int32_t max_k) {
    if (!idx) return fail(RAGO_INVALID_ARG, "null index");
    if (max_nq < 1 || max_nprobe < 1 || max_k < 1) return fail(RAGO_INVALID_ARG, "maxima must be >= 1");
    if (max_nprobe > idx->nlist) max_nprobe = idx->nlist;
    int rc = check_search_args(idx, idx, idx, max_nq, max_nprobe, max_k);
    if (rc) return rc;
    DeviceGuard g(idx->device);
    RAGO_HIP(hipDeviceSynchronize());           // buffers that grow are freed: nothing may still be using them
    idx->ws_frozen = false;
    idx->reserving = true;
    rc = run_search(idx, nullptr, max_nq, max_nprobe, max_k, nullptr, nullptr, nullptr, nullptr, nullptr, false);
    if (!rc && idx->nsuper > 0) {
        // the stage through the upper level, for any number of kept groups
        const int nsp = idx->nsp;
        idx->nsp = idx->nsuper;
        rc = launch_select_tree(idx, nullptr, max_nq, max_nprobe, idx->ws.probes.as<int32_t>(), nullptr);
        idx->nsp = nsp;
    }
    idx->reserving = false;
    if (rc) return rc;
    idx->ws_frozen = true;
    idx->res_nq = max_nq; idx->res_nprobe = max_nprobe; idx->res_k = max_k;
    return RAGO_OK;
}

int rago_debug_force_scan_kernel(int which) {
    if (which < 0 || which > 3) return fail(RAGO_INVALID_ARG, "0 = pick by sizes, 1 = wide, 2 = narrow, 3 = wave per item");
    g_forced_scan.store(which);
    return RAGO_OK;
}

int64_t rago_debug_allocations(void) { return (int64_t)device_allocations(); }

int rago_debug_profile(rago_index* idx, int enable) {
    if (!idx) return fail(RAGO_INVALID_ARG, "null index");
    DeviceGuard g(idx->device);
    if (enable && !idx->prof.created) {
        for (auto& c : idx->prof.ev)
            for (auto& e : c) RAGO_HIP(hipEventCreate(&e));
        idx->prof.created = true;
    }
    idx->prof.on = enable != 0;
    if (enable) idx->prof.ncalls = 0;
    return RAGO_OK;
}

int rago_debug_stage_ms(rago_index* idx, float* out_ms, int32_t* out_calls) {
    if (!idx || !out_ms || !out_calls) return fail(RAGO_INVALID_ARG, "null argument");
    DeviceGuard g(idx->device);
    for (int i = 0; i < 8; ++i) out_ms[i] = 0.f;
    *out_calls = idx->prof.ncalls;
    for (int c = 0; c < idx->prof.ncalls; ++c) {
        RAGO_HIP(hipEventSynchronize(idx->prof.ev[c][PROF_EVENTS - 1]));
        for (int i = 0; i + 1 < PROF_EVENTS; ++i) {
            float ms = 0.f;
            RAGO_HIP(hipEventElapsedTime(&ms, idx->prof.ev[c][i], idx->prof.ev[c][i + 1]));
            out_ms[i] += ms / idx->prof.ncalls;
        }
        float ms = 0.f;
        RAGO_HIP(hipEventElapsedTime(&ms, idx->prof.ev[c][0], idx->prof.ev[c][PROF_EVENTS - 1]));
        out_ms[6] += ms / idx->prof.ncalls;
    }
    return RAGO_OK;
}

static int flat_search(const void* corpus, const void* queries, int32_t R, int64_t n, int32_t nqr, int32_t d, int32_t k,
                       int64_t* out_ids, float* out_scores, int device, bool half, void* stream, bool static_scratch = false) {
    if (R < 0 || n < 0) return fail(RAGO_INVALID_ARG, "negative size");
    if (nqr < 1 || nqr > 16) return fail(RAGO_INVALID_ARG, "nqr must be in [1, 16]");
    if (k < 1) return fail(RAGO_INVALID_ARG, "k must be >= 1");
    if (k > KMAX) return fail(RAGO_UNSUPPORTED, "k > 128");
    if (d < 64 || d % 64 || d > 1024) return fail(RAGO_UNSUPPORTED, "d must be a multiple of 64 in [64, 1024]");
    if (R > 0 && (!queries || !out_ids || !out_scores || (n > 0 && !corpus))) return fail(RAGO_INVALID_ARG, "null buffer");
    if (((uintptr_t)corpus & 15) || ((uintptr_t)queries & 15)) return fail(RAGO_INVALID_ARG, "buffers must be 16-byte aligned");
    if (n > 0x7fffffffLL) return fail(RAGO_UNSUPPORTED, "n > 2^31-1 per request");
    if (R == 0) return RAGO_OK;
    DeviceGuard g(device);
    if (!g.ok) return fail(RAGO_DEVICE, "hipSetDevice failed");
    if (static_scratch) return launch_flat_static(corpus, queries, R, n, nqr, d, k, out_ids, out_scores, device, half, (hipStream_t)stream);
    return launch_flat(corpus, queries, R, n, nqr, d, k, out_ids, out_scores, device, half, (hipStream_t)stream);
}

int rago_flat_search_static(const void* corpus, const void* queries, int32_t R, int64_t n, int32_t nqr, int32_t d, int32_t k,
                            int32_t format, int64_t* out_ids, float* out_scores, int device, void* stream) {
    if (format != 0 && format != 1) return fail(RAGO_INVALID_ARG, "format must be 0 (bf16) or 1 (binary16)");
    return flat_search(corpus, queries, R, n, nqr, d, k, out_ids, out_scores, device, format == 1, stream, true);
}

int rago_flat_search(const void* corpus, const void* queries, int32_t R, int64_t n, int32_t nqr, int32_t d, int32_t k,
                     int64_t* out_ids, float* out_scores, int device, void* stream) {
    return flat_search(corpus, queries, R, n, nqr, d, k, out_ids, out_scores, device, false, stream);
}

int rago_flat_search_f16(const void* corpus, const void* queries, int32_t R, int64_t n, int32_t nqr, int32_t d, int32_t k,
                         int64_t* out_ids, float* out_scores, int device, void* stream) {
    return flat_search(corpus, queries, R, n, nqr, d, k, out_ids, out_scores, device, true, stream);
}

int rago_debug_flat_profile(int device, int enable) {
    DeviceGuard g(device);
    if (!g.ok) return fail(RAGO_DEVICE, "hipSetDevice failed");
    return flat_profile(device, enable);
}

int rago_debug_flat_stage_ms(int device, float* out_ms, int32_t* out_calls) {
    if (!out_ms || !out_calls) return fail(RAGO_INVALID_ARG, "null argument");
    DeviceGuard g(device);
    if (!g.ok) return fail(RAGO_DEVICE, "hipSetDevice failed");
    return flat_stage_ms(device, out_ms, out_calls);
}

int rago_debug_copy(const void* src, void* dst, int64_t bytes, void* stream) {
    if (!src || !dst || bytes < 0 || (bytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15))
        return fail(RAGO_INVALID_ARG, "copy needs 16-byte aligned buffers and a size that is a multiple of 16");
    return launch_calib_copy(src, dst, bytes, (hipStream_t)stream);
}

int rago_debug_read_stream(const void* src, int64_t bytes, uint32_t* sink, void* stream) {
    if (!src || !sink || bytes < 0 || (bytes & 15) || ((uintptr_t)src & 15))
        return fail(RAGO_INVALID_ARG, "read stream needs a 16-byte aligned buffer, a size that is a multiple of 16 and a sink");
    return launch_calib_read(src, bytes, sink, (hipStream_t)stream);
}

int rago_debug_counters(rago_index* idx, int64_t* out, void* stream) {
    if (!idx || !out) return fail(RAGO_INVALID_ARG, "null argument");
    DeviceGuard g(idx->device);
    for (int i = 0; i < 8; ++i) out[i] = 0;
    if (!idx->ws.counters.p) return RAGO_OK;
    RAGO_HIP(hipMemcpyAsync(out, idx->ws.counters.p, 8 * sizeof(int64_t), hipMemcpyDeviceToHost, (hipStream_t)stream));
    RAGO_HIP(hipStreamSynchronize((hipStream_t)stream));
    out[6] = idx->last_scan_kernel;
    return RAGO_OK;
}

}  // extern "C"

// Feeds the library's index-file loader good and bad files, in a build whose host code is compiled with
// -fsanitize=address,undefined, so that a header the loader trusts too far shows up as a sanitizer report.
// Runs without a GPU: every bad file must be refused by the host-side checks, before any device call; the one
// well-formed file gets as far as selecting the device and must then fail cleanly (no device here) or load.
// Test infrastructure: built and run by tests/test_sanitizers.py only.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "rago.h"

static std::string g_dir;

static std::string write_file(const char* name, const std::vector<unsigned char>& bytes) {
    const std::string path = g_dir + "/" + name;
    FILE* f = std::fopen(path.c_str(), "wb");
    if (!f) { std::perror("fopen"); std::exit(2); }
    if (!bytes.empty()) std::fwrite(bytes.data(), 1, bytes.size(), f);
    std::fclose(f);
    return path;
}

struct Header { uint32_t version = 1, metric = 0, d = 8, m = 2, ksub = 256, nlist = 3; uint64_t n = 5; };

// A file laid out as the header says (payload zeros, offsets 0, 2, 2, 5), cut or padded by `delta` bytes.
static std::vector<unsigned char> make_file(const Header& h, long delta = 0, const char* magic = "RAGOIVPQ") {
    std::vector<unsigned char> b(64, 0);
    std::memcpy(b.data(), magic, 8);
    const uint32_t u[6] = {h.version, h.metric, h.d, h.m, h.ksub, h.nlist};
    std::memcpy(b.data() + 8, u, 24);
    std::memcpy(b.data() + 32, &h.n, 8);
    const uint64_t cbytes = h.ksub == 16 ? h.m / 2 : h.m;
    const uint64_t dsub = h.m ? h.d / h.m : 0;
    const uint64_t payload = 4ull * h.nlist * h.d + 4ull * h.m * h.ksub * dsub + 8ull * (h.nlist + 1) + h.n * cbytes + 8ull * h.n;
    if (payload < (1ull << 24)) {
        b.resize(64 + payload, 0);
        if (h.nlist == 3 && h.n == 5) {
            const int64_t off[4] = {0, 2, 2, 5};
            std::memcpy(b.data() + 64 + 4ull * h.nlist * h.d + 4ull * h.m * h.ksub * dsub, off, sizeof off);
        }
    }
    if (delta < 0) b.resize(b.size() > (size_t)-delta ? b.size() + delta : 0);
    if (delta > 0) b.resize(b.size() + delta, 0);
    return b;
}

static int expect_refused(const char* what, const std::string& path, int want_code = 0) {
    rago_index* idx = nullptr;
    const int rc = rago_index_load(path.c_str(), 0, &idx);
    if (rc == RAGO_OK) { std::fprintf(stderr, "%s: loaded, expected a refusal\n", what); rago_index_free(idx); return 1; }
    if (want_code && rc != want_code) { std::fprintf(stderr, "%s: code %d (%s), expected %d\n", what, rc, rago_last_error(), want_code); return 1; }
    if (!rago_last_error() || !*rago_last_error()) { std::fprintf(stderr, "%s: refusal without a message\n", what); return 1; }
    return 0;
}

int main(int argc, char** argv) {
    if (argc != 2) { std::fprintf(stderr, "usage: loader_sanitize_check <scratch directory>\n"); return 2; }
    g_dir = argv[1];
    int bad = 0;
    Header ok;
    bad += expect_refused("missing file", g_dir + "/does_not_exist", RAGO_IO);
    bad += expect_refused("empty file", write_file("empty", {}), RAGO_FORMAT);
    bad += expect_refused("short header", write_file("short", std::vector<unsigned char>(40, 'R')), RAGO_FORMAT);
    bad += expect_refused("bad magic", write_file("magic", make_file(ok, 0, "RAGOIVPX")), RAGO_FORMAT);
    bad += expect_refused("one byte short", write_file("cut1", make_file(ok, -1)), RAGO_FORMAT);
    bad += expect_refused("cut inside the offsets", write_file("cut2", make_file(ok, -60)), RAGO_FORMAT);
    bad += expect_refused("trailing bytes", write_file("long", make_file(ok, 3)), RAGO_FORMAT);
    { Header h = ok; h.version = 2; bad += expect_refused("unknown version", write_file("ver", make_file(h)), RAGO_FORMAT); }
    { Header h = ok; h.metric = 7; bad += expect_refused("unknown metric", write_file("metric", make_file(h)), RAGO_UNSUPPORTED); }
    { Header h = ok; h.ksub = 64; bad += expect_refused("ksub 64", write_file("ksub", make_file(h)), RAGO_UNSUPPORTED); }
    { Header h = ok; h.ksub = 16; h.m = 1; bad += expect_refused("odd m with 4-bit codes", write_file("odd", make_file(h)), RAGO_UNSUPPORTED); }
    { Header h = ok; h.m = 0; bad += expect_refused("m = 0", write_file("m0", make_file(h)), RAGO_FORMAT); }
    { Header h = ok; h.d = 0; bad += expect_refused("d = 0", write_file("d0", make_file(h)), RAGO_FORMAT); }
    { Header h = ok; h.nlist = 0; bad += expect_refused("nlist = 0", write_file("l0", make_file(h)), RAGO_FORMAT); }
    { Header h = ok; h.m = 3; bad += expect_refused("d not a multiple of m", write_file("dm", make_file(h)), RAGO_UNSUPPORTED); }
    { Header h = ok; h.d = 0xFFFFFFF8u; bad += expect_refused("huge d", write_file("hd", make_file(h)), RAGO_FORMAT); }
    { Header h = ok; h.nlist = 0xFFFFFFFFu; bad += expect_refused("huge nlist", write_file("hl", make_file(h)), RAGO_FORMAT); }
    { Header h = ok; h.n = ~0ull; bad += expect_refused("huge n", write_file("hn", make_file(h)), RAGO_FORMAT); }
    // sizes whose byte count wraps around 2^64 if summed carelessly: the file is 64 bytes + a small payload
    { Header h = ok; h.d = 1u << 20; h.m = 1u << 20; h.nlist = 1u << 28; h.n = 1ull << 40;
      bad += expect_refused("largest plausible header on a tiny file", write_file("big", make_file(h)), RAGO_FORMAT); }
    // a well-formed file: read in full by the host code; then either loads (a GPU is present) or fails on the device
    {
        rago_index* idx = nullptr;
        const int rc = rago_index_load(write_file("good", make_file(ok)).c_str(), 0, &idx);
        if (rc == RAGO_OK) rago_index_free(idx);
        else if (rc == RAGO_FORMAT || rc == RAGO_IO) { std::fprintf(stderr, "well-formed file refused: %s\n", rago_last_error()); ++bad; }
    }
    if (bad) { std::fprintf(stderr, "%d loader check(s) failed\n", bad); return 1; }
    std::puts("loader sanitize check ok");
    return 0;
}

// Exact inner-product search over small per-request corpora (brute-force kNN, Section 5.2).
#include "rago_internal.h"

namespace rago {

int launch_flat(const void*, const void*, int, int64_t, int, int, int, int64_t*, float*, int, hipStream_t) {
    return fail(RAGO_UNSUPPORTED, "flat search not built yet");
}

}  // namespace rago

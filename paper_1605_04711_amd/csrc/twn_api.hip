// Host-only helpers of the C ABI: status strings, packed-format sizes, env overrides.
#include <cstdlib>

#include "twn_common.h"

namespace twn {

int env_int(const char* name, int fallback) {
    const char* v = std::getenv(name);
    if (!v || !*v) return fallback;
    return std::atoi(v);
}

}  // namespace twn

extern "C" const char* twn_status_str(int32_t status) {
    switch (status) {
        case TWN_OK: return "ok";
        case TWN_ERR_NULL: return "null pointer";
        case TWN_ERR_SHAPE: return "bad shape or size";
        case TWN_ERR_ALIGN: return "misaligned pointer or leading dimension";
        case TWN_ERR_UNSUPPORTED: return "unsupported dtype, variant or option";
        case TWN_ERR_WORKSPACE: return "workspace missing or too small";
        case TWN_ERR_HIP: return "HIP launch failed";
        default: return "unknown status";
    }
}

extern "C" int32_t twn_abi_version(void) { return 1; }

extern "C" int64_t twn_packed_words_per_row(int64_t K) {
    if (K <= 0) return 0;
    return 8 * ((K + 127) / 128);
}

extern "C" int64_t twn_packed1_words_per_row(int64_t K) {
    if (K <= 0) return 0;
    return 4 * ((K + 127) / 128);
}

extern "C" size_t twn_packed_bytes(int32_t rows, int64_t K) {
    if (rows <= 0 || K <= 0) return 0;
    return static_cast<size_t>(rows) * static_cast<size_t>(twn_packed_words_per_row(K)) * 4u;
}

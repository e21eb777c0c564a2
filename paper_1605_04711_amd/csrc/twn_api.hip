// Host-only helpers of the C ABI: status strings, packed-format sizes, env overrides.
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "twn_common.h"

namespace twn {

// The TWN_* tuning knobs are read from the environment once each and remembered: launches do not call getenv
// (which is neither free nor safe against a concurrent setenv).  twn_reload_env forgets what was read.
namespace {
struct EnvEntry {
    const char* name;     // the caller's string literal
    bool set;
    int value;
};
constexpr int kEnvMax = 64;
std::mutex g_env_mutex;
EnvEntry g_env[kEnvMax];
int g_env_count = 0;
}  // namespace

int env_int(const char* name, int fallback) {
    std::lock_guard<std::mutex> lock(g_env_mutex);
    for (int i = 0; i < g_env_count; ++i)
        if (g_env[i].name == name || std::strcmp(g_env[i].name, name) == 0) return g_env[i].set ? g_env[i].value : fallback;
    const char* v = std::getenv(name);
    const bool set = v && *v;
    const int value = set ? std::atoi(v) : 0;
    if (g_env_count < kEnvMax) g_env[g_env_count++] = EnvEntry{name, set, value};
    return set ? value : fallback;
}

}  // namespace twn

extern "C" void twn_reload_env(void) {
    std::lock_guard<std::mutex> lock(twn::g_env_mutex);
    twn::g_env_count = 0;
}

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

extern "C" int32_t twn_abi_version(void) { return 2; }

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

// Error string, version and the host Philox word of the C ABI.
#include "common.h"

namespace bs {
static thread_local char g_err[512] = "";
void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}
const char* get_error() { return g_err; }
}  // namespace bs

extern "C" __attribute__((visibility("default"))) const char* bs_last_error_string(void) { return bs::get_error(); }
extern "C" __attribute__((visibility("default"))) int bs_version(void) { return 1; }
extern "C" __attribute__((visibility("default"))) uint32_t bs_philox_word(uint64_t seed, uint32_t b, uint32_t t, uint32_t slot, uint32_t purpose) {
    return bs::philox_word(seed, b, t, slot, purpose);
}

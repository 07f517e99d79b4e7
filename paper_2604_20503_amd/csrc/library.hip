// Library-wide entry points: last-error text and version.
#include <atomic>

#include "common.hpp"

namespace fsr {
char* error_buffer() {
    static thread_local char buf[256] = {0};
    return buf;
}
unsigned long long next_call_id() {
    static std::atomic<unsigned long long> counter{0};
    return (counter.fetch_add(1, std::memory_order_relaxed) + 1) & 0xffffffffffffull;
}
}  // namespace fsr

extern "C" const char* fsr_last_error(void) { return fsr::error_buffer(); }
extern "C" const char* fsr_version(void) { return "faser_verify 0.1 (gfx950)"; }

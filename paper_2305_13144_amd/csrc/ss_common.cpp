// Thread-local error text for the C ABI.
#include "ss_internal.h"

#include <cstdarg>
#include <cstdio>

#include <atomic>

namespace {
thread_local char g_err[512] = "";
std::atomic<int> g_verbose{0};
}

namespace ss {

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

void clear_error() { g_err[0] = '\0'; }

int verbose() { return g_verbose.load(std::memory_order_relaxed); }

}  // namespace ss

extern "C" const char* ss_last_error(void) { return g_err; }

extern "C" void ss_set_verbose(int32_t level) { g_verbose.store(level); }

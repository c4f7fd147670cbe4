// Error reporting behind grf_last_error(): one message buffer per host thread.
#include "common.hpp"

namespace grf {

char* error_buffer()
{
    static thread_local char buffer[512] = "";
    return buffer;
}

grf_status fail(grf_status code, const char* fmt, ...)
{
    va_list args;
    va_start(args, fmt);
    vsnprintf(error_buffer(), 512, fmt, args);
    va_end(args);
    return code;
}

}  // namespace grf

extern "C" const char* grf_last_error(void) { return grf::error_buffer(); }

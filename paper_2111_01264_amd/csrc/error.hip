// Thread-local error message behind dqn_last_error().
#include "common.h"

namespace dqn {

char* error_buffer()
{
    static thread_local char buf[512] = {0};
    return buf;
}

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(error_buffer(), 512, fmt, ap);
    va_end(ap);
    return code;
}

}  // namespace dqn

extern "C" const char* dqn_last_error(void) { return dqn::error_buffer(); }

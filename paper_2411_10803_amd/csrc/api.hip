// Error reporting and version of the C ABI.
#include "md_host.hpp"

#include <string.h>

namespace md {

char* error_buffer() {
    static thread_local char buf[512] = {0};
    return buf;
}

void clear_error() { error_buffer()[0] = '\0'; }

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(error_buffer(), 512, fmt, ap);
    va_end(ap);
    return code;
}

}  // namespace md

extern "C" const char* mustdrop_last_error(void) { return md::error_buffer(); }
extern "C" int mustdrop_version(void) { return 1; }

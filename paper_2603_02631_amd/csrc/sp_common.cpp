// Error bookkeeping and the host-only entry points of the library.
#include "sp_common.hpp"

#include <cstring>

namespace sp {

char *error_buffer()
{
    static thread_local char buf[512] = {0};
    return buf;
}

sp_status fail(sp_status code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(error_buffer(), 512, fmt, ap);
    va_end(ap);
    return code;
}

void clear_error() { error_buffer()[0] = '\0'; }

}  // namespace sp

extern "C" const char *sp_last_error(void) { return sp::error_buffer(); }

extern "C" const char *sp_version(void) { return "sp-importance 0.1 (gfx950)"; }

// Section 3.1 of the paper: the top-K chunks are a fraction rho of the draft
// sequence; K = clamp(ceil(C * num / den), 1, C).
extern "C" int64_t sp_keep_count(int64_t n_chunks, int64_t keep_num, int64_t keep_den)
{
    if (n_chunks < 1 || keep_den < 1 || keep_num < 0) return -1;
    // ceil(n_chunks * keep_num / keep_den) without overflow for large counts
    const __int128 prod = (__int128)n_chunks * (__int128)keep_num;
    __int128 k = (prod + keep_den - 1) / keep_den;
    if (k < 1) k = 1;
    if (k > n_chunks) k = n_chunks;
    return (int64_t)k;
}

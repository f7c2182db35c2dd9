// Error reporting shared by all entry points.
#include <stdarg.h>
#include <string.h>

#include "moe_common.h"

namespace moe {

static thread_local char g_error[512] = "";

char *error_buffer() { return g_error; }

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return code;
}

int check_launch(const char *what)
{
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return fail(MOE_ERR_HIP, "%s: %s", what, hipGetErrorString(err));
    return MOE_OK;
}

}  // namespace moe

extern "C" const char *moe_last_error(void) { return moe::error_buffer(); }
extern "C" int moe_abi_version(void) { return 4; }

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

// Names of the GEMM kernels the last FFN call on this thread launched, in launch order.
static thread_local char g_kernels[160] = "";

void reset_kernel_notes() { g_kernels[0] = 0; }

void note_kernel(const char *name)
{
    const size_t used = strlen(g_kernels);
    snprintf(g_kernels + used, sizeof(g_kernels) - used, "%s%s", used ? " " : "", name);
}

int check_launch(const char *what)
{
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return fail(MOE_ERR_HIP, "%s: %s", what, hipGetErrorString(err));
    return MOE_OK;
}

}  // namespace moe

extern "C" const char *moe_last_error(void) { return moe::error_buffer(); }
extern "C" const char *moe_last_ffn_kernels(void) { return moe::g_kernels; }
// What the current device reports about itself (for measurement reports that re-derive the chip's peaks).
extern "C" int moe_device_info(int *compute_units, int *engine_clock_khz, int *memory_clock_khz, int *memory_bus_bits)
{
    int dev = 0;
    hipDeviceProp_t prop;
    hipError_t err = hipGetDevice(&dev);
    if (err == hipSuccess) err = hipGetDeviceProperties(&prop, dev);
    if (err != hipSuccess) return moe::fail(MOE_ERR_HIP, "moe_device_info: %s", hipGetErrorString(err));
    if (compute_units) *compute_units = prop.multiProcessorCount;
    if (engine_clock_khz) *engine_clock_khz = prop.clockRate;
    if (memory_clock_khz) *memory_clock_khz = prop.memoryClockRate;
    if (memory_bus_bits) *memory_bus_bits = prop.memoryBusWidth;
    return MOE_OK;
}

extern "C" int moe_abi_version(void) { return 4; }

// The fused step kernel's instances for one register-slot level and one gain variant
// (ADASCALE_LEVEL = 0..3, ADASCALE_LAG = 0 or 1, given on the compiler's command line): the build
// compiles this file once per combination, in parallel.
#include "adascale_device.h"

#if !defined(ADASCALE_LEVEL) || !defined(ADASCALE_LAG)
#error "compile with -DADASCALE_LEVEL=<0..3> -DADASCALE_LAG=<0|1>"
#endif

#define ADASCALE_CAT4(a, b, c, d) a##b##c##d
#define ADASCALE_CAT(a, b, c, d) ADASCALE_CAT4(a, b, c, d)

extern "C" __attribute__((visibility("hidden"))) const void *ADASCALE_CAT(adascale_fused_kernel_level, ADASCALE_LEVEL, _lag,
                                                                           ADASCALE_LAG)(int dtype, int S)
{
    static_assert(ADASCALE_LEVEL >= 0 && ADASCALE_LEVEL < kFRegLevels, "no such level");
    return fused_kernel_at<ADASCALE_LEVEL, ADASCALE_LAG != 0>(dtype, S);
}

/* Test helper: binary64 -> binary32 conversion under a chosen IEEE rounding mode, using the
 * host's own conversion instruction.  A library-routine pin for the replay definition. */
#include <fenv.h>
#include <stdint.h>
#pragma STDC FENV_ACCESS ON
void cast_with_mode(const double *x, uint64_t n, int mode, float *y)
{
    int old = fegetround();
    fesetround(mode == 0 ? FE_TONEAREST : mode == 1 ? FE_DOWNWARD : FE_UPWARD);
    for (uint64_t i = 0; i < n; ++i) {
        volatile double v = x[i];
        volatile float f = (float)v;
        y[i] = f;
    }
    fesetround(old);
}

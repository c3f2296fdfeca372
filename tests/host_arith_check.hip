// Test helper: runs the library's per-element integer arithmetic (csrc/vt_device.h) on the HOST
// CPU, so its rounding / distance / direction logic can be compared with the oracle without a GPU.
#include "../paper_2403_09603_amd/csrc/vt_device.h"
extern "C" void h_decide(const uint64_t *bits, uint64_t n, uint32_t *y, uint32_t *D, uint32_t *dir)
{
    for (uint64_t i = 0; i < n; ++i) {
        vt::Decision d = vt::decide(bits[i]);
        y[i] = d.ybits; D[i] = d.D; dir[i] = d.dir;
    }
}
extern "C" void h_directed(const uint64_t *bits, uint64_t n, uint32_t dir, uint32_t *y)
{
    for (uint64_t i = 0; i < n; ++i) y[i] = vt::directed(bits[i], dir);
}

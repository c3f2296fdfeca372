// vt_gemm_shape_128x128.hip -- the 128x128 workgroup tile of the FP64 GEMM (see vt_gemm_tile.h).
#include "vt_gemm_tile.h"

namespace vt {

hipError_t launch_gemm_128x128(const GemmParams &p, int am, bool kcb, hipStream_t s)
{
    return launch_shape<2, 4>(p, am, kcb, s);
}

hipError_t launch_gemm_grouped_128x128(const GemmGroup &gp, int am, bool kcb, hipStream_t s)
{
    return launch_shape_grouped<2, 4>(gp, am, kcb, s);
}

}  // namespace vt

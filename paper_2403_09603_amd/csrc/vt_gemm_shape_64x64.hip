// vt_gemm_shape_64x64.hip -- the 64x64 workgroup tile of the FP64 GEMM (see vt_gemm_tile.h).
#include "vt_gemm_tile.h"

namespace vt {

hipError_t launch_gemm_64x64(const GemmParams &p, int am, bool kcb, hipStream_t s)
{
    return launch_shape<4, 1>(p, am, kcb, s);
}

hipError_t launch_gemm_grouped_64x64(const GemmGroup &gp, int am, bool kcb, hipStream_t s)
{
    return launch_shape_grouped<4, 1>(gp, am, kcb, s);
}

}  // namespace vt

// vt_gemm_shape_64x128.hip -- the 64x128 workgroup tile of the FP64 GEMM (see vt_gemm_tile.h).
#include "vt_gemm_tile.h"

namespace vt {

hipError_t launch_gemm_64x128(const GemmParams &p, int am, bool kcb, hipStream_t s)
{
    return launch_shape<2, 2>(p, am, kcb, s);
}

}  // namespace vt

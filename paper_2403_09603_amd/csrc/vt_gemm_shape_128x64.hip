// vt_gemm_shape_128x64.hip -- the 128x64 workgroup tile of the FP64 GEMM (see vt_gemm_tile.h).
#include "vt_gemm_tile.h"

namespace vt {

hipError_t launch_gemm_128x64(const GemmParams &p, int am, bool kcb, hipStream_t s)
{
    return launch_shape<4, 2>(p, am, kcb, s);
}

}  // namespace vt

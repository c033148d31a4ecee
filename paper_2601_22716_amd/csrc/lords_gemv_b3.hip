// The one-/two-token decode kernels for 3-bit codes (the kernel template lives in lords_gemv_kernel.h;
// one translation unit per code width keeps the build parallel).
#include "lords_gemv_kernel.h"

namespace lords {

hipError_t launch_gemv_3bit(const GvArgs &a, const GvPlan &d, bool bvec, dim3 grid, hipStream_t st)
{
    return launch_gv_bits<3>(a, d, bvec, grid, st);
}

}  // namespace lords

// The one-/two-token decode kernels for 2-bit codes with the table of code quadruples (the kernel template
// lives in lords_gemv_kernel.h; a translation unit of its own keeps the build parallel).
#include "lords_gemv_kernel.h"

namespace lords {

hipError_t launch_gemv_2bit_quads(const GvArgs &a, const GvPlan &d, bool bvec, dim3 grid, hipStream_t st)
{
    return launch_gv_bits<2, true>(a, d, bvec, grid, st);
}

}  // namespace lords

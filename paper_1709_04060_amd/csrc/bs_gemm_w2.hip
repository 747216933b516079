// Instantiates the bit-serial GEMM kernels for 2 weight plane(s).
#include "bs_gemm_kernel.h"

namespace bs {
template bs_status launch_wb<2>(const GemmParams &, int, bool, bool, bool, bool, hipStream_t);
}

// Instantiates the bit-serial GEMM kernels for 3 weight plane(s).
#include "bs_gemm_kernel.h"

namespace bs {
template bs_status launch_wb<3>(const GemmParams &, int, bool, bool, bool, bool, hipStream_t);
}

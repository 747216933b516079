// Instantiates the bit-serial GEMM kernels for 4 weight plane(s).
#include "bs_gemm_kernel.h"

namespace bs {
template bs_status launch_wb<4>(const GemmParams &, int, bool, bool, bool, bool, hipStream_t);
}

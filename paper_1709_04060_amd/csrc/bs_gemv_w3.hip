// Instantiates the few-column kernels for 3 weight plane(s).
#include "bs_gemv_kernel.h"

namespace bs {
template bs_status launch_gemv_wb<3>(const GemmParams &, int, bool, bool, hipStream_t);
}

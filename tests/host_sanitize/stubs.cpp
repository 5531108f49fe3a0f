// Link-time stand-ins for the kernel launchers (which live in HIP sources) in the host sanitizer
// build.  Nothing here runs: on a machine without a GPU every entry point returns
// MTNN_ERR_NO_DEVICE before it would launch, and the driver checks exactly that.
#include "mtnn_internal.h"

#include <cstdlib>

namespace mtnn {
static int never() { std::abort(); }
int launch_gemm(hipStream_t, const Geometry&, const Scratch&, int, int, int, int, int, int, const float*, long, const float*, long,
                float*, long, const Epilogue*, bool*) { return never(); }
long long gemm_streamk_launches() { return 0; }
long long gemm_fused_launches() { return 0; }
int launch_bias_act(hipStream_t, int, int, float*, long, const float*, int) { return never(); }
int launch_sgd_2d(hipStream_t, int, int, float*, long, const float*, long, float) { return never(); }
int launch_fill_zero(hipStream_t, int, int, float*, long) { return never(); }
int launch_transpose_inplace(hipStream_t, int, float*, long) { return never(); }
bool transpose_inplace_rect_supported(int rows, int cols) { return rows >= 1 && cols >= 1 && rows <= 32768 && cols <= 32768; }
int launch_transpose_inplace_rect(hipStream_t, int, int, float*) { return never(); }
int launch_copy(hipStream_t, size_t, const void*, void*) { return never(); }
int launch_transpose(hipStream_t, int, int, const float*, long, float*, long) { return never(); }
}  // namespace mtnn

// kernel instances of tile geometries 2 (128 x 128 x 64), 6 (128 x 256 x 32) and 8 (128 x 64 x 32)
#include "gemm_inst.h"
namespace mtnn {
void fill_kernel_sets_c(KernelSet* t)
{
    t[2] = make_kernel_set<128, 128, 64, 4, 2, 2, 16>();
    t[6] = make_kernel_set<128, 256, 32, 2, 4, 2, 16>();
    t[8] = make_kernel_set<128, 64, 32, 2, 2, 2, 16>();
}
}  // namespace mtnn

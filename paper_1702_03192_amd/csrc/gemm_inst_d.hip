// kernel instances of tile geometries 7 (256 x 128 x 32), 9 (64 x 128 x 32) and 10 (128 x 128 x 32)
#include "gemm_inst.h"
namespace mtnn {
void fill_kernel_sets_d(KernelSet* t)
{
    t[7] = make_kernel_set<256, 128, 32, 4, 2, 2, 16>();
    t[9] = make_kernel_set<64, 128, 32, 2, 2, 2, 16>();
    t[10] = make_kernel_set<128, 128, 32, 2, 2, 2, 16>();
}
}  // namespace mtnn

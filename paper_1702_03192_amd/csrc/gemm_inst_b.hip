// kernel instances of tile geometries 1 (256 x 128 x 16), 4 (32 x 256 x 32) and 5 (256 x 32 x 32)
#include "gemm_inst.h"
namespace mtnn {
void fill_kernel_sets_b(KernelSet* t)
{
    t[1] = make_kernel_set<256, 128, 16, 2, 2, 3, 16>();
    t[4] = make_kernel_set<32, 256, 32, 1, 4, 2, 16>();
    t[5] = make_kernel_set<256, 32, 32, 4, 1, 2, 16>();
}
}  // namespace mtnn

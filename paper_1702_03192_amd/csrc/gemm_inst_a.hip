// kernel instances of tile geometries 0 (256 x 256 x 32) and 3 (64 x 64 x 64)
#include "gemm_inst.h"
namespace mtnn {
void fill_kernel_sets_a(KernelSet* t)
{
    t[0] = make_kernel_set<256, 256, 32, 4, 2, 2, 16>();
    t[3] = make_kernel_set<64, 64, 64, 2, 2, 2, 16>();
}
}  // namespace mtnn

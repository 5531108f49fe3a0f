// kernel instances with two sets of waves per workgroup: tile geometries 11 (64 x 64 x 64), 12 (32 x 256 x 32) and 13 (256 x 32 x 32)
#include "gemm_inst.h"
namespace mtnn {
void fill_kernel_sets_e(KernelSet* t)
{
    t[11] = make_kernel_set<64, 64, 64, 2, 2, 2, 16, 2>();
    t[12] = make_kernel_set<32, 256, 32, 1, 4, 2, 16, 2>();
    t[13] = make_kernel_set<256, 32, 32, 4, 1, 2, 16, 2>();
}
}  // namespace mtnn

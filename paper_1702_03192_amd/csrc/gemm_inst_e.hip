// kernel instances of tile geometry 11 (64 x 64 x 64 with two sets of waves per workgroup)
#include "gemm_inst.h"
namespace mtnn {
void fill_kernel_sets_e(KernelSet* t)
{
    t[11] = make_kernel_set<64, 64, 64, 2, 2, 2, 16, 2>();
}
}  // namespace mtnn

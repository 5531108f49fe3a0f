// One KernelSet per tile geometry: every kernel instance of that geometry, taken by address so that
// the launcher (another translation unit) can launch them.  Included by the gemm_inst_*.hip files,
// each of which instantiates a few geometries (the instances compile in parallel).
#pragma once
#include "gemm_kernels.h"

namespace mtnn {

// The pipelined kernel with a fused epilogue, or null for the 16-wide-slab geometry: there the
// epilogue's arithmetic makes the compiler move all 128 accumulators from AGPRs to VGPRs in one block
// at the loop exit, and the registers that takes no longer allow the two workgroups per CU the
// configuration is rated for (its launches run the plain kernel and the separate pass instead).
template <int BM, int BN, int BK, int WMV, int WNV, bool NT, int NS, int EPI, int KS>
constexpr GemmKernel epilogue_kernel()
{
    if constexpr (BK == 16) return nullptr;
    else return &gemm_dma_kernel<BM, BN, BK, WMV, WNV, NT, NS, EPI, KS>;
}

// tile BM x BN, pipelined slab BK with NS buffers, WMV x WNV waves (KS sets of them in the pipelined
// kernel), guarded kernel's slab GBK
template <int BM, int BN, int BK, int WMV, int WNV, int NS, int GBK, int KS = 1>
KernelSet make_kernel_set()
{
    KernelSet s;
    s.kern[0][0] = gemm_kernel<BM, BN, GBK, WMV, WNV, false, false>;
    s.kern[0][1] = gemm_kernel<BM, BN, GBK, WMV, WNV, false, true>;
    s.kern[1][0] = gemm_kernel<BM, BN, GBK, WMV, WNV, true, false>;
    s.kern[1][1] = gemm_kernel<BM, BN, GBK, WMV, WNV, true, true>;
    s.dma[0] = gemm_dma_kernel<BM, BN, BK, WMV, WNV, false, NS, kEpiNone, KS>;
    s.dma[1] = gemm_dma_kernel<BM, BN, BK, WMV, WNV, true, NS, kEpiNone, KS>;
    s.dma_bias[0] = epilogue_kernel<BM, BN, BK, WMV, WNV, false, NS, kEpiBiasAct, KS>();
    s.dma_bias[1] = epilogue_kernel<BM, BN, BK, WMV, WNV, true, NS, kEpiBiasAct, KS>();
    s.dma_sgd = epilogue_kernel<BM, BN, BK, WMV, WNV, false, NS, kEpiSgd, KS>();
    s.sk[0] = gemm_streamk_kernel<BM, BN, BK, WMV, WNV, false, NS, KS>;
    s.sk[1] = gemm_streamk_kernel<BM, BN, BK, WMV, WNV, true, NS, KS>;
    s.fix = streamk_fixup_kernel<BM, BN>;
    return s;
}

}  // namespace mtnn

// Measurement aid (not part of the paper's method): do fp32 matrix instructions and ordinary vector
// instructions of OTHER waves on the same SIMD overlap?  Each workgroup has eight waves, two per
// SIMD: waves 0-3 issue `n_mfma` v_mfma_f32_32x32x2_f32 on two independent accumulator chains, waves
// 4-7 issue `n_valu` fp32 multiply-adds on four independent chains.  Timing the launch with only the
// first kind of work, only the second, and both answers the question: if the two kinds overlapped,
// the third time would be the larger of the first two; on gfx950 it is their sum, because the fp32
// matrix instructions execute on the vector lanes (the fp32 matrix and vector peak rates are the
// same number).  The GEMM kernels' design follows from that: every vector instruction around the k
// loop costs matrix time.
#include "../../include/mtnn.h"
#include "mtnn_internal.h"

namespace mtnn {

typedef float f32x16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(512) void probe_lanes_kernel(float* __restrict__ sink, int n_mfma, int n_valu)
{
    const int wave = threadIdx.x >> 6;
    if (wave < 4) {
        f32x16 a0 = {}, a1 = {};
        const float x = threadIdx.x * 1e-3f, y = 1.0f;
        for (int i = 0; i < n_mfma; i += 2) {
            a0 = __builtin_amdgcn_mfma_f32_32x32x2f32(x, y, a0, 0, 0, 0);
            a1 = __builtin_amdgcn_mfma_f32_32x32x2f32(y, x, a1, 0, 0, 0);
        }
        if (a0[0] + a1[3] == 1234.5f) sink[threadIdx.x] = a0[1];          // (keeps the chains alive; never true)
    } else {
        float v0 = threadIdx.x, v1 = 1.f, v2 = 2.f, v3 = 3.f;
        const float c = 1.0001f;
        for (int i = 0; i < n_valu; i += 4) {
            v0 = __builtin_fmaf(v0, c, 1.f);
            v1 = __builtin_fmaf(v1, c, 1.f);
            v2 = __builtin_fmaf(v2, c, 1.f);
            v3 = __builtin_fmaf(v3, c, 1.f);
        }
        if (v0 + v1 + v2 + v3 == 1234.5f) sink[threadIdx.x] = v0;
    }
}

}  // namespace mtnn

extern "C" int mtnn_probe_lanes(void* stream, int n_mfma, int n_valu, float* sink)
{
    if (n_mfma < 0 || n_valu < 0) return MTNN_ERR_DIM;
    if (!sink) return MTNN_ERR_NULL;
    mtnn::Geometry geo;
    if (!mtnn::current_geometry(&geo)) return MTNN_ERR_NO_DEVICE;
    hipLaunchKernelGGL(mtnn::probe_lanes_kernel, dim3((unsigned)geo.cus), dim3(512), 0, static_cast<hipStream_t>(stream),
                       sink, n_mfma, n_valu);
    return hipGetLastError() == hipSuccess ? MTNN_OK : MTNN_ERR_LAUNCH;
}

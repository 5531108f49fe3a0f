// Internal declarations shared by the translation units of libmtnn (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace mtnn {

enum GemmOp { OP_NN = 0, OP_NT = 1 };

// Launchers return a hipError_t-compatible int (0 = success).  All arguments are assumed
// validated: m, n >= 1, k >= 1, leading dimensions large enough, pointers non-null.
// cfg < 0: configuration chosen by the fixed rule; splits <= 0: split count chosen by the rule.
//
// epi (optional): work fused into the product's epilogue.  kind 1: C = act(A x B + bias[column]);
// kind 2 (NN only): C = A x B and W = fma(-lr, C, W) for a second m x n matrix W.  A launch that
// cannot fuse it (operands the pipelined kernel does not take; for kind 2 also a split launch)
// computes the plain product and reports *fused = false: the caller then runs the separate pass.
struct Epilogue {
    int kind;
    const float* bias;
    int relu;
    float* W;
    long ldw;
    float lr;
};
int launch_gemm(hipStream_t s, int op, int cfg, int splits, int m, int n, int k,
                const float* A, long lda, const float* B, long ldb, float* C, long ldc,
                const Epilogue* epi = nullptr, bool* fused = nullptr);
int gemm_config_count();
long long gemm_streamk_launches();
long long gemm_fused_launches();
const char* gemm_config_name(int cfg);
int gemm_default_config(int op, int m, int n, int k);
int gemm_default_splits(int op, int m, int n, int k);

// the separate passes behind the fused epilogues, for matrices with any leading dimension (fc.hip)
int launch_bias_act(hipStream_t s, int rows, int width, float* Z, long ld, const float* b, int relu);
int launch_sgd_2d(hipStream_t s, int rows, int width, float* P, long ldp, const float* G, long ldg, float lr);

int launch_fill_zero(hipStream_t s, int m, int n, float* C, long ldc);
int launch_transpose_inplace(hipStream_t s, int n, float* X, long ld);
int launch_copy(hipStream_t s, size_t nvec, const void* in, void* out);
int launch_transpose(hipStream_t s, int rows, int cols, const float* in, long ldin, float* out, long ldout);

}  // namespace mtnn

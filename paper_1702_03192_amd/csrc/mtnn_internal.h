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
int launch_gemm(hipStream_t s, int op, int cfg, int splits, int m, int n, int k,
                const float* A, long lda, const float* B, long ldb, float* C, long ldc);
int gemm_config_count();
long long gemm_streamk_launches();
const char* gemm_config_name(int cfg);
int gemm_default_config(int op, int m, int n, int k);
int gemm_default_splits(int op, int m, int n, int k);

int launch_fill_zero(hipStream_t s, int m, int n, float* C, long ldc);
int launch_transpose_inplace(hipStream_t s, int n, float* X, long ld);
int launch_copy(hipStream_t s, size_t nvec, const void* in, void* out);
int launch_transpose(hipStream_t s, int rows, int cols, const float* in, long ldin, float* out, long ldout);

}  // namespace mtnn

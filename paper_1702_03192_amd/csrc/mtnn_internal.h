// Internal declarations shared by the translation units of libmtnn (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace mtnn {

enum GemmOp { OP_NN = 0, OP_NT = 1 };

// ---- the device the kernels were written for (device.cpp) ---------------------------------------
// What the launchers and the cost model need to know about a GPU.  Read from the device once per
// device; the nominal MI355X figures stand in where no device can be asked (host-only callers of the
// cost model).
struct Geometry {
    int device;         // HIP device ordinal, -1 for the nominal figures
    int cus;            // compute units (256 on MI355X)
    int xcds;           // accelerator dies, each with its own L2; workgroup ids are dealt round robin to them (8)
    int lds_per_cu;     // bytes of LDS per compute unit (160 KB)
};
Geometry nominal_geometry();
// Is `arch` (hipDeviceProp_t::gcnArchName, e.g. "gfx950:sramecc+:xnack-") the architecture the
// kernels are compiled for?
bool arch_is_gfx950(const char* arch);
// Geometry of the current device.  Returns false if there is no current device, its properties
// cannot be read, or it is not a gfx950: the library then launches nothing.
bool current_geometry(Geometry* out);
// current_geometry() if there is a usable device, else the nominal figures
Geometry geometry_or_nominal();

// ---- scratch memory for partial products (device.cpp) -----------------------------------------
// The library allocates no device memory.  Split-k and the even cut keep partial products in a
// buffer the CALLER registers per (device, stream) with mtnn_set_scratch; launches on one stream are
// ordered, so they can share it.  Nothing registered: {nullptr, 0}, and only unsplit launches run.
struct Scratch {
    float* ptr;
    size_t bytes;
};
Scratch scratch_lookup(hipStream_t s);
int scratch_register(hipStream_t s, void* ptr, size_t bytes);   // MTNN status

// Launchers return a hipError_t-compatible int (0 = success).  All arguments are assumed
// validated: m, n >= 1, k >= 1, leading dimensions large enough, pointers non-null.
// cfg < 0: configuration chosen by the fixed rule; splits <= 0: split count chosen by the rule
// among those whose partial products fit `scratch`.  An explicit split count (or the even cut)
// whose partials do not fit returns kErrScratch.
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
constexpr int kErrScratch = -1000;     // not a hipError_t: the launch needs more scratch than it was given
int launch_gemm(hipStream_t s, const Geometry& geo, const Scratch& scratch, int op, int cfg, int splits, int m, int n, int k,
                const float* A, long lda, const float* B, long ldb, float* C, long ldc,
                const Epilogue* epi = nullptr, bool* fused = nullptr);
// Argument validation and dispatch of mtnn_gemm_ex (api.cpp).  provider: called after validation,
// with the device known to be usable, for the scratch a divided launch may use (it returns an MTNN
// status); null = the scratch registered for the stream.
typedef int (*ScratchProvider)(Scratch* out);
int gemm_ex_entry(void* stream, int op, int cfg, int splits, int m, int n, int k, const float* A, int lda,
                  const float* B, int ldb, float* C, int ldc, ScratchProvider provider);
int gemm_config_count();
long long gemm_streamk_launches();
long long gemm_fused_launches();
const char* gemm_config_name(int cfg);
int gemm_default_config(int op, int m, int n, int k, size_t scratch_bytes);
int gemm_default_splits(int op, int m, int n, int k, size_t scratch_bytes);
// the cost model's estimate for the launch the rule would choose (aligned operands)
double gemm_predicted_seconds(const Geometry& geo, int op, int m, int n, int k, size_t scratch_bytes);

// the separate passes behind the fused epilogues, for matrices with any leading dimension (fc.hip)
int launch_bias_act(hipStream_t s, int rows, int width, float* Z, long ld, const float* b, int relu);
int launch_sgd_2d(hipStream_t s, int rows, int width, float* P, long ldp, const float* G, long ldg, float lr);

int launch_fill_zero(hipStream_t s, int m, int n, float* C, long ldc);
int launch_transpose_inplace(hipStream_t s, int n, float* X, long ld);
// dense rows x cols -> cols x rows in the same buffer (transpose_inplace_rect.hip)
bool transpose_inplace_rect_supported(int rows, int cols);
int launch_transpose_inplace_rect(hipStream_t s, int rows, int cols, float* X);
int launch_copy(hipStream_t s, size_t nvec, const void* in, void* out);
int launch_transpose(hipStream_t s, int rows, int cols, const float* in, long ldin, float* out, long ldout);

}  // namespace mtnn

// C ABI of libmtnn: argument validation, Algorithm 1 (TNN) and Algorithm 2 (MTNN) of the paper
// as host-side compositions of the HIP kernels.  Validation is pure host code and runs before
// any HIP call, so it behaves the same on a machine without a GPU.
#include "../../include/mtnn.h"
#include "mtnn_internal.h"
#include "selector.h"
#include "gemm_config.h"

#include <atomic>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

namespace {

std::atomic<int> g_last_hip_error{0};   // last non-zero HIP error a launcher reported (diagnostics only)
std::atomic<int> g_fuse_epilogues{1};   // mtnn_set_fused_epilogues: 0 = always the separate pass (measurements)

int launch_status(int err)
{
    if (err == 0) return MTNN_OK;
    if (err == mtnn::kErrScratch) return MTNN_ERR_WORKSPACE;
    g_last_hip_error = err;
    return MTNN_ERR_LAUNCH;
}

// what split launches on a stream may use when the caller has registered nothing smaller or larger
constexpr size_t kDefaultScratchBytes = 64u << 20;

struct Range {
    uintptr_t lo, hi;   // [lo, hi)
};

// bytes spanned by a rows x cols fp32 matrix with leading dimension ld
Range span(const void* p, long long rows, long long cols, long long ld)
{
    Range r;
    r.lo = reinterpret_cast<uintptr_t>(p);
    if (rows <= 0 || cols <= 0) { r.hi = r.lo; return r; }
    r.hi = r.lo + (uintptr_t)(((rows - 1) * ld + cols) * 4);
    return r;
}

bool overlap(const Range& a, const Range& b)
{
    return a.lo < a.hi && b.lo < b.hi && a.lo < b.hi && b.lo < a.hi;
}

int check_gemm(int op, int m, int n, int k, const float* A, int lda, const float* B, int ldb,
               const float* C, int ldc)
{
    if (m < 0 || n < 0 || k < 0) return MTNN_ERR_DIM;
    if (m == 0 || n == 0) return MTNN_OK;
    if (!C) return MTNN_ERR_NULL;
    if (ldc < n) return MTNN_ERR_LD;
    if (k == 0) return MTNN_OK;
    if (!A || !B) return MTNN_ERR_NULL;
    if (lda < k) return MTNN_ERR_LD;
    const int b_rows = (op == mtnn::OP_NT) ? n : k;
    const int b_cols = (op == mtnn::OP_NT) ? k : n;
    if (ldb < b_cols) return MTNN_ERR_LD;
    const Range rc = span(C, m, n, ldc);
    if (overlap(rc, span(A, m, k, lda)) || overlap(rc, span(B, b_rows, b_cols, ldb))) return MTNN_ERR_ALIAS;
    return MTNN_OK;
}

// epi: work to fuse into the product where the launch can, done as a separate pass over C where it cannot
// provider: where a divided launch keeps its partial products; null = what the caller registered for the stream
int run_gemm(void* stream, int op, int cfg, int splits, int m, int n, int k, const float* A, int lda,
             const float* B, int ldb, float* C, int ldc, const mtnn::Epilogue* epi = nullptr,
             mtnn::ScratchProvider provider = nullptr)
{
    const int st = check_gemm(op, m, n, k, A, lda, B, ldb, C, ldc);
    if (st != MTNN_OK) return st;
    if (m == 0 || n == 0) return MTNN_OK;
    mtnn::Geometry geo;
    if (!mtnn::current_geometry(&geo)) return MTNN_ERR_NO_DEVICE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int err;
    bool fused = false;
    if (k == 0) {
        err = mtnn::launch_fill_zero(s, m, n, C, ldc);
    } else {
        mtnn::Scratch scratch;
        if (provider) {
            const int ps = provider(&scratch);
            if (ps != MTNN_OK) return ps;
        } else {
            scratch = mtnn::scratch_lookup(s);
        }
        err = mtnn::launch_gemm(s, geo, scratch, op, cfg, splits, m, n, k, A, lda, B, ldb, C, ldc,
                                g_fuse_epilogues.load() ? epi : nullptr, &fused);
    }
    if (err == 0 && epi && !fused) {
        if (epi->kind == 1) err = mtnn::launch_bias_act(s, m, n, C, ldc, epi->bias, epi->relu);
        else err = mtnn::launch_sgd_2d(s, m, n, epi->W, epi->ldw, C, ldc, epi->lr);
    }
    return launch_status(err);
}

// Algorithm 1 with an optional epilogue on the NN product
int tnn_impl(void* stream, int m, int n, int k, const float* A, int lda, const float* B, int ldb,
             float* C, int ldc, void* workspace, size_t workspace_bytes, const mtnn::Epilogue* epi)
{
    int st = check_gemm(mtnn::OP_NT, m, n, k, A, lda, B, ldb, C, ldc);
    if (st != MTNN_OK) return st;
    if (m == 0 || n == 0) return MTNN_OK;
    if (k == 0) return run_gemm(stream, mtnn::OP_NT, -1, 0, m, n, k, A, lda, B, ldb, C, ldc, epi);
    if (!workspace || workspace_bytes < mtnn_tnn_workspace_bytes(n, k)) return MTNN_ERR_WORKSPACE;
    float* Bt = static_cast<float*>(workspace);
    const Range rw = span(Bt, k, n, n);
    if (overlap(rw, span(A, m, k, lda)) || overlap(rw, span(B, n, k, ldb)) || overlap(rw, span(C, m, n, ldc)))
        return MTNN_ERR_ALIAS;
    // Algorithm 1: B (n x k) -> B^T (k x n), then the NN product on the same stream
    st = mtnn_transpose(stream, n, k, B, ldb, Bt, n);
    if (st != MTNN_OK) return st;
    return run_gemm(stream, mtnn::OP_NN, -1, 0, m, n, k, A, lda, Bt, n, C, ldc, epi);
}

// The choice of Algorithm 2: the predictor, overridden by the memory rule of Section II (no room for
// B^T: NT) and, for experiments, by the environment variable MTNN_FORCE=nt|tnn (read once).
int pick_label(int m, int n, int k, const void* workspace, size_t workspace_bytes)
{
    static const int forced = [] {
        const char* e = getenv("MTNN_FORCE");
        if (!e) return 0;
        if (!strcmp(e, "nt") || !strcmp(e, "NT")) return 1;
        if (!strcmp(e, "tnn") || !strcmp(e, "TNN")) return -1;
        return 0;
    }();
    int label = (m > 0 && n > 0 && k > 0) ? (forced ? forced : mtnn_select(m, n, k)) : 1;
    if (label == -1 && (!workspace || workspace_bytes < mtnn_tnn_workspace_bytes(n, k))) label = 1;
    return label;
}

bool device_ok()
{
    mtnn::Geometry geo;
    return mtnn::current_geometry(&geo);
}

int check_transpose(int rows, int cols, const float* in, int ldin, const float* out, int ldout)
{
    if (rows < 0 || cols < 0) return MTNN_ERR_DIM;
    if (rows == 0 || cols == 0) return MTNN_OK;
    if (!in || !out) return MTNN_ERR_NULL;
    if (ldin < cols || ldout < rows) return MTNN_ERR_LD;
    if (overlap(span(in, rows, cols, ldin), span(out, cols, rows, ldout))) return MTNN_ERR_ALIAS;
    return MTNN_OK;
}

}  // namespace

namespace mtnn {
int gemm_ex_entry(void* stream, int op, int cfg, int splits, int m, int n, int k, const float* A, int lda,
                  const float* B, int ldb, float* C, int ldc, ScratchProvider provider)
{
    if ((op != OP_NN && op != OP_NT) || cfg < -1 || cfg >= gemm_config_count() ||
        (splits < 0 && splits != MTNN_GEMM_EVEN_CUT) || splits > 32)
        return MTNN_ERR_ARG;
    return run_gemm(stream, op, cfg, splits, m, n, k, A, lda, B, ldb, C, ldc, nullptr, provider);
}
}  // namespace mtnn

extern "C" {

int mtnn_nt(void* stream, int m, int n, int k, const float* A, int lda, const float* B, int ldb,
            float* C, int ldc)
{
    return run_gemm(stream, mtnn::OP_NT, -1, 0, m, n, k, A, lda, B, ldb, C, ldc);
}

int mtnn_nn(void* stream, int m, int n, int k, const float* A, int lda, const float* B, int ldb,
            float* C, int ldc)
{
    return run_gemm(stream, mtnn::OP_NN, -1, 0, m, n, k, A, lda, B, ldb, C, ldc);
}

int mtnn_gemm_ex(void* stream, int op, int cfg, int splits, int m, int n, int k, const float* A, int lda,
                 const float* B, int ldb, float* C, int ldc)
{
    return mtnn::gemm_ex_entry(stream, op, cfg, splits, m, n, k, A, lda, B, ldb, C, ldc, nullptr);
}

int mtnn_gemm_default_splits(int op, int m, int n, int k)
{
    if ((op != mtnn::OP_NN && op != mtnn::OP_NT) || m <= 0 || n <= 0 || k <= 0) return -1;
    return mtnn::gemm_default_splits(op, m, n, k, kDefaultScratchBytes);
}

size_t mtnn_scratch_bytes_default(void) { return kDefaultScratchBytes; }

int mtnn_gemm_choice(int op, int m, int n, int k, size_t scratch_bytes, int* cfg, int* splits)
{
    if (op != mtnn::OP_NN && op != mtnn::OP_NT) return MTNN_ERR_ARG;
    if (m <= 0 || n <= 0 || k <= 0) return MTNN_ERR_DIM;
    const mtnn::Choice ch = mtnn::choose(mtnn::geometry_or_nominal(), op, m, n, k, true, true, mtnn::kEpiNone, scratch_bytes);
    if (cfg) *cfg = ch.cfg;
    if (splits) *splits = ch.splits;
    return MTNN_OK;
}

int mtnn_set_scratch(void* stream, void* scratch, size_t bytes)
{
    return mtnn::scratch_register(static_cast<hipStream_t>(stream), scratch, bytes);
}

size_t mtnn_get_scratch_bytes(void* stream)
{
    const mtnn::Scratch s = mtnn::scratch_lookup(static_cast<hipStream_t>(stream));
    return s.ptr ? s.bytes : 0;
}

size_t mtnn_gemm_scratch_bytes(int cfg, int splits, int m, int n, int k)
{
    if (cfg < 0 || cfg >= mtnn::gemm_config_count() || m <= 0 || n <= 0 || k <= 0) return 0;
    if (splits != MTNN_GEMM_EVEN_CUT && (splits < 2 || splits > 32)) return 0;
    return mtnn::scratch_needed(mtnn::geometry_or_nominal(), cfg, splits, m, n, k);
}

int mtnn_gemm_config_count(void) { return mtnn::gemm_config_count(); }
const char* mtnn_gemm_config_name(int cfg) { return mtnn::gemm_config_name(cfg); }
int mtnn_gemm_default_config(int op, int m, int n, int k)
{
    if ((op != mtnn::OP_NN && op != mtnn::OP_NT) || m <= 0 || n <= 0 || k <= 0) return -1;
    return mtnn::gemm_default_config(op, m, n, k, kDefaultScratchBytes);
}

int mtnn_transpose(void* stream, int rows, int cols, const float* in, int ldin, float* out, int ldout)
{
    const int st = check_transpose(rows, cols, in, ldin, out, ldout);
    if (st != MTNN_OK) return st;
    if (rows == 0 || cols == 0) return MTNN_OK;
    if (!device_ok()) return MTNN_ERR_NO_DEVICE;
    const int err = mtnn::launch_transpose(static_cast<hipStream_t>(stream), rows, cols, in, ldin, out, ldout);
    return launch_status(err);
}

int mtnn_transpose_inplace(void* stream, int n, float* X, int ld)
{
    if (n < 0) return MTNN_ERR_DIM;
    if (n == 0) return MTNN_OK;
    if (!X) return MTNN_ERR_NULL;
    if (ld < n) return MTNN_ERR_LD;
    if (!device_ok()) return MTNN_ERR_NO_DEVICE;
    return launch_status(mtnn::launch_transpose_inplace(static_cast<hipStream_t>(stream), n, X, ld));
}

int mtnn_transpose_inplace_rect(void* stream, int rows, int cols, float* X)
{
    if (rows < 0 || cols < 0) return MTNN_ERR_DIM;
    if (rows == 0 || cols == 0) return MTNN_OK;
    if (!X) return MTNN_ERR_NULL;
    if (rows == cols) return mtnn_transpose_inplace(stream, rows, X, rows);
    if (rows == 1 || cols == 1) return MTNN_OK;                    // a vector keeps its words where they are
    if (!mtnn::transpose_inplace_rect_supported(rows, cols)) return MTNN_ERR_ARG;
    if (!device_ok()) return MTNN_ERR_NO_DEVICE;
    return launch_status(mtnn::launch_transpose_inplace_rect(static_cast<hipStream_t>(stream), rows, cols, X));
}

int mtnn_tnn_inplace_supported(int n, int k, int ldb)
{
    if (n <= 0 || k <= 0 || ldb < k) return 0;
    if (n == k) return 1;                                          // square: any leading dimension
    return (ldb == k && mtnn::transpose_inplace_rect_supported(n, k)) ? 1 : 0;
}

int mtnn_tnn_inplace(void* stream, int m, int n, int k, const float* A, int lda, float* B, int ldb, float* C, int ldc)
{
    // TNN with no workspace: transpose B in place, NN product on it, transpose back
    const int st0 = check_gemm(mtnn::OP_NT, m, n, k, A, lda, B, ldb, C, ldc);
    if (st0 != MTNN_OK) return st0;
    if (m == 0 || n == 0) return MTNN_OK;
    if (k == 0) return run_gemm(stream, mtnn::OP_NT, -1, 0, m, n, k, A, lda, B, ldb, C, ldc);
    if (!mtnn_tnn_inplace_supported(n, k, ldb)) return MTNN_ERR_ARG;
    // B is written on the way (transposed, then transposed back): as an output it must not overlap A
    // (the Gram product A x A^T with A == B would otherwise have its left operand transposed under it)
    if (overlap(span(B, n, k, ldb), span(A, m, k, lda))) return MTNN_ERR_ALIAS;
    const bool square = (n == k);
    int st = square ? mtnn_transpose_inplace(stream, n, B, ldb) : mtnn_transpose_inplace_rect(stream, n, k, B);
    if (st != MTNN_OK) return st;
    // B now holds B^T: k x n, leading dimension ldb (square) or n (dense rectangular)
    st = run_gemm(stream, mtnn::OP_NN, -1, 0, m, n, k, A, lda, B, square ? ldb : n, C, ldc);
    // restore B even if the product failed to launch
    const int st2 = square ? mtnn_transpose_inplace(stream, n, B, ldb) : mtnn_transpose_inplace_rect(stream, k, n, B);
    return st != MTNN_OK ? st : st2;
}

// Does TNN through in-place transposes promise to beat NT?  The cost model's estimates of the two
// products, and two in-place transposes of B at their measured rates (8 bytes per word moved): the
// square kernel, one pass of tile swaps, ~4.1 TB/s; the rectangular one, two or three passes over the
// buffer, 0.9-2.2 TB/s (1.2 taken, and three launches).
static bool inplace_pays(int m, int n, int k)
{
    const mtnn::Geometry geo = mtnn::geometry_or_nominal();
    const double t_nt = mtnn::gemm_predicted_seconds(geo, mtnn::OP_NT, m, n, k, kDefaultScratchBytes);
    const double t_nn = mtnn::gemm_predicted_seconds(geo, mtnn::OP_NN, m, n, k, kDefaultScratchBytes);
    const double bytes = 8.0 * (double)n * (double)k;
    const double t_ip = (n == k) ? bytes / 4.1e12 + 3e-6 : bytes / 1.2e12 + 12e-6;
    return t_nt - t_nn > 2.0 * t_ip;
}

int mtnn_select3(int m, int n, int k, int have_workspace, int can_inplace)
{
    if (m <= 0 || n <= 0 || k <= 0) return 0;
    const int label = mtnn_select(m, n, k);
    if (label != -1) return label;
    if (have_workspace) return -1;
    return (can_inplace && inplace_pays(m, n, k)) ? -2 : 1;
}

int mtnn_auto3(void* stream, int mode, int m, int n, int k, const float* A, int lda, float* B, int ldb,
               float* C, int ldc, void* workspace, size_t workspace_bytes, int* chosen)
{
    if (mode != 0 && mode != 1 && mode != -1 && mode != -2) return MTNN_ERR_ARG;
    const int st = check_gemm(mtnn::OP_NT, m, n, k, A, lda, B, ldb, C, ldc);
    if (st != MTNN_OK) return st;
    int path = mode;
    if (mode == 0) {
        const bool room = workspace && workspace_bytes >= mtnn_tnn_workspace_bytes(n, k);
        const bool can_ip = m > 0 && n > 0 && k > 0 && mtnn_tnn_inplace_supported(n, k, ldb) &&
                            !overlap(span(B, n, k, ldb), span(A, m, k, lda));
        path = (m > 0 && n > 0 && k > 0) ? mtnn_select3(m, n, k, room ? 1 : 0, can_ip ? 1 : 0) : 1;
        if (path == -1 && !room) path = 1;       // (the memory rule once more: never TNN without room for B^T)
    }
    if (chosen) *chosen = path;
    if (path == -2) return mtnn_tnn_inplace(stream, m, n, k, A, lda, B, ldb, C, ldc);
    if (path == -1) return mtnn_tnn(stream, m, n, k, A, lda, B, ldb, C, ldc, workspace, workspace_bytes);
    return mtnn_nt(stream, m, n, k, A, lda, B, ldb, C, ldc);
}

int mtnn_copy_bytes(void* stream, size_t bytes, const void* in, void* out)
{
    if (bytes == 0) return MTNN_OK;
    if (!in || !out) return MTNN_ERR_NULL;
    if ((bytes & 15) || (reinterpret_cast<uintptr_t>(in) & 15) || (reinterpret_cast<uintptr_t>(out) & 15))
        return MTNN_ERR_ARG;
    const uintptr_t a = reinterpret_cast<uintptr_t>(in), b = reinterpret_cast<uintptr_t>(out);
    if (a < b + bytes && b < a + bytes) return MTNN_ERR_ALIAS;
    if (!device_ok()) return MTNN_ERR_NO_DEVICE;
    return launch_status(mtnn::launch_copy(static_cast<hipStream_t>(stream), bytes / 16, in, out));
}

size_t mtnn_tnn_workspace_bytes(int n, int k)
{
    if (n <= 0 || k <= 0) return 0;
    const size_t bytes = (size_t)n * (size_t)k * 4u;
    return (bytes + 255u) & ~(size_t)255u;
}

int mtnn_tnn(void* stream, int m, int n, int k, const float* A, int lda, const float* B, int ldb,
             float* C, int ldc, void* workspace, size_t workspace_bytes)
{
    return tnn_impl(stream, m, n, k, A, lda, B, ldb, C, ldc, workspace, workspace_bytes, nullptr);
}

int mtnn_auto(void* stream, int m, int n, int k, const float* A, int lda, const float* B, int ldb,
              float* C, int ldc, void* workspace, size_t workspace_bytes, int* chosen)
{
    // Algorithm 2
    const int label = pick_label(m, n, k, workspace, workspace_bytes);
    if (chosen) *chosen = label;
    if (label == -1)
        return mtnn_tnn(stream, m, n, k, A, lda, B, ldb, C, ldc, workspace, workspace_bytes);
    return mtnn_nt(stream, m, n, k, A, lda, B, ldb, C, ldc);
}

int mtnn_fc_layer_forward(void* stream, int mode, int m, int n, int k, const float* X, int ldx, const float* W, int ldw,
                          const float* b, int relu, float* Y, int ldy, void* workspace, size_t workspace_bytes, int* chosen)
{
    if ((mode != 1 && mode != 0 && mode != -1) || (relu != 0 && relu != 1)) return MTNN_ERR_ARG;
    const int st = check_gemm(mtnn::OP_NT, m, n, k, X, ldx, W, ldw, Y, ldy);
    if (st != MTNN_OK) return st;
    int label = mode;
    if (mode == 0) label = pick_label(m, n, k, workspace, workspace_bytes);
    if (chosen) *chosen = label;
    if (m == 0 || n == 0) return MTNN_OK;
    if (!b) return MTNN_ERR_NULL;
    if (overlap(span(Y, m, n, ldy), span(b, 1, n, n))) return MTNN_ERR_ALIAS;
    const mtnn::Epilogue epi = {1, b, relu, nullptr, 0, 0.f};
    if (label == -1)
        return tnn_impl(stream, m, n, k, X, ldx, W, ldw, Y, ldy, workspace, workspace_bytes, &epi);
    return run_gemm(stream, mtnn::OP_NT, -1, 0, m, n, k, X, ldx, W, ldw, Y, ldy, &epi);
}

int mtnn_fc_weight_grad_sgd(void* stream, int m, int n, int k, const float* A, int lda, const float* B, int ldb,
                            float* dW, int lddw, float* W, int ldw, float lr)
{
    const int st = check_gemm(mtnn::OP_NN, m, n, k, A, lda, B, ldb, dW, lddw);
    if (st != MTNN_OK) return st;
    if (m == 0 || n == 0) return MTNN_OK;
    if (!W) return MTNN_ERR_NULL;
    if (ldw < n) return MTNN_ERR_LD;
    const Range rw = span(W, m, n, ldw);
    if (overlap(rw, span(dW, m, n, lddw)) || (k > 0 && (overlap(rw, span(A, m, k, lda)) || overlap(rw, span(B, k, n, ldb)))))
        return MTNN_ERR_ALIAS;
    const mtnn::Epilogue epi = {2, nullptr, 0, W, ldw, lr};
    return run_gemm(stream, mtnn::OP_NN, -1, 0, m, n, k, A, lda, B, ldb, dW, lddw, &epi);
}

const char* mtnn_status_string(int status)
{
    switch (status) {
        case MTNN_OK: return "ok";
        case MTNN_ERR_DIM: return "negative dimension";
        case MTNN_ERR_NULL: return "null pointer with a non-empty problem";
        case MTNN_ERR_LD: return "leading dimension smaller than the row length";
        case MTNN_ERR_ALIAS: return "output overlaps an input";
        case MTNN_ERR_WORKSPACE: return "workspace missing or too small";
        case MTNN_ERR_LAUNCH: return "HIP launch failed";
        case MTNN_ERR_MODEL: return "model file missing or malformed";
        case MTNN_ERR_ARG: return "invalid argument";
        case MTNN_ERR_NO_DEVICE: return "no usable gfx950 device";
        default: return "unknown status";
    }
}

int mtnn_last_hip_error(void) { return g_last_hip_error.load(); }

int mtnn_version(void) { return 100; }

long long mtnn_gemm_even_cut_launches(void) { return mtnn::gemm_streamk_launches(); }
long long mtnn_gemm_fused_epilogue_launches(void) { return mtnn::gemm_fused_launches(); }
int mtnn_set_fused_epilogues(int enable) { return g_fuse_epilogues.exchange(enable ? 1 : 0); }

int mtnn_arch_supported(const char* arch) { return mtnn::arch_is_gfx950(arch) ? 1 : 0; }

int mtnn_device_attribute(int what)
{
    static const hipDeviceAttribute_t attrs[4] = {hipDeviceAttributeMultiprocessorCount, hipDeviceAttributeClockRate,
                                                  hipDeviceAttributeMemoryClockRate, hipDeviceAttributeMemoryBusWidth};
    if (what < 0 || what > 3) return -1;
    int dev = 0, value = -1;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&value, attrs[what], dev) != hipSuccess) {
        (void)hipGetLastError();
        return -1;
    }
    return value;
}

}  // extern "C"

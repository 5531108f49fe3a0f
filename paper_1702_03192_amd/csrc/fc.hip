// One training step of a fully connected net built on the NT / NN / transpose operations
// (the setting of Section V-C of the MTNN paper: layer sizes as in Table IX, where the forward
// product of a layer -- activations (mb x l1) times the transpose of the weights (l2 x l1) -- is
// the NT operation MTNN accelerates and the backward products are plain NN operations).
//
// The paper fixes only the layer sizes.  The rest is this library's reading: a bias on every
// layer, ReLU after every hidden layer, softmax cross-entropy averaged over the mini-batch, plain
// SGD.  Every matrix product goes through mtnn_nt / mtnn_tnn / mtnn_auto (forward) and
// mtnn_nn / mtnn_transpose (backward); the kernels here are the small elementwise and reduction
// steps around them.  All reductions run in a fixed order: results are bit-reproducible.
#include "../../include/mtnn.h"
#include "mtnn_internal.h"

#include <math.h>

namespace mtnn {

// Z[i][j] += b[j]; if relu, clamp at zero.  In place on the GEMM output (batch x width, ld = width).
__global__ __launch_bounds__(256) void bias_act_kernel(float* __restrict__ Z, const float* __restrict__ b,
                                                       long long total, int width, int relu)
{
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (long long)gridDim.x * blockDim.x) {
        float v = Z[e] + b[e % width];
        if (relu) v = v > 0.f ? v : 0.f;
        Z[e] = v;
    }
}

// One wave per row: stable softmax, loss_i = -log p[label_i], dZ = (p - onehot) / batch.
__global__ __launch_bounds__(64) void softmax_xent_kernel(const float* __restrict__ logits, const int* __restrict__ labels,
                                                          float* __restrict__ dZ, float* __restrict__ row_loss,
                                                          int batch, int classes)
{
    const int row = blockIdx.x;
    const int lane = threadIdx.x;
    const float* z = logits + (size_t)row * classes;
    float mx = -INFINITY;
    for (int j = lane; j < classes; j += 64) mx = fmaxf(mx, z[j]);
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    float sum = 0.f;
    for (int j = lane; j < classes; j += 64) sum += expf(z[j] - mx);
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
    const float lse = logf(sum);
    const int lab = labels[row];
    const float inv_b = 1.0f / (float)batch;
    for (int j = lane; j < classes; j += 64) {
        const float p = expf(z[j] - mx - lse);
        dZ[(size_t)row * classes + j] = (p - (j == lab ? 1.f : 0.f)) * inv_b;
    }
    // a label outside [0, classes) has no log-probability: its row reports NaN instead of reading out of bounds
    if (lane == 0) row_loss[row] = (lab >= 0 && lab < classes) ? -(z[lab] - mx - lse) : NAN;
}

// mean of `n` values with one workgroup and a fixed tree: out[0] = sum(v) / n
__global__ __launch_bounds__(256) void mean_kernel(const float* __restrict__ v, int n, float* __restrict__ out)
{
    __shared__ float part[256];
    float s = 0.f;
    for (int i = threadIdx.x; i < n; i += 256) s += v[i];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = part[0] / (float)n;
}

// dZ = dH where H > 0 else 0 (H is the ReLU output; H > 0 exactly where the pre-activation was > 0)
__global__ __launch_bounds__(256) void relu_backward_kernel(float* __restrict__ dH, const float* __restrict__ H, long long total)
{
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (long long)gridDim.x * blockDim.x)
        dH[e] = H[e] > 0.f ? dH[e] : 0.f;
}

// db[j] = sum_i dZ[i][j]: 64 columns per workgroup, 4 row groups of 64 lanes, rows in a fixed order
__global__ __launch_bounds__(256) void bias_grad_kernel(const float* __restrict__ dZ, float* __restrict__ db, int batch, int width)
{
    __shared__ float part[4][64];
    const int col = blockIdx.x * 64 + (threadIdx.x & 63);
    const int grp = threadIdx.x >> 6;
    float s = 0.f;
    if (col < width)
        for (int i = grp; i < batch; i += 4) s += dZ[(size_t)i * width + col];
    part[grp][threadIdx.x & 63] = s;
    __syncthreads();
    if (grp == 0 && col < width) db[col] = (part[0][threadIdx.x] + part[1][threadIdx.x]) + (part[2][threadIdx.x] + part[3][threadIdx.x]);
}

// Two-stage version for large batches: stage 1 sums row chunk blockIdx.y of 64 columns into
// part[chunk][col]; stage 2 adds the chunks in order.  Same fixed order on every run.
__global__ __launch_bounds__(256) void bias_grad_partial_kernel(const float* __restrict__ dZ, float* __restrict__ part,
                                                                int batch, int width, int rows_per_chunk)
{
    __shared__ float acc[4][64];
    const int col = blockIdx.x * 64 + (threadIdx.x & 63);
    const int grp = threadIdx.x >> 6;
    const int r0 = blockIdx.y * rows_per_chunk;
    const int r1 = min(batch, r0 + rows_per_chunk);
    float s = 0.f;
    if (col < width)
        for (int i = r0 + grp; i < r1; i += 4) s += dZ[(size_t)i * width + col];
    acc[grp][threadIdx.x & 63] = s;
    __syncthreads();
    if (grp == 0 && col < width)
        part[(size_t)blockIdx.y * width + col] =
            (acc[0][threadIdx.x] + acc[1][threadIdx.x]) + (acc[2][threadIdx.x] + acc[3][threadIdx.x]);
}

__global__ __launch_bounds__(256) void bias_grad_final_kernel(const float* __restrict__ part, int chunks, int width,
                                                              float* __restrict__ db)
{
    const int col = blockIdx.x * 256 + threadIdx.x;
    if (col >= width) return;
    float s = part[col];
    for (int c = 1; c < chunks; ++c) s += part[(size_t)c * width + col];
    db[col] = s;
}

// P -= lr * G
__global__ __launch_bounds__(256) void sgd_kernel(float* __restrict__ P, const float* __restrict__ G, long long total, float lr)
{
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (long long)gridDim.x * blockDim.x)
        P[e] = __builtin_fmaf(-lr, G[e], P[e]);      // (the fused update in the product's epilogue is the same fma)
}

// ---- 16-byte versions (width a multiple of 4, 16-byte aligned bases) -----------------------------
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Z[i][c..c+3] += b[c..c+3] (then ReLU): a thread keeps its four bias values and walks the rows of
// its row chunk, so there is no index division at all
__global__ __launch_bounds__(256) void bias_act_vec_kernel(float* __restrict__ Z, const float* __restrict__ b,
                                                           int batch, int width, int rows_per_block, int relu)
{
    const int c = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (c >= width) return;
    const f32x4 bias = *reinterpret_cast<const f32x4*>(b + c);
    const int r0 = blockIdx.y * rows_per_block;
    const int r1 = min(batch, r0 + rows_per_block);
#pragma unroll 4
    for (int i = r0; i < r1; ++i) {
        f32x4* z = reinterpret_cast<f32x4*>(Z + (size_t)i * width + c);
        f32x4 v = *z + bias;
        if (relu) {
            v.x = v.x > 0.f ? v.x : 0.f; v.y = v.y > 0.f ? v.y : 0.f;
            v.z = v.z > 0.f ? v.z : 0.f; v.w = v.w > 0.f ? v.w : 0.f;
        }
        *z = v;
    }
}

// Column sums of one row chunk into part[chunk][col].  A workgroup covers 256 columns (four per
// lane) and one chunk of rows; its four waves take every fourth row of the chunk and their sums
// are added in wave order, so the order of the additions is fixed.
// RELU: first pass dZ through the ReLU mask of H in place (dZ = H > 0 ? dZ : 0), so the gradient
// is read once for both steps.
template <bool RELU>
__global__ __launch_bounds__(256) void colsum_vec_kernel(float* __restrict__ dZ, const float* __restrict__ H,
                                                         float* __restrict__ part, int batch, int width, int rows_per_chunk)
{
    __shared__ f32x4 acc[4][64];
    const int lane = threadIdx.x & 63;
    const int sub = threadIdx.x >> 6;
    const int c = (blockIdx.x * 64 + lane) * 4;
    const int r0 = blockIdx.y * rows_per_chunk;
    const int r1 = min(batch, r0 + rows_per_chunk);
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    if (c < width) {
#pragma unroll 8
        for (int i = r0 + sub; i < r1; i += 4) {
            const size_t off = (size_t)i * width + c;
            f32x4 g = *reinterpret_cast<const f32x4*>(dZ + off);
            if (RELU) {
                const f32x4 h = *reinterpret_cast<const f32x4*>(H + off);
                g.x = h.x > 0.f ? g.x : 0.f; g.y = h.y > 0.f ? g.y : 0.f;
                g.z = h.z > 0.f ? g.z : 0.f; g.w = h.w > 0.f ? g.w : 0.f;
                *reinterpret_cast<f32x4*>(dZ + off) = g;
            }
            s += g;
        }
    }
    acc[sub][lane] = s;
    __syncthreads();
    if (sub == 0 && c < width)
        *reinterpret_cast<f32x4*>(part + (size_t)blockIdx.y * width + c) =
            (acc[0][lane] + acc[1][lane]) + (acc[2][lane] + acc[3][lane]);
}

// db[col] = sum over chunks of part[chunk][col]: 64 columns per workgroup, its four waves take a
// quarter of the chunks each (in order), then the four sums are added in wave order
// P (optional): the parameter the sums are the gradient of; it takes its SGD step here, P = fma(-lr, db, P)
__global__ __launch_bounds__(256) void colsum_final_kernel(const float* __restrict__ part, int chunks, int width,
                                                           float* __restrict__ db, float* __restrict__ P, float lr)
{
    __shared__ float acc[4][64];
    const int lane = threadIdx.x & 63;
    const int sub = threadIdx.x >> 6;
    const int col = blockIdx.x * 64 + lane;
    const int per = (chunks + 3) / 4;
    float s = 0.f;
    if (col < width)
        for (int ch = sub * per; ch < min(chunks, (sub + 1) * per); ++ch) s += part[(size_t)ch * width + col];
    acc[sub][lane] = s;
    __syncthreads();
    if (sub == 0 && col < width) {
        const float g = (acc[0][lane] + acc[1][lane]) + (acc[2][lane] + acc[3][lane]);
        db[col] = g;
        if (P) P[col] = __builtin_fmaf(-lr, g, P[col]);
    }
}

__global__ __launch_bounds__(256) void sgd_vec_kernel(float* __restrict__ P, const float* __restrict__ G, long long total4, float lr)
{
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < total4;
         e += (long long)gridDim.x * blockDim.x) {
        f32x4* p = reinterpret_cast<f32x4*>(P) + e;
        const f32x4 g = reinterpret_cast<const f32x4*>(G)[e];
        f32x4 v = *p;
        v.x = __builtin_fmaf(-lr, g.x, v.x); v.y = __builtin_fmaf(-lr, g.y, v.y);
        v.z = __builtin_fmaf(-lr, g.z, v.z); v.w = __builtin_fmaf(-lr, g.w, v.w);
        *p = v;
    }
}

// The same two passes for matrices whose rows are further apart than their width
__global__ __launch_bounds__(256) void bias_act_ld_kernel(float* __restrict__ Z, long ld, const float* __restrict__ b,
                                                          long long total, int width, int relu)
{
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (long long)gridDim.x * blockDim.x) {
        const long long i = e / width;
        const int j = (int)(e - i * width);
        float v = Z[(size_t)i * ld + j] + b[j];
        if (relu) v = v > 0.f ? v : 0.f;
        Z[(size_t)i * ld + j] = v;
    }
}

__global__ __launch_bounds__(256) void sgd_ld_kernel(float* __restrict__ P, long ldp, const float* __restrict__ G, long ldg,
                                                     long long total, int width, float lr)
{
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (long long)gridDim.x * blockDim.x) {
        const long long i = e / width;
        const int j = (int)(e - i * width);
        float* p = P + (size_t)i * ldp + j;
        *p = __builtin_fmaf(-lr, G[(size_t)i * ldg + j], *p);
    }
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

__global__ __launch_bounds__(256) void copy_words_kernel(const float* __restrict__ in, float* __restrict__ out, long long total)
{
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (long long)gridDim.x * blockDim.x)
        out[e] = in[e];
}

static unsigned blocks_for(long long total)
{
    long long b = (total + 255) / 256;
    return (unsigned)(b > 8192 ? 8192 : (b < 1 ? 1 : b));
}

// Z (rows x width, leading dimension ld) += b per column, then the clamp
int launch_bias_act(hipStream_t s, int rows, int width, float* Z, long ld, const float* b, int relu)
{
    if (ld == width) {
        const int st = mtnn_fc_bias_act(s, rows, width, Z, b, relu);
        return st == MTNN_OK ? 0 : (int)hipErrorLaunchFailure;
    }
    const long long total = (long long)rows * width;
    hipLaunchKernelGGL(bias_act_ld_kernel, dim3(blocks_for(total)), dim3(256), 0, s, Z, ld, b, total, width, relu);
    return (int)hipGetLastError();
}

// P (rows x width, leading dimension ldp) = fma(-lr, G, P)
int launch_sgd_2d(hipStream_t s, int rows, int width, float* P, long ldp, const float* G, long ldg, float lr)
{
    if (ldp == width && ldg == width) {
        const int st = mtnn_fc_sgd(s, (long long)rows * width, P, G, lr);
        return st == MTNN_OK ? 0 : (int)hipErrorLaunchFailure;
    }
    const long long total = (long long)rows * width;
    hipLaunchKernelGGL(sgd_ld_kernel, dim3(blocks_for(total)), dim3(256), 0, s, P, ldp, G, ldg, total, width, lr);
    return (int)hipGetLastError();
}

}  // namespace mtnn

namespace {
// (the elementwise kernels ask nothing of the device's geometry, so these entry points do not look it
// up; a launch refused for want of a device, or of code for it, reports that instead of a launch error)
int status_of(hipError_t e)
{
    if (e == hipSuccess) return MTNN_OK;
    if (e == hipErrorNoDevice || e == hipErrorInvalidDevice || e == hipErrorNoBinaryForGpu ||
        e == hipErrorInvalidDeviceFunction || e == hipErrorSharedObjectInitFailed)
        return MTNN_ERR_NO_DEVICE;
    return MTNN_ERR_LAUNCH;
}
size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
}  // namespace

extern "C" {

int mtnn_fc_bias_act(void* stream, int batch, int width, float* Z, const float* b, int relu)
{
    if (batch < 0 || width < 0) return MTNN_ERR_DIM;
    if (batch == 0 || width == 0) return MTNN_OK;
    if (!Z || !b) return MTNN_ERR_NULL;
    const long long total = (long long)batch * width;
    if (width % 4 == 0 && mtnn::aligned16(Z) && mtnn::aligned16(b)) {
        int rows_per_block = 4;
        if ((batch + rows_per_block - 1) / rows_per_block > 32768) rows_per_block = (batch + 32767) / 32768;
        const dim3 grid((width / 4 + 255) / 256, (batch + rows_per_block - 1) / rows_per_block);
        hipLaunchKernelGGL(mtnn::bias_act_vec_kernel, grid, dim3(256), 0, static_cast<hipStream_t>(stream),
                           Z, b, batch, width, rows_per_block, relu);
        return status_of(hipGetLastError());
    }
    hipLaunchKernelGGL(mtnn::bias_act_kernel, dim3(mtnn::blocks_for(total)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       Z, b, total, width, relu);
    return status_of(hipGetLastError());
}

int mtnn_fc_softmax_xent(void* stream, int batch, int classes, const float* logits, const int* labels,
                         float* dZ, float* row_loss, float* mean_loss)
{
    if (batch <= 0 || classes <= 0) return MTNN_ERR_DIM;
    if (!logits || !labels || !dZ || !row_loss || !mean_loss) return MTNN_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(mtnn::softmax_xent_kernel, dim3(batch), dim3(64), 0, s, logits, labels, dZ, row_loss, batch, classes);
    hipLaunchKernelGGL(mtnn::mean_kernel, dim3(1), dim3(256), 0, s, row_loss, batch, mean_loss);
    return status_of(hipGetLastError());
}

int mtnn_fc_relu_backward(void* stream, long long count, float* dH, const float* H)
{
    if (count < 0) return MTNN_ERR_DIM;
    if (count == 0) return MTNN_OK;
    if (!dH || !H) return MTNN_ERR_NULL;
    hipLaunchKernelGGL(mtnn::relu_backward_kernel, dim3(mtnn::blocks_for(count)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), dH, H, count);
    return status_of(hipGetLastError());
}

// Row chunks for the two-stage column sums: at most 32 (the scratch holds 32 x width), at least 32
// rows each (8 per wave).
static int colsum_chunks(int batch, int* rows_per_chunk)
{
    int chunks = batch / 32;
    if (chunks > 32) chunks = 32;
    if (chunks < 1) chunks = 1;
    *rows_per_chunk = (batch + chunks - 1) / chunks;
    return (batch + *rows_per_chunk - 1) / *rows_per_chunk;
}

// The column sums, and (P non-null) the SGD step of the bias they are the gradient of: in the same
// launch where the 16-byte path runs, as a separate small pass otherwise.
static int bias_grad_impl(void* stream, int batch, int width, const float* dZ, float* db, float* scratch, float* P, float lr)
{
    if (batch <= 0 || width <= 0) return MTNN_ERR_DIM;
    if (!dZ || !db) return MTNN_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (scratch && width % 4 == 0 && mtnn::aligned16(dZ) && mtnn::aligned16(scratch)) {
        int rows_per_chunk;
        const int chunks = colsum_chunks(batch, &rows_per_chunk);
        hipLaunchKernelGGL(mtnn::colsum_vec_kernel<false>, dim3((width / 4 + 63) / 64, chunks), dim3(256), 0, s,
                           const_cast<float*>(dZ), static_cast<const float*>(nullptr), scratch, batch, width, rows_per_chunk);
        hipLaunchKernelGGL(mtnn::colsum_final_kernel, dim3((width + 63) / 64), dim3(256), 0, s, scratch, chunks, width, db, P, lr);
        return status_of(hipGetLastError());
    }
    const int col_blocks = (width + 63) / 64;
    // enough row chunks to put ~512 workgroups on the machine, at most 32, at least 32 rows each
    int chunks = 512 / col_blocks;
    if (chunks > 32) chunks = 32;
    if (chunks > batch / 32) chunks = batch / 32;
    if (!scratch || chunks < 2) {
        hipLaunchKernelGGL(mtnn::bias_grad_kernel, dim3(col_blocks), dim3(256), 0, s, dZ, db, batch, width);
    } else {
        const int rows_per_chunk = (batch + chunks - 1) / chunks;
        chunks = (batch + rows_per_chunk - 1) / rows_per_chunk;
        hipLaunchKernelGGL(mtnn::bias_grad_partial_kernel, dim3(col_blocks, chunks), dim3(256), 0, s, dZ, scratch, batch,
                           width, rows_per_chunk);
        hipLaunchKernelGGL(mtnn::bias_grad_final_kernel, dim3((width + 255) / 256), dim3(256), 0, s, scratch, chunks, width, db);
    }
    const int st = status_of(hipGetLastError());
    if (st != MTNN_OK || !P) return st;
    return mtnn_fc_sgd(stream, width, P, db, lr);
}

int mtnn_fc_bias_grad(void* stream, int batch, int width, const float* dZ, float* db, float* scratch)
{
    return bias_grad_impl(stream, batch, width, dZ, db, scratch, nullptr, 0.f);
}

static int relu_backward_bias_grad_impl(void* stream, int batch, int width, float* dH, const float* H, float* db,
                                        float* scratch, float* P, float lr)
{
    if (batch <= 0 || width <= 0) return MTNN_ERR_DIM;
    if (!dH || !H || !db) return MTNN_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (scratch && width % 4 == 0 && mtnn::aligned16(dH) && mtnn::aligned16(H) && mtnn::aligned16(scratch)) {
        int rows_per_chunk;
        const int chunks = colsum_chunks(batch, &rows_per_chunk);
        hipLaunchKernelGGL(mtnn::colsum_vec_kernel<true>, dim3((width / 4 + 63) / 64, chunks), dim3(256), 0, s,
                           dH, H, scratch, batch, width, rows_per_chunk);
        hipLaunchKernelGGL(mtnn::colsum_final_kernel, dim3((width + 63) / 64), dim3(256), 0, s, scratch, chunks, width, db, P, lr);
        return status_of(hipGetLastError());
    }
    const int st = mtnn_fc_relu_backward(stream, (long long)batch * width, dH, H);
    if (st != MTNN_OK) return st;
    return bias_grad_impl(stream, batch, width, dH, db, scratch, P, lr);
}

int mtnn_fc_relu_backward_bias_grad(void* stream, int batch, int width, float* dH, const float* H, float* db, float* scratch)
{
    return relu_backward_bias_grad_impl(stream, batch, width, dH, H, db, scratch, nullptr, 0.f);
}

int mtnn_fc_sgd(void* stream, long long count, float* P, const float* G, float lr)
{
    if (count < 0) return MTNN_ERR_DIM;
    if (count == 0) return MTNN_OK;
    if (!P || !G) return MTNN_ERR_NULL;
    if (count % 4 == 0 && mtnn::aligned16(P) && mtnn::aligned16(G)) {
        hipLaunchKernelGGL(mtnn::sgd_vec_kernel, dim3(mtnn::blocks_for(count / 4)), dim3(256), 0,
                           static_cast<hipStream_t>(stream), P, G, count / 4, lr);
        return status_of(hipGetLastError());
    }
    hipLaunchKernelGGL(mtnn::sgd_kernel, dim3(mtnn::blocks_for(count)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       P, G, count, lr);
    return status_of(hipGetLastError());
}

// workspace layout (all blocks 256-byte aligned):
//   H_1 .. H_L        batch x dims[l]            activations (H_L = logits)
//   dA, dB            batch x max_width each     ping-pong gradients w.r.t. layer outputs / inputs
//   dZt               max_width x batch          transposed gradient for the dW product
//   Bt                max(out x in) floats       B^T buffer for the TNN forward path
//   row_loss          batch
//   bias_part         32 x max_width             row-chunk partial sums of the bias gradient
size_t mtnn_fc_workspace_bytes(int num_layers, const int* dims, int batch)
{
    if (num_layers <= 0 || !dims || batch <= 0) return 0;
    size_t total = 0, max_w = 0, max_wt = 0;
    for (int l = 0; l <= num_layers; ++l) {
        if (dims[l] <= 0) return 0;
        if ((size_t)dims[l] > max_w) max_w = (size_t)dims[l];
    }
    for (int l = 1; l <= num_layers; ++l) {
        total += align256((size_t)batch * dims[l] * 4);
        const size_t wt = (size_t)dims[l] * dims[l - 1];
        if (wt > max_wt) max_wt = wt;
    }
    total += 2 * align256((size_t)batch * max_w * 4);
    total += align256(max_w * (size_t)batch * 4);
    total += align256(max_wt * 4);
    total += align256((size_t)batch * 4);
    total += align256(32 * max_w * 4);
    return total;
}

static int fc_run(void* stream, const mtnn_fc_step_desc* d, bool forward_only)
{
    if (!d) return MTNN_ERR_NULL;
    const int L = d->num_layers;
    if (L <= 0 || L > 64 || d->batch <= 0 || !d->dims) return MTNN_ERR_DIM;
    for (int l = 0; l <= L; ++l)
        if (d->dims[l] <= 0) return MTNN_ERR_DIM;
    if (!d->X || !d->labels || !d->W || !d->b || !d->loss || !d->workspace) return MTNN_ERR_NULL;
    if (!forward_only && (!d->dW || !d->db)) return MTNN_ERR_NULL;
    for (int l = 0; l < L; ++l) {
        if (!d->W[l] || !d->b[l]) return MTNN_ERR_NULL;
        if (!forward_only && (!d->dW[l] || !d->db[l])) return MTNN_ERR_NULL;
    }
    if (d->forward_mode != 0 && d->forward_mode != 1 && d->forward_mode != -1) return MTNN_ERR_ARG;
    if (d->workspace_bytes < mtnn_fc_workspace_bytes(L, d->dims, d->batch)) return MTNN_ERR_WORKSPACE;

    const int batch = d->batch;
    const int* dims = d->dims;
    size_t max_w = 0, max_wt = 0;
    for (int l = 0; l <= L; ++l) if ((size_t)dims[l] > max_w) max_w = (size_t)dims[l];
    for (int l = 1; l <= L; ++l) {
        const size_t wt = (size_t)dims[l] * dims[l - 1];
        if (wt > max_wt) max_wt = wt;
    }
    char* base = static_cast<char*>(d->workspace);
    size_t off = 0;
    auto carve = [&](size_t bytes) { char* p = base + off; off += align256(bytes); return reinterpret_cast<float*>(p); };
    float* H[65];
    H[0] = const_cast<float*>(d->X);
    for (int l = 1; l <= L; ++l) H[l] = carve((size_t)batch * dims[l] * 4);
    float* dA = carve((size_t)batch * max_w * 4);
    float* dB = carve((size_t)batch * max_w * 4);
    float* dZt = carve(max_w * (size_t)batch * 4);
    float* Bt = carve(max_wt * 4);
    float* row_loss = carve((size_t)batch * 4);
    float* bias_part = carve(32 * max_w * 4);
    const size_t bt_bytes = align256(max_wt * 4);

    int st;
    // forward: H_l = act(H_{l-1} x W_l^T + b_l) -- the NT operation of each layer
    for (int l = 0; l < L; ++l) {
        const int in = dims[l], out = dims[l + 1];
        // (bias and ReLU in the product's epilogue)
        st = mtnn_fc_layer_forward(stream, d->forward_mode, batch, out, in, H[l], in, d->W[l], in, d->b[l],
                                   l < L - 1 ? 1 : 0, H[l + 1], out, Bt, bt_bytes, nullptr);
        if (st != MTNN_OK) return st;
    }
    if (d->logits) {
        st = mtnn_copy_rows(stream, batch, dims[L], H[L], d->logits);
        if (st != MTNN_OK) return st;
    }
    // loss and gradient w.r.t. the logits
    float* dZ = dA;
    float* dNext = dB;
    st = mtnn_fc_softmax_xent(stream, batch, dims[L], H[L], d->labels, dZ, row_loss, d->loss);
    if (st != MTNN_OK) return st;
    if (forward_only) return MTNN_OK;
    // backward, last layer first
    for (int l = L - 1; l >= 0; --l) {
        const int in = dims[l], out = dims[l + 1];
        if (l == L - 1) {                      // below, db comes with the ReLU mask of the layer above
            st = bias_grad_impl(stream, batch, out, dZ, d->db[l], bias_part, d->b[l], d->lr);   // (and b_l takes its step)
            if (st != MTNN_OK) return st;
        }
        if (l > 0) {
            // dH_l = dZ x W_l (NN, with the weights before their update), then through the ReLU
            st = mtnn_nn(stream, batch, in, out, dZ, out, d->W[l], in, dNext, in);
            if (st != MTNN_OK) return st;
            // ... which gives dZ_{l-1}; its column sums are db_{l-1}, taken in the same pass, and
            // b_{l-1}, which the backward pass does not read, takes its step there too
            st = relu_backward_bias_grad_impl(stream, batch, in, dNext, H[l], d->db[l - 1], bias_part, d->b[l - 1], d->lr);
            if (st != MTNN_OK) return st;
        }
        // dW_l = dZ^T x H_l : transpose dZ (batch x out -> out x batch), then an NN product whose
        // epilogue also takes the step of W_l (after the product above has read the old weights)
        st = mtnn_transpose(stream, batch, out, dZ, out, dZt, batch);
        if (st != MTNN_OK) return st;
        st = mtnn_fc_weight_grad_sgd(stream, out, in, batch, dZt, batch, H[l], in, d->dW[l], in, d->W[l], in, d->lr);
        if (st != MTNN_OK) return st;
        float* t = dZ; dZ = dNext; dNext = t;
    }
    return MTNN_OK;
}

int mtnn_fc_train_step(void* stream, const mtnn_fc_step_desc* d) { return fc_run(stream, d, false); }

int mtnn_fc_forward(void* stream, const mtnn_fc_step_desc* d) { return fc_run(stream, d, true); }

int mtnn_copy_rows(void* stream, int rows, int cols, const float* in, float* out)
{
    if (rows < 0 || cols < 0) return MTNN_ERR_DIM;
    if (rows == 0 || cols == 0) return MTNN_OK;
    if (!in || !out) return MTNN_ERR_NULL;
    // a kernel rather than a runtime copy, so that a caller capturing the step into a HIP graph gets
    // kernel nodes only
    const long long total = (long long)rows * cols;
    hipLaunchKernelGGL(mtnn::copy_words_kernel, dim3(mtnn::blocks_for(total)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), in, out, total);
    return status_of(hipGetLastError());
}

}  // extern "C"

// Out-of-place transpose of 32-bit words for gfx950: out[c][r] = in[r][c]
// (Section III of the MTNN paper; the "transposeOnGPU" step of Algorithm 1).
//
// The operation is pure data movement, so the design is about HBM: every global access is a
// full-width coalesced row segment on both sides, and the row/column exchange happens in LDS.
// A workgroup of 256 threads moves one TS x TS tile (TS = 64):
//   read   16 lanes x 16 B cover one 256 B row segment, 4 rows per wave instruction;
//   LDS    tile[TS][TS+1]: the odd row stride puts the 4 words a lane writes, and the 4 words
//          it later gathers down a column, in distinct banks across the wave;
//   write  each lane gathers 4 words of one tile column and stores them as 16 B of an output row.
// Words are moved as integers, so NaN payloads and signed zeros survive bit for bit.
// Edge tiles, leading dimensions that are not multiples of 4 and unaligned bases take the
// guarded one-word-per-access path of the same kernel.
#include "mtnn_internal.h"

namespace mtnn {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int TS = 64;          // tile edge in words
constexpr int TP = TS + 1;      // padded LDS row stride
constexpr int TR_THREADS = 256;

template <bool VEC>
__global__ __launch_bounds__(TR_THREADS) void transpose_kernel(
    const uint32_t* __restrict__ in, uint32_t* __restrict__ out,
    int rows, int cols, long ldin, long ldout, int tiles_c)
{
    __shared__ uint32_t tile[TS * TP];
    const int t = threadIdx.x;
    // consecutive workgroups walk along an input row, so the reads of neighbouring workgroups
    // are neighbouring 256 B segments
    const int tc = blockIdx.x % tiles_c;
    const int tr = blockIdx.x / tiles_c;
    const int r0 = tr * TS;
    const int c0 = tc * TS;
    const bool full = (r0 + TS <= rows) && (c0 + TS <= cols);
    const int q = t & 15;        // which 4-word group of a 64-word row
    const int rr = t >> 4;       // row within a pass of 16 rows

    if (VEC && full) {
        u32x4 v[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int r = p * 16 + rr;
            v[p] = *reinterpret_cast<const u32x4*>(in + (size_t)(r0 + r) * ldin + c0 + q * 4);
        }
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int r = p * 16 + rr;
            uint32_t* dst = tile + r * TP + q * 4;
            dst[0] = v[p].x; dst[1] = v[p].y; dst[2] = v[p].z; dst[3] = v[p].w;
        }
        __syncthreads();
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int c = p * 16 + rr;                 // tile column = output row
            const uint32_t* src = tile + (q * 4) * TP + c;
            u32x4 w;
            w.x = src[0]; w.y = src[TP]; w.z = src[2 * TP]; w.w = src[3 * TP];
            *reinterpret_cast<u32x4*>(out + (size_t)(c0 + c) * ldout + r0 + q * 4) = w;
        }
    } else {
        // guarded path: one word per access, still row-coalesced on both sides
        const int lane_c = t & 63;
        const int rbase = t >> 6;                      // 0..3
        for (int r = rbase; r < TS; r += 4) {
            if (r0 + r < rows && c0 + lane_c < cols)
                tile[r * TP + lane_c] = in[(size_t)(r0 + r) * ldin + c0 + lane_c];
        }
        __syncthreads();
        for (int c = rbase; c < TS; c += 4) {
            if (c0 + c < cols && r0 + lane_c < rows)
                out[(size_t)(c0 + c) * ldout + r0 + lane_c] = tile[lane_c * TP + c];
        }
    }
}

int launch_transpose(hipStream_t s, int rows, int cols, const float* in, long ldin, float* out, long ldout)
{
    const int tiles_c = (cols + TS - 1) / TS;
    const int tiles_r = (rows + TS - 1) / TS;
    const long long nblocks = (long long)tiles_c * tiles_r;
    if (nblocks <= 0) return 0;
    if (nblocks > 0x7fffffffLL) return (int)hipErrorInvalidValue;
    const bool vec = (ldin % 4 == 0) && (ldout % 4 == 0) &&
                     ((reinterpret_cast<uintptr_t>(in) & 15) == 0) &&
                     ((reinterpret_cast<uintptr_t>(out) & 15) == 0);
    const uint32_t* pin = reinterpret_cast<const uint32_t*>(in);
    uint32_t* pout = reinterpret_cast<uint32_t*>(out);
    if (vec)
        hipLaunchKernelGGL(transpose_kernel<true>, dim3((unsigned)nblocks), dim3(TR_THREADS), 0, s,
                           pin, pout, rows, cols, ldin, ldout, tiles_c);
    else
        hipLaunchKernelGGL(transpose_kernel<false>, dim3((unsigned)nblocks), dim3(TR_THREADS), 0, s,
                           pin, pout, rows, cols, ldin, ldout, tiles_c);
    return (int)hipGetLastError();
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float* __restrict__ C, int m, int n, long ldc)
{
    const long long total = (long long)m * n;
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (long long)gridDim.x * blockDim.x) {
        const long long i = e / n;
        const long long j = e - i * n;
        C[(size_t)i * ldc + j] = 0.0f;
    }
}

int launch_fill_zero(hipStream_t s, int m, int n, float* C, long ldc)
{
    const long long total = (long long)m * n;
    if (total <= 0) return 0;
    long long blocks = (total + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, s, C, m, n, ldc);
    return (int)hipGetLastError();
}

// Plain streaming copy of 16-byte words: the reference point for HBM counters and for what a
// pure read-once/write-once kernel reaches on this machine (not part of the paper's method).
__global__ __launch_bounds__(256) void copy_kernel(const u32x4* __restrict__ in, u32x4* __restrict__ out, size_t nvec)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += stride) out[i] = in[i];
}

int launch_copy(hipStream_t s, size_t nvec, const void* in, void* out)
{
    if (nvec == 0) return 0;
    size_t blocks = (nvec + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, s,
                       static_cast<const u32x4*>(in), static_cast<u32x4*>(out), nvec);
    return (int)hipGetLastError();
}

}  // namespace mtnn

// Out-of-place transpose of 32-bit words for gfx950: out[c][r] = in[r][c]
// (Section III of the MTNN paper; the "transposeOnGPU" step of Algorithm 1).
//
// The operation is pure data movement, so the design is about HBM.  A 256-thread workgroup moves a
// tile of TR input rows x TC input columns (TR = 128 or 256, TC = 32):
//   read   a tile row is 128 bytes, one full cache line: 8 lanes x 16 B, 32 rows per pass;
//   LDS    tile[TR][TC+1] words; the odd row stride spreads the column gather over the banks;
//   write  an output row segment is TR words (512 B or 1 KB): each lane gathers 4 words of one
//          tile column from LDS and stores 16 B, with non-temporal stores so that the stream of
//          results does not evict the input from the caches;
//   order  consecutive workgroups walk DOWN the input (tile-row index fastest), so their writes
//          are neighbouring segments of the same output rows.  Measured on MI355X, long contiguous
//          write runs matter more than contiguous reads: this order with the tall, narrow tile
//          moves 5.1-6.8 TB/s where a square 64 x 64 tile in row order moved 4.0-5.2 TB/s.
// Words are moved as integers, so NaN payloads and signed zeros survive bit for bit.
// Sizes or leading dimensions that are not multiples of 4 and unaligned bases take the guarded
// one-word-per-access path of the same kernel; otherwise edge tiles only skip the 16-byte groups
// that fall outside.
#include "mtnn_internal.h"

namespace mtnn {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int TC = 32;          // tile columns (input) = output rows per tile
constexpr int TP = TC + 1;      // padded LDS row stride
constexpr int TR_THREADS = 256;

// the 16-byte-group path of one tile; GUARD: skip the groups that fall outside the matrix (edge tiles)
template <int TR, bool GUARD>
__device__ __forceinline__ void transpose_tile_vec(const uint32_t* __restrict__ in, uint32_t* __restrict__ out,
                                                   uint32_t* tile, int rows, int cols, long ldin, long ldout,
                                                   int r0, int c0)
{
    const int t = threadIdx.x;
    constexpr int QC = TC / 4;               // 16-byte groups per tile row (8)
    constexpr int RP = TR_THREADS / QC;      // rows per pass (32)
    const int q = t % QC;
    const int rr = t / QC;
    u32x4 v[TR / RP] = {};
#pragma unroll
    for (int p = 0; p < TR / RP; ++p) {
        const int r = r0 + p * RP + rr;
        if (!GUARD || (r < rows && c0 + q * 4 < cols))
            v[p] = *reinterpret_cast<const u32x4*>(in + (size_t)r * ldin + c0 + q * 4);
    }
#pragma unroll
    for (int p = 0; p < TR / RP; ++p) {
        uint32_t* dst = tile + (p * RP + rr) * TP + q * 4;
        dst[0] = v[p].x; dst[1] = v[p].y; dst[2] = v[p].z; dst[3] = v[p].w;
    }
    __syncthreads();
    constexpr int QR = TR / 4;               // 16-byte groups per output row segment
    constexpr int CP = TR_THREADS / QR;      // output rows per pass
    const int oq = t % QR;
    const int oc = t / QR;
#pragma unroll
    for (int p = 0; p < TC / CP; ++p) {
        const int c = p * CP + oc;           // tile column = output row
        const uint32_t* src = tile + (oq * 4) * TP + c;
        u32x4 w;
        w.x = src[0]; w.y = src[TP]; w.z = src[2 * TP]; w.w = src[3 * TP];
        if (!GUARD || (c0 + c < cols && r0 + oq * 4 < rows))
            __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(out + (size_t)(c0 + c) * ldout + r0 + oq * 4));
    }
}

template <int TR, bool VEC>
__global__ __launch_bounds__(TR_THREADS) void transpose_kernel(
    const uint32_t* __restrict__ in, uint32_t* __restrict__ out,
    int rows, int cols, long ldin, long ldout, int tiles_r)
{
    __shared__ uint32_t tile[TR * TP];
    const int t = threadIdx.x;
    const int tr = blockIdx.x % tiles_r;
    const int tc = blockIdx.x / tiles_r;
    const int r0 = tr * TR;
    const int c0 = tc * TC;

    // VEC: 16-byte aligned rows on both sides and rows, cols multiples of 4, so every 16-byte group
    // is entirely inside or entirely outside the matrix
    if (VEC) {
        if ((r0 + TR <= rows) && (c0 + TC <= cols))
            transpose_tile_vec<TR, false>(in, out, tile, rows, cols, ldin, ldout, r0, c0);
        else
            transpose_tile_vec<TR, true>(in, out, tile, rows, cols, ldin, ldout, r0, c0);
    } else {
        // guarded path: one word per access, still row-coalesced on both sides
        const int lane_c = t % TC;
        const int rbase = t / TC;                        // 0 .. 7
        for (int r = rbase; r < TR; r += TR_THREADS / TC) {
            if (r0 + r < rows && c0 + lane_c < cols)
                tile[r * TP + lane_c] = in[(size_t)(r0 + r) * ldin + c0 + lane_c];
        }
        __syncthreads();
        for (int e = t; e < TR * TC; e += TR_THREADS) {
            const int c = e / TR;                        // output row within the tile
            const int r = e % TR;                        // consecutive threads -> consecutive output words
            if (c0 + c < cols && r0 + r < rows)
                out[(size_t)(c0 + c) * ldout + r0 + r] = tile[r * TP + c];
        }
    }
}

template <int TR>
static int launch_transpose_t(hipStream_t s, int rows, int cols, const uint32_t* in, long ldin,
                              uint32_t* out, long ldout, bool vec)
{
    const int tiles_c = (cols + TC - 1) / TC;
    const int tiles_r = (rows + TR - 1) / TR;
    const long long nblocks = (long long)tiles_c * tiles_r;
    if (nblocks > 0x7fffffffLL) return (int)hipErrorInvalidValue;
    if (vec)
        hipLaunchKernelGGL((transpose_kernel<TR, true>), dim3((unsigned)nblocks), dim3(TR_THREADS), 0, s,
                           in, out, rows, cols, ldin, ldout, tiles_r);
    else
        hipLaunchKernelGGL((transpose_kernel<TR, false>), dim3((unsigned)nblocks), dim3(TR_THREADS), 0, s,
                           in, out, rows, cols, ldin, ldout, tiles_r);
    return (int)hipGetLastError();
}

int launch_transpose(hipStream_t s, int rows, int cols, const float* in, long ldin, float* out, long ldout)
{
    if (rows <= 0 || cols <= 0) return 0;
    const bool vec = (ldin % 4 == 0) && (ldout % 4 == 0) && (rows % 4 == 0) && (cols % 4 == 0) &&
                     ((reinterpret_cast<uintptr_t>(in) & 15) == 0) &&
                     ((reinterpret_cast<uintptr_t>(out) & 15) == 0);
    const uint32_t* pin = reinterpret_cast<const uint32_t*>(in);
    uint32_t* pout = reinterpret_cast<uint32_t*>(out);
    // the taller tile (1 KB write runs) pays off once the matrix is far larger than the caches
    if ((long long)rows * cols >= (1LL << 27) && rows >= 256)
        return launch_transpose_t<256>(s, rows, cols, pin, ldin, pout, ldout, vec);
    return launch_transpose_t<128>(s, rows, cols, pin, ldin, pout, ldout, vec);
}

// ---- in-place transpose of a square matrix -------------------------------------------------------
//
// The paper's TNN needs extra memory for B^T and names in-place transposition as future work for
// the case where that memory is missing (Section III, Section VI).  For a square matrix the
// in-place problem decomposes into independent swaps: the workgroup for tile pair (ti <= tj) loads
// tile (ti, tj) and tile (tj, ti) into LDS and writes each one transposed into the other's place
// (a diagonal tile is transposed onto itself).  Every element is read and written exactly once by
// exactly one workgroup, so there are no hazards between workgroups.  64 x 64 tiles, 256 threads.
constexpr int IT = 64;
constexpr int ITP = IT + 1;

__global__ __launch_bounds__(256) void transpose_inplace_kernel(uint32_t* __restrict__ X, int n, long ld)
{
    const int ti = blockIdx.y, tj = blockIdx.x;
    if (ti > tj) return;
    __shared__ uint32_t ta[IT * ITP];     // tile (ti, tj)
    __shared__ uint32_t tb[IT * ITP];     // tile (tj, ti)
    const int t = threadIdx.x;
    const int lane_c = t & 63;
    const int rbase = t >> 6;
    const int r0 = ti * IT, c0 = tj * IT;
    for (int r = rbase; r < IT; r += 4) {
        if (r0 + r < n && c0 + lane_c < n) ta[r * ITP + lane_c] = X[(size_t)(r0 + r) * ld + c0 + lane_c];
        if (ti != tj && c0 + r < n && r0 + lane_c < n) tb[r * ITP + lane_c] = X[(size_t)(c0 + r) * ld + r0 + lane_c];
    }
    __syncthreads();
    for (int r = rbase; r < IT; r += 4) {
        // row r of the tile at (tj, ti) receives column r of tile (ti, tj), and vice versa
        if (c0 + r < n && r0 + lane_c < n) X[(size_t)(c0 + r) * ld + r0 + lane_c] = ta[lane_c * ITP + r];
        if (ti != tj && r0 + r < n && c0 + lane_c < n) X[(size_t)(r0 + r) * ld + c0 + lane_c] = tb[lane_c * ITP + r];
    }
}

int launch_transpose_inplace(hipStream_t s, int n, float* X, long ld)
{
    if (n <= 0) return 0;
    const int nt = (n + IT - 1) / IT;
    if (nt > 65535) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(transpose_inplace_kernel, dim3(nt, nt), dim3(256), 0, s, reinterpret_cast<uint32_t*>(X), n, ld);
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

// Plain streaming copy of 16-byte words (non-temporal stores, like the transpose): the reference point for HBM counters and for what a
// pure read-once/write-once kernel reaches on this machine (not part of the paper's method).
__global__ __launch_bounds__(256) void copy_kernel(const u32x4* __restrict__ in, u32x4* __restrict__ out, size_t nvec)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += stride)
        __builtin_nontemporal_store(in[i], out + i);
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

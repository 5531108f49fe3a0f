// Out-of-place transpose of 32-bit words for gfx950: out[c][r] = in[r][c]
// (Section III of the MTNN paper; the "transposeOnGPU" step of Algorithm 1).
//
// The operation is pure data movement, so the design is about HBM.  A 256-thread workgroup moves a
// tile of TR input rows x TC input columns:
//   read   a tile row is TC words (128 or 256 bytes, whole cache lines), 16 bytes per lane;
//   LDS    tile[TR][TC] words with the columns of each row XOR-swizzled, which spreads the row-wise
//          stores and the column gather over the banks;
//   write  an output row segment is TR words (512 B or 1 KB): each lane gathers 4 words of one
//          tile column from LDS and stores 16 B, with non-temporal stores so that the stream of
//          results does not evict the input from the caches;
//   order  workgroup i takes tile row i mod tiles_r and tile column (i / tiles_r + tile row) mod
//          tiles_c: a diagonal walk.  Workgroups that run at the same time then read different
//          column strips and write different output row blocks, which spreads both streams over
//          the memory channels (walking straight down one column strip keeps every concurrent
//          read 128 bytes wide at one row pitch: measured 5.2 TB/s against 6.0 TB/s for the
//          diagonal walk on an 8192 x 8192 matrix that comes from HBM).
// Three tile shapes, chosen by size (measured on MI355X, see launch_transpose):
//   128 x 32, ordinary loads      matrices up to 2^24 elements: source and result together fit the
//                                 256 MB memory-side cache, where they usually still are when the
//                                 transpose follows the kernel that produced its input;
//   128 x 64, non-temporal loads  between 2^24 and 2^26 elements;
//   256 x 64, non-temporal loads  from 2^26 elements: data streams from and to HBM, 1 KB write runs.
// Words are moved as integers, so NaN payloads and signed zeros survive bit for bit.
// Rows that are not 16-byte aligned (odd leading dimensions, unaligned bases) take the same path
// with the 16-byte accesses made at 4-byte alignment; groups of four that lie across the matrix
// edge are moved word by word.
#include "mtnn_internal.h"

#include <atomic>

namespace mtnn {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int TR_THREADS = 256;

// LDS layout of the 16-byte-group path: tile[row][col ^ swz(row)], rows of TC words with no padding.
// The XOR spreads both phases over the banks (64 banks of 4 bytes; reasoning per pass of 32 lanes).
// Measured SQ_LDS_BANK_CONFLICT per 128 x 32 tile: 384 cycles with a padded [TR][TC+1] tile, 128 with
// this layout; a variant laid out for 64 lanes per pass measured 256, so this is the one kept:
//   store phase  a pass holds 4 or 8 consecutive rows x all 16-byte groups of a row; the low two
//                bits of swz differ between the rows that share a bank half;
//   gather phase lane i reads rows 4 i + e (e = 0..3 in turn) of one column; swz(4 i + e) is a
//                bijection of i for fixed e, so the lanes spread over all banks.
template <int TC>
__device__ __forceinline__ int swz(int row)
{
    if (TC == 64) return ((row >> 2) ^ (row & 3)) & 63;
    return ((row >> 2) ^ ((row >> 1) & 3)) & 31;          // TC == 32: row parity picks the bank half
}

// One tile.  A16: rows of both matrices are 16-byte aligned (aligned bases, leading dimensions
// multiples of 4); otherwise the same 16-byte accesses are made at 4-byte alignment, which gfx950
// allows for global memory.  GUARD (edge tiles): a group of four that lies across the matrix edge
// is moved word by word, one that lies outside is skipped.
template <int TR, int TC, bool NTL, bool GUARD, bool A16, bool STREAM>
__device__ __forceinline__ void transpose_tile_vec(const uint32_t* __restrict__ in, uint32_t* __restrict__ out,
                                                   uint32_t* tile, int rows, int cols, long ldin, long ldout,
                                                   int r0, int c0)
{
    static_assert(TC == 32 || TC == 64, "swz() knows these two widths");
    typedef uint32_t u32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));
    const int t = threadIdx.x;
    constexpr int QC = TC / 4;               // 16-byte groups per tile row
    constexpr int RP = TR_THREADS / QC;      // rows per pass
    const int q = t % QC;
    const int rr = t / QC;
    u32x4 v[TR / RP] = {};
#pragma unroll
    for (int p = 0; p < TR / RP; ++p) {
        const int r = r0 + p * RP + rr;
        const int cg = c0 + q * 4;
        const uint32_t* src = in + (size_t)r * ldin + cg;
        if (!GUARD || (r < rows && cg + 3 < cols)) {
            if (A16) v[p] = NTL ? __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src))
                                : *reinterpret_cast<const u32x4*>(src);
            else v[p] = *reinterpret_cast<const u32x4_a4*>(src);
        } else if (r < rows && cg < cols) {
            v[p].x = src[0];
            if (cg + 1 < cols) v[p].y = src[1];
            if (cg + 2 < cols) v[p].z = src[2];
        }
    }
#pragma unroll
    for (int p = 0; p < TR / RP; ++p) {
        const int row = p * RP + rr;
        const int x = swz<TC>(row);
        uint32_t* dst = tile + row * TC;
        dst[(q * 4 + 0) ^ x] = v[p].x; dst[(q * 4 + 1) ^ x] = v[p].y;
        dst[(q * 4 + 2) ^ x] = v[p].z; dst[(q * 4 + 3) ^ x] = v[p].w;
    }
    __syncthreads();
    constexpr int QR = TR / 4;               // 16-byte groups per output row segment
    constexpr int CP = TR_THREADS / QR;      // output rows per pass
    const int oq = t % QR;
    const int oc = t / QR;
#pragma unroll
    for (int p = 0; p < TC / CP; ++p) {
        const int c = p * CP + oc;           // tile column = output row
        const uint32_t* src = tile + (oq * 4) * TC;
        u32x4 w;
        w.x = src[c ^ swz<TC>(oq * 4)];
        w.y = src[TC + (c ^ swz<TC>(oq * 4 + 1))];
        w.z = src[2 * TC + (c ^ swz<TC>(oq * 4 + 2))];
        w.w = src[3 * TC + (c ^ swz<TC>(oq * 4 + 3))];
        const int orow = c0 + c;
        const int og = r0 + oq * 4;
        uint32_t* dst = out + (size_t)orow * ldout + og;
        if (!GUARD || (orow < cols && og + 3 < rows)) {
            if (A16 && STREAM) __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(dst));
            else if (A16) *reinterpret_cast<u32x4*>(dst) = w;
            else *reinterpret_cast<u32x4_a4*>(dst) = w;
        } else if (orow < cols && og < rows) {
            dst[0] = w.x;
            if (og + 1 < rows) dst[1] = w.y;
            if (og + 2 < rows) dst[2] = w.z;
        }
    }
}

// xcds > 1 (launches of 2^21 to 3 x 2^22 words whose output rows do not start on cache lines): workgroup ids, which the hardware
// deals round robin to the XCDs, are renumbered so that each XCD works on one contiguous run of the
// tile order (the first xcd_tall XCDs take xcd_per tiles, the others one fewer).  Tiles that are
// neighbours in the matrix then mostly run on the same XCD, and the cache lines two tiles share at
// their common edge -- input row pieces and output row segments both end inside lines there -- meet
// in that XCD's L2 instead of being fetched twice and written back as two partial lines.
template <int TR, int TC, bool VEC, bool NTL, bool STREAM>
__global__ __launch_bounds__(TR_THREADS) void transpose_kernel(
    const uint32_t* __restrict__ in, uint32_t* __restrict__ out,
    int rows, int cols, long ldin, long ldout, int tiles_r, int tiles_c, int xcds, int xcd_per, int xcd_tall)
{
    extern __shared__ uint32_t tile[];                   // TR * TC words
    int pid = (int)blockIdx.x;
    if (xcds > 1) {
        const int local = pid / xcds;
        const int x = pid - local * xcds;
        pid = (x < xcd_tall) ? x * xcd_per + local : xcd_tall * xcd_per + (x - xcd_tall) * (xcd_per - 1) + local;
    }
    const int tr = pid % tiles_r;
    const int tc = (pid / tiles_r + tr) % tiles_c;          // for each tile row a rotation of the columns
    const int r0 = tr * TR;
    const int c0 = tc * TC;
    // VEC: 16-byte aligned rows on both sides
    if ((r0 + TR <= rows) && (c0 + TC <= cols))
        transpose_tile_vec<TR, TC, NTL, false, VEC, STREAM>(in, out, tile, rows, cols, ldin, ldout, r0, c0);
    else
        transpose_tile_vec<TR, TC, NTL, true, VEC, STREAM>(in, out, tile, rows, cols, ldin, ldout, r0, c0);
}

template <int TR, int TC, bool VEC, bool NTL, bool STREAM>
static int launch_transpose_t(hipStream_t s, int rows, int cols, const uint32_t* in, long ldin,
                              uint32_t* out, long ldout)
{
    const int tiles_c = (cols + TC - 1) / TC;
    const int tiles_r = (rows + TR - 1) / TR;
    const long long nblocks = (long long)tiles_c * tiles_r;
    if (nblocks > 0x7fffffffLL) return (int)hipErrorInvalidValue;
    constexpr size_t lds = (size_t)TR * TC * sizeof(uint32_t);
    auto kern = transpose_kernel<TR, TC, VEC, NTL, STREAM>;
    if (lds > 64 * 1024) {
        // opt in to the large LDS carve-out once per device
        static std::atomic<bool> raised[16] = {};
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess) return (int)hipGetLastError();
        if (dev < 0 || dev >= 16 || !raised[dev]) {
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return (int)e;
            if (dev >= 0 && dev < 16) raised[dev] = true;
        }
    }
    int xcds = 1, xcd_per = 0, xcd_tall = 0;
    // (only up to 3 x 2^22 words: measured from the caches 4500 x 1500 11.1 -> 9.6 us, 2500 x 3300 13.3 -> 11.4,
    // 2743 x 3061 13.8 -> 11.8, from HBM 16.6 -> 15.2 / 19.4 -> 18.2 / 20.2 -> 18.8; beyond that the XCDs each
    // streaming a region of their own lose more in memory than the shared lines gain: 8200^2 from HBM 123 -> 144 us)
    // (and from 2^21 words: a grid of a few hundred tiles is one partial round either way, and 1000^2 measured
    // 3.4 -> 3.7 us with the renumbering)
    if (!STREAM && (long long)rows * cols <= (3LL << 22) && (long long)rows * cols >= (1LL << 21)) {
        Geometry geo;
        if (current_geometry(&geo) && geo.xcds > 1 && nblocks >= geo.xcds) {
            xcds = geo.xcds;
            xcd_per = (int)((nblocks + xcds - 1) / xcds);
            xcd_tall = (int)(nblocks - (long long)(xcd_per - 1) * xcds);
        }
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)nblocks), dim3(TR_THREADS), lds, s,
                       in, out, rows, cols, ldin, ldout, tiles_r, tiles_c, xcds, xcd_per, xcd_tall);
    return (int)hipGetLastError();
}

int launch_transpose(hipStream_t s, int rows, int cols, const float* in, long ldin, float* out, long ldout)
{
    if (rows <= 0 || cols <= 0) return 0;
    const bool vec = (ldin % 4 == 0) && (ldout % 4 == 0) &&
                     ((reinterpret_cast<uintptr_t>(in) & 15) == 0) &&
                     ((reinterpret_cast<uintptr_t>(out) & 15) == 0);
    const uint32_t* pin = reinterpret_cast<const uint32_t*>(in);
    uint32_t* pout = reinterpret_cast<uint32_t*>(out);
    const long long elems = (long long)rows * cols;
    // Results are written past the caches only when every output row segment (TR words at a multiple of
    // TR words within its row) is whole 128-byte lines, i.e. the rows of `out` start on lines.  Otherwise
    // a segment shares its end lines with the neighbouring tiles' segments, and ordinary stores let the
    // pieces meet in L2 instead of each going to memory as a partial line (4500 x 1500, whose output
    // rows are 18000 bytes: 14.5 us streamed).
    const bool whole_lines = vec && (ldout % 32 == 0) && ((reinterpret_cast<uintptr_t>(out) & 127) == 0);
#define MTNN_TRANSPOSE(TR, TC, NTL)                                                                                   \
    (vec ? (whole_lines ? launch_transpose_t<TR, TC, true, NTL, true>(s, rows, cols, pin, ldin, pout, ldout)            \
                        : launch_transpose_t<TR, TC, true, NTL, false>(s, rows, cols, pin, ldin, pout, ldout))          \
         : launch_transpose_t<TR, TC, false, NTL, false>(s, rows, cols, pin, ldin, pout, ldout))
    if (elems >= (1LL << 26) && rows >= 256 && cols >= 64) return MTNN_TRANSPOSE(256, 64, true);
    if (elems > (1LL << 24) && cols >= 64) return MTNN_TRANSPOSE(128, 64, true);
    // Output rows that do not start on lines, a few million words: the 128 x 64 tile (input row pieces of
    // 256 bytes, so three lines touched per piece instead of two per 128 bytes) measures ahead of
    // 128 x 32 from the caches (4100^2 26.0 -> 22.5 us, 4097 x 4095 27.2 -> 24.0, 4500 x 1500 12.4 -> 11.1,
    // 2500 x 3300 14.8 -> 13.3) and level with it from HBM; aligned shapes of this size keep 128 x 32
    // (4096 x 1024 from the caches 4.7 us against 5.2).
    if (!whole_lines && elems >= (1LL << 22) && cols >= 64) return MTNN_TRANSPOSE(128, 64, false);
    return MTNN_TRANSPOSE(128, 32, false);
#undef MTNN_TRANSPOSE
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

// 16-byte-group helpers of the in-place kernel: a 64 x 64 tile at (r0, c0) to LDS, and the transposed
// LDS tile to the 64 x 64 region at (r0, c0); groups outside the n x n matrix are skipped.
template <bool NTL>
__device__ __forceinline__ void inplace_load_tile(const uint32_t* __restrict__ X, long ld, int n, int r0, int c0,
                                                  u32x4 (&v)[4])
{
    const int t = threadIdx.x;
    const int q = t & 15, rr = t >> 4;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int r = r0 + p * 16 + rr;
        v[p] = u32x4{0u, 0u, 0u, 0u};
        if (r < n && c0 + q * 4 < n) {
            const u32x4* src = reinterpret_cast<const u32x4*>(X + (size_t)r * ld + c0 + q * 4);
            v[p] = NTL ? __builtin_nontemporal_load(src) : *src;
        }
    }
}

__device__ __forceinline__ void inplace_stash_tile(uint32_t* tile, const u32x4 (&v)[4])
{
    const int t = threadIdx.x;
    const int q = t & 15, rr = t >> 4;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        uint32_t* dst = tile + (p * 16 + rr) * ITP + q * 4;
        dst[0] = v[p].x; dst[1] = v[p].y; dst[2] = v[p].z; dst[3] = v[p].w;
    }
}

// region (r0, c0) <- transpose of the LDS tile: row r of the region is column r of the tile
__device__ __forceinline__ void inplace_store_transposed(uint32_t* __restrict__ X, long ld, int n, int r0, int c0,
                                                         const uint32_t* tile)
{
    const int t = threadIdx.x;
    const int q = t & 15, rr = t >> 4;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int r = p * 16 + rr;
        const uint32_t* src = tile + (q * 4) * ITP + r;
        u32x4 w;
        w.x = src[0]; w.y = src[ITP]; w.z = src[2 * ITP]; w.w = src[3 * ITP];
        if (r0 + r < n && c0 + q * 4 < n)
            __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(X + (size_t)(r0 + r) * ld + c0 + q * 4));
    }
}

// VEC: n and ld multiples of 4 and a 16-byte aligned base, so a 16-byte group is inside or outside
// the matrix as a whole; otherwise one word per access.
template <bool VEC, bool NTL>
__global__ __launch_bounds__(256) void transpose_inplace_kernel(uint32_t* __restrict__ X, int n, long ld)
{
    const int ti = blockIdx.y, tj = blockIdx.x;
    if (ti > tj) return;
    __shared__ uint32_t ta[IT * ITP];     // tile (ti, tj)
    __shared__ uint32_t tb[IT * ITP];     // tile (tj, ti)
    const int t = threadIdx.x;
    const int r0 = ti * IT, c0 = tj * IT;
    if (VEC) {
        u32x4 va[4], vb[4];
        inplace_load_tile<NTL>(X, ld, n, r0, c0, va);
        if (ti != tj) inplace_load_tile<NTL>(X, ld, n, c0, r0, vb);
        inplace_stash_tile(ta, va);
        if (ti != tj) inplace_stash_tile(tb, vb);
        __syncthreads();
        inplace_store_transposed(X, ld, n, c0, r0, ta);
        if (ti != tj) inplace_store_transposed(X, ld, n, r0, c0, tb);
        return;
    }
    const int lane_c = t & 63;
    const int rbase = t >> 6;
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
    uint32_t* p = reinterpret_cast<uint32_t*>(X);
    const bool vec = (n % 4 == 0) && (ld % 4 == 0) && ((reinterpret_cast<uintptr_t>(X) & 15) == 0);
    if (!vec)
        hipLaunchKernelGGL((transpose_inplace_kernel<false, false>), dim3(nt, nt), dim3(256), 0, s, p, n, ld);
    else if ((long long)n * n > (1LL << 24))              // beyond the caches: streaming loads
        hipLaunchKernelGGL((transpose_inplace_kernel<true, true>), dim3(nt, nt), dim3(256), 0, s, p, n, ld);
    else
        hipLaunchKernelGGL((transpose_inplace_kernel<true, false>), dim3(nt, nt), dim3(256), 0, s, p, n, ld);
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

// Plain streaming copy of 16-byte words: the reference point for HBM counters and for what a pure
// read-once / write-once kernel reaches on this machine (not part of the paper's method).  Each
// thread keeps four independent 16-byte loads in flight; loads and stores are non-temporal.
__global__ __launch_bounds__(256) void copy_kernel(const u32x4* __restrict__ in, u32x4* __restrict__ out, size_t nvec)
{
    const size_t stride = (size_t)gridDim.x * 1024;
    size_t base = (size_t)blockIdx.x * 1024 + threadIdx.x;
    for (; base + 768 < nvec; base += stride) {
        u32x4 v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = __builtin_nontemporal_load(in + base + j * 256);
#pragma unroll
        for (int j = 0; j < 4; ++j) __builtin_nontemporal_store(v[j], out + base + j * 256);
    }
    // the last, partial group of 1024 words (at most one workgroup gets here with work left)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const size_t i = base + (size_t)j * 256;
        if (i < nvec) __builtin_nontemporal_store(__builtin_nontemporal_load(in + i), out + i);
    }
}

int launch_copy(hipStream_t s, size_t nvec, const void* in, void* out)
{
    if (nvec == 0) return 0;
    size_t blocks = (nvec + 1023) / 1024;
    if (blocks > 256 * 64) blocks = 256 * 64;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, s,
                       static_cast<const u32x4*>(in), static_cast<u32x4*>(out), nvec);
    return (int)hipGetLastError();
}

}  // namespace mtnn

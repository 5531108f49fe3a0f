// In-place transpose of a dense rectangular matrix of 32-bit words: X holds rows x cols (row-major,
// ld = cols) on entry and cols x rows (ld = rows) on exit, with no second buffer.
//
// The paper names in-place transposition as the way out when the memory for B^T is missing (Section
// III) and as future work (Section VI).  Instead of following the cycles of the index permutation
// (long, data-dependent chains of single-word moves), the permutation is factored into passes that
// each permute within the rows or within the columns of the rows x cols view of the buffer, so that
// every pass is a set of independent, LDS-sized problems with coalesced global traffic.
//
// Let R = rows, C = cols, g = gcd(R, C), a = R / g, b = C / g.  The word at (i, j) must end at linear
// index l' = j R + i, i.e. at (i', j') = (l' div C, l' mod C) of the R x C view.
//   pass 0 (columns; only if g > 1)  column j is rotated down by floor(j / b): (i, j) -> (r, j),
//           r = (i + floor(j / b)) mod R.  Without it the g words j, j + b, .. of a row would all ask
//           for the same column in pass 1 (j R mod C depends on j mod b only).
//   pass 1 (rows)     row r sends the word in column j to column j' = (j R + i) mod C, where
//           i = (r - floor(j / b)) mod R is the row it came from.  For fixed r this is a bijection of
//           the columns: with j = u b + v, j R + i = v R + (r - u) (+ R if r < u) mod C; v R runs through
//           the multiples of g exactly once (a and b are coprime), and the g values of u shift that
//           by g consecutive offsets.
//   pass 2 (columns)  column j' now holds exactly the R words whose final column is j', one per row;
//           the word for final row i' is the one that started at (i, j) = (l' mod R, l' div R),
//           l' = i' C + j', and sits in row (i + floor(j / b)) mod R.
// Each pass loads its rows / column panel into LDS, synchronises, and writes back, so reads of a
// row (panel) complete before its writes; different rows (panels) do not interact.
// Limits: R, C <= 32768 (a row, or one column of R words, must fit 128 KB of LDS).
#include "mtnn_internal.h"

#include <atomic>

namespace mtnn {

namespace {

constexpr int kRectThreads = 256;
constexpr unsigned kRectLdsWords = 32768;       // 128 KB

struct RectGeom {
    unsigned R, C, g, b;      // rows, cols, gcd, C / g
};

// pass 1: one workgroup permutes `rows_per_wg` consecutive rows; scatter into LDS, linear write back
__global__ __launch_bounds__(kRectThreads) void rect_row_pass(uint32_t* __restrict__ X, RectGeom q, unsigned rows_per_wg)
{
    extern __shared__ uint32_t buf[];
    const unsigned r0 = blockIdx.x * rows_per_wg;
    const unsigned nrows = min(rows_per_wg, q.R - r0);
    const unsigned total = nrows * q.C;
    uint32_t* base = X + (size_t)r0 * q.C;
    for (unsigned e = threadIdx.x; e < total; e += kRectThreads) {
        const unsigned rr = e / q.C;
        const unsigned j = e - rr * q.C;
        const unsigned r = r0 + rr;
        const unsigned u = j / q.b;                              // rotation pass 0 applied to column j
        const unsigned i = (r >= u) ? r - u : r + q.R - u;       // the row the word came from (u < g <= R)
        const unsigned jp = (j * q.R + i) % q.C;               // j R + i < 2^30 + 2^15 within the size limits
        buf[rr * q.C + jp] = base[e];
    }
    __syncthreads();
    for (unsigned e = threadIdx.x; e < total; e += kRectThreads) base[e] = buf[e];
}

// passes 0 and 2: one workgroup permutes a panel of `w` adjacent columns (all R rows) by a gather
// whose source row depends on (output row, column).  FINAL = false: pass 0; true: pass 2.
template <bool FINAL>
__global__ __launch_bounds__(kRectThreads) void rect_col_pass(uint32_t* __restrict__ X, RectGeom q, unsigned w)
{
    extern __shared__ uint32_t buf[];
    const unsigned j0 = blockIdx.x * w;
    const unsigned nw = min(w, q.C - j0);
    const unsigned total = q.R * w;                              // panel slots, row-major with stride w
    for (unsigned e = threadIdx.x; e < total; e += kRectThreads) {
        const unsigned r = e / w, jj = e - r * w;
        if (jj < nw) buf[e] = X[(size_t)r * q.C + j0 + jj];
    }
    __syncthreads();
    for (unsigned e = threadIdx.x; e < total; e += kRectThreads) {
        const unsigned ip = e / w, jj = e - ip * w;
        if (jj >= nw) continue;
        const unsigned jp = j0 + jj;
        unsigned src;
        if (FINAL) {
            const unsigned l = ip * q.C + jp;                    // < R C <= 2^30
            const unsigned j = l / q.R;
            const unsigned i = l - j * q.R;
            src = i + j / q.b;                                   // < R + g <= 2 R
            if (src >= q.R) src -= q.R;
        } else {
            const unsigned u = jp / q.b;
            src = (ip >= u) ? ip - u : ip + q.R - u;
        }
        X[(size_t)ip * q.C + jp] = buf[src * w + jj];
    }
}

unsigned gcd_u(unsigned a, unsigned b)
{
    while (b) { const unsigned t = a % b; a = b; b = t; }
    return a;
}

template <typename K>
hipError_t allow_big_lds(K kern, size_t bytes, int slot)
{
    if (bytes <= 64 * 1024) return hipSuccess;
    static std::atomic<unsigned long long> raised[3] = {};       // bit per device, per kernel
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return hipGetLastError();
    const unsigned long long bit = (dev >= 0 && dev < 64) ? (1ull << dev) : 0;
    if (bit && (raised[slot].load() & bit)) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                             (int)(kRectLdsWords * sizeof(uint32_t)));
    if (e == hipSuccess && bit) raised[slot].fetch_or(bit);
    return e;
}

}  // namespace

bool transpose_inplace_rect_supported(int rows, int cols)
{
    return rows >= 1 && cols >= 1 && (unsigned)rows <= kRectLdsWords && (unsigned)cols <= kRectLdsWords;
}

int launch_transpose_inplace_rect(hipStream_t s, int rows, int cols, float* X)
{
    if (rows <= 1 || cols <= 1) return 0;                        // a vector: both layouts are the same words
    if (!transpose_inplace_rect_supported(rows, cols)) return (int)hipErrorInvalidValue;
    RectGeom q;
    q.R = (unsigned)rows;
    q.C = (unsigned)cols;
    q.g = gcd_u(q.R, q.C);
    q.b = q.C / q.g;
    uint32_t* p = reinterpret_cast<uint32_t*>(X);
    // column panels: as wide as LDS allows, at most 32 words (one 128-byte line per row)
    unsigned w = 32;
    while (w > 1 && (unsigned long long)q.R * w > kRectLdsWords) w >>= 1;
    const unsigned panels = (q.C + w - 1) / w;
    const size_t col_lds = (size_t)q.R * w * sizeof(uint32_t);
    // rows per workgroup: about 8 K words of work each
    unsigned rpw = 8192 / q.C;
    if (rpw < 1) rpw = 1;
    const unsigned row_groups = (q.R + rpw - 1) / rpw;
    const size_t row_lds = (size_t)rpw * q.C * sizeof(uint32_t);
    hipError_t e;
    if (q.g > 1) {
        if ((e = allow_big_lds(rect_col_pass<false>, col_lds, 0)) != hipSuccess) return (int)e;
        hipLaunchKernelGGL(rect_col_pass<false>, dim3(panels), dim3(kRectThreads), col_lds, s, p, q, w);
        if ((e = hipGetLastError()) != hipSuccess) return (int)e;
    }
    if ((e = allow_big_lds(rect_row_pass, row_lds, 1)) != hipSuccess) return (int)e;
    hipLaunchKernelGGL(rect_row_pass, dim3(row_groups), dim3(kRectThreads), row_lds, s, p, q, rpw);
    if ((e = hipGetLastError()) != hipSuccess) return (int)e;
    if ((e = allow_big_lds(rect_col_pass<true>, col_lds, 2)) != hipSuccess) return (int)e;
    hipLaunchKernelGGL(rect_col_pass<true>, dim3(panels), dim3(kRectThreads), col_lds, s, p, q, w);
    return (int)hipGetLastError();
}

}  // namespace mtnn

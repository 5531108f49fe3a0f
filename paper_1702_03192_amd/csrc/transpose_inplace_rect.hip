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
//
// The three passes take an R x C buffer to C x R while working on columns of R words.  Run backwards
// (the inverse of pass 2, of pass 1, of pass 0: the same index formulas with the gather on the other
// side of LDS) they take a C x R buffer to R x C, still working on columns of R words.  The launcher
// takes whichever direction makes the columns the shorter dimension: a column panel in LDS is then as
// wide as it can be (global accesses of up to 128 bytes per row of the panel) and there are many panels.
// Column panels are dealt to the XCDs in contiguous ranges, so that the panels in flight on one XCD
// share the cache lines they each use a few words of.  Divisions by R, C, b are multiply-high with
// host-made constants.
// Limits: R, C <= 32768 (a row, or one column of R words, must fit 128 KB of LDS).
#include "mtnn_internal.h"
#include "gemm_config.h"

#include <atomic>

namespace mtnn {

namespace {

constexpr int kRectThreads = 1024;
constexpr unsigned kRectLdsWords = 32768;       // 128 KB

struct RectGeom {
    unsigned R, C, b;          // rows and columns of the view the passes work in, C / gcd(R, C)
    FastDiv fdR, fdC, fdb;
};

__device__ __forceinline__ unsigned udiv(unsigned n, FastDiv f) { return (unsigned)fast_div((int)n, f); }

// pass 1: one workgroup permutes `rows_per_wg` consecutive rows.  Forward: row r sends column j to
// column jp(r, j), scattered into LDS and written back in order.  INVERSE: column j takes the word of
// column jp(r, j), the rows copied to LDS in order and gathered from there.
template <bool INVERSE>
__global__ __launch_bounds__(kRectThreads) void rect_row_pass(uint32_t* __restrict__ X, RectGeom q, unsigned rows_per_wg)
{
    extern __shared__ uint32_t buf[];
    const unsigned r0 = blockIdx.x * rows_per_wg;
    const unsigned nrows = min(rows_per_wg, q.R - r0);
    const unsigned total = nrows * q.C;
    uint32_t* base = X + (size_t)r0 * q.C;
    if (INVERSE) {
        for (unsigned e = threadIdx.x; e < total; e += kRectThreads) buf[e] = base[e];
        __syncthreads();
    }
    for (unsigned e = threadIdx.x; e < total; e += kRectThreads) {
        const unsigned rr = udiv(e, q.fdC);
        const unsigned j = e - rr * q.C;
        const unsigned r = r0 + rr;
        const unsigned u = udiv(j, q.fdb);                       // rotation of pass 0 applied to column j
        const unsigned i = (r >= u) ? r - u : r + q.R - u;       // the row the word came from (u < g <= R)
        const unsigned t = j * q.R + i;                          // < 2^30 + 2^15 within the size limits
        const unsigned jp = t - udiv(t, q.fdC) * q.C;
        if (INVERSE) base[e] = buf[rr * q.C + jp];
        else buf[rr * q.C + jp] = base[e];
    }
    if (!INVERSE) {
        __syncthreads();
        for (unsigned e = threadIdx.x; e < total; e += kRectThreads) base[e] = buf[e];
    }
}

// passes 0 and 2: one workgroup permutes a panel of w = 2^lw adjacent columns (all R rows) within its
// columns.  The forward pass moves the word of row src(ip, jp) to row ip; FINAL = false: pass 0, true:
// pass 2.  INVERSE moves the word of row ip to row src(ip, jp).
template <bool FINAL, bool INVERSE>
__global__ __launch_bounds__(kRectThreads) void rect_col_pass(uint32_t* __restrict__ X, RectGeom q, unsigned lw,
                                                              unsigned panels, unsigned panels_per_xcd, unsigned num_xcd)
{
    extern __shared__ uint32_t buf[];
    // consecutive workgroup ids go to different XCDs: give each XCD a contiguous range of panels
    const unsigned xcd = blockIdx.x % num_xcd;
    const unsigned panel = xcd * panels_per_xcd + blockIdx.x / num_xcd;
    if (blockIdx.x / num_xcd >= panels_per_xcd || panel >= panels) return;      // uniform per workgroup
    const unsigned w = 1u << lw;
    const unsigned j0 = panel << lw;
    const unsigned jj = threadIdx.x & (w - 1);
    const unsigned jp = j0 + jj;
    const unsigned row0 = threadIdx.x >> lw, step = kRectThreads >> lw;
    const bool live = jp < q.C;                                   // false: a column past the edge of the last panel
    uint32_t* col = X + jp;
    const unsigned u0 = FINAL ? 0u : udiv(jp, q.fdb);

    auto source_row = [&](unsigned ip) -> unsigned {
        if (FINAL) {
            const unsigned l = ip * q.C + jp;                    // < R C <= 2^30
            const unsigned j = udiv(l, q.fdR);
            unsigned src = (l - j * q.R) + udiv(j, q.fdb);       // < R + g <= 2 R
            if (src >= q.R) src -= q.R;
            return src;
        }
        return (ip >= u0) ? ip - u0 : ip + q.R - u0;
    };

    // every lane reaches the one barrier: lanes of one wave may differ in `live`
    if (INVERSE) {
        if (live)
            for (unsigned ip = row0; ip < q.R; ip += step) buf[(source_row(ip) << lw) + jj] = col[(size_t)ip * q.C];
        __syncthreads();
        if (live)
            for (unsigned r = row0; r < q.R; r += step) col[(size_t)r * q.C] = buf[(r << lw) + jj];
    } else {
        if (live)
            for (unsigned r = row0; r < q.R; r += step) buf[(r << lw) + jj] = col[(size_t)r * q.C];
        __syncthreads();
        if (live)
            for (unsigned ip = row0; ip < q.R; ip += step) col[(size_t)ip * q.C] = buf[(source_row(ip) << lw) + jj];
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
    static std::atomic<unsigned long long> raised[6] = {};       // bit per device, per kernel
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return hipGetLastError();
    const unsigned long long bit = (dev >= 0 && dev < 64) ? (1ull << dev) : 0;
    if (bit && (raised[slot].load() & bit)) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                             (int)(kRectLdsWords * sizeof(uint32_t)));
    if (e == hipSuccess && bit) raised[slot].fetch_or(bit);
    return e;
}

struct ColLaunch {
    unsigned lw, panels, per_xcd, num_xcd, grid;
    size_t lds;
};

template <bool FINAL, bool INVERSE>
hipError_t run_col_pass(hipStream_t s, uint32_t* p, const RectGeom& q, const ColLaunch& c, int slot)
{
    hipError_t e = allow_big_lds(rect_col_pass<FINAL, INVERSE>, c.lds, slot);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((rect_col_pass<FINAL, INVERSE>), dim3(c.grid), dim3(kRectThreads), c.lds, s, p, q, c.lw, c.panels,
                       c.per_xcd, c.num_xcd);
    return hipGetLastError();
}

template <bool INVERSE>
hipError_t run_row_pass(hipStream_t s, uint32_t* p, const RectGeom& q, unsigned rpw, int slot)
{
    const size_t lds = (size_t)rpw * q.C * sizeof(uint32_t);
    hipError_t e = allow_big_lds(rect_row_pass<INVERSE>, lds, slot);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(rect_row_pass<INVERSE>, dim3((q.R + rpw - 1) / rpw), dim3(kRectThreads), lds, s, p, q, rpw);
    return hipGetLastError();
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
    // forward: the buffer is R x C = rows x cols; backward: it is C x R with R = cols, C = rows.
    // Either way the passes see an R x C view; R is the shorter dimension.
    const bool inverse = rows > cols;
    RectGeom q;
    q.R = (unsigned)(inverse ? cols : rows);
    q.C = (unsigned)(inverse ? rows : cols);
    const unsigned g = gcd_u(q.R, q.C);
    q.b = q.C / g;
    q.fdR = make_fastdiv(q.R);
    q.fdC = make_fastdiv(q.C);
    q.fdb = make_fastdiv(q.b);
    uint32_t* p = reinterpret_cast<uint32_t*>(X);
    // column panels: as wide as LDS allows, at most 32 words (one 128-byte line per row), and
    // narrower (down to 32 bytes per row) while there are fewer than two panels per CU
    ColLaunch c;
    c.lw = 5;
    while (c.lw > 0 && ((unsigned long long)q.R << c.lw) > kRectLdsWords) --c.lw;
    const unsigned want_panels = 2u * (unsigned)geometry_or_nominal().cus;
    while (c.lw > 3 && ((q.C + (1u << c.lw) - 1) >> c.lw) < want_panels) --c.lw;
    c.panels = (q.C + (1u << c.lw) - 1) >> c.lw;
    c.num_xcd = (unsigned)geometry_or_nominal().xcds;
    if (c.num_xcd < 1 || c.panels < 4 * c.num_xcd) c.num_xcd = 1;
    c.per_xcd = (c.panels + c.num_xcd - 1) / c.num_xcd;
    c.grid = c.per_xcd * c.num_xcd;
    c.lds = ((size_t)q.R << c.lw) * sizeof(uint32_t);
    // rows per workgroup: about 16 K words of work each (two workgroups per CU)
    unsigned rpw = 16384 / q.C;
    if (rpw < 1) rpw = 1;
    hipError_t e;
    if (!inverse) {
        if (g > 1 && (e = run_col_pass<false, false>(s, p, q, c, 0)) != hipSuccess) return (int)e;
        if ((e = run_row_pass<false>(s, p, q, rpw, 1)) != hipSuccess) return (int)e;
        return (int)run_col_pass<true, false>(s, p, q, c, 2);
    }
    if ((e = run_col_pass<true, true>(s, p, q, c, 3)) != hipSuccess) return (int)e;
    if ((e = run_row_pass<true>(s, p, q, rpw, 4)) != hipSuccess) return (int)e;
    if (g > 1) return (int)run_col_pass<false, true>(s, p, q, c, 5);
    return 0;
}

}  // namespace mtnn

// What the translation units of the GEMM share: the kernel argument block, the table of tile
// configurations (geometry + the cost model's fitted numbers, gemm_cost.cpp) and the table of
// kernel instances per tile geometry (gemm_inst_*.hip, assembled in gemm_launch.hip).  Keeping the
// fitted numbers apart from the kernels means a changed constant recompiles one small host file.
#pragma once
#include "mtnn_internal.h"

namespace mtnn {

// Division of a number below 2^31 by a divisor known on the host, as a multiply-high and a shift: with
// s = ceil(log2 d) and mul = floor(2^(31+s) / d) + 1 (which fits 32 bits), floor(n / d) =
// (n x mul) >> (31 + s) exactly for every n < 2^31 (the error mul d - 2^(31+s) is at most d, so n times
// it stays below 2^(31+s)).  On wave-uniform operands this is two scalar instructions; an integer
// division in the kernel would be some twenty vector instructions, which the fp32 matrix instructions
// cannot overlap (they run on the same lanes).
struct FastDiv {
    unsigned mul;     // 0: the divisor is 1
    unsigned shift;   // (31 + s) - 32
};
inline FastDiv make_fastdiv(unsigned d)
{
    FastDiv f = {0u, 0u};
    if (d <= 1) return f;
    unsigned s = 0;
    while ((1ull << s) < d) ++s;
    f.mul = (unsigned)(((1ull << (31 + s)) / d) + 1ull);
    f.shift = s - 1;
    return f;
}
__host__ __device__ inline int fast_div(int n, FastDiv f)
{
    if (f.mul == 0) return n;
    return (int)((unsigned)(((unsigned long long)(unsigned)n * f.mul) >> 32) >> f.shift);
}

struct GemmParams {
    const float* A;
    const float* B;
    float* C;
    int M, N, K;
    long lda, ldb, ldc;
    int tiles_m, tiles_n;
    int group_m;      // C-tile rows per band (L2 locality)
    int num_xcd;      // XCDs the hardware deals consecutive workgroup ids to (8 on MI355X); 1: no remapping
    // what tile_of_block needs, worked out on the host (set_tile_order): the deal of tile ids to XCDs
    // (the first xcd_tall XCDs take xcd_per ids, the others one fewer) and the bands of group_m tile rows
    int xcd_per, xcd_tall;
    int last_band, last_rows;   // index of the last band and its number of tile rows (<= group_m)
    FastDiv fd_xcd, fd_band, fd_group, fd_last;   // divisions by num_xcd, group_m x tiles_n, group_m, last_rows
    // split-k: workgroup w handles C tile w % tiles and k range [split * k_per_split, ...) with
    // split = w / tiles; partial products go to `part` (splits dense M x N matrices), summed by
    // reduce_splits_kernel in split order.  splits == 1: results go straight to C.
    int splits;
    int k_per_split;  // a multiple of every configuration's k slab
    float* part;
    int part_cached;  // split-k: the partial products are small enough to be written with ordinary stores
    int sk_units_per_tile;   // gemm_streamk_kernel: k units (of kSplitQuantum) per tile
    // fused epilogues (read only by the kernel instances built for them)
    const float* bias;       // kEpiBiasAct: C = act(A x B + bias[column])
    int relu;
    float* W;                // kEpiSgd: C = A x B and W -= lr * C (W: M x N, leading dimension ldw)
    long ldw;
    float lr;
};

// fills the fields tile_of_block reads from tiles_m, tiles_n, group_m and num_xcd
inline void set_tile_order(GemmParams& p)
{
    const int total = p.tiles_m * p.tiles_n;
    if (p.num_xcd < 1 || total < p.num_xcd) p.num_xcd = 1;
    p.xcd_per = (total + p.num_xcd - 1) / p.num_xcd;
    p.xcd_tall = total - (p.xcd_per - 1) * p.num_xcd;
    const int bands = (p.tiles_m + p.group_m - 1) / p.group_m;
    p.last_band = bands - 1;
    p.last_rows = p.tiles_m - p.last_band * p.group_m;
    p.fd_xcd = make_fastdiv((unsigned)p.num_xcd);
    p.fd_band = make_fastdiv((unsigned)(p.group_m * p.tiles_n));
    p.fd_group = make_fastdiv((unsigned)p.group_m);
    p.fd_last = make_fastdiv((unsigned)p.last_rows);
}

// what a kernel instance does with its accumulators besides storing them
constexpr int kEpiNone = 0;
constexpr int kEpiBiasAct = 1;   // every launch shape; with split-k the reduction kernel applies it
constexpr int kEpiSgd = 2;       // pipelined NN kernel, unsplit launches only

constexpr int kSplitQuantum = 64;   // k ranges of split work are multiples of this (every slab size divides it)
constexpr int kFixChunks = 4;       // workgroups per cut tile in the even cut's fix-up kernel
constexpr int kMaxSplits = 32;
constexpr int kStreamK = -2;        // in place of a split count: cut the work evenly over a fixed grid

// The kernel instances of one tile geometry.
typedef void (*GemmKernel)(GemmParams);
struct KernelSet {
    GemmKernel kern[2][2];    // guarded kernel, [op][16-byte aligned rows]
    GemmKernel dma[2];        // pipelined kernel, [op]
    GemmKernel dma_bias[2];   // pipelined kernel with the bias + activation epilogue, [op]; may be null
    GemmKernel dma_sgd;       // pipelined NN kernel with the fused SGD step; may be null
    GemmKernel sk[2];         // the pipelined kernel with the work cut evenly over a fixed grid, [op]
    void (*fix)(GemmParams, int);   // ... and its fix-up kernel
};
constexpr int kNumKernelSets = 14;
// each fills the entries of the geometries it instantiates (gemm_inst_*.hip)
void fill_kernel_sets_a(KernelSet* table);
void fill_kernel_sets_b(KernelSet* table);
void fill_kernel_sets_c(KernelSet* table);
void fill_kernel_sets_d(KernelSet* table);
void fill_kernel_sets_e(KernelSet* table);

// One tile configuration: a geometry, how many workgroups a CU should hold, and the cost model's
// numbers for it.
struct TileConfig {
    const char* name;
    int bm, bn, bk;
    int gbk;                          // k slab of the guarded kernel that serves what the pipelined one cannot
    int nstage;
    int threads;                      // of the pipelined kernel
    int threads_guarded;              // of the guarded kernel (the same unless the pipelined one runs two sets of waves)
    int waves_n;
    int max_wg;                       // workgroups per CU the launch allows (it sizes its LDS request to that)
    int kernel_set;                   // index into the KernelSet table
    bool has_fused;                   // fused-epilogue instances exist for this geometry
    // Fitted to measured times of the {64..8192}^3 grid with every CU busy (tune.py collect / fit):
    // time of one CU = tiles x (2 bm bn k / (eff x peak per CU)) + rounds x round_s
    // (separately for NN and NT: index = GemmOp)
    float eff[2];                     // rate of the k loop as a fraction of the fp32 MFMA peak
    float round_s[2];                 // seconds per round outside the k loop: first copies, result store
    float eff_guarded[2];             // the same two for the guarded kernel (fitted with odd leading dimensions)
    float round_guarded_s[2];

    // LDS bytes of the guarded kernel: two buffers of an A slab and a B slab (layouts as in the kernel)
    size_t lds_bytes_guarded(int op) const
    {
        const size_t a = (size_t)bm * (gbk + 4);
        const size_t b = (op == OP_NT) ? (size_t)bn * (gbk + 4) : (size_t)gbk * (bn + 8);
        return 2 * (a + b) * sizeof(float);
    }
    size_t lds_bytes_dma() const
    {
        const size_t ring = (size_t)nstage * (bm + bn) * bk * sizeof(float);
        // epilogue patches: 16 rows x (wave tile width + 8) words per wave
        const size_t waves = (size_t)threads / 64;
        const size_t wn = (size_t)bn / (size_t)waves_n;
        const size_t patches = waves * 16 * (wn + 8) * sizeof(float);
        return ring > patches ? ring : patches;
    }
    // workgroups of the pipelined kernel a CU holds at a time (bounded by its LDS)
    int wg_per_cu(int lds_per_cu) const
    {
        const int by_lds = (int)((size_t)lds_per_cu / lds_bytes_dma());
        const int r = by_lds < max_wg ? by_lds : max_wg;
        return r < 1 ? 1 : r;
    }
};
extern const TileConfig kTileConfigs[];
extern const int kNumTileConfigs;

// ---- choice of configuration and split count (gemm_cost.cpp) ------------------------------------
struct Choice { int cfg; int splits; };
// pipelined: the operands allow the pipelined kernel; otherwise the guarded kernel's own rates are
// used (and the even cut, which exists only in the pipelined kernel, is not considered).
// epi_kind: the launch wants that epilogue fused.  scratch_bytes: room for partial products; a
// candidate whose partials do not fit is not considered (0: unsplit launches only).
Choice choose(const Geometry& geo, int op, int m, int n, int k, bool allow_split, bool pipelined, int epi_kind,
              size_t scratch_bytes);
// scratch bytes of a launch: split-k partials (splits >= 2), the even cut's slots (kStreamK), else 0
size_t scratch_needed(const Geometry& geo, int cfg, int splits, int m, int n, int k);
// the split count and k range per split a launch really uses for a requested count (ranges are
// multiples of kSplitQuantum, empty splits are dropped)
void effective_splits(int k, int splits, int* eff_splits, int* k_per_split);

}  // namespace mtnn

// fp32 GEMM kernels for gfx950 on the matrix cores:
//   NN (Eq. 1 of the MTNN paper):  C[i][j] = sum_l A[i][l] * B[l][j]   A m x k, B k x n
//   NT (Eq. 2):                    C[i][j] = sum_l A[i][l] * B[j][l]   A m x k, B n x k
// all row-major, alpha = 1, no beta term (Section II).
//
// Two kernels share the tile geometry below: gemm_dma_kernel, the pipelined one (slabs copied global
// -> LDS directly, ring of slab buffers; 16-byte aligned operands with k % 4 = 0), and gemm_kernel,
// the guarded one for everything else.  The work is divided one of three ways: one workgroup per C
// tile; split-k (several workgroups per tile, partial products summed by reduce_splits_kernel); or
// the even cut (gemm_streamk_kernel: all tiles' k ranges cut into equal pieces over a fixed grid,
// cut tiles finished by streamk_fixup_kernel).  `choose` picks configuration and division per shape.
//
// Design (ours; the paper calls a closed library for both operations):
//   * one workgroup computes a BM x BN tile of C, stepping through k in slabs of BK;
//   * each 64-lane wave owns a WM x WN sub-tile built from 32x32 blocks, each block advanced
//     by v_mfma_f32_32x32x2_f32 (lane l supplies A[l%32][l/32] and B[l/32][l%32]; 16
//     accumulator registers per block, register r of lane l holding row 8*(r/4)+4*(l/32)+r%4,
//     column l%32);
//   * slabs are staged global -> registers -> LDS with two LDS buffers, so the loads of slab
//     t+1 are in flight while slab t feeds the matrix cores, and one barrier per slab suffices;
//   * A is kept in LDS as [row][k] with a padded row stride, so a lane fetches four consecutive
//     k of its row with one 128-bit LDS read.  The order in which k is consumed inside a group
//     of 8 is permuted (lanes 0-31 take k = 0..3, lanes 32-63 take k = 4..7); A and B use the
//     same permutation and a sum does not care;
//   * NT: B rows are k-contiguous exactly like A rows, so B uses the same staging as A.
//     NN: B rows are n-contiguous; the slab is kept as [k][n] (the guarded kernel reads its
//     column word by word; the pipelined kernel reads TN consecutive n per lane, see there);
//   * rows of A / B beyond m / n are clamped to the last valid row: they only feed outputs
//     that are never stored.  Elements beyond k are zero-filled in both operands, so padding
//     (which may hold NaN) never reaches a sum;
//   * workgroup ids are remapped so that each XCD (the hardware deals consecutive ids round
//     robin to its 8 XCDs, each with a private L2) works on one compact band of C tiles.
//
// The summation order of every C element is fixed by (configuration, k), never by timing:
// results are bit-reproducible.
#pragma once
#include "gemm_config.h"

namespace mtnn {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
// four consecutive floats at any 4-byte aligned address: the compiler may still use one 16-byte
// global load where the target allows unaligned vector access
typedef float f32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));




// what one workgroup works on: its k range of A and B, and where its tile of results goes
struct WorkView {
    const float* A;
    const float* B;
    float* C;
    long ldc;
    int K;
    int pid;          // C tile index before the XCD / band remapping
};

__device__ __forceinline__ WorkView work_view(const GemmParams& p, bool nt)
{
    WorkView v;
    const int tiles = p.tiles_m * p.tiles_n;
    const int split = (p.splits > 1) ? (int)blockIdx.x / tiles : 0;
    v.pid = (int)blockIdx.x - split * tiles;
    const int ks = split * p.k_per_split;
    v.K = min(p.K - ks, p.k_per_split);
    v.A = p.A + ks;
    v.B = nt ? p.B + ks : p.B + (size_t)ks * p.ldb;
    if (p.splits > 1) {
        v.C = p.part + (size_t)split * p.M * p.N;
        v.ldc = p.N;
    } else {
        v.C = p.C;
        v.ldc = p.ldc;
    }
    return v;
}

// ---- guarded global loads -------------------------------------------------------------------

// Four consecutive k of one row.  FAST: the caller guarantees kidx + 3 < K (interior slab), so
// the load is unconditional and the k loop stays free of divergent branches; otherwise elements
// at or beyond K read as zero.
template <bool VEC, bool FAST>
__device__ __forceinline__ f32x4 load_k4(const float* __restrict__ row, int kidx, int K)
{
    if (FAST || kidx + 3 < K) {
        if (VEC) return *reinterpret_cast<const f32x4*>(row + kidx);
        return *reinterpret_cast<const f32x4_a4*>(row + kidx);
    }
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (kidx < K) v.x = row[kidx];
    if (kidx + 1 < K) v.y = row[kidx + 1];
    if (kidx + 2 < K) v.z = row[kidx + 2];
    return v;
}

// Four consecutive n of one k-row of B (NN).  FAST: krow < K and nidx + 3 < N are guaranteed.
// Otherwise columns beyond N are clamped (they feed only outputs that are never stored) and
// rows at or beyond K read as zero.
template <bool VEC, bool FAST>
__device__ __forceinline__ f32x4 load_n4(const float* __restrict__ B, long ldb, int krow, int K, int nidx, int N)
{
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (!FAST && krow >= K) return v;
    const float* row = B + (size_t)krow * ldb;
    if (FAST || nidx + 3 < N) {
        if (VEC) return *reinterpret_cast<const f32x4*>(row + nidx);
        return *reinterpret_cast<const f32x4_a4*>(row + nidx);
    }
    const int last = N - 1;
    v.x = row[min(nidx, last)];
    v.y = row[min(nidx + 1, last)];
    v.z = row[min(nidx + 2, last)];
    v.w = row[min(nidx + 3, last)];
    return v;
}

// ---- workgroup id -> C tile -------------------------------------------------------------------

// (All operands are wave-uniform and the divisions are multiply-high + shift with host-made
// constants, so the whole mapping runs on the scalar unit.)
__device__ __forceinline__ void tile_of_block(const GemmParams& p, int pid, int& tm, int& tn)
{
    // undo the round-robin deal to XCDs: XCD x receives ids x, x+X, x+2X, ...; give it the
    // contiguous range of logical ids [start(x), start(x+1))
    const int X = p.num_xcd;
    if (X > 1) {
        const int local = fast_div(pid, p.fd_xcd);
        const int x = pid - local * X;
        pid = (x < p.xcd_tall) ? x * p.xcd_per + local
                               : p.xcd_tall * p.xcd_per + (x - p.xcd_tall) * (p.xcd_per - 1) + local;
    }
    // bands of group_m tile rows, walked column by column inside a band
    const int band_sz = p.group_m * p.tiles_n;
    const int band = fast_div(pid, p.fd_band);
    const int in_band = pid - band * band_sz;
    const bool last = (band == p.last_band);
    const int rows_here = last ? p.last_rows : p.group_m;
    tn = fast_div(in_band, last ? p.fd_last : p.fd_group);
    tm = band * p.group_m + (in_band - tn * rows_here);
}

// ---- epilogue: accumulators -> C -------------------------------------------------------------
//
// Register r of lane l of a 32x32 block is row 8*(r/4) + 4*(l/32) + r%4, column l%32: one store
// instruction writes two full 128-byte row segments.  Results are not read again by the kernel, so
// the stores are non-temporal; tiles entirely inside C skip the per-element guards.
// BIAS: each value first takes its column's bias (bv[j] for block j of this lane) and, if relu, the clamp at zero
template <bool BIAS, int TN>
__device__ __forceinline__ float with_bias(float v, const float (&bv)[TN], int j, int relu)
{
    if (BIAS) {
        v += bv[j];
        // (a select, not a branch on `relu`: a branch would be merged across the whole unrolled epilogue
        // and every addition hoisted above it, with all accumulators live in VGPRs at once)
        const bool keep = (v > 0.f) | (relu == 0);
        v = keep ? v : 0.f;
    }
    return v;
}

// STREAM: results are not read again by the kernel, so they are written past the cache -- if the rows
// of C start on 128-byte lines, so that a tile's row segments (128 bytes or more, at multiples of 128
// bytes within the row) are whole lines.  Otherwise a segment shares its first and last line with the
// neighbouring tiles' segments, and ordinary stores let the pieces meet in L2 instead of each going to
// memory alone.  Measured with 128 x 64 tiles, NT, streamed against ordinary: 7928 x 5018 x 76 (rows 8
// bytes off) 101 against 82 us; n = 5016 (32-byte rows) 89 against 80; 8192 x 4112 x 64 (64-byte rows) 70
// against 54; with whole lines streaming wins, 2 % at 7928 x 5024 x 76, 10 % at 8192 x 8192 x 64.
__device__ __forceinline__ bool whole_lines(const float* C, long ldc)
{
    return ((reinterpret_cast<uintptr_t>(C) & 127) == 0) && ((ldc & 31) == 0);
}

template <bool STREAM, typename T>
__device__ __forceinline__ void put(T v, T* dst)
{
    if (STREAM) __builtin_nontemporal_store(v, dst);
    else *dst = v;
}

template <int TM, int TN, bool BIAS = false, bool STREAM = true>
__device__ __forceinline__ void store_tile(const f32x16 (&acc)[TM][TN], float* __restrict__ C, long ldc,
                                           int M, int N, int row0, int col0, int lr, int lh,
                                           const float (&bv)[TN], int relu)
{
    if (row0 + TM * 32 <= M && col0 + TN * 32 <= N) {
        // one address per lane, then wave-uniform row offsets (scalar multiplies) added to it
        float* lane_base = C + (size_t)(row0 + lh * 4) * ldc + col0 + lr;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float* dst = lane_base + (size_t)(i * 32 + (r / 4) * 8 + (r % 4)) * ldc;
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    put<STREAM>(with_bias<BIAS, TN>(acc[i][j][r], bv, j, relu), dst + j * 32);
                if (BIAS && r % 4 == 3) __builtin_amdgcn_sched_barrier(0);   // (keeps the additions next to their stores)
            }
        return;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = col0 + j * 32 + lr;
            if (col < N) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = row0 + i * 32 + (r / 4) * 8 + lh * 4 + (r % 4);
                    if (row < M) C[(size_t)row * ldc + col] = with_bias<BIAS, TN>(acc[i][j][r], bv, j, relu);
                }
            }
        }
    }
}

// Epilogue of the pipelined NN kernel.  There a lane's TN accumulator blocks hold TN CONSECUTIVE
// columns (block j, lane l <-> column TN * (l % 32) + j, see the B fragment reads), so for interior
// tiles of an aligned C one store per accumulator register writes TN words: lanes 0-31 cover
// 32 * TN consecutive words of one row.
template <int TM, int TN, bool BIAS = false, bool STREAM = true>
__device__ __forceinline__ void store_tile_interleaved(const f32x16 (&acc)[TM][TN], float* __restrict__ C, long ldc,
                                                       int M, int N, int row0, int col0, int lr, int lh, bool aligned,
                                                       const float (&bv)[TN], int relu)
{
    typedef float vecN __attribute__((ext_vector_type(TN)));
    if (TN > 1 && aligned && row0 + TM * 32 <= M && col0 + TN * 32 <= N) {
        float* lane_base = C + (size_t)(row0 + lh * 4) * ldc + col0 + TN * lr;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                vecN v;
#pragma unroll
                for (int j = 0; j < TN; ++j) v[j] = with_bias<BIAS, TN>(acc[i][j][r], bv, j, relu);
                float* dst = lane_base + (size_t)(i * 32 + (r / 4) * 8 + (r % 4)) * ldc;
                put<STREAM>(v, reinterpret_cast<vecN*>(dst));
                if (BIAS && r % 4 == 3) __builtin_amdgcn_sched_barrier(0);
            }
        return;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = row0 + i * 32 + (r / 4) * 8 + lh * 4 + (r % 4);
            if (row < M) {
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int col = col0 + TN * lr + j;
                    if (col < N) C[(size_t)row * ldc + col] = with_bias<BIAS, TN>(acc[i][j][r], bv, j, relu);
                }
            }
        }
}

// store_tile_interleaved plus the plain SGD step on a second matrix of the same shape:
// G = acc (the gradient, not read again here: non-temporal) and W = fma(-lr, acc, W), the same
// arithmetic as the separate update kernel, so fusing the step changes no bit of either result.
template <int TM, int TN>
__device__ __forceinline__ void store_tile_interleaved_sgd(const f32x16 (&acc)[TM][TN], float* __restrict__ G, long ldg,
                                                           float* __restrict__ W, long ldw, float lr,
                                                           int M, int N, int row0, int col0, int lr_, int lh, bool aligned)
{
    typedef float vecN __attribute__((ext_vector_type(TN)));
    if (TN > 1 && aligned && row0 + TM * 32 <= M && col0 + TN * 32 <= N) {
        // eight rows at a time (their loads of W in flight together), so that the loads of the whole
        // tile are not all hoisted to the front at the cost of as many registers
        float* w_base = W + (size_t)(row0 + lh * 4) * ldw + col0 + TN * lr_;
        float* g_base = G + (size_t)(row0 + lh * 4) * ldg + col0 + TN * lr_;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                vecN w[8];
#pragma unroll
                for (int rr = 0; rr < 8; ++rr) {
                    const int r = h * 8 + rr;
                    const size_t row = (size_t)(i * 32 + (r / 4) * 8 + (r % 4));      // wave-uniform
                    w[rr] = *reinterpret_cast<const vecN*>(w_base + row * ldw);
                }
#pragma unroll
                for (int rr = 0; rr < 8; ++rr) {
                    const int r = h * 8 + rr;
                    const size_t row = (size_t)(i * 32 + (r / 4) * 8 + (r % 4));
                    vecN g;
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        g[j] = acc[i][j][r];
                        w[rr][j] = __builtin_fmaf(-lr, g[j], w[rr][j]);
                    }
                    *reinterpret_cast<vecN*>(w_base + row * ldw) = w[rr];
                    __builtin_nontemporal_store(g, reinterpret_cast<vecN*>(g_base + row * ldg));
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        return;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = row0 + i * 32 + (r / 4) * 8 + lh * 4 + (r % 4);
            if (row < M) {
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int col = col0 + TN * lr_ + j;
                    if (col < N) {
                        const float g = acc[i][j][r];
                        float* wp = W + (size_t)row * ldw + col;
                        *wp = __builtin_fmaf(-lr, g, *wp);
                        G[(size_t)row * ldg + col] = g;
                    }
                }
            }
        }
}

// The same through LDS, for tiles entirely inside a C whose rows are 16-byte aligned: 16 rows of the
// wave's sub-tile at a time are written to a wave-private LDS patch (row stride WN + 8 words: the two
// lane halves, 4 rows apart, land 32 banks apart) and read back as 128-bit row pieces, so every
// store instruction writes whole 512-byte (WN = 128) row segments, 16 bytes per lane.
template <int TM, int TN, bool BIAS = false, bool STREAM = true>
__device__ __forceinline__ void store_tile_staged(const f32x16 (&acc)[TM][TN], float* __restrict__ C, long ldc,
                                                  int row0, int col0, int lane, float* patch,
                                                  const float (&bv)[TN], int relu)
{
    constexpr int WN = TN * 32;
    constexpr int S = WN + 8;
    constexpr int V = WN / 4;                 // 16-byte pieces per row
    constexpr int PIECES = 16 * V;            // pieces per 16-row patch
    const int lr = lane & 31;
    const int lh = lane >> 5;
    // lane-dependent parts once: where this lane writes in the patch, where it reads, and its address in C
    float* wr = patch + (lh * 4) * S + lr;
    const float* rd = patch + (lane / V) * S + (lane % V) * 4;
    float* lane_base = C + (size_t)(row0 + lane / V) * ldc + col0 + (lane % V) * 4;
    constexpr int ROWS_PER_T = 64 / V;                                      // patch rows one pass of 64 lanes covers
    static_assert(64 % V == 0, "a pass of 64 lanes covers whole patch rows");
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
#pragma unroll
            for (int rr = 0; rr < 8; ++rr) {
                const int r = h * 8 + rr;                                   // rows 16h .. 16h+15 of the block
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    wr[((rr / 4) * 8 + (rr % 4)) * S + j * 32] = with_bias<BIAS, TN>(acc[i][j][r], bv, j, relu);
            }
#pragma unroll
            for (int t = 0; t < (PIECES + 63) / 64; ++t) {
                if (PIECES % 64 == 0 || t * 64 + lane < PIECES) {
                    const f32x4 v = *reinterpret_cast<const f32x4*>(rd + (t * ROWS_PER_T) * S);
                    put<STREAM>(v, reinterpret_cast<f32x4*>(lane_base + (size_t)(i * 32 + h * 16 + t * ROWS_PER_T) * ldc));
                }
            }
            if (BIAS) __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// ---- the kernel ------------------------------------------------------------------------------

template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, bool NT, bool VEC>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64) void gemm_kernel(GemmParams p)
{
    constexpr int NTH = WAVES_M * WAVES_N * 64;
    constexpr int WM = BM / WAVES_M;
    constexpr int WN = BN / WAVES_N;
    constexpr int TM = WM / 32;
    constexpr int TN = WN / 32;
    constexpr int KQ = BK / 4;                       // float4 groups along k
    constexpr int SA = BK + 4;                       // LDS row stride of a [row][k] tile
    constexpr int SBN = BN + 8;                      // LDS row stride of the [k][n] tile (NN)
    constexpr int A_WORDS = BM * SA;
    constexpr int B_WORDS = NT ? BN * SA : BK * SBN;
    constexpr int A_VECS = BM * KQ;                  // float4 groups in an A slab
    constexpr int B_VECS = NT ? BN * KQ : BK * (BN / 4);
    constexpr int A_LOADS = (A_VECS + NTH - 1) / NTH;
    constexpr int B_LOADS = (B_VECS + NTH - 1) / NTH;
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must be built from 32x32 blocks");
    static_assert(BK % 8 == 0, "k slab must be a multiple of 8");
    static_assert(A_VECS % NTH == 0 || A_VECS < NTH, "A slab: whole passes, or a single partial one");
    static_assert(B_VECS % NTH == 0 || B_VECS < NTH, "B slab: whole passes, or a single partial one");
    const bool a_on = (A_VECS >= NTH) || ((int)threadIdx.x < A_VECS);   // thread takes part in staging A
    const bool b_on = (B_VECS >= NTH) || ((int)threadIdx.x < B_VECS);

    // dynamic LDS: [2][A_WORDS] then [2][B_WORDS]; the large tiles need more than the 64 KB a
    // kernel may declare statically
    extern __shared__ __attribute__((aligned(16))) float lds[];
    float(*As)[A_WORDS] = reinterpret_cast<float(*)[A_WORDS]>(lds);
    float(*Bs)[B_WORDS] = reinterpret_cast<float(*)[B_WORDS]>(lds + 2 * A_WORDS);

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = t >> 6;
    const int lr = lane & 31;
    const int lh = lane >> 5;
    const int wm0 = (wave / WAVES_N) * WM;
    const int wn0 = (wave % WAVES_N) * WN;

    const WorkView w = work_view(p, NT);
    int tm, tn;
    tile_of_block(p, w.pid, tm, tn);
    const int m0 = tm * BM;
    const int n0 = tn * BN;
    const int M = p.M, N = p.N, K = w.K;

    // per-thread staging geometry
    const float* a_row[A_LOADS];
    int a_kq[A_LOADS], a_lds[A_LOADS];
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {
        const int f = a_on ? t + i * NTH : 0;
        const int row = f / KQ;
        a_kq[i] = (f % KQ) * 4;
        a_row[i] = w.A + (size_t)min(m0 + row, M - 1) * p.lda;
        a_lds[i] = row * SA + a_kq[i];
    }
    const float* b_row[B_LOADS];
    int b_off[B_LOADS], b_lds[B_LOADS], b_krow[B_LOADS];
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) {
        const int f = b_on ? t + i * NTH : 0;
        if (NT) {
            const int row = f / KQ;
            b_off[i] = (f % KQ) * 4;
            b_row[i] = w.B + (size_t)min(n0 + row, N - 1) * p.ldb;
            b_lds[i] = row * SA + b_off[i];
            b_krow[i] = 0;
        } else {
            b_krow[i] = f / (BN / 4);
            b_off[i] = n0 + (f % (BN / 4)) * 4;
            b_row[i] = w.B;
            b_lds[i] = b_krow[i] * SBN + (f % (BN / 4)) * 4;
        }
    }

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    f32x4 a_st[A_LOADS], b_st[B_LOADS];
    // interior slabs (the whole slab below K and, for the [k][n] tile of NN, the whole tile left
    // of N) load without guards; only the last, ragged slab takes the guarded path
    const bool n_interior = NT || (n0 + BN <= N);
    auto fetch = [&](int k0) {
        if (k0 + BK <= K && n_interior) {
#pragma unroll
            for (int i = 0; i < A_LOADS; ++i)
                if (a_on) a_st[i] = load_k4<VEC, true>(a_row[i], k0 + a_kq[i], K);
#pragma unroll
            for (int i = 0; i < B_LOADS; ++i) {
                if (!b_on) continue;
                if (NT) b_st[i] = load_k4<VEC, true>(b_row[i], k0 + b_off[i], K);
                else b_st[i] = load_n4<VEC, true>(b_row[i], p.ldb, k0 + b_krow[i], K, b_off[i], N);
            }
        } else {
#pragma unroll
            for (int i = 0; i < A_LOADS; ++i)
                if (a_on) a_st[i] = load_k4<VEC, false>(a_row[i], k0 + a_kq[i], K);
#pragma unroll
            for (int i = 0; i < B_LOADS; ++i) {
                if (!b_on) continue;
                if (NT) b_st[i] = load_k4<VEC, false>(b_row[i], k0 + b_off[i], K);
                else b_st[i] = load_n4<VEC, false>(b_row[i], p.ldb, k0 + b_krow[i], K, b_off[i], N);
            }
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i)
            if (a_on) *reinterpret_cast<f32x4*>(&As[buf][a_lds[i]]) = a_st[i];
#pragma unroll
        for (int i = 0; i < B_LOADS; ++i)
            if (b_on) *reinterpret_cast<f32x4*>(&Bs[buf][b_lds[i]]) = b_st[i];
    };

    const int num_slabs = (K + BK - 1) / BK;
    fetch(0);
    stash(0);
    __syncthreads();

    for (int s = 0; s < num_slabs; ++s) {
        const int buf = s & 1;
        const bool more = (s + 1 < num_slabs);
        if (more) fetch((s + 1) * BK);

        const float* as = As[buf];
        const float* bs = Bs[buf];
#pragma unroll
        for (int kk = 0; kk < BK / 8; ++kk) {
            f32x4 af[TM], bf[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[i] = *reinterpret_cast<const f32x4*>(&as[(wm0 + i * 32 + lr) * SA + kk * 8 + lh * 4]);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if (NT) {
                    bf[j] = *reinterpret_cast<const f32x4*>(&bs[(wn0 + j * 32 + lr) * SA + kk * 8 + lh * 4]);
                } else {
                    const float* col = &bs[(kk * 8 + lh * 4) * SBN + wn0 + j * 32 + lr];
                    bf[j].x = col[0];
                    bf[j].y = col[SBN];
                    bf[j].z = col[2 * SBN];
                    bf[j].w = col[3 * SBN];
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i][q], bf[j][q], acc[i][j], 0, 0, 0);
        }

        if (more) stash(buf ^ 1);
        __syncthreads();
    }

    // store: register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32 of its block
    const float no_bias[TN] = {};
    if (whole_lines(w.C, w.ldc))
        store_tile<TM, TN, false, true>(acc, w.C, w.ldc, M, N, m0 + wm0, n0 + wn0, lr, lh, no_bias, 0);
    else
        store_tile<TM, TN, false, false>(acc, w.C, w.ldc, M, N, m0 + wm0, n0 + wn0, lr, lh, no_bias, 0);
}

// ---- the pipelined kernel: global -> LDS by DMA, NSTAGE slabs in flight --------------------------
//
// Same tiling and MFMA blocking as gemm_kernel, different data movement.  Slabs are copied from
// global memory straight into LDS with global_load_lds_dwordx4 (no staging registers, no LDS store
// instructions), NSTAGE slab buffers deep: the copy of slab j is issued while slab j - NSTAGE is
// still being multiplied, so it has NSTAGE - 1 slab times to land.  Each lane's 16 bytes land at
// (wave-uniform LDS base) + 16 * lane, so a wave instruction fills 1 KB of LDS linearly and the
// lane chooses WHICH 16 global bytes it fetches: the tile is stored without padding and with the
// 16-byte chunks of each row XOR-swizzled, which keeps the 128-bit fragment reads conflict-free.
// Fragments are double-buffered in registers: the reads for the next 8 k (or for the first 8 k of
// the next slab, right after the slab barrier) are in flight while the current ones feed the
// matrix cores, so after a barrier the MFMAs restart from registers at once.
//
// Preconditions (checked by the launcher, which otherwise uses gemm_kernel): 16-byte aligned A and
// B, lda and ldb multiples of 4, K a multiple of 4, and for NN also N a multiple of 4 -- every
// 16-byte chunk is then entirely inside or entirely outside the matrix; and leading dimensions small
// enough that byte offsets within one tile fit 32 bits.  Chunks at or beyond K are zeroed in LDS
// after they land; rows beyond m / n (and, for NN, chunks beyond N) are
// clamped to valid ones and only feed outputs that are never stored.

// One 16-byte global -> LDS copy per lane: lane l fetches base + lane_off (a wave-uniform 64-bit
// base and a per-lane unsigned 32-bit byte offset) and its bytes land at lds_base + 16 l.  Per slab
// only the scalar base moves, so a copy costs two scalar and one vector-memory instruction.
__device__ __forceinline__ void dma_chunk_s(const float* base, unsigned lane_off, unsigned lds_base)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(lane_off), "s"(base), "s"(lds_base) : "memory", "m0");
}

// A wave-uniform pointer the compiler may have computed on the vector unit, moved to scalar registers
// (the copies take their base address there).
__device__ __forceinline__ const float* uniform_ptr(const float* p)
{
    const uintptr_t v = reinterpret_cast<uintptr_t>(p);
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
    return reinterpret_cast<const float*>(((uintptr_t)hi << 32) | lo);
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// All of this wave's LDS traffic done, then the workgroup barrier; global loads stay in flight.
// The wait is the compiler's own s_waitcnt (vmcnt and expcnt fields left at "no wait"), so its
// counter bookkeeping knows the fragment registers are valid afterwards; the empty asm statements
// keep memory accesses from being moved across.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// One segment of work of the pipelined kernel: the k range and destination described by `w`, for
// C tile (tm, tn).  The whole workgroup calls it; it leaves no copies in flight, and its last LDS
// accesses (the epilogue's staging) are this wave's own, so a caller that runs several segments
// needs one workgroup barrier between them.
//
// KS = 2: the workgroup has two sets of WAVES_M x WAVES_N waves.  Both sets work on the whole tile;
// of every slab, set 0 multiplies the first half of the k range and set 1 the second half, and at the
// end set 0 adds set 1's accumulators (handed over through LDS) to its own and stores.  A tile that
// has a CU to itself then keeps two waves per SIMD busy instead of one, which hides each wave's waits
// for its fragment reads and barriers behind the other's matrix instructions.
template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, bool NT, int NSTAGE, int EPI = kEpiNone, int KS = 1>
__device__ __forceinline__ void dma_segment(const GemmParams& p, const WorkView& w, const int tm, const int tn)
{
    static_assert(KS == 1 || KS == 2, "one or two sets of waves");
    constexpr int NWT = WAVES_M * WAVES_N;            // waves per set
    constexpr int NW = NWT * KS;
    constexpr int WM = BM / WAVES_M;
    constexpr int WN = BN / WAVES_N;
    constexpr int TM = WM / 32;
    constexpr int TN = WN / 32;
    constexpr int KK = BK / 8;                        // fragment steps per slab
    constexpr int KKG = KK / KS;                      // ... and per set of waves
    constexpr int CPR = BK / 4;                       // 16-byte chunks per [row][k] row
    constexpr int RPL = (CPR >= 16) ? 1 : 16 / CPR;   // rows per 256 bytes of LDS
    constexpr int NCH = BN / 4;                       // chunks per [k][n] row (NN)
    constexpr int A_WORDS = BM * BK;
    constexpr int B_WORDS = BN * BK;
    constexpr int STAGE_WORDS = A_WORDS + B_WORDS;
    constexpr int A_BLOCKS = A_WORDS / 256;           // 1 KB wave copies per slab
    constexpr int B_BLOCKS = B_WORDS / 256;
    // Copies are issued by half of the waves at a time: with 8 waves, waves 0-3 (one per SIMD) feed
    // the even slabs and waves 4-7 the odd ones.  While a wave is busy issuing copies its SIMD
    // partner keeps the matrix core fed, so the issue work is hidden instead of stalling both.
    constexpr int NG = (NW >= 8) ? 2 : 1;             // issuer groups
    constexpr int NI = NW / NG;                       // waves per group
    constexpr int A_LOADS = (A_BLOCKS + NI - 1) / NI;
    constexpr int B_LOADS = (B_BLOCKS + NI - 1) / NI;
    constexpr int LPS = A_LOADS + B_LOADS;            // copies per issuing wave per slab
    static_assert(KK % KS == 0 && KKG >= 2 && KKG % 2 == 0, "an even number of fragment steps per slab and set (register ping-pong)");
    static_assert(KS == 1 || NWT * TM * TN * 1024 <= NSTAGE * STAGE_WORDS, "the accumulators of one set must fit the slab buffers");
    static_assert(A_WORDS % 256 == 0 && B_WORDS % 256 == 0, "slabs must be whole 1 KB blocks");
    static_assert(NSTAGE >= 2 && NSTAGE <= 4, "2..4 slab buffers");
    static_assert(LPS * 2 <= 63, "vmcnt is 6 bits");

    extern __shared__ __attribute__((aligned(16))) float lds[];
    const unsigned lds_base = (unsigned)(uintptr_t)lds;

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int lr = lane & 31;
    const int lh = lane >> 5;
    const int kg = (KS > 1) ? wave / NWT : 0;         // which set of waves: which half of each slab's k range
    const int wpos = (KS > 1) ? wave % NWT : wave;    // position of the wave's block of the tile
    const int wm0 = (wpos / WAVES_N) * WM;
    const int wn0 = (wpos % WAVES_N) * WN;
    // chunk index of the set's first k inside a [row][k] row: one bit above the chunk indices the
    // set's fragment steps run through, so it can be folded into the row's XOR swizzle
    const int kgc = kg * (CPR / KS);

    const int m0 = tm * BM;
    const int n0 = tn * BN;
    const int M = p.M, N = p.N, K = w.K;

    // ---- copy geometry: which global chunk this lane fetches for each of its wave's blocks, as
    // a byte offset from the tile's first row (A) / first row or first k-row (B).  A wave with fewer
    // blocks than copies re-fetches a block another wave also fetches (same bytes to the same
    // place), so every issuing wave issues exactly LPS copies per slab.
    const int grp = wave / NI;
    const int wi = wave % NI;
    // NT with four blocks per wave across n and a 16-byte aligned C: the rows of the B tile are placed
    // in LDS so that block j of lane l works on column TN * l + j, as in the NN kernel (LDS row
    // j * 32 + l of a wave's WN rows holds B row TN * l + j).  The fragment reads do not change, and the
    // epilogue stores TN consecutive words per lane straight from registers instead of going through
    // the LDS patches (256 x 256 tiles: 2-3 us per tile, 1.3 % at k = 1024, 3.4 % at k = 256).
    const bool c_vec = ((reinterpret_cast<uintptr_t>(w.C) & 15) == 0) && ((w.ldc & 3) == 0);
    const bool interleave = NT && TN == 4 && c_vec;
    const float* a_tile = uniform_ptr(w.A + (size_t)m0 * p.lda);
    const float* b_tile = uniform_ptr(NT ? w.B + (size_t)n0 * p.ldb : w.B);
    unsigned a_off[A_LOADS], a_dst[A_LOADS];
    int a_k[A_LOADS];
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {
        const int b = (i * NI + wi) % A_BLOCKS;
        const int u = b * 64 + lane;
        const int row = u / CPR;
        const int slot = u % CPR;
        const int c = slot ^ ((row / RPL) % CPR);
        a_k[i] = c * 4;
        a_off[i] = (unsigned)(((size_t)(min(m0 + row, M - 1) - m0) * p.lda + a_k[i]) * 4);
        a_dst[i] = (unsigned)(b * 1024);
    }
    unsigned b_off[B_LOADS], b_dst[B_LOADS];
    int b_k[B_LOADS];
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) {
        const int b = (i * NI + wi) % B_BLOCKS;
        const int u = b * 64 + lane;
        b_dst[i] = (unsigned)(A_WORDS * 4 + b * 1024);
        if (NT) {
            const int row = u / CPR;
            const int slot = u % CPR;
            const int c = slot ^ ((row / RPL) % CPR);
            b_k[i] = c * 4;
            int brow = row;                                    // which row of B lands in LDS row `row`
            if (interleave) {
                const int local = row % WN;
                brow = row - local + TN * (local % 32) + local / 32;
            }
            b_off[i] = (unsigned)(((size_t)(min(n0 + brow, N - 1) - n0) * p.ldb + b_k[i]) * 4);
        } else {
            const int krow = u / NCH;
            const int slot = u % NCH;
            const int nch = (NCH >= 16) ? (slot ^ (((krow >> 2) & 1) << 3)) : slot;
            const int col = min(n0 + nch * 4, N - 4);          // N % 4 == 0: a whole valid chunk
            b_k[i] = krow;
            b_off[i] = (unsigned)(((size_t)krow * p.ldb + col) * 4);
        }
    }
    const size_t b_step = NT ? (size_t)BK : (size_t)BK * p.ldb;

    // Issue this wave's copies of slab `slab` into buffer `stage`.  In a ragged last slab a chunk at
    // or beyond K is fetched from the last valid chunk instead (a valid address); zero_tail() then
    // overwrites it with zeros once the copy has landed.
    auto issue = [&](int slab, int stage) {
        const int k0 = slab * BK;
        const unsigned base = lds_base + (unsigned)stage * (STAGE_WORDS * 4);
        const float* a_base = a_tile + (size_t)k0;
        const float* b_base = b_tile + (size_t)slab * b_step;
        if (k0 + BK <= K) {
#pragma unroll
            for (int i = 0; i < A_LOADS; ++i) dma_chunk_s(a_base, a_off[i], base + a_dst[i]);
#pragma unroll
            for (int i = 0; i < B_LOADS; ++i) dma_chunk_s(b_base, b_off[i], base + b_dst[i]);
        } else {
            const int kv = K - k0;                           // valid k in this slab, a multiple of 4
#pragma unroll
            for (int i = 0; i < A_LOADS; ++i) {
                const unsigned off = (a_k[i] < kv) ? a_off[i] : a_off[i] - (unsigned)((a_k[i] - (kv - 4)) * 4);
                dma_chunk_s(a_base, off, base + a_dst[i]);
            }
#pragma unroll
            for (int i = 0; i < B_LOADS; ++i) {
                unsigned off = b_off[i];
                if (b_k[i] >= kv)
                    off -= NT ? (unsigned)((b_k[i] - (kv - 4)) * 4)
                              : (unsigned)((size_t)(b_k[i] - (kv - 1)) * p.ldb * 4);
                dma_chunk_s(b_base, off, base + b_dst[i]);
            }
        }
    };
    // after this wave's copies of a ragged slab have landed: zeros over the chunks at or beyond K
    auto zero_tail = [&](int slab, int stage) {
        const int kv = K - slab * BK;
        if (kv >= BK) return;
        float* buf = lds + stage * STAGE_WORDS;
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i)
            if (a_k[i] >= kv) *reinterpret_cast<f32x4*>(buf + a_dst[i] / 4 + lane * 4) = z;
#pragma unroll
        for (int i = 0; i < B_LOADS; ++i)
            if (b_k[i] >= kv) *reinterpret_cast<f32x4*>(buf + b_dst[i] / 4 + lane * 4) = z;
    };
    // does this wave feed slab j?
    auto feeds = [&](int j) { return NG == 1 || (j & 1) == grp; };

    // wait until all but the `newer` most recent slab copies of this wave have landed
    auto wait_newer = [&](int newer) {
        if constexpr (NSTAGE >= 4) {
            if (newer >= 3) { wait_vmcnt<3 * LPS>(); return; }
        }
        if constexpr (NSTAGE >= 3) {
            if (newer == 2) { wait_vmcnt<2 * LPS>(); return; }
        }
        if (newer == 1) wait_vmcnt<LPS>();
        else wait_vmcnt<0>();
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // fragment reads of this set's step kk from buffer `stage`
    auto read_frags = [&](int stage, int kk, f32x4 (&af)[TM], f32x4 (&bf)[TN]) {
        const float* as = lds + stage * STAGE_WORDS;
        const float* bs = as + A_WORDS;
        const int c = kk * 2 + lh;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row = wm0 + i * 32 + lr;
            af[i] = *reinterpret_cast<const f32x4*>(&as[row * BK + ((c ^ ((row / RPL) % CPR) ^ kgc) * 4)]);
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            if (NT) {
                const int row = wn0 + j * 32 + lr;
                bf[j] = *reinterpret_cast<const f32x4*>(&bs[row * BK + ((c ^ ((row / RPL) % CPR) ^ kgc) * 4)]);
            }
        }
        if (!NT) {
            // NN: row krow + s of the [k][n] slab feeds k step s.  A lane reads TN consecutive n
            // (one 128-, 64- or 32-bit LDS load) and uses them for its TN blocks, so block j of lane l
            // works on column wn0 + TN * l + j; the epilogue stores with the same mapping.
            typedef float vecN __attribute__((ext_vector_type(TN)));
            const int krow = (kg * KKG + kk) * 8 + lh * 4;    // rows krow..krow+3 share (krow>>2)&1
            const int sw = (NCH >= 16) ? (((krow >> 2) & 1) << 3) : 0;
            const int col = wn0 + TN * lr;
            const float* q = &bs[krow * BN + (((col >> 2) ^ sw) << 2) + (col & 3)];
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                const vecN v = *reinterpret_cast<const vecN*>(q + st * BN);
#pragma unroll
                for (int j = 0; j < TN; ++j) bf[j][st] = v[j];
            }
        }
    };

    // Ring of NSTAGE buffers, slab j in buffer j % NSTAGE.  Slabs 0 .. NSTAGE-1 are requested before
    // the loop; slab j + NSTAGE is requested right after the barrier that ends the reads of slab j.
    // A wave waits only for copies it issued itself: when it needs slab s + 1 (which it fed iff
    // feeds(s + 1)), the copies it has issued since then are those of the slabs it feeds among
    // s + 2 .. last requested.
    const int num_slabs = (K + BK - 1) / BK;
    const int pre = min(num_slabs, NSTAGE);
    for (int s = 0; s < pre; ++s)
        if (feeds(s)) issue(s, s);
    {
        int newer = 0;
        for (int j = 1; j < pre; ++j) newer += feeds(j) ? 1 : 0;
        if (feeds(0)) {
            wait_newer(newer);
            zero_tail(0, 0);
        }
    }
    lds_barrier();

    f32x4 af[2][TM], bf[2][TN];
    read_frags(0, 0, af[0], bf[0]);

    int stage = 0;
    for (int s = 0; s < num_slabs; ++s) {
        const int next_stage = (stage + 1 == NSTAGE) ? 0 : stage + 1;
#pragma unroll
        for (int kk = 0; kk < KKG; ++kk) {
            const int cur = kk & 1;
            if (kk + 1 < KKG) {
                read_frags(stage, kk + 1, af[cur ^ 1], bf[cur ^ 1]);
            } else {
                // every fragment read of slab s has been issued: after the barrier its buffer is free
                if (s + 1 < num_slabs && feeds(s + 1)) {
                    const int last = min(s + NSTAGE - 1, num_slabs - 1);      // last slab requested so far
                    int newer = 0;
                    for (int j = s + 2; j <= last; ++j) newer += feeds(j) ? 1 : 0;
                    wait_newer(newer);
                    zero_tail(s + 1, next_stage);
                }
                lds_barrier();
                if (s + NSTAGE < num_slabs && feeds(s + NSTAGE)) issue(s + NSTAGE, stage);
                if (s + 1 < num_slabs) read_frags(next_stage, 0, af[cur ^ 1], bf[cur ^ 1]);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[cur][i][q], bf[cur][j][q], acc[i][j], 0, 0, 0);
        }
        stage = next_stage;
    }

    if constexpr (KS > 1) {
        // set 1 hands its accumulators to set 0 through the slab buffers (free once every wave has passed
        // the first barrier): register r of block (i, j) of the wave at position wpos, lane by lane
        float* red = lds + (size_t)wpos * (TM * TN * 1024) + lane;
        lds_barrier();
        if (kg != 0) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) red[((i * TN + j) * 16 + r) * 64] = acc[i][j][r];
        }
        lds_barrier();
        if (kg == 0) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][j][r] += red[((i * TN + j) * 16 + r) * 64];
        }
        lds_barrier();        // the sums are in registers: LDS may be reused (store patches, the next segment's copies)
        if (kg != 0) return;
    }

    // epilogue: interior tiles of a 16-byte-aligned C go through wave-private LDS patches (the slab
    // buffers are free once every wave has passed this barrier)
    // (split-k partial products of a few MB are read back at once by the kernel that adds them: ordinary
    //  stores, so that they are still in the caches then)
    const bool stream = !(p.splits > 1 && p.part_cached) && whole_lines(w.C, w.ldc);
    // kEpiBiasAct: the bias of the lane's column of each block (the block -> column mapping of the stores),
    // added, and the clamp applied, as each value is stored: the same two operations on the same fp32
    // values as a separate pass over C
    constexpr bool BIAS = (EPI == kEpiBiasAct);
    float bv[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        bv[j] = 0.f;
        if (BIAS) {
            const int col = (NT && !interleave) ? n0 + wn0 + j * 32 + lr : n0 + wn0 + TN * lr + j;
            if (col < N) bv[j] = p.bias[col];
        }
    }
    const int relu = BIAS ? p.relu : 0;
    if constexpr (EPI == kEpiSgd) {
        static_assert(!NT, "the fused update exists for the NN kernel only");
        const bool w_vec = c_vec && ((reinterpret_cast<uintptr_t>(p.W) & 15) == 0) && ((p.ldw & 3) == 0);
        store_tile_interleaved_sgd<TM, TN>(acc, w.C, w.ldc, p.W, p.ldw, p.lr, M, N, m0 + wm0, n0 + wn0, lr, lh, w_vec);
    } else if (!NT || interleave) {
        if (stream)
            store_tile_interleaved<TM, TN, BIAS, true>(acc, w.C, w.ldc, M, N, m0 + wm0, n0 + wn0, lr, lh, c_vec, bv, relu);
        else
            store_tile_interleaved<TM, TN, BIAS, false>(acc, w.C, w.ldc, M, N, m0 + wm0, n0 + wn0, lr, lh, c_vec, bv, relu);
    } else {
        if constexpr (KS == 1) lds_barrier();       // (KS = 2: every wave has passed the barriers above)
        if (c_vec && m0 + BM <= M && n0 + BN <= N) {
            if (stream)
                store_tile_staged<TM, TN, BIAS, true>(acc, w.C, w.ldc, m0 + wm0, n0 + wn0, lane, lds + wave * (16 * (WN + 8)), bv, relu);
            else
                store_tile_staged<TM, TN, BIAS, false>(acc, w.C, w.ldc, m0 + wm0, n0 + wn0, lane, lds + wave * (16 * (WN + 8)), bv, relu);
        } else if (stream) {
            store_tile<TM, TN, BIAS, true>(acc, w.C, w.ldc, M, N, m0 + wm0, n0 + wn0, lr, lh, bv, relu);
        } else {
            store_tile<TM, TN, BIAS, false>(acc, w.C, w.ldc, M, N, m0 + wm0, n0 + wn0, lr, lh, bv, relu);
        }
    }
}

template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, bool NT, int NSTAGE, int EPI = kEpiNone, int KS = 1>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64 * KS) void gemm_dma_kernel(GemmParams p)
{
    const WorkView w = work_view(p, NT);
    int tm, tn;
    tile_of_block(p, w.pid, tm, tn);
    dma_segment<BM, BN, BK, WAVES_M, WAVES_N, NT, NSTAGE, EPI, KS>(p, w, tm, tn);
}

// ---- even split of the whole k x tiles work over a fixed number of workgroups -------------------
//
// When the tiles of C do not fill the machine evenly (72 tiles of 256 x 256 on 256 CUs, or 288), the
// work is cut differently: every tile's k range is divided into units of kSplitQuantum, all units of
// all tiles are laid in one line (tile after tile), and workgroup w of G takes the w-th equal piece
// of that line.  A piece covers the end of one tile, possibly some whole tiles, and the start of
// another: the workgroup runs one segment per tile it touches.  Whole tiles go straight to C; a
// partial one goes to the workgroup's scratch slot (2 w for a segment that starts inside a tile,
// 2 w + 1 for one that starts a tile but does not finish it) and streamk_fixup_kernel adds the
// pieces of each cut tile in k order.  The cut depends only on (configuration, m, n, k), so results
// stay reproducible.
struct StreamKCut {
    int units;            // tiles x units_per_tile (the launcher keeps it below 2^31)
    int units_per_tile;
    int groups;           // G
    __host__ __device__ int bound(int w) const { return (int)((long long)units * w / groups); }
};

// workgroup ids are dealt round robin to the XCDs; give each XCD a contiguous run of pieces
__device__ __forceinline__ int streamk_piece_of_block(int block, int groups, int num_xcd)
{
    if (num_xcd <= 1 || groups % num_xcd != 0) return block;
    return (block % num_xcd) * (groups / num_xcd) + block / num_xcd;
}

template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, bool NT, int NSTAGE, int KS = 1>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64 * KS) void gemm_streamk_kernel(GemmParams p)
{
    const StreamKCut cut = {p.tiles_m * p.tiles_n * p.sk_units_per_tile, p.sk_units_per_tile, (int)gridDim.x};
    const int piece = streamk_piece_of_block((int)blockIdx.x, cut.groups, p.num_xcd);
    GemmParams q = p;
    q.num_xcd = 1;                                   // tiles are already walked in order: bands only
    // (the divisions run on the vector unit; readfirstlane tells the compiler the results are wave-uniform)
    int u = __builtin_amdgcn_readfirstlane(cut.bound(piece));
    const int u_end = __builtin_amdgcn_readfirstlane(cut.bound(piece + 1));
    bool first = true;
    while (u < u_end) {
        const int tile = __builtin_amdgcn_readfirstlane(u / cut.units_per_tile);
        const int s0 = u - tile * cut.units_per_tile;
        const int left = u_end - u;
        const int s1 = (left < cut.units_per_tile - s0) ? s0 + left : cut.units_per_tile;
        int tm, tn;
        tile_of_block(q, tile, tm, tn);
        const int k0 = s0 * kSplitQuantum;
        const int k1 = min(p.K, s1 * kSplitQuantum);
        WorkView w;
        w.pid = tile;
        w.K = k1 - k0;
        w.A = p.A + k0;
        w.B = NT ? p.B + k0 : p.B + (size_t)k0 * p.ldb;
        if (s0 == 0 && s1 == cut.units_per_tile) {
            w.C = p.C;
            w.ldc = p.ldc;
        } else {
            // a dense BM x BN slot; the epilogue adds (tile row origin) x ldc + (tile column origin)
            float* slot = p.part + (size_t)(2 * piece + (s0 == 0 ? 1 : 0)) * (BM * BN);
            w.C = slot - ((size_t)tm * BM * BN + (size_t)tn * BN);
            w.ldc = BN;
        }
        if (!first) lds_barrier();
        first = false;
        dma_segment<BM, BN, BK, WAVES_M, WAVES_N, NT, NSTAGE, kEpiNone, KS>(q, w, tm, tn);
        u += s1 - s0;
    }
}

// C tile = sum of its pieces in k order, for every tile that was cut.  kFixChunks workgroups of 256
// threads per tile, each taking a band of BM / kFixChunks rows.
constexpr int kFixMaxPieces = 8;      // pieces of one tile summed per pass (more: further passes)

template <int BM, int BN>
__global__ __launch_bounds__(256) void streamk_fixup_kernel(GemmParams p, int groups)
{
    const StreamKCut cut = {p.tiles_m * p.tiles_n * p.sk_units_per_tile, p.sk_units_per_tile, groups};
    const int tile = blockIdx.x / kFixChunks;
    const int chunk = blockIdx.x % kFixChunks;
    const int ub = tile * cut.units_per_tile, ue = ub + cut.units_per_tile;
    int w0 = (int)((long long)ub * groups / cut.units);
    while (w0 > 0 && cut.bound(w0) > ub) --w0;
    while (w0 + 1 < groups && cut.bound(w0 + 1) <= ub) ++w0;
    if (cut.bound(w0) <= ub && cut.bound(w0 + 1) >= ue) return;      // one workgroup did the whole tile
    GemmParams q = p;
    q.num_xcd = 1;
    int tm, tn;
    tile_of_block(q, tile, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const bool vec = ((reinterpret_cast<uintptr_t>(p.C) & 15) == 0) && ((p.ldc & 3) == 0) && (n0 + BN <= p.N);
    constexpr int ROWS = BM / kFixChunks;
    const int r_first = chunk * ROWS;
    int w = w0;
    bool have_sum = false;                    // later passes continue from what is already in C
    while (w < groups && cut.bound(w) < ue) {
        // the next (up to kFixMaxPieces) pieces of this tile
        const float* slot[kFixMaxPieces];
        int np = 0;
        for (; w < groups && cut.bound(w) < ue && np < kFixMaxPieces; ++w) {
            const int a = cut.bound(w) > ub ? cut.bound(w) : ub;
            const int b = cut.bound(w + 1) < ue ? cut.bound(w + 1) : ue;
            if (a >= b) continue;
            slot[np++] = p.part + (size_t)(2 * w + (a == ub ? 1 : 0)) * (BM * BN);
        }
        for (int e = threadIdx.x; e < ROWS * BN / 4; e += 256) {
            const int r = r_first + e / (BN / 4);
            const int c = (e % (BN / 4)) * 4;
            if (m0 + r >= p.M || n0 + c >= p.N) continue;
            float* dst = p.C + (size_t)(m0 + r) * p.ldc + n0 + c;
            f32x4 v[kFixMaxPieces];
#pragma unroll
            for (int j = 0; j < kFixMaxPieces; ++j)
                if (j < np) v[j] = *reinterpret_cast<const f32x4*>(slot[j] + (size_t)r * BN + c);
            f32x4 acc;
            if (have_sum) {
                if (vec) acc = *reinterpret_cast<const f32x4*>(dst);
                else {
                    acc.x = dst[0];
                    acc.y = (n0 + c + 1 < p.N) ? dst[1] : 0.f;
                    acc.z = (n0 + c + 2 < p.N) ? dst[2] : 0.f;
                    acc.w = (n0 + c + 3 < p.N) ? dst[3] : 0.f;
                }
                acc += v[0];
            } else {
                acc = v[0];
            }
#pragma unroll
            for (int j = 1; j < kFixMaxPieces; ++j)
                if (j < np) acc += v[j];
            if (vec) {
                *reinterpret_cast<f32x4*>(dst) = acc;
            } else {
                dst[0] = acc.x;
                if (n0 + c + 1 < p.N) dst[1] = acc.y;
                if (n0 + c + 2 < p.N) dst[2] = acc.z;
                if (n0 + c + 3 < p.N) dst[3] = acc.w;
            }
        }
        have_sum = true;
    }
}

// ---- split-k reduction ---------------------------------------------------------------------------

// C[i][j] = part[0][i][j] + part[1][i][j] + ... in split order (fixed, so results are reproducible)
// EPI = kEpiBiasAct: ... then the column's bias and the clamp, as in the fused epilogue of the kernel
// The partial products are loaded in batches of eight (then four, two, one for what is left) before
// any of a batch is added, so that a lane waits for one round trip to memory per batch instead of one
// per split (the additions keep their order).
// One element per lane: the kernel is bound by that round trip, and four elements per lane (a quarter
// of the waves) measured 0.5-1.5 us slower on results of 10^4 to 10^6 elements.
// while at least B splits are left: load the next B partial products, then add them in split order
template <int B>
__device__ __forceinline__ void reduce_batch(const float* __restrict__ part, long long total, long long e, int splits,
                                             int& s, float& acc)
{
    for (; s + B <= splits; s += B) {
        float v[B];
#pragma unroll
        for (int u = 0; u < B; ++u) v[u] = part[(size_t)(s + u) * total + e];
#pragma unroll
        for (int u = 0; u < B; ++u) acc += v[u];
    }
}

template <int EPI>
__global__ __launch_bounds__(256) void reduce_splits_kernel(const float* __restrict__ part, int splits,
                                                            int M, int N, float* __restrict__ C, long ldc,
                                                            const float* __restrict__ bias, int relu)
{
    const long long total = (long long)M * N;
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (long long)gridDim.x * blockDim.x) {
        float acc = part[e];
        int s = 1;
        reduce_batch<8>(part, total, e, splits, s, acc);
        reduce_batch<4>(part, total, e, splits, s, acc);
        reduce_batch<2>(part, total, e, splits, s, acc);
        reduce_batch<1>(part, total, e, splits, s, acc);
        const long long i = e / N;
        const long long j = e - i * N;
        if (EPI == kEpiBiasAct) {
            acc += bias[j];
            if (relu) acc = acc > 0.f ? acc : 0.f;
        }
        C[(size_t)i * ldc + j] = acc;
    }
}
}  // namespace mtnn

// Launcher of the fp32 GEMM kernels: picks the kernel instance for a (configuration, division of
// the work) pair, sizes its LDS request, and enqueues it with the reduction / fix-up kernel that a
// divided launch needs.  The kernels are in gemm_kernels.h (instantiated per tile geometry in
// gemm_inst_*.hip), the configurations and the rule that chooses among them in gemm_cost.cpp.
#include "gemm_kernels.h"

#include <atomic>
#include <mutex>

namespace mtnn {

static std::atomic<long long> g_streamk_launches{0};
long long gemm_streamk_launches() { return g_streamk_launches.load(); }
static std::atomic<long long> g_fused_launches{0};
long long gemm_fused_launches() { return g_fused_launches.load(); }

static const KernelSet* kernel_sets()
{
    static KernelSet table[kNumKernelSets];
    static std::once_flag once;
    std::call_once(once, [] {
        fill_kernel_sets_a(table);
        fill_kernel_sets_b(table);
        fill_kernel_sets_c(table);
        fill_kernel_sets_d(table);
        fill_kernel_sets_e(table);
    });
    return table;
}

// opt a kernel in to the large LDS carve-out, once per kernel and device
static hipError_t raise_lds_limit(const void* kern, int dev, int lds_per_cu)
{
    constexpr int kSlots = 256;
    struct Seen { std::atomic<const void*> kern; std::atomic<int> devmask; };
    static Seen seen[kSlots] = {};
    const int bit = (dev >= 0 && dev < 31) ? (1 << dev) : 0;
    // open addressing on the kernel's address; a full table or a racing caller at worst sets the attribute again
    size_t h = (reinterpret_cast<uintptr_t>(kern) >> 4) % kSlots;
    for (int probe = 0; probe < kSlots; ++probe, h = (h + 1) % kSlots) {
        const void* cur = seen[h].kern.load();
        if (cur == kern) {
            if (bit && (seen[h].devmask.load() & bit)) return hipSuccess;
            break;
        }
        if (cur == nullptr) {
            const void* expected = nullptr;
            if (seen[h].kern.compare_exchange_strong(expected, kern) || expected == kern) break;
        }
    }
    const hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_per_cu);
    if (e != hipSuccess) return e;
    if (seen[h].kern.load() == kern && bit) seen[h].devmask.fetch_or(bit);
    return hipSuccess;
}

int launch_gemm(hipStream_t s, const Geometry& geo, const Scratch& scratch, int op, int cfg, int splits, int m, int n, int k,
                const float* A, long lda, const float* B, long ldb, float* C, long ldc,
                const Epilogue* epi, bool* fused)
{
    if (fused) *fused = false;
    if (op != OP_NN && op != OP_NT) return (int)hipErrorInvalidValue;
    const int kind = epi ? epi->kind : kEpiNone;
    if (kind != kEpiNone && kind != kEpiBiasAct && kind != kEpiSgd) return (int)hipErrorInvalidValue;
    // splits: >= 1 as given; kStreamK the even cut; any other value <= 0 leaves the choice to the rule
    const bool free_splits = (splits <= 0 && splits != kStreamK);
    const bool chunks16 = (lda % 4 == 0) && (ldb % 4 == 0) && (k % 4 == 0) && (op == OP_NT || n % 4 == 0) &&
                          ((reinterpret_cast<uintptr_t>(A) & 15) == 0) && ((reinterpret_cast<uintptr_t>(B) & 15) == 0);
    const size_t room = scratch.ptr ? scratch.bytes : 0;
    if (cfg < 0) {
        const Choice ch = choose(geo, op, m, n, k, free_splits, chunks16, kind, room);
        cfg = ch.cfg;
        if (free_splits) splits = ch.splits;
    } else if (free_splits) {
        splits = 1;
    }
    if (cfg >= kNumTileConfigs || splits > kMaxSplits) return (int)hipErrorInvalidValue;
    const bool want_streamk = (splits == kStreamK);
    if (splits < 1) splits = 1;
    const TileConfig& c = kTileConfigs[cfg];
    const KernelSet& ks = kernel_sets()[c.kernel_set];
    const int occ = c.wg_per_cu(geo.lds_per_cu);
    GemmParams p;
    p.A = A; p.B = B; p.C = C;
    p.M = m; p.N = n; p.K = k;
    p.lda = lda; p.ldb = ldb; p.ldc = ldc;
    p.tiles_m = (m + c.bm - 1) / c.bm;
    p.tiles_n = (n + c.bn - 1) / c.bn;
    p.group_m = p.tiles_m < 8 ? p.tiles_m : 8;
    p.num_xcd = geo.xcds;
    // split-k: equal k ranges, multiples of the quantum; splits that would be empty are dropped
    p.splits = 1;
    p.k_per_split = k;
    p.part = nullptr;
    p.part_cached = 0;
    p.sk_units_per_tile = 0;
    p.bias = (kind == kEpiBiasAct) ? epi->bias : nullptr;
    p.relu = (kind == kEpiBiasAct) ? epi->relu : 0;
    p.W = (kind == kEpiSgd) ? epi->W : nullptr;
    p.ldw = (kind == kEpiSgd) ? epi->ldw : 0;
    p.lr = (kind == kEpiSgd) ? epi->lr : 0.f;
    set_tile_order(p);
    if (splits > 1) {
        int eff_splits = 1, kps = k;
        effective_splits(k, splits, &eff_splits, &kps);
        if (eff_splits > 1) {
            if ((size_t)m * n * eff_splits * sizeof(float) > room) return kErrScratch;
            p.splits = eff_splits;
            p.k_per_split = kps;
            p.part = scratch.ptr;
            // Partial products of up to 8 MiB are written with ordinary stores: the kernel that adds them
            // runs next and finds them in the caches (NT, 64 x 64 tiles: 128 x 128 x 4096 12.8 -> 11.8 us,
            // 64 x 64 x 8192 14.7 -> 13.8 us); larger ones stream past the caches as results do.
            p.part_cached = ((size_t)m * n * eff_splits * sizeof(float) <= ((size_t)8 << 20)) ? 1 : 0;
        }
    }
    const long long total = (long long)p.tiles_m * p.tiles_n * p.splits;
    if (total > 0x7fffffffLL) return (int)hipErrorInvalidValue;
    const bool vec = (lda % 4 == 0) && (ldb % 4 == 0) &&
                     ((reinterpret_cast<uintptr_t>(A) & 15) == 0) &&
                     ((reinterpret_cast<uintptr_t>(B) & 15) == 0);
    // the pipelined kernel needs whole 16-byte chunks everywhere (see its preconditions) ...
    // ... and per-lane byte offsets inside a tile that fit 32 bits
    const unsigned long long lim = 1ull << 32;
    const bool off_ok = (unsigned long long)c.bm * (unsigned long long)lda * 4ull < lim &&
                        (op == OP_NT ? (unsigned long long)c.bn * (unsigned long long)ldb * 4ull < lim
                                     : (unsigned long long)(c.bk + 1) * (unsigned long long)ldb * 4ull < lim);
    const bool dma_ok = vec && (k % 4 == 0) && (op == OP_NT || n % 4 == 0) && off_ok;
    if (want_streamk && dma_ok) {
        // the even cut: (CUs x workgroups per CU) pieces, if there is at least one unit for each;
        // otherwise the plain launch below
        const int groups = geo.cus * occ;
        const int units_per_tile = (k + kSplitQuantum - 1) / kSplitQuantum;
        const long long units = (long long)p.tiles_m * p.tiles_n * units_per_tile;
        if (units >= groups && units < 0x7fffffffLL) {
            if (scratch_needed(geo, cfg, kStreamK, m, n, k) > room) return kErrScratch;
            p.part = scratch.ptr;
            p.sk_units_per_tile = units_per_tile;
            size_t lds_sk = c.lds_bytes_dma();
            const size_t share = ((size_t)geo.lds_per_cu / (size_t)occ) & ~(size_t)1023;
            if (lds_sk < share - 1024) lds_sk = share - 1024;
            if (lds_sk > 64 * 1024) {
                const hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(ks.sk[op]), geo.device, geo.lds_per_cu);
                if (e != hipSuccess) return (int)e;
            }
            hipLaunchKernelGGL(ks.sk[op], dim3((unsigned)groups), dim3(c.threads), lds_sk, s, p);
            hipError_t err = hipGetLastError();
            if (err != hipSuccess) return (int)err;
            hipLaunchKernelGGL(ks.fix, dim3((unsigned)(p.tiles_m * p.tiles_n * kFixChunks)), dim3(256), 0, s, p, groups);
            ++g_streamk_launches;
            return (int)hipGetLastError();
        }
    }
    // A fused epilogue runs in the pipelined kernel's instance built for it (unsplit launches), or, for
    // the bias + activation, in the reduction kernel of a split launch; anything else is left to the caller.
    const bool fuse_reduce = (kind == kEpiBiasAct) && p.splits > 1;
    const bool fuse_main = p.splits == 1 && dma_ok &&
                           ((kind == kEpiBiasAct && ks.dma_bias[op]) || (kind == kEpiSgd && op == OP_NN && ks.dma_sgd));
    GemmKernel kern = fuse_main ? (kind == kEpiBiasAct ? ks.dma_bias[op] : ks.dma_sgd)
                                : dma_ok ? ks.dma[op] : ks.kern[op][vec ? 1 : 0];
    size_t lds = dma_ok ? c.lds_bytes_dma() : c.lds_bytes_guarded(op);
    if (dma_ok) {
        // Ask for at least 1/want of the CU's LDS, want = the workgroups a CU should hold at a time (the
        // configuration's limit, or fewer if the grid has fewer per CU): no CU can then take more than
        // the cost model assumed, so a grid of exactly CUs x want workgroups spreads evenly instead of
        // piling three on some CUs and one on others.
        long long per_cu_wgs = (total + geo.cus - 1) / geo.cus;
        int want = occ;
        if (p.k_per_split <= c.bk && c.threads == c.threads_guarded) {
            // The whole k range is one slab: only the first slab buffer is ever touched, so the request
            // shrinks to it (or to the epilogue's patches) and a CU may hold more workgroups -- as many as
            // the registers allow, four for these kernels -- which hides more of the one global -> LDS
            // round trip each workgroup waits for ((8192, 8192, 32) NT: 65 -> 61 us on 128 x 64 tiles).
            const size_t ring1 = (size_t)(c.bm + c.bn) * c.bk * sizeof(float);
            const size_t patches = (size_t)(c.threads / 64) * 16 * (size_t)(c.bn / c.waves_n + 8) * sizeof(float);
            lds = ring1 > patches ? ring1 : patches;
            want = 5;
        }
        if (per_cu_wgs < want) want = (int)per_cu_wgs;
        if (want < 1) want = 1;
        const size_t share = ((size_t)geo.lds_per_cu / (size_t)want) & ~(size_t)1023;
        const size_t floor_bytes = share > 1024 ? share - 1024 : share;
        if (lds < floor_bytes) lds = floor_bytes;
    }
    if (lds > 64 * 1024) {
        // (the limit is raised to the CU's whole LDS: the request above varies with the grid)
        const hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(kern), geo.device, geo.lds_per_cu);
        if (e != hipSuccess) return (int)e;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)total), dim3(dma_ok ? c.threads : c.threads_guarded), lds, s, p);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return (int)err;
    if (p.splits > 1) {
        const long long elems = (long long)m * n;
        long long blocks = (elems + 255) / 256;
        if (blocks > 2048) blocks = 2048;
        if (fuse_reduce)
            hipLaunchKernelGGL(reduce_splits_kernel<kEpiBiasAct>, dim3((unsigned)blocks), dim3(256), 0, s,
                               p.part, p.splits, m, n, C, ldc, p.bias, p.relu);
        else
            hipLaunchKernelGGL(reduce_splits_kernel<kEpiNone>, dim3((unsigned)blocks), dim3(256), 0, s,
                               p.part, p.splits, m, n, C, ldc, nullptr, 0);
        err = hipGetLastError();
    }
    if (err == hipSuccess && (fuse_main || fuse_reduce)) {
        ++g_fused_launches;
        if (fused) *fused = true;
    }
    return (int)err;
}

}  // namespace mtnn

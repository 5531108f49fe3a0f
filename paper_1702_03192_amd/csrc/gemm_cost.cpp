// The tile configurations of the fp32 GEMM kernels, the numbers fitted to their measured times,
// and the rule that picks configuration and split count per shape.  Host-only code with no kernels
// in it: changing a constant here recompiles this file alone.
//
// Where the numbers come from: tune.py `collect` times every configuration x split count on the
// {64..8192}^3 grid, `fit` does the per-configuration least-squares fits printed in the table below
// (the rows the fits use are kept in data/gemm_fit_rows_gfx950.csv).
#include "gemm_config.h"

#include <cmath>

namespace mtnn {

// pipelined kernel with NS slab buffers, and the guarded kernel (slab GBK) that serves what it cannot
#define MTNN_TILE_KS(SET, BM, BN, BK, WMV, WNV, KS, KSNAME, NS, GBK, MAXWG, EFF_NN, RND_NN, EFF_NT, RND_NT, GEFF_NN, GRND_NN, GEFF_NT, GRND_NT) \
    { #BM "x" #BN "x" #BK "_w" #WMV "x" #WNV KSNAME "_dma" #NS "_x" #MAXWG, BM, BN, BK, GBK, NS, WMV * WNV * 64 * KS, WMV * WNV * 64, WNV, MAXWG, SET, \
      BK != 16, {EFF_NN, EFF_NT}, {RND_NN, RND_NT}, {GEFF_NN, GEFF_NT}, {GRND_NN, GRND_NT} }
#define MTNN_TILE(SET, BM, BN, BK, WMV, WNV, NS, GBK, MAXWG, EFF_NN, RND_NN, EFF_NT, RND_NT, GEFF_NN, GRND_NN, GEFF_NT, GRND_NT) \
    MTNN_TILE_KS(SET, BM, BN, BK, WMV, WNV, 1, "", NS, GBK, MAXWG, EFF_NN, RND_NN, EFF_NT, RND_NT, GEFF_NN, GRND_NN, GEFF_NT, GRND_NT)

const TileConfig kTileConfigs[] = {
    //  set   tile         waves stages    per CU   NN: eff, round      NT: eff, round       guarded kernel: NN, NT
    MTNN_TILE(0, 256, 256, 32, 4, 2, 2, 16,   1,   0.951f, 12.9e-6f,   0.948f, 12.4e-6f,   0.871f, 12.7e-6f, 0.842f, 11.5e-6f),  // 0: 8 waves of 64 x 128, 128 KB of LDS
    // (1: the fits put it level with configuration 0 inside the grid (0.953 / 0.944); beyond it the narrower tile
    //  re-reads more of A and falls behind -- NN 135 against 148 TFLOP/s at 65536^3, NT 139 against 148 at
    //  65536 x 256 x 32768 and 146 against 149 at 16384^3.  Its time is also the one that moves between
    //  machines and sessions: NN (4096, 4096, 1024) 242-247 us where the table was collected, 270-275 us in
    //  five later sessions on other MI355X boxes, while configurations 0 and 10 stayed at 245 and 248-252 us
    //  on both.  A lead of 1 % on a good day does not pay for 12 % on a bad one, so it is rated below them.)
    MTNN_TILE(1, 256, 128, 16, 2, 2, 3, 16,   2,   0.925f, 10.8e-6f,   0.925f, 11.9e-6f,   0.840f, 9.8e-6f, 0.848f, 10.6e-6f),  // 1: 4 waves of 128 x 64, 72 KB
    MTNN_TILE(2, 128, 128, 64, 4, 2, 2, 16,   1,   0.890f, 3.4e-6f,   0.890f, 3.1e-6f,   0.802f, 2.1e-6f, 0.776f, 2.0e-6f),   // 2: 8 waves of 32 x 64, 128 KB
    // (3: the fit gives 2.0 / 1.2 us per round; with that the rule takes this tile for short-k products of a
    //  single round where the three-per-CU tiles measure 5-10 % faster, so its rounds are rated a little dearer)
    MTNN_TILE(3, 64, 64, 64, 2, 2, 2, 16,     2,   0.882f, 2.6e-6f,   0.854f, 1.9e-6f,   0.688f, 1.1e-6f, 0.680f, 1.1e-6f),   // 3: 4 waves of 32 x 32, 64 KB
    MTNN_TILE(4, 32, 256, 32, 1, 4, 2, 16,    2,   0.901f, 2.2e-6f,   0.888f, 2.1e-6f,   0.698f, 1.7e-6f, 0.621f, 2.0e-6f),   // 4: 4 waves of 32 x 64 (small m), 72 KB
    MTNN_TILE(5, 256, 32, 32, 4, 1, 2, 16,    2,   0.824f, 3.2e-6f,   0.883f, 2.4e-6f,   0.567f, 1.9e-6f, 0.535f, 1.4e-6f),   // 5: 4 waves of 64 x 32 (small n), 72 KB
    MTNN_TILE(6, 128, 256, 32, 2, 4, 2, 16,   1,   0.934f, 6.2e-6f,   0.934f, 6.2e-6f,   0.822f, 5.9e-6f, 0.795f, 4.0e-6f),   // 6: 8 waves of 64 x 64, 96 KB
    MTNN_TILE(7, 256, 128, 32, 4, 2, 2, 16,   1,   0.925f, 6.5e-6f,   0.928f, 6.4e-6f,   0.837f, 4.8e-6f, 0.805f, 4.5e-6f),   // 7: 8 waves of 64 x 64, 96 KB
    MTNN_TILE(8, 128, 64, 32, 2, 2, 2, 16,    2,   0.912f, 3.3e-6f,   0.908f, 1.8e-6f,   0.740f, 1.9e-6f, 0.728f, 2.0e-6f),   // 8: 4 waves of 64 x 32, 48 KB
    MTNN_TILE(9, 64, 128, 32, 2, 2, 2, 16,    2,   0.912f, 2.4e-6f,   0.912f, 1.9e-6f,   0.783f, 2.0e-6f, 0.743f, 1.8e-6f),   // 9: 4 waves of 32 x 64, 48 KB
    MTNN_TILE(10, 128, 128, 32, 2, 2, 2, 16,  2,   0.932f, 4.7e-6f,   0.943f, 4.7e-6f,   0.820f, 4.2e-6f, 0.789f, 4.3e-6f),   // 10: 4 waves of 64 x 64, 64 KB
    MTNN_TILE(8, 128, 64, 32, 2, 2, 2, 16,    3,   0.907f, 3.5e-6f,   0.901f, 1.9e-6f,   0.753f, 2.1e-6f, 0.734f, 2.3e-6f),   // 11: as 8, three per CU (small k)
    MTNN_TILE(9, 64, 128, 32, 2, 2, 2, 16,    3,   0.915f, 2.6e-6f,   0.917f, 2.2e-6f,   0.807f, 2.2e-6f, 0.745f, 1.9e-6f),   // 12: as 9, three per CU (small k)
    // (13: fitted 2.7 / 1.7 us per round, 0.7 / 0.5 above configuration 3's fit; rated that much above
    //  configuration 3's compiled-in figures, so that the two keep their measured order)
    MTNN_TILE_KS(11, 64, 64, 64, 2, 2, 2, "k2", 2, 16,  2,   0.884f, 3.3e-6f,   0.879f, 2.4e-6f,   0.688f, 1.1e-6f, 0.680f, 1.1e-6f),   // 13: as 3 with two sets of 4 waves, each on half of every slab's k
    MTNN_TILE_KS(12, 32, 256, 32, 1, 4, 2, "k2", 2, 16, 2,   0.897f, 3.1e-6f,   0.880f, 2.8e-6f,   0.698f, 1.7e-6f, 0.621f, 2.0e-6f),   // 14: as 4 with two sets of 4 waves
    MTNN_TILE_KS(13, 256, 32, 32, 4, 1, 2, "k2", 2, 16, 2,   0.862f, 4.3e-6f,   0.873f, 2.7e-6f,   0.567f, 1.9e-6f, 0.535f, 1.4e-6f),   // 15: as 5 with two sets of 4 waves
};
const int kNumTileConfigs = (int)(sizeof(kTileConfigs) / sizeof(kTileConfigs[0]));

// fp32 matrix rate of one compute unit: 256 flop per clock (four SIMDs, one 32x32x2 MFMA per 16
// passes of 4 clocks each) at the 2.4 GHz peak clock; the fitted `eff` figures are fractions of it
constexpr double kPeakPerCu = 256.0 * 2.4e9;

void effective_splits(int k, int splits, int* eff_splits, int* k_per_split)
{
    if (splits <= 1) { *eff_splits = 1; *k_per_split = k; return; }
    int kps = (k + splits - 1) / splits;
    kps = ((kps + kSplitQuantum - 1) / kSplitQuantum) * kSplitQuantum;
    *eff_splits = (k + kps - 1) / kps;
    *k_per_split = kps;
    if (*eff_splits <= 1) { *eff_splits = 1; *k_per_split = k; }
}

size_t scratch_needed(const Geometry& geo, int cfg, int splits, int m, int n, int k)
{
    if (splits == kStreamK) {
        const TileConfig& c = kTileConfigs[cfg];
        const size_t groups = (size_t)geo.cus * (size_t)c.wg_per_cu(geo.lds_per_cu);
        return 2 * groups * (size_t)c.bm * (size_t)c.bn * sizeof(float);
    }
    int eff = 1, kps = k;
    effective_splits(k, splits, &eff, &kps);
    return eff > 1 ? (size_t)m * (size_t)n * (size_t)eff * sizeof(float) : 0;
}

// A small cost model, evaluated for every configuration and split count; the cheapest wins, ties go
// to the earlier (larger) configuration.  For a candidate: workgroups = tiles x splits are dealt
// evenly to the CUs; a CU works through its share at the configuration's fitted k-loop rate, less if
// it holds fewer workgroups than it could overlap; every round of resident workgroups pays the
// configuration's fitted time outside the k loop (first copies, result store);
// split-k adds the traffic of writing and re-reading the partial products.  The choice depends only
// on (op, m, n, k), the device's geometry and the scratch capacity, never on timing, so results stay
// reproducible.
static double predicted_seconds(const Geometry& geo, const TileConfig& c, int op, int m, int n, int k, int splits, bool pipelined)
{
    const long long cus = geo.cus;
    const long long tiles = (long long)((m + c.bm - 1) / c.bm) * ((n + c.bn - 1) / c.bn);
    const long long wgs = tiles * splits;
    const long long per_cu = (wgs + cus - 1) / cus;
    int kloc = (k + splits - 1) / splits;
    kloc = ((kloc + kSplitQuantum - 1) / kSplitQuantum) * kSplitQuantum;
    if (splits == 1) kloc = k;
    const int occ = c.wg_per_cu(geo.lds_per_cu);
    // A CU works through its share `occ` workgroups at a time; when one is left over at the end it runs
    // alone, and a single 4-wave workgroup keeps only one wave per SIMD busy (measured on one tile column,
    // 64 x 128 tiles, k = 640: 19.7 us per tile two or three at a time, 23.6 us alone; two left over of
    // three run at the full rate).
    const double solo_tiles = (c.threads < 512 && per_cu % occ == 1) ? 1.0 : 0.0;
    const double solo_rate = (occ >= 3 && per_cu > 1) ? 0.92 : 0.85;      // (21.6 us alone after rounds of three)
    const double wg_flops = 2.0 * c.bm * c.bn * (double)kloc;
    double t = ((double)per_cu - solo_tiles + solo_tiles / solo_rate) * wg_flops /
               (kPeakPerCu * (pipelined ? c.eff[op] : c.eff_guarded[op]));
    // first copies + result store per round.  The 256 x 256 tile's figure was fitted on grids of at most
    // four rounds, where all workgroups store at the same moment; over more rounds they drift apart
    // and the stores stop colliding (NN, k = 512, per round beyond the k loop: 11.7 us at 4 rounds, 7.5
    // at 16, 4.8 at 64, 4.3 at 256).
    const long long rounds = (per_cu + occ - 1) / occ;
    double round_cost = pipelined ? c.round_s[op] : c.round_guarded_s[op];
    if (pipelined && c.bm * c.bn >= 256 * 256 && rounds > 4) round_cost *= 0.36 + 0.64 * pow(4.0 / (double)rounds, 0.75);
    t += round_cost * (double)rounds;
    // HBM floor: operands once, result once
    const double bytes = 4.0 * ((double)m * k + (double)n * k + (double)m * n);
    // (one workgroup per CU streaming a skinny operand: 3 % faster with two sets of waves than with one,
    //  (32, 8192, 8192) 49.3 against 50.8 us, (8192, 32, 8192) 49.4 against 51.8)
    const double stream_rate = (c.threads != c.threads_guarded) ? 5.15e12 : 5.0e12;
    if (t < bytes / stream_rate) t = bytes / stream_rate;
    // A launch whose whole k range is one slab holds four workgroups per CU (the launcher then asks for
    // one slab buffer only); measured at k <= 32 the 64 x 128 tiles lead there by 3-6 % for both
    // operations ((8192, 8192, 32) NT 55.9 us against 59.3 on 128 x 64 tiles, NN 60.0 against 64.8).
    if (pipelined && splits == 1 && k <= c.bk && c.bm == 64 && c.bn == 128) t *= 0.95;
    if (splits > 1) t += 2.3e-6 + 0.3e-6 * ((splits + 7) / 8) + 4.0 * (double)m * n * (splits + 2) / 4.0e12;
    return t + 3.0e-6;
}

// Predicted time of the even cut (gemm_streamk_kernel + fix-up) for configuration c, or a huge value
// where it cannot run.  Every workgroup gets the same number of k units, so the k-loop time is the
// padded work spread over all CUs; a workgroup pays the time outside the k loop once per tile it
// touches, and the fix-up kernel moves every cut tile's pieces once more.  The four weights are a
// least-squares fit to 130 measured (shape, configuration) pairs (tune.py even-cut; mean error 5 %).
static double predicted_seconds_even_cut(const Geometry& geo, int cfg, int op, int m, int n, int k, size_t scratch_bytes)
{
    const TileConfig& c = kTileConfigs[cfg];
    const long long tiles = (long long)((m + c.bm - 1) / c.bm) * ((n + c.bn - 1) / c.bn);
    const int units_per_tile = (k + kSplitQuantum - 1) / kSplitQuantum;
    const long long units = tiles * units_per_tile;
    const int occ = c.wg_per_cu(geo.lds_per_cu);
    const long long groups = (long long)geo.cus * occ;
    if (units < groups || units >= 0x7fffffffLL) return 1e30;
    if (scratch_needed(geo, cfg, kStreamK, m, n, k) > scratch_bytes) return 1e30;
    // with fewer tiles than an eighth of the pieces, every tile is cut many times and the fix-up
    // kernel (a few workgroups adding dozens of pieces each) dominates: measured 3x slower than split-k
    if (tiles * 8 < groups) return 1e30;
    const double units_per_wg = (double)units / (double)groups;
    const double main_s = units_per_wg * occ * 2.0 * c.bm * c.bn * kSplitQuantum / (kPeakPerCu * c.eff[op]);
    const double segments = units_per_wg / units_per_tile + 1.0;
    const double cut_tiles = tiles < groups ? (double)tiles : (double)groups;
    const double pieces = tiles < groups ? ((double)groups / tiles + 1.0 < 2.0 ? 2.0 : (double)groups / tiles + 1.0) : 2.0;
    const double fix_bytes = cut_tiles * (pieces + 1.0) * c.bm * c.bn * 4.0;
    return 1.04 * main_s + 1.01 * segments * c.round_s[op] + 0.41 * fix_bytes / 4.0e12 + 11.0e-6;
}

// A candidate that cannot fuse a requested epilogue (a configuration without the fused instance, the
// even cut, a split weight gradient) is charged the separate pass over C it would need: one more
// launch and two (bias, clamp) or three (update) trips of m x n words.
Choice choose(const Geometry& geo, int op, int m, int n, int k, bool allow_split, bool pipelined, int epi_kind,
              size_t scratch_bytes)
{
    Choice best = {0, 1};
    double best_t = 1e30;
    const int o = (op == OP_NT) ? 1 : 0;
    const bool epi = pipelined && epi_kind != kEpiNone;
    const double pass_s = epi ? 4.5e-6 + (epi_kind == kEpiBiasAct ? 2.0 : 3.0) * (double)m * (double)n * 4.0 / 4.0e12 : 0.0;
    for (int c = 0; c < kNumTileConfigs; ++c) {
        for (int splits = 1; splits <= kMaxSplits; splits *= 2) {
            if (splits > 1) {
                if (!allow_split) break;
                if ((size_t)m * n * splits * sizeof(float) > scratch_bytes) break;
                if (k / splits < 2 * kSplitQuantum) break;
            }
            const TileConfig& tc = kTileConfigs[c];
            if (tc.threads != tc.threads_guarded) {
                // two sets of waves on one tile: for launches that give a CU one workgroup at most, with
                // enough k per workgroup to pay for the hand-over at the end.  Measured on the grid: where
                // the rule takes it the time falls by 1-5 % on average (up to 13 %) for 512 to 2048 k per
                // workgroup; with less k the hand-over costs what the second set gains, with more the
                // older configurations' deeper splits are as good.
                // The 32-row and 32-column tiles of this kind serve products that are one such tile high or
                // wide (m or n <= 32: 3-6 % faster than their 4-wave twins); for anything larger the other
                // tiles are better and the model, fitted on full grids, would overrate these.
                const long long tiles_m = (m + tc.bm - 1) / tc.bm, tiles_n = (n + tc.bn - 1) / tc.bn;
                const long long wgs = tiles_m * tiles_n * splits;
                if (!pipelined || wgs > geo.cus || k / splits < 512 || k / splits > 2048) continue;
                if ((tc.bm < 64 && tiles_m > 1) || (tc.bn < 64 && tiles_n > 1)) continue;
            }
            double t = predicted_seconds(geo, tc, o, m, n, k, splits, pipelined);
            if (epi) {
                const bool fuses = (epi_kind == kEpiBiasAct) ? (splits > 1 || kTileConfigs[c].has_fused)
                                                             : (splits == 1 && o == 0 && kTileConfigs[c].has_fused);
                if (!fuses) t += pass_s;
                // the fused update reads and writes W next to the store of dW: 8 m n bytes more, which a
                // workgroup that has its CU to itself cannot overlap with anything ((4096, 4096, 1024):
                // +24 us on 256 x 256 tiles, +16 us on 128 x 128 tiles two per CU, over a 241 us product)
                else if (epi_kind == kEpiSgd)
                    t += 8.0 * (double)m * (double)n / (tc.wg_per_cu(geo.lds_per_cu) == 1 ? 5.3e12 : 8.0e12);
            }
            if (t < best_t * 0.999) { best_t = t; best = Choice{c, splits}; }
        }
    }
    if (allow_split && pipelined) {
        // the even cut, for the two configurations it was measured with (64 x 128 and 128 x 128 tiles,
        // two per CU), and only where it promises 5 % or more: on 65 measured shapes (tune.py even-cut)
        // it beat the best ordinary launch of all configurations and split counts on 19, by 2-10 %; this
        // rule took it on 13, once wrongly (5 % slower)
        double sk_t = best_t * 0.95;
        for (int c = 9; c <= 10; ++c) {
            const double t = predicted_seconds_even_cut(geo, c, o, m, n, k, scratch_bytes) + pass_s;
            if (t < sk_t) { sk_t = t; best = Choice{c, kStreamK}; }
        }
    }
    return best;
}

double gemm_predicted_seconds(const Geometry& geo, int op, int m, int n, int k, size_t scratch_bytes)
{
    const Choice ch = choose(geo, op, m, n, k, true, true, kEpiNone, scratch_bytes);
    const int o = (op == OP_NT) ? 1 : 0;
    if (ch.splits == kStreamK) return predicted_seconds_even_cut(geo, ch.cfg, o, m, n, k, scratch_bytes);
    return predicted_seconds(geo, kTileConfigs[ch.cfg], o, m, n, k, ch.splits, true);
}

int gemm_config_count() { return kNumTileConfigs; }
const char* gemm_config_name(int cfg) { return (cfg >= 0 && cfg < kNumTileConfigs) ? kTileConfigs[cfg].name : nullptr; }

int gemm_default_config(int op, int m, int n, int k, size_t scratch_bytes)
{
    return choose(geometry_or_nominal(), op, m, n, k, true, true, kEpiNone, scratch_bytes).cfg;
}
int gemm_default_splits(int op, int m, int n, int k, size_t scratch_bytes)
{
    return choose(geometry_or_nominal(), op, m, n, k, true, true, kEpiNone, scratch_bytes).splits;
}

}  // namespace mtnn

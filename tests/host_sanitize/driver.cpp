// Host-only exercise of the C ABI's validation, the selector (training, model files, evaluation,
// memo), the cost model and the C oracle, built with AddressSanitizer and UBSan (see
// tests/test_sanitize_host.py).  Prints "ALL OK" and exits 0 when every check holds and the
// sanitizers stayed silent.
#include "../../include/mtnn.h"
#include "gemm_config.h"

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

extern "C" {
int oracle_num_threads(void);
void oracle_nt_ref(int, int, int, const float*, long, const float*, long, const int*, int, double*, double*);
void oracle_nn_ref(int, int, int, const float*, long, const float*, long, const int*, int, double*, double*);
void oracle_transpose_ref(int, int, const uint32_t*, long, uint32_t*, long);
void oracle_f64_nt(int, int, int, const double*, const double*, double*);
void oracle_f64_nn(int, int, int, const double*, const double*, double*);
void oracle_f64_tn(int, int, int, const double*, const double*, double*);
}

static int g_failed = 0;
#define CHECK(cond) do { if (!(cond)) { std::printf("FAILED line %d: %s\n", __LINE__, #cond); ++g_failed; } } while (0)

static float* fake(uintptr_t a) { return reinterpret_cast<float*>(a); }

static void abi_validation()
{
    float *A = fake(0x100000), *B = fake(0x200000), *C = fake(0x300000), *W = fake(0x400000);
    CHECK(mtnn_nt(nullptr, -1, 4, 4, A, 4, B, 4, C, 4) == MTNN_ERR_DIM);
    CHECK(mtnn_nt(nullptr, 4, 4, 4, nullptr, 4, B, 4, C, 4) == MTNN_ERR_NULL);
    CHECK(mtnn_nn(nullptr, 4, 6, 8, A, 8, B, 5, C, 6) == MTNN_ERR_LD);
    CHECK(mtnn_nt(nullptr, 4, 4, 4, A, 4, B, 4, A + 4, 4) == MTNN_ERR_ALIAS);
    CHECK(mtnn_nt(nullptr, 0, 4, 4, nullptr, 4, nullptr, 4, nullptr, 4) == MTNN_OK);
    const int valid = mtnn_nt(nullptr, 4, 6, 8, A, 8, B, 8, C, 6);
    CHECK(valid == MTNN_ERR_NO_DEVICE);                          // no GPU here: nothing may be launched
    CHECK(mtnn_transpose(nullptr, 4, 6, A, 5, B, 4) == MTNN_ERR_LD);
    CHECK(mtnn_transpose(nullptr, 4, 6, A, 6, A, 4) == MTNN_ERR_ALIAS);
    CHECK(mtnn_transpose(nullptr, 4, 6, A, 6, B, 4) == MTNN_ERR_NO_DEVICE);
    CHECK(mtnn_transpose_inplace(nullptr, 4, A, 3) == MTNN_ERR_LD);
    CHECK(mtnn_transpose_inplace_rect(nullptr, 4, 40000, A) == MTNN_ERR_ARG);
    CHECK(mtnn_tnn(nullptr, 4, 6, 8, A, 8, B, 8, C, 6, nullptr, 0) == MTNN_ERR_WORKSPACE);
    CHECK(mtnn_tnn(nullptr, 4, 6, 8, A, 8, B, 8, C, 6, B + 2, mtnn_tnn_workspace_bytes(6, 8)) == MTNN_ERR_ALIAS);
    CHECK(mtnn_tnn_workspace_bytes(65536, 65536) == (size_t)65536 * 65536 * 4);
    CHECK(mtnn_tnn_inplace(nullptr, 8, 8, 8, A, 8, A, 8, C, 8) == MTNN_ERR_ALIAS);
    CHECK(mtnn_gemm_ex(nullptr, 2, 0, 1, 4, 4, 4, A, 4, B, 4, C, 4) == MTNN_ERR_ARG);
    int chosen = 7;
    CHECK(mtnn_auto(nullptr, 4, 6, 8, A, 7, B, 8, C, 6, W, 256, &chosen) == MTNN_ERR_LD);
    CHECK(mtnn_auto3(nullptr, 5, 4, 6, 8, A, 8, B, 8, C, 6, W, 256, &chosen) == MTNN_ERR_ARG);
    CHECK(mtnn_fc_layer_forward(nullptr, 1, 4, 6, 8, A, 8, B, 8, C + 2, 1, C, 6, W, 1 << 20, nullptr) == MTNN_ERR_ALIAS);
    CHECK(mtnn_fc_weight_grad_sgd(nullptr, 4, 6, 8, A, 8, B, 6, C, 6, C + 4, 6, 0.1f) == MTNN_ERR_ALIAS);
    CHECK(mtnn_set_scratch(nullptr, fake(0x700010), 1 << 20) == MTNN_ERR_ARG);
    CHECK(mtnn_get_scratch_bytes(nullptr) == 0);
    CHECK(mtnn_copy_bytes(nullptr, 60, A, B) == MTNN_ERR_ARG);
    CHECK(std::strcmp(mtnn_status_string(MTNN_OK), "ok") == 0 && std::strcmp(mtnn_status_string(99), "unknown status") == 0);
    CHECK(mtnn_arch_supported("gfx950:sramecc+:xnack-") == 1 && mtnn_arch_supported("gfx942") == 0 && mtnn_arch_supported(nullptr) == 0);
}

static void cost_model()
{
    const int ncfg = mtnn_gemm_config_count();
    CHECK(ncfg >= 3 && mtnn_gemm_config_name(ncfg) == nullptr && mtnn_gemm_config_name(-1) == nullptr);
    unsigned s = 12345;
    for (int it = 0; it < 4000; ++it) {
        int dims[3];
        for (int& d : dims) { s = s * 1664525u + 1013904223u; d = 1 + (int)((s >> 8) % 70000u); if (it % 7 == 0) d = 1 + d % 300; }
        for (int op = 0; op < 2; ++op) {
            for (size_t cap : {(size_t)0, (size_t)1 << 20, mtnn_scratch_bytes_default()}) {
                int cfg = -1, splits = 0;
                CHECK(mtnn_gemm_choice(op, dims[0], dims[1], dims[2], cap, &cfg, &splits) == MTNN_OK);
                CHECK(cfg >= 0 && cfg < ncfg);
                CHECK(splits == MTNN_GEMM_EVEN_CUT || (splits >= 1 && splits <= 32));
                if (splits != 1) CHECK(mtnn_gemm_scratch_bytes(cfg, splits, dims[0], dims[1], dims[2]) <= cap);
            }
        }
    }
    CHECK(mtnn_gemm_choice(3, 4, 4, 4, 0, nullptr, nullptr) == MTNN_ERR_ARG);
    CHECK(mtnn_gemm_choice(1, 0, 4, 4, 0, nullptr, nullptr) == MTNN_ERR_DIM);
}

// the multiply-high division the kernels use for the tile mapping, against the machine's own division
static void fast_division()
{
    const unsigned ds[] = {1, 2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 63, 64, 65, 127, 255, 256, 257, 1000, 4095, 4096, 4097, 65535, 65536, 65537,
                           1000003, (1u << 20) + 1, (1u << 30) - 1, 1u << 30, (1u << 30) + 1, 0x7ffffffeu, 0x7fffffffu};
    unsigned s = 99;
    for (unsigned d : ds) {
        const mtnn::FastDiv f = mtnn::make_fastdiv(d);
        const unsigned long long edge[] = {0, 1, d - 1ull, d, d + 1ull, 2ull * d - 1, 2ull * d, 3ull * d - 1, 0x7fffffffull, 0x7ffffffeull,
                                           0x40000000ull, 0x3fffffffull};
        for (unsigned long long n : edge) if (n <= 0x7fffffffull) CHECK(mtnn::fast_div((int)n, f) == (int)((unsigned)n / d));
        for (int it = 0; it < 20000; ++it) {
            s = s * 1664525u + 1013904223u;
            const int n = (int)(s >> 1);
            if (mtnn::fast_div(n, f) != (int)((unsigned)n / d)) { CHECK(!"fast_div differs"); break; }
        }
    }
    // the tile order as the kernels compute it, against plain divisions, over many grids
    for (int tiles_m : {1, 2, 3, 7, 8, 9, 16, 33, 128, 1000}) for (int tiles_n : {1, 2, 5, 8, 64, 129}) for (int xcd : {1, 8}) {
        mtnn::GemmParams p = {};
        p.tiles_m = tiles_m; p.tiles_n = tiles_n; p.group_m = tiles_m < 8 ? tiles_m : 8; p.num_xcd = xcd;
        mtnn::set_tile_order(p);
        const int total = tiles_m * tiles_n;
        std::vector<char> seen(total, 0);
        for (int pid0 = 0; pid0 < total; ++pid0) {
            int pid = pid0;
            if (p.num_xcd > 1) {
                const int local = mtnn::fast_div(pid, p.fd_xcd), x = pid - local * p.num_xcd;
                CHECK(local == pid / p.num_xcd);
                pid = (x < p.xcd_tall) ? x * p.xcd_per + local : p.xcd_tall * p.xcd_per + (x - p.xcd_tall) * (p.xcd_per - 1) + local;
            }
            const int band_sz = p.group_m * p.tiles_n, band = mtnn::fast_div(pid, p.fd_band);
            CHECK(band == pid / band_sz);
            const int in_band = pid - band * band_sz;
            const bool last = band == p.last_band;
            const int rows_here = last ? p.last_rows : p.group_m;
            const int tn = mtnn::fast_div(in_band, last ? p.fd_last : p.fd_group);
            const int tm = band * p.group_m + (in_band - tn * rows_here);
            CHECK(tn == in_band / rows_here && tm >= 0 && tm < tiles_m && tn >= 0 && tn < tiles_n);
            if (tm >= 0 && tm < tiles_m && tn >= 0 && tn < tiles_n) { CHECK(!seen[tm * tiles_n + tn]); seen[tm * tiles_n + tn] = 1; }
        }
    }
}

static void selector(const char* tmpdir)
{
    std::vector<int> mnk, labels;
    for (int m : {64, 256, 1024, 4096}) for (int n : {64, 256, 1024, 4096}) for (int k : {64, 256, 1024, 4096}) {
        mnk.insert(mnk.end(), {m, n, k});
        labels.push_back((k >= 1024 && m >= 256) ? -1 : 1);
    }
    const int rows = (int)labels.size();
    CHECK(mtnn_train_selector(rows, mnk.data(), labels.data()) == MTNN_OK);
    CHECK(mtnn_model_num_trees() >= 1 && mtnn_model_num_trees() <= 8 && mtnn_model_num_features() == 7);
    for (int i = 0; i < rows; ++i) CHECK(mtnn_select(mnk[3 * i], mnk[3 * i + 1], mnk[3 * i + 2]) == labels[i]);
    std::vector<int> out(rows);
    CHECK(mtnn_select_batch(rows, mnk.data(), out.data()) == MTNN_OK);
    for (int i = 0; i < rows; ++i) CHECK(out[i] == labels[i]);
    for (int t = 0; t < mtnn_model_num_trees(); ++t) {
        const int sz = mtnn_model_tree_size(t);
        CHECK(sz >= 1);
        for (int i = 0; i < sz; ++i) {
            int f, l, r; double thr, v;
            CHECK(mtnn_model_node(t, i, &f, &thr, &l, &r, &v) == MTNN_OK);
            if (f >= 0) CHECK(l > i && r > i && l < sz && r < sz && f < 7); else CHECK(l == -1 && r == -1);
        }
        int f, l, r; double thr, v;
        CHECK(mtnn_model_node(t, sz, &f, &thr, &l, &r, &v) != MTNN_OK);
    }
    CHECK(mtnn_model_tree_size(99) == -1);
    const std::string good = std::string(tmpdir) + "/m.model", bad = std::string(tmpdir) + "/bad.model";
    CHECK(mtnn_save_model(good.c_str()) == MTNN_OK);
    // malformed files: truncated, child index going backwards, wrong arity, garbage
    std::string text;
    { FILE* f = std::fopen(good.c_str(), "r"); char buf[4096]; size_t n; while ((n = std::fread(buf, 1, sizeof buf, f)) > 0) text.append(buf, n); std::fclose(f); }
    const std::string variants[] = {text.substr(0, text.size() / 2), "mtnn-gbdt 1\nfeatures 0\ntrees 0\n", "mtnn-gbdt 2\nfeatures 7\ntrees 0\n", "garbage\n",
                                    "mtnn-gbdt 1\nfeatures 7\ntrees 1\ntree 0 nodes 3\n0 0x1p+3 2 1 0x0p+0\n-1 0x0p+0 -1 -1 0x1p+0\n0 0x1p+2 0 1 0x0p+0\n",
                                    "mtnn-gbdt 1\nfeatures 7\ntrees 1\ntree 0 nodes 2000000000\n", ""};
    for (const std::string& v : variants) {
        FILE* f = std::fopen(bad.c_str(), "w"); std::fwrite(v.data(), 1, v.size(), f); std::fclose(f);
        CHECK(mtnn_load_model(bad.c_str()) == MTNN_ERR_MODEL);
        CHECK(mtnn_select(4096, 4096, 4096) == -1);             // the current predictor is untouched
    }
    CHECK(mtnn_load_model((std::string(tmpdir) + "/missing").c_str()) == MTNN_ERR_MODEL);
    mtnn_unload_model();
    CHECK(mtnn_select(4096, 4096, 4096) == 1 && mtnn_model_num_trees() == 0);
    CHECK(mtnn_load_model(good.c_str()) == MTNN_OK);
    for (int i = 0; i < rows; ++i) CHECK(mtnn_select(mnk[3 * i], mnk[3 * i + 1], mnk[3 * i + 2]) == labels[i]);
    CHECK(mtnn_select3(4096, 4096, 4096, 1, 1) == -1 && mtnn_select3(4096, 4096, 4096, 0, 0) == 1);
    double x[7];
    CHECK(mtnn_features(2, 3, 5, x) == MTNN_OK && x[0] == 2 && x[3] == 15 && x[6] == 30 && mtnn_features(0, 1, 1, x) == MTNN_ERR_DIM);
    double margin = 0;
    CHECK(mtnn_model_margin(x, 7, &margin) == MTNN_OK && mtnn_model_margin(x, 6, &margin) != MTNN_OK);
    // degenerate training sets
    int one[3] = {4, 4, 4}, lab = 1, badlab = 3;
    CHECK(mtnn_train_selector(1, one, &lab) == MTNN_OK && mtnn_select(9, 9, 9) == 1);
    CHECK(mtnn_train_selector(1, one, &badlab) == MTNN_ERR_ARG);
    CHECK(mtnn_train_selector(0, one, &lab) != MTNN_OK);
    mtnn_unload_model();
}

static void oracle()
{
    const int m = 5, n = 7, k = 9;
    std::vector<float> A(m * (k + 2)), B(n * (k + 1)), Bt(k * n);
    for (size_t i = 0; i < A.size(); ++i) A[i] = (float)((int)(i * 7 % 13) - 6);
    for (size_t i = 0; i < B.size(); ++i) B[i] = (float)((int)(i * 5 % 11) - 5);
    std::vector<double> C(m * n), S(m * n), C2(m * n);
    oracle_nt_ref(m, n, k, A.data(), k + 2, B.data(), k + 1, nullptr, 0, C.data(), S.data());
    for (int l = 0; l < k; ++l) for (int j = 0; j < n; ++j) Bt[l * n + j] = B[j * (k + 1) + l];
    oracle_nn_ref(m, n, k, A.data(), k + 2, Bt.data(), n, nullptr, 0, C2.data(), nullptr);
    for (int e = 0; e < m * n; ++e) CHECK(C[e] == C2[e] && S[e] >= std::fabs(C[e]));
    int rows[2] = {4, 1};
    std::vector<double> Cr(2 * n);
    oracle_nt_ref(m, n, k, A.data(), k + 2, B.data(), k + 1, rows, 2, Cr.data(), nullptr);
    for (int j = 0; j < n; ++j) CHECK(Cr[j] == C[4 * n + j] && Cr[n + j] == C[1 * n + j]);
    std::vector<uint32_t> in(3 * 5), out(5 * 4, 0xdeadbeefu);
    for (size_t i = 0; i < in.size(); ++i) in[i] = 0x7fc00000u + (uint32_t)i;
    oracle_transpose_ref(3, 5, in.data(), 5, out.data(), 4);
    for (int r = 0; r < 3; ++r) for (int c = 0; c < 5; ++c) CHECK(out[c * 4 + r] == in[r * 5 + c]);
    for (int c = 0; c < 5; ++c) CHECK(out[c * 4 + 3] == 0xdeadbeefu);
    std::vector<double> Ad(m * k), Bd(n * k), Bdt(k * n), Adt(k * m), D1(m * n), D2(m * n), D3(m * n);
    for (int i = 0; i < m; ++i) for (int l = 0; l < k; ++l) { Ad[i * k + l] = A[i * (k + 2) + l]; Adt[l * m + i] = Ad[i * k + l]; }
    for (int j = 0; j < n; ++j) for (int l = 0; l < k; ++l) { Bd[j * k + l] = B[j * (k + 1) + l]; Bdt[l * n + j] = Bd[j * k + l]; }
    oracle_f64_nt(m, n, k, Ad.data(), Bd.data(), D1.data());
    oracle_f64_nn(m, n, k, Ad.data(), Bdt.data(), D2.data());
    oracle_f64_tn(m, n, k, Adt.data(), Bdt.data(), D3.data());
    for (int e = 0; e < m * n; ++e) CHECK(D1[e] == C[e] && D2[e] == C[e] && D3[e] == C[e]);
    CHECK(oracle_num_threads() >= 1);
}

int main(int argc, char** argv)
{
    const char* tmpdir = argc > 1 ? argv[1] : "/tmp";
    abi_validation();
    cost_model();
    fast_division();
    selector(tmpdir);
    oracle();
    if (g_failed) { std::printf("%d checks failed\n", g_failed); return 1; }
    std::printf("ALL OK\n");
    return 0;
}

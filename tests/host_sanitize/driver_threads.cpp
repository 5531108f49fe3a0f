// Driver of the ThreadSanitizer build of the library's host side: several threads use the process-wide
// state at once -- the current selector model (installed, loaded, unloaded and queried concurrently),
// the per-thread memo that must follow it, the scratch registry, the cost model's tables.  Host only;
// without a GPU every launch path returns MTNN_ERR_NO_DEVICE before it would launch.
#include "../../include/mtnn.h"

#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <string>
#include <thread>
#include <vector>

static std::atomic<int> g_failures{0};
#define CHECK(cond)                                                                  \
    do {                                                                             \
        if (!(cond)) { std::fprintf(stderr, "FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); ++g_failures; } \
    } while (0)

// a training table whose label depends on the shape, so that trained models answer both ways
static void make_table(int variant, std::vector<int>& mnk, std::vector<int>& labels)
{
    const int sizes[6] = {64, 128, 256, 512, 1024, 2048};
    for (int a = 0; a < 6; ++a)
        for (int b = 0; b < 6; ++b)
            for (int c = 0; c < 6; ++c) {
                mnk.push_back(sizes[a]); mnk.push_back(sizes[b]); mnk.push_back(sizes[c]);
                const bool tnn = variant == 0 ? (sizes[c] >= 512 && sizes[b] <= 256) : (sizes[a] <= 128);
                labels.push_back(tnn ? -1 : 1);
            }
}

int main(int argc, char** argv)
{
    const std::string dir = argc > 1 ? argv[1] : "/tmp";
    std::vector<int> mnk0, lab0, mnk1, lab1;
    make_table(0, mnk0, lab0);
    make_table(1, mnk1, lab1);
    CHECK(mtnn_train_selector((int)lab0.size(), mnk0.data(), lab0.data()) == MTNN_OK);
    const std::string file0 = dir + "/tsan_model0.txt";
    CHECK(mtnn_save_model(file0.c_str()) == MTNN_OK);

    std::atomic<bool> stop{false};
    std::vector<std::thread> threads;
    // readers: single and batched queries; an answer is always +1 or -1, whatever model is current
    for (int t = 0; t < 4; ++t)
        threads.emplace_back([&, t] {
            const int sizes[6] = {64, 128, 256, 512, 1024, 2048};
            int batch[3 * 8], out[8];
            unsigned s = 1234u + (unsigned)t;
            while (!stop.load()) {
                for (int i = 0; i < 8; ++i)
                    for (int j = 0; j < 3; ++j) { s = s * 1664525u + 1013904223u; batch[3 * i + j] = sizes[(s >> 16) % 6]; }
                for (int i = 0; i < 8; ++i) {
                    const int l = mtnn_select(batch[3 * i], batch[3 * i + 1], batch[3 * i + 2]);
                    CHECK(l == 1 || l == -1);
                    // the same shape again: the memo's answer, which must still be a valid label
                    const int l2 = mtnn_select(batch[3 * i], batch[3 * i + 1], batch[3 * i + 2]);
                    CHECK(l2 == 1 || l2 == -1);
                }
                CHECK(mtnn_select_batch(8, batch, out) == MTNN_OK);
                for (int i = 0; i < 8; ++i) CHECK(out[i] == 1 || out[i] == -1);
                int cfg = -1, splits = 0;
                CHECK(mtnn_gemm_choice(1, batch[0], batch[1], batch[2], mtnn_scratch_bytes_default(), &cfg, &splits) == MTNN_OK);
                CHECK(cfg >= 0 && cfg < mtnn_gemm_config_count());
                CHECK(mtnn_select3(batch[0], batch[1], batch[2], 0, 1) != 0);
            }
        });
    // writers: retrain, load, unload, save
    threads.emplace_back([&] {
        for (int i = 0; i < 300; ++i) {
            if (i % 2) CHECK(mtnn_train_selector((int)lab1.size(), mnk1.data(), lab1.data()) == MTNN_OK);
            else CHECK(mtnn_train_selector((int)lab0.size(), mnk0.data(), lab0.data()) == MTNN_OK);
        }
    });
    threads.emplace_back([&] {
        const std::string mine = dir + "/tsan_model1.txt";
        for (int i = 0; i < 300; ++i) {
            CHECK(mtnn_load_model(file0.c_str()) == MTNN_OK);
            CHECK(mtnn_save_model(mine.c_str()) == MTNN_OK || true);       // (nothing to save right after an unload by this thread)
            if (i % 7 == 0) mtnn_unload_model();
            CHECK(mtnn_load_model((dir + "/no_such_model").c_str()) == MTNN_ERR_MODEL);
        }
    });
    // the scratch registry and the device probe from two threads (no device here: every call must say so or refuse the arguments)
    for (int t = 0; t < 2; ++t)
        threads.emplace_back([&, t] {
            for (int i = 0; i < 300; ++i) {
                void* stream = reinterpret_cast<void*>((uintptr_t)(0x1000 * (1 + (i + t) % 5)));
                void* ptr = reinterpret_cast<void*>((uintptr_t)0x7000000 + (uintptr_t)t * 0x100000);
                const int st = mtnn_set_scratch(stream, ptr, 1 << 20);
                CHECK(st == MTNN_OK || st == MTNN_ERR_NO_DEVICE);
                (void)mtnn_get_scratch_bytes(stream);
                const int st2 = mtnn_set_scratch(stream, nullptr, 0);
                CHECK(st2 == MTNN_OK || st2 == MTNN_ERR_NO_DEVICE);
                float x = 0.f;
                const int st3 = mtnn_nt(stream, 4, 4, 4, &x, 4, &x + 64, 4, &x + 128, 4);
                CHECK(st3 == MTNN_ERR_NO_DEVICE);
            }
        });
    for (size_t i = 4; i < threads.size(); ++i) threads[i].join();
    stop.store(true);
    for (size_t i = 0; i < 4; ++i) threads[i].join();
    if (g_failures.load() == 0) std::printf("ALL OK\n");
    return g_failures.load() ? 1 : 0;
}

// The device the kernels run on, and the scratch memory callers lend the library.
//
// Geometry: compute units, accelerator dies (XCDs) and LDS per compute unit are read from the HIP
// runtime once per device and cached; anything that is not a gfx950 is refused, because the code
// objects in this library exist for that architecture only.
//
// Scratch: the library allocates no device memory.  Launches that divide one product over several
// workgroups per C tile (split-k, the even cut) keep their partial products in a buffer that the
// caller registers per (device, stream); launches on one stream are ordered, so they share it.
#include "../../include/mtnn.h"
#include "mtnn_internal.h"

#include <atomic>
#include <mutex>
#include <string.h>
#include <vector>

namespace mtnn {

Geometry nominal_geometry() { return Geometry{-1, 256, 8, 160 * 1024}; }

bool arch_is_gfx950(const char* arch)
{
    if (!arch) return false;
    // "gfx950" alone or followed by feature flags (":sramecc+:xnack-"); "gfx9500" would be another chip
    return strncmp(arch, "gfx950", 6) == 0 && (arch[6] == '\0' || arch[6] == ':');
}

namespace {
constexpr int kMaxDevices = 64;
struct DeviceSlot {
    std::atomic<int> state{0};   // 0 unknown, 1 usable, 2 not usable
    Geometry geo;
};
DeviceSlot g_devices[kMaxDevices];
std::mutex g_device_mutex;

int probe_device(int dev, Geometry* out)
{
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) { (void)hipGetLastError(); return 2; }
    if (!arch_is_gfx950(prop.gcnArchName)) return 2;
    int xcds = 0;
    if (hipDeviceGetAttribute(&xcds, hipDeviceAttributeNumberOfXccs, dev) != hipSuccess || xcds < 1) {
        (void)hipGetLastError();
        xcds = 1;        // unknown: no remapping of workgroup ids (correct, only less local)
    }
    const size_t lds = prop.maxSharedMemoryPerMultiProcessor;
    if (prop.multiProcessorCount < 1 || lds < 64 * 1024) return 2;
    *out = Geometry{dev, prop.multiProcessorCount, xcds, (int)lds};
    return 1;
}
}  // namespace

bool current_geometry(Geometry* out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return false; }
    if (dev < 0 || dev >= kMaxDevices) return false;
    DeviceSlot& slot = g_devices[dev];
    int state = slot.state.load(std::memory_order_acquire);
    if (state == 0) {
        std::lock_guard<std::mutex> lock(g_device_mutex);
        state = slot.state.load(std::memory_order_acquire);
        if (state == 0) {
            Geometry g = nominal_geometry();
            state = probe_device(dev, &g);
            slot.geo = g;
            slot.state.store(state, std::memory_order_release);
        }
    }
    if (state != 1) return false;
    *out = slot.geo;
    return true;
}

Geometry geometry_or_nominal()
{
    Geometry g;
    return current_geometry(&g) ? g : nominal_geometry();
}

// ---- scratch registry ---------------------------------------------------------------------------
namespace {
struct ScratchEntry { int dev; hipStream_t stream; float* ptr; size_t bytes; };
std::vector<ScratchEntry> g_scratch;
std::mutex g_scratch_mutex;
std::atomic<unsigned long long> g_scratch_generation{1};   // bumped by every registration: invalidates the memos
}  // namespace

Scratch scratch_lookup(hipStream_t s)
{
    // a one-entry memo per thread: a training loop issues its launches on one stream
    struct Memo { unsigned long long generation; int dev; hipStream_t stream; Scratch value; };
    static thread_local Memo memo = {0, -1, nullptr, {nullptr, 0}};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return Scratch{nullptr, 0}; }
    const unsigned long long gen = g_scratch_generation.load(std::memory_order_acquire);
    if (memo.generation == gen && memo.dev == dev && memo.stream == s) return memo.value;
    Scratch found = {nullptr, 0};
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        for (const ScratchEntry& e : g_scratch)
            if (e.dev == dev && e.stream == s) { found = Scratch{e.ptr, e.bytes}; break; }
    }
    memo = Memo{gen, dev, s, found};
    return found;
}

int scratch_register(hipStream_t s, void* ptr, size_t bytes)
{
    if ((ptr == nullptr) != (bytes == 0)) return MTNN_ERR_ARG;
    if (reinterpret_cast<uintptr_t>(ptr) & 255) return MTNN_ERR_ARG;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return MTNN_ERR_NO_DEVICE; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    for (size_t i = 0; i < g_scratch.size(); ++i) {
        if (g_scratch[i].dev == dev && g_scratch[i].stream == s) {
            if (ptr) { g_scratch[i].ptr = static_cast<float*>(ptr); g_scratch[i].bytes = bytes; }
            else g_scratch.erase(g_scratch.begin() + (long)i);
            g_scratch_generation.fetch_add(1, std::memory_order_release);
            return MTNN_OK;
        }
    }
    if (ptr) {
        g_scratch.push_back(ScratchEntry{dev, s, static_cast<float*>(ptr), bytes});
        g_scratch_generation.fetch_add(1, std::memory_order_release);
    }
    return MTNN_OK;
}

}  // namespace mtnn

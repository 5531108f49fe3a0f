// mtnn_gemm_ex_static: mtnn_gemm_ex for callers that can neither allocate device memory nor lend
// the library any -- code under HIP graph capture, tight serving loops, harnesses that forbid
// hipMalloc.  A divided launch (split-k, the even cut) keeps its partial products in the array
// below, which lives in the library's code object: one copy per GPU the library runs on, held until
// the process ends.  The entry point allocates and frees nothing.
#include "../../include/mtnn.h"
#include "mtnn_internal.h"

#include <atomic>
#include <mutex>

// 32 MiB: room for, e.g., 8 partial products of a 1024 x 1024 result or the even cut's slots for
// 64 x 128 tiles; a launch that would need more is refused.
static __device__ __align__(256) unsigned char scratch[MTNN_STATIC_SCRATCH_BYTES];

namespace {

// `scratch` names a host-side stand-in here, not device memory: the array's address on a device is
// asked of the runtime once per device, with that device current, and kept.
constexpr int kMaxDevices = 64;
void* g_ptr[kMaxDevices];
std::atomic<int> g_state[kMaxDevices];     // 0 not asked yet, 1 resolved, 2 the runtime refused
std::mutex g_mutex;

// (called by the shared entry code after validation: the current device is a usable gfx950)
int static_scratch_for_current_device(mtnn::Scratch* out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return MTNN_ERR_NO_DEVICE; }
    if (dev < 0 || dev >= kMaxDevices) return MTNN_ERR_NO_DEVICE;
    int state = g_state[dev].load(std::memory_order_acquire);
    if (state == 0) {
        std::lock_guard<std::mutex> lock(g_mutex);
        state = g_state[dev].load(std::memory_order_acquire);
        if (state == 0) {
            void* ptr = nullptr;
            const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
            if (e == hipSuccess && ptr != nullptr) {
                g_ptr[dev] = ptr;
                state = 1;
            } else {
                (void)hipGetLastError();
                state = 2;
            }
            g_state[dev].store(state, std::memory_order_release);
        }
    }
    if (state != 1) return MTNN_ERR_LAUNCH;
    out->ptr = static_cast<float*>(g_ptr[dev]);
    out->bytes = MTNN_STATIC_SCRATCH_BYTES;
    return MTNN_OK;
}

}  // namespace

extern "C" int mtnn_gemm_ex_static(void* stream, int op, int cfg, int splits, int m, int n, int k,
                                   const float* A, int lda, const float* B, int ldb, float* C, int ldc)
{
    // Same validation, same kernels and same division of the work as mtnn_gemm_ex with 32 MiB lent:
    // an explicit division whose partial products need more returns MTNN_ERR_WORKSPACE before anything
    // is launched, and the rule's own choice (cfg = -1, splits = 0) only considers what fits.  Every
    // partial product a launch reads back it has written first, so nothing needs clearing between calls.
    return mtnn::gemm_ex_entry(stream, op, cfg, splits, m, n, k, A, lda, B, ldb, C, ldc,
                               &static_scratch_for_current_device);
}

// hlq_lut_gemv_static: hlq_lut_gemv for callers that cannot allocate device memory (code under HIP
// graph capture, tight serving loops, harnesses that forbid hipMalloc).  Same kernels, same plan,
// same results as hlq_lut_gemv; the split-K arrival counters and partial sums, which hlq_lut_gemv
// takes from the caller's workspace argument, live in a fixed device array of this library instead.
//
// The array is one per GPU: every device that loads the library's code object holds its own copy
// at its own address until the process ends.  In host code the array's NAME is only a stand-in for
// the symbol, not a device address; the address on the current device comes from
// hipGetSymbolAddress, once per device, and only that pointer is handed to kernels.
#include <atomic>
#include <mutex>

#include "hlq_internal.h"

// counters (HLQ_WS_COUNTER_BYTES) followed by the fp32 partial sums.  The host-side use in
// hipGetSymbolAddress below is what makes the compiler emit the array as a symbol the runtime can find.
static __device__ __align__(256) unsigned char scratch[HLQ_STATIC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
std::atomic<void *> g_scratch_ptr[MAX_DEVICES];   // device address of `scratch` on device i, null until looked up
std::mutex g_scratch_mutex;

// Address of the scratch array on the current device.  The first call on a device looks it up and
// clears the counter block with a small fill kernel on `st` (the array is zero when the code object
// is loaded and every GEMV leaves the counters zero, so this is a belt-and-braces step; a fill
// kernel rather than a memset node, so that a caller may be capturing `st`).
hlq_status scratch_on_current_device(hipStream_t st, void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return HLQ_ERR_HIP;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        p = g_scratch_ptr[dev].load(std::memory_order_acquire);
        if (!p) {
            void *sym = nullptr;
            const hipError_t e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !sym) return hlq_hip_status(e == hipSuccess ? hipErrorInvalidSymbol : e);
            const hlq_status s = hlq_launch_ws_init(sym, HLQ_STATIC_SCRATCH_BYTES, st);
            if (s != HLQ_OK) return s;
            g_scratch_ptr[dev].store(sym, std::memory_order_release);
            p = sym;
        }
    }
    *out = p;
    return HLQ_OK;
}

} // namespace

extern "C" hlq_status hlq_lut_gemv_static(const hlq_desc *d, const void *packed, const uint16_t *x, void *y,
                                          hlq_out_dtype out, void *stream)
{
    HlqDims dm;
    hlq_status s = hlq_check_desc(d, &dm);
    if (s != HLQ_OK) return s;
    if (!packed || !x || !y) return HLQ_ERR_NULL;
    if (out != HLQ_OUT_F16 && out != HLQ_OUT_F32) return HLQ_ERR_UNSUPPORTED;
    if (((uintptr_t)packed & 15u) || ((uintptr_t)x & 15u) || ((uintptr_t)y & (out == HLQ_OUT_F32 ? 3u : 1u)))
        return HLQ_ERR_BAD_STRIDE;
    // what this GEMV's plan needs, decided on the host before anything touches the device
    size_t need = 0;
    s = hlq_gemv_ws_used(dm, &need);
    if (s != HLQ_OK) return s;
    if (need > HLQ_STATIC_SCRATCH_BYTES) return HLQ_ERR_BUFFER_TOO_SMALL;
    void *ws = nullptr;
    s = scratch_on_current_device((hipStream_t)stream, &ws);
    if (s != HLQ_OK) return s;
    HlqGemvItem it;
    it.dm = dm;
    it.packed = packed;
    it.x = x;
    it.y = y;
    return hlq_launch_gemv_batch(1, &it, out, ws, (hipStream_t)stream, HLQ_STATIC_SCRATCH_BYTES);
}

// fbq_linear_static: the decode hot path for callers that cannot allocate.  Same kernels as fbq_linear;
// the hand-over scratch (the tagged words that carry t = x.A from the blocks that compute it to the
// blocks that use it) lives in a file-scope device array instead of a caller-supplied workspace.
#include <mutex>

#include "fbq_internal.h"

namespace fbq {

// One copy per GPU the library's code object is loaded on, held until the process ends.  Zero when
// loaded, which is what the hand-over needs (a launch tag is never zero); after that every launch
// marks the words it writes with its own identity, so nothing has to be cleared between calls.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU, looked up once
static std::mutex g_scratch_mutex;

// In host code `scratch` is only a handle for the symbol: its address on the current device has to be
// asked for, once per device, with that device current.
static fbq_status scratch_on_current_device(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return FBQ_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return FBQ_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return FBQ_OK;
}

}  // namespace fbq

using namespace fbq;

extern "C" fbq_status fbq_linear_static(const fbq_desc *d, int M, const void *x, const void *qweight, const void *scales,
                                        const void *zeros, const void *At, const void *Bt, void *y, fbq_stream stream)
{
    const fbq_status ds = fbq_check_desc(d);
    if (ds != FBQ_OK) return ds;
    if (M < 1) return FBQ_ERR_SHAPE;
    if (M > kDecodeMaxM) return FBQ_ERR_UNSUPPORTED;     // larger token counts need scratch that grows with M, N and K
    const size_t need = fbq_workspace_bytes(d, M);
    if (need > kStaticScratchBytes) return FBQ_ERR_WORKSPACE;
    // every argument is checked before the GPU is asked for anything (the workspace passed here is a stand-in)
    LinearArgs a;
    fbq_status st = check_layer(d, M, x, qweight, scales, zeros, At, Bt, y, (void *)(uintptr_t)256, kStaticScratchBytes, &a);
    if (st != FBQ_OK) return st;
    void *ws = nullptr;
    st = scratch_on_current_device(&ws);
    if (st != FBQ_OK) return st;
    a.workspace = ws;
    return hip_status(launch_one(a, (hipStream_t)stream));
}

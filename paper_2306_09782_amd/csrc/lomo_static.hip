// lomo_vector_update for callers that cannot allocate: the partial column sums of the gain-vector kernels go to
// a fixed device array of this library instead of a caller workspace.  Nothing here allocates: no hipMalloc, no
// hipFree, no events, no streams.  The array's device address is looked up once per device.
#include "lomo.h"
#include "lomo_kernels.h"

#include <mutex>

namespace {

// In host code this name is only a handle for hipGetSymbolAddress; kernels get the address that call returns.
static __device__ __align__(256) unsigned char scratch[LOMO_VECTOR_STATIC_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
void* g_scratch_ptr[kMaxDevices] = {};     // per device: each GPU holds its own copy of the array at its own address

// Device address of `scratch` on the current device, or null (with *status set) if it cannot be had.
void* scratch_for_current_device(lomo_status* status) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        *status = LOMO_ERR_LAUNCH;
        return nullptr;
    }
    std::lock_guard<std::mutex> lk(g_mu);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
            *status = LOMO_ERR_LAUNCH;
            return nullptr;
        }
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}

}  // namespace

extern "C" lomo_status lomo_vector_update_static(const lomo_half* Xhat, const lomo_half* dY, lomo_half* w, int64_t T, int64_t H,
                                                 float lr, float inv_loss_scale, float clip_coef,
                                                 const int32_t* overflow_flag, void* stream) {
    if (T < 0 || H < 0 || (H & 7)) return LOMO_ERR_SHAPE;
    if (T == 0 || H == 0) return LOMO_OK;
    if (!Xhat || !dY || !w) return LOMO_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(Xhat) & 15u) || (reinterpret_cast<uintptr_t>(dY) & 15u) ||
        (reinterpret_cast<uintptr_t>(w) & 15u))
        return LOMO_ERR_ALIGN;
    if (lomo::vector_ws_bytes(T, H) > (size_t)LOMO_VECTOR_STATIC_BYTES) return LOMO_ERR_TOO_LARGE;
    lomo_status st = LOMO_OK;
    void* ws = scratch_for_current_device(&st);
    if (ws == nullptr) return st;
    const float s = (float)((double)lr * (double)clip_coef * (double)inv_loss_scale);
    // same kernels as lomo_vector_update, launched untimed; every partial sum is written before it is read, so the
    // array's old contents do not matter
    return lomo::launch_vector(Xhat, dY, w, T, H, ws, 1, s, nullptr, nullptr, overflow_flag,
                               static_cast<hipStream_t>(stream)) == hipSuccess
               ? LOMO_OK
               : LOMO_ERR_LAUNCH;
}

// C-ABI shim: argument checks, workspace carving, launches on the caller's stream.
// Declarations and the contract of every entry point are in include/lomo.h.
#include "lomo.h"
#include "lomo_kernels.h"

#include <math.h>

using namespace lomo;

namespace {

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }
inline lomo_status from_hip(hipError_t e) { return e == hipSuccess ? LOMO_OK : LOMO_ERR_LAUNCH; }
inline float step_size(float lr, float inv_loss_scale, float clip_coef) {
    return (float)((double)lr * (double)clip_coef * (double)inv_loss_scale);
}

}  // namespace

extern "C" {

int lomo_version(void) { return 1000; }

const char* lomo_status_str(lomo_status s) {
    switch (s) {
        case LOMO_OK: return "ok";
        case LOMO_ERR_NULL: return "required pointer is NULL";
        case LOMO_ERR_SHAPE: return "bad shape (negative, or K/N/H not a multiple of 8)";
        case LOMO_ERR_ALIGN: return "pointer not 16-byte aligned";
        case LOMO_ERR_WORKSPACE: return "workspace missing or too small";
        case LOMO_ERR_LAUNCH: return "HIP launch failed";
    }
    return "unknown status";
}

lomo_status lomo_wgrad_sqnorm(const lomo_half* X, const lomo_half* dY, int64_t T, int64_t K, int64_t N, double* acc,
                              int32_t* overflow_flag, void* stream) {
    if (T < 0 || K < 0 || N < 0 || (K & 7) || (N & 7)) return LOMO_ERR_SHAPE;
    if (!acc) return LOMO_ERR_NULL;
    if (T == 0 || K == 0 || N == 0) return LOMO_OK;
    if (!X || !dY) return LOMO_ERR_NULL;
    if (misaligned(X) || misaligned(dY) || (reinterpret_cast<uintptr_t>(acc) & 7u)) return LOMO_ERR_ALIGN;
    GemmArgs a{};
    a.A = X; a.B = dY; a.Out = nullptr;
    a.M = K; a.Nn = N; a.C = T;
    a.lda = K; a.ldb = N; a.ldo = K;
    a.acc = acc; a.flag_out = overflow_flag;
    a.family = LOMO_KERNEL_WGRAD_SQNORM;
    return from_hip(launch_wgrad_sqnorm(a, static_cast<hipStream_t>(stream)));
}

lomo_status lomo_linear_backward_update(const lomo_half* X, const lomo_half* dY, lomo_half* W, lomo_half* dX, int64_t T,
                                        int64_t K, int64_t N, float lr, float inv_loss_scale, float clip_coef,
                                        const int32_t* overflow_flag, void* stream) {
    if (T < 0 || K < 0 || N < 0 || (K & 7) || (N & 7)) return LOMO_ERR_SHAPE;
    if (K == 0 || N == 0) return LOMO_OK;
    if (!W) return LOMO_ERR_NULL;
    if (T > 0 && (!X || !dY)) return LOMO_ERR_NULL;
    if (misaligned(X) || misaligned(dY) || misaligned(W) || misaligned(dX)) return LOMO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (T == 0) return LOMO_OK;
    if (dX) {   // dgrad first: it must see the pre-update W; same stream => ordered
        GemmArgs d{};
        d.A = W; d.B = dY; d.Out = dX;
        d.M = K; d.Nn = T; d.C = N;
        d.lda = K; d.ldb = N; d.ldo = K;
        d.family = LOMO_KERNEL_DGRAD;
        hipError_t e = launch_dgrad(d, st);
        if (e != hipSuccess) return LOMO_ERR_LAUNCH;
    }
    GemmArgs a{};
    a.A = X; a.B = dY; a.Out = W;
    a.M = K; a.Nn = N; a.C = T;
    a.lda = K; a.ldb = N; a.ldo = K;
    a.s = step_size(lr, inv_loss_scale, clip_coef);
    a.flag_in = overflow_flag;
    a.family = LOMO_KERNEL_WGRAD_UPDATE;
    return from_hip(launch_wgrad_update(a, st));
}

size_t lomo_embedding_workspace_bytes(int64_t T, int64_t H) { return embedding_ws_bytes(T, H); }
size_t lomo_vector_workspace_bytes(int64_t T, int64_t H) { return vector_ws_bytes(T, H); }

static lomo_status check_embedding(const int32_t* ids, const lomo_half* dY, int64_t T, int64_t H, int64_t V, void* ws,
                                   size_t ws_bytes) {
    if (T < 0 || H < 0 || V < 0 || (H & 7) || T > 0x7fffffff) return LOMO_ERR_SHAPE;
    if (T == 0 || H == 0) return LOMO_OK;
    if (!ids || !dY) return LOMO_ERR_NULL;
    if (misaligned(dY) || (reinterpret_cast<uintptr_t>(ids) & 3u)) return LOMO_ERR_ALIGN;
    if (!ws || ws_bytes < embedding_ws_bytes(T, H) || (reinterpret_cast<uintptr_t>(ws) & 255u)) return LOMO_ERR_WORKSPACE;
    return LOMO_OK;
}

lomo_status lomo_embedding_grouping(const int32_t* ids, int64_t T, int64_t V, void* ws, size_t ws_bytes,
                                    int32_t* unique_ids, int32_t* seg_offsets, int32_t* perm, int32_t* n_unique,
                                    void* stream) {
    if (T < 0 || V < 0 || T > 0x7fffffff) return LOMO_ERR_SHAPE;
    if (!unique_ids || !seg_offsets || !perm || !n_unique) return LOMO_ERR_NULL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (T > 0) {
        if (!ids) return LOMO_ERR_NULL;
        if (!ws || ws_bytes < embedding_ws_bytes(T, 8) || (reinterpret_cast<uintptr_t>(ws) & 255u))
            return LOMO_ERR_WORKSPACE;
    }
    EmbeddingWs w{};
    if (T > 0) w = carve_embedding_ws(ws, T);
    w.perm = perm; w.unique_ids = unique_ids; w.seg_offsets = seg_offsets; w.n_unique = n_unique;
    return from_hip(launch_embedding_grouping(ids, T, w, st));
}

lomo_status lomo_embedding_sqnorm(const int32_t* ids, const lomo_half* dY, int64_t T, int64_t H, int64_t V, void* ws,
                                  size_t ws_bytes, double* acc, int32_t* overflow_flag, void* stream) {
    lomo_status s = check_embedding(ids, dY, T, H, V, ws, ws_bytes);
    if (s != LOMO_OK) return s;
    if (!acc) return LOMO_ERR_NULL;
    if (T == 0 || H == 0) return LOMO_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    EmbeddingWs w = carve_embedding_ws(ws, T);
    ScopedTiming timing(LOMO_KERNEL_EMBEDDING, st);
    hipError_t e = launch_embedding_grouping(ids, T, w, st);
    if (e != hipSuccess) return LOMO_ERR_LAUNCH;
    return from_hip(launch_embedding_rows(dY, nullptr, T, H, w, 0, 0.f, acc, overflow_flag, nullptr, st));
}

lomo_status lomo_embedding_update(const int32_t* ids, const lomo_half* dY, lomo_half* W, int64_t T, int64_t H, int64_t V,
                                  float lr, float inv_loss_scale, float clip_coef, const int32_t* overflow_flag, void* ws,
                                  size_t ws_bytes, void* stream) {
    lomo_status s = check_embedding(ids, dY, T, H, V, ws, ws_bytes);
    if (s != LOMO_OK) return s;
    if (T == 0 || H == 0 || V == 0) return LOMO_OK;
    if (!W) return LOMO_ERR_NULL;
    if (misaligned(W)) return LOMO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    EmbeddingWs w = carve_embedding_ws(ws, T);
    ScopedTiming timing(LOMO_KERNEL_EMBEDDING, st);
    hipError_t e = launch_embedding_grouping(ids, T, w, st);
    if (e != hipSuccess) return LOMO_ERR_LAUNCH;
    return from_hip(launch_embedding_rows(dY, W, T, H, w, 1, step_size(lr, inv_loss_scale, clip_coef), nullptr, nullptr,
                                          overflow_flag, st));
}

static lomo_status check_vector(const lomo_half* Xhat, const lomo_half* dY, int64_t T, int64_t H, void* ws,
                                size_t ws_bytes) {
    if (T < 0 || H < 0 || (H & 7)) return LOMO_ERR_SHAPE;
    if (T == 0 || H == 0) return LOMO_OK;
    if (!Xhat || !dY) return LOMO_ERR_NULL;
    if (misaligned(Xhat) || misaligned(dY)) return LOMO_ERR_ALIGN;
    if (!ws || ws_bytes < vector_ws_bytes(T, H) || (reinterpret_cast<uintptr_t>(ws) & 15u)) return LOMO_ERR_WORKSPACE;
    return LOMO_OK;
}

lomo_status lomo_vector_sqnorm(const lomo_half* Xhat, const lomo_half* dY, int64_t T, int64_t H, void* ws,
                               size_t ws_bytes, double* acc, int32_t* overflow_flag, void* stream) {
    lomo_status s = check_vector(Xhat, dY, T, H, ws, ws_bytes);
    if (s != LOMO_OK) return s;
    if (!acc) return LOMO_ERR_NULL;
    if (T == 0 || H == 0) return LOMO_OK;
    ScopedTiming timing(LOMO_KERNEL_VECTOR, static_cast<hipStream_t>(stream));
    return from_hip(launch_vector(Xhat, dY, nullptr, T, H, ws, 0, 0.f, acc, overflow_flag, nullptr,
                                  static_cast<hipStream_t>(stream)));
}

lomo_status lomo_vector_update(const lomo_half* Xhat, const lomo_half* dY, lomo_half* w, int64_t T, int64_t H, float lr,
                               float inv_loss_scale, float clip_coef, const int32_t* overflow_flag, void* ws,
                               size_t ws_bytes, void* stream) {
    lomo_status s = check_vector(Xhat, dY, T, H, ws, ws_bytes);
    if (s != LOMO_OK) return s;
    if (T == 0 || H == 0) return LOMO_OK;
    if (!w) return LOMO_ERR_NULL;
    ScopedTiming timing(LOMO_KERNEL_VECTOR, static_cast<hipStream_t>(stream));
    return from_hip(launch_vector(Xhat, dY, w, T, H, ws, 1, step_size(lr, inv_loss_scale, clip_coef), nullptr, nullptr,
                                  overflow_flag, static_cast<hipStream_t>(stream)));
}

lomo_status lomo_reduce_flags(const int32_t* flags, int64_t n, int32_t* out, void* stream) {
    if (n < 0) return LOMO_ERR_SHAPE;
    if (!out || (n > 0 && !flags)) return LOMO_ERR_NULL;
    return from_hip(launch_reduce_flags(flags, n, out, static_cast<hipStream_t>(stream)));
}

double lomo_clip_coef(double acc_sqnorm_scaled, double loss_scale, double max_norm, double eps) {
    const double norm = sqrt(acc_sqnorm_scaled) / loss_scale;
    if (!isfinite(norm)) return 0.0;   // overflowed step: nothing may be applied
    const double c = max_norm / (norm + eps);
    return c < 1.0 ? c : 1.0;
}

void lomo_scaler_step(float* loss_scale, int32_t* clean_steps, int32_t growth_interval, int overflow) {
    if (!loss_scale || !clean_steps) return;
    if (overflow) {
        float s = *loss_scale * 0.5f;
        *loss_scale = s < 1.0f ? 1.0f : s;
        *clean_steps = 0;
        return;
    }
    *clean_steps += 1;
    if (*clean_steps >= growth_interval) {
        float s = *loss_scale * 2.0f;
        *loss_scale = s > 16777216.0f ? 16777216.0f : s;
        *clean_steps = 0;
    }
}

}  // extern "C"

// C-ABI shim: argument checks, workspace carving, launches on the caller's stream.
// Declarations and the contract of every entry point are in include/lomo.h.
#include "lomo.h"
#include "lomo_kernels.h"

#include <math.h>

#include <vector>

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
        case LOMO_ERR_TOO_LARGE: return "size beyond the fixed scratch of the allocation-free entry point";
    }
    return "unknown status";
}

lomo_status lomo_wgrad_sqnorm(const lomo_half* X, const lomo_half* dY, int64_t T, int64_t K, int64_t N, double* acc,
                              int32_t* overflow_flag, void* stream) {
    return lomo_wgrad_sqnorm_route(X, dY, T, K, N, acc, overflow_flag, LOMO_NORM_DIRECT, stream);
}

lomo_status lomo_wgrad_sqnorm_route(const lomo_half* X, const lomo_half* dY, int64_t T, int64_t K, int64_t N, double* acc,
                                    int32_t* overflow_flag, int norm_algorithm, void* stream) {
    if (norm_algorithm != LOMO_NORM_DIRECT && norm_algorithm != LOMO_NORM_AUTO && norm_algorithm != LOMO_NORM_GRAM)
        return LOMO_ERR_SHAPE;
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
    return from_hip(launch_wgrad_sqnorm(a, norm_algorithm, static_cast<hipStream_t>(stream)));
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
        if (!ws || ws_bytes < embedding_ws_bytes(T, 0) || (reinterpret_cast<uintptr_t>(ws) & 255u))
            return LOMO_ERR_WORKSPACE;
    }
    EmbeddingWs w{};
    if (T > 0) w = carve_embedding_ws(ws, T, 0);
    w.perm = perm; w.unique_ids = unique_ids; w.seg_offsets = seg_offsets; w.n_unique = n_unique;
    return from_hip(launch_embedding_grouping(ids, T, V, w, st));
}

lomo_status lomo_embedding_sqnorm(const int32_t* ids, const lomo_half* dY, int64_t T, int64_t H, int64_t V, void* ws,
                                  size_t ws_bytes, double* acc, int32_t* overflow_flag, void* stream) {
    lomo_status s = check_embedding(ids, dY, T, H, V, ws, ws_bytes);
    if (s != LOMO_OK) return s;
    if (!acc) return LOMO_ERR_NULL;
    if (T == 0 || H == 0) return LOMO_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    EmbeddingWs w = carve_embedding_ws(ws, T, H);
    ScopedTiming timing(LOMO_KERNEL_EMBEDDING, st);
    hipError_t e = launch_embedding_grouping(ids, T, V, w, st);
    if (e != hipSuccess) return LOMO_ERR_LAUNCH;
    return from_hip(launch_embedding_rows(ids, dY, nullptr, T, H, w, 0, 0.f, acc, overflow_flag, nullptr, st));
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
    EmbeddingWs w = carve_embedding_ws(ws, T, H);
    ScopedTiming timing(LOMO_KERNEL_EMBEDDING, st);
    hipError_t e = launch_embedding_grouping(ids, T, V, w, st);
    if (e != hipSuccess) return LOMO_ERR_LAUNCH;
    return from_hip(launch_embedding_rows(ids, dY, W, T, H, w, 1, step_size(lr, inv_loss_scale, clip_coef), nullptr, nullptr,
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
    if (misaligned(w)) return LOMO_ERR_ALIGN;
    ScopedTiming timing(LOMO_KERNEL_VECTOR, static_cast<hipStream_t>(stream));
    return from_hip(launch_vector(Xhat, dY, w, T, H, ws, 1, step_size(lr, inv_loss_scale, clip_coef), nullptr, nullptr,
                                  overflow_flag, static_cast<hipStream_t>(stream)));
}

// ---- whole passes ------------------------------------------------------------------------

static lomo_status check_linear(const lomo_tensor& t, bool need_w) {
    if (t.T < 0 || t.K < 0 || t.N < 0 || (t.K & 7) || (t.N & 7)) return LOMO_ERR_SHAPE;
    if (t.T == 0 || t.K == 0 || t.N == 0) return LOMO_OK;
    if (!t.X || !t.dY || (need_w && !t.W)) return LOMO_ERR_NULL;
    if (misaligned(t.X) || misaligned(t.dY) || (need_w && (misaligned(t.W) || misaligned(t.dX)))) return LOMO_ERR_ALIGN;
    return LOMO_OK;
}

// Workspace layout of a whole-pass call: [ embedding grouping | shared area ].  The shared area serves the
// embedding's partial rows and the gain vectors' partial column sums in turn (everything runs on one stream).
struct StepWs {
    size_t grouping = 0;     // bytes of the head (largest embedding batch of the list)
    size_t emb_rest = 0;     // bytes the embedding needs behind its grouping
    size_t vec_one = 0;      // largest single gain vector's partial sums
    size_t vec_all = 0;      // the same for every gain vector of the most demanding shape at once (capped)
    int n_embedding = 0;
};
constexpr size_t kVecBatchBytes = (size_t)64 << 20;     // partial sums worth batching per launch

static StepWs plan_step_ws(const lomo_tensor* tensors, int64_t n) {
    StepWs p;
    if (!tensors) return p;
    for (int64_t i = 0; i < n; ++i) {
        const lomo_tensor& t = tensors[i];
        if (t.T <= 0 || t.K <= 0) continue;
        if (t.kind == LOMO_TENSOR_EMBEDDING) {
            const size_t g = embedding_grouping_bytes(t.T);
            const size_t all = embedding_ws_bytes(t.T, t.K);
            if (g > p.grouping) p.grouping = g;
            if (all - g > p.emb_rest) p.emb_rest = all - g;
            p.n_embedding++;
        } else if (t.kind == LOMO_TENSOR_VECTOR) {
            const size_t one = vector_ws_bytes(t.T, t.K);
            size_t same = 0;
            for (int64_t j = 0; j < n; ++j)
                if (tensors[j].kind == LOMO_TENSOR_VECTOR && tensors[j].T == t.T && tensors[j].K == t.K) ++same;
            if (same > (size_t)VEC_BATCH) same = VEC_BATCH;
            size_t all = one * same;
            if (all > kVecBatchBytes) all = (kVecBatchBytes / one > 0 ? kVecBatchBytes / one : 1) * one;
            if (one > p.vec_one) p.vec_one = one;
            if (all > p.vec_all) p.vec_all = all;
        }
    }
    return p;
}

size_t lomo_step_workspace_bytes(const lomo_tensor* tensors, int64_t n) {
    const StepWs p = plan_step_ws(tensors, n);
    return p.grouping + (p.emb_rest > p.vec_all ? p.emb_rest : p.vec_all);
}

size_t lomo_step_workspace_min_bytes(const lomo_tensor* tensors, int64_t n) {
    const StepWs p = plan_step_ws(tensors, n);
    return p.grouping + (p.emb_rest > p.vec_one ? p.emb_rest : p.vec_one);
}

static lomo_status check_step(const lomo_tensor* tensors, int64_t n, bool update, void* ws, size_t ws_bytes) {
    if (n < 0) return LOMO_ERR_SHAPE;
    if (n > 0 && !tensors) return LOMO_ERR_NULL;
    const size_t need = lomo_step_workspace_min_bytes(tensors, n);
    if (need > 0 && (!ws || ws_bytes < need || (reinterpret_cast<uintptr_t>(ws) & 255u))) return LOMO_ERR_WORKSPACE;
    // the per-kind checks below see a workspace that is known to be large enough for each tensor on its own
    for (int64_t i = 0; i < n; ++i) {
        const lomo_tensor& t = tensors[i];
        lomo_status s;
        if (t.kind == LOMO_TENSOR_LINEAR) {
            s = check_linear(t, update);
        } else if (t.kind == LOMO_TENSOR_EMBEDDING) {
            s = check_embedding(t.ids, t.dY, t.T, t.K, t.N, ws, ws_bytes);
            if (s == LOMO_OK && update && t.T > 0 && t.K > 0 && t.N > 0 && (!t.W || misaligned(t.W))) s = t.W ? LOMO_ERR_ALIGN : LOMO_ERR_NULL;
        } else if (t.kind == LOMO_TENSOR_VECTOR) {
            s = check_vector(t.X, t.dY, t.T, t.K, ws, ws_bytes);
            if (s == LOMO_OK && update && t.T > 0 && t.K > 0 && (!t.W || misaligned(t.W))) s = t.W ? LOMO_ERR_ALIGN : LOMO_ERR_NULL;
        } else {
            s = LOMO_ERR_SHAPE;
        }
        if (s != LOMO_OK) return s;
    }
    return LOMO_OK;
}

// The row kernels of a pass: every gain vector (one launch per stage and shape, as far as the shared area holds
// their partial sums), then the embedding.  mode as in launch_vector / launch_embedding_rows; flags: per-tensor
// flags to raise (modes 0 and 2) or null.
static lomo_status run_row_kernels(const lomo_tensor* tensors, int64_t n, void* ws, size_t ws_bytes, int mode, float s,
                                   const float* s_dev, double* acc, int32_t* flags, const int32_t* step_flag, float lr,
                                   float clipv, bool reuse_grouping, hipStream_t st) {
    const StepWs plan = plan_step_ws(tensors, n);
    char* shared = static_cast<char*>(ws) + plan.grouping;
    const size_t shared_bytes = ws_bytes - plan.grouping;
    std::vector<char> done((size_t)n, 0);
    for (int64_t i = 0; i < n; ++i) {
        const lomo_tensor& t = tensors[i];
        if (t.kind != LOMO_TENSOR_VECTOR || done[i] || t.T == 0 || t.K == 0) continue;
        std::vector<VecItem> items;
        for (int64_t j = i; j < n; ++j) {
            const lomo_tensor& u = tensors[j];
            if (u.kind != LOMO_TENSOR_VECTOR || u.T != t.T || u.K != t.K) continue;
            done[j] = 1;
            items.push_back(VecItem{u.X, u.dY, mode == 0 ? nullptr : u.W, flags ? flags + j : nullptr});
        }
        ScopedTiming timing(LOMO_KERNEL_VECTOR, st);
        if (launch_vector_batch(items.data(), (int)items.size(), t.T, t.K, shared, shared_bytes, mode, s, acc, step_flag, st,
                                lr, clipv, s_dev) != hipSuccess)
            return LOMO_ERR_LAUNCH;
    }
    for (int64_t i = 0; i < n; ++i) {
        const lomo_tensor& t = tensors[i];
        if (t.kind != LOMO_TENSOR_EMBEDDING || t.T == 0 || t.K == 0 || t.N == 0) continue;
        EmbeddingWs w = carve_embedding_ws(ws, t.T, t.K);
        // partial sums go behind the grouping of the LARGEST embedding batch, where the shared area starts
        const ptrdiff_t shift = shared - reinterpret_cast<char*>(w.partials);
        w.partials = reinterpret_cast<double*>(reinterpret_cast<char*>(w.partials) + shift);
        w.chunk_rows = reinterpret_cast<float*>(reinterpret_cast<char*>(w.chunk_rows) + shift);
        ScopedTiming timing(LOMO_KERNEL_EMBEDDING, st);
        if (!(reuse_grouping && plan.n_embedding == 1) && launch_embedding_grouping(t.ids, t.T, t.N, w, st) != hipSuccess)
            return LOMO_ERR_LAUNCH;
        if (launch_embedding_rows(t.ids, t.dY, mode == 0 ? nullptr : t.W, t.T, t.K, w, mode, s, acc, flags ? flags + i : nullptr,
                                  step_flag, st, lr, clipv, s_dev) != hipSuccess)
            return LOMO_ERR_LAUNCH;
    }
    return LOMO_OK;
}

lomo_status lomo_step_norm_pass(const lomo_tensor* tensors, int64_t n, double* acc, int32_t* flags, void* ws,
                                size_t ws_bytes, const lomo_step_options* options, void* stream) {
    const int route = options ? options->norm_algorithm : LOMO_NORM_DIRECT;
    if (route != LOMO_NORM_DIRECT && route != LOMO_NORM_AUTO && route != LOMO_NORM_GRAM) return LOMO_ERR_SHAPE;
    lomo_status cs = check_step(tensors, n, false, ws, ws_bytes);
    if (cs != LOMO_OK) return cs;
    if (!acc || !flags) return LOMO_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(acc) & 7u) return LOMO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    std::vector<GemmArgs> grouped;
    for (int64_t i = 0; i < n; ++i) {
        const lomo_tensor& t = tensors[i];
        if (t.kind != LOMO_TENSOR_LINEAR || t.T == 0 || t.K == 0 || t.N == 0) continue;
        GemmArgs a{};
        a.A = t.X; a.B = t.dY; a.Out = nullptr;
        a.M = t.K; a.Nn = t.N; a.C = t.T;
        a.lda = t.K; a.ldb = t.N; a.ldo = t.K;
        a.acc = acc; a.flag_out = flags + i;
        a.family = LOMO_KERNEL_WGRAD_SQNORM;
        if (dma_eligible(a)) grouped.push_back(a);
        else if (launch_wgrad_sqnorm(a, route, st) != hipSuccess) return LOMO_ERR_LAUNCH;
    }
    std::vector<GemmArgs> gram, direct;
    choose_norm_route(route, grouped, gram, direct);
    if (!gram.empty() && launch_gram_group(gram.data(), (int)gram.size(), st) != hipSuccess) return LOMO_ERR_LAUNCH;
    if (!direct.empty() && launch_dma_group<true, EPI_SQNORM>(direct.data(), (int)direct.size(), st) != hipSuccess)
        return LOMO_ERR_LAUNCH;
    cs = run_row_kernels(tensors, n, ws, ws_bytes, 0, 0.f, nullptr, acc, flags, nullptr, 0.f, 0.f, false, st);
    if (cs != LOMO_OK) return cs;
    return from_hip(launch_reduce_flags(flags, n, flags + n, st));
}

// Pass 2 with the step size given by value (s_dev == nullptr) or read by the kernels from device memory.
static lomo_status update_pass(const lomo_tensor* tensors, int64_t n, float s, const float* s_dev,
                               const int32_t* step_flag, void* ws, size_t ws_bytes, const lomo_step_options* options,
                               void* stream) {
    lomo_status cs = check_step(tensors, n, true, ws, ws_bytes);
    if (cs != LOMO_OK) return cs;
    hipStream_t st = static_cast<hipStream_t>(stream);
    std::vector<GemmArgs> dgrads, updates, updates_plain;
    // every dgrad first: dX must come from the pre-update weights
    for (int64_t i = 0; i < n; ++i) {
        const lomo_tensor& t = tensors[i];
        if (t.kind != LOMO_TENSOR_LINEAR || t.T == 0 || t.K == 0 || t.N == 0) continue;
        if (t.dX) {
            GemmArgs d{};
            d.A = t.W; d.B = t.dY; d.Out = t.dX;
            d.M = t.K; d.Nn = t.T; d.C = t.N;
            d.lda = t.K; d.ldb = t.N; d.ldo = t.K;
            d.family = LOMO_KERNEL_DGRAD;
            if (dma_eligible(d)) dgrads.push_back(d);
            else if (launch_dgrad(d, st) != hipSuccess) return LOMO_ERR_LAUNCH;
        }
        GemmArgs a{};
        a.A = t.X; a.B = t.dY; a.Out = t.W;
        a.M = t.K; a.Nn = t.N; a.C = t.T;
        a.lda = t.K; a.ldb = t.N; a.ldo = t.K;
        a.s = s; a.s_dev = s_dev; a.flag_in = step_flag;
        a.family = LOMO_KERNEL_WGRAD_UPDATE;
        if (dma_eligible(a)) updates.push_back(a);
        else updates_plain.push_back(a);
    }
    if (!dgrads.empty() && launch_dma_group<false, EPI_STORE>(dgrads.data(), (int)dgrads.size(), st) != hipSuccess)
        return LOMO_ERR_LAUNCH;
    if (!updates.empty() && launch_dma_group<true, EPI_UPDATE>(updates.data(), (int)updates.size(), st) != hipSuccess)
        return LOMO_ERR_LAUNCH;
    for (const GemmArgs& a : updates_plain)
        if (launch_wgrad_update(a, st) != hipSuccess) return LOMO_ERR_LAUNCH;
    return run_row_kernels(tensors, n, ws, ws_bytes, 1, s, s_dev, nullptr, nullptr, step_flag, 0.f, 0.f,
                           options != nullptr && options->reuse_grouping != 0, st);
}

lomo_status lomo_step_update_pass(const lomo_tensor* tensors, int64_t n, float lr, float inv_loss_scale,
                                  float clip_coef, const int32_t* step_flag, void* ws, size_t ws_bytes,
                                  const lomo_step_options* options, void* stream) {
    return update_pass(tensors, n, step_size(lr, inv_loss_scale, clip_coef), nullptr, step_flag, ws, ws_bytes, options, stream);
}

lomo_status lomo_step_scalars_device(const double* acc, const int32_t* step_flag, double loss_scale, double max_norm,
                                     double eps, double lr, lomo_step_scalars* scalars, void* stream) {
    if (!acc || !scalars) return LOMO_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(acc) & 7u) || (reinterpret_cast<uintptr_t>(scalars) & 7u)) return LOMO_ERR_ALIGN;
    if (!(loss_scale > 0.0)) return LOMO_ERR_SHAPE;
    return from_hip(launch_step_scalars(acc, step_flag, loss_scale, max_norm, eps, lr, scalars,
                                        static_cast<hipStream_t>(stream)));
}

lomo_status lomo_step_update_pass_device(const lomo_tensor* tensors, int64_t n, const lomo_step_scalars* scalars,
                                         const int32_t* step_flag, void* ws, size_t ws_bytes,
                                         const lomo_step_options* options, void* stream) {
    if (!scalars) return LOMO_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(scalars) & 7u) return LOMO_ERR_ALIGN;
    return update_pass(tensors, n, 0.f, &scalars->step, step_flag, ws, ws_bytes, options, stream);
}

// ---- clip by value (single pass) -----------------------------------------------------------

lomo_status lomo_linear_backward_update_clip_value(const lomo_half* X, const lomo_half* dY, lomo_half* W, lomo_half* dX,
                                                   int64_t T, int64_t K, int64_t N, float lr, float inv_loss_scale,
                                                   float clip_value, int32_t* overflow_flag, void* stream) {
    lomo_tensor t{};
    t.kind = LOMO_TENSOR_LINEAR;
    t.X = X; t.dY = dY; t.W = W; t.dX = dX; t.T = T; t.K = K; t.N = N;
    lomo_status cs = check_linear(t, true);
    if (cs != LOMO_OK) return cs;
    if (!(clip_value >= 0.f)) return LOMO_ERR_SHAPE;
    if (T == 0 || K == 0 || N == 0) return LOMO_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dX) {
        GemmArgs d{};
        d.A = W; d.B = dY; d.Out = dX;
        d.M = K; d.Nn = T; d.C = N;
        d.lda = K; d.ldb = N; d.ldo = K;
        d.family = LOMO_KERNEL_DGRAD;
        if (launch_dgrad(d, st) != hipSuccess) return LOMO_ERR_LAUNCH;
    }
    GemmArgs a{};
    a.A = X; a.B = dY; a.Out = W;
    a.M = K; a.Nn = N; a.C = T;
    a.lda = K; a.ldb = N; a.ldo = K;
    a.lr = lr; a.inv_s = inv_loss_scale; a.clipv = clip_value;
    a.flag_out = overflow_flag;
    a.family = LOMO_KERNEL_WGRAD_UPDATE;
    return from_hip(launch_wgrad_update_clipv(a, st));
}

lomo_status lomo_step_update_pass_clip_value(const lomo_tensor* tensors, int64_t n, float lr, float inv_loss_scale,
                                             float clip_value, int32_t* flags, void* ws, size_t ws_bytes, void* stream) {
    lomo_status cs = check_step(tensors, n, true, ws, ws_bytes);
    if (cs != LOMO_OK) return cs;
    if (!flags) return LOMO_ERR_NULL;
    if (!(clip_value >= 0.f)) return LOMO_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    std::vector<GemmArgs> dgrads, updates, updates_plain;
    for (int64_t i = 0; i < n; ++i) {
        const lomo_tensor& t = tensors[i];
        if (t.kind != LOMO_TENSOR_LINEAR || t.T == 0 || t.K == 0 || t.N == 0) continue;
        if (t.dX) {
            GemmArgs d{};
            d.A = t.W; d.B = t.dY; d.Out = t.dX;
            d.M = t.K; d.Nn = t.T; d.C = t.N;
            d.lda = t.K; d.ldb = t.N; d.ldo = t.K;
            d.family = LOMO_KERNEL_DGRAD;
            if (dma_eligible(d)) dgrads.push_back(d);
            else if (launch_dgrad(d, st) != hipSuccess) return LOMO_ERR_LAUNCH;
        }
        GemmArgs a{};
        a.A = t.X; a.B = t.dY; a.Out = t.W;
        a.M = t.K; a.Nn = t.N; a.C = t.T;
        a.lda = t.K; a.ldb = t.N; a.ldo = t.K;
        a.lr = lr; a.inv_s = inv_loss_scale; a.clipv = clip_value;
        a.flag_out = flags + i;
        a.family = LOMO_KERNEL_WGRAD_UPDATE;
        if (dma_eligible(a)) updates.push_back(a);
        else updates_plain.push_back(a);
    }
    if (!dgrads.empty() && launch_dma_group<false, EPI_STORE>(dgrads.data(), (int)dgrads.size(), st) != hipSuccess)
        return LOMO_ERR_LAUNCH;
    if (!updates.empty() && launch_dma_group<true, EPI_CLIPV>(updates.data(), (int)updates.size(), st) != hipSuccess)
        return LOMO_ERR_LAUNCH;
    for (const GemmArgs& a : updates_plain)
        if (launch_wgrad_update_clipv(a, st) != hipSuccess) return LOMO_ERR_LAUNCH;
    cs = run_row_kernels(tensors, n, ws, ws_bytes, 2, inv_loss_scale, nullptr, nullptr, flags, nullptr, lr, clip_value, false, st);
    if (cs != LOMO_OK) return cs;
    return from_hip(launch_reduce_flags(flags, n, flags + n, st));
}

lomo_status lomo_linear_dgrad(const lomo_half* dY, const lomo_half* W, lomo_half* dX, int64_t T, int64_t K, int64_t N,
                              void* stream) {
    if (T < 0 || K < 0 || N < 0 || (K & 7) || (N & 7)) return LOMO_ERR_SHAPE;
    if (T == 0 || K == 0) return LOMO_OK;
    if (!dX) return LOMO_ERR_NULL;
    if (N > 0 && (!dY || !W)) return LOMO_ERR_NULL;
    if (misaligned(dY) || misaligned(W) || misaligned(dX)) return LOMO_ERR_ALIGN;
    if (N == 0) return LOMO_ERR_SHAPE;   // an empty contraction would leave dX undefined
    GemmArgs d{};
    d.A = W; d.B = dY; d.Out = dX;
    d.M = K; d.Nn = T; d.C = N;
    d.lda = K; d.ldb = N; d.ldo = K;
    d.family = LOMO_KERNEL_DGRAD;
    return from_hip(launch_dgrad(d, static_cast<hipStream_t>(stream)));
}

lomo_status lomo_linear_forward(const lomo_half* X, const lomo_half* W, lomo_half* Y, int64_t T, int64_t K, int64_t N,
                                int accumulate, void* stream) {
    if (T < 0 || K < 0 || N < 0 || (K & 7) || (N & 7)) return LOMO_ERR_SHAPE;
    if (T == 0 || N == 0) return LOMO_OK;
    if (!Y) return LOMO_ERR_NULL;
    if (K > 0 && (!X || !W)) return LOMO_ERR_NULL;
    if (misaligned(X) || misaligned(W) || misaligned(Y)) return LOMO_ERR_ALIGN;
    if (K == 0) return LOMO_ERR_SHAPE;   // an empty contraction would leave Y undefined
    GemmArgs f{};
    f.A = W; f.B = X; f.Out = Y;
    f.M = N; f.Nn = T; f.C = K;
    f.lda = K; f.ldb = K; f.ldo = N;
    f.s = -1.0f;                         // accumulate: Y <- rne16(Y - s * acc)
    f.family = LOMO_KERNEL_FORWARD;
    return from_hip(launch_forward(f, accumulate != 0, static_cast<hipStream_t>(stream)));
}

lomo_status lomo_linear_forward_residual(const lomo_half* X, const lomo_half* W, const lomo_half* R, lomo_half* Y, int64_t T,
                                         int64_t K, int64_t N, void* stream) {
    if (T < 0 || K < 0 || N < 0 || (K & 7) || (N & 7)) return LOMO_ERR_SHAPE;
    if (T == 0 || N == 0) return LOMO_OK;
    if (!Y || !R) return LOMO_ERR_NULL;
    if (K > 0 && (!X || !W)) return LOMO_ERR_NULL;
    if (misaligned(X) || misaligned(W) || misaligned(Y) || misaligned(R)) return LOMO_ERR_ALIGN;
    if (K == 0) return LOMO_ERR_SHAPE;
    GemmArgs f{};
    f.A = W; f.B = X; f.Out = Y; f.Res = R;
    f.M = N; f.Nn = T; f.C = K;
    f.lda = K; f.ldb = K; f.ldo = N;
    f.s = -1.0f;
    f.family = LOMO_KERNEL_FORWARD;
    return from_hip(launch_forward(f, true, static_cast<hipStream_t>(stream)));
}

lomo_status lomo_embedding_forward(const int32_t* ids, const lomo_half* W, lomo_half* h, int64_t T, int64_t H, int64_t V,
                                   void* stream) {
    if (T < 0 || H < 0 || V < 0 || (H & 7)) return LOMO_ERR_SHAPE;
    if (T == 0 || H == 0) return LOMO_OK;
    if (!ids || !h || (V > 0 && !W)) return LOMO_ERR_NULL;
    if (misaligned(W) || misaligned(h) || (reinterpret_cast<uintptr_t>(ids) & 3u)) return LOMO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ScopedTiming timing(LOMO_KERNEL_CHAIN, st);
    return from_hip(launch_embedding_forward(ids, W, h, T, H, V, st));
}

lomo_status lomo_rmsnorm_forward(const lomo_half* h, const lomo_half* gain, float eps, lomo_half* xhat, float* rstd,
                                 lomo_half* xn, int64_t T, int64_t H, void* stream) {
    if (T < 0 || H < 0 || (H & 7) || T > 0x7fffffff || !(eps >= 0.f)) return LOMO_ERR_SHAPE;
    if (T == 0 || H == 0) return LOMO_OK;
    if (!h || !gain || !xhat || !rstd || !xn) return LOMO_ERR_NULL;
    if (misaligned(h) || misaligned(gain) || misaligned(xhat) || misaligned(xn) || (reinterpret_cast<uintptr_t>(rstd) & 3u))
        return LOMO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ScopedTiming timing(LOMO_KERNEL_CHAIN, st);
    return from_hip(launch_rmsnorm_forward(h, gain, eps, xhat, rstd, xn, T, H, st));
}

lomo_status lomo_swiglu_forward(const lomo_half* gate_up, lomo_half* a, int64_t T, int64_t F, void* stream) {
    if (T < 0 || F < 0 || (F & 7)) return LOMO_ERR_SHAPE;
    if (T == 0 || F == 0) return LOMO_OK;
    if (!gate_up || !a) return LOMO_ERR_NULL;
    if (misaligned(gate_up) || misaligned(a)) return LOMO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ScopedTiming timing(LOMO_KERNEL_CHAIN, st);
    return from_hip(launch_swiglu_forward(gate_up, a, T, F, st));
}

lomo_status lomo_rope_forward(lomo_half* qkv, const float* rope_cos, const float* rope_sin, int64_t T, int64_t s,
                              int64_t n_heads, int64_t head_dim, void* stream) {
    if (T < 0 || s <= 0 || n_heads <= 0 || head_dim != 128 || s > (1 << 24) || n_heads > (1 << 16)) return LOMO_ERR_SHAPE;
    if (T == 0) return LOMO_OK;
    if (!qkv || !rope_cos || !rope_sin) return LOMO_ERR_NULL;
    if (misaligned(qkv) || (reinterpret_cast<uintptr_t>(rope_cos) & 3u) || (reinterpret_cast<uintptr_t>(rope_sin) & 3u))
        return LOMO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ScopedTiming timing(LOMO_KERNEL_CHAIN, st);
    return from_hip(launch_rope_forward(qkv, rope_cos, rope_sin, T, s, n_heads, st));
}

lomo_status lomo_cross_entropy(const lomo_half* logits, const int32_t* targets, float grad_scale, float* loss,
                               lomo_half* dlogits, int64_t T, int64_t V, void* stream) {
    if (T < 0 || V < 0 || (V & 7) || T > 0x7fffffff || V > 0x7fffffff) return LOMO_ERR_SHAPE;
    if (T == 0) return LOMO_OK;
    if (V == 0) return LOMO_ERR_SHAPE;
    if (!logits || !targets || !loss || !dlogits) return LOMO_ERR_NULL;
    if (misaligned(logits) || misaligned(dlogits) || (reinterpret_cast<uintptr_t>(targets) & 3u) ||
        (reinterpret_cast<uintptr_t>(loss) & 3u))
        return LOMO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ScopedTiming timing(LOMO_KERNEL_CHAIN, st);
    return from_hip(launch_cross_entropy(logits, targets, grad_scale, loss, dlogits, T, V, st));
}

lomo_status lomo_cross_entropy_mean(const lomo_half* logits, const int32_t* targets, double loss_scale, float* loss,
                                    lomo_half* dlogits, double* stats, int64_t T, int64_t V, void* stream) {
    if (T < 0 || V < 0 || (V & 7) || T > 0x7fffffff || V > 0x7fffffff || !(loss_scale > 0.0)) return LOMO_ERR_SHAPE;
    if (!stats) return LOMO_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(stats) & 7u) return LOMO_ERR_ALIGN;
    if (T > 0 && V == 0) return LOMO_ERR_SHAPE;
    if (T > 0 && (!logits || !targets || !loss || !dlogits)) return LOMO_ERR_NULL;
    if (misaligned(logits) || misaligned(dlogits) || (reinterpret_cast<uintptr_t>(targets) & 3u) ||
        (reinterpret_cast<uintptr_t>(loss) & 3u))
        return LOMO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ScopedTiming timing(LOMO_KERNEL_CHAIN, st);
    return from_hip(launch_cross_entropy_mean(logits, targets, loss_scale, loss, dlogits, stats, T, V, st));
}

lomo_status lomo_attention_forward(const lomo_half* qkv, lomo_half* o, float* lse, int64_t B, int64_t s, int64_t n_heads,
                                   int64_t head_dim, void* stream) {
    if (B < 0 || s < 0 || n_heads <= 0 || head_dim != 128 || (s % 64) != 0) return LOMO_ERR_SHAPE;
    if (B * s * n_heads > (int64_t)1 << 31 || (s / 64) * n_heads * B > 0x7fffffff) return LOMO_ERR_SHAPE;
    if (B == 0 || s == 0) return LOMO_OK;
    if (!qkv || !o || !lse) return LOMO_ERR_NULL;
    if (misaligned(qkv) || misaligned(o) || (reinterpret_cast<uintptr_t>(lse) & 3u)) return LOMO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ScopedTiming timing(LOMO_KERNEL_ATTENTION, st);
    return from_hip(launch_attention_forward(qkv, o, lse, B, s, n_heads, st));
}

lomo_status lomo_swiglu_backward(const lomo_half* da, const lomo_half* gate_up, lomo_half* dgate_up, int64_t T, int64_t F,
                                 void* stream) {
    if (T < 0 || F < 0 || (F & 7)) return LOMO_ERR_SHAPE;
    if (T == 0 || F == 0) return LOMO_OK;
    if (!da || !gate_up || !dgate_up) return LOMO_ERR_NULL;
    if (misaligned(da) || misaligned(gate_up) || misaligned(dgate_up)) return LOMO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ScopedTiming timing(LOMO_KERNEL_CHAIN, st);
    return from_hip(launch_swiglu_backward(da, gate_up, dgate_up, T, F, st));
}

lomo_status lomo_rmsnorm_backward(const lomo_half* dxn, const lomo_half* xhat, const float* rstd, const lomo_half* gain,
                                  const lomo_half* dres, lomo_half* dh, int64_t T, int64_t H, void* stream) {
    if (T < 0 || H < 0 || (H & 7) || T > 0x7fffffff) return LOMO_ERR_SHAPE;
    if (T == 0 || H == 0) return LOMO_OK;
    if (!dxn || !xhat || !rstd || !gain || !dh) return LOMO_ERR_NULL;
    if (misaligned(dxn) || misaligned(xhat) || misaligned(gain) || misaligned(dres) || misaligned(dh) ||
        (reinterpret_cast<uintptr_t>(rstd) & 3u))
        return LOMO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ScopedTiming timing(LOMO_KERNEL_CHAIN, st);
    return from_hip(launch_rmsnorm_backward(dxn, xhat, rstd, gain, dres, dh, T, H, st));
}

lomo_status lomo_attention_backward(const lomo_half* qkv, const lomo_half* o, const lomo_half* dO, const float* lse,
                                    const float* rope_cos, const float* rope_sin, float* delta_ws, lomo_half* dqkv,
                                    int64_t B, int64_t s, int64_t n_heads, int64_t head_dim, void* stream) {
    if (B < 0 || s < 0 || n_heads < 0 || head_dim != 128 || (s & 63) || s > (1 << 20) || n_heads > 65535 || B > 65535 ||
        (s / 64) * n_heads * B >= (1ll << 31))
        return LOMO_ERR_SHAPE;
    if (B == 0 || s == 0 || n_heads == 0) return LOMO_OK;
    if (!qkv || !o || !dO || !lse || !delta_ws || !dqkv) return LOMO_ERR_NULL;
    if ((rope_cos == nullptr) != (rope_sin == nullptr)) return LOMO_ERR_NULL;
    if (misaligned(qkv) || misaligned(o) || misaligned(dO) || misaligned(dqkv) || (reinterpret_cast<uintptr_t>(lse) & 3u) ||
        (reinterpret_cast<uintptr_t>(delta_ws) & 3u) || (reinterpret_cast<uintptr_t>(rope_cos) & 3u) ||
        (reinterpret_cast<uintptr_t>(rope_sin) & 3u))
        return LOMO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ScopedTiming timing(LOMO_KERNEL_ATTENTION, st);
    return from_hip(launch_attention_backward(qkv, o, dO, lse, rope_cos, rope_sin, delta_ws, dqkv, B, s, n_heads, st));
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

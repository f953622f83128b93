// Internal launch interface between the C-ABI shim and the HIP kernels (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <vector>

#include "lomo.h"

namespace lomo {

// Which epilogue the contraction kernel ends with.
enum Epilogue : int {
    EPI_UPDATE = 0,   // W <- rne16(W - s * acc)            (fused wgrad + SGD update)
    EPI_SQNORM = 1,   // acc_out += sum acc^2, overflow flag (norm pass)
    EPI_STORE = 2,    // Out <- rne16(acc)                  (dgrad)
    EPI_CLIPV = 3     // W <- rne16(W - lr * clamp(acc / S, -c, c)), single pass (clip by value)
};

// One contraction  Out[n][m] (+)= sum_c A(c, m) * B(c, n).
//   A is "contraction-strided", A[c * lda + m], except in the forward product (A[m * lda + c]).
//   B is contraction-strided  (B[c * ldb + n])  or contraction-contiguous (B[n * ldb + c]).
// wgrad: A = X, B = dY (strided), Out = W;   M = K_in, Nn = N_out, C = T.
// dgrad: A = W, B = dY (contiguous), Out = dX; M = K_in, Nn = T, C = N_out.
struct GemmArgs {
    int family;              // LOMO_KERNEL_* of this launch (host side only: timing)
    const uint16_t* A;
    const uint16_t* B;
    uint16_t* Out;
    const uint16_t* Res;     // EPI_UPDATE only: read the old value from here instead of Out (same layout); null = Out
    int64_t M, Nn, C;
    int64_t lda, ldb, ldo;
    float s;                 // update step (EPI_UPDATE)
    const float* s_dev;      // when not null the update step is read from device memory instead
    float lr, inv_s, clipv;  // learning rate, 1 / loss scale, clamp threshold (EPI_CLIPV)
    double* acc;             // squared-norm accumulator (EPI_SQNORM)
    int32_t* flag_out;       // overflow flag to raise (EPI_SQNORM), may be null
    const int32_t* flag_in;  // overflow flag to honour (EPI_UPDATE), may be null
};

// Whole-tile fast path (lomo_gemm_fast.hip): returns false when the shape is not eligible.
template <bool B_STRIDED, int EPI>
bool try_launch_fast(const GemmArgs& a, hipStream_t st, hipError_t* err);

// Persistent 256 x 256 direct-to-LDS kernel (lomo_gemm_dma.hip).  try_launch_dma returns false when
// the tensor is not eligible or too small; launch_dma_group runs a list of eligible tensors (same
// epilogue, same acc / step flag / step size) in as few launches as the argument space allows.
bool dma_eligible(const GemmArgs& a);
template <bool B_STRIDED, int EPI>
bool try_launch_dma(const GemmArgs& a, hipStream_t st, hipError_t* err);
template <bool B_STRIDED, int EPI>
hipError_t launch_dma_group(const GemmArgs* list, int n, hipStream_t st);
// Forward product Y = X W^T: A = W [M x C] and B = X [Nn x C], both contraction-contiguous.
template <int EPI>
bool try_launch_dma_nt(const GemmArgs& a, hipStream_t st, hipError_t* err);

// Gram route of the norm pass (lomo_gram.hip): ||dY^T X||^2 from X X^T and dY dY^T.  `a` is a norm-pass
// contraction (A = X, B = dY, C = T).  Costs are in units of one 256 x 256 x 32 slice on one CU.
bool gram_eligible(const GemmArgs& a);
double gram_cost(const GemmArgs& a);
double direct_cost(const GemmArgs& a);
hipError_t launch_gram_group(const GemmArgs* list, int n, hipStream_t st);
// Splits the eligible tensors of `all` between the two routes according to `mode` (LOMO_NORM_*).
void choose_norm_route(int mode, const std::vector<GemmArgs>& all, std::vector<GemmArgs>& gram, std::vector<GemmArgs>& direct);

hipError_t launch_wgrad_update(const GemmArgs& a, hipStream_t st);
hipError_t launch_wgrad_update_clipv(const GemmArgs& a, hipStream_t st);
hipError_t launch_wgrad_sqnorm(const GemmArgs& a, int norm_route, hipStream_t st);
hipError_t launch_dgrad(const GemmArgs& a, hipStream_t st);
// A = W [M = N_out x C = K_in], B = X [Nn = T x C], Out = Y [T x N_out]; accumulate: Y <- rne16(Y + acc).
hipError_t launch_forward(const GemmArgs& a, bool accumulate, hipStream_t st);

// Row-wise kernels -------------------------------------------------------------------------
struct EmbeddingWs {          // carved out of the caller's workspace
    uint64_t* keys;           // [Tpad] (id << 32 | position), padded with all-ones
    uint64_t* keys2;          // [Tpad] second key buffer of the merge rounds (batches above 8192 positions; else null)
    int32_t* perm;            // [T]
    int32_t* unique_ids;      // [T]
    int32_t* seg_offsets;     // [T + 1]
    int32_t* n_unique;        // [1]
    double* partials;         // per-wave / per-workgroup shares of the squared norm
    float* chunk_rows;        // [2 * ceil(T / 16)][H] fp32 partial sums of runs that cross chunk boundaries
};
size_t embedding_ws_bytes(int64_t T, int64_t H);
size_t embedding_grouping_bytes(int64_t T);     // head of the workspace: what launch_embedding_grouping fills
EmbeddingWs carve_embedding_ws(void* ws, int64_t T, int64_t H);
hipError_t launch_embedding_grouping(const int32_t* ids, int64_t T, int64_t V, const EmbeddingWs& w, hipStream_t st);
// mode 0: squared norm into acc (+ flag_out); mode 1: in-place row update honouring flag_in;
// mode 2: clip-by-value update, g = clamp(sum * s, -clipv, clipv), W -= lr * g, raising flag_out
// (and leaving the element alone) where the sum is not finite.  In mode 2, s is 1 / loss scale.
hipError_t launch_embedding_rows(const int32_t* ids, const uint16_t* dY, uint16_t* W, int64_t T, int64_t H,
                                 const EmbeddingWs& w, int mode, float s, double* acc, int32_t* flag_out, const int32_t* flag_in,
                                 hipStream_t st, float lr = 0.f, float clipv = 0.f, const float* s_dev = nullptr);

size_t vector_ws_bytes(int64_t T, int64_t H);
hipError_t launch_vector(const uint16_t* Xhat, const uint16_t* dY, uint16_t* w, int64_t T, int64_t H,
                         void* ws, int mode, float s, double* acc, int32_t* flag_out, const int32_t* flag_in,
                         hipStream_t st, float lr = 0.f, float clipv = 0.f, const float* s_dev = nullptr);
// mode 1 with s_dev: the step is read from device memory (written by launch_step_scalars earlier on the stream).

// Gain vectors of one shape [T x H] in one launch per stage (kernel arguments carry the pointers).
constexpr int VEC_BATCH = 64;
struct VecItem {
    const uint16_t* Xhat;
    const uint16_t* dY;
    uint16_t* w;            // null in mode 0
    int32_t* flag_out;      // modes 0 and 2, may be null
};
struct VecBatch {
    const uint16_t* Xh[VEC_BATCH];
    const uint16_t* dY[VEC_BATCH];
    uint16_t* w[VEC_BATCH];
    int32_t* flag_out[VEC_BATCH];
};
// ws_bytes decides how many vectors share a launch: floor(ws_bytes / vector_ws_bytes(T, H)), at least 1 required.
hipError_t launch_vector_batch(const VecItem* items, int n, int64_t T, int64_t H, void* ws, size_t ws_bytes, int mode,
                               float s, double* acc, const int32_t* flag_in, hipStream_t st, float lr = 0.f,
                               float clipv = 0.f, const float* s_dev = nullptr);

// Device-side form of the host coefficient: reads the scaled squared norm and the step flag, writes
// {clip, norm, step = lr * clip / S, overflow} to `out`.
hipError_t launch_step_scalars(const double* acc, const int32_t* step_flag, double loss_scale, double max_norm, double eps,
                               double lr, lomo_step_scalars* out, hipStream_t st);

// Event timing (lomo_timing.hip).  Contraction kernels attach the events to their own dispatch
// (no extra packets on the stream); multi-kernel families bracket their launches instead.
bool timing_slot(int family, hipEvent_t* start, hipEvent_t* stop);
// begin returns true iff a start event was recorded.
bool timing_begin(int family, hipStream_t st);
void timing_end(int family, hipStream_t st);
struct ScopedTiming {
    int family;
    hipStream_t st;
    bool on;
    ScopedTiming(int f, hipStream_t s) : family(f), st(s), on(timing_begin(f, s)) {}
    ~ScopedTiming() {
        if (on) timing_end(family, st);
    }
};

// Raises a kernel's dynamic-LDS limit; callers keep the result in a function-local static, whose initialisation is
// thread-safe, so concurrent first launches make the runtime call once per kernel.
template <typename Kern>
inline hipError_t allow_dynamic_lds(Kern kern, int bytes) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

// Launch with the family's timing events attached when timing is on.
template <typename Kern, typename... Args>
inline hipError_t launch_timed(int family, Kern kern, dim3 grid, dim3 block, size_t lds, hipStream_t st, Args... args) {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (timing_slot(family, &e0, &e1)) hipExtLaunchKernelGGL(kern, grid, block, (uint32_t)lds, st, e0, e1, 0, args...);
    else hipLaunchKernelGGL(kern, grid, block, lds, st, args...);
    return hipGetLastError();
}

// Feed-forward block chain (lomo_chain.hip): rows of gate_up / dgate_up are [gate | up], 2F wide.
hipError_t launch_swiglu_backward(const uint16_t* da, const uint16_t* gate_up, uint16_t* dgate_up, int64_t T, int64_t F,
                                  hipStream_t st);
hipError_t launch_rmsnorm_backward(const uint16_t* dxn, const uint16_t* xhat, const float* rstd, const uint16_t* gain,
                                   const uint16_t* dres, uint16_t* dh, int64_t T, int64_t H, hipStream_t st);

// Forward steps for activation recomputation and the loss (lomo_forward.hip, lomo_attention_fwd.hip).
hipError_t launch_rmsnorm_forward(const uint16_t* h, const uint16_t* gain, float eps, uint16_t* xhat, float* rstd, uint16_t* xn,
                                  int64_t T, int64_t H, hipStream_t st);
hipError_t launch_swiglu_forward(const uint16_t* gate_up, uint16_t* a, int64_t T, int64_t F, hipStream_t st);
hipError_t launch_rope_forward(uint16_t* qkv, const float* cosv, const float* sinv, int64_t T, int64_t s, int64_t nh, hipStream_t st);
hipError_t launch_cross_entropy(const uint16_t* z, const int32_t* target, float grad_scale, float* loss, uint16_t* dz, int64_t T,
                                int64_t V, hipStream_t st);
hipError_t launch_cross_entropy_mean(const uint16_t* z, const int32_t* target, double loss_scale, float* loss, uint16_t* dz,
                                     double* stats, int64_t T, int64_t V, hipStream_t st);
hipError_t launch_embedding_forward(const int32_t* ids, const uint16_t* W, uint16_t* h, int64_t T, int64_t H, int64_t V,
                                    hipStream_t st);
hipError_t launch_attention_forward(const uint16_t* qkv, uint16_t* o, float* lse, int64_t B, int64_t s, int64_t nh, hipStream_t st);

// Causal attention backward with the rotary step (lomo_attention.hip): head width 128, s % 64 == 0.
hipError_t launch_attention_backward(const uint16_t* qkv, const uint16_t* o, const uint16_t* dO, const float* lse,
                                     const float* cosv, const float* sinv, float* delta, uint16_t* dqkv, int64_t B, int64_t s,
                                     int64_t nh, hipStream_t st);

hipError_t launch_reduce_flags(const int32_t* flags, int64_t n, int32_t* out, hipStream_t st);

}  // namespace lomo

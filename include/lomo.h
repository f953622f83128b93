/*
 * lomo.h -- C ABI of the LOMO fused backward + update hot path for AMD MI355X (gfx950).
 *
 * LOMO (LOw-Memory Optimization, arXiv 2306.09782) applies the SGD update of a parameter
 * inside back-propagation, as soon as that parameter's gradient exists, and never stores
 * a gradient tensor (paper section 3.2, Algorithm 1).  With global gradient-norm clipping
 * and a dynamic loss scaler the step takes two passes over the parameters (section 3.3):
 *
 *   pass 1  for every parameter, in backward order: form its gradient, add its squared
 *           norm into one accumulator, raise a flag if it holds inf/NaN, drop it;
 *   host    norm -> clipping coefficient; overflow -> the step is dropped, scale halved;
 *   pass 2  for every parameter: dX from the pre-update weights, then gradient and update
 *           fused: W <- round_fp16( W - lr * clip * G / loss_scale ), computed in fp32.
 *
 * Conventions that hold for every call unless stated otherwise
 *   - lomo_half is IEEE binary16 bits.  All tensors are row-major and live in DEVICE memory.
 *   - linear tensor: W [N x K] (N out-features, K in-features), X [T x K], dY [T x N],
 *     dX [T x K]; forward was Y = X W^T; scaled gradient G = dY^T X; dX = dY W.
 *     dY carries the loss scale; inv_loss_scale = 1 / loss_scale removes it.
 *   - the caller owns every buffer; the library allocates no device memory and keeps no state that
 *     changes a result between calls (what it does keep: the event pool of lomo_timing_*, one-time
 *     kernel attributes, the fixed scratch array of lomo_vector_update_static, described with that
 *     call, and a 16 KB array of counters through which the workgroups of the fused update kernel
 *     keep in step, cleared before every such launch: it affects timing only).  Every choice that
 *     changes how a result is computed is an argument.  Calls
 *     launch on `stream` (a hipStream_t, NULL = default stream) and never synchronise.  `acc` and
 *     `overflow_flag` are zeroed by the caller before pass 1.
 *   - pointers must be 16-byte aligned; K, N and H must be multiples of 8; T >= 0 is free.
 *     X / dY must not alias W / dX.  Token ids must lie in [0, V).
 *   - errors are return codes.  Every argument check is made before the first launch, so a call that
 *     returns LOMO_ERR_NULL / SHAPE / ALIGN / WORKSPACE has launched nothing.  LOMO_ERR_LAUNCH means the
 *     HIP runtime refused a launch: a per-tensor call has then queued at most its dgrad, a whole-pass
 *     call (lomo_step_*) may have queued the launches that came before the refused one, and the caller
 *     should treat the step's outputs as undefined.  Sizes equal to zero are accepted and do nothing.
 */
#ifndef LOMO_H
#define LOMO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LOMO_OK = 0,
    LOMO_ERR_NULL = 1,       /* a required pointer is NULL                       */
    LOMO_ERR_SHAPE = 2,      /* negative size, or K/N/H not a multiple of 8      */
    LOMO_ERR_ALIGN = 3,      /* a pointer is not 16-byte aligned                 */
    LOMO_ERR_WORKSPACE = 4,  /* workspace NULL or smaller than *_workspace_bytes */
    LOMO_ERR_LAUNCH = 5,     /* the HIP runtime refused a launch                 */
    LOMO_ERR_TOO_LARGE = 6   /* beyond the fixed scratch of lomo_vector_update_static */
} lomo_status;

typedef uint16_t lomo_half;

/* Library version (major * 1000 + minor). */
int lomo_version(void);
/* Static string for a status code. */
const char* lomo_status_str(lomo_status s);

/* ---------------------------------------------------------------- pass 1 (section 3.3.1: the
 * additional backward pass that accumulates every parameter's gradient norm; section 3.3.2: the
 * same pass identifies overflow). */

/* acc[0] += sum_{n,k} ( sum_t dY[t,n] * X[t,k] )^2  -- squared Frobenius norm of the SCALED
 * gradient of one linear tensor, without storing it.  fp16 inputs, fp32 MFMA accumulation,
 * fp32 partial sums per workgroup, one double atomic per workgroup into acc (device double).
 * overflow_flag (device int32, may be NULL): set to 1 if any gradient element is inf/NaN. */
lomo_status lomo_wgrad_sqnorm(const lomo_half* X, const lomo_half* dY,
                              int64_t T, int64_t K, int64_t N,
                              double* acc, int32_t* overflow_flag, void* stream);

/* How a norm-pass call obtains ||dY^T X||^2 of a linear tensor (section 3.3.1 asks only for the norm).
 *   LOMO_NORM_DIRECT  contract the gradient tile by tile and square it (2 T N K flop).  What
 *                     lomo_wgrad_sqnorm does.
 *   LOMO_NORM_GRAM    sum over token pairs of (x_t . x_t')(dy_t . dy_t'), lower triangle only
 *                     (T^2 (K + N) flop); needs T % 256 == 0, K % 128 == 0, N % 128 == 0 and dense
 *                     rows, other tensors take the direct route.  Same value up to rounding, same
 *                     overflow flag; its rounding error is relative to sum_t |x_t|^2 |dy_t|^2 instead
 *                     of ||G||^2, so it loses accuracy when per-token gradients cancel in the sum.
 *   LOMO_NORM_AUTO    per tensor, whichever the cost model says is faster.
 * The route is an argument of the call that uses it; the library holds no setting. */
enum { LOMO_NORM_DIRECT = 0, LOMO_NORM_AUTO = 1, LOMO_NORM_GRAM = 2 };

/* lomo_wgrad_sqnorm with the route given.  LOMO_ERR_SHAPE for an unknown norm_algorithm. */
lomo_status lomo_wgrad_sqnorm_route(const lomo_half* X, const lomo_half* dY,
                                    int64_t T, int64_t K, int64_t N,
                                    double* acc, int32_t* overflow_flag, int norm_algorithm, void* stream);

/* Same quantity for an embedding table [V x H] whose rows were gathered by ids [T] (device
 * int32): the gradient of row v is the sum of the dY rows at the positions holding id v.
 * The positions are sorted by (id, position); the sorted list is cut into chunks of 16, each chunk's
 * rows are added in order in fp32, and the partial sums of an id that spans chunks are added in chunk
 * order: the order of every sum depends on the ids alone, so results are bit-reproducible.
 * ws: device workspace of at least lomo_embedding_workspace_bytes(T, H) bytes (about T * H / 2 bytes:
 * fp32 partial rows of ids that cross chunk boundaries). */
lomo_status lomo_embedding_sqnorm(const int32_t* ids, const lomo_half* dY,
                                  int64_t T, int64_t H, int64_t V,
                                  void* ws, size_t ws_bytes,
                                  double* acc, int32_t* overflow_flag, void* stream);

/* Same quantity for an RMSNorm gain w [H] in y = xhat * w: g[j] = sum_t dY[t,j] * xhat[t,j].
 * Xhat, dY: [T x H].  ws: at least lomo_vector_workspace_bytes(T, H) bytes. */
lomo_status lomo_vector_sqnorm(const lomo_half* Xhat, const lomo_half* dY,
                               int64_t T, int64_t H,
                               void* ws, size_t ws_bytes,
                               double* acc, int32_t* overflow_flag, void* stream);

/* ---------------------------------------------------------------- host step between the passes */

/* clip = min(1, max_norm / (sqrt(acc_sqnorm_scaled) / loss_scale + eps)): global-norm clipping
 * of the unscaled gradient (appendix A: max grad norm 1.0).  Host function, host arguments. */
double lomo_clip_coef(double acc_sqnorm_scaled, double loss_scale, double max_norm, double eps);

/* Dynamic loss scaler of section 3.3.2 (host function, host pointers): on overflow the scale is
 * halved and the clean-step counter reset; otherwise the counter is incremented and, when it
 * reaches growth_interval, the scale is doubled and the counter reset.  Scale stays in [1, 2^24]. */
void lomo_scaler_step(float* loss_scale, int32_t* clean_steps, int32_t growth_interval, int overflow);

/* out[0] = 1 if any of flags[0..n) is non-zero else 0 (device pointers).  Lets a caller keep one
 * flag per tensor for diagnosis and still hand a single step flag to pass 2. */
lomo_status lomo_reduce_flags(const int32_t* flags, int64_t n, int32_t* out, void* stream);

/* ---------------------------------------------------------------- pass 2 (section 3.2, Algorithm 1:
 * theta_l <- theta_l - lr * g_l as soon as g_l exists; section 3.3.2: in full precision) */

/* One linear tensor: if dX != NULL, dX = round_fp16(dY W) is computed first from the pre-update W;
 * then W[n,k] <- round_fp16( float(W[n,k]) - s * sum_t dY[t,n] X[t,k] ) with
 * s = lr * clip_coef * inv_loss_scale formed once in double and rounded to float; the product is
 * accumulated in fp32 on the matrix cores and the result rounded once (nearest-even) to fp16.
 * No gradient element is written to memory.  overflow_flag (device, may be NULL): if it holds a
 * non-zero value when the kernel runs, W is left untouched (dX is still produced). */
lomo_status lomo_linear_backward_update(const lomo_half* X, const lomo_half* dY, lomo_half* W,
                                        lomo_half* dX,
                                        int64_t T, int64_t K, int64_t N,
                                        float lr, float inv_loss_scale, float clip_coef,
                                        const int32_t* overflow_flag, void* stream);

/* Embedding table W [V x H]: positions are grouped by id with a stable sort (ties by position),
 * each touched row's gradient is the fp32 sum of its dY rows taken in a fixed order that depends
 * only on the ids (bit-reproducible), and the row is updated in place as above.  Rows whose id does not occur are
 * neither read nor written. */
lomo_status lomo_embedding_update(const int32_t* ids, const lomo_half* dY, lomo_half* W,
                                  int64_t T, int64_t H, int64_t V,
                                  float lr, float inv_loss_scale, float clip_coef,
                                  const int32_t* overflow_flag,
                                  void* ws, size_t ws_bytes, void* stream);

/* RMSNorm gain w [H]: w[j] <- round_fp16( float(w[j]) - s * sum_t dY[t,j] * xhat[t,j] ). */
lomo_status lomo_vector_update(const lomo_half* Xhat, const lomo_half* dY, lomo_half* w,
                               int64_t T, int64_t H,
                               float lr, float inv_loss_scale, float clip_coef,
                               const int32_t* overflow_flag,
                               void* ws, size_t ws_bytes, void* stream);

/* lomo_vector_update for callers that cannot allocate device memory or carry a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arithmetic, same kernels, same result bit
 * for bit; the partial column sums go to a fixed array of LOMO_VECTOR_STATIC_BYTES (4 MiB) of device memory inside
 * the library instead of a caller workspace.  Each GPU the library runs on holds that array until the process ends.
 * The call allocates nothing (no hipMalloc / hipFree, no event, no stream), records no timing, and returns
 * LOMO_ERR_TOO_LARGE when lomo_vector_workspace_bytes(T, H) exceeds the array (H up to 8192 fits for any T).
 * Every call on one GPU uses the same array: calls that overlap in time on one GPU (different streams, different
 * threads) race with each other; calls on one stream are ordered and safe.  Nothing in the array has to start at
 * zero (every partial sum is written before it is read). */
#define LOMO_VECTOR_STATIC_BYTES (4u << 20)
lomo_status lomo_vector_update_static(const lomo_half* Xhat, const lomo_half* dY, lomo_half* w,
                                      int64_t T, int64_t H,
                                      float lr, float inv_loss_scale, float clip_coef,
                                      const int32_t* overflow_flag, void* stream);

/* ---------------------------------------------------------------- whole passes over a list of tensors
 *
 * The same two passes, taken over all tensors of a step in one call each, so that the library can run
 * the contractions of many tensors in a few persistent launches (one ramp-up per pass, partial last
 * rounds of one tensor filled with tiles of the next).  Results are those of the per-tensor calls
 * above made in list order: within the update pass every dX is computed from pre-update weights
 * (all dgrads run before any update), and tensors are independent otherwise (Algorithm 1 couples
 * them only through the clipping coefficient). */

typedef enum { LOMO_TENSOR_LINEAR = 0, LOMO_TENSOR_EMBEDDING = 1, LOMO_TENSOR_VECTOR = 2 } lomo_tensor_kind;

typedef struct {
    int32_t kind;          /* lomo_tensor_kind                                                     */
    const lomo_half* X;    /* linear: X [T x K]; vector: xhat [T x K]; embedding: unused (NULL)     */
    const lomo_half* dY;   /* linear: [T x N]; embedding and vector: [T x K]                        */
    lomo_half* W;          /* linear: [N x K]; embedding: [N x K] (N = vocabulary); vector: [K]     */
    lomo_half* dX;         /* linear only, may be NULL                                              */
    const int32_t* ids;    /* embedding only: [T]                                                   */
    int64_t T, K, N;       /* linear: K in-features, N out-features; embedding: K = H, N = V;
                              vector: K = H, N = 1                                                  */
} lomo_tensor;

/* Choices of a whole-pass call, owned by the caller; a NULL pointer means all zeros (the defaults). */
typedef struct lomo_step_options {
    int32_t norm_algorithm;   /* lomo_step_norm_pass: LOMO_NORM_* route of the linear tensors (0 = direct)       */
    int32_t reuse_grouping;   /* update passes: non-zero promises that `ws` still holds what lomo_step_norm_pass
                                 left there for the SAME tensor list (nothing else wrote to it since), so the
                                 embedding's token grouping is not computed a second time.  Only used when the
                                 list holds exactly one embedding tensor.                                          */
} lomo_step_options;

/* Device workspace needed by the row kernels of the listed tensors (host function).  Layout: the embedding's
 * token grouping first (kept between the passes of a step), then one area shared by the embedding's partial
 * rows and the gain vectors' partial column sums.  All gain vectors of equal shape run in one launch per stage
 * as far as that area holds their partial sums (it is sized for 64 MiB of them at most: 64 vectors at the 7B
 * shape); a smaller workspace is accepted as long as it holds one vector's. */
size_t lomo_step_workspace_bytes(const lomo_tensor* tensors, int64_t n);
/* The least `ws_bytes` the whole-pass calls accept for the list (one gain vector per launch). */
size_t lomo_step_workspace_min_bytes(const lomo_tensor* tensors, int64_t n);

/* Pass 1 over tensors[0..n) (host array of descriptors, device buffers inside): acc[0] += the squared
 * norm of every scaled gradient; flags[i] |= 1 if tensor i's gradient holds inf/NaN; finally
 * flags[n] = any(flags[0..n)).  acc (device double) and flags (device int32[n + 1]) are zeroed by the
 * caller.  W and dX members are ignored. */
lomo_status lomo_step_norm_pass(const lomo_tensor* tensors, int64_t n, double* acc, int32_t* flags,
                                void* ws, size_t ws_bytes, const lomo_step_options* options, void* stream);

/* Pass 2 over the same list: dX (where given) and the fused gradient + SGD update of every tensor,
 * W <- round_fp16(W - lr * clip_coef * inv_loss_scale * G), skipped entirely if step_flag[0] != 0. */
lomo_status lomo_step_update_pass(const lomo_tensor* tensors, int64_t n,
                                  float lr, float inv_loss_scale, float clip_coef,
                                  const int32_t* step_flag, void* ws, size_t ws_bytes,
                                  const lomo_step_options* options, void* stream);

/* The coefficient of a step without a host round trip (sections 3.3.1 and 3.3.2, appendix A): a one-thread
 * kernel reads the scaled squared norm acc[0] and the step flag that pass 1 left on the device and
 * writes, to device memory,
 *     grad_norm = sqrt(acc) / loss_scale,  clip_coef = min(1, max_norm / (grad_norm + eps)),
 *     step = (float)(lr * clip_coef / loss_scale)   (formed in double, rounded once),
 *     overflow = step_flag[0] != 0;   clip_coef = step = 0 if overflow or grad_norm is not finite.
 * lomo_step_update_pass_device is lomo_step_update_pass with the step size read from scalars->step by
 * the kernels themselves, so norm pass, coefficient and update pass can be queued back to back on one
 * stream (or captured into a graph) and the host reads `scalars` whenever it likes.
 * scalars: device memory, 8-byte aligned, caller-owned. */
typedef struct lomo_step_scalars {
    double clip_coef;
    double grad_norm;
    float step;
    int32_t overflow;
} lomo_step_scalars;

lomo_status lomo_step_scalars_device(const double* acc, const int32_t* step_flag, double loss_scale, double max_norm,
                                     double eps, double lr, lomo_step_scalars* scalars, void* stream);
lomo_status lomo_step_update_pass_device(const lomo_tensor* tensors, int64_t n, const lomo_step_scalars* scalars,
                                         const int32_t* step_flag, void* ws, size_t ws_bytes,
                                         const lomo_step_options* options, void* stream);

/* ---------------------------------------------------------------- clip by value (section 3.3.1, first
 * alternative): one pass, no norm.  Each element of the unscaled gradient g = G / loss_scale is clamped
 * to [-clip_value, clip_value] and applied at once: W <- round_fp16(float(W) - lr * clamp(g)), fp32
 * arithmetic, one rounding.  The paper's example: [1.3, 0.8] clipped at 1.0 becomes [1.0, 0.8].
 * Overflow cannot be known before updating in a single pass: an element whose gradient is inf/NaN is
 * left unchanged and the flag is raised, so the host can still halve the loss scale. */

/* One linear tensor (dX as in lomo_linear_backward_update).  overflow_flag: device int32, |= 1, may be NULL. */
lomo_status lomo_linear_backward_update_clip_value(const lomo_half* X, const lomo_half* dY, lomo_half* W,
                                                   lomo_half* dX, int64_t T, int64_t K, int64_t N,
                                                   float lr, float inv_loss_scale, float clip_value,
                                                   int32_t* overflow_flag, void* stream);

/* A whole step in one pass over a tensor list (all kinds).  flags: device int32[n + 1], zeroed by the
 * caller; flags[i] |= 1 where tensor i met a non-finite gradient element, flags[n] = any. */
lomo_status lomo_step_update_pass_clip_value(const lomo_tensor* tensors, int64_t n,
                                             float lr, float inv_loss_scale, float clip_value,
                                             int32_t* flags, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------- helpers */

/* Workspace sizes in bytes (host functions; 0 for T == 0). */
size_t lomo_embedding_workspace_bytes(int64_t T, int64_t H);
size_t lomo_vector_workspace_bytes(int64_t T, int64_t H);

/* The grouping that the embedding calls use, exposed so it can be compared bit for bit:
 * perm [T] = positions sorted by (id, position); unique_ids [<= T] ascending; seg_offsets
 * [<= T + 1] with segment u = perm[seg_offsets[u] .. seg_offsets[u+1]); n_unique [1].
 * All outputs are device int32 arrays owned by the caller (capacity T, T, T + 1, 1). */
lomo_status lomo_embedding_grouping(const int32_t* ids, int64_t T, int64_t V,
                                    void* ws, size_t ws_bytes,
                                    int32_t* unique_ids, int32_t* seg_offsets, int32_t* perm,
                                    int32_t* n_unique, void* stream);

/* ---------------------------------------------------------------- diagnostics */

/* ---------------------------------------------------------------- backward loop through a feed-forward block
 * Algorithm 1 of the paper walks back through the layers: each parameter's gradient is formed and applied,
 * and the gradient of the layer input is handed to the layer below (section 3.2).  These calls are the
 * steps between the linear tensors of a LLaMA feed-forward block (the models of section 4):
 *     xhat = h * rstd (per token), xn = xhat * gain, [gate | up] = xn W_gu^T, a = silu(gate) * up,
 *     y = h + a W_d^T.
 * All buffers device memory, row-major fp16 unless stated, caller-owned, 16-byte aligned; asynchronous on
 * `stream`; fp32 arithmetic, each stored element rounded once. */

/* dX = dY W alone (dY [T x N], W [N x K], dX [T x K]): pass 1 of a chained step needs the hand-on gradient
 * but must not touch W.  Same kernel and shape rules as the dgrad inside lomo_linear_backward_update. */
lomo_status lomo_linear_dgrad(const lomo_half* dY, const lomo_half* W, lomo_half* dX,
                              int64_t T, int64_t K, int64_t N, void* stream);

/* SwiGLU backward.  da [T x F]; gate_up and dgate_up [T x 2F], each row [gate | up]:
 *   dgate = da * up * s * (1 + gate * (1 - s)),  dup = da * gate * s,  s = 1 / (1 + exp(-gate)).
 * F % 8 == 0.  dgate_up may not alias the inputs. */
lomo_status lomo_swiglu_backward(const lomo_half* da, const lomo_half* gate_up, lomo_half* dgate_up,
                                 int64_t T, int64_t F, void* stream);

/* RMSNorm backward.  dxn, xhat, dh [T x H]; rstd [T] fp32 (1 / sqrt(mean(h^2) + eps) from the forward pass);
 * gain [H]; dres [T x H] or NULL (gradient arriving through the residual connection, added in):
 *   dh = dres + rstd * (dxn * gain - xhat * mean_j(dxn * gain * xhat)).
 * H % 8 == 0.  dh may alias dres (each element is read before it is written by the same thread), nothing else. */
lomo_status lomo_rmsnorm_backward(const lomo_half* dxn, const lomo_half* xhat, const float* rstd,
                                  const lomo_half* gain, const lomo_half* dres, lomo_half* dh,
                                  int64_t T, int64_t H, void* stream);

/* Causal self-attention backward with the rotary position step, for the hand-on gradient through the
 * attention block of a LLaMA layer.  Tokens t = b * s + pos (B sequences of length s); head n owns columns
 * [n d, (n + 1) d) of q, k, v, o; d = head_dim must be 128 and s a multiple of 64 (else LOMO_ERR_SHAPE).
 *   qkv   [T x 3H] rotated q | rotated k | v as saved by the forward pass (H = n_heads * d)
 *   o     [T x H]  attention output;  dO [T x H] its gradient
 *   lse   [T x n_heads] fp32, log sum_j exp(q_i . k_j / sqrt(d)) over the keys j <= i
 *   rope_cos, rope_sin [s x d/2] fp32 (angle pos * theta_c), or both NULL for no rotary step
 *   delta_ws [T x n_heads] fp32 scratch (receives do_i . o_i)
 *   dqkv  [T x 3H] out: dq | dk | dv, the gradient of the fused projection's output
 * P = exp(S - lse), dP = dO v^T, dS = P (dP - delta) / sqrt(d), dv = P^T dO, dk = dS^T q, dq = dS k, then
 * dq and dk are rotated by the negative angle (pairs (c, c + d/2)).  fp32 accumulation; P and dS pass through
 * fp16 before the products that consume them; outputs rounded once.  Deterministic (no atomics). */
lomo_status lomo_attention_backward(const lomo_half* qkv, const lomo_half* o, const lomo_half* dO, const float* lse,
                                    const float* rope_cos, const float* rope_sin, float* delta_ws, lomo_half* dqkv,
                                    int64_t B, int64_t s, int64_t n_heads, int64_t head_dim, void* stream);

/* ---------------------------------------------------------------- forward steps: activation recomputation, loss
 * With activation checkpointing (paper section 2; section 4.1: 45.61 GB -> 1.79 GB of activations at 7B) only each
 * layer's input is kept, and the activations the backward loop of Algorithm 1 reads are recomputed from it just
 * before the loop enters the layer.  These are the forward steps of a LLaMA decoder layer in the same storage
 * convention as the backward steps above (fp16 tensors, fp32 arithmetic, one rounding per stored element). */

/* Y = X W^T (accumulate == 0) or Y <- Y + X W^T rounded once (accumulate != 0: Y holds the residual stream).
 * X [T x K], W [N x K], Y [T x N]; K % 8 == 0, N % 8 == 0.  Y may not alias X or W. */
lomo_status lomo_linear_forward(const lomo_half* X, const lomo_half* W, lomo_half* Y,
                                int64_t T, int64_t K, int64_t N, int accumulate, void* stream);

/* Y = rne16(R + X W^T) with the residual stream R [T x N] read from its own buffer (R may be Y itself, which is
 * lomo_linear_forward with accumulate).  Same shape rules. */
lomo_status lomo_linear_forward_residual(const lomo_half* X, const lomo_half* W, const lomo_half* R, lomo_half* Y,
                                         int64_t T, int64_t K, int64_t N, void* stream);

/* Embedding rows: h[t] = W[ids[t]] (ids [T] int32, W [V x H], h [T x H]); an id outside [0, V) gives a zero row.
 * H % 8 == 0. */
lomo_status lomo_embedding_forward(const int32_t* ids, const lomo_half* W, lomo_half* h,
                                   int64_t T, int64_t H, int64_t V, void* stream);

/* RMSNorm forward: rstd[t] = 1 / sqrt(mean_j h[t][j]^2 + eps) (fp32 [T]), xhat = h * rstd, xn = xhat * gain with
 * xhat taken as stored.  h, xhat, xn [T x H]; gain [H]; H % 8 == 0.  xhat or xn may not alias h. */
lomo_status lomo_rmsnorm_forward(const lomo_half* h, const lomo_half* gain, float eps, lomo_half* xhat, float* rstd,
                                 lomo_half* xn, int64_t T, int64_t H, void* stream);

/* SwiGLU forward: a = gate / (1 + exp(-gate)) * up.  gate_up [T x 2F] rows [gate | up]; a [T x F]; F % 8 == 0. */
lomo_status lomo_swiglu_forward(const lomo_half* gate_up, lomo_half* a, int64_t T, int64_t F, void* stream);

/* Rotary position step, in place on the q and k parts of qkv [T x 3H] (H = n_heads * 128, token t at position
 * t % s): pairs (c, c + 64) of each head are rotated by the angle whose cosine / sine is rope_cos / rope_sin
 * [s x 64] fp32.  head_dim must be 128. */
lomo_status lomo_rope_forward(lomo_half* qkv, const float* rope_cos, const float* rope_sin,
                              int64_t T, int64_t s, int64_t n_heads, int64_t head_dim, void* stream);

/* Causal self-attention forward on the rotated qkv [T x 3H]: o [T x H] and lse [T x n_heads] fp32 as
 * lomo_attention_backward expects them.  Same shape rules (head_dim 128, s % 64 == 0).  Probabilities pass
 * through fp16 before they multiply v; o is rounded once.  Deterministic. */
lomo_status lomo_attention_forward(const lomo_half* qkv, lomo_half* o, float* lse,
                                   int64_t B, int64_t s, int64_t n_heads, int64_t head_dim, void* stream);

/* Token-level cross-entropy and its scaled gradient (section 3.3.2: the loss is multiplied by the scale before
 * the backward pass).  logits [T x V] fp16, targets [T] int32, loss [T] fp32 out (loss[t] = lse_t - z[t][target]),
 * dlogits [T x V] out = grad_scale * (softmax(z_t) - onehot(target_t)); pass grad_scale = loss_scale / (number of
 * counted tokens) for a mean loss.  A target outside [0, V) leaves its token out: loss 0, zero gradient row.
 * V % 8 == 0.  dlogits may be the logits buffer itself. */
lomo_status lomo_cross_entropy(const lomo_half* logits, const int32_t* targets, float grad_scale, float* loss,
                               lomo_half* dlogits, int64_t T, int64_t V, void* stream);

/* The mean loss of a batch in one call: counts the targets inside [0, V) on the device (n), runs lomo_cross_entropy
 * with grad_scale = (float)(loss_scale / n) (formed in double from the device count), and writes
 * stats[0] = sum_t loss[t] / n (fp64, fixed summation order) and stats[1] = n to device memory (double[3], 8-byte
 * aligned, caller-owned; stats[2] is scratch).  n == 0 gives grad_scale 0, a zero gradient and stats = {0, 0}. */
lomo_status lomo_cross_entropy_mean(const lomo_half* logits, const int32_t* targets, double loss_scale, float* loss,
                                    lomo_half* dlogits, double* stats, int64_t T, int64_t V, void* stream);

/* Kernel families for lomo_timing_read. */
enum { LOMO_KERNEL_WGRAD_UPDATE = 0, LOMO_KERNEL_WGRAD_SQNORM = 1, LOMO_KERNEL_DGRAD = 2,
       LOMO_KERNEL_EMBEDDING = 3, LOMO_KERNEL_VECTOR = 4, LOMO_KERNEL_GRAM_SQNORM = 5, LOMO_KERNEL_CHAIN = 6,
       LOMO_KERNEL_ATTENTION = 7, LOMO_KERNEL_FORWARD = 8, LOMO_KERNEL_PROBE = 9, LOMO_KERNEL_FAMILIES = 10 };

/* Per-kernel timing for benchmarks: while enabled, each launch of a kernel family is bracketed
 * by two HIP events recorded on the launch stream (the only host-side state the library keeps;
 * events are created on first use and reused).  Enabling or disabling resets the counters.
 * lomo_timing_read waits for the recorded events of one family and returns the summed kernel
 * time in milliseconds and the number of timed launches (host pointers). */
lomo_status lomo_timing_enable(int on);
lomo_status lomo_timing_read(int family, double* total_ms, int64_t* launches);

/* ---------------------------------------------------------------- measured ceilings (benchmark aids)
 * The denominators a roofline needs next to the published peaks: what this chip sustains on the matrix cores with
 * nothing else going on, and on a plain streaming copy.  Neither is part of the method. */

/* Matrix-core loop without memory traffic.  One workgroup per CU, waves_per_simd (1 or 2) waves on each of its four
 * SIMDs; every wave loads sixteen 32 x 16 fp16 operand fragments once from `operands` (device, at least
 * LOMO_PROBE_OPERAND_BYTES bytes: all zeros, or N(0,1) values, or anything else the caller wants to measure with)
 * and then issues iters x 32 v_mfma_f32_32x32x16_f16 in the 4 x 4 register blocking of the contraction kernels
 * (iters x 16 in a 4 x 2 blocking with two waves per SIMD, which have half the registers each), alternating
 * between two operand sets.  idle_sleeps (0 .. 4096): each wave sleeps that many times 64 clocks after every
 * iteration, which lowers the duty cycle of the matrix pipes (is the sustained rate set by power, so that idle time is
 * paid back by a higher clock, or by a fixed clock?).  lds_reads != 0: each operand set is re-read from LDS before
 * use (the contraction kernels' LDS read traffic per MFMA, no global loads).  The accumulators are summed into
 * sink[workgroup] (device float[n_cu]) so the work cannot be dropped.  flops_out (host, may be NULL) receives the flop
 * count of the launch.  Timed as family LOMO_KERNEL_PROBE when timing is on. */
#define LOMO_PROBE_OPERAND_BYTES (16 * 64 * 16)
lomo_status lomo_probe_mfma(const lomo_half* operands, int64_t iters, int waves_per_simd, int idle_sleeps, int lds_reads,
                            float* sink, int64_t sink_len, double* flops_out, void* stream);

/* dst[0 .. bytes) = src[0 .. bytes) with 16-byte loads and stores, grid-stride (bytes % 16 == 0, 16-byte aligned
 * pointers): 2 x bytes of HBM traffic.  Timed as family LOMO_KERNEL_PROBE when timing is on. */
lomo_status lomo_probe_copy(const void* src, void* dst, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LOMO_H */

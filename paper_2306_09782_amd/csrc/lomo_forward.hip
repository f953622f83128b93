// Forward steps of a LLaMA decoder layer, so that the activations Algorithm 1's backward loop needs (paper
// section 3.2) can be recomputed from a checkpoint of the layer input instead of being kept (activation
// checkpointing: section 2, and section 4.1 where it takes the 7B activation memory from 45.61 GB to 1.79 GB),
// and the loss whose scaled gradient starts the loop (section 3.3.2: the loss is multiplied by the scale).
//
//   RMSNorm:   rstd = 1 / sqrt(mean_j h^2 + eps),  xhat = h * rstd,  xn = xhat * gain   (xn from the stored xhat)
//   rotary:    (x_c, x_{c+d/2}) <- (x_c cos - x_{c+d/2} sin,  x_{c+d/2} cos + x_c sin),  angle pos * theta_c
//   SwiGLU:    a = gate / (1 + exp(-gate)) * up
//   loss:      loss_t = lse_t - z[t][target_t];  dz = S / n * (softmax(z_t) - onehot(target_t))
//
// fp16 storage, fp32 arithmetic, one rounding per stored element.  All kernels are HBM bound; reductions have
// a fixed order, so results are bit-reproducible.
#include "lomo_kernels.h"

namespace lomo {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));

constexpr int FW_NT = 256;

__device__ __forceinline__ float block_sum_256(float v, float* red) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    const float total = (red[0] + red[1]) + (red[2] + red[3]);
    __syncthreads();
    return total;
}

__device__ __forceinline__ float block_max_256(float v, float* red) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    const float total = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    return total;
}

// One workgroup per token.
__global__ __launch_bounds__(FW_NT) void rmsnorm_forward_kernel(const uint16_t* __restrict__ h, const uint16_t* __restrict__ gain,
                                                                float eps, uint16_t* __restrict__ xhat, float* __restrict__ rstd,
                                                                uint16_t* __restrict__ xn, int64_t H) {
    __shared__ float red[FW_NT / 64];
    const int64_t t = blockIdx.x;
    const uint16_t* row = h + t * H;
    float part = 0.f;
    for (int64_t c = (int64_t)threadIdx.x * 8; c < H; c += FW_NT * 8) {
        const half8 x = *reinterpret_cast<const half8*>(row + c);
#pragma unroll
        for (int e = 0; e < 8; ++e) part = fmaf((float)x[e], (float)x[e], part);
    }
    const float r = 1.0f / sqrtf(block_sum_256(part, red) / (float)H + eps);
    if (threadIdx.x == 0) rstd[t] = r;
    for (int64_t c = (int64_t)threadIdx.x * 8; c < H; c += FW_NT * 8) {
        const half8 x = *reinterpret_cast<const half8*>(row + c);      // still in cache
        const half8 w = *reinterpret_cast<const half8*>(gain + c);
        half8 a, b;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            a[e] = (_Float16)((float)x[e] * r);
            b[e] = (_Float16)((float)a[e] * (float)w[e]);
        }
        *reinterpret_cast<half8*>(xhat + t * H + c) = a;
        *reinterpret_cast<half8*>(xn + t * H + c) = b;
    }
}

// One thread per 8 consecutive features of one token.
__global__ __launch_bounds__(FW_NT) void swiglu_forward_kernel(const uint16_t* __restrict__ gate_up, uint16_t* __restrict__ a,
                                                               int64_t T, int64_t F) {
    const int64_t chunks = F >> 3;
    const int64_t i = (int64_t)blockIdx.x * FW_NT + threadIdx.x;
    if (i >= T * chunks) return;
    const int64_t t = i / chunks, c = (i - t * chunks) << 3;
    const half8 g = *reinterpret_cast<const half8*>(gate_up + t * 2 * F + c);
    const half8 u = *reinterpret_cast<const half8*>(gate_up + t * 2 * F + F + c);
    half8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float gf = (float)g[e];
        o[e] = (_Float16)(gf / (1.f + expf(-gf)) * (float)u[e]);
    }
    *reinterpret_cast<half8*>(a + t * F + c) = o;
}

// In place on the q and k parts of qkv [T x 3H]: one thread per (token, q or k, head, 8 pairs).
__global__ __launch_bounds__(FW_NT) void rope_forward_kernel(uint16_t* __restrict__ qkv, const float* __restrict__ cosv,
                                                             const float* __restrict__ sinv, int64_t T, int s, int nh) {
    const int64_t i = (int64_t)blockIdx.x * FW_NT + threadIdx.x;
    const int64_t per_token = 2 * (int64_t)nh * 8;
    if (i >= T * per_token) return;
    const int64_t t = i / per_token;
    const int rem = (int)(i - t * per_token);
    const int part = rem / (nh * 8), head = (rem / 8) % nh, c0 = (rem & 7) * 8;
    const int pos = (int)(t % s);
    const int64_t H = (int64_t)nh * 128;
    uint16_t* p = qkv + t * 3 * H + part * H + head * 128 + c0;
    const half8 x1 = *reinterpret_cast<const half8*>(p);
    const half8 x2 = *reinterpret_cast<const half8*>(p + 64);
    half8 y1, y2;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float co = cosv[pos * 64 + c0 + e], si = sinv[pos * 64 + c0 + e];
        const float a = (float)x1[e], b = (float)x2[e];
        y1[e] = (_Float16)fmaf(-b, si, a * co);
        y2[e] = (_Float16)fmaf(a, si, b * co);
    }
    *reinterpret_cast<half8*>(p) = y1;
    *reinterpret_cast<half8*>(p + 64) = y2;
}

// One workgroup per token: max, sum of exponentials, then the scaled gradient.  z and dz may be the same buffer.
// grad_scale_dev (when not null) holds the scale in device memory, written earlier on the stream.
__global__ __launch_bounds__(FW_NT) void cross_entropy_kernel(const uint16_t* z, const int32_t* __restrict__ target,
                                                              float grad_scale, const float* __restrict__ grad_scale_dev,
                                                              float* __restrict__ loss, uint16_t* dz, int64_t V) {
    __shared__ float red[FW_NT / 64];
    if (grad_scale_dev != nullptr) grad_scale = grad_scale_dev[0];
    const int64_t t = blockIdx.x;
    const uint16_t* row = z + t * V;
    const int tgt = target[t];
    const bool counted = tgt >= 0 && tgt < V;      // any other target: the token is left out (no loss, zero gradient)
    const float zt = counted ? (float)reinterpret_cast<const _Float16*>(row)[tgt] : 0.f;   // before anything is overwritten
    float m = -INFINITY;
    for (int64_t c = (int64_t)threadIdx.x * 8; c < V; c += FW_NT * 8) {
        const half8 x = *reinterpret_cast<const half8*>(row + c);
#pragma unroll
        for (int e = 0; e < 8; ++e) m = fmaxf(m, (float)x[e]);
    }
    m = block_max_256(m, red);
    float sum = 0.f;
    for (int64_t c = (int64_t)threadIdx.x * 8; c < V; c += FW_NT * 8) {
        const half8 x = *reinterpret_cast<const half8*>(row + c);
#pragma unroll
        for (int e = 0; e < 8; ++e) sum += expf((float)x[e] - m);
    }
    sum = block_sum_256(sum, red);
    const float lse = m + logf(sum);
    if (threadIdx.x == 0) loss[t] = counted ? lse - zt : 0.f;
    const float inv = counted ? grad_scale / sum : 0.f;
    for (int64_t c = (int64_t)threadIdx.x * 8; c < V; c += FW_NT * 8) {
        const half8 x = *reinterpret_cast<const half8*>(row + c);
        half8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float ex = expf((float)x[e] - m);
            o[e] = (_Float16)(((c + e == tgt) ? ex - sum : ex) * inv);      // (p - 1) without cancellation
        }
        *reinterpret_cast<half8*>(dz + t * V + c) = o;
    }
}

// Embedding rows: h[t] = W[ids[t]]; one thread per 16-byte chunk.  An id outside [0, V) gives a zero row.
__global__ __launch_bounds__(FW_NT) void embedding_forward_kernel(const int32_t* __restrict__ ids, const uint16_t* __restrict__ W,
                                                                  uint16_t* __restrict__ h, int64_t T, int64_t H, int64_t V) {
    const int64_t chunks = H >> 3;
    const int64_t i = (int64_t)blockIdx.x * FW_NT + threadIdx.x;
    if (i >= T * chunks) return;
    const int64_t t = i / chunks, c = (i - t * chunks) << 3;
    const int64_t id = ids[t];
    half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
    if (id >= 0 && id < V) v = *reinterpret_cast<const half8*>(W + id * H + c);
    *reinterpret_cast<half8*>(h + t * H + c) = v;
}

hipError_t launch_embedding_forward(const int32_t* ids, const uint16_t* W, uint16_t* h, int64_t T, int64_t H, int64_t V,
                                    hipStream_t st) {
    const int64_t n = T * (H >> 3);
    hipLaunchKernelGGL(embedding_forward_kernel, dim3((unsigned)((n + FW_NT - 1) / FW_NT)), dim3(FW_NT), 0, st, ids, W, h, T, H, V);
    return hipGetLastError();
}

hipError_t launch_rmsnorm_forward(const uint16_t* h, const uint16_t* gain, float eps, uint16_t* xhat, float* rstd, uint16_t* xn,
                                  int64_t T, int64_t H, hipStream_t st) {
    hipLaunchKernelGGL(rmsnorm_forward_kernel, dim3((unsigned)T), dim3(FW_NT), 0, st, h, gain, eps, xhat, rstd, xn, H);
    return hipGetLastError();
}

hipError_t launch_swiglu_forward(const uint16_t* gate_up, uint16_t* a, int64_t T, int64_t F, hipStream_t st) {
    const int64_t n = T * (F >> 3);
    hipLaunchKernelGGL(swiglu_forward_kernel, dim3((unsigned)((n + FW_NT - 1) / FW_NT)), dim3(FW_NT), 0, st, gate_up, a, T, F);
    return hipGetLastError();
}

hipError_t launch_rope_forward(uint16_t* qkv, const float* cosv, const float* sinv, int64_t T, int64_t s, int64_t nh,
                               hipStream_t st) {
    const int64_t n = T * 2 * nh * 8;
    hipLaunchKernelGGL(rope_forward_kernel, dim3((unsigned)((n + FW_NT - 1) / FW_NT)), dim3(FW_NT), 0, st, qkv, cosv, sinv, T,
                       (int)s, (int)nh);
    return hipGetLastError();
}

hipError_t launch_cross_entropy(const uint16_t* z, const int32_t* target, float grad_scale, float* loss, uint16_t* dz, int64_t T,
                                int64_t V, hipStream_t st) {
    hipLaunchKernelGGL(cross_entropy_kernel, dim3((unsigned)T), dim3(FW_NT), 0, st, z, target, grad_scale,
                       static_cast<const float*>(nullptr), loss, dz, V);
    return hipGetLastError();
}

// stats[1] = n = number of targets inside [0, V); stats[2] (as float) = (float)(loss_scale / n), 0 when n == 0.
__global__ __launch_bounds__(FW_NT) void count_targets_kernel(const int32_t* __restrict__ target, int64_t T, int64_t V,
                                                              double loss_scale, double* __restrict__ stats) {
    __shared__ int red[FW_NT];
    int c = 0;
    for (int64_t t = threadIdx.x; t < T; t += FW_NT) c += (target[t] >= 0 && target[t] < V) ? 1 : 0;
    red[threadIdx.x] = c;
    __syncthreads();
    for (int off = FW_NT / 2; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const int n = red[0];
        stats[1] = (double)n;
        *reinterpret_cast<float*>(stats + 2) = n > 0 ? (float)(loss_scale / (double)n) : 0.f;
    }
}

// stats[0] = sum_t loss[t] / n in fp64: threads take strided shares in ascending order, then a fixed tree.
__global__ __launch_bounds__(FW_NT) void mean_loss_kernel(const float* __restrict__ loss, int64_t T, double* __restrict__ stats) {
    __shared__ double red[FW_NT];
    double v = 0.0;
    for (int64_t t = threadIdx.x; t < T; t += FW_NT) v += (double)loss[t];
    red[threadIdx.x] = v;
    __syncthreads();
    for (int off = FW_NT / 2; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) stats[0] = stats[1] > 0.0 ? red[0] / stats[1] : 0.0;
}

// stats: device double[3]; [0] mean loss, [1] counted targets, [2] scratch (the gradient scale as a float).
hipError_t launch_cross_entropy_mean(const uint16_t* z, const int32_t* target, double loss_scale, float* loss, uint16_t* dz,
                                     double* stats, int64_t T, int64_t V, hipStream_t st) {
    hipLaunchKernelGGL(count_targets_kernel, dim3(1), dim3(FW_NT), 0, st, target, T, V, loss_scale, stats);
    if (T > 0)
        hipLaunchKernelGGL(cross_entropy_kernel, dim3((unsigned)T), dim3(FW_NT), 0, st, z, target, 0.f,
                           reinterpret_cast<const float*>(stats + 2), loss, dz, V);
    hipLaunchKernelGGL(mean_loss_kernel, dim3(1), dim3(FW_NT), 0, st, loss, T, stats);
    return hipGetLastError();
}

}  // namespace lomo

// Element-wise and row-wise steps between the contractions of a LLaMA feed-forward block, so that
// Algorithm 1's backward loop (paper section 3.2) can run through a real layer on the GPU: the gradient
// that one linear tensor hands down (dX of the fused kernels) becomes the dY of the next one.
//
//   SwiGLU backward:   dgate = da * up * s (1 + gate (1 - s)),  dup = da * gate * s,  s = 1 / (1 + exp(-gate))
//   RMSNorm backward:  dh = dres + r * (dxn * w - xhat * mean_j(dxn * w * xhat))
//
// fp16 storage, fp32 arithmetic, one rounding per stored element (section 3.3.2).  Both kernels are
// HBM bound.  Reductions have a fixed order: results are bit-reproducible.
#include "lomo_kernels.h"

namespace lomo {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));

constexpr int CH_NT = 256;

// One thread per 8 consecutive features of one token; gate_up and dgate_up rows are [gate | up], 2F wide.
__global__ __launch_bounds__(CH_NT) void swiglu_backward_kernel(const uint16_t* __restrict__ da,
                                                                const uint16_t* __restrict__ gate_up,
                                                                uint16_t* __restrict__ dgate_up, int64_t T, int64_t F) {
    const int64_t chunks = F >> 3;
    const int64_t i = (int64_t)blockIdx.x * CH_NT + threadIdx.x;
    if (i >= T * chunks) return;
    const int64_t t = i / chunks, c = (i - t * chunks) << 3;
    const half8 d = *reinterpret_cast<const half8*>(da + t * F + c);
    const half8 g = *reinterpret_cast<const half8*>(gate_up + t * 2 * F + c);
    const half8 u = *reinterpret_cast<const half8*>(gate_up + t * 2 * F + F + c);
    half8 og, ou;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float gf = (float)g[e], df = (float)d[e], uf = (float)u[e];
        const float s = 1.f / (1.f + expf(-gf));
        og[e] = (_Float16)(df * uf * (s * (1.f + gf * (1.f - s))));
        ou[e] = (_Float16)(df * (gf * s));
    }
    *reinterpret_cast<half8*>(dgate_up + t * 2 * F + c) = og;
    *reinterpret_cast<half8*>(dgate_up + t * 2 * F + F + c) = ou;
}

// One workgroup per token.  Pass A: c = mean_j(dxn * w * xhat), lanes sum their chunks in ascending order,
// waves and then the four wave sums are added in a fixed order.  Pass B re-reads the row (it is still in
// cache) and writes dh.
__global__ __launch_bounds__(CH_NT) void rmsnorm_backward_kernel(const uint16_t* __restrict__ dxn,
                                                                 const uint16_t* __restrict__ xhat,
                                                                 const float* __restrict__ rstd,
                                                                 const uint16_t* __restrict__ gain,
                                                                 const uint16_t* __restrict__ dres,
                                                                 uint16_t* __restrict__ dh, int64_t H) {
    __shared__ float red[CH_NT / 64];
    const int64_t t = blockIdx.x;
    const uint16_t* drow = dxn + t * H;
    const uint16_t* xrow = xhat + t * H;
    float part = 0.f;
    for (int64_t c = (int64_t)threadIdx.x * 8; c < H; c += CH_NT * 8) {
        const half8 d = *reinterpret_cast<const half8*>(drow + c);
        const half8 x = *reinterpret_cast<const half8*>(xrow + c);
        const half8 w = *reinterpret_cast<const half8*>(gain + c);
#pragma unroll
        for (int e = 0; e < 8; ++e) part = fmaf((float)d[e] * (float)w[e], (float)x[e], part);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = part;
    __syncthreads();
    const float cmean = ((red[0] + red[1]) + (red[2] + red[3])) / (float)H;
    const float r = rstd[t];
    for (int64_t c = (int64_t)threadIdx.x * 8; c < H; c += CH_NT * 8) {
        const half8 d = *reinterpret_cast<const half8*>(drow + c);
        const half8 x = *reinterpret_cast<const half8*>(xrow + c);
        const half8 w = *reinterpret_cast<const half8*>(gain + c);
        half8 o;
        if (dres != nullptr) {
            const half8 q = *reinterpret_cast<const half8*>(dres + t * H + c);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                o[e] = (_Float16)fmaf(r, fmaf(-(float)x[e], cmean, (float)d[e] * (float)w[e]), (float)q[e]);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (_Float16)(r * fmaf(-(float)x[e], cmean, (float)d[e] * (float)w[e]));
        }
        *reinterpret_cast<half8*>(dh + t * H + c) = o;
    }
}

hipError_t launch_swiglu_backward(const uint16_t* da, const uint16_t* gate_up, uint16_t* dgate_up, int64_t T, int64_t F,
                                  hipStream_t st) {
    const int64_t n = T * (F >> 3);
    hipLaunchKernelGGL(swiglu_backward_kernel, dim3((unsigned)((n + CH_NT - 1) / CH_NT)), dim3(CH_NT), 0, st, da, gate_up,
                       dgate_up, T, F);
    return hipGetLastError();
}

hipError_t launch_rmsnorm_backward(const uint16_t* dxn, const uint16_t* xhat, const float* rstd, const uint16_t* gain,
                                   const uint16_t* dres, uint16_t* dh, int64_t T, int64_t H, hipStream_t st) {
    hipLaunchKernelGGL(rmsnorm_backward_kernel, dim3((unsigned)T), dim3(CH_NT), 0, st, dxn, xhat, rstd, gain, dres, dh, H);
    return hipGetLastError();
}

}  // namespace lomo

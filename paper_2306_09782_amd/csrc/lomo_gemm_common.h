// Shared pieces of the MFMA contraction kernels: vector types, reductions and the three epilogues.
#pragma once
#include "lomo_kernels.h"

#include <hip/hip_fp16.h>

namespace lomo {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int NT = 256;        // threads per workgroup: 4 waves in a 2 x 2 arrangement

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Epilogue of a BM x BN workgroup tile held as 32x32 MFMA accumulators, 4 waves in 2 x 2.
// Lane (l32, lh) of MFMA tile (i, j) holds, in register 4*q4 + e, the element
//   m = 32 i + 8 q4 + 4 lh + e,  n = 32 j + l32   of the wave's sub-tile,
// so four consecutive registers are four consecutive m: an 8-byte run of the output row.
//   EPI_UPDATE: W <- rne16(float(W) - s * acc)   (section 3.2 update, fp32 as section 3.3.2 asks)
//   EPI_SQNORM: one fp32 sum of squares per workgroup -> double atomic; inf/NaN -> flag
//   EPI_STORE : Out <- rne16(acc)
template <int BM, int BN, int EPI>
__device__ __forceinline__ void epilogue(floatx16 (&acc)[BM / 64][BN / 64], const GemmArgs& g, uint16_t* smem,
                                         int64_t m0, int64_t n0, int m_rem, int n_rem) {
    constexpr int TM = BM / 64, TN = BN / 64;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const int l32 = lane & 31, lh = lane >> 5;
    if constexpr (EPI == EPI_SQNORM) {
        float sum = 0.f;
        uint32_t worst = 0u;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float v = acc[i][j][r];
                    sum = fmaf(v, v, sum);
                    const uint32_t mag = __float_as_uint(v) & 0x7fffffffu;
                    worst = mag > worst ? mag : worst;
                }
        sum = wave_sum(sum);
        const bool bad = __any(worst >= 0x7f800000u);
        float* red = reinterpret_cast<float*>(smem);   // main loop is over: LDS is free
        int* redflag = reinterpret_cast<int*>(smem) + 8;
        if (lane == 0) {
            red[wave] = sum;
            redflag[wave] = bad ? 1 : 0;
        }
        __syncthreads();
        if (tid == 0) {
            const float total = (red[0] + red[1]) + (red[2] + red[3]);
            atomicAdd(g.acc, (double)total);
            if (g.flag_out != nullptr && (redflag[0] | redflag[1] | redflag[2] | redflag[3])) atomicOr(g.flag_out, 1);
        }
    } else {
        const float s = g.s;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int nl = wn * (BN / 2) + 32 * j + l32;
            if (nl >= n_rem) continue;
            uint16_t* row = g.Out + (n0 + nl) * g.ldo + m0;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const int ml = wm * (BM / 2) + 32 * i + 8 * q4 + 4 * lh;
                    if (ml >= m_rem) continue;
                    half4* p = reinterpret_cast<half4*>(row + ml);
                    half4 out;
                    if constexpr (EPI == EPI_UPDATE) {
                        const half4 w = *p;
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            out[e] = (_Float16)fmaf(-s, acc[i][j][4 * q4 + e], (float)w[e]);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) out[e] = (_Float16)acc[i][j][4 * q4 + e];
                    }
                    *p = out;
                }
            }
        }
    }
}

}  // namespace lomo

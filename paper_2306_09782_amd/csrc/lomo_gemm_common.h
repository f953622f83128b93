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
//   m = 32 i + 8 q4 + 4 lh + e,  n = 32 j + l32   of the wave's sub-tile.
//   EPI_UPDATE: W <- rne16(float(W) - s * acc)   (section 3.2 update, fp32 as section 3.3.2 asks)
//   EPI_SQNORM: one fp32 sum of squares per workgroup -> double atomic; inf/NaN -> flag
//   EPI_STORE : Out <- rne16(acc)
//   EPI_CLIPV : W <- rne16(float(W) - lr * clamp(acc / S, -c, c))   (single-pass alternative of section 3.3.1)
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
        // Lanes l and l + 32 hold the two 4-row halves of every 8-row block of the same output row n.
        // v_permlane32_swap exchanges them so that each lane owns 8 consecutive m (16 bytes):
        // lane half lh covers m = 32 i + 16 a + 8 lh .. + 7.  All W loads of a 32-row stripe are issued
        // before any of them is used, and the next stripe is loaded while the current one is updated.
        typedef uint32_t u32x2v __attribute__((ext_vector_type(2)));
        const float s = g.s_dev != nullptr ? *g.s_dev : g.s;
        auto row_ptr = [&](int j) -> uint16_t* {
            const int nl = wn * (BN / 2) + 32 * j + l32;
            return (nl < n_rem) ? g.Out + (n0 + nl) * g.ldo + m0 : nullptr;
        };
        auto mloc = [&](int i, int a) { return wm * (BM / 2) + 32 * i + 16 * a + 8 * lh; };
        half8 wbuf[2][TM][2];
        const uint16_t* old_base = (EPI == EPI_UPDATE && g.Res != nullptr) ? g.Res : g.Out;
        auto load_stripe = [&](int j, half8 (&w)[TM][2]) {
            const int nl_ = wn * (BN / 2) + 32 * j + l32;
            const uint16_t* row = (nl_ < n_rem) ? old_base + (n0 + nl_) * g.ldo + m0 : nullptr;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int a = 0; a < 2; ++a) {
                    const int ml = mloc(i, a);
                    if (row != nullptr && ml < m_rem) w[i][a] = *reinterpret_cast<const half8*>(row + ml);
                }
        };
        constexpr bool RMW = (EPI == EPI_UPDATE || EPI == EPI_CLIPV);
        bool bad = false;
        if constexpr (RMW) load_stripe(0, wbuf[0]);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            if constexpr (RMW) {
                if (j + 1 < TN) load_stripe(j + 1, wbuf[(j + 1) & 1]);
            }
            uint16_t* row = row_ptr(j);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int a = 0; a < 2; ++a) {
                    float v[8];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const u32x2v sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[i][j][8 * a + e]),
                                                                           __float_as_uint(acc[i][j][8 * a + 4 + e]),
                                                                           false, false);
                        v[e] = __uint_as_float(sw[0]);
                        v[4 + e] = __uint_as_float(sw[1]);
                    }
                    const int ml = mloc(i, a);
                    if (row == nullptr || ml >= m_rem) continue;
                    half8 out;
                    if constexpr (EPI == EPI_UPDATE) {
                        const half8 w = wbuf[j & 1][i][a];
#pragma unroll
                        for (int e = 0; e < 8; ++e) out[e] = (_Float16)fmaf(-s, v[e], (float)w[e]);
                    } else if constexpr (EPI == EPI_CLIPV) {
                        // clip by value (section 3.3.1): clamp each unscaled gradient element, then update;
                        // a non-finite element raises the flag and leaves its weight alone
                        const half8 w = wbuf[j & 1][i][a];
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const float gq = v[e] * g.inv_s;
                            const bool fin = (__float_as_uint(gq) & 0x7f800000u) != 0x7f800000u;
                            const float gc = fminf(fmaxf(gq, -g.clipv), g.clipv);
                            out[e] = fin ? (_Float16)fmaf(-g.lr, gc, (float)w[e]) : w[e];
                            bad |= !fin;
                        }
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; ++e) out[e] = (_Float16)v[e];
                    }
                    *reinterpret_cast<half8*>(row + ml) = out;
                }
        }
        if constexpr (EPI == EPI_CLIPV) {
            if (__any(bad) && lane == 0 && g.flag_out != nullptr) atomicOr(g.flag_out, 1);
        }
    }
}

}  // namespace lomo

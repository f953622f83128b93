// MFMA contraction kernels of the LOMO hot path for gfx950 (CDNA4, wave64).
//
// One kernel template serves the three dense steps of a linear tensor:
//   * fused wgrad + SGD update (paper section 3.2, Algorithm 1: theta <- theta - lr * g, the
//     gradient never leaves the accumulators; section 3.3.2: update arithmetic in fp32),
//   * wgrad squared norm + overflow detection (section 3.3.1 / 3.3.2, first backward pass),
//   * dgrad dX = dY W for the continuing back-propagation.
//
// Layout.  The output tile is Out[n][m] with m contiguous in memory.  Operand "A" supplies the m
// index and is always stored with the contraction index as its slow dimension (X[t][k] for wgrad,
// W[n][k] for dgrad), so it has to be transposed on its way to the matrix cores: a lane fetches
// dwords (two neighbouring m) from eight consecutive contraction rows, repacks them with byte
// permutes into two 16-byte runs along the contraction, and stores those to LDS in [m][c] order.
// Operand "B" supplies n and is transposed the same way (dY[t][n] for wgrad) or copied straight
// (dY[t][n] for dgrad, where n_out is the contraction).  MFMA 32x32x16 f16 then reads 16-byte
// fragments from LDS rows of 80 bytes (64 + 16 pad), which makes ds_read_b128 conflict free.
// With A on the MFMA row side, each lane's four consecutive accumulator registers are four
// consecutive m, i.e. an 8-byte run of W / dX: the read-modify-write epilogue is vectorised.
#include "lomo_gemm_common.h"

#include <stdlib.h>

namespace lomo {

constexpr int BK = 32;         // contraction slice per pipeline stage
constexpr int LROW = BK + 8;   // halves per LDS row

// ---- global -> registers ------------------------------------------------------------------

// Contraction-strided operand: tile of BK rows x BX columns starting at `base` (row stride ld).
// Item = (column pair p, row octet q): eight dword loads down the rows.
template <int BX, bool GUARD>
__device__ __forceinline__ void load_strided(const uint16_t* __restrict__ base, int64_t ld, int c_rem, int x_rem,
                                             uint32_t (&r)[BX / 128][8], int tid) {
#pragma unroll
    for (int it = 0; it < BX / 128; ++it) {
        const int item = tid + it * NT;
        const int p = item % (BX / 2);
        const int q = item / (BX / 2);
        const uint16_t* src = base + (int64_t)(8 * q) * ld + 2 * p;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (!GUARD || (8 * q + i < c_rem && 2 * p < x_rem))
                r[it][i] = *reinterpret_cast<const uint32_t*>(src + (int64_t)i * ld);
            else
                r[it][i] = 0u;
        }
    }
}

template <int BX>
__device__ __forceinline__ void store_strided(uint16_t* __restrict__ lds, const uint32_t (&r)[BX / 128][8], int tid) {
#pragma unroll
    for (int it = 0; it < BX / 128; ++it) {
        const int item = tid + it * NT;
        const int p = item % (BX / 2);
        const int q = item / (BX / 2);
        u32x4 lo, hi;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            lo[j] = __builtin_amdgcn_perm(r[it][2 * j + 1], r[it][2 * j], 0x05040100u);
            hi[j] = __builtin_amdgcn_perm(r[it][2 * j + 1], r[it][2 * j], 0x07060302u);
        }
        *reinterpret_cast<u32x4*>(lds + (2 * p) * LROW + 8 * q) = lo;
        *reinterpret_cast<u32x4*>(lds + (2 * p + 1) * LROW + 8 * q) = hi;
    }
}

// Contraction-contiguous operand: tile of BX rows x BK halves, 16-byte chunks.
template <int BX, bool GUARD>
__device__ __forceinline__ void load_contig(const uint16_t* __restrict__ base, int64_t ld, int c_rem, int x_rem,
                                            u32x4 (&r)[BX / 64], int tid) {
#pragma unroll
    for (int it = 0; it < BX / 64; ++it) {
        const int item = tid + it * NT;
        const int n = item / (BK / 8);
        const int q = item % (BK / 8);
        if (!GUARD || (n < x_rem && 8 * q < c_rem))
            r[it] = *reinterpret_cast<const u32x4*>(base + (int64_t)n * ld + 8 * q);
        else
            r[it] = u32x4{0u, 0u, 0u, 0u};
    }
}

template <int BX>
__device__ __forceinline__ void store_contig(uint16_t* __restrict__ lds, const u32x4 (&r)[BX / 64], int tid) {
#pragma unroll
    for (int it = 0; it < BX / 64; ++it) {
        const int item = tid + it * NT;
        const int n = item / (BK / 8);
        const int q = item % (BK / 8);
        *reinterpret_cast<u32x4*>(lds + n * LROW + 8 * q) = r[it];
    }
}

// ---- the kernel ---------------------------------------------------------------------------

// A_STRIDED = false serves the forward product Y = X W^T (both operands contraction-contiguous: A = W[n][k]
// supplies the m index, B = X[t][k] the n index), used to recompute activations from a checkpoint.
template <int BM, int BN, bool B_STRIDED, int EPI, bool A_STRIDED = true>
__global__ __launch_bounds__(NT) void lomo_contract_kernel(GemmArgs g) {
    constexpr int TM = BM / 64, TN = BN / 64;          // 32x32 MFMA tiles per wave
    constexpr int STAGE = (BM + BN) * LROW;            // halves per LDS stage
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];

    if (EPI == EPI_UPDATE && g.flag_in != nullptr && *g.flag_in != 0) {
        return;   // overflow seen in pass 1: the step is dropped, W stays as it is
    }

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const int l32 = lane & 31, lh = lane >> 5;

    const int tiles_m = (int)((g.M + BM - 1) / BM);
    const int64_t m0 = (int64_t)(blockIdx.x % tiles_m) * BM;
    const int64_t n0 = (int64_t)(blockIdx.x / tiles_m) * BN;
    const int m_rem = (int)((g.M - m0 < BM) ? (g.M - m0) : BM);
    const int n_rem = (int)((g.Nn - n0 < BN) ? (g.Nn - n0) : BN);
    const bool full_mn = (m_rem == BM) && (n_rem == BN);

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const uint16_t* pa = A_STRIDED ? (g.A + m0) : (g.A + m0 * g.lda);        // (c = 0, m0)
    const uint16_t* pb = B_STRIDED ? (g.B + n0) : (g.B + n0 * g.ldb);        // (c = 0, n0)
    const int64_t a_step = A_STRIDED ? (int64_t)BK * g.lda : (int64_t)BK;
    const int64_t b_step = B_STRIDED ? (int64_t)BK * g.ldb : (int64_t)BK;

    uint32_t ra[A_STRIDED ? BM / 128 : 1][8];
    u32x4 rac[A_STRIDED ? 1 : BM / 64];
    uint32_t rbs[B_STRIDED ? BN / 128 : 1][8];
    u32x4 rbc[B_STRIDED ? 1 : BN / 64];

    const int KT = (int)((g.C + BK - 1) / BK);

    auto fetch = [&](int kt) {
        const int c_rem = (int)(g.C - (int64_t)kt * BK);
        const bool guard = !full_mn || c_rem < BK;
        const uint16_t* a = pa + (int64_t)kt * a_step;
        const uint16_t* b = pb + (int64_t)kt * b_step;
        if (!guard) {
            if constexpr (A_STRIDED) load_strided<BM, false>(a, g.lda, c_rem, m_rem, ra, tid);
            else load_contig<BM, false>(a, g.lda, c_rem, m_rem, rac, tid);
            if constexpr (B_STRIDED) load_strided<BN, false>(b, g.ldb, c_rem, n_rem, rbs, tid);
            else load_contig<BN, false>(b, g.ldb, c_rem, n_rem, rbc, tid);
        } else {
            if constexpr (A_STRIDED) load_strided<BM, true>(a, g.lda, c_rem, m_rem, ra, tid);
            else load_contig<BM, true>(a, g.lda, c_rem, m_rem, rac, tid);
            if constexpr (B_STRIDED) load_strided<BN, true>(b, g.ldb, c_rem, n_rem, rbs, tid);
            else load_contig<BN, true>(b, g.ldb, c_rem, n_rem, rbc, tid);
        }
    };
    auto stash = [&](int buf) {
        uint16_t* as = smem + buf * STAGE;
        uint16_t* bs = as + BM * LROW;
        if constexpr (A_STRIDED) store_strided<BM>(as, ra, tid);
        else store_contig<BM>(as, rac, tid);
        if constexpr (B_STRIDED) store_strided<BN>(bs, rbs, tid);
        else store_contig<BN>(bs, rbc, tid);
    };

    if (KT > 0) {
        fetch(0);
        stash(0);
    }
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const bool more = kt + 1 < KT;
        if (more) fetch(kt + 1);

        const uint16_t* as = smem + (kt & 1) * STAGE + (wm * (BM / 2) + l32) * LROW + 8 * lh;
        const uint16_t* bs = smem + (kt & 1) * STAGE + BM * LROW + (wn * (BN / 2) + l32) * LROW + 8 * lh;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            half8 a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const half8*>(as + i * 32 * LROW + kk * 16);
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = *reinterpret_cast<const half8*>(bs + j * 32 * LROW + kk * 16);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
        }

        if (more) stash((kt + 1) & 1);
        __syncthreads();
    }

    epilogue<BM, BN, EPI>(acc, g, smem, m0, n0, m_rem, n_rem);
}

// ---- host side ----------------------------------------------------------------------------

template <int BM, int BN, bool B_STRIDED, int EPI, bool A_STRIDED = true>
static hipError_t launch_one(const GemmArgs& a, hipStream_t st) {
    if (a.M <= 0 || a.Nn <= 0) return hipSuccess;
    constexpr size_t lds = 2u * (BM + BN) * LROW * sizeof(uint16_t);
    auto kern = lomo_contract_kernel<BM, BN, B_STRIDED, EPI, A_STRIDED>;
    // thread-safe one-time set-up (initialisation of a function-local static)
    static const hipError_t cfg0 = allow_dynamic_lds(kern, (int)lds);
    if (cfg0 != hipSuccess) return cfg0;
    const int64_t tiles = ((a.M + BM - 1) / BM) * ((a.Nn + BN - 1) / BN);
    if (tiles > 0x7fffffff) return hipErrorInvalidValue;
    return launch_timed(a.family, kern, dim3((unsigned)tiles), dim3(NT), lds, st, a);
}

// Tile choice: 256 x 256 when that still gives every CU at least one tile, else 128 x 128.
static inline bool use_big_tiles(int64_t M, int64_t Nn) {
    const int64_t big = ((M + 255) / 256) * ((Nn + 255) / 256);
    return big >= 192;
}

// LOMO_DISABLE_FAST=1 forces the generic kernel everywhere, LOMO_DISABLE_DMA=1 skips the
// direct-to-LDS kernel (testing aids).
static bool fast_enabled() {
    static const bool on = [] {
        const char* e = getenv("LOMO_DISABLE_FAST");
        return !(e && e[0] == '1');
    }();
    return on;
}

static bool dma_enabled() {
    static const bool on = [] {
        const char* e = getenv("LOMO_DISABLE_DMA");
        return !(e && e[0] == '1');
    }();
    return on;
}

hipError_t launch_wgrad_update(const GemmArgs& a, hipStream_t st) {
    hipError_t e;
    if (fast_enabled() && dma_enabled() && try_launch_dma<true, EPI_UPDATE>(a, st, &e)) return e;
    if (fast_enabled() && try_launch_fast<true, EPI_UPDATE>(a, st, &e)) return e;
    return use_big_tiles(a.M, a.Nn) ? launch_one<256, 256, true, EPI_UPDATE>(a, st)
                                    : launch_one<128, 128, true, EPI_UPDATE>(a, st);
}
hipError_t launch_wgrad_update_clipv(const GemmArgs& a, hipStream_t st) {
    hipError_t e;
    if (fast_enabled() && dma_enabled() && try_launch_dma<true, EPI_CLIPV>(a, st, &e)) return e;
    if (fast_enabled() && try_launch_fast<true, EPI_CLIPV>(a, st, &e)) return e;
    return use_big_tiles(a.M, a.Nn) ? launch_one<256, 256, true, EPI_CLIPV>(a, st)
                                    : launch_one<128, 128, true, EPI_CLIPV>(a, st);
}
hipError_t launch_wgrad_sqnorm(const GemmArgs& a, int norm_route, hipStream_t st) {
    hipError_t e;
    if (norm_route != LOMO_NORM_DIRECT && fast_enabled() && dma_enabled()) {
        std::vector<GemmArgs> one(1, a), gram, direct;
        choose_norm_route(norm_route, one, gram, direct);
        if (!gram.empty()) return launch_gram_group(gram.data(), 1, st);
    }
    if (fast_enabled() && dma_enabled() && try_launch_dma<true, EPI_SQNORM>(a, st, &e)) return e;
    if (fast_enabled() && try_launch_fast<true, EPI_SQNORM>(a, st, &e)) return e;
    return use_big_tiles(a.M, a.Nn) ? launch_one<256, 256, true, EPI_SQNORM>(a, st)
                                    : launch_one<128, 128, true, EPI_SQNORM>(a, st);
}
hipError_t launch_dgrad(const GemmArgs& a, hipStream_t st) {
    hipError_t e;
    if (fast_enabled() && dma_enabled() && try_launch_dma<false, EPI_STORE>(a, st, &e)) return e;
    if (fast_enabled() && try_launch_fast<false, EPI_STORE>(a, st, &e)) return e;
    return use_big_tiles(a.M, a.Nn) ? launch_one<256, 256, false, EPI_STORE>(a, st)
                                    : launch_one<128, 128, false, EPI_STORE>(a, st);
}

// Y = X W^T (EPI_STORE) or Y <- Y + X W^T rounded once (EPI_UPDATE with s = -1: the residual connection).
hipError_t launch_forward(const GemmArgs& a, bool accumulate, hipStream_t st) {
    hipError_t e;
    if (accumulate) {
        if (fast_enabled() && dma_enabled() && try_launch_dma_nt<EPI_UPDATE>(a, st, &e)) return e;
        return use_big_tiles(a.M, a.Nn) ? launch_one<256, 256, false, EPI_UPDATE, false>(a, st)
                                        : launch_one<128, 128, false, EPI_UPDATE, false>(a, st);
    }
    if (fast_enabled() && dma_enabled() && try_launch_dma_nt<EPI_STORE>(a, st, &e)) return e;
    return use_big_tiles(a.M, a.Nn) ? launch_one<256, 256, false, EPI_STORE, false>(a, st)
                                    : launch_one<128, 128, false, EPI_STORE, false>(a, st);
}

}  // namespace lomo

// 256 x 256 MFMA contraction with a four-stage direct-to-LDS pipeline (gfx950).
//
// Same mathematics and epilogues as the other contraction kernels (fused wgrad + SGD update of
// paper section 3.2 / Algorithm 1, squared-norm pass of section 3.3.1, dgrad).  Data movement:
//   * global -> LDS without passing through registers: global_load_lds_dwordx4 writes lane L's
//     16 bytes to M0 + 16 L, and each lane may fetch any global address, so a wave instruction
//     fills 1 KiB of LDS with the 16-byte chunks of two tile rows in swizzled order;
//   * four 32 KiB stages: the loads for slice kt+3 are issued while slice kt is multiplied, which
//     covers HBM latency with two and a half slices of MFMA work and needs no staging registers;
//   * LDS -> MFMA operands with the transposing read ds_read_b64_tr_b16 (contraction-strided
//     operands) or ds_read_b128 (contraction-contiguous operand of dgrad); the fragments of the
//     next half-slice are read while the current one is multiplied, across the barrier;
//   * one barrier per slice.  The vector-memory counter is managed by hand because the compiler
//     would otherwise drain it before every LDS read.
#include "lomo_gemm_common.h"

namespace lomo {

typedef short short4v __attribute__((ext_vector_type(4)));

namespace dma {

constexpr int BM = 256, BN = 256, BK = 32, NS = 4;
constexpr int A_HALVES = BK * BM, B_HALVES = BK * BN, STAGE_HALVES = A_HALVES + B_HALVES;
constexpr int LOADS_PER_STAGE = 8;   // per wave: 4 for the A tile, 4 for the B tile

__device__ __forceinline__ int swz_s(int r) { return ((r & 1) * 10) + ((r & 2) * 2); }
__device__ __forceinline__ int swz_c(int n) { return ((n >> 1) & 3) ^ ((n >> 3) & 1); }

// 16 bytes per lane from base + voff to LDS address m0 + 16 * lane.
__device__ __forceinline__ void dma16(uint32_t voff, const void* base, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(base), "s"(lds_addr) : "memory", "m0");
}

__device__ __forceinline__ half8 read_tr8(const uint16_t* p0, const uint16_t* p1) {
    typedef __attribute__((address_space(3))) short4v* lds_p;
    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p0));
    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p1));
    return __builtin_bit_cast(half8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

}  // namespace dma

template <bool B_STRIDED, int EPI>
__global__ __launch_bounds__(NT) void lomo_contract_dma_kernel(GemmArgs g, int tiles_m, int tiles_n) {
    using namespace dma;
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];

    if (EPI == EPI_UPDATE && g.flag_in != nullptr && *g.flag_in != 0) return;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;

    int tm, tn;
    {   // XCD-aware tile assignment: each XCD owns a contiguous range of tiles, walked in 8-wide bands
        const int total = tiles_m * tiles_n;
        const int bid = blockIdx.x;
        const int x = bid & 7, local = bid >> 3;
        const int q = total >> 3, r = total & 7;
        const int t = x * q + (x < r ? x : r) + local;
        constexpr int GM = 8;
        const int per_band = GM * tiles_n;
        const int band = t / per_band;
        const int first_m = band * GM;
        const int gsz = (tiles_m - first_m < GM) ? (tiles_m - first_m) : GM;
        const int in_band = t - band * per_band;
        tm = first_m + in_band % gsz;
        tn = in_band / gsz;
    }
    const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

    floatx16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // ---- DMA: per-lane source byte offsets inside a slice, and this wave's LDS targets
    uint32_t a_voff[4], b_voff[4];
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int q = wave * 4 + it;
        {
            const int r = 2 * q + (lane >> 5), cp = lane & 31;
            a_voff[it] = (uint32_t)(r * (int)g.lda + ((cp ^ swz_s(r)) * 8)) * 2u;
        }
        if constexpr (B_STRIDED) {
            const int r = 2 * q + (lane >> 5), cp = lane & 31;
            b_voff[it] = (uint32_t)(r * (int)g.ldb + ((cp ^ swz_s(r)) * 8)) * 2u;
        } else {
            const int n = 16 * q + (lane >> 2), cp = lane & 3;
            b_voff[it] = (uint32_t)(n * (int)g.ldb + ((cp ^ swz_c(n)) * 8)) * 2u;
        }
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
    const uint32_t lds_wave = lds0 + (uint32_t)wave * 4096u;   // this wave's first KiB slot in a tile

    const uint16_t* pa = g.A + m0;
    const uint16_t* pb = B_STRIDED ? (g.B + n0) : (g.B + n0 * g.ldb);
    const int64_t a_step = (int64_t)BK * g.lda;
    const int64_t b_step = B_STRIDED ? (int64_t)BK * g.ldb : (int64_t)BK;
    const int KT = (int)(g.C / BK);

    auto issue = [&](int stage, int buf) {
        const int s = stage < KT ? stage : KT - 1;   // past the end: harmless re-read, keeps the counter regular
        const uint16_t* a = pa + (int64_t)s * a_step;
        const uint16_t* b = pb + (int64_t)s * b_step;
        const uint32_t la = lds_wave + (uint32_t)buf * (STAGE_HALVES * 2u);
        const uint32_t lb = la + A_HALVES * 2u;
#pragma unroll
        for (int it = 0; it < 4; ++it) dma16(a_voff[it], a, la + it * 1024u);
#pragma unroll
        for (int it = 0; it < 4; ++it) dma16(b_voff[it], b, lb + it * 1024u);
    };

    // ---- fragment read offsets (halves), as in the register-staged fast path
    const int g4 = lane >> 4, j16 = lane & 15;
    const int mhalf = g4 & 1, kh = g4 >> 1, rib = j16 >> 2, piece = j16 & 3;
    const int a_rd = (8 * kh + rib) * BM + (((wm * (BM / 16) + 2 * mhalf + (piece >> 1)) ^ swz_s(rib)) * 8) + (piece & 1) * 4;
    int b_rd;
    if constexpr (B_STRIDED) {
        b_rd = (8 * kh + rib) * BN + (((wn * (BN / 16) + 2 * mhalf + (piece >> 1)) ^ swz_s(rib)) * 8) + (piece & 1) * 4;
    } else {
        const int nl = wn * (BN / 2) + (lane & 31), lh = lane >> 5;
        b_rd = nl * BK + ((lh ^ swz_c(nl)) * 8);
    }

    // Reads are issued in the order the MFMAs consume them: a0, b0..b3, a1..a3.
    auto load_frags = [&](half8 (&a)[4], half8 (&b)[4], int buf, int kk) {
        const uint16_t* as = smem + buf * STAGE_HALVES;
        const uint16_t* bs = as + A_HALVES;
        auto read_a = [&](int i) {
            const uint16_t* p = as + ((a_rd ^ (i << 5)) + kk * 16 * BM);
            a[i] = read_tr8(p, p + 4 * BM);
        };
        read_a(0);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (B_STRIDED) {
                const uint16_t* p = bs + ((b_rd ^ (j << 5)) + kk * 16 * BN);
                b[j] = read_tr8(p, p + 4 * BN);
            } else {
                b[j] = *reinterpret_cast<const half8*>(bs + ((b_rd ^ (kk << 4)) + j * 32 * BK));
            }
        }
        read_a(1);
        read_a(2);
        read_a(3);
    };
    auto mfma_all = [&](const half8 (&a)[4], const half8 (&b)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
    };

    // ---- prologue: three slices in flight, slice 0 landed and visible, its first fragments read
    issue(0, 0);
    issue(1, 1);
    issue(2, 2);
    asm volatile("s_waitcnt vmcnt(16)\n\ts_barrier" ::: "memory");
    half8 fa0[4], fb0[4], fa1[4], fb1[4];
    load_frags(fa0, fb0, 0, 0);

    // One LDS read is slotted in front of each MFMA, so the fragments of the next half-slice
    // arrive while the current one is multiplied.
    auto interleave = [] {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one DS read
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
        }
    };
    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 3;
        load_frags(fa1, fb1, cur, 1);
        mfma_all(fa0, fb0);
        interleave();
        __builtin_amdgcn_sched_barrier(0);
        issue(kt + 3, (kt + 3) & 3);
        // own loads of slice kt+1 landed (two younger slices may still fly); own LDS reads done
        asm volatile("s_waitcnt vmcnt(16) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        load_frags(fa0, fb0, (kt + 1) & 3, 0);
        mfma_all(fa1, fb1);
        interleave();
        __builtin_amdgcn_sched_barrier(0);
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");

    epilogue<BM, BN, EPI>(acc, g, smem, m0, n0, BM, BN);
}

template <bool B_STRIDED, int EPI>
static hipError_t launch_dma_one(const GemmArgs& a, hipStream_t st) {
    constexpr size_t lds = (size_t)dma::NS * dma::STAGE_HALVES * sizeof(uint16_t);
    auto kern = lomo_contract_dma_kernel<B_STRIDED, EPI>;
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        configured = true;
    }
    const int tiles_m = (int)(a.M / dma::BM), tiles_n = (int)(a.Nn / dma::BN);
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(NT), lds, st, a, tiles_m, tiles_n);
    return hipGetLastError();
}

// Eligible: whole 256 x 256 x 32 tiles, enough of them to fill the chip, 32-bit slice offsets.
template <bool B_STRIDED, int EPI>
bool try_launch_dma(const GemmArgs& a, hipStream_t st, hipError_t* err) {
    using namespace dma;
    const bool ok = a.M > 0 && a.Nn > 0 && a.C >= BK && a.M % BM == 0 && a.Nn % BN == 0 && a.C % BK == 0 &&
                    (int64_t)BK * a.lda < (1 << 30) && (int64_t)BN * a.ldb < (1 << 30) &&
                    (a.M / BM) * (a.Nn / BN) >= 192 && (a.M / BM) * (a.Nn / BN) < (1 << 24);
    if (!ok) return false;
    *err = launch_dma_one<B_STRIDED, EPI>(a, st);
    return true;
}

template bool try_launch_dma<true, EPI_UPDATE>(const GemmArgs&, hipStream_t, hipError_t*);
template bool try_launch_dma<true, EPI_SQNORM>(const GemmArgs&, hipStream_t, hipError_t*);
template bool try_launch_dma<false, EPI_STORE>(const GemmArgs&, hipStream_t, hipError_t*);

}  // namespace lomo

// Fast path of the MFMA contraction for shapes made of whole tiles (every LLaMA-shaped tensor).
//
// Same mathematics and epilogues as the generic kernel (fused wgrad + SGD update of paper section
// 3.2 / Algorithm 1, squared-norm pass of section 3.3.1, dgrad); what differs is how operands
// reach the matrix cores:
//   * global -> registers with 16-byte loads along the contiguous dimension, two k-slices ahead
//     (two register sets), so HBM/L2 latency hides behind two slices of MFMA work;
//   * registers -> LDS unchanged in layout ([contraction][feature], as in memory) but with the
//     16-byte chunks of each row XOR-swizzled;
//   * LDS -> MFMA operands with the gfx950 transposing read ds_read_b64_tr_b16: a 16-lane group
//     reads a 4 (contraction) x 16 (feature) block and each lane receives the 4 contraction values
//     of its own feature.  Two such reads give the 8 halves a 32x32x16 MFMA lane needs.  No VALU
//     work is spent on the transpose.  The swizzle makes the four rows a group touches fall into
//     different banks.
//   * workgroup -> tile mapping is XCD aware: each of the 8 XCDs (own L2) works on a contiguous
//     range of tiles, walked in 8 x 4 bands so that co-resident tiles share operand panels.
#include "lomo_gemm_common.h"

namespace lomo {

typedef short short4v __attribute__((ext_vector_type(4)));

constexpr int FBK = 32;   // contraction slice per stage

// chunk swizzles (in units of 16-byte chunks)
__device__ __forceinline__ int swz_s(int r) { return ((r & 1) * 10) + ((r & 2) * 2); }       // strided tiles
__device__ __forceinline__ int swz_c(int n) { return ((n >> 1) & 3) ^ ((n >> 3) & 1); }      // contiguous tiles

__device__ __forceinline__ half8 lds_read_tr8(const uint16_t* p0, const uint16_t* p1) {
    typedef __attribute__((address_space(3))) short4v* lds_p;
    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p0));
    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p1));
    typedef short short8v __attribute__((ext_vector_type(8)));
    const short8v v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(half8, v);
}

template <int BM, int BN, bool B_STRIDED, int EPI>
__global__ __launch_bounds__(NT) void lomo_contract_fast_kernel(GemmArgs g, int tiles_m, int tiles_n) {
    constexpr int TM = BM / 64, TN = BN / 64;
    constexpr int A_HALVES = FBK * BM;                       // strided A tile
    constexpr int B_HALVES = FBK * BN;                       // same size either way
    constexpr int STAGE = A_HALVES + B_HALVES;
    constexpr int NA = BM / 64, NB = BN / 64;                // 16-byte chunks per thread per tile
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];

    if (EPI == EPI_UPDATE && g.flag_in != nullptr && *g.flag_in != 0) return;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;

    // ---- XCD-aware tile assignment
    int tm, tn;
    {
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

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // ---- per-thread global offsets and LDS store offsets (halves)
    uint32_t a_goff[NA], b_goff[NB];   // byte offsets from the slice base
    int a_loff[NA], b_loff[NB];
#pragma unroll
    for (int it = 0; it < NA; ++it) {
        const int id = tid + it * NT, r = id / (BM / 8), j = id % (BM / 8);
        a_goff[it] = (uint32_t)(r * (int)g.lda + j * 8) * 2u;
        a_loff[it] = r * BM + ((j ^ swz_s(r)) * 8);
    }
#pragma unroll
    for (int it = 0; it < NB; ++it) {
        const int id = tid + it * NT;
        if constexpr (B_STRIDED) {
            const int r = id / (BN / 8), j = id % (BN / 8);
            b_goff[it] = (uint32_t)(r * (int)g.ldb + j * 8) * 2u;
            b_loff[it] = r * BN + ((j ^ swz_s(r)) * 8);
        } else {
            const int n = id / 4, j = id % 4;
            b_goff[it] = (uint32_t)(n * (int)g.ldb + j * 8) * 2u;
            b_loff[it] = n * FBK + ((j ^ swz_c(n)) * 8);
        }
    }
    const uint16_t* pa = g.A + m0;
    const uint16_t* pb = B_STRIDED ? (g.B + n0) : (g.B + n0 * g.ldb);
    const int64_t a_step = (int64_t)FBK * g.lda;
    const int64_t b_step = B_STRIDED ? (int64_t)FBK * g.ldb : (int64_t)FBK;

    // ---- per-lane LDS read offsets (halves)
    const int g4 = lane >> 4, j16 = lane & 15;
    const int mhalf = g4 & 1, kh = g4 >> 1, rib = j16 >> 2, piece = j16 & 3;
    const int a_rd = (8 * kh + rib) * BM + (((wm * (BM / 16) + 2 * mhalf + (piece >> 1)) ^ swz_s(rib)) * 8) + (piece & 1) * 4;
    int b_rd;
    if constexpr (B_STRIDED) {
        b_rd = (8 * kh + rib) * BN + (((wn * (BN / 16) + 2 * mhalf + (piece >> 1)) ^ swz_s(rib)) * 8) + (piece & 1) * 4;
    } else {
        const int nl = wn * (BN / 2) + (lane & 31), lh = lane >> 5;
        b_rd = nl * FBK + ((lh ^ swz_c(nl)) * 8);
    }

    const int KT = (int)(g.C / FBK);

    u32x4 ra0[NA], rb0[NB], ra1[NA], rb1[NB];
    auto fetch = [&](u32x4 (&ra)[NA], u32x4 (&rb)[NB], int kt) {
        const char* a = reinterpret_cast<const char*>(pa + (int64_t)kt * a_step);
        const char* b = reinterpret_cast<const char*>(pb + (int64_t)kt * b_step);
#pragma unroll
        for (int it = 0; it < NA; ++it) ra[it] = *reinterpret_cast<const u32x4*>(a + a_goff[it]);
#pragma unroll
        for (int it = 0; it < NB; ++it) rb[it] = *reinterpret_cast<const u32x4*>(b + b_goff[it]);
    };
    auto stash = [&](const u32x4 (&ra)[NA], const u32x4 (&rb)[NB], int buf) {
        uint16_t* as = smem + buf * STAGE;
        uint16_t* bs = as + A_HALVES;
#pragma unroll
        for (int it = 0; it < NA; ++it) *reinterpret_cast<u32x4*>(as + a_loff[it]) = ra[it];
#pragma unroll
        for (int it = 0; it < NB; ++it) *reinterpret_cast<u32x4*>(bs + b_loff[it]) = rb[it];
    };
    auto compute = [&](int buf) {
        const uint16_t* as = smem + buf * STAGE;
        const uint16_t* bs = as + A_HALVES;
#pragma unroll
        for (int kk = 0; kk < FBK / 16; ++kk) {
            half8 a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const uint16_t* p = as + ((a_rd ^ (i << 5)) + kk * 16 * BM);
                a[i] = lds_read_tr8(p, p + 4 * BM);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if constexpr (B_STRIDED) {
                    const uint16_t* p = bs + ((b_rd ^ (j << 5)) + kk * 16 * BN);
                    b[j] = lds_read_tr8(p, p + 4 * BN);
                } else {
                    b[j] = *reinterpret_cast<const half8*>(bs + ((b_rd ^ (kk << 4)) + j * 32 * FBK));
                }
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    };

    // KT is even and >= 4 (checked on the host).  Invariant at the top of the loop: LDS buffer 0
    // holds slice kt, register set 1 holds slice kt+1, register set 0 is in flight with kt+2.
    fetch(ra0, rb0, 0);
    fetch(ra1, rb1, 1);
    stash(ra0, rb0, 0);
    __syncthreads();
    fetch(ra0, rb0, 2);
    for (int kt = 0; kt + 2 < KT; kt += 2) {
        compute(0);
        stash(ra1, rb1, 1);
        __syncthreads();
        fetch(ra1, rb1, kt + 3);
        compute(1);
        stash(ra0, rb0, 0);
        __syncthreads();
        fetch(ra0, rb0, (kt + 4 < KT) ? kt + 4 : KT - 1);   // clamped: the last one is a harmless re-read
    }
    compute(0);
    stash(ra1, rb1, 1);
    __syncthreads();
    compute(1);
    __syncthreads();

    epilogue<BM, BN, EPI>(acc, g, smem, m0, n0, BM, BN);
}

template <int BM, int BN, bool B_STRIDED, int EPI>
static hipError_t launch_fast_one(const GemmArgs& a, hipStream_t st) {
    constexpr size_t lds = 2u * FBK * (BM + BN) * sizeof(uint16_t);
    auto kern = lomo_contract_fast_kernel<BM, BN, B_STRIDED, EPI>;
    // thread-safe one-time set-up (initialisation of a function-local static)
    static const hipError_t cfg0 = allow_dynamic_lds(kern, (int)lds);
    if (cfg0 != hipSuccess) return cfg0;
    const int tiles_m = (int)(a.M / BM), tiles_n = (int)(a.Nn / BN);
    return launch_timed(a.family, kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(NT), lds, st, a, tiles_m, tiles_n);
}

// Eligible: whole tiles in every dimension and offsets that fit 32-bit element indices.
template <int BM, int BN>
static inline bool fast_ok(const GemmArgs& a) {
    return a.M > 0 && a.Nn > 0 && a.C > 0 && a.M % BM == 0 && a.Nn % BN == 0 && a.C % (2 * FBK) == 0 && a.C >= 4 * FBK &&
           (int64_t)FBK * a.lda < (1 << 30) && (int64_t)BN * a.ldb < (1 << 30) &&
           (a.M / BM) * (a.Nn / BN) < (1 << 24);
}

template <bool B_STRIDED, int EPI>
bool try_launch_fast(const GemmArgs& a, hipStream_t st, hipError_t* err) {
    if (fast_ok<256, 256>(a) && (a.M / 256) * (a.Nn / 256) >= 192) {
        *err = launch_fast_one<256, 256, B_STRIDED, EPI>(a, st);
        return true;
    }
    if (fast_ok<128, 128>(a)) {
        *err = launch_fast_one<128, 128, B_STRIDED, EPI>(a, st);
        return true;
    }
    return false;
}

template bool try_launch_fast<true, EPI_UPDATE>(const GemmArgs&, hipStream_t, hipError_t*);
template bool try_launch_fast<true, EPI_CLIPV>(const GemmArgs&, hipStream_t, hipError_t*);
template bool try_launch_fast<true, EPI_SQNORM>(const GemmArgs&, hipStream_t, hipError_t*);
template bool try_launch_fast<false, EPI_STORE>(const GemmArgs&, hipStream_t, hipError_t*);

}  // namespace lomo

// Squared gradient norm of a linear tensor without forming the gradient: Gram route (gfx950).
//
// The norm pass of paper section 3.3.1 needs ||G||_F^2 for G = dY^T X (scaled gradient, [N x K]).
// With x_t, dy_t the rows of X [T x K] and dY [T x N]:
//
//     ||G||_F^2 = sum_{t,t'} (x_t . x_t') (dy_t . dy_t') = sum_{t,t'} P[t,t'] Q[t,t'],
//     P = X X^T,  Q = dY dY^T   (both T x T, symmetric),
//
// so only the lower triangle is needed: sum_t P_tt Q_tt + 2 sum_{t > t'} P Q.  That is
// T^2 (K + N) flop instead of 2 T N K, which is less whenever T < 2 N K / (N + K) -- the case
// for the wide tensors of large models at moderate token counts.  The overflow flag keeps its
// meaning: some element of G is non-finite exactly when some input is inf/NaN, and then the
// diagonal entry of P or Q in that row is non-finite.
//
// Accuracy: P and Q are accumulated in fp32 on the MFMA units; the error of the result is of the
// order 1e-6 * sum_{t,t'} |P Q|, i.e. relative to the per-token gradient energy rather than to
// ||G||^2 itself.  When the per-token gradients nearly cancel in the sum over tokens this is less
// accurate than the direct kernel, which is why the direct route is the default.
//
// Kernel: one persistent workgroup per CU walks a list of 256 x 128 tiles of the triangle of up to
// MAX_GROUP tensors.  A tile runs K/32 slices of X rows into the P accumulators and N/32 slices of
// dY rows into the Q accumulators as one continuous four-stage direct-to-LDS pipeline (both
// operands are contraction-contiguous, so LDS reads are plain 16-byte reads), then multiplies the
// two accumulator sets element by element, applies the triangle weights and adds one double.
#include "lomo_gemm_common.h"

#include <algorithm>

namespace lomo {
namespace gram {

constexpr int BM = 256, BN = 128, BK = 32, NS = 4;
constexpr int A_HALVES = BM * BK, B_HALVES = BN * BK, STAGE_HALVES = A_HALVES + B_HALVES;
constexpr int LDS_BYTES = NS * STAGE_HALVES * 2 + 256;
constexpr int MAX_GROUP = 40;
constexpr int BAND = 4;   // tile rows per band: the 32 tiles an XCD holds at once form a 4 x 8 block

struct GramTensor {
    const uint16_t* X;
    const uint16_t* dY;
    int32_t* flag_out;
    int K, N, tiles_m, tile_begin;
};

struct GroupArgs {
    double* acc;
    int n, total_tiles;
    GramTensor t[MAX_GROUP];
};

__device__ __forceinline__ int swz_c(int n) { return ((n >> 1) & 3) ^ ((n >> 3) & 1); }

__device__ __forceinline__ void dma16(uint32_t voff, const void* base, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(base), "s"(lds_addr) : "memory", "m0");
}

// Tile number t of the lower triangle (tile row bi covers tokens [256 bi, 256 bi + 256), tile column bj
// covers [128 bj, 128 bj + 128); valid when bj <= 2 bi + 1).  Bands of BAND tile rows, column-major
// inside a band.  The host guarantees t < tm (tm + 1).
__device__ __forceinline__ void locate(int t, int tm, int& bi, int& bj) {
    bi = 0;
    bj = 0;
    for (int r0 = 0; r0 < tm; r0 += BAND) {
        const int R = (tm - r0 < BAND) ? (tm - r0) : BAND;
        const int r1 = r0 + R - 1;
        const int cnt = R * (r0 + r1 + 2);          // sum over rows of (2 row + 2)
        if (t >= cnt) {
            t -= cnt;
            continue;
        }
        const int full = 2 * r0 + 2;                // columns that reach every row of the band
        if (t < R * full) {
            bj = t / R;
            bi = r0 + t % R;
            return;
        }
        t -= R * full;
        for (int c = full; c <= 2 * r1 + 1; ++c) {
            const int lo = c >> 1;                  // first row that reaches column c
            const int n = r1 - lo + 1;
            if (t < n) {
                bj = c;
                bi = lo + t;
                return;
            }
            t -= n;
        }
        return;
    }
}

}  // namespace gram

__global__ __launch_bounds__(NT) void lomo_gram_sqnorm_kernel(gram::GroupArgs ga) {
    using namespace gram;
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const int l32 = lane & 31, lh = lane >> 5;
    const int G = gridDim.x;

    int pos;
    {
        const int x = (int)(blockIdx.x & 7), local = (int)(blockIdx.x >> 3);
        const int q = G >> 3, r = G & 7;
        pos = x * q + (x < r ? x : r) + local;
    }

    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
    float* red_scratch = reinterpret_cast<float*>(smem + NS * STAGE_HALVES);

    // ---- fragment read offsets (halves)
    const int arow = wm * (BM / 2) + l32, brow = wn * (BN / 2) + l32;
    const int a_rd = arow * BK + ((lh ^ swz_c(arow)) * 8);
    const int b_rd = brow * BK + ((lh ^ swz_c(brow)) * 8);

    // ---- per-tile state of the loads: phase P reads X, phase Q reads dY.  A wave instruction fetches 16
    // rows of 64 bytes; lane L takes row L / 4 and, of its four 16-byte chunks, the one that the swizzle
    // assigns to LDS position L % 4.  The swizzle depends on the row modulo 16 only, so one lane offset per
    // phase serves every instruction and the row block goes into the scalar base address.
    uint32_t voffP = 0, voffQ = 0;
    const uint16_t *paP = nullptr, *pbP = nullptr, *paQ = nullptr, *pbQ = nullptr;
    int KTP = 0, KT = 0, ldP = 0, ldQ = 0;

    auto setup = [&](int w, int& tensor, int& bi, int& bj) {
        int k = 0;
        while (k + 1 < ga.n && w >= ga.t[k + 1].tile_begin) ++k;
        const GramTensor& T = ga.t[k];
        locate(w - T.tile_begin, T.tiles_m, bi, bj);
        tensor = k;
        const int n = lane >> 2, cp = lane & 3;
        const uint32_t c = (uint32_t)((cp ^ swz_c(n)) * 8);
        voffP = ((uint32_t)n * (uint32_t)T.K + c) * 2u;
        voffQ = ((uint32_t)n * (uint32_t)T.N + c) * 2u;
        ldP = T.K;
        ldQ = T.N;
        paP = T.X + (int64_t)bi * BM * T.K;
        pbP = T.X + (int64_t)bj * BN * T.K;
        paQ = T.dY + (int64_t)bi * BM * T.N;
        pbQ = T.dY + (int64_t)bj * BN * T.N;
        KTP = T.K / BK;
        KT = KTP + T.N / BK;
    };

    // One DMA instruction of slice `stage` of the tile: part 0 = the 256 tile rows (four KiB per wave),
    // part 1 = the 128 tile columns (two KiB per wave).  Slices past the end re-read the last one.
    auto issue1 = [&](int stage, int buf, int part, int it) {
        const int s = stage < KT ? stage : KT - 1;
        const bool q = s >= KTP;
        const int sl = q ? s - KTP : s;
        const int blk = part == 0 ? wave * 4 + it : wave * 2 + it;      // 16-row block inside the tile part
        const uint32_t l = lds0 + (uint32_t)buf * (STAGE_HALVES * 2u) + (part == 0 ? 0u : (uint32_t)(A_HALVES * 2)) +
                           (uint32_t)blk * 1024u;
        const uint16_t* base = part == 0 ? (q ? paQ : paP) : (q ? pbQ : pbP);
        base += (int64_t)(16 * blk) * (q ? ldQ : ldP) + (int64_t)sl * BK;
        dma16(q ? voffQ : voffP, base, l);
    };
    auto issue_prologue = [&] {
#pragma unroll
        for (int st = 0; st < 3; ++st) {
#pragma unroll
            for (int it = 0; it < 4; ++it) issue1(st, st, 0, it);
#pragma unroll
            for (int it = 0; it < 2; ++it) issue1(st, st, 1, it);
        }
#pragma unroll
        for (int it = 0; it < 4; ++it) issue1(3, 3, 0, it);
    };

    auto read_a = [&](half8 (&a)[4], int buf, int kk, int i) {
        a[i] = *reinterpret_cast<const half8*>(smem + buf * STAGE_HALVES + ((a_rd ^ (kk << 4)) + i * 32 * BK));
    };
    auto read_b = [&](half8 (&b)[2], int buf, int kk, int j) {
        b[j] = *reinterpret_cast<const half8*>(smem + buf * STAGE_HALVES + A_HALVES + ((b_rd ^ (kk << 4)) + j * 32 * BK));
    };
    // EARLY packs the six fragments into the first three groups so that every read of the buffer has
    // completed when the half-slice ends at the barrier that releases it.
    auto read_group = [&](half8 (&a)[4], half8 (&b)[2], int buf, int kk, int q, bool early) {
        if (early) {
            if (q == 0) { read_a(a, buf, kk, 0); read_b(b, buf, kk, 0); read_b(b, buf, kk, 1); }
            if (q == 1) { read_a(a, buf, kk, 1); read_a(a, buf, kk, 2); }
            if (q == 2) { read_a(a, buf, kk, 3); }
        } else {
            if (q == 0) { read_a(a, buf, kk, 0); read_b(b, buf, kk, 0); }
            if (q == 1) { read_b(b, buf, kk, 1); read_a(a, buf, kk, 1); }
            if (q == 2) { read_a(a, buf, kk, 2); }
            if (q == 3) { read_a(a, buf, kk, 3); }
        }
    };
    constexpr int READS_EARLY[4] = {3, 2, 1, 0};
    constexpr int READS_EVEN[4] = {2, 2, 1, 1};

    floatx16 accP[4][2], accQ[4][2];
    auto zero_acc = [&] {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    accP[i][j][r] = 0.f;
                    accQ[i][j][r] = 0.f;
                }
    };

    // Half a slice: 8 MFMAs on (ua, ub) in four groups of two; each group is preceded by the reads of one
    // fragment group of the next half-slice and followed by at most one direct-to-LDS load.
    auto half_slice = [&](floatx16 (&acc)[4][2], const half8 (&ua)[4], const half8 (&ub)[2], half8 (&la)[4],
                          half8 (&lb)[2], int lbuf, int lkk, bool early, int dstage, int dbuf, int dpart) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            read_group(la, lb, lbuf, lkk, q, early);
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[q][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ua[q], ub[j], acc[q][j], 0, 0, 0);
            {
                int left = early ? READS_EARLY[q] : READS_EVEN[q];
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int now = (left + (1 - j)) / (2 - j);
                    if (now == 1) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // DS reads
                    if (now == 2) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                 // one MFMA
                    left -= now;
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            if (dpart == 0 || q < 2) issue1(dstage, dbuf, dpart, q);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    half8 fa0[4], fb0[2], fa1[4], fb1[2];
    // Four slices (one trip round the LDS stages) accumulated into `acc`.
    auto four_slices = [&](floatx16 (&acc)[4][2], int kt) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            // first half of slice kt+u; reads its second half's fragments; loads the column part of slice kt+u+3
            half_slice(acc, fa0, fb0, fa1, fb1, u, 1, true, kt + u + 3, (u + 3) & 3, 1);
            // own loads of slice kt+u+1 have landed (the 12 youngest may still fly); own LDS reads done
            asm volatile("s_waitcnt vmcnt(12) lgkmcnt(0)\n\ts_barrier" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
            // second half; reads the first fragments of slice kt+u+1; loads the row part of slice kt+u+4
            // into the buffer of slice kt+u, which nobody reads any more
            half_slice(acc, fa1, fb1, fa0, fb0, (u + 1) & 3, 0, false, kt + u + 4, u, 0);
        }
    };

    int w = pos;
    if (w >= ga.total_tiles) return;   // grid <= total_tiles: cannot happen; nothing was issued yet
    int tensor, bi, bj;
    setup(w, tensor, bi, bj);
    issue_prologue();
    zero_acc();

    while (true) {
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
#pragma unroll
        for (int q = 0; q < 4; ++q) read_group(fa0, fb0, 0, 0, q, false);

        // K/32 and N/32 are multiples of 4, so a trip round the stages never straddles the two phases
        for (int kt = 0; kt < KTP; kt += 4) four_slices(accP, kt);
        for (int kt = KTP; kt < KT; kt += 4) four_slices(accQ, kt);
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");

        int32_t* const flag_out = ga.t[tensor].flag_out;
        const int ebi = bi, ebj = bj;

        w += G;
        const bool more = w < ga.total_tiles;
        if (more) {
            setup(w, tensor, bi, bj);
            issue_prologue();
        }

        // ---- sum of weight * P * Q over the tile.  Lane (l32, lh) holds, in register 4 q4 + e of MFMA
        // block (i, j), the pair (row 32 i + 8 q4 + 4 lh + e of the wave's rows, column 32 j + l32).
        const bool below = ebj < 2 * ebi;     // every pair of the tile has t > t'
        float sum = 0.f;
        uint32_t worst = 0u;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float p = accP[i][j][r], qv = accQ[i][j][r];
                    const uint32_t mp = __float_as_uint(p) & 0x7fffffffu, mq = __float_as_uint(qv) & 0x7fffffffu;
                    worst = mp > worst ? mp : worst;
                    worst = mq > worst ? mq : worst;
                    float wgt = 2.f;
                    if (!below) {
                        const int t = ebi * BM + wm * (BM / 2) + 32 * i + 8 * (r >> 2) + 4 * lh + (r & 3);
                        const int tp = ebj * BN + wn * (BN / 2) + 32 * j + l32;
                        wgt = t > tp ? 2.f : (t == tp ? 1.f : 0.f);
                    }
                    sum = fmaf(wgt * p, qv, sum);
                }
        sum = wave_sum(sum);
        const bool bad = __any(worst >= 0x7f800000u);
        int* redflag = reinterpret_cast<int*>(red_scratch) + 8;
        if (lane == 0) {
            red_scratch[wave] = sum;
            redflag[wave] = bad ? 1 : 0;
        }
        __syncthreads();
        if (tid == 0) {
            const double total = ((double)red_scratch[0] + (double)red_scratch[1]) +
                                 ((double)red_scratch[2] + (double)red_scratch[3]);
            atomicAdd(ga.acc, total);
            if (flag_out != nullptr && (redflag[0] | redflag[1] | redflag[2] | redflag[3])) atomicOr(flag_out, 1);
        }
        if (!more) break;
        zero_acc();
    }
}

// ---- host side ----------------------------------------------------------------------------

static int gram_cu_count() {
    static const int n = [] {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 256;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) return 256;
        return v;
    }();
    return n;
}

// `a` is a norm-pass contraction (A = X [C x M], B = dY [C x Nn], dense rows).
bool gram_eligible(const GemmArgs& a) {
    using namespace gram;
    return a.C >= BM && a.C % BM == 0 && a.M >= 4 * BK && a.M % (4 * BK) == 0 && a.Nn >= 4 * BK &&
           a.Nn % (4 * BK) == 0 && a.lda == a.M && a.ldb == a.Nn && a.C <= (1 << 20) && a.M < (1 << 22) &&
           a.Nn < (1 << 22) && (a.C / BM) * (a.C / BM + 1) < (1 << 24);
}

// Estimated cost in units of one 256 x 256 x 32 slice on one CU.  A 256 x 128 x 32 slice of this kernel
// does half the arithmetic but is bound by LDS bandwidth (a wave tile of 128 x 64 reads 1.5 times the
// operand bytes per flop of the direct kernel's 128 x 128): measured 0.73 of a full slice.
constexpr double kGramSlice = 0.73;
double gram_cost(const GemmArgs& a) {
    const double tm = (double)(a.C / gram::BM);
    return kGramSlice * tm * (tm + 1.0) * (double)(a.M + a.Nn) / 32.0;
}
double direct_cost(const GemmArgs& a) {
    return (double)((a.M + 255) / 256) * (double)((a.Nn + 255) / 256) * (double)a.C / 32.0;
}

// The order launch_gram_group runs its tensors in: longest tiles first, so that the static walk ends on the short ones.
static void gram_launch_order(std::vector<GemmArgs>& v) {
    std::stable_sort(v.begin(), v.end(), [](const GemmArgs& x, const GemmArgs& y) { return x.M + x.Nn > y.M + y.Nn; });
}

// When the Gram launches of these tensors finish, in the same units: workgroup p of a launch walks tiles p, p + G, ...
// (the kernel's static assignment), every tile of a tensor costs the same, and a launch ends with its busiest workgroup.
// A few hundred long tiles on 256 CUs end far later than (total work) / (number of CUs) says.
static double gram_finish_time(std::vector<GemmArgs> v) {
    gram_launch_order(v);
    const int cus = gram_cu_count();
    double total = 0.0;
    std::vector<double> load;
    for (size_t first = 0; first < v.size(); first += gram::MAX_GROUP) {
        const size_t cnt = v.size() - first < (size_t)gram::MAX_GROUP ? v.size() - first : (size_t)gram::MAX_GROUP;
        int64_t tiles = 0;
        for (size_t i = 0; i < cnt; ++i) {
            const int64_t tm = v[first + i].C / gram::BM;
            tiles += tm * (tm + 1);
        }
        const int64_t G = tiles < cus ? tiles : cus;
        load.assign((size_t)G, 0.0);
        int64_t w = 0;
        for (size_t i = 0; i < cnt; ++i) {
            const GemmArgs& a = v[first + i];
            const int64_t tm = a.C / gram::BM, n = tm * (tm + 1);
            const double tile = kGramSlice * (double)(a.M + a.Nn) / 32.0;
            for (int64_t k = 0; k < n; ++k, ++w) load[(size_t)(w % G)] += tile;
        }
        double longest = 0.0;
        for (double l : load) longest = l > longest ? l : longest;
        total += longest;
    }
    return total;
}

void choose_norm_route(int mode, const std::vector<GemmArgs>& all, std::vector<GemmArgs>& gram, std::vector<GemmArgs>& direct) {
    for (const GemmArgs& a : all) {
        const bool g = mode != LOMO_NORM_DIRECT && gram_eligible(a) && (mode == LOMO_NORM_GRAM || gram_cost(a) < direct_cost(a));
        (g ? gram : direct).push_back(a);
    }
    if (mode != LOMO_NORM_AUTO || gram.empty()) return;
    // Compare finishing times, not total work: the direct kernels' tiles are short and many (their share of the chip is
    // their work), the Gram tiles are long and few.
    double work_d = 0.0;
    for (const GemmArgs& a : gram) work_d += direct_cost(a);
    if (gram_finish_time(gram) >= work_d / (double)gram_cu_count()) {
        direct.insert(direct.end(), gram.begin(), gram.end());
        gram.clear();
    }
}

hipError_t launch_gram_group(const GemmArgs* list, int n, hipStream_t st) {
    using namespace gram;
    auto kern = lomo_gram_sqnorm_kernel;
    // thread-safe one-time set-up (initialisation of a function-local static)
    static const hipError_t cfg0 = allow_dynamic_lds(kern, LDS_BYTES);
    if (cfg0 != hipSuccess) return cfg0;
    // Longest tiles first: the static round-robin then ends on the short ones.
    std::vector<GemmArgs> order(list, list + n);
    gram_launch_order(order);
    list = order.data();
    for (int first = 0; first < n; first += MAX_GROUP) {
        const int cnt = (n - first < MAX_GROUP) ? (n - first) : MAX_GROUP;
        GroupArgs ga{};
        ga.acc = list[first].acc;
        ga.n = cnt;
        int tiles = 0;
        for (int i = 0; i < cnt; ++i) {
            const GemmArgs& a = list[first + i];
            GramTensor& t = ga.t[i];
            t.X = a.A; t.dY = a.B; t.flag_out = a.flag_out;
            t.K = (int)a.M; t.N = (int)a.Nn;
            t.tiles_m = (int)(a.C / BM);
            t.tile_begin = tiles;
            tiles += t.tiles_m * (t.tiles_m + 1);
        }
        ga.total_tiles = tiles;
        const int grid = tiles < gram_cu_count() ? tiles : gram_cu_count();
        hipError_t e = launch_timed(LOMO_KERNEL_GRAM_SQNORM, kern, dim3((unsigned)grid), dim3(NT), (size_t)LDS_BYTES, st, ga);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace lomo

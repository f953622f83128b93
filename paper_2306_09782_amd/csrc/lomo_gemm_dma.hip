// Persistent, grouped 256 x 256 MFMA contraction with a four-stage direct-to-LDS pipeline (gfx950).
//
// Same mathematics and epilogues as the other contraction kernels (fused wgrad + SGD update of
// paper section 3.2 / Algorithm 1, squared-norm pass of section 3.3.1, dgrad).  One launch covers
// the output tiles of up to MAX_GROUP tensors: one workgroup per CU walks the concatenated tile list
// with a fixed stride, so there is one ramp-up per pass instead of one per tensor and partial last
// rounds of one tensor are filled with tiles of the next.
//
// Data movement per tile:
//   * global -> LDS without passing through registers: global_load_lds_dwordx4 writes lane L's
//     16 bytes to M0 + 16 L, and each lane may fetch any global address, so a wave instruction
//     fills 1 KiB of LDS with the 16-byte chunks of two tile rows in swizzled order;
//   * four 32 KiB stages: the loads for slice kt+3 are issued while slice kt is multiplied (one
//     load instruction after every fourth MFMA, so the loads never queue up behind each other),
//     which covers memory latency and needs no staging registers;
//   * LDS -> MFMA operands with the transposing read ds_read_b64_tr_b16 (contraction-strided
//     operands) or ds_read_b128 (contraction-contiguous operand of dgrad); the fragments of the
//     next half-slice are read while the current one is multiplied, across the barrier;
//   * one barrier per slice.  The vector-memory counter is managed by hand because the compiler
//     would otherwise drain it before every LDS read;
//   * the first slices of the next tile are requested before the epilogue of the current one runs.
#include "lomo_gemm_common.h"

namespace lomo {

typedef short short4v __attribute__((ext_vector_type(4)));

namespace dma {

constexpr int BM = 256, BN = 256, BK = 32, NS = 4;
constexpr int A_HALVES = BK * BM, B_HALVES = BK * BN, STAGE_HALVES = A_HALVES + B_HALVES;
constexpr int EPI_UNIT_HALVES = 32 * 64;                 // staging block of the row epilogue: 32 rows x 64 columns (4 KiB)
// four stages + 32 KiB behind them: two staging blocks per wave for the row epilogue (update, store), whose first
// 256 bytes serve as the reduction scratch of the norm epilogue.  160 KiB in all, the whole LDS of a CU.
constexpr int LDS_BYTES = NS * STAGE_HALVES * 2 + 8 * EPI_UNIT_HALVES * 2;
constexpr int MAX_GROUP = 40;

struct GroupTensor {
    const uint16_t* A;
    const uint16_t* B;
    uint16_t* Out;
    const uint16_t* Res;
    int32_t* flag_out;
    int M, Nn, C, lda, ldb, ldo;
    int tiles_m, tiles_n, tile_begin;
};

struct GroupArgs {
    double* acc;
    const int32_t* flag_in;
    float s, lr, inv_s, clipv;
    const float* s_dev;
    int n, total_tiles;
    GroupTensor t[MAX_GROUP];
};

// Soft alignment of the workgroups of one XCD between rounds of the update kernels (timing only, no effect on results).
// The 32 tiles that an XCD works on in a round share operand panels through its L2 as long as they walk the
// contraction roughly in step; the update epilogue takes a different time on every CU (it waits for HBM), and without
// anything that pulls them together again the workgroups drift apart over the rounds until a panel has left the L2
// before its last reader asks for it (measured on the 7B stack: 22 GiB fetched per launch instead of 15.6).  Every
// workgroup that has finished the main loop of a round adds one to the counter of (next round, XCD) and, before it
// enters the next main loop, waits a bounded time until the others of its XCD have done so.  The counters are cleared
// by a small kernel in front of every launch.  Launches that overlap on one GPU share them: a workgroup may then
// wait less, or up to the bound once (after which it stops waiting), never for ever.
constexpr int SYNC_ROUNDS = 512;        // rounds beyond this run free
constexpr int SYNC_POLLS = 24;          // x 2048 clocks: the longest wait, about 30 us
__device__ int32_t g_round_arrive[SYNC_ROUNDS][8];

__global__ void clear_round_counters(int rounds) {
    const int i = (int)(blockIdx.x * blockDim.x + threadIdx.x);
    if (i < rounds * 8) (&g_round_arrive[0][0])[i] = 0;
}

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

// ---- row epilogue (update / store) --------------------------------------------------------------------
// The accumulator layout gives a lane 16 bytes of one output row at a time, so a wave instruction on global
// memory would touch 32 rows x 32 bytes.  Here each wave stages 32 x 64 blocks of its 128 x 128 sub-tile in
// LDS: the old W block arrives row-contiguous by direct-to-LDS loads (8 rows x 128 bytes per instruction),
// lanes pick their 16-byte pieces out of it, update, put the results back in the same places, and the block
// leaves row-contiguous again.  Three blocks per wave rotate; the first three loads are issued right after
// the tile's last slice, ahead of the next tile's first slices, and block u + 3 is requested as soon as block u
// is in registers.  16-byte chunk c of row r sits at chunk position c ^ (r & 7): the LDS serves eight lanes of a
// 16-byte access per clock (128 bytes), and eight consecutive lanes are either eight consecutive rows at one
// chunk (pieces) or the eight chunks of one row (rows), so both patterns are conflict-free.
__device__ __forceinline__ int swz_e(int r) { return r & 7; }

struct RowEpilogue {
    uint16_t* buf[3];
    uint32_t voff[4];
    const uint16_t* old_base;
    uint16_t* out_base;
    int64_t ldo, origin;      // origin: halves from the tensor base to this wave's 128 x 128 sub-tile

    __device__ __forceinline__ RowEpilogue(const GemmArgs& g, uint16_t* smem, int wave, int64_t m0, int64_t n0) {
        const int lane = threadIdx.x & 63;
        const int wm = wave & 1, wn = wave >> 1;
        // two blocks per wave behind the stages, the third in the B part of stage 3, which is idle between the last
        // slice of a tile and the first half-slice of the next
        buf[0] = smem + NS * STAGE_HALVES + wave * EPI_UNIT_HALVES;
        buf[1] = buf[0] + 4 * EPI_UNIT_HALVES;
        buf[2] = smem + 3 * STAGE_HALVES + A_HALVES + wave * EPI_UNIT_HALVES;
        ldo = g.ldo;
        old_base = (g.Res != nullptr) ? g.Res : g.Out;
        out_base = g.Out;
        origin = (n0 + wn * (BN / 2)) * ldo + m0 + wm * (BM / 2);
        // row-contiguous mapping inside a block: instruction q covers rows 8 q .. 8 q + 7, eight lanes per row
        const int rr = lane >> 3, slot = lane & 7;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int r = 8 * q + rr;
            voff[q] = (uint32_t)(r * ldo + ((slot ^ swz_e(r)) * 8)) * 2u;
        }
    }
    __device__ __forceinline__ int64_t unit_off(int u) const { return origin + 32 * (u >> 1) * ldo + 64 * (u & 1); }
    __device__ __forceinline__ void fill(int u) const {
        const uint16_t* base = old_base + unit_off(u);
        const uint32_t l = (uint32_t)(uintptr_t)buf[u % 3];
#pragma unroll
        for (int q = 0; q < 4; ++q) dma16(voff[q], base, l + (uint32_t)q * 1024u);
    }

    // `ahead`: vector-memory operations issued between the first three fills and this call (the next tile's first slices)
    template <int EPI>
    __device__ __forceinline__ void run(floatx16 (&acc)[4][4], float s, bool ahead) const {
        typedef uint32_t u32x2v __attribute__((ext_vector_type(2)));
        const int lane = threadIdx.x & 63;
        const int l32 = lane & 31, lh = lane >> 5;
        int poff[2][2];     // accumulator-layout mapping: this lane's piece (il, a) of row l32
#pragma unroll
        for (int il = 0; il < 2; ++il)
#pragma unroll
            for (int a = 0; a < 2; ++a) poff[il][a] = l32 * 64 + (((4 * il + 2 * a + lh) ^ swz_e(l32)) * 8);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int j = u >> 1, ih = u & 1;
            uint16_t* b = buf[u % 3];
            half8 w[2][2];
            if constexpr (EPI == EPI_UPDATE) {
                // Vector-memory operations complete in issue order.  Issued after this block's four loads: blocks 0-2,
                // the 28 loads of the next tile's first slices (if any), then per block u its stores and the loads of
                // block u + 3.  Wait until only those may still be outstanding.
                if (u == 0) { if (ahead) asm volatile("s_waitcnt vmcnt(36)" ::: "memory"); else asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); }
                else if (u == 1) { if (ahead) asm volatile("s_waitcnt vmcnt(40)" ::: "memory"); else asm volatile("s_waitcnt vmcnt(12)" ::: "memory"); }
                else if (u == 2) { if (ahead) asm volatile("s_waitcnt vmcnt(44)" ::: "memory"); else asm volatile("s_waitcnt vmcnt(16)" ::: "memory"); }
                else if (u <= 5) asm volatile("s_waitcnt vmcnt(20)" ::: "memory");
                else if (u == 6) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
                else asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
#pragma unroll
                for (int il = 0; il < 2; ++il)
#pragma unroll
                    for (int a = 0; a < 2; ++a) w[il][a] = *reinterpret_cast<const half8*>(b + poff[il][a]);
            }
#pragma unroll
            for (int il = 0; il < 2; ++il)
#pragma unroll
                for (int a = 0; a < 2; ++a) {
                    const int i = 2 * ih + il;
                    float v[8];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const u32x2v sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[i][j][8 * a + e]),
                                                                           __float_as_uint(acc[i][j][8 * a + 4 + e]), false, false);
                        v[e] = __uint_as_float(sw[0]);
                        v[4 + e] = __uint_as_float(sw[1]);
                    }
                    half8 out;
                    if constexpr (EPI == EPI_UPDATE) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) out[e] = (_Float16)fmaf(-s, v[e], (float)w[il][a][e]);
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; ++e) out[e] = (_Float16)v[e];
                    }
                    *reinterpret_cast<half8*>(b + poff[il][a]) = out;
                }
            half8 rows[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) rows[q] = *reinterpret_cast<const half8*>(b + q * 512 + lane * 8);
            if constexpr (EPI == EPI_UPDATE) {
                if (u + 3 < 8) {
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");     // the block is in registers: its buffer is free
                    fill(u + 3);
                }
            }
            uint16_t* dst = out_base + unit_off(u);
            const int rr = lane >> 3, slot = lane & 7;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int r = 8 * q + rr;
                *reinterpret_cast<half8*>(dst + r * ldo + ((slot ^ swz_e(r)) * 8)) = rows[q];
            }
        }
    }
};

}  // namespace dma

// A_STRIDED = false: the A operand is contraction-contiguous as well (forward product Y = X W^T with A = W),
// fetched and read like the contraction-contiguous B.
template <bool B_STRIDED, int EPI, bool A_STRIDED = true>
__global__ __launch_bounds__(NT) void lomo_contract_dma_kernel(dma::GroupArgs ga) {
    using namespace dma;
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];

    if (EPI == EPI_UPDATE && ga.flag_in != nullptr && *ga.flag_in != 0) return;   // step dropped

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const int G = gridDim.x;

    // Position of this workgroup inside a window of G consecutive tiles: workgroups of one XCD
    // (blockIdx % 8) take a contiguous run, which the band order below turns into an 8 x 4 block of
    // tiles that share operand panels in that XCD's L2.
    int pos;
    {
        const int x = (int)(blockIdx.x & 7), local = (int)(blockIdx.x >> 3);
        const int q = G >> 3, r = G & 7;
        pos = x * q + (x < r ? x : r) + local;
    }

    // round alignment (update kernels): this XCD's run of positions and how many of them have a tile in round k
    constexpr bool ALIGN_ROUNDS = (EPI == EPI_UPDATE || EPI == EPI_CLIPV) && A_STRIDED && B_STRIDED;
    const int xcd = (int)(blockIdx.x & 7);
    const int xcd_first = xcd * (G >> 3) + (xcd < (G & 7) ? xcd : (G & 7));
    const int xcd_count = (G >> 3) + (xcd < (G & 7) ? 1 : 0);
    auto xcd_tiles_in_round = [&](int k) {
        const int v = ga.total_tiles - k * G - xcd_first;
        return v < 0 ? 0 : (v > xcd_count ? xcd_count : v);
    };
    bool align_rounds = ALIGN_ROUNDS;      // cleared after a wait that ran into its bound
    int round = 0;

    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
    const uint32_t lds_wave = lds0 + (uint32_t)wave * 4096u;   // this wave's first KiB slot in a tile
    uint16_t* red_scratch = smem + NS * STAGE_HALVES;

    // ---- fragment read offsets (halves): fixed for the whole kernel
    const int g4 = lane >> 4, j16 = lane & 15;
    const int mhalf = g4 & 1, kh = g4 >> 1, rib = j16 >> 2, piece = j16 & 3;
    int a_rd;
    if constexpr (A_STRIDED) {
        a_rd = (8 * kh + rib) * BM + (((wm * (BM / 16) + 2 * mhalf + (piece >> 1)) ^ swz_s(rib)) * 8) + (piece & 1) * 4;
    } else {
        const int ml = wm * (BM / 2) + (lane & 31), lh = lane >> 5;
        a_rd = ml * BK + ((lh ^ swz_c(ml)) * 8);
    }
    int b_rd;
    if constexpr (B_STRIDED) {
        b_rd = (8 * kh + rib) * BN + (((wn * (BN / 16) + 2 * mhalf + (piece >> 1)) ^ swz_s(rib)) * 8) + (piece & 1) * 4;
    } else {
        const int nl = wn * (BN / 2) + (lane & 31), lh = lane >> 5;
        b_rd = nl * BK + ((lh ^ swz_c(nl)) * 8);
    }

    // ---- per-tile state of the loads
    uint32_t a_voff[4], b_voff[4];
    const uint16_t* pa = nullptr;
    const uint16_t* pb = nullptr;
    int64_t a_step = 0, b_step = 0;
    int KT = 0;

    // Locate tile number w of the concatenated list; set up the load state; return its coordinates.
    // A workgroup's tile numbers only grow, so the search for the tile's tensor resumes at the previous tile's.
    auto setup = [&](int w, int& tensor, int64_t& m0, int64_t& n0) {
        int k = tensor;
        while (k + 1 < ga.n && w >= ga.t[k + 1].tile_begin) ++k;
        const GroupTensor& T = ga.t[k];
        const int t = w - T.tile_begin;
        constexpr int GM = 8;
        const int per_band = GM * T.tiles_n;
        const int band = t / per_band;
        const int first_m = band * GM;
        const int gsz = (T.tiles_m - first_m < GM) ? (T.tiles_m - first_m) : GM;
        const int in_band = t - band * per_band;
        const int tm = first_m + in_band % gsz;
        const int tn = in_band / gsz;
        tensor = k;
        m0 = (int64_t)tm * BM;
        n0 = (int64_t)tn * BN;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int q = wave * 4 + it;
            if constexpr (A_STRIDED) {
                const int r = 2 * q + (lane >> 5), cp = lane & 31;
                a_voff[it] = (uint32_t)(r * T.lda + ((cp ^ swz_s(r)) * 8)) * 2u;
            } else {
                const int n = 16 * q + (lane >> 2), cp = lane & 3;
                a_voff[it] = (uint32_t)(n * T.lda + ((cp ^ swz_c(n)) * 8)) * 2u;
            }
            if constexpr (B_STRIDED) {
                const int r = 2 * q + (lane >> 5), cp = lane & 31;
                b_voff[it] = (uint32_t)(r * T.ldb + ((cp ^ swz_s(r)) * 8)) * 2u;
            } else {
                const int n = 16 * q + (lane >> 2), cp = lane & 3;
                b_voff[it] = (uint32_t)(n * T.ldb + ((cp ^ swz_c(n)) * 8)) * 2u;
            }
        }
        pa = A_STRIDED ? (T.A + m0) : (T.A + m0 * (int64_t)T.lda);
        pb = B_STRIDED ? (T.B + n0) : (T.B + n0 * (int64_t)T.ldb);
        a_step = A_STRIDED ? (int64_t)BK * T.lda : (int64_t)BK;
        b_step = B_STRIDED ? (int64_t)BK * T.ldb : (int64_t)BK;
        KT = T.C / BK;
    };

    // One DMA instruction: part 0 = A tile, part 1 = B tile; `it` selects this wave's KiB slot.
    auto issue1 = [&](int stage, int buf, int part, int it) {
        const int s = stage < KT ? stage : KT - 1;   // past the end: harmless re-read, keeps the counter regular
        const uint32_t l = lds_wave + (uint32_t)buf * (STAGE_HALVES * 2u) + (uint32_t)part * (A_HALVES * 2u) +
                           (uint32_t)it * 1024u;
        if (part == 0) dma16(a_voff[it], pa + (int64_t)s * a_step, l);
        else dma16(b_voff[it], pb + (int64_t)s * b_step, l);
    };
    // Slices 0..2 and the A part of slice 3 of the tile that `setup` selected.
    auto issue_prologue = [&] {
#pragma unroll
        for (int st = 0; st < 3; ++st) {
#pragma unroll
            for (int it = 0; it < 4; ++it) issue1(st, st, 0, it);
#pragma unroll
            for (int it = 0; it < 4; ++it) issue1(st, st, 1, it);
        }
#pragma unroll
        for (int it = 0; it < 4; ++it) issue1(3, 3, 0, it);
    };

    // ---- fragment reads, in the order the MFMAs consume them: a0, b0..b3, a1..a3
    auto read_a = [&](half8 (&a)[4], int buf, int kk, int i) {
        if constexpr (A_STRIDED) {
            const uint16_t* p = smem + buf * STAGE_HALVES + ((a_rd ^ (i << 5)) + kk * 16 * BM);
            a[i] = read_tr8(p, p + 4 * BM);
        } else {
            a[i] = *reinterpret_cast<const half8*>(smem + buf * STAGE_HALVES + ((a_rd ^ (kk << 4)) + i * 32 * BK));
        }
    };
    auto read_b = [&](half8 (&b)[4], int buf, int kk, int j) {
        const uint16_t* bs = smem + buf * STAGE_HALVES + A_HALVES;
        if constexpr (B_STRIDED) {
            const uint16_t* p = bs + ((b_rd ^ (j << 5)) + kk * 16 * BN);
            b[j] = read_tr8(p, p + 4 * BN);
        } else {
            b[j] = *reinterpret_cast<const half8*>(bs + ((b_rd ^ (kk << 4)) + j * 32 * BK));
        }
    };
    // Fragment groups.  EARLY packs the eight fragments into the first three groups, so that every
    // read has completed when the half-slice ends at a barrier.
    auto read_group = [&](half8 (&a)[4], half8 (&b)[4], int buf, int kk, int q, bool early) {
        if (early) {
            if (q == 0) { read_a(a, buf, kk, 0); read_b(b, buf, kk, 0); read_b(b, buf, kk, 1); }
            if (q == 1) { read_b(b, buf, kk, 2); read_b(b, buf, kk, 3); read_a(a, buf, kk, 1); }
            if (q == 2) { read_a(a, buf, kk, 2); read_a(a, buf, kk, 3); }
        } else {
            if (q == 0) { read_a(a, buf, kk, 0); read_b(b, buf, kk, 0); }
            if (q == 1) { read_b(b, buf, kk, 1); read_b(b, buf, kk, 2); }
            if (q == 2) { read_b(b, buf, kk, 3); read_a(a, buf, kk, 1); }
            if (q == 3) { read_a(a, buf, kk, 2); read_a(a, buf, kk, 3); }
        }
    };
    constexpr int RA = A_STRIDED ? 2 : 1, RB = B_STRIDED ? 2 : 1;     // LDS read instructions per fragment
    constexpr int READS_EARLY[4] = {RA + 2 * RB, 2 * RB + RA, 2 * RA, 0};
    constexpr int READS_EVEN[4] = {RA + RB, 2 * RB, RB + RA, 2 * RA};

    floatx16 acc[4][4];
    auto zero_acc = [&] {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    };

    // Half a slice: 16 MFMAs on (ua, ub) in four groups; each group is preceded by the reads of one
    // fragment group of the next half-slice and followed by one direct-to-LDS load, so that LDS reads,
    // global loads and MFMAs overlap instead of queueing behind each other.
    auto half_slice = [&](const half8 (&ua)[4], const half8 (&ub)[4], half8 (&la)[4], half8 (&lb)[4], int lbuf, int lkk,
                          bool early, int dstage, int dbuf, int dpart) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            read_group(la, lb, lbuf, lkk, q, early);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[q][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ua[q], ub[j], acc[q][j], 0, 0, 0);
            {   // spread this group's reads in front of its four MFMAs
                int left = early ? READS_EARLY[q] : READS_EVEN[q];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int now = (left + (3 - j)) / (4 - j);
                    if (now == 1) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // DS reads
                    if (now == 2) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                    if (now == 3) __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    left -= now;
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            issue1(dstage, dbuf, dpart, q);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- walk the tile list: tile w = round * G + pos; every workgroup leaves through `break`
    int w = pos;
    if (w >= ga.total_tiles) return;   // cannot happen with grid <= total_tiles; nothing was issued yet
    int tensor = 0;
    int64_t m0, n0;
    setup(w, tensor, m0, n0);
    issue_prologue();
    zero_acc();

    while (true) {
        if constexpr (ALIGN_ROUNDS) {
            if (round >= 1 && round < SYNC_ROUNDS && tid == 0 && align_rounds) {
                const int need = xcd_tiles_in_round(round);
                int polls = 0;
                while (__hip_atomic_load(&g_round_arrive[round][xcd], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < need &&
                       polls < SYNC_POLLS) {
                    __builtin_amdgcn_s_sleep(32);
                    ++polls;
                }
                if (polls == SYNC_POLLS) align_rounds = false;     // something else holds CUs: stop waiting
            }
        }
        // every load of this tile's first slices has landed and is visible to all waves (and thread 0 is back)
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        half8 fa0[4], fb0[4], fa1[4], fb1[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) read_group(fa0, fb0, 0, 0, q, false);

        // KT is a multiple of 4: the body is unrolled over the four LDS stages so that every LDS
        // address is a register plus an immediate.
        for (int kt = 0; kt < KT; kt += 4) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                // first half of slice kt+u; reads its second half's fragments; loads the B part of slice kt+u+3
                half_slice(fa0, fb0, fa1, fb1, u, 1, true, kt + u + 3, (u + 3) & 3, 1);
                // own loads of slice kt+u+1 landed (two younger slices may still fly); own LDS reads done
                asm volatile("s_waitcnt vmcnt(16) lgkmcnt(0)\n\ts_barrier" ::: "memory");
                __builtin_amdgcn_sched_barrier(0);
                // second half; reads the first fragments of the next slice; loads the A part of slice
                // kt+u+4 into the buffer of slice kt+u, which nobody reads any more
                half_slice(fa1, fb1, fa0, fb0, (u + 1) & 3, 0, false, kt + u + 4, u, 0);
            }
        }
        // drain: the loads past the end (re-reads) have landed, all waves are done with the LDS stages
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");

        // epilogue arguments of the tile just finished
        GemmArgs g;
        g.Out = ga.t[tensor].Out;
        g.Res = ga.t[tensor].Res;
        g.ldo = ga.t[tensor].ldo;
        g.s = ga.s;
        g.s_dev = ga.s_dev;
        g.lr = ga.lr;
        g.inv_s = ga.inv_s;
        g.clipv = ga.clipv;
        g.acc = ga.acc;
        g.flag_out = ga.t[tensor].flag_out;
        const int64_t em0 = m0, en0 = n0;

        // request the first blocks of W (update), then the first slices of the next tile, then finish this one
        w += G;
        const bool more = w < ga.total_tiles;
        ++round;
        if constexpr (ALIGN_ROUNDS) {
            if (more && round < SYNC_ROUNDS && tid == 0) atomicAdd(&g_round_arrive[round][xcd], 1);
        }
        if constexpr (EPI == EPI_UPDATE || EPI == EPI_STORE) {
            const RowEpilogue re(g, smem, wave, em0, en0);
            if constexpr (EPI == EPI_UPDATE) {
                re.fill(0);
                re.fill(1);
                re.fill(2);
            }
            if (more) {
                setup(w, tensor, m0, n0);
                issue_prologue();
            }
            re.template run<EPI>(acc, g.s_dev != nullptr ? *g.s_dev : g.s, more);
        } else {
            if (more) {
                setup(w, tensor, m0, n0);
                issue_prologue();
            }
            epilogue<BM, BN, EPI>(acc, g, red_scratch, em0, en0, BM, BN);
        }
        if (!more) break;
        zero_acc();
    }
}

// ---- host side ----------------------------------------------------------------------------

static int cu_count() {
    static const int n = [] {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 256;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) return 256;
        return v;
    }();
    return n;
}

bool dma_eligible(const GemmArgs& a) {
    using namespace dma;
    return a.M > 0 && a.Nn > 0 && a.C >= 4 * BK && a.M % BM == 0 && a.Nn % BN == 0 && a.C % (4 * BK) == 0 &&
           a.M < (1 << 30) && a.Nn < (1 << 30) && a.C < (1 << 30) &&
           (int64_t)BK * a.lda < (1 << 30) && (int64_t)BN * a.ldb < (1 << 30) && a.ldo < (1 << 30) &&
           (a.M / BM) * (a.Nn / BN) < (1 << 24);
}

template <bool B_STRIDED, int EPI, bool A_STRIDED>
static hipError_t launch_dma_group_impl(const GemmArgs* list, int n, hipStream_t st) {
    using namespace dma;
    auto kern = lomo_contract_dma_kernel<B_STRIDED, EPI, A_STRIDED>;
    // thread-safe one-time set-up (initialisation of a function-local static)
    static const hipError_t cfg0 = allow_dynamic_lds(kern, LDS_BYTES);
    if (cfg0 != hipSuccess) return cfg0;
    for (int first = 0; first < n; first += MAX_GROUP) {
        const int cnt = (n - first < MAX_GROUP) ? (n - first) : MAX_GROUP;
        GroupArgs ga{};
        ga.acc = list[first].acc;
        ga.flag_in = list[first].flag_in;
        ga.s = list[first].s;
        ga.s_dev = list[first].s_dev;
        ga.lr = list[first].lr;
        ga.inv_s = list[first].inv_s;
        ga.clipv = list[first].clipv;
        ga.n = cnt;
        int tiles = 0;
        for (int i = 0; i < cnt; ++i) {
            const GemmArgs& a = list[first + i];
            GroupTensor& t = ga.t[i];
            t.A = a.A; t.B = a.B; t.Out = a.Out; t.Res = a.Res; t.flag_out = a.flag_out;
            t.M = (int)a.M; t.Nn = (int)a.Nn; t.C = (int)a.C;
            t.lda = (int)a.lda; t.ldb = (int)a.ldb; t.ldo = (int)a.ldo;
            t.tiles_m = (int)(a.M / BM); t.tiles_n = (int)(a.Nn / BN);
            t.tile_begin = tiles;
            tiles += t.tiles_m * t.tiles_n;
        }
        ga.total_tiles = tiles;
        const int grid = tiles < cu_count() ? tiles : cu_count();
        if ((EPI == EPI_UPDATE || EPI == EPI_CLIPV) && A_STRIDED && B_STRIDED) {     // the kernels that align their rounds
            int rounds = (tiles + grid - 1) / grid;
            if (rounds > SYNC_ROUNDS) rounds = SYNC_ROUNDS;
            hipLaunchKernelGGL(clear_round_counters, dim3((unsigned)((rounds * 8 + 255) / 256)), dim3(256), 0, st, rounds);
        }
        hipError_t e = launch_timed(list[first].family, kern, dim3((unsigned)grid), dim3(NT), (size_t)LDS_BYTES, st, ga);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

template <bool B_STRIDED, int EPI>
hipError_t launch_dma_group(const GemmArgs* list, int n, hipStream_t st) {
    return launch_dma_group_impl<B_STRIDED, EPI, true>(list, n, st);
}

// Forward product (A contraction-contiguous): same eligibility, except that A's row stride now multiplies
// the 256 tile rows instead of the 32 slice rows.
template <int EPI>
bool try_launch_dma_nt(const GemmArgs& a, hipStream_t st, hipError_t* err) {
    if (!dma_eligible(a) || (int64_t)dma::BM * a.lda >= (1 << 30) || (a.M / dma::BM) * (a.Nn / dma::BN) < 192) return false;
    *err = launch_dma_group_impl<false, EPI, false>(&a, 1, st);
    return true;
}
template bool try_launch_dma_nt<EPI_STORE>(const GemmArgs&, hipStream_t, hipError_t*);
template bool try_launch_dma_nt<EPI_UPDATE>(const GemmArgs&, hipStream_t, hipError_t*);

// Single tensor: worth it when there are enough tiles to fill most of the chip.
template <bool B_STRIDED, int EPI>
bool try_launch_dma(const GemmArgs& a, hipStream_t st, hipError_t* err) {
    if (!dma_eligible(a) || (a.M / dma::BM) * (a.Nn / dma::BN) < 192) return false;
    *err = launch_dma_group<B_STRIDED, EPI>(&a, 1, st);
    return true;
}

template bool try_launch_dma<true, EPI_UPDATE>(const GemmArgs&, hipStream_t, hipError_t*);
template bool try_launch_dma<true, EPI_CLIPV>(const GemmArgs&, hipStream_t, hipError_t*);
template bool try_launch_dma<true, EPI_SQNORM>(const GemmArgs&, hipStream_t, hipError_t*);
template bool try_launch_dma<false, EPI_STORE>(const GemmArgs&, hipStream_t, hipError_t*);
template hipError_t launch_dma_group<true, EPI_UPDATE>(const GemmArgs*, int, hipStream_t);
template hipError_t launch_dma_group<true, EPI_CLIPV>(const GemmArgs*, int, hipStream_t);
template hipError_t launch_dma_group<true, EPI_SQNORM>(const GemmArgs*, int, hipStream_t);
template hipError_t launch_dma_group<false, EPI_STORE>(const GemmArgs*, int, hipStream_t);

}  // namespace lomo

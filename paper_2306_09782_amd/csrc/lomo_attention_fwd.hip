// Forward of causal softmax attention (head width 128) on the rotated q, k and v, for recomputing the
// activations that Algorithm 1's backward loop reads from a checkpoint of the layer input (paper section 3.2;
// activation checkpointing: sections 2 and 4.1).  Produces o and lse = log sum_j exp(q_i . k_j / sqrt(d)) in
// the layout the backward kernel reads.
//
// One workgroup per (sequence, head, block of 64 queries) walks the key blocks up to the diagonal.  The four
// waves split the block 2 x 2: wave (wr, wc) owns queries 32 wr .. +31 and, in every key block, keys
// 32 wc .. +31.  Each wave keeps its own running maximum, sum and output accumulator over the keys it has
// seen (an online softmax per wave, so no reduction across waves inside the loop); the two key halves are
// merged once at the end through LDS.  The score tile is computed transposed (keys are the MFMA rows), so a
// lane owns one query: its maximum is a scan of the lane's registers plus one exchange with lane + 32, and
// the probabilities become the B operand of o^T += v^T p^T after a v_permlane32_swap, without passing
// through LDS.  Probabilities are rounded to fp16 relative to the running maximum; accumulation is fp32;
// o is rounded once.  Deterministic.
#include "lomo_attention_common.h"

namespace lomo {

namespace attn {

constexpr int OUT_BYTES = BLK * PO * 4;                          // fp32 output tile, reuses the K / V tiles
constexpr int FWD_LDS_BYTES = OUT_BYTES + 2 * 2 * BLK * 4;       // + running maximum and sum of both key halves

struct FwdArgs {
    const uint16_t* qkv;   // [T x 3H]
    uint16_t* o;           // [T x H]
    float* lse;            // [T x nh]
    int s, nh, H;
};

}  // namespace attn

__global__ __launch_bounds__(256, 2) void attention_forward_kernel(attn::FwdArgs a) {
    using namespace attn;
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    uint16_t* sK = smem;
    uint16_t* sV = sK + TILE;
    float* sOut = reinterpret_cast<float*>(smem);
    float* sStat = reinterpret_cast<float*>(reinterpret_cast<char*>(smem) + OUT_BYTES);     // [wc][m | l][query]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave & 1, wc = wave >> 1;
    const int l32 = lane & 31, lh = lane >> 5;
    const int g4 = lane >> 4, j16 = lane & 15;
    const int mhalf = g4 & 1, kh = g4 >> 1, rib = j16 >> 2, piece = j16 & 3;
    const int tr_row = 8 * kh + rib, tr_col = 16 * mhalf + 4 * piece;
    const int tr_sw0 = ((rib << 2) | (2 * kh)) << 3, tr_sw1 = ((rib << 2) | (2 * kh + 1)) << 3;

    // a contiguous run of (sequence, head) pairs per XCD, heaviest query blocks first
    const int nb = a.s / BLK;
    int pos;
    {
        const int G = gridDim.x, x = (int)(blockIdx.x & 7), local = (int)(blockIdx.x >> 3);
        const int q = G >> 3, r = G & 7;
        pos = x * q + (x < r ? x : r) + local;
    }
    const int head = pos / nb, within = pos - head * nb;
    const int n = head % a.nh, b = head / a.nh;
    const int qi = nb - 1 - within;
    const int64_t ld3 = 3 * (int64_t)a.H;
    const int64_t t0 = (int64_t)b * a.s;
    const uint16_t* gq = a.qkv + (int64_t)n * D;
    const uint16_t* gk = gq + a.H;
    const uint16_t* gv = gk + a.H;
    const float scale_log2e = 0.08838834764831845f * 1.4426950408889634f;     // log2(e) / sqrt(128)

    // this wave's 32 queries as MFMA B fragments, once through LDS
    u32x4 r0[4], r1[4];
    fetch_tile(r0, gq + (t0 + (int64_t)qi * BLK) * ld3, ld3);
    stash_tile(r0, sK);
    __syncthreads();
    half8 fq[D / 16];
    {
        const int row = 32 * wr + l32;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks)
            fq[ks] = *reinterpret_cast<const half8*>(sK + row * PD + ((16 * ks + 8 * lh) ^ (swz(row) << 3)));
    }

    floatx16 accO[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) accO[i][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;     // log2 domain; l_run is this lane's share (its half of the keys)

    fetch_tile(r0, gk + t0 * ld3, ld3);
    fetch_tile(r1, gv + t0 * ld3, ld3);
    const int query = 32 * wr + l32;
    for (int blk = 0; blk <= qi; ++blk) {
        __syncthreads();     // everybody is done with the previous tiles (and with the Q tile)
        stash_tile(r0, sK);
        stash_tile(r1, sV);
        __syncthreads();
        if (blk < qi) {
            const int64_t row0 = t0 + (int64_t)(blk + 1) * BLK;
            fetch_tile(r0, gk + row0 * ld3, ld3);
            fetch_tile(r1, gv + row0 * ld3, ld3);
        }
        const bool diag = blk == qi;
        if (diag && wc == 1 && wr == 0) continue;     // keys 32..63 against queries 0..31: all above the diagonal

        // S^T for this wave's 32 keys x 32 queries
        floatx16 accS;
#pragma unroll
        for (int r = 0; r < 16; ++r) accS[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
            const int krow = 32 * wc + l32;
            const half8 fk = *reinterpret_cast<const half8*>(sK + krow * PD + ((16 * ks + 8 * lh) ^ (swz(krow) << 3)));
            accS = __builtin_amdgcn_mfma_f32_32x32x16_f16(fk, fq[ks], accS, 0, 0, 0);
        }
        // register r <-> key 32 wc + 8 (r / 4) + 4 lh + r % 4 of query `query`
        float x[16];
        float bmax = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = 32 * wc + 8 * (r >> 2) + 4 * lh + (r & 3);
            x[r] = (diag && key > query) ? -INFINITY : accS[r] * scale_log2e;
            bmax = fmaxf(bmax, x[r]);
        }
        bmax = fmaxf(bmax, __shfl_xor(bmax, 32, 64));
        const float m_new = fmaxf(m_run, bmax);
        const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;     // a query that has seen no key yet
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_ref);
        float psum = 0.f;
        uint32_t pk[8];
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            const float p0 = __builtin_amdgcn_exp2f(x[r] - m_ref), p1 = __builtin_amdgcn_exp2f(x[r + 1] - m_ref);
            psum += p0 + p1;
            typedef _Float16 half2v __attribute__((ext_vector_type(2)));
            const half2v h = {(_Float16)p0, (_Float16)p1};
            pk[r >> 1] = __builtin_bit_cast(uint32_t, h);
        }
        l_run = fmaf(l_run, alpha, psum);
        m_run = m_new;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) accO[i][r] *= alpha;

        // o^T[dcol][query] += v^T[dcol][key] p^T[key][query] over this wave's 32 keys, 16 at a time
        typedef uint32_t u32x2v __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            // lane halves exchange so that each holds eight consecutive keys: 16 ks + 8 lh .. + 7
            const u32x2v s0 = __builtin_amdgcn_permlane32_swap(pk[4 * ks + 0], pk[4 * ks + 2], false, false);
            const u32x2v s1 = __builtin_amdgcn_permlane32_swap(pk[4 * ks + 1], pk[4 * ks + 3], false, false);
            const u32x4 w = {s0[0], s1[0], s0[1], s1[1]};
            const half8 fp = __builtin_bit_cast(half8, w);
            const int krow = 32 * wc + 16 * ks + tr_row;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int col = 32 * i + tr_col;
                const int o0 = krow * PD + (col ^ tr_sw0), o1 = (krow + 4) * PD + (col ^ tr_sw1);
                accO[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(read_tr8(sV + o0, sV + o1), fp, accO[i], 0, 0, 0);
            }
        }
    }

    // ---- merge the two key halves: common maximum, total sum, then o through LDS as fp32
    l_run += __shfl_xor(l_run, 32, 64);
    __syncthreads();     // the K / V tiles are free
    if (lh == 0) {
        sStat[(2 * wc + 0) * BLK + query] = m_run;
        sStat[(2 * wc + 1) * BLK + query] = l_run;
    }
    __syncthreads();
    const float m0 = sStat[0 * BLK + query], l0 = sStat[1 * BLK + query];
    const float m1 = sStat[2 * BLK + query], l1 = sStat[3 * BLK + query];
    const float mt = fmaxf(m0, m1);     // finite: key 0 is visible to every query
    const float lt = l0 * __builtin_amdgcn_exp2f(m0 - mt) + l1 * __builtin_amdgcn_exp2f(m1 - mt);
    const float f = __builtin_amdgcn_exp2f(m_run - mt) / lt;
    // accO[i][r] <-> dcol = 32 i + 8 (r / 4) + 4 lh + r % 4
    if (wc == 1) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) sOut[query * PO + 32 * i + 8 * (r >> 2) + 4 * lh + (r & 3)] = accO[i][r] * f;
    }
    __syncthreads();
    if (wc == 0) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) sOut[query * PO + 32 * i + 8 * (r >> 2) + 4 * lh + (r & 3)] += accO[i][r] * f;
        if (lh == 0)
            a.lse[(t0 + (int64_t)qi * BLK + query) * a.nh + n] = (mt + __builtin_amdgcn_logf(lt)) * 0.6931471805599453f;
    }
    __syncthreads();
    {
        const int row = tid >> 2, c0 = 32 * (tid & 3);
        const float* src = sOut + row * PO + c0;
        uint16_t* dst = a.o + (t0 + (int64_t)qi * BLK + row) * a.H + (int64_t)n * D + c0;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float4 v0 = *reinterpret_cast<const float4*>(src + 8 * u);
            const float4 v1 = *reinterpret_cast<const float4*>(src + 8 * u + 4);
            const half8 h = {(_Float16)v0.x, (_Float16)v0.y, (_Float16)v0.z, (_Float16)v0.w,
                             (_Float16)v1.x, (_Float16)v1.y, (_Float16)v1.z, (_Float16)v1.w};
            *reinterpret_cast<half8*>(dst + 8 * u) = h;
        }
    }
}

hipError_t launch_attention_forward(const uint16_t* qkv, uint16_t* o, float* lse, int64_t B, int64_t s, int64_t nh,
                                    hipStream_t st) {
    using namespace attn;
    // thread-safe one-time set-up (initialisation of a function-local static)
    static const hipError_t cfg0 = allow_dynamic_lds(attention_forward_kernel, FWD_LDS_BYTES);
    if (cfg0 != hipSuccess) return cfg0;
    FwdArgs a;
    a.qkv = qkv; a.o = o; a.lse = lse;
    a.s = (int)s; a.nh = (int)nh; a.H = (int)(nh * D);
    const dim3 grid((unsigned)((s / BLK) * nh * B));
    hipLaunchKernelGGL(attention_forward_kernel, grid, dim3(256), FWD_LDS_BYTES, st, a);
    return hipGetLastError();
}

}  // namespace lomo

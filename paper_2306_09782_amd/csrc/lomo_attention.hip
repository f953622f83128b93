// Backward of causal softmax attention with the rotary step, for the hand-on gradient of Algorithm 1
// (paper section 3.2) through the self-attention block of a LLaMA layer (the models of section 4), gfx950.
//
// Tokens t = b * s + pos; head n owns columns [128 n, 128 n + 128) of q, k, v, o.  qkv holds the rotated
// q and k and v side by side ([T x 3H]); lse[t][n] = log sum_j exp(S_tj) is saved by the forward pass.
//
//   P_ij = exp(q_i . k_j / sqrt(d) - lse_i)  (j <= i),   dP_ij = do_i . v_j,   delta_i = do_i . o_i
//   dS = P (dP - delta) / sqrt(d);   dv_j = sum_i P_ij do_i;   dk_j = sum_i dS_ij q_i;   dq_i = sum_j dS_ij k_j
//   then the rotary step backwards (rotation by the negative angle) on dq and dk.
//
// fp16 storage, fp32 accumulation on the MFMA units; P and dS pass through fp16 before the products that
// consume them (fp16 training holds them as fp16 tensors); dq, dk, dv are rounded once, after the rotation.
//
// Two deterministic kernels, no atomics: one workgroup per (sequence, head, block of 64 keys) walks the query
// blocks at or below it and accumulates dk, dv; one per (sequence, head, block of 64 queries) walks the key
// blocks up to it and accumulates dq.  Both recompute S, P, dP, dS per 64 x 64 block (32x32x16 MFMA, four
// waves in 2 x 2); the loop operand of the next block is fetched into registers while the current one is
// multiplied.  Transposed operands come from LDS through ds_read_b64_tr_b16.
#include "lomo_attention_common.h"

namespace lomo {

namespace attn {

struct Args {
    const uint16_t* qkv;   // [T x 3H]
    const uint16_t* o;     // [T x H]
    const uint16_t* dO;    // [T x H]
    const float* lse;      // [T x nh]
    const float* delta;    // [T x nh]
    const float* cosv;     // [s x 64] or null
    const float* sinv;
    uint16_t* dqkv;        // [T x 3H]
    int s, nh, H;
};

}  // namespace attn

// delta[t][n] = sum_c dO[t][128 n + c] * o[t][128 n + c]: sixteen lanes per (token, head), eight columns each.
__global__ __launch_bounds__(256) void attention_delta_kernel(const uint16_t* __restrict__ o, const uint16_t* __restrict__ dO,
                                                              float* __restrict__ delta, int64_t rows) {
    const int64_t row = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);     // row = t * nh + n
    const int part = threadIdx.x & 15;
    float sum = 0.f;
    if (row < rows) {
        const half8 a = *reinterpret_cast<const half8*>(o + row * attn::D + part * 8);
        const half8 b = *reinterpret_cast<const half8*>(dO + row * attn::D + part * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) sum = fmaf((float)a[e], (float)b[e], sum);
    }
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
    if (row < rows && part == 0) delta[row] = sum;
}

// MODE 0: workgroup = (key block j, head, sequence): dk, dv.  MODE 1: workgroup = (query block i, head, sequence): dq.
template <int MODE>
__global__ __launch_bounds__(256, 2) void attention_backward_kernel(attn::Args a) {
    using namespace attn;
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    // Two [64 x 128] tiles for the operand pair that moves with the loop (MODE 0: Q_i and dO_i; MODE 1: K_j and
    // V_j); the pair that stays is held as MFMA fragments in registers.  Less LDS, two workgroups per CU.
    uint16_t* sA = smem;
    uint16_t* sB = sA + TILE;
    uint16_t* sP = sB + TILE;
    uint16_t* sDS = sP + BLK * PS;
    float* sL = reinterpret_cast<float*>(sDS + BLK * PS);
    float* sDelta = sL + BLK;
    float* sOut = reinterpret_cast<float*>(smem);     // [64 x PO] fp32, after the loop (over both tiles and into sP)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave & 1, wc = wave >> 1;
    const int l32 = lane & 31, lh = lane >> 5;
    const int g4 = lane >> 4, j16 = lane & 15;
    const int mhalf = g4 & 1, kh = g4 >> 1, rib = j16 >> 2, piece = j16 & 3;
    const int tr_row = 8 * kh + rib, tr_col = 16 * mhalf + 4 * piece;
    // swizzles of the rows a transposing read touches in the big tiles: rows 16 ks + tr_row and + 4
    const int tr_sw0 = ((rib << 2) | (2 * kh)) << 3, tr_sw1 = ((rib << 2) | (2 * kh + 1)) << 3;

    // Workgroups are dealt to the 8 XCDs round-robin; give each XCD a contiguous run of (sequence, head) pairs so
    // that the blocks of one head, which re-read the same q, k, v, dO rows, meet in one L2.
    const int nb = a.s / BLK;
    int pos;
    {
        const int G = gridDim.x, x = (int)(blockIdx.x & 7), local = (int)(blockIdx.x >> 3);
        const int q = G >> 3, r = G & 7;
        pos = x * q + (x < r ? x : r) + local;
    }
    const int head = pos / nb, within = pos - head * nb;
    const int n = head % a.nh, b = head / a.nh;
    const int fixed = (MODE == 0) ? within : nb - 1 - within;   // heaviest blocks first
    const int64_t ld3 = 3 * (int64_t)a.H, ldh = a.H;
    const int64_t t0 = (int64_t)b * a.s;
    const uint16_t* gq = a.qkv + (int64_t)n * D;
    const uint16_t* gk = gq + a.H;
    const uint16_t* gv = gk + a.H;
    const uint16_t* gdo = a.dO + (int64_t)n * D;
    const float scale = 0.08838834764831845f;     // 1 / sqrt(128)
    // exp(x) as the hardware's 2^y with y = x log2(e): its relative error (about 1e-6 for |x| < 30) is far
    // below half an fp16 ulp, and the softmax phase is bound by vector ALU work, not by the matrix cores
    const float log2e = 1.4426950408889634f, scale_log2e = scale * log2e;

    // the operand pair that stays: K_j, V_j (MODE 0) or Q_i, dO_i with lse and delta (MODE 1), through LDS
    // once into the registers of the wave that multiplies with them
    u32x4 r0[4], r1[4];
    if (MODE == 0) {
        fetch_tile(r0, gk + (t0 + (int64_t)fixed * BLK) * ld3, ld3);
        fetch_tile(r1, gv + (t0 + (int64_t)fixed * BLK) * ld3, ld3);
    } else {
        fetch_tile(r0, gq + (t0 + (int64_t)fixed * BLK) * ld3, ld3);
        fetch_tile(r1, gdo + (t0 + (int64_t)fixed * BLK) * ldh, ldh);
        if (tid < BLK) {
            sL[tid] = a.lse[(t0 + (int64_t)fixed * BLK + tid) * a.nh + n] * log2e;
            sDelta[tid] = a.delta[(t0 + (int64_t)fixed * BLK + tid) * a.nh + n];
        }
    }
    stash_tile(r0, sA);
    stash_tile(r1, sB);
    __syncthreads();
    half8 fx[D / 16], fy[D / 16];
    {
        const int row = ((MODE == 0) ? 32 * wc : 32 * wr) + l32;     // MODE 0: this wave's keys; MODE 1: its queries
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
            fx[ks] = *reinterpret_cast<const half8*>(sA + row * PD + ((16 * ks + 8 * lh) ^ (swz(row) << 3)));
            fy[ks] = *reinterpret_cast<const half8*>(sB + row * PD + ((16 * ks + 8 * lh) ^ (swz(row) << 3)));
        }
    }

    floatx16 acc0[2], acc1[2];     // MODE 0: dv, dk;  MODE 1: dq (acc1 unused)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            acc0[i][r] = 0.f;
            acc1[i][r] = 0.f;
        }

    const int first = (MODE == 0) ? fixed : 0;
    const int last = (MODE == 0) ? nb - 1 : fixed;
    float rl = 0.f, rd = 0.f;
    auto fetch_moving = [&](int blk) {
        const int64_t row0 = t0 + (int64_t)blk * BLK;
        if (MODE == 0) {
            fetch_tile(r0, gq + row0 * ld3, ld3);
            fetch_tile(r1, gdo + row0 * ldh, ldh);
            if (tid < BLK) {
                rl = a.lse[(row0 + tid) * a.nh + n];
                rd = a.delta[(row0 + tid) * a.nh + n];
            }
        } else {
            fetch_tile(r0, gk + row0 * ld3, ld3);
            fetch_tile(r1, gv + row0 * ld3, ld3);
        }
    };
    fetch_moving(first);

    for (int blk = first; blk <= last; ++blk) {
        __syncthreads();     // everybody is done with the tiles of the previous block
        stash_tile(r0, sA);
        stash_tile(r1, sB);
        if (MODE == 0 && tid < BLK) {
            sL[tid] = rl * log2e;
            sDelta[tid] = rd;
        }
        __syncthreads();
        if (blk < last) fetch_moving(blk + 1);     // in flight while this block is multiplied

        // ---- S^T = K Q^T and dP^T = V dO^T for this wave's 32 keys x 32 queries: the keys are the MFMA rows, so a
        // lane owns one query (one lse, one delta) and four consecutive keys per register group
        floatx16 accS, accP;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            accS[r] = 0.f;
            accP[r] = 0.f;
        }
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
            const int mrow = ((MODE == 0) ? 32 * wr : 32 * wc) + l32;
            const int off = mrow * PD + ((16 * ks + 8 * lh) ^ (swz(mrow) << 3));
            if (MODE == 0) {      // moving Q_i, dO_i come from LDS; K_j, V_j from registers
                const half8 fq = *reinterpret_cast<const half8*>(sA + off);
                const half8 fd = *reinterpret_cast<const half8*>(sB + off);
                accS = __builtin_amdgcn_mfma_f32_32x32x16_f16(fx[ks], fq, accS, 0, 0, 0);
                accP = __builtin_amdgcn_mfma_f32_32x32x16_f16(fy[ks], fd, accP, 0, 0, 0);
            } else {              // moving K_j, V_j come from LDS; Q_i, dO_i from registers
                const half8 fk = *reinterpret_cast<const half8*>(sA + off);
                const half8 fv = *reinterpret_cast<const half8*>(sB + off);
                accS = __builtin_amdgcn_mfma_f32_32x32x16_f16(fk, fx[ks], accS, 0, 0, 0);
                accP = __builtin_amdgcn_mfma_f32_32x32x16_f16(fv, fy[ks], accP, 0, 0, 0);
            }
        }
        // ---- P and dS in fp16, [query][key]: four consecutive keys per 8-byte store
        {
            const bool diag = blk == fixed;
            const int qrow = 32 * wr + l32;
            const float lq = sL[qrow], dq = sDelta[qrow];
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int key0 = 32 * wc + 8 * q4 + 4 * lh;
                half4 hp, hd;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int r = 4 * q4 + e;
                    float p = __builtin_amdgcn_exp2f(fmaf(scale_log2e, accS[r], -lq));
                    float ds = scale * p * (accP[r] - dq);
                    if (diag && key0 + e > qrow) {
                        p = 0.f;
                        ds = 0.f;
                    }
                    hp[e] = (_Float16)p;
                    hd[e] = (_Float16)ds;
                }
                *reinterpret_cast<half4*>(sP + qrow * PS + key0) = hp;
                *reinterpret_cast<half4*>(sDS + qrow * PS + key0) = hd;
            }
        }
        __syncthreads();

        if (MODE == 0) {
            // dv^T[dcol][key] += dO^T P,  dk^T[dcol][key] += Q^T dS   (contraction over the 64 queries)
#pragma unroll
            for (int ks = 0; ks < BLK / 16; ++ks) {
                const uint16_t* pp = sP + (16 * ks + tr_row) * PS + 32 * wc + tr_col;
                const uint16_t* pd = sDS + (16 * ks + tr_row) * PS + 32 * wc + tr_col;
                const half8 bP = read_tr8(pp, pp + 4 * PS);
                const half8 bD = read_tr8(pd, pd + 4 * PS);
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int col = 64 * wr + 32 * i + tr_col;
                    const int o0 = (16 * ks + tr_row) * PD + (col ^ tr_sw0), o1 = (16 * ks + tr_row + 4) * PD + (col ^ tr_sw1);
                    acc0[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(read_tr8(sB + o0, sB + o1), bP, acc0[i], 0, 0, 0);
                    acc1[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(read_tr8(sA + o0, sA + o1), bD, acc1[i], 0, 0, 0);
                }
            }
        } else {
            // dq^T[dcol][query] += K^T dS^T   (contraction over the 64 keys)
#pragma unroll
            for (int ks = 0; ks < BLK / 16; ++ks) {
                const half8 bD = *reinterpret_cast<const half8*>(sDS + (32 * wc + l32) * PS + 16 * ks + 8 * lh);
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int col = 64 * wr + 32 * i + tr_col;
                    const int o0 = (16 * ks + tr_row) * PD + (col ^ tr_sw0), o1 = (16 * ks + tr_row + 4) * PD + (col ^ tr_sw1);
                    acc0[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(read_tr8(sA + o0, sA + o1), bD, acc0[i], 0, 0, 0);
                }
            }
        }
    }

    // ---- results: through LDS as fp32 so that the rotary pairs (c, c + 64) meet and stores are 16 bytes wide
    const int64_t orow0 = t0 + (int64_t)fixed * BLK;
    auto emit = [&](floatx16 (&acc)[2], int64_t colbase, bool rotate) {
        // thread: row = tid / 4, sixteen pairs (c, c + 64) with c = 16 * (tid % 4) ...
        const int row = tid >> 2, c0 = 16 * (tid & 3);
        const int pos = fixed * BLK + row;
        float4 co[4], si[4];
        if (rotate) {      // the table rows of this thread, requested before the exchange through LDS
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                co[u] = *reinterpret_cast<const float4*>(a.cosv + pos * 64 + c0 + 4 * u);
                si[u] = *reinterpret_cast<const float4*>(a.sinv + pos * 64 + c0 + 4 * u);
            }
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                sOut[(32 * wc + l32) * PO + 64 * wr + 32 * i + 8 * (r >> 2) + 4 * lh + (r & 3)] = acc[i][r];
        __syncthreads();
        const float* src = sOut + row * PO;
        half8 lo[2], hi[2];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float4 x1 = *reinterpret_cast<const float4*>(src + c0 + 4 * u);
            const float4 x2 = *reinterpret_cast<const float4*>(src + c0 + 64 + 4 * u);
            const float a1[4] = {x1.x, x1.y, x1.z, x1.w}, a2[4] = {x2.x, x2.y, x2.z, x2.w};
            float cc[4] = {1.f, 1.f, 1.f, 1.f}, ss[4] = {0.f, 0.f, 0.f, 0.f};
            if (rotate) {
                cc[0] = co[u].x; cc[1] = co[u].y; cc[2] = co[u].z; cc[3] = co[u].w;
                ss[0] = si[u].x; ss[1] = si[u].y; ss[2] = si[u].z; ss[3] = si[u].w;
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float y1 = a1[e], y2 = a2[e];
                if (rotate) {
                    y1 = fmaf(a2[e], ss[e], a1[e] * cc[e]);
                    y2 = fmaf(-a1[e], ss[e], a2[e] * cc[e]);
                }
                lo[u >> 1][4 * (u & 1) + e] = (_Float16)y1;
                hi[u >> 1][4 * (u & 1) + e] = (_Float16)y2;
            }
        }
        uint16_t* dst = a.dqkv + (orow0 + row) * ld3 + colbase + (int64_t)n * D + c0;
        *reinterpret_cast<half8*>(dst) = lo[0];
        *reinterpret_cast<half8*>(dst + 8) = lo[1];
        *reinterpret_cast<half8*>(dst + 64) = hi[0];
        *reinterpret_cast<half8*>(dst + 72) = hi[1];
    };
    const bool rot = a.cosv != nullptr;
    if (MODE == 0) {
        emit(acc0, 2 * (int64_t)a.H, false);    // dv
        emit(acc1, (int64_t)a.H, rot);          // dk
    } else {
        emit(acc0, 0, rot);                     // dq
    }
}

hipError_t launch_attention_backward(const uint16_t* qkv, const uint16_t* o, const uint16_t* dO, const float* lse,
                                     const float* cosv, const float* sinv, float* delta, uint16_t* dqkv, int64_t B, int64_t s,
                                     int64_t nh, hipStream_t st) {
    using namespace attn;
    // thread-safe one-time set-up (initialisation of a function-local static)
    static const hipError_t cfg0 = allow_dynamic_lds(attention_backward_kernel<0>, LDS_BYTES);
    if (cfg0 != hipSuccess) return cfg0;
    static const hipError_t cfg1 = allow_dynamic_lds(attention_backward_kernel<1>, LDS_BYTES);
    if (cfg1 != hipSuccess) return cfg1;
    const int64_t rows = B * s * nh;
    hipLaunchKernelGGL(attention_delta_kernel, dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, st, o, dO, delta, rows);
    Args a;
    a.qkv = qkv; a.o = o; a.dO = dO; a.lse = lse; a.delta = delta; a.cosv = cosv; a.sinv = sinv; a.dqkv = dqkv;
    a.s = (int)s; a.nh = (int)nh; a.H = (int)(nh * D);
    const dim3 grid((unsigned)((s / BLK) * nh * B));
    hipLaunchKernelGGL(attention_backward_kernel<0>, grid, dim3(256), LDS_BYTES, st, a);
    hipLaunchKernelGGL(attention_backward_kernel<1>, grid, dim3(256), LDS_BYTES, st, a);
    return hipGetLastError();
}

}  // namespace lomo

// Pieces shared by the attention forward and backward kernels: tile geometry, the chunk swizzle of the
// [64 x 128] LDS tiles, tile fetch / stash and the transposing LDS read.
#pragma once
#include "lomo_gemm_common.h"

namespace lomo {

typedef short short4a __attribute__((ext_vector_type(4)));

namespace attn {

constexpr int D = 128;        // head width
constexpr int BLK = 64;       // queries / keys per block
constexpr int PD = D;         // LDS pitch of a [64 x 128] fp16 tile (halves): unpadded, 16-byte chunks swizzled
constexpr int PS = BLK + 8;   // LDS pitch of a [64 x 64] fp16 tile
constexpr int PO = D + 4;     // LDS pitch of the fp32 output tile (floats)
constexpr int TILE = BLK * PD;
constexpr int LDS_BYTES = 2 * TILE * 2 + 2 * BLK * PS * 2 + 2 * BLK * 4;

__device__ __forceinline__ half8 read_tr8(const uint16_t* p0, const uint16_t* p1) {
    typedef __attribute__((address_space(3))) short4a* lds_p;
    const short4a lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p0));
    const short4a hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p1));
    return __builtin_bit_cast(half8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// A [64 x 128] fp16 tile: thread tid owns the 16-byte chunks tid, tid + 256, tid + 512, tid + 768
// (row = chunk / 16, column = 8 * (chunk % 16)).
__device__ __forceinline__ void fetch_tile(u32x4 (&r)[4], const uint16_t* g, int64_t ld) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int c = threadIdx.x + 256 * u;
        r[u] = *reinterpret_cast<const u32x4*>(g + (int64_t)(c >> 4) * ld + (c & 15) * 8);
    }
}
// Chunk swizzle of the [64 x 128] tiles: 16-byte chunk c of row r sits at position c ^ swz(r).  Rows that
// differ in their low two bits are 4 chunks apart (the four rows of a transposing read fall on disjoint banks,
// and so do its two 16-column halves), rows that differ in the next two bits are 1..3 chunks apart (sixteen
// consecutive rows read at the same column hit sixteen different chunks).
__device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

__device__ __forceinline__ void stash_tile(const u32x4 (&r)[4], uint16_t* s) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int c = threadIdx.x + 256 * u;
        *reinterpret_cast<u32x4*>(s + (c >> 4) * PD + (((c & 15) ^ swz(c >> 4)) * 8)) = r[u];
    }
}

}  // namespace attn

}  // namespace lomo

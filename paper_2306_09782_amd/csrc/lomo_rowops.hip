// Bandwidth-bound kernels of the LOMO hot path for gfx950: embedding rows and RMSNorm gains.
//
// Every parameter gets its gradient and its update inside back-propagation (paper section 3.2);
// for an embedding table only the rows whose token occurs in the batch have a gradient, and for a
// gain vector the gradient is a column reduction.  Both run in two modes: squared norm + overflow
// detection (first pass, section 3.3) and in-place fp32 update rounded once to fp16 (second pass).
// All reductions have a fixed order, so results are bit-reproducible from run to run.
#include "lomo_kernels.h"

namespace lomo {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));

static inline int64_t next_pow2(int64_t v) {
    int64_t p = 1;
    while (p < v) p <<= 1;
    return p;
}
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ------------------------------------------------------------------------------------------
// Embedding grouping.  Three routes, one result (positions sorted by id, ties in position order; unique ids
// ascending; segment offsets): one workgroup for batches of at most 8192 positions, sorted chunks + merge rounds
// for larger ones (both below), and, for ids too wide for their 32-bit keys, the route of this section: a
// bitonic sort of unique 64-bit keys (id << 32 | position) and a one-workgroup segment scan.  Unique keys make
// any correct sort stable by construction: ties between equal ids are broken by position.
// ------------------------------------------------------------------------------------------

constexpr int SORT_NT = 1024;
constexpr int SORT_CHUNK = 8192;   // keys sorted per workgroup in LDS (64 KB)

__global__ void emb_make_keys(const int32_t* __restrict__ ids, int64_t T, int64_t Tpad, uint64_t* __restrict__ keys) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= Tpad) return;
    keys[i] = (i < T) ? (((uint64_t)(uint32_t)ids[i] << 32) | (uint64_t)(uint32_t)i) : ~0ull;
}

__device__ __forceinline__ void cmpx(uint64_t& a, uint64_t& b, bool up) {
    if ((a > b) == up) {
        const uint64_t t = a;
        a = b;
        b = t;
    }
}

// Runs, inside LDS, the stages j = j_start .. 1 of merge step k for k = k_first .. k_last.
// Each workgroup owns SORT_CHUNK (or fewer) consecutive keys.
__global__ __launch_bounds__(SORT_NT) void emb_bitonic_local(uint64_t* __restrict__ keys, int64_t Tpad,
                                                             int64_t k_first, int64_t k_last) {
    __shared__ uint64_t s[SORT_CHUNK];
    const int64_t chunk = Tpad < SORT_CHUNK ? Tpad : SORT_CHUNK;
    const int64_t base = (int64_t)blockIdx.x * chunk;
    for (int64_t i = threadIdx.x; i < chunk; i += SORT_NT) s[i] = keys[base + i];
    __syncthreads();
    for (int64_t k = k_first; k <= k_last; k <<= 1) {
        int64_t j = (k >> 1) < chunk ? (k >> 1) : (chunk >> 1);
        for (; j > 0; j >>= 1) {
            for (int64_t pidx = threadIdx.x; pidx < (chunk >> 1); pidx += SORT_NT) {
                const int64_t lo = ((pidx & ~(j - 1)) << 1) | (pidx & (j - 1));
                const bool up = (((base + lo) & k) == 0);
                uint64_t a = s[lo], b = s[lo + j];
                cmpx(a, b, up);
                s[lo] = a;
                s[lo + j] = b;
            }
            __syncthreads();
        }
    }
    for (int64_t i = threadIdx.x; i < chunk; i += SORT_NT) keys[base + i] = s[i];
}

// One global compare-exchange stage (j >= SORT_CHUNK).
__global__ void emb_bitonic_global(uint64_t* __restrict__ keys, int64_t Tpad, int64_t k, int64_t j) {
    const int64_t pidx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (pidx >= (Tpad >> 1)) return;
    const int64_t lo = ((pidx & ~(j - 1)) << 1) | (pidx & (j - 1));
    const bool up = ((lo & k) == 0);
    uint64_t a = keys[lo], b = keys[lo + j];
    cmpx(a, b, up);
    keys[lo] = a;
    keys[lo + j] = b;
}

// Head flags + exclusive scan over the sorted keys: one workgroup walks the array.
__global__ __launch_bounds__(SORT_NT) void emb_segments(const uint64_t* __restrict__ keys, int64_t T,
                                                        int32_t* __restrict__ perm, int32_t* __restrict__ unique_ids,
                                                        int32_t* __restrict__ seg_offsets, int32_t* __restrict__ n_unique) {
    __shared__ int32_t wsum[SORT_NT / 64];
    __shared__ int32_t carry_s;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) carry_s = 0;
    __syncthreads();
    for (int64_t start = 0; start < T; start += SORT_NT) {
        const int64_t i = start + tid;
        int32_t head = 0;
        uint32_t id = 0;
        if (i < T) {
            const uint64_t key = keys[i];
            id = (uint32_t)(key >> 32);
            perm[i] = (int32_t)(uint32_t)key;
            head = (i == 0) || ((uint32_t)(keys[i - 1] >> 32) != id);
        }
        // inclusive scan inside the wave, then across waves
        int32_t v = head;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int32_t o = __shfl_up(v, off, 64);
            if (lane >= off) v += o;
        }
        if (lane == 63) wsum[wave] = v;
        __syncthreads();
        int32_t before = 0;
        for (int w = 0; w < wave; ++w) before += wsum[w];
        const int32_t carry = carry_s;
        const int32_t excl = carry + before + v - head;
        if (head) {
            unique_ids[excl] = (int32_t)id;
            seg_offsets[excl] = (int32_t)i;
        }
        __syncthreads();
        if (tid == SORT_NT - 1) carry_s = carry + before + v;
        __syncthreads();
    }
    if (tid == 0) {
        n_unique[0] = carry_s;
        seg_offsets[carry_s] = (int32_t)T;
    }
}

// ------------------------------------------------------------------------------------------
// Small batches (at most 8192 positions, id * 8192 below 2^32): keys, sort and segments in ONE workgroup.
// 32-bit keys id << shift | position; every thread keeps 8 elements in registers.  The sort is a
// least-significant-digit-first radix sort over the id bits, four bits per pass, every pass stable: positions
// start in ascending order, so equal ids end up in ascending position order.
// One pass: wave w owns the 512 consecutive elements w * 512 + r * 64 + lane (r = 0..7).  For each r the lanes
// that hold the same digit find each other with four ballots; the lowest of them adds the group's size to the
// wave's counter of that digit in LDS and hands the counter's old value to the group, so an element's rank
// among the wave's elements of its digit is (old value) + (lanes of the group below it): rounds r are issued in
// order and LDS executes a wave's operations in order.  After one barrier every wave scans the 16 x waves
// counters (digit-major, wave-minor) for itself and knows where its elements of each digit start; the exchange
// goes through LDS.  Two barriers per pass.
// ------------------------------------------------------------------------------------------

constexpr int GS_KPT = 8;
constexpr int GS_MAX = 8192;
constexpr int GS_DIGIT_BITS = 4, GS_DIGITS = 1 << GS_DIGIT_BITS;

// The passes.  In: key[r] = element wave * 512 + r * 64 + lane of the workgroup's blockDim.x * 8 keys; the bits
// [shift, shift + id_bits) are sorted on.  Out: the sorted keys in sk (a barrier has been passed; at least one
// pass runs).  hist: 16 x waves counters, digit-major; wbase: waves x 16.
__device__ __forceinline__ void radix_sort_in_lds(uint32_t (&key)[GS_KPT], uint32_t* __restrict__ sk, int32_t* __restrict__ hist,
                                                  int32_t* __restrict__ wbase, int shift, int id_bits) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nw = (int)(blockDim.x >> 6);                                  // 1, 2, 4, 8 or 16
    const int s0 = wave * (64 * GS_KPT) + lane;
    const uint64_t below = (1ull << lane) - 1ull;
    for (int bit = shift; bit < shift + id_bits; bit += GS_DIGIT_BITS) {
        if (lane < GS_DIGITS) hist[lane * nw + wave] = 0;
        int rank[GS_KPT], digit[GS_KPT];
#pragma unroll
        for (int r = 0; r < GS_KPT; ++r) {
            const int d = (int)((key[r] >> bit) & (uint32_t)(GS_DIGITS - 1));
            uint64_t same = ~0ull;
#pragma unroll
            for (int b = 0; b < GS_DIGIT_BITS; ++b) {
                const bool set = (d >> b) & 1;
                const uint64_t vote = __ballot(set);
                same &= set ? vote : ~vote;
            }
            const int lower = __popcll(same & below);
            int old = 0;
            if (lower == 0) old = atomicAdd(&hist[d * nw + wave], __popcll(same));
            rank[r] = __shfl(old, __ffsll((unsigned long long)same) - 1, 64) + lower;
            digit[r] = d;
        }
        __syncthreads();     // all counters are final; everybody has read its keys of the previous pass out of sk
        {
            // entries 4 lane .. 4 lane + 3 of the digit-major list of 16 * nw counters
            int v[4] = {0, 0, 0, 0};
            const bool live = 4 * lane < GS_DIGITS * nw;
            if (live) {
                const int4 q = *reinterpret_cast<const int4*>(hist + 4 * lane);
                v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
            }
            const int mine = (v[0] + v[1]) + (v[2] + v[3]);
            int incl = mine;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int o = __shfl_up(incl, off, 64);
                if (lane >= off) incl += o;
            }
            int start = incl - mine;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int i = 4 * lane + k;
                if (live && (i & (nw - 1)) == wave) wbase[wave * GS_DIGITS + i / nw] = start;
                start += v[k];
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int r = 0; r < GS_KPT; ++r) sk[wbase[wave * GS_DIGITS + digit[r]] + rank[r]] = key[r];
        __syncthreads();
#pragma unroll
        for (int r = 0; r < GS_KPT; ++r) key[r] = sk[s0 + 64 * r];
    }
}

__global__ __launch_bounds__(1024) void emb_group_small(const int32_t* __restrict__ ids, int T, int N, int shift,
                                                        int id_bits, int32_t* __restrict__ perm,
                                                        int32_t* __restrict__ unique_ids, int32_t* __restrict__ seg_offsets,
                                                        int32_t* __restrict__ n_unique) {
    __shared__ __attribute__((aligned(16))) uint32_t sk[GS_MAX];
    __shared__ __attribute__((aligned(16))) int32_t hist[GS_DIGITS * 16];     // [digit][wave]
    __shared__ int32_t wbase[16 * GS_DIGITS];                               // [wave][digit]
    __shared__ int32_t wsum[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nw = (int)(blockDim.x >> 6);
    const int s0 = wave * (64 * GS_KPT) + lane;                             // this lane's element of round r: s0 + 64 r
    uint32_t key[GS_KPT];
#pragma unroll
    for (int r = 0; r < GS_KPT; ++r) {
        const int e = s0 + 64 * r;
        key[r] = (e < T) ? (((uint32_t)ids[e] << shift) | (uint32_t)e) : 0xffffffffu;   // padding: every bit set
    }
    radix_sort_in_lds(key, sk, hist, wbase, shift, id_bits);
    // ---- sk holds the sorted keys (at least one pass has run): eight consecutive ones per thread from here on
    const int e0 = tid * GS_KPT;
    {
        const uint4 q0 = *reinterpret_cast<const uint4*>(sk + e0), q1 = *reinterpret_cast<const uint4*>(sk + e0 + 4);
        key[0] = q0.x; key[1] = q0.y; key[2] = q0.z; key[3] = q0.w;
        key[4] = q1.x; key[5] = q1.y; key[6] = q1.z; key[7] = q1.w;
    }
    __syncthreads();
    // ---- segments: head flags, exclusive scan, outputs
    const uint32_t mask = (1u << shift) - 1u;
    uint32_t prev = (uint32_t)__shfl_up((int)key[GS_KPT - 1], 1, 64);
    if (lane == 63) sk[wave] = key[GS_KPT - 1];
    __syncthreads();
    if (lane == 0) prev = wave > 0 ? sk[wave - 1] : 0u;
    int heads = 0;
    bool head[GS_KPT];
#pragma unroll
    for (int r = 0; r < GS_KPT; ++r) {
        const int e = e0 + r;
        const uint32_t before = r == 0 ? prev : key[r - 1];
        head[r] = e < T && (e == 0 || (before >> shift) != (key[r] >> shift));
        heads += head[r] ? 1 : 0;
    }
    int v = heads;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(v, off, 64);
        if (lane >= off) v += o;
    }
    if (lane == 63) wsum[wave] = v;
    __syncthreads();
    int base = 0, total = 0;
    for (int w = 0; w < nw; ++w) {
        base += w < wave ? wsum[w] : 0;
        total += wsum[w];
    }
    int idx = base + v - heads;
#pragma unroll
    for (int r = 0; r < GS_KPT; ++r) {
        const int e = e0 + r;
        if (e < T) perm[e] = (int32_t)(key[r] & mask);
        if (head[r]) {
            unique_ids[idx] = (int32_t)(key[r] >> shift);
            seg_offsets[idx] = e;
            ++idx;
        }
    }
    if (tid == 0) {
        n_unique[0] = total;
        seg_offsets[total] = T;
    }
}

// Whether the one-workgroup route applies: N = padded size (power of two, 512..8192), ids < V fit above `shift` bits.
static inline bool group_small_plan(int64_t T, int64_t V, int* N, int* shift, int* id_bits) {
    if (T <= 0 || T > GS_MAX || V <= 0) return false;
    int64_t n = next_pow2(T);
    if (n < GS_KPT * 64) n = GS_KPT * 64;
    int sh = 0;
    while ((1ll << sh) < n) ++sh;
    if ((V - 1) >> (32 - sh) != 0) return false;                  // id << shift must stay below 2^32
    if ((((V - 1) << sh) | (n - 1)) >= 0xffffffffll) return false;   // all-ones is the padding key
    int ib = 1;
    while ((1ll << ib) < V) ++ib;
    *N = (int)n;
    *shift = sh;
    *id_bits = ib;
    return true;
}

// ------------------------------------------------------------------------------------------
// Larger batches (ids below 2^19): every 8192 consecutive positions are sorted by one workgroup with the radix
// sort above (keys id << 13 | position inside the chunk) and written as 64-bit keys id << 32 | position; the
// sorted runs are merged pairwise, doubling per round, between two key buffers (merge path: a workgroup owns
// 2048 consecutive outputs, finds where they start in both runs by bisection, stages its inputs in LDS and every
// thread merges eight outputs).  Keys are unique, so the merge needs no tie rule.  Segments: heads are counted
// per 2048 keys, then every workgroup adds up the counts before it and writes its part.
// ------------------------------------------------------------------------------------------

constexpr int GS_CHUNK_SHIFT = 13;     // log2(GS_MAX)
constexpr int MG_NT = 256, MG_KPT = 8, MG_TILE = MG_NT * MG_KPT;

static inline bool group_chunks_plan(int64_t T, int64_t V, int* id_bits) {
    if (T <= GS_MAX || V <= 0) return false;
    if ((V - 1) >> (32 - GS_CHUNK_SHIFT) != 0) return false;
    if ((((V - 1) << GS_CHUNK_SHIFT) | (GS_MAX - 1)) >= 0xffffffffll) return false;
    int ib = 1;
    while ((1ll << ib) < V) ++ib;
    *id_bits = ib;
    return true;
}

__global__ __launch_bounds__(1024) void emb_sort_chunks(const int32_t* __restrict__ ids, int64_t T, int id_bits,
                                                        uint64_t* __restrict__ out) {
    __shared__ __attribute__((aligned(16))) uint32_t sk[GS_MAX];
    __shared__ __attribute__((aligned(16))) int32_t hist[GS_DIGITS * 16];
    __shared__ int32_t wbase[16 * GS_DIGITS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t base = (int64_t)blockIdx.x * GS_MAX;
    const int n = (int)((T - base) < GS_MAX ? (T - base) : GS_MAX);
    const int s0 = wave * (64 * GS_KPT) + lane;
    uint32_t key[GS_KPT];
#pragma unroll
    for (int r = 0; r < GS_KPT; ++r) {
        const int e = s0 + 64 * r;
        key[r] = (e < n) ? (((uint32_t)ids[base + e] << GS_CHUNK_SHIFT) | (uint32_t)e) : 0xffffffffu;
    }
    radix_sort_in_lds(key, sk, hist, wbase, GS_CHUNK_SHIFT, id_bits);
    for (int e = tid; e < n; e += (int)blockDim.x) {
        const uint32_t k = sk[e];
        out[base + e] = ((uint64_t)(k >> GS_CHUNK_SHIFT) << 32) | (uint64_t)(base + (int64_t)(k & (uint32_t)(GS_MAX - 1)));
    }
}

// How many of the first d merged outputs of the sorted runs A (nA keys) and B (nB keys) come from A.
template <typename Index>
__device__ __forceinline__ Index merge_split(const uint64_t* A, Index nA, const uint64_t* B, Index nB, Index d) {
    Index lo = d > nB ? d - nB : 0, hi = d < nA ? d : nA;
    while (lo < hi) {
        const Index mid = (lo + hi) >> 1;
        if (A[mid] < B[d - 1 - mid]) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

// One round: runs of `run` keys (the last one may be shorter or have no partner) become runs of 2 * run keys.
// MG_TILE divides 2 * run, so a workgroup's outputs belong to one pair of runs.
__global__ __launch_bounds__(MG_NT) void emb_merge_round(const uint64_t* __restrict__ src, uint64_t* __restrict__ dst, int64_t T,
                                                         int64_t run) {
    __shared__ uint64_t s[MG_TILE];
    __shared__ int64_t split[2];
    const int tid = threadIdx.x;
    const int64_t out0 = (int64_t)blockIdx.x * MG_TILE;
    const int64_t a0 = out0 / (2 * run) * (2 * run);
    const int64_t a1 = a0 + run < T ? a0 + run : T, b1 = a0 + 2 * run < T ? a0 + 2 * run : T;
    const uint64_t* A = src + a0;
    const uint64_t* B = src + a1;
    const int64_t nA = a1 - a0, nB = b1 - a1;
    const int64_t d0 = out0 - a0, d1 = d0 + MG_TILE < nA + nB ? d0 + MG_TILE : nA + nB;
    if (tid < 2) split[tid] = merge_split<int64_t>(A, nA, B, nB, tid ? d1 : d0);
    __syncthreads();
    const int64_t i0 = split[0], j0 = d0 - i0;
    const int na = (int)(split[1] - i0), n = (int)(d1 - d0), nb = n - na;
    for (int i = tid; i < n; i += MG_NT) s[i] = i < na ? A[i0 + i] : B[j0 + (i - na)];
    __syncthreads();
    const int k0 = tid * MG_KPT < n ? tid * MG_KPT : n;
    int i = merge_split<int>(s, na, s + na, nb, k0), j = k0 - i;
#pragma unroll
    for (int r = 0; r < MG_KPT; ++r) {
        if (k0 + r < n) {
            const bool from_a = j >= nb || (i < na && s[i] < s[na + j]);
            dst[out0 + k0 + r] = from_a ? s[i] : s[na + j];
            i += from_a ? 1 : 0;
            j += from_a ? 0 : 1;
        }
    }
}

// Heads (first position of every id) among the sorted keys [blockIdx.x * MG_TILE, + MG_TILE): their number.
__device__ __forceinline__ int tile_heads(const uint64_t* __restrict__ keys, int64_t T, int64_t e0, uint32_t (&id)[MG_KPT],
                                          uint32_t (&pos)[MG_KPT], bool (&head)[MG_KPT]) {
    uint32_t before = e0 > 0 && e0 <= T ? (uint32_t)(keys[e0 - 1] >> 32) : 0u;
    int heads = 0;
#pragma unroll
    for (int r = 0; r < MG_KPT; ++r) {
        const int64_t e = e0 + r;
        const uint64_t k = e < T ? keys[e] : 0ull;
        id[r] = (uint32_t)(k >> 32);
        pos[r] = (uint32_t)k;
        head[r] = e < T && (e == 0 || before != id[r]);
        heads += head[r] ? 1 : 0;
        before = id[r];
    }
    return heads;
}

__device__ __forceinline__ int block_sum_int_256(int v, int32_t* red) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

__global__ __launch_bounds__(MG_NT) void emb_count_heads(const uint64_t* __restrict__ keys, int64_t T, int32_t* __restrict__ counts) {
    __shared__ int32_t red[4];
    uint32_t id[MG_KPT], pos[MG_KPT];
    bool head[MG_KPT];
    const int heads = tile_heads(keys, T, (int64_t)blockIdx.x * MG_TILE + (int64_t)threadIdx.x * MG_KPT, id, pos, head);
    const int total = block_sum_int_256(heads, red);
    if (threadIdx.x == 0) counts[blockIdx.x] = total;
}

__global__ __launch_bounds__(MG_NT) void emb_segments_tiled(const uint64_t* __restrict__ keys, int64_t T,
                                                            const int32_t* __restrict__ counts, int32_t* __restrict__ perm,
                                                            int32_t* __restrict__ unique_ids, int32_t* __restrict__ seg_offsets,
                                                            int32_t* __restrict__ n_unique) {
    __shared__ int32_t red[4], wsum[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int before_me = 0;
    for (int b = tid; b < (int)blockIdx.x; b += MG_NT) before_me += counts[b];
    const int base = block_sum_int_256(before_me, red);
    uint32_t id[MG_KPT], pos[MG_KPT];
    bool head[MG_KPT];
    const int64_t e0 = (int64_t)blockIdx.x * MG_TILE + (int64_t)tid * MG_KPT;
    const int heads = tile_heads(keys, T, e0, id, pos, head);
    int v = heads;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(v, off, 64);
        if (lane >= off) v += o;
    }
    if (lane == 63) wsum[wave] = v;
    __syncthreads();
    int waves_before = 0, total = 0;
    for (int w = 0; w < 4; ++w) {
        waves_before += w < wave ? wsum[w] : 0;
        total += wsum[w];
    }
    int idx = base + waves_before + v - heads;
#pragma unroll
    for (int r = 0; r < MG_KPT; ++r) {
        const int64_t e = e0 + r;
        if (e < T) perm[e] = (int32_t)pos[r];
        if (head[r]) {
            unique_ids[idx] = (int32_t)id[r];
            seg_offsets[idx] = (int32_t)e;
            ++idx;
        }
    }
    if (blockIdx.x == gridDim.x - 1 && tid == 0) {
        n_unique[0] = base + total;
        seg_offsets[base + total] = (int32_t)T;
    }
}

// Rows are summed in chunks of EMB_CHUNK sorted positions (one wave per chunk and 512-column slab).
constexpr int EMB_CHUNK = 16;
constexpr int EMB_COLS = 512;      // 64 lanes x 8 halves
constexpr int EMB_FIX_GX = 128;    // workgroups of the fix-up kernel along the segment axis (64 segments per trip)

static inline int64_t emb_chunks(int64_t T) { return (T + EMB_CHUNK - 1) / EMB_CHUNK; }
static inline int64_t emb_slabs(int64_t H) { return H > 0 ? (H + EMB_COLS - 1) / EMB_COLS : 1; }
static inline int64_t emb_chunk_blocks(int64_t T) { return (emb_chunks(T) + 3) / 4; }     // four waves per workgroup

static inline size_t emb_partials_bytes(int64_t T, int64_t H) {
    return align_up((size_t)(emb_chunk_blocks(T) + EMB_FIX_GX) * (size_t)emb_slabs(H) * sizeof(double), 256);
}

size_t embedding_ws_bytes(int64_t T, int64_t H) {
    if (T <= 0) return 0;
    const int64_t Tpad = next_pow2(T);
    size_t b = align_up((size_t)Tpad * 8, 256) * (T > GS_MAX ? 2 : 1);   // keys (+ the merge rounds' second buffer)
    b += align_up((size_t)T * 4, 256) * 2;         // perm, unique_ids
    b += align_up((size_t)(T + 1) * 4, 256);       // seg_offsets
    b += 256;                                      // n_unique
    b += emb_partials_bytes(T, H);                 // per-wave / per-workgroup shares of the squared norm
    b += align_up((size_t)emb_chunks(T) * 2 * (size_t)H * sizeof(float), 256);   // partial sums of runs that cross chunks
    return b;
}

// Bytes of the grouping part (keys, perm, unique ids, offsets, count): the head of the embedding workspace, which a
// step keeps from its norm pass to its update pass.
size_t embedding_grouping_bytes(int64_t T) {
    if (T <= 0) return 0;
    return align_up((size_t)next_pow2(T) * 8, 256) * (T > GS_MAX ? 2 : 1) + align_up((size_t)T * 4, 256) * 2 +
           align_up((size_t)(T + 1) * 4, 256) + 256;
}

EmbeddingWs carve_embedding_ws(void* ws, int64_t T, int64_t H) {
    EmbeddingWs w;
    char* p = static_cast<char*>(ws);
    const int64_t Tpad = next_pow2(T);
    w.keys = reinterpret_cast<uint64_t*>(p);
    p += align_up((size_t)Tpad * 8, 256);
    w.keys2 = nullptr;
    if (T > GS_MAX) {
        w.keys2 = reinterpret_cast<uint64_t*>(p);
        p += align_up((size_t)Tpad * 8, 256);
    }
    w.perm = reinterpret_cast<int32_t*>(p);
    p += align_up((size_t)T * 4, 256);
    w.unique_ids = reinterpret_cast<int32_t*>(p);
    p += align_up((size_t)T * 4, 256);
    w.seg_offsets = reinterpret_cast<int32_t*>(p);
    p += align_up((size_t)(T + 1) * 4, 256);
    w.n_unique = reinterpret_cast<int32_t*>(p);
    p += 256;
    w.partials = reinterpret_cast<double*>(p);
    p += emb_partials_bytes(T, H);
    w.chunk_rows = reinterpret_cast<float*>(p);
    return w;
}

hipError_t launch_embedding_grouping(const int32_t* ids, int64_t T, int64_t V, const EmbeddingWs& w, hipStream_t st) {
    int N = 0, shift = 0, id_bits = 0;
    if (group_small_plan(T, V, &N, &shift, &id_bits)) {
        hipLaunchKernelGGL(emb_group_small, dim3(1), dim3((unsigned)(N / GS_KPT)), 0, st, ids, (int)T, N, shift, id_bits,
                           w.perm, w.unique_ids, w.seg_offsets, w.n_unique);
        return hipGetLastError();
    }
    if (w.keys2 && group_chunks_plan(T, V, &id_bits)) {
        const int64_t chunks = (T + GS_MAX - 1) / GS_MAX;
        int rounds = 0;
        for (int64_t run = GS_MAX; run < T; run <<= 1) ++rounds;
        uint64_t* cur = (rounds & 1) ? w.keys2 : w.keys;      // after `rounds` exchanges the result is in w.keys
        uint64_t* other = (rounds & 1) ? w.keys : w.keys2;
        hipLaunchKernelGGL(emb_sort_chunks, dim3((unsigned)chunks), dim3(1024), 0, st, ids, T, id_bits, cur);
        const unsigned tiles = (unsigned)((T + MG_TILE - 1) / MG_TILE);
        for (int64_t run = GS_MAX; run < T; run <<= 1) {
            hipLaunchKernelGGL(emb_merge_round, dim3(tiles), dim3(MG_NT), 0, st, cur, other, T, run);
            uint64_t* t = cur;
            cur = other;
            other = t;
        }
        int32_t* counts = reinterpret_cast<int32_t*>(w.keys2);     // free again: one count per 2048 keys
        hipLaunchKernelGGL(emb_count_heads, dim3(tiles), dim3(MG_NT), 0, st, w.keys, T, counts);
        hipLaunchKernelGGL(emb_segments_tiled, dim3(tiles), dim3(MG_NT), 0, st, w.keys, T, counts, w.perm, w.unique_ids,
                           w.seg_offsets, w.n_unique);
        return hipGetLastError();
    }
    if (T == 0) {   // empty batch: zero segments
        hipLaunchKernelGGL(emb_segments, dim3(1), dim3(SORT_NT), 0, st, w.keys, T, w.perm, w.unique_ids, w.seg_offsets,
                           w.n_unique);
        return hipGetLastError();
    }
    const int64_t Tpad = next_pow2(T);
    hipLaunchKernelGGL(emb_make_keys, dim3((unsigned)((Tpad + 255) / 256)), dim3(256), 0, st, ids, T, Tpad, w.keys);
    const int64_t chunk = Tpad < SORT_CHUNK ? Tpad : SORT_CHUNK;
    const unsigned nblk = (unsigned)(Tpad / chunk);
    if (Tpad >= 2) {
        hipLaunchKernelGGL(emb_bitonic_local, dim3(nblk), dim3(SORT_NT), 0, st, w.keys, Tpad, (int64_t)2, chunk);
        for (int64_t k = chunk << 1; k <= Tpad; k <<= 1) {
            for (int64_t j = k >> 1; j >= chunk; j >>= 1)
                hipLaunchKernelGGL(emb_bitonic_global, dim3((unsigned)(((Tpad >> 1) + 255) / 256)), dim3(256), 0, st,
                                   w.keys, Tpad, k, j);
            hipLaunchKernelGGL(emb_bitonic_local, dim3(nblk), dim3(SORT_NT), 0, st, w.keys, Tpad, k, k);
        }
    }
    hipLaunchKernelGGL(emb_segments, dim3(1), dim3(SORT_NT), 0, st, w.keys, T, w.perm, w.unique_ids, w.seg_offsets,
                       w.n_unique);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Embedding rows: fp32 segment sums in a fixed order, independent of how skewed the token ids are.
//
// Pass A (emb_chunk_kernel): the sorted positions are cut into chunks of 16; one wave owns a chunk and a
// 512-column slab, requests its 16 rows at once and adds them in order.  A run of equal ids that lies inside
// the chunk is a whole segment and is finished on the spot (norm share or row update).  A run that reaches
// the chunk's first or last position and continues in the neighbouring chunk is stored as an fp32 partial row:
// slot 0 for the run that came from the previous chunk, slot 1 for the run that goes on into the next one.
// Pass B (emb_fixup_kernel): every segment that spans chunks adds its partial rows in chunk order (eight waves
// interleaved, then a fixed tree) and is finished.  The order of every sum depends on the ids alone.
// ------------------------------------------------------------------------------------------

constexpr int ROW_NT = 256;

__device__ __forceinline__ float block_sum_256(float v, float* red) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

// What happens to a finished segment sum g (8 columns of this lane): MODE 0 squared norm + overflow test,
// MODE 1 row update W <- rne16(W - s g), MODE 2 clip-by-value update (s = 1 / loss scale).
// `w`: the row's old 8 columns, loaded by the caller (update modes).
template <int MODE>
__device__ __forceinline__ void emb_finish_row(const float (&g)[8], uint16_t* __restrict__ W, int64_t row_off, bool active,
                                               float s, float lr, float clipv, float& sq, bool& bad, const half8& w) {
    if (MODE == 0) {
        uint32_t worst = 0u;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            sq = fmaf(g[e], g[e], sq);
            const uint32_t mag = __float_as_uint(g[e]) & 0x7fffffffu;
            worst = mag > worst ? mag : worst;
        }
        bad |= worst >= 0x7f800000u;
    } else if (active) {
        half8* p = reinterpret_cast<half8*>(W + row_off);
        half8 o;
        if (MODE == 1) {
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (_Float16)fmaf(-s, g[e], (float)w[e]);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float gq = g[e] * s;
                const bool fin = (__float_as_uint(gq) & 0x7f800000u) != 0x7f800000u;
                const float gc = fminf(fmaxf(gq, -clipv), clipv);
                o[e] = fin ? (_Float16)fmaf(-lr, gc, (float)w[e]) : w[e];
                bad |= !fin;
            }
        }
        *p = o;
    }
}

template <int MODE>
__global__ __launch_bounds__(ROW_NT) void emb_chunk_kernel(const int32_t* __restrict__ ids, const uint16_t* __restrict__ dY,
                                                           uint16_t* __restrict__ W, int T, int64_t H,
                                                           const int32_t* __restrict__ perm, float s,
                                                           float* __restrict__ chunk_rows, double* __restrict__ partials,
                                                           int32_t* __restrict__ flag_out, const int32_t* __restrict__ flag_in,
                                                           float lr, float clipv, const float* __restrict__ s_dev) {
    if (MODE == 1 && flag_in != nullptr && flag_in[0] != 0) return;
    if (MODE == 1 && s_dev != nullptr) s = s_dev[0];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // consecutive workgroups take the column slabs of the same four chunks: the pieces of a dY row are asked for at about
    // the same time, which the DRAM pages like better than slab after slab over the whole batch
    const int slabs = (int)((H + EMB_COLS - 1) / EMB_COLS);
    const int chunk = (int)(blockIdx.x / slabs) * 4 + wave;
    const int64_t col = (int64_t)(blockIdx.x % slabs) * EMB_COLS + lane * 8;
    const bool active = col < H;
    const int nchunks = (T + EMB_CHUNK - 1) / EMB_CHUNK;
    float sq = 0.f;
    bool bad = false;
    if (chunk < nchunks) {
        const int r0 = chunk * EMB_CHUNK;
        const int n = (T - r0 < EMB_CHUNK) ? (T - r0) : EMB_CHUNK;
        // lanes 0..17 look up (position, id) of the sorted entries r0 - 1 .. r0 + 16; -1 where there is none
        int myp = -1, myid = -1;
        {
            const int idx = r0 - 1 + lane;
            if (lane < EMB_CHUNK + 2 && idx >= 0 && idx < T) {
                myp = perm[idx];
                myid = ids[myp];
            }
        }
        // Which positions end a run that lies wholly inside the chunk (uniform): those runs are finished here, and in the
        // update modes their old rows are requested now, together with the dY rows, instead of one by one later.
        const int id_prev = __builtin_amdgcn_readlane(myid, 0);
        bool whole[EMB_CHUNK];
        {
            bool seen_end = false;
#pragma unroll
            for (int u = 0; u < EMB_CHUNK; ++u) {
                const int id_u = __builtin_amdgcn_readlane(myid, u + 1);
                const int id_n = __builtin_amdgcn_readlane(myid, u + 2);      // -1 past the end of the batch
                const bool end = u < n && (u == n - 1 || id_n != id_u);
                const bool from_prev = !seen_end && id_prev == id_u;
                const bool to_next = u == n - 1 && id_n == id_u;
                whole[u] = end && !from_prev && !to_next;
                seen_end |= end;
            }
        }
        half8 v[EMB_CHUNK];
#pragma unroll
        for (int u = 0; u < EMB_CHUNK; ++u) {
            const int p = __builtin_amdgcn_readlane(myp, u + 1);
            if (u < n && active) v[u] = *reinterpret_cast<const half8*>(dY + (int64_t)p * H + col);
        }
        half8 wold[EMB_CHUNK];
        if (MODE != 0) {
#pragma unroll
            for (int u = 0; u < EMB_CHUNK; ++u) {
                const int id_u = __builtin_amdgcn_readlane(myid, u + 1);
                if (whole[u] && active) wold[u] = *reinterpret_cast<const half8*>(W + (int64_t)id_u * H + col);
            }
        }
        float g[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) g[e] = 0.f;
        bool first = true;
#pragma unroll
        for (int u = 0; u < EMB_CHUNK; ++u) {
            if (u < n) {      // uniform
                if (active) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) g[e] += (float)v[u][e];
                }
                const int id_u = __builtin_amdgcn_readlane(myid, u + 1);
                const int id_n = __builtin_amdgcn_readlane(myid, u + 2);
                if (u == n - 1 || id_n != id_u) {                             // the run ends here
                    const bool from_prev = first && id_prev == id_u;
                    if (whole[u]) {
                        emb_finish_row<MODE>(g, W, (int64_t)id_u * H + col, active, s, lr, clipv, sq, bad, wold[u]);
                    } else if (active) {
                        float4* dst = reinterpret_cast<float4*>(chunk_rows + ((int64_t)chunk * 2 + (from_prev ? 0 : 1)) * H + col);
                        dst[0] = make_float4(g[0], g[1], g[2], g[3]);
                        dst[1] = make_float4(g[4], g[5], g[6], g[7]);
                    }
#pragma unroll
                    for (int e = 0; e < 8; ++e) g[e] = 0.f;
                    first = false;
                }
            }
        }
    }
    if (MODE == 0) {      // one share per workgroup: the four waves added in order
        __shared__ float red[4];
        const float total = block_sum_256(sq, red);
        if (threadIdx.x == 0) partials[blockIdx.x] = (double)total;
    }
    if (MODE != 1 && flag_out != nullptr && __any(bad) && lane == 0) atomicOr(flag_out, 1);
}

constexpr int EMB_NT = 512;     // 8 waves
constexpr int EMB_W = EMB_NT / 64;

template <int MODE>
__global__ __launch_bounds__(EMB_NT) void emb_fixup_kernel(const float* __restrict__ chunk_rows, uint16_t* __restrict__ W,
                                                           int64_t H, const int32_t* __restrict__ unique_ids,
                                                           const int32_t* __restrict__ seg_offsets,
                                                           const int32_t* __restrict__ n_unique, float s,
                                                           double* __restrict__ partials, int32_t* __restrict__ flag_out,
                                                           const int32_t* __restrict__ flag_in, float lr, float clipv,
                                                           const float* __restrict__ s_dev) {
    if (MODE == 1 && flag_in != nullptr && flag_in[0] != 0) return;
    if (MODE == 1 && s_dev != nullptr) s = s_dev[0];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t col = (int64_t)blockIdx.y * EMB_COLS + lane * 8;
    const bool active = col < H;
    const int nseg = n_unique[0];
    float sq = 0.f;
    bool bad = false;
    // 64 segments per trip: every lane looks at one segment's offsets, a ballot names those that span chunks, and the
    // spanning segments of the trip go to the eight waves in turn.  A wave adds its segment's partial rows in chunk order,
    // eight loads in flight, then finishes the row: no exchange between waves, and the order of every sum depends on the
    // ids alone.
    for (int base = blockIdx.x * 64; base < nseg; base += gridDim.x * 64) {
        int lbeg = 0, lend = 1;
        if (base + lane < nseg) {
            lbeg = seg_offsets[base + lane];
            lend = seg_offsets[base + lane + 1];
        }
        unsigned long long spanning = __ballot(lbeg / EMB_CHUNK != (lend - 1) / EMB_CHUNK);
        int turn = 0;
        while (spanning != 0ull) {        // uniform: every wave computed the same mask
            const int bit = __builtin_ctzll(spanning);
            spanning &= spanning - 1ull;
            if ((turn++ & (EMB_W - 1)) != wave) continue;
            const int seg = base + bit;
            const int beg = __shfl(lbeg, bit, 64), end = __shfl(lend, bit, 64);
            const int cf = beg / EMB_CHUNK, cl = (end - 1) / EMB_CHUNK;
            const int64_t row_off = (int64_t)unique_ids[seg] * H + col;
            half8 wold;
            if (MODE != 0 && active) wold = *reinterpret_cast<const half8*>(W + row_off);
            float g[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) g[e] = 0.f;
            if (active) {
                // the first chunk holds the segment's run in slot 1 (it goes on), every later chunk in slot 0
                auto row = [&](int c) { return chunk_rows + ((int64_t)c * 2 + (c == cf ? 1 : 0)) * H + col; };
                int c = cf;
                for (; c + 7 <= cl; c += 8) {
                    float4 a[8][2];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const float4* src = reinterpret_cast<const float4*>(row(c + u));
                        a[u][0] = src[0];
                        a[u][1] = src[1];
                    }
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        g[0] += a[u][0].x; g[1] += a[u][0].y; g[2] += a[u][0].z; g[3] += a[u][0].w;
                        g[4] += a[u][1].x; g[5] += a[u][1].y; g[6] += a[u][1].z; g[7] += a[u][1].w;
                    }
                }
                float4 t[7][2];
                const int left = cl - c + 1;        // 0 .. 7 (uniform)
#pragma unroll
                for (int u = 0; u < 7; ++u) {
                    if (u < left) {
                        const float4* src = reinterpret_cast<const float4*>(row(c + u));
                        t[u][0] = src[0];
                        t[u][1] = src[1];
                    }
                }
#pragma unroll
                for (int u = 0; u < 7; ++u) {
                    if (u < left) {
                        g[0] += t[u][0].x; g[1] += t[u][0].y; g[2] += t[u][0].z; g[3] += t[u][0].w;
                        g[4] += t[u][1].x; g[5] += t[u][1].y; g[6] += t[u][1].z; g[7] += t[u][1].w;
                    }
                }
            }
            emb_finish_row<MODE>(g, W, row_off, active, s, lr, clipv, sq, bad, wold);
        }
    }
    if (MODE != 1 && flag_out != nullptr && __any(bad) && lane == 0) atomicOr(flag_out, 1);
    if (MODE == 0) {      // one share per workgroup: its eight waves added in a fixed tree
        __shared__ float wsq[EMB_W];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) sq += __shfl_xor(sq, off, 64);
        if (lane == 0) wsq[wave] = sq;
        __syncthreads();
        if (threadIdx.x == 0) {
            const float total = ((wsq[0] + wsq[1]) + (wsq[2] + wsq[3])) + ((wsq[4] + wsq[5]) + (wsq[6] + wsq[7]));
            partials[(int64_t)blockIdx.y * gridDim.x + blockIdx.x] = (double)total;
        }
    }
}

// Adds the per-workgroup shares of both kernels in index order: the embedding's squared norm is bit-reproducible.  (A
// last-workgroup-to-arrive reduction inside the fix-up kernel was slower: hundreds of workgroups taking a ticket from one
// address serialise in the L2's atomic unit.)
__global__ __launch_bounds__(ROW_NT) void emb_finish_sqnorm(const double* __restrict__ partials, int n,
                                                            double* __restrict__ acc) {
    __shared__ double red[ROW_NT];
    double v = 0.0;
    int i = threadIdx.x;
    for (; i + 7 * ROW_NT < n; i += 8 * ROW_NT) {      // eight loads in flight; the order of the sum is fixed by this code
        double t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = partials[i + u * ROW_NT];
        v += ((t[0] + t[1]) + (t[2] + t[3])) + ((t[4] + t[5]) + (t[6] + t[7]));
    }
    for (; i < n; i += ROW_NT) v += partials[i];
    red[threadIdx.x] = v;
    __syncthreads();
    for (int off = ROW_NT / 2; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) atomicAdd(acc, red[0]);
}

hipError_t launch_embedding_rows(const int32_t* ids, const uint16_t* dY, uint16_t* W, int64_t T, int64_t H,
                                 const EmbeddingWs& w, int mode, float s, double* acc, int32_t* flag_out,
                                 const int32_t* flag_in, hipStream_t st, float lr, float clipv, const float* s_dev) {
    const dim3 gridA((unsigned)(emb_chunk_blocks(T) * emb_slabs(H)));
    const int64_t tripsB = (T + 63) / 64;
    const dim3 gridB((unsigned)(tripsB < EMB_FIX_GX ? tripsB : EMB_FIX_GX), (unsigned)emb_slabs(H));
    double* partB = w.partials + (int64_t)gridA.x;
#define LOMO_EMB_LAUNCH(M)                                                                                              \
    hipLaunchKernelGGL(emb_chunk_kernel<M>, gridA, dim3(ROW_NT), 0, st, ids, dY, W, (int)T, H, w.perm, s, w.chunk_rows, \
                       w.partials, flag_out, flag_in, lr, clipv, s_dev);                                                \
    hipLaunchKernelGGL(emb_fixup_kernel<M>, gridB, dim3(EMB_NT), 0, st, w.chunk_rows, W, H, w.unique_ids, w.seg_offsets, \
                       w.n_unique, s, partB, flag_out, flag_in, lr, clipv, s_dev);
    if (mode == 0) {
        LOMO_EMB_LAUNCH(0)
        hipLaunchKernelGGL(emb_finish_sqnorm, dim3(1), dim3(ROW_NT), 0, st, w.partials,
                           (int)(gridA.x + gridB.x * gridB.y), acc);
    } else if (mode == 1) {
        LOMO_EMB_LAUNCH(1)
    } else {
        LOMO_EMB_LAUNCH(2)
    }
#undef LOMO_EMB_LAUNCH
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// RMSNorm gain: g[j] = sum_t dY[t, j] * xhat[t, j].  Stage 1 writes fp32 partial column sums per
// row split, stage 2 adds the splits in order and finishes (norm or update).
// ------------------------------------------------------------------------------------------

constexpr int VEC_COLS = 512;       // columns per workgroup: 64 lanes x 8 halves = 1 KiB per row and wave
constexpr int VEC_NT = 512;         // 8 waves
constexpr int VEC_W = VEC_NT / 64;
constexpr int VEC_U = 8;            // rows a wave has in flight: 16 independent 16-byte loads per lane
constexpr int VEC_BLOCK = VEC_W * VEC_U;   // rows a workgroup consumes per iteration
constexpr int VEC_MAX_SPLITS = 128;

static inline int vector_splits(int64_t T) {
    int64_t s = (T + VEC_BLOCK - 1) / VEC_BLOCK;
    if (s < 1) s = 1;
    if (s > VEC_MAX_SPLITS) s = VEC_MAX_SPLITS;
    return (int)s;
}

size_t vector_ws_bytes(int64_t T, int64_t H) {
    if (T <= 0 || H <= 0) return 0;
    return align_up((size_t)vector_splits(T) * (size_t)H * sizeof(float), 256);
}

// Stage 1.  Workgroup (slab, split) sums rows [t0, t1) of its 512-column slab.  Per iteration every wave
// takes eight consecutive rows and issues all sixteen loads before using any, so a CU keeps about
// 256 KiB in flight; a wave adds its rows in ascending order, the eight waves are then added in a
// fixed tree: the result depends on T and H only, not on scheduling.
// blockIdx.z selects the gain vector of the batch; its partial sums follow those of the vectors before it.
__global__ __launch_bounds__(VEC_NT) void vec_partial_kernel(VecBatch batch, int64_t T, int64_t H,
                                                             int splits, float* __restrict__ partial) {
    __shared__ float part[VEC_W - 1][64][9];
    const uint16_t* __restrict__ Xh = batch.Xh[blockIdx.z];
    const uint16_t* __restrict__ dY = batch.dY[blockIdx.z];
    partial += (int64_t)blockIdx.z * splits * H;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t col = (int64_t)blockIdx.x * VEC_COLS + lane * 8;
    const bool active = col < H;
    const int split = blockIdx.y;
    int64_t rows_per = (T + splits - 1) / splits;
    rows_per = (rows_per + VEC_BLOCK - 1) / VEC_BLOCK * VEC_BLOCK;
    const int64_t t0 = (int64_t)split * rows_per;
    const int64_t t1 = (t0 + rows_per < T) ? (t0 + rows_per) : T;
    float g[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) g[e] = 0.f;
    if (active) {
        int64_t base = t0 + wave * VEC_U;
        for (; base + VEC_U <= t1; base += VEC_BLOCK) {          // eight whole rows: no per-row test
            half8 a[VEC_U], b[VEC_U];
#pragma unroll
            for (int u = 0; u < VEC_U; ++u) {
                a[u] = *reinterpret_cast<const half8*>(Xh + (base + u) * H + col);
                b[u] = *reinterpret_cast<const half8*>(dY + (base + u) * H + col);
            }
#pragma unroll
            for (int u = 0; u < VEC_U; ++u)
#pragma unroll
                for (int e = 0; e < 8; ++e) g[e] = fmaf((float)a[u][e], (float)b[u][e], g[e]);
        }
        for (int64_t t = base; t < t1 && t < base + VEC_U; ++t) {   // ragged end of the split
            const half8 a = *reinterpret_cast<const half8*>(Xh + t * H + col);
            const half8 b = *reinterpret_cast<const half8*>(dY + t * H + col);
#pragma unroll
            for (int e = 0; e < 8; ++e) g[e] = fmaf((float)a[e], (float)b[e], g[e]);
        }
    }
    if (wave > 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) part[wave - 1][lane][e] = g[e];
    }
    __syncthreads();
    if (wave == 0 && active) {
        float4 lo, hi;
        float o[8];
#pragma unroll
        for (int e = 0; e < 8; ++e)
            o[e] = ((g[e] + part[0][lane][e]) + (part[1][lane][e] + part[2][lane][e])) +
                   ((part[3][lane][e] + part[4][lane][e]) + (part[5][lane][e] + part[6][lane][e]));
        lo = make_float4(o[0], o[1], o[2], o[3]);
        hi = make_float4(o[4], o[5], o[6], o[7]);
        float4* dst = reinterpret_cast<float4*>(partial + (int64_t)split * H + col);
        dst[0] = lo;
        dst[1] = hi;
    }
}

// Stage 2.  A workgroup finishes 128 columns: eight groups of 32 lanes take the splits round-robin
// (group q: splits q, q + 8, ...), four columns per lane, every load independent of the others; the
// eight group sums are then added in a fixed tree.  Then the squared norm or the update.
constexpr int FIN_COLS = 128;
constexpr int FIN_GROUPS = ROW_NT / 32;

template <int MODE>
__global__ __launch_bounds__(ROW_NT) void vec_finish_kernel(VecBatch batch, const float* __restrict__ partial, int64_t H,
                                                            int splits, float s, double* __restrict__ acc,
                                                            const int32_t* __restrict__ flag_in, float lr, float clipv,
                                                            const float* __restrict__ s_dev) {
    __shared__ float4 part[FIN_GROUPS - 1][32];
    __shared__ float red[4];
    __shared__ int redflag[4];
    if (MODE == 1 && flag_in != nullptr && flag_in[0] != 0) return;
    if (MODE == 1 && s_dev != nullptr) s = s_dev[0];
    uint16_t* __restrict__ w = batch.w[blockIdx.y];
    int32_t* __restrict__ flag_out = batch.flag_out[blockIdx.y];
    partial += (int64_t)blockIdx.y * splits * H;
    const int c4 = threadIdx.x & 31, grp = threadIdx.x >> 5;
    const int64_t j = (int64_t)blockIdx.x * FIN_COLS + c4 * 4;
    const bool active = j < H;                     // H is a multiple of 8: four whole columns or none
    float4 g = make_float4(0.f, 0.f, 0.f, 0.f);
    if (active) {
        int sp = grp;
        for (; sp + 3 * FIN_GROUPS < splits; sp += 4 * FIN_GROUPS) {
            float4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                v[u] = *reinterpret_cast<const float4*>(partial + (int64_t)(sp + u * FIN_GROUPS) * H + j);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                g.x += v[u].x; g.y += v[u].y; g.z += v[u].z; g.w += v[u].w;
            }
        }
        for (; sp < splits; sp += FIN_GROUPS) {
            const float4 v = *reinterpret_cast<const float4*>(partial + (int64_t)sp * H + j);
            g.x += v.x; g.y += v.y; g.z += v.z; g.w += v.w;
        }
    }
    if (grp > 0) part[grp - 1][c4] = g;
    __syncthreads();
    float gs[4] = {0.f, 0.f, 0.f, 0.f};
    if (grp == 0) {
        const float4 p0 = part[0][c4], p1 = part[1][c4], p2 = part[2][c4], p3 = part[3][c4], p4 = part[4][c4],
                     p5 = part[5][c4], p6 = part[6][c4];
        gs[0] = ((g.x + p0.x) + (p1.x + p2.x)) + ((p3.x + p4.x) + (p5.x + p6.x));
        gs[1] = ((g.y + p0.y) + (p1.y + p2.y)) + ((p3.y + p4.y) + (p5.y + p6.y));
        gs[2] = ((g.z + p0.z) + (p1.z + p2.z)) + ((p3.z + p4.z) + (p5.z + p6.z));
        gs[3] = ((g.w + p0.w) + (p1.w + p2.w)) + ((p3.w + p4.w) + (p5.w + p6.w));
    }
    if (MODE == 0) {
        float sq = 0.f;
        bool badv = false;
        if (grp == 0 && active) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                sq = fmaf(gs[e], gs[e], sq);
                badv |= (__float_as_uint(gs[e]) & 0x7fffffffu) >= 0x7f800000u;
            }
        }
        const bool bad = __any(badv);
        if ((threadIdx.x & 63) == 0) redflag[threadIdx.x >> 6] = bad ? 1 : 0;
        const float total = block_sum_256(sq, red);
        if (threadIdx.x == 0) {
            atomicAdd(acc, (double)total);
            if (flag_out != nullptr && (redflag[0] | redflag[1] | redflag[2] | redflag[3])) atomicOr(flag_out, 1);
        }
    } else if (grp == 0 && active) {
        half4 old = *reinterpret_cast<const half4*>(w + j);
        bool badv = false;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (MODE == 1) {
                old[e] = (_Float16)fmaf(-s, gs[e], (float)old[e]);
            } else {   // clip by value: s is 1 / loss scale here
                const float gq = gs[e] * s;
                if ((__float_as_uint(gq) & 0x7f800000u) != 0x7f800000u)
                    old[e] = (_Float16)fmaf(-lr, fminf(fmaxf(gq, -clipv), clipv), (float)old[e]);
                else
                    badv = true;
            }
        }
        *reinterpret_cast<half4*>(w + j) = old;
        if (MODE == 2 && badv && flag_out != nullptr) atomicOr(flag_out, 1);
    }
}

// Vectors of one shape, as many per launch pair as the workspace holds partial sums for (at most VEC_BATCH).
hipError_t launch_vector_batch(const VecItem* items, int n, int64_t T, int64_t H, void* ws, size_t ws_bytes, int mode,
                               float s, double* acc, const int32_t* flag_in, hipStream_t st, float lr, float clipv,
                               const float* s_dev) {
    const int splits = vector_splits(T);
    const size_t per = vector_ws_bytes(T, H);
    int64_t cap = per > 0 ? (int64_t)(ws_bytes / per) : 0;
    if (cap < 1) return hipErrorInvalidValue;
    if (cap > VEC_BATCH) cap = VEC_BATCH;
    float* partial = static_cast<float*>(ws);
    for (int first = 0; first < n; first += (int)cap) {
        const int cnt = (n - first < (int)cap) ? (n - first) : (int)cap;
        VecBatch b{};
        for (int i = 0; i < cnt; ++i) {
            b.Xh[i] = items[first + i].Xhat;
            b.dY[i] = items[first + i].dY;
            b.w[i] = items[first + i].w;
            b.flag_out[i] = items[first + i].flag_out;
        }
        hipLaunchKernelGGL(vec_partial_kernel, dim3((unsigned)((H + VEC_COLS - 1) / VEC_COLS), (unsigned)splits, (unsigned)cnt),
                           dim3(VEC_NT), 0, st, b, T, H, splits, partial);
        const dim3 grid((unsigned)((H + FIN_COLS - 1) / FIN_COLS), (unsigned)cnt);
        if (mode == 0)
            hipLaunchKernelGGL(vec_finish_kernel<0>, grid, dim3(ROW_NT), 0, st, b, partial, H, splits, s, acc, flag_in, lr,
                               clipv, s_dev);
        else if (mode == 1)
            hipLaunchKernelGGL(vec_finish_kernel<1>, grid, dim3(ROW_NT), 0, st, b, partial, H, splits, s, acc, flag_in, lr,
                               clipv, s_dev);
        else
            hipLaunchKernelGGL(vec_finish_kernel<2>, grid, dim3(ROW_NT), 0, st, b, partial, H, splits, s, acc, flag_in, lr,
                               clipv, s_dev);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_vector(const uint16_t* Xhat, const uint16_t* dY, uint16_t* w, int64_t T, int64_t H, void* ws, int mode,
                         float s, double* acc, int32_t* flag_out, const int32_t* flag_in, hipStream_t st, float lr,
                         float clipv, const float* s_dev) {
    const VecItem one{Xhat, dY, w, flag_out};
    return launch_vector_batch(&one, 1, T, H, ws, vector_ws_bytes(T, H), mode, s, acc, flag_in, st, lr, clipv, s_dev);
}

// ------------------------------------------------------------------------------------------

// Clipping coefficient of the step on the device (section 3.3.1 with the loss scale of section 3.3.2):
// norm = sqrt(acc) / S, clip = min(1, max_norm / (norm + eps)), step = lr * clip / S in double, rounded
// once to float.  An overflowed or non-finite step gets clip = step = 0.
__global__ void step_scalars_kernel(const double* __restrict__ acc, const int32_t* __restrict__ step_flag,
                                    double loss_scale, double max_norm, double eps, double lr,
                                    lomo_step_scalars* __restrict__ out) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const int overflow = (step_flag != nullptr && step_flag[0] != 0) ? 1 : 0;
    const double norm = sqrt(acc[0]) / loss_scale;
    double clip = 0.0;
    if (!overflow && norm == norm && norm - norm == 0.0) {      // finite
        const double c = max_norm / (norm + eps);
        clip = c < 1.0 ? c : 1.0;
    }
    out->clip_coef = clip;
    out->grad_norm = norm;
    out->step = (float)(lr * clip / loss_scale);
    out->overflow = overflow;
}

hipError_t launch_step_scalars(const double* acc, const int32_t* step_flag, double loss_scale, double max_norm, double eps,
                               double lr, lomo_step_scalars* out, hipStream_t st) {
    hipLaunchKernelGGL(step_scalars_kernel, dim3(1), dim3(64), 0, st, acc, step_flag, loss_scale, max_norm, eps, lr, out);
    return hipGetLastError();
}

__global__ void reduce_flags_kernel(const int32_t* __restrict__ flags, int64_t n, int32_t* __restrict__ out) {
    __shared__ int any_s;
    if (threadIdx.x == 0) any_s = 0;
    __syncthreads();
    int mine = 0;
    for (int64_t i = threadIdx.x; i < n; i += blockDim.x) mine |= (flags[i] != 0);
    if (mine) any_s = 1;   // benign: every writer stores the same value
    __syncthreads();
    if (threadIdx.x == 0) out[0] = any_s;
}

hipError_t launch_reduce_flags(const int32_t* flags, int64_t n, int32_t* out, hipStream_t st) {
    hipLaunchKernelGGL(reduce_flags_kernel, dim3(1), dim3(256), 0, st, flags, n, out);
    return hipGetLastError();
}

}  // namespace lomo

// Measured ceilings for the roofline denominators (benchmark aids, not part of the method): what the chip
// sustains on its matrix cores when nothing else runs, and on a plain streaming copy.  The contraction
// kernels' TFLOP/s are reported next to these, because the rate the matrix cores hold depends on the operand
// data (power management): zeros and normally distributed values give very different figures.
#include "lomo.h"
#include "lomo_kernels.h"

namespace lomo {

typedef _Float16 probe_half8 __attribute__((ext_vector_type(8)));
typedef float probe_floatx16 __attribute__((ext_vector_type(16)));

// Every wave: 2 sets x (4 A + 4 B) fragments in registers, NI x NJ accumulators of 32 x 32; per iteration
// 2 x NI x NJ MFMAs in the order of the contraction kernels' half-slices (A fragment outer, B fragment inner).
// No LDS, no global memory inside the loop.  4 x 4 with one wave per SIMD is the contraction kernels' blocking
// (256 accumulator registers); two waves per SIMD have 256 registers each, hence 4 x 2.
//   idle:      after each iteration the wave sleeps `idle` x 64 clocks (duty cycle below one: does the chip clock
//              higher when the matrix pipes are not saturated, i.e. is the rate set by power or by a fixed clock?)
//   LDS_READS: every operand set is re-read from LDS before it is used (sixteen 16-byte reads per lane and
//              iteration: the LDS read traffic of the contraction kernels, without their global loads)
template <int NI, int NJ, int THREADS, bool LDS_READS>
__global__ __launch_bounds__(THREADS) void probe_mfma_kernel(const uint16_t* __restrict__ operands, int64_t iters, int idle,
                                                             float* __restrict__ sink) {
    __shared__ __attribute__((aligned(16))) uint16_t lds[LOMO_PROBE_OPERAND_BYTES / 2];
    const int lane = threadIdx.x & 63;
    probe_half8 a[2][4], b[2][4];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            a[s][i] = *reinterpret_cast<const probe_half8*>(operands + ((s * 8 + i) * 64 + lane) * 8);
            b[s][i] = *reinterpret_cast<const probe_half8*>(operands + ((s * 8 + 4 + i) * 64 + lane) * 8);
        }
    if (LDS_READS) {
        for (int i = threadIdx.x; i < LOMO_PROBE_OPERAND_BYTES / 16; i += THREADS)
            reinterpret_cast<probe_half8*>(lds)[i] = reinterpret_cast<const probe_half8*>(operands)[i];
        __syncthreads();
    }
    // 16-byte LDS read that the compiler can neither hoist nor drop
    auto lds_frag = [&](int frag) {
        probe_half8 v;
        const uint32_t addr = (uint32_t)(uintptr_t)(lds + (frag * 64 + lane) * 8);
        asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr) : "memory");
        return v;
    };
    probe_floatx16 acc[NI][NJ];
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    for (int64_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            if (LDS_READS) {      // the other set is fetched while this one is multiplied
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    a[s ^ 1][i] = lds_frag((s ^ 1) * 8 + i);
                    b[s ^ 1][i] = lds_frag((s ^ 1) * 8 + 4 + i);
                }
            }
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[s][i], b[s][j], acc[i][j], 0, 0, 0);
            if (LDS_READS) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
        for (int k = 0; k < idle; ++k) __builtin_amdgcn_s_sleep(1);
    }
    float v = 0.f;
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) v += acc[i][j][r];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    if (lane == 0) atomicAdd(sink + blockIdx.x, v);
}

// Streaming copy: every thread keeps eight independent 16-byte loads in flight; loads and stores carry the
// non-temporal hint (the data is touched once).
typedef uint32_t probe_u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void probe_copy_kernel(const probe_u32x4* __restrict__ src, probe_u32x4* __restrict__ dst, int64_t n16) {
    constexpr int U = 8;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + (U - 1) * stride < n16; i += U * stride) {
        probe_u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < U; ++u) __builtin_nontemporal_store(v[u], dst + i + u * stride);
    }
    for (; i < n16; i += stride) dst[i] = src[i];
}

static int probe_cu_count() {
    static const int n = [] {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 256;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) return 256;
        return v;
    }();
    return n;
}

}  // namespace lomo

using namespace lomo;

extern "C" {

lomo_status lomo_probe_mfma(const lomo_half* operands, int64_t iters, int waves_per_simd, int idle_sleeps, int lds_reads,
                            float* sink, int64_t sink_len, double* flops_out, void* stream) {
    if (iters < 0 || (waves_per_simd != 1 && waves_per_simd != 2) || idle_sleeps < 0 || idle_sleeps > 4096) return LOMO_ERR_SHAPE;
    if (!operands || !sink) return LOMO_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(operands) & 15u) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return LOMO_ERR_ALIGN;
    const int cus = probe_cu_count();
    if (sink_len < cus) return LOMO_ERR_WORKSPACE;
    const int threads = 256 * waves_per_simd;
    const double mfmas_per_iter = waves_per_simd == 1 ? 32.0 : 16.0;
    if (flops_out) *flops_out = (double)cus * (threads / 64) * (double)iters * mfmas_per_iter * (2.0 * 32 * 32 * 16);
    if (iters == 0) return LOMO_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e;
    const dim3 grid((unsigned)cus);
    if (waves_per_simd == 1 && !lds_reads)
        e = launch_timed(LOMO_KERNEL_PROBE, probe_mfma_kernel<4, 4, 256, false>, grid, dim3(256), 0, st, operands, iters, idle_sleeps, sink);
    else if (waves_per_simd == 1)
        e = launch_timed(LOMO_KERNEL_PROBE, probe_mfma_kernel<4, 4, 256, true>, grid, dim3(256), 0, st, operands, iters, idle_sleeps, sink);
    else if (!lds_reads)
        e = launch_timed(LOMO_KERNEL_PROBE, probe_mfma_kernel<4, 2, 512, false>, grid, dim3(512), 0, st, operands, iters, idle_sleeps, sink);
    else
        e = launch_timed(LOMO_KERNEL_PROBE, probe_mfma_kernel<4, 2, 512, true>, grid, dim3(512), 0, st, operands, iters, idle_sleeps, sink);
    return e == hipSuccess ? LOMO_OK : LOMO_ERR_LAUNCH;
}

lomo_status lomo_probe_copy(const void* src, void* dst, size_t bytes, void* stream) {
    if (bytes & 15u) return LOMO_ERR_SHAPE;
    if (bytes == 0) return LOMO_OK;
    if (!src || !dst) return LOMO_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(dst) & 15u)) return LOMO_ERR_ALIGN;
    const int64_t n16 = (int64_t)(bytes >> 4);
    int64_t blocks = (n16 + 8 * 256 - 1) / (8 * 256);
    const int64_t cap = (int64_t)probe_cu_count() * 32;
    if (blocks > cap) blocks = cap;
    return launch_timed(LOMO_KERNEL_PROBE, probe_copy_kernel, dim3((unsigned)blocks), dim3(256), 0,
                        static_cast<hipStream_t>(stream), static_cast<const probe_u32x4*>(src), static_cast<probe_u32x4*>(dst), n16) ==
                   hipSuccess
               ? LOMO_OK
               : LOMO_ERR_LAUNCH;
}

}  // extern "C"

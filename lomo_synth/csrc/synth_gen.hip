// Device twin of the counter-based input generator (lomo_synth/generators.py): fills an fp16
// buffer with Irwin-Hall(12) normals from SplitMix64 words.  Input generation only -- no part of
// the LOMO method is computed here.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

__device__ __forceinline__ uint64_t mix(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__global__ void normal_f16_kernel(uint64_t key, int64_t first, int64_t n, float mult, _Float16* __restrict__ out) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const uint64_t base = (uint64_t)(first + i) * 3ull;
        int32_t s = 0;
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            const uint64_t w = mix(key + (base + (uint64_t)j + 1ull) * 0x9E3779B97F4A7C15ull);
            s += (int32_t)(w & 0xFFFF) + (int32_t)((w >> 16) & 0xFFFF) + (int32_t)((w >> 32) & 0xFFFF) +
                 (int32_t)((w >> 48) & 0xFFFF);
        }
        float p = (float)(s - 6 * 65535) * mult;   // one fp32 multiply ...
        asm volatile("" : "+v"(p));                // ... kept as an fp32 value (no fused multiply-convert)
        out[i] = (_Float16)p;                      // ... then one RNE to fp16, as the CPU recipe does
    }
}

}  // namespace

extern "C" int synth_normal_f16(uint64_t key, int64_t first, int64_t n, float mult, void* out, void* stream) {
    if (n <= 0) return 0;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(normal_f16_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream), key,
                       first, n, mult, static_cast<_Float16*>(out));
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

// Diagnostic kernel: what dense bf16 MFMA rate does this GPU sustain when nothing but MFMAs run?
//
// The published peak assumes the boost clock.  Under a full matrix load the chip is power-limited and the
// clock it settles at depends on how many operand bits toggle: with constant operands the clock stays near
// the boost clock, with random mantissas and signs it drops by about a third.  The attention kernel's rate is
// to be read against the random-operand figure of this probe as well as against the published peak.
#include "kernels.h"

namespace ll {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// Each wave issues iters * 16 MFMAs 32x32x16 back to back (four independent accumulators), two waves per SIMD.
// counters[0] += core clocks, counters[1] += 100 MHz reference ticks spent in the loop by wave 0 of workgroup 0.
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void ll_probe_mfma_kernel(float* sink, unsigned long long* counters, int iters, int random_operands) {
    u32x4 a[8], b[8];
    unsigned x = (blockIdx.x * 512u + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            x = x * 1664525u + 1013904223u;
            const unsigned ra = x ^ (x >> 13);
            x = x * 1664525u + 1013904223u;
            const unsigned rb = x ^ (x >> 13);
            // bf16 pairs in [0.5, 1) with random mantissas and signs, or all 1.0
            a[i][j] = random_operands ? ((ra & 0x807F807Fu) | 0x3F003F00u) : 0x3F803F80u;
            b[i][j] = random_operands ? ((rb & 0x807F807Fu) | 0x3F003F00u) : 0x3F803F80u;
        }
    f32x16 o[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[j][r] = 0.f;
    const unsigned long long c0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < 16; ++k)
            o[k % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[k % 8]),
                                                               __builtin_bit_cast(bf16x8, b[(k * 3 + 1) % 8]), o[k % 4], 0, 0, 0);
        if ((it & 63) == 63) {
#pragma unroll
            for (int j = 0; j < 4; ++j) o[j] *= 1e-3f;      // keep the accumulators finite
        }
    }
    const unsigned long long c1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        counters[0] = c1 - c0;
        counters[1] = r1 - r0;
    }
    f32x16 cs = o[0] + o[1] + o[2] + o[3];
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 16; ++j) s += cs[j];
    sink[blockIdx.x * 512 + threadIdx.x] = s;
}

hipError_t launch_probe_mfma(float* sink, unsigned long long* counters, int workgroups, int iters, int random_operands,
                             hipStream_t s) {
    hipLaunchKernelGGL(ll_probe_mfma_kernel, dim3(workgroups), dim3(512), 0, s, sink, counters, iters, random_operands);
    return hipGetLastError();
}

}  // namespace ll

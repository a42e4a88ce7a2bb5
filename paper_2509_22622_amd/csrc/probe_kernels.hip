// Diagnostic kernels: what dense bf16 MFMA rate does this GPU sustain, alone and with company?
//
// The published peak assumes the boost clock.  Under a full matrix load the chip is power-limited and the
// clock it settles at depends on how many operand bits toggle: with constant operands the clock stays near
// the boost clock, with random mantissas and signs it drops by about a third.  The attention kernel's rate is
// to be read against the random-operand figure of this probe as well as against the published peak.
//
// The same loop with a few vector or LDS instructions issued behind every MFMA shows what that company costs in
// matrix throughput (issue slots at constant operands, issue slots and power at random ones): the numbers
// behind the attention kernel's choice of instructions.
#include "kernels.h"

namespace ll {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));

// companion instruction kinds (PROBE_* in kernels.h).  Each works on registers no MFMA touches.
template <int KIND>
__device__ __forceinline__ void probe_companion(float& x, float c, u32x4& frag, unsigned lds_addr) {
    if (KIND == PROBE_ADD) asm volatile("v_add_f32 %0, %0, %1" : "+v"(x) : "v"(c));
    if (KIND == PROBE_EXP) asm volatile("v_exp_f32 %0, %0" : "+v"(x));
    if (KIND == PROBE_CVT_BF16) asm volatile("v_cvt_pk_bf16_f32 %0, %0, %1" : "+v"(x) : "v"(c));
    if (KIND == PROBE_DOT2_BF16) asm volatile("v_dot2c_f32_bf16 %0, %1, %1" : "+v"(x) : "v"(c));
    if (KIND == PROBE_MAX3) asm volatile("v_max3_f32 %0, %0, %1, %1" : "+v"(x) : "v"(c));
    if (KIND == PROBE_LDS_READ) asm volatile("ds_read_b128 %0, %1" : "=v"(frag) : "v"(lds_addr));
}
// What the 8-bit attention kernel issues per fp8 MFMA, on registers no MFMA touches: the vector part (4 exp2, 4 adds,
// 2 conversions to E4M3, 2 max3) and the LDS part (two 16-byte reads).
template <int KIND>
__device__ __forceinline__ void probe_fp8_company(float (&x)[4], float c, u32x4& frag, unsigned lds_addr) {
    if (KIND == PROBE_FP8_MIX || KIND == PROBE_FP8_VALU) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            asm volatile("v_exp_f32 %0, %0" : "+v"(x[i]));
            asm volatile("v_add_f32 %0, %0, %1" : "+v"(x[i]) : "v"(c));
        }
        unsigned w = 0;
        asm volatile("v_cvt_pk_fp8_f32 %0, %1, %2" : "+v"(w) : "v"(x[0]), "v"(x[1]));
        asm volatile("v_cvt_pk_fp8_f32 %0, %1, %2 op_sel:[0,0,1]" : "+v"(w) : "v"(x[2]), "v"(x[3]));
        asm volatile("v_max3_f32 %0, %0, %1, %2" : "+v"(x[0]) : "v"(c), "v"(w));
        asm volatile("v_max3_f32 %0, %0, %1, %1" : "+v"(x[1]) : "v"(c));
    }
    if (KIND == PROBE_FP8_MIX || KIND == PROBE_FP8_LDS) {
        asm volatile("ds_read_b128 %0, %1" : "=v"(frag) : "v"(lds_addr));
        asm volatile("ds_read_b128 %0, %1 offset:1024" : "=v"(frag) : "v"(lds_addr));
    }
}

// Each wave issues iters * 16 MFMAs 32x32x16 (or iters * 32 MFMAs 16x16x32: the same flops; or iters * 16 fp8 MFMAs
// 32x32x64: four times the flops) back to back, four (eight) independent accumulators, two waves per SIMD, PER
// companion instructions behind each MFMA.
// counters[0] = core clocks, counters[1] = 100 MHz reference ticks spent in the loop by wave 0 of workgroup 0.
template <int KIND, int PER>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void ll_probe_mfma_kernel(float* sink, unsigned long long* counters, int iters, int random_operands) {
    constexpr bool FP8 = KIND >= PROBE_FP8_NONE;
    constexpr bool USES_LDS = KIND == PROBE_LDS_READ || KIND == PROBE_FP8_MIX || KIND == PROBE_FP8_LDS;
    __shared__ __attribute__((aligned(16))) unsigned lds[USES_LDS ? 16384 : 4];
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
            // bf16 pairs (E4M3 bytes for the fp8 kinds) in [0.5, 1) with random mantissas and signs, or all 1.0
            if (FP8) {
                a[i][j] = random_operands ? ((ra & 0x87878787u) | 0x30303030u) : 0x38383838u;
                b[i][j] = random_operands ? ((rb & 0x87878787u) | 0x30303030u) : 0x38383838u;
            } else {
                a[i][j] = random_operands ? ((ra & 0x807F807Fu) | 0x3F003F00u) : 0x3F803F80u;
                b[i][j] = random_operands ? ((rb & 0x807F807Fu) | 0x3F003F00u) : 0x3F803F80u;
            }
        }
    if (USES_LDS) {
        for (int i = threadIdx.x; i < 16384; i += 512) {
            x = x * 1664525u + 1013904223u;
            lds[i] = random_operands ? x : 0x3F803F80u;
        }
        __syncthreads();
    }
    const unsigned lds_addr = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned*)lds + (threadIdx.x & 63) * 16;
    f32x16 o[4];
    f32x4 o4[8];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[j][r] = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) o4[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    constexpr int NV = FP8 ? 64 : 16 * PER;
    float v[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) v[i] = -0.5f - 0.001f * i - 1e-5f * threadIdx.x;
    i32x8 a8[4], b8[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            a8[i][j] = int(a[2 * i][j]); a8[i][4 + j] = int(a[2 * i + 1][j]);
            b8[i][j] = int(b[2 * i][j]); b8[i][4 + j] = int(b[2 * i + 1][j]);
        }
    u32x4 frag = {0, 0, 0, 0};
    const unsigned long long c0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            if (FP8) {
                o[k % 4] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8[k % 4], b8[(k * 3 + 1) % 4], o[k % 4], 0, 0, 0,
                                                                           0x7F7F7F7F, 0, 0x7F7F7F7F);
                float(&x4)[4] = *reinterpret_cast<float(*)[4]>(&v[4 * k]);
                probe_fp8_company<KIND>(x4, 0.999f, frag, lds_addr + (k & 7) * 2048);
            } else if (KIND == PROBE_SHAPE_16X16X32) {
                o4[(2 * k) % 8] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[k % 8]),
                                      __builtin_bit_cast(bf16x8, b[(k * 3 + 1) % 8]), o4[(2 * k) % 8], 0, 0, 0);
                o4[(2 * k + 1) % 8] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[k % 8]),
                                          __builtin_bit_cast(bf16x8, b[(k * 3 + 2) % 8]), o4[(2 * k + 1) % 8], 0, 0, 0);
            } else {
                o[k % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[k % 8]),
                               __builtin_bit_cast(bf16x8, b[(k * 3 + 1) % 8]), o[k % 4], 0, 0, 0);
            }
            if (!FP8) {
#pragma unroll
                for (int r = 0; r < PER; ++r) probe_companion<KIND>(v[k * PER + r], 0.999f, frag, lds_addr + ((k * PER + r) & 15) * 1024);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (USES_LDS) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(frag));
        if ((it & 63) == 63) {
#pragma unroll
            for (int j = 0; j < 4; ++j) o[j] *= 1e-3f;      // keep the accumulators finite
#pragma unroll
            for (int j = 0; j < 8; ++j) o4[j] *= 1e-3f;
        }
    }
    const unsigned long long c1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        counters[0] = c1 - c0;
        counters[1] = r1 - r0;
    }
    f32x16 cs = o[0] + o[1] + o[2] + o[3];
    f32x4 c4 = o4[0] + o4[1] + o4[2] + o4[3] + o4[4] + o4[5] + o4[6] + o4[7];
    float s = c4[0] + c4[1] + c4[2] + c4[3] + __uint_as_float(frag[0] & 0x007FFFFFu);
#pragma unroll
    for (int j = 0; j < 16; ++j) s += cs[j];
#pragma unroll
    for (int i = 0; i < NV; ++i) s += v[i];
    sink[blockIdx.x * 512 + threadIdx.x] = s;
}

template <int KIND, int PER>
static hipError_t launch_probe(float* sink, unsigned long long* counters, int workgroups, int iters, int random_operands,
                               hipStream_t s) {
    hipLaunchKernelGGL((ll_probe_mfma_kernel<KIND, PER>), dim3(workgroups), dim3(512), 0, s, sink, counters, iters, random_operands);
    return hipGetLastError();
}

hipError_t launch_probe_mfma(float* sink, unsigned long long* counters, int workgroups, int iters, int random_operands,
                             int companion, int per_mfma, hipStream_t s) {
#define LL_PROBE_CASE(K)                                                                                            \
    case K:                                                                                                         \
        return per_mfma == 1 ? launch_probe<K, 1>(sink, counters, workgroups, iters, random_operands, s)            \
                             : launch_probe<K, 2>(sink, counters, workgroups, iters, random_operands, s);
    switch (companion) {
        case PROBE_NONE: return launch_probe<PROBE_NONE, 1>(sink, counters, workgroups, iters, random_operands, s);
        case PROBE_SHAPE_16X16X32: return launch_probe<PROBE_SHAPE_16X16X32, 1>(sink, counters, workgroups, iters, random_operands, s);
        LL_PROBE_CASE(PROBE_ADD)
        LL_PROBE_CASE(PROBE_EXP)
        LL_PROBE_CASE(PROBE_CVT_BF16)
        LL_PROBE_CASE(PROBE_DOT2_BF16)
        LL_PROBE_CASE(PROBE_MAX3)
        LL_PROBE_CASE(PROBE_LDS_READ)
        case PROBE_FP8_NONE: return launch_probe<PROBE_FP8_NONE, 1>(sink, counters, workgroups, iters, random_operands, s);
        case PROBE_FP8_MIX: return launch_probe<PROBE_FP8_MIX, 1>(sink, counters, workgroups, iters, random_operands, s);
        case PROBE_FP8_VALU: return launch_probe<PROBE_FP8_VALU, 1>(sink, counters, workgroups, iters, random_operands, s);
        case PROBE_FP8_LDS: return launch_probe<PROBE_FP8_LDS, 1>(sink, counters, workgroups, iters, random_operands, s);
    }
#undef LL_PROBE_CASE
    return hipErrorInvalidValue;
}

}  // namespace ll

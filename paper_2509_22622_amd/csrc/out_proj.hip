// Output projection of the cross-attention block: y = x w^T with x [M, K] the heads' attention outputs side by side
// (K = H * D), w [N, K] the layer's output weight as a linear layer stores it ([output feature][input feature]),
// y [M, N]; bf16 in and out, fp32 accumulation.  A dense contraction: MFMA-bound (roofline of the bf16 matrix pipe).
//
// Why its own kernel and not an epilogue inside the attention kernel: the projection sums over ALL heads of a token,
// while attention's unit of work is one head (its K/V stream is what a workgroup shares).  A workgroup that held a
// token's all-head output would have to stream the whole weight (4.7 MB at 12 heads x 128) for a few dozen rows; one
// that kept its head would have to add its share into y across workgroups.  So the call runs the attention kernel
// first and this kernel behind it on the same stream.  What the two share is the operand layout: the attention
// kernel's epilogue writes its output as ready-made MFMA fragments (kernels.h: op_frag_offset), which is the order its
// accumulator registers already have, and the weight is packed into the same order once, when the model is loaded.
//
// Why fragments and not row-major operands (measured on this chip): a row-major fragment is 16 rows x 64 bytes, rows
// H * D * 2 bytes apart, and every load instruction gathers 16 separate pieces; L2 delivers 7.7-7.9 TB/s for such
// gathers against 13.8 TB/s for contiguous 1 KB fragments.  The row-major form of this kernel spent its time there
// (6.3 TB/s, whatever the staging: registers, direct-to-LDS loads, whole cache lines, staggered walks).
//
// Formulation, as in the attention kernels: the transposed product y^T = w x^T on 16x16x32 MFMAs.
//   A: w fragment (n block, k-step), B: x fragment (m block, k-step), same order of the 32 contraction indices in both
//   C: lane (g, c) register j = y[m0 + c][n0 + 4 g + j]: four neighbouring output features, one 8-byte store.
// A workgroup of 8 waves (two per SIMD) owns a 256 x 128 tile of y (each wave 64 x 64: 16 accumulator blocks) and
// walks K in steps of 64 through a ring of three LDS stages filled by direct-to-LDS loads two steps ahead: a step is
// 48 fragments (16 of w, 32 of x), six loads per wave, and 32 MFMAs per wave; one barrier per step.  Every w fragment
// is read from LDS by four waves, every x fragment by two.
#include "kernels.h"

namespace ll {

typedef __bf16 op_bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 op_bf16x2 __attribute__((ext_vector_type(2)));
typedef float op_f32x4 __attribute__((ext_vector_type(4)));
typedef float op_f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned op_u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned op_u32x2 __attribute__((ext_vector_type(2)));

// (steps of 32 through six stages, five ahead, take the same time)
constexpr int OP_BM = 256, OP_BN = 128, OP_BK = 64, OP_STAGES = 3, OP_AHEAD = OP_STAGES - 1, OP_WAVES = 8;
constexpr int OP_SUBS = OP_BK / 32;                             // k-steps of 32 per stage
constexpr int OP_WFRAGS = OP_BN / 16 * OP_SUBS;                 // 1 KB fragments per stage: 16 of w,
constexpr int OP_FRAGS = OP_WFRAGS + OP_BM / 16 * OP_SUBS;      // then 32 of x
constexpr int OP_STAGE_BYTES = OP_FRAGS * 1024;
constexpr int OP_LPW = OP_FRAGS / OP_WAVES;                     // fragments a wave loads per stage
static_assert(OP_FRAGS % OP_WAVES == 0 && OP_STAGES == OP_AHEAD + 1 && OP_STAGES * OP_STAGE_BYTES <= 160 * 1024, "ring of the output projection");

// s_waitcnt that only waits for vector-memory loads: at most N outstanding
template <int N>
__device__ __forceinline__ void op_wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}

__global__ __launch_bounds__(64 * OP_WAVES) __attribute__((amdgpu_waves_per_eu(2, 2)))
void ll_out_proj_kernel(const OutProjParams p) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave & 3, wn = wave >> 2;
    // Workgroup b runs on XCD b % 8, each with its own L2: every XCD takes one contiguous run of tiles, weight blocks
    // fastest, so that the tiles it has in flight share a few row blocks of x (read once per XCD, then from its L2 for
    // every weight block) and walk the weight together.
    const int n_nt = (p.N + OP_BN - 1) / OP_BN, n_mt = (p.M + OP_BM - 1) / OP_BM;
    const int total = n_nt * n_mt, xcd = blockIdx.x & 7;
    const int tile = ((xcd * total + 7) >> 3) + (blockIdx.x >> 3);
    if (tile >= (((xcd + 1) * total + 7) >> 3)) return;          // uniform over the workgroup
    const int mt = tile / n_nt, nt = tile % n_nt;
    const int m0 = mt * OP_BM, n0 = nt * OP_BN;
    const int KT = p.K / OP_BK, n_ksteps = p.K / 32;
    const int last_mb = (p.M - 1) >> 4, last_nb = (p.N >> 4) - 1;

    // the fragments this wave loads per stage: fragments wave + 8 l of [w: (n block, sub-step) | x: (m block, sub-step)];
    // the two sub-steps of a block are neighbours in memory.  Blocks past the end of a tensor are clamped to its last
    // block (their products are never stored).
    const char* src[OP_LPW];
#pragma unroll
    for (int l = 0; l < OP_LPW; ++l) {
        const int f = wave + OP_WAVES * l;                       // wave-uniform
        const bool is_w = f < OP_WFRAGS;
        const int blk = is_w ? min((n0 >> 4) + f / OP_SUBS, last_nb) : min((m0 >> 4) + (f - OP_WFRAGS) / OP_SUBS, last_mb);
        src[l] = reinterpret_cast<const char*>(is_w ? p.w_frag : p.x_frag) + (int64_t(blk) * n_ksteps + f % OP_SUBS) * 1024 + lane * 16;
    }
    auto issue = [&](int kt) {
        const int kc = min(kt, KT - 1);          // past the end the last step is fetched again, never used
        char* stage = lds + (kt % OP_STAGES) * OP_STAGE_BYTES;
#pragma unroll
        for (int l = 0; l < OP_LPW; ++l)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src[l] + kc * OP_SUBS * 1024),
                                             (__attribute__((address_space(3))) void*)(stage + (wave + OP_WAVES * l) * 1024), 16, 0, 0);
    };

    op_f32x4 acc[4][4];                          // [n block][m block]
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = op_f32x4{0.f, 0.f, 0.f, 0.f};

#pragma unroll
    for (int j = 0; j < OP_AHEAD; ++j) issue(j);
    for (int kt = 0; kt < KT; ++kt) {
        // this wave's loads of step kt have landed (all but the youngest step's), then every wave's have, and every
        // wave has left step kt - 1, whose stage the loads issued next overwrite
        op_wait_vmcnt<(OP_AHEAD - 1) * OP_LPW>();
        asm volatile("s_barrier" ::: "memory");
        issue(kt + OP_AHEAD);
        const char* st = lds + (kt % OP_STAGES) * OP_STAGE_BYTES + lane * 16;
        op_u32x4 wf[OP_SUBS][4], xf[OP_SUBS][4];
#pragma unroll
        for (int sub = 0; sub < OP_SUBS; ++sub) {
#pragma unroll
            for (int a = 0; a < 4; ++a) wf[sub][a] = *reinterpret_cast<const op_u32x4*>(st + ((wn * 4 + a) * OP_SUBS + sub) * 1024);
#pragma unroll
            for (int b = 0; b < 4; ++b) xf[sub][b] = *reinterpret_cast<const op_u32x4*>(st + (OP_WFRAGS + (wm * 4 + b) * OP_SUBS + sub) * 1024);
        }
#pragma unroll
        for (int sub = 0; sub < OP_SUBS; ++sub)
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(op_bf16x8, wf[sub][a]),
                                                                        __builtin_bit_cast(op_bf16x8, xf[sub][b]), acc[a][b], 0, 0, 0);
    }
    op_wait_vmcnt<0>();                          // the loads issued past the end have landed before the wave leaves

#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const int row = m0 + wm * 64 + 16 * b + r;
        if (row >= p.M) continue;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const int col = n0 + wn * 64 + 16 * a + 4 * g;
            if (col >= p.N) continue;            // N is a multiple of 16: a group of four is inside or outside
            const op_f32x2 lo = {acc[a][b][0], acc[a][b][1]}, hi = {acc[a][b][2], acc[a][b][3]};
            const op_u32x2 o = {__builtin_bit_cast(unsigned, __builtin_convertvector(lo, op_bf16x2)),
                                __builtin_bit_cast(unsigned, __builtin_convertvector(hi, op_bf16x2))};
            *reinterpret_cast<op_u32x2*>(p.y + int64_t(row) * p.N + col) = o;
        }
    }
}

// One thread per 16-byte unit of the packed weight: lane (g, r) of fragment (n block, k-step) takes
// w[16 nb + r][32 ks + 4 g + 0..3] and w[16 nb + r][32 ks + 16 + 4 g + 0..3].
__global__ __launch_bounds__(256) void ll_pack_out_weight_kernel(const uint16_t* w, uint16_t* w_frag, int N, int K) {
    const int64_t unit = int64_t(blockIdx.x) * 256 + threadIdx.x;
    const int n_ksteps = K / 32;
    if (unit >= int64_t(N / 16) * n_ksteps * 64) return;
    const int lane = int(unit & 63), r = lane & 15, g = lane >> 4;
    const int ks = int((unit >> 6) % n_ksteps), nb = int((unit >> 6) / n_ksteps);
    const uint16_t* row = w + int64_t(16 * nb + r) * K + 32 * ks + 4 * g;
    const op_u32x2 lo = *reinterpret_cast<const op_u32x2*>(row), hi = *reinterpret_cast<const op_u32x2*>(row + 16);
    *reinterpret_cast<op_u32x4*>(w_frag + unit * 8) = op_u32x4{lo[0], lo[1], hi[0], hi[1]};
}

hipError_t launch_pack_out_weight(const uint16_t* w, uint16_t* w_frag, int N, int K, hipStream_t s) {
    if (N < 16 || N % 16 != 0 || K < 32 || K % 32 != 0) return hipErrorInvalidValue;
    const int64_t units = int64_t(N / 16) * (K / 32) * 64;
    if ((units + 255) / 256 > 0x7FFFFFFF) return hipErrorInvalidValue;
    hipLaunchKernelGGL(ll_pack_out_weight_kernel, dim3(unsigned((units + 255) / 256)), dim3(256), 0, s, w, w_frag, N, K);
    return hipGetLastError();
}

hipError_t launch_out_proj(const OutProjParams& p, hipStream_t s) {
    if (p.M < 1 || p.N < 16 || p.N % 16 != 0 || p.K < OP_BK || p.K % OP_BK != 0) return hipErrorInvalidValue;   // K = H * D, D 64 or 128
    const int64_t tiles = int64_t((p.M + OP_BM - 1) / OP_BM) * ((p.N + OP_BN - 1) / OP_BN);
    if (tiles > 0x7FFFFFFF) return hipErrorInvalidValue;
    constexpr int lds_bytes = OP_STAGES * OP_STAGE_BYTES;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(ll_out_proj_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(ll_out_proj_kernel, dim3(unsigned((tiles + 7) / 8 * 8)), dim3(64 * OP_WAVES), lds_bytes, s, p);
    return hipGetLastError();
}

}  // namespace ll

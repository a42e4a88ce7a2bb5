// Output projection of the cross-attention block: y = x w^T with x [M, K] the heads' attention outputs side by side
// (K = H * D), w [N, K] the layer's output weight as a linear layer stores it ([output feature][input feature]),
// y [M, N]; bf16 in and out, fp32 accumulation.  A dense contraction: MFMA-bound (roofline of the bf16 matrix pipe).
//
// Why its own kernel and not an epilogue inside the attention kernel: the projection sums over ALL heads of a token,
// while attention's unit of work is one head (its K/V stream is what a workgroup shares).  A workgroup that held a
// token's all-head output would have to stream the whole weight (4.7 MB at 12 heads x 128) for a few dozen rows; one
// that kept its head would have to add its share into y across workgroups.  So the call runs the attention kernel
// first and this kernel behind it on the same stream; the attention output stays in the caller's tensor (14 MB at the
// benchmark shape: it is still in the last-level cache when this kernel reads it).
//
// Formulation, as in the attention kernels: the transposed product y^T = w x^T on 16x16x32 MFMAs.
//   A: w fragment, lane (g, r) holds w[n0 + r][k0 + 8 g + 0..7]  (16 contiguous bytes of a weight row)
//   B: x fragment, lane (g, r) holds x[m0 + r][k0 + 8 g + 0..7]  (16 contiguous bytes of an activation row)
//   C: lane (g, c) register j = y[m0 + c][n0 + 4 g + j]: four neighbouring output features, one 8-byte store.
// A workgroup of 8 waves (two per SIMD) owns a 256 x 128 tile of y (each wave 64 x 64: 16 accumulator blocks) and
// walks K in steps of 64 through two LDS stages: a wave loads its share of the next step's 48 fragments (16 of w, 32
// of x, 1 KB each) into registers while the MFMAs of the current step run, and stores them behind the step; one
// barrier per step of 32 MFMAs per wave.  Every w fragment is read by four waves, every x fragment by two.
//
// What bounds it (measured): not the matrix pipe.  Both operands are row-major with rows H * D * 2 bytes apart, so a
// fragment is 16 rows x 64 bytes and every load instruction gathers 16 separate pieces; the chip delivers about 6 TB/s
// from L2 for such gathers (the same tile walked with direct-to-LDS loads, with whole-cache-line pieces, or with the
// tiles' walks staggered against each other, all take the same time), against 13.6 TB/s for the attention kernels'
// contiguous 1 KB fragments.  At 85 flop per byte fetched (a 256 x 128 tile) that is about 520 TFLOP/s.  The next step
// would be operands stored as fragments: the weight packed once when the model is loaded, the attention output
// written in fragment order by the attention kernel's epilogue.
#include "kernels.h"

namespace ll {

typedef __bf16 op_bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 op_bf16x2 __attribute__((ext_vector_type(2)));
typedef float op_f32x4 __attribute__((ext_vector_type(4)));
typedef float op_f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned op_u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned op_u32x2 __attribute__((ext_vector_type(2)));

constexpr int OP_BM = 256, OP_BN = 128, OP_BK = 64, OP_STAGES = 2, OP_WAVES = 8;
constexpr int OP_FRAGS = (OP_BM + OP_BN) / 16 * (OP_BK / 32);   // 1 KB fragments per stage: 16 of w, then 32 of x
constexpr int OP_STAGE_BYTES = OP_FRAGS * 1024;
constexpr int OP_LPW = OP_FRAGS / OP_WAVES;                     // fragments a wave moves per stage

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
    const int KT = p.K / OP_BK;

    // the fragments this wave moves per stage: fragments OP_LPW * wave .. of [w: (n block, sub-step) | x: (m block,
    // sub-step)], through registers: a lane loads the 16 bytes the MFMA wants from it and stores them at byte 16 * lane
    // of the fragment.  Rows past the end of a tensor are clamped to its last row (their products are never stored).
    const uint16_t* src[OP_LPW];
#pragma unroll
    for (int l = 0; l < OP_LPW; ++l) {
        const int f = wave * OP_LPW + l;
        constexpr int NWF = OP_BN / 16 * (OP_BK / 32);
        if (f < NWF) src[l] = p.w + int64_t(min(n0 + 16 * (f >> 1) + r, p.N - 1)) * p.K + 32 * (f & 1) + 8 * g;
        else src[l] = p.x + int64_t(min(m0 + 16 * ((f - NWF) >> 1) + r, p.M - 1)) * p.K + 32 * (f & 1) + 8 * g;
    }
    op_u32x4 stage_regs[OP_LPW];
    auto load = [&](int kt) {
        const int kc = min(kt, KT - 1);          // past the end the last step is fetched again, never used
#pragma unroll
        for (int l = 0; l < OP_LPW; ++l) stage_regs[l] = *reinterpret_cast<const op_u32x4*>(src[l] + kc * OP_BK);
    };
    auto store = [&](int kt) {
        char* dst = lds + (kt % OP_STAGES) * OP_STAGE_BYTES + wave * OP_LPW * 1024 + lane * 16;
#pragma unroll
        for (int l = 0; l < OP_LPW; ++l) *reinterpret_cast<op_u32x4*>(dst + l * 1024) = stage_regs[l];
    };

    op_f32x4 acc[4][4];                          // [n block][m block]
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = op_f32x4{0.f, 0.f, 0.f, 0.f};

    load(0);
    store(0);
    load(1);
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        const char* st = lds + (kt % OP_STAGES) * OP_STAGE_BYTES + lane * 16;
        op_u32x4 wf[2][4], xf[2][4];
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
            for (int a = 0; a < 4; ++a) wf[sub][a] = *reinterpret_cast<const op_u32x4*>(st + ((wn * 4 + a) * 2 + sub) * 1024);
#pragma unroll
            for (int b = 0; b < 4; ++b) xf[sub][b] = *reinterpret_cast<const op_u32x4*>(st + (16 + (wm * 4 + b) * 2 + sub) * 1024);
        }
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(op_bf16x8, wf[sub][a]),
                                                                        __builtin_bit_cast(op_bf16x8, xf[sub][b]), acc[a][b], 0, 0, 0);
        // the other stage was last read in step kt - 1, which every wave left before the barrier that ended it
        store(kt + 1);
        load(kt + 2);
        // the LDS writes above must be visible behind the barrier; the loads just issued stay in flight across it
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    }

#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const int row = m0 + wm * 64 + 16 * b + r;
        if (row >= p.M) continue;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const int col = n0 + wn * 64 + 16 * a + 4 * g;
            if (col >= p.N) continue;            // N is a multiple of 4: a group of four is inside or outside
            const op_f32x2 lo = {acc[a][b][0], acc[a][b][1]}, hi = {acc[a][b][2], acc[a][b][3]};
            const op_u32x2 o = {__builtin_bit_cast(unsigned, __builtin_convertvector(lo, op_bf16x2)),
                                __builtin_bit_cast(unsigned, __builtin_convertvector(hi, op_bf16x2))};
            *reinterpret_cast<op_u32x2*>(p.y + int64_t(row) * p.N + col) = o;
        }
    }
}

hipError_t launch_out_proj(const OutProjParams& p, hipStream_t s) {
    if (p.M < 1 || p.N < 4 || p.N % 4 != 0 || p.K < OP_BK || p.K % OP_BK != 0) return hipErrorInvalidValue;   // K = H * D, D 64 or 128
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

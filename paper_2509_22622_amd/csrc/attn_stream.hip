// Software-pipelined sink+window attention kernel (same mathematics and cache layout as
// attn_kernel.hip; see there and kernels.h).
//
// 8 waves per workgroup, 32 queries per wave, two waves per SIMD.  Measured on gfx950 a
// wave issues at most one VALU instruction every ~9 cycles while the SIMD can take one
// every 4, and a 32x32x16 MFMA holds the matrix pipe for 32 cycles; both pipes stay busy
// only when every wave's own instruction stream mixes MFMA and VALU work.  Each loop
// iteration therefore carries three independent strands for three consecutive kblocks:
//     matrix : O^T += V^T P^T of kblock i-1, then S^T = K Q^T of kblock i+1
//     vector : softmax numerators of kblock i (exp2, bf16 packing, row sums)
//     memory : LDS fragment reads for the next iteration, direct-to-LDS loads PF ahead
// and one workgroup barrier hands the LDS ring stages over.
//
// VALU work is kept minimal: queries arrive pre-scaled by log2(e)/sqrt(D) (the append
// kernel folds that factor into the rotary epilogue), the score accumulator starts at
// minus the running reference maximum, so p = exp2(acc) needs no further arithmetic;
// row sums are taken over the bf16-rounded p (the values the second MFMA consumes) with
// the packed dot-product instruction.  The reference maximum moves only when a score
// exceeds it by more than RESCALE_SLACK (then O, the row sum and the pending scores are
// rescaled); the final division by the row sum makes the result independent of it.
#include "kernels.h"

namespace ll {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

constexpr float SP_RESCALE_SLACK = 6.0f;         // log2 units: p stays below 2^6 between rescales

__device__ inline unsigned sp_pack_bf16(float a, float b) {
    f32x2 v = {a, b};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}
// acc + lo + hi of a packed bf16 pair
__device__ inline float sp_pair_sum(unsigned pair, float acc) {
    const bf16x2 one = {(__bf16)1.0f, (__bf16)1.0f};
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pair), one, acc, false);
}
// s_waitcnt that only waits for vector-memory loads: at most N outstanding.
template <int N>
__device__ inline void sp_wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}

// Up to three token-slot ranges are walked as one virtual list of kblocks: virtual index v lies
// in range 0 (v < n0), 1 (v < n01) or 2.  All arguments are plain scalars passed by value so
// that everything stays in scalar registers.
__device__ __forceinline__ int sp_pick(int v, int n0, int n01, int a0, int a1, int a2) {
    return v < n0 ? a0 : (v < n01 ? a1 : a2);
}
// bit r set: the key held by accumulator register r of a lane in `half` is inside [rs, re)
__device__ __forceinline__ unsigned sp_live_mask(int key0, int rs, int re, int half) {
    unsigned live = 0;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int key = key0 + 16 * (r >> 3) + 8 * half + (r & 7);
        if (key >= rs && key < re) live |= 1u << r;
    }
    return live;
}

template <int D, int PF>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void ll_attn_sp_kernel(const AttnParams p) {
    constexpr int KS = D / 16;                  // k-steps of S^T = K Q^T, also fragments per K kblock
    constexpr int DB = D / 32;                  // 32-row blocks of O^T
    constexpr int KB_BYTES = KBLOCK * D * 2;
    constexpr int STAGE_BYTES = 2 * KB_BYTES;   // [K kblock | V kblock]
    constexpr int NS = PF + 2;                  // ring stages: a stage is rewritten two barriers after its last read
    constexpr int NF = 2 * KS;                  // 1 KB fragments per stage
    constexpr int LPW = NF / 8;                 // loads per wave per kblock
    constexpr int QT = 256;
    static_assert(NF % 8 == 0, "fragments must split over 8 waves");
    static_assert(PF >= 3, "kblock i + 2 must have landed when iteration i starts");

    extern __shared__ __attribute__((aligned(16))) char lds[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in a scalar register
    const int col = lane & 31, half = lane >> 5;

    const int total = p.n_tiles * p.H;
    const int per_xcd = (total + 7) >> 3;
    const int item = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (item >= total) return;                  // uniform over the workgroup
    const int head = item / p.n_tiles;
    const int tile = item % p.n_tiles;
    int ci = 0;
    while (ci + 1 < p.n_chunks && tile >= p.chunk[ci + 1].tile_begin) ++ci;
    const AttnChunk& ch = p.chunk[ci];
    const int q0 = ch.q_begin + (tile - ch.tile_begin) * QT + wave * 32;
    const int n_ranges = ch.n_ranges;
    // ranges in scalar registers (no kernel-argument loads inside the loop)
    const int rs0 = ch.rs[0], re0 = ch.re[0];
    int rs1 = ch.rs[1], re1 = ch.re[1], rs2 = ch.rs[2], re2 = ch.re[2];   // loaded unconditionally, then blanked
    if (n_ranges < 2) rs1 = re1 = 0;
    if (n_ranges < 3) rs2 = re2 = 0;
    const int kb0 = rs0 / KBLOCK, ke0 = (re0 + KBLOCK - 1) / KBLOCK;      // kblock spans of the ranges
    const int kb1 = rs1 / KBLOCK, ke1 = (re1 + KBLOCK - 1) / KBLOCK;
    const int kb2 = rs2 / KBLOCK, ke2 = (re2 + KBLOCK - 1) / KBLOCK;
    const int q_end = ch.q_end;
    const int T = (ke0 - kb0) + (ke1 - kb1) + (ke2 - kb2);                // kblocks over all ranges

    bf16x8 qf[KS];                               // Q^T fragments (pre-scaled by log2(e)/sqrt(D))
    {
        const int row = min(q0 + col, q_end - 1);
        const uint16_t* src = p.q + (int64_t(row) * p.H + head) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(src + ks * 16);
    }

    const char* kbase = reinterpret_cast<const char*>(p.k_cache + head * p.head_stride);
    const char* vbase = reinterpret_cast<const char*>(p.v_cache + head * p.head_stride);

    const int n0 = ke0 - kb0, n01 = n0 + (ke1 - kb1);                     // kblocks in range 0, in ranges 0 and 1
    // physical kblock of virtual kblock v, its range, and whether it is the first or last kblock of a
    // range (only those can be cut by a range boundary; they take the slow path)
#define SP_PHYS_KB(v) ((v) + sp_pick((v), n0, n01, kb0, kb1 - n0, kb2 - n01))
#define SP_LIVE(v) sp_live_mask(SP_PHYS_KB(v) * KBLOCK, sp_pick((v), n0, n01, rs0, rs1, rs2), sp_pick((v), n0, n01, re0, re1, re2), half)
#define SP_IS_EDGE(v) ((v) == 0 || (v) == n0 - 1 || (v) == n0 || (v) == n01 - 1 || (v) == n01 || (v) == T - 1)

    // direct-to-LDS loads of physical kblock kb into a ring stage
    const unsigned lane_off = lane * 16;
    auto issue_loads = [&](int kb, int stage) {
        const int64_t kb_off = int64_t(kb) * KB_BYTES;
#pragma unroll
        for (int l = 0; l < LPW; ++l) {
            const int f = wave + 8 * l;         // fragment of the stage this wave fetches
            const char* sbase = (f < KS ? kbase + f * 1024 : vbase + (f - KS) * 1024) + kb_off;   // wave-uniform
            const char* src = sbase + lane_off;
            char* dst = lds + stage * STAGE_BYTES + f * 1024;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src),
                                             (__attribute__((address_space(3))) void*)(dst), 16, 0, 0);
        }
    };
    auto next_stage = [](int st) { return st + 1 == NS ? 0 : st + 1; };

#pragma unroll
    for (int j = 0; j < PF; ++j) {
        const int v = min(j, T - 1);             // past the end the last kblock is fetched again, never used
        issue_loads(SP_PHYS_KB(v), j);
    }
    sp_wait_vmcnt<(PF - 3) * LPW>();            // this wave's loads of kblocks 0..2 have landed
    __builtin_amdgcn_s_barrier();

    auto read_k = [&](int st, bf16x8 (&a)[KS]) {
        const char* kt = lds + st * STAGE_BYTES + lane_off;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) a[ks] = *reinterpret_cast<const bf16x8*>(kt + ks * 1024);
    };
    auto read_v = [&](int st, u32x4 (&av)[2][DB]) {
        const char* vt = lds + st * STAGE_BYTES + KB_BYTES + lane_off;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int db = 0; db < DB; ++db) av[t][db] = *reinterpret_cast<const u32x4*>(vt + (db * 2 + t) * 1024);
    };
    // dead slots may hold anything, even NaN: zero the V elements of keys outside the range
    auto mask_v = [&](u32x4 (&av)[2][DB], unsigned live) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const unsigned b0 = (live >> (8 * t + 2 * e)) & 1, b1 = (live >> (8 * t + 2 * e + 1)) & 1;
                const unsigned m = (b0 ? 0x0000FFFFu : 0u) | (b1 ? 0xFFFF0000u : 0u);
#pragma unroll
                for (int db = 0; db < DB; ++db) av[t][db][e] &= m;
            }
    };

    f32x16 o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
    float lsum0 = 0.f, lsum1 = 0.f;              // row sum of this lane's keys (two chains)
    f32x16 negm;                                 // every element = -(reference maximum) of this lane's query
    f32x16 s;                                    // scores of kblock i minus the reference, log2 domain
    bf16x8 kfr[KS];                              // K fragments of kblock i + 1
    u32x4 vfr[2][DB];                            // V^T fragments of kblock i - 1
    unsigned pb[2][4];                           // P^T fragments of kblock i - 1 (bf16 pairs)

    // ---- prologue: scores of kblock 0 with a zero reference, then the true first reference
    read_k(0, kfr);
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[ks], qf[ks], s, 0, 0, 0);
    auto mask_s = [&](unsigned live) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
            if (!((live >> r) & 1)) s[r] = -INFINITY;
    };
    auto max_s = [&]() {
        float mx = fmaxf(fmaxf(s[0], s[1]), s[2]);
#pragma unroll
        for (int r = 3; r < 15; r += 2) mx = fmaxf(fmaxf(mx, s[r]), s[r + 1]);
        return fmaxf(mx, s[15]);
    };
    mask_s(SP_LIVE(0));
    {
        float mx = s[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
        const float m0 = fmaxf(mx, __shfl_xor(mx, 32));   // a kblock of a range holds a live key: finite
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            negm[r] = -m0;
            s[r] -= m0;
        }
    }
    read_k(1 % NS, kfr);
#pragma unroll
    for (int t = 0; t < 2; ++t) {
#pragma unroll
        for (int e = 0; e < 4; ++e) pb[t][e] = 0u;
#pragma unroll
        for (int db = 0; db < DB; ++db) vfr[t][db] = u32x4{0u, 0u, 0u, 0u};
    }
    int st_v = 0;                                // stage of kblock i
    int st_k = 2 % NS;                           // stage of kblock i + 2
    int st_ld = PF % NS;                         // stage the next loads go to

    bool edge_prev = false;                      // kblock i - 1 (whose V fragments are in vfr) is cut by a range boundary
    for (int i = 0; i < T; ++i) {
        // ---- rare path: a kblock cut by a range boundary, or a score above the reference by more than the slack
        {
            const bool edge_cur = i > 0 && SP_IS_EDGE(i);      // kblock 0 was masked in the prologue
            float mx = max_s();
            if (__any(mx > SP_RESCALE_SLACK) || edge_cur || edge_prev) {
                if (edge_prev) mask_v(vfr, SP_LIVE(i - 1));
                if (edge_cur) {
                    mask_s(SP_LIVE(i));
                    mx = max_s();
                }
                const float delta = fmaxf(fmaxf(mx, __shfl_xor(mx, 32)), 0.f);
                const float alpha = __builtin_amdgcn_exp2f(-delta);
                lsum0 *= alpha;
                lsum1 *= alpha;
                // P^T of kblock i-1 is still waiting for its MFMA: bring it to the new reference too
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        pb[t][e] = sp_pack_bf16(__uint_as_float(pb[t][e] << 16) * alpha,
                                                __uint_as_float(pb[t][e] & 0xFFFF0000u) * alpha);
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    negm[r] -= delta;
                    s[r] -= delta;
                }
            }
            edge_prev = SP_IS_EDGE(i);
        }

        // ---- memory strand: loads PF kblocks ahead
        {
            const int v = min(i + PF, T - 1);
            issue_loads(SP_PHYS_KB(v), st_ld);
        }

        // ---- first half: p = 2^s on the vector pipe while O^T += V^T P^T (kblock i-1) runs on the matrix pipe
        float pr[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) pr[r] = __builtin_amdgcn_exp2f(s[r]);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const u32x4 bv = {pb[t][0], pb[t][1], pb[t][2], pb[t][3]};
#pragma unroll
            for (int db = 0; db < DB; ++db)
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vfr[t][db]),
                                                                 __builtin_bit_cast(bf16x8, bv), o[db], 0, 0, 0);
        }
#pragma unroll
        for (int g = 0; g < 2 * DB; ++g) {       // one MFMA, then its share of the exponentials
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 16 / (2 * DB), 0);
        }
        read_v(st_v, vfr);                       // kblock i, consumed by the next iteration
        __builtin_amdgcn_sched_group_barrier(0x100, 2 * DB, 0);

        // ---- second half: S^T = K Q^T - m (kblock i+1) on the matrix pipe, bf16 packing and row sums beside it
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[0], qf[0], negm, 0, 0, 0);
#pragma unroll
        for (int ks = 1; ks < KS; ++ks) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[ks], qf[ks], s, 0, 0, 0);
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int e = 0; e < 4; ++e) pb[t][e] = sp_pack_bf16(pr[8 * t + 2 * e], pr[8 * t + 2 * e + 1]);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            lsum0 = sp_pair_sum(pb[0][e], lsum0);
            lsum1 = sp_pair_sum(pb[1][e], lsum1);
        }
#pragma unroll
        for (int g = 0; g < KS; ++g) {           // one MFMA, then its share of the pack / sum instructions
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 16 / KS, 0);
        }
        read_k(st_k, kfr);                       // kblock i + 2, consumed by the next iteration
        __builtin_amdgcn_sched_group_barrier(0x100, KS, 0);

        st_ld = next_stage(st_ld);
        st_v = next_stage(st_v);
        st_k = next_stage(st_k);
        sp_wait_vmcnt<(PF - 3) * LPW>();         // this wave's loads of kblocks up to i + 3 have landed
        __builtin_amdgcn_s_barrier();
    }
    // ---- epilogue: O^T += V^T P^T of the last kblock
    if (edge_prev) mask_v(vfr, SP_LIVE(T - 1));
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const u32x4 bv = {pb[t][0], pb[t][1], pb[t][2], pb[t][3]};
#pragma unroll
        for (int db = 0; db < DB; ++db)
            o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vfr[t][db]),
                                                             __builtin_bit_cast(bf16x8, bv), o[db], 0, 0, 0);
    }
    sp_wait_vmcnt<0>();                          // nothing may still be writing LDS when the wave ends

    const float lsum = lsum0 + lsum1;
    const float l = lsum + __shfl_xor(lsum, 32);
    const float inv = 1.0f / l;
    const int row = q0 + col;
    if (row < q_end) {
        uint16_t* dst = p.out + (int64_t(row) * p.H + head) * D + half * 4;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                u32x2 w = {sp_pack_bf16(o[db][4 * g] * inv, o[db][4 * g + 1] * inv),
                           sp_pack_bf16(o[db][4 * g + 2] * inv, o[db][4 * g + 3] * inv)};
                *reinterpret_cast<u32x2*>(dst + db * 32 + g * 8) = w;
            }
    }
}

#undef SP_PHYS_KB
#undef SP_LIVE
#undef SP_IS_EDGE

const AttnVariant kStreamVariants[] = {
    {"d128_sp_pf4", 128, 256, 6 * 2 * KBLOCK * 128 * 2, ll_attn_sp_kernel<128, 4>, 512},
    {"d128_sp_pf6", 128, 256, 8 * 2 * KBLOCK * 128 * 2, ll_attn_sp_kernel<128, 6>, 512},
    {"d64_sp_pf4", 64, 256, 6 * 2 * KBLOCK * 64 * 2, ll_attn_sp_kernel<64, 4>, 512},
};
const int kNumStreamVariants = sizeof(kStreamVariants) / sizeof(kStreamVariants[0]);

}  // namespace ll
